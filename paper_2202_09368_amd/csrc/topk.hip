// G, I = TopK(S^T, k): every expert takes its k best tokens (Sec. 3.2, Eq. 2).
//
// One 1024-thread workgroup per expert works on that expert's row of S^T
// (n contiguous floats).  Scores are non-negative, so their bit patterns order
// like unsigned integers, and (score bits, ~token) is a total order in which
// "larger" means "admitted first".  Steps:
//   1. stage the row in LDS when it fits (one HBM read), find min and max;
//   2. radix-select on (bits - min), 8 bits per pass starting at the top bit of
//      the actual range, until the bin holding the k-th score has at most
//      TOPK_CAND_MAX members or all 32 bits are decided;
//   3. find the cut-off key, the k-th largest (score, ~token): among few
//      candidates by counting, among many exact ties by token order;
//   4. every wavefront owns a contiguous range of tokens: count the admitted
//      ones per range, prefix the counts, then write the bucket in ascending
//      token order with ballot ranks.  No sort is needed.
#include "ec_common.h"

namespace ecmoe {

constexpr int TOPK_THREADS = 1024;
constexpr int TOPK_WAVES = TOPK_THREADS / kWave;
constexpr int TOPK_CAND_MAX = 256;

// Optional token-major by-products for the combine stage, written while the bucket is emitted:
// either a slot list per token (slot_cnt[l] counts the experts that chose token l, the first
// `slot_cap` of them leave their bucket row i*k+j in slots[l*slot_cap + ...], in arrival order)
// or one bit per (token, expert) in `bitmap` (`bitmap_words` 32-bit words per token).
// Integer atomics only: the set of entries does not depend on the order of arrival.
struct TopkEmit {
    int32_t* slot_cnt;
    int32_t* slots;
    int slot_cap;
    uint32_t* bitmap;
    int bitmap_words;
};

__device__ __forceinline__ void topk_emit(const TopkEmit& em, int expert, int k, int rank, int tok) {
    if (em.slot_cnt != nullptr) {
        int s = atomicAdd(&em.slot_cnt[tok], 1);
        if (s < em.slot_cap) em.slots[(size_t)tok * em.slot_cap + s] = expert * k + rank;
    }
    if (em.bitmap != nullptr) atomicOr(&em.bitmap[(size_t)tok * em.bitmap_words + (expert >> 5)], 1u << (expert & 31));
}

struct TopkShared {
    unsigned int hist[256];
    unsigned int red[2 * TOPK_WAVES];
    unsigned int wave_cnt[TOPK_WAVES];
    unsigned long long cand[TOPK_CAND_MAX];
    unsigned long long cutoff;
    unsigned int bin, remaining, ncand, slot;
};

__device__ __forceinline__ unsigned long long topk_key(unsigned int bits, unsigned int tok) {
    return ((unsigned long long)bits << 32) | (unsigned long long)(0xFFFFFFFFu - tok);
}

template <bool STAGED>
__global__ void __launch_bounds__(TOPK_THREADS)
topk_tokens_kernel(const float* __restrict__ St, int n, int k, float* __restrict__ G, int32_t* __restrict__ I,
                   TopkEmit emit) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ TopkShared sh;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int expert = blockIdx.x;
    const unsigned int* __restrict__ colg = reinterpret_cast<const unsigned int*>(St) + (size_t)expert * n;
    unsigned int* cols = reinterpret_cast<unsigned int*>(smem);

    // ---- 1. stage + min/max ------------------------------------------------
    unsigned int vmin = 0xFFFFFFFFu, vmax = 0u;
    const bool vec_ok = (n & 3) == 0;  // rows are 16-byte aligned: four scores per load
    if (vec_ok) {
        const uint4* __restrict__ colg4 = reinterpret_cast<const uint4*>(colg);
#pragma unroll 4
        for (int q = tid; q < (n >> 2); q += TOPK_THREADS) {
            const uint4 v = colg4[q];
            if (STAGED) reinterpret_cast<uint4*>(cols)[q] = v;
            const unsigned int lo4 = min(min(v.x, v.y), min(v.z, v.w)), hi4 = max(max(v.x, v.y), max(v.z, v.w));
            vmin = lo4 < vmin ? lo4 : vmin;
            vmax = hi4 > vmax ? hi4 : vmax;
        }
    } else {
        for (int idx = tid; idx < n; idx += TOPK_THREADS) {
            unsigned int v = colg[idx];
            if (STAGED) cols[idx] = v;
            vmin = v < vmin ? v : vmin;
            vmax = v > vmax ? v : vmax;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        unsigned int a = __shfl_xor(vmin, off, kWave), b = __shfl_xor(vmax, off, kWave);
        vmin = a < vmin ? a : vmin;
        vmax = b > vmax ? b : vmax;
    }
    if (lane == 0) { sh.red[wave] = vmin; sh.red[TOPK_WAVES + wave] = vmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < TOPK_WAVES; ++w) {
        unsigned int a = sh.red[w], b = sh.red[TOPK_WAVES + w];
        vmin = a < vmin ? a : vmin;
        vmax = b > vmax ? b : vmax;
    }
    auto ld = [&](int idx) -> unsigned int { return STAGED ? cols[idx] : colg[idx]; };

    // ---- 2. radix select on key = v - vmin --------------------------------
    const unsigned int range = vmax - vmin;
    int lo = range == 0 ? 0 : 32 - __clz(range);  // bits [lo, 32) of the key are decided so far
    unsigned int prefix = 0;                      // their value for the k-th score
    unsigned int remaining = (unsigned int)k;     // how many to take among the candidates
    unsigned int cand = (unsigned int)n;          // scores matching the prefix
    while (cand > (unsigned int)TOPK_CAND_MAX && lo > 0) {
        const int nlo = lo > 8 ? lo - 8 : 0;
        const unsigned int dmask = (1u << (lo - nlo)) - 1u;
        const unsigned int hmask = lo >= 32 ? 0u : ~((1u << lo) - 1u);
        if (tid < 256) sh.hist[tid] = 0;
        __syncthreads();
        if (!STAGED && vec_ok) {
            const uint4* __restrict__ colg4 = reinterpret_cast<const uint4*>(colg);
#pragma unroll 4
            for (int q = tid; q < (n >> 2); q += TOPK_THREADS) {
                const uint4 v = colg4[q];
                const unsigned int k4[4] = {v.x - vmin, v.y - vmin, v.z - vmin, v.w - vmin};
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if ((k4[u] & hmask) == prefix) atomicAdd(&sh.hist[(k4[u] >> nlo) & dmask], 1u);
            }
        } else {
            for (int idx = tid; idx < n; idx += TOPK_THREADS) {
                unsigned int key = ld(idx) - vmin;
                if ((key & hmask) == prefix) atomicAdd(&sh.hist[(key >> nlo) & dmask], 1u);
            }
        }
        __syncthreads();
        if (wave == 0) {
            // lane owns bins 4*lane .. 4*lane+3; find the bin where the count from the top reaches `remaining`
            unsigned int h0 = sh.hist[4 * lane], h1 = sh.hist[4 * lane + 1], h2 = sh.hist[4 * lane + 2],
                         h3 = sh.hist[4 * lane + 3];
            unsigned int tot = h0 + h1 + h2 + h3;
            unsigned int incl = tot;  // inclusive suffix sum over lanes >= this one
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                unsigned int o = __shfl_down(incl, off, kWave);
                if (lane + off < 64) incl += o;
            }
            unsigned int above = incl - tot;  // scores in bins of higher lanes
            if (above < remaining && remaining <= incl) {
                unsigned int a3 = above, a2 = a3 + h3, a1 = a2 + h2, a0 = a1 + h1;
                unsigned int b, ab, hb;
                if (remaining <= a2) { b = 3; ab = a3; hb = h3; }
                else if (remaining <= a1) { b = 2; ab = a2; hb = h2; }
                else if (remaining <= a0) { b = 1; ab = a1; hb = h1; }
                else { b = 0; ab = a0; hb = h0; }
                sh.bin = 4 * lane + b;
                sh.remaining = remaining - ab;
                sh.ncand = hb;
            }
        }
        __syncthreads();
        prefix |= sh.bin << nlo;
        remaining = sh.remaining;
        cand = sh.ncand;
        lo = nlo;
        __syncthreads();
    }
    const unsigned int hmask = lo >= 32 ? 0u : ~((1u << lo) - 1u);

    // Token range of every wavefront (multiple of 64 so chunks stay aligned).
    const int per_wave = ((n + TOPK_WAVES - 1) / TOPK_WAVES + kWave - 1) / kWave * kWave;
    const int w_beg = wave * per_wave;
    const int w_end = (w_beg + per_wave) < n ? (w_beg + per_wave) : n;

    // ---- 3. the cut-off key ---------------------------------------------------
    if (cand <= (unsigned int)TOPK_CAND_MAX) {
        // Few candidates: gather their keys, then the one with exactly remaining-1 keys above it is the cut-off.
        if (tid == 0) sh.slot = 0;
        __syncthreads();
        const int n_round = (n + TOPK_THREADS - 1) / TOPK_THREADS * TOPK_THREADS;
        for (int idx = tid; idx < n_round; idx += TOPK_THREADS) {
            bool is_cand = false;
            unsigned int v = 0;
            if (idx < n) {
                v = ld(idx);
                is_cand = ((v - vmin) & hmask) == prefix;
            }
            unsigned long long bal = __ballot(is_cand);
            unsigned int base = 0;
            if (bal != 0ull) {
                if (lane == 0) base = atomicAdd(&sh.slot, (unsigned int)__popcll(bal));
                base = __shfl(base, 0, kWave);
            }
            if (is_cand) sh.cand[base + __popcll(bal & ((1ull << lane) - 1ull))] = topk_key(v, (unsigned int)idx);
        }
        __syncthreads();
        if (tid < (int)cand) {
            const unsigned long long mine = sh.cand[tid];
            const unsigned int mhi = (unsigned int)(mine >> 32), mlo = (unsigned int)mine;
            unsigned int above = 0;
            for (unsigned int j = 0; j < cand; ++j) {
                const unsigned long long o = sh.cand[j];
                const unsigned int ohi = (unsigned int)(o >> 32), olo = (unsigned int)o;
                above += (ohi > mhi) | ((ohi == mhi) & (olo > mlo));
            }
            if (above == remaining - 1u) sh.cutoff = mine;
        }
    } else {
        // All 32 bits decided and still many candidates: exact ties at the threshold score.  The cut-off is
        // the `remaining`-th tied token in token order.
        const unsigned int tbits = prefix + vmin;
        unsigned int ties = 0;
        for (int base = w_beg; base < w_end; base += kWave) {
            int idx = base + lane;
            bool eq = idx < w_end && ld(idx) == tbits;
            ties += (unsigned int)__popcll(__ballot(eq));
        }
        if (lane == 0) sh.wave_cnt[wave] = ties;
        __syncthreads();
        unsigned int before = 0;
#pragma unroll
        for (int w = 0; w < TOPK_WAVES; ++w) before += w < wave ? sh.wave_cnt[w] : 0u;
        if (before < remaining && remaining <= before + ties) {  // this wavefront holds the cut-off token
            unsigned int seen = before;
            for (int base = w_beg; base < w_end; base += kWave) {
                int idx = base + lane;
                bool eq = idx < w_end && ld(idx) == tbits;
                unsigned long long bal = __ballot(eq);
                unsigned int c = (unsigned int)__popcll(bal);
                if (seen + c >= remaining) {
                    unsigned int rank = seen + (unsigned int)__popcll(bal & ((1ull << lane) - 1ull));
                    if (eq && rank == remaining - 1u) sh.cutoff = topk_key(tbits, (unsigned int)idx);
                    break;
                }
                seen += c;
            }
        }
    }
    __syncthreads();
    const unsigned long long cutoff = sh.cutoff;
    const unsigned int chi = (unsigned int)(cutoff >> 32), clo = (unsigned int)cutoff;
    auto admitted = [&](unsigned int v, int idx) -> bool {
        const unsigned int klo = 0xFFFFFFFFu - (unsigned int)idx;
        return (v > chi) | ((v == chi) & (klo >= clo));
    };

    // ---- 4. count per wavefront range, prefix, emit in token order ------------
    unsigned int mine_cnt = 0;
    for (int base = w_beg; base < w_end; base += kWave) {
        int idx = base + lane;
        bool sel = idx < w_end && admitted(ld(idx), idx);
        mine_cnt += (unsigned int)__popcll(__ballot(sel));
    }
    __syncthreads();  // wave_cnt may still be read by the tie path above
    if (lane == 0) sh.wave_cnt[wave] = mine_cnt;
    __syncthreads();
    unsigned int pos = 0;
#pragma unroll
    for (int w = 0; w < TOPK_WAVES; ++w) pos += w < wave ? sh.wave_cnt[w] : 0u;
    for (int base = w_beg; base < w_end; base += kWave) {
        int idx = base + lane;
        unsigned int v = idx < w_end ? ld(idx) : 0u;
        bool sel = idx < w_end && admitted(v, idx);
        unsigned long long bal = __ballot(sel);
        if (sel) {
            const unsigned int j = pos + (unsigned int)__popcll(bal & ((1ull << lane) - 1ull));
            if (j < (unsigned int)k) {  // always true for a correct selection; guards the stores
                G[(size_t)expert * k + j] = __uint_as_float(v);
                I[(size_t)expert * k + j] = idx;
                topk_emit(emit, expert, k, (int)j, idx);
            }
        }
        pos += (unsigned int)__popcll(bal);
    }
}

// LDS the top-k kernel may use for the staged row.
static size_t topk_lds_budget() {
    static size_t budget = 0;
    if (budget == 0) {
        int dev = 0, v = 0;
        size_t b = 64 * 1024;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v > 0)
            b = (size_t)v;
        (void)hipGetLastError();
        const size_t reserve = sizeof(TopkShared) + 256;
        budget = b > reserve + 4096 ? b - reserve : 4096;
    }
    return budget;
}

// The selection needs no scratch in global memory.
size_t topk_ws_bytes(int64_t, int64_t, int64_t) { return 0; }

int launch_topk(const float* St, int64_t n, int64_t e, int64_t k, float* G, int32_t* I,
                unsigned long long* sortkeys_ws, int32_t* slot_cnt, int32_t* slots, int slot_cap, uint32_t* bitmap,
                hipStream_t stream) {
    (void)sortkeys_ws;
    TopkEmit emit;
    emit.slot_cnt = slot_cnt; emit.slots = slots; emit.slot_cap = slot_cap;
    emit.bitmap = bitmap; emit.bitmap_words = (int)ceil_div(e, 32);
    const size_t stage_bytes = align_up((size_t)n * 4, 16);
    const bool staged = stage_bytes <= topk_lds_budget();
    const size_t dyn = staged ? stage_bytes : 0;
    dim3 grid((unsigned)e), block(TOPK_THREADS);
    if (staged) {
        auto kern = topk_tokens_kernel<true>;
        if (dyn > 64 * 1024)
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)dyn);
        hipLaunchKernelGGL(kern, grid, block, dyn, stream, St, (int)n, (int)k, G, I, emit);
    } else {
        hipLaunchKernelGGL(topk_tokens_kernel<false>, grid, block, 0, stream, St, (int)n, (int)k, G, I, emit);
    }
    return check_launch();
}

}  // namespace ecmoe
