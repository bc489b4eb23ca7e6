// G, I = TopK(S^T, k): every expert takes its k best tokens (Sec. 3.2, Eq. 2).
//
// One 1024-thread workgroup per expert works on that expert's row of S^T
// (n contiguous floats).  Scores are non-negative, so their bit patterns order
// like unsigned integers.  Steps:
//   1. stage the row in LDS when it fits (one HBM read), find min and max;
//   2. radix-select on (bits - min), 8 bits per pass starting at the top bit of
//      the actual range, until the bin holding the k-th score has at most
//      TOPK_CAND_MAX members (usually one or two passes);
//   3. compact the surely selected scores and the candidates into 64-bit keys
//      (score bits << 32 | ~token), wavefront-aggregated slot allocation;
//      if all bits are used up and too many candidates remain they are exact
//      ties: admit them in token order with ballot prefix ranks instead;
//   4. bitonic sort of the keys, descending: score descending, then token
//      ascending -- the order the interface promises -- and write the first k.
#include "ec_common.h"

namespace ecmoe {

constexpr int TOPK_THREADS = 1024;
constexpr int TOPK_WAVES = TOPK_THREADS / kWave;
constexpr int TOPK_CAND_MAX = 1024;

__host__ __device__ inline int64_t topk_next_pow2(int64_t v) {
    int64_t p = 1;
    while (p < v) p <<= 1;
    return p;
}

// Capacity (in keys) of the sort buffer for bucket size k over n tokens.
__host__ __device__ inline int64_t topk_key_capacity(int64_t n, int64_t k) {
    int64_t m = k + TOPK_CAND_MAX;
    if (m > n) m = n;  // never more keys than tokens
    if (m < 2) m = 2;
    return topk_next_pow2(m);
}

struct TopkShared {
    unsigned int hist[256];
    unsigned int red[2 * TOPK_WAVES];
    unsigned int wave_cnt[TOPK_WAVES];
    unsigned int bin, remaining, cand, slot;
};

template <bool STAGED, bool KEYS_LDS>
__global__ void __launch_bounds__(TOPK_THREADS)
topk_tokens_kernel(const float* __restrict__ St, int n, int k, int kcap, float* __restrict__ G,
                   int32_t* __restrict__ I, unsigned long long* __restrict__ keys_ws, int stage_words) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ TopkShared sh;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int expert = blockIdx.x;
    const unsigned int* __restrict__ colg = reinterpret_cast<const unsigned int*>(St) + (size_t)expert * n;
    unsigned int* cols = reinterpret_cast<unsigned int*>(smem);
    unsigned long long* keys = KEYS_LDS
        ? reinterpret_cast<unsigned long long*>(smem + (STAGED ? (size_t)stage_words * 4 : 0))
        : keys_ws + (size_t)expert * kcap;

    // ---- 1. stage + min/max ------------------------------------------------
    unsigned int vmin = 0xFFFFFFFFu, vmax = 0u;
    for (int idx = tid; idx < n; idx += TOPK_THREADS) {
        unsigned int v = colg[idx];
        if (STAGED) cols[idx] = v;
        vmin = v < vmin ? v : vmin;
        vmax = v > vmax ? v : vmax;
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
        for (int idx = tid; idx < n; idx += TOPK_THREADS) {
            unsigned int key = ld(idx) - vmin;
            if ((key & hmask) == prefix) atomicAdd(&sh.hist[(key >> nlo) & dmask], 1u);
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
                sh.cand = hb;
            }
        }
        __syncthreads();
        prefix |= sh.bin << nlo;
        remaining = sh.remaining;
        cand = sh.cand;
        lo = nlo;
        __syncthreads();
    }
    const unsigned int hmask = lo >= 32 ? 0u : ~((1u << lo) - 1u);
    const unsigned int n_sure = (unsigned int)k - remaining;  // scores strictly above the candidate bin
    const bool take_all_cand = (unsigned long long)n_sure + cand <= (unsigned long long)kcap;

    // ---- 3. compaction into keys ------------------------------------------
    if (tid == 0) sh.slot = 0;
    __syncthreads();
    const int n_round = (n + TOPK_THREADS - 1) / TOPK_THREADS * TOPK_THREADS;
    for (int idx = tid; idx < n_round; idx += TOPK_THREADS) {
        bool sel = false;
        unsigned int v = 0;
        if (idx < n) {
            v = ld(idx);
            unsigned int hk = (v - vmin) & hmask;
            sel = hk > prefix || (take_all_cand && hk == prefix);
        }
        unsigned long long bal = __ballot(sel);
        unsigned int base = 0;
        if (bal != 0ull) {
            if (lane == 0) base = atomicAdd(&sh.slot, (unsigned int)__popcll(bal));
            base = __shfl(base, 0, kWave);
        }
        if (sel) {
            unsigned int slot = base + __popcll(bal & ((1ull << lane) - 1ull));
            keys[slot] = ((unsigned long long)v << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned int)idx);
        }
    }
    __syncthreads();
    unsigned int m = sh.slot;  // keys written so far
    if (!take_all_cand) {
        // Exact ties at the threshold (all 32 bits equal): admit the first `remaining` in token order.
        unsigned int running = 0;
        for (int idx0 = 0; idx0 < n && running < remaining; idx0 += TOPK_THREADS) {
            int idx = idx0 + tid;
            bool eq = idx < n && ((ld(idx) - vmin) == prefix);
            unsigned long long bal = __ballot(eq);
            if (lane == 0) sh.wave_cnt[wave] = (unsigned int)__popcll(bal);
            __syncthreads();
            unsigned int before = 0, total = 0;
#pragma unroll
            for (int w = 0; w < TOPK_WAVES; ++w) {
                unsigned int c = sh.wave_cnt[w];
                before += w < wave ? c : 0u;
                total += c;
            }
            unsigned int rank = running + before + (unsigned int)__popcll(bal & ((1ull << lane) - 1ull));
            if (eq && rank < remaining)
                keys[n_sure + rank] = ((unsigned long long)(prefix + vmin) << 32) |
                                      (unsigned long long)(0xFFFFFFFFu - (unsigned int)idx);
            running += total;
            __syncthreads();
        }
        m = (unsigned int)k;
    }

    // ---- 4. bitonic sort, descending --------------------------------------
    unsigned int mp = 2;
    while (mp < m) mp <<= 1;
    for (unsigned int idx = m + tid; idx < mp; idx += TOPK_THREADS) keys[idx] = 0ull;  // below every real key
    __syncthreads();
    for (unsigned int size = 2; size <= mp; size <<= 1) {
        for (unsigned int stride = size >> 1; stride > 0; stride >>= 1) {
            for (unsigned int p = tid; p < (mp >> 1); p += TOPK_THREADS) {
                unsigned int lo_i = 2 * p - (p & (stride - 1));  // index with the `stride` bit clear
                unsigned int hi_i = lo_i + stride;
                bool desc = (lo_i & size) == 0;
                unsigned long long a = keys[lo_i], b = keys[hi_i];
                if ((a < b) == desc) { keys[lo_i] = b; keys[hi_i] = a; }
            }
            if (!KEYS_LDS) __threadfence_block();
            __syncthreads();
        }
    }
    for (int j = tid; j < k; j += TOPK_THREADS) {
        unsigned long long key = keys[j];
        G[(size_t)expert * k + j] = __uint_as_float((unsigned int)(key >> 32));
        I[(size_t)expert * k + j] = (int32_t)(0xFFFFFFFFu - (unsigned int)(key & 0xFFFFFFFFull));
    }
}

// LDS the top-k kernel may use for the staged row plus the keys.
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

// Sort keys that do not fit in LDS live in the workspace: bytes for all experts (0 when LDS suffices).
size_t topk_ws_bytes(int64_t n, int64_t e, int64_t k) {
    // Sized for the smallest LDS any supported device offers (64 KiB) so that the
    // workspace size does not depend on the device that later runs the call.
    int64_t kcap = topk_key_capacity(n, k);
    if ((size_t)kcap * 8 <= 48 * 1024) return 0;
    return (size_t)e * (size_t)kcap * 8;
}

int launch_topk(const float* St, int64_t n, int64_t e, int64_t k, float* G, int32_t* I,
                unsigned long long* sortkeys_ws, hipStream_t stream) {
    const int64_t kcap = topk_key_capacity(n, k);
    const size_t budget = topk_lds_budget();
    const size_t key_bytes = (size_t)kcap * 8;
    const bool keys_lds = key_bytes <= 48 * 1024;  // same rule as topk_ws_bytes
    const size_t stage_bytes = align_up((size_t)n * 4, 16);
    const bool staged = stage_bytes + (keys_lds ? key_bytes : 0) <= budget;
    size_t dyn = (staged ? stage_bytes : 0) + (keys_lds ? key_bytes : 0);
    if (!keys_lds && sortkeys_ws == nullptr) return EC_ERR_WORKSPACE;
    dim3 grid((unsigned)e), block(TOPK_THREADS);
#define EC_TOPK_LAUNCH(ST, KL)                                                                             \
    do {                                                                                                   \
        auto kern = topk_tokens_kernel<ST, KL>;                                                            \
        if (dyn > 64 * 1024)                                                                               \
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                 \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);               \
        hipLaunchKernelGGL(kern, grid, block, dyn, stream, St, (int)n, (int)k, (int)kcap, G, I,            \
                           sortkeys_ws, (int)(stage_bytes / 4));                                           \
    } while (0)
    if (staged && keys_lds) EC_TOPK_LAUNCH(true, true);
    else if (staged) EC_TOPK_LAUNCH(true, false);
    else if (keys_lds) EC_TOPK_LAUNCH(false, true);
    else EC_TOPK_LAUNCH(false, false);
#undef EC_TOPK_LAUNCH
    return check_launch();
}

}  // namespace ecmoe
