// G, I = TopK(S^T, k): every expert takes its k best tokens (Sec. 3.2, Eq. 2).
//
// One 1024-thread workgroup per expert works on that expert's row of S^T
// (n contiguous floats).  Scores are non-negative, so their bit patterns order
// like unsigned integers, and (score bits, ~token) is a total order in which
// "larger" means "admitted first".  Steps:
//   1. read the row once and keep it on chip -- in the registers of the workgroup (rows up to 65536
//      tokens, the kernel further down) or in LDS -- and find min and max; rows that fit neither are
//      re-read from memory in every pass;
//   2. radix-select on (bits - min), 8 bits per pass starting at the top bit of
//      the actual range, until the bin holding the k-th score has at most
//      TOPK_CAND_MAX members or all 32 bits are decided;
//   3. find the cut-off key, the k-th largest (score, ~token): among few
//      candidates by counting, among many exact ties by token order;
//   4. every wavefront owns a contiguous range of tokens: count the admitted
//      ones per range, prefix the counts, then write the bucket in ascending
//      token order with ballot ranks.  No sort is needed.
// Rows of more than 32768 scores with k <= 512 first try a threshold taken from the per-thread maxima, which
// replaces steps 2-4 by work on about 1.3 k candidates (see the register-resident kernel).
#include <atomic>

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

// ---------------------------------------------------------------------------
// Selection among at most 1024 keys held one per thread (the threshold pass of the register-resident kernel).
// ---------------------------------------------------------------------------
constexpr int TOPK_FAST_K = 512;      // largest bucket the threshold pass is tried for
constexpr int TOPK_FAST_CAND = 1024;  // candidates it may keep: one per thread

struct TopkSelectShared {
    unsigned int hist[3][256];
    unsigned long long red[2 * TOPK_WAVES];
    unsigned long long cand[TOPK_CAND_MAX];
    unsigned int above[TOPK_CAND_MAX];
    unsigned int slot;
    unsigned long long result;
};

// The kth largest (1 <= kth <= count) of `count` distinct 64-bit keys, one per thread where `valid`.  Every thread
// of the block calls it.  Radix select, 8 bits per pass from the top bit of the actual range, until at most
// TOPK_CAND_MAX keys are left; those are ranked by counting, four threads per key.
__device__ unsigned long long block_kth_largest(unsigned long long key, bool valid, unsigned int kth, unsigned int count,
                                                TopkSelectShared& s) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned long long kmin = valid ? key : ~0ull, kmax = valid ? key : 0ull;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned long long a = __shfl_xor(kmin, off, kWave), b = __shfl_xor(kmax, off, kWave);
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
    }
    if (lane == 0) { s.red[wave] = kmin; s.red[TOPK_WAVES + wave] = kmax; }
    if (tid < 768) (&s.hist[0][0])[tid] = 0u;
    if (tid < TOPK_CAND_MAX) s.above[tid] = 0u;
    if (tid == 0) s.slot = 0u;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < TOPK_WAVES; ++w) {
        const unsigned long long a = s.red[w], b = s.red[TOPK_WAVES + w];
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
    }
    const unsigned long long range = kmax - kmin;
    int lo = range == 0 ? 0 : 64 - __clzll((long long)range);
    unsigned long long prefix = 0;
    unsigned int remaining = kth, cand = count;
    int pass = 0;
    while (cand > (unsigned int)TOPK_CAND_MAX && lo > 0) {
        const int nlo = lo > 8 ? lo - 8 : 0;
        const unsigned long long base = kmin + prefix, span_m1 = lo >= 64 ? ~0ull : (1ull << lo) - 1ull;
        const unsigned long long t = key - base;
        if (valid && t <= span_m1) atomicAdd(&s.hist[pass % 3][(unsigned int)(t >> nlo)], 1u);
        __syncthreads();
        // the buffer of the pass after the next one was last scanned before this barrier
        if (tid < 256) s.hist[(pass + 2) % 3][tid] = 0u;
        const uint4 q = *reinterpret_cast<const uint4*>(&s.hist[pass % 3][4 * lane]);  // lane owns bins 4*lane .. +3
        const unsigned int h[4] = {q.x, q.y, q.z, q.w};
        const unsigned int tot = h[0] + h[1] + h[2] + h[3];
        unsigned int incl = tot;  // inclusive suffix sum over lanes >= this one
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const unsigned int o = __shfl_down(incl, off, kWave);
            if (lane + off < 64) incl += o;
        }
        const unsigned int above = incl - tot;
        const bool own = above < remaining && remaining <= incl;  // exactly one lane
        unsigned int b = 0, ab = 0, hb = 0;
        if (own) {
            const unsigned int a3 = above, a2 = a3 + h[3], a1 = a2 + h[2], a0 = a1 + h[1];
            if (remaining <= a2) { b = 3; ab = a3; hb = h[3]; }
            else if (remaining <= a1) { b = 2; ab = a2; hb = h[2]; }
            else if (remaining <= a0) { b = 1; ab = a1; hb = h[1]; }
            else { b = 0; ab = a0; hb = h[0]; }
            b += 4u * (unsigned int)lane;
        }
        const int src = __ffsll((long long)__ballot(own)) - 1;
        b = __builtin_amdgcn_readlane(b, src);
        ab = __builtin_amdgcn_readlane(ab, src);
        hb = __builtin_amdgcn_readlane(hb, src);
        prefix |= (unsigned long long)b << nlo;
        remaining -= ab;
        cand = hb;
        lo = nlo;
        ++pass;
    }
    // at most TOPK_CAND_MAX keys are left in the window (with every bit decided the keys left are equal, and keys
    // are distinct: one key)
    const unsigned long long base = kmin + prefix, span_m1 = lo >= 64 ? ~0ull : (1ull << lo) - 1ull;
    if (valid && key - base <= span_m1) {
        const unsigned int p = atomicAdd(&s.slot, 1u);
        if (p < (unsigned int)TOPK_CAND_MAX) s.cand[p] = key;
    }
    __syncthreads();
    const unsigned int c = (unsigned int)tid & (TOPK_CAND_MAX - 1), part = (unsigned int)tid / TOPK_CAND_MAX;
    if (c < cand) {
        const unsigned long long mine = s.cand[c];
        unsigned int above = 0;
        for (unsigned int j = part; j < cand; j += 4) above += s.cand[j] > mine ? 1u : 0u;
        if (above != 0u) atomicAdd(&s.above[c], above);
    }
    __syncthreads();
    if ((unsigned int)tid < cand && s.above[tid] == remaining - 1u) s.result = s.cand[tid];
    __syncthreads();
    return s.result;
}

// ---------------------------------------------------------------------------
// Register-resident variant: the whole row lives in the registers of the 1024 threads (R quads of
// four scores per thread, n <= 4096 * R <= 65536), so S^T is read exactly once and every later
// pass (radix digits, cut-off, counting, emission) runs out of registers.  Wavefront w owns the
// contiguous tokens [w * 256 R, (w + 1) * 256 R); quad r of a lane covers tokens
// w * 256 R + 256 r + 4 lane .. + 3, so a wavefront's loads are whole 1-KiB pieces of the row.
// Histograms: four copies (one per wavefront residue) in three rotating buffers, which leaves one
// barrier per radix pass; every wavefront scans the histogram itself instead of waiting for a
// broadcast.  Requires n % 4 == 0 (16-byte aligned rows).
//
// gridDim.y > 1 selects per group of tokens: the row is cut into gridDim.y equal segments of n
// tokens and every (expert, segment) pair takes its own k best; a bucket then lists its segments
// one after the other, which keeps it in ascending token order.
// ---------------------------------------------------------------------------
struct TopkRegShared {
    unsigned int hist[3][4][256];
    unsigned int red[2 * TOPK_WAVES];
    unsigned int wave_cnt[TOPK_WAVES];
    unsigned int cand_key[TOPK_CAND_MAX];  // candidates for the cut-off: key and ~token, kept as separate
    unsigned int cand_ntok[TOPK_CAND_MAX]; // 32-bit words (64-bit keys would double the register need)
    unsigned int above_cnt[TOPK_CAND_MAX]; // candidates ranked above each candidate
    unsigned int cut_key, cut_ntok;
    unsigned int slot;
};

// What the threshold pass adds: its candidates, and one bit per token of the segment with the prefix of the
// bit counts (two words per thread), from which an admitted token reads its place in the bucket.
struct TopkFastShared {
    TopkSelectShared sel;
    unsigned int key[TOPK_FAST_CAND];
    unsigned int ntok[TOPK_FAST_CAND];
    unsigned int tokbits[2 * TOPK_THREADS];
    unsigned int tokpre[TOPK_THREADS];
};

template <int R>
__global__ void __launch_bounds__(TOPK_THREADS)
topk_tokens_reg_kernel(const float* __restrict__ St, int n_total, int n, int k, float* __restrict__ G,
                       int32_t* __restrict__ I, TopkEmit emit) {
    __shared__ TopkRegShared sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int expert = blockIdx.x, tok0 = blockIdx.y * n;
    const size_t out0 = ((size_t)expert * gridDim.y + blockIdx.y) * (size_t)k;
    const unsigned int* __restrict__ colg = reinterpret_cast<const unsigned int*>(St) + (size_t)expert * n_total + tok0;
    constexpr int PER_WAVE = 256 * R;
    const int t_base = wave * PER_WAVE + 4 * lane;  // token of quad 0, element 0
    // quads r < rv are inside the row (n % 4 == 0: a quad is inside or outside as a whole)
    const int rv = t_base >= n ? 0 : ((n - t_base + 255) >> 8) < R ? ((n - t_base + 255) >> 8) : R;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;

    // ---- 1. one read of the row; min / max ----------------------------------
    unsigned int v[R][4];
    unsigned int vmin = 0xFFFFFFFFu, vmax = 0u;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        // Quads outside the row hold 0xFFFFFFFF: scores are non-negative floats (bits below 2^31), so this
        // value is never inside a radix window and, compared as a signed number, never passes the cut-off.
        uint4 q = make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu);
        if (r < rv) {
            q = *reinterpret_cast<const uint4*>(colg + t_base + 256 * r);
            vmin = min(vmin, min(min(q.x, q.y), min(q.z, q.w)));
            vmax = max(vmax, max(max(q.x, q.y), max(q.z, q.w)));
        }
        v[r][0] = q.x; v[r][1] = q.y; v[r][2] = q.z; v[r][3] = q.w;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        vmin = min(vmin, (unsigned int)__shfl_xor(vmin, off, kWave));
        vmax = max(vmax, (unsigned int)__shfl_xor(vmax, off, kWave));
    }
    if (lane == 0) { sh.red[wave] = vmin; sh.red[TOPK_WAVES + wave] = vmax; }
    (&sh.hist[0][0][0])[tid] = 0u;         // buffers 0 and 1 start clean (1024 words each)
    (&sh.hist[1][0][0])[tid] = 0u;
    if (tid == 0) sh.slot = 0u;
    if (tid < TOPK_CAND_MAX) sh.above_cnt[tid] = 0u;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < TOPK_WAVES; ++w) {
        vmin = min(vmin, sh.red[w]);
        vmax = max(vmax, sh.red[TOPK_WAVES + w]);
    }
    // block-uniform values are moved to scalar registers: fewer vector registers, scalar branches
    vmin = __builtin_amdgcn_readfirstlane(vmin);
    vmax = __builtin_amdgcn_readfirstlane(vmax);
    // ---- 1b. threshold pass (rows of more than 32768 scores, small buckets) ------
    // The k-th largest of the 1024 per-thread maxima is a lower bound T of the k-th largest score: the k maxima
    // at or above it are k scores at or above it.  So every admitted score is >= T, and on scores in no special
    // order few others are (a thread's other scores rarely reach the median of the maxima): they become the
    // candidates, one per thread, the cut-off is selected among them, and the bucket is written from them -- the
    // row in the registers is looked at once more only, by one comparison per score.  More than 1024 candidates
    // (ties at T, sorted rows): the general path below.
    if (R >= 16 && k <= TOPK_FAST_K) {  // measured: 65536 scores 49 -> 32 us; 32768 scores no gain, so not there
        __shared__ TopkFastShared fs;
        unsigned int tmax = 0u;
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (r < rv) tmax = max(tmax, max(max(v[r][0], v[r][1]), max(v[r][2], v[r][3])));
        int nvt = 0;  // threads that hold scores: lanes with 4 * lane below what is left of the row for their wavefront
#pragma unroll
        for (int w = 0; w < TOPK_WAVES; ++w) {
            const int rem = n - w * PER_WAVE;
            nvt += rem <= 0 ? 0 : (rem >= 256 ? 64 : rem >> 2);
        }
        unsigned int T = 0u;  // fewer maxima than k: everything is a candidate
        if (k <= nvt)
            T = (unsigned int)(block_kth_largest(((unsigned long long)tmax << 32) | (unsigned int)tid, rv > 0,
                                                 (unsigned int)k, (unsigned int)nvt, fs.sel) >> 32);
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if ((int)v[r][c] >= (int)T) {  // signed: the padding value 0xFFFFFFFF never passes
                    const unsigned int p = atomicAdd(&sh.slot, 1u);
                    if (p < (unsigned int)TOPK_FAST_CAND) {
                        fs.key[p] = v[r][c];
                        fs.ntok[p] = 0xFFFFFFFFu - (unsigned int)(t_base + 256 * r + c);
                    }
                }
            }
        }
        fs.tokbits[2 * tid] = 0u;
        fs.tokbits[2 * tid + 1] = 0u;
        __syncthreads();
        const unsigned int C = sh.slot;  // >= k
        if (C <= (unsigned int)TOPK_FAST_CAND) {
            const bool mine = (unsigned int)tid < C;
            const unsigned int ck = mine ? fs.key[tid] : 0u, cn = mine ? fs.ntok[tid] : 0u;
            const unsigned long long key = ((unsigned long long)ck << 32) | cn;
            const unsigned long long cut = block_kth_largest(key, mine, (unsigned int)k, C, fs.sel);
            const bool adm = mine && key >= cut;
            const unsigned int tok = 0xFFFFFFFFu - cn;  // index inside the segment
            if (adm) atomicOr(&fs.tokbits[tok >> 5], 1u << (tok & 31));
            __syncthreads();
            const unsigned int c2 = (unsigned int)__popc(fs.tokbits[2 * tid]) + (unsigned int)__popc(fs.tokbits[2 * tid + 1]);
            unsigned int incl = c2;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const unsigned int o = __shfl_up(incl, off, kWave);
                if (lane >= off) incl += o;
            }
            if (lane == 63) sh.wave_cnt[wave] = incl;
            __syncthreads();
            unsigned int before = 0;
#pragma unroll
            for (int w = 0; w < TOPK_WAVES; ++w) before += w < wave ? sh.wave_cnt[w] : 0u;
            fs.tokpre[tid] = before + incl - c2;
            __syncthreads();
            if (adm) {
                const unsigned int word = tok >> 5;
                const unsigned int j = fs.tokpre[word >> 1] + ((word & 1u) ? (unsigned int)__popc(fs.tokbits[word - 1]) : 0u) +
                                       (unsigned int)__popc(fs.tokbits[word] & ((1u << (tok & 31)) - 1u));
                if (j < (unsigned int)k) {  // always true for a correct selection; guards the stores
                    const int gtok = tok0 + (int)tok;
                    G[out0 + j] = __uint_as_float(ck);
                    I[out0 + j] = gtok;
                    if (emit.slot_cnt != nullptr) {
                        const int at = atomicAdd(&emit.slot_cnt[gtok], 1);
                        if (at < emit.slot_cap) emit.slots[(size_t)gtok * emit.slot_cap + at] = (int32_t)(out0 + j);
                    }
                    if (emit.bitmap != nullptr)
                        atomicOr(&emit.bitmap[(size_t)gtok * emit.bitmap_words + (expert >> 5)], 1u << (expert & 31));
                }
            }
            return;
        }
        if (tid == 0) sh.slot = 0u;
        __syncthreads();
    }

    // ---- 2. radix select on key = bits - vmin ---------------------------------
    const unsigned int range = vmax - vmin;
    int lo = range == 0 ? 0 : 32 - __clz(range);
    unsigned int prefix = 0, remaining = (unsigned int)k, cand = (unsigned int)n;
    int pass = 0;
    while (cand > (unsigned int)TOPK_CAND_MAX && lo > 0) {
        const int nlo = lo > 8 ? lo - 8 : 0;
        // scores whose key (bits - vmin) matches the decided prefix: bits - (vmin + prefix) < 2^lo; what is
        // left after the subtraction is the undecided part of the key, its top digit the histogram bin
        const unsigned int base = vmin + prefix, span_m1 = lo >= 32 ? 0xFFFFFFFFu : (1u << lo) - 1u;
        unsigned int* H = sh.hist[pass % 3][wave & 3];
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const unsigned int t = v[r][c] - base;
                if (t <= span_m1) atomicAdd(&H[t >> nlo], 1u);
            }
        }
        __syncthreads();
        // The buffer of the pass after the next one was last scanned before this barrier: clear it now.
        (&sh.hist[(pass + 2) % 3][0][0])[tid] = 0u;
        // Every wavefront scans for itself: lane owns bins 4*lane .. 4*lane+3.
        unsigned int h[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int cpy = 0; cpy < 4; ++cpy) {
            const uint4 q = *reinterpret_cast<const uint4*>(&sh.hist[pass % 3][cpy][4 * lane]);
            h[0] += q.x; h[1] += q.y; h[2] += q.z; h[3] += q.w;
        }
        const unsigned int tot = h[0] + h[1] + h[2] + h[3];
        unsigned int incl = tot;  // inclusive suffix sum over lanes >= this one
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const unsigned int o = __shfl_down(incl, off, kWave);
            if (lane + off < 64) incl += o;
        }
        const unsigned int above = incl - tot;
        const bool own = above < remaining && remaining <= incl;  // exactly one lane
        unsigned int b = 0, ab = 0, hb = 0;
        if (own) {
            const unsigned int a3 = above, a2 = a3 + h[3], a1 = a2 + h[2], a0 = a1 + h[1];
            if (remaining <= a2) { b = 3; ab = a3; hb = h[3]; }
            else if (remaining <= a1) { b = 2; ab = a2; hb = h[2]; }
            else if (remaining <= a0) { b = 1; ab = a1; hb = h[1]; }
            else { b = 0; ab = a0; hb = h[0]; }
            b += 4u * (unsigned int)lane;
        }
        const int src = __ffsll((long long)__ballot(own)) - 1;
        b = __builtin_amdgcn_readlane(b, src);
        ab = __builtin_amdgcn_readlane(ab, src);
        hb = __builtin_amdgcn_readlane(hb, src);
        prefix |= b << nlo;
        remaining -= ab;
        cand = hb;
        lo = nlo;
        ++pass;
    }
    const unsigned int base = vmin + prefix, span_m1 = lo >= 32 ? 0xFFFFFFFFu : (1u << lo) - 1u;

    // ---- 3. the cut-off key ----------------------------------------------------
    if (cand <= (unsigned int)TOPK_CAND_MAX) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (v[r][c] - base <= span_m1) {
                    const unsigned int p = atomicAdd(&sh.slot, 1u);
                    if (p < (unsigned int)TOPK_CAND_MAX) {
                        sh.cand_key[p] = v[r][c];
                        sh.cand_ntok[p] = 0xFFFFFFFFu - (unsigned int)(t_base + 256 * r + c);
                    }
                }
            }
        }
        __syncthreads();
        // the candidate with exactly remaining-1 candidates above it is the cut-off; four threads share
        // the count of one candidate
        static_assert(TOPK_THREADS == 4 * TOPK_CAND_MAX, "four threads per candidate");
        const unsigned int c = (unsigned int)tid & (TOPK_CAND_MAX - 1), part = (unsigned int)tid / TOPK_CAND_MAX;
        if (c < cand) {
            const unsigned int mhi = sh.cand_key[c], mlo = sh.cand_ntok[c];
            unsigned int above = 0;
            for (unsigned int j = part; j < cand; j += 4) {
                const unsigned int ohi = sh.cand_key[j], olo = sh.cand_ntok[j];
                above += (ohi > mhi) | ((ohi == mhi) & (olo > mlo));
            }
            if (above != 0u) atomicAdd(&sh.above_cnt[c], above);
        }
        __syncthreads();
        if (tid < (int)cand && sh.above_cnt[tid] == remaining - 1u) {
            sh.cut_key = sh.cand_key[tid];
            sh.cut_ntok = sh.cand_ntok[tid];
        }
    } else {
        // Exact ties at the threshold score: the cut-off is the `remaining`-th tied token in token order.
        const unsigned int tbits = base;  // every bit of the threshold score is decided
        unsigned int ties = 0;
#pragma unroll
        for (int r = 0; r < R; ++r)
            ties += (v[r][0] == tbits) + (v[r][1] == tbits) + (v[r][2] == tbits) + (v[r][3] == tbits);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) ties += __shfl_xor(ties, off, kWave);
        if (lane == 0) sh.wave_cnt[wave] = ties;
        __syncthreads();
        unsigned int before = 0;
#pragma unroll
        for (int w = 0; w < TOPK_WAVES; ++w) before += w < wave ? sh.wave_cnt[w] : 0u;
        if (before < remaining && remaining <= before + ties) {  // this wavefront holds the cut-off token
            unsigned int seen = before;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                unsigned int pre = 0, tot = 0;
                bool eq[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    eq[c] = v[r][c] == tbits;
                    const unsigned long long bal = __ballot(eq[c]);
                    pre += (unsigned int)__popcll(bal & lt_mask);
                    tot += (unsigned int)__popcll(bal);
                }
                // token order inside a quad row: lane-major, then element
                unsigned int rank = seen + pre;
                // lanes below contribute all four of their elements before this lane's first one
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (eq[c] && rank == remaining - 1u) {
                        sh.cut_key = tbits;
                        sh.cut_ntok = 0xFFFFFFFFu - (unsigned int)(t_base + 256 * r + c);
                    }
                    rank += eq[c] ? 1u : 0u;
                }
                seen += tot;
            }
        }
        __syncthreads();  // wave_cnt is reused below
    }
    __syncthreads();
    const unsigned int chi = __builtin_amdgcn_readfirstlane(sh.cut_key);
    const int cut_tok = (int)(0xFFFFFFFFu - (unsigned int)__builtin_amdgcn_readfirstlane(sh.cut_ntok));
    // score above the cut-off score, or equal to it with a token index up to the cut-off token; `ofs` is the
    // compile-time offset of the element from the lane's first token, so the comparison needs no index register
    auto admitted = [&](unsigned int key, int ofs) -> bool {
        return ((int)key > (int)chi) | ((key == chi) & (t_base <= cut_tok - ofs));
    };

    // ---- 4. count per wavefront, prefix, emit in token order ---------------------
    unsigned int mine_cnt = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int c = 0; c < 4; ++c) mine_cnt += admitted(v[r][c], 256 * r + c) ? 1u : 0u;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mine_cnt += __shfl_xor(mine_cnt, off, kWave);
    if (lane == 0) sh.wave_cnt[wave] = mine_cnt;
    __syncthreads();
    unsigned int pos = 0;
#pragma unroll
    for (int w = 0; w < TOPK_WAVES; ++w) pos += w < wave ? sh.wave_cnt[w] : 0u;
    if (mine_cnt == 0u) return;  // uniform per wavefront; no barrier follows

#pragma unroll
    for (int r = 0; r < R; ++r) {
        bool sel[4];
        unsigned int pre = 0, tot = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            sel[c] = admitted(v[r][c], 256 * r + c);
            const unsigned long long bal = __ballot(sel[c]);
            pre += (unsigned int)__popcll(bal & lt_mask);
            tot += (unsigned int)__popcll(bal);
        }
        if (tot != 0u) {  // uniform
            const int tok_q = tok0 + t_base + 256 * r;
            int slot_at[4] = {0, 0, 0, 0};
            if (emit.slot_cnt != nullptr) {  // the four atomics are in flight together; their results feed the stores below
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (sel[c]) slot_at[c] = atomicAdd(&emit.slot_cnt[tok_q + c], 1);
            }
            unsigned int j = pos + pre;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (sel[c] && j < (unsigned int)k) {  // j < k always holds for a correct selection; guards the stores
                    G[out0 + j] = __uint_as_float(v[r][c]);
                    I[out0 + j] = tok_q + c;
                    if (emit.slot_cnt != nullptr && slot_at[c] < emit.slot_cap)
                        emit.slots[(size_t)(tok_q + c) * emit.slot_cap + slot_at[c]] = (int32_t)(out0 + j);
                    if (emit.bitmap != nullptr)
                        atomicOr(&emit.bitmap[(size_t)(tok_q + c) * emit.bitmap_words + (expert >> 5)], 1u << (expert & 31));
                }
                j += sel[c] ? 1u : 0u;
            }
        }
        pos += tot;
    }
}

// ---------------------------------------------------------------------------
// Small segments (at most 256 tokens, a multiple of 4): one wavefront per (expert, segment), four scores
// per lane, no LDS and no barrier -- the batched small selection that routing per group of tokens needs
// when the groups are short (Limitations section: small batches at serving time).  The k-th largest
// score is found bit by bit (31 counting steps with ballots: scores are non-negative floats), ties at
// that score are admitted in token order, and the bucket is written in ascending token order.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
topk_small_kernel(const float* __restrict__ St, int n_total, int n, int k, int e, int groups,
                  float* __restrict__ G, int32_t* __restrict__ I, TopkEmit emit) {
    const int lane = threadIdx.x & 63;
    const long long job = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);  // (expert, segment), segment fastest
    if (job >= (long long)e * groups) return;                              // uniform per wavefront
    const int expert = (int)(job / groups), group = (int)(job % groups);
    const int tok0 = group * n;
    const size_t out0 = (size_t)job * (size_t)k;
    const unsigned int* __restrict__ colg = reinterpret_cast<const unsigned int*>(St) + (size_t)expert * n_total + tok0;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const bool valid = 4 * lane < n;  // n % 4 == 0: a lane's quad is inside or outside as a whole
    unsigned int v[4] = {0u, 0u, 0u, 0u};
    if (valid) {
        const uint4 q = *reinterpret_cast<const uint4*>(colg + 4 * lane);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
    auto count_ge = [&](unsigned int t) -> int {
        int c = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) c += __popcll(__ballot(valid && v[j] >= t));
        return c;
    };
    // largest T with at least k scores >= T: the k-th largest score
    unsigned int T = 0u;
    for (int bit = 30; bit >= 0; --bit) {
        const unsigned int cand = T | (1u << bit);
        if (count_ge(cand) >= k) T = cand;
    }
    int above = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) above += __popcll(__ballot(valid && v[j] > T));
    const int need = k - above;  // ties at T to admit, lowest token indices first
    // rank among the ties and position in the bucket, both in token order (lane-major, then element)
    unsigned long long tie_bal[4];
    int tie_before = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        tie_bal[j] = __ballot(valid && v[j] == T);
        tie_before += __popcll(tie_bal[j] & lt_mask);
    }
    bool sel[4];
    int tr = tie_before;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool tie = valid && v[j] == T;
        sel[j] = valid && (v[j] > T || (tie && tr < need));
        tr += tie ? 1 : 0;
    }
    int pos = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) pos += __popcll(__ballot(sel[j]) & lt_mask);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (sel[j] && pos < k) {  // pos < k always holds for a correct selection; guards the stores
            const int tok = tok0 + 4 * lane + j;
            G[out0 + pos] = __uint_as_float(v[j]);
            I[out0 + pos] = tok;
            if (emit.slot_cnt != nullptr) {
                const int s = atomicAdd(&emit.slot_cnt[tok], 1);
                if (s < emit.slot_cap) emit.slots[(size_t)tok * emit.slot_cap + s] = (int32_t)(out0 + pos);
            }
            if (emit.bitmap != nullptr)
                atomicOr(&emit.bitmap[(size_t)tok * emit.bitmap_words + (expert >> 5)], 1u << (expert & 31));
        }
        pos += sel[j] ? 1 : 0;
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

template <int R>
static void launch_topk_reg(const float* St, int n_total, int n_seg, int k, int e, int groups, float* G, int32_t* I,
                            const TopkEmit& emit, hipStream_t stream) {
    hipLaunchKernelGGL(topk_tokens_reg_kernel<R>, dim3((unsigned)e, (unsigned)groups), dim3(TOPK_THREADS), 0, stream, St,
                       n_total, n_seg, k, G, I, emit);
}

// n tokens in all, cut into `groups` equal segments; k is the bucket size per (expert, segment).
int launch_topk(const float* St, int64_t n, int64_t e, int64_t k, float* G, int32_t* I,
                int32_t* slot_cnt, int32_t* slots, int slot_cap, uint32_t* bitmap, hipStream_t stream, int64_t groups) {
    TopkEmit emit;
    emit.slot_cnt = slot_cnt; emit.slots = slots; emit.slot_cap = slot_cap;
    emit.bitmap = bitmap; emit.bitmap_words = (int)ceil_div(e, 32);
    const int64_t seg = n / groups;
    if ((seg & 3) == 0 && seg <= 256 && e * groups >= 64) {
        // many short segments: a wavefront each
        const long long jobs = (long long)e * groups;
        hipLaunchKernelGGL(topk_small_kernel, dim3((unsigned)((jobs + 3) / 4)), dim3(256), 0, stream, St, (int)n, (int)seg,
                           (int)k, (int)e, (int)groups, G, I, emit);
        return check_launch();
    }
    if ((seg & 3) == 0 && seg <= 65536 && groups <= 65535) {
        // the row (segment) fits the registers of one workgroup: S^T is read once
        const int ni = (int)n, si = (int)seg, ki = (int)k, ei = (int)e, gi = (int)groups;
        if (seg <= 4096) launch_topk_reg<1>(St, ni, si, ki, ei, gi, G, I, emit, stream);
        else if (seg <= 8192) launch_topk_reg<2>(St, ni, si, ki, ei, gi, G, I, emit, stream);
        else if (seg <= 16384) launch_topk_reg<4>(St, ni, si, ki, ei, gi, G, I, emit, stream);
        else if (seg <= 32768) launch_topk_reg<8>(St, ni, si, ki, ei, gi, G, I, emit, stream);
        else launch_topk_reg<16>(St, ni, si, ki, ei, gi, G, I, emit, stream);
        return check_launch();
    }
    if (groups != 1) return EC_ERR_UNSUPPORTED;  // segments must be multiples of 4 tokens, at most 65536 long
    const size_t stage_bytes = align_up((size_t)n * 4, 16);
    const bool staged = stage_bytes <= topk_lds_budget();
    const size_t dyn = staged ? stage_bytes : 0;
    dim3 grid((unsigned)e), block(TOPK_THREADS);
    if (staged) {
        auto kern = topk_tokens_kernel<true>;
        if (dyn > 64 * 1024) {
            // the limit is raised once per GPU, to the whole budget, so later launches of any size are covered
            static std::atomic<bool> raised[64];
            int dev = 0;
            if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
            if (!raised[dev].load(std::memory_order_acquire)) {
                (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                          (int)topk_lds_budget());
                raised[dev].store(true, std::memory_order_release);
            }
        }
        hipLaunchKernelGGL(kern, grid, block, dyn, stream, St, (int)n, (int)k, G, I, emit);
    } else {
        hipLaunchKernelGGL(topk_tokens_kernel<false>, grid, block, 0, stream, St, (int)n, (int)k, G, I, emit);
    }
    return check_launch();
}

}  // namespace ecmoe
