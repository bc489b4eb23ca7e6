// Token-choice routing, the conventional baseline of Sec. 3.1: every token independently takes its
// top-m experts (m = 1: Switch Transformer, m = 2: GShard; Sec. 3.4), an expert's buffer holds at
// most `cap` tokens and what is routed to it beyond that is dropped.  Placement order: all first
// choices before any second choice, ascending token index inside one rank of choice; ties between
// experts go to the lower expert index; gate weight = the raw score.  Empty buffer rows get
// I = -1, G = 0.  The buffers have the [e, cap] shape of expert choice's buckets, so Eq. 3-4 run on
// the same dispatch / expert / combine kernels.
//
// Two kernels:
//  * tc_choices_kernel: one wavefront per token finds the m best experts of the token's row of S
//    by repeated maximum of the key (score bits, ~expert) and stores them rank-major, choice[r][l].
//  * tc_place_kernel: one workgroup per expert.  Every wavefront owns a contiguous range of tokens;
//    per rank it counts the tokens that chose this expert, a prefix over (rank, wavefront) gives
//    every range its first buffer row, and ballot ranks inside a wavefront keep token order.
//    No sort and no floating-point atomics.
#include "ec_common.h"

namespace ecmoe {

constexpr int TC_MAX_M = 8;
constexpr int TC_THREADS = 1024;
constexpr int TC_WAVES = TC_THREADS / kWave;

__global__ void __launch_bounds__(256)
tc_choices_kernel(const float* __restrict__ S, int n, int e, int m, int32_t* __restrict__ choice) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned int* __restrict__ Su = reinterpret_cast<const unsigned int*>(S);
    for (int l = blockIdx.x * 4 + wave; l < n; l += gridDim.x * 4) {
        const unsigned int* row = Su + (size_t)l * e;
        int taken[TC_MAX_M];
#pragma unroll
        for (int r = 0; r < TC_MAX_M; ++r) taken[r] = -1;
#pragma unroll
        for (int r = 0; r < TC_MAX_M; ++r) {
            if (r < m) {
                // key = (score bits, ~expert): the maximum is the largest score, the lowest expert among equals;
                // 0 stands for "nothing" (a real key has a non-zero low word because expert < 2^32 - 1)
                unsigned int bhi = 0u, blo = 0u;
                for (int i = lane; i < e; i += kWave) {
                    bool free_ = true;
#pragma unroll
                    for (int q = 0; q < TC_MAX_M; ++q) free_ = free_ && taken[q] != i;
                    const unsigned int hi = row[i], lo = 0xFFFFFFFFu - (unsigned int)i;
                    if (free_ && (hi > bhi || (hi == bhi && lo > blo))) { bhi = hi; blo = lo; }
                }
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) {
                    const unsigned int ohi = __shfl_xor(bhi, off, kWave), olo = __shfl_xor(blo, off, kWave);
                    if (ohi > bhi || (ohi == bhi && olo > blo)) { bhi = ohi; blo = olo; }
                }
                const int best = (int)(0xFFFFFFFFu - blo);
                taken[r] = best;
                if (lane == 0) choice[(size_t)r * n + l] = best;
            }
        }
    }
}

struct TcEmit {          // token-major by-products for the combine stage (see the top-k kernel)
    int32_t* slot_cnt;
    int32_t* slots;
    int slot_cap;
    uint32_t* bitmap;
    int bitmap_words;
};

__global__ void __launch_bounds__(TC_THREADS)
tc_place_kernel(const float* __restrict__ S, const int32_t* __restrict__ choice, int n, int e, int m, int cap,
                float* __restrict__ G, int32_t* __restrict__ I, int32_t* __restrict__ load, TcEmit emit) {
    __shared__ unsigned int cnt[TC_MAX_M][TC_WAVES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int expert = blockIdx.x;
    const int per_wave = ((n + TC_WAVES - 1) / TC_WAVES + kWave - 1) / kWave * kWave;
    const int w_beg = wave * per_wave;
    const int w_end = (w_beg + per_wave) < n ? (w_beg + per_wave) : n;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;

    for (int r = 0; r < m; ++r) {
        const int32_t* ch = choice + (size_t)r * n;
        unsigned int c = 0;
        for (int base = w_beg; base < w_end; base += kWave) {
            const int l = base + lane;
            c += (unsigned int)__popcll(__ballot(l < w_end && ch[l] == expert));
        }
        if (lane == 0) cnt[r][wave] = c;
    }
    __syncthreads();
    unsigned int total = 0;
    for (int r = 0; r < m; ++r) {
        unsigned int before = total;  // rows taken by the earlier ranks
        unsigned int rank_total = 0;
        for (int w = 0; w < TC_WAVES; ++w) {
            const unsigned int c = cnt[r][w];
            before += w < wave ? c : 0u;
            rank_total += c;
        }
        total += rank_total;
        // this wavefront's tokens of rank r start at buffer row `before`
        if (before < (unsigned int)cap) {  // uniform per wavefront: nothing of this range fits otherwise
            const int32_t* ch = choice + (size_t)r * n;
            unsigned int pos = before;
            for (int base = w_beg; base < w_end && pos < (unsigned int)cap; base += kWave) {
                const int l = base + lane;
                const bool sel = l < w_end && ch[l] == expert;
                const unsigned long long bal = __ballot(sel);
                const unsigned int j = pos + (unsigned int)__popcll(bal & lt_mask);
                if (sel && j < (unsigned int)cap) {
                    const size_t row = (size_t)expert * cap + j;
                    I[row] = l;
                    G[row] = S[(size_t)l * e + expert];
                    if (emit.slot_cnt != nullptr) {
                        const int s = atomicAdd(&emit.slot_cnt[l], 1);
                        if (s < emit.slot_cap) emit.slots[(size_t)l * emit.slot_cap + s] = (int32_t)row;
                    }
                    if (emit.bitmap != nullptr)
                        atomicOr(&emit.bitmap[(size_t)l * emit.bitmap_words + (expert >> 5)], 1u << (expert & 31));
                }
                pos += (unsigned int)__popcll(bal);
            }
        }
    }
    // rows nobody took, and the load before dropping
    for (unsigned int j = total + tid; j < (unsigned int)cap; j += TC_THREADS) {
        I[(size_t)expert * cap + j] = -1;
        G[(size_t)expert * cap + j] = 0.0f;
    }
    if (tid == 0 && load != nullptr) load[expert] = (int32_t)total;
}

int launch_token_choice(const float* S, int64_t n, int64_t e, int64_t m, int64_t cap, float* G, int32_t* I,
                        int32_t* load, int32_t* choice_ws, int32_t* slot_cnt, int32_t* slots, int slot_cap,
                        uint32_t* bitmap, hipStream_t stream) {
    long long blocks = ceil_div(n, 4);
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(tc_choices_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, S, (int)n, (int)e, (int)m,
                       choice_ws);
    int rc = check_launch();
    if (rc != EC_OK) return rc;
    TcEmit emit;
    emit.slot_cnt = slot_cnt; emit.slots = slots; emit.slot_cap = slot_cap;
    emit.bitmap = bitmap; emit.bitmap_words = (int)ceil_div(e, 32);
    hipLaunchKernelGGL(tc_place_kernel, dim3((unsigned)e), dim3(TC_THREADS), 0, stream, S, choice_ws, (int)n, (int)e,
                       (int)m, (int)cap, G, I, load, emit);
    return check_launch();
}

}  // namespace ecmoe
