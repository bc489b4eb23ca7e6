// Grouped bf16 GEMM on the matrix cores, shared by the forward expert FFN and the backward pass:
//   C[g] = epilogue( opA(A[g]) . opB(B[g]) ),   M x K times K x N, fp32 accumulation,
// one launch for all groups g (experts).
//
// Operand storage (template flags):
//   A_MC = false  A[g] is [M][K]  (contraction-contiguous rows)
//   A_MC = true   A[g] is [K][M]  (the transposed operand of a weight-gradient product)
//   B_KC = false  B[g] is [K][N]  (row-major weights, as in X.W)
//   B_KC = true   B[g] is [N][K]  (the transposed operand of X.W^T)
// A contraction-contiguous tile sits in LDS as [rows][64 + 8] and fragments are 16-byte reads.
// The other kind keeps the matrix's own [k][columns] form in LDS ([64][columns + 32], 64 bytes of
// padding put four consecutive rows in four bank groups) and fragments come from two transposing
// LDS reads (ds_read_b64_tr_b16): in a 16-lane group, lane L points at row kbase + L/4, columns
// base + 4*(L%4)..+3 and receives rows kbase..kbase+3 of column base + L.
//
// Tiling: BM x BN block tile, 4 wavefronts in a 2 x 2 arrangement, each (BM/2) x (BN/2) as TM x TN
// tiles of v_mfma_f32_32x32x16_bf16; K in stages of 64 through one or two LDS stages; global loads
// are raw buffer loads (the range check returns zeros past the end of a group's matrix, so ragged
// M and N need no branches: such rows/columns only feed outputs that are never stored).
// The N-side operand feeds the MFMA "A" port and the M-side operand the "B" port, so an accumulator
// quad holds four consecutive output columns of one row; the epilogue stages 32-row strips through
// LDS and stores full 16-byte vectors.
#pragma once

#include <atomic>

#include "ec_common.h"

namespace ecmoe {

constexpr int GEMM_BK = 64;                   // contraction elements per LDS stage
constexpr int GEMM_LDS_STRIDE = GEMM_BK + 8;  // bf16 elements per LDS row of a contraction-contiguous tile

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

enum GemmEpilogue {
    EPI_ACT = 0,       // C (bf16) = act(acc); optionally C3 (bf16) = act(acc) - C, what the rounding of C dropped
    EPI_ACT_SAVE = 1,  // additionally C2 (bf16) = acc
    EPI_MULGRAD = 2,   // C (bf16) = v = acc * act'(C2[m][n]) [* row_scale[m]],  C2 = bf16 pre-activations (read);
                       // optionally C3 (bf16) = v - C, the part of v that the rounding of C dropped
    EPI_F32 = 3,       // C (fp32) = acc; optionally C3 (bf16) = acc rounded
    EPI_SOFTMAX = 4    // one group, N <= BN: C (fp32, [N][M]) = softmax over n of acc[m][:], transposed;
                       // C2 (fp32, [M][N], optional) the same untransposed.  `gather` is not used for
                       // loads here: it names `gather_rows` 32-bit words that the launch sets to zero.
};

// GeLU with the exact-erf definition a * Phi(a); erfc by the Abramowitz-Stegun rational form 7.1.26
// (|error| < 1.5e-7).  Used where the result is rounded to bf16 anyway, so the hardware reciprocal
// and exp2 (1 ulp each) replace the IEEE division and the library exp.  Constants are folded:
//   x = |a| / sqrt 2,  t = 1 / (1 + p x),  0.5 erfc(x) = t (c1 + t (c2 + ...)) exp(-x^2) with c_i halved.
__device__ __forceinline__ float phi_tail_fast(float a, float* gauss) {  // returns 0.5*erfc(|a|/sqrt 2)
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752440f, fabsf(a), 1.0f));
    float p = fmaf(t, 0.5f * 1.061405429f, 0.5f * -1.453152027f);
    p = fmaf(t, p, 0.5f * 1.421413741f);
    p = fmaf(t, p, 0.5f * -0.284496736f);
    p = fmaf(t, p, 0.5f * 0.254829592f);
    const float g = __builtin_amdgcn_exp2f((a * a) * (-0.5f * 1.44269504088896340736f));  // exp(-a^2/2)
    *gauss = g;
    return (p * t) * g;
}
// a Phi(a) = max(a, 0) - |a| * (0.5 erfc(|a| / sqrt 2)): no cancellation in either tail, no select.
__device__ __forceinline__ float gelu_erf_fast(float a) {
    float g;
    const float tail = phi_tail_fast(a, &g);
    return fmaf(-fabsf(a), tail, fmaxf(a, 0.0f));
}
// d/da of a * Phi(a) = Phi(a) + a * phi(a), phi the standard normal density.
__device__ __forceinline__ float gelu_grad_fast(float a) {
    float g;
    const float tail = phi_tail_fast(a, &g);
    const float Phi = a >= 0.0f ? 1.0f - tail : tail;
    return fmaf(a * 0.39894228040143267794f, g, Phi);
}

template <int ACT>
__device__ __forceinline__ float apply_act_bf16(float a) {
    if (ACT == EC_ACT_GELU) return gelu_erf_fast(a);
    return apply_act<ACT>(a);
}
template <int ACT>
__device__ __forceinline__ float apply_act_grad_bf16(float a) {
    if (ACT == EC_ACT_GELU) return gelu_grad_fast(a);
    if (ACT == EC_ACT_RELU) return a > 0.0f ? 1.0f : 0.0f;
    return 1.0f;
}

// SPLIT: one operand is the sum of two bf16 matrices (a value carried as high part + remainder), the second part
// given as `X2all`: the contraction takes 64 steps of k with the first part, then the same 64 steps with the second,
// against the same piece of the other operand, so the product sees that operand to 2^-17 at twice the work.
//   SPLIT_LEFT   the left operand, contraction-contiguous (A_MC = false): A[g] + X2[g]
//   SPLIT_RIGHT  the right operand in its [K][N] form (B_KC = false):     B[g] + X2[g]
enum GemmSplit { SPLIT_NONE = 0, SPLIT_LEFT = 1, SPLIT_RIGHT = 2 };

template <int BM, int BN, int STAGES, int OCC, bool A_MC, bool B_KC, int EPI, int ACT, int SPLIT = SPLIT_NONE>
__global__ void __launch_bounds__(256, OCC)
gemm_bf16_kernel(const bf16_t* __restrict__ Aall, const bf16_t* __restrict__ Ball, void* __restrict__ Call,
                 void* __restrict__ C2all, int M, int N, int K, int G, int tiles_m, int tiles_n,
                 const int32_t* __restrict__ gather, int gather_rows, const float* __restrict__ row_scale,
                 const bf16_t* __restrict__ X2all, void* __restrict__ C3all) {
    static_assert(SPLIT != SPLIT_LEFT || !A_MC, "the two-part left operand is contraction-contiguous");
    static_assert(SPLIT != SPLIT_RIGHT || !B_KC, "the two-part right operand keeps k as its row index");
    constexpr bool SPLIT_A = SPLIT == SPLIT_LEFT, SPLIT_B = SPLIT == SPLIT_RIGHT;
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_CHUNKS = BM / 32, B_CHUNKS = BN / 32;  // 16-byte chunks per thread and stage
    constexpr int A_PITCH = A_MC ? BM + 32 : GEMM_LDS_STRIDE;
    constexpr int B_PITCH = B_KC ? GEMM_LDS_STRIDE : BN + 32;
    constexpr int A_ELEMS = A_MC ? GEMM_BK * A_PITCH : BM * A_PITCH;
    constexpr int B_ELEMS = B_KC ? BN * B_PITCH : GEMM_BK * B_PITCH;
    constexpr int STAGE = A_ELEMS + B_ELEMS;
    constexpr bool F32_STRIP = EPI == EPI_MULGRAD || EPI == EPI_F32;
    constexpr int EPI_STRIDE = F32_STRIP ? WN + 4 : WN + 8;  // elements per staged output row
    static_assert(TM >= 1 && TN >= 1, "tile too small");
    static_assert(EPI == EPI_SOFTMAX || (F32_STRIP ? 1 : 2) * 4 * 32 * EPI_STRIDE * (F32_STRIP ? 4 : 2) <= STAGES * STAGE * 2,
                  "epilogue staging must fit (bf16 outputs: two sets of strips, values and remainders)");
    static_assert(STAGES == 1 || STAGES == 2, "one or two LDS stages");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);

    // XCD-aware tile order: workgroups are handed to the 8 XCDs round-robin, so give each XCD a
    // contiguous run of logical tiles; consecutive logical tiles share an operand panel, which then
    // stays in that XCD's L2.
    const int total = G * tiles_m * tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (EPI != EPI_SOFTMAX && logical >= total) return;
    // the axis with fewer tiles varies fastest, so that the 32 tiles an XCD works on at a time span all of the
    // short axis and a few panels of the long one: both operands' panels then fit its L2 and are read from
    // HBM once (a tall product walked m-first re-read its whole M-side operand for every column of tiles)
    const bool n_fast = tiles_m > tiles_n;
    const int tm = n_fast ? (logical / tiles_n) % tiles_m : logical % tiles_m;
    const int tn = n_fast ? logical % tiles_n : (logical / tiles_m) % tiles_n;
    const int g = logical / (tiles_m * tiles_n);
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int col = lane & 31, half = lane >> 5, l16 = lane & 15;

    if (EPI == EPI_SOFTMAX) {
        uint32_t* zero_buf = reinterpret_cast<uint32_t*>(const_cast<int32_t*>(gather));
        for (int i = blockIdx.x * 256 + threadIdx.x; i < gather_rows; i += gridDim.x * 256) zero_buf[i] = 0u;
        gather = nullptr;
        if (logical >= total) return;
    }

    // With `gather` (A_MC = false only), row m of group g's left operand is row gather[g*M + m] of one
    // shared [gather_rows, K] matrix: the dispatch of Eq. 3 fused into the tile loads.
    const __amdgpu_buffer_rsrc_t rsrcA = (!A_MC && gather != nullptr)
        ? __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(Aall), 0, gather_rows * K * 2, 0x00020000)
        : __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(Aall + (size_t)g * M * K), 0, M * K * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcA2 = SPLIT_A
        ? __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(X2all + (size_t)g * M * K), 0, M * K * 2, 0x00020000)
        : rsrcA;
    const __amdgpu_buffer_rsrc_t rsrcB = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(Ball + (size_t)g * K * N), 0, K * N * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcB2 = SPLIT_B
        ? __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(X2all + (size_t)g * K * N), 0, K * N * 2, 0x00020000)
        : rsrcB;
    const int a_kstep = A_MC ? M * 2 : 2;  // bytes per unit of k in the scalar stage offset
    const int b_kstep = B_KC ? 2 : N * 2;

    // Per-thread byte offsets inside the group's matrices (the stage offset is added as a scalar) and
    // element offsets inside an LDS stage.  Every load instruction covers whole contiguous row pieces.
    int a_voff[A_CHUNKS], a_lds[A_CHUNKS], b_voff[B_CHUNKS], b_lds[B_CHUNKS];
#pragma unroll
    for (int r = 0; r < A_CHUNKS; ++r) {
        const int c = tid + 256 * r;
        if (A_MC) {
            const int krow = c / (BM / 8), ch = c % (BM / 8);
            a_voff[r] = (krow * M + m0 + ch * 8) * 2;
            a_lds[r] = krow * A_PITCH + ch * 8;
        } else {
            const int row = c >> 3, kch = c & 7;
            if (gather != nullptr) {
                const int gm = m0 + row;  // rows past M and empty rows (index -1) point outside the buffer: zeros
                const int src = gm < M ? gather[(size_t)g * M + gm] : -1;
                a_voff[r] = src >= 0 ? (src * K + kch * 8) * 2 : 0x7FFFFF00;
            } else {
                a_voff[r] = ((m0 + row) * K + kch * 8) * 2;
            }
            a_lds[r] = row * A_PITCH + kch * 8;
        }
    }
#pragma unroll
    for (int r = 0; r < B_CHUNKS; ++r) {
        const int c = tid + 256 * r;
        if (B_KC) {
            const int row = c >> 3, kch = c & 7;
            b_voff[r] = ((n0 + row) * K + kch * 8) * 2;
            b_lds[r] = A_ELEMS + row * B_PITCH + kch * 8;
        } else {
            const int krow = c / (BN / 8), ch = c % (BN / 8);
            b_voff[r] = (krow * N + n0 + ch * 8) * 2;
            b_lds[r] = A_ELEMS + krow * B_PITCH + ch * 8;
        }
    }

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    u32x4 areg[A_CHUNKS];
    u32x4 breg[B_CHUNKS];
    // Stage at contraction offset k0.  With a two-part left operand the stages alternate between the parts: stages
    // 2j and 2j+1 multiply the first and the second part's columns 64j.. by the same 64 rows of B, which the second
    // of them finds in the cache.
    auto load_tiles = [&](int k0) {
        const bool second = SPLIT != SPLIT_NONE && ((k0 / GEMM_BK) & 1) != 0;
        const int kk = SPLIT != SPLIT_NONE ? (k0 / (2 * GEMM_BK)) * GEMM_BK : k0;
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r)
            areg[r] = (SPLIT_A && second) ? __builtin_amdgcn_raw_buffer_load_b128(rsrcA2, a_voff[r], kk * a_kstep, 0)
                                          : __builtin_amdgcn_raw_buffer_load_b128(rsrcA, a_voff[r], kk * a_kstep, 0);
#pragma unroll
        for (int r = 0; r < B_CHUNKS; ++r)
            breg[r] = (SPLIT_B && second) ? __builtin_amdgcn_raw_buffer_load_b128(rsrcB2, b_voff[r], kk * b_kstep, 0)
                                          : __builtin_amdgcn_raw_buffer_load_b128(rsrcB, b_voff[r], kk * b_kstep, 0);
    };
    auto store_tiles = [&](int buf) {
        bf16_t* base = smem + buf * STAGE;
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r) *reinterpret_cast<u32x4*>(&base[a_lds[r]]) = areg[r];
#pragma unroll
        for (int r = 0; r < B_CHUNKS; ++r) *reinterpret_cast<u32x4*>(&base[b_lds[r]]) = breg[r];
    };

    // Fragment addresses (element offsets in a stage) for step 0, tile 0.
    const int a_frag = A_MC ? (half * 8 + (l16 >> 2)) * A_PITCH + wr * WM + ((lane >> 4) & 1) * 16 + (l16 & 3) * 4
                            : (wr * WM + col) * A_PITCH + half * 8;
    const int b_frag = A_ELEMS + (B_KC ? (wc * WN + col) * B_PITCH + half * 8
                                       : (half * 8 + (l16 >> 2)) * B_PITCH + wc * WN + ((lane >> 4) & 1) * 16 +
                                             (l16 & 3) * 4);
    bf16x4 alo[2][TM], ahi[2][TM], blo[2][TN], bhi[2][TN];
    typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
    constexpr int A_READS = A_MC ? 2 * TM : TM, B_READS = B_KC ? TN : 2 * TN;
    constexpr int N_READS = A_READS + B_READS;  // LDS reads that fetch one step's fragments
    auto read_one = [&](int set, const bf16_t* stage, int s, int idx) {
        if (idx < A_READS) {
            if (A_MC) {
                const int i = idx >> 1;
                const bf16_t* p0 = &stage[a_frag + s * 16 * A_PITCH + i * 32];
                if ((idx & 1) == 0) alo[set][i] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0));
                else ahi[set][i] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0 + 4 * A_PITCH));
            } else {
                const bf16x8 v = *reinterpret_cast<const bf16x8*>(&stage[a_frag + idx * 32 * A_PITCH + s * 16]);
                alo[set][idx] = __builtin_shufflevector(v, v, 0, 1, 2, 3);
                ahi[set][idx] = __builtin_shufflevector(v, v, 4, 5, 6, 7);
            }
        } else if (idx < N_READS) {
            const int t = idx - A_READS;
            if (B_KC) {
                const bf16x8 v = *reinterpret_cast<const bf16x8*>(&stage[b_frag + t * 32 * B_PITCH + s * 16]);
                blo[set][t] = __builtin_shufflevector(v, v, 0, 1, 2, 3);
                bhi[set][t] = __builtin_shufflevector(v, v, 4, 5, 6, 7);
            } else {
                const int j = t >> 1;
                const bf16_t* p0 = &stage[b_frag + s * 16 * B_PITCH + j * 32];
                if ((t & 1) == 0) blo[set][j] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0));
                else bhi[set][j] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0 + 4 * B_PITCH));
            }
        }
    };
    auto read_frags = [&](int set, const bf16_t* stage, int s) {
#pragma unroll
        for (int idx = 0; idx < N_READS; ++idx) read_one(set, stage, s, idx);
    };

    // One staging chunk: its register goes to the other LDS buffer, then the same register is refilled
    // with the chunk of the stage after that.  Spreading these pairs between the MFMAs keeps the
    // vector-memory and LDS queues from ever seeing a burst, and gives every global load a whole
    // iteration of flight time.
    constexpr int N_CHUNKS = A_CHUNKS + B_CHUNKS;
    constexpr int STEPS = GEMM_BK / 16;
    constexpr int NMF = TM * TN;              // MFMAs per step = issue slots per step
    constexpr int STAGING_STEPS = STEPS - 1;  // staging happens before the barrier, i.e. not in the last step
    constexpr int CHUNKS_PER_STEP = (N_CHUNKS + STAGING_STEPS - 1) / STAGING_STEPS;
    constexpr int READS_PER_SLOT = (N_READS + NMF - 1) / NMF;
    static_assert(STAGES == 1 || 2 * CHUNKS_PER_STEP <= NMF, "a step has too few MFMAs to hide its staging traffic");
    constexpr int STAGE_SLOT0 = NMF > 2 * CHUNKS_PER_STEP ? NMF - 2 * CHUNKS_PER_STEP : 0;  // chunk pairs fill the back of a step
    auto stage_write = [&](int r, bf16_t* dst) {
        if (r < A_CHUNKS) *reinterpret_cast<u32x4*>(&dst[a_lds[r]]) = areg[r];
        else if (r < N_CHUNKS) *reinterpret_cast<u32x4*>(&dst[b_lds[r - A_CHUNKS]]) = breg[r - A_CHUNKS];
    };
    auto stage_load = [&](int r, int k_next) {
        const bool second = SPLIT != SPLIT_NONE && ((k_next / GEMM_BK) & 1) != 0;
        const int kk = SPLIT != SPLIT_NONE ? (k_next / (2 * GEMM_BK)) * GEMM_BK : k_next;
        if (r < A_CHUNKS)
            areg[r] = (SPLIT_A && second) ? __builtin_amdgcn_raw_buffer_load_b128(rsrcA2, a_voff[r], kk * a_kstep, 0)
                                          : __builtin_amdgcn_raw_buffer_load_b128(rsrcA, a_voff[r], kk * a_kstep, 0);
        else if (r < N_CHUNKS)
            breg[r - A_CHUNKS] =
                (SPLIT_B && second) ? __builtin_amdgcn_raw_buffer_load_b128(rsrcB2, b_voff[r - A_CHUNKS], kk * b_kstep, 0)
                                    : __builtin_amdgcn_raw_buffer_load_b128(rsrcB, b_voff[r - A_CHUNKS], kk * b_kstep, 0);
    };
    // One step (16 contraction elements) written in issue order.  After every MFMA comes at most one
    // fragment read for the following step (taken from `next_stage` at step `next_s`) and, in the
    // staging steps, either the LDS write or the global load of a staging chunk: an LDS write of 1 KiB
    // keeps the wavefront's issue port busy about as long as one MFMA executes, so no two of them may
    // sit between the same pair of MFMAs.  Scheduling barriers pin this order.
    auto step = [&](int s, const bf16_t* next_stage, int next_s, bf16_t* dst, int k_next, bool staging) {
#pragma unroll
        for (int m = 0; m < NMF; ++m) {
            const int i = m / TN, j = m % TN;
            const bf16x8 bop = __builtin_shufflevector(blo[s & 1][j], bhi[s & 1][j], 0, 1, 2, 3, 4, 5, 6, 7);
            const bf16x8 aop = __builtin_shufflevector(alo[s & 1][i], ahi[s & 1][i], 0, 1, 2, 3, 4, 5, 6, 7);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bop, aop, acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < READS_PER_SLOT; ++c) read_one((s + 1) & 1, next_stage, next_s, m * READS_PER_SLOT + c);
            if (staging && m >= STAGE_SLOT0) {
                const int r = s * CHUNKS_PER_STEP + ((m - STAGE_SLOT0) >> 1);
                if (((m - STAGE_SLOT0) & 1) == 0) stage_write(r, dst);
                else stage_load(r, k_next);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Loads past the last stage read zeros or in-range data of the same group: harmless, never consumed.
    // a ragged K is legal only when both operands keep k as the row index; a two-part left operand doubles the stages
    const int nk = (SPLIT != SPLIT_NONE ? 2 : 1) * ((K + GEMM_BK - 1) / GEMM_BK);
    if (STAGES == 2) {
        // Both of the first two stages are requested at once (one trip to memory instead of two in a row): stage 0
        // into a second set of registers that only lives here, stage 1 into the set the loop works with.
        u32x4 areg0[A_CHUNKS], breg0[B_CHUNKS];
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r) areg0[r] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, a_voff[r], 0, 0);
#pragma unroll
        for (int r = 0; r < B_CHUNKS; ++r) breg0[r] = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, b_voff[r], 0, 0);
        load_tiles(GEMM_BK);
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r) *reinterpret_cast<u32x4*>(&smem[a_lds[r]]) = areg0[r];
#pragma unroll
        for (int r = 0; r < B_CHUNKS; ++r) *reinterpret_cast<u32x4*>(&smem[b_lds[r]]) = breg0[r];
        __syncthreads();
        read_frags(0, smem, 0);
        for (int kc = 0; kc < nk; ++kc) {
            const int cur = kc & 1;
            const bf16_t* stage = smem + cur * STAGE;
            bf16_t* other = smem + (cur ^ 1) * STAGE;
            // Registers hold stage kc+1: it goes to the other buffer (last read before the previous
            // barrier) while stage kc+2 is requested, all within the first steps.
#pragma unroll
            for (int s = 0; s + 1 < STEPS; ++s) step(s, stage, s + 1, other, (kc + 2) * GEMM_BK, true);
            __syncthreads();  // stage kc+1 is complete in `other`; nobody reads `stage` any more
            // last step: its fragments are already in registers; fetch the next stage's first ones meanwhile
            step(STEPS - 1, other, 0, nullptr, 0, false);
        }
        __syncthreads();  // every wavefront is done with the tile buffers before the epilogue reuses them
    } else {
        load_tiles(0);
        for (int kc = 0; kc < nk; ++kc) {
            store_tiles(0);  // the buffer is free: every wavefront passed the barrier that ends the previous phase
            __syncthreads();
            load_tiles((kc + 1) * GEMM_BK);
            read_frags(0, smem, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < STEPS; ++s) step(s, smem, s + 1 < STEPS ? s + 1 : 0, nullptr, 0, false);
            __syncthreads();
        }
    }

    // Epilogue.  acc[i][j][4q+t] = C[row m = i*32 + col][column n = j*32 + 8q + 4*half + t] of the wave tile.
    // Per wavefront: stage one 32-row strip (all WN columns) in LDS, then store it with 16-byte vectors.
    const size_t gofs = (size_t)g * M * N;
    if (EPI == EPI_SOFTMAX) {
        // A row of the tile is a token's logits over all N columns (tiles_n == 1).  A lane holds 64 of
        // them per 32-row strip i; the other half-wave holds 64 more and the wavefront next to it (wc ^ 1)
        // the remaining 128: one shuffle and one exchange through LDS complete a row's maximum and sum.
        float* __restrict__ Ct = reinterpret_cast<float*>(Call);   // [N][M]
        float* __restrict__ Cn = reinterpret_cast<float*>(C2all);  // [M][N] or null
        float* xch = reinterpret_cast<float*>(smem_raw);           // [wave][TM][32]
        float mx[TM], part[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            float m = -INFINITY;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ex = n0 + wc * WN + j * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                    if (ex < N) m = fmaxf(m, acc[i][j][r]);
                }
            mx[i] = fmaxf(m, __shfl_xor(m, 32, kWave));
            if (half == 0) xch[(wave * TM + i) * 32 + col] = mx[i];
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < TM; ++i) mx[i] = fmaxf(mx[i], xch[((wave ^ 1) * TM + i) * 32 + col]);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            float sum = 0.0f;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ex = n0 + wc * WN + j * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                    // exp through the hardware exp2: the rounding of (z - max) * log2(e) costs a relative
                    // 6e-8 * |z - max|, far inside the tolerance of the scores wherever they are not negligible
                    const float p = ex < N ? __builtin_amdgcn_exp2f((acc[i][j][r] - mx[i]) * 1.44269504088896340736f) : 0.0f;
                    acc[i][j][r] = p;
                    sum += p;
                }
            sum += __shfl_xor(sum, 32, kWave);
            part[i] = sum;
            if (half == 0) xch[(wave * TM + i) * 32 + col] = sum;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const float other = xch[((wave ^ 1) * TM + i) * 32 + col];
            const float total_sum = part[i] + other;  // the same two addends in both wavefronts: the same sum
            const float inv_sum = 1.0f / total_sum;    // one division per row, then multiplications
            const int gm = m0 + wr * WM + i * 32 + col;
            if (gm < M) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int ex0 = n0 + wc * WN + j * 32 + 8 * q + 4 * half;
                        if (ex0 < N) {  // N % 8 == 0: a quad is all columns or all padding
                            floatx4 o;
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                o[t] = acc[i][j][4 * q + t] * inv_sum;
                                if (Ct != nullptr) Ct[(size_t)(ex0 + t) * M + gm] = o[t];
                            }
                            if (Cn != nullptr) *reinterpret_cast<floatx4*>(Cn + (size_t)gm * N + ex0) = o;
                        }
                    }
            }
        }
    } else if (!F32_STRIP) {
        bf16_t* __restrict__ C = reinterpret_cast<bf16_t*>(Call) + gofs;
        bf16_t* __restrict__ Cpre = EPI == EPI_ACT_SAVE ? reinterpret_cast<bf16_t*>(C2all) + gofs : nullptr;
        bf16_t* __restrict__ Clo = C3all != nullptr ? reinterpret_cast<bf16_t*>(C3all) + gofs : nullptr;
        bf16_t* strip = smem + wave * 32 * EPI_STRIDE;
        bf16_t* strip_lo = smem + (4 + wave) * 32 * EPI_STRIDE;  // second set of strips, for the remainders
        constexpr int CHUNKS_PER_ROW = WN / 8;
        constexpr int ROWS_PER_PASS = 64 / CHUNKS_PER_ROW;  // lanes past ROWS_PER_PASS rows idle (WN = 96)
        const int er = lane / CHUNKS_PER_ROW, ec = lane % CHUNKS_PER_ROW;
#pragma unroll
        for (int pass = 0; pass < (EPI == EPI_ACT_SAVE ? 2 : 1); ++pass) {
            const bool pre = EPI == EPI_ACT_SAVE && pass == 0;
            const bool with_lo = !pre && Clo != nullptr;  // uniform
            bf16_t* __restrict__ dst = pre ? Cpre : C;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        bf16x4 v;
                        float y[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const float x = acc[i][j][4 * q + t];
                            y[t] = pre ? x : apply_act_bf16<ACT>(x);
                            v[t] = static_cast<bf16_t>(y[t]);
                        }
                        *reinterpret_cast<bf16x4*>(&strip[col * EPI_STRIDE + j * 32 + 8 * q + 4 * half]) = v;
                        if (with_lo) {
                            bf16x4 vl;
#pragma unroll
                            for (int t = 0; t < 4; ++t) vl[t] = static_cast<bf16_t>(y[t] - static_cast<float>(v[t]));
                            *reinterpret_cast<bf16x4*>(&strip_lo[col * EPI_STRIDE + j * 32 + 8 * q + 4 * half]) = vl;
                        }
                    }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int rr = 0; rr < 32; rr += ROWS_PER_PASS) {
                    const int row = rr + er;
                    const int gm = m0 + wr * WM + i * 32 + row;
                    const int gn = n0 + wc * WN + ec * 8;
                    if (er < ROWS_PER_PASS && row < 32 && gm < M && gn < N) {
                        *reinterpret_cast<uint4*>(dst + (size_t)gm * N + gn) =
                            *reinterpret_cast<const uint4*>(&strip[row * EPI_STRIDE + ec * 8]);
                        if (with_lo)
                            *reinterpret_cast<uint4*>(Clo + (size_t)gm * N + gn) =
                                *reinterpret_cast<const uint4*>(&strip_lo[row * EPI_STRIDE + ec * 8]);
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
    } else {
        float* strip = reinterpret_cast<float*>(smem_raw) + wave * 32 * EPI_STRIDE;
        // EPI_MULGRAD: the pre-activations and row weights this lane will need are requested for the whole wave tile
        // up front (the staging registers of the main loop are free now), so the strips below wait for memory once.
        constexpr int MG_CHUNKS_PER_ROW = WN / 8, MG_ROWS_PER_PASS = 64 / MG_CHUNKS_PER_ROW;
        constexpr int MG_PASSES = EPI == EPI_MULGRAD ? 32 / MG_ROWS_PER_PASS : 1;
        bf16x8 mg_aux[EPI == EPI_MULGRAD ? TM : 1][MG_PASSES];
        float mg_rs[EPI == EPI_MULGRAD ? TM : 1][MG_PASSES];
        if (EPI == EPI_MULGRAD) {
            const bf16_t* __restrict__ Aux = reinterpret_cast<const bf16_t*>(C2all) + gofs;
            const int er = lane / MG_CHUNKS_PER_ROW, ec = lane % MG_CHUNKS_PER_ROW;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int p = 0; p < MG_PASSES; ++p) {
                    const int row = p * MG_ROWS_PER_PASS + er;
                    const int gm = m0 + wr * WM + i * 32 + row;
                    const int gn = n0 + wc * WN + ec * 8;
                    const bool in = er < MG_ROWS_PER_PASS && row < 32 && gm < M && gn < N;
                    bf16x8 a = {};
                    if (in) a = *reinterpret_cast<const bf16x8*>(Aux + (size_t)gm * N + gn);
                    mg_aux[i][p] = a;
                    mg_rs[i][p] = (in && row_scale != nullptr) ? row_scale[(size_t)g * M + gm] : 1.0f;
                }
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    floatx4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    *reinterpret_cast<floatx4*>(&strip[col * EPI_STRIDE + j * 32 + 8 * q + 4 * half]) = v;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (EPI == EPI_F32) {
                float* __restrict__ C = reinterpret_cast<float*>(Call) + gofs;
                constexpr int CHUNKS_PER_ROW = WN / 4;  // 16-byte chunks of 4 floats
                constexpr int ROWS_PER_PASS = 64 / CHUNKS_PER_ROW;
                const int er = lane / CHUNKS_PER_ROW, ec = lane % CHUNKS_PER_ROW;
#pragma unroll
                for (int rr = 0; rr < 32; rr += ROWS_PER_PASS) {
                    const int row = rr + er;
                    const int gm = m0 + wr * WM + i * 32 + row;
                    const int gn = n0 + wc * WN + ec * 4;
                    if (er < ROWS_PER_PASS && row < 32 && gm < M && gn < N) {
                        const floatx4 val = *reinterpret_cast<const floatx4*>(&strip[row * EPI_STRIDE + ec * 4]);
                        *reinterpret_cast<floatx4*>(C + (size_t)gm * N + gn) = val;
                        if (C3all != nullptr) {  // the same values rounded to bf16 (uniform branch)
                            bf16x4 h;
#pragma unroll
                            for (int t = 0; t < 4; ++t) h[t] = static_cast<bf16_t>(val[t]);
                            *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16_t*>(C3all) + gofs + (size_t)gm * N + gn) = h;
                        }
                    }
                }
            } else {
                bf16_t* __restrict__ C = reinterpret_cast<bf16_t*>(Call) + gofs;
                bf16_t* __restrict__ Clo = C3all != nullptr ? reinterpret_cast<bf16_t*>(C3all) + gofs : nullptr;
                constexpr int CHUNKS_PER_ROW = MG_CHUNKS_PER_ROW;
                constexpr int ROWS_PER_PASS = MG_ROWS_PER_PASS;
                const int er = lane / CHUNKS_PER_ROW, ec = lane % CHUNKS_PER_ROW;
#pragma unroll
                for (int rr = 0; rr < 32; rr += ROWS_PER_PASS) {
                    const int row = rr + er;
                    const int gm = m0 + wr * WM + i * 32 + row;
                    const int gn = n0 + wc * WN + ec * 8;
                    if (er < ROWS_PER_PASS && row < 32 && gm < M && gn < N) {
                        const floatx4 v0 = *reinterpret_cast<const floatx4*>(&strip[row * EPI_STRIDE + ec * 8]);
                        const floatx4 v1 = *reinterpret_cast<const floatx4*>(&strip[row * EPI_STRIDE + ec * 8 + 4]);
                        const bf16x8 a = mg_aux[EPI == EPI_MULGRAD ? i : 0][EPI == EPI_MULGRAD ? rr / ROWS_PER_PASS : 0];
                        const float rs = mg_rs[EPI == EPI_MULGRAD ? i : 0][EPI == EPI_MULGRAD ? rr / ROWS_PER_PASS : 0];
                        bf16x8 o, lo;
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const float w0 = (rs * v0[t]) * apply_act_grad_bf16<ACT>(static_cast<float>(a[t]));
                            const float w1 = (rs * v1[t]) * apply_act_grad_bf16<ACT>(static_cast<float>(a[t + 4]));
                            o[t] = static_cast<bf16_t>(w0);
                            o[t + 4] = static_cast<bf16_t>(w1);
                            lo[t] = static_cast<bf16_t>(w0 - static_cast<float>(o[t]));
                            lo[t + 4] = static_cast<bf16_t>(w1 - static_cast<float>(o[t + 4]));
                        }
                        *reinterpret_cast<bf16x8*>(C + (size_t)gm * N + gn) = o;
                        if (Clo != nullptr) *reinterpret_cast<bf16x8*>(Clo + (size_t)gm * N + gn) = lo;
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// LDS bytes of a configuration.
template <int BM, int BN, int STAGES>
constexpr size_t gemm_bf16_lds_bytes() {
    // both storage kinds of an operand tile take the same space: ROWS * 72 == 64 * (ROWS + 32) for ROWS = 256,
    // and the padded form is the larger one below that
    return (size_t)STAGES * ((BM * GEMM_LDS_STRIDE > GEMM_BK * (BM + 32) ? BM * GEMM_LDS_STRIDE : GEMM_BK * (BM + 32)) +
                             (BN * GEMM_LDS_STRIDE > GEMM_BK * (BN + 32) ? BN * GEMM_LDS_STRIDE : GEMM_BK * (BN + 32))) *
           sizeof(bf16_t);
}

// True when the kernel covers the shape (otherwise callers fall back or refuse).  A contraction-
// contiguous operand needs K % 64 == 0 (the tail of a row would run into the next row); operands that
// keep k as the row index are zero-filled past K by the buffer range check.
inline bool gemm_bf16_shape_ok(int64_t M, int64_t N, int64_t K, bool k_contiguous_operand = true,
                               bool m_contiguous_operand = false) {
    return (!k_contiguous_operand || (K % GEMM_BK) == 0) && (N % 8) == 0 && (!m_contiguous_operand || (M % 8) == 0) &&
           M * K * 2 < ((int64_t)1 << 31) && K * N * 2 < ((int64_t)1 << 31) && M * N < ((int64_t)1 << 31);
}

// Raises a kernel's dynamic-LDS limit once per kernel and GPU (the attribute belongs to the function on the
// current device); `done` is the instantiation's own flag array.
inline void gemm_allow_lds(const void* kern, size_t lds, std::atomic<bool>* done /*[64]*/) {
    if (lds <= 64 * 1024) return;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    if (done[dev].load(std::memory_order_acquire)) return;
    (void)hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    done[dev].store(true, std::memory_order_release);
}

// X2 (with SPLIT): the second part of the split operand.  C3 (optional): see GemmEpilogue.
template <int BM, int BN, int STAGES, int OCC, bool A_MC, bool B_KC, int EPI, int ACT, int SPLIT = SPLIT_NONE>
static void gemm_bf16_launch(const bf16_t* A, const bf16_t* B, void* C, void* C2, int G, int M, int N, int K,
                             const int32_t* gather, int gather_rows, hipStream_t stream,
                             const float* row_scale = nullptr, const bf16_t* X2 = nullptr, void* C3 = nullptr) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int total = G * tiles_m * tiles_n;
    const size_t lds = gemm_bf16_lds_bytes<BM, BN, STAGES>();
    auto kern = gemm_bf16_kernel<BM, BN, STAGES, OCC, A_MC, B_KC, EPI, ACT, SPLIT>;
    static std::atomic<bool> lds_allowed[64];
    gemm_allow_lds(reinterpret_cast<const void*>(kern), lds, lds_allowed);
    hipLaunchKernelGGL(kern, dim3((unsigned)((total + 7) / 8 * 8)), dim3(256), lds, stream, A, B, C, C2, M, N, K, G,
                       tiles_m, tiles_n, gather, gather_rows, row_scale, X2, C3);
}

}  // namespace ecmoe
