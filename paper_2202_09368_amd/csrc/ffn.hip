// Expert FFN: X_e[i] = act(X_in[i].W1[i]).W2[i] for every expert i (Sec. 3.2, Eq. 3).
//
// Two grouped (one launch covers all experts) GEMMs: A = X_in.W1 with the
// activation fused into the epilogue, then X_e = H.W2.
//  * bf16: matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation, LDS-staged
//    tiles.  Both products are "row-major x row-major": the left operand is
//    contraction-contiguous, the right operand (the weights) is not, so its
//    tile is transposed in registers on the way into LDS and both MFMA operands
//    are then read as 16-byte contraction-contiguous vectors.
//  * fp32: plain FMA tiles (small parity configuration only).
#include <cmath>
#include <cstdlib>

#include "ec_common.h"

namespace ecmoe {

// ===========================================================================
// bf16 grouped GEMM on MFMA:  C[g] = epilogue(A[g] (M x K)  .  B[g] (K x N))
// ===========================================================================
constexpr int GEMM_BK = 64;                 // contraction elements per LDS stage
constexpr int GEMM_LDS_STRIDE = GEMM_BK + 8;  // bf16 elements per LDS row (144 B: conflict-free 16 B reads)

struct GemmArgs {
    const bf16_t* A;   // [G, M, K]
    const bf16_t* B;   // [G, K, N]
    bf16_t* C;         // [G, M, N]  act(acc)
    bf16_t* Cpre;      // [G, M, N]  acc before the activation, or nullptr
    int M, N, K, G;
    int tiles_m, tiles_n;
};

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) {  // (a.lo16, b.lo16) -> a.lo | b.lo << 16
    return __builtin_amdgcn_perm(b, a, 0x05040100u);
}
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) {  // a.hi | b.hi << 16
    return __builtin_amdgcn_perm(b, a, 0x07060302u);
}

// General-shape kernel (any K that is a multiple of 8): same tiling as the fast
// kernel below but with predicated, zero-filling loads.  Used when K % 64 != 0.
template <int BM, int BN, int ACT, bool SAVE_PRE>
__global__ void __launch_bounds__(256, 1)
gemm_bf16_generic_kernel(GemmArgs p) {
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_CHUNKS = BM * 8 / 256;                    // 16-byte chunks of the A tile per thread
    constexpr int B_BLOCKS = (GEMM_BK / 4) * (BN / 8) / 256;  // 4(k) x 8(n) sub-blocks of the B tile per thread
    constexpr int STAGE = (BM + BN) * GEMM_LDS_STRIDE;        // bf16 elements per stage
    constexpr int EPI_STRIDE = WN + 8;                        // bf16 elements per staged output row
    static_assert(A_CHUNKS >= 1 && B_BLOCKS >= 1 && TM >= 1 && TN >= 1, "tile too small");
    static_assert(4 * 32 * EPI_STRIDE <= 2 * STAGE, "epilogue staging must fit in the tile buffers");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);

    // XCD-aware tile order: workgroups are handed to the 8 XCDs round-robin, so
    // give each XCD a contiguous run of logical tiles; consecutive logical tiles
    // share the weight panel (m fastest), which then stays in that XCD's L2.
    const int total = p.G * p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    const int tm = logical % p.tiles_m;
    const int tn = (logical / p.tiles_m) % p.tiles_n;
    const int g = logical / (p.tiles_m * p.tiles_n);

    const int M = p.M, N = p.N, K = p.K;
    const bf16_t* __restrict__ A = p.A + (size_t)g * M * K;
    const bf16_t* __restrict__ B = p.B + (size_t)g * K * N;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int col = lane & 31, half = lane >> 5;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    uint4 areg[A_CHUNKS];
    uint4 breg[B_BLOCKS][4];
    const uint4 zero4 = {0u, 0u, 0u, 0u};

    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r) {
            int c = tid + 256 * r;
            int row = c >> 3, kch = c & 7;
            int gm = m0 + row, gk = k0 + kch * 8;
            areg[r] = (gm < M && gk < K) ? *reinterpret_cast<const uint4*>(A + (size_t)gm * K + gk) : zero4;
        }
#pragma unroll
        for (int r = 0; r < B_BLOCKS; ++r) {
            int blk = tid + 256 * r;
            int kg = blk & 15, ng = blk >> 4;  // 16 k-groups of 4 rows, BN/8 n-groups of 8 columns
            int gn = n0 + ng * 8;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int gk = k0 + kg * 4 + q;
                breg[r][q] = (gk < K && gn < N) ? *reinterpret_cast<const uint4*>(B + (size_t)gk * N + gn) : zero4;
            }
        }
    };
    auto store_tiles = [&](int buf) {
        bf16_t* As = smem + buf * STAGE;
        bf16_t* Bs = As + BM * GEMM_LDS_STRIDE;  // transposed: [n][k]
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r) {
            int c = tid + 256 * r;
            int row = c >> 3, kch = c & 7;
            *reinterpret_cast<uint4*>(&As[row * GEMM_LDS_STRIDE + kch * 8]) = areg[r];
        }
#pragma unroll
        for (int r = 0; r < B_BLOCKS; ++r) {
            int blk = tid + 256 * r;
            int kg = blk & 15, ng = blk >> 4;
            // 4 x 8 block held as 4 rows of 8 bf16 -> 8 columns of 4 bf16 (contraction-contiguous)
            const uint32_t* r0 = reinterpret_cast<const uint32_t*>(&breg[r][0]);
            const uint32_t* r1 = reinterpret_cast<const uint32_t*>(&breg[r][1]);
            const uint32_t* r2 = reinterpret_cast<const uint32_t*>(&breg[r][2]);
            const uint32_t* r3 = reinterpret_cast<const uint32_t*>(&breg[r][3]);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint2 even = {pack_lo(r0[w], r1[w]), pack_lo(r2[w], r3[w])};  // column 2w
                uint2 odd = {pack_hi(r0[w], r1[w]), pack_hi(r2[w], r3[w])};   // column 2w+1
                *reinterpret_cast<uint2*>(&Bs[(ng * 8 + 2 * w) * GEMM_LDS_STRIDE + kg * 4]) = even;
                *reinterpret_cast<uint2*>(&Bs[(ng * 8 + 2 * w + 1) * GEMM_LDS_STRIDE + kg * 4]) = odd;
            }
        }
    };

    const int nk = (K + GEMM_BK - 1) / GEMM_BK;
    load_tiles(0);
    store_tiles(0);
    if (nk > 1) load_tiles(GEMM_BK);
    __syncthreads();
    for (int kc = 0; kc < nk; ++kc) {
        const int cur = kc & 1;
        if (kc + 1 < nk) {
            store_tiles(cur ^ 1);  // registers hold stage kc+1; that buffer was last read in iteration kc-1
            if (kc + 2 < nk) load_tiles((kc + 2) * GEMM_BK);
        }
        const bf16_t* As = smem + cur * STAGE + (wr * WM + col) * GEMM_LDS_STRIDE + half * 8;
        const bf16_t* Bs = smem + cur * STAGE + BM * GEMM_LDS_STRIDE + (wc * WN + col) * GEMM_LDS_STRIDE + half * 8;
#pragma unroll
        for (int s = 0; s < GEMM_BK / 16; ++s) {
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(&As[i * 32 * GEMM_LDS_STRIDE + s * 16]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8*>(&Bs[j * 32 * GEMM_LDS_STRIDE + s * 16]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // Epilogue.  acc[i][j][4q+t] = C[row m = i*32 + col][column n = j*32 + 8q + 4*half + t] of the wave tile.
    // Per wavefront: stage one 32-row strip (all WN columns) in LDS, then store it with 16-byte vectors.
    bf16_t* __restrict__ C = p.C + (size_t)g * M * N;
    bf16_t* __restrict__ Cpre = SAVE_PRE ? p.Cpre + (size_t)g * M * N : nullptr;
    bf16_t* strip = smem + wave * 32 * EPI_STRIDE;
    constexpr int CHUNKS_PER_ROW = WN / 8;            // 16-byte chunks per staged row
    constexpr int ROWS_PER_PASS = 64 / CHUNKS_PER_ROW;
    const int er = lane / CHUNKS_PER_ROW, ec = lane % CHUNKS_PER_ROW;
#pragma unroll
    for (int pass = 0; pass < (SAVE_PRE ? 2 : 1); ++pass) {
        bf16_t* __restrict__ dst = (SAVE_PRE && pass == 0) ? Cpre : C;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bf16x4 v;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        float x = acc[i][j][4 * q + t];
                        v[t] = static_cast<bf16_t>((SAVE_PRE && pass == 0) ? x : apply_act<ACT>(x));
                    }
                    *reinterpret_cast<bf16x4*>(&strip[col * EPI_STRIDE + j * 32 + 8 * q + 4 * half]) = v;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int rr = 0; rr < 32; rr += ROWS_PER_PASS) {
                const int row = rr + er;
                const int gm = m0 + wr * WM + i * 32 + row;
                const int gn = n0 + wc * WN + ec * 8;
                uint4 v = *reinterpret_cast<const uint4*>(&strip[row * EPI_STRIDE + ec * 8]);
                if (gm < M && gn < N) *reinterpret_cast<uint4*>(dst + (size_t)gm * N + gn) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// ---------------------------------------------------------------------------
// Fast kernel: K % 64 == 0.  Global loads are raw buffer loads (the hardware
// range check returns zeros past the end of an expert's matrix, so ragged M
// needs no branch; ragged N only produces columns that are never stored).
// Per stage: write the prefetched stage to the other LDS buffer, issue the
// loads of the stage after it, then 4 x (TM x TN) MFMAs with the operands of
// step s+1 read from LDS while step s is in the matrix cores.
// ---------------------------------------------------------------------------
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// GeLU with the exact-erf definition a * Phi(a); erf by the Abramowitz-Stegun
// rational form 7.1.26 (|error| < 1.5e-7), written so the negative tail has no
// cancellation.  Used where the result is rounded to bf16 anyway.
__device__ __forceinline__ float gelu_erf_fast(float a) {
    const float x = fabsf(a) * 0.70710678118654752440f;
    const float t = __frcp_rn(fmaf(0.3275911f, x, 1.0f));
    float p = fmaf(t, 1.061405429f, -1.453152027f);
    p = fmaf(t, p, 1.421413741f);
    p = fmaf(t, p, -0.284496736f);
    p = fmaf(t, p, 0.254829592f);
    const float tail = 0.5f * p * t * __expf(-x * x);  // 0.5 * erfc(|a|/sqrt 2)
    const float phi = a >= 0.0f ? 1.0f - tail : tail;
    return a * phi;
}

template <int ACT>
__device__ __forceinline__ float apply_act_bf16(float a) {
    if (ACT == EC_ACT_GELU) return gelu_erf_fast(a);
    return apply_act<ACT>(a);
}

template <int BM, int BN, int STAGES, int OCC, int ACT, bool SAVE_PRE>
__global__ void __launch_bounds__(256, OCC)
gemm_bf16_fast_kernel(const bf16_t* __restrict__ Aall, const bf16_t* __restrict__ Ball, bf16_t* __restrict__ Call,
                      bf16_t* __restrict__ Cpreall, int M, int N, int K, int G, int tiles_m, int tiles_n,
                      const int32_t* __restrict__ gather, int gather_rows) {
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_CHUNKS = BM * 8 / 256;              // 16-byte chunks of the A tile per thread
    constexpr int B_CHUNKS = GEMM_BK * (BN / 8) / 256;  // 16-byte chunks of the B tile per thread
    constexpr int B_PITCH = BN + 32;                    // bf16 elements per LDS row of the B tile: 64 B of padding
                                                        // put four consecutive rows in four distinct bank groups
    constexpr int A_ELEMS = BM * GEMM_LDS_STRIDE;
    constexpr int STAGE = A_ELEMS + GEMM_BK * B_PITCH;
    constexpr int EPI_STRIDE = WN + 8;
    static_assert(A_CHUNKS >= 1 && B_CHUNKS >= 1 && TM >= 1 && TN >= 1, "tile too small");
    static_assert(4 * 32 * EPI_STRIDE <= STAGES * STAGE, "epilogue staging must fit in the tile buffers");
    static_assert(STAGES == 1 || STAGES == 2, "one or two LDS stages");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);

    // XCD-aware tile order (see the generic kernel).
    const int total = G * tiles_m * tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    const int tm = logical % tiles_m;
    const int tn = (logical / tiles_m) % tiles_n;
    const int g = logical / (tiles_m * tiles_n);
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int col = lane & 31, half = lane >> 5;

    // With `gather`, row m of group g's left operand is row gather[g*M + m] of one shared
    // [gather_rows, K] matrix (the dispatch of Eq. 3 fused into the tile loads).
    const __amdgpu_buffer_rsrc_t rsrcA = gather != nullptr
        ? __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(Aall), 0, gather_rows * K * 2, 0x00020000)
        : __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(Aall + (size_t)g * M * K), 0, M * K * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcB = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(Ball + (size_t)g * K * N), 0, K * N * 2, 0x00020000);

    // Per-thread byte offsets inside the expert's matrices (the stage offset is added as a scalar).
    // A tile: 8 lanes cover one 128-byte row segment.  B tile: BN/8 lanes cover one whole row of
    // the tile, so every load instruction reads full contiguous rows of the weight matrix.
    int a_voff[A_CHUNKS], a_lds[A_CHUNKS];
#pragma unroll
    for (int r = 0; r < A_CHUNKS; ++r) {
        int c = tid + 256 * r;
        int row = c >> 3, kch = c & 7;
        if (gather != nullptr) {
            const int gm = m0 + row;  // rows past M point outside the buffer: they load zeros
            a_voff[r] = gm < M ? (gather[(size_t)g * M + gm] * K + kch * 8) * 2 : 0x7FFFFF00;
        } else {
            a_voff[r] = ((m0 + row) * K + kch * 8) * 2;
        }
        a_lds[r] = row * GEMM_LDS_STRIDE + kch * 8;
    }
    int b_voff[B_CHUNKS], b_lds[B_CHUNKS];
#pragma unroll
    for (int r = 0; r < B_CHUNKS; ++r) {
        int c = tid + 256 * r;
        int krow = c / (BN / 8), nch = c % (BN / 8);
        b_voff[r] = (krow * N + n0 + nch * 8) * 2;
        b_lds[r] = A_ELEMS + krow * B_PITCH + nch * 8;
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

    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r)
            areg[r] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, a_voff[r], k0 * 2, 0);
#pragma unroll
        for (int r = 0; r < B_CHUNKS; ++r)
            breg[r] = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, b_voff[r], k0 * N * 2, 0);
    };
    auto store_tiles = [&](int buf) {
        bf16_t* base = smem + buf * STAGE;
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r) *reinterpret_cast<u32x4*>(&base[a_lds[r]]) = areg[r];
#pragma unroll
        for (int r = 0; r < B_CHUNKS; ++r) *reinterpret_cast<u32x4*>(&base[b_lds[r]]) = breg[r];
    };

    // A fragments: 16-byte contraction-contiguous reads.  B fragments: the B tile keeps the weight
    // matrix's own row-major [k][n] form; two transposing LDS reads (ds_read_b64_tr_b16) hand every
    // lane the 2 x 4 consecutive-k values of its column.  In a 16-lane group, lane L points at row
    // kbase + L/4, columns nbase + 4*(L%4) .. +3, and receives rows kbase..kbase+3 of column nbase + L.
    const int a_frag = (wr * WM + col) * GEMM_LDS_STRIDE + half * 8;
    const int l16 = lane & 15;
    const int b_frag = A_ELEMS + (half * 8 + (l16 >> 2)) * B_PITCH + wc * WN + ((lane >> 4) & 1) * 16 + (l16 & 3) * 4;
    bf16x8 af[2][TM];
    bf16x4 blo[2][TN], bhi[2][TN];
    typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
    constexpr int N_READS = TM + 2 * TN;  // LDS reads that fetch one step's fragments
    auto read_one = [&](int set, const bf16_t* stage, int s, int idx) {
        if (idx < TM) {
            af[set][idx] = *reinterpret_cast<const bf16x8*>(&stage[a_frag + idx * 32 * GEMM_LDS_STRIDE + s * 16]);
        } else if (idx < N_READS) {
            const int j = (idx - TM) >> 1;
            const bf16_t* p0 = &stage[b_frag + s * 16 * B_PITCH + j * 32];
            if (((idx - TM) & 1) == 0) blo[set][j] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0));
            else bhi[set][j] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0 + 4 * B_PITCH));
        }
    };
    auto read_frags = [&](int set, const bf16_t* stage, int s) {
#pragma unroll
        for (int idx = 0; idx < N_READS; ++idx) read_one(set, stage, s, idx);
    };

    // One staging chunk: its register goes to the other LDS buffer, then the same register is
    // refilled with the chunk of the stage after that.  Spreading these pairs between the MFMAs
    // keeps the vector-memory and LDS queues from ever seeing a burst, and gives every global
    // load a whole iteration of flight time.
    constexpr int N_CHUNKS = A_CHUNKS + B_CHUNKS;
    constexpr int STEPS = GEMM_BK / 16;
    constexpr int NMF = TM * TN;                      // MFMAs per step = issue slots per step
    constexpr int STAGING_STEPS = STEPS - 1;          // staging happens before the barrier, i.e. not in the last step
    constexpr int CHUNKS_PER_STEP = (N_CHUNKS + STAGING_STEPS - 1) / STAGING_STEPS;
    constexpr int READS_PER_SLOT = (N_READS + NMF - 1) / NMF;
    static_assert(STAGES == 1 || 2 * CHUNKS_PER_STEP <= NMF, "a step has too few MFMAs to hide its staging traffic");
    constexpr int STAGE_SLOT0 = NMF > 2 * CHUNKS_PER_STEP ? NMF - 2 * CHUNKS_PER_STEP : 0;  // chunk pairs fill the back of a step
    // One step (16 contraction elements) written in issue order.  After every MFMA comes at most
    // one fragment read for the following step (taken from `next_stage` at step `next_s`) and, in
    // the staging steps, either the LDS write or the global load of a staging chunk: an LDS write
    // of 1 KiB keeps the wavefront's issue port busy about as long as one MFMA executes, so no two
    // of them may sit between the same pair of MFMAs.  Scheduling barriers pin this order.
    auto stage_write = [&](int r, bf16_t* dst) {
        if (r < A_CHUNKS) *reinterpret_cast<u32x4*>(&dst[a_lds[r]]) = areg[r];
        else if (r < N_CHUNKS) *reinterpret_cast<u32x4*>(&dst[b_lds[r - A_CHUNKS]]) = breg[r - A_CHUNKS];
    };
    auto stage_load = [&](int r, int k_next) {
        if (r < A_CHUNKS) areg[r] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, a_voff[r], k_next * 2, 0);
        else if (r < N_CHUNKS)
            breg[r - A_CHUNKS] = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, b_voff[r - A_CHUNKS], k_next * N * 2, 0);
    };
    auto step = [&](int s, const bf16_t* next_stage, int next_s, bf16_t* dst, int k_next, bool staging) {
#pragma unroll
        for (int m = 0; m < NMF; ++m) {
            const int i = m / TN, j = m % TN;
            const bf16x8 bop = __builtin_shufflevector(blo[s & 1][j], bhi[s & 1][j], 0, 1, 2, 3, 4, 5, 6, 7);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bop, af[s & 1][i], acc[i][j], 0, 0, 0);
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

    // Loads past the last stage read zeros or in-range rows of the same expert: harmless, never consumed.
    const int nk = K / GEMM_BK;
    load_tiles(0);
    if (STAGES == 2) {
        store_tiles(0);
        load_tiles(GEMM_BK);
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
    bf16_t* __restrict__ C = Call + (size_t)g * M * N;
    bf16_t* __restrict__ Cpre = SAVE_PRE ? Cpreall + (size_t)g * M * N : nullptr;
    bf16_t* strip = smem + wave * 32 * EPI_STRIDE;
    constexpr int CHUNKS_PER_ROW = WN / 8;
    constexpr int ROWS_PER_PASS = 64 / CHUNKS_PER_ROW;
    const int er = lane / CHUNKS_PER_ROW, ec = lane % CHUNKS_PER_ROW;
#pragma unroll
    for (int pass = 0; pass < (SAVE_PRE ? 2 : 1); ++pass) {
        bf16_t* __restrict__ dst = (SAVE_PRE && pass == 0) ? Cpre : C;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bf16x4 v;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        float x = acc[i][j][4 * q + t];
                        v[t] = static_cast<bf16_t>((SAVE_PRE && pass == 0) ? x : apply_act_bf16<ACT>(x));
                    }
                    *reinterpret_cast<bf16x4*>(&strip[col * EPI_STRIDE + j * 32 + 8 * q + 4 * half]) = v;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int rr = 0; rr < 32; rr += ROWS_PER_PASS) {
                const int row = rr + er;
                const int gm = m0 + wr * WM + i * 32 + row;
                const int gn = n0 + wc * WN + ec * 8;
                uint4 v = *reinterpret_cast<const uint4*>(&strip[row * EPI_STRIDE + ec * 8]);
                if (gm < M && gn < N) *reinterpret_cast<uint4*>(dst + (size_t)gm * N + gn) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

template <int BM, int BN, int STAGES, int OCC>
static void launch_gemm_bf16(const bf16_t* A, const bf16_t* B, bf16_t* C, bf16_t* Cpre, int G, int M, int N, int K,
                             int act, const int32_t* gather, int gather_rows, hipStream_t stream) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int total = G * tiles_m * tiles_n;
    dim3 grid((unsigned)((total + 7) / 8 * 8)), block(256);
    const bool fast = (K % GEMM_BK) == 0 && (int64_t)M * K * 2 < ((int64_t)1 << 31) &&
                      (int64_t)K * N * 2 < ((int64_t)1 << 31);
    const size_t lds = fast ? (size_t)STAGES * (BM * GEMM_LDS_STRIDE + GEMM_BK * (BN + 32)) * sizeof(bf16_t)
                            : (size_t)2 * (BM + BN) * GEMM_LDS_STRIDE * sizeof(bf16_t);
    GemmArgs p;
    p.A = A; p.B = B; p.C = C; p.Cpre = Cpre;
    p.M = M; p.N = N; p.K = K; p.G = G;
    p.tiles_m = tiles_m; p.tiles_n = tiles_n;
#define EC_GEMM_LAUNCH(ACTV, SAVE)                                                                          \
    do {                                                                                                    \
        if (fast) {                                                                                         \
            auto kern = gemm_bf16_fast_kernel<BM, BN, STAGES, OCC, ACTV, SAVE>;                             \
            if (lds > 64 * 1024)                                                                            \
                (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                              \
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);            \
            hipLaunchKernelGGL(kern, grid, block, lds, stream, A, B, C, Cpre, M, N, K, G, tiles_m, tiles_n,     \
                               gather, gather_rows);                                                        \
        } else {                                                                                            \
            auto kern = gemm_bf16_generic_kernel<BM, BN, ACTV, SAVE>;                                       \
            if (lds > 64 * 1024)                                                                            \
                (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                              \
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);            \
            hipLaunchKernelGGL(kern, grid, block, lds, stream, p);                                          \
        }                                                                                                   \
    } while (0)
#define EC_GEMM_CASE(ACTV)                                                                                  \
    if (Cpre) EC_GEMM_LAUNCH(ACTV, true);                                                                   \
    else EC_GEMM_LAUNCH(ACTV, false)
    if (act == EC_ACT_RELU) { EC_GEMM_CASE(EC_ACT_RELU); }
    else if (act == EC_ACT_GELU) { EC_GEMM_CASE(EC_ACT_GELU); }
    else { EC_GEMM_CASE(EC_ACT_IDENTITY); }
#undef EC_GEMM_CASE
#undef EC_GEMM_LAUNCH
}

// Tile configuration of a grouped product: the candidate with the lowest estimated time, taken as
// (rounds of 256 compute units) x (tile area) / (relative rate of that configuration).
static void gemm_bf16_dispatch(const bf16_t* A, const bf16_t* B, bf16_t* C, bf16_t* Cpre, int G, int M, int N,
                               int K, int act, const int32_t* gather, int gather_rows, hipStream_t stream) {
    auto cost = [&](int bm, int bn, int occ, double rate) {
        double tiles = (double)G * ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
        double rounds = std::ceil(tiles / (256.0 * occ)) * occ;
        return rounds * bm * bn / rate;
    };
    const double c0 = cost(256, 256, 1, 1.0), c1 = cost(256, 128, 1, 0.85), c2 = cost(128, 128, 2, 0.6);
    int pick = (c0 <= c1 && c0 <= c2) ? 0 : (c1 <= c2 ? 1 : 2);
    // Short contractions leave the epilogue (activation, stores) as large as the MFMA phase: two
    // co-resident 256 x 128 workgroups per compute unit overlap one's epilogue with the other's MFMAs.
    if (pick == 0 && K <= 1024 && cost(256, 128, 2, 1.0) <= 1.25 * c0) pick = 3;
    static const int forced = [] {  // tuning knob: EC_MOE_GEMM_TILE=0..3 forces one configuration
        const char* v = std::getenv("EC_MOE_GEMM_TILE");
        return v ? std::atoi(v) : -1;
    }();
    if (forced >= 0 && forced <= 3) pick = forced;
    switch (pick) {
        case 0: launch_gemm_bf16<256, 256, 2, 1>(A, B, C, Cpre, G, M, N, K, act, gather, gather_rows, stream); break;
        case 1: launch_gemm_bf16<256, 128, 2, 1>(A, B, C, Cpre, G, M, N, K, act, gather, gather_rows, stream); break;
        case 2: launch_gemm_bf16<128, 128, 1, 2>(A, B, C, Cpre, G, M, N, K, act, gather, gather_rows, stream); break;
        default: launch_gemm_bf16<256, 128, 1, 2>(A, B, C, Cpre, G, M, N, K, act, gather, gather_rows, stream); break;
    }
}

// ===========================================================================
// fp32 grouped GEMM, 64 x 64 tiles, 4 x 4 outputs per thread.
// ===========================================================================
template <int ACT, bool SAVE_PRE>
__global__ void __launch_bounds__(256)
gemm_f32_kernel(const float* __restrict__ Ag, const float* __restrict__ Bg, float* __restrict__ Cg,
                float* __restrict__ Cpreg, int M, int N, int K) {
    __shared__ float As[16][64 + 4];  // [k][m]
    __shared__ float Bs[16][64 + 4];  // [k][n]
    const int g = blockIdx.z;
    const float* A = Ag + (size_t)g * M * K;
    const float* B = Bg + (size_t)g * K * N;
    float* C = Cg + (size_t)g * M * N;
    float* Cpre = SAVE_PRE ? Cpreg + (size_t)g * M * N : nullptr;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int c = tid; c < 64 * 16; c += 256) {
            int m = c >> 4, kk = c & 15;  // A: consecutive threads walk the contraction axis
            int gm = m0 + m, gk = k0 + kk;
            As[kk][m] = (gm < M && gk < K) ? A[(size_t)gm * K + gk] : 0.0f;
            int kb = c >> 6, nn = c & 63;  // B: consecutive threads walk the column axis
            int gkb = k0 + kb, gn = n0 + nn;
            Bs[kb][nn] = (gkb < K && gn < N) ? B[(size_t)gkb * N + gn] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) { a[q] = As[kk][ty * 4 + q]; b[q] = Bs[kk][tx * 4 + q]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int gm = m0 + ty * 4 + i, gn = n0 + tx * 4 + j;
            if (gm < M && gn < N) {
                if (SAVE_PRE) Cpre[(size_t)gm * N + gn] = acc[i][j];
                C[(size_t)gm * N + gn] = apply_act<ACT>(acc[i][j]);
            }
        }
}

static void launch_gemm_f32(const float* A, const float* B, float* C, float* Cpre, int G, int M, int N, int K,
                            int act, hipStream_t stream) {
    dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64), (unsigned)G), block(256);
#define EC_SGEMM_CASE(ACTV)                                                                         \
    if (Cpre) hipLaunchKernelGGL((gemm_f32_kernel<ACTV, true>), grid, block, 0, stream, A, B, C, Cpre, M, N, K); \
    else hipLaunchKernelGGL((gemm_f32_kernel<ACTV, false>), grid, block, 0, stream, A, B, C, Cpre, M, N, K)
    if (act == EC_ACT_RELU) { EC_SGEMM_CASE(EC_ACT_RELU); }
    else if (act == EC_ACT_GELU) { EC_SGEMM_CASE(EC_ACT_GELU); }
    else { EC_SGEMM_CASE(EC_ACT_IDENTITY); }
#undef EC_SGEMM_CASE
}

// ---------------------------------------------------------------------------
// Xe = act(Xin.W1).W2 ; H is the [e,k,d_ff] hidden buffer (workspace or caller's).
// ---------------------------------------------------------------------------
// True when the first product can gather its rows straight from X (no X_in buffer needed).
bool ffn_can_gather(int dtype, int64_t n, int64_t k, int64_t d, int64_t d_ff) {
    return dtype == EC_BF16 && (d % GEMM_BK) == 0 && n * d * 2 < ((int64_t)1 << 31) - 65536 &&
           d * d_ff * 2 < ((int64_t)1 << 31) && k > 0;
}

// Xin == nullptr: gather mode, rows of the buckets are read from X through I (needs ffn_can_gather).
int launch_ffn(const void* Xin, const void* X, const int32_t* I, int64_t n, const void* W1, const void* W2, void* Xe,
               void* A_save, void* H, int64_t e, int64_t k, int64_t d, int64_t d_ff, int act, int dtype,
               hipStream_t stream) {
    const int G = (int)e, M = (int)k;
    if (dtype == EC_BF16) {
        if (Xin == nullptr)
            gemm_bf16_dispatch((const bf16_t*)X, (const bf16_t*)W1, (bf16_t*)H, (bf16_t*)A_save, G, M, (int)d_ff, (int)d,
                               act, I, (int)n, stream);
        else
            gemm_bf16_dispatch((const bf16_t*)Xin, (const bf16_t*)W1, (bf16_t*)H, (bf16_t*)A_save, G, M, (int)d_ff,
                               (int)d, act, nullptr, 0, stream);
        int rc = check_launch();
        if (rc != EC_OK) return rc;
        gemm_bf16_dispatch((const bf16_t*)H, (const bf16_t*)W2, (bf16_t*)Xe, nullptr, G, M, (int)d, (int)d_ff,
                           EC_ACT_IDENTITY, nullptr, 0, stream);
        return check_launch();
    }
    launch_gemm_f32((const float*)Xin, (const float*)W1, (float*)H, (float*)A_save, G, M, (int)d_ff, (int)d, act,
                    stream);
    int rc = check_launch();
    if (rc != EC_OK) return rc;
    launch_gemm_f32((const float*)H, (const float*)W2, (float*)Xe, nullptr, G, M, (int)d, (int)d_ff,
                    EC_ACT_IDENTITY, stream);
    return check_launch();
}

}  // namespace ecmoe
