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

// BM x BN block tile, 4 wavefronts arranged WR x WC, each computing
// (BM/WR) x (BN/WC) as TM x TN MFMA tiles of 32 x 32.
template <int BM, int BN, int WR, int WC, int ACT, bool SAVE_PRE>
__global__ void __launch_bounds__(256)
gemm_bf16_kernel(GemmArgs p) {
    static_assert(WR * WC == 4, "four wavefronts");
    constexpr int TM = BM / WR / 32, TN = BN / WC / 32;
    constexpr int A_CHUNKS = BM * 8 / 256;        // 16-byte chunks of the A tile per thread
    constexpr int B_BLOCKS = (GEMM_BK / 4) * (BN / 8) / 256;  // 4(k) x 8(n) sub-blocks of the B tile per thread
    static_assert(A_CHUNKS >= 1 && B_BLOCKS >= 1, "tile too small");

    __shared__ __attribute__((aligned(16))) bf16_t As[BM * GEMM_LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[BN * GEMM_LDS_STRIDE];  // transposed: [n][k]

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
    const int wr = wave / WC, wc = wave % WC;
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
            int kg = blk & 15, ng = blk >> 4;      // 16 k-groups of 4 rows, BN/8 n-groups of 8 columns
            int gn = n0 + ng * 8;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int gk = k0 + kg * 4 + q;
                breg[r][q] = (gk < K && gn < N) ? *reinterpret_cast<const uint4*>(B + (size_t)gk * N + gn) : zero4;
            }
        }
    };
    auto store_tiles = [&]() {
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
    for (int kc = 0; kc < nk; ++kc) {
        __syncthreads();
        store_tiles();
        __syncthreads();
        if (kc + 1 < nk) load_tiles((kc + 1) * GEMM_BK);
#pragma unroll
        for (int s = 0; s < GEMM_BK / 16; ++s) {
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(
                    &As[(wr * TM * 32 + i * 32 + col) * GEMM_LDS_STRIDE + s * 16 + half * 8]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8*>(
                    &Bs[(wc * TN * 32 + j * 32 + col) * GEMM_LDS_STRIDE + s * 16 + half * 8]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
    }

    // Epilogue.  acc[i][j][r] is C[row = 8*(r/4) + 4*half + r%4][column = col] of its 32 x 32 tile.
    bf16_t* __restrict__ C = p.C + (size_t)g * M * N;
    bf16_t* __restrict__ Cpre = SAVE_PRE ? p.Cpre + (size_t)g * M * N : nullptr;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int gn = n0 + wc * TN * 32 + j * 32 + col;
            const int mbase = m0 + wr * TM * 32 + i * 32 + 4 * half;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int gm = mbase + 8 * (r >> 2) + (r & 3);
                if (gm < M && gn < N) {
                    float v = acc[i][j][r];
                    if (SAVE_PRE) Cpre[(size_t)gm * N + gn] = static_cast<bf16_t>(v);
                    C[(size_t)gm * N + gn] = static_cast<bf16_t>(apply_act<ACT>(v));
                }
            }
        }
}

template <int BM, int BN, int WR, int WC>
static void launch_gemm_bf16(const bf16_t* A, const bf16_t* B, bf16_t* C, bf16_t* Cpre, int G, int M, int N, int K,
                             int act, hipStream_t stream) {
    GemmArgs p;
    p.A = A; p.B = B; p.C = C; p.Cpre = Cpre;
    p.M = M; p.N = N; p.K = K; p.G = G;
    p.tiles_m = (M + BM - 1) / BM;
    p.tiles_n = (N + BN - 1) / BN;
    const int total = G * p.tiles_m * p.tiles_n;
    dim3 grid((unsigned)((total + 7) / 8 * 8)), block(256);
#define EC_GEMM_CASE(ACTV)                                                                                  \
    if (Cpre) hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WR, WC, ACTV, true>), grid, block, 0, stream, p); \
    else hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WR, WC, ACTV, false>), grid, block, 0, stream, p)
    if (act == EC_ACT_RELU) { EC_GEMM_CASE(EC_ACT_RELU); }
    else if (act == EC_ACT_GELU) { EC_GEMM_CASE(EC_ACT_GELU); }
    else { EC_GEMM_CASE(EC_ACT_IDENTITY); }
#undef EC_GEMM_CASE
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
int launch_ffn(const void* Xin, const void* W1, const void* W2, void* Xe, void* A_save, void* H,
               int64_t e, int64_t k, int64_t d, int64_t d_ff, int act, int dtype, hipStream_t stream) {
    const int G = (int)e, M = (int)k;
    if (dtype == EC_BF16) {
        launch_gemm_bf16<128, 128, 2, 2>((const bf16_t*)Xin, (const bf16_t*)W1, (bf16_t*)H, (bf16_t*)A_save, G, M,
                                         (int)d_ff, (int)d, act, stream);
        int rc = check_launch();
        if (rc != EC_OK) return rc;
        launch_gemm_bf16<128, 128, 2, 2>((const bf16_t*)H, (const bf16_t*)W2, (bf16_t*)Xe, nullptr, G, M, (int)d,
                                         (int)d_ff, EC_ACT_IDENTITY, stream);
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
