// Expert FFN: X_e[i] = act(X_in[i].W1[i]).W2[i] for every expert i (Sec. 3.2, Eq. 3).
//
// Two grouped (one launch covers all experts) GEMMs: A = X_in.W1 with the
// activation fused into the epilogue, then X_e = H.W2.
//  * bf16: matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation, LDS-staged
//    tiles (gemm_bf16.h).  Both products are "row-major x row-major": the left
//    operand is contraction-contiguous and read from LDS as 16-byte fragments;
//    the right operand (the weights) keeps its own [k][columns] form in LDS and
//    its fragments come from transposing LDS reads.  Widths that are not
//    multiples of 64 take a predicated kernel that transposes the weight tile
//    in registers instead.
//  * fp32: plain FMA tiles (small parity configuration only).
#include <cmath>

#include "ec_common.h"
#include "gemm_bf16.h"

namespace ecmoe {

// ===========================================================================
// bf16 grouped GEMM on MFMA:  C[g] = epilogue(A[g] (M x K)  .  B[g] (K x N))
// ===========================================================================

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

// True when the matrix-core kernel covers the product (with rows gathered from a [gather_rows, K] matrix if asked).
static bool gemm_bf16_fast_ok(int64_t M, int64_t N, int64_t K, bool gather, int64_t gather_rows) {
    return gemm_bf16_shape_ok(M, N, K) && (!gather || gather_rows * K * 2 < ((int64_t)1 << 31) - 65536);
}

template <int BM, int BN, int STAGES, int OCC>
static int launch_gemm_bf16(const bf16_t* A, const bf16_t* B, bf16_t* C, bf16_t* Cpre, int G, int M, int N, int K,
                            int act, const int32_t* gather, int gather_rows, hipStream_t stream, bf16_t* Clo) {
    if (gemm_bf16_fast_ok(M, N, K, gather != nullptr, gather_rows)) {
#define EC_GEMM_CASE(ACTV)                                                                                       \
    if (Cpre) gemm_bf16_launch<BM, BN, STAGES, OCC, false, false, EPI_ACT_SAVE, ACTV>(                           \
                  A, B, C, Cpre, G, M, N, K, gather, gather_rows, stream, nullptr, nullptr, Clo);                \
    else gemm_bf16_launch<BM, BN, STAGES, OCC, false, false, EPI_ACT, ACTV>(A, B, C, nullptr, G, M, N, K, gather, \
                                                                           gather_rows, stream, nullptr, nullptr, Clo)
        if (act == EC_ACT_RELU) { EC_GEMM_CASE(EC_ACT_RELU); }
        else if (act == EC_ACT_GELU) { EC_GEMM_CASE(EC_ACT_GELU); }
        else { EC_GEMM_CASE(EC_ACT_IDENTITY); }
#undef EC_GEMM_CASE
        return check_launch();
    }
    // general shapes: predicated kernel, 128 x 128 tiles.  It reads its left operand as stored and writes one
    // output: a caller that asked for gathered rows or for the remainders gets an error instead of a wrong product.
    if (gather != nullptr || Clo != nullptr) return EC_ERR_UNSUPPORTED;
    if ((int64_t)M * K >= ((int64_t)1 << 31) || (int64_t)K * N >= ((int64_t)1 << 31) || (int64_t)M * N >= ((int64_t)1 << 31))
        return EC_ERR_UNSUPPORTED;
    constexpr int GBM = 128, GBN = 128;
    GemmArgs p;
    p.A = A; p.B = B; p.C = C; p.Cpre = Cpre;
    p.M = M; p.N = N; p.K = K; p.G = G;
    p.tiles_m = (M + GBM - 1) / GBM; p.tiles_n = (N + GBN - 1) / GBN;
    const int total = G * p.tiles_m * p.tiles_n;
    const size_t lds = (size_t)2 * (GBM + GBN) * GEMM_LDS_STRIDE * sizeof(bf16_t);
    dim3 grid((unsigned)((total + 7) / 8 * 8)), block(256);
#define EC_GEMM_CASE(ACTV)                                                                                       \
    do {                                                                                                         \
        auto k1 = gemm_bf16_generic_kernel<GBM, GBN, ACTV, true>;                                                \
        auto k0 = gemm_bf16_generic_kernel<GBM, GBN, ACTV, false>;                                               \
        auto kern = Cpre ? k1 : k0;                                                                              \
        static std::atomic<bool> allowed[2][64];                                                                 \
        gemm_allow_lds(reinterpret_cast<const void*>(kern), lds, allowed[Cpre ? 1 : 0]);                         \
        hipLaunchKernelGGL(kern, grid, block, lds, stream, p);                                                   \
    } while (0)
    if (act == EC_ACT_RELU) { EC_GEMM_CASE(EC_ACT_RELU); }
    else if (act == EC_ACT_GELU) { EC_GEMM_CASE(EC_ACT_GELU); }
    else { EC_GEMM_CASE(EC_ACT_IDENTITY); }
#undef EC_GEMM_CASE
    return check_launch();
}

// Tile configuration of a grouped product: the candidate with the lowest estimated time, taken as
// (rounds of 256 compute units) x (tile area) / (relative rate of that configuration).
static int gemm_tile_pick(int G, int M, int N, int K) {
    auto cost = [&](int bm, int bn, int occ, double rate) {
        double tiles = (double)G * ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
        double rounds = std::ceil(tiles / (256.0 * occ)) * occ;
        return rounds * bm * bn / rate;
    };
    const double c0 = cost(256, 256, 1, 1.0), c1 = cost(256, 128, 1, 0.85), c2 = cost(128, 128, 2, 0.6);
    const double c4 = cost(256, 192, 1, 0.95);  // fills the chip exactly when 256 x 256 tiles leave units idle
    int pick = (c0 <= c1 && c0 <= c2) ? 0 : (c1 <= c2 ? 1 : 2);
    if (c4 < c0 && c4 < c1 && c4 < c2) pick = 4;
    // Short contractions leave the epilogue (activation, stores) as large as the MFMA phase: 128 x 128 tiles, two
    // workgroups per compute unit, overlap one's epilogue with the other's MFMAs.  Measured with the GeLU epilogue:
    // K = 768 (16 x 1024 x 3072): 103 us against 105 (256 x 256) and 111 (256 x 128 pairs); from K = 1024 on
    // (64 x 512 x 4096) the 256 x 256 tile wins, 344 us against 356 and 369.
    if (pick == 0 && K <= 768 && cost(128, 128, 2, 1.0) <= 1.25 * c0) pick = 2;
    return pick;
}

// Clo (optional): receives act(acc) - C, the part of the activated value that the bf16 rounding of C dropped.
static int gemm_bf16_dispatch(const bf16_t* A, const bf16_t* B, bf16_t* C, bf16_t* Cpre, int G, int M, int N,
                              int K, int act, const int32_t* gather, int gather_rows, hipStream_t stream,
                              bf16_t* Clo = nullptr) {
    switch (gemm_tile_pick(G, M, N, K)) {
        case 1: return launch_gemm_bf16<256, 128, 2, 1>(A, B, C, Cpre, G, M, N, K, act, gather, gather_rows, stream, Clo);
        case 2: return launch_gemm_bf16<128, 128, 1, 2>(A, B, C, Cpre, G, M, N, K, act, gather, gather_rows, stream, Clo);
        case 4: return launch_gemm_bf16<256, 192, 2, 1>(A, B, C, Cpre, G, M, N, K, act, gather, gather_rows, stream, Clo);
        default: return launch_gemm_bf16<256, 256, 2, 1>(A, B, C, Cpre, G, M, N, K, act, gather, gather_rows, stream, Clo);
    }
}

// The second product of Eq. 3 with its left operand carried as high part + remainder (A + Alo): C32 (fp32) = the
// product unrounded, Cb (bf16, optional) = the same rounded.  The tile is chosen for the doubled contraction.
static int gemm_bf16_dispatch_split(const bf16_t* A, const bf16_t* Alo, const bf16_t* B, float* C32, bf16_t* Cb, int G,
                                    int M, int N, int K, hipStream_t stream) {
    if (!gemm_bf16_shape_ok(M, N, K)) return EC_ERR_UNSUPPORTED;
#define EC_SPLIT_CASE(BM, BN, ST, OCC)                                                                              \
    gemm_bf16_launch<BM, BN, ST, OCC, false, false, EPI_F32, EC_ACT_IDENTITY, SPLIT_LEFT>(A, B, C32, nullptr, G, M, N, K, \
                                                                                         nullptr, 0, stream, nullptr, Alo, Cb)
    switch (gemm_tile_pick(G, M, N, 2 * K)) {
        case 1: EC_SPLIT_CASE(256, 128, 2, 1); break;
        case 2: EC_SPLIT_CASE(128, 128, 1, 2); break;
        case 4: EC_SPLIT_CASE(256, 192, 2, 1); break;
        default: EC_SPLIT_CASE(256, 256, 2, 1); break;
    }
#undef EC_SPLIT_CASE
    return check_launch();
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

static int launch_gemm_f32(const float* A, const float* B, float* C, float* Cpre, int G, int M, int N, int K,
                           int act, hipStream_t stream) {
    if ((M + 63) / 64 > 65535 || G > 65535) return EC_ERR_UNSUPPORTED;  // grid.y / grid.z limits
    dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64), (unsigned)G), block(256);
#define EC_SGEMM_CASE(ACTV)                                                                         \
    if (Cpre) hipLaunchKernelGGL((gemm_f32_kernel<ACTV, true>), grid, block, 0, stream, A, B, C, Cpre, M, N, K); \
    else hipLaunchKernelGGL((gemm_f32_kernel<ACTV, false>), grid, block, 0, stream, A, B, C, Cpre, M, N, K)
    if (act == EC_ACT_RELU) { EC_SGEMM_CASE(EC_ACT_RELU); }
    else if (act == EC_ACT_GELU) { EC_SGEMM_CASE(EC_ACT_GELU); }
    else { EC_SGEMM_CASE(EC_ACT_IDENTITY); }
#undef EC_SGEMM_CASE
    return check_launch();
}

// ---------------------------------------------------------------------------
// Xe = act(Xin.W1).W2 ; H is the [e,k,d_ff] hidden buffer (workspace or caller's).
// ---------------------------------------------------------------------------
// True when the first product can gather its rows straight from X (no X_in buffer needed).
// It is used only while X is small (16 MiB: it then stays in the L2 caches): the tile loader reads every bucket row
// once per column of tiles, and rows scattered over a large X cost more there than one pass of the dispatch kernel
// (measured: 8192 x 768 tokens, gathered product 99 us against 103 + 13 for the dispatch; 16384 x 1024 tokens,
// 383 us against 344 + 25).
bool ffn_can_gather(int dtype, int64_t n, int64_t k, int64_t d, int64_t d_ff) {
    return dtype == EC_BF16 && k > 0 && n * d * 2 <= ((int64_t)16 << 20) && gemm_bf16_fast_ok(k, d_ff, d, true, n);
}


// True when the products can carry H as high part + remainder (the matrix-core kernel covers both shapes).
bool ffn_can_hilo(int dtype, int64_t k, int64_t d, int64_t d_ff) {
    return dtype == EC_BF16 && k > 0 && gemm_bf16_shape_ok(k, d_ff, d) && gemm_bf16_shape_ok(k, d, d_ff);
}

// Xin == nullptr: gather mode, rows of the buckets are read from X through I (needs ffn_can_gather).
// H_lo / Xe32 (both or neither; need ffn_can_hilo): the first product also leaves H_lo = act(A) - H, the second
// multiplies (H + H_lo) by W2 and writes X_e unrounded to Xe32 [e,k,d] (fp32), and rounded to Xe if Xe is given.
int launch_ffn(const void* Xin, const void* X, const int32_t* I, int64_t n, const void* W1, const void* W2, void* Xe,
               void* A_save, void* H, int64_t e, int64_t k, int64_t d, int64_t d_ff, int act, int dtype,
               hipStream_t stream, void* H_lo, float* Xe32) {
    const int G = (int)e, M = (int)k;
    if (dtype == EC_BF16) {
        int rc;
        if (Xin == nullptr)
            rc = gemm_bf16_dispatch((const bf16_t*)X, (const bf16_t*)W1, (bf16_t*)H, (bf16_t*)A_save, G, M, (int)d_ff,
                                    (int)d, act, I, (int)n, stream, (bf16_t*)H_lo);
        else
            rc = gemm_bf16_dispatch((const bf16_t*)Xin, (const bf16_t*)W1, (bf16_t*)H, (bf16_t*)A_save, G, M, (int)d_ff,
                                    (int)d, act, nullptr, 0, stream, (bf16_t*)H_lo);
        if (rc != EC_OK) return rc;
        if (H_lo != nullptr)
            return gemm_bf16_dispatch_split((const bf16_t*)H, (const bf16_t*)H_lo, (const bf16_t*)W2, Xe32, (bf16_t*)Xe, G,
                                            M, (int)d, (int)d_ff, stream);
        return gemm_bf16_dispatch((const bf16_t*)H, (const bf16_t*)W2, (bf16_t*)Xe, nullptr, G, M, (int)d, (int)d_ff,
                                  EC_ACT_IDENTITY, nullptr, 0, stream);
    }
    if (Xin == nullptr || H_lo != nullptr) return EC_ERR_UNSUPPORTED;
    int rc = launch_gemm_f32((const float*)Xin, (const float*)W1, (float*)H, (float*)A_save, G, M, (int)d_ff, (int)d, act,
                             stream);
    if (rc != EC_OK) return rc;
    return launch_gemm_f32((const float*)H, (const float*)W2, (float*)Xe, nullptr, G, M, (int)d, (int)d_ff,
                           EC_ACT_IDENTITY, stream);
}

}  // namespace ecmoe
