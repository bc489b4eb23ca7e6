// Backward of the expert-choice layer: gradient of <dY, X_out> through Sec. 3.2, Eq. 2-4 with the TopK
// selection I held constant and the gate values G = S[I[i,j], i] differentiable (Sec. 3.4: the gating
// network is trained through the top-k function).  With r = (i,j) a bucket row and l = I[i,j]:
//   dX_e[r,:] = G[r] dY[l,:]                 dG[r]  = <dY[l,:], X_e[r,:]>               (Eq. 4)
//   dW2[i] = H[i]^T dX_e[i]                  dH[r,:] = dX_e[r,:] W2[i]^T = G[r] (dY[l,:] W2[i]^T)
//   dA = dH * act'(A)                        dW1[i] = X_in[i]^T dA[i]    dX_in[i] = dA[i] W1[i]^T   (Eq. 3)
//   dS[l,i] = dG[r] on selected pairs, else 0;  dZ[l,:] = S[l,:] * (dS[l,:] - <dS[l,:], S[l,:]>)   (softmax)
//   dWg = X^T dZ                             dX[l,:] = dZ[l,:] Wg^T + sum_{r: I[r]=l} dX_in[r,:]   (Eq. 2, 3)
// bf16 with d, d_ff multiples of 64: the four expert products run on the matrix cores (gemm_bf16.h);
// everything else, and fp32, uses a plain tiled FMA kernel.  Sums over a token's experts run in
// ascending expert order, sums over tokens in fixed split order: no floating-point atomics.
#include "ec_common.h"
#include "gemm_bf16.h"

namespace ecmoe {

// ---------------------------------------------------------------------------
// dX_e and dG: one wavefront per bucket row.
// ---------------------------------------------------------------------------
template <typename T, int VEC, typename TOut>
__global__ void __launch_bounds__(256)
bwd_rows_kernel(const T* __restrict__ dY, const T* __restrict__ Xe, const float* __restrict__ G,
                const int32_t* __restrict__ I, TOut* __restrict__ dXe, float* __restrict__ dG, long long rows, int d,
                TOut* __restrict__ dXe_lo) {  // dXe_lo (optional): G dY - dXe, what the rounding of dXe dropped
    typedef T vec_t __attribute__((ext_vector_type(VEC)));  // VEC elements = 16 bytes when the rows allow it
    typedef TOut ovec_t __attribute__((ext_vector_type(VEC)));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nvec = d / VEC;
    for (long long r = (long long)blockIdx.x * 4 + wave; r < rows; r += (long long)gridDim.x * 4) {
        const int tok = I[r];  // -1: an empty buffer row (token-choice routing) fed nothing: zero gradient
        const vec_t* src = reinterpret_cast<const vec_t*>(dY + (size_t)(tok < 0 ? 0 : tok) * d);
        const vec_t* xe = reinterpret_cast<const vec_t*>(Xe + (size_t)r * d);
        ovec_t* dst = reinterpret_cast<ovec_t*>(dXe + (size_t)r * d);
        ovec_t* dst_lo = dXe_lo != nullptr ? reinterpret_cast<ovec_t*>(dXe_lo + (size_t)r * d) : nullptr;
        const float g = tok < 0 ? 0.0f : G[r];
        float dot = 0.0f;
        for (int t = lane; t < nvec; t += kWave) {
            const vec_t y = src[t], x = xe[t];
            ovec_t o, lo;
#pragma unroll
            for (int q = 0; q < VEC; ++q) {
                const float yf = Cvt<T>::to_f32(y[q]);
                dot = fmaf(yf, Cvt<T>::to_f32(x[q]), dot);
                o[q] = Cvt<TOut>::from_f32(g * yf);
                lo[q] = Cvt<TOut>::from_f32(g * yf - Cvt<TOut>::to_f32(o[q]));
            }
            dst[t] = o;
            if (dst_lo != nullptr) dst_lo[t] = lo;
        }
        dot = wave_reduce_sum(dot);
        if (lane == 0) dG[r] = tok < 0 ? 0.0f : dot;
    }
}

// ---------------------------------------------------------------------------
// Softmax backward per token (one wavefront per token).  The token's selected pairs come from its
// expert-ascending row list; dZ is written densely as fp32 [n,e] and, optionally, as bf16.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
bwd_dz_kernel(const float* __restrict__ S, const float* __restrict__ dG, const int32_t* __restrict__ offsets,
              const int32_t* __restrict__ inv, float* __restrict__ dZ, bf16_t* __restrict__ dZb, int n, int e, int k) {
    __shared__ float ds[4][EC_MOE_MAX_EXPERTS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int base = blockIdx.x * 4; base < n; base += gridDim.x * 4) {
        const int l = base + wave;
        const bool active = l < n;
        for (int i = lane; i < e; i += kWave) ds[wave][i] = 0.0f;
        __syncthreads();
        float dot = 0.0f;
        if (active) {
            const int beg = offsets[l], end = offsets[l + 1];
            for (int p = beg + lane; p < end; p += kWave) {
                const int r = inv[p];
                const int i = r / k;
                const float v = dG[r];
                ds[wave][i] = v;  // a token appears at most once per expert
                dot = fmaf(v, S[(size_t)l * e + i], dot);
            }
        }
        dot = wave_reduce_sum(dot);
        __syncthreads();
        if (active) {
            for (int i = lane; i < e; i += kWave) {
                const float z = S[(size_t)l * e + i] * (ds[wave][i] - dot);
                dZ[(size_t)l * e + i] = z;
                if (dZb != nullptr) {  // z = hi + lo with both in bf16 (error 2^-17 |z|), row layout [hi(e) | lo(e)]
                    const bf16_t hi = static_cast<bf16_t>(z);
                    dZb[(size_t)l * 2 * e + i] = hi;
                    dZb[(size_t)l * 2 * e + e + i] = static_cast<bf16_t>(z - static_cast<float>(hi));
                }
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Plain tiled FMA GEMM, any shape: C[g] = opA(A[g]) . opB(B[g]) (+ epilogue), fp32 accumulation.
//   TRA: A[g] stored [K][M] instead of [M][K];  TRB: B[g] stored [N][K] instead of [K][N].
//   MULGRAD: C = acc * act'(aux[m][n]).
// ---------------------------------------------------------------------------
template <typename TA, typename TB, typename TC, bool TRA, bool TRB, bool MULGRAD, int ACT, typename TAux = TC>
__global__ void __launch_bounds__(256)
gemm_plain_kernel(const TA* __restrict__ Ag, const TB* __restrict__ Bg, TC* __restrict__ Cg,
                  const TAux* __restrict__ auxg, int M, int N, int K, long long sA, long long sB, long long sC) {
    __shared__ float As[16][64 + 4];  // [k][m]
    __shared__ float Bs[16][64 + 4];  // [k][n]
    const int g = blockIdx.z;
    const TA* A = Ag + (size_t)g * sA;
    const TB* B = Bg + (size_t)g * sB;
    TC* C = Cg + (size_t)g * sC;
    const TAux* aux = MULGRAD ? auxg + (size_t)g * sC : nullptr;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int c = tid; c < 64 * 16; c += 256) {
            {   // A tile: walk the contiguous axis with consecutive threads
                const int m = TRA ? (c & 63) : (c >> 4), kk = TRA ? (c >> 6) : (c & 15);
                const int gm = m0 + m, gk = k0 + kk;
                float v = 0.0f;
                if (gm < M && gk < K) v = Cvt<TA>::to_f32(TRA ? A[(size_t)gk * M + gm] : A[(size_t)gm * K + gk]);
                As[kk][m] = v;
            }
            {
                const int nn = TRB ? (c >> 4) : (c & 63), kk = TRB ? (c & 15) : (c >> 6);
                const int gn = n0 + nn, gk = k0 + kk;
                float v = 0.0f;
                if (gn < N && gk < K) v = Cvt<TB>::to_f32(TRB ? B[(size_t)gn * K + gk] : B[(size_t)gk * N + gn]);
                Bs[kk][nn] = v;
            }
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
            const int gm = m0 + ty * 4 + i, gn = n0 + tx * 4 + j;
            if (gm < M && gn < N) {
                float v = acc[i][j];
                if (MULGRAD) {
                    const float a = Cvt<TAux>::to_f32(aux[(size_t)gm * N + gn]);
                    float gr = 1.0f;
                    if (ACT == EC_ACT_RELU) gr = a > 0.0f ? 1.0f : 0.0f;
                    if (ACT == EC_ACT_GELU) {
                        const float Phi = 0.5f * (1.0f + erff(a * 0.70710678118654752440f));
                        gr = Phi + a * 0.39894228040143267794f * expf(-0.5f * a * a);
                    }
                    v *= gr;
                }
                C[(size_t)gm * N + gn] = Cvt<TC>::from_f32(v);
            }
        }
}

// grid.y carries the row tiles and grid.z the groups: both are limited to 65535
static bool plain_grid_ok(int G, int M) { return (M + 63) / 64 <= 65535 && G <= 65535; }

template <typename TA, typename TB, typename TC, bool TRA, bool TRB>
static int gemm_plain(const TA* A, const TB* B, TC* C, int G, int M, int N, int K, long long sA, long long sB,
                      long long sC, hipStream_t stream) {
    if (!plain_grid_ok(G, M)) return EC_ERR_UNSUPPORTED;
    dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64), (unsigned)G);
    hipLaunchKernelGGL((gemm_plain_kernel<TA, TB, TC, TRA, TRB, false, EC_ACT_IDENTITY>), grid, dim3(256), 0, stream, A, B,
                       C, (const TC*)nullptr, M, N, K, sA, sB, sC);
    return EC_OK;
}
template <typename T>
static int gemm_plain_mulgrad(const float* A, const T* B, float* C, const T* aux, int G, int M, int N, int K, int act,
                              hipStream_t stream) {  // A [M][K] fp32, B stored [N][K]
    if (!plain_grid_ok(G, M)) return EC_ERR_UNSUPPORTED;
    dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64), (unsigned)G);
    const long long sA = (long long)M * K, sB = (long long)N * K, sC = (long long)M * N;
    if (act == EC_ACT_RELU)
        hipLaunchKernelGGL((gemm_plain_kernel<float, T, float, false, true, true, EC_ACT_RELU, T>), grid, dim3(256), 0,
                           stream, A, B, C, aux, M, N, K, sA, sB, sC);
    else if (act == EC_ACT_GELU)
        hipLaunchKernelGGL((gemm_plain_kernel<float, T, float, false, true, true, EC_ACT_GELU, T>), grid, dim3(256), 0,
                           stream, A, B, C, aux, M, N, K, sA, sB, sC);
    else
        hipLaunchKernelGGL((gemm_plain_kernel<float, T, float, false, true, true, EC_ACT_IDENTITY, T>), grid, dim3(256), 0,
                           stream, A, B, C, aux, M, N, K, sA, sB, sC);
    return EC_OK;
}

// Sum of `splits` partial [rows] vectors in split order.
__global__ void __launch_bounds__(256)
reduce_splits_kernel(const float* __restrict__ part, float* __restrict__ out, long long count, int splits) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < count; i += (long long)gridDim.x * 256) {
        float s = 0.0f;
        for (int p = 0; p < splits; ++p) s += part[(size_t)p * count + i];
        out[i] = s;
    }
}

// Partials laid out [splits][d][2e] (products with the high and the low half of dZ side by side):
// out[t][i] = sum over splits, in split order, of (part[s][t][i] + part[s][t][e + i]).
__global__ void __launch_bounds__(256)
reduce_splits_halves_kernel(const float* __restrict__ part, float* __restrict__ out, int d, int e, int splits) {
    const long long count = (long long)d * e;
    for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < count; q += (long long)gridDim.x * 256) {
        const long long t = q / e, i = q % e;
        float s = 0.0f;
        for (int p = 0; p < splits; ++p) {
            const float* row = part + ((size_t)p * d + t) * 2 * e;
            s += row[i] + row[e + i];
        }
        out[q] = s;
    }
}

// Wg2[t][:] = [Wg[t][:] | Wg[t][:]]: the other operand of the product with [hi | lo].
__global__ void __launch_bounds__(256)
duplicate_columns_kernel(const bf16_t* __restrict__ Wg, bf16_t* __restrict__ Wg2, int d, int e) {
    const long long count = (long long)d * e;
    for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < count; q += (long long)gridDim.x * 256) {
        const long long t = q / e, i = q % e;
        const bf16_t v = Wg[q];
        Wg2[t * 2 * e + i] = v;
        Wg2[t * 2 * e + e + i] = v;
    }
}

// ---------------------------------------------------------------------------
// Workspace of the backward pass (after the forward layout, at L.bwd).
// ---------------------------------------------------------------------------
struct BwdLayout {
    size_t dxe, dxe_lo, dg, da, da_lo, dxin, dz, dzb, dxz, wg_part, wg2, total;
    int splits;
    int64_t split_len;
    bool mfma;  // the four expert products run on the matrix cores
};

static BwdLayout bwd_layout(int64_t n, int64_t d, int64_t e, int64_t k, int64_t d_ff, int dtype, bool hilo) {
    BwdLayout B;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t a = off; off = align_up(off + bytes, 256); return a; };
    B.split_len = 512;  // tokens per partial sum of dWg
    B.splits = (int)ceil_div(n, B.split_len);
    // matrix-core path: bf16, contraction-contiguous operands need d, d_ff % 64 == 0, the rows of dY are gathered
    // through one buffer descriptor
    B.mfma = dtype == EC_BF16 && gemm_bf16_shape_ok(k, d_ff, d) && gemm_bf16_shape_ok(k, d, d_ff) &&
             gemm_bf16_shape_ok(d_ff, d, k, false, true) && gemm_bf16_shape_ok(d, d_ff, k, false, true) &&
             n * d * 2 < ((int64_t)1 << 31) - 65536;
    // Intermediates: bf16 where they are matrix-core operands (dA as high part + remainder), fp32 on the plain path.
    const size_t is = B.mfma ? 2 : 4;
    B.dxe = take((size_t)e * k * d * is);
    B.dxe_lo = take((B.mfma && hilo) ? (size_t)e * k * d * 2 : 0);
    B.dg = take((size_t)e * k * 4);
    B.da = take((size_t)e * k * d_ff * is);
    B.da_lo = take(B.mfma ? (size_t)e * k * d_ff * 2 : 0);
    B.dxin = take((size_t)e * k * d * 4);  // fp32 on both paths: it is only summed into dX
    B.dz = take((size_t)n * e * 4);
    B.dzb = take((size_t)n * e * 2 * 2);                   // [n][hi | lo]
    B.dxz = take((size_t)n * d * 4);
    B.wg_part = take((size_t)B.splits * d * e * 2 * 4);    // [splits][d][2e] on the matrix-core path
    B.wg2 = take((size_t)d * e * 2 * 2);
    B.total = off;
    return B;
}

size_t bwd_ws_bytes(int64_t n, int64_t d, int64_t e, int64_t k, int64_t d_ff, int dtype, bool hilo) {
    return bwd_layout(n, d, e, k, d_ff, dtype, hilo).total;
}

template <typename T>
static int backward_typed(const T* dY, const T* X, const T* Wg, const T* W1, const T* W2, const float* S, const float* G,
                          const int32_t* I, const T* Xin, const T* A, const T* H, const T* Xe, T* dX, float* dWg,
                          float* dW1, float* dW2, int64_t n, int64_t d, int64_t e, int64_t k, int64_t d_ff, int act,
                          int dtype, void* ws, const WsLayout& L, hipStream_t stream, hipEvent_t* marks, bool hilo) {
    // marks (optional, BWD_STAGES + 1 events): recorded on the stream before the first stage and after every stage
    int mark_at = 0;
    auto mark = [&]() {
        if (marks != nullptr) (void)hipEventRecord(marks[mark_at], stream);
        ++mark_at;
    };
    mark();
    unsigned char* base = static_cast<unsigned char*>(ws) + L.bwd;
    const BwdLayout B = bwd_layout(n, d, e, k, d_ff, dtype, hilo);
    if (hilo && !B.mfma) return EC_ERR_UNSUPPORTED;  // the two-part operands exist on the matrix-core path only
    float* dG = reinterpret_cast<float*>(base + B.dg);
    float* dXin = reinterpret_cast<float*>(base + B.dxin);
    float* dZ = reinterpret_cast<float*>(base + B.dz);
    bf16_t* dZb = reinterpret_cast<bf16_t*>(base + B.dzb);
    float* dXz = reinterpret_cast<float*>(base + B.dxz);
    float* wg_part = reinterpret_cast<float*>(base + B.wg_part);
    const long long rows = (long long)e * k;
    const int Gn = (int)e, Mk = (int)k, D = (int)d, F = (int)d_ff;
    constexpr bool BF = sizeof(T) == 2;
    const bool mfma = BF && B.mfma;

    // Matrix-core path for the two gate products (dWg = X^T dZ, dZ Wg^T): whole splits of 512 tokens, experts
    // a multiple of 32 (the contraction of the second product is 2e), 16-byte rows.  dZ enters as hi + lo,
    // two bf16 numbers per value, so the products see it to 2^-17: dZ is a gradient of the fp32 scores and a
    // single bf16 rounding would cost a third of the error budget of dWg.
    const bool mfma_gate = BF && (n % B.split_len) == 0 && (e % 32) == 0 && (d % 8) == 0 &&
                           gemm_bf16_shape_ok(d, 2 * e, B.split_len, false, true) && gemm_bf16_shape_ok(n, d, 2 * e);
    bf16_t* Wg2 = reinterpret_cast<bf16_t*>(base + B.wg2);

    // Eq. 4 backwards: dX_e, dG (dX_e in bf16 as a matrix-core operand, in fp32 on the plain path)
    {
        long long blocks = ceil_div(rows, 4);
        if (blocks > (1 << 20)) blocks = 1 << 20;
        constexpr int V16 = 16 / (int)sizeof(T);
        const dim3 grid((unsigned)blocks), block(256);
        void* dXe = base + B.dxe;
        if (mfma) {
            T* dXe_lo = hilo ? reinterpret_cast<T*>(base + B.dxe_lo) : nullptr;
            if (d % V16 == 0)
                hipLaunchKernelGGL((bwd_rows_kernel<T, V16, T>), grid, block, 0, stream, dY, Xe, G, I, (T*)dXe, dG, rows, D,
                                   dXe_lo);
            else
                hipLaunchKernelGGL((bwd_rows_kernel<T, 1, T>), grid, block, 0, stream, dY, Xe, G, I, (T*)dXe, dG, rows, D,
                                   dXe_lo);
        } else {
            if (d % V16 == 0)
                hipLaunchKernelGGL((bwd_rows_kernel<T, V16, float>), grid, block, 0, stream, dY, Xe, G, I, (float*)dXe, dG,
                                   rows, D, (float*)nullptr);
            else
                hipLaunchKernelGGL((bwd_rows_kernel<T, 1, float>), grid, block, 0, stream, dY, Xe, G, I, (float*)dXe, dG,
                                   rows, D, (float*)nullptr);
        }
    }
    mark();  // 0: rows
    // Eq. 3 backwards
    if (mfma) {
        if constexpr (BF) {
            const bf16_t *bdXe = reinterpret_cast<const bf16_t*>(base + B.dxe), *bH = (const bf16_t*)H,
                         *bXin = (const bf16_t*)Xin;
            bf16_t* dA = reinterpret_cast<bf16_t*>(base + B.da);       // high part: bf16(dA)
            bf16_t* dAlo = reinterpret_cast<bf16_t*>(base + B.da_lo);  // remainder: bf16(dA - high part)
            // dW2[i] = H[i]^T dX_e[i]     (A stored [k][d_ff], B [k][d]) -> fp32 [d_ff][d]; with the two-part dX_e the
            // contraction runs over its high part and its remainder
            if (hilo)
                gemm_bf16_launch<256, 256, 2, 1, true, false, EPI_F32, EC_ACT_IDENTITY, SPLIT_RIGHT>(
                    bH, bdXe, dW2, nullptr, Gn, F, D, Mk, nullptr, 0, stream, nullptr,
                    reinterpret_cast<const bf16_t*>(base + B.dxe_lo), nullptr);
            else
                gemm_bf16_launch<256, 256, 2, 1, true, false, EPI_F32, EC_ACT_IDENTITY>(bH, bdXe, dW2, nullptr, Gn, F, D, Mk,
                                                                                        nullptr, 0, stream);
            mark();  // 1: dW2
            // dA[i] = (dX_e[i] W2[i]^T) * act'(A[i]) with dX_e[r,:] = G[r] dY[I[r],:]: the rows of dY are gathered by
            // the tile loader (exact bf16 operands) and G[r] multiplies the fp32 result in the epilogue, so dA -- and
            // through it dX -- does not inherit the bf16 rounding of dX_e   (B = W2 stored [d_ff][d] = [N][K]).
            // The epilogue also keeps what the bf16 rounding of dA drops (dAlo), for the product that feeds dX.
#define EC_BWD_DA(ACTV)                                                                                              \
    gemm_bf16_launch<256, 256, 2, 1, false, true, EPI_MULGRAD, ACTV>((const bf16_t*)dY, (const bf16_t*)W2, dA, (void*)A, \
                                                                     Gn, Mk, F, D, I, (int)n, stream, G, nullptr, dAlo)
            if (act == EC_ACT_RELU) EC_BWD_DA(EC_ACT_RELU);
            else if (act == EC_ACT_GELU) EC_BWD_DA(EC_ACT_GELU);
            else EC_BWD_DA(EC_ACT_IDENTITY);
#undef EC_BWD_DA
            mark();  // 2: dA
            // dW1[i] = X_in[i]^T dA[i]    -> fp32 [d][d_ff]
            gemm_bf16_launch<256, 256, 2, 1, true, false, EPI_F32, EC_ACT_IDENTITY>(bXin, (const bf16_t*)dA, dW1, nullptr, Gn,
                                                                                    D, F, Mk, nullptr, 0, stream);
            mark();  // 3: dW1
            // dX_in[i] = (dA[i] + dAlo[i]) W1[i]^T    (B = W1 stored [d][d_ff] = [N][K]); kept in fp32: it is only
            // summed into dX.  A token's gradient row scales with its gate value while the error bar is relative to
            // the whole tensor, so a single bf16 rounding of dA (2^-9) is what decides the worst element of dX;
            // with the remainder the product sees dA to 2^-17, at twice the work of this one product.
            gemm_bf16_launch<256, 256, 2, 1, false, true, EPI_F32, EC_ACT_IDENTITY, SPLIT_LEFT>(
                (const bf16_t*)dA, (const bf16_t*)W1, dXin, nullptr, Gn, Mk, D, F, nullptr, 0, stream, nullptr, dAlo, nullptr);
            mark();  // 4: dX_in
        }
    } else {
        // plain path: every intermediate (dX_e, dA, dX_in) stays in fp32
        const float* dXe = reinterpret_cast<const float*>(base + B.dxe);
        float* dA = reinterpret_cast<float*>(base + B.da);
        int prc = gemm_plain<T, float, float, true, false>(H, dXe, dW2, Gn, F, D, Mk, (long long)k * d_ff, (long long)k * d,
                                                           (long long)d_ff * d, stream);
        mark();
        if (prc == EC_OK) prc = gemm_plain_mulgrad<T>(dXe, W2, dA, A, Gn, Mk, F, D, act, stream);
        mark();
        if (prc == EC_OK)
            prc = gemm_plain<T, float, float, true, false>(Xin, dA, dW1, Gn, D, F, Mk, (long long)k * d,
                                                           (long long)k * d_ff, (long long)d * d_ff, stream);
        mark();
        if (prc == EC_OK)
            prc = gemm_plain<float, T, float, false, true>(dA, W1, dXin, Gn, Mk, D, F, (long long)k * d_ff,
                                                           (long long)d * d_ff, (long long)k * d, stream);
        mark();
        if (prc != EC_OK) return prc;
    }
    int rc = check_launch();
    if (rc != EC_OK) return rc;

    // token-major row lists (CSR form, expert-ascending) rebuilt from I
    CombineIndex ix = combine_index_at(ws, L, e);
    ix.use_slots = false;
    rc = launch_combine_index(I, n, e, k, ix, stream);
    if (rc != EC_OK) return rc;
    rc = launch_combine_csr(I, n, e, k, ix, stream);
    if (rc != EC_OK) return rc;
    mark();  // 5: token-major index

    // Eq. 2 backwards: dZ, then dWg = X^T dZ (fixed-order split sums) and the dense part of dX
    {
        long long blocks = ceil_div(n, 4);
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(bwd_dz_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, S, dG, ix.offsets, ix.inv, dZ,
                           mfma_gate ? dZb : (bf16_t*)nullptr, (int)n, (int)e, (int)k);
    }
    mark();  // 6: dZ
    if (mfma_gate) {
        if constexpr (BF) {
            // partial[s] = X[s*512 ..]^T [hi | lo][s*512 ..]: one group per split, both operands row-indexed
            // by the token; the fixed-order sum over the splits folds the two halves
            gemm_bf16_launch<256, 128, 2, 1, true, false, EPI_F32, EC_ACT_IDENTITY>(
                (const bf16_t*)X, dZb, wg_part, nullptr, B.splits, D, 2 * (int)e, (int)B.split_len, nullptr, 0, stream);
            const long long cnt = (long long)d * e, blocks = (cnt + 255) / 256;
            const unsigned gridr = (unsigned)(blocks > 4096 ? 4096 : blocks);
            hipLaunchKernelGGL(reduce_splits_halves_kernel, dim3(gridr), dim3(256), 0, stream, wg_part, dWg, D, (int)e,
                               B.splits);
            // dXz = [hi | lo] [Wg | Wg]^T: contraction over 2e, the second operand stored [d][2e] = [N][K]
            hipLaunchKernelGGL(duplicate_columns_kernel, dim3(gridr), dim3(256), 0, stream, (const bf16_t*)Wg, Wg2, D, (int)e);
            gemm_bf16_launch<256, 256, 2, 1, false, true, EPI_F32, EC_ACT_IDENTITY>(dZb, Wg2, dXz, nullptr, 1, (int)n, D,
                                                                                    2 * (int)e, nullptr, 0, stream);
        }
    } else {
    {   // partial[s] = X[s*len .. ]^T dZ[s*len .. ]   (the last split is shorter; its K is passed per launch)
        const int full = (int)(n / B.split_len);
        int prc = EC_OK;
        if (full > 0)
            prc = gemm_plain<T, float, float, true, false>(X, dZ, wg_part, full, D, (int)e, (int)B.split_len,
                                                           (long long)B.split_len * d, (long long)B.split_len * e,
                                                           (long long)d * e, stream);
        const int64_t rest = n - (int64_t)full * B.split_len;
        if (prc == EC_OK && rest > 0)
            prc = gemm_plain<T, float, float, true, false>(X + (size_t)full * B.split_len * d,
                                                           dZ + (size_t)full * B.split_len * e,
                                                           wg_part + (size_t)full * d * e, 1, D, (int)e, (int)rest, 0, 0,
                                                           0, stream);
        if (prc != EC_OK) return prc;
        long long cnt = (long long)d * e, blocks = (cnt + 255) / 256;
        hipLaunchKernelGGL(reduce_splits_kernel, dim3((unsigned)(blocks > 4096 ? 4096 : blocks)), dim3(256), 0, stream,
                           wg_part, dWg, cnt, B.splits);
    }
    // dXz = dZ Wg^T  (Wg stored [d][e] = [N][K])
    const int prc = gemm_plain<float, T, float, false, true>(dZ, Wg, dXz, 1, (int)n, D, (int)e, 0, 0, 0, stream);
    if (prc != EC_OK) return prc;
    }
    rc = check_launch();
    if (rc != EC_OK) return rc;
    mark();  // 7: gate products (dWg, dZ Wg^T)
    // dX = dXz + scatter-add of dX_in rows, expert-ascending, rounded once
    rc = launch_combine(dXin, nullptr, I, dX, n, d, e, k, dtype, ix, stream, dXz, true, nullptr, BF);
    mark();  // 8: scatter into dX
    return rc;
}

int launch_backward(const void* dY, const void* X, const void* Wg, const void* W1, const void* W2, const float* S,
                    const float* G, const int32_t* I, const void* Xin, const void* A, const void* H, const void* Xe,
                    void* dX, float* dWg, float* dW1, float* dW2, int64_t n, int64_t d, int64_t e, int64_t k,
                    int64_t d_ff, int act, int dtype, void* ws, const WsLayout& L, hipStream_t stream,
                    hipEvent_t* marks, bool hilo) {
    if (dtype == EC_BF16)
        return backward_typed<bf16_t>((const bf16_t*)dY, (const bf16_t*)X, (const bf16_t*)Wg, (const bf16_t*)W1,
                                      (const bf16_t*)W2, S, G, I, (const bf16_t*)Xin, (const bf16_t*)A, (const bf16_t*)H,
                                      (const bf16_t*)Xe, (bf16_t*)dX, dWg, dW1, dW2, n, d, e, k, d_ff, act, dtype, ws, L,
                                      stream, marks, hilo);
    return backward_typed<float>((const float*)dY, (const float*)X, (const float*)Wg, (const float*)W1, (const float*)W2,
                                 S, G, I, (const float*)Xin, (const float*)A, (const float*)H, (const float*)Xe, (float*)dX,
                                 dWg, dW1, dW2, n, d, e, k, d_ff, act, dtype, ws, L, stream, marks, false);
}

}  // namespace ecmoe
