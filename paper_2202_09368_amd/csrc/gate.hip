// Gating scores S = Softmax(X.Wg) over the expert axis (Sec. 3.2, Eq. 2; Sec. 3.4).
//
// Two kernels:
//  * gate_mfma_kernel   bf16 inputs, d % 64 == 0, e <= 256.  Computes Z^T = Wg^T.X^T
//    on the matrix cores with experts as the MFMA row axis and tokens as the
//    column axis, so that one token's logits sit in the registers of two lanes
//    (lane and lane^32) and the softmax needs a single cross-lane exchange.
//    Stores S^T [e,n] with 32 consecutive tokens per store instruction.
//  * gate_generic_kernel  any dtype / shape; one wavefront per token, plain fp32 FMAs.
#include "ec_common.h"

namespace ecmoe {

// ---------------------------------------------------------------------------
// Wg [d,e] -> Wgt [e_pad, d] bf16 (rows >= e are zero).  Tiny; runs once per call.
// ---------------------------------------------------------------------------
__global__ void wg_transpose_kernel(const bf16_t* __restrict__ Wg, bf16_t* __restrict__ Wgt,
                                    int d, int e, int e_pad) {
    __shared__ bf16_t tile[32][33];
    const int t0 = blockIdx.x * 32;  // d index
    const int i0 = blockIdx.y * 32;  // expert index
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        int t = t0 + r, i = i0 + tx;
        tile[r][tx] = (t < d && i < e) ? Wg[(size_t)t * e + i] : static_cast<bf16_t>(0.0f);
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        int i = i0 + r, t = t0 + tx;
        if (i < e_pad && t < d) Wgt[(size_t)i * d + t] = tile[tx][r];
    }
}

// ---------------------------------------------------------------------------
// MFMA gate.  Block = 256 threads = 4 wavefronts, 32 tokens per wavefront.
// ET = number of 32-expert tiles held per wavefront (e_pad = 32*ET).
// ---------------------------------------------------------------------------
constexpr int GATE_BK = 64;       // contraction elements per LDS stage
constexpr int GATE_LDS_STRIDE = GATE_BK + 8;  // bf16 elements; 144-byte rows keep 16-byte reads conflict-free

template <int ET>
__global__ void __launch_bounds__(256)
gate_mfma_kernel(const bf16_t* __restrict__ X, const bf16_t* __restrict__ Wgt,
                 float* __restrict__ S, float* __restrict__ St, int n, int d, int e) {
    constexpr int E_PAD = 32 * ET;
    __shared__ __attribute__((aligned(16))) bf16_t Wt[E_PAD * GATE_LDS_STRIDE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int tok = blockIdx.x * 128 + wave * 32 + col;
    const int tok_ld = tok < n ? tok : n - 1;  // clamp loads, predicate stores
    const bf16_t* xrow = X + (size_t)tok_ld * d + half * 32;

    floatx16 acc[ET];
#pragma unroll
    for (int te = 0; te < ET; ++te)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[te][r] = 0.0f;

    bf16x8 wreg[ET];
    bf16x8 xreg[4];
    auto load_chunk = [&](int kc) {
#pragma unroll
        for (int r = 0; r < ET; ++r) {
            int c = tid + 256 * r;
            int row = c >> 3, kch = c & 7;
            wreg[r] = *reinterpret_cast<const bf16x8*>(Wgt + (size_t)row * d + kc * GATE_BK + kch * 8);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
            xreg[s] = *reinterpret_cast<const bf16x8*>(xrow + kc * GATE_BK + s * 8);
    };

    const int nk = d / GATE_BK;
    load_chunk(0);
    for (int kc = 0; kc < nk; ++kc) {
        __syncthreads();
#pragma unroll
        for (int r = 0; r < ET; ++r) {
            int c = tid + 256 * r;
            int row = c >> 3, kch = c & 7;
            *reinterpret_cast<bf16x8*>(&Wt[row * GATE_LDS_STRIDE + kch * 8]) = wreg[r];
        }
        __syncthreads();
        bf16x8 xcur[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) xcur[s] = xreg[s];
        if (kc + 1 < nk) load_chunk(kc + 1);
        // The contraction index is consumed in the order (half, s): lanes 0-31 own
        // elements [0,32) of the stage, lanes 32-63 own [32,64); both operands agree.
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int te = 0; te < ET; ++te) {
                bf16x8 a = *reinterpret_cast<const bf16x8*>(
                    &Wt[(te * 32 + col) * GATE_LDS_STRIDE + half * 32 + s * 8]);
                acc[te] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xcur[s], acc[te], 0, 0, 0);
            }
        }
    }

    // acc[te][r] = Z[expert = 32*te + 8*(r/4) + 4*half + r%4][token = col]
    float m = -INFINITY;
#pragma unroll
    for (int te = 0; te < ET; ++te)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int ex = te * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
            if (ex < e) m = fmaxf(m, acc[te][r]);
        }
    m = fmaxf(m, __shfl_xor(m, 32, kWave));
    float sum = 0.0f;
#pragma unroll
    for (int te = 0; te < ET; ++te)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int ex = te * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
            float p = ex < e ? expf(acc[te][r] - m) : 0.0f;
            acc[te][r] = p;
            sum += p;
        }
    sum += __shfl_xor(sum, 32, kWave);
    if (tok >= n) return;
    const bool s_vec = (S != nullptr) && ((e & 3) == 0);
#pragma unroll
    for (int te = 0; te < ET; ++te)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int ex0 = te * 32 + 8 * q + 4 * half;
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = acc[te][4 * q + j] / sum;
            if (St != nullptr) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (ex0 + j < e) St[(size_t)(ex0 + j) * n + tok] = v[j];
            }
            if (S != nullptr) {
                if (s_vec) {
                    if (ex0 < e) {
                        floatx4 o = {v[0], v[1], v[2], v[3]};
                        *reinterpret_cast<floatx4*>(S + (size_t)tok * e + ex0) = o;
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (ex0 + j < e) S[(size_t)tok * e + ex0 + j] = v[j];
                }
            }
        }
}

// ---------------------------------------------------------------------------
// Generic gate: one wavefront per token, lanes split the model dimension,
// experts in chunks of 16, logits staged in LDS, softmax by the same wavefront.
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
gate_generic_kernel(const T* __restrict__ X, const T* __restrict__ Wg, float* __restrict__ S,
                    float* __restrict__ St, int n, int d, int e) {
    __shared__ float z[4][EC_MOE_MAX_EXPERTS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int tok = blockIdx.x * 4 + wave; tok < n; tok += gridDim.x * 4) {
        const T* xrow = X + (size_t)tok * d;
        for (int i0 = 0; i0 < e; i0 += 16) {
            float acc[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[j] = 0.0f;
            for (int t = lane; t < d; t += kWave) {
                float x = Cvt<T>::to_f32(xrow[t]);
                const T* wrow = Wg + (size_t)t * e + i0;
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (i0 + j < e) acc[j] = fmaf(x, Cvt<T>::to_f32(wrow[j]), acc[j]);
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                float v = wave_reduce_sum(acc[j]);
                if (lane == 0 && i0 + j < e) z[wave][i0 + j] = v;
            }
        }
        __builtin_amdgcn_wave_barrier();
        __threadfence_block();
        float m = -INFINITY;
        for (int i = lane; i < e; i += kWave) m = fmaxf(m, z[wave][i]);
        m = wave_reduce_max(m);
        float sum = 0.0f;
        for (int i = lane; i < e; i += kWave) sum += expf(z[wave][i] - m);
        sum = wave_reduce_sum(sum);
        for (int i = lane; i < e; i += kWave) {
            float v = expf(z[wave][i] - m) / sum;
            if (S != nullptr) S[(size_t)tok * e + i] = v;
            if (St != nullptr) St[(size_t)i * n + tok] = v;
        }
        __builtin_amdgcn_wave_barrier();
        __threadfence_block();
    }
}

int launch_gate(const void* X, const void* Wg, float* S, float* St, int64_t n, int64_t d, int64_t e,
                int dtype, void* wgt_ws, hipStream_t stream) {
    const bool mfma = dtype == EC_BF16 && (d % GATE_BK) == 0 && e <= 256 && wgt_ws != nullptr;
    if (mfma) {
        int et = e <= 32 ? 1 : e <= 64 ? 2 : e <= 128 ? 4 : 8;
        int e_pad = 32 * et;
        dim3 tg((unsigned)ceil_div(d, 32), (unsigned)(e_pad / 32));
        hipLaunchKernelGGL(wg_transpose_kernel, tg, dim3(256), 0, stream, (const bf16_t*)Wg, (bf16_t*)wgt_ws,
                           (int)d, (int)e, e_pad);
        dim3 grid((unsigned)ceil_div(n, 128));
#define EC_GATE_LAUNCH(ETV)                                                                              \
    hipLaunchKernelGGL(gate_mfma_kernel<ETV>, grid, dim3(256), 0, stream, (const bf16_t*)X,              \
                       (const bf16_t*)wgt_ws, S, St, (int)n, (int)d, (int)e)
        switch (et) {
            case 1: EC_GATE_LAUNCH(1); break;
            case 2: EC_GATE_LAUNCH(2); break;
            case 4: EC_GATE_LAUNCH(4); break;
            default: EC_GATE_LAUNCH(8); break;
        }
#undef EC_GATE_LAUNCH
        return check_launch();
    }
    int64_t blocks = ceil_div(n, 4);
    if (blocks > 65536) blocks = 65536;
    if (dtype == EC_BF16)
        hipLaunchKernelGGL(gate_generic_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const bf16_t*)X, (const bf16_t*)Wg, S, St, (int)n, (int)d, (int)e);
    else
        hipLaunchKernelGGL(gate_generic_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const float*)X, (const float*)Wg, S, St, (int)n, (int)d, (int)e);
    return check_launch();
}

}  // namespace ecmoe
