// Gating scores S = Softmax(X.Wg) over the expert axis (Sec. 3.2, Eq. 2; Sec. 3.4).
//
// Two kernels:
//  * gate_mfma_kernel   bf16 inputs, d % 64 == 0, e % 8 == 0, e <= 256.  Computes Z^T = Wg^T.X^T
//    on the matrix cores with experts as the MFMA row axis and tokens as the
//    column axis, so that one token's logits sit in the registers of two lanes
//    (lane and lane^32) and the softmax needs a single cross-lane exchange.
//    Stores S^T [e,n] with 32 consecutive tokens per store instruction.
//  * gate_generic_kernel  any dtype / shape; one wavefront per token, plain fp32 FMAs.
// With more than 64 experts and enough tokens to fill the chip the product runs on the grouped-GEMM
// kernel instead (gemm_bf16.h, softmax epilogue).
#include "ec_common.h"
#include "gemm_bf16.h"

namespace ecmoe {

// ---------------------------------------------------------------------------
// MFMA gate.  Block = NW wavefronts, 32 tokens per wavefront.  ET = number of
// 32-expert tiles held per wavefront (e_pad = 32*ET).  A stage of 64 rows of Wg
// sits in LDS in the matrix's own row-major [k][expert] form; transposing LDS
// reads (ds_read_b64_tr_b16) hand each lane the 2 x 4 consecutive-k values of
// its expert, so Wg needs no transposed copy.  The block also clears
// `zero_words` 32-bit words at `zero_buf` (counters the later stages use).
// ---------------------------------------------------------------------------
constexpr int GATE_BK = 64;  // contraction elements per LDS stage

template <int ET, int NW>
__global__ void __launch_bounds__(64 * NW)
gate_mfma_kernel(const bf16_t* __restrict__ X, const bf16_t* __restrict__ Wg, float* __restrict__ S,
                 float* __restrict__ St, int n, int d, int e, uint32_t* __restrict__ zero_buf, int zero_words) {
    constexpr int E_PAD = 32 * ET;
    constexpr int NT = 64 * NW;
    constexpr int PITCH = ET == 1 ? 32 : E_PAD + 32;  // four consecutive rows fall in four distinct 64-byte bank groups
    constexpr int CHUNKS = GATE_BK * (E_PAD / 8);     // 16-byte chunks per stage
    constexpr int CPT = (CHUNKS + NT - 1) / NT;       // chunks per thread
    __shared__ __attribute__((aligned(16))) bf16_t Wk[GATE_BK * PITCH];
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

    const int tid = threadIdx.x;
    for (int i = blockIdx.x * NT + tid; i < zero_words; i += gridDim.x * NT) zero_buf[i] = 0u;

    const int lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5, l16 = lane & 15;
    const int tok = blockIdx.x * (32 * NW) + wave * 32 + col;
    const int tok_ld = tok < n ? tok : n - 1;  // clamp loads, predicate stores
    const bf16_t* xrow = X + (size_t)tok_ld * d + half * 32;

    floatx16 acc[ET];
#pragma unroll
    for (int te = 0; te < ET; ++te)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[te][r] = 0.0f;

    // Loads run PD stages ahead of their use: a wavefront has only a few MFMAs per stage, far too little to
    // cover a trip to memory, and with one wavefront per block nothing else on the SIMD would cover it either.
    constexpr int PD = 4;
    u32x4 wq[PD][CPT];
    bf16x8 xq[PD][4];
    auto load_chunk = [&](int kc, int slot) {
#pragma unroll
        for (int r = 0; r < CPT; ++r) {
            const int c = tid + NT * r;
            const int krow = c / (E_PAD / 8), ech = c % (E_PAD / 8);
            u32x4 v = {0u, 0u, 0u, 0u};
            if (c < CHUNKS && ech * 8 < e)  // e % 8 == 0: a chunk is all experts or all padding
                v = *reinterpret_cast<const u32x4*>(Wg + (size_t)(kc * GATE_BK + krow) * e + ech * 8);
            wq[slot][r] = v;
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) xq[slot][s] = *reinterpret_cast<const bf16x8*>(xrow + kc * GATE_BK + s * 8);
    };

    // The contraction index of a stage is consumed in the order (half, step): lanes 0-31 own elements
    // [0,32) of the stage, lanes 32-63 own [32,64), so a lane's X values are 64 contiguous bytes.
    const int w_frag = (half * 32 + (l16 >> 2)) * PITCH + ((lane >> 4) & 1) * 16 + (l16 & 3) * 4;
    const int nk = d / GATE_BK;
#pragma unroll
    for (int u = 0; u < PD; ++u)
        if (u < nk) load_chunk(u, u);
    for (int kc0 = 0; kc0 < nk; kc0 += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const int kc = kc0 + u;
            if (kc < nk) {  // uniform
                __syncthreads();
#pragma unroll
                for (int r = 0; r < CPT; ++r) {
                    const int c = tid + NT * r;
                    const int krow = c / (E_PAD / 8), ech = c % (E_PAD / 8);
                    if (c < CHUNKS) *reinterpret_cast<u32x4*>(&Wk[krow * PITCH + ech * 8]) = wq[u][r];
                }
                __syncthreads();
                bf16x8 xcur[4];
#pragma unroll
                for (int s = 0; s < 4; ++s) xcur[s] = xq[u][s];
                if (kc + PD < nk) load_chunk(kc + PD, u);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
#pragma unroll
                    for (int te = 0; te < ET; ++te) {
                        const bf16_t* p0 = &Wk[w_frag + s * 8 * PITCH + te * 32];
                        bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0));
                        bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0 + 4 * PITCH));
                        bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        acc[te] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xcur[s], acc[te], 0, 0, 0);
                    }
                }
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
            // exp through the hardware exp2 (relative 6e-8 * |z - max| from rounding the scaled argument)
            float p = ex < e ? __builtin_amdgcn_exp2f((acc[te][r] - m) * 1.44269504088896340736f) : 0.0f;
            acc[te][r] = p;
            sum += p;
        }
    sum += __shfl_xor(sum, 32, kWave);
    if (tok >= n) return;
    const float inv_sum = 1.0f / sum;
#pragma unroll
    for (int te = 0; te < ET; ++te)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int ex0 = te * 32 + 8 * q + 4 * half;
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = acc[te][4 * q + j] * inv_sum;
            if (ex0 >= e) continue;  // e % 8 == 0: a quad is all experts or all padding
            if (St != nullptr) {
#pragma unroll
                for (int j = 0; j < 4; ++j) St[(size_t)(ex0 + j) * n + tok] = v[j];
            }
            if (S != nullptr) {
                floatx4 o = {v[0], v[1], v[2], v[3]};
                *reinterpret_cast<floatx4*>(S + (size_t)tok * e + ex0) = o;
            }
        }
}

__global__ void __launch_bounds__(256)
zero_words_kernel(uint32_t* __restrict__ p, long long count) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < count; i += (long long)gridDim.x * 256) p[i] = 0u;
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
                int dtype, uint32_t* zero_buf, int64_t zero_words, hipStream_t stream) {
    const bool mfma = dtype == EC_BF16 && (d % GATE_BK) == 0 && e <= 256 && (e % 8) == 0;
    // Many experts and many tokens: X.Wg is a real matrix product.  It runs on the grouped-GEMM kernel
    // (one group, all experts inside one tile) whose epilogue does the softmax and clears the counters.
    if (mfma && e > 64 && gemm_bf16_shape_ok(n, e, d)) {
        if (e > 128 && n >= 128 * 256) {
            gemm_bf16_launch<256, 256, 2, 1, false, false, EPI_SOFTMAX, EC_ACT_IDENTITY>(
                (const bf16_t*)X, (const bf16_t*)Wg, St, S, 1, (int)n, (int)e, (int)d,
                reinterpret_cast<const int32_t*>(zero_buf), (int)zero_words, stream);
            return check_launch();
        }
        if (e <= 128 && n >= 128 * 128) {
            gemm_bf16_launch<128, 128, 1, 2, false, false, EPI_SOFTMAX, EC_ACT_IDENTITY>(
                (const bf16_t*)X, (const bf16_t*)Wg, St, S, 1, (int)n, (int)e, (int)d,
                reinterpret_cast<const int32_t*>(zero_buf), (int)zero_words, stream);
            return check_launch();
        }
    }
    if (mfma) {
        const int et = e <= 32 ? 1 : e <= 64 ? 2 : e <= 128 ? 4 : 8;
        // one wavefront per block while that still leaves blocks for every compute unit, four otherwise
        const bool small = n <= 32 * 1024 && et <= 2;
        const int tok_per_block = small ? 32 : 128;
        dim3 grid((unsigned)ceil_div(n, tok_per_block));
#define EC_GATE_LAUNCH(ETV, NWV)                                                                          \
    hipLaunchKernelGGL((gate_mfma_kernel<ETV, NWV>), grid, dim3(64 * NWV), 0, stream, (const bf16_t*)X,   \
                       (const bf16_t*)Wg, S, St, (int)n, (int)d, (int)e, zero_buf, (int)zero_words)
        if (small) {
            if (et == 1) EC_GATE_LAUNCH(1, 1); else EC_GATE_LAUNCH(2, 1);
        } else {
            switch (et) {
                case 1: EC_GATE_LAUNCH(1, 4); break;
                case 2: EC_GATE_LAUNCH(2, 4); break;
                case 4: EC_GATE_LAUNCH(4, 4); break;
                default: EC_GATE_LAUNCH(8, 4); break;
            }
        }
#undef EC_GATE_LAUNCH
        return check_launch();
    }
    if (zero_words > 0) {
        long long zb = (zero_words + 255) / 256;
        hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)(zb > 4096 ? 4096 : zb)), dim3(256), 0, stream, zero_buf,
                           (long long)zero_words);
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
