// Dispatch ("shuffle", Sec. 3.2 Eq. 3 first line) and combine ("unshuffle", Eq. 4).
//
// dispatch: X_in[i,j,:] = X[I[i,j],:] -- a row gather with 16-byte lanes.
// combine:  X_out[l,:] = sum_{(i,j): I[i,j]=l} G[i,j] X_e[i,j,:], deterministic.
//   A token-major index is built from I without sorting and without float atomics:
//     a) bitmap[l] |= 1 << i          (integer OR commutes: order-free)
//     b) offsets = exclusive scan of popcount(bitmap[l])
//     c) inv[offsets[l] + popcount(bitmap[l] & bits below i)] = i*k + j
//   so each token's list is already in ascending expert order, and
//     d) one group of lanes per token adds its rows in that order in fp32.
#include "ec_common.h"

namespace ecmoe {

// ------------------------------------------------------------------ dispatch
// One row per group of `tpr` threads; each thread moves 16 bytes per step.
__global__ void __launch_bounds__(256)
dispatch_kernel(const uint4* __restrict__ X, const int32_t* __restrict__ I, uint4* __restrict__ Xin,
                long long rows, int vec_per_row, int tpr) {
    const int rows_per_block = 256 / tpr;
    const int sub = threadIdx.x / tpr, t = threadIdx.x % tpr;
    for (long long r = (long long)blockIdx.x * rows_per_block + sub; r < rows;
         r += (long long)gridDim.x * rows_per_block) {
        const uint4* src = X + (size_t)I[r] * vec_per_row;
        uint4* dst = Xin + (size_t)r * vec_per_row;
        for (int v = t; v < vec_per_row; v += tpr) dst[v] = src[v];
    }
}

// Rows whose byte length is not a multiple of 16 (fp32 with d % 4 != 0).
__global__ void __launch_bounds__(256)
dispatch_scalar_kernel(const float* __restrict__ X, const int32_t* __restrict__ I, float* __restrict__ Xin,
                       long long rows, int d) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (long long r = (long long)blockIdx.x * 4 + wave; r < rows; r += (long long)gridDim.x * 4) {
        const float* src = X + (size_t)I[r] * d;
        float* dst = Xin + (size_t)r * d;
        for (int v = lane; v < d; v += kWave) dst[v] = src[v];
    }
}

static int pick_threads_per_row(int64_t vec_per_row) {
    int tpr = 8;
    while (tpr < 256 && tpr < vec_per_row) tpr <<= 1;
    return tpr;
}

int launch_dispatch(const void* X, const int32_t* I, void* Xin, int64_t n, int64_t d, int64_t e, int64_t k,
                    int dtype, hipStream_t stream) {
    (void)n;
    const long long rows = (long long)e * k;
    const size_t row_bytes = (size_t)d * elem_size(dtype);
    if (row_bytes % 16 == 0) {
        int vec = (int)(row_bytes / 16);
        int tpr = pick_threads_per_row(vec);
        long long blocks = ceil_div(rows, 256 / tpr);
        if (blocks > (1 << 20)) blocks = 1 << 20;
        hipLaunchKernelGGL(dispatch_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4*)X, I,
                           (uint4*)Xin, rows, vec, tpr);
    } else {
        long long blocks = ceil_div(rows, 4);
        if (blocks > (1 << 20)) blocks = 1 << 20;
        hipLaunchKernelGGL(dispatch_scalar_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const float*)X,
                           I, (float*)Xin, rows, (int)d);
    }
    return check_launch();
}

// ------------------------------------------------------------------- combine
__global__ void __launch_bounds__(256)
fill_u32_kernel(uint32_t* __restrict__ p, long long count, uint32_t v) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < count; i += (long long)gridDim.x * 256) p[i] = v;
}

__global__ void __launch_bounds__(256)
bitmap_kernel(const int32_t* __restrict__ I, uint32_t* __restrict__ bitmap, long long rows, int k, int words) {
    for (long long r = (long long)blockIdx.x * 256 + threadIdx.x; r < rows; r += (long long)gridDim.x * 256) {
        int i = (int)(r / k);
        atomicOr(&bitmap[(size_t)I[r] * words + (i >> 5)], 1u << (i & 31));
    }
}

// Exclusive scan of per-token expert counts.  One 1024-thread workgroup; tokens
// are taken in consecutive chunks of 1024 so loads stay coalesced.
__global__ void __launch_bounds__(1024)
offsets_kernel(const uint32_t* __restrict__ bitmap, int32_t* __restrict__ offsets, int n, int words) {
    __shared__ unsigned int wave_tot[16];
    __shared__ unsigned int carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int l0 = 0; l0 < n; l0 += 1024) {
        int l = l0 + tid;
        unsigned int c = 0;
        if (l < n)
            for (int w = 0; w < words; ++w) c += __popc(bitmap[(size_t)l * words + w]);
        unsigned int incl = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            unsigned int o = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += o;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        unsigned int before = carry, total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            unsigned int t = wave_tot[w];
            before += w < wave ? t : 0u;
            total += t;
        }
        if (l < n) offsets[l] = (int32_t)(before + incl - c);
        __syncthreads();
        if (tid == 0) carry += total;
        __syncthreads();
    }
    if (tid == 0) offsets[n] = (int32_t)carry;
}

__global__ void __launch_bounds__(256)
inverse_index_kernel(const int32_t* __restrict__ I, const uint32_t* __restrict__ bitmap,
                     const int32_t* __restrict__ offsets, int32_t* __restrict__ inv, long long rows, int k,
                     int words) {
    for (long long r = (long long)blockIdx.x * 256 + threadIdx.x; r < rows; r += (long long)gridDim.x * 256) {
        int i = (int)(r / k);
        int l = I[r];
        const uint32_t* bm = bitmap + (size_t)l * words;
        int rank = 0;
        for (int w = 0; w < (i >> 5); ++w) rank += __popc(bm[w]);
        rank += __popc(bm[i >> 5] & ((1u << (i & 31)) - 1u));
        inv[offsets[l] + rank] = (int32_t)r;
    }
}

// One token per group of `tpr` threads; each thread owns 16 bytes of the row
// (8 bf16 / 4 fp32) per step and accumulates in fp32.
template <typename T, int VEC>
__global__ void __launch_bounds__(256)
combine_kernel(const T* __restrict__ Xe, const float* __restrict__ G, const int32_t* __restrict__ offsets,
               const int32_t* __restrict__ inv, T* __restrict__ Xout, int n, int d, int tpr) {
    typedef T vec_t __attribute__((ext_vector_type(VEC)));
    const int tok_per_block = 256 / tpr;
    const int sub = threadIdx.x / tpr, t = threadIdx.x % tpr;
    const int vec_per_row = d / VEC;
    for (int l = blockIdx.x * tok_per_block + sub; l < n; l += gridDim.x * tok_per_block) {
        const int beg = offsets[l], end = offsets[l + 1];
        for (int v = t; v < vec_per_row; v += tpr) {
            float acc[VEC];
#pragma unroll
            for (int q = 0; q < VEC; ++q) acc[q] = 0.0f;
            for (int p = beg; p < end; ++p) {
                const int r = inv[p];
                const float g = G[r];
                vec_t x = *reinterpret_cast<const vec_t*>(Xe + (size_t)r * d + (size_t)v * VEC);
#pragma unroll
                for (int q = 0; q < VEC; ++q) acc[q] = fmaf(g, Cvt<T>::to_f32(x[q]), acc[q]);
            }
            vec_t o;
#pragma unroll
            for (int q = 0; q < VEC; ++q) o[q] = Cvt<T>::from_f32(acc[q]);
            *reinterpret_cast<vec_t*>(Xout + (size_t)l * d + (size_t)v * VEC) = o;
        }
    }
}

int launch_combine(const void* Xe, const float* G, const int32_t* I, void* Xout, int64_t n, int64_t d,
                   int64_t e, int64_t k, int dtype, uint32_t* bitmap, int32_t* offsets, int32_t* inv,
                   hipStream_t stream) {
    const long long rows = (long long)e * k;
    const int words = (int)ceil_div(e, 32);
    const long long bm_words = (long long)n * words;
    auto blocks_for = [](long long items) {
        long long b = (items + 255) / 256;
        return (unsigned)(b > 16384 ? 16384 : (b < 1 ? 1 : b));
    };
    hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(bm_words)), dim3(256), 0, stream, bitmap, bm_words, 0u);
    hipLaunchKernelGGL(bitmap_kernel, dim3(blocks_for(rows)), dim3(256), 0, stream, I, bitmap, rows, (int)k, words);
    hipLaunchKernelGGL(offsets_kernel, dim3(1), dim3(1024), 0, stream, bitmap, offsets, (int)n, words);
    hipLaunchKernelGGL(inverse_index_kernel, dim3(blocks_for(rows)), dim3(256), 0, stream, I, bitmap, offsets, inv,
                       rows, (int)k, words);
    int rc = check_launch();
    if (rc != EC_OK) return rc;

    if (dtype == EC_BF16) {
        int vec = (int)(d / 8);
        int tpr = pick_threads_per_row(vec);
        long long blocks = ceil_div(n, 256 / tpr);
        if (blocks > (1 << 20)) blocks = 1 << 20;
        hipLaunchKernelGGL((combine_kernel<bf16_t, 8>), dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const bf16_t*)Xe, G, offsets, inv, (bf16_t*)Xout, (int)n, (int)d, tpr);
    } else if (d % 4 == 0) {
        int vec = (int)(d / 4);
        int tpr = pick_threads_per_row(vec);
        long long blocks = ceil_div(n, 256 / tpr);
        if (blocks > (1 << 20)) blocks = 1 << 20;
        hipLaunchKernelGGL((combine_kernel<float, 4>), dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const float*)Xe, G, offsets, inv, (float*)Xout, (int)n, (int)d, tpr);
    } else {
        int tpr = pick_threads_per_row(d);
        long long blocks = ceil_div(n, 256 / tpr);
        if (blocks > (1 << 20)) blocks = 1 << 20;
        hipLaunchKernelGGL((combine_kernel<float, 1>), dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const float*)Xe, G, offsets, inv, (float*)Xout, (int)n, (int)d, tpr);
    }
    return check_launch();
}

}  // namespace ecmoe
