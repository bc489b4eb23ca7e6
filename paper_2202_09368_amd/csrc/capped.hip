// Expert choice with a cap on the experts per token (Sec. 3.3): the matrix A[e,n] of the
// entropy-regularised linear programme
//     max <S^T, A> + lambda H(A),  rows sum to k, columns sum to at most b, 0 <= A <= 1,
// by Dykstra's algorithm over the three constraint sets; the buckets are then TopK(A, k).
// The paper prints neither the projections nor a stopping rule.  Here the projections are the KL
// (Bregman) ones, which are scalings -- rows by k / rowsum, columns by min(1, b / colsum), entries
// clipped at 1 -- with Dykstra's correction terms for the two inequality sets (one scale per column,
// one value per entry), and a fixed number of sweeps (rows, columns, box) is run.  Everything is
// kept in the log domain in float64: exp(S / lambda) overflows any float type for lambda = 0.001.
//
// One sweep is two launches over the [e][n] state:
//   capped_row_kernel   per expert row: r[i] = log k - logsumexp_j logA[i,j]   (read only)
//   capped_col_kernel   per token column: applies r, the column scale and the box step, and keeps
//                       the two correction terms.  Lanes run along the token axis (contiguous).
// Reductions use a fixed order (online log-sum-exp per thread, then a fixed tree), so results do
// not depend on timing.  Bound: HBM / L2 traffic, 2 reads + 2 writes of 8 e n bytes per sweep
// plus one more read for the row sums.
#include <cmath>

#include "ec_common.h"

namespace ecmoe {

struct Lse {  // running log-sum-exp: sum = s * exp(m)
    double m, s;
};
__device__ __forceinline__ Lse lse_empty() { return {-INFINITY, 0.0}; }
__device__ __forceinline__ Lse lse_add(Lse a, double x) {
    if (x > a.m) { a.s = a.s * exp(a.m - x) + 1.0; a.m = x; }
    else if (x > -INFINITY) a.s += exp(x - a.m);
    return a;
}
__device__ __forceinline__ Lse lse_merge(Lse a, Lse b) {
    if (b.m > a.m) { Lse t = a; a = b; b = t; }
    if (b.m > -INFINITY) a.s += b.s * exp(b.m - a.m);
    return a;
}
__device__ __forceinline__ double lse_value(Lse a) { return a.m + log(a.s); }

__global__ void __launch_bounds__(256)
capped_init_kernel(const float* __restrict__ St, double inv_lambda, double* __restrict__ logA,
                   double* __restrict__ lq_box, double* __restrict__ lq_col, long long count, int n) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < count; i += (long long)gridDim.x * 256) {
        logA[i] = (double)St[i] * inv_lambda;
        lq_box[i] = 0.0;
        if (i < n) lq_col[i] = 0.0;
    }
}

__global__ void __launch_bounds__(1024)
capped_row_kernel(const double* __restrict__ logA, double* __restrict__ r, int n, double log_k) {
    __shared__ double sm[16], ss[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double* row = logA + (size_t)blockIdx.x * n;
    Lse a = lse_empty();
    for (int j = tid; j < n; j += 1024) a = lse_add(a, row[j]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        Lse o = {__shfl_xor(a.m, off, kWave), __shfl_xor(a.s, off, kWave)};
        a = lse_merge(a, o);  // symmetric in its arguments: both partners end with the same value
    }
    if (lane == 0) { sm[wave] = a.m; ss[wave] = a.s; }
    __syncthreads();
    if (tid == 0) {
        Lse t = {sm[0], ss[0]};
        for (int w = 1; w < 16; ++w) t = lse_merge(t, Lse{sm[w], ss[w]});
        r[blockIdx.x] = log_k - lse_value(t);
    }
}

// Block = 64 tokens x 4 slices of the expert axis (wavefront w takes experts w, w+4, ...).
__global__ void __launch_bounds__(256)
capped_col_kernel(double* __restrict__ logA, double* __restrict__ lq_box, double* __restrict__ lq_col,
                  const double* __restrict__ r, int n, int e, double log_b) {
    __shared__ double sm[4][64], ss[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = blockIdx.x * 64 + lane;
    const bool live = j < n;
    const double qc = live ? lq_col[j] : 0.0;
    Lse a = lse_empty();
    if (live)
        for (int i = wave; i < e; i += 4) a = lse_add(a, logA[(size_t)i * n + j] + r[i] + qc);
    sm[wave][lane] = a.m;
    ss[wave][lane] = a.s;
    __syncthreads();
    Lse t = {sm[0][lane], ss[0][lane]};
#pragma unroll
    for (int w = 1; w < 4; ++w) t = lse_merge(t, Lse{sm[w][lane], ss[w][lane]});
    if (!live) return;
    const double s = fmin(0.0, log_b - lse_value(t));  // log of the column's scale
    for (int i = wave; i < e; i += 4) {
        const size_t at = (size_t)i * n + j;
        const double B = logA[at] + r[i] + qc + s + lq_box[at];
        logA[at] = fmin(B, 0.0);
        lq_box[at] = fmax(B, 0.0);
    }
    if (wave == 0) lq_col[j] = -s;
}

__global__ void __launch_bounds__(256)
capped_exp_kernel(const double* __restrict__ logA, float* __restrict__ A, long long count) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < count; i += (long long)gridDim.x * 256)
        A[i] = (float)exp(logA[i]);
}

// G[i,j] = St[i, I[i,j]]: the gate weights stay the scores, only the indices come from A.
__global__ void __launch_bounds__(256)
gather_scores_kernel(const float* __restrict__ St, const int32_t* __restrict__ I, float* __restrict__ G,
                     long long rows, int k, int n) {
    for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < rows; q += (long long)gridDim.x * 256)
        G[q] = St[(size_t)(q / k) * n + I[q]];
}

size_t capped_ws_bytes(int64_t n, int64_t e) {
    return 2 * align_up((size_t)e * n * 8, 256) + align_up((size_t)n * 8, 256) + align_up((size_t)e * 8, 256);
}

static unsigned grid_for(long long items) {
    long long b = (items + 255) / 256;
    return (unsigned)(b > 65536 ? 65536 : (b < 1 ? 1 : b));
}

int launch_capped_assignment(const float* St, int64_t n, int64_t e, int64_t k, double b, double lambda,
                             int64_t iters, float* A, void* ws, hipStream_t stream) {
    char* p = (char*)ws;
    double* logA = (double*)p;    p += align_up((size_t)e * n * 8, 256);
    double* lq_box = (double*)p;  p += align_up((size_t)e * n * 8, 256);
    double* lq_col = (double*)p;  p += align_up((size_t)n * 8, 256);
    double* r = (double*)p;
    const long long count = (long long)e * n;
    hipLaunchKernelGGL(capped_init_kernel, dim3(grid_for(count)), dim3(256), 0, stream, St, 1.0 / lambda, logA, lq_box,
                       lq_col, count, (int)n);
    const double log_k = std::log((double)k), log_b = std::log(b);
    for (int64_t it = 0; it < iters; ++it) {
        hipLaunchKernelGGL(capped_row_kernel, dim3((unsigned)e), dim3(1024), 0, stream, logA, r, (int)n, log_k);
        hipLaunchKernelGGL(capped_col_kernel, dim3((unsigned)ceil_div(n, 64)), dim3(256), 0, stream, logA, lq_box, lq_col,
                           r, (int)n, (int)e, log_b);
    }
    hipLaunchKernelGGL(capped_exp_kernel, dim3(grid_for(count)), dim3(256), 0, stream, logA, A, count);
    return check_launch();
}

int launch_gather_scores(const float* St, const int32_t* I, float* G, int64_t n, int64_t e, int64_t k,
                         hipStream_t stream) {
    const long long rows = (long long)e * k;
    hipLaunchKernelGGL(gather_scores_kernel, dim3(grid_for(rows)), dim3(256), 0, stream, St, I, G, rows, (int)k, (int)n);
    return check_launch();
}

}  // namespace ecmoe
