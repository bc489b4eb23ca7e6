// Dispatch ("shuffle", Sec. 3.2 Eq. 3 first line) and combine ("unshuffle", Eq. 4).
//
// dispatch: X_in[i,j,:] = X[I[i,j],:] -- a row gather with 16-byte lanes (I = -1: a row of zeros).
// combine:  X_out[l,:] = sum_{(i,j): I[i,j]=l} G[i,j] X_e[i,j,:], deterministic.
//   A token-major index is built from I with integer atomics only (see below); one group of
//   lanes per token then adds that token's bucket rows in ascending expert order in fp32.
#include <mutex>

#include "ec_common.h"

namespace ecmoe {

// Scratch of ec_moe_combine_static: the token-major index lives here instead of in a caller's
// workspace.  One copy per GPU, held until the process ends; every call on a GPU shares it.
static __device__ __align__(256) unsigned char scratch[EC_MOE_STATIC_SCRATCH_BYTES];

// ------------------------------------------------------------------ dispatch
// One row per group of `tpr` threads; each thread moves 16 bytes per step.
__global__ void __launch_bounds__(256)
dispatch_kernel(const uint4* __restrict__ X, const int32_t* __restrict__ I, uint4* __restrict__ Xin,
                long long rows, int vec_per_row, int tpr) {
    const int rows_per_block = 256 / tpr;
    const int sub = threadIdx.x / tpr, t = threadIdx.x % tpr;
    for (long long r = (long long)blockIdx.x * rows_per_block + sub; r < rows;
         r += (long long)gridDim.x * rows_per_block) {
        const int tok = I[r];  // -1: an empty buffer row (token-choice routing), filled with zeros
        const uint4* src = X + (size_t)(tok < 0 ? 0 : tok) * vec_per_row;
        uint4* dst = Xin + (size_t)r * vec_per_row;
        for (int v = t; v < vec_per_row; v += tpr) dst[v] = tok < 0 ? make_uint4(0u, 0u, 0u, 0u) : src[v];
    }
}

// Rows whose byte length is not a multiple of 16 (fp32 with d % 4 != 0).
__global__ void __launch_bounds__(256)
dispatch_scalar_kernel(const float* __restrict__ X, const int32_t* __restrict__ I, float* __restrict__ Xin,
                       long long rows, int d) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (long long r = (long long)blockIdx.x * 4 + wave; r < rows; r += (long long)gridDim.x * 4) {
        const int tok = I[r];
        const float* src = X + (size_t)(tok < 0 ? 0 : tok) * d;
        float* dst = Xin + (size_t)r * d;
        for (int v = lane; v < d; v += kWave) dst[v] = tok < 0 ? 0.0f : src[v];
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
// Token-major index of the routing, two forms:
//  * slot lists (e <= COMBINE_SLOT_CAP): slot_cnt[l] experts chose token l and left their bucket rows
//    in slots[l*cap ...] in arrival order; the combine kernel visits them in ascending row order,
//    which is ascending expert order because an expert holds a token at most once.
//  * CSR (any e): bitmap[l] has one bit per expert, offsets = exclusive scan of its popcounts,
//    inv[offsets[l] + (number of set bits below i)] = i*k + j -- already expert-ascending.
// Both are built with integer atomics only (OR / counting), so the result never depends on timing.
__global__ void __launch_bounds__(256)
fill_u32_kernel(uint32_t* __restrict__ p, long long count, uint32_t v) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < count; i += (long long)gridDim.x * 256) p[i] = v;
}

__global__ void __launch_bounds__(256)
bitmap_kernel(const int32_t* __restrict__ I, uint32_t* __restrict__ bitmap, long long rows, int k, int words) {
    for (long long r = (long long)blockIdx.x * 256 + threadIdx.x; r < rows; r += (long long)gridDim.x * 256) {
        int i = (int)(r / k);
        if (I[r] >= 0) atomicOr(&bitmap[(size_t)I[r] * words + (i >> 5)], 1u << (i & 31));  // -1: empty row
    }
}

__global__ void __launch_bounds__(256)
slots_kernel(const int32_t* __restrict__ I, int32_t* __restrict__ slot_cnt, int32_t* __restrict__ slots,
             long long rows, int cap) {
    for (long long r = (long long)blockIdx.x * 256 + threadIdx.x; r < rows; r += (long long)gridDim.x * 256) {
        const int l = I[r];
        if (l < 0) continue;  // empty buffer row
        const int s = atomicAdd(&slot_cnt[l], 1);
        if (s < cap) slots[(size_t)l * cap + s] = (int32_t)r;
    }
}

// Exclusive scan of per-token expert counts (popcounts of the bitmap rows) in two launches:
// block_counts_kernel sums the counts of each block's token range; offsets_kernel adds up the
// totals of the blocks before it (at most 1024 of them, one per thread) and scans its own range.
// A block owns `tpb` consecutive tokens (a multiple of 1024), walked 1024 at a time so that
// loads stay coalesced.
__device__ __forceinline__ unsigned int token_count(const uint32_t* __restrict__ bitmap, int l, int n, int words) {
    unsigned int v = 0;
    if (l < n)
        for (int w = 0; w < words; ++w) v += __popc(bitmap[(size_t)l * words + w]);
    return v;
}

__device__ __forceinline__ unsigned int block_sum_1024(unsigned int v, unsigned int* red /*[16]*/) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    __syncthreads();  // red may still be read from a previous use
    if (lane == 0) red[wave] = v;
    __syncthreads();
    unsigned int total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) total += red[w];
    return total;
}

__global__ void __launch_bounds__(1024)
block_counts_kernel(const uint32_t* __restrict__ bitmap, uint32_t* __restrict__ block_tot, int n, int words, int tpb) {
    __shared__ unsigned int red[16];
    const int beg = blockIdx.x * tpb;
    unsigned int v = 0;
    for (int l0 = beg; l0 < beg + tpb && l0 < n; l0 += 1024) v += token_count(bitmap, l0 + threadIdx.x, n, words);
    const unsigned int total = block_sum_1024(v, red);
    if (threadIdx.x == 0) block_tot[blockIdx.x] = total;
}

__global__ void __launch_bounds__(1024)
offsets_kernel(const uint32_t* __restrict__ bitmap, const uint32_t* __restrict__ block_tot,
               int32_t* __restrict__ offsets, int n, int words, int tpb) {
    __shared__ unsigned int red[16];
    __shared__ unsigned int wave_tot[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned int carry = block_sum_1024(tid < (int)blockIdx.x ? block_tot[tid] : 0u, red);  // gridDim.x <= 1024
    const int beg = blockIdx.x * tpb;
    for (int l0 = beg; l0 < beg + tpb && l0 < n; l0 += 1024) {
        const int l = l0 + tid;
        const unsigned int c = token_count(bitmap, l, n, words);
        unsigned int incl = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            unsigned int o = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += o;
        }
        __syncthreads();  // wave_tot of the previous round has been read
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        unsigned int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            unsigned int t = wave_tot[w];
            before += w < wave ? t : 0u;
            total += t;
        }
        if (l < n) offsets[l] = (int32_t)(carry + before + incl - c);
        carry += total;
    }
    if (blockIdx.x == gridDim.x - 1 && tid == 0) offsets[n] = (int32_t)carry;
}

__global__ void __launch_bounds__(256)
inverse_index_kernel(const int32_t* __restrict__ I, const uint32_t* __restrict__ bitmap,
                     const int32_t* __restrict__ offsets, int32_t* __restrict__ inv, long long rows, int k,
                     int words) {
    for (long long r = (long long)blockIdx.x * 256 + threadIdx.x; r < rows; r += (long long)gridDim.x * 256) {
        int i = (int)(r / k);
        int l = I[r];
        if (l < 0) continue;  // empty buffer row
        const uint32_t* bm = bitmap + (size_t)l * words;
        int rank = 0;
        for (int w = 0; w < (i >> 5); ++w) rank += __popc(bm[w]);
        rank += __popc(bm[i >> 5] & ((1u << (i & 31)) - 1u));
        inv[offsets[l] + rank] = (int32_t)r;
    }
}

// A block works on runs of `chunk` (at most COMBINE_CHUNK) consecutive tokens.  Phase 1 resolves the index of the whole run at once:
// the run's list entries (bucket row -> source row and weight) go to LDS, so the chain offsets -> list -> weight
// is waited for once per run and not once per token.  Phase 2 streams the rows: one token per group of `tpr`
// threads, each thread owning 16 bytes of the row (8 bf16 / 4 fp32) per step and accumulating in fp32, with
// nothing but the row loads left to wait for.  CAP = 0: entries come from the CSR lists (expert-ascending).
// CAP > 0: from the token's slot list (capacity CAP), put in ascending row order by repeated minimum -- the
// lists are short, the capacity factor on average.  A run with more than COMBINE_ENTRIES entries (tokens that
// many experts chose) reads its index from memory entry by entry instead.  The order of the additions of a
// token is the order of its list in every case.
constexpr int COMBINE_CHUNK = 32;
constexpr int COMBINE_ENTRIES = 1024;

// Tokens per run: long runs amortise the index look-up, short ones leave the hardware many more blocks than it can
// hold at once, which evens out runs of unequal length (measured on 65536 tokens: 2048 blocks 178 us, 16384 blocks 165).
static int combine_chunk(int64_t n, int tpr) {
    const int tok_per_block = 256 / tpr;
    int chunk = COMBINE_CHUNK;
    while (chunk > tok_per_block && n / chunk < 16384) chunk >>= 1;
    return chunk < tok_per_block ? tok_per_block : chunk;
}

template <typename T, int VEC, int CAP, typename TRow = T>
__global__ void __launch_bounds__(256)
combine_kernel(const TRow* __restrict__ Xe, const float* __restrict__ G, const int32_t* __restrict__ offsets,
               const int32_t* __restrict__ inv, T* __restrict__ Xout, int n, int d, int tpr,
               const float* __restrict__ addend, const int32_t* __restrict__ src_rows, int chunk) {
    typedef T vec_t __attribute__((ext_vector_type(VEC)));
    typedef TRow row_vec_t __attribute__((ext_vector_type(VEC)));  // bucket rows may be fp32 where the output is bf16
    static_assert(COMBINE_CHUNK * (CAP > 0 ? CAP : 1) <= COMBINE_ENTRIES, "slot lists of a run fit the staging arrays");
    __shared__ int ent_src[COMBINE_ENTRIES];
    __shared__ float ent_g[COMBINE_ENTRIES];
    __shared__ int tok_beg[COMBINE_CHUNK + 1];  // CSR: offsets of the run; slots: first entry of token j is j * CAP
    __shared__ int tok_cnt[COMBINE_CHUNK];
    const int tok_per_block = 256 / tpr;
    const int sub = threadIdx.x / tpr, t = threadIdx.x % tpr;
    const int vec_per_row = d / VEC;
    const int chunks = (n + chunk - 1) / chunk;  // chunk <= COMBINE_CHUNK tokens per run
    for (int ch = blockIdx.x; ch < chunks; ch += gridDim.x) {
        const int l0 = ch * chunk;
        const int ntok = n - l0 < chunk ? n - l0 : chunk;
        bool staged = true;
        int beg0 = 0;
        __syncthreads();  // the previous run's rows have been read through these arrays
        if (CAP > 0) {
            if ((int)threadIdx.x < ntok) {
                const int l = l0 + (int)threadIdx.x;
                int cnt = offsets[l];  // experts that chose this token
                cnt = cnt < CAP ? cnt : CAP;
                int raw[CAP > 0 ? CAP : 1];
#pragma unroll
                for (int q = 0; q < CAP; ++q) raw[q] = q < cnt ? inv[(size_t)l * CAP + q] : 0x7FFFFFFF;
                int last = -1;
                for (int p = 0; p < cnt; ++p) {
                    int best = 0x7FFFFFFF;
#pragma unroll
                    for (int q = 0; q < CAP; ++q) best = (raw[q] > last && raw[q] < best) ? raw[q] : best;
                    last = best;
                    ent_src[threadIdx.x * CAP + p] = src_rows != nullptr ? src_rows[best] : best;
                    ent_g[threadIdx.x * CAP + p] = G != nullptr ? G[best] : 1.0f;
                }
                tok_beg[threadIdx.x] = (int)threadIdx.x * CAP;
                tok_cnt[threadIdx.x] = cnt;
            }
            __syncthreads();
        } else {
            if ((int)threadIdx.x <= ntok) tok_beg[threadIdx.x] = offsets[l0 + (int)threadIdx.x];
            __syncthreads();
            beg0 = tok_beg[0];
            const int total = tok_beg[ntok] - beg0;
            staged = total <= COMBINE_ENTRIES;  // the same for every thread of the block
            if (staged) {
                for (int idx = threadIdx.x; idx < total; idx += 256) {
                    const int r = inv[beg0 + idx];
                    ent_src[idx] = src_rows != nullptr ? src_rows[r] : r;
                    ent_g[idx] = G != nullptr ? G[r] : 1.0f;
                }
            }
            if ((int)threadIdx.x < ntok) tok_cnt[threadIdx.x] = tok_beg[threadIdx.x + 1] - tok_beg[threadIdx.x];
            __syncthreads();
        }
        for (int tt = sub; tt < ntok; tt += tok_per_block) {
            const int l = l0 + tt;
            const int cnt = tok_cnt[tt];
            const int eb = tok_beg[tt] - beg0;  // first entry of this token in the staging arrays
            for (int v = t; v < vec_per_row; v += tpr) {
                float acc[VEC];
#pragma unroll
                for (int q = 0; q < VEC; ++q) acc[q] = addend != nullptr ? addend[(size_t)l * d + (size_t)v * VEC + q] : 0.0f;
                // entry p of this token: source row and weight.  src_rows: bucket row r is row src_rows[r] of Xe
                // (identity experts: X_e[i,j,:] = X[I[i,j],:], the gather of Eq. 3 read in place instead of through a
                // materialised X_in); no weights: plain scatter-add of rows
                auto entry = [&](int p, size_t& src, float& g) {
                    if (staged) {
                        src = (size_t)ent_src[eb + p];
                        g = ent_g[eb + p];
                    } else {
                        const int r = inv[beg0 + eb + p];
                        src = src_rows != nullptr ? (size_t)src_rows[r] : (size_t)r;
                        g = G != nullptr ? G[r] : 1.0f;
                    }
                };
                int p = 0;
                // four rows requested together, added in list order: a token that many experts chose does not pay one
                // trip to memory per expert
                for (; p + 4 <= cnt; p += 4) {
                    size_t src[4];
                    float g[4];
                    row_vec_t x[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) entry(p + u, src[u], g[u]);
#pragma unroll
                    for (int u = 0; u < 4; ++u) x[u] = *reinterpret_cast<const row_vec_t*>(Xe + src[u] * d + (size_t)v * VEC);
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int q = 0; q < VEC; ++q) acc[q] = fmaf(g[u], Cvt<TRow>::to_f32(x[u][q]), acc[q]);
                }
                for (; p < cnt; ++p) {
                    size_t src;
                    float g;
                    entry(p, src, g);
                    row_vec_t x = *reinterpret_cast<const row_vec_t*>(Xe + src * d + (size_t)v * VEC);
#pragma unroll
                    for (int q = 0; q < VEC; ++q) acc[q] = fmaf(g, Cvt<TRow>::to_f32(x[q]), acc[q]);
                }
                vec_t o;
#pragma unroll
                for (int q = 0; q < VEC; ++q) o[q] = Cvt<T>::from_f32(acc[q]);
                *reinterpret_cast<vec_t*>(Xout + (size_t)l * d + (size_t)v * VEC) = o;
            }
        }
    }
}

static unsigned blocks_for(long long items) {
    long long b = (items + 255) / 256;
    return (unsigned)(b > 16384 ? 16384 : (b < 1 ? 1 : b));
}

// Builds the token-major index from I alone (stand-alone combine; the forward pass gets it
// from the gate and top-k kernels instead).
int launch_combine_index(const int32_t* I, int64_t n, int64_t e, int64_t k, const CombineIndex& ix,
                         hipStream_t stream) {
    const long long rows = (long long)e * k;
    if (ix.use_slots) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(n)), dim3(256), 0, stream, (uint32_t*)ix.slot_cnt,
                           (long long)n, 0u);
        hipLaunchKernelGGL(slots_kernel, dim3(blocks_for(rows)), dim3(256), 0, stream, I, ix.slot_cnt, ix.slots, rows,
                           ix.slot_cap);
    } else {
        const int words = (int)ceil_div(e, 32);
        hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for((long long)n * words)), dim3(256), 0, stream, ix.bitmap,
                           (long long)n * words, 0u);
        hipLaunchKernelGGL(bitmap_kernel, dim3(blocks_for(rows)), dim3(256), 0, stream, I, ix.bitmap, rows, (int)k,
                           words);
    }
    return check_launch();
}

// Finishes the CSR form from a filled bitmap: offsets (exclusive scan) and the expert-ascending row lists.
int launch_combine_csr(const int32_t* I, int64_t n, int64_t e, int64_t k, const CombineIndex& ix, hipStream_t stream) {
    const long long rows = (long long)e * k;
    const int words = (int)ceil_div(e, 32);
    // token range of a scan block: 1024 tokens, more only when that would need over 1024 blocks
    const int tpb = (int)(ceil_div(ceil_div(n, 1024), 1024) * 1024);
    const unsigned scan_blocks = (unsigned)ceil_div(n, tpb);
    uint32_t* block_tot = reinterpret_cast<uint32_t*>(ix.slot_cnt);  // [n] words, idle in the CSR form
    hipLaunchKernelGGL(block_counts_kernel, dim3(scan_blocks), dim3(1024), 0, stream, ix.bitmap, block_tot, (int)n,
                       words, tpb);
    hipLaunchKernelGGL(offsets_kernel, dim3(scan_blocks), dim3(1024), 0, stream, ix.bitmap, block_tot, ix.offsets,
                       (int)n, words, tpb);
    hipLaunchKernelGGL(inverse_index_kernel, dim3(blocks_for(rows)), dim3(256), 0, stream, I, ix.bitmap, ix.offsets,
                       ix.inv, rows, (int)k, words);
    return check_launch();
}

// Applies Eq. 4 given a filled index (slot lists, or the bitmap from which the CSR lists are finished here).
// G == nullptr adds the rows unweighted; `addend` (fp32 [n,d], optional) is the starting value of every row;
// `src_rows` (optional, [e*k]) redirects bucket row r to row src_rows[r] of Xe; `rows_f32`: the bucket rows are
// fp32 although the output is bf16 (the last product of the backward pass is kept unrounded).
int launch_combine(const void* Xe, const float* G, const int32_t* I, void* Xout, int64_t n, int64_t d,
                   int64_t e, int64_t k, int dtype, const CombineIndex& ix, hipStream_t stream,
                   const float* addend, bool csr_ready, const int32_t* src_rows, bool rows_f32) {
    const int32_t* offs = ix.slot_cnt;
    const int32_t* list = ix.slots;
    if (!ix.use_slots) {
        if (!csr_ready) {
            int rc = launch_combine_csr(I, n, e, k, ix, stream);
            if (rc != EC_OK) return rc;
        }
        offs = ix.offsets;
        list = ix.inv;
    }
#define EC_COMBINE_LAUNCH(TYPE, VECV, NVEC)                                                                   \
    do {                                                                                                      \
        int tpr = pick_threads_per_row(NVEC);                                                                 \
        const int chunk = combine_chunk(n, tpr);                                                              \
        long long blocks = ceil_div(n, chunk);                                                                \
        if (blocks > (1 << 20)) blocks = 1 << 20;                                                             \
        dim3 grid((unsigned)blocks), block(256);                                                              \
        if (!ix.use_slots)                                                                                    \
            hipLaunchKernelGGL((combine_kernel<TYPE, VECV, 0>), grid, block, 0, stream, (const TYPE*)Xe, G,   \
                               offs, list, (TYPE*)Xout, (int)n, (int)d, tpr, addend, src_rows, chunk);                                 \
        else if (ix.slot_cap == 4)                                                                            \
            hipLaunchKernelGGL((combine_kernel<TYPE, VECV, 4>), grid, block, 0, stream, (const TYPE*)Xe, G,   \
                               offs, list, (TYPE*)Xout, (int)n, (int)d, tpr, addend, src_rows, chunk);                                 \
        else if (ix.slot_cap == 8)                                                                            \
            hipLaunchKernelGGL((combine_kernel<TYPE, VECV, 8>), grid, block, 0, stream, (const TYPE*)Xe, G,   \
                               offs, list, (TYPE*)Xout, (int)n, (int)d, tpr, addend, src_rows, chunk);                                 \
        else                                                                                                  \
            hipLaunchKernelGGL((combine_kernel<TYPE, VECV, 16>), grid, block, 0, stream, (const TYPE*)Xe, G,  \
                               offs, list, (TYPE*)Xout, (int)n, (int)d, tpr, addend, src_rows, chunk);                                 \
    } while (0)
    if (dtype == EC_BF16 && rows_f32) {
        int tpr = pick_threads_per_row(d / 8);
        const int chunk = combine_chunk(n, tpr);
        long long blocks = ceil_div(n, chunk);
        if (blocks > (1 << 20)) blocks = 1 << 20;
        const dim3 grid((unsigned)blocks), block(256);
#define EC_COMBINE_F32ROWS(CAPV)                                                                                   \
    hipLaunchKernelGGL((combine_kernel<bf16_t, 8, CAPV, float>), grid, block, 0, stream, (const float*)Xe, G, offs, list, \
                       (bf16_t*)Xout, (int)n, (int)d, tpr, addend, src_rows, chunk)
        if (!ix.use_slots) EC_COMBINE_F32ROWS(0);
        else if (ix.slot_cap == 4) EC_COMBINE_F32ROWS(4);
        else if (ix.slot_cap == 8) EC_COMBINE_F32ROWS(8);
        else EC_COMBINE_F32ROWS(16);
#undef EC_COMBINE_F32ROWS
    } else if (dtype == EC_BF16) EC_COMBINE_LAUNCH(bf16_t, 8, d / 8);
    else if (d % 4 == 0) EC_COMBINE_LAUNCH(float, 4, d / 4);
    else EC_COMBINE_LAUNCH(float, 1, d);
#undef EC_COMBINE_LAUNCH
    return check_launch();
}

// Eq. 4 with the token-major index in the library's own static device array (nothing is allocated).
// The array's device address is looked up once per GPU, with that GPU current; host code only ever
// uses that address, never the array's name.
int combine_static(const void* Xe, const float* G, const int32_t* I, void* Xout, int64_t n, int64_t d, int64_t e,
                   int64_t k, int dtype, hipStream_t stream) {
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static unsigned char* scratch_ptr[MAX_DEVICES] = {};
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        set_last_hip_error(err != hipSuccess ? err : hipErrorInvalidDevice);
        return EC_ERR_HIP;
    }
    unsigned char* base;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (scratch_ptr[dev] == nullptr) {
            void* p = nullptr;
            err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (err != hipSuccess || p == nullptr) {
                set_last_hip_error(err != hipSuccess ? err : hipErrorInvalidSymbol);
                return EC_ERR_HIP;
            }
            scratch_ptr[dev] = static_cast<unsigned char*>(p);
        }
        base = scratch_ptr[dev];
    }
    // carve-up: only the form of the index that this expert count uses
    CombineIndex ix;
    ix.use_slots = e <= COMBINE_SLOT_CAP;
    ix.slot_cap = e <= 4 ? 4 : e <= 8 ? 8 : 16;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t a = off; off = align_up(off + bytes, 256); return a; };
    size_t o_cnt, o_slots = 0, o_bitmap = 0, o_offsets = 0, o_inv = 0;
    if (ix.use_slots) {
        o_cnt = take((size_t)n * 4);
        o_slots = take((size_t)n * ix.slot_cap * 4);
    } else {
        o_cnt = take(1024 * 4);  // totals of the scan blocks (at most 1024 of them)
        o_bitmap = take((size_t)n * (size_t)ceil_div(e, 32) * 4);
        o_offsets = take((size_t)(n + 1) * 4);
        o_inv = take((size_t)e * k * 4);
    }
    if (off > (size_t)EC_MOE_STATIC_SCRATCH_BYTES) return EC_ERR_UNSUPPORTED;
    ix.slot_cnt = reinterpret_cast<int32_t*>(base + o_cnt);
    ix.slots = reinterpret_cast<int32_t*>(base + o_slots);
    ix.bitmap = reinterpret_cast<uint32_t*>(base + o_bitmap);
    ix.offsets = reinterpret_cast<int32_t*>(base + o_offsets);
    ix.inv = reinterpret_cast<int32_t*>(base + o_inv);
    int rc = launch_combine_index(I, n, e, k, ix, stream);  // clears the counters / bitmap with a fill kernel first
    if (rc != EC_OK) return rc;
    return launch_combine(Xe, G, I, Xout, n, d, e, k, dtype, ix, stream);
}

}  // namespace ecmoe
