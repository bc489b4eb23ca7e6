// Internal helpers shared by the HIP translation units of libec_moe.so.
// Nothing here is part of the public ABI (include/ec_moe.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ec_moe.h"

namespace ecmoe {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;  // CDNA wavefront width

// Per-thread record of the last failing HIP call (read by ec_moe_last_hip_error).
void set_last_hip_error(hipError_t err);

// Returns EC_OK or records the error and returns EC_ERR_HIP.
inline int check_launch() {
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        set_last_hip_error(err);
        return EC_ERR_HIP;
    }
    return EC_OK;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t elem_size(int dtype) { return (dtype == EC_BF16 || dtype == EC_BF16_HILO) ? 2 : 4; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---------------------------------------------------------------------------
// Workspace layout.  One carve-up serves every entry point; regions that are
// never live together in ec_moe_forward are still kept apart, the sizes are
// small next to the activations.
// ---------------------------------------------------------------------------
struct WsLayout {
    size_t st;         // float [e, n]: S^T
    size_t g;          // float [e, k]
    size_t i;          // int32 [e, k]
    size_t xin;        // dtype [e, k, d]
    size_t h;          // dtype [e, k, d_ff]
    size_t xe;         // dtype [e, k, d]
    size_t h_lo;       // bf16 [e, k, d_ff]: act(A) - H                            (EC_BF16_HILO only)
    size_t xe32;       // float [e, k, d]: X_e unrounded                           (EC_BF16_HILO only)
    size_t bitmap;     // uint32 [n, ceil(e/32)]: which experts chose a token      (CSR form, e > COMBINE_SLOT_CAP)
    size_t offsets;    // int32 [n+1]: CSR row starts of the token-major index
    size_t inv;        // int32 [e*k]: bucket rows (i*k+j) grouped by token, expert-ascending
    size_t slot_cnt;   // int32 [n]: experts that chose a token                     (slot form, e <= COMBINE_SLOT_CAP)
    size_t slots;      // int32 [n, COMBINE_SLOT_CAP]: their bucket rows, arrival order
    size_t choice;     // int32 [8, n]: every token's chosen experts, rank-major (token-choice routing)
    size_t bwd;        // start of the backward-only region
    size_t total;
};

WsLayout ws_layout(int64_t n, int64_t d, int64_t e, int64_t k, int64_t d_ff, int dtype, int with_backward);

// Sizes of the backward-only region (defined with the backward kernels).
size_t bwd_ws_bytes(int64_t n, int64_t d, int64_t e, int64_t k, int64_t d_ff, int dtype, bool hilo = false);

// Token-major index of the routing handed from the top-k stage to the combine stage.
constexpr int COMBINE_SLOT_CAP = 16;
struct CombineIndex {
    bool use_slots;      // e <= COMBINE_SLOT_CAP: per-token slot lists; otherwise bitmap + CSR
    int32_t* slot_cnt;   // [n]
    int32_t* slots;      // [n, slot_cap]
    int slot_cap;
    uint32_t* bitmap;    // [n, ceil(e/32)]
    int32_t* offsets;    // [n+1]
    int32_t* inv;        // [e*k]
};
CombineIndex combine_index_at(void* ws_base, const WsLayout& L, int64_t e);
// 32-bit words that must be zero before the index is filled, and where they start.
inline uint32_t* combine_zero_ptr(const CombineIndex& ix) { return ix.use_slots ? (uint32_t*)ix.slot_cnt : ix.bitmap; }
inline int64_t combine_zero_words(const CombineIndex& ix, int64_t n, int64_t e) {
    return ix.use_slots ? n : n * ceil_div(e, 32);
}

// ---------------------------------------------------------------------------
// Launchers (host side, arguments already validated by the ABI layer).
// ---------------------------------------------------------------------------
int launch_gate(const void* X, const void* Wg, float* S, float* St, int64_t n, int64_t d, int64_t e,
                int dtype, uint32_t* zero_buf, int64_t zero_words, hipStream_t stream);
int launch_topk(const float* St, int64_t n, int64_t e, int64_t k, float* G, int32_t* I,
                int32_t* slot_cnt, int32_t* slots, int slot_cap, uint32_t* bitmap, hipStream_t stream,
                int64_t groups = 1);
int launch_token_choice(const float* S, int64_t n, int64_t e, int64_t m, int64_t cap, float* G, int32_t* I,
                        int32_t* load, int32_t* choice_ws, int32_t* slot_cnt, int32_t* slots, int slot_cap,
                        uint32_t* bitmap, hipStream_t stream);
size_t capped_ws_bytes(int64_t n, int64_t e);
int launch_capped_assignment(const float* St, int64_t n, int64_t e, int64_t k, double b, double lambda,
                             int64_t iters, float* A, void* ws, hipStream_t stream);
int launch_gather_scores(const float* St, const int32_t* I, float* G, int64_t n, int64_t e, int64_t k,
                         hipStream_t stream);
int launch_combine_index(const int32_t* I, int64_t n, int64_t e, int64_t k, const CombineIndex& ix,
                         hipStream_t stream);
int launch_dispatch(const void* X, const int32_t* I, void* Xin, int64_t n, int64_t d, int64_t e, int64_t k,
                    int dtype, hipStream_t stream);
bool ffn_can_gather(int dtype, int64_t n, int64_t k, int64_t d, int64_t d_ff);
bool ffn_can_hilo(int dtype, int64_t k, int64_t d, int64_t d_ff);
int launch_ffn(const void* Xin, const void* X, const int32_t* I, int64_t n, const void* W1, const void* W2, void* Xe,
               void* A_save, void* H, int64_t e, int64_t k, int64_t d, int64_t d_ff, int act, int dtype,
               hipStream_t stream, void* H_lo = nullptr, float* Xe32 = nullptr);
int launch_combine_csr(const int32_t* I, int64_t n, int64_t e, int64_t k, const CombineIndex& ix, hipStream_t stream);
int launch_combine(const void* Xe, const float* G, const int32_t* I, void* Xout, int64_t n, int64_t d,
                   int64_t e, int64_t k, int dtype, const CombineIndex& ix, hipStream_t stream,
                   const float* addend = nullptr, bool csr_ready = false, const int32_t* src_rows = nullptr,
                   bool rows_f32 = false);
int combine_static(const void* Xe, const float* G, const int32_t* I, void* Xout, int64_t n, int64_t d, int64_t e,
                   int64_t k, int dtype, hipStream_t stream);
int launch_backward(const void* dY, const void* X, const void* Wg, const void* W1, const void* W2,
                    const float* S, const float* G, const int32_t* I, const void* Xin, const void* A,
                    const void* H, const void* Xe, void* dX, float* dWg, float* dW1, float* dW2,
                    int64_t n, int64_t d, int64_t e, int64_t k, int64_t d_ff, int act, int dtype,
                    void* ws, const WsLayout& L, hipStream_t stream, hipEvent_t* marks = nullptr, bool hilo = false);
constexpr int BWD_STAGES = 9;  // rows, dW2, dA, dW1, dX_in, index, dZ, gate products, scatter

// ---------------------------------------------------------------------------
// Device helpers.
// ---------------------------------------------------------------------------
template <typename T> struct Cvt;
template <> struct Cvt<float> {
    static __device__ __forceinline__ float to_f32(float v) { return v; }
    static __device__ __forceinline__ float from_f32(float v) { return v; }
};
template <> struct Cvt<bf16_t> {
    static __device__ __forceinline__ float to_f32(bf16_t v) { return static_cast<float>(v); }
    static __device__ __forceinline__ bf16_t from_f32(float v) { return static_cast<bf16_t>(v); }  // RNE
};

__device__ __forceinline__ float wave_reduce_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}
__device__ __forceinline__ float wave_reduce_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Exact-erf GeLU, a * Phi(a) (Hendrycks & Gimpel), evaluated in fp32.
__device__ __forceinline__ float gelu_erf(float a) { return 0.5f * a * (1.0f + erff(a * 0.70710678118654752440f)); }

template <int ACT>
__device__ __forceinline__ float apply_act(float a) {
    if (ACT == EC_ACT_RELU) return fmaxf(a, 0.0f);
    if (ACT == EC_ACT_GELU) return gelu_erf(a);
    return a;
}

}  // namespace ecmoe
