// C ABI of libec_moe.so: argument validation, workspace carving, and the
// forward chain gate -> TopK over tokens -> dispatch -> expert FFN -> combine
// (Sec. 3.2, Eq. 1-4).  All arithmetic lives in the kernels of the other files.
#include <cmath>

#include "ec_common.h"

namespace ecmoe {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t err) { g_last_hip_error = (int)err; }

WsLayout ws_layout(int64_t n, int64_t d, int64_t e, int64_t k, int64_t d_ff, int dtype, int with_backward) {
    WsLayout L;
    const bool hilo = dtype == EC_BF16_HILO && d_ff > 0;  // identity experts: no product, nothing to carry in two parts
    if (dtype == EC_BF16_HILO) dtype = EC_BF16;
    const size_t es = elem_size(dtype);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    L.st = take((size_t)e * n * 4);
    L.g = take((size_t)e * k * 4);
    L.i = take((size_t)e * k * 4);
    L.xin = take((size_t)e * k * d * es);
    L.h = take((size_t)e * k * (size_t)(d_ff > 0 ? d_ff : 0) * es);
    L.xe = take((size_t)e * k * d * es);
    L.h_lo = take(hilo ? (size_t)e * k * (size_t)(d_ff > 0 ? d_ff : 0) * 2 : 0);
    L.xe32 = take(hilo ? (size_t)e * k * d * 4 : 0);
    L.bitmap = take((size_t)n * (size_t)ceil_div(e, 32) * 4);
    L.offsets = take((size_t)(n + 1) * 4);
    L.inv = take((size_t)e * k * 4);
    L.slot_cnt = take((size_t)n * 4);
    L.slots = take((size_t)n * COMBINE_SLOT_CAP * 4);
    L.choice = take((size_t)n * 8 * 4);
    L.bwd = off;
    if (with_backward) take(bwd_ws_bytes(n, d, e, k, d_ff, dtype, hilo));
    L.total = off;
    return L;
}

static bool sizes_ok(int64_t n, int64_t d, int64_t e, int64_t k) {
    return n > 0 && d > 0 && e > 0 && k >= 1 && k <= n && n < (int64_t)1 << 31 && d < (int64_t)1 << 31 &&
           e <= EC_MOE_MAX_EXPERTS && e * k < (int64_t)1 << 31;
}
static bool dtype_ok(int dtype) { return dtype == EC_F32 || dtype == EC_BF16 || dtype == EC_BF16_HILO; }
// EC_BF16_HILO stores what EC_BF16 stores; `*hilo` says whether the two-part operands were asked for.
static int storage_dtype(int dtype, bool* hilo = nullptr) {
    if (hilo != nullptr) *hilo = dtype == EC_BF16_HILO;
    return dtype == EC_BF16_HILO ? EC_BF16 : dtype;
}
static bool act_ok(int act) { return act == EC_ACT_RELU || act == EC_ACT_GELU || act == EC_ACT_IDENTITY; }
static bool width_ok(int64_t w, int dtype) { return dtype == EC_F32 || (w % 8) == 0; }
template <typename... P>
static bool all_aligned(P... ptrs) {
    bool ok = true;
    const void* list[] = {ptrs...};
    for (const void* q : list) ok = ok && (q == nullptr || aligned16(q));
    return ok;
}
static bool ws_ok(const void* ws, size_t ws_bytes, size_t need) {
    return need == 0 || (ws != nullptr && ws_bytes >= need && (reinterpret_cast<uintptr_t>(ws) & 255u) == 0);
}
static unsigned char* at(void* ws, size_t off) { return static_cast<unsigned char*>(ws) + off; }

CombineIndex combine_index_at(void* ws, const WsLayout& L, int64_t e) {
    CombineIndex ix;
    ix.use_slots = e <= COMBINE_SLOT_CAP;
    ix.slot_cap = e <= 4 ? 4 : e <= 8 ? 8 : 16;
    ix.slot_cnt = (int32_t*)at(ws, L.slot_cnt);
    ix.slots = (int32_t*)at(ws, L.slots);
    ix.bitmap = (uint32_t*)at(ws, L.bitmap);
    ix.offsets = (int32_t*)at(ws, L.offsets);
    ix.inv = (int32_t*)at(ws, L.inv);
    return ix;
}

}  // namespace ecmoe

using namespace ecmoe;

extern "C" {

int ec_moe_capacity(int64_t n, int64_t e, double c, int64_t* k) {
    if (k == nullptr || n <= 0 || e <= 0 || !(c > 0.0) || !std::isfinite(c)) return EC_ERR_INVALID_ARG;
    double kd = std::floor((double)n * c / (double)e);
    if (!(kd >= 1.0) || kd > (double)n) return EC_ERR_INVALID_ARG;
    *k = (int64_t)kd;
    return EC_OK;
}

size_t ec_moe_workspace_bytes(int64_t n, int64_t d, int64_t e, int64_t k, int64_t d_ff, int dtype,
                              int with_backward) {
    if (!sizes_ok(n, d, e, k) || d_ff < 0 || !dtype_ok(dtype)) return 0;
    if (dtype == EC_BF16_HILO && d_ff > 0 && !ffn_can_hilo(EC_BF16, k, d, d_ff)) return 0;  // no such layer: see EC_ERR_UNSUPPORTED
    return ws_layout(n, d, e, k, d_ff, dtype, with_backward).total;
}

int ec_moe_gate(const void* X, const void* Wg, float* S, float* St, int64_t n, int64_t d, int64_t e, int dtype,
                void* ws, size_t ws_bytes, void* stream) {
    if (!X || !Wg || (!S && !St) || n <= 0 || d <= 0 || e <= 0 || e > EC_MOE_MAX_EXPERTS || n >= (int64_t)1 << 31 ||
        !dtype_ok(dtype) || !all_aligned(X, Wg, S, St))
        return EC_ERR_INVALID_ARG;
    dtype = storage_dtype(dtype);
    (void)ws; (void)ws_bytes;  // the gate needs no scratch
    return launch_gate(X, Wg, S, St, n, d, e, dtype, nullptr, 0, (hipStream_t)stream);
}

int ec_moe_topk_tokens(const float* St, int64_t n, int64_t e, int64_t k, float* G, int32_t* I, void* ws,
                       size_t ws_bytes, void* stream) {
    if (!St || !G || !I || !sizes_ok(n, 1, e, k) || !all_aligned(St, G, I)) return EC_ERR_INVALID_ARG;
    (void)ws; (void)ws_bytes;  // the selection needs no scratch in global memory
    return launch_topk(St, n, e, k, G, I, nullptr, nullptr, 0, nullptr, (hipStream_t)stream);
}

int ec_moe_topk_tokens_grouped(const float* St, int64_t n, int64_t e, int64_t groups, int64_t k_g, float* G,
                               int32_t* I, void* ws, size_t ws_bytes, void* stream) {
    if (groups <= 0 || n <= 0 || n % groups != 0) return EC_ERR_INVALID_ARG;
    if (!St || !G || !I || !sizes_ok(n / groups, 1, e, k_g) || !sizes_ok(n, 1, e, groups * k_g) ||
        !all_aligned(St, G, I))
        return EC_ERR_INVALID_ARG;
    (void)ws; (void)ws_bytes;
    return launch_topk(St, n, e, k_g, G, I, nullptr, nullptr, 0, nullptr, (hipStream_t)stream, groups);
}

int ec_moe_dispatch(const void* X, const int32_t* I, void* Xin, int64_t n, int64_t d, int64_t e, int64_t k,
                    int dtype, void* stream) {
    if (!X || !I || !Xin || !sizes_ok(n, d, e, k) || !dtype_ok(dtype) || !width_ok(d, dtype) ||
        !all_aligned(X, I, Xin))
        return EC_ERR_INVALID_ARG;
    dtype = storage_dtype(dtype);
    return launch_dispatch(X, I, Xin, n, d, e, k, dtype, (hipStream_t)stream);
}

int ec_moe_expert_ffn(const void* Xin, const void* W1, const void* W2, void* Xe, void* A_save, void* H_save,
                      int64_t e, int64_t k, int64_t d, int64_t d_ff, int act, int dtype, void* ws, size_t ws_bytes,
                      void* stream) {
    if (!Xin || !W1 || !W2 || !Xe || e <= 0 || k <= 0 || d <= 0 || d_ff <= 0 || e > EC_MOE_MAX_EXPERTS ||
        k >= (int64_t)1 << 31 || d >= (int64_t)1 << 31 || d_ff >= (int64_t)1 << 31 || !dtype_ok(dtype) ||
        !act_ok(act) || !width_ok(d, dtype) || !width_ok(d_ff, dtype) ||
        !all_aligned(Xin, W1, W2, Xe, A_save, H_save))
        return EC_ERR_INVALID_ARG;
    bool hilo = false;
    dtype = storage_dtype(dtype, &hilo);
    if (hilo && !ffn_can_hilo(dtype, k, d, d_ff)) return EC_ERR_UNSUPPORTED;
    // workspace: H unless the caller keeps it; with two-part operands the remainder of H and X_e unrounded
    const size_t h_bytes = H_save ? 0 : align_up((size_t)e * k * d_ff * elem_size(dtype), 256);
    const size_t hlo_bytes = hilo ? align_up((size_t)e * k * d_ff * 2, 256) : 0;
    const size_t xe32_bytes = hilo ? align_up((size_t)e * k * d * 4, 256) : 0;
    if (!ws_ok(ws, ws_bytes, h_bytes + hlo_bytes + xe32_bytes)) return EC_ERR_WORKSPACE;
    void* H = H_save ? H_save : ws;
    void* H_lo = hilo ? at(ws, h_bytes) : nullptr;
    float* Xe32 = hilo ? (float*)at(ws, h_bytes + hlo_bytes) : nullptr;
    return launch_ffn(Xin, nullptr, nullptr, 0, W1, W2, Xe, A_save, H, e, k, d, d_ff, act, dtype, (hipStream_t)stream, H_lo,
                      Xe32);
}

int ec_moe_combine(const void* Xe, const float* G, const int32_t* I, void* Xout, int64_t n, int64_t d, int64_t e,
                   int64_t k, int dtype, void* ws, size_t ws_bytes, void* stream) {
    if (!Xe || !G || !I || !Xout || !sizes_ok(n, d, e, k) || !dtype_ok(dtype) || !width_ok(d, dtype) ||
        !all_aligned(Xe, G, I, Xout))
        return EC_ERR_INVALID_ARG;
    dtype = storage_dtype(dtype);
    // token-major index: carved from the front of the workspace
    WsLayout L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t a = off; off = align_up(off + bytes, 256); return a; };
    L.bitmap = take((size_t)n * (size_t)ceil_div(e, 32) * 4);
    L.offsets = take((size_t)(n + 1) * 4);
    L.inv = take((size_t)e * k * 4);
    L.slot_cnt = take((size_t)n * 4);
    L.slots = take((size_t)n * COMBINE_SLOT_CAP * 4);
    if (!ws_ok(ws, ws_bytes, off)) return EC_ERR_WORKSPACE;
    const CombineIndex ix = combine_index_at(ws, L, e);
    int rc = launch_combine_index(I, n, e, k, ix, (hipStream_t)stream);
    if (rc != EC_OK) return rc;
    return launch_combine(Xe, G, I, Xout, n, d, e, k, dtype, ix, (hipStream_t)stream);
}

int ec_moe_combine_static(const void* Xe, const float* G, const int32_t* I, void* Xout, int64_t n, int64_t d,
                          int64_t e, int64_t k, int dtype, void* stream) {
    if (!Xe || !G || !I || !Xout || !sizes_ok(n, d, e, k) || !dtype_ok(dtype) || !width_ok(d, dtype) ||
        !all_aligned(Xe, G, I, Xout))
        return EC_ERR_INVALID_ARG;
    dtype = storage_dtype(dtype);
    return combine_static(Xe, G, I, Xout, n, d, e, k, dtype, (hipStream_t)stream);
}

// The expert products of Eq. 3 and the sum of Eq. 4 on filled buckets: rows of the buckets come from Xin, or from X
// through I when Xin == nullptr (the gather fused into the first product).  `hilo`: H leaves the first product as
// high part + remainder and X_e reaches the sum unrounded (the bf16 X_e is written only for a caller who asks for it).
static int experts_then_combine(const void* Xin, const void* X, const int32_t* I, const float* G, const void* W1,
                                const void* W2, void* Xout, void* Xe_out, void* A_out, void* H_out, int64_t n, int64_t d,
                                int64_t e, int64_t k, int64_t d_ff, int act, int dtype, bool hilo, void* ws,
                                const WsLayout& L, const CombineIndex& ix, hipStream_t st) {
    void* H = H_out ? H_out : at(ws, L.h);
    if (hilo) {
        float* Xe32 = (float*)at(ws, L.xe32);
        int rc = launch_ffn(Xin, X, I, n, W1, W2, Xe_out, A_out, H, e, k, d, d_ff, act, dtype, st, at(ws, L.h_lo), Xe32);
        if (rc != EC_OK) return rc;
        return launch_combine(Xe32, G, I, Xout, n, d, e, k, dtype, ix, st, nullptr, false, nullptr, true);
    }
    void* Xe = Xe_out ? Xe_out : at(ws, L.xe);
    int rc = launch_ffn(Xin, X, I, n, W1, W2, Xe, A_out, H, e, k, d, d_ff, act, dtype, st);
    if (rc != EC_OK) return rc;
    return launch_combine(Xe, G, I, Xout, n, d, e, k, dtype, ix, st);
}

// The layer with TopK taken inside each of `groups` equal runs of tokens (groups = 1: Eq. 2 as printed).
static int forward_impl(const void* X, const void* Wg, const void* W1, const void* W2, double c, int64_t groups,
                        void* Xout, float* S_out, float* G_out, int32_t* I_out, void* Xin_out, void* A_out,
                        void* H_out, void* Xe_out, int64_t n, int64_t d, int64_t e, int64_t d_ff, int act, int dtype,
                        void* ws, size_t ws_bytes, void* stream) {
    if (groups <= 0 || n <= 0 || n % groups != 0) return EC_ERR_INVALID_ARG;
    int64_t k_g = 0;
    if (ec_moe_capacity(n / groups, e, c, &k_g) != EC_OK) return EC_ERR_INVALID_ARG;
    const int64_t k = groups * k_g;  // rows of an expert's bucket
    const bool identity = (W1 == nullptr && W2 == nullptr);
    if (!X || !Wg || !Xout || !sizes_ok(n, d, e, k) || !dtype_ok(dtype) || !act_ok(act) || !width_ok(d, dtype) ||
        !all_aligned(X, Wg, W1, W2, Xout, S_out, G_out, I_out, Xin_out, A_out, H_out, Xe_out))
        return EC_ERR_INVALID_ARG;
    if (identity) {
        if (act != EC_ACT_IDENTITY) return EC_ERR_INVALID_ARG;
        d_ff = 0;
    } else {
        if (!W1 || !W2 || d_ff <= 0 || d_ff >= (int64_t)1 << 31 || !width_ok(d_ff, dtype))
            return EC_ERR_INVALID_ARG;
    }
    const WsLayout L = ws_layout(n, d, e, k, d_ff, dtype, 0);
    if (!ws_ok(ws, ws_bytes, L.total)) return EC_ERR_WORKSPACE;
    bool hilo = false;
    dtype = storage_dtype(dtype, &hilo);
    if (identity) hilo = false;  // no product, nothing to carry in two parts
    if (hilo && !ffn_can_hilo(dtype, k, d, d_ff)) return EC_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;

    float* St = (float*)at(ws, L.st);
    float* G = G_out ? G_out : (float*)at(ws, L.g);
    int32_t* I = I_out ? I_out : (int32_t*)at(ws, L.i);
    void* Xin = Xin_out ? Xin_out : at(ws, L.xin);

    const CombineIndex ix = combine_index_at(ws, L, e);
    int rc = launch_gate(X, Wg, S_out, St, n, d, e, dtype, combine_zero_ptr(ix), combine_zero_words(ix, n, e), st);
    if (rc != EC_OK) return rc;
    rc = launch_topk(St, n, e, k_g, G, I, ix.use_slots ? ix.slot_cnt : nullptr, ix.slots, ix.slot_cap,
                     ix.use_slots ? nullptr : ix.bitmap, st, groups);
    if (rc != EC_OK) return rc;
    // The bucket gather is fused into the first expert product unless the caller wants X_in itself.  With
    // identity experts X_e = X_in = the gathered rows of X: unless the caller asks for one of them, the
    // combine reads those rows in place through I.
    const bool fused_gather = !identity && Xin_out == nullptr && ffn_can_gather(dtype, n, k, d, d_ff);
    if (identity) {
        void* rows = Xin_out ? Xin_out : Xe_out;
        if (rows == nullptr) return launch_combine(X, G, I, Xout, n, d, e, k, dtype, ix, st, nullptr, false, I);
        rc = launch_dispatch(X, I, rows, n, d, e, k, dtype, st);
        if (rc != EC_OK) return rc;
        if (Xin_out && Xe_out) {
            rc = launch_dispatch(X, I, Xe_out, n, d, e, k, dtype, st);
            if (rc != EC_OK) return rc;
        }
        return launch_combine(rows, G, I, Xout, n, d, e, k, dtype, ix, st);
    }
    if (!fused_gather) {
        rc = launch_dispatch(X, I, Xin, n, d, e, k, dtype, st);
        if (rc != EC_OK) return rc;
    }
    return experts_then_combine(fused_gather ? nullptr : Xin, X, I, G, W1, W2, Xout, Xe_out, A_out, H_out, n, d, e, k,
                                d_ff, act, dtype, hilo, ws, L, ix, st);
}

int ec_moe_forward(const void* X, const void* Wg, const void* W1, const void* W2, double c, void* Xout,
                   float* S_out, float* G_out, int32_t* I_out, void* Xin_out, void* A_out, void* H_out,
                   void* Xe_out, int64_t n, int64_t d, int64_t e, int64_t d_ff, int act, int dtype, void* ws,
                   size_t ws_bytes, void* stream) {
    return forward_impl(X, Wg, W1, W2, c, 1, Xout, S_out, G_out, I_out, Xin_out, A_out, H_out, Xe_out, n, d, e, d_ff,
                        act, dtype, ws, ws_bytes, stream);
}

int ec_moe_forward_grouped(const void* X, const void* Wg, const void* W1, const void* W2, double c, int64_t groups,
                           void* Xout, float* S_out, float* G_out, int32_t* I_out, void* Xin_out, void* A_out,
                           void* H_out, void* Xe_out, int64_t n, int64_t d, int64_t e, int64_t d_ff, int act,
                           int dtype, void* ws, size_t ws_bytes, void* stream) {
    return forward_impl(X, Wg, W1, W2, c, groups, Xout, S_out, G_out, I_out, Xin_out, A_out, H_out, Xe_out, n, d, e,
                        d_ff, act, dtype, ws, ws_bytes, stream);
}

int ec_moe_token_choice(const float* S, int64_t n, int64_t e, int64_t m, int64_t cap, float* G, int32_t* I,
                        int32_t* load, void* ws, size_t ws_bytes, void* stream) {
    if (!S || !G || !I || n <= 0 || e <= 0 || e > EC_MOE_MAX_EXPERTS || n >= (int64_t)1 << 31 || m < 1 || m > e ||
        m > 8 || cap < 1 || cap > n || e * cap >= (int64_t)1 << 31 || !all_aligned(S, G, I, load))
        return EC_ERR_INVALID_ARG;
    if (!ws_ok(ws, ws_bytes, (size_t)n * 8 * 4)) return EC_ERR_WORKSPACE;
    return launch_token_choice(S, n, e, m, cap, G, I, load, (int32_t*)ws, nullptr, nullptr, 0, nullptr,
                               (hipStream_t)stream);
}

int ec_moe_forward_token_choice(const void* X, const void* Wg, const void* W1, const void* W2, double c, int64_t m,
                                void* Xout, float* S_out, float* G_out, int32_t* I_out, int32_t* load_out,
                                void* Xin_out, void* A_out, void* H_out, void* Xe_out, int64_t n, int64_t d, int64_t e,
                                int64_t d_ff, int act, int dtype, void* ws, size_t ws_bytes, void* stream) {
    int64_t k = 0;  // rows of an expert's buffer
    if (ec_moe_capacity(n, e, c, &k) != EC_OK || m < 1 || m > e || m > 8) return EC_ERR_INVALID_ARG;
    const bool identity = (W1 == nullptr && W2 == nullptr);
    if (!X || !Wg || !Xout || !sizes_ok(n, d, e, k) || !dtype_ok(dtype) || !act_ok(act) || !width_ok(d, dtype) ||
        !all_aligned(X, Wg, W1, W2, Xout, S_out, G_out, I_out, load_out, Xin_out, A_out, H_out, Xe_out))
        return EC_ERR_INVALID_ARG;
    if (identity) {
        if (act != EC_ACT_IDENTITY) return EC_ERR_INVALID_ARG;
        d_ff = 0;
    } else {
        if (!W1 || !W2 || d_ff <= 0 || d_ff >= (int64_t)1 << 31 || !width_ok(d_ff, dtype))
            return EC_ERR_INVALID_ARG;
    }
    const WsLayout L = ws_layout(n, d, e, k, d_ff, dtype, 0);
    if (!ws_ok(ws, ws_bytes, L.total)) return EC_ERR_WORKSPACE;
    bool hilo = false;
    dtype = storage_dtype(dtype, &hilo);
    if (identity) hilo = false;
    if (hilo && !ffn_can_hilo(dtype, k, d, d_ff)) return EC_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;

    float* S = S_out ? S_out : (float*)at(ws, L.st);  // [n, e]: the same size as the S^T region
    float* G = G_out ? G_out : (float*)at(ws, L.g);
    int32_t* I = I_out ? I_out : (int32_t*)at(ws, L.i);
    void* Xin = Xin_out ? Xin_out : at(ws, L.xin);

    const CombineIndex ix = combine_index_at(ws, L, e);
    int rc = launch_gate(X, Wg, S, nullptr, n, d, e, dtype, combine_zero_ptr(ix), combine_zero_words(ix, n, e), st);
    if (rc != EC_OK) return rc;
    rc = launch_token_choice(S, n, e, m, k, G, I, load_out, (int32_t*)at(ws, L.choice),
                             ix.use_slots ? ix.slot_cnt : nullptr, ix.slots, ix.slot_cap,
                             ix.use_slots ? nullptr : ix.bitmap, st);
    if (rc != EC_OK) return rc;
    const bool fused_gather = !identity && Xin_out == nullptr && ffn_can_gather(dtype, n, k, d, d_ff);
    if (!fused_gather) {
        rc = launch_dispatch(X, I, Xin, n, d, e, k, dtype, st);
        if (rc != EC_OK) return rc;
    }
    if (identity) return launch_combine(Xin, G, I, Xout, n, d, e, k, dtype, ix, st);
    return experts_then_combine(fused_gather ? nullptr : Xin, X, I, G, W1, W2, Xout, Xe_out, A_out, H_out, n, d, e, k,
                                d_ff, act, dtype, hilo, ws, L, ix, st);
}

size_t ec_moe_capped_workspace_bytes(int64_t n, int64_t e) {
    if (n <= 0 || e <= 0 || e > EC_MOE_MAX_EXPERTS || n >= (int64_t)1 << 31) return 0;
    return capped_ws_bytes(n, e);
}

static bool capped_args_ok(double b, double lambda, int64_t iters) {
    return std::isfinite(b) && b > 0.0 && std::isfinite(lambda) && lambda > 0.0 && iters >= 0 && iters <= 100000;
}

int ec_moe_capped_assignment(const float* St, int64_t n, int64_t e, int64_t k, double b, double lambda,
                             int64_t iters, float* A, void* ws, size_t ws_bytes, void* stream) {
    if (!St || !A || !sizes_ok(n, 1, e, k) || !capped_args_ok(b, lambda, iters) || !all_aligned(St, A))
        return EC_ERR_INVALID_ARG;
    if (!ws_ok(ws, ws_bytes, capped_ws_bytes(n, e))) return EC_ERR_WORKSPACE;
    return launch_capped_assignment(St, n, e, k, b, lambda, iters, A, ws, (hipStream_t)stream);
}

int ec_moe_forward_capped(const void* X, const void* Wg, const void* W1, const void* W2, double c, double b,
                          double lambda, int64_t iters, void* Xout, float* S_out, float* G_out, int32_t* I_out,
                          float* A_out, void* Xe_out, int64_t n, int64_t d, int64_t e, int64_t d_ff, int act,
                          int dtype, void* ws, size_t ws_bytes, void* stream) {
    int64_t k = 0;
    if (ec_moe_capacity(n, e, c, &k) != EC_OK || !capped_args_ok(b, lambda, iters)) return EC_ERR_INVALID_ARG;
    const bool identity = (W1 == nullptr && W2 == nullptr);
    if (!X || !Wg || !Xout || !sizes_ok(n, d, e, k) || !dtype_ok(dtype) || !act_ok(act) || !width_ok(d, dtype) ||
        !all_aligned(X, Wg, W1, W2, Xout, S_out, G_out, I_out, A_out, Xe_out))
        return EC_ERR_INVALID_ARG;
    if (identity) {
        if (act != EC_ACT_IDENTITY) return EC_ERR_INVALID_ARG;
        d_ff = 0;
    } else {
        if (!W1 || !W2 || d_ff <= 0 || d_ff >= (int64_t)1 << 31 || !width_ok(d_ff, dtype))
            return EC_ERR_INVALID_ARG;
    }
    const WsLayout L = ws_layout(n, d, e, k, d_ff, dtype, 0);
    // after the layer's own regions: the solver's state, then A when the caller does not want it
    const size_t a_bytes = align_up((size_t)e * n * 4, 256);
    if (!ws_ok(ws, ws_bytes, L.total + capped_ws_bytes(n, e) + a_bytes)) return EC_ERR_WORKSPACE;
    bool hilo = false;
    dtype = storage_dtype(dtype, &hilo);
    if (identity) hilo = false;
    if (hilo && !ffn_can_hilo(dtype, k, d, d_ff)) return EC_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;

    float* St = (float*)at(ws, L.st);
    float* G = G_out ? G_out : (float*)at(ws, L.g);
    int32_t* I = I_out ? I_out : (int32_t*)at(ws, L.i);
    void* Xin = at(ws, L.xin);
    void* solver = at(ws, L.total);
    float* A = A_out ? A_out : (float*)at(ws, L.total + capped_ws_bytes(n, e));

    const CombineIndex ix = combine_index_at(ws, L, e);
    int rc = launch_gate(X, Wg, S_out, St, n, d, e, dtype, combine_zero_ptr(ix), combine_zero_words(ix, n, e), st);
    if (rc != EC_OK) return rc;
    rc = launch_capped_assignment(St, n, e, k, b, lambda, iters, A, solver, st);
    if (rc != EC_OK) return rc;
    // indices from TopK(A, k); the values it returns are entries of A and are replaced by the scores
    rc = launch_topk(A, n, e, k, G, I, ix.use_slots ? ix.slot_cnt : nullptr, ix.slots, ix.slot_cap,
                     ix.use_slots ? nullptr : ix.bitmap, st);
    if (rc != EC_OK) return rc;
    rc = launch_gather_scores(St, I, G, n, e, k, st);
    if (rc != EC_OK) return rc;
    const bool fused_gather = !identity && ffn_can_gather(dtype, n, k, d, d_ff);
    if (!fused_gather) {
        rc = launch_dispatch(X, I, Xin, n, d, e, k, dtype, st);
        if (rc != EC_OK) return rc;
    }
    if (identity) return launch_combine(Xin, G, I, Xout, n, d, e, k, dtype, ix, st);
    return experts_then_combine(fused_gather ? nullptr : Xin, X, I, G, W1, W2, Xout, Xe_out, nullptr, nullptr, n, d, e, k,
                                d_ff, act, dtype, hilo, ws, L, ix, st);
}

int ec_moe_backward(const void* dY, const void* X, const void* Wg, const void* W1, const void* W2, const float* S,
                    const float* G, const int32_t* I, const void* Xin, const void* A, const void* H,
                    const void* Xe, void* dX, float* dWg, float* dW1, float* dW2, int64_t n, int64_t d, int64_t e,
                    int64_t k, int64_t d_ff, int act, int dtype, void* ws, size_t ws_bytes, void* stream) {
    if (!dY || !X || !Wg || !W1 || !W2 || !S || !G || !I || !Xin || !A || !H || !Xe || !dX || !dWg || !dW1 ||
        !dW2 || !sizes_ok(n, d, e, k) || d_ff <= 0 || d_ff >= (int64_t)1 << 31 || !dtype_ok(dtype) ||
        !act_ok(act) || !width_ok(d, dtype) || !width_ok(d_ff, dtype) ||
        !all_aligned(dY, X, Wg, W1, W2, S, G, I, Xin, A, H, Xe, dX, dWg, dW1, dW2))
        return EC_ERR_INVALID_ARG;
    const WsLayout L = ws_layout(n, d, e, k, d_ff, dtype, 1);
    if (!ws_ok(ws, ws_bytes, L.total)) return EC_ERR_WORKSPACE;
    bool hilo = false;
    dtype = storage_dtype(dtype, &hilo);
    return launch_backward(dY, X, Wg, W1, W2, S, G, I, Xin, A, H, Xe, dX, dWg, dW1, dW2, n, d, e, k, d_ff, act,
                           dtype, ws, L, (hipStream_t)stream, nullptr, hilo);
}

int ec_moe_backward_timed(const void* dY, const void* X, const void* Wg, const void* W1, const void* W2, const float* S,
                          const float* G, const int32_t* I, const void* Xin, const void* A, const void* H,
                          const void* Xe, void* dX, float* dWg, float* dW1, float* dW2, int64_t n, int64_t d, int64_t e,
                          int64_t k, int64_t d_ff, int act, int dtype, void* ws, size_t ws_bytes, void* stream,
                          float* stage_ms) {
    if (!stage_ms || !dY || !X || !Wg || !W1 || !W2 || !S || !G || !I || !Xin || !A || !H || !Xe || !dX || !dWg || !dW1 ||
        !dW2 || !sizes_ok(n, d, e, k) || d_ff <= 0 || d_ff >= (int64_t)1 << 31 || !dtype_ok(dtype) ||
        !act_ok(act) || !width_ok(d, dtype) || !width_ok(d_ff, dtype) ||
        !all_aligned(dY, X, Wg, W1, W2, S, G, I, Xin, A, H, Xe, dX, dWg, dW1, dW2))
        return EC_ERR_INVALID_ARG;
    const WsLayout L = ws_layout(n, d, e, k, d_ff, dtype, 1);
    if (!ws_ok(ws, ws_bytes, L.total)) return EC_ERR_WORKSPACE;
    bool hilo = false;
    dtype = storage_dtype(dtype, &hilo);
    hipEvent_t marks[BWD_STAGES + 1];
    int made = 0;
    hipError_t err = hipSuccess;
    for (; made <= BWD_STAGES && err == hipSuccess; ++made) err = hipEventCreate(&marks[made]);
    int rc = EC_OK;
    if (err != hipSuccess) {
        --made;  // the last create failed
        set_last_hip_error(err);
        rc = EC_ERR_HIP;
    } else {
        rc = launch_backward(dY, X, Wg, W1, W2, S, G, I, Xin, A, H, Xe, dX, dWg, dW1, dW2, n, d, e, k, d_ff, act, dtype,
                             ws, L, (hipStream_t)stream, marks, hilo);
        if (rc == EC_OK) {
            err = hipEventSynchronize(marks[BWD_STAGES]);
            for (int s = 0; s < BWD_STAGES && err == hipSuccess; ++s)
                err = hipEventElapsedTime(&stage_ms[s], marks[s], marks[s + 1]);
            if (err != hipSuccess) {
                set_last_hip_error(err);
                rc = EC_ERR_HIP;
            }
        } else {
            (void)hipStreamSynchronize((hipStream_t)stream);  // nothing may still refer to the events
        }
    }
    for (int s = 0; s < made; ++s) (void)hipEventDestroy(marks[s]);
    return rc;
}

const char* ec_moe_backward_stage_name(int stage) {
    static const char* const names[BWD_STAGES] = {"bwd_rows", "bwd_dW2", "bwd_dA", "bwd_dW1", "bwd_dX_in",
                                                  "bwd_index", "bwd_dZ", "bwd_gate_products", "bwd_scatter"};
    return stage >= 0 && stage < BWD_STAGES ? names[stage] : nullptr;
}

int ec_moe_last_hip_error(void) { return g_last_hip_error; }

const char* ec_moe_status_string(int status) {
    switch (status) {
        case EC_OK: return "EC_OK";
        case EC_ERR_INVALID_ARG: return "EC_ERR_INVALID_ARG";
        case EC_ERR_WORKSPACE: return "EC_ERR_WORKSPACE";
        case EC_ERR_HIP: return "EC_ERR_HIP";
        case EC_ERR_UNSUPPORTED: return "EC_ERR_UNSUPPORTED";
        default: return "EC_UNKNOWN_STATUS";
    }
}

const char* ec_moe_version(void) { return "0.2"; }

}  // extern "C"
