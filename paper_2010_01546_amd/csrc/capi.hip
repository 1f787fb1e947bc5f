// C ABI of the feature-whitening library: argument validation, workspace carving, dispatch to the kernels.
#include "fw_internal.h"

using namespace fw;

namespace {

bool desc_ok(const fw_conv_desc* d, fw_layout lay) {
    if (!d) return false;
    if (d->B <= 0 || d->Cin <= 0 || d->H <= 0 || d->W <= 0 || d->kh <= 0 || d->kw <= 0 || d->stride <= 0 || d->pad < 0) return false;
    if (d->H + 2 * d->pad < d->kh || d->W + 2 * d->pad < d->kw) return false;
    if (d->pad > 0 && (d->pad >= d->kh || d->pad >= d->kw)) return false;  // a window lying wholly in the padding
    if (d->form < FW_COV_FORM_AUTO || d->form > FW_COV_FORM_SPLIT) return false;
    if (lay == FW_LAYOUT_ROWS && (d->H != 1 || d->W != 1 || d->kh != 1 || d->kw != 1 || d->stride != 1 || d->pad != 0)) return false;
    return true;
}

bool dtype_ok(fw_dtype dt) { return dt == FW_F32 || dt == FW_BF16; }
bool layout_ok(fw_layout l) { return l == FW_LAYOUT_ROWS || l == FW_LAYOUT_NCHW || l == FW_LAYOUT_NHWC || l == FW_LAYOUT_NHWC_KKC; }

// Q = T^T T built in the workspace: Q itself, a dummy vector of column sums, and the larger of the covariance kernel's
// scratch (float32 form) and the packed planes of T^T (split form, from FW_REFRESH_SPLIT_MIN_M features on)
bool q_build_split(int M) { return M >= FW_REFRESH_SPLIT_MIN_M; }
size_t grad_ws_bytes(int M) {
    fw_conv_desc d = {M, M, 1, 1, 1, 1, 1, 0, FW_COV_FORM_DIRECT};   // products in float32, never the split form
    const size_t cov = cov_workspace_bytes(M, &d, FW_F32, FW_LAYOUT_ROWS);
    const size_t packed = q_build_split(M) ? gemm_split_packed_bytes(M, M) : 0;
    return align_up((size_t)M * M * sizeof(float), 256) + align_up((size_t)M * sizeof(float), 256) + (cov > packed ? cov : packed);
}

// bfloat16 (or per-tap) gradients: a float32 copy of the gradient as [rows, M]
size_t grad_wide_bytes(long long rows, int M) { return align_up((size_t)rows * M * sizeof(float), 256); }

// float32 gradients of large layers: the product on the bfloat16 matrix cores with hi + lo split operands
// (gemm_split.hip) needs the packed planes of Q and of G and room for partial results
// measured break-even against the float32 strip kernel: the packing of Q costs M^2, the product gains with S M
bool grad_split_applies(int S, int M) {
    return M >= 1024 && S >= 128 && (long long)S * M >= (M >= 2048 ? FW_GRAD_SPLIT_MIN_SM_WIDE : FW_GRAD_SPLIT_MIN_SM);
}
size_t grad_split_bytes(int S, int M) {
    return grad_split_applies(S, M) ? gemm_split_packed_bytes(M, M) + gemm_split_packed_bytes(S, M) + gemm_split_partial_bytes(S, M, M) : 0;
}

// rows [n, M] float32 times Q on the bfloat16 matrix cores (split form), the runs of the contraction index added by the
// epilogue `e`; tail: grad_split_bytes(n, M) bytes
fw_status split_rows_apply(const float* rows, int n, int M, const float* Q, const GemmEpilogue& e, void* tail, hipStream_t st) {
    char* base = reinterpret_cast<char*>(tail);
    void* Qp = base;
    void* Gp = base + gemm_split_packed_bytes(M, M);
    float* sp = reinterpret_cast<float*>(base + gemm_split_packed_bytes(M, M) + gemm_split_packed_bytes(n, M));
    fw_status rc = gemm_split_pack(Q, M, M, Qp, st);              // Q is symmetric: its rows stand for its columns
    if (rc != FW_OK) return rc;
    rc = gemm_split_pack(rows, n, M, Gp, st);
    if (rc != FW_OK) return rc;
    int runs = 1;
    rc = gemm_split_run(Gp, Qp, n, M, M, 0, sp, st, sp, &runs);
    if (rc != FW_OK) return rc;
    return grad_epilogue_from_runs(sp, runs, e, n, M, st);
}

}  // namespace

extern "C" {

fw_status fw_cov_accumulate(const void* X, fw_dtype dt, fw_layout lay, const fw_conv_desc* d, float* A, float* s, void* ws,
                            size_t ws_bytes, void* stream) {
    if (!X || !A || !s || !d || !dtype_ok(dt) || !layout_ok(lay) || !desc_ok(d, lay)) return FW_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(A) || !aligned16(s) || (ws && !aligned16(ws))) return FW_ERR_ALIGNMENT;
    const size_t need = cov_workspace_bytes(0, d, dt, lay);
    if (need == 0) return FW_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < need) return FW_ERR_WORKSPACE;
    return cov_accumulate(X, dt, lay, d, A, s, ws, ws_bytes, reinterpret_cast<hipStream_t>(stream));
}

fw_status fw_cov_finalize(const float* A, const float* s, long long n, int M, float alpha, int first_block, float* mu, float* Phi_x,
                          float* phi_x, float* lambda_bar, void* stream) {
    if (!A || !s || !mu || !Phi_x || !phi_x || !lambda_bar || n <= 0 || M <= 0) return FW_ERR_INVALID_ARG;
    if (!first_block && !(alpha >= 0.f && alpha < 1.f)) return FW_ERR_INVALID_ARG;
    if (!aligned16(A) || !aligned16(s) || !aligned16(mu) || !aligned16(Phi_x) || !aligned16(phi_x)) return FW_ERR_ALIGNMENT;
    return cov_finalize(A, s, n, M, alpha, first_block ? 1 : 0, mu, Phi_x, phi_x, lambda_bar, reinterpret_cast<hipStream_t>(stream));
}

fw_status fw_grad_transform(const void* G, fw_dtype dt, int S, int M, const float* T, const float* Q, void* G_out, void* ws,
                            size_t ws_bytes, void* stream) {
    if (!G || !G_out || S <= 0 || M <= 0 || !dtype_ok(dt) || (!Q && !T) || G == G_out) return FW_ERR_INVALID_ARG;
    if (M > 16384) return FW_ERR_UNSUPPORTED;
    if (!aligned16(G) || !aligned16(G_out) || (Q && !aligned16(Q)) || (T && !aligned16(T)) || (ws && !aligned16(ws)))
        return FW_ERR_ALIGNMENT;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!Q) {
        if (!ws || ws_bytes < grad_ws_bytes(M)) return FW_ERR_WORKSPACE;
        char* base = reinterpret_cast<char*>(ws);
        float* Qb = reinterpret_cast<float*>(base);
        const size_t qbytes = align_up((size_t)M * M * sizeof(float), 256);
        float* sdummy = reinterpret_cast<float*>(base + qbytes);
        const size_t sbytes = align_up((size_t)M * sizeof(float), 256);
        fw_status rc;
        if (q_build_split(M)) {
            // Q = T^T T = (T^T)(T^T)^T on the bfloat16 matrix cores: the columns of T, packed as hi + lo planes, are both
            // operands; only the tiles that touch the lower triangle are multiplied (eq. (vQ))
            void* Tp = base + qbytes + sbytes;
            rc = gemm_split_pack_transposed(T, M, M, Tp, st);
            if (rc != FW_OK) return rc;
            rc = gemm_split_run(Tp, Tp, M, M, M, 1, Qb, st);
            if (rc != FW_OK) return rc;
        } else {
            const fw_conv_desc d = {M, M, 1, 1, 1, 1, 1, 0, FW_COV_FORM_DIRECT};   // products in float32, never the split form
            rc = fill_f32(Qb, (size_t)M * M, 0.f, st);
            if (rc != FW_OK) return rc;
            rc = fill_f32(sdummy, (size_t)M, 0.f, st);
            if (rc != FW_OK) return rc;
            // Q = T^T T: the rows of T are the "samples" of a symmetric rank-M update (eq. (vQ))
            rc = cov_accumulate(T, FW_F32, FW_LAYOUT_ROWS, &d, Qb, sdummy, base + qbytes + sbytes, ws_bytes - qbytes - sbytes, st);
            if (rc != FW_OK) return rc;
        }
        rc = symmetrize_from_lower(Qb, M, st);
        if (rc != FW_OK) return rc;
        Q = Qb;
    }
    // workspace beyond the Q build (and the widened gradient): partial strips, so that a product with few tiles can cut
    // its contraction index into runs over more workgroups
    const size_t fixed = grad_ws_bytes(M) + (dt == FW_BF16 ? grad_wide_bytes(S, M) : 0);
    float* part = (ws && ws_bytes >= fixed + grad_gemm_partial_bytes(S, M))
                      ? reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + fixed) : nullptr;
    if (dt == FW_BF16 && ws && ws_bytes >= grad_ws_bytes(M) + grad_wide_bytes(S, M)) {
        // widened to float32 in the workspace, multiplied in float32, rounded to bfloat16 as the results are stored
        float* G32 = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + grad_ws_bytes(M));
        const fw_status rc = grad_stage_rows(G, FW_BF16, S, M, 1, G32, st);
        if (rc != FW_OK) return rc;
        GemmEpilogue e = {};
        e.out = G_out; e.out_bf16 = 1; e.taps = 1;
        // a large product takes the split form from the widened copy, its runs summed and rounded by the epilogue pass
        if (grad_split_applies(S, M) && (M & 3) == 0 && ws_bytes >= fixed + grad_gemm_partial_bytes(S, M) + grad_split_bytes(S, M))
            return split_rows_apply(G32, S, M, Q, e, reinterpret_cast<char*>(ws) + fixed + grad_gemm_partial_bytes(S, M), st);
        return grad_gemm_f32(G32, S, M, Q, e, st, part);
    }
    if (dt == FW_F32 && grad_split_applies(S, M) && ws &&
        ws_bytes >= fixed + grad_gemm_partial_bytes(S, M) + grad_split_bytes(S, M)) {
        char* base = reinterpret_cast<char*>(ws) + fixed + grad_gemm_partial_bytes(S, M);
        void* Qp = base;
        void* Gp = base + gemm_split_packed_bytes(M, M);
        float* sp = reinterpret_cast<float*>(base + gemm_split_packed_bytes(M, M) + gemm_split_packed_bytes(S, M));
        fw_status rc = gemm_split_pack(Q, M, M, Qp, st);          // Q is symmetric: its rows stand for its columns
        if (rc != FW_OK) return rc;
        rc = gemm_split_pack(reinterpret_cast<const float*>(G), S, M, Gp, st);
        if (rc != FW_OK) return rc;
        return gemm_split_run(Gp, Qp, S, M, M, 0, reinterpret_cast<float*>(G_out), st, sp);
    }
    return grad_gemm(G, dt, S, M, Q, G_out, st, dt == FW_F32 ? part : nullptr);
}

fw_status fw_grad_transform_taps(const void* G, fw_dtype dt, int S, int M, int taps, const float* Q, void* G_out, void* ws,
                                 size_t ws_bytes, void* stream) {
    if (!G || !G_out || !Q || S <= 0 || M <= 0 || taps <= 0 || !dtype_ok(dt) || G == G_out) return FW_ERR_INVALID_ARG;
    if (M > 16384 || (long long)S * taps >= (1ll << 31) / 64) return FW_ERR_UNSUPPORTED;
    if (!aligned16(G) || !aligned16(G_out) || !aligned16(Q) || (ws && !aligned16(ws))) return FW_ERR_ALIGNMENT;
    if (!ws || ws_bytes < grad_wide_bytes((long long)S * taps, M)) return FW_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    float* rows = reinterpret_cast<float*>(ws);
    const fw_status rc = grad_stage_rows(G, dt, S, M, taps, rows, st);
    if (rc != FW_OK) return rc;
    GemmEpilogue e = {};
    e.out = G_out; e.out_bf16 = dt == FW_BF16 ? 1 : 0; e.taps = taps;
    const size_t wide = grad_wide_bytes((long long)S * taps, M);
    if (grad_split_applies(S * taps, M) && (M & 3) == 0 && ws_bytes >= wide + grad_split_bytes(S * taps, M))
        return split_rows_apply(rows, S * taps, M, Q, e, reinterpret_cast<char*>(ws) + wide, st);
    return grad_gemm_f32(rows, S * taps, M, Q, e, st);
}

fw_status fw_sgd_update(const void* G, fw_dtype dt, int S, int M, int taps, const float* Q, const fw_sgd_params* p, float* W, float* V,
                        void* ws, size_t ws_bytes, void* stream) {
    if (!G || !Q || !p || !W || S <= 0 || M <= 0 || taps <= 0 || !dtype_ok(dt) || G == (const void*)W || G == (const void*)V || W == V)
        return FW_ERR_INVALID_ARG;
    if (!(p->lr >= 0.f) || !(p->momentum >= 0.f && p->momentum < 1.f) || !(p->weight_decay >= 0.f)) return FW_ERR_INVALID_ARG;
    if (p->momentum > 0.f && !V) return FW_ERR_INVALID_ARG;
    if (M > 16384 || (long long)S * taps >= (1ll << 31) / 64) return FW_ERR_UNSUPPORTED;
    if (!aligned16(G) || !aligned16(Q) || !aligned16(W) || (V && !aligned16(V)) || (ws && !aligned16(ws))) return FW_ERR_ALIGNMENT;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const float* rows = reinterpret_cast<const float*>(G);
    if (dt == FW_BF16 || taps > 1) {
        if (!ws || ws_bytes < grad_wide_bytes((long long)S * taps, M)) return FW_ERR_WORKSPACE;
        const fw_status rc = grad_stage_rows(G, dt, S, M, taps, reinterpret_cast<float*>(ws), st);
        if (rc != FW_OK) return rc;
        rows = reinterpret_cast<const float*>(ws);
    }
    GemmEpilogue e = {};
    e.taps = taps; e.W = W; e.V = p->momentum > 0.f ? V : nullptr;
    e.lr = p->lr; e.momentum = p->momentum; e.wd = p->weight_decay;
    const size_t wide = grad_wide_bytes((long long)S * taps, M);
    if (grad_split_applies(S * taps, M) && (M & 3) == 0 && ws && ws_bytes >= wide + grad_split_bytes(S * taps, M))
        return split_rows_apply(rows, S * taps, M, Q, e, reinterpret_cast<char*>(ws) + wide, st);
    return grad_gemm_f32(rows, S * taps, M, Q, e, st);
}

fw_status fw_bias_compensate(float* b, const float* W, int S, int M, int taps, const float* mu_old, const float* mu_new, float scale,
                             void* stream) {
    if (!b || !W || !mu_old || !mu_new || S <= 0 || M <= 0 || taps <= 0) return FW_ERR_INVALID_ARG;
    return bias_compensate(b, W, S, M, taps, mu_old, mu_new, scale, reinterpret_cast<hipStream_t>(stream));
}

fw_status fw_diagnostics(const float* Phi_y, const float* lambda, int M, float* out, void* ws, size_t ws_bytes, void* stream) {
    if ((!Phi_y && !lambda) || !out || M <= 0) return FW_ERR_INVALID_ARG;
    if (M > 16384) return FW_ERR_UNSUPPORTED;
    if ((Phi_y && !aligned16(Phi_y)) || (ws && !aligned16(ws))) return FW_ERR_ALIGNMENT;
    if (Phi_y && (!ws || ws_bytes < diagnostics_workspace_bytes(M))) return FW_ERR_WORKSPACE;
    return diagnostics(Phi_y, lambda, M, out, ws, reinterpret_cast<hipStream_t>(stream));
}

fw_status fw_cond_probe(const float* Phi_y, int M, const float* b0, int k, float* out, void* ws, size_t ws_bytes, void* stream) {
    if (!Phi_y || !out || M <= 0 || k < 1 || k > FW_COND_PROBE_MAX_K) return FW_ERR_INVALID_ARG;
    if (M > 16384) return FW_ERR_UNSUPPORTED;
    if (!aligned16(Phi_y) || (ws && !aligned16(ws))) return FW_ERR_ALIGNMENT;
    if (!ws || ws_bytes < cond_probe_workspace_bytes(M, k)) return FW_ERR_WORKSPACE;
    return cond_probe(Phi_y, M, b0, k, out, ws, reinterpret_cast<hipStream_t>(stream));
}

fw_status fw_mfma_rate_probe(int zero_operands, int iters, float* sink, double* flops_host, void* stream) {
    if (!sink || iters <= 0 || iters > (1 << 24)) return FW_ERR_INVALID_ARG;
    return mfma_rate_probe(zero_operands ? 1 : 0, iters, sink, flops_host, reinterpret_cast<hipStream_t>(stream));
}

fw_status fw_cond_state_init(const fw_cond_state* st, void* stream) {
    if (!st || st->M <= 0 || !st->Phi_x || !st->T || !st->Q || !st->Qs || !st->Phi_y || !st->xi2) return FW_ERR_INVALID_ARG;
    if (!aligned16(st->Phi_x) || !aligned16(st->T) || !aligned16(st->Q) || !aligned16(st->Qs) || !aligned16(st->Phi_y) ||
        !aligned16(st->xi2) || (st->Psi && !aligned16(st->Psi)))
        return FW_ERR_ALIGNMENT;
    return cond_state_init(st, reinterpret_cast<hipStream_t>(stream));
}

fw_status fw_cond_state_refresh(const fw_cond_state* st, void* ws, size_t ws_bytes, void* stream) {
    if (!st || st->M <= 0 || !st->Phi_x || !st->T || !st->Phi_y || !st->xi2) return FW_ERR_INVALID_ARG;
    if (st->M > 16384) return FW_ERR_UNSUPPORTED;
    if (!aligned16(st->Phi_x) || !aligned16(st->T) || !aligned16(st->Phi_y) || !aligned16(st->xi2) || (st->Psi && !aligned16(st->Psi)) ||
        (ws && !aligned16(ws)))
        return FW_ERR_ALIGNMENT;
    if (!st->Psi && (!ws || ws_bytes < align_up((size_t)st->M * st->M * sizeof(float), 256))) return FW_ERR_WORKSPACE;
    return cond_state_refresh(st, ws, ws_bytes, reinterpret_cast<hipStream_t>(stream));
}

// argument checks shared by the two forms of the recursive step (everything except the workspace)
static fw_status cond_step_check(const fw_cond_state* st, const fw_cond_params* p) {
    if (!st || !p || st->M <= 0 || !st->Phi_x || !st->lambda_bar || !st->T || !st->Q || !st->Qs || !st->Phi_y || !st->xi2)
        return FW_ERR_INVALID_ARG;
    if (!(p->gamma > 0.f && p->gamma <= 1.f) || !(p->delta > 0.f) || !(p->eps > 0.f) || !(p->beta >= 0.f && p->beta < 1.f) ||
        !(p->c_rel >= 0.f) || !(p->c_abs >= 0.f) || p->n_power_iters < 0 || p->n_power_iters > 1024)
        return FW_ERR_INVALID_ARG;
    if (p->gamma < 1.f && !st->Psi) return FW_ERR_INVALID_ARG;
    if (st->M > 16384) return FW_ERR_UNSUPPORTED;
    if (!aligned16(st->Phi_x) || !aligned16(st->T) || !aligned16(st->Q) || !aligned16(st->Qs) || !aligned16(st->Phi_y) ||
        !aligned16(st->xi2) || (st->Psi && !aligned16(st->Psi)))
        return FW_ERR_ALIGNMENT;
    return FW_OK;
}

fw_status fw_grad_plan_query(fw_dtype dt, int S, int M, size_t ws_bytes, fw_grad_plan* plan) {
    if (!plan || S <= 0 || M <= 0 || (dt != FW_F32 && dt != FW_BF16)) return FW_ERR_INVALID_ARG;
    if (M > 16384) return FW_ERR_UNSUPPORTED;
    const size_t fixed = grad_ws_bytes(M) + (dt == FW_BF16 ? grad_wide_bytes(S, M) : 0);
    plan->split = dt == FW_F32 && grad_split_applies(S, M) &&
                  ws_bytes >= fixed + grad_gemm_partial_bytes(S, M) + grad_split_bytes(S, M);
    plan->mfma_flops_issued = plan->split ? gemm_split_flops_issued(S, M, M, 0, true) : 2.0 * (double)S * M * M;
    return FW_OK;
}

fw_status fw_cond_refresh_plan_query(int M, size_t ws_bytes, fw_refresh_plan* plan) {
    if (!plan || M <= 0) return FW_ERR_INVALID_ARG;
    return cond_refresh_plan(M, ws_bytes, plan) ? FW_OK : FW_ERR_UNSUPPORTED;
}

fw_status fw_cond_reduce_step(const fw_cond_state* st, const fw_cond_params* p, fw_cond_info* info_dev, void* ws, size_t ws_bytes,
                              void* stream) {
    const fw_status rc = cond_step_check(st, p);
    if (rc != FW_OK) return rc;
    if (ws && !aligned16(ws)) return FW_ERR_ALIGNMENT;
    if (!ws || ws_bytes < cond_workspace_bytes(st->M)) return FW_ERR_WORKSPACE;
    return cond_reduce_step(st, p, info_dev, ws, reinterpret_cast<hipStream_t>(stream));
}

fw_status fw_cond_reduce_step_static(const fw_cond_state* st, const fw_cond_params* p, fw_cond_info* info_dev, void* stream) {
    fw_status rc = cond_step_check(st, p);
    if (rc != FW_OK) return rc;
    if (st->M > FW_COND_STATIC_MAX_M) return FW_ERR_UNSUPPORTED;
    void* ws = nullptr;
    size_t ws_bytes = 0;
    rc = cond_static_scratch(&ws, &ws_bytes);   // no allocation: the address of a static device array
    if (rc != FW_OK) return rc;
    if (cond_workspace_bytes(st->M) > ws_bytes) return FW_ERR_UNSUPPORTED;
    return cond_reduce_step(st, p, info_dev, ws, reinterpret_cast<hipStream_t>(stream));
}

fw_status fw_whiten_evd(const float* Phi_x, int M, const fw_evd_params* p, float* T, float* Q, float* Qs, float* lambda, void* ws,
                        size_t ws_bytes, void* stream) {
    if (!Phi_x || !p || !T || !Q || !lambda || M <= 0) return FW_ERR_INVALID_ARG;
    if (!(p->eps > 0.f) || (p->gain_mode != 0 && p->gain_mode != 1) || (p->gain_mode == 1 && !(p->g_max > 0.f)) ||
        (Qs && !(p->beta >= 0.f && p->beta < 1.f)))
        return FW_ERR_INVALID_ARG;
    if (M > 16384) return FW_ERR_UNSUPPORTED;
    if (!aligned16(Phi_x) || !aligned16(T) || !aligned16(Q) || !aligned16(lambda) || (Qs && !aligned16(Qs)) || (ws && !aligned16(ws)))
        return FW_ERR_ALIGNMENT;
    if (!ws || ws_bytes < evd_workspace_bytes(M)) return FW_ERR_WORKSPACE;
    return whiten_evd(Phi_x, M, p, T, Q, Qs, lambda, ws, ws_bytes, reinterpret_cast<hipStream_t>(stream));
}

fw_status fw_cov_plan_query(fw_dtype dt, fw_layout lay, const fw_conv_desc* d, fw_cov_plan* plan) {
    if (!plan || !d || !dtype_ok(dt) || !layout_ok(lay) || !desc_ok(d, lay)) return FW_ERR_INVALID_ARG;
    return cov_plan(d, dt, lay, plan) ? FW_OK : FW_ERR_UNSUPPORTED;
}

size_t fw_workspace_bytes(fw_op op, int M, int S, const fw_conv_desc* d, fw_dtype dt) {
    switch (op) {
        case FW_OP_COV_ACCUMULATE: {
            if (!d || !dtype_ok(dt)) return 0;
            // the call has no layout argument: the largest need over the tensor layouts (rows split like a 1x1 tensor)
            const bool rows = d->H == 1 && d->W == 1 && d->kh == 1 && d->kw == 1;
            if (!desc_ok(d, rows ? FW_LAYOUT_ROWS : FW_LAYOUT_NHWC)) return 0;
            size_t need = cov_workspace_bytes(M, d, dt, FW_LAYOUT_NHWC);
            const size_t n1 = cov_workspace_bytes(M, d, dt, FW_LAYOUT_NCHW), n2 = cov_workspace_bytes(M, d, dt, FW_LAYOUT_NHWC_KKC);
            if (n1 > need) need = n1;
            if (n2 > need) need = n2;
            return need;
        }
        case FW_OP_GRAD_TRANSFORM:
            if (M <= 0 || M > 16384) return 0;
            return grad_ws_bytes(M) + ((dt == FW_BF16 && S > 0) ? grad_wide_bytes(S, M) : 0) + (S > 0 ? grad_gemm_partial_bytes(S, M) : 0) +
                   (S > 0 ? grad_split_bytes(S, M) : 0);
        case FW_OP_COND_REDUCE_STEP: return M > 0 && M <= 16384 ? cond_workspace_bytes(M) : 0;
        case FW_OP_WHITEN_EVD: return M > 0 && M <= 16384 ? evd_workspace_bytes(M) : 0;
        case FW_OP_COND_STATE_REFRESH: return M > 0 && M <= 16384 ? cond_refresh_workspace_bytes(M) : 0;
        case FW_OP_GRAD_TRANSFORM_TAPS:
        case FW_OP_SGD_UPDATE: return (M > 0 && M <= 16384 && S > 0) ? grad_wide_bytes(S, M) + grad_split_bytes(S, M) : 0;
        case FW_OP_DIAGNOSTICS: return M > 0 && M <= 16384 ? diagnostics_workspace_bytes(M) : 0;
        case FW_OP_COND_PROBE: return M > 0 && M <= 16384 ? cond_probe_workspace_bytes(M, S > 0 ? S : FW_COND_PROBE_MAX_K) : 0;
    }
    return 0;
}

const char* fw_status_string(fw_status st) {
    switch (st) {
        case FW_OK: return "ok";
        case FW_ERR_INVALID_ARG: return "invalid argument";
        case FW_ERR_UNSUPPORTED: return "unsupported size or mode";
        case FW_ERR_ALIGNMENT: return "device pointer not 16-byte aligned";
        case FW_ERR_WORKSPACE: return "workspace missing or too small";
        case FW_ERR_HIP: return "HIP runtime error";
        case FW_ERR_NOT_CONVERGED: return "eigen-decomposition did not converge";
    }
    return "unknown status";
}

int fw_version(void) { return 103; }

}  // extern "C"
