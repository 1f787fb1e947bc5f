// EVD / ZCA whitening matrix (Sec. 2, eqs. (vPhix_evd), (vT_EVD), (vg); Sec. 3.2, eqs. (hMs), (g_mod)) for gfx950.
//
// Phi_x is symmetric positive semi-definite, so a one-sided Jacobi iteration on its rows yields the decomposition:
// plane rotations J are applied to the rows of W (initially Phi_x) and of V (initially I) until the rows of W are
// mutually orthogonal; then W = Lambda V, the rows of V are the eigenvectors and lambda_k = w_k . v_k.
// A round of the round-robin schedule rotates M/2 disjoint row pairs, one workgroup per pair; rotations are
// independent inside a round.  All of it runs in float64 inside the workspace so that small eigenvalues, which
// carry the largest gains, keep their relative accuracy.  T = V^T diag(sqrt g) V and Q = V^T diag(g) V are then
// symmetric rank-M updates of row-scaled copies of V and reuse the float32 matrix-core covariance kernel.
#include "fw_internal.h"

namespace fw {
namespace {

struct EvdWs {
    size_t W, V, lam, gq, gh, cnt, X, dummy_s, cov, total;
};
inline size_t cov_ws_for(int M) {
    fw_conv_desc d = {M, M, 1, 1, 1, 1, 1, 0};
    return cov_workspace_bytes(M, &d, FW_F32, FW_LAYOUT_ROWS);
}
inline EvdWs evd_layout(int M) {
    EvdWs L;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes, 256); return at; };
    L.W = take((size_t)M * M * sizeof(double));
    L.V = take((size_t)M * M * sizeof(double));
    L.lam = take((size_t)M * sizeof(double));
    L.gq = take((size_t)M * sizeof(double));
    L.gh = take((size_t)M * sizeof(double));
    L.cnt = take(256);
    L.X = take((size_t)M * M * sizeof(float));
    L.dummy_s = take((size_t)M * sizeof(float));
    L.cov = take(cov_ws_for(M));
    L.total = o;
    return L;
}

__global__ __launch_bounds__(256) void evd_init_kernel(const float* __restrict__ Phi, int M, double* __restrict__ W, double* __restrict__ V) {
    const size_t n = (size_t)M * M;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256) {
        const int i = (int)(e / M), j = (int)(e - (size_t)i * M);
        // symmetric part, so that a slightly asymmetric input still has a well-defined decomposition
        W[e] = 0.5 * ((double)Phi[e] + (double)Phi[(size_t)j * M + i]);
        V[e] = i == j ? 1.0 : 0.0;
    }
}

__device__ __forceinline__ double block_sum256(double v, double* red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// One round of the round-robin ordering over n (even) players; pair k of round r.
__device__ __forceinline__ void rr_pair(int n, int r, int k, int* a, int* b) {
    const int m = n - 1;
    if (k == 0) { *a = m; *b = r; }
    else { *a = (r + k) % m; *b = (r - k + m) % m; }
}

__global__ __launch_bounds__(256) void jacobi_round_kernel(double* __restrict__ W, double* __restrict__ V, int M, int n_even, int round,
                                                           double tol, int* __restrict__ counter) {
    __shared__ double red[4];
    int a, b;
    rr_pair(n_even, round, blockIdx.x, &a, &b);
    const int p = min(a, b), q = max(a, b);
    if (q >= M) return;  // pair with the padding player
    double* wp = W + (size_t)p * M;
    double* wq = W + (size_t)q * M;
    double al = 0.0, be = 0.0, ga = 0.0;
    for (int j = threadIdx.x; j < M; j += 256) {
        const double x = wp[j], y = wq[j];
        al += x * x; be += y * y; ga += x * y;
    }
    al = block_sum256(al, red);
    be = block_sum256(be, red);
    ga = block_sum256(ga, red);
    if (!(fabs(ga) > tol * sqrt(al * be)) || ga == 0.0) return;
    const double zeta = (be - al) / (2.0 * ga);
    const double tt = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
    const double c = 1.0 / sqrt(1.0 + tt * tt), s = c * tt;
    double* vp = V + (size_t)p * M;
    double* vq = V + (size_t)q * M;
    for (int j = threadIdx.x; j < M; j += 256) {
        const double x = wp[j], y = wq[j];
        wp[j] = c * x - s * y;
        wq[j] = s * x + c * y;
        const double e = vp[j], f = vq[j];
        vp[j] = c * e - s * f;
        vq[j] = s * e + c * f;
    }
    if (threadIdx.x == 0) atomicAdd(counter, 1);
}

__global__ void zero_int_kernel(int* p) { *p = 0; }

// lambda_k = w_k . v_k (signed), one wavefront per row
__global__ __launch_bounds__(256) void eig_kernel(const double* __restrict__ W, const double* __restrict__ V, int M, double* __restrict__ lam) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= M) return;
    double acc = 0.0;
    for (int j = lane; j < M; j += 64) acc += W[(size_t)r * M + j] * V[(size_t)r * M + j];
    acc = wave_sum(acc);
    if (lane == 0) lam[r] = acc;
}

// Sorted eigenvalues (decreasing) and per-row gain roots.  One workgroup.
//  mode 0: g = 1/max(lambda, eps)                                          eq. (vg)
//  mode 1: g = min(1/(M lb), g_max) for sorted position < round(Ms_hat), 1 otherwise, lb = lambda/sum(lambda),
//          Ms_hat = exp(-sum lb log lb)  (exponential of the spectral entropy; reading of eq. (hMs))   eq. (g_mod)
__global__ __launch_bounds__(1024) void gains_kernel(const double* __restrict__ lam, int M, float eps, float g_max, int mode,
                                                     float* __restrict__ lam_sorted, double* __restrict__ gq, double* __restrict__ gh) {
    __shared__ double red[16];
    __shared__ double s_tot, s_ent;
    double tot = 0.0;
    for (int k = threadIdx.x; k < M; k += 1024) tot += fmax(lam[k], 0.0);
    tot = wave_sum(tot);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = tot;
    __syncthreads();
    if (threadIdx.x == 0) { double t = 0; for (int i = 0; i < 16; ++i) t += red[i]; s_tot = t; }
    __syncthreads();
    tot = s_tot;
    double ent = 0.0;
    for (int k = threadIdx.x; k < M; k += 1024) {
        const double lb = tot > 0.0 ? fmax(lam[k], 0.0) / tot : 0.0;
        if (lb > 0.0) ent -= lb * log(lb);
    }
    ent = wave_sum(ent);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ent;
    __syncthreads();
    if (threadIdx.x == 0) { double t = 0; for (int i = 0; i < 16; ++i) t += red[i]; s_ent = t; }
    __syncthreads();
    int rank_sig = M;
    if (mode == 1) {
        const double ms = tot > 0.0 ? exp(s_ent) : 1.0;
        double r = floor(ms + 0.5);
        if (r < 1.0) r = 1.0;
        if (r > (double)M) r = (double)M;
        rank_sig = (int)r;
    }
    for (int k = threadIdx.x; k < M; k += 1024) {
        const double lk = lam[k];
        int pos = 0;  // sorted position: number of eigenvalues ahead of this one
        for (int j = 0; j < M; ++j) {
            const double lj = lam[j];
            pos += (lj > lk || (lj == lk && j < k)) ? 1 : 0;
        }
        lam_sorted[pos] = (float)lk;
        double g;
        if (mode == 0) g = 1.0 / fmax(lk, (double)eps);
        else if (pos >= rank_sig) g = 1.0;
        else if (lk <= 0.0 || tot <= 0.0) g = (double)g_max;
        else g = fmin(tot / ((double)M * lk), (double)g_max);
        gh[k] = sqrt(g);
        gq[k] = sqrt(sqrt(g));
    }
}

// X[k][j] = scale[k] * V[k][j] as float32
__global__ __launch_bounds__(256) void scale_rows_kernel(const double* __restrict__ V, const double* __restrict__ scale, int M,
                                                         float* __restrict__ X) {
    const size_t n = (size_t)M * M;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256)
        X[e] = (float)(scale[e / M] * V[e]);
}

__global__ __launch_bounds__(256) void fill_kernel(float* __restrict__ p, size_t n, float v) {
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256) p[e] = v;
}

__global__ __launch_bounds__(256) void ema_kernel(float* __restrict__ Qs, const float* __restrict__ Q, size_t n, float beta) {
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256)
        Qs[e] = beta * Qs[e] + (1.f - beta) * Q[e];
}

inline int grid_for(size_t n) {
    size_t b = (n + 255) / 256;
    return (int)(b > 8192 ? 8192 : b);
}

}  // namespace

size_t evd_workspace_bytes(int M) { return evd_layout(M).total; }

fw_status whiten_evd(const float* Phi_x, int M, const fw_evd_params* p, float* T, float* Q, float* Qs, float* lambda, void* ws,
                     size_t ws_bytes, hipStream_t st) {
    const EvdWs L = evd_layout(M);
    if (ws_bytes < L.total) return FW_ERR_WORKSPACE;
    char* base = reinterpret_cast<char*>(ws);
    double* W = reinterpret_cast<double*>(base + L.W);
    double* V = reinterpret_cast<double*>(base + L.V);
    double* lam = reinterpret_cast<double*>(base + L.lam);
    double* gq = reinterpret_cast<double*>(base + L.gq);
    double* gh = reinterpret_cast<double*>(base + L.gh);
    int* cnt = reinterpret_cast<int*>(base + L.cnt);
    float* X = reinterpret_cast<float*>(base + L.X);
    float* dummy_s = reinterpret_cast<float*>(base + L.dummy_s);
    void* cov_ws = base + L.cov;
    const size_t cov_ws_bytes = cov_ws_for(M);
    const size_t n = (size_t)M * M;
    const double tol = p->tol > 0.f ? (double)p->tol : 1e-12;
    const int max_sweeps = p->max_sweeps > 0 ? p->max_sweeps : 30;

    hipLaunchKernelGGL(evd_init_kernel, dim3(grid_for(n)), dim3(256), 0, st, Phi_x, M, W, V);
    FW_LAUNCH_CHECK();
    const int n_even = (M + 1) & ~1;
    bool converged = M == 1;
    for (int sweep = 0; sweep < max_sweeps && !converged; ++sweep) {
        hipLaunchKernelGGL(zero_int_kernel, dim3(1), dim3(1), 0, st, cnt);
        for (int r = 0; r < n_even - 1; ++r)
            hipLaunchKernelGGL(jacobi_round_kernel, dim3(n_even / 2), dim3(256), 0, st, W, V, M, n_even, r, tol, cnt);
        FW_LAUNCH_CHECK();
        int rotations = -1;
        FW_HIP_TRY(hipMemcpyAsync(&rotations, cnt, sizeof(int), hipMemcpyDeviceToHost, st));
        FW_HIP_TRY(hipStreamSynchronize(st));
        converged = rotations == 0;
    }
    hipLaunchKernelGGL(eig_kernel, dim3((M + 3) / 4), dim3(256), 0, st, W, V, M, lam);
    hipLaunchKernelGGL(gains_kernel, dim3(1), dim3(1024), 0, st, lam, M, p->eps, p->g_max, p->gain_mode, lambda, gq, gh);
    FW_LAUNCH_CHECK();

    const fw_conv_desc d = {M, M, 1, 1, 1, 1, 1, 0};
    for (int which = 0; which < 2; ++which) {
        float* out = which == 0 ? T : Q;
        hipLaunchKernelGGL(scale_rows_kernel, dim3(grid_for(n)), dim3(256), 0, st, V, which == 0 ? gq : gh, M, X);
        hipLaunchKernelGGL(fill_kernel, dim3(grid_for(n)), dim3(256), 0, st, out, n, 0.f);
        hipLaunchKernelGGL(fill_kernel, dim3(grid_for(M)), dim3(256), 0, st, dummy_s, (size_t)M, 0.f);
        FW_LAUNCH_CHECK();
        fw_status rc = cov_accumulate(X, FW_F32, FW_LAYOUT_ROWS, &d, out, dummy_s, cov_ws, cov_ws_bytes, st);
        if (rc != FW_OK) return rc;
        rc = symmetrize_from_lower(out, M, st);
        if (rc != FW_OK) return rc;
    }
    if (Qs) {
        hipLaunchKernelGGL(ema_kernel, dim3(grid_for(n)), dim3(256), 0, st, Qs, Q, n, p->beta);
        FW_LAUNCH_CHECK();
    }
    return converged ? FW_OK : FW_ERR_NOT_CONVERGED;
}

}  // namespace fw
