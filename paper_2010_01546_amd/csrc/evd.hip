// EVD / ZCA whitening matrix (Sec. 2, eqs. (vPhix_evd), (vT_EVD), (vg); Sec. 3.2, eqs. (hMs), (g_mod)) for gfx950.
//
// Phi_x is symmetric positive semi-definite, so a one-sided Jacobi iteration on its rows yields the decomposition:
// orthogonal transformations are applied to the rows of W (initially Phi_x) and of V (initially I) until the rows of
// W are mutually orthogonal; then W = Lambda V, the rows of V are the eigenvectors and lambda_k = w_k . v_k.
// The iteration is blocked: rows are cut into blocks of 32, a round of the round-robin schedule takes disjoint pairs
// of blocks, and for every pair (64 rows) three kernels run: the 64x64 Gram matrix of the rows (partial sums over
// column slices), its diagonalisation by a cyclic two-sided Jacobi iteration in LDS, which yields the 64x64 rotation
// that makes the 64 rows orthogonal to each other, and the application of that rotation to the rows of W and V.
// A round therefore streams W and V once for 64 rows per pair instead of once per single row pair.  All of it runs
// in float64 inside the workspace so that small eigenvalues, which carry the largest gains, keep their relative
// accuracy.  T = V^T diag(sqrt g) V and Q = V^T diag(g) V are then symmetric rank-M updates of row-scaled copies of V:
// through the float32 matrix-core covariance kernel, or for many features as split products on the bfloat16 matrix
// cores (gemm_split.hip).
#include "fw_internal.h"

namespace fw {
namespace {

constexpr int JB = 32;        // rows per block
constexpr int JP = 2 * JB;    // rows per pair of blocks
constexpr int JSW = 512;      // columns per slice of the Gram kernel

struct EvdWs {
    size_t W, V, lam, gq, gh, cnt, X, dummy_s, cov, gpart, rot, flags, total;
    int nblk, nblk_even, npairs, nslices;
};
// T and Q from the scaled eigenvectors: from FW_REFRESH_SPLIT_MIN_M features on as split products on the bfloat16 matrix
// cores (the packed planes of X^T live where the covariance kernel's scratch would), below that through the float32
// covariance kernel
inline bool evd_products_split(int M) { return M >= FW_REFRESH_SPLIT_MIN_M; }
inline size_t cov_ws_for(int M) {
    if (evd_products_split(M)) return gemm_split_packed_bytes(M, M);
    fw_conv_desc d = {M, M, 1, 1, 1, 1, 1, 0, FW_COV_FORM_DIRECT};   // products in float32, never the split form
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
    L.nblk = (M + JB - 1) / JB;
    L.nblk_even = (L.nblk + 1) & ~1;
    L.npairs = L.nblk_even / 2;
    L.nslices = (M + JSW - 1) / JSW;
    L.gpart = take((size_t)L.npairs * L.nslices * JP * JP * sizeof(double));
    L.rot = take((size_t)L.npairs * JP * JP * sizeof(double));
    L.flags = take((size_t)L.npairs * sizeof(int));
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

// One round of the round-robin ordering over n (even) players; pair k of round r.
__device__ __forceinline__ void rr_pair(int n, int r, int k, int* a, int* b) {
    const int m = n - 1;
    if (k == 0) { *a = m; *b = r; }
    else { *a = (r + k) % m; *b = (r - k + m) % m; }
}

// global row of member k (0..63) of the block pair (p, q); -1 if it does not exist
__device__ __forceinline__ int pair_row(int p, int q, int nblk, int M, int k) {
    const int blk = k < JB ? p : q;
    const int r = blk * JB + (k & (JB - 1));
    return (blk < nblk && r < M) ? r : -1;
}

typedef double doublex4 __attribute__((ext_vector_type(4)));

// Partial Gram matrices: Gpart[pair][slice] = R_slice R_slice^T for the 64 rows R of the pair restricted to a slice of
// JSW columns, on v_mfma_f64_16x16x4_f64 (operand lane l: row l % 16, contraction entry l / 16; result register v of
// lane l: row 4 v + l / 16, column l % 16).  Chunks of 32 columns are staged in LDS; the four wavefronts take
// different 4-column steps of a chunk and each of them updates the ten 16x16 tiles of the lower triangle, both
// operands of a tile being fragments of the same staged rows; the four partial results are summed through LDS in
// wavefront order.
__global__ __launch_bounds__(256) void gram_kernel(const double* __restrict__ W, int M, int nblk, int nblk_even, int round, int nslices,
                                                   double* __restrict__ Gpart) {
    __shared__ double Xs[JP][33];
    __shared__ double red[40][64];
    int a, b;
    rr_pair(nblk_even, round, blockIdx.y, &a, &b);
    const int p = min(a, b), q = max(a, b);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane & 15, lq = lane >> 4;
    doublex4 acc[10];
#pragma unroll
    for (int t = 0; t < 10; ++t) acc[t] = doublex4{0.0, 0.0, 0.0, 0.0};
    const int c_begin = blockIdx.x * JSW, c_end = min(M, c_begin + JSW);
    // this thread's eight entries of a chunk: row (tid + 256 m) / 32, column (tid + 256 m) % 32; fetched one chunk ahead
    int grow[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) grow[m] = pair_row(p, q, nblk, M, (threadIdx.x + 256 * m) >> 5);
    const int cc = threadIdx.x & 31;
    double nxt[8];
    auto fetch = [&](int c0) {
#pragma unroll
        for (int m = 0; m < 8; ++m) nxt[m] = (grow[m] >= 0 && c0 + cc < c_end) ? W[(size_t)grow[m] * M + c0 + cc] : 0.0;
    };
    fetch(c_begin);
    for (int c0 = c_begin; c0 < c_end; c0 += 32) {
#pragma unroll
        for (int m = 0; m < 8; ++m) Xs[(threadIdx.x + 256 * m) >> 5][cc] = nxt[m];
        __syncthreads();
        if (c0 + 32 < c_end) fetch(c0 + 32);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int ks = wave + 4 * h;
            double f[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) f[t] = Xs[16 * t + lr][4 * ks + lq];
            int n = 0;
#pragma unroll
            for (int ta = 0; ta < 4; ++ta)
#pragma unroll
                for (int tb = 0; tb <= ta; ++tb, ++n) acc[n] = __builtin_amdgcn_mfma_f64_16x16x4f64(f[ta], f[tb], acc[n], 0, 0, 0);
        }
        __syncthreads();
    }
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int t = 0; t < 10; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    double* slot = &red[t * 4 + v][lane];
                    *slot = w == 0 ? acc[t][v] : *slot + acc[t][v];
                }
        }
        __syncthreads();
    }
    double* dst = Gpart + ((size_t)blockIdx.y * nslices + blockIdx.x) * (JP * JP);
    for (int e = threadIdx.x; e < 40 * 64; e += 256) {
        const int tv = e >> 6, l = e & 63;
        const int t = tv >> 2, v = tv & 3;
        int ta = 0, base = 0;
        while (base + ta + 1 <= t) { base += ta + 1; ++ta; }   // tile t = ta (ta + 1) / 2 + tb
        const int tb = t - base;
        const int i = 16 * ta + 4 * v + (l >> 4), j = 16 * tb + (l & 15);
        const double g = red[tv][l];
        dst[i * JP + j] = g;
        dst[j * JP + i] = g;
    }
}

// Diagonalisation of the 64x64 Gram matrix of a pair: cyclic Jacobi with 32 disjoint index pairs per step (32 threads
// per index pair: half a wavefront).  The accumulated rotation R (new rows = R old rows, R G R^T diagonal) goes to Rot[pair];
// flags[pair] = 1 if any rotation was applied, and the counter gets the number applied in the first inner sweep.
__global__ __launch_bounds__(1024) void pair_evd_kernel(const double* __restrict__ Gpart, int nslices, double tol, int inner_sweeps,
                                                       double* __restrict__ Rot,
                                                       int* __restrict__ flags, int* __restrict__ counter) {
    __shared__ double Gs[JP][JP + 1], Rs[JP][JP + 1];
    __shared__ int n_rot, n_first;
    const int tid = threadIdx.x;
    const int kk = tid >> 5, sub = tid & 31;
    for (int e = tid; e < JP * JP; e += 1024) {
        const double* src = Gpart + (size_t)blockIdx.x * nslices * (JP * JP) + e;
        double g = 0.0;
        for (int sl = 0; sl < nslices; ++sl) g += src[(size_t)sl * (JP * JP)];
        Gs[e >> 6][e & 63] = g;
        Rs[e >> 6][e & 63] = (e >> 6) == (e & 63) ? 1.0 : 0.0;
    }
    if (tid == 0) { n_rot = 0; n_first = 0; }
    __syncthreads();
    int total = 0;
    for (int sweep = 0; sweep < inner_sweeps; ++sweep) {
        for (int step = 0; step < JP - 1; ++step) {
            int i, j;
            rr_pair(JP, step, kk, &i, &j);
            if (i > j) { const int t = i; i = j; j = t; }
            // every thread of the index pair works out the rotation for itself: the 32 of them sit in one wavefront,
            // so all of them have read the three entries before any of them rewrites rows i and j
            const double al = Gs[i][i], be = Gs[j][j], ga = Gs[i][j];
            double c = 1.0, s = 0.0;
            if (fabs(ga) > tol * sqrt(fabs(al * be)) && ga != 0.0) {
                const double tau = be - al;
                const double tt = (tau >= 0.0 ? 2.0 : -2.0) * ga / (fabs(tau) + sqrt(tau * tau + 4.0 * ga * ga));
                c = rsqrt(1.0 + tt * tt);
                s = c * tt;
                if (sub == 0) atomicAdd(&n_rot, 1);
            }
            if (s != 0.0) {   // rows i, j of G and of R
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    const int col = sub + 32 * m;
                    const double x = Gs[i][col], y = Gs[j][col];
                    Gs[i][col] = c * x - s * y; Gs[j][col] = s * x + c * y;
                    const double e = Rs[i][col], f = Rs[j][col];
                    Rs[i][col] = c * e - s * f; Rs[j][col] = s * e + c * f;
                }
            }
            __syncthreads();
            if (s != 0.0) {   // columns i, j of G
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    const int row = sub + 32 * m;
                    const double x = Gs[row][i], y = Gs[row][j];
                    Gs[row][i] = c * x - s * y; Gs[row][j] = s * x + c * y;
                }
            }
            __syncthreads();
        }
        const int r = n_rot;      // every thread reads the same value: the last barrier of the step loop has passed
        __syncthreads();
        if (tid == 0) { if (sweep == 0) n_first = r; n_rot = 0; }
        __syncthreads();
        total += r;
        if (r == 0) break;
    }
    if (total > 0)
        for (int e = tid; e < JP * JP; e += 1024) Rot[(size_t)blockIdx.x * (JP * JP) + e] = Rs[e >> 6][e & 63];
    if (tid == 0) {
        flags[blockIdx.x] = total > 0 ? 1 : 0;
        if (n_first > 0) atomicAdd(counter, n_first);
    }
}

// rows of the pair <- R rows, for W (blockIdx.z = 0) and V (1), on v_mfma_f64_16x16x4_f64: a wavefront keeps all
// fragments of R in registers and takes groups of 16 columns; the 64 x 16 block of a group is read into registers
// before any of it is written back.
__global__ __launch_bounds__(256) void rotate_rows_kernel(double* __restrict__ W, double* __restrict__ V, int M, int nblk, int nblk_even,
                                                          int round, const double* __restrict__ Rot, const int* __restrict__ flags) {
    __shared__ double Rs[JP][JP + 1];
    if (flags[blockIdx.y] == 0) return;
    int a, b;
    rr_pair(nblk_even, round, blockIdx.y, &a, &b);
    const int p = min(a, b), q = max(a, b);
    for (int e = threadIdx.x; e < JP * JP; e += 256) Rs[e >> 6][e & 63] = Rot[(size_t)blockIdx.y * (JP * JP) + e];
    __syncthreads();
    double* Mat = blockIdx.z == 0 ? W : V;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane & 15, lq = lane >> 4;
    double ra[4][16];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) ra[t][ks] = Rs[16 * t + lr][4 * ks + lq];
    int rowk[16];   // global rows of this lane's contraction entries 4 ks + lq
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) rowk[ks] = pair_row(p, q, nblk, M, 4 * ks + lq);
    for (int gi = 0; gi < 8; ++gi) {
        const int col0 = blockIdx.x * 512 + (wave * 8 + gi) * 16;
        if (col0 >= M) break;
        const int col = col0 + lr;
        const bool cok = col < M;
        double xb[16];
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) xb[ks] = (rowk[ks] >= 0 && cok) ? Mat[(size_t)rowk[ks] * M + col] : 0.0;
        doublex4 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = doublex4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int ks = 0; ks < 16; ++ks)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(ra[t][ks], xb[ks], acc[t], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gr = pair_row(p, q, nblk, M, 16 * t + 4 * v + lq);
                if (gr >= 0 && cok) Mat[(size_t)gr * M + col] = acc[t][v];
            }
    }
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
    double* Gpart = reinterpret_cast<double*>(base + L.gpart);
    double* Rot = reinterpret_cast<double*>(base + L.rot);
    int* flags = reinterpret_cast<int*>(base + L.flags);
    const int ncolblk = (M + 511) / 512;
    const int inner = 1;   // inner sweeps per visit of a pair: one was the fastest overall (more inner sweeps, fewer outer ones)
    bool converged = false;
    for (int sweep = 0; sweep < max_sweeps && !converged; ++sweep) {
        hipLaunchKernelGGL(zero_int_kernel, dim3(1), dim3(1), 0, st, cnt);
        for (int r = 0; r < L.nblk_even - 1; ++r) {
            hipLaunchKernelGGL(gram_kernel, dim3(L.nslices, L.npairs), dim3(256), 0, st, W, M, L.nblk, L.nblk_even, r, L.nslices, Gpart);
            hipLaunchKernelGGL(pair_evd_kernel, dim3(L.npairs), dim3(1024), 0, st, Gpart, L.nslices, tol, inner, Rot, flags, cnt);
            hipLaunchKernelGGL(rotate_rows_kernel, dim3(ncolblk, L.npairs, 2), dim3(256), 0, st, W, V, M, L.nblk, L.nblk_even, r, Rot,
                               flags);
        }
        FW_LAUNCH_CHECK();
        int rotations = -1;
        FW_HIP_TRY(hipMemcpyAsync(&rotations, cnt, sizeof(int), hipMemcpyDeviceToHost, st));
        FW_HIP_TRY(hipStreamSynchronize(st));
        converged = rotations == 0;
    }
    hipLaunchKernelGGL(eig_kernel, dim3((M + 3) / 4), dim3(256), 0, st, W, V, M, lam);
    hipLaunchKernelGGL(gains_kernel, dim3(1), dim3(1024), 0, st, lam, M, p->eps, p->g_max, p->gain_mode, lambda, gq, gh);
    FW_LAUNCH_CHECK();

    const fw_conv_desc d = {M, M, 1, 1, 1, 1, 1, 0, FW_COV_FORM_DIRECT};   // products in float32, never the split form
    for (int which = 0; which < 2; ++which) {
        float* out = which == 0 ? T : Q;
        hipLaunchKernelGGL(scale_rows_kernel, dim3(grid_for(n)), dim3(256), 0, st, V, which == 0 ? gq : gh, M, X);
        FW_LAUNCH_CHECK();
        fw_status rc;
        if (evd_products_split(M)) {
            // X^T X = (X^T)(X^T)^T: the columns of X as hi + lo planes are both operands; lower triangle only
            rc = gemm_split_pack_transposed(X, M, M, cov_ws, st);
            if (rc != FW_OK) return rc;
            rc = gemm_split_run(cov_ws, cov_ws, M, M, M, 1, out, st);
            if (rc != FW_OK) return rc;
        } else {
            hipLaunchKernelGGL(fill_kernel, dim3(grid_for(n)), dim3(256), 0, st, out, n, 0.f);
            hipLaunchKernelGGL(fill_kernel, dim3(grid_for(M)), dim3(256), 0, st, dummy_s, (size_t)M, 0.f);
            FW_LAUNCH_CHECK();
            rc = cov_accumulate(X, FW_F32, FW_LAYOUT_ROWS, &d, out, dummy_s, cov_ws, cov_ws_bytes, st);
            if (rc != FW_OK) return rc;
        }
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
