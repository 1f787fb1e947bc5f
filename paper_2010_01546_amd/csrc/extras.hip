// Companions of the hot path: bias compensation when the tracked mean moves (Sec. 3.1, eq. (vtb_corr)) and the two
// monitoring figures of Sec. 6, whiteness rho (eq. (rho)) and normalised rank kappa (Sec. 3.2, eq. (hMs)).
#include "fw_internal.h"

namespace fw {
namespace {

// b[s] += scale * sum_{c,t} W[s][c][t] (mu_new[c] - mu_old[c]); one wavefront per output feature s, float64 sum.
// Sign: the layer output sum W~ (x - mu) + b must not change when mu moves, which needs the NEW mean minus the OLD one
// (the printed equation has them the other way round, against the relation it is derived from).
__global__ __launch_bounds__(256) void bias_compensate_kernel(float* __restrict__ b, const float* __restrict__ W, int S, int M, int taps,
                                                              const float* __restrict__ mu_old, const float* __restrict__ mu_new,
                                                              float scale) {
    const int lane = threadIdx.x & 63;
    const int s = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (s >= S) return;
    const size_t n = (size_t)M * taps;
    const float* w = W + (size_t)s * n;
    double acc = 0.0;
    for (size_t e = lane; e < n; e += 64) {
        const int c = (int)(e / taps);
        acc += (double)w[e] * ((double)mu_new[c] - (double)mu_old[c]);
    }
    acc = wave_sum(acc);
    if (lane == 0) b[s] = (float)((double)b[s] + (double)scale * acc);
}

__global__ __launch_bounds__(256) void diag_extract_kernel(const float* __restrict__ P, int M, float* __restrict__ d) {
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m < M) d[m] = P[(size_t)m * M + m];
}

// rowsum[r] = (1 / d[r]) sum_c P[r][c]^2 / d[c]; one wavefront per row, 16-byte loads when the rows allow them
__global__ __launch_bounds__(256) void whiteness_rows_kernel(const float* __restrict__ P, const float* __restrict__ d, int M,
                                                             double* __restrict__ rowsum) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= M) return;
    const float* row = P + (size_t)r * M;
    double acc = 0.0;
    if ((M & 3) == 0) {
        const float4* row4 = reinterpret_cast<const float4*>(row);
        const float4* d4 = reinterpret_cast<const float4*>(d);
        const int n4 = M >> 2;
        int c = lane;
        for (; c + 64 < n4; c += 128) {
            const float4 p0 = row4[c], p1 = row4[c + 64], q0 = d4[c], q1 = d4[c + 64];
            acc += (double)(p0.x * p0.x / q0.x + p0.y * p0.y / q0.y) + (double)(p0.z * p0.z / q0.z + p0.w * p0.w / q0.w);
            acc += (double)(p1.x * p1.x / q1.x + p1.y * p1.y / q1.y) + (double)(p1.z * p1.z / q1.z + p1.w * p1.w / q1.w);
        }
        for (; c < n4; c += 64) {
            const float4 p0 = row4[c], q0 = d4[c];
            acc += (double)(p0.x * p0.x / q0.x + p0.y * p0.y / q0.y) + (double)(p0.z * p0.z / q0.z + p0.w * p0.w / q0.w);
        }
    } else {
        for (int c = lane; c < M; c += 64) {
            const float p = row[c];
            acc += (double)(p * p / d[c]);
        }
    }
    acc = wave_sum(acc);
    if (lane == 0) rowsum[r] = acc / (double)d[r];
}

__device__ __forceinline__ double block_sum_1024(double v, double* red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += red[i];
    return t;
}

// out[0] = rho = M / sum of the row sums (when rowsum is given);
// out[1] = kappa = Ms_hat / M, out[2] = Ms_hat = exp(-sum lb log lb), lb = max(lambda, 0) / sum, 0 log 0 = 0 (when
// lambda is given; the exponential of the spectral entropy is the reading of eq. (hMs) that has the two stated extremes)
__global__ __launch_bounds__(1024) void diagnostics_final_kernel(const double* __restrict__ rowsum, const float* __restrict__ lambda,
                                                                 int M, float* __restrict__ out) {
    __shared__ double red[16];
    if (rowsum) {
        double v = 0.0;
        for (int k = threadIdx.x; k < M; k += 1024) v += rowsum[k];
        const double tot = block_sum_1024(v, red);
        if (threadIdx.x == 0) out[0] = (float)((double)M / tot);
    }
    if (lambda) {
        double v = 0.0;
        for (int k = threadIdx.x; k < M; k += 1024) v += fmax((double)lambda[k], 0.0);
        const double tot = block_sum_1024(v, red);
        double ent = 0.0;
        for (int k = threadIdx.x; k < M; k += 1024) {
            const double lb = tot > 0.0 ? fmax((double)lambda[k], 0.0) / tot : 0.0;
            if (lb > 0.0) ent -= lb * log(lb);
        }
        ent = block_sum_1024(ent, red);
        if (threadIdx.x == 0) {
            const double ms = tot > 0.0 ? exp(ent) : 1.0;
            out[1] = (float)(ms / (double)M);
            out[2] = (float)ms;
        }
    }
}

}  // namespace

fw_status bias_compensate(float* b, const float* W, int S, int M, int taps, const float* mu_old, const float* mu_new, float scale,
                          hipStream_t st) {
    hipLaunchKernelGGL(bias_compensate_kernel, dim3((S + 3) / 4), dim3(256), 0, st, b, W, S, M, taps, mu_old, mu_new, scale);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

size_t diagnostics_workspace_bytes(int M) { return align_up((size_t)M * sizeof(float), 256) + align_up((size_t)M * sizeof(double), 256); }

fw_status diagnostics(const float* Phi_y, const float* lambda, int M, float* out, void* ws, hipStream_t st) {
    double* rowsum = nullptr;
    if (Phi_y) {
        float* d = reinterpret_cast<float*>(ws);
        rowsum = reinterpret_cast<double*>(reinterpret_cast<char*>(ws) + align_up((size_t)M * sizeof(float), 256));
        hipLaunchKernelGGL(diag_extract_kernel, dim3((M + 255) / 256), dim3(256), 0, st, Phi_y, M, d);
        hipLaunchKernelGGL(whiteness_rows_kernel, dim3((M + 3) / 4), dim3(256), 0, st, Phi_y, d, M, rowsum);
        FW_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(diagnostics_final_kernel, dim3(1), dim3(1024), 0, st, rowsum, lambda, M, out);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
