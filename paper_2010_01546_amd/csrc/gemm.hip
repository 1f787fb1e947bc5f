// Gradient transformation G_out = G Q (Sec. 3.1, eqs. (mod_weight_grad), (vQ)) on the gfx950 matrix cores.
//
// A workgroup of four wavefronts owns a 64 x 128 tile of G_out; each wavefront a 32 x 64 part of it (two MFMA
// 32x32 tiles).  The contraction index runs over the M features in chunks staged through LDS.
//   float32: v_mfma_f32_32x32x2_f32, G panel [row][k], Q panel [k][col].
//   bfloat16: v_mfma_f32_32x32x16_bf16, both panels K-major; Q is symmetric, so the K-major panel of Q is read
//   along its rows (contiguous) and rounded to bfloat16 while it is staged.
#include "fw_internal.h"

namespace fw {
namespace {

constexpr int TM = 64;    // rows of G per workgroup
constexpr int TN = 128;   // columns per workgroup
constexpr int KC32 = 16;  // contraction chunk, float32
constexpr int KC16 = 32;  // contraction chunk, bfloat16
constexpr int ROWB = KC16 * 2 + 16;  // bytes of one K-major bf16 LDS row

__global__ __launch_bounds__(256) void grad_gemm_f32_kernel(const float* __restrict__ G, const float* __restrict__ Q,
                                                            float* __restrict__ Out, int S, int M) {
    __shared__ float Gt[TM][KC32 + 1];
    __shared__ float Qt[KC32][TN];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int row0 = blockIdx.y * TM, col0 = blockIdx.x * TN;
    const int wr = wave & 1, wc = wave >> 1;
    floatx16 acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    for (int k0 = 0; k0 < M; k0 += KC32) {
        {   // G panel: 64 rows x 16 k
            const int k = tid & 15;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = (tid >> 4) + 16 * j;
                float v = 0.f;
                if (row0 + r < S && k0 + k < M) v = G[(size_t)(row0 + r) * M + k0 + k];
                Gt[r][k] = v;
            }
        }
        {   // Q panel: 16 k x 128 columns
            const int c = tid & 127;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int k = (tid >> 7) + 2 * j;
                float v = 0.f;
                if (k0 + k < M && col0 + c < M) v = Q[(size_t)(k0 + k) * M + col0 + c];
                Qt[k][c] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < KC32; kk += 2) {
            const float a = Gt[32 * wr + l32][kk + half];
            const float b0 = Qt[kk + half][64 * wc + l32];
            const float b1 = Qt[kk + half][64 * wc + 32 + l32];
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc[1], 0, 0, 0);
        }
        __syncthreads();
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int r = row0 + 32 * wr + 8 * (i >> 2) + 4 * half + (i & 3);
            const int c = col0 + 64 * wc + 32 * t + l32;
            if (r < S && c < M) Out[(size_t)r * M + c] = acc[t][i];
        }
}

// Small problems (too few 64x128 tiles to fill the chip): a workgroup owns a 32x32 tile of G_out and its four
// wavefronts split the contraction index four ways; operands come straight from global memory / L2 (G is small and
// Q rows are read coalesced), partial tiles are combined through LDS.  Latency-bound by design.
__global__ __launch_bounds__(256) void grad_gemm_f32_small_kernel(const float* __restrict__ G, const float* __restrict__ Q,
                                                                  float* __restrict__ Out, int S, int M) {
    __shared__ float red[3][32 * 32];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int row0 = blockIdx.y * 32, col0 = blockIdx.x * 32;
    int kq = ((M + 3) / 4 + 1) & ~1;             // even slice length per wavefront
    const int kb = wave * kq, ke = min(M, kb + kq);
    const int r = row0 + l32, c = col0 + l32;
    const bool r_ok = r < S, c_ok = c < M;
    const float* gp = G + (size_t)(r_ok ? r : 0) * M;
    const float* qp = Q + (c_ok ? c : 0);
    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    int k = kb;
    for (; k + 16 <= ke; k += 16) {
        float a[8], b[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int kk = k + 2 * j + half;
            a[j] = r_ok ? gp[kk] : 0.f;
            b[j] = c_ok ? qp[(size_t)kk * M] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b[j], acc, 0, 0, 0);
    }
    for (; k < ke; k += 2) {
        const int kk = k + half;
        const bool k_ok = kk < ke;
        const float a = (r_ok && k_ok) ? gp[kk] : 0.f;
        const float b = (c_ok && k_ok) ? qp[(size_t)kk * M] : 0.f;
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
    }
    if (wave > 0) {
#pragma unroll
        for (int i = 0; i < 16; ++i) red[wave - 1][(8 * (i >> 2) + 4 * half + (i & 3)) * 32 + l32] = acc[i];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int rr = 8 * (i >> 2) + 4 * half + (i & 3);
            const float v = acc[i] + red[0][rr * 32 + l32] + red[1][rr * 32 + l32] + red[2][rr * 32 + l32];
            if (row0 + rr < S && c_ok) Out[(size_t)(row0 + rr) * M + c] = v;
        }
    }
}

__global__ __launch_bounds__(256) void grad_gemm_bf16_kernel(const unsigned short* __restrict__ G, const float* __restrict__ Q,
                                                             unsigned short* __restrict__ Out, int S, int M) {
    __shared__ __attribute__((aligned(16))) unsigned char Gt[TM][ROWB];   // [row][k] bf16
    __shared__ __attribute__((aligned(16))) unsigned char Qt[TN][ROWB];   // [col][k] bf16
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int row0 = blockIdx.y * TM, col0 = blockIdx.x * TN;
    const int wr = wave & 1, wc = wave >> 1;
    floatx16 acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    for (int k0 = 0; k0 < M; k0 += KC16) {
        const int k = tid & 31;
#pragma unroll
        for (int j = 0; j < 8; ++j) {   // G panel: 64 rows x 32 k
            const int r = (tid >> 5) + 8 * j;
            unsigned short v = 0;
            if (row0 + r < S && k0 + k < M) v = G[(size_t)(row0 + r) * M + k0 + k];
            *reinterpret_cast<unsigned short*>(&Gt[r][2 * k]) = v;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {  // Q panel, read along row (col0 + c): Q[c][k] = Q[k][c]
            const int c = (tid >> 5) + 8 * j;
            float v = 0.f;
            if (col0 + c < M && k0 + k < M) v = Q[(size_t)(col0 + c) * M + k0 + k];
            *reinterpret_cast<unsigned short*>(&Qt[c][2 * k]) = f32_to_bf16_rne(v);
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < KC16; kk += 16) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Gt[32 * wr + l32][2 * (kk + 8 * half)]);
            const bf16x8 b0 = *reinterpret_cast<const bf16x8*>(&Qt[64 * wc + l32][2 * (kk + 8 * half)]);
            const bf16x8 b1 = *reinterpret_cast<const bf16x8*>(&Qt[64 * wc + 32 + l32][2 * (kk + 8 * half)]);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b0, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b1, acc[1], 0, 0, 0);
        }
        __syncthreads();
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int r = row0 + 32 * wr + 8 * (i >> 2) + 4 * half + (i & 3);
            const int c = col0 + 64 * wc + 32 * t + l32;
            if (r < S && c < M) Out[(size_t)r * M + c] = f32_to_bf16_rne(acc[t][i]);
        }
}

}  // namespace

fw_status grad_gemm(const void* G, fw_dtype dt, int S, int M, const float* Q, void* G_out, hipStream_t st) {
    const dim3 grid((M + TN - 1) / TN, (S + TM - 1) / TM);
    if (dt == FW_BF16)
        hipLaunchKernelGGL(grad_gemm_bf16_kernel, grid, dim3(256), 0, st, reinterpret_cast<const unsigned short*>(G), Q,
                           reinterpret_cast<unsigned short*>(G_out), S, M);
    else if ((long long)grid.x * grid.y < 200)
        hipLaunchKernelGGL(grad_gemm_f32_small_kernel, dim3((M + 31) / 32, (S + 31) / 32), dim3(256), 0, st,
                           reinterpret_cast<const float*>(G), Q, reinterpret_cast<float*>(G_out), S, M);
    else
        hipLaunchKernelGGL(grad_gemm_f32_kernel, grid, dim3(256), 0, st, reinterpret_cast<const float*>(G), Q,
                           reinterpret_cast<float*>(G_out), S, M);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
