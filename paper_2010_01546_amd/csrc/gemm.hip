// Gradient transformation G_out = G Q (Sec. 3.1, eqs. (mod_weight_grad), (vQ)) on the gfx950 matrix cores.
//
// A workgroup of four wavefronts owns a tile of G_out (64 x 64 in float32, 64 x 128 in bfloat16); the contraction
// index runs over the M features in chunks staged through LDS.
//   float32: v_mfma_f32_32x32x2_f32, G panel [row][k], Q panel [k][col].
//   bfloat16: v_mfma_f32_32x32x16_bf16, both panels K-major; Q is symmetric, so the K-major panel of Q is read
//   along its rows (contiguous) and rounded to bfloat16 while it is staged.
#include "fw_internal.h"

namespace fw {
namespace {

constexpr int TM = 64;    // rows of G per workgroup
constexpr int TN = 128;   // columns per workgroup
constexpr int KC16 = 32;  // contraction chunk, bfloat16
constexpr int ROWB = KC16 * 2 + 16;  // bytes of one K-major bf16 LDS row

// float32, large problems: 64x64 tile per workgroup, one 32x32 MFMA tile per wavefront.  Chunks of 32 contraction
// entries are fetched with 16-byte loads one chunk ahead of the MFMAs and double-buffered in LDS, both panels
// K-major ([k][row] for G, [k][col] for Q), so that a chunk costs one barrier.  Needs M % 4 == 0.
struct GemmSmem {
    float Gt[2][32][65];   // [buffer][k][row], row stride 65 words: the transposing stores spread over the banks
    alignas(16) float Qt[2][32][64];   // [buffer][k][col]
};

__global__ __launch_bounds__(256) void grad_gemm_f32_kernel(const float* __restrict__ G, const float* __restrict__ Q,
                                                            float* __restrict__ Out, int S, int M) {
    constexpr int KC = 32;
    __shared__ GemmSmem sm;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int row0 = blockIdx.y * 64, col0 = blockIdx.x * 64;
    const int wr = wave & 1, wc = wave >> 1;
    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;

    // staging roles: G panel 64 rows x 32 k = 512 float4 (row = e / 8, k quad = e % 8), Q panel 32 k x 64 cols = 512 float4
    float4 pg[2], pq[2];
    const int nchunks = (M + KC - 1) / KC;
    auto load_chunk = [&](int c) {
        const int k0 = c * KC;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int e = tid + 256 * j;
            const int gr = row0 + (e >> 3), gk = k0 + 4 * (e & 7);
            pg[j] = (gr < S && gk < M) ? *reinterpret_cast<const float4*>(G + (size_t)gr * M + gk) : make_float4(0.f, 0.f, 0.f, 0.f);
            const int qk = k0 + (e >> 4), qc = col0 + 4 * (e & 15);
            pq[j] = (qk < M && qc < M) ? *reinterpret_cast<const float4*>(Q + (size_t)qk * M + qc) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto store_chunk = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int e = tid + 256 * j;
            const int r = e >> 3, kq = 4 * (e & 7);
            sm.Gt[buf][kq + 0][r] = pg[j].x; sm.Gt[buf][kq + 1][r] = pg[j].y;
            sm.Gt[buf][kq + 2][r] = pg[j].z; sm.Gt[buf][kq + 3][r] = pg[j].w;
            *reinterpret_cast<float4*>(&sm.Qt[buf][e >> 4][4 * (e & 15)]) = pq[j];
        }
    };
    load_chunk(0);
    store_chunk(0);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        const bool more = c + 1 < nchunks;
        if (more) load_chunk(c + 1);
#pragma unroll
        for (int kk = 0; kk < KC; kk += 2) {
            const float a = sm.Gt[buf][kk + half][32 * wr + l32];
            const float b = sm.Qt[buf][kk + half][32 * wc + l32];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        if (more) store_chunk(buf ^ 1);
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int r = row0 + 32 * wr + 8 * (i >> 2) + 4 * half + (i & 3);
        const int c = col0 + 32 * wc + l32;
        if (r < S && c < M) Out[(size_t)r * M + c] = acc[i];
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
    else if ((long long)((M + 63) / 64) * ((S + 63) / 64) < 400 || (M & 3) != 0)
        hipLaunchKernelGGL(grad_gemm_f32_small_kernel, dim3((M + 31) / 32, (S + 31) / 32), dim3(256), 0, st,
                           reinterpret_cast<const float*>(G), Q, reinterpret_cast<float*>(G_out), S, M);
    else
        hipLaunchKernelGGL(grad_gemm_f32_kernel, dim3((M + 63) / 64, (S + 63) / 64), dim3(256), 0, st,
                           reinterpret_cast<const float*>(G), Q, reinterpret_cast<float*>(G_out), S, M);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
