// Internal declarations shared by the gfx950 kernels of the feature-whitening library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fw.h"

#define FW_HIP_TRY(expr)                            \
    do {                                            \
        hipError_t e__ = (expr);                    \
        if (e__ != hipSuccess) return FW_ERR_HIP;   \
    } while (0)

#define FW_LAUNCH_CHECK()                                        \
    do {                                                         \
        if (hipGetLastError() != hipSuccess) return FW_ERR_HIP;  \
    } while (0)

namespace fw {

constexpr int kWave = 64;

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short shortx8 __attribute__((ext_vector_type(8)));

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// bfloat16 bit pattern <-> float
__device__ __forceinline__ float bf16_to_f32(unsigned short h) { return __uint_as_float(((unsigned)h) << 16); }
__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

// 64-lane butterfly reductions.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ---- direct global-to-LDS loads with hand-counted completion
// s_waitcnt vmcnt(n), the other counters left alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
#define FW_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)
// s_waitcnt lgkmcnt(0): the LDS reads (and scalar loads) of this wavefront have returned
#define FW_WAIT_LGKM0() __builtin_amdgcn_s_waitcnt(0xC07F)
// keeps the compiler from moving memory accesses across this point (no instruction)
#define FW_COMPILER_FENCE() asm volatile("" ::: "memory")

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at lds_base + 16 l (lds_base is
// wavefront-uniform and travels in M0).  Written as assembly so that the compiler does not track it as a pending LDS
// store (it would then wait for ALL outstanding loads before every LDS read): completion is awaited by hand with
// FW_WAIT_VM, counting these loads in issue order, followed by a workgroup barrier.
// M0 is named as clobbered; the compiler warns that it does not save reserved registers around assembly, which is what
// is wanted here: it never keeps a value in M0 (it writes M0 itself right before each instruction of its own that
// reads it), so nothing is lost.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const void* src, void* lds_dst) {
    const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)lds_dst;
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(lds_addr) : "memory", "m0");
}
#pragma clang diagnostic pop

// ---- cov.hip
size_t cov_workspace_bytes(int M, const fw_conv_desc* d, fw_dtype dt, fw_layout lay);
fw_status cov_accumulate(const void* X, fw_dtype dt, fw_layout lay, const fw_conv_desc* d, float* A, float* s,
                         void* ws, size_t ws_bytes, hipStream_t st);
fw_status cov_finalize(const float* A, const float* s, long long n, int M, float alpha, int first_block, float* mu,
                       float* Phi_x, float* phi_x, float* lambda_bar, hipStream_t st);
fw_status symmetrize_from_lower(float* A, int M, hipStream_t st);
fw_status fill_f32(float* p, size_t n, float v, hipStream_t st);
bool cov_plan(const fw_conv_desc* d, fw_dtype dt, fw_layout lay, fw_cov_plan* plan);

// ---- shift correlations of stride-1 windows (cov_shift.hip, cov_bf16.hip)
// tap differences kept, in order: (0, 0..kw-1), then (dy, -(kw-1)..kw-1) for dy = 1..kh-1
__device__ __host__ inline void shift_diff_of(int di, int kw, int* dy, int* dx) {
    if (di < kw) { *dy = 0; *dx = di; return; }
    const int e = di - kw, w2 = 2 * kw - 1;
    *dy = 1 + e / w2;
    *dx = e % w2 - (kw - 1);
}
__device__ __host__ inline int shift_diff_index(int dy, int dx, int kw) { return dy == 0 ? dx : kw + (dy - 1) * (2 * kw - 1) + dx + kw - 1; }
// bands of one image axis: maximal runs of coordinates y that serve the same set of taps t (bit t of mask: the output
// coordinate y - t + pad lies in [0, Ho)); returns the number of bands, -1 if more than cap
struct ShiftBand { int begin, len, mask; };
inline int shift_bands(int H, int k, int pad, int Ho, ShiftBand* out, int cap) {
    auto mask_of = [&](int yy) {
        int m = 0;
        for (int t = 0; t < k; ++t) {
            const int p = yy - t + pad;
            if (p >= 0 && p <= Ho - 1) m |= 1 << t;
        }
        return m;
    };
    int n = 0, y = 0;
    while (y < H) {
        const int m = mask_of(y);
        int y1 = y;
        while (y1 + 1 < H && mask_of(y1 + 1) == m) ++y1;
        if (m) {
            if (n == cap) return -1;
            out[n].begin = y; out[n].len = y1 - y + 1; out[n].mask = m;
            ++n;
        }
        y = y1 + 1;
    }
    return n;
}

// ---- cov_shift.hip
bool cov_shift_applies(const fw_conv_desc* d, fw_layout lay);
size_t cov_shift_workspace_bytes(const fw_conv_desc* d, fw_layout lay);
fw_status cov_shift_accumulate(const float* X, fw_layout lay, const fw_conv_desc* d, float* A, float* s, void* ws, size_t ws_bytes,
                               hipStream_t st);

bool cov_shift_plan(const fw_conv_desc* d, fw_layout lay, fw_cov_plan* plan);

// ---- cov_skinny.hip
bool cov_skinny_applies(const fw_conv_desc* d, fw_layout lay);
size_t cov_skinny_workspace_bytes(const fw_conv_desc* d, fw_layout lay);
bool cov_skinny_plan(const fw_conv_desc* d, fw_layout lay, fw_cov_plan* plan);
fw_status cov_skinny_accumulate(const void* X, fw_dtype dt, fw_layout lay, const fw_conv_desc* d, float* A, float* s, void* ws,
                                size_t ws_bytes, hipStream_t st);

// ---- cov_bf16.hip
bool cov_bf16_plan(const fw_conv_desc* d, fw_layout lay, fw_cov_plan* plan);
size_t cov_bf16_workspace_bytes(const fw_conv_desc* d, fw_layout lay);
fw_status cov_bf16_accumulate(const void* X, fw_layout lay, const fw_conv_desc* d, float* A, float* s, void* ws,
                              size_t ws_bytes, hipStream_t st, bool split_f32 = false);

// ---- gemm.hip
// what the float32 product does with its result (see emit() in gemm.hip)
struct GemmEpilogue {
    void* out;        // transformed gradient, float32 or bfloat16 bits, or null
    int out_bf16;
    int taps;         // 1: [S, M]; > 1: the product ran on [S * taps, M] rows and results go to [S, M, taps]
    float* W;         // stored weights to update in place, or null
    float* V;         // momentum buffer, or null
    float lr, momentum, wd;
};
// `part`: optional scratch of grad_gemm_partial_bytes(S, M) bytes that lets the float32 product cut its contraction index
// into runs over more workgroups (few tiles otherwise leave compute units idle); null = never cut
size_t grad_gemm_partial_bytes(int S, int M);
fw_status grad_gemm(const void* G, fw_dtype dt, int S, int M, const float* Q, void* G_out, hipStream_t st, float* part = nullptr);
fw_status grad_gemm_f32(const float* G, int S, int M, const float* Q, const GemmEpilogue& e, hipStream_t st, float* part = nullptr);
fw_status grad_stage_rows(const void* G, fw_dtype dt, int S, int M, int taps, float* dst, hipStream_t st);
fw_status grad_epilogue_from_runs(const float* part, int nks, const GemmEpilogue& e, int S, int M, hipStream_t st);

// ---- gemm_split.hip: C = A B^T in float32-grade accuracy on the bfloat16 matrix cores (operands split in hi + lo)
size_t gemm_split_packed_bytes(int rows, int K);
fw_status gemm_split_pack(const float* X, int rows, int K, void* Xp, hipStream_t st);
fw_status gemm_split_pack_transposed(const float* X, int K, int rows, void* Xp, hipStream_t st);
double gemm_split_flops_issued(int R, int N, int K, int lower, bool with_runs = false);
int gemm_split_runs(int R, int N, int K);
size_t gemm_split_partial_bytes(int R, int N, int K);
fw_status gemm_split_run(const void* Ap, const void* Bp, int R, int N, int K, int lower, float* C, hipStream_t st,
                         float* part = nullptr, int* runs_out = nullptr);

// ---- extras.hip
fw_status mfma_rate_probe(int zero_operands, int iters, float* sink, double* flops, hipStream_t st);
fw_status bias_compensate(float* b, const float* W, int S, int M, int taps, const float* mu_old, const float* mu_new, float scale,
                          hipStream_t st);
size_t diagnostics_workspace_bytes(int M);
fw_status diagnostics(const float* Phi_y, const float* lambda, int M, float* out, void* ws, hipStream_t st);
size_t cond_probe_workspace_bytes(int M, int k);
fw_status cond_probe(const float* Phi_y, int M, const float* b0, int k, float* out, void* ws, hipStream_t st);

// ---- cond.hip
size_t cond_workspace_bytes(int M);
fw_status cond_state_init(const fw_cond_state* s, hipStream_t st);
fw_status cond_reduce_step(const fw_cond_state* s, const fw_cond_params* p, fw_cond_info* info, void* ws, hipStream_t st);
size_t cond_refresh_workspace_bytes(int M);
bool cond_refresh_plan(int M, size_t ws_bytes, fw_refresh_plan* plan);
fw_status cond_state_refresh(const fw_cond_state* s, void* ws, size_t ws_bytes, hipStream_t st);
fw_status cond_static_scratch(void** ptr, size_t* bytes);

// ---- evd.hip
size_t evd_workspace_bytes(int M);
fw_status whiten_evd(const float* Phi_x, int M, const fw_evd_params* p, float* T, float* Q, float* Qs, float* lambda,
                     void* ws, size_t ws_bytes, hipStream_t st);

}  // namespace fw
