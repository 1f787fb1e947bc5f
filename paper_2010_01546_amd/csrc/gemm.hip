// Gradient transformation G_out = G Q (Sec. 3.1, eqs. (mod_weight_grad), (vQ)) on the gfx950 matrix cores.
//
// Q = T^T T is symmetric, so column c of Q is read as row c: both operands are contiguous along the contraction index.
//   float32: v_mfma_f32_32x32x2_f32 or v_mfma_f32_16x16x4_f32, strips of output tiles per workgroup (see below).
//   bfloat16: v_mfma_f32_32x32x16_bf16, 64 x 128 tile per workgroup, Q rounded to bfloat16 while it is staged.
#include "fw_internal.h"
#include <type_traits>

namespace fw {
namespace {

constexpr int TM = 64;    // rows of G per workgroup
constexpr int TN = 128;   // columns per workgroup
constexpr int KC16 = 32;  // contraction chunk, bfloat16
constexpr int ROWB = KC16 * 2 + 16;  // bytes of one K-major bf16 LDS row

// float32: a workgroup of four wavefronts owns a strip of C output tiles (MF x MF each, MF = 32 or 16) that share one
// row tile of G.  The contraction index is cut into chunks; a chunk of the G rows and of the Q rows that belong to
// the strip's columns (Q is symmetric: column c of Q is row c, contiguous along the contraction index) travels from
// global memory straight into LDS (global_load_lds_dwordx4) into a ring of two or three stages, that many chunks ahead of
// the MFMAs, laid out [panel][row][16-byte group] with the group index XOR-ed by a function of the row so that the
// fragment reads of 16 consecutive rows hit distinct banks.  Inside a chunk the four wavefronts take disjoint quarters
// of the contraction index and each of them updates ALL tiles of the strip, so every SIMD gets the same number of
// MFMAs whatever the tile count; the fragments of the next chunk are read into registers while the MFMAs of the
// current one run, and the four partial strips are summed through LDS at the end, in wavefront order.  A ragged last
// chunk is staged through registers with zero fill.  The host picks (MF, C) so that the workgroup count comes close
// to a multiple of the 256 compute units.  Needs M % 4 == 0.
template <int MF>
struct Mfma;
template <>
struct Mfma<32> {
    typedef floatx16 acc_t;
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }
    // register i of lane (lr, lk) holds row 8*(i/4) + 4*lk + i%4, column lr
    static __device__ __forceinline__ int row(int i, int lk) { return 8 * (i >> 2) + 4 * lk + (i & 3); }
};
template <>
struct Mfma<16> {
    typedef floatx4 acc_t;
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }
    // register i of lane (lr, lk) holds row 4*lk + i, column lr
    static __device__ __forceinline__ int row(int i, int lk) { return 4 * lk + i; }
};

// What the float32 kernels do with a finished element (row, col) of G Q, value v:
//   taps == 1: element index row * M + col.  taps > 1 (per-tap form): the product ran on rows (s, tap) of the permuted
//   gradient, and the element belongs at [s][col][tap] of an [S, M, taps] array (the layout of a convolution weight).
//   out (float32, or bfloat16 bits when out_bf16): the transformed gradient, written when non-null.
//   W (and V): the update  d = v + wd W;  V = momentum V + d (if V);  W -= lr (V or d)   (eq. (vtWrn_SGD)).
__device__ __forceinline__ void emit(const GemmEpilogue& e, int row, int col, int M, float v) {
    size_t idx;
    if (e.taps > 1) {
        const int s = row / e.taps, t = row - s * e.taps;
        idx = ((size_t)s * M + col) * e.taps + t;
    } else {
        idx = (size_t)row * M + col;
    }
    if (e.out) {
        if (e.out_bf16) reinterpret_cast<unsigned short*>(e.out)[idx] = f32_to_bf16_rne(v);
        else reinterpret_cast<float*>(e.out)[idx] = v;
    }
    if (e.W) {
        const float w = e.W[idx];
        float d = v + e.wd * w;
        if (e.V) {
            d = e.momentum * e.V[idx] + d;
            e.V[idx] = d;
        }
        e.W[idx] = w - e.lr * d;
    }
}

// float4 per lane, panel and chunk: enough for about 2000 cycles of MFMAs per chunk and wavefront, within an LDS stage
// of at most 80 KB
__host__ __device__ constexpr int strip_u(int mf, int c) {
    return mf == 32 ? (c >= 9 ? 1 : c >= 4 ? 2 : c >= 2 ? 4 : 8) : (c >= 5 ? 2 : c >= 2 ? 4 : 8);
}

template <int MF, int C>
struct StripCfg {
    static constexpr int KL = 64 / MF;                       // lanes of one row along the contraction index
    static constexpr int KW = 4 * KL;                        // contraction entries one float4 per lane covers
    static constexpr int U = strip_u(MF, C);
    static constexpr int KC = 4 * KW * U;                    // contraction entries per chunk (four wavefronts)
    static constexpr int QR = KC / 4;                        // 16-byte groups per staged row: 8, 16, 32 or 64
    static constexpr int NP = 1 + C;                         // staged panels: G rows, then C tiles of Q rows
    static constexpr int IPW = NP * U;                       // direct-to-LDS loads per wavefront and chunk
    static constexpr int NACC = MF * MF / 64;
    static constexpr int PANEL = MF * KC;                    // floats of one staged panel = 256 U groups
    static constexpr int STAGE = NP * PANEL;
    static constexpr int NST = 3 * STAGE * 4 <= 160 * 1024 ? 3 : 2;   // stages of the LDS ring
    static constexpr int RED = 16 * MF * MF;                 // epilogue: 4 tiles x 4 wavefronts
    static constexpr int SMEM = NST * STAGE > RED ? NST * STAGE : RED;
    // group g of row r is stored at group g ^ swz(r): 16 consecutive rows reading one g then cover 16 distinct
    // 16-byte bank groups
    static __device__ __forceinline__ int swz(int r) { return QR == 8 ? (r >> 1) & 7 : r & 15; }
};

// PLAIN: the result is a float32 [S, M] array and nothing else happens to it (the epilogue's other fields are ignored);
// kept as an instantiation of its own so that the general epilogue costs the plain product no registers.
// With gridDim.z > 1 the contraction index is cut into gridDim.z runs of `kchunks` whole chunks (the last run takes what
// is left, the ragged end included); workgroup z then writes its partial strip to part[z][S][M] instead of finishing
// the result, and strip_reduce_kernel adds the runs in a fixed order and applies the epilogue.
template <int MF, int C, bool PLAIN>
__global__ __launch_bounds__(256) void grad_gemm_f32_strip_kernel(const float* __restrict__ G, const float* __restrict__ Q,
                                                                  GemmEpilogue Out, int S, int M, int kchunks, float* __restrict__ part) {
    typedef StripCfg<MF, C> K;
    typedef typename Mfma<MF>::acc_t acc_t;
    __shared__ __attribute__((aligned(16))) float sm[K::SMEM];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane % MF, lk = lane / MF;
    const int row0 = blockIdx.y * MF, col0 = blockIdx.x * (C * MF);
    acc_t acc[C];
#pragma unroll
    for (int j = 0; j < C; ++j)
#pragma unroll
        for (int i = 0; i < K::NACC; ++i) acc[j][i] = 0.f;

    // Load i of this wavefront fills groups ((i % U)*4 + wave)*64 .. +63 of panel i / U; lane l brings group +l.
    // Rows past the end of G or Q are clamped: they only feed outputs that are never stored.
    int doff[K::IPW];
#pragma unroll
    for (int i = 0; i < K::IPW; ++i) {
        const int p = i / K::U;
        const int sgrp = ((i % K::U) * 4 + wave) * 64 + lane;
        const int r = sgrp / K::QR, q = (sgrp % K::QR) ^ K::swz(r);
        const int grow = p == 0 ? min(row0 + r, S - 1) : min(col0 + (p - 1) * MF + r, M - 1);
        doff[i] = grow * M + 4 * q;
    }
    // this workgroup's run of the contraction index: [kbeg, kbeg + klen)
    const int kbeg = (int)blockIdx.z * kchunks * K::KC;
    const int klen = blockIdx.z + 1 == gridDim.z ? M - kbeg : kchunks * K::KC;
    auto dma_one = [&](int k0, int stage, int i) {   // i is a compile-time constant after unrolling
        const int p = i / K::U;
        dma16((p == 0 ? G : Q) + doff[i] + kbeg + k0, &sm[stage * K::STAGE + p * K::PANEL + ((i % K::U) * 4 + wave) * 256]);
    };
    auto issue = [&](int c, int stage) {
#pragma unroll
        for (int i = 0; i < K::IPW; ++i) dma_one(c * K::KC, stage, i);
    };
    // operand fragments of a chunk for this wavefront's quarter of it
    int foff[K::U];
#pragma unroll
    for (int u = 0; u < K::U; ++u) foff[u] = 4 * (lr * K::QR + (((wave * K::U + u) * K::KL + lk) ^ K::swz(lr)));
    float4 fr[2][K::IPW];
    auto read_one = [&](int stage, float4* f, int i) {   // fragment i = u * NP + p
        f[i] = *reinterpret_cast<const float4*>(&sm[stage * K::STAGE + (i % K::NP) * K::PANEL + foff[i / K::NP]]);
    };
    auto read_frags = [&](int stage, float4* f) {
#pragma unroll
        for (int i = 0; i < K::IPW; ++i) read_one(stage, f, i);
    };
    // MFMA t of a chunk, 0 <= t < NT: t = (u*4 + s)*C + j updates tile j with entry s of the float4 pair u
    constexpr int NT = 4 * K::U * C;
    auto mfma_one = [&](const float4* f, int t) {
        const int j = t % C, s4 = (t / C) % 4, u = t / (4 * C);
        const float4 a = f[u * K::NP], b = f[u * K::NP + 1 + j];
        const float av = s4 == 0 ? a.x : s4 == 1 ? a.y : s4 == 2 ? a.z : a.w;
        const float bv = s4 == 0 ? b.x : s4 == 1 ? b.y : s4 == 2 ? b.z : b.w;
        acc[j] = Mfma<MF>::run(av, bv, acc[j]);
    };
    auto mfmas = [&](const float4* f) {
#pragma unroll
        for (int t = 0; t < NT; ++t) mfma_one(f, t);
    };

    const int nfull = klen / K::KC;
    if (nfull > 0) {
        issue(0, 0);
        if (nfull > 1) issue(1, 1);
        if (K::NST > 2 && nfull > 2) issue(2, 2);
        if (K::NST > 2 && nfull > 2) FW_WAIT_VM(2 * K::IPW);
        else if (nfull > 1) FW_WAIT_VM(K::IPW);
        else FW_WAIT_VM(0);
        __builtin_amdgcn_s_barrier();
        FW_COMPILER_FENCE();
        read_frags(0, fr[0]);
        int sc = 0;   // stage of chunk c
        // Iteration c.  On entry every wavefront has asked for its fragments of chunk c (registers `cur`).  After the
        // first half of the MFMAs: chunk c+1 must have landed (later chunks may still be on their way) and, past the
        // barrier, nobody reads the stage of chunk c any more, so it takes chunk c+NST.  The loads of that chunk and
        // the fragment reads of chunk c+1 are then issued one by one between the remaining MFMAs, which keeps the
        // matrix pipe fed while a single wavefront per SIMD does the issuing.
        constexpr int H = NT / 2, REST = NT - H;
        auto iteration = [&](int c, const float4* cur, float4* nxt, auto STEADY) {
            constexpr bool steady = decltype(STEADY)::value;   // c + NST < nfull known: no branches around the MFMAs
            const int sn = sc == K::NST - 1 ? 0 : sc + 1;
            FW_WAIT_LGKM0();
#pragma unroll
            for (int t = 0; t < H; ++t) mfma_one(cur, t);
            __builtin_amdgcn_sched_barrier(0);
            if (K::NST > 2 && (steady || c + 2 < nfull)) FW_WAIT_VM(K::IPW);
            else FW_WAIT_VM(0);
            __builtin_amdgcn_s_barrier();
            FW_COMPILER_FENCE();
#pragma unroll
            for (int i = 0; i < K::IPW; ++i) {
                if (steady || c + K::NST < nfull) dma_one((c + K::NST) * K::KC, sc, i);
                if (steady || c + 1 < nfull) read_one(sn, nxt, i);
#pragma unroll
                for (int t = H + i * REST / K::IPW; t < H + (i + 1) * REST / K::IPW; ++t) mfma_one(cur, t);
                __builtin_amdgcn_sched_barrier(0);
            }
            sc = sn;
        };
        int c = 0;
        for (; c + 1 + K::NST < nfull; c += 2) {
            iteration(c, fr[0], fr[1], std::true_type());
            iteration(c + 1, fr[1], fr[0], std::true_type());
        }
        for (; c < nfull; c += 2) {   // the last few chunks
            iteration(c, fr[0], fr[1], std::false_type());
            if (c + 1 < nfull) iteration(c + 1, fr[1], fr[0], std::false_type());
        }
    }
    if (nfull * K::KC < klen) {   // ragged last chunk through registers, zero beyond the end
        const int k0 = kbeg + nfull * K::KC;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < K::IPW; ++i) {
            const int p = i / K::U;
            const int sgrp = ((i % K::U) * 4 + wave) * 64 + lane;
            const int r = sgrp / K::QR, q = (sgrp % K::QR) ^ K::swz(r);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k0 + 4 * q < M) v = *reinterpret_cast<const float4*>((p == 0 ? G : Q) + doff[i] + k0);
            *reinterpret_cast<float4*>(&sm[p * K::PANEL + 4 * sgrp]) = v;
        }
        __syncthreads();
        read_frags(0, fr[0]);
        mfmas(fr[0]);
    }
    __syncthreads();

    // sum of the four partial strips: rounds of four tiles, wavefront q owns tile q of the round
    float* red = sm;   // [tile of the round][wavefront][register][lane]
#pragma unroll
    for (int g = 0; g < (C + 3) / 4; ++g) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (4 * g + q < C && wave != q) {
#pragma unroll
                for (int i = 0; i < K::NACC; ++i) red[((q * 4 + wave) * K::NACC + i) * 64 + lane] = acc[(4 * g + q) % C][i];
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (4 * g + q < C && wave == q) {
                const int col = col0 + (4 * g + q) * MF + lr;
#pragma unroll
                for (int i = 0; i < K::NACC; ++i) {
                    float v = 0.f;
#pragma unroll
                    for (int w = 0; w < 4; ++w) v += (w == q) ? acc[(4 * g + q) % C][i] : red[((q * 4 + w) * K::NACC + i) * 64 + lane];
                    const int row = row0 + Mfma<MF>::row(i, lk);
                    if (row < S && col < M) {
                        if (gridDim.z > 1) part[((size_t)blockIdx.z * S + row) * M + col] = v;
                        else if (PLAIN) reinterpret_cast<float*>(Out.out)[(size_t)row * M + col] = v;
                        else emit(Out, row, col, M, v);
                    }
                }
            }
        }
        __syncthreads();
    }
}

// (MF, C) with the lowest cost: rounds of 256 workgroups x MFMA time of a workgroup, contraction padded to whole chunks.
// When that choice still leaves three quarters of the compute units without a workgroup (few rows of G), and a
// workspace for partial strips is at hand, the contraction index is cut into up to STRIP_MAX_RUNS runs of whole chunks;
// a run shorter than about 16 chunks is not worth it (filling the LDS ring and summing the four wavefronts' strips at
// the end take about as long as ten chunks: measured, a 256 x 2304 x 2304 product got slower when cut in four).
struct StripChoice { int mf, c, nks, kchunks; };
constexpr int STRIP_MAX_RUNS = 8;
inline StripChoice pick_strip(int S, int M, bool plain, bool can_split) {
    static const int cs[6] = {9, 6, 4, 3, 2, 1};
    StripChoice best = {32, 1, 1, 0};
    double best_cost = 1e300;
    long long best_wgs = 1;
    for (int mf = 32; mf >= 16; mf -= 16)
        for (int ci = 0; ci < 6; ++ci) {
            const int c = cs[ci];
            if (!plain && mf == 32 && c == 9) continue;   // the general epilogue does not fit beside 9 x 16 accumulators
            const int kw = mf == 32 ? 8 : 16, u = strip_u(mf, c), kc = 4 * kw * u;
            const long long tr = (S + mf - 1) / mf, tc = (M + mf - 1) / mf;
            const long long wgs = tr * ((tc + c - 1) / c);
            const double rounds = (double)((wgs + 255) / 256);
            const double kpad = (double)((M + kc - 1) / kc * kc) / M;
            // a 16x16 tile is a quarter of the MFMA work of a 32x32 tile and reads twice the operands per flop;
            // a wider strip reads fewer operands per MFMA
            const double cost = rounds * c * (mf == 32 ? 1.0 : 0.25 * 1.06) * kpad * (1.0 + 0.02 / c);
            if (cost < best_cost) { best_cost = cost; best = {mf, c, 1, 0}; best_wgs = wgs; }
        }
    if (can_split && best_wgs <= 64) {
        const int kc = 4 * (best.mf == 32 ? 8 : 16) * strip_u(best.mf, best.c);
        const int nchunks = M / kc;
        int nks = (int)(256 / best_wgs);
        if (nks > STRIP_MAX_RUNS) nks = STRIP_MAX_RUNS;
        while (nks > 1 && nchunks / nks < 16) --nks;
        if (nks > 1) { best.nks = nks; best.kchunks = (nchunks + nks - 1) / nks; }
    }
    return best;
}

// sum of the partial strips of the runs, in run order, then the epilogue
template <bool PLAIN>
__global__ __launch_bounds__(256) void strip_reduce_kernel(const float* __restrict__ part, int nks, GemmEpilogue Out, int S, int M) {
    const size_t n4 = (size_t)S * M / 4;
    const size_t stride = (size_t)S * M;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n4; e += (size_t)gridDim.x * 256) {
        float4 v = *reinterpret_cast<const float4*>(part + 4 * e);
        for (int z = 1; z < nks; ++z) {
            const float4 w = *reinterpret_cast<const float4*>(part + (size_t)z * stride + 4 * e);
            v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
        }
        if (PLAIN) {
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(Out.out) + 4 * e) = v;
        } else {
            const int row = (int)((4 * e) / M), col = (int)((4 * e) - (size_t)row * M);
            emit(Out, row, col, M, v.x); emit(Out, row, col + 1, M, v.y); emit(Out, row, col + 2, M, v.z); emit(Out, row, col + 3, M, v.w);
        }
    }
}

template <int MF>
void launch_strip(const StripChoice& ch, const float* G, const float* Q, const GemmEpilogue& Out, int S, int M, float* part, hipStream_t st) {
    const int c = ch.c;
    const dim3 grid(((M + MF - 1) / MF + c - 1) / c, (S + MF - 1) / MF, ch.nks);
    const bool plain = Out.out && !Out.out_bf16 && Out.taps == 1 && !Out.W;
#define FW_STRIP_LAUNCH(CC)                                                                                                \
    if (plain) hipLaunchKernelGGL((grad_gemm_f32_strip_kernel<MF, CC, true>), grid, dim3(256), 0, st, G, Q, Out, S, M, ch.kchunks, part);   \
    else if constexpr (!(MF == 32 && CC == 9))                                                                             \
        hipLaunchKernelGGL((grad_gemm_f32_strip_kernel<MF, CC, false>), grid, dim3(256), 0, st, G, Q, Out, S, M, ch.kchunks, part)
    switch (c) {
        case 9: FW_STRIP_LAUNCH(9); break;
        case 6: FW_STRIP_LAUNCH(6); break;
        case 4: FW_STRIP_LAUNCH(4); break;
        case 3: FW_STRIP_LAUNCH(3); break;
        case 2: FW_STRIP_LAUNCH(2); break;
        default: FW_STRIP_LAUNCH(1); break;
    }
#undef FW_STRIP_LAUNCH
    if (ch.nks > 1) {
        size_t blocks = ((size_t)S * M / 4 + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        if (plain) hipLaunchKernelGGL(strip_reduce_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, part, ch.nks, Out, S, M);
        else hipLaunchKernelGGL(strip_reduce_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, part, ch.nks, Out, S, M);
    }
}

// M not a multiple of 4 (rows of G and Q not 16-byte aligned): a workgroup owns a 32x32 tile of G_out and its four
// wavefronts split the contraction index four ways; operands come straight from global memory / L2 with scalar
// loads (Q along its rows, like the other kernels), partial tiles are combined through LDS.
__global__ __launch_bounds__(256) void grad_gemm_f32_small_kernel(const float* __restrict__ G, const float* __restrict__ Q,
                                                                  GemmEpilogue Out, int S, int M) {
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
    const float* qp = Q + (size_t)(c_ok ? c : 0) * M;   // row c of Q stands for its column c (Q is symmetric)
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
            b[j] = c_ok ? qp[kk] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b[j], acc, 0, 0, 0);
    }
    for (; k < ke; k += 2) {
        const int kk = k + half;
        const bool k_ok = kk < ke;
        const float a = (r_ok && k_ok) ? gp[kk] : 0.f;
        const float b = (c_ok && k_ok) ? qp[kk] : 0.f;
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
            if (row0 + rr < S && c_ok) emit(Out, row0 + rr, c, M, v);
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

// bfloat16 -> float32 copy of G for the widened path of the bfloat16 gradient transform
__global__ __launch_bounds__(256) void widen_bf16_kernel(const unsigned short* __restrict__ src, float* __restrict__ dst, size_t n) {
    for (size_t e = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8; e < n; e += (size_t)gridDim.x * 256 * 8) {
        if (e + 8 <= n) {
            const uint4 v = *reinterpret_cast<const uint4*>(src + e);
            float4 lo, hi;
            lo.x = __uint_as_float(v.x << 16); lo.y = __uint_as_float(v.x & 0xffff0000u);
            lo.z = __uint_as_float(v.y << 16); lo.w = __uint_as_float(v.y & 0xffff0000u);
            hi.x = __uint_as_float(v.z << 16); hi.y = __uint_as_float(v.z & 0xffff0000u);
            hi.z = __uint_as_float(v.w << 16); hi.w = __uint_as_float(v.w & 0xffff0000u);
            *reinterpret_cast<float4*>(dst + e) = lo;
            *reinterpret_cast<float4*>(dst + e + 4) = hi;
        } else {
            for (size_t k = e; k < n; ++k) dst[k] = bf16_to_f32(src[k]);
        }
    }
}

// [S, M, taps] (float32 or bfloat16 bits) -> [S * taps, M] float32; one thread per element of the destination, so the
// writes are contiguous and the strided reads of a wavefront fall into taps-times as many cache lines
__global__ __launch_bounds__(256) void taps_to_rows_kernel(const void* __restrict__ src, int is_bf16, int S, int M, int taps,
                                                           float* __restrict__ dst) {
    const size_t n = (size_t)S * M * taps;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256) {
        const size_t row = e / M;
        const int c = (int)(e - row * M);
        const size_t s = row / taps;
        const int t = (int)(row - s * taps);
        const size_t i = (s * M + c) * taps + t;
        dst[e] = is_bf16 ? bf16_to_f32(reinterpret_cast<const unsigned short*>(src)[i]) : reinterpret_cast<const float*>(src)[i];
    }
}

}  // namespace

size_t grad_gemm_partial_bytes(int S, int M) { return align_up((size_t)STRIP_MAX_RUNS * S * M * sizeof(float), 256); }

// part: room for grad_gemm_partial_bytes(S, M) bytes, or null (then the contraction index is not cut into runs)
fw_status grad_gemm_f32(const float* G, int S, int M, const float* Q, const GemmEpilogue& e, hipStream_t st, float* part) {
    if ((M & 3) != 0)
        hipLaunchKernelGGL(grad_gemm_f32_small_kernel, dim3((M + 31) / 32, (S + 31) / 32), dim3(256), 0, st, G, Q, e, S, M);
    else {
        const bool plain = e.out && !e.out_bf16 && e.taps == 1 && !e.W;
        const StripChoice ch = pick_strip(S, M, plain, part != nullptr);
        if (ch.mf == 32) launch_strip<32>(ch, G, Q, e, S, M, part, st);
        else launch_strip<16>(ch, G, Q, e, S, M, part, st);
    }
    FW_LAUNCH_CHECK();
    return FW_OK;
}

// Epilogue applied to a product that sits in the workspace as `nks` partial results [nks][S][M] (M a multiple of 4): the
// runs are added in order and every element goes where `e` says (store, per-tap position, rounding, weight update)
fw_status grad_epilogue_from_runs(const float* part, int nks, const GemmEpilogue& e, int S, int M, hipStream_t st) {
    if ((M & 3) != 0 || nks < 1) return FW_ERR_UNSUPPORTED;
    size_t blocks = ((size_t)S * M / 4 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(strip_reduce_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, part, nks, e, S, M);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

fw_status grad_gemm(const void* G, fw_dtype dt, int S, int M, const float* Q, void* G_out, hipStream_t st, float* part) {
    if (dt == FW_BF16) {
        const dim3 grid((M + TN - 1) / TN, (S + TM - 1) / TM);
        hipLaunchKernelGGL(grad_gemm_bf16_kernel, grid, dim3(256), 0, st, reinterpret_cast<const unsigned short*>(G), Q,
                           reinterpret_cast<unsigned short*>(G_out), S, M);
        FW_LAUNCH_CHECK();
        return FW_OK;
    }
    GemmEpilogue e = {};
    e.out = G_out; e.taps = 1;
    return grad_gemm_f32(reinterpret_cast<const float*>(G), S, M, Q, e, st, part);
}

// bfloat16 (or per-tap) gradient -> float32 rows in scratch.  src is [S, M] (taps == 1) or [S, M, taps]; dst is
// [S * taps, M] float32 with row s * taps + t holding src[s][:][t].
fw_status grad_stage_rows(const void* G, fw_dtype dt, int S, int M, int taps, float* dst, hipStream_t st) {
    const size_t n = (size_t)S * M * taps;
    if (taps == 1 && dt == FW_BF16) {
        size_t blocks = (n / 8 + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        if (blocks == 0) blocks = 1;
        hipLaunchKernelGGL(widen_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, reinterpret_cast<const unsigned short*>(G), dst, n);
    } else {
        size_t blocks = (n + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        hipLaunchKernelGGL(taps_to_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, G, dt == FW_BF16 ? 1 : 0, S, M, taps, dst);
    }
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
