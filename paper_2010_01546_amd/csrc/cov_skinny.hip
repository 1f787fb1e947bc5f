// Moment accumulation for inputs with few features and many rows (the sums inside eqs. (vmuxi), (vPhixi) of Sec. 2):
// 1x1 windows with M <= 128 -- the per-channel variant (whitening in front of a convolution, M = Cin, Sec. 6),
// pointwise and shortcut convolutions, narrow fully connected layers.  Such a call is bound by reading the rows once,
// so there is no staging at all: a wavefront streams its own run of rows straight into MFMA operands
// (v_mfma_f32_32x32x2_f32: lanes 0..31 hold 32 features of one row, lanes 32..63 the same features of the next row),
// keeps the lower-triangle tiles of the M x M result in registers, and the four wavefronts of a workgroup are summed
// through LDS before one partial result per workgroup goes to the workspace.  bfloat16 rows are widened in registers
// (their products are exact in float32 either way); a lane then loads two neighbouring features as one 32-bit word, so
// operand group t of a bfloat16 call holds the features 64 (t / 2) + 2 lane + (t & 1) instead of 32 t + lane.
#include "fw_internal.h"

namespace fw {
namespace {

constexpr int SK_UMAX = 8;   // row pairs per batch of loads: 8 for M <= 64, 4 above (registers)

struct SkinnyGeom {
    int n_rows, M, H, W, Ho, Wo, stride;
    int rows_per_wave;   // multiple of 2 * SK_UMAX
    int nwg;
};

// feature held by lane l (of 32) of operand group t
__host__ __device__ inline int skinny_feature(int t, int l, bool paired) { return paired ? 64 * (t >> 1) + 2 * l + (t & 1) : 32 * t + l; }

// PAIRED (bfloat16, even NB, even M): two neighbouring features per 32-bit load
// CONTIG: the rows follow each other in memory (stride 1, or plain rows)
template <int NB, bool BF16, bool PAIRED, bool CONTIG>
__global__ __launch_bounds__(256) void cov_skinny_kernel(const void* __restrict__ Xv, SkinnyGeom g, float* __restrict__ part,
                                                         float* __restrict__ spart) {
    constexpr int NT = NB * (NB + 1) / 2;             // 32x32 tiles of the lower triangle
    constexpr int SK_U = NB <= 2 ? 8 : 4;
    __shared__ float red[2][NT][1024];                // two wavefronts' tiles
    __shared__ float sred[4][NB][32];
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wid = blockIdx.x * 4 + wave;
    const int r_begin = min(g.n_rows, wid * g.rows_per_wave), r_end = min(g.n_rows, r_begin + g.rows_per_wave);

    floatx16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
    float cs[NB];
    bool f_ok[NB];
#pragma unroll
    for (int t = 0; t < NB; ++t) { cs[t] = 0.f; f_ok[t] = skinny_feature(t, l32, PAIRED) < g.M; }

    // this lane's row: r_begin + half, then two further per step; its element index (the tensor has fewer than 2^31
    // elements) moves along with it
    int r = r_begin + half;
    int oy = 0, ox = 0, base;
    if (CONTIG) {
        base = r * g.M;
    } else {
        const int P = g.Ho * g.Wo;
        const int b = r / P, p = r - b * P;
        oy = p / g.Wo; ox = p - oy * g.Wo;
        base = ((b * g.H + oy * g.stride) * g.W + ox * g.stride) * g.M;
    }
    const int step_x = g.stride * g.M;                              // one output column on
    const int wrap_x = (g.stride * g.W - g.Wo * g.stride) * g.M;    // to the next output row
    const int wrap_y = (g.H - g.Ho * g.stride) * g.W * g.M;         // to the next image
    auto advance2 = [&]() {
        if (CONTIG) { r += 2; base += 2 * g.M; return; }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            ++r; ++ox; base += step_x;
            if (ox == g.Wo) { ox = 0; ++oy; base += wrap_x; }
            if (oy == g.Ho) { oy = 0; base += wrap_y; }
        }
    };
    // Loads are issued unconditionally (a masked lane reads element 0) and masked when they are used; the raw words
    // pass through an empty asm statement at the point of use, which keeps the compiler from moving the loads into a
    // branch on the mask (it would then wait for every load on the spot).
    constexpr int NW = PAIRED ? NB / 2 : NB;          // loads per row pair
    auto load = [&](unsigned* raw, unsigned& okbits) {
        const bool row_ok = r < r_end;
        okbits = 0;
#pragma unroll
        for (int t = 0; t < NW; ++t) {
            const bool ok = row_ok && f_ok[PAIRED ? 2 * t : t];   // a pair 64 t + 2 lane, + 1 lies inside or outside together
            const int idx = ok ? base + (PAIRED ? 64 * t + 2 * l32 : 32 * t + l32) : 0;
            if (PAIRED) raw[t] = *reinterpret_cast<const unsigned*>(reinterpret_cast<const unsigned short*>(Xv) + idx);
            else if (BF16) raw[t] = reinterpret_cast<const unsigned short*>(Xv)[idx];
            else raw[t] = reinterpret_cast<const unsigned*>(Xv)[idx];
            okbits |= (ok ? 1u : 0u) << t;
        }
    };
    auto unpack = [&](unsigned* raw, unsigned okbits, float* a) {
#pragma unroll
        for (int t = 0; t < NW; ++t) {
            unsigned w = raw[t];
            asm volatile("" : "+v"(w));
            const bool ok = (okbits >> t) & 1u;
            if (PAIRED) {
                a[2 * t] = ok ? __uint_as_float(w << 16) : 0.f;
                a[2 * t + 1] = ok ? __uint_as_float(w & 0xffff0000u) : 0.f;
            } else if (BF16) {
                a[t] = ok ? __uint_as_float(w << 16) : 0.f;
            } else {
                a[t] = ok ? __uint_as_float(w) : 0.f;
            }
        }
    };

    // the rows of the next batch are on their way while the current one is multiplied
    const int npairs = (r_end - r_begin + 1) / 2;
    unsigned raw[2][SK_U][NW], okb[2][SK_U];
#pragma unroll
    for (int u = 0; u < SK_U; ++u) { load(raw[0][u], okb[0][u]); advance2(); }   // past the end of the run the loads are masked
    for (int p0 = 0; p0 < npairs; p0 += 2 * SK_U) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int u = 0; u < SK_U; ++u) { load(raw[h ^ 1][u], okb[h ^ 1][u]); advance2(); }
#pragma unroll
            for (int u = 0; u < SK_U; ++u) {
                float a[NB];
                unpack(raw[h][u], okb[h][u], a);
#pragma unroll
                for (int t = 0; t < NB; ++t) cs[t] += a[t];
#pragma unroll
                for (int ta = 0; ta < NB; ++ta)
#pragma unroll
                    for (int tb = 0; tb <= ta; ++tb)
                        acc[ta * (ta + 1) / 2 + tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta], a[tb], acc[ta * (ta + 1) / 2 + tb], 0, 0, 0);
            }
        }
    }

    // the four wavefronts of the workgroup, summed in a fixed order: (0 + 2) + (1 + 3)
    auto put = [&](int slot) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) red[slot][t][(8 * (i >> 2) + 4 * half + (i & 3)) * 32 + l32] = acc[t][i];
    };
    auto add = [&](int slot) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[t][i] += red[slot][t][(8 * (i >> 2) + 4 * half + (i & 3)) * 32 + l32];
    };
#pragma unroll
    for (int t = 0; t < NB; ++t) {
        const float v = cs[t] + __shfl_xor(cs[t], 32, 64);
        if (half == 0) sred[wave][t][l32] = v;
    }
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) add(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave == 0) {
        add(0);
        float* dst = part + (size_t)blockIdx.x * NT * 1024;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) dst[t * 1024 + (8 * (i >> 2) + 4 * half + (i & 3)) * 32 + l32] = acc[t][i];
        if (half == 0) {
#pragma unroll
            for (int t = 0; t < NB; ++t)
                spart[(size_t)blockIdx.x * (NB * 32) + 32 * t + l32] = (sred[0][t][l32] + sred[2][t][l32]) + (sred[1][t][l32] + sred[3][t][l32]);
        }
    }
}

// partial results of the workgroups -> A (lower triangle) and s.  A workgroup takes 16 consecutive entries of the
// partial layout; 16 threads per entry sum every sixteenth workgroup's value (float64, eight loads in flight) and are
// combined through LDS in a fixed order.
__global__ __launch_bounds__(256) void cov_skinny_reduce_kernel(SkinnyGeom g, int nb, int paired, const float* __restrict__ part,
                                                                const float* __restrict__ spart, float* __restrict__ A, float* __restrict__ s) {
    __shared__ double red[16][17];
    const int nt = nb * (nb + 1) / 2;
    const int el = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int e = blockIdx.x * 16 + el;
    const float* src = nullptr;
    size_t stride = 0;
    float* dst = nullptr;
    if (e < nt * 1024) {
        const int t = e >> 10, w = e & 1023;
        int ta = 0;
        while ((ta + 1) * (ta + 2) / 2 <= t) ++ta;
        const int tb = t - ta * (ta + 1) / 2;
        const int i = skinny_feature(ta, w >> 5, paired != 0), j = skinny_feature(tb, w & 31, paired != 0);
        // the tiles on and below the diagonal of the tile grid hold every unordered pair once, except that a diagonal
        // tile holds both (i, j) and (j, i): keep the one with j <= i
        if (i < g.M && j < g.M && !(ta == tb && j > i)) {
            src = part + e; stride = (size_t)nt * 1024;
            dst = A + (size_t)max(i, j) * g.M + min(i, j);
        }
    } else {
        const int q = e - nt * 1024;          // group-major position of a column sum
        if (q < nb * 32) {
            const int f = skinny_feature(q >> 5, q & 31, paired != 0);
            if (f < g.M) { src = spart + q; stride = (size_t)nb * 32; dst = s + f; }
        }
    }
    double v = 0.0;
    if (src) {
        int w = grp;
        for (; w + 112 < g.nwg; w += 128) {
            float x[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) x[q] = src[(size_t)(w + 16 * q) * stride];
#pragma unroll
            for (int q = 0; q < 8; ++q) v += (double)x[q];
        }
        for (; w < g.nwg; w += 16) v += (double)src[(size_t)w * stride];
    }
    red[grp][el] = v;
    __syncthreads();
    if (grp == 0 && dst) {
        double t = 0.0;
#pragma unroll
        for (int q = 0; q < 16; ++q) t += red[q][el];
        *dst = (float)((double)*dst + t);
    }
}

bool make_skinny_geom(const fw_conv_desc* d, fw_layout lay, SkinnyGeom* g) {
    if (lay == FW_LAYOUT_NCHW && !(d->H == 1 && d->W == 1)) return false;
    if (d->kh != 1 || d->kw != 1 || d->pad != 0 || d->Cin > 128) return false;
    const int Ho = (d->H - 1) / d->stride + 1, Wo = (d->W - 1) / d->stride + 1;
    const long long n_rows = (long long)d->B * Ho * Wo;
    if (n_rows < 2048 || n_rows >= (1ll << 31) - 64 || (long long)d->B * d->H * d->W * d->Cin >= (1ll << 30)) return false;   // element indices stay far inside int
    g->n_rows = (int)n_rows; g->M = d->Cin; g->H = d->H; g->W = d->W; g->Ho = Ho; g->Wo = Wo; g->stride = d->stride;
    // as many workgroups as the registers let a compute unit hold (4, 2 or 1), each wavefront with at least 128 rows: what
    // hides the latency of the loads is wavefronts x batches in flight.  With 3 or 4 blocks of 32 features a row pair
    // costs 6 or 10 matrix instructions, and it is those that want to be spread over all SIMDs: 64 and 32 rows then.
    long long nwg = d->Cin <= 64 ? 1024 : d->Cin <= 96 ? 512 : 256;
    const int min_rows = d->Cin <= 64 ? 128 : d->Cin <= 96 ? 64 : 32;
    while (nwg > 1 && n_rows / (nwg * 4) < min_rows) nwg >>= 1;
    long long rpw = (n_rows + nwg * 4 - 1) / (nwg * 4);
    rpw = (rpw + 2 * SK_UMAX - 1) / (2 * SK_UMAX) * (2 * SK_UMAX);
    g->rows_per_wave = (int)rpw;
    g->nwg = (int)((n_rows + rpw * 4 - 1) / (rpw * 4));
    return true;
}

size_t skinny_part_bytes(const SkinnyGeom& g) {
    const int nb = (g.M + 31) / 32;
    return align_up((size_t)g.nwg * (nb * (nb + 1) / 2) * 1024 * sizeof(float), 256);
}

}  // namespace

bool cov_skinny_applies(const fw_conv_desc* d, fw_layout lay) {
    SkinnyGeom g;
    return d && make_skinny_geom(d, lay, &g);
}

size_t cov_skinny_workspace_bytes(const fw_conv_desc* d, fw_layout lay) {
    SkinnyGeom g;
    if (!d || !make_skinny_geom(d, lay, &g)) return 0;
    const int nb = (g.M + 31) / 32;
    return skinny_part_bytes(g) + align_up((size_t)g.nwg * nb * 32 * sizeof(float), 256);
}

bool cov_skinny_plan(const fw_conv_desc* d, fw_layout lay, fw_cov_plan* plan) {
    SkinnyGeom g;
    if (!d || !make_skinny_geom(d, lay, &g)) return false;
    const int nb = (g.M + 31) / 32;
    plan->workgroups = g.nwg; plan->ranges = g.nwg * 4;
    plan->mfma_flops_issued = 2.0 * 1024.0 * (nb * (nb + 1) / 2) * (double)g.nwg * 4.0 * g.rows_per_wave;
    return true;
}

fw_status cov_skinny_accumulate(const void* X, fw_dtype dt, fw_layout lay, const fw_conv_desc* d, float* A, float* s, void* ws,
                                size_t ws_bytes, hipStream_t st) {
    SkinnyGeom g;
    if (!make_skinny_geom(d, lay, &g)) return FW_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < cov_skinny_workspace_bytes(d, lay)) return FW_ERR_WORKSPACE;
    float* part = reinterpret_cast<float*>(ws);
    float* spart = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + skinny_part_bytes(g));
    const int nb = (g.M + 31) / 32;
    const bool bf = dt == FW_BF16;
    const bool paired = bf && (nb % 2) == 0 && (g.M % 2) == 0;
    const bool contig = g.stride == 1 || (g.H == 1 && g.W == 1);
#define FW_SKINNY_C(NBV, C)                                                                                                         \
    if (paired) hipLaunchKernelGGL((cov_skinny_kernel<NBV, true, (NBV % 2 == 0), C>), dim3(g.nwg), dim3(256), 0, st, X, g, part, spart); \
    else if (bf) hipLaunchKernelGGL((cov_skinny_kernel<NBV, true, false, C>), dim3(g.nwg), dim3(256), 0, st, X, g, part, spart);   \
    else hipLaunchKernelGGL((cov_skinny_kernel<NBV, false, false, C>), dim3(g.nwg), dim3(256), 0, st, X, g, part, spart)
#define FW_SKINNY(NBV)                 \
    if (contig) { FW_SKINNY_C(NBV, true); } \
    else { FW_SKINNY_C(NBV, false); }
    switch (nb) {
        case 1: FW_SKINNY(1); break;
        case 2: FW_SKINNY(2); break;
        case 3: FW_SKINNY(3); break;
        default: FW_SKINNY(4); break;
    }
#undef FW_SKINNY
#undef FW_SKINNY_C
    FW_LAUNCH_CHECK();
    const int n = (nb * (nb + 1) / 2) * 1024 + nb * 32;
    hipLaunchKernelGGL(cov_skinny_reduce_kernel, dim3((n + 15) / 16), dim3(256), 0, st, g, nb, paired ? 1 : 0, part, spart, A, s);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
