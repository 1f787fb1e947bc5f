// bfloat16 moment accumulation A += X^T X (sums inside eqs. (vmuxi), (vPhixi), (phixmi)) on the gfx950 matrix cores.
//
// v_mfma_f32_32x32x16_bf16 wants, per lane, eight consecutive entries of the reduction index for one feature.
// The reduction index of X^T X is the patch row (image, oy, ox); any order of it gives the same sums, so the
// eight entries of a lane are taken from EIGHT IMAGES at one output position.  A bandwidth-bound pre-pass packs
// the activation tensor into
//     P[image group][y + pad][x + pad][channel] -> 8 x bf16 (16 bytes: the same pixel and channel of 8 images)
// with a zero border of `pad` pixels, so that every tap of every output position is one aligned 16-byte load with
// no bounds test, for any window, stride and input layout.  A "unit" is (image group, oy, ox); an MFMA consumes two.
//
// The contraction kernel cuts the lower triangle of A into 256x256 tiles.  A workgroup of 8 wavefronts (2 x 4, each
// 128x64 = 4x2 MFMA tiles) owns one tile over a range of units; panels of 8 units are prefetched into registers one
// chunk ahead and double-buffered in LDS as [unit][feature][16 B], which both the staging writes and the
// ds_read_b128 operand reads traverse contiguously.  Diagonal tiles stage one panel and accumulate the column sums.
// With one range per tile the result is added straight into A; otherwise partial tiles go to the workspace and are
// summed in float64.
#include "fw_internal.h"
#include <math.h>
#include <stdlib.h>

namespace fw {
namespace {

constexpr int TB = 256;  // tile edge (features)
constexpr int KU = 8;    // units per staged chunk (64 reduction entries)

struct TileGeom {
    int M, nb, ntiles;
    int B, Bg, Cin, H, W, Hp, Wp, kh, kw, stride, pad, Ho, Wo;
    int layout;
    int n_units, units_per_split, nsplit;
    int direct;   // one range per tile and external order == internal order: tiles are added straight into A
};

typedef unsigned short u16;

// ---- pre-pass: pack 8 images per 16 bytes, zero border ---------------------------------------------------------
__global__ __launch_bounds__(256) void pack_images_kernel(const u16* __restrict__ X, TileGeom g, uint4* __restrict__ P) {
    const long long total = (long long)g.Bg * g.Hp * g.Wp * g.Cin;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
        int c, xp, yp, bg;
        long long t = e;
        if (g.layout == FW_LAYOUT_NCHW) {  // walk the source along x for coalescing; the packed order stays [bg][yp][xp][c]
            xp = (int)(t % g.Wp); t /= g.Wp;
            yp = (int)(t % g.Hp); t /= g.Hp;
            c = (int)(t % g.Cin); bg = (int)(t / g.Cin);
        } else {
            c = (int)(t % g.Cin); t /= g.Cin;
            xp = (int)(t % g.Wp); t /= g.Wp;
            yp = (int)(t % g.Hp); bg = (int)(t / g.Hp);
        }
        const int y = yp - g.pad, x = xp - g.pad;
        unsigned v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int b = bg * 8 + i;
            unsigned val = 0;
            if (b < g.B && (unsigned)y < (unsigned)g.H && (unsigned)x < (unsigned)g.W) {
                const long long src = g.layout == FW_LAYOUT_NCHW ? (((long long)b * g.Cin + c) * g.H + y) * g.W + x
                                                                 : (((long long)b * g.H + y) * g.W + x) * g.Cin + c;
                val = X[src];
            }
            v[i] = val;
        }
        uint4 o;
        o.x = v[0] | (v[1] << 16); o.y = v[2] | (v[3] << 16); o.z = v[4] | (v[5] << 16); o.w = v[6] | (v[7] << 16);
        P[(((long long)bg * g.Hp + yp) * g.Wp + xp) * g.Cin + c] = o;
    }
}

// offset (in 16-byte elements) of the top-left tap of every unit
__global__ __launch_bounds__(256) void unit_table_kernel(TileGeom g, int* __restrict__ utab) {
    const int u = blockIdx.x * 256 + threadIdx.x;
    if (u >= g.n_units) return;
    const int P = g.Ho * g.Wo;
    const int bg = u / P, p = u - bg * P;
    const int oy = p / g.Wo, ox = p - oy * g.Wo;
    utab[u] = ((bg * g.Hp + oy * g.stride) * g.Wp + ox * g.stride) * g.Cin;
}

// internal feature (tap-major, channel-minor) -> offset inside a unit, external index m = (c*kh + ky)*kw + kx
// (or the internal index itself when the caller works in channels-last feature order)
__device__ __forceinline__ void feat_map(int fi, const TileGeom& g, int* off, int* ext) {
    const int t = fi / g.Cin, c = fi - t * g.Cin;
    const int ky = t / g.kw, kx = t - ky * g.kw;
    *off = (ky * g.Wp + kx) * g.Cin + c;
    *ext = g.layout == FW_LAYOUT_NHWC_KKC ? fi : c * (g.kh * g.kw) + t;
}

__device__ __forceinline__ float sum8_bf16(const uint4& v) {
    float s = 0.f;
    s += __uint_as_float(v.x << 16) + __uint_as_float(v.x & 0xffff0000u);
    s += __uint_as_float(v.y << 16) + __uint_as_float(v.y & 0xffff0000u);
    s += __uint_as_float(v.z << 16) + __uint_as_float(v.z & 0xffff0000u);
    s += __uint_as_float(v.w << 16) + __uint_as_float(v.w & 0xffff0000u);
    return s;
}

struct SmemTile {
    alignas(16) uint4 pan[2][2][KU][TB];  // [buffer][row panel / column panel][unit][feature], 128 KB
};

__global__ __launch_bounds__(512) void cov_bf16_tile_kernel(const uint4* __restrict__ P, const int* __restrict__ utab, TileGeom g,
                                                            float* __restrict__ part, float* __restrict__ spart, float* __restrict__ A) {
    __shared__ SmemTile sm;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave >> 2, wj = wave & 3;
    const int half = lane >> 5, l32 = lane & 31;
    const int tile = blockIdx.x, split = blockIdx.y;
    int I = (int)((sqrtf(8.f * tile + 1.f) - 1.f) * 0.5f);
    while ((I + 1) * (I + 2) / 2 <= tile) ++I;
    while (I * (I + 1) / 2 > tile) --I;
    const int J = tile - I * (I + 1) / 2;
    const bool diag = I == J;

    const int f = tid & 255, ul = tid >> 8;
    int offA, offB, extA, extB;
    const bool okA = I * TB + f < g.M, okB = J * TB + f < g.M;
    feat_map(okA ? I * TB + f : 0, g, &offA, &extA);
    feat_map(okB ? J * TB + f : 0, g, &offB, &extB);

    floatx16 acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    const int u_begin = split * g.units_per_split;
    const int u_end = min(g.n_units, u_begin + g.units_per_split);
    const int nchunks = (u_end - u_begin + KU - 1) / KU;

    uint4 pa[KU / 2], pb[KU / 2];
    int base[KU / 2];      // unit offsets of the chunk whose loads come next; -1 past the end of the range
    float ssum = 0.f;
    auto load_bases = [&](int c) {
#pragma unroll
        for (int j = 0; j < KU / 2; ++j) {
            const int u = u_begin + c * KU + ul + 2 * j;
            base[j] = (c < nchunks && u < u_end) ? utab[u] : -1;
        }
    };
    auto load_chunk = [&]() {
#pragma unroll
        for (int j = 0; j < KU / 2; ++j) {
            pa[j] = make_uint4(0, 0, 0, 0);
            pb[j] = make_uint4(0, 0, 0, 0);
            if (base[j] >= 0) {
                if (okA) pa[j] = P[base[j] + offA];
                if (!diag && okB) pb[j] = P[base[j] + offB];
            }
        }
    };
    auto store_chunk = [&](int buf) {
#pragma unroll
        for (int j = 0; j < KU / 2; ++j) {
            sm.pan[buf][0][ul + 2 * j][f] = pa[j];
            if (!diag) sm.pan[buf][1][ul + 2 * j][f] = pb[j];
            else ssum += sum8_bf16(pa[j]);
        }
    };

    // L2 warm-up: every chunk ahead of the register prefetch is touched with one 4-byte load per 128-byte line, so that
    // the 16-byte panel loads find their lines in L2 instead of waiting, all lanes at a barrier, for the slowest miss.
    // Thread -> (panel, unit, line): 2 x 8 x 32 lines of 8 features.  The value is never used; the empty asm at the top
    // of the next iteration is only there to retire the load one iteration after it was issued.
    constexpr int PD = 3;   // chunks between the touch and the MFMAs that consume the chunk
    const int t_unit = (tid >> 5) & 7, t_panel = tid >> 8;
    int t_off, t_ext;
    const int t_feat = (t_panel ? J : I) * TB + 8 * (tid & 31);
    const bool t_ok = t_feat < g.M && !(diag && t_panel);
    feat_map(t_ok ? t_feat : 0, g, &t_off, &t_ext);
    unsigned pending = 0;
    int t_base = -1;
    auto touch_base = [&](int c) {
        const int u = u_begin + c * KU + t_unit;
        return (c < nchunks && u < u_end) ? utab[u] : -1;
    };
    t_base = touch_base(PD);

    load_bases(0);
    if (nchunks > 0) {
        load_chunk();
        load_bases(1);
        store_chunk(0);
    }
    __syncthreads();
    const int pj = diag ? 0 : 1;
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        const bool more = c + 1 < nchunks;
        asm volatile("" ::"v"(pending));
        if (more) { load_chunk(); load_bases(c + 2); }
        if (t_ok && t_base >= 0) pending = *reinterpret_cast<const unsigned*>(P + t_base + t_off);
        t_base = touch_base(c + PD + 1);
        // operand fragments are read one k-step ahead of the MFMAs that use them (two register sets)
        bf16x8 fa[2][4], fb[2][2];
        auto read_frags = [&](int ks, int set) {
            const int unit = 2 * ks + half;
#pragma unroll
            for (int t = 0; t < 4; ++t) fa[set][t] = *reinterpret_cast<const bf16x8*>(&sm.pan[buf][0][unit][128 * wi + 32 * t + l32]);
#pragma unroll
            for (int t = 0; t < 2; ++t) fb[set][t] = *reinterpret_cast<const bf16x8*>(&sm.pan[buf][pj][unit][64 * wj + 32 * t + l32]);
        };
        read_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < KU / 2; ++ks) {
            if (ks + 1 < KU / 2) read_frags(ks + 1, (ks + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);   // keep the reads of the next step ahead of this step's MFMAs
#pragma unroll
            for (int ta = 0; ta < 4; ++ta)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
                    acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][ta], fb[ks & 1][tb], acc[ta][tb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (more) store_chunk(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue
    if (!g.direct) {
        float* dst = part + ((size_t)split * g.ntiles + tile) * (TB * TB);
#pragma unroll
        for (int ta = 0; ta < 4; ++ta)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = 128 * wi + 32 * ta + 8 * (i >> 2) + 4 * half + (i & 3);
                    const int col = 64 * wj + 32 * tb + l32;
                    dst[row * TB + col] = acc[ta][tb][i];
                }
    } else {
        // one range per tile, feature order kept: add into the lower triangle of A, 32 lanes along a row
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            const int col = 64 * wj + 32 * tb + l32;
            const int gj = J * TB + col;
#pragma unroll
            for (int ta = 0; ta < 4; ++ta)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = 128 * wi + 32 * ta + 8 * (i >> 2) + 4 * half + (i & 3);
                    const int gi = I * TB + row;
                    if (gi >= g.M || gj >= g.M || gj > gi) continue;
                    A[(size_t)gi * g.M + gj] += acc[ta][tb][i];
                }
        }
    }
    if (diag) {
        // column sums of this block: the two unit groups of a feature meet in LDS
        float* red = reinterpret_cast<float*>(&sm.pan[1][0][0][0]);
        red[tid] = ssum;
        __syncthreads();
        if (tid < 256 && okA) spart[(size_t)split * g.nb * TB + I * TB + f] = red[f] + red[256 + f];
    }
}

// partial tiles -> A (float64 sum over the ranges), one thread per tile element
__global__ __launch_bounds__(256) void tile_reduce_kernel(TileGeom g, const float* __restrict__ part, float* __restrict__ A) {
    const int tile = blockIdx.x >> 8;            // 256 blocks of 256 threads per tile
    const int e = ((blockIdx.x & 255) << 8) + threadIdx.x;
    int I = (int)((sqrtf(8.f * tile + 1.f) - 1.f) * 0.5f);
    while ((I + 1) * (I + 2) / 2 <= tile) ++I;
    while (I * (I + 1) / 2 > tile) --I;
    const int J = tile - I * (I + 1) / 2;
    const int row = e >> 8, col = e & 255;
    const int fi = I * TB + row, fj = J * TB + col;
    if (fi >= g.M || fj >= g.M || (I == J && row < col)) return;
    const size_t stride = (size_t)g.ntiles * TB * TB;
    const float* src = part + (size_t)tile * (TB * TB) + e;
    double v = 0.0;
    for (int sp = 0; sp < g.nsplit; ++sp) v += (double)src[sp * stride];
    int o, ei, ej;
    feat_map(fi, g, &o, &ei);
    feat_map(fj, g, &o, &ej);
    float* dst = A + (size_t)max(ei, ej) * g.M + min(ei, ej);
    *dst = (float)((double)*dst + v);
}

__global__ __launch_bounds__(256) void tile_reduce_sums_kernel(TileGeom g, const float* __restrict__ spart, float* __restrict__ s) {
    __shared__ double red[4][64];
    const int fi = blockIdx.x * 64 + (threadIdx.x & 63), grp = threadIdx.x >> 6;
    double v = 0.0;
    if (fi < g.M)
        for (int sp = grp; sp < g.nsplit; sp += 4) v += (double)spart[(size_t)sp * g.nb * TB + fi];
    red[grp][threadIdx.x & 63] = v;
    __syncthreads();
    if (grp == 0 && fi < g.M) {
        v = red[0][threadIdx.x] + red[1][threadIdx.x] + red[2][threadIdx.x] + red[3][threadIdx.x];
        int o, e;
        feat_map(fi, g, &o, &e);
        s[e] = (float)((double)s[e] + v);
    }
}

bool make_tile_geom(const fw_conv_desc* d, fw_layout lay, TileGeom* g) {
    g->B = d->B; g->Cin = d->Cin; g->H = d->H; g->W = d->W;
    g->kh = d->kh; g->kw = d->kw; g->stride = d->stride; g->pad = d->pad;
    g->layout = (int)lay;
    g->Ho = (d->H + 2 * d->pad - d->kh) / d->stride + 1;
    g->Wo = (d->W + 2 * d->pad - d->kw) / d->stride + 1;
    g->Hp = d->H + 2 * d->pad; g->Wp = d->W + 2 * d->pad;
    g->Bg = (d->B + 7) / 8;
    const long long M = (long long)d->Cin * d->kh * d->kw;
    const long long n_units = (long long)g->Bg * g->Ho * g->Wo;
    const long long packed = (long long)g->Bg * g->Hp * g->Wp * d->Cin;
    if (M <= 0 || M > 16384 || n_units <= 0 || n_units >= (1ll << 31) || packed >= (1ll << 31)) return false;
    if ((long long)d->B * d->Cin * d->H * d->W >= (1ll << 31)) return false;
    g->M = (int)M; g->nb = (int)((M + TB - 1) / TB); g->ntiles = g->nb * (g->nb + 1) / 2;
    g->n_units = (int)n_units;
    // Number of unit ranges per tile: minimise  rounds x units per range x t_unit  +  traffic of the partial tiles,
    // with rounds = ceil(tiles x ranges / 256 compute units); one range means no partial tiles at all.
    const double t_unit = 0.15e-6, bw = 4.0e12;
    const long long nchunks = (n_units + KU - 1) / KU;
    double best = 1e30;
    int best_ns = 1;
    for (int ns = 1; ns <= 512 && ns <= nchunks; ++ns) {
        const long long wgs = (long long)g->ntiles * ns;
        const long long rounds = (wgs + 255) / 256;
        const long long cps = (nchunks + ns - 1) / ns;
        double cost = (double)rounds * (double)cps * KU * t_unit;
        if (ns > 1) cost += (double)wgs * TB * TB * 4.0 * 2.0 / bw;
        if (cost < best * 0.999) { best = cost; best_ns = ns; }
    }
    if (const char* e = getenv("FW_COV_BF16_SPLITS")) best_ns = atoi(e) > 0 ? atoi(e) : best_ns;
    if (best_ns > nchunks) best_ns = (int)nchunks;
    const long long cps = (nchunks + best_ns - 1) / best_ns;
    g->units_per_split = (int)(cps * KU);
    g->nsplit = (int)((n_units + g->units_per_split - 1) / g->units_per_split);
    const bool ident = lay == FW_LAYOUT_NHWC_KKC || lay == FW_LAYOUT_ROWS || d->kh * d->kw == 1;
    g->direct = (g->nsplit == 1 && ident) ? 1 : 0;
    return true;
}

struct Bf16Ws { size_t packed, utab, part, spart, total; };
Bf16Ws ws_layout(const TileGeom& g) {
    Bf16Ws L;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes, 256); return at; };
    L.packed = take((size_t)g.Bg * g.Hp * g.Wp * g.Cin * 16);
    L.utab = take((size_t)g.n_units * 4);
    L.part = take(g.direct ? 0 : (size_t)g.nsplit * g.ntiles * TB * TB * 4);
    L.spart = take((size_t)g.nsplit * g.nb * TB * 4);
    L.total = o;
    return L;
}

}  // namespace

size_t cov_bf16_workspace_bytes(const fw_conv_desc* d, fw_layout lay) {
    TileGeom g;
    if (!d || !make_tile_geom(d, lay, &g)) return 0;
    return ws_layout(g).total;
}

fw_status cov_bf16_accumulate(const void* X, fw_layout lay, const fw_conv_desc* d, float* A, float* s, void* ws, size_t ws_bytes,
                              hipStream_t st) {
    TileGeom g;
    if (!make_tile_geom(d, lay, &g)) return FW_ERR_UNSUPPORTED;
    const Bf16Ws L = ws_layout(g);
    if (!ws || ws_bytes < L.total) return FW_ERR_WORKSPACE;
    char* base = reinterpret_cast<char*>(ws);
    uint4* P = reinterpret_cast<uint4*>(base + L.packed);
    int* utab = reinterpret_cast<int*>(base + L.utab);
    float* part = reinterpret_cast<float*>(base + L.part);
    float* spart = reinterpret_cast<float*>(base + L.spart);
    const long long total = (long long)g.Bg * g.Hp * g.Wp * g.Cin;
    long long pb = (total + 255) / 256;
    if (pb > 65536) pb = 65536;
    hipLaunchKernelGGL(pack_images_kernel, dim3((unsigned)pb), dim3(256), 0, st, reinterpret_cast<const u16*>(X), g, P);
    hipLaunchKernelGGL(unit_table_kernel, dim3((g.n_units + 255) / 256), dim3(256), 0, st, g, utab);
    FW_LAUNCH_CHECK();
    hipLaunchKernelGGL(cov_bf16_tile_kernel, dim3(g.ntiles, g.nsplit), dim3(512), 0, st, P, utab, g, part, spart, A);
    FW_LAUNCH_CHECK();
    if (!g.direct) hipLaunchKernelGGL(tile_reduce_kernel, dim3(g.ntiles * 256), dim3(256), 0, st, g, part, A);
    hipLaunchKernelGGL(tile_reduce_sums_kernel, dim3((g.M + 63) / 64), dim3(256), 0, st, g, spart, s);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
