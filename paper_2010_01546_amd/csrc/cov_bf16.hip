// bfloat16 moment accumulation A += X^T X, s += X^T 1 (sums inside eqs. (vmuxi), (vPhixi), (phixmi)) on the gfx950
// matrix cores.
//
// v_mfma_f32_32x32x16_bf16 wants, per lane, eight consecutive entries of the reduction index for one feature.
// The reduction index of X^T X is the patch row (image, oy, ox); any order of it gives the same sums, so the
// eight entries of a lane are taken from EIGHT IMAGES at one output position.  A bandwidth-bound pre-pass packs
// the activation tensor into
//     P[image group][y + pad][x + pad][channel] -> 8 x bf16 (16 bytes: the same pixel and channel of 8 images)
// with a zero border of `pad` pixels, so that every tap of every output position is one aligned 16-byte load with
// no bounds test, for any window, stride and input layout.  A "unit" is (image group, oy, ox); an MFMA consumes two.
// The same pass adds up, per padded pixel and channel, the values it packs; the column sums s are sums of those
// per-pixel sums over the output positions of a tap, so the contraction kernel does not touch them.
//
// The contraction kernel cuts the lower triangle of A into 256x256 tiles.  A workgroup of 8 wavefronts (2 x 4, each
// 128x64 = 4x2 MFMA tiles) owns one tile over a range of units.  Panels of 4 units travel from global memory
// straight into LDS (global_load_lds_dwordx4, no register staging) into a ring of four stages laid out as
// [unit][feature][16 B], three chunks ahead of the MFMAs; a chunk costs one s_waitcnt and one barrier, and the
// operand fragments of every group of eight MFMAs are read from LDS while the previous group executes.
// With one range per tile and the feature order kept, the result is added straight into A; otherwise partial
// tiles go to the workspace and are summed in float64 (and permuted to the caller's feature order).
#include "fw_internal.h"
#include <math.h>

namespace fw {
namespace {

constexpr int TB = 256;  // tile edge (features)
constexpr int KU = 4;    // units per staged chunk (32 reduction entries)
constexpr int NST = 4;   // stages of the LDS ring

struct TileGeom {
    int M, nb, ntiles;
    int B, Bg, Cin, H, W, Hp, Wp, kh, kw, stride, pad, Ho, Wo;
    int layout;
    int n_units, units_per_split, nsplit;
    int direct;   // one range per tile and external order == internal order: tiles are added straight into A
    int bg_chunks, bg_per_chunk;   // the pre-pass deals the image groups to this many thread groups
    int zero_off;                  // 16-byte element of P that is always zero (target of masked-off loads)
};

typedef unsigned short u16;

// ---- pre-pass: pack 8 images per 16 bytes, zero border; per-pixel sums for the column sums ----------------------
// One thread per (chunk of image groups, padded pixel, channel); it walks its image groups, so the sum it leaves in
// S8[chunk][yp][xp][c] has a fixed order of additions.
__global__ __launch_bounds__(256) void pack_images_kernel(const u16* __restrict__ X, TileGeom g, uint4* __restrict__ P,
                                                          float* __restrict__ S8) {
    const int per_img = g.Hp * g.Wp * g.Cin;
    const int e = blockIdx.x * 256 + threadIdx.x;
    const int chunk = blockIdx.y;
    if (blockIdx.x == 0 && chunk == 0 && threadIdx.x < 16) P[g.zero_off + threadIdx.x] = make_uint4(0, 0, 0, 0);
    if (e >= per_img) return;
    int c, xp, yp;
    if (g.layout == FW_LAYOUT_NCHW) {  // walk the source along x for coalescing; the packed order stays [yp][xp][c]
        xp = e % g.Wp; const int t = e / g.Wp;
        yp = t % g.Hp; c = t / g.Hp;
    } else {
        c = e % g.Cin; const int t = e / g.Cin;
        xp = t % g.Wp; yp = t / g.Wp;
    }
    const int y = yp - g.pad, x = xp - g.pad;
    const bool inside = (unsigned)y < (unsigned)g.H && (unsigned)x < (unsigned)g.W;
    const long long img_stride = (long long)g.Cin * g.H * g.W;
    const long long src0 = g.layout == FW_LAYOUT_NCHW ? ((long long)c * g.H + y) * g.W + x : ((long long)y * g.W + x) * g.Cin + c;
    const int dst0 = (yp * g.Wp + xp) * g.Cin + c;
    const int bg0 = chunk * g.bg_per_chunk, bg1 = min(g.Bg, bg0 + g.bg_per_chunk);
    float acc = 0.f;
    for (int bg = bg0; bg < bg1; ++bg) {
        unsigned v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int b = bg * 8 + i;
            v[i] = (inside && b < g.B) ? X[(long long)b * img_stride + src0] : 0u;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) acc += __uint_as_float(v[i] << 16);
        uint4 o;
        o.x = v[0] | (v[1] << 16); o.y = v[2] | (v[3] << 16); o.z = v[4] | (v[5] << 16); o.w = v[6] | (v[7] << 16);
        P[(long long)bg * per_img + dst0] = o;
    }
    S8[(size_t)chunk * per_img + dst0] = acc;
}

// s[m] += sum over the output positions of the per-pixel sums under tap (ky,kx): one workgroup per feature
__global__ __launch_bounds__(256) void column_sums_kernel(TileGeom g, const float* __restrict__ S8, float* __restrict__ s);

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

struct SmemTile {
    alignas(16) uint4 pan[NST][2][KU][TB];  // [stage][row panel / column panel][unit][feature], 128 KB
};

// s_waitcnt vmcnt(n) with the other counters left alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
#define FW_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)
// the same, and lgkmcnt(0): LDS reads of this wavefront have returned as well
#define FW_WAIT_VM_LGKM0(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0070)

__global__ __launch_bounds__(512) void cov_bf16_tile_kernel(const uint4* __restrict__ P, const int* __restrict__ utab, TileGeom g,
                                                            float* __restrict__ part, float* __restrict__ A) {
    __shared__ SmemTile sm;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave >> 2, wj = wave & 3;
    const int half = lane >> 5, l32 = lane & 31;
    // Workgroups are handed to the 8 XCDs round-robin by their linear index.  Re-index so that each XCD works on a
    // contiguous run of (range, tile) pairs: neighbours in that run share the unit range and mostly the row panel, which
    // keeps what one XCD pulls into its own L2 small.
    const int total = g.ntiles * g.nsplit;
    const int per_xcd = (total + 7) / 8;
    int tile, split;
    {
        const int w = blockIdx.x;
        const int n = (w & 7) * per_xcd + (w >> 3);
        if (n >= total || (w >> 3) >= per_xcd) return;   // padding of the last run
        split = n / g.ntiles;
        tile = n - split * g.ntiles;
    }
    int I = (int)((sqrtf(8.f * tile + 1.f) - 1.f) * 0.5f);
    while ((I + 1) * (I + 2) / 2 <= tile) ++I;
    while (I * (I + 1) / 2 > tile) --I;
    const int J = tile - I * (I + 1) / 2;
    const bool diag = I == J;

    // Staging: a wavefront-wide 16-byte load fills 64 consecutive features of one unit of one panel (1 KB of LDS).
    // Wavefront w always takes feature quarter w & 3; its loads of a chunk are (panel, unit) = (0, g2), (0, g2 + 2),
    // (1, g2), (1, g2 + 2) with g2 = w >> 2.  Lanes whose feature lies beyond M, and units beyond the range, read
    // the zero element instead, so every stage is completely rewritten by every chunk.
    const int q = wave & 3, g2 = wave >> 2;
    int off[2], ext_unused;
    bool ok[2];
    {
        const int fA = I * TB + 64 * q + lane, fB = J * TB + 64 * q + lane;
        ok[0] = fA < g.M; ok[1] = fB < g.M;
        feat_map(ok[0] ? fA : 0, g, &off[0], &ext_unused);
        feat_map(ok[1] ? fB : 0, g, &off[1], &ext_unused);
    }

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
    const int npanels = diag ? 1 : 2;

    // unit offsets of the chunk whose loads are issued next (wavefront-uniform, fetched one iteration early)
    int nbase[2];
    auto fetch_bases = [&](int c) {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int uu = u_begin + c * KU + g2 + 2 * k;
            nbase[k] = (c < nchunks && uu < u_end) ? utab[uu] : -1;
        }
    };
    auto issue = [&](int c) {
        const int stage = c & (NST - 1);
#pragma unroll
        for (int pnl = 0; pnl < 2; ++pnl) {
            if (pnl >= npanels) break;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int u = g2 + 2 * k;
                const int idx = (nbase[k] >= 0 && ok[pnl]) ? nbase[k] + off[pnl] : g.zero_off;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(P + idx),
                                                 (__attribute__((address_space(3))) void*)(&sm.pan[stage][pnl][u][64 * q]), 16, 0, 0);
            }
        }
        fetch_bases(c + 1);
    };

    const int pj = diag ? 0 : 1;
    // Operand fragments of k-step ks (units 2ks, 2ks+1) of chunk c; two register sets alternate so that the reads
    // for the next group of MFMAs are always issued before the current group.
    bf16x8 fa[2][4], fb[2][2];
    auto read_frags = [&](int c, int ks, int set) {
        const int stage = c & (NST - 1);
        const int unit = 2 * ks + half;
#pragma unroll
        for (int t = 0; t < 4; ++t) fa[set][t] = *reinterpret_cast<const bf16x8*>(&sm.pan[stage][0][unit][128 * wi + 32 * t + l32]);
#pragma unroll
        for (int t = 0; t < 2; ++t) fb[set][t] = *reinterpret_cast<const bf16x8*>(&sm.pan[stage][pj][unit][64 * wj + 32 * t + l32]);
    };
    auto mfma_group = [&](int set) {
#pragma unroll
        for (int ta = 0; ta < 4; ++ta)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][ta], fb[set][tb], acc[ta][tb], 0, 0, 0);
    };
    static_assert(KU == 4 && NST == 4, "the loop below is written for two k-steps per chunk and a ring of four");

    // Ring protocol.  Loads of one wavefront complete in order, so "at most the loads of two chunks outstanding" means
    // the chunk before those two has landed for this wavefront; the barrier extends that to all wavefronts.  The
    // barrier sits in the middle of a chunk: by then every wavefront has its last fragments of chunk c in registers
    // (lgkmcnt 0), so the stage of chunk c is free for the loads of chunk c+4, and chunk c+1 is ready to be read while
    // the second half of chunk c is still being multiplied.  Every iteration issues the same number of loads (past the
    // end they fetch the zero element), which keeps the outstanding-load arithmetic valid in the tail.
    // The barrier is the bare instruction: __syncthreads() would first drain every outstanding load, which is exactly
    // what the ring is there to avoid.
    fetch_bases(0);
    issue(0); issue(1); issue(2);
    if (diag) FW_WAIT_VMCNT(4); else FW_WAIT_VMCNT(8);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue(3);
    read_frags(0, 0, 0);
    for (int c = 0; c < nchunks; ++c) {
        read_frags(c, 1, 1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_group(0);
        __builtin_amdgcn_sched_barrier(0);
        if (diag) FW_WAIT_VM_LGKM0(4); else FW_WAIT_VM_LGKM0(8);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue(c + 4);
        read_frags(c + 1, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma_group(1);
        __builtin_amdgcn_sched_barrier(0);
    }
    FW_WAIT_VMCNT(0);
    __syncthreads();

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
}

__global__ __launch_bounds__(256) void column_sums_kernel(TileGeom g, const float* __restrict__ S8, float* __restrict__ s) {
    __shared__ double red[4];
    const int fi = blockIdx.x;
    int off, ext;
    feat_map(fi, g, &off, &ext);
    const int per_img = g.Hp * g.Wp * g.Cin;
    const int npos = g.Ho * g.Wo;
    double v = 0.0;
    for (int k = 0; k < g.bg_chunks; ++k)
        for (int p = threadIdx.x; p < npos; p += 256) {
            const int oy = p / g.Wo, ox = p - oy * g.Wo;
            v += (double)S8[(size_t)k * per_img + ((oy * g.stride) * g.Wp + ox * g.stride) * g.Cin + off];
        }
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) s[ext] = (float)((double)s[ext] + red[0] + red[1] + red[2] + red[3]);
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
    if (M <= 0 || M > 16384 || n_units <= 0 || n_units >= (1ll << 31) || packed + 16 >= (1ll << 31)) return false;
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
    if (best_ns > nchunks) best_ns = (int)nchunks;
    const long long cps = (nchunks + best_ns - 1) / best_ns;
    g->units_per_split = (int)(cps * KU);
    g->nsplit = (int)((n_units + g->units_per_split - 1) / g->units_per_split);
    // the pre-pass wants about half a million threads: split the image groups when one image gives fewer
    {
        const long long per_img = (long long)g->Hp * g->Wp * d->Cin;
        long long ch = (524288 + per_img - 1) / per_img;
        if (ch > g->Bg) ch = g->Bg;
        if (ch < 1) ch = 1;
        g->bg_per_chunk = (int)((g->Bg + ch - 1) / ch);
        g->bg_chunks = (g->Bg + g->bg_per_chunk - 1) / g->bg_per_chunk;
        g->zero_off = (int)packed;
    }
    const bool ident = lay == FW_LAYOUT_NHWC_KKC || lay == FW_LAYOUT_ROWS || d->kh * d->kw == 1;
    g->direct = (g->nsplit == 1 && ident) ? 1 : 0;
    return true;
}

struct Bf16Ws { size_t packed, utab, part, s8, total; };
Bf16Ws ws_layout(const TileGeom& g) {
    Bf16Ws L;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes, 256); return at; };
    L.packed = take(((size_t)g.Bg * g.Hp * g.Wp * g.Cin + 16) * 16);
    L.utab = take((size_t)g.n_units * 4);
    L.part = take(g.direct ? 0 : (size_t)g.nsplit * g.ntiles * TB * TB * 4);
    L.s8 = take((size_t)g.bg_chunks * g.Hp * g.Wp * g.Cin * 4);
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
    float* S8 = reinterpret_cast<float*>(base + L.s8);
    const int per_img = g.Hp * g.Wp * g.Cin;
    hipLaunchKernelGGL(pack_images_kernel, dim3((per_img + 255) / 256, g.bg_chunks), dim3(256), 0, st, reinterpret_cast<const u16*>(X),
                       g, P, S8);
    hipLaunchKernelGGL(unit_table_kernel, dim3((g.n_units + 255) / 256), dim3(256), 0, st, g, utab);
    FW_LAUNCH_CHECK();
    const int per_xcd = (g.ntiles * g.nsplit + 7) / 8;
    hipLaunchKernelGGL(cov_bf16_tile_kernel, dim3(per_xcd * 8), dim3(512), 0, st, P, utab, g, part, A);
    FW_LAUNCH_CHECK();
    if (!g.direct) hipLaunchKernelGGL(tile_reduce_kernel, dim3(g.ntiles * 256), dim3(256), 0, st, g, part, A);
    hipLaunchKernelGGL(column_sums_kernel, dim3(g.M), dim3(256), 0, st, g, S8, s);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
