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
// The contraction kernel covers the lower triangle of A with tiles of 64 NRT rows x 64 NCT columns (4 >= NRT >= NCT >= 2;
// the host takes the shape and the number of unit ranges per tile that fill the 256 compute units best).  A workgroup
// of 4 wavefronts, one per SIMD, each with 32 NRT x 32 NCT outputs (NRT x NCT MFMA tiles in accumulation registers), owns
// one tile over a range of units.  Chunks of 4 units travel from global memory straight into LDS
// (global_load_lds_dwordx4, no register staging; wavefront w brings unit w) into a ring of five or six stages (all of
// the 160 KB of LDS) laid out as [unit][feature][16 B], four or five chunks ahead of the MFMAs: in flight is what
// covers the latency of the loads, which all workgroups of an XCD see at full length because they stream through
// the units in step.  A chunk costs one barrier; the loads of the chunk
// after next, and the fragment reads of the next 16-entry step, are issued one by one between the MFMAs of the
// current step, so that the matrix pipe stays busy while a single wavefront per SIMD does all the issuing.
// With one range per tile and the feature order kept, the result is added straight into A; otherwise partial
// tiles go to the workspace and are summed in float64 (and permuted to the caller's feature order).
#include "fw_internal.h"
#include <math.h>

namespace fw {
namespace {

constexpr int KU = 4;    // units per staged chunk (32 reduction entries) = wavefronts of a workgroup

struct TileGeom {
    int M, ntiles;
    int nrt, nct, tr, tc, ncb, nrb;  // MFMA row / column tiles per wavefront, tile = 64 nrt x 64 nct, column / row blocks of A
    int B, Bg, Cin, H, W, Hp, Wp, kh, kw, stride, pad, Ho, Wo;
    int layout;
    int n_units, nchunks, chunks_per_split, nsplit;
    int direct;   // one range per tile and external order == internal order: tiles are added straight into A
    int bg_chunks, bg_per_chunk;   // the pre-pass deals the image groups to this many thread groups
    int zero_off;                  // 16-byte element of P that is always zero (target of masked-off loads)
};

// column blocks of row block I that touch the lower triangle
__host__ __device__ inline int cols_of_row(int I, int tr, int tc, int ncb) {
    const int n = (I * tr + tr - 1) / tc + 1;
    return n < ncb ? n : ncb;
}

typedef unsigned short u16;

// ---- pre-pass: pack 8 images per 16 bytes, zero border; per-pixel sums for the column sums ----------------------
// One thread per (chunk of image groups, padded pixel, channel); it walks its image groups, so the sum it leaves in
// S8[chunk][yp][xp][c] has a fixed order of additions.
// The first row of workgroups also writes the unit table: offset (in 16-byte elements) of the top-left tap of every
// unit, -1 for the padding up to a whole number of chunks.
__global__ __launch_bounds__(256) void pack_images_kernel(const u16* __restrict__ X, TileGeom g, uint4* __restrict__ P,
                                                          float* __restrict__ S8, int* __restrict__ utab) {
    const int per_img = g.Hp * g.Wp * g.Cin;
    const int e = blockIdx.x * 256 + threadIdx.x;
    const int chunk = blockIdx.y;
    if (blockIdx.x == 0 && chunk == 0 && threadIdx.x < 16) P[g.zero_off + threadIdx.x] = make_uint4(0, 0, 0, 0);
    if (chunk == 0) {
        const int npos = g.Ho * g.Wo;
        for (int u = e; u < g.nchunks * KU; u += gridDim.x * 256) {
            int v = -1;
            if (u < g.n_units) {
                const int bg = u / npos, p = u - bg * npos;
                const int oy = p / g.Wo, ox = p - oy * g.Wo;
                v = ((bg * g.Hp + oy * g.stride) * g.Wp + ox * g.stride) * g.Cin;
            }
            utab[u] = v;
        }
    }
    if (e >= per_img) return;
    int c, xp, yp;
    if (g.layout == FW_LAYOUT_NCHW) {  // walk the source along x for coalescing; the packed order stays [yp][xp][c]
        xp = e % g.Wp; const int t = e / g.Wp;
        yp = t % g.Hp; c = t / g.Hp;
    } else {
        c = e % g.Cin; const int t = e / g.Cin;
        xp = t % g.Wp; yp = t / g.Wp;
    }
    // a padded pixel that no window touches (stride larger than the window) is neither read nor written
    if (g.stride > g.kh || g.stride > g.kw) {
        bool ry = false, rx = false;
        for (int ky = 0; ky < g.kh; ++ky) { const int o = yp - ky; ry |= o >= 0 && o % g.stride == 0 && o / g.stride < g.Ho; }
        for (int kx = 0; kx < g.kw; ++kx) { const int o = xp - kx; rx |= o >= 0 && o % g.stride == 0 && o / g.stride < g.Wo; }
        if (!(ry && rx)) return;
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

// internal feature (tap-major, channel-minor) -> offset inside a unit, external index m = (c*kh + ky)*kw + kx
// (or the internal index itself when the caller works in channels-last feature order)
__device__ __forceinline__ void feat_map(int fi, const TileGeom& g, int* off, int* ext) {
    const int t = fi / g.Cin, c = fi - t * g.Cin;
    const int ky = t / g.kw, kx = t - ky * g.kw;
    *off = (ky * g.Wp + kx) * g.Cin + c;
    *ext = g.layout == FW_LAYOUT_NHWC_KKC ? fi : c * (g.kh * g.kw) + t;
}

__device__ __forceinline__ void tile_coords(int tile, const TileGeom& g, int* I, int* J) {
    int i = 0;
    for (;;) {
        const int n = cols_of_row(i, g.tr, g.tc, g.ncb);
        if (tile < n) break;
        tile -= n; ++i;
    }
    *I = i; *J = tile;
}

template <int NRT, int NCT>
__global__ __launch_bounds__(256) void cov_bf16_tile_kernel(const uint4* __restrict__ P, const int* __restrict__ utab, TileGeom g,
                                                            float* __restrict__ part, float* __restrict__ A) {
    constexpr int TR = 64 * NRT;      // tile rows
    constexpr int TC = 64 * NCT;      // tile columns
    constexpr int NF = NRT + NCT;     // groups of 64 features per unit: NRT of the row panel, NCT of the column panel
    constexpr int ROW = TR + TC;      // 16-byte elements per unit
    constexpr int NM = NRT * NCT;     // MFMAs per 16-entry step and wavefront
    constexpr int NST = 160 * 1024 / (KU * ROW * 16);   // stages of the LDS ring: all of the 160 KB (5, 5, 6)
    __shared__ uint4 pan[NST][KU][ROW];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave >> 1, wj = wave & 1;
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
    int I, J;
    tile_coords(tile, g, &I, &J);

    // Staging: a wavefront-wide 16-byte load fills 64 consecutive features of one unit (1 KB of LDS); wavefront w
    // brings unit w of every chunk, NF loads.  Lanes whose feature lies beyond M, and units beyond the range, read the
    // zero element instead, so every stage is completely rewritten by every chunk.
    int off[NF];
    unsigned okmask = 0;
#pragma unroll
    for (int k = 0; k < NF; ++k) {
        const int f = k < NRT ? I * TR + 64 * k + lane : J * TC + 64 * (k - NRT) + lane;
        const bool ok = f < g.M;
        int ext_unused;
        feat_map(ok ? f : 0, g, &off[k], &ext_unused);
        okmask |= (ok ? 1u : 0u) << k;
    }

    floatx16 acc[NRT][NCT];
#pragma unroll
    for (int a = 0; a < NRT; ++a)
#pragma unroll
        for (int b = 0; b < NCT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    const int c_begin = split * g.chunks_per_split;
    const int nchunks = min(g.nchunks, c_begin + g.chunks_per_split) - c_begin;

    // offset of the unit this wavefront loads next (wavefront-uniform; -1 past the end of the range)
    int nb = -1;
    auto fetch_base = [&](int c) { nb = c < nchunks ? utab[(c_begin + c) * KU + wave] : -1; };
    auto dma_one = [&](int stage, int k) {   // k is a compile-time constant after unrolling
        const int idx = (nb >= 0 && ((okmask >> k) & 1u)) ? nb + off[k] : g.zero_off;
        dma16(P + idx, &pan[stage][wave][64 * k]);
    };
    auto issue = [&](int stage) {
#pragma unroll
        for (int k = 0; k < NF; ++k) dma_one(stage, k);
    };

    // Operand fragments of 16-entry step ks (units 2ks, 2ks+1) of a stage; fragment r < NRT is row tile r, the others
    // are the column tiles.  Two register sets alternate between the two steps of a chunk.
    bf16x8 fr[2][NF];
    auto read_one = [&](int stage, int ks, int set, int r) {
        const int col = r < NRT ? 32 * NRT * wi + 32 * r : TR + 32 * NCT * wj + 32 * (r - NRT);
        fr[set][r] = *reinterpret_cast<const bf16x8*>(&pan[stage][2 * ks + half][col + l32]);
    };
    auto mfma_one = [&](int set, int m) {   // m = ta * NCT + tb
        const int ta = m / NCT, tb = m % NCT;
        acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[set][ta], fr[set][NRT + tb], acc[ta][tb], 0, 0, 0);
    };

    // Ring protocol.  Loads of one wavefront complete in order, so "at most the loads of NST-2 chunks outstanding" means
    // the chunk before those has landed for this wavefront; the barrier extends that to all wavefronts.  The
    // barrier sits in the middle of a chunk: by then every wavefront has its last fragments of chunk c in registers
    // (lgkmcnt 0), so the stage of chunk c is free for the loads of chunk c+NST, and chunk c+1 is ready to be read while
    // the second step of chunk c is still being multiplied.  Every iteration issues the same number of loads (past the
    // end they fetch the zero element), which keeps the outstanding-load arithmetic valid in the tail.
#pragma unroll
    for (int i = 0; i < NST - 1; ++i) { fetch_base(i); issue(i); }
    fetch_base(NST - 1);
    FW_WAIT_VM((NST - 2) * NF);
    __builtin_amdgcn_s_barrier();
    FW_COMPILER_FENCE();
    issue(NST - 1);
#pragma unroll
    for (int r = 0; r < NF; ++r) read_one(0, 0, 0, r);
    int sc = 0;   // stage of chunk c
    for (int c = 0; c < nchunks; ++c) {
        const int sn = sc == NST - 1 ? 0 : sc + 1;
        fetch_base(c + NST);
        // step 0 of chunk c; the fragment reads of step 1 go out between its first MFMAs, so that they have returned
        // by the time the last one is issued
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            if (m < NF) read_one(sc, 1, 1, m);
            mfma_one(0, m);
            __builtin_amdgcn_sched_barrier(0);
        }
        FW_WAIT_LGKM0();
        FW_WAIT_VM((NST - 2) * NF);
        __builtin_amdgcn_s_barrier();
        FW_COMPILER_FENCE();
        // step 1 of chunk c; first the fragment reads of step 0 of chunk c+1, then the loads of chunk c+NST, one
        // between every two MFMAs
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            if (m < NF) read_one(sn, 0, 0, m);
            else if (m - NF < NF) dma_one(sc, m - NF);
            mfma_one(1, m);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int k = NM - NF; k < NF; ++k) dma_one(sc, k);   // loads that did not fit between the MFMAs
        sc = sn;
    }
    FW_WAIT_VM(0);
    FW_WAIT_LGKM0();
    __syncthreads();

    // ---- epilogue
    if (!g.direct) {
        float* dst = part + ((size_t)split * g.ntiles + tile) * (TR * TC);
#pragma unroll
        for (int ta = 0; ta < NRT; ++ta)
#pragma unroll
            for (int tb = 0; tb < NCT; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = 32 * NRT * wi + 32 * ta + 8 * (i >> 2) + 4 * half + (i & 3);
                    const int col = 32 * NCT * wj + 32 * tb + l32;
                    dst[row * TC + col] = acc[ta][tb][i];
                }
    } else {
        // one range per tile, feature order kept: add into the lower triangle of A, 32 lanes along a row, the 16 loads of
        // an MFMA tile in flight together
#pragma unroll
        for (int tb = 0; tb < NCT; ++tb) {
            const int gj = J * TC + 32 * NCT * wj + 32 * tb + l32;
#pragma unroll
            for (int ta = 0; ta < NRT; ++ta) {
                const int gi0 = I * TR + 32 * NRT * wi + 32 * ta + 4 * half;
                if (gi0 + 27 < J * TC + 32 * NCT * wj + 32 * tb) continue;   // MFMA tile entirely above the diagonal
                float old[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int gi = gi0 + 8 * (i >> 2) + (i & 3);
                    old[i] = (gi < g.M && gj < g.M && gj <= gi) ? A[(size_t)gi * g.M + gj] : 0.f;
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int gi = gi0 + 8 * (i >> 2) + (i & 3);
                    if (gi < g.M && gj < g.M && gj <= gi) A[(size_t)gi * g.M + gj] = old[i] + acc[ta][tb][i];
                }
            }
        }
    }
}

// s[m] += sum over the output positions of the per-pixel sums under the tap of feature m: 16 features per workgroup
// of 1024 threads, 64 lanes per feature over (position, image-group chunk), four loads in flight, float64
__global__ __launch_bounds__(1024) void column_sums_kernel(TileGeom g, const float* __restrict__ S8, float* __restrict__ s) {
    __shared__ double red[64][16];
    const int fl = threadIdx.x & 15, pl = threadIdx.x >> 4;
    const int fi = blockIdx.x * 16 + fl;
    const bool ok = fi < g.M;
    int off = 0, ext = 0;
    if (ok) feat_map(fi, g, &off, &ext);
    const int per_img = g.Hp * g.Wp * g.Cin;
    const int npos = g.Ho * g.Wo;
    const int total = npos * g.bg_chunks;
    auto at = [&](int idx) {
        const int k = idx / npos, p = idx - k * npos;
        const int oy = p / g.Wo, ox = p - oy * g.Wo;
        return S8[(size_t)k * per_img + ((oy * g.stride) * g.Wp + ox * g.stride) * g.Cin + off];
    };
    double v = 0.0;
    if (ok) {
        int idx = pl;
        for (; idx + 192 < total; idx += 256) {
            const float x0 = at(idx), x1 = at(idx + 64), x2 = at(idx + 128), x3 = at(idx + 192);
            v += ((double)x0 + (double)x1) + ((double)x2 + (double)x3);
        }
        for (; idx < total; idx += 64) v += (double)at(idx);
    }
    red[pl][fl] = v;
    __syncthreads();
    if (pl == 0 && ok) {
        double t = 0.0;
#pragma unroll 8
        for (int q = 0; q < 64; ++q) t += red[q][fl];
        s[ext] = (float)((double)s[ext] + t);
    }
}

// partial tiles -> A (float64 sum over the ranges), one thread per tile element
__global__ __launch_bounds__(256) void tile_reduce_kernel(TileGeom g, const float* __restrict__ part, float* __restrict__ A) {
    const int bpt = g.tr * g.tc / 256;             // blocks of 256 threads per tile of tr x tc
    const int tile = blockIdx.x / bpt;
    const int e = (blockIdx.x - tile * bpt) * 256 + threadIdx.x;
    int I, J;
    tile_coords(tile, g, &I, &J);
    const int row = e / g.tc, col = e - row * g.tc;
    const int fi = I * g.tr + row, fj = J * g.tc + col;
    if (fi >= g.M || fj >= g.M || fj > fi) return;
    const size_t tsz = (size_t)g.tr * g.tc;
    const size_t stride = (size_t)g.ntiles * tsz;
    const float* src = part + (size_t)tile * tsz + e;
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
    if (M <= 0 || M > 16384 || n_units <= 0 || n_units >= (1ll << 31) - KU || packed + 16 >= (1ll << 31)) return false;
    if ((long long)d->B * d->Cin * d->H * d->W >= (1ll << 31)) return false;
    g->M = (int)M;
    g->n_units = (int)n_units;
    g->nchunks = (int)((n_units + KU - 1) / KU);
    const bool ident = lay == FW_LAYOUT_NHWC_KKC || lay == FW_LAYOUT_ROWS || d->kh * d->kw == 1;
    // Tile shape (64 nrt x 64 nct, nct <= nrt) and number of unit ranges per tile: minimise
    //   rounds x chunks per range x time of a chunk  +  traffic of the partial tiles,
    // with rounds = ceil(tiles x ranges / 256 compute units).  A chunk costs the larger of its MFMAs (2 steps x nrt nct
    // x 32 cycles, plus a share for the barrier) and its loads into LDS, which a compute unit sustains at about 23 bytes
    // per cycle next to the fragment reads; one range per tile in the caller's feature order needs no partial tiles.
    const double clk = 2.0e9, bw = 4.0e12, lds_load_rate = 23.0;
    double best = 1e300;
    int best_nrt = 4, best_nct = 4, best_ns = 1;
    for (int nrt = 4; nrt >= 2; --nrt)
        for (int nct = nrt; nct >= 2; --nct) {
            const int tr = 64 * nrt, tc = 64 * nct, ncb = (int)((M + tc - 1) / tc), nrb = (int)((M + tr - 1) / tr);
            long long ntiles = 0;
            for (int I = 0; I < nrb; ++I) ntiles += cols_of_row(I, tr, tc, ncb);
            const double t_mfma = 64.0 * nrt * nct + 150.0, t_load = (double)(tr + tc) * KU * 16.0 / lds_load_rate;
            const double t_chunk = (t_mfma > t_load ? t_mfma : t_load) / clk;
            for (int ns = 1; ns <= 512 && ns <= g->nchunks; ++ns) {
                const long long wgs = ntiles * ns;
                const long long rounds = (wgs + 255) / 256;
                const long long cps = (g->nchunks + ns - 1) / ns;
                double cost = (double)rounds * (double)cps * t_chunk;
                if (ns > 1 || !ident) cost += (double)wgs * tr * tc * 4.0 * 2.0 / bw;
                if (cost < best * 0.999) { best = cost; best_nrt = nrt; best_nct = nct; best_ns = ns; }
            }
        }
    g->nrt = best_nrt; g->nct = best_nct; g->tr = 64 * best_nrt; g->tc = 64 * best_nct;
    g->ncb = (int)((M + g->tc - 1) / g->tc); g->nrb = (int)((M + g->tr - 1) / g->tr);
    g->ntiles = 0;
    for (int I = 0; I < g->nrb; ++I) g->ntiles += cols_of_row(I, g->tr, g->tc, g->ncb);
    g->chunks_per_split = (g->nchunks + best_ns - 1) / best_ns;
    g->nsplit = (g->nchunks + g->chunks_per_split - 1) / g->chunks_per_split;
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
    g->direct = (g->nsplit == 1 && ident) ? 1 : 0;
    return true;
}

struct Bf16Ws { size_t packed, utab, part, s8, total; };
Bf16Ws ws_layout(const TileGeom& g) {
    Bf16Ws L;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes, 256); return at; };
    L.packed = take(((size_t)g.Bg * g.Hp * g.Wp * g.Cin + 16) * 16);
    L.utab = take((size_t)g.nchunks * KU * 4);
    L.part = take(g.direct ? 0 : (size_t)g.nsplit * g.ntiles * g.tr * g.tc * 4);
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
                       g, P, S8, utab);
    FW_LAUNCH_CHECK();
    const dim3 grid((g.ntiles * g.nsplit + 7) / 8 * 8);
#define FW_TILE_LAUNCH(R, C) hipLaunchKernelGGL((cov_bf16_tile_kernel<R, C>), grid, dim3(256), 0, st, P, utab, g, part, A)
    switch (g.nrt * 10 + g.nct) {
        case 44: FW_TILE_LAUNCH(4, 4); break;
        case 43: FW_TILE_LAUNCH(4, 3); break;
        case 42: FW_TILE_LAUNCH(4, 2); break;
        case 33: FW_TILE_LAUNCH(3, 3); break;
        case 32: FW_TILE_LAUNCH(3, 2); break;
        default: FW_TILE_LAUNCH(2, 2); break;
    }
#undef FW_TILE_LAUNCH
    FW_LAUNCH_CHECK();
    if (!g.direct) hipLaunchKernelGGL(tile_reduce_kernel, dim3(g.ntiles * (g.tr * g.tc / 256)), dim3(256), 0, st, g, part, A);
    hipLaunchKernelGGL(column_sums_kernel, dim3((g.M + 15) / 16), dim3(1024), 0, st, g, S8, s);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
