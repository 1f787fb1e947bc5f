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
//
// Stride-1 windows take the shift-correlation form instead (same sums, see cov_shift.hip for the derivation): the same
// kernel runs on a rectangular grid of tiles whose rows are the channels of a pixel and whose columns are (tap
// difference, channel) of the pixel shifted back by that difference; units are pixels listed region by region, ranges
// never cross a region, and an assembly kernel adds, per pair of taps, the partial tiles of the regions that serve the
// row tap.  Up to 128 channels a unit is a pair of horizontally neighbouring pixels (2 Cin "channels"), which fills the
// row tiles and halves the units.
#include "fw_internal.h"
#include <math.h>
#include <string.h>
#include <algorithm>
#include <queue>
#include <type_traits>
#include <vector>

namespace fw {
namespace {

constexpr int KU = 4;    // units per staged chunk (32 reduction entries) = wavefronts of a workgroup

constexpr int MAXREG = 32;

// region of the image whose pixels serve the same set of taps (shift-correlation mode, see below)
struct TileRegion {
    int y0, x0, rh, rw;          // rectangle of pixels
    int rowmask, colmask;        // bit ty / tx: its pixels serve taps of row ty / column tx
    int colmask2;                // pixel pairs (gx = 2): the column taps served by the odd pixel of a pair
    int chunk_begin, nchunks;    // its units in the unit table, padded to whole chunks
    int split_begin, nsplit;     // its unit ranges
    unsigned dmask[4];           // bit di: some pair of taps (t1 >= t2, t1 served by this region) has the difference di
};

// does column tile J (features J*tc .. J*tc + tc - 1 of the nd*Cin shifted features) hold a difference the region uses?
__host__ __device__ inline bool region_needs_tile(const TileRegion& R, int J, int tc, int Cin, int nd) {
    const int d0 = (J * tc) / Cin;
    int d1 = (J * tc + tc - 1) / Cin;
    if (d1 > nd - 1) d1 = nd - 1;
    for (int di = d0; di <= d1; ++di)
        if ((R.dmask[di >> 5] >> (di & 31)) & 1u) return true;
    return false;
}

// everything about a layer's launch geometry except the regions (kernels that do not need those take this part only:
// a kernel argument of 2 KB makes a launch noticeably slower on the host)
struct TileCore {
    int M, ntiles;
    int nrt, nct, tr, tc, ncb, nrb;  // MFMA row / column tiles per wavefront, tile = 64 nrt x 64 nct, column / row blocks of A
    int B, Bg, Cin, H, W, Hp, Wp, kh, kw, stride, pad, Ho, Wo;
    int layout;
    int n_units, nchunks, chunks_per_split, nsplit;
    int direct;   // one range per tile and external order == internal order: tiles are added straight into A
    int bg_chunks, bg_per_chunk;   // the pre-pass deals the image groups to this many thread groups
    int zero_off;                  // 16-byte element of P that is always zero (target of masked-off loads)
    int py, px;                    // zero rows above / columns left of the image in P (Hp, Wp count the border on all sides)
    int sum_shift;                 // offset of the tap (0,0) of output position (0,0) in P
    // shift-correlation mode (stride-1 windows): rows = Cin channels of a pixel, columns = nd tap differences x Cin
    int shift, nd, F, nreg;
    int spread;                  // shift mode: how workgroups map to (tile, range), see the tile kernel
    // Few channels (Cin <= 128): a unit of the shift mode is a PAIR of horizontally neighbouring pixels, i.e. the image is
    // read as W/2 pixels of 2 Cin channels (the packed layout is the same memory either way).  Row features: both pixels'
    // channels (a full 128-row tile); kept differences: those of a window half as wide, (dy, e) with e counted in pairs.
    // A product of pixel 2X+a with pixel 2X+a-dx of the original differences is the entry (a, c1) x (a', c2) of the pair
    // difference e = -floor((a - dx) / 2), a' = (a - dx) mod 2.
    int gx;                      // pixels per unit along x: 1 or 2
    int t_cin, t_wp, t_kw;       // the contraction's view: channels per unit, units per packed row, width of the difference window
};
struct TileGeom : TileCore {
    TileRegion reg[MAXREG];
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
// SPLIT: the source is a float32 tensor with g.Cin / 2 channels; packed channel c < Cin / 2 takes hi = bf16(x) of source
// channel c, packed channel Cin / 2 + c takes lo = bf16(x - hi) (the split form of float32 moments, see cov.hip).
template <bool SHIFT, bool SPLIT>
__global__ __launch_bounds__(256) void pack_images_kernel(const void* __restrict__ Xv, std::conditional_t<SHIFT, TileGeom, TileCore> g,
                                                          uint4* __restrict__ P,
                                                          float* __restrict__ S8, int* __restrict__ utab) {
    const u16* __restrict__ X = reinterpret_cast<const u16*>(Xv);
    const float* __restrict__ Xf = reinterpret_cast<const float*>(Xv);
    const int per_img = g.Hp * g.Wp * g.Cin;
    const int e = blockIdx.x * 256 + threadIdx.x;
    const int chunk = blockIdx.y;
    if (blockIdx.x == 0 && chunk == 0 && threadIdx.x < 16) P[g.zero_off + threadIdx.x] = make_uint4(0, 0, 0, 0);
    if (chunk == 0 && !SHIFT) {
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
    if constexpr (SHIFT) if (chunk == 0) {
        // units are pixels (of an image group), listed region by region, every region padded to whole chunks
        for (int u = e; u < g.nchunks * KU; u += gridDim.x * 256) {
            int ri = 0;
            for (int r = 0; r < g.nreg; ++r)
                if (u >= g.reg[r].chunk_begin * KU) ri = r;
            const int l = u - g.reg[ri].chunk_begin * KU;
            const int area = g.reg[ri].rh * g.reg[ri].rw;
            int v = -1;
            if (l < g.Bg * area) {
                const int bg = l / area, p = l - bg * area;
                const int yy = p / g.reg[ri].rw, xx = p - yy * g.reg[ri].rw;
                v = ((bg * g.Hp + g.reg[ri].y0 + yy + g.py) * g.Wp + g.gx * (g.reg[ri].x0 + xx) + g.px) * g.Cin;
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
    const int y = yp - g.py, x = xp - g.px;
    const bool inside = (unsigned)y < (unsigned)g.H && (unsigned)x < (unsigned)g.W;
    const int Csrc = SPLIT ? g.Cin >> 1 : g.Cin;            // channels of the source tensor
    const int csrc = SPLIT ? (c >= Csrc ? c - Csrc : c) : c;
    const bool lo_plane = SPLIT && c >= Csrc;
    const long long img_stride = (long long)Csrc * g.H * g.W;
    const long long src0 = g.layout == FW_LAYOUT_NCHW ? ((long long)csrc * g.H + y) * g.W + x : ((long long)y * g.W + x) * Csrc + csrc;
    const int dst0 = (yp * g.Wp + xp) * g.Cin + c;
    const int bg0 = chunk * g.bg_per_chunk, bg1 = min(g.Bg, bg0 + g.bg_per_chunk);
    float acc = 0.f;
    for (int bg = bg0; bg < bg1; ++bg) {
        // eight loads in flight: issued unconditionally (a masked one reads element 0) and masked afterwards; the empty
        // asm statement keeps the compiler from moving them into branches, where each would be waited for on the spot
        unsigned v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int b = bg * 8 + i;
            const long long idx = (inside && b < g.B) ? (long long)b * img_stride + src0 : 0;
            if constexpr (SPLIT) v[i] = __float_as_uint(Xf[idx]);
            else v[i] = X[idx];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            asm volatile("" : "+v"(v[i]));
            if (!(inside && bg * 8 + i < g.B)) v[i] = 0u;
            if constexpr (SPLIT) {
                const float xf = __uint_as_float(v[i]);
                const unsigned short h = f32_to_bf16_rne(xf);
                v[i] = lo_plane ? (unsigned)f32_to_bf16_rne(xf - bf16_to_f32(h)) : (unsigned)h;   // the difference is exact
            }
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
__device__ __forceinline__ void feat_map(int fi, const TileCore& g, int* off, int* ext) {
    const int t = fi / g.Cin, c = fi - t * g.Cin;
    const int ky = t / g.kw, kx = t - ky * g.kw;
    *off = (ky * g.Wp + kx) * g.Cin + c;
    *ext = g.layout == FW_LAYOUT_NHWC_KKC ? fi : c * (g.kh * g.kw) + t;
}

__device__ __forceinline__ void tile_coords(int tile, const TileCore& g, int* I, int* J) {
    int i = 0;
    for (;;) {
        const int n = cols_of_row(i, g.tr, g.tc, g.ncb);
        if (tile < n) break;
        tile -= n; ++i;
    }
    *I = i; *J = tile;
}

template <int NRT, int NCT, bool SHIFT>
__global__ __launch_bounds__(256) void cov_bf16_tile_kernel(const uint4* __restrict__ P, const int* __restrict__ utab,
                                                            std::conditional_t<SHIFT, TileGeom, TileCore> g,
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
    int I, J, c_begin, nchunks;
    if constexpr (!SHIFT) {
        const int w = blockIdx.x;
        const int n = (w & 7) * per_xcd + (w >> 3);
        if (n >= total || (w >> 3) >= per_xcd) return;   // padding of the last run
        split = n / g.ntiles;
        tile = n - split * g.ntiles;
        tile_coords(tile, g, &I, &J);
        c_begin = split * g.chunks_per_split;
        nchunks = min(g.nchunks, c_begin + g.chunks_per_split) - c_begin;
    } else {
        // shift-correlation mode: rectangular grid of tiles; the ranges differ in length (they never cross a region).
        // Many ranges: XCD x takes the ranges x, x + 8, ... with all their tiles (each XCD reads its own units only).
        // Few ranges cannot be dealt evenly to 8 XCDs: then the tiles of every range are spread over the XCDs (workgroup
        // index = range-major, tile-minor; every XCD reads all units, which are few in that case).
        const int w = blockIdx.x;
        if (g.spread) {
            split = w / g.ntiles;
            tile = w - split * g.ntiles;
        } else {
            tile = (w >> 3) % g.ntiles;
            split = (w & 7) + 8 * ((w >> 3) / g.ntiles);
        }
        if (split >= g.nsplit) return;
        I = tile / g.ncb;
        J = tile - I * g.ncb;
        int ri = 0;
        for (int r = 0; r < g.nreg; ++r)
            if (split >= g.reg[r].split_begin) ri = r;
        const int first = (split - g.reg[ri].split_begin) * g.chunks_per_split;
        c_begin = g.reg[ri].chunk_begin + first;
        nchunks = min(g.chunks_per_split, g.reg[ri].nchunks - first);
        // a border region serves few taps, and so only some of the differences: its other tiles are never read
        if (!region_needs_tile(g.reg[ri], J, g.tc, g.t_cin, g.nd)) return;
    }
    // all of these are the same for the whole workgroup: keep them in scalar registers
    tile = __builtin_amdgcn_readfirstlane(tile); split = __builtin_amdgcn_readfirstlane(split);
    I = __builtin_amdgcn_readfirstlane(I); J = __builtin_amdgcn_readfirstlane(J);
    c_begin = __builtin_amdgcn_readfirstlane(c_begin); nchunks = __builtin_amdgcn_readfirstlane(nchunks);

    // Staging: a wavefront-wide 16-byte load fills 64 consecutive features of one unit (1 KB of LDS); wavefront w
    // brings unit w of every chunk, NF loads.  Lanes whose feature lies beyond M, and units beyond the range, read the
    // zero element instead, so every stage is completely rewritten by every chunk.
    int off[NF];
    unsigned okmask = 0;
#pragma unroll
    for (int k = 0; k < NF; ++k) {
        const int f = k < NRT ? I * TR + 64 * k + lane : J * TC + 64 * (k - NRT) + lane;
        bool ok;
        if (!SHIFT) {
            ok = f < g.M;
            int ext_unused;
            feat_map(ok ? f : 0, g, &off[k], &ext_unused);
        } else if (k < NRT) {           // channel f of the unit (pixel, or pixel pair) itself
            ok = f < g.t_cin;
            off[k] = ok ? f : 0;
        } else {                        // channel c of the unit shifted back by difference di
            ok = f < g.F;
            const int di = ok ? f / g.t_cin : 0, c = ok ? f - di * g.t_cin : 0;
            int dy, dx;
            shift_diff_of(di, g.t_kw, &dy, &dx);
            off[k] = -(dy * g.t_wp + dx) * g.t_cin + c;
        }
        okmask |= (ok ? 1u : 0u) << k;
    }

    floatx16 acc[NRT][NCT];
#pragma unroll
    for (int a = 0; a < NRT; ++a)
#pragma unroll
        for (int b = 0; b < NCT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

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
#pragma unroll
                for (int h = 0; h < 16; h += 8) {   // eight loads in flight (sixteen do not fit beside 256 accumulators)
                    float old[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int gi = gi0 + 8 * ((h + i) >> 2) + ((h + i) & 3);
                        old[i] = (gi < g.M && gj < g.M && gj <= gi) ? A[(size_t)gi * g.M + gj] : 0.f;
                    }
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int gi = gi0 + 8 * ((h + i) >> 2) + ((h + i) & 3);
                        if (gi < g.M && gj < g.M && gj <= gi) A[(size_t)gi * g.M + gj] = old[i] + acc[ta][tb][h + i];
                    }
                }
            }
        }
    }
}

// Column sums from the per-pixel sums: s[m] += sum over the output positions of S8 under the tap of feature m, in two
// steps.  First: 64 consecutive features (consecutive channels of a tap lie next to each other in S8: a wavefront reads
// 256 contiguous bytes) x one of up to CS_SLICES slices of the positions per workgroup of 1024 threads, the slice dealt
// to its 16 wavefronts in runs of eight positions along an output row: eight loads in flight and no index arithmetic
// between them, float64 (the loop is a chain of load latencies: many short slices beat few long ones).  Second: the slices are added in a fixed order, 16 lanes per feature.
constexpr int CS_SLICES = 64;
__global__ __launch_bounds__(1024) void column_sums_kernel(TileCore g, const float* __restrict__ S8, double* __restrict__ cpart,
                                                           float* __restrict__ s) {
    __shared__ double red[16][64];
    const int fl = threadIdx.x & 63, pl = threadIdx.x >> 6;
    const int fi = blockIdx.x * 64 + fl;
    const bool ok = fi < g.M;
    int off = 0, ext = 0;
    if (ok) feat_map(fi, g, &off, &ext);
    const int per_img = g.Hp * g.Wp * g.Cin;
    // items: runs of eight positions along an output row (one batch of loads, no index arithmetic inside)
    const int nseg = (g.Wo + 7) >> 3;
    const int total = g.Ho * g.bg_chunks * nseg;
    const int per_slice = (total + (int)gridDim.y - 1) / (int)gridDim.y;
    const int i0 = blockIdx.y * per_slice, i1 = min(total, i0 + per_slice);
    const int step = g.stride * g.Cin;
    double v = 0.0;
    if (ok)
        for (int it = i0 + pl; it < i1; it += 16) {
            const int row = it / nseg, seg = it - row * nseg;
            const int k = row / g.Ho, oy = row - k * g.Ho;
            const float* src = S8 + (size_t)k * per_img + ((oy * g.stride) * g.Wp + seg * 8 * g.stride) * g.Cin + g.sum_shift + off;
            const int n = min(8, g.Wo - seg * 8);
            float x[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) x[q] = src[(q < n ? q : 0) * step];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                asm volatile("" : "+v"(x[q]));      // all eight loads are issued before the first is used
                if (q >= n) x[q] = 0.f;
            }
            v += (((double)x[0] + (double)x[1]) + ((double)x[2] + (double)x[3])) + (((double)x[4] + (double)x[5]) + ((double)x[6] + (double)x[7]));
        }
    red[pl][fl] = v;
    __syncthreads();
    if (pl == 0 && ok) {
        double t = 0.0;
#pragma unroll
        for (int q = 0; q < 16; ++q) t += red[q][fl];
        if (gridDim.y == 1) s[ext] = (float)((double)s[ext] + t);   // few positions: one slice, no second step
        else cpart[(size_t)blockIdx.y * g.M + ext] = t;
    }
}

__global__ __launch_bounds__(256) void column_sums_final_kernel(int M, int nslices, const double* __restrict__ cpart, float* __restrict__ s) {
    const int m = blockIdx.x * 16 + (threadIdx.x & 15), part = threadIdx.x >> 4;   // 16 features x 16 lanes
    double t = 0.0;
    if (m < M)
        for (int q = part; q < nslices; q += 16) t += cpart[(size_t)q * M + m];
    __shared__ double red[16][17];
    red[part][threadIdx.x & 15] = t;
    __syncthreads();
    if (part == 0 && m < M) {
        double v = 0.0;
#pragma unroll
        for (int q = 0; q < 16; ++q) v += red[q][threadIdx.x];
        s[m] = (float)((double)s[m] + v);
    }
}

// partial tiles -> A (float64 sum over the ranges).  A workgroup takes 256 / NG consecutive tile elements; its NG groups
// of threads share the ranges (group q takes the ranges q, q + NG, ..., eight loads in flight) and are added in a fixed
// order, so that many ranges do not become a long chain of loads in few threads.
template <int NG>
__global__ __launch_bounds__(256) void tile_reduce_kernel(TileCore g, const float* __restrict__ part, float* __restrict__ A) {
    constexpr int EPB = 256 / NG;                  // elements per workgroup
    const int bpt = g.tr * g.tc / EPB;             // workgroups per tile of tr x tc
    const int tile = blockIdx.x / bpt;
    const int le = threadIdx.x % EPB, grp = threadIdx.x / EPB;
    const int e = (blockIdx.x - tile * bpt) * EPB + le;
    int I, J;
    tile_coords(tile, g, &I, &J);
    const int row = e / g.tc, col = e - row * g.tc;
    const int fi = I * g.tr + row, fj = J * g.tc + col;
    const bool active = fi < g.M && fj < g.M && fj <= fi;
    const size_t tsz = (size_t)g.tr * g.tc;
    const size_t stride = (size_t)g.ntiles * tsz;
    const float* src = part + (size_t)tile * tsz + e;
    double v = 0.0;
    if (active) {
        int sp = grp;
        for (; sp + 7 * NG < g.nsplit; sp += 8 * NG) {
            float x[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) x[q] = src[(size_t)(sp + q * NG) * stride];
#pragma unroll
            for (int q = 0; q < 8; ++q) v += (double)x[q];
        }
        for (; sp < g.nsplit; sp += NG) v += (double)src[(size_t)sp * stride];
    }
    if (NG > 1) {
        __shared__ double red[NG > 1 ? NG - 1 : 1][EPB];
        if (grp > 0) red[grp - 1][le] = v;
        __syncthreads();
        if (grp > 0) return;
#pragma unroll
        for (int q = 0; q < NG - 1; ++q) v += red[q][le];
    }
    if (!active) return;
    int o, ei, ej;
    feat_map(fi, g, &o, &ei);
    feat_map(fj, g, &o, &ej);
    float* dst = A + (size_t)max(ei, ej) * g.M + min(ei, ej);
    *dst = (float)((double)*dst + v);
}

// Shift-correlation mode: the block of A that pairs row tap t1 with column tap t2 <= t1 (in tap order) is the sum, over
// the regions whose pixels serve t1 and over their unit ranges, of the partial tiles' entries R(t1 - t2)[c1][c2].  A
// workgroup takes 16 / NG channels c1 x 64 channels c2 of one pair of taps, so the window and the ranges are uniform
// and the loads (16 bytes per lane along c2, four in flight) and the writes run along rows; its NG groups of threads
// share the ranges and are added in a fixed order; float64 sums.
template <int NG>
__global__ __launch_bounds__(256) void shift_tile_assemble_kernel(TileGeom g, const float* __restrict__ part, float* __restrict__ A) {
    const int kk = g.kh * g.kw;
    int t1 = 0;
    {
        int pr = blockIdx.z;                          // pair index: t1 (t1 + 1) / 2 + t2
        while ((t1 + 1) * (t1 + 2) / 2 <= pr) ++t1;
        pr -= t1 * (t1 + 1) / 2;
        const int t2 = pr;
        const int t1y = t1 / g.kw, t1x = t1 - t1y * g.kw, t2y = t2 / g.kw, t2x = t2 - t2y * g.kw;
        int dy = t1y - t2y, dx = t1x - t2x;           // >= 0 in lexicographic order because t1 >= t2
        constexpr int R = 16 / NG;                     // channels c1 per workgroup; NG groups of 16 R threads share the ranges
        const int lane = threadIdx.x % (16 * R), grp = threadIdx.x / (16 * R);
        const int c1 = blockIdx.y * R + (lane >> 4);
        const int c2 = blockIdx.x * 64 + 4 * (lane & 15);
        // entries right of the diagonal of a diagonal block are not kept
        const bool active = c1 < g.Cin && c2 < g.Cin && !(t1 == t2 && c2 > c1 + 3);
        const size_t tsz = (size_t)g.tr * g.tc;
        const size_t stride = (size_t)g.ntiles * tsz;
        double v0 = 0.0, v1 = 0.0, v2 = 0.0, v3 = 0.0;
        for (int a = 0; a < g.gx && active; ++a) {    // the pixel of a pair that plays the row tap (one pass without pairs)
            int row, f;
            if (g.gx == 1) {
                row = c1;
                f = shift_diff_index(dy, dx, g.kw) * g.Cin + c2;
            } else {
                const int sft = a - dx;               // the column pixel is 2X + a - dx: pair X + floor(sft / 2), parity sft mod 2
                const int fl = sft >= 0 ? sft / 2 : -((1 - sft) / 2);
                const int ap = sft - 2 * fl;
                row = a * g.Cin + c1;
                f = shift_diff_index(dy, -fl, g.t_kw) * g.t_cin + ap * g.Cin + c2;
            }
            // four consecutive columns f .. f+3 lie in one tile (Cin % 4 == 0)
            const int I = row / g.tr, J = f / g.tc;
            const float* src = part + (size_t)(I * g.ncb + J) * tsz + (size_t)(row - I * g.tr) * g.tc + (f - J * g.tc);
            for (int r = 0; r < g.nreg; ++r) {
                const int cm = a == 0 ? g.reg[r].colmask : g.reg[r].colmask2;
                if (!(((g.reg[r].rowmask >> t1y) & 1) && ((cm >> t1x) & 1))) continue;
                const int s0 = g.reg[r].split_begin, s1 = s0 + g.reg[r].nsplit;
                for (int sp = s0 + 4 * grp; sp < s1; sp += 4 * NG) {   // group grp: every NG-th batch of four ranges
                    float4 x[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) x[q] = *reinterpret_cast<const float4*>(src + (size_t)(sp + q < s1 ? sp + q : s0) * stride);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        asm volatile("" : "+v"(x[q].x), "+v"(x[q].y), "+v"(x[q].z), "+v"(x[q].w));
                        if (sp + q < s1) { v0 += (double)x[q].x; v1 += (double)x[q].y; v2 += (double)x[q].z; v3 += (double)x[q].w; }
                    }
                }
            }
        }
        if (NG > 1) {
            __shared__ double red[NG > 1 ? NG - 1 : 1][4][16 * R];
            if (grp > 0) { red[grp - 1][0][lane] = v0; red[grp - 1][1][lane] = v1; red[grp - 1][2][lane] = v2; red[grp - 1][3][lane] = v3; }
            __syncthreads();
            if (grp > 0) return;
#pragma unroll
            for (int q = 0; q < NG - 1; ++q) { v0 += red[q][0][lane]; v1 += red[q][1][lane]; v2 += red[q][2][lane]; v3 += red[q][3][lane]; }
        }
        if (!active) return;
        const double v[4] = {v0, v1, v2, v3};
        const bool kkc = g.layout == FW_LAYOUT_NHWC_KKC;
        if (kkc && (t1 != t2 || c2 + 3 <= c1)) {
            // channels-last order: the four columns are contiguous in A (16-byte aligned: Cin and c2 are multiples of 4)
            float4* dst = reinterpret_cast<float4*>(A + (size_t)(t1 * g.Cin + c1) * g.M + (size_t)t2 * g.Cin + c2);
            float4 o = *dst;
            o.x = (float)((double)o.x + v0); o.y = (float)((double)o.y + v1);
            o.z = (float)((double)o.z + v2); o.w = (float)((double)o.w + v3);
            *dst = o;
            return;
        }
        // the four old values are read before the first new one is written (a read behind a write would wait for it)
        float* dst[4];
        float old[4];
        bool keep[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int cc = c2 + q;
            keep[q] = !(t1 == t2 && cc > c1);
            const int ei = kkc ? t1 * g.Cin + c1 : c1 * kk + t1;
            const int ej = kkc ? t2 * g.Cin + cc : cc * kk + t2;
            dst[q] = A + (keep[q] ? (size_t)max(ei, ej) * g.M + min(ei, ej) : 0);
            old[q] = *dst[q];
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (keep[q]) *dst[q] = (float)((double)old[q] + v[q]);
    }
}

// Geometry of the shift-correlation mode; false when it does not apply.  *cost is an estimate of its run time in the
// same terms as the direct form's (see make_tile_geom).
bool make_shift_tile_geom(const fw_conv_desc* d, TileGeom* g, double* cost) {
    if (d->stride != 1 || d->kh * d->kw <= 1 || d->kh > 8 || d->kw > 8 || (d->Cin & 3) != 0) return false;
    if (d->form == FW_COV_FORM_DIRECT) return false;
    const int Cin = d->Cin;
    const int gx = Cin <= 128 && d->W >= 4 ? 2 : 1;    // few channels: pairs of pixels fill the rows of a larger tile
    g->gx = gx;
    g->t_cin = gx * Cin;
    g->t_kw = gx == 1 ? d->kw : d->kw / 2 + 1;        // pairs back: 0 .. kw / 2 (and as many forward under dy > 0)
    g->nd = g->t_kw + (d->kh - 1) * (2 * g->t_kw - 1);
    const long long F = (long long)g->nd * g->t_cin;
    if (F > (1 << 20)) return false;
    g->F = (int)F;
    g->shift = 1;
    // border of zeros: what the differences reach above and to both sides, the windows' own padding below
    const int reach = gx * (g->t_kw - 1);
    const int hy = d->kh - 1 > d->pad ? d->kh - 1 : d->pad, hx = reach > d->pad ? reach : d->pad;
    const int wu = (d->W + gx - 1) / gx;               // units per image row; an odd last pixel pairs with the border
    g->py = hy; g->px = hx;
    g->Hp = d->H + hy + d->pad; g->Wp = hx + gx * wu + hx;
    if (g->Wp % gx) ++g->Wp;
    g->t_wp = g->Wp / gx;
    g->sum_shift = ((g->py - d->pad) * g->Wp + (g->px - d->pad)) * Cin;
    const long long packed = (long long)g->Bg * g->Hp * g->Wp * Cin;
    if (packed + 16 >= (1ll << 31)) return false;
    ShiftBand rows[16], cols[16];
    const int nr = shift_bands(d->H, d->kh, d->pad, g->Ho, rows, 16);
    int nc = shift_bands(d->W, d->kw, d->pad, g->Wo, cols, 16);
    if (nr <= 0 || nc <= 0) return false;
    int colmask2[16] = {0};
    if (gx == 2) {
        // bands of pairs: runs of pairs X whose pixels 2X and 2X + 1 serve the same two sets of column taps
        auto mask_at = [&](int x) {
            for (int b = 0; b < nc; ++b)
                if (x >= cols[b].begin && x < cols[b].begin + cols[b].len) return cols[b].mask;
            return 0;                                  // beyond the image, or a pixel that serves no tap
        };
        ShiftBand pc[16];
        int np = 0, X = 0;
        while (X < wu) {
            const int m0 = mask_at(2 * X), m1 = mask_at(2 * X + 1);
            int X1 = X;
            while (X1 + 1 < wu && mask_at(2 * X1 + 2) == m0 && mask_at(2 * X1 + 3) == m1) ++X1;
            if (m0 | m1) {
                if (np == 16) return false;
                pc[np] = ShiftBand{X, X1 - X + 1, m0};
                colmask2[np++] = m1;
            }
            X = X1 + 1;
        }
        nc = np;
        for (int b = 0; b < nc; ++b) cols[b] = pc[b];
        if (nc <= 0) return false;
    }
    if (nr * nc > MAXREG) return false;
    g->nreg = nr * nc;
    g->nrt = g->t_cin > 192 ? 4 : g->t_cin > 128 ? 3 : 2;
    g->nct = 4;
    g->tr = 64 * g->nrt; g->tc = 64 * g->nct;
    g->nrb = (g->t_cin + g->tr - 1) / g->tr; g->ncb = (g->F + g->tc - 1) / g->tc;
    g->ntiles = g->nrb * g->ncb;
    // regions, largest first: their ranges are dispatched in this order, so the short ones fill the end
    int nregs = 0;
    for (int a = 0; a < nr; ++a)
        for (int b = 0; b < nc; ++b) {
            TileRegion& R = g->reg[nregs++];
            R.y0 = rows[a].begin; R.rh = rows[a].len; R.rowmask = rows[a].mask;
            R.x0 = cols[b].begin; R.rw = cols[b].len; R.colmask = cols[b].mask; R.colmask2 = colmask2[b];
            R.nchunks = (int)(((long long)g->Bg * R.rh * R.rw + KU - 1) / KU);
            for (int q = 0; q < 4; ++q) R.dmask[q] = 0;
            for (int pa = 0; pa < gx; ++pa)
                for (int t1 = 0; t1 < d->kh * d->kw; ++t1) {
                    const int t1y = t1 / d->kw, t1x = t1 - t1y * d->kw;
                    if (!(((R.rowmask >> t1y) & 1) && (((pa ? R.colmask2 : R.colmask) >> t1x) & 1))) continue;
                    for (int t2 = 0; t2 <= t1; ++t2) {
                        const int dy = t1y - t2 / d->kw, dx = t1x - t2 % d->kw;
                        int di;
                        if (gx == 1) di = shift_diff_index(dy, dx, d->kw);
                        else {
                            const int sft = pa - dx;
                            di = shift_diff_index(dy, sft >= 0 ? -(sft / 2) : (1 - sft) / 2, g->t_kw);
                        }
                        R.dmask[di >> 5] |= 1u << (di & 31);
                    }
                }
        }
    std::stable_sort(g->reg, g->reg + nregs, [](const TileRegion& x, const TileRegion& y) { return x.nchunks > y.nchunks; });
    long long total_chunks = 0;
    for (int r = 0; r < nregs; ++r) {
        g->reg[r].chunk_begin = (int)total_chunks;
        total_chunks += g->reg[r].nchunks;
    }
    if (total_chunks * KU >= (1ll << 31) - KU) return false;
    for (int r = g->nreg; r < MAXREG; ++r) g->reg[r] = TileRegion{0, 0, 1, 1, 0, 0, 0, 0, 0, 0, 0, {0, 0, 0, 0}};
    g->nchunks = (int)total_chunks;
    g->n_units = (int)(total_chunks * KU);
    g->direct = 0;
    g->zero_off = (int)packed;
    // Length of a unit range (ranges never cross a region): simulate the dispatch of the workgroups, in launch order, onto
    // the 256 compute units for a ladder of lengths and keep the cheapest: time of the longest compute unit plus the
    // traffic of the partial tiles (written once, read back by the assembly about 0.6 times per tap pair of a window).
    const double clk = 2.0e9, bw = 4.0e12, lds_load_rate = 23.0;
    const double t_mfma = 64.0 * g->nrt * g->nct + 150.0, t_load = (double)(g->tr + g->tc) * KU * 16.0 / lds_load_rate;
    const double t_chunk = (t_mfma > t_load ? t_mfma : t_load) / clk;
    const double ideal = (double)total_chunks * g->ntiles / 256.0;
    const int kk = d->kh * d->kw;
    double best = 1e300;
    long long best_cps = 8;
    int best_spread = 0;
    // what the spread mapping costs: seven more XCDs pull the packed units into their L2 (from the shared last-level cache)
    const double spread_penalty = 7.0 * (double)packed * 16.0 / 8.0e12;
    long long last_cps = -1;
    for (int step = -24; step <= 24; ++step) {
        long long cps = (long long)(ideal * pow(2.0, step / 12.0) + 0.5);
        if (cps < 8) cps = 8;
        if (cps > total_chunks) cps = total_chunks;
        if (cps == last_cps) continue;
        last_cps = cps;
        int nsplit = 0;
        int len[MAXREG], cnt[MAXREG];
        for (int r = 0; r < nregs; ++r) {
            cnt[r] = (int)((g->reg[r].nchunks + cps - 1) / cps);
            len[r] = g->reg[r].nchunks - (cnt[r] - 1) * (int)cps;   // the last range of a region
            nsplit += cnt[r];
        }
        if ((long long)nsplit * g->ntiles > 8192) continue;
        int r = 0, within = 0;
        std::vector<int> range_len(nsplit), range_reg(nsplit);
        for (int sp = 0; sp < nsplit; ++sp) {
            range_len[sp] = within == cnt[r] - 1 ? len[r] : (int)cps;
            range_reg[sp] = r;
            if (++within == cnt[r]) { within = 0; ++r; }
        }
        for (int spread = 0; spread < 2; ++spread) {
            // workgroup w goes to XCD w % 8, which hands its workgroups, in launch order, to its 32 compute units
            // (one workgroup each): a min-heap of finish times per XCD
            std::priority_queue<double, std::vector<double>, std::greater<double>> cu[8];
            for (int x = 0; x < 8; ++x)
                for (int i = 0; i < 32; ++i) cu[x].push(0.0);
            double makespan = 0.0, wgs = 0.0;
            auto place = [&](int w, int sp, int t) {
                if (!region_needs_tile(g->reg[range_reg[sp]], t % g->ncb, g->tc, g->t_cin, g->nd)) return;   // leaves at once
                auto& q = cu[w & 7];
                const double f = q.top() + range_len[sp] + 6.0;   // fill of the ring and write-out of the tile
                q.pop(); q.push(f);
                if (f > makespan) makespan = f;
                wgs += 1.0;
            };
            if (spread) {
                for (int w = 0; w < nsplit * g->ntiles; ++w) place(w, w / g->ntiles, w % g->ntiles);
            } else {
                int w = 0;
                for (int g8 = 0; g8 < nsplit; g8 += 8)
                    for (int t = 0; t < g->ntiles; ++t)
                        for (int sp = g8; sp < g8 + 8; ++sp, ++w)
                            if (sp < nsplit) place(w, sp, t);
            }
            const double c = makespan * t_chunk + wgs * g->tr * g->tc * 4.0 / bw + (spread ? spread_penalty : 0.0) +
                             0.5 * kk * (kk + 1) * (double)Cin * Cin * 4.0 * 0.6 * gx * nsplit / bw + 0.5 * (double)g->M * g->M * 8.0 / bw;
            if (c < best) { best = c; best_cps = cps; best_spread = spread; }
        }
    }
    g->spread = best_spread;
    g->chunks_per_split = (int)best_cps;
    int nsplit = 0;
    for (int r = 0; r < nregs; ++r) {
        g->reg[r].split_begin = nsplit;
        g->reg[r].nsplit = (int)((g->reg[r].nchunks + best_cps - 1) / best_cps);
        nsplit += g->reg[r].nsplit;
    }
    g->nsplit = nsplit;
    *cost = best;
    return true;
}

bool build_tile_geom(const fw_conv_desc* d, fw_layout lay, TileGeom* g) {
    g->B = d->B; g->Cin = d->Cin; g->H = d->H; g->W = d->W;
    g->kh = d->kh; g->kw = d->kw; g->stride = d->stride; g->pad = d->pad;
    g->layout = (int)lay;
    g->Ho = (d->H + 2 * d->pad - d->kh) / d->stride + 1;
    g->Wo = (d->W + 2 * d->pad - d->kw) / d->stride + 1;
    g->Hp = d->H + 2 * d->pad; g->Wp = d->W + 2 * d->pad;
    g->py = g->px = d->pad; g->sum_shift = 0;
    g->shift = 0; g->nd = 0; g->F = 0; g->nreg = 0; g->spread = 0;
    for (int r = 0; r < MAXREG; ++r) g->reg[r] = TileRegion{0, 0, 1, 1, 0, 0, 0, 0, 0, 0, 0, {0, 0, 0, 0}};
    g->gx = 1; g->t_cin = d->Cin; g->t_wp = g->Wp; g->t_kw = d->kw;
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
    {
        // stride-1 windows: tap pairs with the same difference share their products (shift-correlation mode)
        TileGeom gs = *g;
        double cs = 0.0;
        if (lay != FW_LAYOUT_ROWS && make_shift_tile_geom(d, &gs, &cs) && (cs < best || d->form == FW_COV_FORM_SHIFT)) {
            const long long per_img = (long long)gs.Hp * gs.Wp * d->Cin;
            long long ch = (524288 + per_img - 1) / per_img;
            if (ch > gs.Bg) ch = gs.Bg;
            if (ch < 1) ch = 1;
            gs.bg_per_chunk = (int)((gs.Bg + ch - 1) / ch);
            gs.bg_chunks = (gs.Bg + gs.bg_per_chunk - 1) / gs.bg_per_chunk;
            *g = gs;
            return true;
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

// The geometries of the layers asked for most recently (64 of them) are kept per host thread: a call computes one for the
// workspace check and for the launches, the dispatch simulation behind it takes milliseconds, and a training loop asks for
// the same layers over and over.
bool make_tile_geom(const fw_conv_desc* d, fw_layout lay, TileGeom* g) {
    struct Entry { bool ok; fw_conv_desc d; fw_layout lay; TileGeom g; };
    static thread_local std::vector<Entry> cache;     // most recent first
    for (size_t i = 0; i < cache.size(); ++i)
        if (cache[i].lay == lay && memcmp(&cache[i].d, d, sizeof(*d)) == 0) {
            if (i) std::swap(cache[i], cache[0]);
            if (cache[0].ok) *g = cache[0].g;
            return cache[0].ok;
        }
    Entry e;
    memset(&e, 0, sizeof(e));
    e.ok = build_tile_geom(d, lay, &e.g);
    e.d = *d; e.lay = lay;
    if (cache.size() >= 64) cache.pop_back();
    cache.insert(cache.begin(), e);
    if (e.ok) *g = e.g;
    return e.ok;
}

struct Bf16Ws { size_t packed, utab, part, s8, cpart, total; };
Bf16Ws ws_layout(const TileGeom& g) {
    Bf16Ws L;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes, 256); return at; };
    L.packed = take(((size_t)g.Bg * g.Hp * g.Wp * g.Cin + 16) * 16);
    L.utab = take((size_t)g.nchunks * KU * 4);
    L.part = take(g.direct ? 0 : (size_t)g.nsplit * g.ntiles * g.tr * g.tc * 4);
    L.s8 = take((size_t)g.bg_chunks * g.Hp * g.Wp * g.Cin * 4);
    L.cpart = take((size_t)CS_SLICES * g.M * sizeof(double));
    L.total = o;
    return L;
}

}  // namespace

bool cov_bf16_plan(const fw_conv_desc* d, fw_layout lay, fw_cov_plan* plan) {
    TileGeom g;
    if (!d || !make_tile_geom(d, lay, &g)) return false;
    plan->shift = g.shift; plan->regions = g.nreg; plan->differences = g.nd;
    plan->workgroups = g.ntiles * g.nsplit; plan->ranges = g.nsplit;
    plan->covered_pixels = 0;
    for (int r = 0; r < g.nreg; ++r)
        plan->covered_pixels += (long long)g.B * g.reg[r].rh * g.reg[r].rw * ((g.reg[r].colmask != 0) + (g.gx == 2 && g.reg[r].colmask2 != 0));
    // every tile is multiplied over all chunks of its ranges: 32 reduction entries (4 units of 8 images) per chunk
    plan->mfma_flops_issued = 2.0 * (double)g.ntiles * g.tr * g.tc * 32.0 * (double)g.nchunks;
    if (g.shift) {   // border regions skip the column tiles whose differences they never use
        double chunk_tiles = 0.0;
        for (int r = 0; r < g.nreg; ++r)
            for (int t = 0; t < g.ntiles; ++t)
                if (region_needs_tile(g.reg[r], t % g.ncb, g.tc, g.t_cin, g.nd)) chunk_tiles += g.reg[r].nchunks;
        plan->mfma_flops_issued = 2.0 * chunk_tiles * g.tr * g.tc * 32.0;
    }
    return true;
}

size_t cov_bf16_workspace_bytes(const fw_conv_desc* d, fw_layout lay) {
    TileGeom g;
    if (!d || !make_tile_geom(d, lay, &g)) return 0;
    return ws_layout(g).total;
}

// split_f32: X is a float32 tensor with d->Cin / 2 channels, taken as hi + lo bfloat16 planes (d describes the doubled tensor)
fw_status cov_bf16_accumulate(const void* X, fw_layout lay, const fw_conv_desc* d, float* A, float* s, void* ws, size_t ws_bytes,
                              hipStream_t st, bool split_f32) {
    TileGeom g;
    if (!make_tile_geom(d, lay, &g)) return FW_ERR_UNSUPPORTED;
    const Bf16Ws L = ws_layout(g);
    if (!ws || ws_bytes < L.total) return FW_ERR_WORKSPACE;
    char* base = reinterpret_cast<char*>(ws);
    uint4* P = reinterpret_cast<uint4*>(base + L.packed);
    int* utab = reinterpret_cast<int*>(base + L.utab);
    float* part = reinterpret_cast<float*>(base + L.part);
    float* S8 = reinterpret_cast<float*>(base + L.s8);
    double* cpart = reinterpret_cast<double*>(base + L.cpart);
    const int per_img = g.Hp * g.Wp * g.Cin;
    const TileCore& core = g;   // the direct form's kernels take the geometry without the regions
    const dim3 pgrid((per_img + 255) / 256, g.bg_chunks);
    if (g.shift && split_f32) hipLaunchKernelGGL((pack_images_kernel<true, true>), pgrid, dim3(256), 0, st, X, g, P, S8, utab);
    else if (g.shift) hipLaunchKernelGGL((pack_images_kernel<true, false>), pgrid, dim3(256), 0, st, X, g, P, S8, utab);
    else if (split_f32) hipLaunchKernelGGL((pack_images_kernel<false, true>), pgrid, dim3(256), 0, st, X, core, P, S8, utab);
    else hipLaunchKernelGGL((pack_images_kernel<false, false>), pgrid, dim3(256), 0, st, X, core, P, S8, utab);
    FW_LAUNCH_CHECK();
    const dim3 grid(g.shift && !g.spread ? 8 * g.ntiles * ((g.nsplit + 7) / 8) : (g.ntiles * g.nsplit + 7) / 8 * 8);
#define FW_TILE_LAUNCH(R, C, S, G) hipLaunchKernelGGL((cov_bf16_tile_kernel<R, C, S>), grid, dim3(256), 0, st, P, utab, G, part, A)
    if (g.shift) switch (g.nrt) {      // the shift form's tiles are 64 nrt x 256
        case 4: FW_TILE_LAUNCH(4, 4, true, g); break;
        case 3: FW_TILE_LAUNCH(3, 4, true, g); break;
        default: FW_TILE_LAUNCH(2, 4, true, g); break;
    }
    else switch (g.nrt * 10 + g.nct) {
        case 44: FW_TILE_LAUNCH(4, 4, false, core); break;
        case 43: FW_TILE_LAUNCH(4, 3, false, core); break;
        case 42: FW_TILE_LAUNCH(4, 2, false, core); break;
        case 33: FW_TILE_LAUNCH(3, 3, false, core); break;
        case 32: FW_TILE_LAUNCH(3, 2, false, core); break;
        default: FW_TILE_LAUNCH(2, 2, false, core); break;
    }
#undef FW_TILE_LAUNCH
    FW_LAUNCH_CHECK();
    if (g.shift) {
        // few channels: too few workgroups of 16 x 64 entries to hide the chain of loads over the ranges; share them
        const int pairs = g.kh * g.kw * (g.kh * g.kw + 1) / 2, cb = (g.Cin + 63) / 64;
        if ((long long)cb * ((g.Cin + 15) / 16) * pairs < 512)
            hipLaunchKernelGGL(shift_tile_assemble_kernel<4>, dim3(cb, (g.Cin + 3) / 4, pairs), dim3(256), 0, st, g, part, A);
        else
            hipLaunchKernelGGL(shift_tile_assemble_kernel<1>, dim3(cb, (g.Cin + 15) / 16, pairs), dim3(256), 0, st, g, part, A);
    }
    else if (!g.direct) {
        // many ranges and few tiles: share the ranges inside a workgroup
        const int elems = g.ntiles * g.tr * g.tc;
        if (g.nsplit >= 64 && elems / 16 <= 65536 * 4)
            hipLaunchKernelGGL(tile_reduce_kernel<16>, dim3(elems / 16), dim3(256), 0, st, g, part, A);
        else if (g.nsplit >= 24)
            hipLaunchKernelGGL(tile_reduce_kernel<4>, dim3(elems / 64), dim3(256), 0, st, g, part, A);
        else
            hipLaunchKernelGGL(tile_reduce_kernel<1>, dim3(elems / 256), dim3(256), 0, st, g, part, A);
    }
    {
        // slices of the positions: enough workgroups to fill the chip, none when a workgroup per 64 features already does
        const long long total = (long long)g.Ho * g.bg_chunks * ((g.Wo + 7) / 8);   // runs of eight positions
        const int nfb = (g.M + 63) / 64;
        int ns = (int)((1024 + nfb - 1) / nfb);
        if ((long long)ns * 32 > total) ns = (int)(total / 32);                     // two runs per wavefront at least
        if (ns > CS_SLICES) ns = CS_SLICES;
        if (ns < 1) ns = 1;
        hipLaunchKernelGGL(column_sums_kernel, dim3(nfb, ns), dim3(1024), 0, st, g, S8, cpart, s);
        if (ns > 1) hipLaunchKernelGGL(column_sums_final_kernel, dim3((g.M + 15) / 16), dim3(256), 0, st, g.M, ns, cpart, s);
    }
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
