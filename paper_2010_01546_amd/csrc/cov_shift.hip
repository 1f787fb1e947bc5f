// Moment accumulation for stride-1 convolutions through shift correlations (float32 activations).
//
// The patch rows of a stride-1 convolution repeat every pixel kh*kw times, and the block of A = X^T X that pairs tap
// t1 with tap t2 (the sums inside eqs. (vmuxi), (vPhixi) of Sec. 2 over the unfolded rows),
//     A[(t1,c1),(t2,c2)] = sum over output positions p of  x[p + t1, c1] x[p + t2, c2]      (x = 0 outside the image)
// becomes, with q = p + t1 and d = t2 - t1,
//     sum over pixels q with q - t1 inside the output grid of  x[q, c1] x[q + d, c2].
// It depends on the pair of taps only through their difference d and through WHICH pixels q take part, and the latter
// differs between taps only in a border of the image.  So the image is cut into regions (row band x column band) inside
// which the set of taps a pixel serves is the same, and for every region r and every tap difference d
//     R_r(d)[c1][c2] = sum over pixels q of region r of  x[q, c1] x[q + d, c2]
// is accumulated on the matrix cores: a product with Cin rows and nd*Cin columns over all pixels, nd = (number of tap
// differences d >= 0 in lexicographic order) = 13 for a 3x3 window instead of the 45 tap pairs of the lower triangle.
// A block of A is then the sum of R_r(d) over the regions whose pixels serve t1; for d < 0 the transposed block of the
// mirrored pair is used.  Nothing is subtracted, the regions are disjoint, so the rounding is that of the plain sums:
// float32 inside a range of pixels, float64 across ranges and regions.  The column sums follow from per-region channel
// sums in the same way.
//
// Work decomposition of the product: a workgroup stages one row panel (64 channels at q) and up to 14 column panels
// (64 of the nd*Cin shifted features each) per chunk of 16 pixels; its eight wavefronts share out the 32x32 output
// tiles (v_mfma_f32_32x32x2_f32) evenly; the pixel axis is split into ranges that never cross a region.
#include "fw_internal.h"
#include <type_traits>

namespace fw {
namespace {

constexpr int BLK = 64;
constexpr int KT = 16;         // pixels per staged chunk
constexpr int NCP = 14;        // column panels per workgroup item
constexpr int NPAN = 2 + NCP;  // staged panels: the row panel, the column panels, one never read (keeps the staging uniform)
constexpr int NLD = NPAN / 2;   // panels one thread stages = pixel pairs of a chunk
constexpr int MAXT = 7;        // 32x32 output tiles per wavefront
constexpr int MAXREG = 32;

struct ShiftRegion {
    int y0, x0, rh, rw;        // rectangle of pixels
    int rowmask, colmask;      // bit ty / tx set: the pixels of this region serve taps of row ty / column tx
    int split_begin, nsplit;   // its pixel ranges
};

struct ShiftGeom {
    int B, Cin, H, W, kh, kw, pad, Ho, Wo;
    int M;
    int nd;                    // tap differences kept: (0, 0..kw-1), then (dy, -(kw-1)..kw-1) for dy = 1..kh-1
    int F;                     // nd * Cin column features
    int nbr, nbc;              // 64-blocks of the Cin rows and of the F columns
    int ipr;                   // workgroup items per row block = ceil(nbc / NCP)
    int nitems;
    int nreg, nsplit;
    int rps;                   // pixels per range (multiple of KT); the last range of a region may be shorter
    int kkc;                   // 1: A in (ky, kx, c) feature order, 0: (c, ky, kx)
    ShiftRegion reg[MAXREG];
};

struct SmemShift {
    alignas(16) float tile[2][NPAN][KT][BLK];   // [buffer][panel][pixel][feature], feature position rotated by 32 on odd pixels
};

// A workgroup of eight wavefronts owns one row panel (64 channels, two row tiles of 32) and up to NCP column panels
// (28 column tiles of 32 features).  Wavefront w takes row tile w & 1 and one of four runs of column tiles, at most
// seven, whose lengths differ by at most one; runs 0 and 2, and 1 and 3, add up to the same length, so the two
// wavefronts that share a SIMD carry the same load.  For a 3x3 window on 64 channels that is 52 tiles on 8 wavefronts,
// 6 or 7 each, nothing idle.  Two wavefronts per SIMD hide each other's staging and barriers.
__global__ __launch_bounds__(512) void shift_partial_f32_kernel(const float* __restrict__ X, ShiftGeom g, float* __restrict__ part,
                                                                float* __restrict__ spart) {
    __shared__ SmemShift sm;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // workgroups go to the 8 XCDs round-robin by linear index: every XCD gets whole pixel ranges (all items of a range)
    const int item_idx = (blockIdx.x >> 3) % g.nitems;
    const int split = (blockIdx.x & 7) + 8 * ((blockIdx.x >> 3) / g.nitems);
    if (split >= g.nsplit) return;
    const int rb = item_idx / g.ipr, ci = item_idx - rb * g.ipr;
    const int cb0 = ci * NCP;                              // first column block of the item
    const int ncp = min(NCP, g.nbc - cb0);                 // its column panels
    const int k = (tid >> 4) & 15, q = tid & 15, ph = wave >> 2;

    // region of this range
    int ri = 0;
    for (int r = 0; r < g.nreg; ++r)
        if (split >= g.reg[r].split_begin && split < g.reg[r].split_begin + g.reg[r].nsplit) ri = r;
    const int y0 = g.reg[ri].y0, x0 = g.reg[ri].x0, rh = g.reg[ri].rh, rw = g.reg[ri].rw;
    const int npix = g.B * rh * rw;
    const int r_begin = (split - g.reg[ri].split_begin) * g.rps;
    const int r_end = min(npix, r_begin + g.rps);

    // what this thread stages: 4 consecutive channels of one (shifted) pixel for the panels ph, ph + 2, ph + 4, ...
    int f_off[NLD], f_dy[NLD], f_dx[NLD];
    bool f_ok[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        const int pan = 2 * j + ph;
        int dy = 0, dx = 0, c = 0;
        bool ok;
        if (pan == 0) {
            c = rb * BLK + 4 * q;
            ok = c < g.Cin;
        } else {
            const int f = (cb0 + pan - 1) * BLK + 4 * q;
            ok = pan <= ncp && f < g.F;
            const int di = ok ? f / g.Cin : 0;
            c = ok ? f - di * g.Cin : 0;
            shift_diff_of(di, g.kw, &dy, &dx);
        }
        f_off[j] = (dy * g.W + dx) * g.Cin + (ok ? c : 0);
        f_dy[j] = dy; f_dx[j] = dx; f_ok[j] = ok;
    }
    const bool sums = ci == 0 && ph == 0;
    float4 ssum = make_float4(0.f, 0.f, 0.f, 0.f);

    // this wavefront's tiles: row tile rt, column tiles ct0 .. ct0 + nt - 1 of the item
    const int rt = wave & 1, cg = wave >> 1;
    const int nct = min(2 * ncp, (g.F - cb0 * BLK + 31) / 32);   // column tiles of the item that hold features
    const int tbase = nct >> 2, textra = nct & 3;
    const int nt = tbase + (cg < textra ? 1 : 0);
    const int ct0 = cg * tbase + min(cg, textra);
    const int half = lane >> 5, l32 = lane & 31;
    floatx16 acc[MAXT];
#pragma unroll
    for (int j = 0; j < MAXT; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    // LDS float offsets (inside a buffer) of the fragments this lane reads at pixel pair 0; a pixel pair further is
    // 2 * BLK floats further.  Lanes 32..63 read the odd pixel, whose features are rotated by 32.
    const int rot = half << 5;
    const int a_off = (0 * KT + half) * BLK + ((32 * rt + l32 + rot) & 63);
    int b_off[MAXT];
#pragma unroll
    for (int j = 0; j < MAXT; ++j) {
        const int ct = ct0 + (j < nt ? j : 0);
        b_off[j] = ((1 + (ct >> 1)) * KT + half) * BLK + ((32 * (ct & 1) + l32 + rot) & 63);
    }

    // Position of this thread's pixel in the first chunk, and the step from chunk to chunk.  `base` is the element index
    // of the pixel's first channel (the whole activation has fewer than 2^30 elements) and moves by precomputed steps,
    // so a chunk costs no multiplications.
    const int area = rh * rw;
    int r = r_begin + k;
    int yy, xx, base;
    {
        const int pb = r / area;
        const int p = r - pb * area;
        yy = p / rw;
        xx = p - yy * rw;
        base = ((pb * g.H + y0 + yy) * g.W + x0 + xx) * g.Cin;
    }
    const int adv_y = (KT % area) / rw, adv_x = (KT % area) % rw;
    const int step = ((KT / area) * g.H * g.W + adv_y * g.W + adv_x) * g.Cin;
    const int wrap_x = (g.W - rw) * g.Cin;            // one region row down instead of rw pixels to the right
    const int wrap_y = (g.H - rh) * g.W * g.Cin;      // first row of the next image instead of rh rows down

    // Loads are issued unconditionally (a masked-out lane reads element 0 instead) and masked when they are stored:
    // no branches around the loads.  pre[j] holds this thread's 16 bytes of panel 2 j + ph of the chunk after the one
    // being multiplied; bit j of okmask says whether they are real.
    static_assert(NLD == KT / 2, "one staged panel per pixel pair");
    float4 pre[NLD];
    unsigned okmask = 0;
    int cy = 0, cx = 0;
    bool row_ok = false;
    auto locate = [&]() { cy = y0 + yy; cx = x0 + xx; row_ok = r < r_end; };
    auto load_slot = [&](int j) {
        const bool ok = row_ok && f_ok[j] && (unsigned)(cy + f_dy[j]) < (unsigned)g.H && (unsigned)(cx + f_dx[j]) < (unsigned)g.W;
        const int idx = ok ? base + f_off[j] : 0;
        pre[j] = *reinterpret_cast<const float4*>(X + idx);
        okmask = (okmask & ~(1u << j)) | ((ok ? 1u : 0u) << j);
    };
    auto advance = [&]() {
        r += KT;
        base += step; yy += adv_y; xx += adv_x;
        if (xx >= rw) { xx -= rw; ++yy; base += wrap_x; }
        if (yy >= rh) { yy -= rh; base += wrap_y; }
    };
    const int pos = (4 * q + ((k & 1) << 5)) & 63;
    auto store_slot = [&](int j, int buf) {
        const bool ok = (okmask >> j) & 1u;
        float4 v;
        v.x = ok ? pre[j].x : 0.f; v.y = ok ? pre[j].y : 0.f; v.z = ok ? pre[j].z : 0.f; v.w = ok ? pre[j].w : 0.f;
        *reinterpret_cast<float4*>(&sm.tile[buf][2 * j + ph][k][pos]) = v;
        if (j == 0 && sums) { ssum.x += v.x; ssum.y += v.y; ssum.z += v.z; ssum.w += v.w; }
    };

    const int nchunks = (r_end - r_begin + KT - 1) / KT;
    // chunk 0 into buffer 0, chunk 1 into the registers
    locate();
#pragma unroll
    for (int j = 0; j < NLD; ++j) load_slot(j);
#pragma unroll
    for (int j = 0; j < NLD; ++j) store_slot(j, 0);
    advance();
    locate();
#pragma unroll
    for (int j = 0; j < NLD; ++j) load_slot(j);
    __syncthreads();
    // While chunk c is multiplied out of one buffer, chunk c + 1 moves from the registers into the other buffer and the
    // loads of chunk c + 2 are issued, one panel per pixel pair, between the matrix instructions (past the end of the
    // range the loads read element 0 and what is stored is never read).  One copy of the loop per tile count, so that
    // no matrix instruction sits behind a branch; a wavefront without tiles (NT = 0) only stages.
    auto run = [&](auto nt_const) {
        constexpr int NT = decltype(nt_const)::value;
        for (int c = 0; c < nchunks; ++c) {
            const int buf = c & 1;
            const float* tb = &sm.tile[buf][0][0][0];
            advance();
            locate();
#pragma unroll
            for (int k0 = 0; k0 < KT; k0 += 2) {
                if constexpr (NT > 0) {
                    const float a = tb[a_off + k0 * BLK];
                    float b[NT];
#pragma unroll
                    for (int j = 0; j < NT; ++j) b[j] = tb[b_off[j] + k0 * BLK];
#pragma unroll
                    for (int j = 0; j < NT; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b[j], acc[j], 0, 0, 0);
                }
                store_slot(k0 >> 1, buf ^ 1);
                load_slot(k0 >> 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();
        }
    };
    switch (nt) {
        case 7: run(std::integral_constant<int, 7>{}); break;
        case 6: run(std::integral_constant<int, 6>{}); break;
        case 5: run(std::integral_constant<int, 5>{}); break;
        case 4: run(std::integral_constant<int, 4>{}); break;
        case 3: run(std::integral_constant<int, 3>{}); break;
        case 2: run(std::integral_constant<int, 2>{}); break;
        case 1: run(std::integral_constant<int, 1>{}); break;
        default: run(std::integral_constant<int, 0>{}); break;
    }

    // partial blocks: [range][row block * nbc + column block][64 x 64]
#pragma unroll
    for (int j = 0; j < MAXT; ++j) {
        if (j >= nt) continue;
        const int ct = ct0 + j;
        float* dst = part + ((size_t)split * g.nbr * g.nbc + (size_t)rb * g.nbc + cb0 + (ct >> 1)) * (BLK * BLK);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = 32 * rt + 8 * (i >> 2) + 4 * half + (i & 3);
            const int col = 32 * (ct & 1) + l32;
            dst[row * BLK + col] = acc[j][i];
        }
    }
    if (ci == 0) {
        // channel sums of the row panel: 16 pixel-threads share a channel quad; combine through LDS (the tiles are dead)
        float* red = &sm.tile[0][0][0][0];
        if (ph == 0) *reinterpret_cast<float4*>(&red[k * 64 + 4 * q]) = ssum;
        __syncthreads();
        if (wave == 0) {
            float v = 0.f;
#pragma unroll
            for (int kk = 0; kk < 16; ++kk) v += red[kk * 64 + lane];
            spart[((size_t)split * g.nbr + rb) * BLK + lane] = v;
        }
    }
}

// R_r = sum of the partial blocks over the ranges of region r, float64.  A workgroup sums 256 consecutive elements of a
// block, 16 bytes per lane: its four wavefronts take every fourth range (four loads in flight each) and combine through
// LDS in a fixed order.  The last nreg * nbr workgroups do the same for the channel sums.
__global__ __launch_bounds__(256) void shift_region_reduce_kernel(ShiftGeom g, const float* __restrict__ part, const float* __restrict__ spart,
                                                                  double* __restrict__ Rr, double* __restrict__ Sr) {
    __shared__ double red[4][256];
    const int ln = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int per_reg = g.nbr * g.nbc * 16;
    const int nblk = g.nreg * per_reg;
    if ((int)blockIdx.x >= nblk) {
        const int idx = (int)blockIdx.x - nblk;
        const int ri = idx / g.nbr, rb = idx - ri * g.nbr;
        const int s0 = g.reg[ri].split_begin, s1 = s0 + g.reg[ri].nsplit;
        double v = 0.0;
        for (int sp = s0 + grp; sp < s1; sp += 4) v += (double)spart[((size_t)sp * g.nbr + rb) * BLK + ln];
        red[grp][ln] = v;
        __syncthreads();
        if (grp == 0) Sr[((size_t)ri * g.nbr + rb) * BLK + ln] = red[0][ln] + red[1][ln] + red[2][ln] + red[3][ln];
        return;
    }
    const int ri = blockIdx.x / per_reg;
    const int rem = blockIdx.x - ri * per_reg;
    const size_t e = (size_t)rem * 256 + 4 * ln;      // first of this lane's four elements of [block][64 x 64]
    const int s0 = g.reg[ri].split_begin, s1 = s0 + g.reg[ri].nsplit;
    const size_t stride = (size_t)g.nbr * g.nbc * BLK * BLK;
    const float* src = part + e;
    double v0 = 0.0, v1 = 0.0, v2 = 0.0, v3 = 0.0;
    int sp = s0 + grp;
    for (; sp + 12 < s1; sp += 16) {
        float4 x[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) x[j] = *reinterpret_cast<const float4*>(src + (size_t)(sp + 4 * j) * stride);
#pragma unroll
        for (int j = 0; j < 4; ++j) { v0 += (double)x[j].x; v1 += (double)x[j].y; v2 += (double)x[j].z; v3 += (double)x[j].w; }
    }
    for (; sp < s1; sp += 4) {
        const float4 x = *reinterpret_cast<const float4*>(src + (size_t)sp * stride);
        v0 += (double)x.x; v1 += (double)x.y; v2 += (double)x.z; v3 += (double)x.w;
    }
    red[grp][4 * ln] = v0; red[grp][4 * ln + 1] = v1; red[grp][4 * ln + 2] = v2; red[grp][4 * ln + 3] = v3;
    __syncthreads();
    const int t = threadIdx.x;
    Rr[(size_t)ri * stride + (size_t)rem * 256 + t] = red[0][t] + red[1][t] + red[2][t] + red[3][t];
}

__device__ __forceinline__ void tap_channel(int e, const ShiftGeom& g, int* ty, int* tx, int* c) {
    int t;
    if (g.kkc) { t = e / g.Cin; *c = e - t * g.Cin; }
    else { const int kk = g.kh * g.kw; *c = e / kk; t = e - *c * kk; }
    *ty = t / g.kw;
    *tx = t - *ty * g.kw;
}

// A[i][j] += sum over the regions that serve the row tap of R_r(d)[c1][c2], one thread per element of the lower
// triangle in the caller's feature order; workgroups with blockIdx.y == M add the column sums
__global__ __launch_bounds__(256) void shift_assemble_kernel(ShiftGeom g, const double* __restrict__ Rr, const double* __restrict__ Sr,
                                                             float* __restrict__ A, float* __restrict__ s) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if ((int)blockIdx.y == g.M) {
        if (j >= g.M) return;
        int ty, tx, c;
        tap_channel(j, g, &ty, &tx, &c);
        double v = 0.0;
        for (int r = 0; r < g.nreg; ++r)
            if (((g.reg[r].rowmask >> ty) & 1) && ((g.reg[r].colmask >> tx) & 1)) v += Sr[(size_t)r * g.nbr * BLK + c];
        s[j] = (float)((double)s[j] + v);
        return;
    }
    const int i = blockIdx.y;
    if (j > i) return;
    int t1y, t1x, c1, t2y, t2x, c2;
    tap_channel(i, g, &t1y, &t1x, &c1);
    tap_channel(j, g, &t2y, &t2x, &c2);
    int dy = t2y - t1y, dx = t2x - t1x;
    if (dy < 0 || (dy == 0 && dx < 0)) {   // the mirrored pair has the kept difference: A[i][j] = A[j][i]
        dy = -dy; dx = -dx;
        int t = t1y; t1y = t2y; t2y = t;
        t = t1x; t1x = t2x; t2x = t;
        t = c1; c1 = c2; c2 = t;
    }
    const int f = shift_diff_index(dy, dx, g.kw) * g.Cin + c2;
    const int rb = c1 >> 6, cb = f >> 6;
    const size_t stride = (size_t)g.nbr * g.nbc * BLK * BLK;
    const size_t idx = ((size_t)rb * g.nbc + cb) * (BLK * BLK) + (size_t)(c1 & 63) * BLK + (f & 63);
    double v = 0.0;
    for (int r = 0; r < g.nreg; ++r)
        if (((g.reg[r].rowmask >> t1y) & 1) && ((g.reg[r].colmask >> t1x) & 1)) v += Rr[(size_t)r * stride + idx];
    float* dst = A + (size_t)i * g.M + j;
    *dst = (float)((double)*dst + v);
}

struct ShiftWs { size_t part, spart, Rr, Sr, total; };
ShiftWs shift_ws_layout(const ShiftGeom& g) {
    ShiftWs L;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o += align_up(bytes, 256); return at; };
    const size_t blocks = (size_t)g.nbr * g.nbc * BLK * BLK;
    L.part = take((size_t)g.nsplit * blocks * sizeof(float));
    L.spart = take((size_t)g.nsplit * g.nbr * BLK * sizeof(float));
    L.Rr = take((size_t)g.nreg * blocks * sizeof(double));
    L.Sr = take((size_t)g.nreg * g.nbr * BLK * sizeof(double));
    L.total = o;
    return L;
}

}  // namespace

// Fills g and returns true when the shift-correlation path applies to this layer and needs fewer matrix instructions
// than the direct lower-triangle product.
static bool make_shift_geom(const fw_conv_desc* d, fw_layout lay, ShiftGeom* g) {
    if (lay != FW_LAYOUT_NHWC && lay != FW_LAYOUT_NHWC_KKC) return false;
    if (d->stride != 1 || d->kh * d->kw <= 1 || d->kh > 8 || d->kw > 8 || (d->Cin & 3) != 0) return false;
    if (d->form == FW_COV_FORM_DIRECT) return false;
    g->B = d->B; g->Cin = d->Cin; g->H = d->H; g->W = d->W; g->kh = d->kh; g->kw = d->kw; g->pad = d->pad;
    g->Ho = d->H + 2 * d->pad - d->kh + 1;
    g->Wo = d->W + 2 * d->pad - d->kw + 1;
    const long long M = (long long)d->Cin * d->kh * d->kw;
    const long long npix = (long long)d->B * d->H * d->W;
    if (g->Ho <= 0 || g->Wo <= 0 || M > 16384 || npix * d->Cin >= (1ll << 30)) return false;   // element indices stay far inside int
    g->M = (int)M;
    g->nd = d->kw + (d->kh - 1) * (2 * d->kw - 1);
    g->F = g->nd * d->Cin;
    g->nbr = (d->Cin + BLK - 1) / BLK;
    g->nbc = (g->F + BLK - 1) / BLK;
    g->ipr = (g->nbc + NCP - 1) / NCP;
    g->nitems = g->nbr * g->ipr;
    g->kkc = lay == FW_LAYOUT_NHWC_KKC ? 1 : 0;
    // fewer 64x64 block products than the lower triangle of the direct form
    const long long nb = (M + BLK - 1) / BLK;
    const double direct = 0.5 * (double)nb * (double)(nb + 1);
    const double shifted = (double)g->nbr * (double)g->nbc;
    if (shifted * 1.1 >= direct && d->form != FW_COV_FORM_SHIFT) return false;
    ShiftBand rows[8 * 2], cols[8 * 2];
    const int nr = shift_bands(d->H, d->kh, d->pad, g->Ho, rows, 16), nc = shift_bands(d->W, d->kw, d->pad, g->Wo, cols, 16);
    if (nr <= 0 || nc <= 0 || nr * nc > MAXREG) return false;
    g->nreg = nr * nc;
    // pixel ranges: one workgroup is resident per compute unit, and the grid should fit in ONE such round (a
    // workgroup that starts late holds up the end).  Ranges never cross a region, so the count
    // is found by shrinking the target until the rounded-up ranges of all regions fit; at least four chunks per range.
    const long long capacity = 256 / g->nitems > 0 ? 256 / g->nitems : 1;
    const long long max_split = (npix + 4 * KT - 1) / (4 * KT);
    int nsplit = 0;
    for (long long want = capacity > 1 ? capacity : 1;; --want) {
        long long w = want > max_split ? max_split : want;
        if (w < 1) w = 1;
        long long rps = (npix + w - 1) / w;
        rps = (rps + KT - 1) / KT * KT;
        g->rps = (int)rps;
        nsplit = 0;
        for (int a = 0; a < nr; ++a)
            for (int b = 0; b < nc; ++b) {
                ShiftRegion& R = g->reg[a * nc + b];
                R.y0 = rows[a].begin; R.rh = rows[a].len; R.rowmask = rows[a].mask;
                R.x0 = cols[b].begin; R.rw = cols[b].len; R.colmask = cols[b].mask;
                const long long pix = (long long)d->B * R.rh * R.rw;
                R.split_begin = nsplit;
                R.nsplit = (int)((pix + rps - 1) / rps);
                nsplit += R.nsplit;
            }
        if (nsplit <= capacity || want <= 1 || nsplit <= g->nreg) break;
    }
    for (int r = g->nreg; r < MAXREG; ++r) g->reg[r] = ShiftRegion{0, 0, 1, 1, 0, 0, 0, 0};
    g->nsplit = nsplit;
    return true;
}

size_t cov_shift_workspace_bytes(const fw_conv_desc* d, fw_layout lay) {
    ShiftGeom g;
    if (!d || !make_shift_geom(d, lay, &g)) return 0;
    return shift_ws_layout(g).total;
}

bool cov_shift_applies(const fw_conv_desc* d, fw_layout lay) {
    ShiftGeom g;
    return d && make_shift_geom(d, lay, &g);
}

bool cov_shift_plan(const fw_conv_desc* d, fw_layout lay, fw_cov_plan* plan) {
    ShiftGeom g;
    if (!d || !make_shift_geom(d, lay, &g)) return false;
    plan->shift = 1; plan->regions = g.nreg; plan->differences = g.nd;
    plan->workgroups = g.nitems * g.nsplit; plan->ranges = g.nsplit;
    plan->covered_pixels = 0;
    for (int r = 0; r < g.nreg; ++r) plan->covered_pixels += (long long)g.B * g.reg[r].rh * g.reg[r].rw;
    // every item multiplies its 64 rows by the 32-feature column tiles that hold features, over all pixels
    plan->mfma_flops_issued = 2.0 * (g.nbr * 64.0) * (((g.F + 31) / 32) * 32.0) * (double)g.B * g.H * g.W;
    return true;
}

fw_status cov_shift_accumulate(const float* X, fw_layout lay, const fw_conv_desc* d, float* A, float* s, void* ws, size_t ws_bytes,
                               hipStream_t st) {
    ShiftGeom g;
    if (!make_shift_geom(d, lay, &g)) return FW_ERR_UNSUPPORTED;
    const ShiftWs L = shift_ws_layout(g);
    if (!ws || ws_bytes < L.total) return FW_ERR_WORKSPACE;
    char* base = reinterpret_cast<char*>(ws);
    float* part = reinterpret_cast<float*>(base + L.part);
    float* spart = reinterpret_cast<float*>(base + L.spart);
    double* Rr = reinterpret_cast<double*>(base + L.Rr);
    double* Sr = reinterpret_cast<double*>(base + L.Sr);
    hipLaunchKernelGGL(shift_partial_f32_kernel, dim3(8 * g.nitems * ((g.nsplit + 7) / 8)), dim3(512), 0, st, X, g, part, spart);
    FW_LAUNCH_CHECK();
    hipLaunchKernelGGL(shift_region_reduce_kernel, dim3(g.nreg * g.nbr * g.nbc * 16 + g.nreg * g.nbr), dim3(256), 0, st, g, part, spart, Rr, Sr);
    FW_LAUNCH_CHECK();
    hipLaunchKernelGGL(shift_assemble_kernel, dim3((g.M + 255) / 256, g.M + 1), dim3(256), 0, st, g, Rr, Sr, A, s);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
