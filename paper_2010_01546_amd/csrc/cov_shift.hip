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
// Work decomposition of the product: as in the direct kernel, a wavefront owns a 64x64 block (2x2 MFMA 32x32x2 tiles);
// a workgroup stages one row panel (64 channels at q) and up to four column panels (64 of the nd*Cin shifted features)
// and its four wavefronts take one column block each; the pixel axis is split into ranges that never cross a region.
#include "fw_internal.h"
#include <type_traits>

namespace fw {
namespace {

constexpr int BLK = 64;
constexpr int KT = 16;         // pixels per staged chunk
constexpr int NSLOT = 5;       // one row panel + four column panels
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
    int ipr;                   // workgroup items per row block = ceil(nbc / 4)
    int nitems;
    int nreg, nsplit;
    int rps;                   // pixels per range (multiple of KT); the last range of a region may be shorter
    int kkc;                   // 1: A in (ky, kx, c) feature order, 0: (c, ky, kx)
    ShiftRegion reg[MAXREG];
};

__device__ __host__ inline void diff_of(int di, int kw, int* dy, int* dx) {
    if (di < kw) { *dy = 0; *dx = di; return; }
    const int e = di - kw, w2 = 2 * kw - 1;
    *dy = 1 + e / w2;
    *dx = e % w2 - (kw - 1);
}
__device__ __host__ inline int diff_index(int dy, int dx, int kw) { return dy == 0 ? dx : kw + (dy - 1) * (2 * kw - 1) + dx + kw - 1; }

struct SmemShift {
    alignas(16) float tile[2][NSLOT][KT][BLK];   // [buffer][panel][pixel][feature], feature position rotated by 32 on odd pixels
};

__global__ __launch_bounds__(256) void shift_partial_f32_kernel(const float* __restrict__ X, ShiftGeom g, float* __restrict__ part,
                                                                float* __restrict__ spart) {
    __shared__ SmemShift sm;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // workgroups go to the 8 XCDs round-robin by linear index: every XCD gets whole pixel ranges (all items of a range)
    const int item_idx = (blockIdx.x >> 3) % g.nitems;
    const int split = (blockIdx.x & 7) + 8 * ((blockIdx.x >> 3) / g.nitems);
    if (split >= g.nsplit) return;
    const int rb = item_idx / g.ipr, ci = item_idx - rb * g.ipr;
    const int k = tid >> 4, q = tid & 15;

    // region of this range
    int ri = 0;
    for (int r = 0; r < g.nreg; ++r)
        if (split >= g.reg[r].split_begin && split < g.reg[r].split_begin + g.reg[r].nsplit) ri = r;
    const int y0 = g.reg[ri].y0, x0 = g.reg[ri].x0, rh = g.reg[ri].rh, rw = g.reg[ri].rw;
    const int npix = g.B * rh * rw;
    const int r_begin = (split - g.reg[ri].split_begin) * g.rps;
    const int r_end = min(npix, r_begin + g.rps);

    // what this thread stages per panel: 4 consecutive channels of one shifted pixel
    int f_off[NSLOT], f_dy[NSLOT], f_dx[NSLOT];
    bool slot_on[NSLOT], f_ok[NSLOT];
#pragma unroll
    for (int s = 0; s < NSLOT; ++s) {
        int dy = 0, dx = 0, c;
        bool ok;
        if (s == 0) {
            c = rb * BLK + 4 * q;
            ok = c < g.Cin;
            slot_on[s] = true;
        } else {
            const int cb = 4 * ci + (s - 1);
            const int f = cb * BLK + 4 * q;
            slot_on[s] = cb < g.nbc;
            ok = slot_on[s] && f < g.F;
            const int di = ok ? f / g.Cin : 0;
            c = ok ? f - di * g.Cin : 0;
            diff_of(di, g.kw, &dy, &dx);
        }
        f_off[s] = (dy * g.W + dx) * g.Cin + (ok ? c : 0);
        f_dy[s] = dy; f_dx[s] = dx; f_ok[s] = ok;
    }
    const bool sums = ci == 0;
    float4 ssum = make_float4(0.f, 0.f, 0.f, 0.f);

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
    const bool active = 4 * ci + wave < g.nbc;
    const int sb = 1 + wave;
    const int half = lane >> 5, l32 = lane & 31;

    // Position of this thread's pixel in the first chunk, and the step from chunk to chunk.  `base` is the element index
    // of the pixel's first channel (the whole activation has fewer than 2^31 elements) and moves by precomputed steps,
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
    // no divergent branches around the loads.
    float4 pre[NSLOT];
    unsigned okmask = 0;
    auto load_chunk = [&]() {
        const int y = y0 + yy, x = x0 + xx;
        const bool row_ok = r < r_end;
        okmask = 0;
#pragma unroll
        for (int s = 0; s < NSLOT; ++s) {
            if (!slot_on[s]) continue;
            const bool ok = row_ok && f_ok[s] && (unsigned)(y + f_dy[s]) < (unsigned)g.H && (unsigned)(x + f_dx[s]) < (unsigned)g.W;
            const int idx = ok ? base + f_off[s] : 0;
            pre[s] = *reinterpret_cast<const float4*>(X + idx);
            okmask |= (ok ? 1u : 0u) << s;
        }
    };
    auto advance = [&]() {
        r += KT;
        base += step; yy += adv_y; xx += adv_x;
        if (xx >= rw) { xx -= rw; ++yy; base += wrap_x; }
        if (yy >= rh) { yy -= rh; base += wrap_y; }
    };
    auto store_chunk = [&](int buf) {
        const int pos = (4 * q + ((k & 1) << 5)) & 63;
#pragma unroll
        for (int s = 0; s < NSLOT; ++s) {
            if (!slot_on[s]) continue;
            const bool ok = (okmask >> s) & 1u;
            float4 v;
            v.x = ok ? pre[s].x : 0.f; v.y = ok ? pre[s].y : 0.f; v.z = ok ? pre[s].z : 0.f; v.w = ok ? pre[s].w : 0.f;
            *reinterpret_cast<float4*>(&sm.tile[buf][s][k][pos]) = v;
            if (s == 0 && sums) { ssum.x += v.x; ssum.y += v.y; ssum.z += v.z; ssum.w += v.w; }
        }
    };

    const int nchunks = (r_end - r_begin + KT - 1) / KT;
    if (nchunks > 0) {
        load_chunk();
        store_chunk(0);
    }
    __syncthreads();
    // the loop exists with and without the matrix instructions: a wavefront without a block keeps staging and meeting
    // the barriers, and the accumulators of the others never sit behind a branch
    auto run = [&](auto with_mfma) {
        for (int c = 0; c < nchunks; ++c) {
            const int buf = c & 1;
            const bool more = c + 1 < nchunks;
            if (more) { advance(); load_chunk(); }
            if constexpr (decltype(with_mfma)::value) {
                const float* ta_base = &sm.tile[buf][0][0][0];
                const float* tb_base = &sm.tile[buf][sb][0][0];
#pragma unroll
                for (int k0 = 0; k0 < KT; k0 += 2) {
                    const int kk = k0 + half;
                    const int rot = half << 5;
                    float a[2], b[2];
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        a[t] = ta_base[kk * BLK + ((32 * t + l32 + rot) & 63)];
                        b[t] = tb_base[kk * BLK + ((32 * t + l32 + rot) & 63)];
                    }
#pragma unroll
                    for (int ta = 0; ta < 2; ++ta)
#pragma unroll
                        for (int tb = 0; tb < 2; ++tb)
                            acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta], b[tb], acc[ta][tb], 0, 0, 0);
                }
            }
            if (more) store_chunk(buf ^ 1);
            __syncthreads();
        }
    };
    if (active) run(std::true_type{}); else run(std::false_type{});

    if (active) {
        float* dst = part + (((size_t)split * g.nitems + item_idx) * 4 + wave) * (BLK * BLK);
#pragma unroll
        for (int ta = 0; ta < 2; ++ta)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = 32 * ta + 8 * (i >> 2) + 4 * half + (i & 3);
                    const int col = 32 * tb + l32;
                    dst[row * BLK + col] = acc[ta][tb][i];
                }
    }
    if (sums) {
        // channel sums of the row panel: 16 pixel-threads share a channel quad; combine through LDS (the tiles are dead)
        float* red = &sm.tile[0][0][0][0];
        *reinterpret_cast<float4*>(&red[k * 64 + 4 * q]) = ssum;
        __syncthreads();
        if (wave == 0) {
            float v = 0.f;
#pragma unroll
            for (int kk = 0; kk < 16; ++kk) v += red[kk * 64 + lane];
            spart[((size_t)split * g.nbr + rb) * BLK + lane] = v;
        }
    }
}

// R_r = sum of the partial blocks over the ranges of region r, float64; the last nreg * nbr workgroups do the same for
// the channel sums
__global__ __launch_bounds__(256) void shift_region_reduce_kernel(ShiftGeom g, const float* __restrict__ part, const float* __restrict__ spart,
                                                                  double* __restrict__ Rr, double* __restrict__ Sr) {
    __shared__ double red[4][64];
    const int per_reg = g.nitems * 4 * 16;
    const int nblk = g.nreg * per_reg;
    if ((int)blockIdx.x >= nblk) {
        const int idx = (int)blockIdx.x - nblk;
        const int ri = idx / g.nbr, rb = idx - ri * g.nbr;
        const int ln = threadIdx.x & 63, grp = threadIdx.x >> 6;
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
    const int blk = rem >> 4;                         // (item, wavefront)
    const int e = ((rem & 15) << 8) + threadIdx.x;    // element of the 64x64 block
    const int item_idx = blk >> 2, wave = blk & 3;
    const int ci = item_idx % g.ipr;
    if (4 * ci + wave >= g.nbc) return;
    const int s0 = g.reg[ri].split_begin, s1 = s0 + g.reg[ri].nsplit;
    const size_t stride = (size_t)g.nitems * 4 * BLK * BLK;
    const float* src = part + (size_t)blk * (BLK * BLK) + e;
    double v = 0.0;
    int sp = s0;
    for (; sp + 8 <= s1; sp += 8) {
        float x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = src[(size_t)(sp + j) * stride];
#pragma unroll
        for (int j = 0; j < 8; ++j) v += (double)x[j];
    }
    for (; sp < s1; ++sp) v += (double)src[(size_t)sp * stride];
    Rr[(size_t)ri * stride + (size_t)blk * (BLK * BLK) + e] = v;
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
    const int f = diff_index(dy, dx, g.kw) * g.Cin + c2;
    const int rb = c1 >> 6, cb = f >> 6;
    const int item_idx = rb * g.ipr + (cb >> 2), wave = cb & 3;
    const size_t stride = (size_t)g.nitems * 4 * BLK * BLK;
    const size_t idx = ((size_t)item_idx * 4 + wave) * (BLK * BLK) + (size_t)(c1 & 63) * BLK + (f & 63);
    double v = 0.0;
    for (int r = 0; r < g.nreg; ++r)
        if (((g.reg[r].rowmask >> t1y) & 1) && ((g.reg[r].colmask >> t1x) & 1)) v += Rr[(size_t)r * stride + idx];
    float* dst = A + (size_t)i * g.M + j;
    *dst = (float)((double)*dst + v);
}

// bands of one axis: maximal runs of coordinates that serve the same set of taps
struct Band { int begin, len, mask; };
int make_bands(int H, int k, int pad, int Ho, Band* out, int cap) {
    int n = 0;
    int y = 0;
    auto mask_of = [&](int yy) {
        int m = 0;
        for (int t = 0; t < k; ++t) {
            const int p = yy - t + pad;
            if (p >= 0 && p <= Ho - 1) m |= 1 << t;
        }
        return m;
    };
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

struct ShiftWs { size_t part, spart, Rr, Sr, total; };
ShiftWs shift_ws_layout(const ShiftGeom& g) {
    ShiftWs L;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o += align_up(bytes, 256); return at; };
    const size_t blocks = (size_t)g.nitems * 4 * BLK * BLK;
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
    g->ipr = (g->nbc + 3) / 4;
    g->nitems = g->nbr * g->ipr;
    g->kkc = lay == FW_LAYOUT_NHWC_KKC ? 1 : 0;
    // fewer 64x64 block products than the lower triangle of the direct form (idle wavefronts of a ragged last item
    // counted at half weight)
    const long long nb = (M + BLK - 1) / BLK;
    const double direct = 0.5 * (double)nb * (double)(nb + 1);
    const double shifted = (double)g->nbr * (0.5 * g->nbc + 0.5 * 4 * g->ipr);
    if (shifted * 1.1 >= direct) return false;
    Band rows[8 * 2], cols[8 * 2];
    const int nr = make_bands(d->H, d->kh, d->pad, g->Ho, rows, 16), nc = make_bands(d->W, d->kw, d->pad, g->Wo, cols, 16);
    if (nr <= 0 || nc <= 0 || nr * nc > MAXREG) return false;
    g->nreg = nr * nc;
    // pixel ranges: three workgroups are resident per compute unit, and the grid should fit in ONE such round (a
    // workgroup that starts late runs almost alone and is bound by latency).  Ranges never cross a region, so the count
    // is found by shrinking the target until the rounded-up ranges of all regions fit; at least four chunks per range.
    const long long capacity = (256 * 3) / g->nitems;
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
    hipLaunchKernelGGL(shift_partial_f32_kernel, dim3(8 * g.nitems * ((g.nsplit + 7) / 8)), dim3(256), 0, st, X, g, part, spart);
    FW_LAUNCH_CHECK();
    hipLaunchKernelGGL(shift_region_reduce_kernel, dim3(g.nreg * g.nitems * 4 * 16 + g.nreg * g.nbr), dim3(256), 0, st, g, part, spart, Rr, Sr);
    FW_LAUNCH_CHECK();
    hipLaunchKernelGGL(shift_assemble_kernel, dim3((g.M + 255) / 256, g.M + 1), dim3(256), 0, st, g, Rr, Sr, A, s);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
