// Moment accumulation (the block sums of Sec. 2, eqs. (vmuxi)/(vPhixi), and Sec. 4.1, eq. (phixmi)) and the
// block-moment epilogue, for gfx950.
//
// A += X^T X over the patch rows of a layer input is a symmetric rank-N_rows update.  The output is cut into
// 64x64 blocks of the lower triangle; one wavefront owns one block (2x2 MFMA 32x32 tiles) and four wavefronts
// that share operand panels form a workgroup.  The reduction axis (patch rows) is split across workgroups;
// partial blocks go to the workspace and a second kernel sums them in float64 and adds them into A.
// Patch rows are never materialised: every staged element is gathered from the activation tensor through a
// per-row table (image, top-left corner) and a per-feature offset (tap, channel), zero outside the image.
//
// Internally features are ordered tap-major / channel-minor for NHWC and ROWS inputs so that consecutive lanes
// read consecutive channels; the reduce kernel maps back to the external order m = (c*kh + ky)*kw + kx, or keeps the
// internal order when the caller asked for it (FW_LAYOUT_NHWC_KKC).
#include "fw_internal.h"
#include <atomic>
#include <type_traits>

namespace fw {
namespace {

constexpr int BLK = 64;        // features per operand panel = edge of a wavefront's output block
constexpr int MAX_SLOTS = 5;   // operand panels a workgroup may stage
constexpr int KT_F32 = 16;     // patch rows per staged chunk, float32 path

struct CovGeom {
    int n_rows, M, nb;
    int B, Cin, H, W, kh, kw, stride, pad, Ho, Wo;
    int layout;
    int rows_per_split, nsplit;
    int n0, n1, n2, nitems;
    int adv_b, adv_y, adv_x;  // a chunk of KT_F32 rows ahead = adv_b images + adv_y output rows + adv_x output columns
};

struct Item {
    int slot_blk[MAX_SLOTS];  // 64-feature block staged in each LDS slot, -1 = unused
    int ja[4], jb[4];         // per wavefront: slots of the row panel and the column panel of its block, -1 = idle
    int summask;              // slots whose column sums this workgroup accumulates
};

// Closed-form enumeration of workgroup items covering every 64x64 block (bi >= bj) of the lower triangle once.
// h = nb/2 is the number of 128-blocks; with an odd number of 64-blocks the last block row r = nb-1 is left over.
//  type 0: 2x2 squares of blocks strictly below the diagonal of the 128-block grid (4 blocks, 4 panels)
//  type 1: diagonal 128-block I: (2I,2I), (2I+1,2I), (2I+1,2I+1) and, if nb is odd, (r,2I) for the fourth wavefront
//  type 2: (nb odd) what is left of row r: (r,r), (r,1), (r,3), ..., (r,2h-1), four per item
__device__ __host__ inline Item get_item(int idx, int nb) {
    Item it;
    for (int i = 0; i < MAX_SLOTS; ++i) it.slot_blk[i] = -1;
    for (int w = 0; w < 4; ++w) it.ja[w] = it.jb[w] = -1;
    it.summask = 0;
    const int h = nb >> 1;
    const bool odd = nb & 1;
    const int r = nb - 1;
    const int n0 = h * (h - 1) / 2, n1 = h;
    if (idx < n0) {
        int I = 1;
        while ((I + 1) * I / 2 <= idx) ++I;  // I*(I-1)/2 <= idx < (I+1)*I/2
        const int J = idx - I * (I - 1) / 2;
        it.slot_blk[0] = 2 * I; it.slot_blk[1] = 2 * I + 1; it.slot_blk[2] = 2 * J; it.slot_blk[3] = 2 * J + 1;
        it.ja[0] = 0; it.jb[0] = 2;
        it.ja[1] = 0; it.jb[1] = 3;
        it.ja[2] = 1; it.jb[2] = 2;
        it.ja[3] = 1; it.jb[3] = 3;
    } else if (idx < n0 + n1) {
        const int I = idx - n0;
        it.slot_blk[0] = 2 * I; it.slot_blk[1] = 2 * I + 1;
        it.ja[0] = 0; it.jb[0] = 0;
        it.ja[1] = 1; it.jb[1] = 0;
        it.ja[2] = 1; it.jb[2] = 1;
        if (odd) { it.slot_blk[2] = r; it.ja[3] = 2; it.jb[3] = 0; }
        it.summask = 3;
    } else {
        const int K = idx - n0 - n1;
        it.slot_blk[0] = r;
        for (int w = 0; w < 4; ++w) {
            const int li = 4 * K + w;  // position in the list (r,r), (r,1), (r,3), ..., (r,2h-1)
            if (li > h) break;
            if (li == 0) { it.ja[w] = 0; it.jb[w] = 0; }
            else { it.slot_blk[1 + w] = 2 * (li - 1) + 1; it.ja[w] = 0; it.jb[w] = 1 + w; }
        }
        if (K == 0) it.summask = 1;
    }
    return it;
}

// selection by compare chain: keeps the item in scalar registers (a dynamically indexed array would go to scratch)
__device__ __forceinline__ int pick4(const int* a, int w) { return w == 0 ? a[0] : w == 1 ? a[1] : w == 2 ? a[2] : a[3]; }
__device__ __forceinline__ int pick_slot(const Item& it, int s) {
    return s == 0 ? it.slot_blk[0] : s == 1 ? it.slot_blk[1] : s == 2 ? it.slot_blk[2] : s == 3 ? it.slot_blk[3] : it.slot_blk[4];
}

inline void item_counts(int nb, int* n0, int* n1, int* n2) {
    const int h = nb >> 1;
    *n0 = h * (h - 1) / 2;
    *n1 = h;
    *n2 = (nb & 1) ? (h + 1 + 3) / 4 : 0;
}

// internal feature index -> (offset inside a patch, ky, kx, external feature index)
struct Feat { int off, ky, kx, ext; };
__device__ __forceinline__ Feat feat_of(int fi, const CovGeom& g) {
    Feat f;
    if (g.layout == FW_LAYOUT_NCHW) {
        const int kk = g.kh * g.kw;
        const int c = fi / kk, t = fi - c * kk;
        f.ky = t / g.kw; f.kx = t - f.ky * g.kw;
        f.off = (c * g.H + f.ky) * g.W + f.kx;
        f.ext = fi;
    } else {  // NHWC and ROWS: tap-major, channel-minor
        const int t = fi / g.Cin, c = fi - t * g.Cin;
        f.ky = t / g.kw; f.kx = t - f.ky * g.kw;
        f.off = (f.ky * g.W + f.kx) * g.Cin + c;
        f.ext = g.layout == FW_LAYOUT_NHWC_KKC ? fi : c * (g.kh * g.kw) + t;
    }
    return f;
}

struct RowInfo { long long base; int iy0, ix0; };

__device__ __forceinline__ RowInfo row_of(int r, bool valid, const CovGeom& g) {
    RowInfo ri;
    if (!valid) { ri.base = 0; ri.iy0 = -(1 << 28); ri.ix0 = -(1 << 28); return ri; }
    const int P = g.Ho * g.Wo;
    const int b = r / P, p = r - b * P;
    const int oy = p / g.Wo, ox = p - oy * g.Wo;
    ri.iy0 = oy * g.stride - g.pad;
    ri.ix0 = ox * g.stride - g.pad;
    if (g.layout == FW_LAYOUT_NCHW)
        ri.base = ((long long)b * g.Cin * g.H + ri.iy0) * g.W + ri.ix0;
    else
        ri.base = (((long long)b * g.H + ri.iy0) * g.W + ri.ix0) * g.Cin;
    return ri;
}

struct Smem {
    alignas(16) float tile[MAX_SLOTS][KT_F32][BLK];  // [slot][row][feature], feature position rotated by 32 on odd rows
    RowInfo rows[KT_F32];
};

// Generic float32 path (any layout, any Cin): one element per load through a per-row table.  bfloat16 inputs take
// the packed-tile path of cov_bf16.hip.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 2))) void cov_partial_kernel(const float* __restrict__ X, CovGeom g, float* __restrict__ part,
                                                          float* __restrict__ spart) {
    constexpr int KT = KT_F32;
    __shared__ Smem sm;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int item_idx = blockIdx.x, split = blockIdx.y;
    const Item it = get_item(item_idx, g.nb);

    // this thread stages feature `lane` of every slot, rows wave, wave+4, ...
    int f_off[MAX_SLOTS], f_ky[MAX_SLOTS], f_kx[MAX_SLOTS];
    bool f_ok[MAX_SLOTS];
#pragma unroll
    for (int s = 0; s < MAX_SLOTS; ++s) {
        const int fi = it.slot_blk[s] * BLK + lane;
        f_ok[s] = it.slot_blk[s] >= 0 && fi < g.M;
        Feat f = feat_of(f_ok[s] ? fi : 0, g);
        f_off[s] = f.off; f_ky[s] = f.ky; f_kx[s] = f.kx;
    }
    float ssum[MAX_SLOTS];
#pragma unroll
    for (int s = 0; s < MAX_SLOTS; ++s) ssum[s] = 0.f;

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    const int sa = pick4(it.ja, wave), sb = pick4(it.jb, wave);
    const int r_begin = split * g.rows_per_split;
    const int r_end = min(g.n_rows, r_begin + g.rows_per_split);
    const int half = lane >> 5, l32 = lane & 31;

    for (int r0 = r_begin; r0 < r_end; r0 += KT) {
        if (tid < KT) sm.rows[tid] = row_of(r0 + tid, r0 + tid < r_end, g);
        __syncthreads();
#pragma unroll
        for (int s = 0; s < MAX_SLOTS; ++s) {
            if (it.slot_blk[s] < 0) continue;
#pragma unroll
            for (int j = 0; j < KT / 4; ++j) {
                const int k = wave + 4 * j;
                const RowInfo ri = sm.rows[k];
                const bool ok = f_ok[s] && (unsigned)(ri.iy0 + f_ky[s]) < (unsigned)g.H &&
                                (unsigned)(ri.ix0 + f_kx[s]) < (unsigned)g.W;
                float v = 0.f;
                if (ok) v = X[ri.base + f_off[s]];
                sm.tile[s][k][(lane + ((k & 1) << 5)) & 63] = v;
                ssum[s] += v;
            }
        }
        __syncthreads();
        if (sa >= 0) {
            {
#pragma unroll
                for (int k0 = 0; k0 < KT; k0 += 2) {
                    const int k = k0 + half;
                    const int rot = (k & 1) << 5;
                    float a[2], b[2];
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        a[t] = sm.tile[sa][k][(32 * t + l32 + rot) & 63];
                        b[t] = sm.tile[sb][k][(32 * t + l32 + rot) & 63];
                    }
#pragma unroll
                    for (int ta = 0; ta < 2; ++ta)
#pragma unroll
                        for (int tb = 0; tb < 2; ++tb)
                            acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta], b[tb], acc[ta][tb], 0, 0, 0);
                }
            }
        }
    }

    // partial 64x64 block of this wavefront: element (i, j) = sum over this split's rows of x_i x_j
    if (sa >= 0) {
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
    // column sums: combine the four row groups through LDS
    if (it.summask) {
        __syncthreads();
        float* red = reinterpret_cast<float*>(&sm.tile[0][0][0]);  // [slot][wave][lane]
#pragma unroll
        for (int s = 0; s < MAX_SLOTS; ++s)
            if ((it.summask >> s) & 1) red[(s * 4 + wave) * 64 + lane] = ssum[s];
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int s = 0; s < MAX_SLOTS; ++s)
                if ((it.summask >> s) & 1) {
                    const float v = red[(s * 4 + 0) * 64 + lane] + red[(s * 4 + 1) * 64 + lane] +
                                    red[(s * 4 + 2) * 64 + lane] + red[(s * 4 + 3) * 64 + lane];
                    spart[(size_t)split * g.nb * BLK + it.slot_blk[s] * BLK + lane] = v;
                }
        }
    }
}

// ------------------------------------------------------------------------------------------------------------
// float32 fast path: NHWC / ROWS inputs with Cin % 4 == 0.  In the internal (tap-major, channel-minor) feature order
// four consecutive features are four consecutive channels of one tap, i.e. 16 contiguous bytes of the activation.
// Thread (k = tid / 16, q = tid % 16) stages features 4q..4q+3 of row k of every panel with one 16-byte load; its
// row position (image, oy, ox) is advanced incrementally from chunk to chunk.  Loads for chunk c+1 are issued before
// the MFMAs of chunk c and written to the other LDS buffer afterwards, so a chunk costs one barrier.
struct SmemVec {
    alignas(16) float tile[2][MAX_SLOTS][KT_F32][BLK];
};

__global__ __launch_bounds__(256) void cov_partial_f32v4_kernel(const float* __restrict__ X, CovGeom g, float* __restrict__ part,
                                                                float* __restrict__ spart) {
    constexpr int KT = KT_F32;
    __shared__ SmemVec sm;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroups go to the 8 XCDs round-robin by linear index; give every XCD whole row ranges (all items of a
    // split), so that a range of the activation is pulled into one L2 only.
    const int item_idx = (blockIdx.x >> 3) % g.nitems;
    const int split = (blockIdx.x & 7) + 8 * ((blockIdx.x >> 3) / g.nitems);
    if (split >= g.nsplit) return;
    const Item it = get_item(item_idx, g.nb);
    const int k = tid >> 4, q = tid & 15;

    int f_off[MAX_SLOTS], f_tap[MAX_SLOTS];  // tap packed as ky << 16 | kx; -1 = nothing to stage
#pragma unroll
    for (int s = 0; s < MAX_SLOTS; ++s) {
        const int fi = it.slot_blk[s] * BLK + 4 * q;
        const bool ok = it.slot_blk[s] >= 0 && fi < g.M;
        Feat f = feat_of(ok ? fi : 0, g);
        f_off[s] = f.off;
        f_tap[s] = ok ? ((f.ky << 16) | f.kx) : -1;
    }
    float4 ssum[2];  // column sums are only ever asked for panels 0 and 1
    ssum[0] = ssum[1] = make_float4(0.f, 0.f, 0.f, 0.f);

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    const int sa = pick4(it.ja, wave), sb = pick4(it.jb, wave);
    const int r_begin = split * g.rows_per_split;
    const int r_end = min(g.n_rows, r_begin + g.rows_per_split);
    const int half = lane >> 5, l32 = lane & 31;

    // position of this thread's row in the first chunk
    int r = r_begin + k;
    int rb, oy, ox;
    {
        const int P = g.Ho * g.Wo;
        rb = r / P;
        const int p = r - rb * P;
        oy = p / g.Wo;
        ox = p - oy * g.Wo;
    }
    float4 pre[MAX_SLOTS];
    auto load_chunk = [&]() {
        const int iy0 = oy * g.stride - g.pad, ix0 = ox * g.stride - g.pad;
        const long long base = (((long long)rb * g.H + iy0) * g.W + ix0) * g.Cin;
        const bool row_ok = r < r_end;
#pragma unroll
        for (int s = 0; s < MAX_SLOTS; ++s) {
            pre[s] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (it.slot_blk[s] < 0) continue;
            const bool ok = row_ok && f_tap[s] >= 0 && (unsigned)(iy0 + (f_tap[s] >> 16)) < (unsigned)g.H &&
                            (unsigned)(ix0 + (f_tap[s] & 0xffff)) < (unsigned)g.W;
            if (ok) pre[s] = *reinterpret_cast<const float4*>(X + base + f_off[s]);
        }
    };
    auto advance = [&]() {
        r += KT;
        rb += g.adv_b; oy += g.adv_y; ox += g.adv_x;
        if (ox >= g.Wo) { ox -= g.Wo; ++oy; }
        if (oy >= g.Ho) { oy -= g.Ho; ++rb; }
    };
    auto store_chunk = [&](int buf) {
        const int pos = (4 * q + ((k & 1) << 5)) & 63;
#pragma unroll
        for (int s = 0; s < MAX_SLOTS; ++s) {
            if (it.slot_blk[s] < 0) continue;
            *reinterpret_cast<float4*>(&sm.tile[buf][s][k][pos]) = pre[s];
            if (s < 2 && ((it.summask >> s) & 1)) {
                ssum[s].x += pre[s].x; ssum[s].y += pre[s].y; ssum[s].z += pre[s].z; ssum[s].w += pre[s].w;
            }
        }
    };

    const int nchunks = (r_end - r_begin + KT - 1) / KT;
    if (nchunks > 0) {
        load_chunk();
        store_chunk(0);
    }
    __syncthreads();
    // The loop exists twice, with and without the matrix instructions, so that a wavefront without a block keeps
    // staging and meeting the barriers while the accumulators of the others never sit behind a branch.
    auto run = [&](auto active) {
        for (int c = 0; c < nchunks; ++c) {
            const int buf = c & 1;
            const bool more = c + 1 < nchunks;
            if (more) { advance(); load_chunk(); }
            if constexpr (decltype(active)::value) {
                const float* ta_base = &sm.tile[buf][sa][0][0];
                const float* tb_base = &sm.tile[buf][sb][0][0];
#pragma unroll
                for (int k0 = 0; k0 < KT; k0 += 2) {
                    const int kk = k0 + half;
                    const int rot = half << 5;  // k0 is even, so the parity of the row is `half`
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
    if (sa >= 0) run(std::true_type{}); else run(std::false_type{});

    if (sa >= 0) {
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
    if (it.summask) {
        // column sums: 16 row-threads share a feature quad; combine them through LDS (the tiles are dead by now)
        float* red = &sm.tile[0][0][0][0];  // [slot][k][64 features]
#pragma unroll
        for (int s = 0; s < 2; ++s)
            if ((it.summask >> s) & 1) *reinterpret_cast<float4*>(&red[(s * 16 + k) * 64 + 4 * q]) = ssum[s];
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
                if ((it.summask >> s) & 1) {
                    float v = 0.f;
#pragma unroll
                    for (int kk = 0; kk < 16; ++kk) v += red[(s * 16 + kk) * 64 + lane];
                    spart[(size_t)split * g.nb * BLK + it.slot_blk[s] * BLK + lane] = v;
                }
        }
    }
}

// Sum of the partial blocks over the row ranges in float64, added into A in the caller's feature order: one thread per
// element, the loads of eight ranges in flight at a time.  The last (M+63)/64 workgroups do the same for the column
// sums: 64 features each, the ranges dealt to four groups of threads and combined through LDS.
__global__ __launch_bounds__(256) void cov_reduce_kernel(CovGeom g, const float* __restrict__ part, const float* __restrict__ spart,
                                                         float* __restrict__ A, float* __restrict__ s) {
    __shared__ double red[4][64];
    const int nblk = g.nitems * 4 * 16;
    if ((int)blockIdx.x >= nblk) {
        const int f = ((int)blockIdx.x - nblk) * 64 + (threadIdx.x & 63), grp = threadIdx.x >> 6;
        double v = 0.0;
        if (f < g.M)
            for (int sp = grp; sp < g.nsplit; sp += 4) v += (double)spart[(size_t)sp * g.nb * BLK + f];
        red[grp][threadIdx.x & 63] = v;
        __syncthreads();
        if (grp == 0 && f < g.M) {
            v = red[0][threadIdx.x] + red[1][threadIdx.x] + red[2][threadIdx.x] + red[3][threadIdx.x];
            const int e = feat_of(f, g).ext;
            s[e] = (float)((double)s[e] + v);
        }
        return;
    }
    const int blk = blockIdx.x >> 4;                       // (item, wavefront)
    const int e = ((blockIdx.x & 15) << 8) + threadIdx.x;  // element of the 64x64 block
    const int item_idx = blk >> 2, wave = blk & 3;
    const Item it = get_item(item_idx, g.nb);
    const int ja = pick4(it.ja, wave), jb = pick4(it.jb, wave);
    if (ja < 0) return;
    const int bi = pick_slot(it, ja), bj = pick_slot(it, jb);
    const int row = e >> 6, col = e & 63;
    const int fi = bi * BLK + row, fj = bj * BLK + col;
    if (fi >= g.M || fj >= g.M) return;
    if (bi == bj && row < col) return;  // diagonal block: its upper half duplicates the lower
    const size_t stride = (size_t)g.nitems * 4 * BLK * BLK;
    const float* src = part + (size_t)blk * (BLK * BLK) + e;
    double v = 0.0;
    int sp = 0;
    for (; sp + 8 <= g.nsplit; sp += 8) {
        float x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = src[(size_t)(sp + j) * stride];
#pragma unroll
        for (int j = 0; j < 8; ++j) v += (double)x[j];
    }
    for (; sp < g.nsplit; ++sp) v += (double)src[(size_t)sp * stride];
    const int ei = feat_of(fi, g).ext, ej = feat_of(fj, g).ext;
    const int hi = max(ei, ej), lo = min(ei, ej);
    float* dst = A + (size_t)hi * g.M + lo;
    *dst = (float)((double)*dst + v);
}

bool make_geom(const fw_conv_desc* d, fw_dtype dt, fw_layout lay, CovGeom* g) {
    g->B = d->B; g->Cin = d->Cin; g->H = d->H; g->W = d->W;
    g->kh = d->kh; g->kw = d->kw; g->stride = d->stride; g->pad = d->pad;
    g->layout = (int)lay;
    g->Ho = (d->H + 2 * d->pad - d->kh) / d->stride + 1;
    g->Wo = (d->W + 2 * d->pad - d->kw) / d->stride + 1;
    const long long n_rows = (long long)d->B * g->Ho * g->Wo;
    const long long M = (long long)d->Cin * d->kh * d->kw;
    if (n_rows <= 0 || n_rows >= (1ll << 31) || M <= 0 || M > 16384) return false;
    if ((long long)d->B * d->Cin * d->H * d->W >= (1ll << 31)) return false;
    g->n_rows = (int)n_rows; g->M = (int)M; g->nb = (int)((M + BLK - 1) / BLK);
    item_counts(g->nb, &g->n0, &g->n1, &g->n2);
    g->nitems = g->n0 + g->n1 + g->n2;
    const int KT = KT_F32;
    // Split the rows so that the grid is close to a whole number of resident rounds: 256 compute units times the
    // workgroups one of them holds (LDS-limited), with at least four chunks of rows per split.
    const long long capacity = 256 * 3;
    long long want = capacity / g->nitems;
    const long long max_split = (n_rows + 4 * KT - 1) / (4 * KT);
    if (want > max_split) want = max_split;
    if (want < 1) want = 1;
    long long rps = (n_rows + want - 1) / want;
    rps = (rps + KT - 1) / KT * KT;
    g->rows_per_split = (int)rps;
    g->nsplit = (int)((n_rows + rps - 1) / rps);
    const int P = g->Ho * g->Wo;
    g->adv_b = KT_F32 / P;
    g->adv_y = (KT_F32 % P) / g->Wo;
    g->adv_x = (KT_F32 % P) % g->Wo;
    return true;
}

// mu, phi_x (updated in place AFTER finalize_phi_kernel has consumed the old mean) and lambda_bar = mean(phi_x): one
// workgroup
__global__ __launch_bounds__(1024) void finalize_vec_kernel(const float* __restrict__ A, const float* __restrict__ s, double inv_n, int M,
                                                            float alpha, int first, float* __restrict__ mu, float* __restrict__ phi,
                                                            float* __restrict__ lambda_bar) {
    __shared__ double red[16];
    double sum = 0.0;
    for (int i = threadIdx.x; i < M; i += 1024) {
        const double mh = (double)s[i] * inv_n;
        const double raw = (double)A[(size_t)i * M + i] * inv_n;
        double m, p;
        if (first) { m = mh; p = raw; }
        else {
            m = (double)alpha * (double)mu[i] + (1.0 - (double)alpha) * mh;
            p = (double)alpha * (double)phi[i] + (1.0 - (double)alpha) * raw;
        }
        const float pf = (float)p;
        mu[i] = (float)m;
        phi[i] = pf;
        sum += (double)pf;
    }
    sum = wave_sum(sum);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < 16; ++w) t += red[w];
        *lambda_bar = (float)(t / (double)M);
    }
}

// Covariance centred on the updated mean, expanded into the raw sums (float64 per element):
//   C_ij = A_ij/n - mhat_i mu_j - mu_i mhat_j + mu_i mu_j,  mhat = s/n,  mu = alpha*mu_old + (1-alpha)*mhat.
// A workgroup takes a 32x32 tile (I, J) of the lower triangle: rows of 32 lanes read A and the old Phi_x and write the
// new values; the mirrored tile (J, I) is written from a transposed copy in LDS, again along rows.
__global__ __launch_bounds__(256) void finalize_phi_kernel(const float* __restrict__ A, const float* __restrict__ s,
                                                           const float* __restrict__ mu_old, double inv_n, int M, float alpha,
                                                           int first, float* __restrict__ Phi) {
    const int I = blockIdx.y, J = blockIdx.x;
    if (J > I) return;
    __shared__ float tr[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int j = J * 32 + tx;
    double mhj = 0.0, mj = 0.0;
    if (j < M) {
        mhj = (double)s[j] * inv_n;
        mj = first ? mhj : (double)alpha * (double)mu_old[j] + (1.0 - (double)alpha) * mhj;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int yy = ty + 8 * r;
        const int i = I * 32 + yy;
        float o = 0.f;
        if (i < M && j < M && j <= i) {
            const double mhi = (double)s[i] * inv_n;
            const double mi = first ? mhi : (double)alpha * (double)mu_old[i] + (1.0 - (double)alpha) * mhi;
            double c = (double)A[(size_t)i * M + j] * inv_n - mhi * mj - mi * mhj + mi * mj;
            if (!first) c = (double)alpha * (double)Phi[(size_t)i * M + j] + (1.0 - (double)alpha) * c;
            o = (float)c;
            Phi[(size_t)i * M + j] = o;
        }
        tr[yy][tx] = o;
    }
    __syncthreads();
    // mirror: element (J*32 + yy, I*32 + tx) = tile element (tx, yy); on a diagonal tile only the part above the diagonal
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int yy = ty + 8 * r;
        const int mi_row = J * 32 + yy, mj_col = I * 32 + tx;
        if (mi_row < M && mj_col < M && mj_col > mi_row) Phi[(size_t)mi_row * M + mj_col] = tr[tx][yy];
    }
}

// The same for M a multiple of 4, on 64x64 tiles with 16-byte accesses: thread (ty, tx) takes rows ty, ty + 16, ty + 32,
// ty + 48 and columns 4 tx .. 4 tx + 3; all its loads are issued before the first is used.  Off the diagonal the tile is
// stored from registers and its mirror image from a transposed read of LDS; a diagonal tile is stored once, made
// symmetric from its lower half (A holds nothing above the diagonal).
__global__ __launch_bounds__(256) void finalize_phi64_kernel(const float* __restrict__ A, const float* __restrict__ s,
                                                             const float* __restrict__ mu_old, double inv_n, int M, float alpha,
                                                             int first, float* __restrict__ Phi) {
    const int I = blockIdx.y, J = blockIdx.x;
    if (J > I) return;
    __shared__ float tr[64][65];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int j0 = J * 64 + 4 * tx;
    const bool col_ok = j0 < M;
    float4 a[4], ph[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = I * 64 + ty + 16 * r;
        const size_t e = (col_ok && i < M) ? (size_t)i * M + j0 : 0;
        a[r] = *reinterpret_cast<const float4*>(A + e);
        ph[r] = first ? make_float4(0.f, 0.f, 0.f, 0.f) : *reinterpret_cast<const float4*>(Phi + e);
    }
    double mhj[4], mj[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int j = j0 + q;
        mhj[q] = j < M ? (double)s[j] * inv_n : 0.0;
        mj[q] = j < M ? (first ? mhj[q] : (double)alpha * (double)mu_old[j] + (1.0 - (double)alpha) * mhj[q]) : 0.0;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int yy = ty + 16 * r;
        const int i = I * 64 + yy;
        asm volatile("" : "+v"(a[r].x), "+v"(a[r].y), "+v"(a[r].z), "+v"(a[r].w));
        const bool row_ok = col_ok && i < M;
        const double mhi = row_ok ? (double)s[i] * inv_n : 0.0;
        const double mi = first ? mhi : (double)alpha * (double)(row_ok ? mu_old[i] : 0.f) + (1.0 - (double)alpha) * mhi;
        const float av[4] = {a[r].x, a[r].y, a[r].z, a[r].w}, pv[4] = {ph[r].x, ph[r].y, ph[r].z, ph[r].w};
        float o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            double c = (double)av[q] * inv_n - mhi * mj[q] - mi * mhj[q] + mi * mj[q];
            if (!first) c = (double)alpha * (double)pv[q] + (1.0 - (double)alpha) * c;
            o[q] = (row_ok && j0 + q <= i) ? (float)c : 0.f;     // nothing is taken from above the diagonal
            tr[yy][4 * tx + q] = o[q];
        }
        if (I != J && row_ok) *reinterpret_cast<float4*>(Phi + (size_t)i * M + j0) = make_float4(o[0], o[1], o[2], o[3]);
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int yy = ty + 16 * r;
        if (I != J) {
            // mirror image: element (J*64 + yy, I*64 + x) = tile element (x, yy)
            const int row = J * 64 + yy, c0 = I * 64 + 4 * tx;
            if (row < M && c0 < M)
                *reinterpret_cast<float4*>(Phi + (size_t)row * M + c0) =
                    make_float4(tr[4 * tx][yy], tr[4 * tx + 1][yy], tr[4 * tx + 2][yy], tr[4 * tx + 3][yy]);
        } else {
            const int row = I * 64 + yy, c0 = I * 64 + 4 * tx;
            if (row < M && c0 < M) {
                float v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) { const int x = 4 * tx + q; v[q] = x <= yy ? tr[yy][x] : tr[x][yy]; }
                *reinterpret_cast<float4*>(Phi + (size_t)row * M + c0) = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
    }
}

__global__ __launch_bounds__(256) void mirror_lower_kernel(float* __restrict__ A, int M) {
    const int i = blockIdx.y * 16 + threadIdx.y, j = blockIdx.x * 16 + threadIdx.x;
    if (i >= M || j >= M || j >= i) return;
    A[(size_t)j * M + i] = A[(size_t)i * M + j];
}

// [B][C][HW] -> [B][HW][C] through 32x32 LDS tiles: float32 activations in NCHW order are brought into the
// channels-last order that the fast accumulation kernel reads with 16-byte loads
__global__ __launch_bounds__(256) void nchw_to_nhwc_kernel(const float* __restrict__ src, float* __restrict__ dst, int C, int HW) {
    __shared__ float t[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const size_t img = (size_t)blockIdx.z * C * HW;
    const int p0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int c = c0 + ty + 8 * r, p = p0 + tx;
        t[ty + 8 * r][tx] = (c < C && p < HW) ? src[img + (size_t)c * HW + p] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int p = p0 + ty + 8 * r, c = c0 + tx;
        if (p < HW && c < C) dst[img + (size_t)p * C + c] = t[tx][ty + 8 * r];
    }
}

__global__ __launch_bounds__(256) void fill_f32_kernel(float* __restrict__ p, size_t n, float v) {
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256) p[e] = v;
}

// ---- float32 activations on the bfloat16 matrix cores (split form).
// Every value x is written as two bfloat16 numbers, hi = bf16(x) and lo = bf16(x - hi) (hi + lo carries 16 significant
// bits of x, residual at most 2^-17 |x| and of either sign with equal likelihood), taken as a tensor with twice the
// channels, [pixel][hi 0..C-1 | lo 0..C-1] (formed by the packing pre-pass of the bfloat16 kernels as it reads the float32
// tensor: no copy of its own).  The bfloat16 kernels then accumulate the moments of that tensor, and
//     sum x_i x_j  ~  sum (hi_i + lo_i)(hi_j + lo_j)  =  the four blocks (hi,hi) + (hi,lo) + (lo,hi) + (lo,lo)
// of its second moments, which split_fold_kernel adds up: four bfloat16 products per float32 product on a pipe sixteen
// times faster.  The residuals are rounding errors of zero mean, so over N rows their sum grows like sqrt(N) against N
// for the moment itself.
// A[i][j] += the four blocks of A2 (moments of the doubled tensor, features ordered (tap, plane, channel), lower triangle
// valid) that belong to the pair of features (i, j), j <= i, in the caller's order: ckk = 1: m = c * kk + t, else m = t * C + c.
// The last row of workgroups does the same for the column sums.
__global__ __launch_bounds__(256) void split_fold_kernel(const float* __restrict__ A2, const float* __restrict__ s2, int M, int C, int kk,
                                                         int ckk, float* __restrict__ A, float* __restrict__ s) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    auto split_index = [&](int m, int* t, int* c) {
        if (ckk) { *c = m / kk; *t = m - *c * kk; }
        else { *t = m / C; *c = m - *t * C; }
    };
    const int M2 = 2 * M;
    if ((int)blockIdx.y == M) {
        if (j >= M) return;
        int t, c;
        split_index(j, &t, &c);
        s[j] = (float)((double)s[j] + (double)s2[t * 2 * C + c] + (double)s2[t * 2 * C + C + c]);
        return;
    }
    const int i = blockIdx.y;
    if (j > i) return;
    int t1, c1, t2, c2;
    split_index(i, &t1, &c1);
    split_index(j, &t2, &c2);
    double v = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int p = t1 * 2 * C + (k & 1 ? C : 0) + c1, q = t2 * 2 * C + (k & 2 ? C : 0) + c2;
        if (p < q) { const int x = p; p = q; q = x; }      // A2 holds its lower triangle
        v += (double)A2[(size_t)p * M2 + q];
    }
    float* dst = A + (size_t)i * M + j;
    *dst = (float)((double)*dst + v);
}

}  // namespace

fw_status fill_f32(float* p, size_t n, float v, hipStream_t st) {
    size_t b = (n + 255) / 256;
    if (b > 8192) b = 8192;
    if (b == 0) return FW_OK;
    hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)b), dim3(256), 0, st, p, n, v);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

// float32 NCHW input with Cin % 4 == 0 is transposed into the workspace and then treated as NHWC (the feature order
// m = (c*kh + ky)*kw + kx is the same for both tensor layouts)
static bool nchw_through_copy(const fw_conv_desc* d, fw_dtype dt, fw_layout lay) {
    return dt == FW_F32 && lay == FW_LAYOUT_NCHW && (d->Cin % 4) == 0 && d->B <= 65535;
}
static size_t act_copy_bytes(const fw_conv_desc* d) { return align_up((size_t)d->B * d->Cin * d->H * d->W * sizeof(float), 256); }

// The split form (float32 activations as hi + lo bfloat16 planes on the bfloat16 kernels): taken when asked for, or by
// the estimate for layers that are large enough for the matrix cores to matter (the float32 MFMA peak is a sixteenth of
// the bfloat16 one, the split form issues four times the products).  `lay` is the layout after the NCHW copy, if any.
struct SplitPlan { fw_conv_desc d2; fw_layout lay2; size_t a2, s2, inner, total; int ckk; };
static bool split_plan(const fw_conv_desc* d, fw_layout lay, SplitPlan* sp) {
    if (d->form != FW_COV_FORM_AUTO && d->form != FW_COV_FORM_SPLIT) return false;
    if (lay == FW_LAYOUT_NCHW) return false;
    const long long M = (long long)d->Cin * d->kh * d->kw;
    const long long Ho = (d->H + 2 * d->pad - d->kh) / d->stride + 1, Wo = (d->W + 2 * d->pad - d->kw) / d->stride + 1;
    const long long n_rows = (long long)d->B * Ho * Wo;
    if (2 * M > 16384 || (long long)d->B * d->H * d->W * 2 * d->Cin >= (1ll << 31)) return false;
    if (d->form == FW_COV_FORM_AUTO) {
        // Measured break-even against the float32 kernels (rows and 3 x 3 windows alike): the split form pays a fixed
        // price in M^2 (A2 is four times A: filled, accumulated and folded), the float32 kernels lose ground as M grows
        // (64 x 64 blocks re-read their panels per block: 15 TFLOP/s at M = 4608 against 70 at M = 576).
        const long long least_rows = M >= 4096 ? 256 : M >= 2048 ? 1024 : M >= 1024 ? 8192 : M >= 512 ? 32768 : -1;
        if (least_rows < 0 || n_rows < least_rows) return false;
    }
    sp->d2 = *d;
    sp->d2.Cin = 2 * d->Cin;
    sp->d2.form = FW_COV_FORM_AUTO;                       // the bfloat16 kernels choose between their own two forms
    sp->lay2 = lay == FW_LAYOUT_ROWS ? FW_LAYOUT_ROWS : FW_LAYOUT_NHWC_KKC;
    sp->ckk = (lay == FW_LAYOUT_NHWC) ? 1 : 0;             // caller's feature order (c, ky, kx) against the kernels' (ky, kx, c)
    sp->inner = cov_bf16_workspace_bytes(&sp->d2, sp->lay2);
    if (sp->inner == 0) return false;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o += align_up(bytes, 256); return at; };
    sp->a2 = take((size_t)4 * M * M * sizeof(float));
    sp->s2 = take((size_t)2 * M * sizeof(float));
    const size_t in = take(sp->inner);
    sp->inner = in;                                        // from here on: offset of the bfloat16 kernels' own workspace
    sp->total = o;
    return true;
}

size_t cov_workspace_bytes(int /*M*/, const fw_conv_desc* d, fw_dtype dt, fw_layout lay) {
    if (d && cov_skinny_applies(d, lay)) return cov_skinny_workspace_bytes(d, lay);
    if (dt == FW_BF16) return cov_bf16_workspace_bytes(d, lay);
    if (!d) return 0;
    const bool copy = nchw_through_copy(d, dt, lay);
    {
        SplitPlan sp;
        if (split_plan(d, copy ? FW_LAYOUT_NHWC : lay, &sp)) return sp.total + (copy ? act_copy_bytes(d) : 0);
    }
    if (cov_shift_applies(d, copy ? FW_LAYOUT_NHWC : lay))
        return cov_shift_workspace_bytes(d, copy ? FW_LAYOUT_NHWC : lay) + (copy ? act_copy_bytes(d) : 0);
    CovGeom g;
    if (!make_geom(d, dt, copy ? FW_LAYOUT_NHWC : lay, &g)) return 0;
    const size_t part = (size_t)g.nsplit * g.nitems * 4 * BLK * BLK * sizeof(float);
    const size_t sp = (size_t)g.nsplit * g.nb * BLK * sizeof(float);
    return align_up(part, 256) + align_up(sp, 256) + (copy ? act_copy_bytes(d) : 0);
}

bool cov_plan(const fw_conv_desc* d, fw_dtype dt, fw_layout lay, fw_cov_plan* plan) {
    *plan = fw_cov_plan{};
    if (cov_skinny_plan(d, lay, plan)) return true;
    if (dt == FW_BF16) return cov_bf16_plan(d, lay, plan);
    if (nchw_through_copy(d, dt, lay)) lay = FW_LAYOUT_NHWC;
    {
        SplitPlan sp;
        if (split_plan(d, lay, &sp)) {
            if (!cov_bf16_plan(&sp.d2, sp.lay2, plan)) return false;
            plan->split_bf16 = 1;
            return true;
        }
    }
    if (cov_shift_plan(d, lay, plan)) return true;
    CovGeom g;
    if (!make_geom(d, dt, lay, &g)) return false;
    plan->workgroups = g.nitems * g.nsplit; plan->ranges = g.nsplit;
    // 64x64 blocks of the lower triangle, diagonal blocks in full
    plan->mfma_flops_issued = 2.0 * 64.0 * 64.0 * (0.5 * g.nb * (g.nb + 1)) * (double)g.n_rows;
    return true;
}

fw_status cov_accumulate(const void* X, fw_dtype dt, fw_layout lay, const fw_conv_desc* d, float* A, float* s, void* ws,
                         size_t ws_bytes, hipStream_t st) {
    // few features, many rows, 1x1 window: streamed once, no staging (cov_skinny.hip)
    if (cov_skinny_applies(d, lay)) return cov_skinny_accumulate(X, dt, lay, d, A, s, ws, ws_bytes, st);
    if (dt == FW_BF16) return cov_bf16_accumulate(X, lay, d, A, s, ws, ws_bytes, st);
    const bool copy = nchw_through_copy(d, dt, lay);
    if (copy) lay = FW_LAYOUT_NHWC;
    {
        SplitPlan sp;
        if (split_plan(d, lay, &sp)) {
            const size_t need = sp.total + (copy ? act_copy_bytes(d) : 0);
            if (!ws || ws_bytes < need) return FW_ERR_WORKSPACE;
            char* base = reinterpret_cast<char*>(ws);
            if (copy) {
                float* Xc = reinterpret_cast<float*>(base + sp.total);
                const int HW = d->H * d->W;
                hipLaunchKernelGGL(nchw_to_nhwc_kernel, dim3((HW + 31) / 32, (d->Cin + 31) / 32, d->B), dim3(256), 0, st,
                                   reinterpret_cast<const float*>(X), Xc, d->Cin, HW);
                FW_LAUNCH_CHECK();
                X = Xc;
            }
            float* A2 = reinterpret_cast<float*>(base + sp.a2);
            float* s2 = reinterpret_cast<float*>(base + sp.s2);
            const int M = d->Cin * d->kh * d->kw;
            // A2 and s2 lie next to each other (a2 then s2): one fill
            fw_status rc = fill_f32(A2, (sp.s2 - sp.a2) / sizeof(float) + 2 * (size_t)M, 0.f, st);
            if (rc != FW_OK) return rc;
            rc = cov_bf16_accumulate(X, sp.lay2, &sp.d2, A2, s2, base + sp.inner, sp.total - sp.inner, st, true);
            if (rc != FW_OK) return rc;
            hipLaunchKernelGGL(split_fold_kernel, dim3((M + 255) / 256, M + 1), dim3(256), 0, st, A2, s2, M, d->Cin, d->kh * d->kw, sp.ckk, A, s);
            FW_LAUNCH_CHECK();
            return FW_OK;
        }
    }
    if (cov_shift_applies(d, lay)) {
        // stride-1 window: tap pairs with the same offset share their products (cov_shift.hip)
        const size_t need = cov_shift_workspace_bytes(d, lay) + (copy ? act_copy_bytes(d) : 0);
        if (!ws || ws_bytes < need) return FW_ERR_WORKSPACE;
        if (copy) {
            float* Xc = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + cov_shift_workspace_bytes(d, lay));
            const int HW = d->H * d->W;
            hipLaunchKernelGGL(nchw_to_nhwc_kernel, dim3((HW + 31) / 32, (d->Cin + 31) / 32, d->B), dim3(256), 0, st,
                               reinterpret_cast<const float*>(X), Xc, d->Cin, HW);
            FW_LAUNCH_CHECK();
            X = Xc;
        }
        return cov_shift_accumulate(reinterpret_cast<const float*>(X), lay, d, A, s, ws, ws_bytes, st);
    }
    CovGeom g;
    if (!make_geom(d, dt, lay, &g)) return FW_ERR_UNSUPPORTED;
    const size_t part_bytes = align_up((size_t)g.nsplit * g.nitems * 4 * BLK * BLK * sizeof(float), 256);
    const size_t sp_bytes = align_up((size_t)g.nsplit * g.nb * BLK * sizeof(float), 256);
    const size_t need = part_bytes + sp_bytes + (copy ? act_copy_bytes(d) : 0);
    if (!ws || ws_bytes < need) return FW_ERR_WORKSPACE;
    float* part = reinterpret_cast<float*>(ws);
    float* spart = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + part_bytes);
    if (copy) {
        float* Xc = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + part_bytes + sp_bytes);
        const int HW = d->H * d->W;
        hipLaunchKernelGGL(nchw_to_nhwc_kernel, dim3((HW + 31) / 32, (d->Cin + 31) / 32, d->B), dim3(256), 0, st,
                           reinterpret_cast<const float*>(X), Xc, d->Cin, HW);
        FW_LAUNCH_CHECK();
        X = Xc;
    }
    const dim3 grid(g.nitems, g.nsplit);
    const bool vec4 = dt == FW_F32 && lay != FW_LAYOUT_NCHW && (g.Cin % 4) == 0;
    if (vec4)
        hipLaunchKernelGGL(cov_partial_f32v4_kernel, dim3(8 * g.nitems * ((g.nsplit + 7) / 8)), dim3(256), 0, st,
                           reinterpret_cast<const float*>(X), g, part, spart);
    else
        hipLaunchKernelGGL(cov_partial_kernel, grid, dim3(256), 0, st, reinterpret_cast<const float*>(X), g, part, spart);
    FW_LAUNCH_CHECK();
    hipLaunchKernelGGL(cov_reduce_kernel, dim3(g.nitems * 4 * 16 + (g.M + 63) / 64), dim3(256), 0, st, g, part, spart, A, s);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

fw_status cov_finalize(const float* A, const float* s, long long n, int M, float alpha, int first_block, float* mu, float* Phi_x,
                       float* phi_x, float* lambda_bar, hipStream_t st) {
    const double inv_n = 1.0 / (double)n;
    if ((M & 3) == 0) {
        const int tb = (M + 63) / 64;
        hipLaunchKernelGGL(finalize_phi64_kernel, dim3(tb, tb), dim3(256), 0, st, A, s, mu, inv_n, M, alpha, first_block, Phi_x);
    } else {
        const int tb = (M + 31) / 32;
        hipLaunchKernelGGL(finalize_phi_kernel, dim3(tb, tb), dim3(256), 0, st, A, s, mu, inv_n, M, alpha, first_block, Phi_x);
    }
    FW_LAUNCH_CHECK();
    hipLaunchKernelGGL(finalize_vec_kernel, dim3(1), dim3(1024), 0, st, A, s, inv_n, M, alpha, first_block, mu, phi_x, lambda_bar);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

fw_status symmetrize_from_lower(float* A, int M, hipStream_t st) {
    const int tb = (M + 15) / 16;
    hipLaunchKernelGGL(mirror_lower_kernel, dim3(tb, tb), dim3(16, 16), 0, st, A, M);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
