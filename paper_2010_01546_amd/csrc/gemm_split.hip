// Float32-grade matrix products on the bfloat16 matrix cores of gfx950:  C = A B^T  for row-major float32 A [R, K] and
// B [N, K] (both contiguous along the contraction index), used where the method needs M x M x M products every block:
//   Psi = T Phi_x  (Phi_x symmetric, so its rows stand for its columns)  and  Phi_y = Psi T^T   (Sec. 4: the recursion
//   works on the covariance of the transformed input; a new block's Phi_x invalidates both).
//
// Every float32 operand x is split into two bfloat16 numbers, hi = bf16(x) and lo = bf16(x - hi); hi + lo carries 16
// significant bits of x.  The product is accumulated in float32 as  hi hi + hi lo + lo hi  (three
// v_mfma_f32_32x32x16_bf16 per tile and 16 contraction entries; lo lo is below the split's own residual).  Per operand
// the relative residual is at most 2^-17, so a product of two splits is accurate to about 2^-16 per term and the result
// to a few 1e-6 in relative Frobenius norm (measured 3.6e-6 for T Phi_x, 5.3e-6 after the second product): twenty
// times inside the 1e-4 float32 tolerance, at three times the multiplications on a pipe sixteen times faster.
//
// A bandwidth-bound pre-pass packs an operand X [R, K] as
//     Xp[plane][kb][r] -> 8 x bf16 (16 bytes: entries k = 8 kb .. 8 kb + 7 of row r), plane 0 = hi, plane 1 = lo,
// rows padded to a multiple of 64 and the contraction index to a multiple of 16 with zeros, so that 64 consecutive rows
// of one (plane, kb) are 1 KB of contiguous memory: one wavefront-wide 16-byte load straight into LDS.
// The product kernel is the tile kernel of the bfloat16 covariance re-targeted: a workgroup of four wavefronts (one per
// SIMD) owns a tile of 64 NRT x 256 outputs, each wavefront 32 NRT x 128 of them (NRT x 4 MFMA tiles in accumulation
// registers); a stage of the LDS ring holds 16 contraction entries of both panels in both planes, wavefront w brings the
// slab (plane, kb parity) = (w >> 1, w & 1); four stages are in flight ahead of the MFMAs, one barrier per stage, the
// fragment reads of the next stage and the loads of the stage NST ahead are placed one by one between the MFMAs.
#include "fw_internal.h"
#include <type_traits>

namespace fw {
namespace {

constexpr int SP_NCT = 4;          // column MFMA tile pairs: tile width 256
constexpr int SP_TC = 64 * SP_NCT;
constexpr int GEMM_SPLIT_MAX_RUNS = 8;
constexpr int SP_SBR = 4, SP_SBC = 8;   // super-block of tiles an XCD works through together (full grids)

struct SplitGeom {
    int R, N, K;          // C is [R, N], contraction length K
    int Rp, Np, KB;       // padded rows of the packed operands, 16-byte groups along k (even)
    int nrt, tr, nrb, ncb, ntiles;
    int lower;            // 1: only tiles that touch the lower triangle (C symmetric), entries above the diagonal not written
    int zero_a, zero_b;   // a 16-byte element of each packed operand that is always zero
    int nks, spk;         // runs the contraction index is cut into (few tiles: more workgroups), stages per run
};

__host__ __device__ inline int sp_cols_of_row(int I, int tr, int ncb, int lower) {
    if (!lower) return ncb;
    const int n = (I * tr + tr - 1) / SP_TC + 1;
    return n < ncb ? n : ncb;
}

// ---- pre-pass: float32 [R, K] -> packed hi / lo planes.  A workgroup takes 64 rows x 64 contraction entries: coalesced
// reads along k into LDS, then thread (r, kb) forms the two 16-byte elements; consecutive threads write consecutive rows.
__global__ __launch_bounds__(256) void split_pack_kernel(const float* __restrict__ X, int R, int K, int Rp, int KB, uint4* __restrict__ Xp) {
    __shared__ float tile[64][65];
    const int r0 = blockIdx.y * 64, k0 = blockIdx.x * 64;
    const bool vec = (K & 3) == 0;
    for (int e = threadIdx.x; e < 64 * 16; e += 256) {
        const int rr = e >> 4, q = e & 15;
        const int r = r0 + rr, k = k0 + 4 * q;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < R) {
            if (vec) {
                if (k < K) v = *reinterpret_cast<const float4*>(X + (size_t)r * K + k);
            } else {
                const float* p = X + (size_t)r * K;
                if (k < K) v.x = p[k];
                if (k + 1 < K) v.y = p[k + 1];
                if (k + 2 < K) v.z = p[k + 2];
                if (k + 3 < K) v.w = p[k + 3];
            }
        }
        tile[rr][4 * q] = v.x; tile[rr][4 * q + 1] = v.y; tile[rr][4 * q + 2] = v.z; tile[rr][4 * q + 3] = v.w;
    }
    __syncthreads();
    const int rr = threadIdx.x & 63;
    for (int g = threadIdx.x >> 6; g < 8; g += 4) {
        const int kb = (k0 >> 3) + g;
        if (kb >= KB || r0 + rr >= Rp) continue;
        unsigned hi[8], lo[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float x = tile[rr][8 * g + i];
            const unsigned short h = f32_to_bf16_rne(x);
            const float rest = x - bf16_to_f32(h);      // exact in float32
            hi[i] = h;
            lo[i] = f32_to_bf16_rne(rest);
        }
        uint4 oh, ol;
        oh.x = hi[0] | (hi[1] << 16); oh.y = hi[2] | (hi[3] << 16); oh.z = hi[4] | (hi[5] << 16); oh.w = hi[6] | (hi[7] << 16);
        ol.x = lo[0] | (lo[1] << 16); ol.y = lo[2] | (lo[3] << 16); ol.z = lo[4] | (lo[5] << 16); ol.w = lo[6] | (lo[7] << 16);
        Xp[(size_t)kb * Rp + r0 + rr] = oh;
        Xp[((size_t)KB + kb) * Rp + r0 + rr] = ol;
    }
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 16) Xp[(size_t)2 * KB * Rp + threadIdx.x] = make_uint4(0, 0, 0, 0);
}

// The same packed planes for the TRANSPOSE of X: X is [K, R] row-major (contraction index along its rows), the packed
// operand has R rows.  Thread (kb, r) reads the eight entries X[8 kb .. 8 kb + 7][r]; consecutive threads read and write
// consecutive addresses, so no staging is needed.
__global__ __launch_bounds__(256) void split_pack_transposed_kernel(const float* __restrict__ X, int K, int R, int Rp, int KB,
                                                                    uint4* __restrict__ Xp) {
    const int r = blockIdx.x * 256 + threadIdx.x, kb = blockIdx.y;
    if (blockIdx.x == 0 && kb == 0 && threadIdx.x < 16) Xp[(size_t)2 * KB * Rp + threadIdx.x] = make_uint4(0, 0, 0, 0);
    if (r >= Rp) return;
    float x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int k = 8 * kb + i;
        x[i] = (r < R && k < K) ? X[(size_t)k * R + r] : 0.f;
    }
    unsigned hi[8], lo[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const unsigned short h = f32_to_bf16_rne(x[i]);
        hi[i] = h;
        lo[i] = f32_to_bf16_rne(x[i] - bf16_to_f32(h));      // the difference is exact in float32
    }
    uint4 oh, ol;
    oh.x = hi[0] | (hi[1] << 16); oh.y = hi[2] | (hi[3] << 16); oh.z = hi[4] | (hi[5] << 16); oh.w = hi[6] | (hi[7] << 16);
    ol.x = lo[0] | (lo[1] << 16); ol.y = lo[2] | (lo[3] << 16); ol.z = lo[4] | (lo[5] << 16); ol.w = lo[6] | (lo[7] << 16);
    Xp[(size_t)kb * Rp + r] = oh;
    Xp[((size_t)KB + kb) * Rp + r] = ol;
}

// With g.nks > 1 workgroup (tile, run) multiplies only the stages of its run and writes the tile to part[run][R][N];
// split_reduce_kernel adds the runs in a fixed order.
template <int NRT>
__global__ __launch_bounds__(256) void gemm_split_kernel(const uint4* __restrict__ Ap, const uint4* __restrict__ Bp, SplitGeom g,
                                                         float* __restrict__ C, float* __restrict__ part) {
    constexpr int NCT = SP_NCT;
    constexpr int TR = 64 * NRT, TC = 64 * NCT;
    constexpr int NF = NRT + NCT;       // groups of 64 rows per slab: NRT of the A panel, NCT of the B panel
    constexpr int ROW = TR + TC;        // 16-byte elements per slab
    constexpr int NM = NRT * NCT;       // MFMAs per product term and stage
    constexpr int NST = 160 * 1024 / (4 * ROW * 16) > 6 ? 6 : 160 * 1024 / (4 * ROW * 16);   // stages of the LDS ring (5, 5, 6)
    __shared__ uint4 pan[NST][4][ROW];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave >> 1, wj = wave & 1;
    const int half = lane >> 5, l32 = lane & 31;
    // workgroups go to the 8 XCDs round-robin by linear index: give each XCD a contiguous run of tiles (row-major:
    // neighbours share the A panel and walk through B), so that its L2 serves the panels to several compute units
    const int total = g.ntiles * g.nks;
    const int per_xcd = (total + 7) / 8;
    int tile = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (tile >= total || ((int)blockIdx.x >> 3) >= per_xcd) return;
    const int run = __builtin_amdgcn_readfirstlane(tile / g.ntiles);   // run-major: neighbours share the contraction range
    tile -= run * g.ntiles;
    int I = 0, J = 0;
    if (g.lower) {
        for (;;) {
            const int n = sp_cols_of_row(I, TR, g.ncb, g.lower);
            if (tile < n) break;
            tile -= n; ++I;
        }
        J = tile;
    } else {
        // full grid: the run of an XCD walks super-blocks of SP_SBR x SP_SBC tiles (row-major inside), so that the 32 tiles
        // its compute units hold at a time share few row panels AND few column panels
        for (int sI = 0; sI < g.nrb; sI += SP_SBR) {
            const int hr = min(SP_SBR, g.nrb - sI);
            bool found = false;
            for (int sJ = 0; sJ < g.ncb; sJ += SP_SBC) {
                const int wc = min(SP_SBC, g.ncb - sJ);
                if (tile < hr * wc) { I = sI + tile / wc; J = sJ + tile % wc; found = true; break; }
                tile -= hr * wc;
            }
            if (found) break;
        }
    }
    I = __builtin_amdgcn_readfirstlane(I); J = __builtin_amdgcn_readfirstlane(J);

    // slab this wavefront brings: plane = wave >> 1, parity of the 16-byte group along k = wave & 1
    const int plane = wave >> 1, kbl = wave & 1;
    int off[NF];
    unsigned okmask = 0;
#pragma unroll
    for (int k = 0; k < NF; ++k) {
        const int r = k < NRT ? I * TR + 64 * k + lane : J * TC + 64 * (k - NRT) + lane;
        const bool ok = r < (k < NRT ? g.Rp : g.Np);
        off[k] = ok ? r : 0;
        okmask |= (ok ? 1u : 0u) << k;
    }
    // stages of 16 contraction entries: this workgroup's run is [c0, c0 + nch)
    const int c0 = run * g.spk;
    const int nch = min(g.spk, (g.KB >> 1) - c0);
    auto dma_one = [&](int stage, int c, int k) {   // k is a compile-time constant after unrolling
        const bool live = c < nch && ((okmask >> k) & 1u);
        const int kb = plane * g.KB + 2 * (c0 + c) + kbl;
        const uint4* src = k < NRT ? Ap + (live ? (size_t)kb * g.Rp + off[k] : (size_t)g.zero_a)
                                   : Bp + (live ? (size_t)kb * g.Np + off[k] : (size_t)g.zero_b);
        dma16(src, &pan[stage][wave][64 * k]);
    };
    auto issue = [&](int stage, int c) {
#pragma unroll
        for (int k = 0; k < NF; ++k) dma_one(stage, c, k);
    };

    floatx16 acc[NRT][NCT];
#pragma unroll
    for (int a = 0; a < NRT; ++a)
#pragma unroll
        for (int b = 0; b < NCT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // fragments of a stage: index f < NF hi plane (A tiles then B tiles), NF <= f < 2 NF lo plane
    bf16x8 fr[2][2 * NF];
    auto read_one = [&](int stage, int set, int f) {
        const int pl = f / NF, r = f % NF;
        const int col = r < NRT ? 32 * NRT * wi + 32 * r : TR + 32 * NCT * wj + 32 * (r - NRT);
        fr[set][f] = *reinterpret_cast<const bf16x8*>(&pan[stage][2 * pl + half][col + l32]);
    };
    auto mfma_one = [&](int set, int m) {   // m = term * NM + ta * NCT + tb; terms: hi hi, hi lo, lo hi
        const int term = m / NM, ta = (m % NM) / NCT, tb = m % NCT;
        const int fa = (term == 2 ? NF : 0) + ta, fb = (term == 1 ? NF : 0) + NRT + tb;
        acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[set][fa], fr[set][fb], acc[ta][tb], 0, 0, 0);
    };

    // Ring protocol (the loads of one wavefront complete in order): "at most the loads of NST-2 stages outstanding" means
    // the stage before those has landed for this wavefront, the barrier extends that to all four.  At the barrier of
    // iteration c every wavefront holds its fragments of stage c in registers, so the buffer of stage c is free for the
    // loads of stage c + NST, and stage c + 1 is ready to be read while stage c is being multiplied.  Every iteration
    // issues the same number of loads (past the end they fetch the zero element), which keeps the count valid in the tail.
#pragma unroll
    for (int i = 0; i < NST - 1; ++i) issue(i, i);
    FW_WAIT_VM((NST - 2) * NF);
    __builtin_amdgcn_s_barrier();
    FW_COMPILER_FENCE();
    issue(NST - 1, NST - 1);
#pragma unroll
    for (int f = 0; f < 2 * NF; ++f) read_one(0, 0, f);
    int sc = 0;
    auto iteration = [&](int c, auto SET) {
        constexpr int set = decltype(SET)::value;    // register set of stage c: a compile-time index into fr
        const int sn = sc == NST - 1 ? 0 : sc + 1;
        FW_WAIT_LGKM0();
        FW_WAIT_VM((NST - 2) * NF);
        __builtin_amdgcn_s_barrier();
        FW_COMPILER_FENCE();
#pragma unroll
        for (int m = 0; m < 3 * NM; ++m) {
            if (m < 2 * NF) read_one(sn, set ^ 1, m);
            else if (m - 2 * NF < NF) dma_one(sc, c + NST, m - 2 * NF);
            mfma_one(set, m);
            __builtin_amdgcn_sched_barrier(0);
        }
        sc = sn;
    };
    int c = 0;
    for (; c + 1 < nch; c += 2) {
        iteration(c, std::integral_constant<int, 0>());
        iteration(c + 1, std::integral_constant<int, 1>());
    }
    if (c < nch) iteration(c, std::integral_constant<int, 0>());
    FW_WAIT_VM(0);
    FW_WAIT_LGKM0();

    // ---- write-out: 32 lanes along a row of C (or of this run's partial result)
    if (g.nks > 1) C = part + (size_t)run * g.R * g.N;
#pragma unroll
    for (int ta = 0; ta < NRT; ++ta)
#pragma unroll
        for (int tb = 0; tb < NCT; ++tb) {
            const int gj = J * TC + 32 * NCT * wj + 32 * tb + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int gi = I * TR + 32 * NRT * wi + 32 * ta + 8 * (i >> 2) + 4 * half + (i & 3);
                if (gi < g.R && gj < g.N && (!g.lower || gj <= gi)) C[(size_t)gi * g.N + gj] = acc[ta][tb][i];
            }
        }
}

struct SplitWs { size_t a, b, total; };

inline bool make_split_geom(int R, int N, int K, int lower, SplitGeom* g, int max_runs = 1) {
    if (R <= 0 || N <= 0 || K <= 0 || R > 16384 || N > 16384 || K > 16384) return false;
    g->R = R; g->N = N; g->K = K; g->lower = lower;
    g->Rp = (R + 63) / 64 * 64; g->Np = (N + 63) / 64 * 64;
    g->KB = (K + 15) / 16 * 2;
    g->zero_a = 2 * g->KB * g->Rp;
    g->zero_b = 2 * g->KB * g->Np;
    // Tile height (64 nrt) and, when partial results may be used (max_runs > 1) and the tiles are few, the number of runs
    // the contraction index is cut into: least estimated time = rounds of 256 workgroups x (stages of a run + ring fill) x
    // time of a stage (its MFMAs, or its loads into LDS at about 23 bytes per cycle and compute unit), plus the pass that
    // adds runs + 1 copies of the result.  A run keeps at least 32 stages.
    const int nst = (g->KB) >> 1;
    double best = 1e300;
    for (int nrt = 4; nrt >= 2; --nrt) {
        const int tr = 64 * nrt, nrb = (R + tr - 1) / tr, ncb = (N + SP_TC - 1) / SP_TC;
        long long nt = 0;
        for (int I = 0; I < nrb; ++I) nt += sp_cols_of_row(I, tr, ncb, lower);
        const double t_mfma = 3.0 * nrt * SP_NCT * 32.0 + 100.0, t_load = (double)(tr + SP_TC) * 64.0 / 23.0;
        const double t_stage = t_mfma > t_load ? t_mfma : t_load;
        int kmax = 1;
        if (max_runs > 1 && nt <= 128) {
            kmax = (int)(256 / nt);
            if (kmax > max_runs) kmax = max_runs;
            while (kmax > 1 && nst / kmax < 32) --kmax;
        }
        for (int nks = 1; nks <= kmax; ++nks) {
            const int spk = (nst + nks - 1) / nks;
            const int runs = (nst + spk - 1) / spk;
            const double rounds = (double)((nt * runs + 255) / 256);
            double cost = rounds * (spk + 5.0) * t_stage;
            if (runs > 1) cost += (runs + 1.0) * R * (double)N * 4.0 / 4.0e12 * 2.0e9 + 4000.0;
            if (cost < best * 0.999) {
                best = cost;
                g->nrt = nrt; g->tr = tr; g->nrb = nrb; g->ncb = ncb; g->ntiles = (int)nt; g->nks = runs; g->spk = spk;
            }
        }
    }
    return true;
}

// C = sum of the runs' partial results, in run order
__global__ __launch_bounds__(256) void split_reduce_kernel(const float* __restrict__ part, int nks, size_t n, float* __restrict__ C) {
    const size_t n4 = n / 4;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n4; e += (size_t)gridDim.x * 256) {
        float4 v = *reinterpret_cast<const float4*>(part + 4 * e);
        for (int z = 1; z < nks; ++z) {
            const float4 w = *reinterpret_cast<const float4*>(part + (size_t)z * n + 4 * e);
            v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
        }
        *reinterpret_cast<float4*>(C + 4 * e) = v;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0)
        for (size_t e = 4 * n4; e < n; ++e) {
            float v = part[e];
            for (int z = 1; z < nks; ++z) v += part[(size_t)z * n + e];
            C[e] = v;
        }
}

}  // namespace

size_t gemm_split_packed_bytes(int rows, int K) {
    const size_t Rp = (size_t)(rows + 63) / 64 * 64, KB = (size_t)(K + 15) / 16 * 2;
    return align_up((2 * KB * Rp + 16) * 16, 256);
}

// Xp = packed hi / lo planes of X [rows, K]
fw_status gemm_split_pack(const float* X, int rows, int K, void* Xp, hipStream_t st) {
    const int Rp = (rows + 63) / 64 * 64, KB = (K + 15) / 16 * 2;
    hipLaunchKernelGGL(split_pack_kernel, dim3((8 * KB + 63) / 64, Rp / 64), dim3(256), 0, st, X, rows, K, Rp, KB,
                       reinterpret_cast<uint4*>(Xp));
    FW_LAUNCH_CHECK();
    return FW_OK;
}

// Xp = packed hi / lo planes of X^T for X [K, rows] (the operand has `rows` rows and contraction length K)
fw_status gemm_split_pack_transposed(const float* X, int K, int rows, void* Xp, hipStream_t st) {
    const int Rp = (rows + 63) / 64 * 64, KB = (K + 15) / 16 * 2;
    hipLaunchKernelGGL(split_pack_transposed_kernel, dim3((Rp + 255) / 256, KB), dim3(256), 0, st, X, K, rows, Rp, KB,
                       reinterpret_cast<uint4*>(Xp));
    FW_LAUNCH_CHECK();
    return FW_OK;
}

// flops the matrix cores execute for one product (three bfloat16 terms per float32 multiplication, whole tiles)
// runs gemm_split_run cuts the contraction index of a full product into when it is given room for partial results
int gemm_split_runs(int R, int N, int K) {
    SplitGeom g;
    if (!make_split_geom(R, N, K, 0, &g, GEMM_SPLIT_MAX_RUNS)) return 1;
    return g.nks;
}
// room for those runs (for one result at least: a caller that sums the runs itself gets a single run there too)
size_t gemm_split_partial_bytes(int R, int N, int K) {
    return align_up((size_t)gemm_split_runs(R, N, K) * R * N * sizeof(float), 256);
}

// with_runs: as gemm_split_run chooses the tiles when it is given room for partial results
double gemm_split_flops_issued(int R, int N, int K, int lower, bool with_runs) {
    SplitGeom g;
    if (!make_split_geom(R, N, K, lower, &g, (with_runs && !lower) ? GEMM_SPLIT_MAX_RUNS : 1)) return 0.0;
    return 3.0 * 2.0 * (double)g.ntiles * g.tr * SP_TC * (8.0 * g.KB);
}

// C [R, N] = A B^T from the packed operands (A [R, K], B [N, K]); lower != 0: C is known to be symmetric (R == N) and
// only its lower triangle is written.
// part: room for gemm_split_partial_bytes(R, N, K) bytes, or null (then the contraction index is never cut into runs)
// runs_out: when given (with part, and C == part), the runs are left unsummed in part[run][R][N] (a single run: part[0]) and
//   their number is returned, for a caller that adds them in an epilogue of its own
fw_status gemm_split_run(const void* Ap, const void* Bp, int R, int N, int K, int lower, float* C, hipStream_t st, float* part,
                         int* runs_out) {
    if (runs_out && (!part || C != part || lower)) return FW_ERR_INVALID_ARG;
    SplitGeom g;
    if (!make_split_geom(R, N, K, lower, &g, (part && !lower) ? GEMM_SPLIT_MAX_RUNS : 1)) return FW_ERR_UNSUPPORTED;
    const dim3 grid((g.ntiles * g.nks + 7) / 8 * 8);
    const uint4* a = reinterpret_cast<const uint4*>(Ap);
    const uint4* b = reinterpret_cast<const uint4*>(Bp);
    switch (g.nrt) {
        case 4: hipLaunchKernelGGL(gemm_split_kernel<4>, grid, dim3(256), 0, st, a, b, g, C, part); break;
        case 3: hipLaunchKernelGGL(gemm_split_kernel<3>, grid, dim3(256), 0, st, a, b, g, C, part); break;
        default: hipLaunchKernelGGL(gemm_split_kernel<2>, grid, dim3(256), 0, st, a, b, g, C, part); break;
    }
    FW_LAUNCH_CHECK();
    if (runs_out) { *runs_out = g.nks; return FW_OK; }
    if (g.nks > 1) {
        const size_t n = (size_t)R * N;
        size_t blocks = (n / 4 + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        if (blocks == 0) blocks = 1;
        hipLaunchKernelGGL(split_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st, part, g.nks, n, C);
        FW_LAUNCH_CHECK();
    }
    return FW_OK;
}

}  // namespace fw
