// Recursive condition-number reduction (Sec. 4) for gfx950: one step is a chain of bandwidth-bound passes over
// M x M float32 matrices.
//
//   estimate (Sec. 4.2):  m' = argmax xi   ->  c = Phi_y Phi_y e_m'  ->  coherence set, weights w  ->
//                         v~ = Phi_y w  ->  v = v~/|v~|   [optional refinements v <- Phi_y v / |Phi_y v|]
//   step (Sec. 4.1):      u = Phi_y v, lambda_e = v^T u, g_e, a_e;  t = T^T v;  p = Phi_x t = Psi^T v (only if gamma < 1)
//   The small reductions in between (arg-max, size of the set, |v~|) are done by every workgroup of the pass that
//   needs them, for itself, from vectors of M entries, so that a step is six launches, four of which touch M x M data:
//   c | v~ | u and the partial products of t and p | t, p and the scalars | update | squared row norms.
//   p = Phi_x T^T v is taken as Psi^T v (Psi = T Phi_x is part of the state): all three products of the third launch
//   then need nothing but v, and no pass has to wait for t.
//   update, one fused pass over pairs of mirrored 32x32 tiles:
//       T'     = gamma (T + a v t^T) + (1-gamma) I                                               eq. (vT_rec)
//       Q'     = gamma^2 (Q + a(a+2) t t^T) + (1-gamma)^2 I
//                + gamma(1-gamma) (a (v t^T + t v^T) + T + T^T)                                  eq. (vQ_rec)
//       Qs'    = beta Qs + (1-beta) Q'                                                           eq. (vQs)
//       Phi_y' = gamma^2 (Phi_y + a (v u^T + u v^T) + a^2 lambda_e v v^T)
//                + gamma(1-gamma) (Psi + Psi^T + a (v p^T + p v^T)) + (1-gamma)^2 Phi_x          (= T' Phi_x T'^T)
//       Psi'   = gamma (Psi + a v p^T) + (1-gamma) Phi_x                                         (= T' Phi_x)
//     and the squared row norms of Phi_y' for the next step's arg-max.
// t = T^T v (the transposed reading of eq. (vtve)) is what makes T' equal gamma T~ T + (1-gamma) I.
// Matrix-vector products use one wavefront per row with a 64-lane shuffle reduction.
#include "fw_internal.h"
#include <mutex>

// Scratch of the allocation-free variant of the step (fw_cond_reduce_step_static): the workspace of one step for
// M <= 4608, held by every GPU the library runs on until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress; the address kernels are given comes from static_scratch() below.
static __device__ __align__(256) unsigned char scratch[6u << 20];

namespace fw {
namespace {

struct Scal {
    int m_prime, set_size, applied, flags;
    float xi_mp, lambda_e, g_e, a_e, vnorm;
};

constexpr int TILE = 32;
constexpr int VM_ROWS_MIN = 16;  // fewest rows a workgroup takes in the T^T v partial products

struct WsLayout {
    size_t c, w, vt, v, u, t, p, tpart, ppart, xpart, scal, total;
    int Mp, nrb, vm_rows, nt;
};
inline WsLayout ws_layout(int M) {
    WsLayout L;
    L.Mp = (M + 63) / 64 * 64;
    // rows per workgroup of the T^T v pass: about 1024 workgroups in all, a multiple of 16 rows, at least 16
    {
        const long long colblocks = (M + 255) / 256;
        long long rows = ((long long)M * colblocks + 1023) / 1024;
        rows = (rows + VM_ROWS_MIN - 1) / VM_ROWS_MIN * VM_ROWS_MIN;
        L.vm_rows = (int)rows;
    }
    L.nrb = (M + L.vm_rows - 1) / L.vm_rows;
    L.nt = (M + TILE - 1) / TILE;
    size_t o = 0;
    auto take = [&](size_t floats) { size_t at = o; o += align_up(floats * sizeof(float), 256); return at; };
    L.c = take(L.Mp); L.w = take(L.Mp); L.vt = take(L.Mp); L.v = take(L.Mp); L.u = take(L.Mp); L.t = take(L.Mp); L.p = take(L.Mp);
    L.tpart = take((size_t)L.nrb * L.Mp);
    L.ppart = take((size_t)L.nrb * L.Mp);
    L.xpart = take((size_t)L.nt * L.Mp);
    L.scal = take(64);
    L.total = o;
    return L;
}

// sum over the workgroup, the same value in every thread
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < (int)(blockDim.x >> 6); ++i) t += red[i];
    return t;
}

// m' = argmax_m xi2[m], lowest index on ties (eq. (mt)), computed by a whole workgroup of 256 threads; every
// workgroup that calls it gets the same answer
__device__ __forceinline__ void block_argmax(const float* __restrict__ xi2, int M, float* bv, int* bi, float* best_out, int* idx_out) {
    float best = -1.f;
    int idx = 0x7fffffff;
    // ascending scan per thread with a strict comparison keeps the lowest index; four 16-byte loads in flight
    if ((M & 3) == 0) {
        const float4* x4 = reinterpret_cast<const float4*>(xi2);
        const int n4 = M >> 2, nt = blockDim.x;
        for (int k = threadIdx.x; k < n4; k += 4 * nt) {
            float4 q[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) q[j] = (k + j * nt < n4) ? x4[k + j * nt] : make_float4(-1.f, -1.f, -1.f, -1.f);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int m = 4 * (k + j * nt);
                if (q[j].x > best) { best = q[j].x; idx = m; }
                if (q[j].y > best) { best = q[j].y; idx = m + 1; }
                if (q[j].z > best) { best = q[j].z; idx = m + 2; }
                if (q[j].w > best) { best = q[j].w; idx = m + 3; }
            }
        }
    } else {
        for (int m = threadIdx.x; m < M; m += blockDim.x) {
            const float v = xi2[m];
            if (v > best) { best = v; idx = m; }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best, o, 64);
        const int oi = __shfl_xor(idx, o, 64);
        if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
    }
    if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = idx; }
    __syncthreads();
    best = bv[0]; idx = bi[0];
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i)
        if (bv[i] > best || (bv[i] == best && bi[i] < idx)) { best = bv[i]; idx = bi[i]; }
    if (idx < 0 || idx >= M) idx = 0;  // every norm was NaN: keep the index in range
    *best_out = best; *idx_out = idx;
}

// dot product of a row of P with x (global memory or LDS), one wavefront per row, four 16-byte loads of the row in flight
__device__ __forceinline__ float row_dot(const float* __restrict__ row, const float* __restrict__ x, int M, int lane) {
    float acc = 0.f;
    if ((M & 3) == 0) {
        const float4* r4 = reinterpret_cast<const float4*>(row);
        const float4* x4 = reinterpret_cast<const float4*>(x);
        const int n4 = M >> 2;
        int k = lane;
        for (; k + 192 < n4; k += 256) {
            float4 a[4], b[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) { a[j] = r4[k + 64 * j]; b[j] = x4[k + 64 * j]; }
#pragma unroll
            for (int j = 0; j < 4; ++j) acc += a[j].x * b[j].x + a[j].y * b[j].y + a[j].z * b[j].z + a[j].w * b[j].w;
        }
        for (; k < n4; k += 64) {
            const float4 a = r4[k], b = x4[k];
            acc += a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
        }
    } else {
        for (int k = lane; k < M; k += 64) acc += row[k] * x[k];
    }
    return wave_sum(acc);
}

// The first four 16-byte loads of a row, issued before a workgroup's preparation (arg-max, weights, norm) so that the
// memory pipe is already busy while the small reductions run; row_dot_pref consumes them and continues like row_dot.
struct RowPref { float4 a[4]; };
__device__ __forceinline__ void row_prefetch(const float* __restrict__ row, int M, int lane, RowPref& p) {
    if ((M & 3) != 0) return;
    const float4* r4 = reinterpret_cast<const float4*>(row);
    const int n4 = M >> 2;
#pragma unroll
    for (int j = 0; j < 4; ++j) p.a[j] = r4[lane + 64 * j < n4 ? lane + 64 * j : 0];
#pragma unroll
    for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(p.a[j].x), "+v"(p.a[j].y), "+v"(p.a[j].z), "+v"(p.a[j].w));   // issued here, not later
}
__device__ __forceinline__ float row_dot_pref(const float* __restrict__ row, const float* __restrict__ x, int M, int lane, const RowPref& p) {
    if ((M & 3) != 0) return row_dot(row, x, M, lane);
    const float4* r4 = reinterpret_cast<const float4*>(row);
    const float4* x4 = reinterpret_cast<const float4*>(x);
    const int n4 = M >> 2;
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (lane + 64 * j < n4) {
            const float4 a = p.a[j], b = x4[lane + 64 * j];
            acc += a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
        }
    int k = lane + 256;
    for (; k + 192 < n4; k += 256) {
        float4 a[4], b[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) { a[j] = r4[k + 64 * j]; b[j] = x4[k + 64 * j]; }
#pragma unroll
        for (int j = 0; j < 4; ++j) acc += a[j].x * b[j].x + a[j].y * b[j].y + a[j].z * b[j].z + a[j].w * b[j].w;
    }
    for (; k < n4; k += 64) {
        const float4 a = r4[k], b = x4[k];
        acc += a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
    }
    return wave_sum(acc);
}

// c = Phi_y (Phi_y e_m') (eq. (vc)) with the arg-max of eq. (mt) found by every workgroup for itself; four rows per
// workgroup, one wavefront each.  Workgroup 0 records m' and xi_m'.
__global__ __launch_bounds__(256) void matvec_c_kernel(const float* __restrict__ P, const float* __restrict__ xi2, int M,
                                                       Scal* __restrict__ sc, float* __restrict__ c) {
    __shared__ float bv[4];
    __shared__ int bi[4];
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    RowPref pre;
    row_prefetch(P + (size_t)(r < M ? r : 0) * M, M, lane, pre);
    float best; int mp;
    block_argmax(xi2, M, bv, bi, &best, &mp);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        sc->m_prime = mp;
        sc->xi_mp = sqrtf(fmaxf(best, 0.f));
        sc->flags = 0;
    }
    if (r >= M) return;
    const float acc = row_dot_pref(P + (size_t)r * M, P + (size_t)mp * M, M, lane, pre);
    if (lane == 0) c[r] = acc;
}

// v~ = Phi_y w (first line of eq. (tve)) with the coherence set and the alignment weights w_m = 1/(|set| c_m) on the
// set, 0 elsewhere (rule after eq. (vc)) formed on the fly: every workgroup counts the set for itself.
__global__ __launch_bounds__(256) void matvec_vt_kernel(const float* __restrict__ P, const float* __restrict__ c,
                                                        const float* __restrict__ xi2, int M, float c_rel, float c_abs,
                                                        Scal* __restrict__ sc, float* __restrict__ vt) {
    extern __shared__ __attribute__((aligned(16))) float wl[];   // M weights
    __shared__ float red[4];
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    RowPref pre;
    row_prefetch(P + (size_t)(r < M ? r : 0) * M, M, lane, pre);
    const float xi_mp = sc->xi_mp;
    // first pass: c_m on the set and 0 elsewhere into LDS, and the size of the set
    float cnt = 0.f;
    auto weight = [&](float cm, float x2) {
        const float thr = fmaxf(c_rel * xi_mp * sqrtf(fmaxf(x2, 0.f)), c_abs);
        const bool in = fabsf(cm) >= thr;
        cnt += in ? 1.f : 0.f;
        return in ? cm : 0.f;
    };
    if ((M & 3) == 0) {
        const float4* c4 = reinterpret_cast<const float4*>(c);
        const float4* x4 = reinterpret_cast<const float4*>(xi2);
        float4* w4 = reinterpret_cast<float4*>(wl);
        const int n4 = M >> 2, nt = blockDim.x;
        for (int k = threadIdx.x; k < n4; k += 2 * nt) {
            const bool two = k + nt < n4;
            const float4 ca = c4[k], xa = x4[k];
            const float4 cb = two ? c4[k + nt] : ca, xb = two ? x4[k + nt] : xa;
            w4[k] = make_float4(weight(ca.x, xa.x), weight(ca.y, xa.y), weight(ca.z, xa.z), weight(ca.w, xa.w));
            if (two) w4[k + nt] = make_float4(weight(cb.x, xb.x), weight(cb.y, xb.y), weight(cb.z, xb.z), weight(cb.w, xb.w));
        }
    } else {
        for (int m = threadIdx.x; m < M; m += blockDim.x) wl[m] = weight(c[m], xi2[m]);
    }
    const float total = block_sum(cnt, red);   // has the barriers that publish wl
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        sc->set_size = (int)total;
        if (total == 0.f) sc->flags |= 1;
    }
    // second pass over LDS: w_m = 1/(|set| c_m) on the set
    for (int m = threadIdx.x; m < M; m += blockDim.x) {
        const float cm = wl[m];
        wl[m] = cm != 0.f ? 1.f / (total * cm) : 0.f;
    }
    __syncthreads();
    if (r >= M) return;
    const float acc = row_dot_pref(P + (size_t)r * M, wl, M, lane, pre);
    if (lane == 0) vt[r] = acc;
}

// |v~| by a whole workgroup (the same value in every workgroup) and the factor that normalises it (second line of
// eq. (tve)); an empty set gives v = 0
__device__ __forceinline__ float block_inv_norm(const float* __restrict__ vt, int M, const Scal* __restrict__ sc, float* red, float* nrm_out) {
    float ss = 0.f;
    if ((M & 3) == 0) {
        const float4* v4 = reinterpret_cast<const float4*>(vt);
        const int n4 = M >> 2, nt = blockDim.x;
        for (int k = threadIdx.x; k < n4; k += 4 * nt) {
            float4 q[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) q[j] = (k + j * nt < n4) ? v4[k + j * nt] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int j = 0; j < 4; ++j) ss += q[j].x * q[j].x + q[j].y * q[j].y + q[j].z * q[j].z + q[j].w * q[j].w;
        }
    } else {
        for (int m = threadIdx.x; m < M; m += blockDim.x) ss += vt[m] * vt[m];
    }
    const float nrm = sqrtf(block_sum(ss, red));
    *nrm_out = nrm;
    return (nrm > 0.f && (sc->flags & 1) == 0) ? 1.f / nrm : 0.f;
}

// One refinement v <- Phi_y v / |Phi_y v| in unnormalised form: out = Phi_y (v~ / |v~|)
__global__ __launch_bounds__(256) void matvec_refine_kernel(const float* __restrict__ P, const float* __restrict__ vt, int M,
                                                            const Scal* __restrict__ sc, float* __restrict__ out) {
    __shared__ float red[4];
    float nrm;
    const float inv = block_inv_norm(vt, M, sc, red, &nrm);
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= M) return;
    const float acc = row_dot(P + (size_t)r * M, vt, M, lane) * inv;
    if (lane == 0) out[r] = acc;
}

// v = v~/|v~|, u = Phi_y v (workgroups below nmv: four rows each) and the partial products of t = T^T v and, with leak,
// p = Psi^T v over bands of vm_rows rows, tpart[band][j] = sum_{i in band} T[i][j] v[i] (the other workgroups: first
// those of T, then those of Psi), in one launch.
__global__ __launch_bounds__(256) void matvec_u_vecmat_kernel(const float* __restrict__ P, const float* __restrict__ T,
                                                              const float* __restrict__ Psi,
                                                              const float* __restrict__ vt, int M, int Mp, int vm_rows, int nmv, int nvm,
                                                              Scal* __restrict__ sc, float* __restrict__ v, float* __restrict__ u,
                                                              float* __restrict__ tpart, float* __restrict__ ppart) {
    __shared__ float red[4];
    float nrm;
    RowPref pre;
    const int ur = blockIdx.x * 4 + (threadIdx.x >> 6);
    if ((int)blockIdx.x < nmv) row_prefetch(P + (size_t)(ur < M ? ur : 0) * M, M, threadIdx.x & 63, pre);
    const float inv = block_inv_norm(vt, M, sc, red, &nrm);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        sc->vnorm = nrm;
        if (!(nrm == nrm) || nrm > 3.0e38f) sc->flags |= 4;
    }
    if ((int)blockIdx.x < nmv) {
        const int lane = threadIdx.x & 63;
        const int r = ur;
        if (r >= M) return;
        const float acc = row_dot_pref(P + (size_t)r * M, vt, M, lane, pre) * inv;
        if (lane == 0) { u[r] = acc; v[r] = vt[r] * inv; }
        return;
    }
    const int ncol = (M + 255) / 256;
    int b = (int)blockIdx.x - nmv;
    if (b >= nvm) {        // the second set of bands multiplies Psi
        b -= nvm;
        T = Psi;
        tpart = ppart;
    }
    const int j = (b % ncol) * 256 + threadIdx.x;
    const int band = b / ncol;
    const int i0 = band * vm_rows;
    const int i1 = min(M, i0 + vm_rows);
    if (j >= M) return;
    float acc = 0.f;
    int i = i0;
    for (; i + 8 <= i1; i += 8) {
        float x[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) x[q] = T[(size_t)(i + q) * M + j];
#pragma unroll
        for (int q = 0; q < 8; ++q) acc += x[q] * vt[i + q];
    }
    for (; i < i1; ++i) acc += T[(size_t)i * M + j] * vt[i];
    tpart[(size_t)band * Mp + j] = acc * inv;
}

// out[m] = sum over b < nparts of part[b][m]: 16 entries per workgroup, the parts dealt to sixteen groups of threads
// (eight loads in flight each) in a fixed order and combined through LDS
__device__ __forceinline__ void partial_sum_block(const float* __restrict__ part, int nparts, int M, int Mp, int blk, float* __restrict__ out,
                                                  float (*red)[16]) {
    const int e = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int m = blk * 16 + e;
    float acc = 0.f;
    if (m < M) {
        int b = grp;
        for (; b + 7 * 16 < nparts; b += 8 * 16) {
            float x[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) x[q] = part[(size_t)(b + 16 * q) * Mp + m];
#pragma unroll
            for (int q = 0; q < 8; ++q) acc += x[q];
        }
        for (; b < nparts; b += 16) acc += part[(size_t)b * Mp + m];
    }
    red[grp][e] = acc;
    __syncthreads();
    if (grp == 0 && m < M) {
        float t = 0.f;
#pragma unroll
        for (int g = 0; g < 16; ++g) t += red[g][e];
        out[m] = t;
    }
}

// squared row norms of the new Phi_y from the partial sums of the update pass
__global__ __launch_bounds__(256) void partial_sum_kernel(const float* __restrict__ part, int nparts, int M, int Mp, float* __restrict__ out) {
    __shared__ float red[16][16];
    partial_sum_block(part, nparts, M, Mp, blockIdx.x, out, red);
}

// t = T^T v (workgroups below nred) and p = Psi^T v (the next nred, with leak) from their partial products, and in the
// last workgroup lambda_e = v^T u (eq. (lambda)), g_e, a_e (eqs. (ge), (xi)), the guard and the diagnostics
__global__ __launch_bounds__(256) void t_reduce_scalars_kernel(const float* __restrict__ tpart, const float* __restrict__ ppart,
                                                               int nparts, int M, int Mp, int nred, int last,
                                                               float* __restrict__ t, float* __restrict__ pv, const float* __restrict__ v,
                                                               const float* __restrict__ u, const float* __restrict__ lambda_bar,
                                                               fw_cond_params prm, Scal* __restrict__ sc, fw_cond_info* __restrict__ info) {
    __shared__ float red[16][16];
    if ((int)blockIdx.x < nred) {
        partial_sum_block(tpart, nparts, M, Mp, blockIdx.x, t, red);
        return;
    }
    if ((int)blockIdx.x < last) {
        partial_sum_block(ppart, nparts, M, Mp, blockIdx.x - nred, pv, red);
        return;
    }
    float dot = 0.f;
    for (int m = threadIdx.x; m < M; m += blockDim.x) dot += v[m] * u[m];
    const float lam_e = block_sum(dot, &red[0][0]);
    if (threadIdx.x == 0) {
        int flags = sc->flags;
        float g_e = 1.f, a_e = 0.f;
        int applied = 0;
        if ((flags & 1) == 0) {
            g_e = prm.delta * (*lambda_bar) / fmaxf(lam_e, prm.eps);
            if (prm.guard && g_e >= 1.f) flags |= 2;
            else if (!(g_e == g_e) || g_e > 3.0e38f) flags |= 4;
            else { a_e = sqrtf(g_e) - 1.f; applied = 1; }
        }
        sc->lambda_e = (flags & 1) ? 0.f : lam_e;
        sc->g_e = g_e; sc->a_e = a_e; sc->applied = applied; sc->flags = flags;
        if (info) {
            info->lambda_e = sc->lambda_e; info->g_e = g_e; info->a_e = a_e; info->v_norm = sc->vnorm;
            info->m_prime = sc->m_prime; info->set_size = sc->set_size; info->applied = applied; info->flags = flags;
        }
    }
}

// Fused update over the pair of mirrored tiles (I,J) and (J,I), I >= J, one workgroup per pair (pairs enumerated along a
// one-dimensional grid).  Q, Qs, Phi_y and Phi_x are symmetric and kept exactly so: only their tile (I,J) is read, the
// mirrored position takes its old values from that tile transposed through LDS, so the pass reads 4 of the 16 M^2 words
// of a step only half (9 M^2 words move instead of 11).  T and Psi are not symmetric: both of their tiles are read, each
// position needs its own element and, for the terms T + T^T and Psi + Psi^T, the other tile's transposed one.
__global__ __launch_bounds__(256) void update_kernel(fw_cond_state s, const float* __restrict__ v, const float* __restrict__ u,
                                                     const float* __restrict__ t, const float* __restrict__ p, const Scal* __restrict__ sc,
                                                     float gamma, float beta, int Mp, float* __restrict__ xpart) {
    // pair index -> (I, J), I >= J: I (I + 1) / 2 + J
    int I = (int)((sqrtf(8.f * (float)blockIdx.x + 1.f) - 1.f) * 0.5f);
    while ((I + 1) * (I + 2) / 2 <= (int)blockIdx.x) ++I;
    while (I * (I + 1) / 2 > (int)blockIdx.x) --I;
    const int J = (int)blockIdx.x - I * (I + 1) / 2;
    const int M = s.M;
    const bool leak = gamma < 1.f;
    // four LDS tiles, used twice: first for the transposed elements of T and Psi, then for those of the symmetric
    // matrices (a workgroup's LDS decides how many of them a compute unit holds, and with them the loads in flight)
    __shared__ float L0[TILE][TILE + 1], L1[TILE][TILE + 1], L2[TILE][TILE + 1], L3[TILE][TILE + 1];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const float a = sc->a_e, lam = sc->lambda_e;
    const float g1 = 1.f - gamma, g2 = gamma * gamma, gg1 = gamma * g1, g1sq = g1 * g1, b1 = 1.f - beta;
    const float aa2 = a * (a + 2.f), a2lam = a * a * lam;

    // Everything this workgroup reads is asked for before anything is stored (the state pointers may not be told apart
    // by the compiler, so a load behind a store would wait for it: a chain of round trips that dominates small M).
    const int npos = (I == J) ? 1 : 2;
    float Qv[4], Yv[4], Sv[4], Xv[4], Tv[2][4], Pv[2][4], Tt[2][4], Pt[2][4];
    {
        const int j = J * TILE + tx;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = I * TILE + ty + 8 * r;
            const bool ok = i < M && j < M;
            const size_t e = ok ? (size_t)i * M + j : 0;
            Qv[r] = s.Q[e]; Yv[r] = s.Phi_y[e]; Sv[r] = s.Qs[e];
            Xv[r] = leak ? s.Phi_x[e] : 0.f;
        }
    }
#pragma unroll
    for (int pos = 0; pos < 2; ++pos) {
        const int rowblk = pos == 0 ? I : J, colblk = pos == 0 ? J : I;
        const int j = colblk * TILE + tx;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = rowblk * TILE + ty + 8 * r;
            const bool ok = pos < npos && i < M && j < M;
            const size_t e = ok ? (size_t)i * M + j : 0;
            Tv[pos][r] = s.T[e];
            Pv[pos][r] = leak ? s.Psi[e] : 0.f;
            Tt[pos][r] = 0.f; Pt[pos][r] = 0.f;
            if (!ok) { Tv[pos][r] = 0.f; Pv[pos][r] = 0.f; }
        }
    }
    if (leak) {
        // transposed elements of T and Psi: position a reads tile b transposed and the other way round (the diagonal
        // tile reads itself)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int yy = ty + 8 * r;
            L0[yy][tx] = Tv[0][r]; L1[yy][tx] = Pv[0][r];
            if (npos == 2) { L2[yy][tx] = Tv[1][r]; L3[yy][tx] = Pv[1][r]; }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int yy = ty + 8 * r;
            if (npos == 2) { Tt[0][r] = L2[tx][yy]; Pt[0][r] = L3[tx][yy]; Tt[1][r] = L0[tx][yy]; Pt[1][r] = L1[tx][yy]; }
            else { Tt[0][r] = L0[tx][yy]; Pt[0][r] = L1[tx][yy]; }
        }
    }
    if (npos == 2) {
        // old values of the symmetric matrices at the mirrored position: the tile (I,J), read transposed where used
        if (leak) __syncthreads();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int yy = ty + 8 * r;
            L0[yy][tx] = Qv[r]; L1[yy][tx] = Yv[r]; L2[yy][tx] = Sv[r]; L3[yy][tx] = Xv[r];
        }
        __syncthreads();
    }

#pragma unroll
    for (int pos = 0; pos < 2; ++pos) {
        if (pos >= npos) break;
        const int rowblk = pos == 0 ? I : J, colblk = pos == 0 ? J : I;
        const int j = colblk * TILE + tx;
        const float vj = j < M ? v[j] : 0.f, uj = j < M ? u[j] : 0.f, tj = j < M ? t[j] : 0.f;
        const float pj = (leak && j < M) ? p[j] : 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int yy = ty + 8 * r;
            const int i = rowblk * TILE + yy;
            float sq = 0.f;
            if (i < M && j < M) {
                const size_t e = (size_t)i * M + j;
                const float vi = v[i], ui = u[i], ti = t[i];
                const float dij = (i == j) ? 1.f : 0.f;
                const float Told = Tv[pos][r];
                const float Qold = pos == 0 ? Qv[r] : L0[tx][yy], Yold = pos == 0 ? Yv[r] : L1[tx][yy];
                const float Sold = pos == 0 ? Sv[r] : L2[tx][yy];
                const float Tn = gamma * (Told + a * vi * tj) + g1 * dij;
                float Qn = g2 * (Qold + aa2 * (ti * tj)) + g1sq * dij;
                float Yn = g2 * (Yold + a * (vi * uj + ui * vj) + a2lam * (vi * vj));
                if (leak) {
                    const float Psiold = Pv[pos][r], phix = pos == 0 ? Xv[r] : L3[tx][yy], pi = p[i];
                    Qn += gg1 * (a * (vi * tj + ti * vj) + Told + Tt[pos][r]);
                    Yn += gg1 * (Psiold + Pt[pos][r] + a * (vi * pj + pi * vj)) + g1sq * phix;
                    s.Psi[e] = gamma * (Psiold + a * vi * pj) + g1 * phix;
                }
                s.T[e] = Tn;
                s.Q[e] = Qn;
                s.Qs[e] = beta * Sold + b1 * Qn;
                s.Phi_y[e] = Yn;
                sq = Yn * Yn;
            }
            // sum over the 32 lanes that share row i
#pragma unroll
            for (int o = 16; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
            if (tx == 0 && i < M) xpart[(size_t)colblk * Mp + i] = sq;
        }
    }
}

__global__ __launch_bounds__(256) void state_init_kernel(fw_cond_state s) {
    const int M = s.M;
    const size_t n = (size_t)M * M;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256) {
        const int i = (int)(e / M), j = (int)(e - (size_t)i * M);
        const float d = i == j ? 1.f : 0.f;
        const float ph = s.Phi_x[e];
        s.T[e] = d; s.Q[e] = d; s.Qs[e] = d;
        s.Phi_y[e] = ph;
        if (s.Psi) s.Psi[e] = ph;
    }
}

// Lower triangle -> full symmetric matrix, and the squared row norms of the result, in one pass over pairs of 64 x 64 tiles
// (I, J), I >= J (M a multiple of 4): the tile (I,J) is read once with 16-byte loads, written transposed as (J,I) through
// LDS, and leaves two sets of partial sums of squares: over its columns for the rows of block I, over its rows for the
// rows of block J (the mirrored tile's rows).  xpart[colblock][row], summed by partial_sum_kernel.
__global__ __launch_bounds__(256) void mirror_rownorm_kernel(float* __restrict__ P, int M, int Mp, float* __restrict__ xpart) {
    __shared__ float t[64][65];
    int I = (int)((sqrtf(8.f * (float)blockIdx.x + 1.f) - 1.f) * 0.5f);
    while ((I + 1) * (I + 2) / 2 <= (int)blockIdx.x) ++I;
    while (I * (I + 1) / 2 > (int)blockIdx.x) --I;
    const int J = (int)blockIdx.x - I * (I + 1) / 2;
    const int q = threadIdx.x & 15, r0 = threadIdx.x >> 4;     // 16 threads along a row (4 floats each), 16 rows per pass
    const int j = J * 64 + 4 * q;
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int rr = r0 + 16 * pass, i = I * 64 + rr;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < M && j < M) {
            v = *reinterpret_cast<const float4*>(P + (size_t)i * M + j);
            if (I == J) {            // diagonal tile: what lies above the diagonal is taken from below it, after the barrier
                if (j > i) v.x = 0.f;
                if (j + 1 > i) v.y = 0.f;
                if (j + 2 > i) v.z = 0.f;
                if (j + 3 > i) v.w = 0.f;
            }
        }
        t[rr][4 * q] = v.x; t[rr][4 * q + 1] = v.y; t[rr][4 * q + 2] = v.z; t[rr][4 * q + 3] = v.w;
    }
    __syncthreads();
    if (I == J) {
        // complete the tile in LDS (upper = lower transposed), write it back whole, one set of row sums
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int rr = r0 + 16 * pass, i = I * 64 + rr;
            float x[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) { const int cc = 4 * q + k; x[k] = cc > rr ? t[cc][rr] : t[rr][cc]; }
            float sq = x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3];
            if (i < M && j < M) *reinterpret_cast<float4*>(P + (size_t)i * M + j) = make_float4(x[0], x[1], x[2], x[3]);
            else sq = 0.f;
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
            if (q == 0 && i < M) xpart[(size_t)J * Mp + i] = sq;
        }
        return;
    }
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int rr = r0 + 16 * pass;
        // row sums of the tile as read (rows of block I, column block J)
        const int i = I * 64 + rr;
        float sq = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) { const float x = t[rr][4 * q + k]; sq += x * x; }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
        if (q == 0 && i < M) xpart[(size_t)J * Mp + i] = sq;
        // the mirrored tile: row rr of (J, I) is column rr of (I, J)
        const int im = J * 64 + rr, jm = I * 64 + 4 * q;
        float x[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] = t[4 * q + k][rr];
        float sm = x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3];
        if (im < M && jm < M) *reinterpret_cast<float4*>(P + (size_t)im * M + jm) = make_float4(x[0], x[1], x[2], x[3]);
        else sm = 0.f;
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) sm += __shfl_xor(sm, o, 64);
        if (q == 0 && im < M) xpart[(size_t)I * Mp + im] = sm;
    }
}

__global__ __launch_bounds__(256) void rownorm2_kernel(const float* __restrict__ P, int M, float* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= M) return;
    float acc = 0.f;
    for (int k = lane; k < M; k += 64) { const float x = P[(size_t)r * M + k]; acc += x * x; }
    acc = wave_sum(acc);
    if (lane == 0) out[r] = acc;
}

}  // namespace

size_t cond_workspace_bytes(int M) { return ws_layout(M).total; }

fw_status cond_state_init(const fw_cond_state* s, hipStream_t st) {
    const size_t n = (size_t)s->M * s->M;
    int blocks = (int)((n + 255) / 256);
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(state_init_kernel, dim3(blocks), dim3(256), 0, st, *s);
    FW_LAUNCH_CHECK();
    hipLaunchKernelGGL(rownorm2_kernel, dim3((s->M + 3) / 4), dim3(256), 0, st, s->Phi_x, s->M, s->xi2);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

// Workspace of the refresh: room for Psi when the state has none, then the packed hi / lo planes of T, Phi_x and Psi.
static size_t refresh_xpart_bytes(int M) {
    const size_t nt = (size_t)(M + 63) / 64, Mp = (size_t)(M + 63) / 64 * 64;
    return align_up(nt * Mp * sizeof(float), 256);
}
size_t cond_refresh_workspace_bytes(int M) {
    return align_up((size_t)M * M * sizeof(float), 256) + 3 * gemm_split_packed_bytes(M, M) + refresh_xpart_bytes(M);
}

bool cond_refresh_plan(int M, size_t ws_bytes, fw_refresh_plan* plan) {
    if (M <= 0 || M > 16384) return false;
    plan->split = (ws_bytes >= cond_refresh_workspace_bytes(M) && M >= FW_REFRESH_SPLIT_MIN_M) ? 1 : 0;
    if (plan->split) plan->mfma_flops_issued = gemm_split_flops_issued(M, M, M, 0) + gemm_split_flops_issued(M, M, M, 1);
    else plan->mfma_flops_issued = 4.0 * (double)M * M * M;
    return true;
}

// New block, new Phi_x: Psi = T Phi_x and Phi_y = T Phi_x T^T = Psi T^T by two M x M x M products, Phi_y made exactly
// symmetric from its lower triangle, and the squared row norms for the arg-max.  Both products have the form A B^T with
// row-major operands: Phi_x is symmetric (its rows stand for its columns), and T is exactly the factor wanted.
// With the full workspace the operands are split into bfloat16 hi + lo planes and multiplied on the bfloat16 matrix
// cores (three products per term, float32 accumulation: see gemm_split.hip), only the lower triangle of Phi_y being
// computed; without it (allowed when the state carries Psi) the products run in plain float32 on the matrix cores.
fw_status cond_state_refresh(const fw_cond_state* s, void* ws, size_t ws_bytes, hipStream_t st) {
    const int M = s->M;
    const size_t psi_bytes = align_up((size_t)M * M * sizeof(float), 256);
    char* base = reinterpret_cast<char*>(ws);
    float* Psi = s->Psi ? s->Psi : reinterpret_cast<float*>(base);
    fw_status rc;
    // Below about 1500 features the float32 kernel is as fast (too few 256-wide tiles for 256 compute units, and the
    // three packing passes cost as much as a product); FW_REFRESH_SPLIT_MIN_M is where the split form starts.
    if (ws && ws_bytes >= cond_refresh_workspace_bytes(M) && M >= FW_REFRESH_SPLIT_MIN_M) {
        const size_t pb = gemm_split_packed_bytes(M, M);
        void* Tp = base + psi_bytes;
        void* Xp = base + psi_bytes + pb;
        void* Pp = base + psi_bytes + 2 * pb;
        if ((rc = gemm_split_pack(s->T, M, M, Tp, st)) != FW_OK) return rc;
        if ((rc = gemm_split_pack(s->Phi_x, M, M, Xp, st)) != FW_OK) return rc;
        if ((rc = gemm_split_run(Tp, Xp, M, M, M, 0, Psi, st)) != FW_OK) return rc;
        if ((rc = gemm_split_pack(Psi, M, M, Pp, st)) != FW_OK) return rc;
        if ((rc = gemm_split_run(Pp, Tp, M, M, M, 1, s->Phi_y, st)) != FW_OK) return rc;
        if ((M & 3) == 0) {
            // mirror and squared row norms in one pass
            float* xpart = reinterpret_cast<float*>(base + psi_bytes + 3 * pb);
            const int nt = (M + 63) / 64, Mp = nt * 64;
            hipLaunchKernelGGL(mirror_rownorm_kernel, dim3(nt * (nt + 1) / 2), dim3(256), 0, st, s->Phi_y, M, Mp, xpart);
            hipLaunchKernelGGL(partial_sum_kernel, dim3((M + 15) / 16), dim3(256), 0, st, xpart, nt, M, Mp, s->xi2);
            FW_LAUNCH_CHECK();
            return FW_OK;
        }
    } else {
        rc = grad_gemm(s->T, FW_F32, M, M, s->Phi_x, Psi, st);
        if (rc != FW_OK) return rc;
        rc = grad_gemm(Psi, FW_F32, M, M, s->T, s->Phi_y, st);
        if (rc != FW_OK) return rc;
    }
    rc = symmetrize_from_lower(s->Phi_y, M, st);
    if (rc != FW_OK) return rc;
    hipLaunchKernelGGL(rownorm2_kernel, dim3((M + 3) / 4), dim3(256), 0, st, s->Phi_y, M, s->xi2);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

// Device address of `scratch` on the current device, looked up once per device (every GPU holds its own copy of the
// array at its own address).
fw_status cond_static_scratch(void** ptr, size_t* bytes) {
    constexpr int kMaxDevices = 64;
    static void* table[kMaxDevices] = {};
    static std::mutex mu;
    int dev = -1;
    FW_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return FW_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (!table[dev]) {
        void* p = nullptr;
        FW_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return FW_ERR_HIP;
        table[dev] = p;
    }
    *ptr = table[dev];
    *bytes = sizeof(scratch);
    return FW_OK;
}

fw_status cond_reduce_step(const fw_cond_state* s, const fw_cond_params* p, fw_cond_info* info, void* ws, hipStream_t st) {
    const int M = s->M;
    const WsLayout L = ws_layout(M);
    char* base = reinterpret_cast<char*>(ws);
    float* c = reinterpret_cast<float*>(base + L.c);
    float* w = reinterpret_cast<float*>(base + L.w);
    float* vt = reinterpret_cast<float*>(base + L.vt);
    float* v = reinterpret_cast<float*>(base + L.v);
    float* u = reinterpret_cast<float*>(base + L.u);
    float* t = reinterpret_cast<float*>(base + L.t);
    float* pv = reinterpret_cast<float*>(base + L.p);
    float* tpart = reinterpret_cast<float*>(base + L.tpart);
    float* ppart = reinterpret_cast<float*>(base + L.ppart);
    float* xpart = reinterpret_cast<float*>(base + L.xpart);
    Scal* sc = reinterpret_cast<Scal*>(base + L.scal);
    const dim3 mv_grid((M + 3) / 4), mv_blk(256);

    const int nmv = (M + 3) / 4, ncol = (M + 255) / 256, nred = (M + 15) / 16;
    hipLaunchKernelGGL(matvec_c_kernel, mv_grid, mv_blk, 0, st, s->Phi_y, s->xi2, M, sc, c);
    hipLaunchKernelGGL(matvec_vt_kernel, mv_grid, mv_blk, (size_t)L.Mp * sizeof(float), st, s->Phi_y, c, s->xi2, M, p->c_rel, p->c_abs, sc, vt);
    float* cur = vt;
    float* other = w;   // scratch vector for the optional refinements
    for (int it = 0; it < p->n_power_iters; ++it) {
        hipLaunchKernelGGL(matvec_refine_kernel, mv_grid, mv_blk, 0, st, s->Phi_y, cur, M, sc, other);
        float* tmp = cur; cur = other; other = tmp;
    }
    const bool leak = p->gamma < 1.f;
    const int nvm = ncol * L.nrb, last = nred * (leak ? 2 : 1);
    hipLaunchKernelGGL(matvec_u_vecmat_kernel, dim3(nmv + nvm * (leak ? 2 : 1)), mv_blk, 0, st, s->Phi_y, s->T, s->Psi, cur, M, L.Mp,
                       L.vm_rows, nmv, nvm, sc, v, u, tpart, ppart);
    hipLaunchKernelGGL(t_reduce_scalars_kernel, dim3(last + 1), mv_blk, 0, st, tpart, ppart, L.nrb, M, L.Mp, nred, last, t, pv, v, u,
                       s->lambda_bar, *p, sc, info);
    hipLaunchKernelGGL(update_kernel, dim3(L.nt * (L.nt + 1) / 2), dim3(256), 0, st, *s, v, u, t, pv, sc, p->gamma, p->beta, L.Mp, xpart);
    hipLaunchKernelGGL(partial_sum_kernel, dim3(nred), dim3(256), 0, st, xpart, L.nt, M, L.Mp, s->xi2);
    FW_LAUNCH_CHECK();
    return FW_OK;
}

}  // namespace fw
