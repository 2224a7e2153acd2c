// conv.h -- the two mesh convolutions of the Picasso paper in their depth-wise
// form (Sec. 4 "Mesh Convolution": vertex2facet with barycentric interpolation,
// facet2vertex with Gaussian-mixture fuzzy coefficients; supplementary section
// "Backward propagations of different convolutions").
//
// Features are fp32 [rows, C] row-major; one lane owns VEC consecutive channels
// of one output row, so neighbouring lanes read neighbouring addresses.  Sums
// over a vertex's facets run over its corners in ascending order (the corner
// CSR), filter gradients are reduced in two fixed stages; there are no fp
// atomics, so results do not depend on scheduling.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pooling.h"

#pragma clang fp contract(off)

namespace conv {

using pool::BLOCK;
using pool::Pack;
using pool::load_pack;
using pool::store_pack;

// Index arrays come from the caller.  They are checked once, where the corner lists are built
// (corner_keys_kernel reports a bad index); the kernels below only make sure that a bad one
// cannot reach outside the arrays: it is read as index 0.
__device__ __forceinline__ int in_range_or_zero(int i, int n) { return ((unsigned)i < (unsigned)n) ? i : 0; }

// Workgroups are handed to the 8 accelerator dies in turn, and each die has its own L2.  The facet
// rows that neighbouring vertices gather overlap (mesh numbering has locality), so the facet2vertex
// forward kernel deals its work out in 8 contiguous parts, one per die: workgroup b works as
// number (b % 8) * (G / 8) + b / 8 of a grid of G workgroups, G a multiple of 8 (xcd_grid).
__device__ __forceinline__ long long xcd_block() {
    const unsigned g8 = gridDim.x >> 3;
    return (long long)(blockIdx.x & 7u) * g8 + (blockIdx.x >> 3);
}
inline int xcd_grid(long long threads) {
    const long long g = (threads + BLOCK - 1) / BLOCK;
    return (int)((g + 7) / 8 * 8 > 0 ? (g + 7) / 8 * 8 : 8);
}

// ---------------------------------------------------------------------------
// Facet geometry: unit normal, area (Sec. 4, first paragraph) and the level k
// of Eq. "interpolate_num", k = floor((A - A_min) / (A_max - A_min)) * alpha +
// beta with A_min, A_max over the facet's own mesh.  Areas are non-negative,
// so their bit patterns order like their values and the per-mesh extremes are
// taken with integer atomics (order-independent).
// ---------------------------------------------------------------------------
__device__ __forceinline__ int mesh_of_facet(const int* __restrict__ foff, int B, int f) {
    int lo = 0, hi = B;  // invariant: foff[lo] <= f < foff[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (foff[mid] <= f) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(BLOCK) void facet_geometry_kernel(const float* __restrict__ verts, int N,
                                                               const int* __restrict__ facets, int F, int B,
                                                               const int* __restrict__ foff,
                                                               float* __restrict__ normals, float* __restrict__ areas,
                                                               unsigned* __restrict__ amin, unsigned* __restrict__ amax,
                                                               int* __restrict__ err) {
    __shared__ unsigned smin, smax;
    __shared__ int smesh, mixed;
    const int f = blockIdx.x * BLOCK + threadIdx.x;
    const bool in = f < F;
    if (threadIdx.x == 0) {
        smin = 0xFFFFFFFFu;
        smax = 0u;
        mixed = 0;
        smesh = amin ? mesh_of_facet(foff, B, blockIdx.x * BLOCK) : 0;
    }
    __syncthreads();
    int i0 = 0, i1 = 0, i2 = 0;
    if (in) {
        i0 = facets[3 * (size_t)f];
        i1 = facets[3 * (size_t)f + 1];
        i2 = facets[3 * (size_t)f + 2];
        if (i0 < 0 || i0 >= N || i1 < 0 || i1 >= N || i2 < 0 || i2 >= N) {
            atomicOr(err, 1);
            i0 = i1 = i2 = 0;
        }
    }
    const float* p0 = verts + 3 * (size_t)i0;
    const float* p1 = verts + 3 * (size_t)i1;
    const float* p2 = verts + 3 * (size_t)i2;
    const float ax = p1[0] - p0[0], ay = p1[1] - p0[1], az = p1[2] - p0[2];
    const float bx = p2[0] - p0[0], by = p2[1] - p0[1], bz = p2[2] - p0[2];
    const float nx = ay * bz - az * by;
    const float ny = az * bx - ax * bz;
    const float nz = ax * by - ay * bx;
    const float len = sqrtf((nx * nx + ny * ny) + nz * nz);
    const float area = 0.5f * len;
    if (in && areas) areas[f] = area;
    if (in && normals) {
        normals[3 * (size_t)f] = len > 0.0f ? nx / len : 0.0f;
        normals[3 * (size_t)f + 1] = len > 0.0f ? ny / len : 0.0f;
        normals[3 * (size_t)f + 2] = len > 0.0f ? nz / len : 0.0f;
    }
    if (!amin) return;
    // Extremes per mesh.  Thousands of atomics on one address queue up, so a workgroup whose facets
    // all belong to one mesh (nearly every one) first combines them in LDS and issues one pair.
    const bool counts = in && area == area;  // (a NaN area takes no part in the extremes)
    const int m = counts ? mesh_of_facet(foff, B, f) : smesh;
    if (m != smesh) mixed = 1;
    __syncthreads();
    if (mixed) {
        if (counts) {
            atomicMin(&amin[m], __float_as_uint(area));
            atomicMax(&amax[m], __float_as_uint(area));
        }
        return;
    }
    if (counts) {
        atomicMin(&smin, __float_as_uint(area));
        atomicMax(&smax, __float_as_uint(area));
    }
    __syncthreads();
    if (threadIdx.x == 0 && smin <= smax) {
        atomicMin(&amin[smesh], smin);
        atomicMax(&amax[smesh], smax);
    }
}

__global__ __launch_bounds__(BLOCK) void facet_level_kernel(const float* __restrict__ areas, int F, int B,
                                                            const int* __restrict__ foff,
                                                            const unsigned* __restrict__ amin,
                                                            const unsigned* __restrict__ amax, int alpha, int beta,
                                                            int* __restrict__ level) {
    const int f = blockIdx.x * BLOCK + threadIdx.x;
    if (f >= F) return;
    const int m = mesh_of_facet(foff, B, f);
    const float lo = __uint_as_float(amin[m]), hi = __uint_as_float(amax[m]);
    const float ratio = hi > lo ? (areas[f] - lo) / (hi - lo) : 0.0f;
    level[f] = (int)floorf(ratio) * alpha + beta;
}

// Fuzzy coefficients of the facets (Sec. 4.2): z_ft = |n_f - mu_t|^2 * inv_var_t,
// pi_ft = exp(-z_ft) / sum_m exp(-z_fm).  One lane per facet, two passes over t.
__global__ __launch_bounds__(BLOCK) void fuzzy_kernel(const float* __restrict__ normals, int F,
                                                      const float* __restrict__ mu, const float* __restrict__ inv_var,
                                                      int T, float* __restrict__ pi) {
    const int f = blockIdx.x * BLOCK + threadIdx.x;
    if (f >= F) return;
    const float nx = normals[3 * (size_t)f], ny = normals[3 * (size_t)f + 1], nz = normals[3 * (size_t)f + 2];
    float sum = 0.0f;
    for (int t = 0; t < T; ++t) {
        const float dx = nx - mu[3 * t], dy = ny - mu[3 * t + 1], dz = nz - mu[3 * t + 2];
        const float e = expf(-(((dx * dx + dy * dy) + dz * dz) * inv_var[t]));
        pi[(size_t)f * T + t] = e;
        sum = sum + e;
    }
    for (int t = 0; t < T; ++t) pi[(size_t)f * T + t] = pi[(size_t)f * T + t] / sum;
}

// ---------------------------------------------------------------------------
// Corners at every vertex: key (vertex << cbits) | corner for the sort, then the
// corner list is the keys' low part.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void corner_keys_kernel(const int* __restrict__ facets, int H, int N, int cbits,
                                                            unsigned long long* __restrict__ key,
                                                            int* __restrict__ err) {
    const int i = blockIdx.x * BLOCK + threadIdx.x;
    if (i >= H) return;
    int v = facets[i];
    if (v < 0 || v >= N) {
        atomicOr(err, 1);
        v = 0;
    }
    key[i] = ((unsigned long long)(unsigned)v << cbits) | (unsigned long long)(unsigned)i;
}

__global__ __launch_bounds__(BLOCK) void corner_list_kernel(const unsigned long long* __restrict__ skey, int H,
                                                            int cbits, int* __restrict__ corners) {
    const int i = blockIdx.x * BLOCK + threadIdx.x;
    if (i < H) corners[i] = (int)(skey[i] & ((1ull << cbits) - 1ull));
}

// ---------------------------------------------------------------------------
// Vertex2facet (Sec. 4.1).  With I_k = sum_s xi_ks I_s, W_k = sum_s xi_ks w_s and
// J = (1/K) sum_k W_k I_k the facet feature is the bilinear form J = w^T M I,
// M = (1/K) sum_k xi_k xi_k^T.  The K = k (k + 1) / 2 points of level k are the
// triangular lattice (i, j, l) / (k - 1) (the centroid alone for k = 1), whose
// moment matrix has the diagonal a = k / (6 (k - 1)) and the off-diagonal
// b = (k - 2) / (12 (k - 1)) (a = b = 1/9 for k = 1; a + 2 b = 1/3 always), so
// J = (a - b) sum_s w_s I_s + b (sum_s w_s) (sum_s I_s).
// ---------------------------------------------------------------------------
__device__ __forceinline__ void lattice_moments(int k, float& a_minus_b, float& b) {
    if (k <= 1) {
        a_minus_b = 0.0f;
        b = 1.0f / 9.0f;
        return;
    }
    const float n = (float)(k - 1);
    a_minus_b = (n + 3.0f) / (12.0f * n);
    b = (n - 1.0f) / (12.0f * n);
}

template <int VEC>
__global__ __launch_bounds__(BLOCK) void v2f_forward_kernel(const float* __restrict__ x, int N, int C,
                                                            const int* __restrict__ facets, int F,
                                                            const int* __restrict__ level,
                                                            const float* __restrict__ w, float* __restrict__ y) {
    const int Q = C / VEC;
    const long long idx = (long long)blockIdx.x * BLOCK + threadIdx.x;
    const int f = (int)(idx / Q), q = (int)(idx % Q);
    if (f >= F) return;
    float amb, b;
    lattice_moments(level ? level[f] : 1, amb, b);
    const size_t co = (size_t)q * VEC;
    Pack<VEC> xs[3], ws[3];
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        xs[s] = load_pack<VEC>(x + (size_t)in_range_or_zero(facets[3 * (size_t)f + s], N) * C + co);
        ws[s] = load_pack<VEC>(w + (size_t)s * C + co);
    }
    Pack<VEC> out;
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        const float dot = (ws[0].v[k] * xs[0].v[k] + ws[1].v[k] * xs[1].v[k]) + ws[2].v[k] * xs[2].v[k];
        const float wsum = (ws[0].v[k] + ws[1].v[k]) + ws[2].v[k];
        const float xsum = (xs[0].v[k] + xs[1].v[k]) + xs[2].v[k];
        out.v[k] = amb * dot + b * (wsum * xsum);
    }
    store_pack<VEC>(y + (size_t)f * C + co, out);
}

// dJ/dI_s = (M w)_s = (a - b) w_s + b sum_r w_r (supplementary, vertex2facet kernel), summed over
// the corners of the vertex in ascending order.
template <int VEC>
__global__ __launch_bounds__(BLOCK) void v2f_backward_x_kernel(const float* __restrict__ gy, int C,
                                                               const int* __restrict__ level,
                                                               const float* __restrict__ w,
                                                               const int* __restrict__ off,
                                                               const int* __restrict__ corners, int N, int H,
                                                               float* __restrict__ gx) {
    const int Q = C / VEC;
    const long long idx = (long long)blockIdx.x * BLOCK + threadIdx.x;
    const int v = (int)(idx / Q), q = (int)(idx % Q);
    if (v >= N) return;
    const size_t co = (size_t)q * VEC;
    Pack<VEC> ws[3], wsum, acc;
#pragma unroll
    for (int s = 0; s < 3; ++s) ws[s] = load_pack<VEC>(w + (size_t)s * C + co);
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        wsum.v[k] = (ws[0].v[k] + ws[1].v[k]) + ws[2].v[k];
        acc.v[k] = 0.0f;
    }
    const int jb = max(off[v], 0), je = min(off[v + 1], H);
    for (int j = jb; j < je; ++j) {
        const int i = in_range_or_zero(corners[j], H);
        const int f = i / 3, s = i - 3 * f;
        float amb, b;
        lattice_moments(level ? level[f] : 1, amb, b);
        const Pack<VEC> g = load_pack<VEC>(gy + (size_t)f * C + co);
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const float wk = s == 0 ? ws[0].v[k] : (s == 1 ? ws[1].v[k] : ws[2].v[k]);
            acc.v[k] = acc.v[k] + g.v[k] * (amb * wk + b * wsum.v[k]);
        }
    }
    store_pack<VEC>(gx + (size_t)v * C + co, acc);
}

// ---------------------------------------------------------------------------
// Filter gradients: a sum over all rows (facets) of ROWS values per channel, in
// two fixed stages.  Stage 1: workgroup g sums the rows [g * chunk, (g + 1) *
// chunk); lane (r, q) of it takes every R-th row of the chunk for channel pack
// q (a launch covers up to BLOCK packs), then the R lanes of a pack are summed in LDS in a fixed tree.  Stage 2
// adds the workgroups' partial sums in ascending order.
// ---------------------------------------------------------------------------
template <int ROWS, int VEC, class Term>
__global__ __launch_bounds__(BLOCK) void reduce_rows_stage1_kernel(Term term, int n_rows, int C, int chunk,
                                                                   float* __restrict__ partial, int q0, int Q) {
    extern __shared__ float lds[];  // [BLOCK][ROWS * VEC]
    // this launch takes the channel packs q0 .. q0 + Q - 1, Q <= BLOCK (the host makes as many launches as
    // the channels need)
    const int R = BLOCK / Q;
    const int r = threadIdx.x / Q, q = q0 + threadIdx.x % Q;
    float acc[ROWS * VEC];
#pragma unroll
    for (int k = 0; k < ROWS * VEC; ++k) acc[k] = 0.0f;
    const int begin = blockIdx.x * chunk;
    const int end = begin + chunk < n_rows ? begin + chunk : n_rows;
    if (r < R)
        for (int f = begin + r; f < end; f += R) term.template add<VEC>(f, q, acc);
#pragma unroll
    for (int k = 0; k < ROWS * VEC; ++k) lds[(size_t)threadIdx.x * (ROWS * VEC) + k] = (r < R) ? acc[k] : 0.0f;
    __syncthreads();
    // lanes r = 0 .. R-1 of pack q sit at threads r * Q + q: halve the number of live r each step
    for (int live = R; live > 1;) {
        const int half = (live + 1) >> 1;
        if (r < live - half) {
#pragma unroll
            for (int k = 0; k < ROWS * VEC; ++k)
                lds[(size_t)threadIdx.x * (ROWS * VEC) + k] =
                    lds[(size_t)threadIdx.x * (ROWS * VEC) + k] + lds[(size_t)(threadIdx.x + half * Q) * (ROWS * VEC) + k];
        }
        __syncthreads();
        live = half;
    }
    if (r == 0) {
#pragma unroll
        for (int row = 0; row < ROWS; ++row)
#pragma unroll
            for (int k = 0; k < VEC; ++k)
                partial[((size_t)blockIdx.x * ROWS + row) * C + (size_t)q * VEC + k] =
                    lds[(size_t)threadIdx.x * (ROWS * VEC) + row * VEC + k];
    }
}

// out[row][c] = sum over the workgroups' partials, rows < rows_used: one wave per output value,
// lane l adds the groups l, l + 64, ... in ascending order, then the 64 lanes are added in a fixed
// butterfly.
__global__ __launch_bounds__(BLOCK) void reduce_rows_stage2_kernel(const float* __restrict__ partial, int groups,
                                                                   int rows, int rows_used, int C,
                                                                   float* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int idx = blockIdx.x * (BLOCK / 64) + (threadIdx.x >> 6);
    if (idx >= rows_used * C) return;  // (whole waves leave together)
    const int row = idx / C, c = idx % C;
    float acc = 0.0f;
    for (int g = lane; g < groups; g += 64) acc = acc + partial[((size_t)g * rows + row) * C + c];
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) acc = acc + __shfl_xor(acc, d, 64);
    if (lane == 0) out[(size_t)row * C + c] = acc;
}

// dJ/dw_s = (M I)_s = (a - b) I_s + b sum_r I_r, times the incoming gradient (supplementary,
// vertex2facet kernel): the three rows of gw.
struct V2fWeightTerm {
    const float* gy;
    const float* x;
    const int* facets;
    const int* level;
    int C, N;
    template <int VEC>
    __device__ __forceinline__ void add(int f, int q, float* acc) const {
        const size_t co = (size_t)q * VEC;
        float amb, b;
        lattice_moments(level ? level[f] : 1, amb, b);
        const Pack<VEC> g = load_pack<VEC>(gy + (size_t)f * C + co);
        Pack<VEC> xs[3];
#pragma unroll
        for (int s = 0; s < 3; ++s)
            xs[s] = load_pack<VEC>(x + (size_t)in_range_or_zero(facets[3 * (size_t)f + s], N) * C + co);
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const float xsum = (xs[0].v[k] + xs[1].v[k]) + xs[2].v[k];
#pragma unroll
            for (int s = 0; s < 3; ++s) acc[s * VEC + k] = acc[s * VEC + k] + g.v[k] * (amb * xs[s].v[k] + b * xsum);
        }
    }
};

// ---------------------------------------------------------------------------
// Facet2facet (Sec. 4.1, for meshes rendered with textures): every facet has
// Gamma_f texture points with features of their own and barycentric coordinates;
// only the filter is interpolated, W_k = sum_s xi_ks w_s, and J_f = (1 / Gamma_f)
// sum_k W_k T_k.  Points of facet f = poff[f] .. poff[f+1]; tex [P,C], bary [P,3].
// One lane owns VEC channels of one facet and walks the facet's points in order.
// ---------------------------------------------------------------------------
template <int VEC>
__device__ __forceinline__ Pack<VEC> point_filter(const float* __restrict__ bary, const Pack<VEC>* ws, int k) {
    const float x0 = bary[3 * (size_t)k], x1 = bary[3 * (size_t)k + 1], x2 = bary[3 * (size_t)k + 2];
    Pack<VEC> wk;
#pragma unroll
    for (int i = 0; i < VEC; ++i) wk.v[i] = (x0 * ws[0].v[i] + x1 * ws[1].v[i]) + x2 * ws[2].v[i];
    return wk;
}

template <int VEC>
__global__ __launch_bounds__(BLOCK) void f2f_forward_kernel(const float* __restrict__ tex,
                                                            const float* __restrict__ bary,
                                                            const int* __restrict__ poff, int F, int P, int C,
                                                            const float* __restrict__ w, float* __restrict__ y) {
    const int Q = C / VEC;
    const long long idx = (long long)blockIdx.x * BLOCK + threadIdx.x;
    const int f = (int)(idx / Q), q = (int)(idx % Q);
    if (f >= F) return;
    const size_t co = (size_t)q * VEC;
    Pack<VEC> ws[3], acc;
#pragma unroll
    for (int s = 0; s < 3; ++s) ws[s] = load_pack<VEC>(w + (size_t)s * C + co);
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc.v[i] = 0.0f;
    const int kb = max(poff[f], 0), ke = min(poff[f + 1], P);
    for (int k = kb; k < ke; ++k) {
        const Pack<VEC> wk = point_filter<VEC>(bary, ws, k);
        const Pack<VEC> t = load_pack<VEC>(tex + (size_t)k * C + co);
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc.v[i] = acc.v[i] + wk.v[i] * t.v[i];
    }
    const float g = (float)(ke - kb);
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc.v[i] = (ke > kb) ? acc.v[i] / g : 0.0f;
    store_pack<VEC>(y + (size_t)f * C + co, acc);
}

// dJ/dT_k = W_k / Gamma_f, times the facet's incoming gradient: the same walk, one row written per point.
template <int VEC>
__global__ __launch_bounds__(BLOCK) void f2f_backward_tex_kernel(const float* __restrict__ gy,
                                                                 const float* __restrict__ bary,
                                                                 const int* __restrict__ poff, int F, int P, int C,
                                                                 const float* __restrict__ w,
                                                                 float* __restrict__ gtex) {
    const int Q = C / VEC;
    const long long idx = (long long)blockIdx.x * BLOCK + threadIdx.x;
    const int f = (int)(idx / Q), q = (int)(idx % Q);
    if (f >= F) return;
    const size_t co = (size_t)q * VEC;
    Pack<VEC> ws[3];
#pragma unroll
    for (int s = 0; s < 3; ++s) ws[s] = load_pack<VEC>(w + (size_t)s * C + co);
    const Pack<VEC> g = load_pack<VEC>(gy + (size_t)f * C + co);
    const int kb = max(poff[f], 0), ke = min(poff[f + 1], P);
    const float n = (float)(ke - kb);
    for (int k = kb; k < ke; ++k) {
        Pack<VEC> wk = point_filter<VEC>(bary, ws, k);
#pragma unroll
        for (int i = 0; i < VEC; ++i) wk.v[i] = (g.v[i] * wk.v[i]) / n;
        store_pack<VEC>(gtex + (size_t)k * C + co, wk);
    }
}

// dJ/dw_s = (1 / Gamma_f) sum_k xi_ks T_k, times the incoming gradient: the three rows of gw.
struct F2fWeightTerm {
    const float* gy;
    const float* tex;
    const float* bary;
    const int* poff;
    int C, P;
    template <int VEC>
    __device__ __forceinline__ void add(int f, int q, float* acc) const {
        const size_t co = (size_t)q * VEC;
        const int kb = max(poff[f], 0), ke = min(poff[f + 1], P);
        if (ke <= kb) return;
        const Pack<VEC> g = load_pack<VEC>(gy + (size_t)f * C + co);
        float m[3 * VEC];
#pragma unroll
        for (int i = 0; i < 3 * VEC; ++i) m[i] = 0.0f;
        for (int k = kb; k < ke; ++k) {
            const Pack<VEC> t = load_pack<VEC>(tex + (size_t)k * C + co);
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const float x = bary[3 * (size_t)k + s];
#pragma unroll
                for (int i = 0; i < VEC; ++i) m[s * VEC + i] = m[s * VEC + i] + x * t.v[i];
            }
        }
        const float n = (float)(ke - kb);
#pragma unroll
        for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[s * VEC + i] = acc[s * VEC + i] + (g.v[i] * m[s * VEC + i]) / n;
    }
};

// ---------------------------------------------------------------------------
// Facet2vertex (Sec. 4.2): I_v = (1 / |N(v)|) sum_{f in N(v)} (sum_t pi_ft w_t) J_f,
// N(v) = the corners at v in ascending order.
// ---------------------------------------------------------------------------
template <int VEC>
__device__ __forceinline__ Pack<VEC> fuzzy_filter(const float* __restrict__ pi, const float* __restrict__ w, int T,
                                                  int C, int f, size_t co) {
    Pack<VEC> coef;
#pragma unroll
    for (int k = 0; k < VEC; ++k) coef.v[k] = 0.0f;
    for (int t = 0; t < T; ++t) {
        const float p = pi[(size_t)f * T + t];
        const Pack<VEC> wt = load_pack<VEC>(w + (size_t)t * C + co);
#pragma unroll
        for (int k = 0; k < VEC; ++k) coef.v[k] = coef.v[k] + p * wt.v[k];
    }
    return coef;
}

// W_IN_LDS: the filter (T x C floats, at most F2V_LDS_FLOATS) is copied to LDS first, so the T
// reads per corner and lane do not go to memory.
constexpr int F2V_LDS_FLOATS = 12288;

template <int VEC, bool W_IN_LDS>
__global__ __launch_bounds__(BLOCK) void f2v_forward_kernel(const float* __restrict__ y, int C,
                                                            const float* __restrict__ pi, int T,
                                                            const float* __restrict__ w,
                                                            const int* __restrict__ off,
                                                            const int* __restrict__ corners, int N, int H,
                                                            float* __restrict__ x) {
    extern __shared__ float wl[];
    if (W_IN_LDS) {
        for (int i = threadIdx.x; i < T * C; i += BLOCK) wl[i] = w[i];
        __syncthreads();
    }
    const float* wsrc = W_IN_LDS ? wl : w;
    const int Q = C / VEC;
    const long long idx = xcd_block() * BLOCK + threadIdx.x;
    const int v = (int)(idx / Q), q = (int)(idx % Q);
    if (v >= N) return;
    const size_t co = (size_t)q * VEC;
    const int s = max(off[v], 0), e = min(off[v + 1], H);
    Pack<VEC> acc;
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc.v[k] = 0.0f;
    for (int j = s; j < e; ++j) {
        const int f = in_range_or_zero(corners[j], H) / 3;
        const Pack<VEC> coef = fuzzy_filter<VEC>(pi, wsrc, T, C, f, co);
        const Pack<VEC> yf = load_pack<VEC>(y + (size_t)f * C + co);
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc.v[k] = acc.v[k] + coef.v[k] * yf.v[k];
    }
    const float n = (float)(e - s);
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc.v[k] = (e > s) ? acc.v[k] / n : 0.0f;
    store_pack<VEC>(x + (size_t)v * C + co, acc);
}

// Incoming gradient of a facet's three vertices, each divided by its vertex's |N(v)|, summed.
template <int VEC>
__device__ __forceinline__ Pack<VEC> gathered_vertex_gradient(const float* __restrict__ gx,
                                                              const int* __restrict__ facets,
                                                              const int* __restrict__ off, int N, int C, int f,
                                                              size_t co) {
    Pack<VEC> g;
#pragma unroll
    for (int k = 0; k < VEC; ++k) g.v[k] = 0.0f;
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        const int v = in_range_or_zero(facets[3 * (size_t)f + s], N);
        const float n = (float)(off[v + 1] - off[v]);
        const Pack<VEC> gv = load_pack<VEC>(gx + (size_t)v * C + co);
#pragma unroll
        for (int k = 0; k < VEC; ++k) g.v[k] = g.v[k] + gv.v[k] / n;
    }
    return g;
}

// dI_v/dJ_f = (sum_t pi_ft w_t) / |N(v)| (supplementary, facet2vertex kernel), summed over the
// facet's three corners.
template <int VEC>
__global__ __launch_bounds__(BLOCK) void f2v_backward_y_kernel(const float* __restrict__ gx, int C,
                                                               const float* __restrict__ pi, int T,
                                                               const float* __restrict__ w,
                                                               const int* __restrict__ facets, int F,
                                                               const int* __restrict__ off, int N,
                                                               float* __restrict__ gy) {
    const int Q = C / VEC;
    const long long idx = (long long)blockIdx.x * BLOCK + threadIdx.x;
    const int f = (int)(idx / Q), q = (int)(idx % Q);
    if (f >= F) return;
    const size_t co = (size_t)q * VEC;
    const Pack<VEC> coef = fuzzy_filter<VEC>(pi, w, T, C, f, co);
    Pack<VEC> g = gathered_vertex_gradient<VEC>(gx, facets, off, N, C, f, co);
#pragma unroll
    for (int k = 0; k < VEC; ++k) g.v[k] = coef.v[k] * g.v[k];
    store_pack<VEC>(gy + (size_t)f * C + co, g);
}

// dI_v/dw_t = (1 / |N(v)|) sum_f pi_ft J_f: rows t0 .. t0 + ROWS - 1 of gw.
template <int ROWS>
struct F2vWeightTerm {
    const float* gx;
    const float* y;
    const float* pi;
    const int* facets;
    const int* off;
    int N, C, T, t0;
    template <int VEC>
    __device__ __forceinline__ void add(int f, int q, float* acc) const {
        const size_t co = (size_t)q * VEC;
        const Pack<VEC> g = gathered_vertex_gradient<VEC>(gx, facets, off, N, C, f, co);
        const Pack<VEC> yf = load_pack<VEC>(y + (size_t)f * C + co);
#pragma unroll
        for (int row = 0; row < ROWS; ++row) {
            const float p = (t0 + row < T) ? pi[(size_t)f * T + t0 + row] : 0.0f;
#pragma unroll
            for (int k = 0; k < VEC; ++k) acc[row * VEC + k] = acc[row * VEC + k] + p * (yf.v[k] * g.v[k]);
        }
    }
};

// dI_v/dpi_ft = w_t J_f / |N(v)|, summed over channels and the facet's corners: one lane per (f, t).
__global__ __launch_bounds__(BLOCK) void f2v_backward_pi_kernel(const float* __restrict__ gx, const float* __restrict__ y,
                                                                int C, int T, const float* __restrict__ w,
                                                                const int* __restrict__ facets, int F,
                                                                const int* __restrict__ off, int N,
                                                                float* __restrict__ gpi) {
    const long long idx = (long long)blockIdx.x * BLOCK + threadIdx.x;
    const int f = (int)(idx / T), t = (int)(idx % T);
    if (f >= F) return;
    float acc = 0.0f;
    for (int c = 0; c < C; ++c) {
        const Pack<1> g = gathered_vertex_gradient<1>(gx, facets, off, N, C, f, (size_t)c);
        acc = acc + w[(size_t)t * C + c] * (y[(size_t)f * C + c] * g.v[0]);
    }
    gpi[(size_t)f * T + t] = acc;
}

}  // namespace conv
