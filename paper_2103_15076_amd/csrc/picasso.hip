// picasso.hip -- round-based QEM mesh decimation for gfx950 behind the C-ABI of
// include/picasso.h.  Follows Algorithm 2 of the Picasso paper (Sec. 3) and
// the quadric equations of its supplementary section "Quadric error
// computation"; the greedy grouping that the paper leaves on the CPU
// (Alg. 2 lines 3-10) is done here on the GPU by a parallel construction of
// the same matching.
//
// All fp32 arithmetic is written as single IEEE operations in a fixed order
// and compiled without contraction, so that results are reproducible to the bit.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "../../include/picasso.h"
#include "primitives.h"
#include "pooling.h"
#include "conv.h"

#pragma clang fp contract(off)

using prim::u32;
using prim::u64;

namespace {

constexpr int BLOCK = prim::BLOCK;
constexpr u64 VMIN_NONE = ~0ull;

// ---------------------------------------------------------------------------
// Device-resident bookkeeping
// ---------------------------------------------------------------------------
struct State {
    int err;       // bit0: bad facet index, bit1: non-finite coordinate
    int nv[2];     // vertex count, ping-pong by round parity
    int nf[2];     // facet count, ping-pong
    int nh;        // 3 * nf of the current round (half-edge keys to sort)
    int ne;        // distinct edges of the current round
    int live[3];   // worklist lengths of the selection sub-rounds (rotating)
    int trunc_n;   // matched edges entering the budget truncation
    int sel_k;     // sub-round index the selection has reached (buffer rotation phase)
    int absorb_n;  // edges through which an un-paired vertex would join a pair's cluster (Alg. 2 line 11)
    int pad[3];
};

// One vertex = 64 bytes: position and the 10 quadric coefficients.
struct __attribute__((aligned(16))) VRec {
    float x, y, z, w0;
    float a00, a01, a02, a11;
    float a12, a22, b0, b1;
    float b2, c, w1, w2;
};

constexpr int MATCH_SLOTS = 32;
constexpr int MATCH_PAD = 32;  // ints: one 128-byte line per slot

struct MeshTab {       // per-mesh tables, all device pointers, B entries (+1 for offsets)
    int B;
    const int* voff;   // [B+1] current vertex offsets
    const int* target; // [B]
    const int* active; // [B] mesh takes part in this round
    const int* nrem;   // [B] pairs still to contract (budget of Alg. 2 line 4)
    int* matched;      // [B] pairs formed this round
    int* mslots;       // [B][MATCH_SLOTS][MATCH_PAD] partial pair counts, spread over cache lines so that
                       // the counting atomics of thousands of waves do not queue on one address
};

__device__ __forceinline__ int mesh_of(const int* __restrict__ voff, int B, int v) {
    if (B <= 1) return 0;
    int lo = 0, hi = B;  // invariant: voff[lo] <= v < voff[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (voff[mid] <= v) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ u32 cost_key(float c) {
    u32 u = __float_as_uint(c);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Order among pairs of equal cost (Alg. 2 line 3; Sec. 3, footnote on the shuffle inserted into the
// sorting): by edge index, or with a seed by a seeded bijection of the 32-bit integers applied to
// the edge index, so that flat regions are clustered differently from epoch to epoch.  Every step
// of enc() is invertible (xor with a constant, multiplication by an odd number, xor with a right
// shift of itself, addition of a constant); dec() undoes them in reverse.
constexpr u32 inverse_mod_2_32(u32 a) {
    u32 x = a;  // correct to 3 bits for odd a; each step doubles the number of correct bits
    for (int i = 0; i < 5; ++i) x *= 2u - a * x;
    return x;
}
constexpr u32 TIE_M1 = 0x9E3779B1u, TIE_M2 = 0x85EBCA77u;
constexpr u32 TIE_M1_INV = inverse_mod_2_32(TIE_M1), TIE_M2_INV = inverse_mod_2_32(TIE_M2);
static_assert(TIE_M1 * TIE_M1_INV == 1u && TIE_M2 * TIE_M2_INV == 1u, "modular inverses");

struct TieBreak {
    u32 on, s0, s1;
    __device__ __forceinline__ u32 enc(u32 e) const {
        if (!on) return e;
        u32 x = e ^ s0;
        x *= TIE_M1;
        x ^= x >> 15;
        x *= TIE_M2;
        x ^= x >> 13;
        return x + s1;
    }
    __device__ __forceinline__ u32 dec(u32 x) const {
        if (!on) return x;
        x -= s1;
        x ^= x >> 13;
        x ^= x >> 26;
        x *= TIE_M2_INV;
        x ^= x >> 15;
        x ^= x >> 30;
        x *= TIE_M1_INV;
        return x ^ s0;
    }
    __device__ __forceinline__ u64 priority(u32 cost_key_, int e) const { return ((u64)cost_key_ << 32) | enc((u32)e); }
};

// The same for the kernels every round runs, where the choice is made at compile time so that
// the path without shuffle carries no test of it.
template <bool SHUFFLE>
__device__ __forceinline__ u64 edge_priority(const TieBreak& tb, u32 cost_key_, int e) {
    if constexpr (SHUFFLE) return tb.priority(cost_key_, e);
    return ((u64)cost_key_ << 32) | (u32)e;
}
template <bool SHUFFLE>
__device__ __forceinline__ u32 edge_of_priority(const TieBreak& tb, u64 p) {
    if constexpr (SHUFFLE) return tb.dec((u32)p);
    return (u32)p;
}

// ---------------------------------------------------------------------------
// S0: vertex quadrics (supplementary: facet quadric Q=(nn^T, dn, d^2); vertex
// quadric = sum over adjacent facets, here in ascending facet order)
// ---------------------------------------------------------------------------

// Validates and copies the inputs into the workspace; emits the (vertex,
// incidence) pairs whose stable sort is the vertex->facet CSR.
enum { COUNT_NONE = 0, COUNT_SMALL = 1, COUNT_LARGE = 2 };

// Incidence key of corner i of the facet array: (vertex << fbits) | facet.
struct IncidenceKeys {
    const int* fcur;
    int fbits;
    __device__ __forceinline__ u64 operator()(long long i) const {
        return ((u64)(u32)fcur[i] << fbits) | (u64)(u32)(i / 3);
    }
};

// Edge key of corner i of the facet array: the side from corner i to the facet's next corner as
// (lower vertex << vbits) | higher vertex; a side with equal ends gets the all-ones key.
struct EdgeKeys {
    const int* fcur;
    int vbits;
    u64 sentinel;
    __device__ __forceinline__ u64 operator()(long long i) const {
        const long long f = i / 3;
        const int sl = (int)(i - 3 * f);
        const int a = fcur[i], b = fcur[3 * f + (sl == 2 ? 0 : sl + 1)];
        const int lo = min(a, b), hi = max(a, b);
        return (lo == hi) ? sentinel : (((u64)(u32)lo << vbits) | (u64)(u32)hi);
    }
};

// Incidence keys for S0: (vertex << fbits) | facet, one per facet corner, so that sorting the keys
// alone lists every vertex's facets in ascending facet order.  With COUNT_SMALL / COUNT_LARGE the
// kernel also adds the keys' top 8- / 12-bit digits (bits [ishift, ...)) to ihist, the histogram
// that the sort of the keys starts from (zero on entry; see quadric_reduce_kernel); that sort makes
// the keys again from the validated facet array (IncidenceKeys), so they are written out (ikey)
// only for a sort that needs them in memory.
template <int COUNT>
__global__ __launch_bounds__(BLOCK) void init_kernel(const float* __restrict__ verts, int N,
                                                     const int* __restrict__ facets, int F, int B,
                                                     const int* __restrict__ voff, const int* __restrict__ foff,
                                                     VRec* __restrict__ vrec, int* __restrict__ cid,
                                                     int* __restrict__ fcur, u64* __restrict__ ikey, int fbits,
                                                     int ishift, u32* __restrict__ ihist, State* st,
                                                     u32* __restrict__ msd_hist, int s0_follows) {
    constexpr int RADIX = COUNT == COUNT_LARGE ? (1 << prim::BUCKET_LARGE_MSD_BITS) : (1 << prim::BUCKET_MSD_BITS);
    __shared__ u32 hist[COUNT != COUNT_NONE ? RADIX : 1];
    const int stride = gridDim.x * BLOCK;
    const int g = blockIdx.x * BLOCK + threadIdx.x;
    // the edge-key sort's digit counts and cursors start every round at zero (see edge_keys_kernel)
    for (int i = g; i < 2 * prim::MSD_HIST_WORDS; i += stride) msd_hist[i] = 0;
    if constexpr (COUNT != COUNT_NONE) {
        for (int i = threadIdx.x; i < RADIX; i += BLOCK) hist[i] = 0;
        __syncthreads();
    }
    int err = 0;
    for (int w = g; w < N; w += stride) {
        float x = verts[3 * (size_t)w], y = verts[3 * (size_t)w + 1], z = verts[3 * (size_t)w + 2];
        if (!(isfinite(x) && isfinite(y) && isfinite(z))) err |= 2;
        if (!s0_follows) {  // (else quadric_reduce_kernel writes the whole record)
            VRec r;
            r.x = x; r.y = y; r.z = z; r.w0 = 0.f;
            r.a00 = r.a01 = r.a02 = r.a11 = r.a12 = r.a22 = r.b0 = r.b1 = r.b2 = r.c = r.w1 = r.w2 = 0.f;
            vrec[w] = r;
        }
        cid[w] = w;
    }
    for (int f0 = blockIdx.x * BLOCK; f0 < F; f0 += stride) {  // (whole waves, for the ballots below)
        const int f = f0 + threadIdx.x;
        const bool ok = f < F;
        int lo = 0, hi = 0;
        if (ok) {
            const int m = mesh_of(foff, B, f);
            lo = voff[m];
            hi = voff[m + 1];
        }
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            u64 k = 0;
            if (ok) {
                int a = facets[3 * (size_t)f + c];
                if (a < lo || a >= hi) { err |= 1; a = lo; }
                fcur[3 * (size_t)f + c] = a;
                k = ((u64)(u32)a << fbits) | (u64)(u32)f;
                if (ikey) ikey[3 * (size_t)f + c] = k;
            }
            if constexpr (COUNT != COUNT_NONE) {
                // neighbouring facets mostly refer to vertices with the same leading bits: a wave
                // whose keys all have one digit counts itself with a single LDS atomic
                const u32 d = (u32)(k >> ishift) & (u32)(RADIX - 1);
                const u64 on = __ballot(ok);
                if (on != 0) {
                    const u32 d0 = (u32)__builtin_amdgcn_readfirstlane((int)d);
                    if (__ballot(ok && d == d0) == on) {
                        if (ok && (on & prim::lanemask_lt()) == 0) atomicAdd(&hist[d0], (u32)__popcll(on));
                    } else if (ok) {
                        atomicAdd(&hist[d], 1u);
                    }
                }
            }
        }
    }
    if constexpr (COUNT != COUNT_NONE) {
        __syncthreads();
        for (int i = threadIdx.x; i < RADIX; i += BLOCK) {
            const u32 c = hist[i];
            if (c) atomicAdd(&ihist[i], c);
        }
    }
    if (err) atomicOr(&st->err, err);
}

// off[v] = first position of row v = key >> fbits in the sorted keys (CSR row starts)
template <typename K>
__global__ __launch_bounds__(BLOCK) void csr_offsets_kernel(const K* __restrict__ skey, int fbits, int H, int N,
                                                            int* __restrict__ off) {
    const int i = blockIdx.x * BLOCK + threadIdx.x;
    if (i >= H) return;
    const int k = (int)(skey[i] >> fbits);
    const int kp = i ? (int)(skey[i - 1] >> fbits) : -1;
    for (int v = kp + 1; v <= k; ++v) off[v] = i;
    if (i == H - 1)
        for (int v = k + 1; v <= N; ++v) off[v] = H;
}

struct Quadric10 {
    float q[10];
};

// Positions come from the caller's packed [N,3] array (12-byte stride), not from the 64-byte
// vertex records: the three gathers per incidence then touch five times fewer cache lines.
__device__ __forceinline__ Quadric10 facet_quadric(const float* __restrict__ verts, int i0, int i1, int i2) {
    Quadric10 Q;
#pragma unroll
    for (int k = 0; k < 10; ++k) Q.q[k] = 0.0f;
    if (i0 == i1 || i1 == i2 || i0 == i2) return Q;
    const float3 p0 = make_float3(verts[3 * (size_t)i0], verts[3 * (size_t)i0 + 1], verts[3 * (size_t)i0 + 2]);
    const float3 p1 = make_float3(verts[3 * (size_t)i1], verts[3 * (size_t)i1 + 1], verts[3 * (size_t)i1 + 2]);
    const float3 p2 = make_float3(verts[3 * (size_t)i2], verts[3 * (size_t)i2 + 1], verts[3 * (size_t)i2 + 2]);
    float ax = p1.x - p0.x, ay = p1.y - p0.y, az = p1.z - p0.z;
    float bx = p2.x - p0.x, by = p2.y - p0.y, bz = p2.z - p0.z;
    float nx = ay * bz - az * by;
    float ny = az * bx - ax * bz;
    float nz = ax * by - ay * bx;
    float len = sqrtf((nx * nx + ny * ny) + nz * nz);
    if (len == 0.0f) return Q;
    nx = nx / len;
    ny = ny / len;
    nz = nz / len;
    float d = -((nx * p0.x + ny * p0.y) + nz * p0.z);
    Q.q[0] = nx * nx; Q.q[1] = nx * ny; Q.q[2] = nx * nz;
    Q.q[3] = ny * ny; Q.q[4] = ny * nz; Q.q[5] = nz * nz;
    Q.q[6] = d * nx;  Q.q[7] = d * ny;  Q.q[8] = d * nz;
    Q.q[9] = d * d;
    return Q;
}

// Ordered segmented reduction: one lane per vertex walks its CSR row in
// ascending incidence order and adds the facet quadrics left to right.
__global__ __launch_bounds__(BLOCK) void quadric_reduce_kernel(VRec* __restrict__ vrec,
                                                               const float* __restrict__ verts, int N,
                                                               const int* __restrict__ fcur,
                                                               const int* __restrict__ off,
                                                               const u64* __restrict__ inc, int fbits,
                                                               u32* __restrict__ ihist) {
    const int w = blockIdx.x * BLOCK + threadIdx.x;
    // last kernel of S0: the incidence sort's digit counts and cursors go back to zero for the next call
    for (int i = w; i < 2 * prim::MSD_HIST_WORDS; i += gridDim.x * BLOCK) ihist[i] = 0;
    if (w >= N) return;
    float acc[10];
#pragma unroll
    for (int k = 0; k < 10; ++k) acc[k] = 0.0f;
    if (off) {
        const int s = off[w], e = off[w + 1];
        for (int j = s; j < e; ++j) {
            const int f = (int)(inc[j] & ((1ull << fbits) - 1ull));
            const Quadric10 Q = facet_quadric(verts, fcur[3 * (size_t)f], fcur[3 * (size_t)f + 1], fcur[3 * (size_t)f + 2]);
#pragma unroll
            for (int k = 0; k < 10; ++k) acc[k] = acc[k] + Q.q[k];
        }
    }
    float4* r = reinterpret_cast<float4*>(&vrec[w]);
    r[0] = make_float4(verts[3 * (size_t)w], verts[3 * (size_t)w + 1], verts[3 * (size_t)w + 2], 0.f);
    r[1] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    r[2] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    r[3] = make_float4(acc[8], acc[9], 0.f, 0.f);
}

// ---------------------------------------------------------------------------
// Round set-up
// ---------------------------------------------------------------------------
struct RoundTab {
    int B;
    const int* voff;
    const int* target;
    int* active;
    int* stuck;
    int* nrem;
    int* matched;
    int* mslots;
    int first_round;
};

// Per-mesh budgets and the round's counters, by one workgroup.
__device__ __forceinline__ void round_begin_block(const RoundTab& R, int cur, State* st) {
    for (int i = threadIdx.x; i < R.B * MATCH_SLOTS; i += blockDim.x) R.mslots[(size_t)i * MATCH_PAD] = 0;
    for (int b = threadIdx.x; b < R.B; b += blockDim.x) {
        const int nvb = R.voff[b + 1] - R.voff[b];
        if (!R.first_round && R.active[b] && R.matched[b] == 0) R.stuck[b] = 1;
        const int act = (nvb > R.target[b]) && !R.stuck[b];
        R.active[b] = act;
        R.nrem[b] = act ? nvb - R.target[b] : 0;
        R.matched[b] = 0;
    }
    if (threadIdx.x == 0) {
        st->nh = 3 * st->nf[cur];
        st->ne = 0;
        st->live[0] = 0;
        st->live[1] = 0;
        st->live[2] = 0;
        st->trunc_n = 0;
        st->sel_k = 0;
        st->absorb_n = 0;
    }
}

// ---------------------------------------------------------------------------
// S1: candidate pairs = distinct mesh edges (Alg. 2 line 1)
//
// First kernel of a round: the round's set-up (block 0), the per-vertex selection state, and one
// 64-bit key (lower vertex, higher vertex) per half-edge, key i for corner i of the facet array.
// With COUNT_SMALL / COUNT_LARGE the kernel also adds the keys' top 8- / 12-bit digits to the
// histogram that the sort of the keys starts from (prim::bucket_sort / prim::bucket_sort_large
// with `counted`; zeroed beforehand), so the sort needs no counting pass of its own.
// ---------------------------------------------------------------------------
template <int COUNT>
__global__ __launch_bounds__(BLOCK) void edge_keys_kernel(const int* __restrict__ fcur, State* st, int cur, int vbits,
                                                          u64* __restrict__ keys, u64* __restrict__ vmin0,
                                                          u64* __restrict__ vmin1, int* __restrict__ mate,
                                                          RoundTab R, int shift, u32* __restrict__ msd_hist) {
    constexpr int ITEMS = COUNT == COUNT_LARGE ? prim::SORT_ITEMS_BIG : prim::SORT_ITEMS_SMALL;
    constexpr int TILE = BLOCK * ITEMS;
    constexpr int RADIX = COUNT == COUNT_LARGE ? (1 << prim::BUCKET_LARGE_MSD_BITS) : (1 << prim::BUCKET_MSD_BITS);
    __shared__ u32 hist[COUNT != COUNT_NONE ? RADIX : 1];
    const int nf = st->nf[cur], nv = st->nv[cur];
    const long long n = 3ll * nf;
    const int stride = gridDim.x * BLOCK;
    const int t = threadIdx.x, g = blockIdx.x * BLOCK + t;
    const u64 sentinel = (vbits >= 32) ? ~0ull : ((1ull << (2 * vbits)) - 1ull);
    for (int w = g; w < nv; w += stride) {
        vmin0[w] = VMIN_NONE;
        vmin1[w] = VMIN_NONE;
        mate[w] = -1;
    }
    if (blockIdx.x == 0) round_begin_block(R, cur, st);
    for (long long tile = blockIdx.x; tile * TILE < n; tile += gridDim.x) {
        if constexpr (COUNT != COUNT_NONE) {
            for (int i = t; i < RADIX; i += BLOCK) hist[i] = 0;
            __syncthreads();
        }
#pragma unroll 4
        for (int i = 0; i < ITEMS; ++i) {
            const long long idx = tile * TILE + (long long)i * BLOCK + t;
            const bool ok = idx < n;
            u64 k = 0;
            if (ok) {
                k = EdgeKeys{fcur, vbits, sentinel}(idx);
                if (keys) keys[idx] = k;  // (the counted sorts make the keys again from fcur)
            }
            if constexpr (COUNT != COUNT_NONE) {
                // the lower vertices of neighbouring corners mostly share their leading bits: a wave
                // whose keys all have one digit counts itself with a single LDS atomic
                const u32 d = (u32)(k >> shift) & (u32)(RADIX - 1);
                const u64 on = __ballot(ok);
                if (on != 0) {
                    const u32 d0 = (u32)__builtin_amdgcn_readfirstlane((int)d);
                    if (__ballot(ok && d == d0) == on) {
                        if (ok && (on & prim::lanemask_lt()) == 0) atomicAdd(&hist[d0], (u32)__popcll(on));
                    } else if (ok) {
                        atomicAdd(&hist[d], 1u);
                    }
                }
            }
        }
        if constexpr (COUNT != COUNT_NONE) {
            __syncthreads();
            for (int i = t; i < RADIX; i += BLOCK) {
                const u32 c = hist[i];
                if (c) atomicAdd(&msd_hist[i], c);
            }
            __syncthreads();
        }
    }
}

struct UniquePred {
    const u64* keys;
    u64 sentinel;
    __device__ bool operator()(int i) const {
        const u64 k = keys[i];
        return k != sentinel && (i == 0 || k != keys[i - 1]);
    }
};

// Where a pair is contracted to.
enum { PLACE_MEAN = 0, PLACE_INVERSE = 1 };

// Point of least quadric error, the solution of A x = -b (supplementary,
// inverse placement equation), for a positive semi-definite A = sum of n n^T.
// The three axes are eliminated in the order of the largest remaining diagonal
// entry (P A P^T = L D L^T); A counts as of full rank when all three pivots are
// positive and the last exceeds rcond_min times the first, their ratio standing
// for the reciprocal condition number.  Returns false, leaving (x, y, z) as
// they are, when A is not of full rank or the solution is not finite.
__device__ __forceinline__ bool quadric_minimiser(float a00, float a01, float a02, float a11, float a12, float a22,
                                                  float b0, float b1, float b2, float rcond_min, float& x, float& y,
                                                  float& z) {
    float r0 = -b0, r1 = -b1, r2 = -b2, t;
    int first = 0;
    float top = a00;
    if (a11 > top) { first = 1; top = a11; }
    if (a22 > top) { first = 2; top = a22; }
    if (first == 1) {  // axes 0 and 1 change places
        t = a00; a00 = a11; a11 = t;
        t = a02; a02 = a12; a12 = t;
        t = r0; r0 = r1; r1 = t;
    } else if (first == 2) {  // axes 0 and 2 change places
        t = a00; a00 = a22; a22 = t;
        t = a01; a01 = a12; a12 = t;
        t = r0; r0 = r2; r2 = t;
    }
    const float d1 = a00;
    if (!(d1 > 0.0f)) return false;
    float l1 = a01 / d1, l2 = a02 / d1;
    float s11 = a11 - (a01 * a01) / d1;
    const float s12 = a12 - (a01 * a02) / d1;
    float s22 = a22 - (a02 * a02) / d1;
    const bool flip = s22 > s11;  // the larger entry of the remaining block goes next
    if (flip) {
        t = s11; s11 = s22; s22 = t;
        t = l1; l1 = l2; l2 = t;
        t = r1; r1 = r2; r2 = t;
    }
    const float d2 = s11;
    if (!(d2 > 0.0f)) return false;
    const float l3 = s12 / d2;
    const float d3 = s22 - l3 * s12;
    if (!(d3 > 0.0f) || !(d3 > rcond_min * d1)) return false;
    const float y1 = r1 - l1 * r0;
    const float y2 = (r2 - l2 * r0) - l3 * y1;
    float w2 = y2 / d3;
    float w1 = y1 / d2 - l3 * w2;
    float w0 = (r0 / d1 - l1 * w1) - l2 * w2;
    if (flip) { t = w1; w1 = w2; w2 = t; }
    if (first == 1) { t = w0; w0 = w1; w1 = t; }
    else if (first == 2) { t = w0; w0 = w2; w2 = t; }
    if (!isfinite(w0) || !isfinite(w1) || !isfinite(w2)) return false;
    x = w0; y = w1; z = w2;
    return true;
}

// S2: cost of a pair = quadric error of the summed quadric at the point the
// pair would be contracted to: the pair's mean, or with PLACE_INVERSE the point
// of least error where the quadric has one (Alg. 2 line 2; supplementary
// Q(x) = x^T A x + 2 b^T x + c and the two placement equations).
template <int PLACE>
__device__ __forceinline__ float pair_cost(const VRec* __restrict__ vrec, int u, int v, float rcond_min) {
    const float4* ru = reinterpret_cast<const float4*>(&vrec[u]);
    const float4* rv = reinterpret_cast<const float4*>(&vrec[v]);
    const float4 u0 = ru[0], u1 = ru[1], u2 = ru[2], u3 = ru[3];
    const float4 v0 = rv[0], v1 = rv[1], v2 = rv[2], v3 = rv[3];
    const float a00 = u1.x + v1.x, a01 = u1.y + v1.y, a02 = u1.z + v1.z, a11 = u1.w + v1.w;
    const float a12 = u2.x + v2.x, a22 = u2.y + v2.y, b0 = u2.z + v2.z, b1 = u2.w + v2.w;
    const float b2 = u3.x + v3.x, c = u3.y + v3.y;
    float mx = (u0.x + v0.x) * 0.5f;
    float my = (u0.y + v0.y) * 0.5f;
    float mz = (u0.z + v0.z) * 0.5f;
    if (PLACE == PLACE_INVERSE) quadric_minimiser(a00, a01, a02, a11, a12, a22, b0, b1, b2, rcond_min, mx, my, mz);
    const float t0 = (a00 * mx + a01 * my) + a02 * mz;
    const float t1 = (a01 * mx + a11 * my) + a12 * mz;
    const float t2 = (a02 * mx + a12 * my) + a22 * mz;
    const float xAx = (mx * t0 + my * t1) + mz * t2;
    const float bx = (b0 * mx + b1 * my) + b2 * mz;
    return (xAx + 2.0f * bx) + c;
}

// Bids of the lanes of one wave on their vertices x, where lanes with equal x are neighbours among
// the lanes that bid (edges are sorted by their lower vertex, so that end of consecutive edges is
// often the same vertex).  Atomics of one wave on one address are served one after the other, so
// each such group first takes the minimum of its priorities across lanes and its last lane issues
// the group's single atomicMin.  Every lane of the wave must call this.
__device__ __forceinline__ void bid_grouped(u64* __restrict__ vmin, bool on, int x, u64 p) {
    const int lane = prim::lane_id();
    const u64 ab = __ballot(on);
    if (ab == 0) return;
    const u64 lt = prim::lanemask_lt();
    const u64 below = ab & lt;
    const int prev = below ? 63 - __clzll((long long)below) : lane;
    const int xprev = __shfl(x, prev, 64);
    const bool head = on && (below == 0 || xprev != x);
    const u64 hb = __ballot(head);
    const u64 hle = hb & (lt | (1ull << lane));
    const int dist = hle ? lane - (63 - __clzll((long long)hle)) : 0;  // lanes back to the group's head
    u64 q = on ? p : ~0ull;
    for (int d = 1; d < 64; d <<= 1) {
        if (!__any(dist >= d)) break;
        const u64 o = __shfl_up(q, d, 64);
        if (dist >= d) q = (o < q) ? o : q;
    }
    const u64 above = ab & ~(lt | (1ull << lane));
    const bool tail = on && (above == 0 || ((hb >> (__ffsll((long long)above) - 1)) & 1ull));
    if (tail) atomicMin(&vmin[x], q);
}

// Writes the distinct edges, their cost keys, and places each edge's first bid
// (sub-round 0 of the selection) on both of its vertices.
template <int PLACE, bool SHUFFLE>
struct UniqueOutT {
    static constexpr bool WAVE_WIDE = true;
    const u64* keys;
    u64* ekey;
    u32* ecost;
    const VRec* vrec;
    u64* vmin0;
    unsigned char* estate;
    int vbits;
    MeshTab mt;
    float rcond_min;
    TieBreak tb;
    __device__ void wave(int i, bool in_range, bool flagged, int e) const {
        bool act = false;
        int u = 0;
        u64 p = 0;
        if (flagged) {
            const u64 k = keys[i];
            u = (int)(k >> vbits);
            const int v = (int)(k & ((1ull << vbits) - 1ull));
            ekey[e] = k;
            const u32 ck = cost_key(pair_cost<PLACE>(vrec, u, v, rcond_min));
            ecost[e] = ck;
            act = mt.active[mesh_of(mt.voff, mt.B, u)] != 0;
            estate[e] = act ? 0 : 1;
            p = edge_priority<SHUFFLE>(tb, ck, e);
            if (act) atomicMin(&vmin0[v], p);
        }
        (void)in_range;
        bid_grouped(vmin0, act, u, p);
    }
};

// ---------------------------------------------------------------------------
// S3: greedy disjoint grouping of Alg. 2 lines 3-10, computed in parallel.
//
// Priority of edge e = (cost key, e) packed in 64 bits; the sequential loop of
// the paper visits edges in ascending priority.  An edge is LIVE while neither
// end is paired.  A live edge whose priority is the minimum among the live
// edges at BOTH ends is exactly one the sequential loop accepts, so every
// sub-round accepts all such edges at once, retires the edges touching newly
// paired vertices, and lets the survivors bid again.  vmin buffers rotate:
// sub-round k reads bids in vmin[k%3], places the survivors' bids in
// vmin[(k+1)%3] and clears their slots in vmin[(k+2)%3].
// ---------------------------------------------------------------------------
constexpr int SEL_ITEMS = 1;
constexpr int SEL_TILE = BLOCK * SEL_ITEMS;
constexpr int TAIL_THREADS = 1024;
constexpr int TAIL_MAX = 3584;  // live edges the single-workgroup tail takes over (sized by its LDS state)

struct SelArgs {
    const u64* ekey;
    const u32* ecost;
    u64* vmin[3];
    int* mate;
    int* list;              // live edges gathered for the tail
    unsigned char* estate;  // per edge: 0 = live, 1 = retired (paired, or an end was paired)
    State* st;
    MeshTab mt;
    int vbits;
    int* host_img;     // pinned host memory, device view: the tail leaves [State][matched] there
    int publish_ints;  // for the host, which then needs no copy of its own before it looks
    TieBreak tb;       // order among edges of equal cost
};

// Bids are read with device-scope atomic loads where the same kernel also
// changes them (the tail), with plain loads otherwise.
template <bool COHERENT>
__device__ __forceinline__ u64 load_bid(const u64* p) {
    if (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
}

template <bool COHERENT, bool SHUFFLE>
__device__ __forceinline__ bool vertex_pairs_now(const u64* __restrict__ cur, const u64* __restrict__ ekey, int vbits,
                                                 const TieBreak& tb, int x, u64 mx) {
    // The best live edge at x is accepted in this sub-round iff it is also the best at its other end.
    if (mx == VMIN_NONE) return false;  // no bid on x (cannot happen for an end of a live edge)
    const u64 k = ekey[edge_of_priority<SHUFFLE>(tb, mx)];
    const int a = (int)(k >> vbits), b = (int)(k & ((1ull << vbits) - 1ull));
    const int other = (a == x) ? b : a;
    return load_bid<COHERENT>(&cur[other]) == mx;
}

// One edge of one sub-round.  Returns true if the edge stays live.
template <bool COHERENT, bool SHUFFLE>
__device__ __forceinline__ bool subround_edge(const SelArgs& A, const u64* __restrict__ cur, int k, int e, int& u,
                                              int& v, int& m, u64& p, bool& sel) {
    const u64 key = A.ekey[e];
    u = (int)(key >> A.vbits);
    v = (int)(key & ((1ull << A.vbits) - 1ull));
    p = edge_priority<SHUFFLE>(A.tb, A.ecost[e], e);
    m = mesh_of(A.mt.voff, A.mt.B, u);
    sel = false;
    if (k == 0 && !A.mt.active[m]) return false;
    const u64 mu = load_bid<COHERENT>(&cur[u]), mv = load_bid<COHERENT>(&cur[v]);
    if (mu == p && mv == p) {
        sel = true;
        A.mate[u] = v;
        A.mate[v] = u;
        return false;
    }
    return !(vertex_pairs_now<COHERENT, SHUFFLE>(cur, A.ekey, A.vbits, A.tb, u, mu) ||
             vertex_pairs_now<COHERENT, SHUFFLE>(cur, A.ekey, A.vbits, A.tb, v, mv));
}

// pairs formed, counted per mesh: one atomic per wave and mesh
__device__ __forceinline__ void count_pairs(const SelArgs& A, bool sel, int m) {
    const int lane = prim::lane_id();
    u64 sb = __ballot(sel);
    while (sb) {
        const int leader = __ffsll((long long)sb) - 1;
        const int m0 = __shfl(m, leader, 64);
        const u64 same = __ballot(sel && m == m0);
        if (lane == leader)
            atomicAdd(&A.mt.mslots[((size_t)m0 * MATCH_SLOTS + (blockIdx.x & (MATCH_SLOTS - 1))) * MATCH_PAD],
                      (int)__popcll(same));
        sb &= ~same;
    }
}

// The same into an LDS array (one workgroup's own tally).
__device__ __forceinline__ void count_pairs_lds(int* pairs, bool sel, int m) {
    const int lane = prim::lane_id();
    u64 sb = __ballot(sel);
    while (sb) {
        const int leader = __ffsll((long long)sb) - 1;
        const int m0 = __shfl(m, leader, 64);
        const u64 same = __ballot(sel && m == m0);
        if (lane == leader) atomicAdd(&pairs[m0], (int)__popcll(same));
        sb &= ~same;
    }
}

// Grid-wide sub-round over ALL edges of the round; retired edges are skipped by
// their state byte.  No worklist is kept here: appending survivors would need
// one returning atomic per workgroup on a single counter, and thousands of
// those queue up for longer than the sub-round itself takes.
template <bool SHUFFLE>
__global__ __launch_bounds__(BLOCK) void select_subround_kernel(SelArgs A, int k) {
    const u64* __restrict__ cur = A.vmin[k % 3];
    u64* __restrict__ nxt = A.vmin[(k + 1) % 3];
    u64* __restrict__ rst = A.vmin[(k + 2) % 3];
    const int n = A.st->ne;
    if (blockIdx.x == 0 && threadIdx.x == 0) A.st->sel_k = k + 1;
    for (long long base = (long long)blockIdx.x * BLOCK; base < n; base += (long long)gridDim.x * BLOCK) {
        const long long i = base + threadIdx.x;
        bool alive = false, sel = false;
        int u = 0, v = 0, m = 0;
        u64 p = 0;
        const bool live_in = (i < n) && A.estate[i] == 0;
        if (live_in) alive = subround_edge<false, SHUFFLE>(A, cur, k, (int)i, u, v, m, p, sel);
        count_pairs(A, sel, m);
        if (alive) {
            atomicMin(&nxt[v], p);
            rst[u] = VMIN_NONE;
            rst[v] = VMIN_NONE;
        } else if (live_in) {
            A.estate[i] = 1;
        }
        bid_grouped(nxt, alive, u, p);
    }
}

// The same sub-round for large rounds once most edges are retired (every sub-round but the
// first).  One lane per edge would then spend a wave, and a trip to memory, on every 64 state
// bytes; here a lane reads the state of 16 consecutive edges at once, the wave lists its live
// edges in LDS in ascending order (1024 edges per wave), and the lanes then work through that
// list 64 edges at a time exactly as above.
constexpr int SPARSE_MIN_EDGES = 1 << 20;  // below this the one-lane-per-edge kernel is at its launch floor anyway

template <int SPARSE_EDGES_PER_LANE, bool SHUFFLE>  // 4 while about a third of the edges are live, 16 later
__global__ __launch_bounds__(BLOCK) void select_subround_sparse_kernel(SelArgs A, int k) {
    static_assert(SPARSE_EDGES_PER_LANE == 4 || SPARSE_EDGES_PER_LANE == 16, "one 4- or 16-byte load per lane");
    constexpr int PER_WAVE = 64 * SPARSE_EDGES_PER_LANE;
    __shared__ int slist[prim::WAVES][PER_WAVE];
    const u64* __restrict__ cur = A.vmin[k % 3];
    u64* __restrict__ nxt = A.vmin[(k + 1) % 3];
    u64* __restrict__ rst = A.vmin[(k + 2) % 3];
    const int n = A.st->ne;
    if (blockIdx.x == 0 && threadIdx.x == 0) A.st->sel_k = k + 1;
    const int lane = prim::lane_id(), w = prim::wave_id();
    int* list = slist[w];
    for (long long cbase = ((long long)blockIdx.x * prim::WAVES + w) * PER_WAVE; cbase < n;
         cbase += (long long)gridDim.x * prim::WAVES * PER_WAVE) {
        const long long b0 = cbase + (long long)lane * SPARSE_EDGES_PER_LANE;
        u32 sw[4] = {0x01010101u, 0x01010101u, 0x01010101u, 0x01010101u};  // "retired" beyond the end
        if (b0 + SPARSE_EDGES_PER_LANE <= n) {
            if constexpr (SPARSE_EDGES_PER_LANE == 16) {
                const uint4 q = *reinterpret_cast<const uint4*>(A.estate + b0);
                sw[0] = q.x; sw[1] = q.y; sw[2] = q.z; sw[3] = q.w;
            } else {
                sw[0] = *reinterpret_cast<const u32*>(A.estate + b0);
            }
        } else {
            for (int j = 0; j < SPARSE_EDGES_PER_LANE; ++j)
                if (b0 + j < n && A.estate[b0 + j] == 0) sw[j >> 2] &= ~(0xFFu << (8 * (j & 3)));
        }
        u32 livebits = 0;
#pragma unroll
        for (int j = 0; j < SPARSE_EDGES_PER_LANE; ++j)
            if (((sw[j >> 2] >> (8 * (j & 3))) & 0xFFu) == 0) livebits |= 1u << j;
        const int c = __popc(livebits);
        int incl = c;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(incl, d, 64);
            if (lane >= d) incl += o;
        }
        const int total = __shfl(incl, 63, 64);
        int pos = incl - c;
        while (livebits) {
            const int j = __ffs((int)livebits) - 1;
            livebits &= livebits - 1;
            list[pos++] = (int)(b0 + j);
        }
        __builtin_amdgcn_wave_barrier();  // (a wave's LDS operations complete in order)
        for (int q = 0; q < total; q += 64) {
            const bool has = q + lane < total;
            const int i = has ? list[q + lane] : 0;
            bool alive = false, sel = false;
            int u = 0, v = 0, m = 0;
            u64 p = 0;
            if (has) alive = subround_edge<false, SHUFFLE>(A, cur, k, i, u, v, m, p, sel);
            count_pairs(A, sel, m);
            if (alive) {
                atomicMin(&nxt[v], p);
                rst[u] = VMIN_NONE;
                rst[v] = VMIN_NONE;
            } else if (has) {
                A.estate[i] = 1;
            }
            bid_grouped(nxt, alive, u, p);
        }
        __builtin_amdgcn_wave_barrier();
    }
}

struct LivePred {
    const unsigned char* estate;
    __device__ bool operator()(int e) const { return estate[e] == 0; }
};

struct LiveOut {
    int* list;
    __device__ void operator()(int e, int pos) const { list[pos] = e; }
};

// Tail: once few edges are live, one workgroup finishes the matching with all
// of its state in LDS: the live edges' priorities, a hash map from the (at
// most 2 x TAIL_MAX) vertices they touch to LDS slots, and one 64-bit bid per
// slot.  A sub-round then costs four workgroup barriers instead of a kernel
// launch and several trips to memory.  The live count falls in every
// sub-round (the best live edge is always accepted), so the loop ends.
// A slot's bid doubles as its "paired" mark (TAIL_PAIRED is below every real
// priority: a finite cost never has cost key 0).
constexpr int TAIL_SLOTS = 8192;  // power of two, >= 2 * TAIL_MAX
constexpr int TAIL_LDS_MESHES = 1024;
constexpr u64 TAIL_PAIRED = 0ull;

struct TailLds {
    u64 prio[TAIL_MAX];
    u64 bid[TAIL_SLOTS];
    int vkey[TAIL_SLOTS];
    unsigned short su[TAIL_MAX], sv[TAIL_MAX];
    unsigned short lst[2][TAIL_MAX];
    int cnt[2];
    int pairs[TAIL_LDS_MESHES];  // pairs this kernel formed, per mesh (batches of up to this many meshes)
};

__device__ __forceinline__ int tail_slot(int* vkey, int v) {
    u32 h = ((u32)v * 0x9E3779B1u) >> 19;  // 13 bits
    for (;;) {
        const int old = atomicCAS(&vkey[h], -1, v);
        if (old == -1 || old == v) return (int)h;
        h = (h + 1) & (TAIL_SLOTS - 1);
    }
}

// The round's counters and pair counts, written straight into the host's pinned memory (read at
// the L2, where this kernel's own stores to them already are).
__device__ __forceinline__ void tail_publish(const SelArgs& A, int tid) {
    const int* hdr = reinterpret_cast<const int*>(A.st);
    for (int i = tid; i < A.publish_ints; i += TAIL_THREADS)
        A.host_img[i] = __hip_atomic_load(&hdr[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(TAIL_THREADS) void select_tail_kernel(SelArgs A) {
    __shared__ TailLds L;
    int n = A.st->live[0];     // live edges, gathered into A.list just before this kernel
    const int tid = threadIdx.x, lane = prim::lane_id();
    if (n > TAIL_MAX) {        // too many: the host runs more grid-wide sub-rounds
        tail_publish(A, tid);
        return;
    }
    const u64 lt = prim::lanemask_lt();
    const u64 vmask = (1ull << A.vbits) - 1ull;

    // Up to TAIL_LDS_MESHES meshes, the pairs formed here are tallied in LDS and added to the earlier
    // kernels' counters at the end; that way nothing this kernel writes to memory is read back by
    // it, and it needs no device-wide fence (which costs several microseconds here).
    const bool lds_pairs = A.mt.B <= TAIL_LDS_MESHES;
    if (lds_pairs)
        for (int b = tid; b < A.mt.B; b += TAIL_THREADS) L.pairs[b] = 0;
    for (int h = tid; h < TAIL_SLOTS; h += TAIL_THREADS) L.vkey[h] = -1;
    __syncthreads();
    for (int i = tid; i < n; i += TAIL_THREADS) {
        const int e = A.list[i];
        const u64 key = A.ekey[e];
        L.prio[i] = A.tb.priority(A.ecost[e], e);
        L.su[i] = (unsigned short)tail_slot(L.vkey, (int)(key >> A.vbits));
        L.sv[i] = (unsigned short)tail_slot(L.vkey, (int)(key & vmask));
        L.lst[0][i] = (unsigned short)i;
    }
    int side = 0;
    __syncthreads();

    while (n > 0) {
        const int padded = (n + 63) & ~63;  // whole waves run each step so that the ballots are uniform
        // clear the bids of every vertex that still has a live edge
        for (int j = tid; j < n; j += TAIL_THREADS) {
            const int i = L.lst[side][j];
            L.bid[L.su[i]] = VMIN_NONE;
            L.bid[L.sv[i]] = VMIN_NONE;
        }
        if (tid == 0) L.cnt[side ^ 1] = 0;
        __syncthreads();
        for (int j = tid; j < n; j += TAIL_THREADS) {
            const int i = L.lst[side][j];
            atomicMin(&L.bid[L.su[i]], L.prio[i]);
            atomicMin(&L.bid[L.sv[i]], L.prio[i]);
        }
        __syncthreads();
        // accept the edges that hold the best bid at both ends
        bool mine[(TAIL_MAX + TAIL_THREADS - 1) / TAIL_THREADS];
        int q = 0;
        for (int j = tid; j < padded; j += TAIL_THREADS, ++q) {
            bool sel = false;
            int m = 0;
            if (j < n) {
                const int i = L.lst[side][j];
                const u64 p = L.prio[i];
                sel = (L.bid[L.su[i]] == p) && (L.bid[L.sv[i]] == p);
                if (sel) {
                    const int u = L.vkey[L.su[i]], v = L.vkey[L.sv[i]];
                    A.mate[u] = v;
                    A.mate[v] = u;
                    m = mesh_of(A.mt.voff, A.mt.B, u);
                }
            }
            mine[q] = sel;
            if (lds_pairs) count_pairs_lds(L.pairs, sel, m);
            else count_pairs(A, sel, m);
        }
        __syncthreads();
        q = 0;
        for (int j = tid; j < n; j += TAIL_THREADS, ++q)
            if (mine[q]) {
                const int i = L.lst[side][j];
                L.bid[L.su[i]] = TAIL_PAIRED;
                L.bid[L.sv[i]] = TAIL_PAIRED;
            }
        __syncthreads();
        // keep the edges whose ends are both still free
        for (int j = tid; j < padded; j += TAIL_THREADS) {
            bool alive = false;
            int i = 0;
            if (j < n) {
                i = L.lst[side][j];
                alive = (L.bid[L.su[i]] != TAIL_PAIRED) && (L.bid[L.sv[i]] != TAIL_PAIRED);
            }
            const u64 ab = __ballot(alive);
            if (ab) {
                int wbase = 0;
                if (lane == 0) wbase = atomicAdd(&L.cnt[side ^ 1], (int)__popcll(ab));
                wbase = __shfl(wbase, 0, 64);
                if (alive) L.lst[side ^ 1][wbase + (int)__popcll(ab & lt)] = (unsigned short)i;
            }
        }
        __syncthreads();
        side ^= 1;
        n = L.cnt[side];
        __syncthreads();
    }

    static_assert(MATCH_SLOTS == 32, "a mesh's slots fill half a wave");
    constexpr int STATE_INTS = (int)(sizeof(State) / sizeof(int));
    if (!lds_pairs) {
        __threadfence();  // the pair counts added above are at the L2 before they are summed
        __syncthreads();
    }
    // one lane per counter slot (a mesh's MATCH_SLOTS slots sit in neighbouring lanes), so that the
    // loads are in flight together; whole waves run each step for the shuffles
    for (int base = 0; base < A.mt.B * MATCH_SLOTS; base += TAIL_THREADS) {
        const int idx = base + tid;
        const bool ok = idx < A.mt.B * MATCH_SLOTS;
        int sum = 0;
        if (ok) sum = __hip_atomic_load(&A.mt.mslots[(size_t)idx * MATCH_PAD], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int d = MATCH_SLOTS / 2; d > 0; d >>= 1) sum += __shfl_xor(sum, d, 64);
        if (ok && (idx & (MATCH_SLOTS - 1)) == 0) {
            const int b = idx / MATCH_SLOTS;
            if (lds_pairs) sum += L.pairs[b];
            A.mt.matched[b] = sum;
            if (lds_pairs && STATE_INTS + b < A.publish_ints) A.host_img[STATE_INTS + b] = sum;
        }
    }
    if (tid == 0) A.st->live[0] = 0;
    if (lds_pairs) {
        // the host's copy of the counters: everything but live[0] was written by earlier kernels
        constexpr int LIVE0 = (int)(offsetof(State, live) / sizeof(int));
        const int* hdr = reinterpret_cast<const int*>(A.st);
        if (tid < STATE_INTS && tid < A.publish_ints) A.host_img[tid] = (tid == LIVE0) ? 0 : hdr[tid];
    } else {
        __threadfence();
        __syncthreads();
        tail_publish(A, tid);
    }
}

// ---------------------------------------------------------------------------
// S2b + budget (Alg. 2 lines 3-4, 6): when a mesh formed more pairs than it may
// remove, only its n_rem pairs of smallest (cost, edge index) stay.  The pairs
// are gathered in edge order, sorted stably by (mesh, cost key), and the tail
// of each mesh's run is released.
// ---------------------------------------------------------------------------
struct TruncPred {
    const u64* ekey;
    const int* mate;
    MeshTab mt;
    int vbits;
    __device__ bool operator()(int e) const {
        const u64 k = ekey[e];
        const int u = (int)(k >> vbits), v = (int)(k & ((1ull << vbits) - 1ull));
        if (mate[u] != v) return false;
        const int m = mesh_of(mt.voff, mt.B, u);
        return mt.matched[m] > mt.nrem[m];
    }
};

struct TruncOut {
    const u64* ekey;
    const u32* ecost;
    u64* tkey;
    u32* tval;
    MeshTab mt;
    int vbits;
    __device__ void operator()(int e, int pos) const {
        const int u = (int)(ekey[e] >> vbits);
        tkey[pos] = ((u64)(u32)mesh_of(mt.voff, mt.B, u) << 32) | (u64)ecost[e];
        tval[pos] = (u32)e;
    }
};

// The same gather for the one-workgroup-per-mesh selection below: cost keys and edges apart.
struct TruncOutSplit {
    const u32* ecost;
    u32* tcost;
    u32* tval;
    __device__ void operator()(int e, int pos) const {
        tcost[pos] = ecost[e];
        tval[pos] = (u32)e;
    }
};

// With the seeded tie-break the sorted variant first orders the gathered pairs by their tie-break
// values (TruncOutTie, 32-bit keys), then gives them their (mesh, cost key) keys in that order
// (trunc_rekey_kernel) for the stable sort that follows.
struct TruncOutTie {
    TieBreak tb;
    u64* tkey;
    u32* tval;
    __device__ void operator()(int e, int pos) const {
        tkey[pos] = (u64)tb.enc((u32)e);
        tval[pos] = (u32)e;
    }
};

__global__ __launch_bounds__(BLOCK) void trunc_rekey_kernel(const u32* __restrict__ tval, const State* st,
                                                            const u64* __restrict__ ekey,
                                                            const u32* __restrict__ ecost, MeshTab mt, int vbits,
                                                            u64* __restrict__ tkey) {
    const int i = blockIdx.x * BLOCK + threadIdx.x;
    if (i >= st->trunc_n) return;
    const u32 e = tval[i];
    tkey[i] = ((u64)(u32)mesh_of(mt.voff, mt.B, (int)(ekey[e] >> vbits)) << 32) | (u64)ecost[e];
}

// Budget for meshes with a moderate number of pairs: no sort.  The gathered pairs of a mesh are a
// contiguous run in edge order; one workgroup per mesh reads the run's cost keys once, into
// registers (item r * TRUNC_THREADS + t sits in register r of thread t), finds the cost key of the
// nrem-th smallest (cost key, edge) by a bitwise search on "how many keys are <= x" (a compare
// and an add per key and bit), and flags every pair above that key and, among the pairs with
// exactly that key, all but the first ones in edge order.  A wide kernel then releases the
// flagged pairs.  One compute unit does the whole search, so runs longer than TRUNC_BLOCK_CAP go
// to the sort instead.
constexpr int TRUNC_THREADS = 1024;
constexpr int TRUNC_REGS_MAX = 32;
constexpr int TRUNC_BLOCK_CAP = TRUNC_THREADS * TRUNC_REGS_MAX;

// Sum over the 64 lanes of a wave (all active), the same value returned to every lane.
__device__ __forceinline__ u32 wave_sum_u32(u32 x) {
    int v = (int)x;
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);  // row_half_mirror
    v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);  // row_mirror: each row of 16 holds its sum
    return (u32)(__builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
                 __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48));
}

template <int R, bool SHUFFLE>
__global__ __launch_bounds__(TRUNC_THREADS) void trunc_block_kernel(u32* __restrict__ tcost,
                                                                    const u32* __restrict__ tval, TieBreak tb,
                                                                    const int* __restrict__ matched,
                                                                    const int* __restrict__ nrem) {
    constexpr int NW = TRUNC_THREADS / 64;
    __shared__ u32 wsum[NW];
    __shared__ u32 wsum2[2][NW];
    __shared__ u32 cnt[R * NW];
    const int b = blockIdx.x;
    const int n = matched[b], keep = nrem[b];
    if (n <= keep) return;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const u64 lt = prim::lanemask_lt();

    u32 before = 0, s0;  // pairs gathered for meshes in front of this one
    for (int j = tid; j < b; j += TRUNC_THREADS)
        if (matched[j] > nrem[j]) before += (u32)matched[j];
    prim::wide_block_exclusive_scan<NW>(before, wsum, s0);
    tcost += s0;
    tval += s0;
    if (n > R * TRUNC_THREADS) {  // not for this kernel (the host does not launch it so): release nothing
        for (int i = tid; i < n; i += TRUNC_THREADS) tcost[i] = 0u;
        return;
    }

    u32 key[R];  // empty slots hold the largest key
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i = r * TRUNC_THREADS + tid;
        key[r] = i < n ? tcost[i] : 0xFFFFFFFFu;
    }

    // Number of the run's keys <= x, known to every thread after one barrier (`slot` alternates so
    // that the next count does not overwrite sums that are still being read).
    auto count_le = [&](u32 x, int slot) -> u32 {
        u32 c = 0;
#pragma unroll
        for (int r = 0; r < R; ++r) c += (key[r] <= x) ? 1u : 0u;
        c = wave_sum_u32(c);
        if (lane == 0) wsum2[slot][w] = c;
        __syncthreads();
        u32 tot = 0;
#pragma unroll
        for (int j = 0; j < NW; ++j) tot += wsum2[slot][j];
        return tot < (u32)n ? tot : (u32)n;  // (empty slots count when x is the largest key)
    };

    // prefix = smallest key x with at least `keep` keys <= x, found bit by bit from the top
    u32 prefix = 0, kk = 0;
    if (keep > 0) {
        for (int bit = 31; bit >= 0; --bit)
            if (count_le(prefix | ((1u << bit) - 1u), bit & 1) < (u32)keep) prefix |= 1u << bit;
        __syncthreads();
        kk = (u32)keep - (prefix ? count_le(prefix - 1u, 0) : 0u);
    }
    // kk = how many pairs with exactly the key `prefix` stay (the first kk in edge order)
    if constexpr (SHUFFLE) {
        // ... the first kk in the order of the seeded tie-break, which is distinct from pair to pair:
        // the same search once more, on the tie-break values of the pairs with that key
        u32 tie[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int i = r * TRUNC_THREADS + tid;
            tie[r] = (i < n && key[r] == prefix) ? tb.enc(tval[i]) : 0xFFFFFFFFu;
        }
        auto count_tie_le = [&](u32 x, int slot) -> u32 {
            u32 c = 0;
#pragma unroll
            for (int r = 0; r < R; ++r)
                c += (r * TRUNC_THREADS + tid < n && key[r] == prefix && tie[r] <= x) ? 1u : 0u;
            c = wave_sum_u32(c);
            __syncthreads();  // (the sums of the count before this one have been read)
            if (lane == 0) wsum2[slot][w] = c;
            __syncthreads();
            u32 tot = 0;
#pragma unroll
            for (int j = 0; j < NW; ++j) tot += wsum2[slot][j];
            return tot;
        };
        u32 t2 = 0;
        if (kk > 0)
            for (int bit = 31; bit >= 0; --bit)
                if (count_tie_le(t2 | ((1u << bit) - 1u), bit & 1) < kk) t2 |= 1u << bit;
        __syncthreads();
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int i = r * TRUNC_THREADS + tid;
            if (i < n) tcost[i] = (key[r] > prefix || (key[r] == prefix && (kk == 0 || tie[r] > t2))) ? 1u : 0u;
        }
        return;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const bool eq = (r * TRUNC_THREADS + tid < n) && key[r] == prefix;
        const u64 eb = __ballot(eq);
        if (lane == 0) cnt[r * NW + w] = (u32)__popcll(eb);
    }
    __syncthreads();
    {
        const u32 v = tid < R * NW ? cnt[tid] : 0u;
        u32 tot;
        const u32 ex = prim::wide_block_exclusive_scan<NW>(v, wsum, tot);
        if (tid < R * NW) cnt[tid] = ex;  // equal keys in front of wave w's part of row r
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i = r * TRUNC_THREADS + tid;
        const bool valid = i < n;
        const bool eq = valid && key[r] == prefix, gt = valid && key[r] > prefix;
        const u64 eb = __ballot(eq);
        const u32 rank = cnt[r * NW + w] + (u32)__popcll(eb & lt);
        if (valid) tcost[i] = (gt || (eq && rank >= kk)) ? 1u : 0u;  // the key's slot now holds the flag
    }
}

constexpr u64 ABID_NONE = ~0ull;

// The end of an edge that line 11 of Alg. 2 could add to the other end's cluster: the un-paired
// one when exactly one end is paired, else -1.
__device__ __forceinline__ int joining_end(const int* __restrict__ mate, int u, int v) {
    const bool pu = mate[u] >= 0, pv = mate[v] >= 0;
    return pu == pv ? -1 : (pu ? v : u);
}

// Gives up what the budget does not cover: a pair is dissolved (ABSORB = false), or the vertex
// that would have joined through the edge stays on its own (ABSORB = true: its bid is withdrawn).
template <bool ABSORB>
__device__ __forceinline__ void release_edge(u64 k, int vbits, int* __restrict__ mate, u64* __restrict__ abid) {
    const int u = (int)(k >> vbits), v = (int)(k & ((1ull << vbits) - 1ull));
    if (ABSORB) {
        const int w = joining_end(mate, u, v);
        if (w >= 0) abid[w] = ABID_NONE;
    } else {
        mate[u] = -1;
        mate[v] = -1;
    }
}

// Releases the flagged pairs; block 0 also clamps the pair counts of the meshes to their budgets.
template <bool ABSORB>
__global__ __launch_bounds__(BLOCK) void trunc_release_kernel(const u32* __restrict__ tflag,
                                                              const u32* __restrict__ tval, const State* st,
                                                              const u64* __restrict__ ekey, int vbits,
                                                              int* __restrict__ mate, int B, int* __restrict__ matched,
                                                              const int* __restrict__ nrem, u64* __restrict__ abid) {
    const int i = blockIdx.x * BLOCK + threadIdx.x;
    if (i < st->trunc_n && tflag[i]) release_edge<ABSORB>(ekey[tval[i]], vbits, mate, abid);
    if (blockIdx.x == 0)
        for (int b = threadIdx.x; b < B; b += BLOCK)
            if (matched[b] > nrem[b]) matched[b] = nrem[b];
}

// segstart[b] = number of gathered pairs that belong to meshes before b
__global__ void trunc_segments_kernel(int B, const int* __restrict__ matched, const int* __restrict__ nrem,
                                      int* __restrict__ segstart) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        int run = 0;
        for (int b = 0; b < B; ++b) {
            segstart[b] = run;
            if (matched[b] > nrem[b]) run += matched[b];
        }
    }
}

template <bool ABSORB>
__global__ __launch_bounds__(BLOCK) void trunc_apply_kernel(const u64* __restrict__ tkey, const u32* __restrict__ tval,
                                                            const State* st, const int* __restrict__ segstart,
                                                            const int* __restrict__ nrem,
                                                            const u64* __restrict__ ekey, int vbits,
                                                            int* __restrict__ mate, u64* __restrict__ abid) {
    const int i = blockIdx.x * BLOCK + threadIdx.x;
    if (i >= st->trunc_n) return;
    const int m = (int)(tkey[i] >> 32);
    if (i - segstart[m] >= nrem[m]) release_edge<ABSORB>(ekey[tval[i]], vbits, mate, abid);
}

__global__ void trunc_finish_kernel(int B, int* __restrict__ matched, const int* __restrict__ nrem) {
    for (int b = threadIdx.x; b < B; b += blockDim.x)
        if (matched[b] > nrem[b]) matched[b] = nrem[b];
}

// ---------------------------------------------------------------------------
// Alg. 2 line 11 (option), under the vertex budget: after the pairs are final,
// an un-paired vertex next to a paired one joins that pair's cluster through
// its cheapest such edge (cost key, edge index) -- the first the sequential
// walk over the sorted pairs would reach.  Every joining vertex has its own
// edge, so the priorities are distinct; where a mesh has more candidates than
// budget left, the cheapest stay (the same machinery as for the pairs).  Only
// the two founders of a cluster attract: a vertex that joined pulls in nobody.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void absorb_begin_kernel(u64* __restrict__ abid, int* __restrict__ arep,
                                                             int* __restrict__ acnt, const State* st, int cur, int B,
                                                             const int* __restrict__ nrem,
                                                             const int* __restrict__ matched, int* __restrict__ arem,
                                                             int* __restrict__ acand) {
    const int nv = st->nv[cur];
    const int stride = gridDim.x * BLOCK;
    const int g = blockIdx.x * BLOCK + threadIdx.x;
    for (int w = g; w < nv; w += stride) {
        abid[w] = ABID_NONE;
        arep[w] = -1;
        acnt[w] = 0;
    }
    for (int b = g; b < B; b += stride) {
        const int left = nrem[b] - matched[b];
        arem[b] = (matched[b] > 0 && left > 0) ? left : 0;  // budget left once the pairs are formed
        acand[b] = 0;
    }
}

__global__ __launch_bounds__(BLOCK) void absorb_bid_kernel(const u64* __restrict__ ekey, const u32* __restrict__ ecost,
                                                           const State* st, int vbits, const int* __restrict__ mate,
                                                           MeshTab mt, const int* __restrict__ arem,
                                                           u64* __restrict__ abid, TieBreak tb) {
    const int n = st->ne;
    for (int e = blockIdx.x * BLOCK + threadIdx.x; e < n; e += gridDim.x * BLOCK) {
        const u64 k = ekey[e];
        const int u = (int)(k >> vbits), v = (int)(k & ((1ull << vbits) - 1ull));
        const int w = joining_end(mate, u, v);
        if (w >= 0 && arem[mesh_of(mt.voff, mt.B, w)] > 0) atomicMin(&abid[w], tb.priority(ecost[e], e));
    }
}

// Edge e is the one through which its un-paired end joins (its bid stands at that vertex).
struct JoinPred {
    const u64* ekey;
    const u32* ecost;
    const int* mate;
    const u64* abid;
    int vbits;
    TieBreak tb;
    __device__ bool operator()(int e) const {
        const u64 k = ekey[e];
        const int w = joining_end(mate, (int)(k >> vbits), (int)(k & ((1ull << vbits) - 1ull)));
        return w >= 0 && abid[w] == tb.priority(ecost[e], e);
    }
};

struct JoinListOut {
    int* list;
    __device__ void operator()(int e, int pos) const { list[pos] = e; }
};

// ... and its mesh has more such edges than budget left.
struct JoinOverPred {
    JoinPred jp;
    MeshTab mt;
    const int* acand;
    const int* arem;
    __device__ bool operator()(int e) const {
        if (!jp(e)) return false;
        const int m = mesh_of(mt.voff, mt.B, (int)(jp.ekey[e] >> jp.vbits));
        return acand[m] > arem[m];
    }
};

// The joining edges are listed in edge order, hence by mesh: acand[b] = how many belong to mesh b.
// Also written to host memory (`host_out`), which the host reads after waiting for the stream.
__global__ __launch_bounds__(BLOCK) void absorb_count_kernel(const int* __restrict__ list, const State* st,
                                                             const u64* __restrict__ ekey, int vbits, int B,
                                                             const int* __restrict__ voff, int* __restrict__ acand,
                                                             int* __restrict__ host_out) {
    const int n = st->absorb_n;
    for (int b = threadIdx.x; b < B; b += BLOCK) {
        int pos[2];
        for (int side = 0; side < 2; ++side) {
            if (b + side == 0 || b + side == B) {  // the ends of the list need no search
                pos[side] = (b + side == 0) ? 0 : n;
                continue;
            }
            const int v0 = voff[b + side];
            int lo = 0, hi = n;  // first listed edge whose lower vertex is at or past v0
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if ((int)(ekey[list[mid]] >> vbits) >= v0) hi = mid; else lo = mid + 1;
            }
            pos[side] = lo;
        }
        acand[b] = pos[1] - pos[0];
        host_out[b] = pos[1] - pos[0];
    }
}

// For every listed edge that still stands: the joining vertex records its cluster's representative
// (the founding pair's smaller index) and emits the key (representative, vertex); withdrawn ones
// emit the all-ones key, which sorts behind every real one.
__global__ __launch_bounds__(BLOCK) void absorb_keys_kernel(const int* __restrict__ list, const State* st,
                                                            const u64* __restrict__ ekey,
                                                            const u32* __restrict__ ecost, int vbits,
                                                            const int* __restrict__ mate, const u64* __restrict__ abid,
                                                            int* __restrict__ arep, int* __restrict__ acnt,
                                                            u64* __restrict__ akey, TieBreak tb) {
    const int i = blockIdx.x * BLOCK + threadIdx.x;
    if (i >= st->absorb_n) return;
    const int e = list[i];
    const u64 k = ekey[e];
    const int u = (int)(k >> vbits), v = (int)(k & ((1ull << vbits) - 1ull));
    const int w = joining_end(mate, u, v);
    u64 out = (vbits >= 32) ? ~0ull : ((1ull << (2 * vbits)) - 1ull);
    if (w >= 0 && abid[w] == tb.priority(ecost[e], e)) {
        const int o = (w == u) ? v : u;
        const int mo = mate[o];
        const int r = o < mo ? o : mo;
        arep[w] = r;
        atomicAdd(&acnt[r], 1);  // (so that representatives nobody joined need not look)
        out = ((u64)(u32)r << vbits) | (u64)(u32)w;
    }
    akey[i] = out;
}

// ---------------------------------------------------------------------------
// S4 + S6: contraction (Alg. 2 lines 12-16) and survivor renumbering
// ---------------------------------------------------------------------------
template <bool ABSORB>
struct AlivePredT {
    const int* mate;
    const int* arep;
    __device__ bool operator()(int w) const {
        const int m = mate[w];
        if (m >= 0 && m < w) return false;  // the larger index of a pair is replaced by the smaller
        return !(ABSORB && arep[w] >= 0);   // as is a vertex that joined a pair's cluster
    }
};

struct AliveOut {
    int* newid;
    __device__ void operator()(int w, int pos) const { newid[w] = pos; }
};

// Survivors move to their new slot; a pair's representative takes the summed
// quadric and the pair's target position (the mean; with PLACE_INVERSE the
// point of least error where there is one).  With ABSORB a cluster may have
// more members than its pair: `akey` lists (representative, member) in
// ascending order for the vertices that joined, and quadric and position are
// summed over all members in ascending index order, the position sum divided
// by their number.  vmap[w] = output slot of w's cluster.
template <int PLACE, bool ABSORB>
__global__ __launch_bounds__(BLOCK) void contract_kernel(const VRec* __restrict__ vin, VRec* __restrict__ vout,
                                                         const int* __restrict__ mate, const int* __restrict__ newid,
                                                         int* __restrict__ vmap, const State* st, int cur, int B,
                                                         const int* __restrict__ voff_cur, int* __restrict__ voff_nxt,
                                                         int* __restrict__ htab, int hsize,
                                                         u32* __restrict__ msd_hist, float rcond_min,
                                                         const int* __restrict__ arep, const int* __restrict__ acnt,
                                                         const u64* __restrict__ akey, int vbits) {
    const int nv = st->nv[cur];
    const int stride = gridDim.x * BLOCK;
    const int g = blockIdx.x * BLOCK + threadIdx.x;
    // this round's edge keys are long sorted: their digit counts and cursors go back to zero for the next round
    for (int i = g; i < 2 * prim::MSD_HIST_WORDS; i += stride) msd_hist[i] = 0;
    for (int w = g; w < nv; w += stride) {
        const int m = mate[w];
        if (m >= 0 && m < w) {
            vmap[w] = newid[m];
            continue;
        }
        if (ABSORB) {
            const int r = arep[w];
            if (r >= 0) {
                vmap[w] = newid[r];
                continue;
            }
        }
        const int nw = newid[w];
        vmap[w] = nw;
        const float4* a = reinterpret_cast<const float4*>(&vin[w]);
        float4 r0 = a[0], r1 = a[1], r2 = a[2], r3 = a[3];
        if (m >= 0) {
            int j = 0, jend = 0;  // this cluster's part of akey
            if (ABSORB && acnt[w] > 0) {
                const int n = st->absorb_n;
                const u64 first = (u64)(u32)w << vbits;
                int lo = 0, hi = n;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (akey[mid] >= first) hi = mid; else lo = mid + 1;
                }
                j = lo;
                jend = min(lo + acnt[w], n);
            }
            if (!ABSORB || j == jend) {
                const float4* b = reinterpret_cast<const float4*>(&vin[m]);
                const float4 s0 = b[0], s1 = b[1], s2 = b[2], s3 = b[3];
                r0.x = (r0.x + s0.x) * 0.5f; r0.y = (r0.y + s0.y) * 0.5f; r0.z = (r0.z + s0.z) * 0.5f;
                r1.x = r1.x + s1.x; r1.y = r1.y + s1.y; r1.z = r1.z + s1.z; r1.w = r1.w + s1.w;
                r2.x = r2.x + s2.x; r2.y = r2.y + s2.y; r2.z = r2.z + s2.z; r2.w = r2.w + s2.w;
                r3.x = r3.x + s3.x; r3.y = r3.y + s3.y;
            } else {
                // merge w < m with the ascending list of joined vertices
                const u64 low = (1ull << vbits) - 1ull;
                bool done_w = false, done_m = false;
                int cnt = 0;
                while (!done_w || !done_m || j < jend) {
                    int x = 0x7FFFFFFF, from = -1;
                    if (!done_w) { x = w; from = 0; }
                    else if (!done_m) { x = m; from = 1; }
                    if (j < jend) {
                        const int y = (int)(akey[j] & low);
                        if (y < x) { x = y; from = 2; }
                    }
                    if (from == 0) done_w = true;
                    else if (from == 1) done_m = true;
                    else ++j;
                    const float4* b = reinterpret_cast<const float4*>(&vin[x]);
                    const float4 s0 = b[0], s1 = b[1], s2 = b[2], s3 = b[3];
                    if (cnt == 0) {
                        r0 = s0; r1 = s1; r2 = s2; r3 = s3;
                    } else {
                        r0.x = r0.x + s0.x; r0.y = r0.y + s0.y; r0.z = r0.z + s0.z;
                        r1.x = r1.x + s1.x; r1.y = r1.y + s1.y; r1.z = r1.z + s1.z; r1.w = r1.w + s1.w;
                        r2.x = r2.x + s2.x; r2.y = r2.y + s2.y; r2.z = r2.z + s2.z; r2.w = r2.w + s2.w;
                        r3.x = r3.x + s3.x; r3.y = r3.y + s3.y;
                    }
                    ++cnt;
                }
                const float k = (float)cnt;
                r0.x = r0.x / k; r0.y = r0.y / k; r0.z = r0.z / k;
                r0.w = 0.f; r3.z = 0.f; r3.w = 0.f;
            }
            if (PLACE == PLACE_INVERSE)
                quadric_minimiser(r1.x, r1.y, r1.z, r1.w, r2.x, r2.y, r2.z, r2.w, r3.x, rcond_min, r0.x, r0.y, r0.z);
        }
        float4* o = reinterpret_cast<float4*>(&vout[nw]);
        o[0] = r0; o[1] = r1; o[2] = r2; o[3] = r3;
    }
    // a mesh's first vertex always survives when only pairs are contracted (a removed vertex has a
    // smaller partner in its own mesh); one that joined a cluster may not, and then the mesh starts
    // at its first survivor (every cluster has one)
    for (int b = g; b <= B; b += stride) {
        int nb = st->nv[cur ^ 1];
        if (b < B) {
            int w = voff_cur[b];
            if (ABSORB)
                while (w + 1 < voff_cur[b + 1] && arep[w] >= 0) ++w;
            nb = newid[w];
        }
        voff_nxt[b] = nb;
    }
    for (int h = g; h < hsize; h += stride) htab[h] = -1;
}

// ---------------------------------------------------------------------------
// S5: facet re-indexing, removal of collapsed and repeated facets, compaction
// ---------------------------------------------------------------------------
__device__ __forceinline__ void sort3(int& a, int& b, int& c) {
    int t;
    if (a > b) { t = a; a = b; b = t; }
    if (b > c) { t = b; b = c; c = t; }
    if (a > b) { t = a; a = b; b = t; }
}

__device__ __forceinline__ u32 hash3(int a, int b, int c) {
    u32 h = (u32)a * 0x9E3779B1u;
    h ^= (u32)b * 0x85EBCA77u + (h << 6) + (h >> 2);
    h ^= (u32)c * 0xC2B2AE3Du + (h << 6) + (h >> 2);
    h ^= h >> 15;
    h *= 0x2C1B3C6Du;
    h ^= h >> 12;
    return h;
}

// Re-indexes every facet and enters the non-collapsed ones into an open-
// addressing table keyed by the unordered vertex triple.  A slot stores a
// facet index; the slot's identity is that facet's triple, and among equal
// triples the slot converges to the smallest facet index (atomicMin), so the
// survivor does not depend on the order in which lanes arrive.
constexpr int FSLOT_KEEP = -1, FSLOT_DROP = -2;

__global__ __launch_bounds__(BLOCK) void facet_insert_kernel(const int* __restrict__ fcur, int* __restrict__ fmap,
                                                             const int* __restrict__ vmap, const State* st, int cur,
                                                             int* __restrict__ htab, u32 hmask, MeshTab mt,
                                                             const int* __restrict__ voff_cur,
                                                             int* __restrict__ cid, int n_orig,
                                                             int* __restrict__ fslot) {
    const int nf = st->nf[cur];
    const int stride = gridDim.x * BLOCK;
    const int g = blockIdx.x * BLOCK + threadIdx.x;
    for (int f = g; f < nf; f += stride) {
        const int a0 = fcur[3 * (size_t)f], b0 = fcur[3 * (size_t)f + 1], c0 = fcur[3 * (size_t)f + 2];
        const int a = vmap[a0], b = vmap[b0], c = vmap[c0];
        fmap[3 * (size_t)f] = a;
        fmap[3 * (size_t)f + 1] = b;
        fmap[3 * (size_t)f + 2] = c;
        // fslot[f]: the table slot that decides about the facet (it survives iff the slot ends up
        // holding f), or FSLOT_KEEP / FSLOT_DROP where no slot is involved
        if (!mt.active[mesh_of(voff_cur, mt.B, a0)]) {  // mesh sits this round out: facets kept as they are
            fslot[f] = FSLOT_KEEP;
            continue;
        }
        if (a == b || b == c || a == c) {
            fslot[f] = FSLOT_DROP;
            continue;
        }
        int x = a, y = b, z = c;
        sort3(x, y, z);
        u32 h = hash3(x, y, z) & hmask;
        for (;;) {
            const int old = atomicCAS(&htab[h], -1, f);
            if (old == -1) break;
            if (old == f) break;
            int p = vmap[fcur[3 * (size_t)old]], q = vmap[fcur[3 * (size_t)old + 1]], r = vmap[fcur[3 * (size_t)old + 2]];
            sort3(p, q, r);
            if (p == x && q == y && r == z) {
                atomicMin(&htab[h], f);
                break;
            }
            h = (h + 1) & hmask;
        }
        fslot[f] = (int)h;
    }
    for (int o = g; o < n_orig; o += stride) cid[o] = vmap[cid[o]];
}

// keep[f] = 1 iff the facet survives: not collapsed and the first of its triple (the slot that
// facet_insert_kernel left for it holds the smallest facet index of the triple).
struct FacetKeepPred {
    const int* fslot;
    const int* htab;
    unsigned char* keep;
    __device__ bool operator()(int f) const {
        const int h = fslot[f];
        const bool k = h >= 0 ? htab[h] == f : h == FSLOT_KEEP;
        keep[f] = k ? 1 : 0;
        return k;
    }
};

struct FlagPred {
    const unsigned char* keep;
    __device__ bool operator()(int f) const { return keep[f] != 0; }
};

struct FacetOut {
    const int* fmap;
    int* fnxt;
    __device__ void operator()(int f, int pos) const {
        fnxt[3 * (size_t)pos] = fmap[3 * (size_t)f];
        fnxt[3 * (size_t)pos + 1] = fmap[3 * (size_t)f + 1];
        fnxt[3 * (size_t)pos + 2] = fmap[3 * (size_t)f + 2];
    }
};

// ---------------------------------------------------------------------------
// Results
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void copy_out_kernel(const VRec* __restrict__ vrec, const int* __restrict__ fcur,
                                                         const int* __restrict__ cid, const State* st, int cur,
                                                         int n_orig, float* __restrict__ verts_out,
                                                         int* __restrict__ facets_out, int* __restrict__ cid_out,
                                                         int B, const int* __restrict__ voff,
                                                         int* __restrict__ foff_out) {
    const int nv = st->nv[cur], nf = st->nf[cur];
    const int stride = gridDim.x * BLOCK;
    const int g = blockIdx.x * BLOCK + threadIdx.x;
    for (int w = g; w < nv; w += stride) {
        const float4 p = *reinterpret_cast<const float4*>(&vrec[w]);
        verts_out[3 * (size_t)w] = p.x;
        verts_out[3 * (size_t)w + 1] = p.y;
        verts_out[3 * (size_t)w + 2] = p.z;
    }
    for (long long i = g; i < 3ll * nf; i += stride) facets_out[i] = fcur[i];
    for (int o = g; o < n_orig; o += stride) cid_out[o] = cid[o];
    // facets stay grouped by mesh: first facet whose leading vertex is at or past the mesh's first vertex
    for (int b = g; b <= B; b += stride) {
        int lo = 0, hi = nf;
        if (b == B) lo = nf;
        else {
            const int v0 = voff[b];
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (fcur[3 * (size_t)mid] >= v0) hi = mid; else lo = mid + 1;
            }
        }
        foff_out[b] = lo;
    }
}

// Plain streaming copy, 16 bytes per lane per step: the yardstick for the
// achievable HBM rate and for calibrating the profiler's byte counters.
__global__ __launch_bounds__(BLOCK) void copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                     size_t n16) {
    const size_t stride = (size_t)gridDim.x * BLOCK;
    for (size_t i = (size_t)blockIdx.x * BLOCK + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(BLOCK) void export_quadrics_kernel(const VRec* __restrict__ vrec, int N,
                                                                float* __restrict__ out) {
    const int w = blockIdx.x * BLOCK + threadIdx.x;
    if (w >= N) return;
    const float4* r = reinterpret_cast<const float4*>(&vrec[w]);
    const float4 r1 = r[1], r2 = r[2], r3 = r[3];
    float* o = out + 10 * (size_t)w;
    o[0] = r1.x; o[1] = r1.y; o[2] = r1.z; o[3] = r1.w;
    o[4] = r2.x; o[5] = r2.y; o[6] = r2.z; o[7] = r2.w;
    o[8] = r3.x; o[9] = r3.y;
}

__global__ __launch_bounds__(BLOCK) void export_edges_kernel(const u64* __restrict__ ekey, const u32* __restrict__ ecost,
                                                             const State* st, int vbits, int* __restrict__ edges,
                                                             float* __restrict__ cost) {
    const int e = blockIdx.x * BLOCK + threadIdx.x;
    if (e >= st->ne) return;
    const u64 k = ekey[e];
    edges[2 * (size_t)e] = (int)(k >> vbits);
    edges[2 * (size_t)e + 1] = (int)(k & ((1ull << vbits) - 1ull));
    const u32 ck = ecost[e];
    cost[e] = __uint_as_float((ck & 0x80000000u) ? (ck & 0x7FFFFFFFu) : ~ck);
}

inline int ceil_log2(long long n) {
    int b = 0;
    while ((1ll << b) < n) ++b;
    return b < 1 ? 1 : b;
}

inline int grid_for(long long n, int cap = 0x7FFFFFFF) {
    long long g = (n + BLOCK - 1) / BLOCK;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

}  // namespace

// ---------------------------------------------------------------------------
// Context
// ---------------------------------------------------------------------------
struct picasso_ctx {
    int device = 0;
    int64_t max_verts = 0, max_facets = 0;
    int32_t max_meshes = 0;
    int64_t opt_max_rounds = -1;
    int64_t opt_stage_timing = 0;
    int64_t opt_subround_batch = 16;
    char hip_err[256] = {0};

    char* ws = nullptr;  // one device allocation, carved below
    size_t ws_bytes = 0;
    int* hdr = nullptr;  // State followed by the per-mesh tables (see carve)
    int cap_b = 1;       // per-mesh capacity the header was laid out for
    State* st = nullptr;
    VRec* vrec[2] = {nullptr, nullptr};
    int* fbuf[2] = {nullptr, nullptr};  // facet lists, ping-pong
    int* fmap = nullptr;                // re-indexed facets before compaction
    int* cid = nullptr;
    u64* key64[2] = {nullptr, nullptr};  // sort buffers (3F keys); also hold 32-bit keys for S0
    u32* val32[2] = {nullptr, nullptr};
    u64* ekey = nullptr;
    u32* ecost = nullptr;
    u64* vmin[3] = {nullptr, nullptr, nullptr};
    int* mate = nullptr;
    int* newid = nullptr;
    int* vmap = nullptr;
    int* csr_off = nullptr;
    int* list = nullptr;
    unsigned char* estate = nullptr;
    int* htab = nullptr;
    size_t hcap = 0;
    unsigned char* keep = nullptr;
    int* fslot = nullptr;  // per facet: the hash-table slot that decides about it
    int* tilesum = nullptr;
    prim::SortScratch sort_sc{};
    u32* hist12 = nullptr;  // the bucket sorts' top-digit counts, cursors and first positions (3 x prim::MSD_HIST_WORDS)
    // The vertex->facet sort has buffers and scratch of its own, so that in the first round it can
    // run beside the edge-key sort (neither depends on the other) on a second stream.
    u64* s0_key[2] = {nullptr, nullptr};  // incidence keys (vertex, facet) of S0 and their sort's second buffer
    prim::SortScratch sort_sc_s0{};
    u32* hist12_s0 = nullptr;
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    int64_t opt_overlap = 1;
    int64_t opt_trunc_block_max = TRUNC_BLOCK_CAP;
    // per-mesh tables
    int* voff[2] = {nullptr, nullptr};
    int* foff = nullptr;
    int* foff_out = nullptr;
    int* target = nullptr;
    int* active = nullptr;
    int* stuck = nullptr;
    int* nrem = nullptr;
    int* matched = nullptr;
    int* segstart = nullptr;
    int* mslots = nullptr;
    // pinned host staging
    // pinned host staging: read-back image of the header's front, then the upload image of the whole header
    int* h_pin = nullptr;
    int* h_pin_dev = nullptr;  // the same memory as the device addresses it
    size_t h_up_off = 0;
    size_t h_pin_ints = 0;
    hipEvent_t ev[2 * PICASSO_STATS_ROUNDS * PICASSO_ST_COUNT + 4];
    int n_ev = 0;
    hipEvent_t ev_total[2];
    // hipEvent brackets around the edge-key sort's main kernel (benchmark roofline)
    int64_t opt_kernel_timing = 0;  // N > 0: events around the kernel in every N-th decimate call
    int opt_placement = PLACE_MEAN;
    float opt_rcond_min = 1e-3f;
    int opt_absorb = 0;
    uint64_t opt_shuffle_seed = 0;  // != 0: pairs of equal cost in the order of the seeded tie-break
    u64* abid = nullptr;   // per vertex: cheapest edge through which it could join a pair's cluster
    int* arep = nullptr;   // per vertex: representative of the cluster it joined, or -1
    int* acnt = nullptr;   // per vertex: how many vertices joined the cluster it represents
    int* acand = nullptr;  // per mesh: vertices that could join
    int* arem = nullptr;   // per mesh: budget left after the pairs
    int64_t kt_calls = 0;           // decimate calls since the option was set
    bool kt_this_call = false;
    hipEvent_t kt_pool[512];
    prim::LaunchTimer::Rec kt_recs[256];
    prim::LaunchTimer kt;
    int64_t kt_launches = 0;
    double kt_ms = 0.0, kt_bytes = 0.0;
};

namespace {

constexpr int HDR_STATE_INTS = (int)(sizeof(State) / sizeof(int));

struct Carver {
    size_t off = 0;
    char* base = nullptr;
    template <typename T>
    T* take(size_t count) {
        size_t o = off;
        off = align_up(off + count * sizeof(T));
        return base ? reinterpret_cast<T*>(base + o) : nullptr;
    }
};

size_t next_pow2(size_t x) {
    size_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

// Lays the workspace out; with base == nullptr only measures it.
size_t carve(picasso_ctx* c, char* base, int64_t N, int64_t F, int32_t B) {
    Carver cv;
    cv.base = base;
    const size_t n = (size_t)std::max<int64_t>(N, 1), f = (size_t)std::max<int64_t>(F, 1), h = 3 * f;
    const size_t b = (size_t)std::max<int32_t>(B, 1);
    picasso_ctx dummy;
    picasso_ctx* x = c ? c : &dummy;
    // header: everything the host uploads or reads back, contiguous so that one copy moves it.
    //   [State][matched B][foff_out B+1] | [voff0 B+1][foff B+1][target B][stuck B][active B]
    //   <-------- read back ----------->
    int* hdr = cv.take<int>(HDR_STATE_INTS + 8 * b + 3);
    x->hdr = hdr;
    x->st = reinterpret_cast<State*>(hdr);
    if (hdr) {
        int* q = hdr + HDR_STATE_INTS;
        x->matched = q; q += b;
        x->foff_out = q; q += b + 1;
        x->voff[0] = q; q += b + 1;
        x->foff = q; q += b + 1;
        x->target = q; q += b;
        x->stuck = q; q += b;
        x->active = q; q += b;
    }
    x->vrec[0] = cv.take<VRec>(n);
    x->vrec[1] = cv.take<VRec>(n);
    x->fbuf[0] = cv.take<int>(3 * f);
    x->fbuf[1] = cv.take<int>(3 * f);
    x->fmap = cv.take<int>(3 * f);
    x->cid = cv.take<int>(n);
    x->key64[0] = cv.take<u64>(h);
    x->key64[1] = cv.take<u64>(h);
    x->val32[0] = cv.take<u32>(h);
    x->val32[1] = cv.take<u32>(h);
    x->ekey = cv.take<u64>(h);
    x->ecost = cv.take<u32>(h);
    for (int i = 0; i < 3; ++i) x->vmin[i] = cv.take<u64>(n);
    x->mate = cv.take<int>(n);
    x->newid = cv.take<int>(n);
    x->vmap = cv.take<int>(n);
    x->csr_off = cv.take<int>(n + 1);
    x->list = cv.take<int>(h);
    x->estate = cv.take<unsigned char>(h);
    x->hcap = next_pow2(2 * f);
    x->htab = cv.take<int>(x->hcap);
    x->keep = cv.take<unsigned char>(f);
    x->fslot = cv.take<int>(f);
    x->tilesum = cv.take<int>((size_t)prim::compact_tilesum_capacity((long long)std::max(h, n)));
    x->sort_sc.T = prim::sort_table_stride((long long)h);
    x->sort_sc.table = cv.take<u32>((size_t)256 * x->sort_sc.T);
    x->sort_sc.totals = cv.take<u32>(256);
    x->hist12 = cv.take<u32>(3 * prim::MSD_HIST_WORDS);
    for (int i = 0; i < 2; ++i) {
        x->s0_key[i] = cv.take<u64>(h);
    }
    x->sort_sc_s0.T = x->sort_sc.T;
    x->sort_sc_s0.table = cv.take<u32>((size_t)256 * x->sort_sc_s0.T);
    x->sort_sc_s0.totals = cv.take<u32>(256);
    x->hist12_s0 = cv.take<u32>(3 * prim::MSD_HIST_WORDS);
    x->voff[1] = cv.take<int>(b + 1);
    x->nrem = cv.take<int>(b);
    x->segstart = cv.take<int>(b);
    x->mslots = cv.take<int>(b * MATCH_SLOTS * MATCH_PAD);
    x->abid = cv.take<u64>(n);
    x->arep = cv.take<int>(n);
    x->acnt = cv.take<int>(n);
    x->acand = cv.take<int>(b);
    x->arem = cv.take<int>(b);
    return cv.off;
}

#define HIP_TRY(ctx, expr)                                                                          \
    do {                                                                                            \
        hipError_t e__ = (expr);                                                                    \
        if (e__ != hipSuccess) {                                                                    \
            snprintf((ctx)->hip_err, sizeof((ctx)->hip_err), "%s at %s:%d: %s", #expr, __FILE__, __LINE__, \
                     hipGetErrorString(e__));                                                       \
            return PICASSO_ERR_HIP;                                                                 \
        }                                                                                           \
    } while (0)

struct StageTimer {
    picasso_ctx* c;
    hipStream_t s;
    bool on;
    struct Rec { int round, stage, e0, e1; };
    std::vector<Rec> recs;
    int open = -1;
    void begin(int round, int stage) {
        if (!on || c->n_ev + 2 > (int)(sizeof(c->ev) / sizeof(c->ev[0]))) return;
        Rec r{round, stage, c->n_ev, c->n_ev + 1};
        c->n_ev += 2;
        (void)hipEventRecord(c->ev[r.e0], s);
        recs.push_back(r);
        open = (int)recs.size() - 1;
    }
    void end() {
        if (!on || open < 0) return;
        (void)hipEventRecord(c->ev[recs[open].e1], s);
        open = -1;
    }
    void collect(picasso_stats* stats) {
        if (!on || !stats) return;
        for (const Rec& r : recs) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, c->ev[r.e0], c->ev[r.e1]) == hipSuccess && r.round < PICASSO_STATS_ROUNDS)
                stats->ms_stage[r.round][r.stage] += ms;
        }
    }
};

// Sort for keys whose leading bits are vertex ids (evenly spread): bucket sort
// when the input is small enough for it, plain LSD passes otherwise.
// which sort sort_by_vertex takes, named by the counting a producer of the keys may do for it
inline int sort_by_vertex_path(long long n_max, int key_bits) {
    if (n_max <= 0) return COUNT_NONE;
    if (n_max <= prim::BUCKET_SORT_MAX_KEYS && key_bits > prim::BUCKET_MSD_BITS) return COUNT_SMALL;
    if (n_max <= prim::BUCKET_SORT_LARGE_MAX_KEYS && key_bits > prim::BUCKET_LARGE_MSD_BITS) return COUNT_LARGE;
    return COUNT_NONE;
}

template <typename K, bool HAS_VAL, int LARGE_KEYS_ONLY_ITEMS = 8, class Src = prim::ArrayKeys<K>>
int sort_by_vertex(hipStream_t s, K* k0, K* k1, u32* v0, u32* v1, const int* n_ptr, int n_max, int key_bits,
                   const prim::SortScratch& sc, u32* hist12, prim::LaunchTimer* lt = nullptr, int tag = 0,
                   bool counted = false, const Src* src = nullptr) {
    const int how = sort_by_vertex_path(n_max, key_bits);
    if (how == COUNT_SMALL)
        return prim::bucket_sort<K, HAS_VAL, Src>(s, k0, k1, v0, v1, n_ptr, n_max, key_bits, sc, lt, tag, counted,
                                                  hist12, src);
    if (how == COUNT_LARGE)
        return prim::bucket_sort_large<K, HAS_VAL, LARGE_KEYS_ONLY_ITEMS, Src>(s, k0, k1, v0, v1, n_ptr, n_max, key_bits,
                                                                               sc, hist12, lt, tag, counted, src);
    return prim::radix_sort<K, HAS_VAL>(s, k0, k1, v0, v1, n_ptr, n_max, key_bits, sc, lt, tag);
}

// Edge keys, their sort and the count half of the unique step (S1 up to where costs are needed)
// for the round that starts with `nvt` vertices and at most `nfb` facets, on stream `st_`.
// *skeys_out = the sorted keys.
int issue_edge_prefix(picasso_ctx* c, hipStream_t st_, int B, int round_, int cur_, int nvt, int nfb,
                      const u64** skeys_out) {
    const u64* skeys = nullptr;
    const int vbits_ = ceil_log2(nvt);
    const int H_ = 3 * nfb;
    const RoundTab rt{B, c->voff[cur_], c->target, c->active, c->stuck, c->nrem, c->matched, c->mslots, round_ == 0};
    // the kernel that writes the keys also counts their top digits for the sort they go to (the
    // histogram and the cursors were zeroed by init_kernel, or by the contraction of the round before)
    const int kb = 2 * vbits_;
    const int how = sort_by_vertex_path(H_, kb);
    const bool counted = how != COUNT_NONE;
    if (how == COUNT_SMALL)
        edge_keys_kernel<COUNT_SMALL><<<prim::sort_tiles(H_, prim::SORT_ITEMS_SMALL), BLOCK, 0, st_>>>(
            c->fbuf[cur_], c->st, cur_, vbits_, nullptr, c->vmin[0], c->vmin[1], c->mate, rt,
            prim::bucket_sort_low_bits(kb), c->hist12);
    else if (how == COUNT_LARGE)
        edge_keys_kernel<COUNT_LARGE><<<prim::sort_tiles(H_, prim::SORT_ITEMS_BIG), BLOCK, 0, st_>>>(
            c->fbuf[cur_], c->st, cur_, vbits_, nullptr, c->vmin[0], c->vmin[1], c->mate, rt,
            kb - prim::BUCKET_LARGE_MSD_BITS, c->hist12);
    else
        edge_keys_kernel<COUNT_NONE><<<grid_for(std::max(3 * nfb, nvt), 8192), BLOCK, 0, st_>>>(
            c->fbuf[cur_], c->st, cur_, vbits_, c->key64[0], c->vmin[0], c->vmin[1], c->mate, rt, 0, nullptr);
    skeys = c->key64[0];
    const u64 sentinel_ = (vbits_ >= 32) ? ~0ull : ((1ull << (2 * vbits_)) - 1ull);
    if (H_ > 0) {
        const EdgeKeys src{c->fbuf[cur_], vbits_, sentinel_};  // (the counted sorts read the keys from here)
        int where = sort_by_vertex<u64, false, 8, EdgeKeys>(st_, c->key64[0], c->key64[1], nullptr, nullptr, &c->st->nh,
                                                            H_, 2 * vbits_, c->sort_sc, c->hist12,
                                                            c->kt_this_call ? &c->kt : nullptr, round_, counted, &src);
        if (where < 0) return PICASSO_ERR_HIP;
        skeys = where ? c->key64[1] : c->key64[0];
    }
    UniquePred up_{skeys, sentinel_};
    prim::compact_count(st_, up_, &c->st->nh, H_, c->tilesum);
    *skeys_out = skeys;
    return PICASSO_OK;
}

constexpr int64_t OVERLAP_MIN_FACETS = 1 << 18;

// Bits of the incidence keys: vertex id above, facet id below.
inline int incidence_fbits(int F) { return ceil_log2(std::max(F, 1)); }
inline int incidence_key_bits(int N, int F) { return ceil_log2(N) + incidence_fbits(F); }

// The validating kernel, instantiated for the sort the incidence keys go to.
int launch_init(picasso_ctx* c, hipStream_t s, const float* d_verts, int N, const int32_t* d_facets, int F, int B,
                bool with_keys) {
    const int fbits = incidence_fbits(F), kb = incidence_key_bits(N, F);
    const int how = with_keys ? sort_by_vertex_path(3ll * F, kb) : COUNT_NONE;
    // only a sort that cannot make the keys itself (the plain LSD fallback) needs them written out
    u64* ikey = (with_keys && how == COUNT_NONE) ? c->s0_key[0] : nullptr;
    const int s0 = with_keys ? 1 : 0;
    const int grid = grid_for(std::max(N, F), 4096);
    if (how == COUNT_SMALL)
        init_kernel<COUNT_SMALL><<<grid, BLOCK, 0, s>>>(d_verts, N, d_facets, F, B, c->voff[0], c->foff, c->vrec[0],
                                                        c->cid, c->fbuf[0], ikey, fbits, prim::bucket_sort_low_bits(kb),
                                                        c->hist12_s0, c->st, c->hist12, s0);
    else if (how == COUNT_LARGE)
        init_kernel<COUNT_LARGE><<<grid, BLOCK, 0, s>>>(d_verts, N, d_facets, F, B, c->voff[0], c->foff, c->vrec[0],
                                                        c->cid, c->fbuf[0], ikey, fbits,
                                                        kb - prim::BUCKET_LARGE_MSD_BITS, c->hist12_s0, c->st, c->hist12,
                                                        s0);
    else
        init_kernel<COUNT_NONE><<<grid, BLOCK, 0, s>>>(d_verts, N, d_facets, F, B, c->voff[0], c->foff, c->vrec[0],
                                                       c->cid, c->fbuf[0], ikey, fbits, 0, nullptr, c->st, c->hist12,
                                                       s0);
    return hipGetLastError() == hipSuccess ? PICASSO_OK : PICASSO_ERR_HIP;
}

// S0 on the incidence keys written by init_kernel (whose digit counts are in hist12_s0).
int run_vertex_quadrics(picasso_ctx* c, hipStream_t s, const float* d_verts, int N, int F) {
    const int H = 3 * F;
    const int fbits = incidence_fbits(F), kb = incidence_key_bits(N, F);
    if (F > 0) {
        const bool counted = sort_by_vertex_path(H, kb) != COUNT_NONE;
        const IncidenceKeys src{c->fbuf[0], fbits};  // (the counted sorts read the keys from here)
        int where = sort_by_vertex<u64, false, 16, IncidenceKeys>(s, c->s0_key[0], c->s0_key[1], nullptr, nullptr,
                                                                  nullptr, H, kb, c->sort_sc_s0, c->hist12_s0, nullptr,
                                                                  0, counted, &src);
        if (where < 0) return PICASSO_ERR_HIP;
        const u64* skey = where ? c->s0_key[1] : c->s0_key[0];
        csr_offsets_kernel<u64><<<grid_for(H), BLOCK, 0, s>>>(skey, fbits, H, N, c->csr_off);
        quadric_reduce_kernel<<<grid_for(N), BLOCK, 0, s>>>(c->vrec[0], d_verts, N, c->fbuf[0], c->csr_off, skey, fbits,
                                                            c->hist12_s0);
    } else {
        quadric_reduce_kernel<<<grid_for(N), BLOCK, 0, s>>>(c->vrec[0], d_verts, N, c->fbuf[0], nullptr, nullptr, 0,
                                                            c->hist12_s0);
    }
    return PICASSO_OK;
}

// Fills the pinned image of the header (State + per-mesh tables) and sends it with one copy.
int upload_header(picasso_ctx* c, hipStream_t s, int B, const int32_t* nv_in, const int32_t* nf_in,
                  const int32_t* target, int64_t* N_out, int64_t* F_out) {
    const int cb = c->cap_b;
    int* img = c->h_pin + c->h_up_off;
    const int total = HDR_STATE_INTS + 8 * cb + 3;
    memset(img, 0, sizeof(int) * total);
    int* hv = img + (c->voff[0] - c->hdr);
    int* hf = img + (c->foff - c->hdr);
    int* ht = img + (c->target - c->hdr);
    int64_t nacc = 0, facc = 0;
    for (int b = 0; b < B; ++b) {
        if (nv_in[b] < 1 || nf_in[b] < 0 || target[b] < 1) return PICASSO_ERR_INVALID_ARG;
        hv[b] = (int)nacc;
        hf[b] = (int)facc;
        ht[b] = target[b];
        nacc += nv_in[b];
        facc += nf_in[b];
        if (nacc > c->max_verts || facc > c->max_facets) return PICASSO_ERR_WORKSPACE;
    }
    hv[B] = (int)nacc;
    hf[B] = (int)facc;
    State* h = reinterpret_cast<State*>(img);
    h->nv[0] = (int)nacc;
    h->nf[0] = (int)facc;
    *N_out = nacc;
    *F_out = facc;
    HIP_TRY(c, hipMemcpyAsync(c->hdr, img, sizeof(int) * total, hipMemcpyHostToDevice, s));
    return PICASSO_OK;
}

// One copy of [State][matched][foff_out] to the pinned read-back area, then waits for the stream.
int read_header(picasso_ctx* c, hipStream_t s) {
    const int n = HDR_STATE_INTS + 2 * c->cap_b + 1;
    HIP_TRY(c, hipMemcpyAsync(c->h_pin, c->hdr, sizeof(int) * n, hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    return PICASSO_OK;
}

int status_from_err_bits(int bits) {
    if (bits & 1) return PICASSO_ERR_BAD_INDEX;
    if (bits & 2) return PICASSO_ERR_NONFINITE;
    return PICASSO_OK;
}

// Budget step: among the edges `over` selects (the formed pairs, or the joining edges of line 11, of
// the meshes that have more of them than they may use: counts[b] > budgets[b]) each mesh keeps its
// budgets[b] first ones in ascending (cost key, tie-break) order; the others are released
// (release_edge<ABSORB>) and counts[] is clamped.  n_over = sum of those meshes' counts, seg_max
// their largest.
template <bool ABSORB, class Over>
int budget_step(picasso_ctx* c, hipStream_t s, Over over, int B, int ne, int vbits, const MeshTab& mt,
                const TieBreak& tb, long long n_over, int seg_max, int* counts, int* budgets) {
    if (seg_max <= c->opt_trunc_block_max) {
        u32* tcost = reinterpret_cast<u32*>(c->key64[0]);
        TruncOutSplit to{c->ecost, tcost, c->val32[0]};
        prim::compact(s, over, over, to, &c->st->ne, ne, c->tilesum, &c->st->trunc_n);
#define PICASSO_TRUNC_BLOCK(R)                                                                                       \
    do {                                                                                                             \
        if (tb.on) trunc_block_kernel<R, true><<<B, TRUNC_THREADS, 0, s>>>(tcost, c->val32[0], tb, counts, budgets);  \
        else trunc_block_kernel<R, false><<<B, TRUNC_THREADS, 0, s>>>(tcost, c->val32[0], tb, counts, budgets);       \
    } while (0)
        if (seg_max <= 4 * TRUNC_THREADS) PICASSO_TRUNC_BLOCK(4);
        else if (seg_max <= 8 * TRUNC_THREADS) PICASSO_TRUNC_BLOCK(8);
        else if (seg_max <= 16 * TRUNC_THREADS) PICASSO_TRUNC_BLOCK(16);
        else PICASSO_TRUNC_BLOCK(32);
#undef PICASSO_TRUNC_BLOCK
        trunc_release_kernel<ABSORB><<<grid_for(n_over), BLOCK, 0, s>>>(tcost, c->val32[0], c->st, c->ekey, vbits,
                                                                        c->mate, B, counts, budgets, c->abid);
        return PICASSO_OK;
    }
    u64* k0 = c->key64[0];
    u64* k1 = c->key64[1];
    u32* v0 = c->val32[0];
    u32* v1 = c->val32[1];
    if (tb.on) {
        TruncOutTie to{tb, k0, v0};
        prim::compact(s, over, over, to, &c->st->ne, ne, c->tilesum, &c->st->trunc_n);
        const int w0 = prim::radix_sort<u64, true>(s, k0, k1, v0, v1, &c->st->trunc_n, (int)n_over, 32, c->sort_sc);
        if (w0 < 0) return PICASSO_ERR_HIP;
        if (w0) { std::swap(k0, k1); std::swap(v0, v1); }
        trunc_rekey_kernel<<<grid_for(n_over), BLOCK, 0, s>>>(v0, c->st, c->ekey, c->ecost, mt, vbits, k0);
    } else {
        TruncOut to{c->ekey, c->ecost, k0, v0, mt, vbits};
        prim::compact(s, over, over, to, &c->st->ne, ne, c->tilesum, &c->st->trunc_n);
    }
    const int where = prim::radix_sort<u64, true>(s, k0, k1, v0, v1, &c->st->trunc_n, (int)n_over,
                                                  32 + (B > 1 ? ceil_log2(B) : 0), c->sort_sc);
    if (where < 0) return PICASSO_ERR_HIP;
    trunc_segments_kernel<<<1, 64, 0, s>>>(B, counts, budgets, c->segstart);
    trunc_apply_kernel<ABSORB><<<grid_for(n_over), BLOCK, 0, s>>>(where ? k1 : k0, where ? v1 : v0, c->st, c->segstart,
                                                                  budgets, c->ekey, vbits, c->mate, c->abid);
    trunc_finish_kernel<<<1, BLOCK, 0, s>>>(B, counts, budgets);
    return PICASSO_OK;
}

// Alg. 2 line 11 on the device for the round whose pairs are final (see the kernels).  nrem /
// h_matched: per-mesh budget and pairs kept (host mirrors); h_joined receives the vertices that
// join per mesh; *akeys the sorted (representative, vertex) keys, st->absorb_n of them.  Waits for
// the stream once (the per-mesh candidate counts decide whether the budget step is needed).
int run_absorb(picasso_ctx* c, hipStream_t s, int B, int cur, int vbits, int ne, int nv_total, const MeshTab& mt,
               const TieBreak& tb, const std::vector<int>& nrem, const std::vector<int>& h_matched, std::vector<int>& h_joined,
               const u64** akeys) {
    absorb_begin_kernel<<<grid_for(std::max(nv_total, B), 4096), BLOCK, 0, s>>>(c->abid, c->arep, c->acnt, c->st, cur, B, c->nrem,
                                                                              c->matched, c->arem, c->acand);
    absorb_bid_kernel<<<grid_for(std::max(ne, 1), 8192), BLOCK, 0, s>>>(c->ekey, c->ecost, c->st, vbits, c->mate, mt,
                                                                      c->arem, c->abid, tb);
    JoinPred jp{c->ekey, c->ecost, c->mate, c->abid, vbits, tb};
    JoinListOut jl{c->list};
    prim::compact(s, jp, jp, jl, &c->st->ne, ne, c->tilesum, &c->st->absorb_n);
    int* host_counts = c->h_pin_dev + HDR_STATE_INTS + c->cap_b;  // (the offsets' slots of the read-back area: free until the end)
    absorb_count_kernel<<<1, BLOCK, 0, s>>>(c->list, c->st, c->ekey, vbits, B, c->voff[cur], c->acand, host_counts);
    HIP_TRY(c, hipStreamSynchronize(s));
    const int* h_cand = c->h_pin + HDR_STATE_INTS + c->cap_b;
    long long n_list = 0, n_over = 0;
    int seg_max = 0;
    for (int b = 0; b < B; ++b) {
        const int left = (h_matched[b] > 0 && nrem[b] > h_matched[b]) ? nrem[b] - h_matched[b] : 0;
        const int cand = h_cand[b];
        n_list += cand;
        if (cand > left) {
            n_over += cand;
            seg_max = std::max(seg_max, cand);
        }
        h_joined[b] = std::min(cand, left);
    }
    if (n_list == 0) return PICASSO_OK;
    if (n_over > 0) {  // the cheapest `left` candidates of each such mesh stay
        JoinOverPred op{jp, mt, c->acand, c->arem};
        const int rc = budget_step<true>(c, s, op, B, ne, vbits, mt, tb, n_over, seg_max, c->acand, c->arem);
        if (rc != PICASSO_OK) return rc;
    }
    absorb_keys_kernel<<<grid_for(n_list), BLOCK, 0, s>>>(c->list, c->st, c->ekey, c->ecost, vbits, c->mate, c->abid,
                                                         c->arep, c->acnt, c->key64[0], tb);
    const int where = sort_by_vertex<u64, false>(s, c->key64[0], c->key64[1], nullptr, nullptr, &c->st->absorb_n,
                                                 (int)n_list, 2 * vbits, c->sort_sc, c->hist12);
    if (where < 0) return PICASSO_ERR_HIP;
    *akeys = where ? c->key64[1] : c->key64[0];
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int decimate_impl(picasso_ctx* c, hipStream_t s, int B, const float* d_verts, const int32_t* d_facets,
                  const int32_t* nv_in, const int32_t* nf_in, const int32_t* target_nv, float* d_verts_out,
                  int32_t* d_facets_out, int32_t* d_cluster_id, int32_t* h_nv_out, int32_t* h_nf_out,
                  picasso_stats* stats) {
    if (!c || !d_verts || !nv_in || !nf_in || !target_nv || !d_verts_out || !d_facets_out || !d_cluster_id ||
        !h_nv_out || !h_nf_out || B < 1)
        return PICASSO_ERR_INVALID_ARG;
    if (B > c->max_meshes) return PICASSO_ERR_WORKSPACE;
    HIP_TRY(c, hipSetDevice(c->device));
    if (stats) memset(stats, 0, sizeof(*stats));

    int64_t N64 = 0, F64 = 0;
    int rc = upload_header(c, s, B, nv_in, nf_in, target_nv, &N64, &F64);
    if (rc != PICASSO_OK) return rc;
    if (F64 > 0 && !d_facets) return PICASSO_ERR_INVALID_ARG;
    const int N = (int)N64, F = (int)F64;

    c->n_ev = 0;
    c->kt.pool = c->kt_pool;
    c->kt.cap = (int)(sizeof(c->kt_pool) / sizeof(c->kt_pool[0]));
    c->kt.recs = c->kt_recs;
    c->kt.used = 0;
    c->kt.nrec = 0;
    c->kt_this_call = c->opt_kernel_timing > 0 && (c->kt_calls++ % c->opt_kernel_timing) == 0;
    std::vector<int> nf_round;
    StageTimer tm{c, s, c->opt_stage_timing != 0 && stats != nullptr, {}, -1};
    if (stats) HIP_TRY(c, hipEventRecord(c->ev_total[0], s));  // (an event costs queue time: only when asked for)

    // host mirror of the per-mesh vertex counts
    std::vector<int> nvb(nv_in, nv_in + B), stuck(B, 0), act(B, 0), nrem(B, 0);
    auto any_active = [&]() {
        bool any = false;
        for (int b = 0; b < B; ++b) {
            act[b] = (nvb[b] > target_nv[b]) && !stuck[b];
            nrem[b] = act[b] ? nvb[b] - target_nv[b] : 0;
            any |= (act[b] != 0);
        }
        return any;
    };
    bool work = any_active() && c->opt_max_rounds != 0;

    // In the first round the vertex quadrics (S0) and the edge keys (S1) depend only on the validated
    // input, not on each other: S1's prefix goes to the context's side stream and joins before the
    // costs are computed.  (Serial when stage times are being recorded, to keep them attributable.)
    // The fork and join cost about as much as a few small kernels, so small inputs stay on one stream.
    const u64* skeys = nullptr;
    const bool overlap = work && c->opt_overlap && c->side && !tm.on && F >= OVERLAP_MIN_FACETS;
    tm.begin(0, PICASSO_ST_QUADRICS);
    rc = launch_init(c, s, d_verts, N, d_facets, F, B, work);
    if (rc != PICASSO_OK) return rc;
    if (overlap) {
        HIP_TRY(c, hipEventRecord(c->ev_fork, s));
        HIP_TRY(c, hipStreamWaitEvent(c->side, c->ev_fork, 0));
        rc = issue_edge_prefix(c, c->side, B, 0, 0, N, F, &skeys);
        if (rc != PICASSO_OK) return rc;
        HIP_TRY(c, hipEventRecord(c->ev_join, c->side));
    }
    if (work) {
        rc = run_vertex_quadrics(c, s, d_verts, N, F);
        if (rc != PICASSO_OK) return rc;
    }
    if (overlap) HIP_TRY(c, hipStreamWaitEvent(s, c->ev_join, 0));
    tm.end();

    State* hst = reinterpret_cast<State*>(c->h_pin);  // read-back area
    std::vector<int> h_matched(B, 0), h_joined(B, 0);
    const TieBreak tb{c->opt_shuffle_seed != 0 ? 1u : 0u, (u32)c->opt_shuffle_seed, (u32)(c->opt_shuffle_seed >> 32)};

    int cur = 0;        // ping-pong index of vrec / facets / voff / State counts
    int nv_total = N;   // exact (host mirror)
    int nf_bound = F;   // upper bound on the current facet count
    int round = 0;
    int ne_prev = 0, nv_prev = 0;  // edge and vertex counts of the round before
    bool validated = false;

    while (work && (c->opt_max_rounds < 0 || round < c->opt_max_rounds)) {
        const int vbits = ceil_log2(nv_total);
        const int H = 3 * nf_bound;
        MeshTab mt{B, c->voff[cur], c->target, c->active, c->nrem, c->matched, c->mslots};

        // ---- S1 (+S2): edges and costs
        tm.begin(round, PICASSO_ST_EDGES);
        if (!(round == 0 && overlap)) {
            rc = issue_edge_prefix(c, s, B, round, cur, nv_total, nf_bound, &skeys);
            if (rc != PICASSO_OK) return rc;
        }
        const u64 sentinel = (vbits >= 32) ? ~0ull : ((1ull << (2 * vbits)) - 1ull);
        UniquePred up{skeys, sentinel};
#define PICASSO_UNIQUE(PLACE, SHUFFLE, RCOND)                                                                       \
    do {                                                                                                             \
        UniqueOutT<PLACE, SHUFFLE> uo{skeys, c->ekey, c->ecost, c->vrec[cur], c->vmin[0], c->estate, vbits, mt,       \
                                      RCOND, tb};                                                                    \
        prim::compact_scatter(s, up, uo, &c->st->nh, H, c->tilesum, &c->st->ne);                                     \
    } while (0)
        if (c->opt_placement == PLACE_INVERSE) {
            if (tb.on) PICASSO_UNIQUE(PLACE_INVERSE, true, c->opt_rcond_min);
            else PICASSO_UNIQUE(PLACE_INVERSE, false, c->opt_rcond_min);
        } else {
            if (tb.on) PICASSO_UNIQUE(PLACE_MEAN, true, 0.0f);
            else PICASSO_UNIQUE(PLACE_MEAN, false, 0.0f);
        }
#undef PICASSO_UNIQUE
        tm.end();

        // ---- S3: selection sub-rounds
        tm.begin(round, PICASSO_ST_SELECT);
        SelArgs sa;
        sa.ekey = c->ekey;
        sa.ecost = c->ecost;
        for (int i = 0; i < 3; ++i) sa.vmin[i] = c->vmin[i];
        sa.mate = c->mate;
        sa.list = c->list;
        sa.estate = c->estate;
        sa.st = c->st;
        sa.mt = mt;
        sa.vbits = vbits;
        sa.host_img = c->h_pin_dev;
        sa.publish_ints = HDR_STATE_INTS + B;
        sa.tb = tb;
        int sel_k = 0;
        // Grid-wide sub-rounds while many edges are live (the live count falls about 3x per
        // sub-round), then the live edges are gathered and one workgroup finishes; the host
        // looks once per batch.
        int launched = 0;
        const int ne_bound = H;  // distinct edges <= half-edges
        // edges of this round: about half the half-edges at first, later the previous round's
        // count scaled by the drop in vertices (the facet bound lags one round behind)
        long long live_est = std::max(H / 2, 1);
        if (round > 0 && ne_prev > 0 && nv_prev > 0)
            live_est = std::max<long long>(1, std::min<long long>(H, (long long)ne_prev * nv_total / nv_prev * 21 / 20));
        for (;;) {
            // live edges fall by about 2.8x, 2.7x, 3.2x, 4x, 5x, ... per sub-round on meshes with varied costs
            static const int decay_x10[] = {28, 27, 32, 40, 50, 60};
            int wide = 0;
            for (long long l = live_est; l > TAIL_MAX; ++wide) l = l * 10 / decay_x10[std::min(wide, 5)];
            wide = std::min<int>(wide, (int)std::max<int64_t>(1, c->opt_subround_batch));
            for (int j = 0; j < wide; ++j) {
                const int g4 = (ne_bound + BLOCK * 4 - 1) / (BLOCK * 4), g16 = (ne_bound + BLOCK * 16 - 1) / (BLOCK * 16);
                if (sel_k + j == 1 && ne_bound >= SPARSE_MIN_EDGES) {
                    if (tb.on) select_subround_sparse_kernel<4, true><<<g4, BLOCK, 0, s>>>(sa, sel_k + j);
                    else select_subround_sparse_kernel<4, false><<<g4, BLOCK, 0, s>>>(sa, sel_k + j);
                } else if (sel_k + j > 1 && ne_bound >= SPARSE_MIN_EDGES) {
                    if (tb.on) select_subround_sparse_kernel<16, true><<<g16, BLOCK, 0, s>>>(sa, sel_k + j);
                    else select_subround_sparse_kernel<16, false><<<g16, BLOCK, 0, s>>>(sa, sel_k + j);
                } else {
                    if (tb.on) select_subround_kernel<true><<<grid_for(ne_bound, 1 << 16), BLOCK, 0, s>>>(sa, sel_k + j);
                    else select_subround_kernel<false><<<grid_for(ne_bound, 1 << 16), BLOCK, 0, s>>>(sa, sel_k + j);
                }
            }
            sel_k += wide;
            LivePred lp{c->estate};
            LiveOut lo{c->list};
            prim::compact(s, lp, lp, lo, &c->st->ne, ne_bound, c->tilesum, &c->st->live[0]);
            select_tail_kernel<<<1, TAIL_THREADS, 0, s>>>(sa);
            launched += wide + 3;
            HIP_TRY(c, hipStreamSynchronize(s));  // the tail has left [State][matched] in the read-back area
            if (!validated) {
                const int st_err = status_from_err_bits(hst->err);
                if (st_err != PICASSO_OK) return st_err;
                validated = true;
            }
            sel_k = hst->sel_k;
            const int live = hst->live[0];
            if (live == 0) break;
            live_est = live;
        }
        for (int b = 0; b < B; ++b) h_matched[b] = c->h_pin[HDR_STATE_INTS + b];
        nf_bound = std::min(nf_bound, hst->nf[cur]);
        nf_round.push_back(hst->nf[cur]);
        ne_prev = hst->ne;
        nv_prev = nv_total;
        if (stats && round < PICASSO_STATS_ROUNDS) {
            stats->nv[round] = nv_total;
            stats->nf[round] = hst->nf[cur];
            stats->ne[round] = hst->ne;
            stats->subrounds[round] = launched;
        }

        // ---- budget truncation (only where a mesh formed more pairs than it may remove)
        bool need_trunc = false;
        long long n_trunc = 0;
        int n_sel = 0, seg_max = 0;
        for (int b = 0; b < B; ++b) {
            if (h_matched[b] > nrem[b]) {
                need_trunc = true;
                n_trunc += h_matched[b];
                seg_max = std::max(seg_max, h_matched[b]);
                h_matched[b] = nrem[b];
            }
            n_sel += h_matched[b];
        }
        if (need_trunc) {
            TruncPred tp{c->ekey, c->mate, mt, vbits};
            rc = budget_step<false>(c, s, tp, B, hst->ne, vbits, mt, tb, n_trunc, seg_max, c->matched, c->nrem);
            if (rc != PICASSO_OK) return rc;
        }

        // ---- Alg. 2 line 11 (option): un-paired vertices join a neighbouring pair's cluster while budget is left
        int n_joined = 0;
        const u64* akeys = nullptr;
        std::fill(h_joined.begin(), h_joined.end(), 0);
        bool budget_left = false;
        for (int b = 0; b < B; ++b) budget_left |= (h_matched[b] > 0 && nrem[b] > h_matched[b]);
        if (c->opt_absorb && budget_left) {
            rc = run_absorb(c, s, B, cur, vbits, hst->ne, nv_total, mt, tb, nrem, h_matched, h_joined, &akeys);
            if (rc != PICASSO_OK) return rc;
            for (int b = 0; b < B; ++b) n_joined += h_joined[b];
        }
        tm.end();
        if (stats && round < PICASSO_STATS_ROUNDS) stats->nsel[round] = n_sel + n_joined;

        // host mirror of the outcome
        for (int b = 0; b < B; ++b) {
            if (act[b] && h_matched[b] == 0) stuck[b] = 1;
            nvb[b] -= h_matched[b] + h_joined[b];
        }
        if (n_sel == 0) {  // nothing contracted anywhere: the meshes are unchanged
            work = any_active();
            break;
        }

        // ---- S4 + S6: contraction and renumbering
        tm.begin(round, PICASSO_ST_CONTRACT);
        const int nxt = cur ^ 1;
        AliveOut ao{c->newid};
        if (n_joined > 0) {
            AlivePredT<true> ap{c->mate, c->arep};
            prim::compact(s, ap, ap, ao, nullptr, nv_total, c->tilesum, &c->st->nv[nxt]);
        } else {
            AlivePredT<false> ap{c->mate, nullptr};
            prim::compact(s, ap, ap, ao, nullptr, nv_total, c->tilesum, &c->st->nv[nxt]);
        }
        const size_t hsize = next_pow2((size_t)2 * std::max(nf_bound, 1));
        const int cgrid = grid_for(std::max<long long>(nv_total, (long long)hsize), 8192);
#define PICASSO_CONTRACT(PLACE, ABSORB, RCOND)                                                                       \
    contract_kernel<PLACE, ABSORB><<<cgrid, BLOCK, 0, s>>>(c->vrec[cur], c->vrec[nxt], c->mate, c->newid, c->vmap,    \
                                                           c->st, cur, B, c->voff[cur], c->voff[nxt], c->htab,        \
                                                           (int)hsize, c->hist12, RCOND, c->arep, c->acnt, akeys, vbits)
        if (c->opt_placement == PLACE_INVERSE) {
            if (n_joined > 0) PICASSO_CONTRACT(PLACE_INVERSE, true, c->opt_rcond_min);
            else PICASSO_CONTRACT(PLACE_INVERSE, false, c->opt_rcond_min);
        } else {
            if (n_joined > 0) PICASSO_CONTRACT(PLACE_MEAN, true, 0.0f);
            else PICASSO_CONTRACT(PLACE_MEAN, false, 0.0f);
        }
#undef PICASSO_CONTRACT
        tm.end();

        // ---- S5: facets
        tm.begin(round, PICASSO_ST_FACETS);
        facet_insert_kernel<<<grid_for(std::max(nf_bound, N), 8192), BLOCK, 0, s>>>(
            c->fbuf[cur], c->fmap, c->vmap, c->st, cur, c->htab, (u32)(hsize - 1), mt, c->voff[cur], c->cid, N,
            c->fslot);
        FacetKeepPred kp{c->fslot, c->htab, c->keep};
        FlagPred fp{c->keep};
        FacetOut fo{c->fmap, c->fbuf[nxt]};
        prim::compact(s, kp, fp, fo, &c->st->nf[cur], nf_bound, c->tilesum, &c->st->nf[nxt]);
        tm.end();

        nv_total -= n_sel + n_joined;
        cur = nxt;
        ++round;
        work = any_active();
    }

    if (!validated) {
        rc = read_header(c, s);
        if (rc != PICASSO_OK) return rc;
        const int st_err = status_from_err_bits(hst->err);
        if (st_err != PICASSO_OK) return st_err;
    }

    copy_out_kernel<<<grid_for(std::max(std::max(N, 3 * nf_bound), 1), 8192), BLOCK, 0, s>>>(
        c->vrec[cur], c->fbuf[cur], c->cid, c->st, cur, N, d_verts_out, d_facets_out, d_cluster_id, B, c->voff[cur],
        c->foff_out);
    if (stats) HIP_TRY(c, hipEventRecord(c->ev_total[1], s));
    rc = read_header(c, s);
    if (rc != PICASSO_OK) return rc;
    HIP_TRY(c, hipGetLastError());
    const int* h_foff = c->h_pin + HDR_STATE_INTS + c->cap_b;

    // edge-key sort, main kernel: one read and one write of every 8-byte key per launch
    for (int i = 0; i < c->kt.nrec; ++i) {
        const prim::LaunchTimer::Rec& r = c->kt.recs[i];
        float ms = 0.f;
        if (r.tag < (int)nf_round.size() && hipEventElapsedTime(&ms, c->kt_pool[r.e0], c->kt_pool[r.e1]) == hipSuccess) {
            c->kt_launches += 1;
            c->kt_ms += ms;
            c->kt_bytes += 16.0 * 3.0 * (double)nf_round[r.tag];
        }
    }

    int warn = PICASSO_OK;
    for (int b = 0; b < B; ++b) {
        h_nv_out[b] = nvb[b];
        h_nf_out[b] = h_foff[b + 1] - h_foff[b];
        if (nvb[b] > target_nv[b] && (c->opt_max_rounds < 0 || stuck[b])) warn = PICASSO_WARN_BUDGET_UNMET;
    }
    if (stats) {
        stats->rounds = round;
        stats->nv_out = hst->nv[cur];
        stats->nf_out = hst->nf[cur];
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->ev_total[0], c->ev_total[1]) == hipSuccess) stats->ms_total = ms;
        tm.collect(stats);
    }
    return warn;
}

// channels per lane for row-major [rows, C] features at these addresses
inline bool conv_vec4(int C, std::initializer_list<const void*> ptrs) {
    if (C % 4 != 0) return false;
    for (const void* p : ptrs)
        if ((uintptr_t)p % 16 != 0) return false;
    return true;
}

// 8 channels per lane where there are enough of them: indices, levels and fuzzy coefficients are then
// read half as often per channel
inline int conv_vec(int C, std::initializer_list<const void*> ptrs) {
    if (!conv_vec4(C, ptrs)) return 1;
    return (C % 8 == 0 && C >= 32) ? 8 : 4;
}

// Two-stage sum of ROWS x C filter-gradient rows over n_rows rows (conv::reduce_rows_stage1/2):
// partial sums in the context's sort buffer.
template <int ROWS, class Term>
int reduce_filter_rows(picasso_ctx* c, hipStream_t s, Term term, int n_rows, int C, bool vec4, int rows_used,
                       float* d_out) {
    const int Q = vec4 ? C / 4 : C;
    if (Q > pool::BLOCK) return PICASSO_ERR_INVALID_ARG;
    const size_t cap = (size_t)3 * (size_t)c->max_facets * sizeof(u64) / sizeof(float);  // floats in key64[0]
    const size_t per_group = (size_t)ROWS * C;
    if (per_group > cap) return PICASSO_ERR_WORKSPACE;
    const int R = pool::BLOCK / Q;
    long long groups = std::min<long long>(1024, ((long long)n_rows + 4ll * R - 1) / (4ll * R));
    groups = std::max<long long>(1, std::min<long long>(groups, (long long)(cap / per_group)));
    const int chunk = (int)(((long long)n_rows + groups - 1) / groups);
    float* partial = reinterpret_cast<float*>(c->key64[0]);
    const size_t lds = (size_t)pool::BLOCK * ROWS * (vec4 ? 4 : 1) * sizeof(float);
    if (vec4)
        conv::reduce_rows_stage1_kernel<ROWS, 4, Term><<<(int)groups, pool::BLOCK, lds, s>>>(term, n_rows, C, chunk, partial);
    else
        conv::reduce_rows_stage1_kernel<ROWS, 1, Term><<<(int)groups, pool::BLOCK, lds, s>>>(term, n_rows, C, chunk, partial);
    conv::reduce_rows_stage2_kernel<<<pool::grid_for((long long)rows_used * C * 64), pool::BLOCK, 0, s>>>(
        partial, (int)groups, ROWS, rows_used, C, d_out);
    return PICASSO_OK;
}

}  // namespace

// ---------------------------------------------------------------------------
// C-ABI
// ---------------------------------------------------------------------------
extern "C" {

size_t picasso_workspace_bytes(int64_t max_verts, int64_t max_facets, int32_t max_meshes) {
    return carve(nullptr, nullptr, max_verts, max_facets, max_meshes);
}

int picasso_create(picasso_ctx** out, int device, int64_t max_verts, int64_t max_facets, int32_t max_meshes) {
    if (!out || max_verts < 1 || max_facets < 0 || max_meshes < 1) return PICASSO_ERR_INVALID_ARG;
    // 32-bit indices throughout: half-edge slots (3 per facet) and the facet hash table
    // (next power of two above 2 * facets) must fit an int
    if (max_verts > 0x7FFFFFF0ll || max_facets > (1ll << 29)) return PICASSO_ERR_INVALID_ARG;
    picasso_ctx* c = new (std::nothrow) picasso_ctx();
    if (!c) return PICASSO_ERR_HIP;
    c->device = device;
    c->max_verts = max_verts;
    c->max_facets = max_facets;
    c->max_meshes = max_meshes;
    if (hipSetDevice(device) != hipSuccess) { delete c; return PICASSO_ERR_HIP; }
    c->ws_bytes = carve(nullptr, nullptr, max_verts, max_facets, max_meshes);
    if (hipMalloc((void**)&c->ws, c->ws_bytes) != hipSuccess) { delete c; return PICASSO_ERR_HIP; }
    carve(c, c->ws, max_verts, max_facets, max_meshes);
    c->cap_b = max_meshes;
    c->h_up_off = (size_t)HDR_STATE_INTS + 2 * (size_t)max_meshes + 16;
    c->h_pin_ints = c->h_up_off + HDR_STATE_INTS + 8 * (size_t)max_meshes + 16;
    if (hipHostMalloc((void**)&c->h_pin, c->h_pin_ints * sizeof(int), hipHostMallocDefault) != hipSuccess) {
        (void)hipFree(c->ws);
        delete c;
        return PICASSO_ERR_HIP;
    }
    memset(c->h_pin, 0, c->h_pin_ints * sizeof(int));
    // the incidence sort's digit counts start at zero; every S0 leaves them at zero again
    if (hipMemset(c->hist12_s0, 0, sizeof(u32) * 2 * prim::MSD_HIST_WORDS) != hipSuccess) {
        (void)hipHostFree(c->h_pin);
        (void)hipFree(c->ws);
        delete c;
        return PICASSO_ERR_HIP;
    }
    if (hipHostGetDevicePointer((void**)&c->h_pin_dev, c->h_pin, 0) != hipSuccess) {
        (void)hipHostFree(c->h_pin);
        (void)hipFree(c->ws);
        delete c;
        return PICASSO_ERR_HIP;
    }
    const int nev = (int)(sizeof(c->ev) / sizeof(c->ev[0]));
    for (int i = 0; i < nev; ++i) (void)hipEventCreate(&c->ev[i]);
    (void)hipEventCreate(&c->ev_total[0]);
    (void)hipEventCreate(&c->ev_total[1]);
    for (hipEvent_t& e : c->kt_pool) (void)hipEventCreate(&e);
    if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess) c->side = nullptr;
    (void)hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming);
    (void)hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming);
    *out = c;
    return PICASSO_OK;
}

void picasso_destroy(picasso_ctx* c) {
    if (!c) return;
    (void)hipSetDevice(c->device);
    (void)hipDeviceSynchronize();
    const int nev = (int)(sizeof(c->ev) / sizeof(c->ev[0]));
    for (int i = 0; i < nev; ++i) (void)hipEventDestroy(c->ev[i]);
    (void)hipEventDestroy(c->ev_total[0]);
    (void)hipEventDestroy(c->ev_total[1]);
    for (hipEvent_t& e : c->kt_pool) (void)hipEventDestroy(e);
    if (c->side) (void)hipStreamDestroy(c->side);
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    if (c->h_pin) (void)hipHostFree(c->h_pin);
    if (c->ws) (void)hipFree(c->ws);
    delete c;
}

int picasso_set_option(picasso_ctx* c, int option, int64_t value) {
    if (!c) return PICASSO_ERR_INVALID_ARG;
    switch (option) {
        case PICASSO_OPT_MAX_ROUNDS: c->opt_max_rounds = value; return PICASSO_OK;
        case PICASSO_OPT_STAGE_TIMING: c->opt_stage_timing = value; return PICASSO_OK;
        case PICASSO_OPT_KERNEL_TIMING:
            if (value < 0) return PICASSO_ERR_INVALID_ARG;
            c->opt_kernel_timing = value;
            c->kt_calls = 0;
            return PICASSO_OK;
        case PICASSO_OPT_OVERLAP: c->opt_overlap = value; return PICASSO_OK;
        case PICASSO_OPT_TRUNC_BLOCK_MAX:
            if (value < 0) return PICASSO_ERR_INVALID_ARG;
            c->opt_trunc_block_max = std::min<int64_t>(value, TRUNC_BLOCK_CAP);
            return PICASSO_OK;
        case PICASSO_OPT_SHUFFLE_SEED:
            c->opt_shuffle_seed = (uint64_t)value;
            return PICASSO_OK;
        case PICASSO_OPT_ABSORB:
            if (value != 0 && value != 1) return PICASSO_ERR_INVALID_ARG;
            c->opt_absorb = (int)value;
            return PICASSO_OK;
        case PICASSO_OPT_PLACEMENT:
            if (value != PLACE_MEAN && value != PLACE_INVERSE) return PICASSO_ERR_INVALID_ARG;
            c->opt_placement = (int)value;
            return PICASSO_OK;
        case PICASSO_OPT_RCOND_MIN_BITS: {
            if (value < 0 || value > 0xFFFFFFFFll) return PICASSO_ERR_INVALID_ARG;
            const u32 bits = (u32)value;
            float f;
            memcpy(&f, &bits, sizeof f);
            if (!(f >= 0.0f) || !std::isfinite(f)) return PICASSO_ERR_INVALID_ARG;
            c->opt_rcond_min = f;
            return PICASSO_OK;
        }
        case PICASSO_OPT_SUBROUND_BATCH:
            if (value < 1 || value > 1024) return PICASSO_ERR_INVALID_ARG;
            c->opt_subround_batch = value;
            return PICASSO_OK;
        default: return PICASSO_ERR_INVALID_ARG;
    }
}

const char* picasso_strerror(int status) {
    switch (status) {
        case PICASSO_OK: return "ok";
        case PICASSO_WARN_BUDGET_UNMET: return "warning: a mesh ran out of edges before reaching its vertex budget";
        case PICASSO_ERR_INVALID_ARG: return "invalid argument";
        case PICASSO_ERR_BAD_INDEX: return "facet index out of range";
        case PICASSO_ERR_NONFINITE: return "non-finite vertex coordinate";
        case PICASSO_ERR_WORKSPACE: return "input exceeds the capacity the context was created with";
        case PICASSO_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

const char* picasso_last_hip_error(picasso_ctx* c) { return c ? c->hip_err : ""; }

int picasso_kernel_timing(picasso_ctx* c, int reset, int64_t* launches, double* ms_total, double* bytes_total) {
    if (!c) return PICASSO_ERR_INVALID_ARG;
    if (launches) *launches = c->kt_launches;
    if (ms_total) *ms_total = c->kt_ms;
    if (bytes_total) *bytes_total = c->kt_bytes;
    if (reset) {
        c->kt_launches = 0;
        c->kt_ms = 0.0;
        c->kt_bytes = 0.0;
    }
    return PICASSO_OK;
}

int picasso_decimate_batch(picasso_ctx* c, void* stream, int32_t B, const float* d_verts, const int32_t* d_facets,
                           const int32_t* h_nv_in, const int32_t* h_nf_in, const int32_t* h_target_nv,
                           float* d_verts_out, int32_t* d_facets_out, int32_t* d_cluster_id, int32_t* h_nv_out,
                           int32_t* h_nf_out, picasso_stats* stats) {
    return decimate_impl(c, (hipStream_t)stream, B, d_verts, d_facets, h_nv_in, h_nf_in, h_target_nv, d_verts_out,
                         d_facets_out, d_cluster_id, h_nv_out, h_nf_out, stats);
}

int picasso_decimate(picasso_ctx* c, void* stream, const float* d_verts, int32_t N, const int32_t* d_facets,
                     int32_t F, int32_t target_nv, float* d_verts_out, int32_t* d_facets_out, int32_t* d_cluster_id,
                     int32_t* h_nv_out, int32_t* h_nf_out, picasso_stats* stats) {
    if (N < 1 || F < 0 || target_nv < 1) return PICASSO_ERR_INVALID_ARG;
    return decimate_impl(c, (hipStream_t)stream, 1, d_verts, d_facets, &N, &F, &target_nv, d_verts_out, d_facets_out,
                         d_cluster_id, h_nv_out, h_nf_out, stats);
}

int picasso_device_copy(void* stream, void* d_dst, const void* d_src, size_t nbytes) {
    if (!d_dst || !d_src || (nbytes & 15) || ((uintptr_t)d_dst & 15) || ((uintptr_t)d_src & 15))
        return PICASSO_ERR_INVALID_ARG;
    if (nbytes == 0) return PICASSO_OK;
    const size_t n16 = nbytes / 16;
    const int g = (int)std::min<size_t>((n16 + BLOCK - 1) / BLOCK, 256 * 32);
    copy_kernel<<<g, BLOCK, 0, (hipStream_t)stream>>>((const float4*)d_src, (float4*)d_dst, n16);
    return hipGetLastError() == hipSuccess ? PICASSO_OK : PICASSO_ERR_HIP;
}

int picasso_vertex_quadrics(picasso_ctx* c, void* stream, const float* d_verts, int32_t N, const int32_t* d_facets,
                            int32_t F, float* d_quadrics_out) {
    if (!c || !d_verts || N < 1 || F < 0 || (F > 0 && !d_facets) || !d_quadrics_out) return PICASSO_ERR_INVALID_ARG;
    if (N > c->max_verts || F > c->max_facets) return PICASSO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    int32_t big = 0x7FFFFFFF;
    int64_t n64, f64;
    int rc = upload_header(c, s, 1, &N, &F, &big, &n64, &f64);
    if (rc != PICASSO_OK) return rc;
    rc = launch_init(c, s, d_verts, N, d_facets, F, 1, true);
    if (rc != PICASSO_OK) return rc;
    State* hst = reinterpret_cast<State*>(c->h_pin);
    rc = read_header(c, s);
    if (rc != PICASSO_OK) return rc;
    rc = status_from_err_bits(hst->err);
    if (rc != PICASSO_OK) {  // S0 will not run: take back the digit counts the validating kernel has added
        prim::fill_u32_kernel<<<2 * prim::MSD_HIST_WORDS / BLOCK, BLOCK, 0, s>>>(c->hist12_s0, 2 * prim::MSD_HIST_WORDS, 0u);
        return rc;
    }
    rc = run_vertex_quadrics(c, s, d_verts, N, F);
    if (rc != PICASSO_OK) return rc;
    export_quadrics_kernel<<<grid_for(N), BLOCK, 0, s>>>(c->vrec[0], N, d_quadrics_out);
    HIP_TRY(c, hipStreamSynchronize(s));
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int picasso_edge_costs(picasso_ctx* c, void* stream, const float* d_verts, int32_t N, const int32_t* d_facets,
                       int32_t F, int32_t* d_edges_out, float* d_cost_out, int32_t* h_ne_out) {
    if (!c || !d_verts || N < 1 || F < 0 || (F > 0 && !d_facets) || !d_edges_out || !d_cost_out || !h_ne_out)
        return PICASSO_ERR_INVALID_ARG;
    if (N > c->max_verts || F > c->max_facets) return PICASSO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    int32_t one = 1;
    int64_t n64, f64;
    int rc = upload_header(c, s, 1, &N, &F, &one, &n64, &f64);
    if (rc != PICASSO_OK) return rc;
    rc = launch_init(c, s, d_verts, N, d_facets, F, 1, true);
    if (rc != PICASSO_OK) return rc;
    State* hst = reinterpret_cast<State*>(c->h_pin);
    rc = read_header(c, s);
    if (rc != PICASSO_OK) return rc;
    rc = status_from_err_bits(hst->err);
    if (rc != PICASSO_OK) {  // S0 will not run: take back the digit counts the validating kernel has added
        prim::fill_u32_kernel<<<2 * prim::MSD_HIST_WORDS / BLOCK, BLOCK, 0, s>>>(c->hist12_s0, 2 * prim::MSD_HIST_WORDS, 0u);
        return rc;
    }
    rc = run_vertex_quadrics(c, s, d_verts, N, F);
    if (rc != PICASSO_OK) return rc;
    const int vbits = ceil_log2(N), H = 3 * F;
    MeshTab mt{1, c->voff[0], c->target, c->active, c->nrem, c->matched, c->mslots};
    const u64* skeys = nullptr;
    rc = issue_edge_prefix(c, s, 1, 0, 0, N, F, &skeys);
    if (rc != PICASSO_OK) return rc;
    const u64 sentinel = (vbits >= 32) ? ~0ull : ((1ull << (2 * vbits)) - 1ull);
    UniquePred up{skeys, sentinel};
    if (c->opt_placement == PLACE_INVERSE) {
        UniqueOutT<PLACE_INVERSE, false> uo{skeys, c->ekey, c->ecost, c->vrec[0], c->vmin[0], c->estate, vbits, mt,
                                            c->opt_rcond_min, TieBreak{0u, 0u, 0u}};
        prim::compact_scatter(s, up, uo, &c->st->nh, H, c->tilesum, &c->st->ne);
    } else {
        UniqueOutT<PLACE_MEAN, false> uo{skeys, c->ekey, c->ecost, c->vrec[0], c->vmin[0], c->estate, vbits, mt, 0.0f,
                                         TieBreak{0u, 0u, 0u}};
        prim::compact_scatter(s, up, uo, &c->st->nh, H, c->tilesum, &c->st->ne);
    }
    export_edges_kernel<<<grid_for(std::max(H, 1)), BLOCK, 0, s>>>(c->ekey, c->ecost, c->st, vbits, d_edges_out,
                                                                   d_cost_out);
    rc = read_header(c, s);
    if (rc != PICASSO_OK) return rc;
    HIP_TRY(c, hipGetLastError());
    *h_ne_out = hst->ne;
    return PICASSO_OK;
}

// ---- pooling / unpooling over cluster_id (Sec. 3, "Pooling and unpooling")

int picasso_cluster_csr(picasso_ctx* c, void* stream, const int32_t* d_cluster_id, int32_t n_in, int32_t n_out,
                        int32_t* d_offsets, int32_t* d_members) {
    if (!c || !d_cluster_id || n_in < 1 || n_out < 1 || !d_offsets || !d_members) return PICASSO_ERR_INVALID_ARG;
    if (n_in > 3 * c->max_facets || n_out > c->max_verts) return PICASSO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    u32* k0 = reinterpret_cast<u32*>(c->key64[0]);
    u32* k1 = reinterpret_cast<u32*>(c->key64[1]);
    prim::fill_u32_kernel<<<1, BLOCK, 0, s>>>(reinterpret_cast<u32*>(&c->st->err), 1, 0u);
    pool::emit_cluster_pairs_kernel<<<pool::grid_for(n_in), pool::BLOCK, 0, s>>>(d_cluster_id, n_in, n_out, k0,
                                                                                 c->val32[0], &c->st->err);
    const int where = sort_by_vertex<u32, true>(s, k0, k1, c->val32[0], c->val32[1], nullptr, n_in, ceil_log2(n_out),
                                                c->sort_sc, c->hist12);
    if (where < 0) return PICASSO_ERR_HIP;
    csr_offsets_kernel<u32><<<grid_for(n_in), BLOCK, 0, s>>>(where ? k1 : k0, 0, n_in, n_out, d_offsets);
    HIP_TRY(c, hipMemcpyAsync(d_members, where ? c->val32[1] : c->val32[0], sizeof(int32_t) * (size_t)n_in,
                              hipMemcpyDeviceToDevice, s));
    int rc = read_header(c, s);
    if (rc != PICASSO_OK) return rc;
    HIP_TRY(c, hipGetLastError());
    return (reinterpret_cast<State*>(c->h_pin)->err & 1) ? PICASSO_ERR_BAD_INDEX : PICASSO_OK;
}

// ---- mesh convolutions, depth-wise (Sec. 4 "Mesh Convolution"; supplementary, backward propagations)

int picasso_vertex_corner_csr(picasso_ctx* c, void* stream, const int32_t* d_facets, int32_t F, int32_t N,
                              int32_t* d_offsets, int32_t* d_corners) {
    if (!c || !d_facets || F < 1 || N < 1 || !d_offsets || !d_corners) return PICASSO_ERR_INVALID_ARG;
    if (F > c->max_facets) return PICASSO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    const int H = 3 * F, cbits = ceil_log2(H), vbits = ceil_log2(N);
    prim::fill_u32_kernel<<<1, BLOCK, 0, s>>>(reinterpret_cast<u32*>(&c->st->err), 1, 0u);
    conv::corner_keys_kernel<<<pool::grid_for(H), pool::BLOCK, 0, s>>>(d_facets, H, N, cbits, c->key64[0], &c->st->err);
    const int where = sort_by_vertex<u64, false>(s, c->key64[0], c->key64[1], nullptr, nullptr, nullptr, H,
                                                 cbits + vbits, c->sort_sc, c->hist12);
    if (where < 0) return PICASSO_ERR_HIP;
    const u64* skey = where ? c->key64[1] : c->key64[0];
    csr_offsets_kernel<u64><<<grid_for(H), BLOCK, 0, s>>>(skey, cbits, H, N, d_offsets);
    conv::corner_list_kernel<<<pool::grid_for(H), pool::BLOCK, 0, s>>>(skey, H, cbits, d_corners);
    int rc = read_header(c, s);
    if (rc != PICASSO_OK) return rc;
    HIP_TRY(c, hipGetLastError());
    return (reinterpret_cast<State*>(c->h_pin)->err & 1) ? PICASSO_ERR_BAD_INDEX : PICASSO_OK;
}

int picasso_facet_geometry(picasso_ctx* c, void* stream, const float* d_verts, int32_t N, const int32_t* d_facets,
                           int32_t F, int32_t B, const int32_t* h_nf, int32_t alpha, int32_t beta, float* d_normals,
                           float* d_areas, int32_t* d_level) {
    if (!c || !d_verts || !d_facets || N < 1 || F < 1 || B < 1 || (B > 1 && !h_nf) || alpha < 0 || beta < 1 ||
        (!d_normals && !d_areas && !d_level))
        return PICASSO_ERR_INVALID_ARG;
    if (B > c->max_meshes || (d_level && !d_areas && F > 3 * c->max_facets)) return PICASSO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    // facet offsets of the meshes, staged in pinned memory like the decimation's header
    int* img = c->h_pin + c->h_up_off;
    long long acc = 0;
    for (int b = 0; b < B; ++b) {
        img[b] = (int)acc;
        const long long nb = (B > 1) ? h_nf[b] : F;
        if (nb < 0) return PICASSO_ERR_INVALID_ARG;
        acc += nb;
    }
    img[B] = (int)acc;
    if (acc != F) return PICASSO_ERR_INVALID_ARG;
    HIP_TRY(c, hipMemcpyAsync(c->foff, img, sizeof(int) * (B + 1), hipMemcpyHostToDevice, s));
    unsigned* amin = reinterpret_cast<unsigned*>(c->acand);
    unsigned* amax = reinterpret_cast<unsigned*>(c->arem);
    float* areas = d_areas ? d_areas : reinterpret_cast<float*>(c->ecost);  // scratch when only levels are wanted
    prim::fill_u32_kernel<<<1, BLOCK, 0, s>>>(reinterpret_cast<u32*>(&c->st->err), 1, 0u);
    if (d_level) {
        prim::fill_u32_kernel<<<grid_for(B), BLOCK, 0, s>>>(amin, B, 0xFFFFFFFFu);
        prim::fill_u32_kernel<<<grid_for(B), BLOCK, 0, s>>>(amax, B, 0u);
    }
    conv::facet_geometry_kernel<<<pool::grid_for(F), pool::BLOCK, 0, s>>>(
        d_verts, N, d_facets, F, B, c->foff, d_normals, (d_areas || d_level) ? areas : nullptr,
        d_level ? amin : nullptr, d_level ? amax : nullptr, &c->st->err);
    if (d_level)
        conv::facet_level_kernel<<<pool::grid_for(F), pool::BLOCK, 0, s>>>(areas, F, B, c->foff, amin, amax, alpha, beta,
                                                                          d_level);
    int rc = read_header(c, s);
    if (rc != PICASSO_OK) return rc;
    HIP_TRY(c, hipGetLastError());
    return (reinterpret_cast<State*>(c->h_pin)->err & 1) ? PICASSO_ERR_BAD_INDEX : PICASSO_OK;
}

int picasso_fuzzy_coefficients(picasso_ctx* c, void* stream, const float* d_normals, int32_t F, const float* d_mu,
                               const float* d_inv_var, int32_t T, float* d_pi) {
    if (!c || !d_normals || F < 1 || !d_mu || !d_inv_var || T < 1 || !d_pi) return PICASSO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    conv::fuzzy_kernel<<<pool::grid_for(F), pool::BLOCK, 0, s>>>(d_normals, F, d_mu, d_inv_var, T, d_pi);
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int picasso_v2f_forward(picasso_ctx* c, void* stream, const float* d_x, int32_t N, int32_t C, const int32_t* d_facets,
                        int32_t F, const int32_t* d_level, const float* d_w, float* d_y) {
    if (!c || !d_x || N < 1 || C < 1 || !d_facets || F < 1 || !d_w || !d_y) return PICASSO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    const int vec = conv_vec(C, {d_x, d_w, d_y});
    if (vec == 8)
        conv::v2f_forward_kernel<8><<<pool::grid_for((long long)F * (C / 8)), pool::BLOCK, 0, s>>>(d_x, N, C, d_facets, F, d_level, d_w, d_y);
    else if (vec == 4)
        conv::v2f_forward_kernel<4><<<pool::grid_for((long long)F * (C / 4)), pool::BLOCK, 0, s>>>(d_x, N, C, d_facets, F, d_level, d_w, d_y);
    else
        conv::v2f_forward_kernel<1><<<pool::grid_for((long long)F * C), pool::BLOCK, 0, s>>>(d_x, N, C, d_facets, F, d_level, d_w, d_y);
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int picasso_v2f_backward(picasso_ctx* c, void* stream, const float* d_gy, const float* d_x, int32_t N, int32_t C,
                         const int32_t* d_facets, int32_t F, const int32_t* d_level, const float* d_w,
                         const int32_t* d_offsets, const int32_t* d_corners, float* d_gx, float* d_gw) {
    if (!c || !d_gy || !d_x || N < 1 || C < 1 || !d_facets || F < 1 || !d_w || !d_offsets || !d_corners ||
        (!d_gx && !d_gw))
        return PICASSO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    const bool vec4 = conv_vec4(C, {d_gy, d_x, d_w, d_gx});
    if (d_gx) {
        if (conv_vec(C, {d_gy, d_w, d_gx}) == 8)
            conv::v2f_backward_x_kernel<8><<<pool::grid_for((long long)N * (C / 8)), pool::BLOCK, 0, s>>>(d_gy, C, d_level, d_w, d_offsets, d_corners, N, 3 * F, d_gx);
        else if (vec4)
            conv::v2f_backward_x_kernel<4><<<pool::grid_for((long long)N * (C / 4)), pool::BLOCK, 0, s>>>(d_gy, C, d_level, d_w, d_offsets, d_corners, N, 3 * F, d_gx);
        else
            conv::v2f_backward_x_kernel<1><<<pool::grid_for((long long)N * C), pool::BLOCK, 0, s>>>(d_gy, C, d_level, d_w, d_offsets, d_corners, N, 3 * F, d_gx);
    }
    if (d_gw) {
        conv::V2fWeightTerm term{d_gy, d_x, d_facets, d_level, C, N};
        const int rc = reduce_filter_rows<3>(c, s, term, F, C, vec4, 3, d_gw);
        if (rc != PICASSO_OK) return rc;
    }
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int picasso_f2v_forward(picasso_ctx* c, void* stream, const float* d_y, int32_t F, int32_t C, const float* d_pi,
                        int32_t T, const float* d_w, const int32_t* d_offsets, const int32_t* d_corners, int32_t N,
                        float* d_x) {
    if (!c || !d_y || F < 1 || C < 1 || !d_pi || T < 1 || !d_w || !d_offsets || !d_corners || N < 1 || !d_x)
        return PICASSO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    const bool vec4 = conv_vec4(C, {d_y, d_w, d_x});
    const bool lds = (long long)T * C <= conv::F2V_LDS_FLOATS;
    const size_t lds_bytes = lds ? sizeof(float) * (size_t)T * C : 0;
    const bool vec8 = conv_vec(C, {d_y, d_w, d_x}) == 8;
    const int grid = pool::grid_for((long long)N * (vec8 ? C / 8 : (vec4 ? C / 4 : C)));
#define PICASSO_F2V(VEC, LDS) \
    conv::f2v_forward_kernel<VEC, LDS><<<grid, pool::BLOCK, lds_bytes, s>>>(d_y, C, d_pi, T, d_w, d_offsets, d_corners, N, 3 * F, d_x)
    if (vec8) {
        if (lds) PICASSO_F2V(8, true);
        else PICASSO_F2V(8, false);
    } else if (vec4) {
        if (lds) PICASSO_F2V(4, true);
        else PICASSO_F2V(4, false);
    } else {
        if (lds) PICASSO_F2V(1, true);
        else PICASSO_F2V(1, false);
    }
#undef PICASSO_F2V
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int picasso_f2v_backward(picasso_ctx* c, void* stream, const float* d_gx, const float* d_y, int32_t F, int32_t C,
                         const float* d_pi, int32_t T, const float* d_w, const int32_t* d_facets,
                         const int32_t* d_offsets, int32_t N, float* d_gy, float* d_gw, float* d_gpi) {
    if (!c || !d_gx || !d_y || F < 1 || C < 1 || !d_pi || T < 1 || !d_w || !d_facets || !d_offsets || N < 1 ||
        (!d_gy && !d_gw && !d_gpi))
        return PICASSO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    const bool vec4 = conv_vec4(C, {d_gx, d_y, d_w, d_gy});
    if (d_gy) {
        if (conv_vec(C, {d_gx, d_w, d_gy}) == 8)
            conv::f2v_backward_y_kernel<8><<<pool::grid_for((long long)F * (C / 8)), pool::BLOCK, 0, s>>>(d_gx, C, d_pi, T, d_w, d_facets, F, d_offsets, N, d_gy);
        else if (vec4)
            conv::f2v_backward_y_kernel<4><<<pool::grid_for((long long)F * (C / 4)), pool::BLOCK, 0, s>>>(d_gx, C, d_pi, T, d_w, d_facets, F, d_offsets, N, d_gy);
        else
            conv::f2v_backward_y_kernel<1><<<pool::grid_for((long long)F * C), pool::BLOCK, 0, s>>>(d_gx, C, d_pi, T, d_w, d_facets, F, d_offsets, N, d_gy);
    }
    if (d_gw) {
        constexpr int ROWS = 8;  // filter rows per pass
        for (int t0 = 0; t0 < T; t0 += ROWS) {
            conv::F2vWeightTerm<ROWS> term{d_gx, d_y, d_pi, d_facets, d_offsets, N, C, T, t0};
            const int rc = reduce_filter_rows<ROWS>(c, s, term, F, C, vec4, std::min(ROWS, T - t0), d_gw + (size_t)t0 * C);
            if (rc != PICASSO_OK) return rc;
        }
    }
    if (d_gpi)
        conv::f2v_backward_pi_kernel<<<pool::grid_for((long long)F * T), pool::BLOCK, 0, s>>>(d_gx, d_y, C, T, d_w, d_facets, F, d_offsets, N, d_gpi);
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int picasso_replace_mapping(picasso_ctx* c, void* stream, const int32_t* d_cluster_id, int32_t n_in, int32_t n_out,
                            int32_t* d_replace, int32_t* d_mapping) {
    if (!c || !d_cluster_id || n_in < 1 || n_out < 1 || !d_replace || !d_mapping) return PICASSO_ERR_INVALID_ARG;
    if (n_out > c->max_verts) return PICASSO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    prim::fill_u32_kernel<<<1, BLOCK, 0, s>>>(reinterpret_cast<u32*>(&c->st->err), 1, 0u);
    prim::fill_u32_kernel<<<grid_for(n_out), BLOCK, 0, s>>>(reinterpret_cast<u32*>(c->newid), n_out, 0x7FFFFFFFu);
    pool::cluster_first_kernel<<<pool::grid_for(n_in), pool::BLOCK, 0, s>>>(d_cluster_id, n_in, n_out, c->newid,
                                                                            &c->st->err);
    pool::replace_mapping_kernel<<<pool::grid_for(n_in), pool::BLOCK, 0, s>>>(d_cluster_id, n_in, n_out, c->newid,
                                                                              d_replace, d_mapping);
    int rc = read_header(c, s);
    if (rc != PICASSO_OK) return rc;
    HIP_TRY(c, hipGetLastError());
    return (reinterpret_cast<State*>(c->h_pin)->err & 1) ? PICASSO_ERR_BAD_INDEX : PICASSO_OK;
}

int picasso_pool_forward(picasso_ctx* c, void* stream, int mode, const float* d_x, int32_t n_in, int32_t C,
                         const int32_t* d_offsets, const int32_t* d_members, int32_t n_out, const float* d_weight,
                         float* d_y, int32_t* d_argmax) {
    if (!c || !d_x || !d_offsets || !d_members || !d_y || n_in < 1 || n_out < 1 || C < 1 || mode < 0 || mode > 3 ||
        (mode == pool::WEIGHTED && !d_weight))
        return PICASSO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    const bool vec4 = (C % 4 == 0) && (((uintptr_t)d_x | (uintptr_t)d_y) % 16 == 0);
    if (vec4) pool::launch_pool_forward<4>(s, mode, d_x, C, d_offsets, d_members, n_out, d_weight, d_y, d_argmax);
    else pool::launch_pool_forward<1>(s, mode, d_x, C, d_offsets, d_members, n_out, d_weight, d_y, d_argmax);
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int picasso_pool_backward(picasso_ctx* c, void* stream, int mode, const float* d_gy, int32_t n_in, int32_t C,
                          const int32_t* d_cluster_id, const int32_t* d_offsets, const int32_t* d_members,
                          int32_t n_out, const float* d_weight, const int32_t* d_argmax, float* d_gx) {
    if (!c || !d_gy || !d_cluster_id || !d_offsets || !d_members || !d_gx || n_in < 1 || n_out < 1 || C < 1 ||
        mode < 0 || mode > 3 || (mode == pool::WEIGHTED && !d_weight) || (mode == pool::MAX && !d_argmax))
        return PICASSO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    const bool vec4 = (C % 4 == 0) && (((uintptr_t)d_gy | (uintptr_t)d_gx) % 16 == 0);
    if (vec4)
        pool::launch_pool_backward<4>(s, mode, d_gy, n_in, C, d_cluster_id, d_offsets, d_members, d_weight, d_argmax, d_gx);
    else
        pool::launch_pool_backward<1>(s, mode, d_gy, n_in, C, d_cluster_id, d_offsets, d_members, d_weight, d_argmax, d_gx);
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int picasso_unpool_forward(picasso_ctx* c, void* stream, const float* d_y, int32_t n_in, int32_t C,
                           const int32_t* d_cluster_id, float* d_x) {
    if (!c || !d_y || !d_cluster_id || !d_x || n_in < 1 || C < 1) return PICASSO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    const bool vec4 = (C % 4 == 0) && (((uintptr_t)d_y | (uintptr_t)d_x) % 16 == 0);
    if (vec4)
        pool::unpool_forward_kernel<4><<<pool::grid_for((long long)n_in * (C / 4)), pool::BLOCK, 0, s>>>(d_y, n_in, C, d_cluster_id, d_x);
    else
        pool::unpool_forward_kernel<1><<<pool::grid_for((long long)n_in * C), pool::BLOCK, 0, s>>>(d_y, n_in, C, d_cluster_id, d_x);
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int picasso_unpool_backward(picasso_ctx* c, void* stream, const float* d_gx, int32_t n_in, int32_t C,
                            const int32_t* d_offsets, const int32_t* d_members, int32_t n_out, float* d_gy) {
    return picasso_pool_forward(c, stream, pool::SUM, d_gx, n_in, C, d_offsets, d_members, n_out, nullptr, d_gy, nullptr);
}

int picasso_bucket_sort(picasso_ctx* c, void* stream, int key_bytes, void* d_keys, uint32_t* d_vals, int64_t n,
                        int key_bits) {
    if (!c || !d_keys || n < 0 || (key_bytes != 4 && key_bytes != 8) || key_bits < 1 || key_bits > 8 * key_bytes)
        return PICASSO_ERR_INVALID_ARG;
    if (n > 3 * c->max_facets || n > prim::BUCKET_SORT_LARGE_MAX_KEYS) return PICASSO_ERR_WORKSPACE;
    if (n == 0) return PICASSO_OK;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    int rc;
    const bool large = n > prim::BUCKET_SORT_MAX_KEYS;
    if (large && key_bits <= prim::BUCKET_LARGE_MSD_BITS) return PICASSO_ERR_INVALID_ARG;
    if (key_bytes == 8) {
        u64* k1 = c->key64[1];
        if (large)
            rc = d_vals ? prim::bucket_sort_large<u64, true>(s, (u64*)d_keys, k1, d_vals, c->val32[1], nullptr, (int)n, key_bits, c->sort_sc, c->hist12)
                        : prim::bucket_sort_large<u64, false>(s, (u64*)d_keys, k1, nullptr, nullptr, nullptr, (int)n, key_bits, c->sort_sc, c->hist12);
        else
            rc = d_vals ? prim::bucket_sort<u64, true>(s, (u64*)d_keys, k1, d_vals, c->val32[1], nullptr, (int)n, key_bits, c->sort_sc)
                        : prim::bucket_sort<u64, false>(s, (u64*)d_keys, k1, nullptr, nullptr, nullptr, (int)n, key_bits, c->sort_sc);
        if (rc == 1) HIP_TRY(c, hipMemcpyAsync(d_keys, k1, sizeof(u64) * n, hipMemcpyDeviceToDevice, s));
    } else {
        u32* k1 = reinterpret_cast<u32*>(c->key64[1]);
        if (large)
            rc = d_vals ? prim::bucket_sort_large<u32, true>(s, (u32*)d_keys, k1, d_vals, c->val32[1], nullptr, (int)n, key_bits, c->sort_sc, c->hist12)
                        : prim::bucket_sort_large<u32, false>(s, (u32*)d_keys, k1, nullptr, nullptr, nullptr, (int)n, key_bits, c->sort_sc, c->hist12);
        else
            rc = d_vals ? prim::bucket_sort<u32, true>(s, (u32*)d_keys, k1, d_vals, c->val32[1], nullptr, (int)n, key_bits, c->sort_sc)
                        : prim::bucket_sort<u32, false>(s, (u32*)d_keys, k1, nullptr, nullptr, nullptr, (int)n, key_bits, c->sort_sc);
        if (rc == 1) HIP_TRY(c, hipMemcpyAsync(d_keys, k1, sizeof(u32) * n, hipMemcpyDeviceToDevice, s));
    }
    if (rc < 0) return PICASSO_ERR_HIP;
    if (rc == 1 && d_vals) HIP_TRY(c, hipMemcpyAsync(d_vals, c->val32[1], sizeof(u32) * n, hipMemcpyDeviceToDevice, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int picasso_radix_sort(picasso_ctx* c, void* stream, int key_bytes, void* d_keys, uint32_t* d_vals, int64_t n,
                       int key_bits) {
    if (!c || !d_keys || n < 0 || (key_bytes != 4 && key_bytes != 8) || key_bits < 1 || key_bits > 8 * key_bytes)
        return PICASSO_ERR_INVALID_ARG;
    if (n > 3 * c->max_facets) return PICASSO_ERR_WORKSPACE;
    if (n == 0) return PICASSO_OK;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    int where;
    if (key_bytes == 8) {
        u64* k = (u64*)d_keys;
        where = d_vals ? prim::radix_sort<u64, true>(s, k, c->key64[1], d_vals, c->val32[1], nullptr, (int)n, key_bits, c->sort_sc)
                       : prim::radix_sort<u64, false>(s, k, c->key64[1], nullptr, nullptr, nullptr, (int)n, key_bits, c->sort_sc);
        if (where < 0) return PICASSO_ERR_HIP;
        if (where == 1) {
            HIP_TRY(c, hipMemcpyAsync(k, c->key64[1], sizeof(u64) * n, hipMemcpyDeviceToDevice, s));
            if (d_vals) HIP_TRY(c, hipMemcpyAsync(d_vals, c->val32[1], sizeof(u32) * n, hipMemcpyDeviceToDevice, s));
        }
    } else {
        u32* k = (u32*)d_keys;
        u32* k1 = reinterpret_cast<u32*>(c->key64[1]);
        where = d_vals ? prim::radix_sort<u32, true>(s, k, k1, d_vals, c->val32[1], nullptr, (int)n, key_bits, c->sort_sc)
                       : prim::radix_sort<u32, false>(s, k, k1, nullptr, nullptr, nullptr, (int)n, key_bits, c->sort_sc);
        if (where < 0) return PICASSO_ERR_HIP;
        if (where == 1) {
            HIP_TRY(c, hipMemcpyAsync(k, k1, sizeof(u32) * n, hipMemcpyDeviceToDevice, s));
            if (d_vals) HIP_TRY(c, hipMemcpyAsync(d_vals, c->val32[1], sizeof(u32) * n, hipMemcpyDeviceToDevice, s));
        }
    }
    HIP_TRY(c, hipStreamSynchronize(s));
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

}  // extern "C"
