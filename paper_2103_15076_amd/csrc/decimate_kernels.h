// decimate_kernels.h -- device side of the round-based QEM mesh decimation for
// gfx950: Algorithm 2 of the Picasso paper (Sec. 3) and the quadric equations of
// its supplementary section "Quadric error computation".  The greedy grouping
// that the paper leaves on the CPU (Alg. 2 lines 3-10) is done on the GPU by a
// parallel construction of the same matching.  Host side: picasso.hip.
//
// All fp32 arithmetic is written as single IEEE operations in a fixed order
// and compiled without contraction, so that results are reproducible to the bit.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <type_traits>

#include "primitives.h"

#pragma clang fp contract(off)

using prim::u32;
using prim::u64;

namespace {

constexpr int BLOCK = prim::BLOCK;
constexpr u64 VMIN_NONE = ~0ull;
constexpr int ERR_BIT_BAD_INDEX = 1, ERR_BIT_NONFINITE = 2, ERR_BIT_INTERNAL = 4;  // State::err

// ---------------------------------------------------------------------------
// Device-resident bookkeeping
// ---------------------------------------------------------------------------
struct State {
    int err;       // bit0: bad facet index, bit1: non-finite coordinate, bit2: a kernel was launched for sizes it does not take
    int nv[2];     // vertex count, ping-pong by round parity
    int nf[2];     // facet count, ping-pong
    int nh;        // 3 * nf of the current round (half-edge keys to sort)
    int ne;        // distinct edges of the current round
    int live[3];   // worklist lengths of the selection sub-rounds (rotating)
    int trunc_n;   // matched edges entering the budget truncation
    int sel_k;     // sub-round index the selection has reached (buffer rotation phase)
    int absorb_n;  // edges through which an un-paired vertex would join a pair's cluster (Alg. 2 line 11)
    int nv_kept;   // output vertices that some output facet refers to (option: degenerated vertices dropped)
    // Written by every selection tail for kernels that the host queued behind it before looking
    // (they run only if the tail finished the matching): 1 / nv / nf / ne of the round then, else zeros.
    int go, guard_nv, guard_nf, guard_ne;
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

// Plane of a facet as (unit normal, d) with n . x + d = 0 (supplementary, facet quadric equation);
// a facet of zero area or with a repeated index gets the zero plane, hence the zero quadric.
// Positions come from the caller's packed [N,3] array.
__device__ __forceinline__ float4 facet_plane(const float* __restrict__ verts, int i0, int i1, int i2) {
    const float4 none = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (i0 == i1 || i1 == i2 || i0 == i2) return none;
    const float3 p0 = make_float3(verts[3 * (size_t)i0], verts[3 * (size_t)i0 + 1], verts[3 * (size_t)i0 + 2]);
    const float3 p1 = make_float3(verts[3 * (size_t)i1], verts[3 * (size_t)i1 + 1], verts[3 * (size_t)i1 + 2]);
    const float3 p2 = make_float3(verts[3 * (size_t)i2], verts[3 * (size_t)i2 + 1], verts[3 * (size_t)i2 + 2]);
    float ax = p1.x - p0.x, ay = p1.y - p0.y, az = p1.z - p0.z;
    float bx = p2.x - p0.x, by = p2.y - p0.y, bz = p2.z - p0.z;
    float nx = ay * bz - az * by;
    float ny = az * bx - ax * bz;
    float nz = ax * by - ay * bx;
    float len = sqrtf((nx * nx + ny * ny) + nz * nz);
    if (len == 0.0f) return none;
    nx = nx / len;
    ny = ny / len;
    nz = nz / len;
    const float d = -((nx * p0.x + ny * p0.y) + nz * p0.z);
    return make_float4(nx, ny, nz, d);
}

// A single mesh's header (State and the per-mesh tables) written by init_kernel itself instead of
// a copy from the host in front of it: everything zero except the counts, the mesh's vertex and
// facet ranges and its target.  State::err is left alone (other workgroups of the same kernel flag
// errors there): it is zero between calls.  hdr == nullptr: the header has been uploaded.
struct HeaderInit {
    int* hdr;
    int total;                           // ints in the header
    int at_voff0, at_foff, at_target;    // where the tables start
    int N, F, target;
};

// Incidence keys for S0: (vertex << fbits) | facet, one per facet corner, so that sorting the keys
// alone lists every vertex's facets in ascending facet order.  With COUNT_SMALL / COUNT_LARGE the
// kernel also adds the keys' top 8- / 12-bit digits (bits [ishift, ...)) to ihist, the histogram
// that the sort of the keys starts from (zero on entry; see quadric_rows_kernel); that sort makes
// the keys again from the validated facet array (IncidenceKeys), so they are written out (ikey)
// only for a sort that needs them in memory.
template <int COUNT>
__global__ __launch_bounds__(BLOCK) void init_kernel(const float* __restrict__ verts, int N,
                                                     const int* __restrict__ facets, int F, int B,
                                                     const int* __restrict__ voff, const int* __restrict__ foff,
                                                     VRec* __restrict__ vrec, int* __restrict__ cid,
                                                     int* __restrict__ fcur, u64* __restrict__ ikey, int fbits,
                                                     int ishift, u32* __restrict__ ihist, State* st,
                                                     u32* __restrict__ msd_hist, int s0_follows, HeaderInit init,
                                                     float4* __restrict__ planes) {
    constexpr int RADIX = COUNT == COUNT_LARGE ? (1 << prim::BUCKET_LARGE_MSD_BITS) : (1 << prim::BUCKET_MSD_BITS);
    __shared__ u32 hist[COUNT != COUNT_NONE ? RADIX : 1];
    const int stride = gridDim.x * BLOCK;
    const int g = blockIdx.x * BLOCK + threadIdx.x;
    const bool single = init.hdr != nullptr;  // one mesh, whose ranges are [0, N) and [0, F): the tables are not read here
    if (single && blockIdx.x == 0) {
        constexpr int ERR = (int)(offsetof(State, err) / sizeof(int));
        constexpr int NV0 = (int)(offsetof(State, nv) / sizeof(int)), NF0 = (int)(offsetof(State, nf) / sizeof(int));
        for (int i = threadIdx.x; i < init.total; i += BLOCK) {
            if (i == ERR) continue;
            int v = 0;
            if (i == NV0 || i == init.at_voff0 + 1) v = init.N;
            else if (i == NF0 || i == init.at_foff + 1) v = init.F;
            else if (i == init.at_target) v = init.target;
            init.hdr[i] = v;
        }
    }
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
        if (!s0_follows) {  // (else quadric_rows_kernel writes the whole record)
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
            if (single) {
                hi = N;
            } else {
                const int m = mesh_of(foff, B, f);
                lo = voff[m];
                hi = voff[m + 1];
            }
        }
        int corner[3] = {0, 0, 0};
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            u64 k = 0;
            if (ok) {
                int a = facets[3 * (size_t)f + c];
                if (a < lo || a >= hi) { err |= 1; a = lo; }
                fcur[3 * (size_t)f + c] = a;
                corner[c] = a;
                k = ((u64)(u32)a << fbits) | (u64)(u32)f;
                if (ikey) ikey[3 * (size_t)f + c] = k;
            }
            if constexpr (COUNT != COUNT_NONE) {
                // neighbouring facets mostly refer to vertices with the same leading bits: the lanes of a
                // wave that share a digit count themselves with a single LDS atomic
                const u32 d = (u32)(k >> ishift) & (u32)(RADIX - 1);
                const u64 same = prim::wave_same_digit_lanes(ok, d);
                if (ok && (same & prim::lanemask_lt()) == 0) atomicAdd(&hist[d], (u32)__popcll(same));
            }
        }
        // the facet's plane, once per facet, for the vertex quadrics that S0 sums from it
        if (planes && ok) planes[f] = facet_plane(verts, corner[0], corner[1], corner[2]);
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

// Ordered segmented reduction over the sorted incidence keys (vertex << fbits | facet): the keys of
// one vertex are consecutive and ascend in facet index, which is the order of the sum.  A
// workgroup takes a tile of the keys; every lane fetches the planes of its share of the tile's
// incidences into LDS (16 bytes gathered per incidence, all of a tile's gathers in flight together:
// the plane was computed once per facet by init_kernel); the positions where a new vertex starts
// are listed, and every such row goes to one lane, which adds up the facets' quadrics
// Q = (n n^T, d n, d^2) left to right and writes the vertex's whole 64-byte record, position
// included.  A row that runs past the end of its tile is followed into the next one (whose first
// keys are then no row start).  Vertices without any facet appear in no key: the row of the next
// vertex that has one notes the run of them in front of it (the last row also the run behind it),
// and the workgroup writes their records (zero quadric) together.
constexpr int QR_ITEMS = 4;
constexpr int QR_TILE = BLOCK * QR_ITEMS;
constexpr int QR_GAPS = 64;  // runs of facet-less vertices a tile lists (further ones are written by the lane that meets them)

__device__ __forceinline__ void write_vertex_record(VRec* __restrict__ vrec, const float* __restrict__ verts, int v,
                                                    const float (&acc)[10]) {
    float4* r = reinterpret_cast<float4*>(&vrec[v]);
    r[0] = make_float4(verts[3 * (size_t)v], verts[3 * (size_t)v + 1], verts[3 * (size_t)v + 2], 0.f);
    r[1] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    r[2] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    r[3] = make_float4(acc[8], acc[9], 0.f, 0.f);
}

// acc += the quadric of the plane (n, d), coefficient by coefficient
__device__ __forceinline__ void add_plane_quadric(float (&acc)[10], const float4 pl) {
    const float q0 = pl.x * pl.x, q1 = pl.x * pl.y, q2 = pl.x * pl.z, q3 = pl.y * pl.y, q4 = pl.y * pl.z;
    const float q5 = pl.z * pl.z, q6 = pl.w * pl.x, q7 = pl.w * pl.y, q8 = pl.w * pl.z, q9 = pl.w * pl.w;
    acc[0] = acc[0] + q0; acc[1] = acc[1] + q1; acc[2] = acc[2] + q2; acc[3] = acc[3] + q3;
    acc[4] = acc[4] + q4; acc[5] = acc[5] + q5; acc[6] = acc[6] + q6; acc[7] = acc[7] + q7;
    acc[8] = acc[8] + q8; acc[9] = acc[9] + q9;
}

__global__ __launch_bounds__(BLOCK) void quadric_rows_kernel(VRec* __restrict__ vrec, const float* __restrict__ verts,
                                                             int N, const float4* __restrict__ planes,
                                                             const u64* __restrict__ inc, int H, int fbits,
                                                             u32* __restrict__ ihist) {
    __shared__ float4 splane[QR_TILE];         // plane of the facet of the key at position base + i
    __shared__ int svert[QR_TILE + 1];         // svert[i + 1] = vertex of that key; svert[0] = of the key in front of the tile (-1: none)
    __shared__ unsigned short hpos[QR_TILE];   // positions (within the tile) where a vertex's row starts, ascending
    __shared__ u32 smem[prim::WAVES];
    __shared__ int gap[2 * QR_GAPS];           // runs [first, end) of vertices without facets met by this tile's rows
    __shared__ int n_gaps;
    const int t = threadIdx.x;
    // last kernel of S0: the incidence sort's digit counts and cursors go back to zero for the next call
    for (int i = blockIdx.x * BLOCK + t; i < 2 * prim::MSD_HIST_WORDS; i += gridDim.x * BLOCK) ihist[i] = 0;
    const float zero[10] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (H <= 0) {  // no facets at all: every vertex gets the zero quadric
        for (int v = blockIdx.x * BLOCK + t; v < N; v += gridDim.x * BLOCK) write_vertex_record(vrec, verts, v, zero);
        return;
    }
    const long long tile = blockIdx.x;
    const long long base = tile * QR_TILE;
    if (base >= H) return;
    const int tile_n = (int)((long long)H - base < QR_TILE ? (long long)H - base : QR_TILE);
    const u64 fmask = (1ull << fbits) - 1ull;
#pragma unroll
    for (int j = 0; j < QR_ITEMS; ++j) {
        const int i = j * BLOCK + t;
        if (i < tile_n) {
            const u64 key = inc[base + i];
            svert[i + 1] = (int)(key >> fbits);
            splane[i] = planes[(size_t)(key & fmask)];
        }
    }
    if (t == 0) {
        svert[0] = base > 0 ? (int)(inc[base - 1] >> fbits) : -1;
        n_gaps = 0;
    }
    __syncthreads();
    // thread t looks at positions t * QR_ITEMS .. + QR_ITEMS - 1, so that the list of starts is in order
    u32 mine = 0;
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < QR_ITEMS; ++j) {
        const int i = t * QR_ITEMS + j;
        if (i < tile_n && svert[i + 1] != svert[i]) {
            mine |= 1u << j;
            ++cnt;
        }
    }
    u32 n_rows;
    u32 at = prim::block_exclusive_scan((u32)cnt, smem, n_rows);
#pragma unroll
    for (int j = 0; j < QR_ITEMS; ++j)
        if (mine & (1u << j)) hpos[at++] = (unsigned short)(t * QR_ITEMS + j);
    __syncthreads();
    auto note_gap = [&](int first, int end) {
        const int slot = atomicAdd(&n_gaps, 1);
        if (slot < QR_GAPS) {
            gap[2 * slot] = first;
            gap[2 * slot + 1] = end;
        } else {
            for (int g = first; g < end; ++g) write_vertex_record(vrec, verts, g, zero);
        }
    };
    for (int r = t; r < (int)n_rows; r += BLOCK) {
        const int hp = hpos[r];
        const int row_end = r + 1 < (int)n_rows ? (int)hpos[r + 1] : tile_n;  // (within the tile)
        const int v = svert[hp + 1];
        const int pv = svert[hp];  // vertices between the row in front of this one and this one have no facet
        if (pv + 1 < v) note_gap(pv + 1, v);
        float acc[10];
#pragma unroll
        for (int k = 0; k < 10; ++k) acc[k] = 0.0f;
        for (int j = hp; j < row_end; ++j) add_plane_quadric(acc, splane[j]);
        bool last_of_all = false;
        if (row_end == tile_n) {  // the tile's last row may go on in the next tile
            long long j = base + tile_n;
            for (; j < H; ++j) {
                const u64 key = inc[j];
                if ((int)(key >> fbits) != v) break;
                add_plane_quadric(acc, planes[(size_t)(key & fmask)]);
            }
            last_of_all = j >= H;
        }
        write_vertex_record(vrec, verts, v, acc);
        if (last_of_all && v + 1 < N) note_gap(v + 1, N);  // the vertices behind the last row have no facet either
    }
    __syncthreads();
    const int ng = n_gaps < QR_GAPS ? n_gaps : QR_GAPS;
    for (int i = 0; i < ng; ++i)
        for (int g = gap[2 * i] + t; g < gap[2 * i + 1]; g += BLOCK) write_vertex_record(vrec, verts, g, zero);
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
                // the lower vertices of neighbouring corners mostly share their leading bits: the lanes of
                // a wave that share a digit count themselves with a single LDS atomic
                const u32 d = (u32)(k >> shift) & (u32)(RADIX - 1);
                const u64 same = prim::wave_same_digit_lanes(ok, d);
                if (ok && (same & prim::lanemask_lt()) == 0) atomicAdd(&hist[d], (u32)__popcll(same));
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

// A word in the context's pinned host memory and the number to store there: the last kernel
// before a look of the host stores it once its results are written, so that the host may watch
// that word instead of waiting for the stream.
struct HostSignal {
    int* word;
    int seq;
};

// By every thread of the (single) workgroup, as its last act: the workgroup's stores to host
// memory are complete before one thread stores the sequence number.  `wrote`: this thread has
// stored something the host will read (only those threads need the fence, which is not cheap).
__device__ __forceinline__ void signal_host(const HostSignal& h, int tid, bool wrote) {
    if (wrote) __threadfence_system();
    __syncthreads();
    if (tid == 0) __hip_atomic_store(h.word, h.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

struct SelArgs {
    const u64* ekey;
    const u32* ecost;
    u64* vmin[3];
    int* mate;
    int* list;              // live edges gathered for the tail,
    const u64* lkey;        // ... their keys
    const u32* lcost;       // ... and cost keys, in the same order
    unsigned char* estate;  // per edge: 0 = live, 1 = retired (paired, or an end was paired)
    State* st;
    MeshTab mt;
    int vbits;
    int* host_img;     // pinned host memory, device view: the tail leaves [State][matched] there
    int publish_ints;  // for the host, which then needs no copy of its own before it looks
    int* host_check;   // ... and, behind them, the number that the kernel after it will store in the
    int host_seq;      // sequence word (the host compares the two before it trusts what it reads)
    TieBreak tb;       // order among edges of equal cost
    int cur;           // which of the ping-pong vertex / facet counts belong to this round
    int* tile_live;    // not null (last grid-wide sub-round before the tail, one edge per lane and no
                       // striding): workgroup b leaves here how many of its edges stay live, which is
                       // the count pass of the gather that follows
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
    bool alive = false;
    for (long long base = (long long)blockIdx.x * BLOCK; base < n; base += (long long)gridDim.x * BLOCK) {
        const long long i = base + threadIdx.x;
        bool sel = false;
        alive = false;
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
    if (A.tile_live) {  // (the host has made the grid cover every edge in one step)
        __shared__ int wave_live[BLOCK / 64];
        const u64 b = __ballot(alive);
        if (prim::lane_id() == 0) wave_live[prim::wave_id()] = (int)__popcll(b);
        __syncthreads();
        if (threadIdx.x == 0) {
            int tot = 0;
#pragma unroll
            for (int j = 0; j < BLOCK / 64; ++j) tot += wave_live[j];
            A.tile_live[blockIdx.x] = tot;
        }
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

// The gathered live edges, with their keys and cost keys beside them: the tail then reads three
// contiguous arrays at once, not the list and then, through it, the edge arrays.
struct LiveOut {
    int* list;
    const u64* ekey;
    const u32* ecost;
    u64* lkey;
    u32* lcost;
    __device__ void operator()(int e, int pos) const {
        list[pos] = e;
        lkey[pos] = ekey[e];
        lcost[pos] = ecost[e];
    }
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

// A word for the host: stored at system scope (not left in a cache of the device), so that it is in
// host memory when the kernel has ended.
__device__ __forceinline__ void host_store(int* p, int v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// By every thread of the tail, after its last store for the host: once all of them are issued, the
// copy of the sequence number follows them.
__device__ __forceinline__ void tail_mark_published(const SelArgs& A, int tid) {
    __syncthreads();
    if (tid == 0) host_store(A.host_check, A.host_seq);
}

// The round's counters and pair counts, written straight into the host's pinned memory (read at
// the L2, where this kernel's own stores to them already are).
__device__ __forceinline__ void tail_publish(const SelArgs& A, int tid) {
    const int* hdr = reinterpret_cast<const int*>(A.st);
    constexpr int GO0 = (int)(offsetof(State, go) / sizeof(int)), STATE_INTS = (int)(sizeof(State) / sizeof(int));
    for (int i = tid; i < A.publish_ints; i += TAIL_THREADS)
        if (i < GO0 || i >= STATE_INTS)  // (the guard fields are for the device only; the tail is writing them)
            host_store(&A.host_img[i], __hip_atomic_load(&hdr[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

// What the kernels queued behind the tail go by (see State).
__device__ __forceinline__ void tail_set_guard(const SelArgs& A, bool finished) {
    A.st->go = finished ? 1 : 0;
    A.st->guard_nv = finished ? A.st->nv[A.cur] : 0;
    A.st->guard_nf = finished ? A.st->nf[A.cur] : 0;
    A.st->guard_ne = finished ? A.st->ne : 0;
}

__global__ __launch_bounds__(TAIL_THREADS) void select_tail_kernel(SelArgs A) {
    __shared__ TailLds L;
    int n = A.st->live[0];     // live edges, gathered into A.list just before this kernel
    const int tid = threadIdx.x, lane = prim::lane_id();
    if (n > TAIL_MAX) {        // too many: the host runs more grid-wide sub-rounds
        if (tid == 0) tail_set_guard(A, false);
        tail_publish(A, tid);
        tail_mark_published(A, tid);
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
        const u64 key = A.lkey[i];
        L.prio[i] = A.tb.priority(A.lcost[i], e);
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
            if (lds_pairs && STATE_INTS + b < A.publish_ints) host_store(&A.host_img[STATE_INTS + b], sum);
        }
    }
    if (tid == 0) {
        A.st->live[0] = 0;
        tail_set_guard(A, true);
    }
    if (lds_pairs) {
        // the host's copy of the counters: everything but live[0] was written by earlier kernels
        constexpr int LIVE0 = (int)(offsetof(State, live) / sizeof(int)), GO0 = (int)(offsetof(State, go) / sizeof(int));
        const int* hdr = reinterpret_cast<const int*>(A.st);
        if (tid < GO0 && tid < A.publish_ints) host_store(&A.host_img[tid], (tid == LIVE0) ? 0 : hdr[tid]);
    } else {
        __threadfence();
        __syncthreads();
        tail_publish(A, tid);
    }
    tail_mark_published(A, tid);
}

// The selection tail does not tell the host itself (a system-scope fence inside it, with the pairs it
// has just written still in the cache, costs more than a launch): the kernel after it on the stream
// does, as its first act, with a release store at system scope: what the kernels before that one
// have written is visible to it when it starts, so the release carries those writes along (there
// is next to nothing left in the cache to write back then, so it costs nothing measurable).  Either the first of the kernels queued ahead of the host's
// look (through the counting predicate's on_start) ...
template <class Pred>
struct SignalingPred {
    Pred pred;
    HostSignal done;
    __device__ void on_start() const {
        if (done.word) __hip_atomic_store(done.word, done.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    __device__ bool operator()(int i) const { return pred(i); }
};
// ... or a kernel of its own.
__global__ void signal_kernel(HostSignal done) {
    if (threadIdx.x == 0) __hip_atomic_store(done.word, done.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
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
// and an add per key and bit; the keys that share the bits decided so far are dealt out again
// once they are few and then decided 8 bits at a time by counts per digit, and in the end one wave
// decides the remaining bits without barriers), and
// flags every pair
// above that key and, among the pairs with exactly that key, all but the first ones in edge order.  A wide kernel then releases the
// flagged pairs.  One compute unit does the whole search, so runs longer than TRUNC_BLOCK_CAP go
// to the sort instead.
constexpr int TRUNC_THREADS = 1024;
constexpr int TRUNC_REGS_MAX = 32;
constexpr int TRUNC_BLOCK_CAP = TRUNC_THREADS * TRUNC_REGS_MAX;
constexpr int TRUNC_NARROW_BLOCK = 4 * TRUNC_THREADS;  // candidates that are dealt out again, 4 to a thread
constexpr int TRUNC_NARROW_WAVE = 4 * 64;              // candidates that one wave takes over, 4 to a lane

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
                                                                    const int* __restrict__ nrem,
                                                                    const int* __restrict__ guard, State* st) {
    if (guard && *guard == 0) return;  // queued ahead of the host's look, and the selection was not finished
    constexpr int NW = TRUNC_THREADS / 64;
    __shared__ u32 wsum[NW];
    __shared__ u32 wsum2[2][NW];
    __shared__ u32 cnt[R * NW];
    __shared__ u32 cbuf[TRUNC_NARROW_BLOCK];
    __shared__ u32 found[3];
    __shared__ u32 dhist[256];  // the narrow phase's counts per 8-bit digit
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
    if (n > R * TRUNC_THREADS) {
        // More pairs than this instance holds: the host never launches it so.  Nothing is released, and
        // the call is made to fail (ERR_BIT_INTERNAL) instead of returning a budget that was not applied.
        for (int i = tid; i < n; i += TRUNC_THREADS) tcost[i] = 0u;
        if (tid == 0) atomicOr(&st->err, ERR_BIT_INTERNAL);
        return;
    }

    u32 key[R];  // empty slots hold the largest key
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i = r * TRUNC_THREADS + tid;
        key[r] = i < n ? tcost[i] : 0xFFFFFFFFu;
    }

    // Number of values <= x among the RR that every thread holds, known to every thread after one
    // barrier (`slot` alternates so that the next count does not overwrite sums still being read).
    auto count_le = [&](const auto& a, auto rr, u32 x, int slot) -> u32 {
        constexpr int RR = decltype(rr)::value;
        u32 c = 0;
#pragma unroll
        for (int r = 0; r < RR; ++r) c += (a[r] <= x) ? 1u : 0u;
        c = wave_sum_u32(c);
        if (lane == 0) wsum2[slot][w] = c;
        __syncthreads();
        u32 tot = 0;
#pragma unroll
        for (int j = 0; j < NW; ++j) tot += wsum2[slot][j];
        return tot;
    };
    // One wave alone finishes a search over at most TRUNC_NARROW_WAVE values held in `cbuf` (the
    // first `m` entries): the smallest x whose low bits (`bit` and below) extend `pre` such that at
    // least `want` values are <= x, `outside` values that are not in `cbuf` being below every
    // candidate.  Returns x and how many values are < x; no barriers, 4 compares per lane and bit.
    auto wave_search = [&](u32 m, u32 pre, int bit, u32 outside, u32 want, u32& less_out) -> u32 {
        u32 less = outside;  // values < pre: those outside `cbuf`, then the candidates passed over
        u32 ck[TRUNC_NARROW_WAVE / 64];
#pragma unroll
        for (int j = 0; j < TRUNC_NARROW_WAVE / 64; ++j) ck[j] = (u32)(j * 64 + lane) < m ? cbuf[j * 64 + lane] : 0xFFFFFFFFu;
        for (; bit >= 0; --bit) {
            const u32 x = pre | ((1u << bit) - 1u);
            u32 c = 0;
#pragma unroll
            for (int j = 0; j < TRUNC_NARROW_WAVE / 64; ++j) c += (u32)__popcll(__ballot(ck[j] <= x));
            c = outside + (c < m ? c : m);  // (the empty places count when x is the largest value)
            if (c < want) {
                pre |= 1u << bit;
                less = c;
            }
        }
        less_out = less;
        return pre;
    };
    // Those of the RR values a thread holds that satisfy `is_cand` go to consecutive places of
    // `cbuf`; returns how many there are in the workgroup (the caller knows that they fit).
    auto gather_candidates = [&](auto rr, auto is_cand, auto value_of) -> u32 {
        constexpr int RR = decltype(rr)::value;
        u32 mc = 0;
#pragma unroll
        for (int r = 0; r < RR; ++r) mc += is_cand(r) ? 1u : 0u;
        u32 m;
        u32 at = prim::wide_block_exclusive_scan<NW>(mc, wsum, m);
#pragma unroll
        for (int r = 0; r < RR; ++r)
            if (is_cand(r) && at < (u32)TRUNC_NARROW_BLOCK) cbuf[at++] = value_of(r);
        __syncthreads();
        return m;
    };

    // The search: the smallest x with at least `want` of the values a[] <= x, bit by bit from the
    // top.  Every thread holds R values, `valid` of them in the workgroup are real (is_real(r)), the
    // others hold the largest value.  below = values < prefix, upper = values <= prefix | (undecided
    // bits all set): upper - below values share the bits decided so far.  Once there are at most
    // TRUNC_NARROW_BLOCK of them they are dealt out again, 4 to a thread; once at most
    // TRUNC_NARROW_WAVE, one wave takes them and finishes alone.  Leaves x in `prefix` and the
    // number of values < x in `below`.
    u32 prefix = 0, below = 0, upper = 0, want = 0;
    int bit = -1;
    // steps over the values in `a` (of which `real` are real, `outside` more lie below them all)
    auto steps = [&](const auto& a, auto rr, u32 real, u32 outside, u32 until) {
        while (bit >= 0 && upper - below > until) {
            u32 c = count_le(a, rr, prefix | ((1u << bit) - 1u), bit & 1);
            c = outside + (c < real ? c : real);  // (the other slots count when x is the largest value)
            if (c < want) {
                prefix |= 1u << bit;
                below = c;
            } else {
                upper = c;
            }
            --bit;
        }
    };
    auto finish_in_one_wave = [&](auto rr, auto is_cand, auto value_of) {
        const u32 outside = below;
        const u32 m = gather_candidates(rr, is_cand, value_of);
        if (w == 0) {
            u32 less;
            const u32 x = wave_search(m, prefix, bit, outside, want, less);
            if (lane == 0) {
                found[0] = x;
                found[1] = less;
            }
        }
        __syncthreads();
        prefix = found[0];
        below = found[1];
    };
    auto search = [&](const auto& a, auto is_real, u32 valid, u32 want_) {
        const auto all_r = std::integral_constant<int, R>{};
        const auto four = std::integral_constant<int, 4>{};
        auto decided_mask = [&]() -> u32 { return bit == 31 ? 0u : ~0u << (bit + 1); };
        prefix = 0;
        below = 0;
        upper = valid;
        want = want_;
        bit = 31;
        __syncthreads();  // (a search before this one has finished with the shared arrays)
        steps(a, all_r, valid, 0u, R > 4 ? (u32)TRUNC_NARROW_BLOCK : (u32)TRUNC_NARROW_WAVE);
        if (R > 4 && bit >= 0 && upper - below > (u32)TRUNC_NARROW_WAVE) {
            const u32 decided = decided_mask(), outside = below;
            const u32 m = gather_candidates(
                all_r, [&](int r) { return is_real(r) && (a[r] & decided) == prefix; }, [&](int r) { return a[r]; });
            u32 k4[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) k4[j] = (u32)(j * TRUNC_THREADS + tid) < m ? cbuf[j * TRUNC_THREADS + tid] : 0xFFFFFFFFu;
            (void)outside;
            // ... and decided 8 bits at a time from here on: the candidates that share the decided bits are
            // counted per digit in LDS (the lanes of a wave that hold one digit with a single atomic: where
            // many pairs tie at the threshold they all hold the same), and the digit in which the running
            // count reaches what is still wanted is found by one scan: three barriers per 8 bits instead
            // of one per bit
            while (bit >= 0 && upper - below > (u32)TRUNC_NARROW_WAVE) {
                const int nb = bit >= 7 ? 8 : bit + 1, shift = bit + 1 - nb;
                const u32 dec = decided_mask();
                if (tid < 256) dhist[tid] = 0;
                __syncthreads();
#pragma unroll
                for (int j = 0; j < 4; ++j) {  // (whole waves, for the ballots)
                    const bool ok = (u32)(j * TRUNC_THREADS + tid) < m && (k4[j] & dec) == prefix;
                    const u32 dg = (k4[j] >> shift) & ((1u << nb) - 1u);
                    const u64 same = prim::wave_same_digit_lanes(ok, dg);
                    if (ok && (same & lt) == 0) atomicAdd(&dhist[dg], (u32)__popcll(same));
                }
                __syncthreads();
                const u32 c = tid < 256 ? dhist[tid] : 0u;
                u32 tot;
                const u32 run = prim::wide_block_exclusive_scan<NW>(c, wsum, tot);
                const u32 need = want - below;  // >= 1, and at most the number of candidates
                if (tid < 256 && run < need && need <= run + c) {
                    found[0] = (u32)tid;
                    found[1] = run;
                    found[2] = c;
                }
                __syncthreads();
                prefix |= found[0] << shift;
                below += found[1];
                upper = below + found[2];
                bit -= nb;
            }
            if (bit >= 0) {
                const u32 d2 = decided_mask();
                finish_in_one_wave(
                    four, [&](int j) { return (u32)(j * TRUNC_THREADS + tid) < m && (k4[j] & d2) == prefix; },
                    [&](int j) { return k4[j]; });
            }
        } else if (bit >= 0) {
            const u32 decided = decided_mask();
            finish_in_one_wave(
                all_r, [&](int r) { return is_real(r) && (a[r] & decided) == prefix; }, [&](int r) { return a[r]; });
        }
    };

    // the cost key of the keep-th smallest pair, and how many pairs with exactly that key stay
    u32 kk = 0;
    if (keep > 0) {
        search(key, [&](int r) { return r * TRUNC_THREADS + tid < n; }, (u32)n, (u32)keep);
        kk = (u32)keep - below;
    }
    const u32 kprefix = prefix;
    if constexpr (SHUFFLE) {
        // ... the first kk in the order of the seeded tie-break, which is distinct from pair to pair:
        // the same search once more, on the tie-break values of the pairs with that key
        u32 tie[R];
        u32 neq = 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int i = r * TRUNC_THREADS + tid;
            const bool eq = i < n && key[r] == kprefix;
            tie[r] = eq ? tb.enc(tval[i]) : 0xFFFFFFFFu;
            neq += eq ? 1u : 0u;
        }
        {
            u32 tot;
            (void)prim::wide_block_exclusive_scan<NW>(neq, wsum, tot);
            neq = tot;
        }
        u32 t2 = 0;
        if (kk > 0) {
            search(tie, [&](int r) { return r * TRUNC_THREADS + tid < n && key[r] == kprefix; }, neq, kk);
            t2 = prefix;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int i = r * TRUNC_THREADS + tid;
            if (i < n) tcost[i] = (key[r] > kprefix || (key[r] == kprefix && (kk == 0 || tie[r] > t2))) ? 1u : 0u;
        }
        return;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const bool eq = (r * TRUNC_THREADS + tid < n) && key[r] == kprefix;
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
        const bool eq = valid && key[r] == kprefix, gt = valid && key[r] > kprefix;
        const u64 eb = __ballot(eq);
        const u32 rank = cnt[r * NW + w] + (u32)__popcll(eb & lt);
        if (valid) tcost[i] = (gt || (eq && rank >= kk)) ? 1u : 0u;  // the key's slot now holds the flag
    }
}

// ---------------------------------------------------------------------------
// Budget for ONE long run (a single mesh that formed more pairs than one workgroup's registers hold)
// without sorting it: the cost key of the nrem-th smallest pair is found digit by digit, from the top,
// by histograms over the gathered cost keys (tcost, in edge order): three passes of 11, 11 and 10 bits,
// each a wide kernel that counts the keys which share the digits decided so far, and one small
// workgroup that picks the digit in which the count crosses nrem.  Then the pairs with exactly that
// key are ranked in edge order by the atomic-free scan, and every pair above the key, or at the key but
// beyond the budget, is flagged for trunc_release_kernel, as trunc_block_kernel does it.
// ---------------------------------------------------------------------------
constexpr int SELECT_BINS = 1 << 11;
struct SelectState {
    u32 prefix;  // the digits decided so far, right-aligned (after the last pass: the threshold key)
    u32 below;   // keys smaller than every key that starts with `prefix`
    u32 keep;    // (after the last pass) how many of the pairs with exactly the threshold key stay
    u32 pad;
    u32 hist[SELECT_BINS];
};
__device__ __forceinline__ int select_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ int select_bits(int pass) { return pass == 2 ? 10 : 11; }

constexpr int SELECT_ITEMS = 8;
template <int PASS>
__global__ __launch_bounds__(BLOCK) void trunc_select_hist_kernel(const u32* __restrict__ tcost, const State* st,
                                                                  SelectState* __restrict__ S) {
    __shared__ u32 h[SELECT_BINS];
    const int n = st->trunc_n;
    const long long base = (long long)blockIdx.x * (BLOCK * SELECT_ITEMS);
    if (base >= n) return;
    const int t = threadIdx.x;
    for (int i = t; i < SELECT_BINS; i += BLOCK) h[i] = 0;
    const u32 prefix = PASS == 0 ? 0u : S->prefix;
    const int shift = select_shift(PASS), bits = select_bits(PASS);
    __syncthreads();
    u32 key[SELECT_ITEMS];
#pragma unroll
    for (int i = 0; i < SELECT_ITEMS; ++i) {
        const long long idx = base + (long long)i * BLOCK + t;
        key[i] = idx < n ? tcost[idx] : 0u;
    }
#pragma unroll
    for (int i = 0; i < SELECT_ITEMS; ++i) {  // (whole waves run every step, for the ballots)
        const long long idx = base + (long long)i * BLOCK + t;
        // keys that share the digits decided so far; cost keys cluster, so the lanes of a wave that hold
        // one digit count themselves with a single LDS atomic
        const bool ok = idx < n && (PASS == 0 || (key[i] >> (shift + bits)) == prefix);
        const u32 d = (key[i] >> shift) & ((1u << bits) - 1u);
        const u64 same = prim::wave_same_digit_lanes(ok, d);
        if (ok && (same & prim::lanemask_lt()) == 0) atomicAdd(&h[d], (u32)__popcll(same));
    }
    __syncthreads();
    for (int i = t; i < SELECT_BINS; i += BLOCK) {
        const u32 c = h[i];
        if (c) atomicAdd(&S->hist[i], c);
    }
}

// One workgroup: the digit in which the running count of the histogram reaches the budget; the
// histogram is left zero for the next pass.
template <int PASS>
__global__ __launch_bounds__(BLOCK) void trunc_select_pick_kernel(SelectState* __restrict__ S,
                                                                  const int* __restrict__ nrem) {
    constexpr int PER = SELECT_BINS / BLOCK;
    __shared__ u32 smem[prim::WAVES];
    const int t = threadIdx.x;
    const u32 below = PASS == 0 ? 0u : S->below, prefix = PASS == 0 ? 0u : S->prefix;
    const u32 need = (u32)nrem[0] - below;  // >= 1: the key sought is among those counted
    u32 c[PER], sum = 0, tot;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        c[j] = S->hist[t * PER + j];
        S->hist[t * PER + j] = 0;
        sum += c[j];
    }
    u32 run = prim::block_exclusive_scan(sum, smem, tot);
    if (run < need && need <= run + sum) {  // (exactly one thread, as tot >= need)
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            if (run < need && need <= run + c[j]) {
                S->prefix = (prefix << select_bits(PASS)) | (u32)(t * PER + j);
                S->below = below + run;
                if (PASS == 2) S->keep = need - run;
            }
            run += c[j];
        }
    }
}

struct SelectTiePred {
    const u32* tcost;
    const SelectState* S;
    __device__ bool operator()(int i) const { return tcost[i] == S->prefix; }
};

// Called for every gathered pair i; `tie`: its key is the threshold key, and `pos` pairs with that key
// come before it in edge order.  The key's slot then holds the flag (1 = give the pair up).
struct SelectFlagOut {
    static constexpr bool WAVE_WIDE = true;
    u32* tcost;
    const SelectState* S;
    __device__ void wave(int i, bool in_range, bool tie, int pos) const {
        if (!in_range) return;
        const u32 k = tcost[i];
        tcost[i] = (k > S->prefix || (tie && (u32)pos >= S->keep)) ? 1u : 0u;
    }
};

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
                                                              const int* __restrict__ nrem, u64* __restrict__ abid,
                                                              const int* __restrict__ guard) {
    if (guard && *guard == 0) return;  // (as in trunc_block_kernel)
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
// Also written to host memory (`host_out`), which the host reads once `done` tells it to.
__global__ __launch_bounds__(BLOCK) void absorb_count_kernel(const int* __restrict__ list, const State* st,
                                                             const u64* __restrict__ ekey, int vbits, int B,
                                                             const int* __restrict__ voff, int* __restrict__ acand,
                                                             int* __restrict__ host_out, HostSignal done) {
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
    signal_host(done, threadIdx.x, (int)threadIdx.x < B);
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
                                                         const u64* __restrict__ akey, int vbits,
                                                         const int* __restrict__ guard) {
    if (guard && *guard == 0) return;  // queued ahead of the host's look, and the selection was not finished
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

// Where a triple's search of the table starts: the table follows the vertex numbering (the triple's
// smallest vertex x, scaled from the round's new vertex count to the number of slots; the same x always
// gives the same place, which is all the table needs), plus a few bits of the triple's hash.
// Facets that are neighbours in the mesh are neighbours in the facet list and have nearby smallest
// vertices, so the lanes that handle them meet in the same cache lines of the table, where a uniform
// hash would fetch, and later write back, a whole line for nearly every facet (and the keep test
// that follows reads the table the same way).  Measured at 1.2 M vertices: 3 hash bits are best; with
// none the facets of one vertex collide, with 6 or 9 the lines are shared by fewer facets.
constexpr int FACET_HOME_WINDOW_BITS = 3;
constexpr int FACET_HOME_PROBES = 8;
__device__ __forceinline__ u32 facet_home(int x, u32 hx, float slots_per_vertex) {
    const float at = (float)x * slots_per_vertex;  // (below 2^32: x is below the vertex count)
    return (u32)at + (hx & ((1u << FACET_HOME_WINDOW_BITS) - 1u));
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
                                                             int* __restrict__ fslot, const int* __restrict__ guard) {
    if (guard && *guard == 0) return;  // (as in contract_kernel)
    const int nf = st->nf[cur];
    const int stride = gridDim.x * BLOCK;
    const int g = blockIdx.x * BLOCK + threadIdx.x;
    const int nv_new = st->nv[cur ^ 1];  // (the renumbering before this kernel has left the count there)
    const float slots_per_vertex = ((float)hmask + 1.0f) / (float)(nv_new > 0 ? nv_new : 1);
    // (the label of this thread's first original vertex is asked for now, so that it arrives while the
    // facet is being worked on; it is composed with the new numbering at the end)
    const int first_label = g < n_orig ? cid[g] : 0;
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
        const u32 hx = hash3(x, y, z);
        u32 h = facet_home(x, hx, slots_per_vertex) & hmask;
        for (int probe = 1;; ++probe) {
            const int old = atomicCAS(&htab[h], -1, f);
            if (old == -1) break;
            if (old == f) break;
            int p = vmap[fcur[3 * (size_t)old]], q = vmap[fcur[3 * (size_t)old + 1]], r = vmap[fcur[3 * (size_t)old + 2]];
            sort3(p, q, r);
            if (p == x && q == y && r == z) {
                atomicMin(&htab[h], f);
                break;
            }
            // a few steps along the line, then (a crowded stretch: a vertex with very many facets) on from
            // a place that the whole triple decides
            h = (probe == FACET_HOME_PROBES ? hx : h + 1u) & hmask;
        }
        fslot[f] = (int)h;
    }
    if (g < n_orig) cid[g] = vmap[first_label];
    for (int o = g + stride; o < n_orig; o += stride) cid[o] = vmap[cid[o]];
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
// The call's last kernel, one workgroup: the header's first n ints ([State][matched][foff_out])
// copied to the host's read-back area, then the host is told.
__global__ __launch_bounds__(BLOCK) void publish_header_kernel(int* __restrict__ hdr, int n,
                                                               int* __restrict__ host_img, HostSignal done) {
    for (int i = threadIdx.x; i < n; i += BLOCK) host_img[i] = hdr[i];
    // (the error flags are zero between calls: a single mesh's next call does not upload a header)
    if (threadIdx.x == 0) hdr[offsetof(State, err) / sizeof(int)] = 0;
    signal_host(done, threadIdx.x, (int)threadIdx.x < n);
}

// Degenerated vertices (option): ref[v] = 1 for every vertex that a facet of the final mesh refers to
// (ref is cleared beforehand; all writers store the same value).
__global__ __launch_bounds__(BLOCK) void mark_referenced_kernel(const int* __restrict__ fcur, const State* st, int cur,
                                                                int* __restrict__ ref) {
    const long long n = 3ll * st->nf[cur];
    for (long long i = (long long)blockIdx.x * BLOCK + threadIdx.x; i < n; i += (long long)gridDim.x * BLOCK) ref[fcur[i]] = 1;
}

struct RefPred {
    const int* ref;
    __device__ bool operator()(int v) const { return ref[v] != 0; }
};

// newid[v] = number of referenced vertices in front of v, for EVERY vertex (so that the count in front
// of a mesh's first vertex can be read off as well)
struct RefOut {
    static constexpr bool WAVE_WIDE = true;
    int* newid;
    __device__ void wave(int v, bool in_range, bool flagged, int pos) const {
        (void)flagged;
        if (in_range) newid[v] = pos;
    }
};

// DROP: only the vertices with ref[v] != 0 go out, at newid[v]; facets and cluster ids follow that
// numbering, cluster ids of dropped vertices become -1, and kept_per_mesh[b] receives mesh b's count.
template <bool DROP>
__global__ __launch_bounds__(BLOCK) void copy_out_kernel(const VRec* __restrict__ vrec, const int* __restrict__ fcur,
                                                         const int* __restrict__ cid, const State* st, int cur,
                                                         int n_orig, float* __restrict__ verts_out,
                                                         int* __restrict__ facets_out, int* __restrict__ cid_out,
                                                         int B, const int* __restrict__ voff,
                                                         int* __restrict__ foff_out, const int* __restrict__ ref,
                                                         const int* __restrict__ newid,
                                                         int* __restrict__ kept_per_mesh) {
    const int nv = st->nv[cur], nf = st->nf[cur];
    const int stride = gridDim.x * BLOCK;
    const int g = blockIdx.x * BLOCK + threadIdx.x;
    for (int w = g; w < nv; w += stride) {
        if (DROP && !ref[w]) continue;
        const int o = DROP ? newid[w] : w;
        const float4 p = *reinterpret_cast<const float4*>(&vrec[w]);
        verts_out[3 * (size_t)o] = p.x;
        verts_out[3 * (size_t)o + 1] = p.y;
        verts_out[3 * (size_t)o + 2] = p.z;
    }
    for (long long i = g; i < 3ll * nf; i += stride) facets_out[i] = DROP ? newid[fcur[i]] : fcur[i];
    for (int o = g; o < n_orig; o += stride) {
        const int c = cid[o];
        cid_out[o] = DROP ? (ref[c] ? newid[c] : -1) : c;
    }
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
        if (DROP && b < B) {
            const int before = voff[b] < nv ? newid[voff[b]] : st->nv_kept;
            const int upto = voff[b + 1] < nv ? newid[voff[b + 1]] : st->nv_kept;
            kept_per_mesh[b] = upto - before;
        }
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

}  // namespace
