// pooling.h -- pooling and unpooling over the vertex clusters recorded by the
// decimation (Picasso paper, Sec. 3, paragraph "Pooling and unpooling").
//
// Features are fp32 [N, C] row-major.  A cluster's members are visited in
// ascending vertex order (CSR built by a stable sort of (cluster_id, vertex)),
// every sum is a left-to-right fp32 sum in that order and there are no fp
// atomics, so results do not depend on scheduling.  One lane owns VEC
// consecutive channels of one cluster (or of one vertex), so neighbouring
// lanes read neighbouring addresses of the same feature row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#pragma clang fp contract(off)

namespace pool {

constexpr int BLOCK = 256;
enum Mode { AVG = 0, MAX = 1, WEIGHTED = 2, SUM = 3 };

template <int VEC>
struct Pack {
    float v[VEC];
};

template <int VEC>
__device__ __forceinline__ Pack<VEC> load_pack(const float* __restrict__ p) {
    Pack<VEC> r;
    if (VEC == 4) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        r.v[0] = t.x; r.v[1 % VEC] = t.y; r.v[2 % VEC] = t.z; r.v[3 % VEC] = t.w;
    } else if (VEC == 8) {
        const float4 t = *reinterpret_cast<const float4*>(p), u = *reinterpret_cast<const float4*>(p + 4);
        r.v[0] = t.x; r.v[1 % VEC] = t.y; r.v[2 % VEC] = t.z; r.v[3 % VEC] = t.w;
        r.v[4 % VEC] = u.x; r.v[5 % VEC] = u.y; r.v[6 % VEC] = u.z; r.v[7 % VEC] = u.w;
    } else {
#pragma unroll
        for (int k = 0; k < VEC; ++k) r.v[k] = p[k];
    }
    return r;
}

template <int VEC>
__device__ __forceinline__ void store_pack(float* __restrict__ p, const Pack<VEC>& r) {
    if (VEC == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(r.v[0], r.v[1 % VEC], r.v[2 % VEC], r.v[3 % VEC]);
    } else if (VEC == 8) {
        *reinterpret_cast<float4*>(p) = make_float4(r.v[0], r.v[1 % VEC], r.v[2 % VEC], r.v[3 % VEC]);
        *reinterpret_cast<float4*>(p + 4) = make_float4(r.v[4 % VEC], r.v[5 % VEC], r.v[6 % VEC], r.v[7 % VEC]);
    } else {
#pragma unroll
        for (int k = 0; k < VEC; ++k) p[k] = r.v[k];
    }
}

// y[c] = pooled feature of cluster c.  MAX also writes the first member that attains the maximum.
template <int MODE, int VEC>
__global__ __launch_bounds__(BLOCK) void pool_forward_kernel(const float* __restrict__ x, int C,
                                                             const int* __restrict__ off,
                                                             const int* __restrict__ mem, int n_out,
                                                             const float* __restrict__ w, float* __restrict__ y,
                                                             int* __restrict__ argmax) {
    const int Q = C / VEC;
    const long long idx = (long long)blockIdx.x * BLOCK + threadIdx.x;
    const int c = (int)(idx / Q), q = (int)(idx % Q);
    if (c >= n_out) return;
    const int s = off[c], e = off[c + 1];
    Pack<VEC> acc;
    int arg[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        acc.v[k] = 0.0f;
        arg[k] = -1;
    }
    float wsum = 0.0f;
    for (int m = s; m < e; ++m) {
        const int v = mem[m];
        const Pack<VEC> xv = load_pack<VEC>(x + (size_t)v * C + (size_t)q * VEC);
        if (MODE == MAX) {
#pragma unroll
            for (int k = 0; k < VEC; ++k)
                if (m == s || xv.v[k] > acc.v[k]) {
                    acc.v[k] = xv.v[k];
                    arg[k] = v;
                }
        } else if (MODE == WEIGHTED) {
            const float wv = w[v];
#pragma unroll
            for (int k = 0; k < VEC; ++k) acc.v[k] = acc.v[k] + wv * xv.v[k];
            wsum = wsum + wv;
        } else {
#pragma unroll
            for (int k = 0; k < VEC; ++k) acc.v[k] = acc.v[k] + xv.v[k];
        }
    }
    if (MODE == AVG) {
        const float n = (float)(e - s);
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc.v[k] = (e > s) ? acc.v[k] / n : 0.0f;
    }
    if (MODE == WEIGHTED) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc.v[k] = (wsum != 0.0f) ? acc.v[k] / wsum : 0.0f;
    }
    store_pack<VEC>(y + (size_t)c * C + (size_t)q * VEC, acc);
    if (MODE == MAX && argmax) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) argmax[(size_t)c * C + (size_t)q * VEC + k] = arg[k];
    }
}

// gx[v] = adjoint of the pooling applied to gy, for the features (weights are constants)
template <int MODE, int VEC>
__global__ __launch_bounds__(BLOCK) void pool_backward_kernel(const float* __restrict__ gy, int n_in, int C,
                                                              const int* __restrict__ cid,
                                                              const int* __restrict__ off,
                                                              const int* __restrict__ mem,
                                                              const float* __restrict__ w,
                                                              const int* __restrict__ argmax,
                                                              float* __restrict__ gx) {
    const int Q = C / VEC;
    const long long idx = (long long)blockIdx.x * BLOCK + threadIdx.x;
    const int v = (int)(idx / Q), q = (int)(idx % Q);
    if (v >= n_in) return;
    const int c = cid[v];
    Pack<VEC> g = load_pack<VEC>(gy + (size_t)c * C + (size_t)q * VEC);
    if (MODE == AVG) {
        const float n = (float)(off[c + 1] - off[c]);
#pragma unroll
        for (int k = 0; k < VEC; ++k) g.v[k] = g.v[k] / n;
    } else if (MODE == MAX) {
#pragma unroll
        for (int k = 0; k < VEC; ++k)
            if (argmax[(size_t)c * C + (size_t)q * VEC + k] != v) g.v[k] = 0.0f;
    } else if (MODE == WEIGHTED) {
        float wsum = 0.0f;
        for (int m = off[c]; m < off[c + 1]; ++m) wsum = wsum + w[mem[m]];
        const float wv = w[v];
#pragma unroll
        for (int k = 0; k < VEC; ++k) g.v[k] = (wsum != 0.0f) ? (g.v[k] * wv) / wsum : 0.0f;
    }
    store_pack<VEC>(gx + (size_t)v * C + (size_t)q * VEC, g);
}

// Unpooling: every vertex takes its cluster's feature.
template <int VEC>
__global__ __launch_bounds__(BLOCK) void unpool_forward_kernel(const float* __restrict__ y, int n_in, int C,
                                                               const int* __restrict__ cid, float* __restrict__ x) {
    const int Q = C / VEC;
    const long long idx = (long long)blockIdx.x * BLOCK + threadIdx.x;
    const int v = (int)(idx / Q), q = (int)(idx % Q);
    if (v >= n_in) return;
    store_pack<VEC>(x + (size_t)v * C + (size_t)q * VEC, load_pack<VEC>(y + (size_t)cid[v] * C + (size_t)q * VEC));
}

// (cluster id, vertex) pairs for the CSR sort; flags ids outside [0, n_out)
__global__ __launch_bounds__(BLOCK) void emit_cluster_pairs_kernel(const int* __restrict__ cid, int n_in, int n_out,
                                                                   uint32_t* __restrict__ key,
                                                                   uint32_t* __restrict__ val, int* __restrict__ err) {
    const int v = blockIdx.x * BLOCK + threadIdx.x;
    if (v >= n_in) return;
    int c = cid[v];
    if (c < 0 || c >= n_out) {
        atomicOr(err, 1);
        c = 0;
    }
    key[v] = (uint32_t)c;
    val[v] = (uint32_t)v;
}

// The two per-input-vertex tensors of Alg. 2's output list from cluster_id: first[c] = smallest
// member of cluster c (first pass, atomicMin: the result does not depend on order), then
// replace[v] = first[cluster_id[v]] and mapping[v] = cluster_id[v] for that member, -1 otherwise.
__global__ __launch_bounds__(BLOCK) void cluster_first_kernel(const int* __restrict__ cid, int n_in, int n_out,
                                                              int* __restrict__ first, int* __restrict__ err) {
    const int v = blockIdx.x * BLOCK + threadIdx.x;
    if (v >= n_in) return;
    const int c = cid[v];
    if (c == -1) return;  // (the vertex's cluster was dropped: nothing represents it)
    if (c < 0 || c >= n_out) {
        atomicOr(err, 1);
        return;
    }
    atomicMin(&first[c], v);
}

__global__ __launch_bounds__(BLOCK) void replace_mapping_kernel(const int* __restrict__ cid, int n_in, int n_out,
                                                                const int* __restrict__ first,
                                                                int* __restrict__ replace, int* __restrict__ mapping) {
    const int v = blockIdx.x * BLOCK + threadIdx.x;
    if (v >= n_in) return;
    const int c = cid[v];
    if (c < -1 || c >= n_out) return;  // (flagged by the first pass; the call reports it)
    const int r = c >= 0 ? first[c] : -1;
    replace[v] = r;
    mapping[v] = (c >= 0 && r == v) ? c : -1;
}

// The two kernels in front of and behind cluster_first_kernel when the table of first members is the
// library's static array (picasso_replace_mapping_static): the fill, which also clears the flag, and
// replace_mapping_kernel's work plus the status word for the caller.
__global__ __launch_bounds__(BLOCK) void static_begin_kernel(int* __restrict__ first, int n_out, int* __restrict__ flag) {
    const int i = blockIdx.x * BLOCK + threadIdx.x;
    if (i < n_out) first[i] = 0x7FFFFFFF;
    if (i == 0) *flag = 0;
}

__global__ __launch_bounds__(BLOCK) void replace_mapping_status_kernel(const int* __restrict__ cid, int n_in, int n_out,
                                                                       const int* __restrict__ first,
                                                                       const int* __restrict__ flag,
                                                                       int* __restrict__ replace, int* __restrict__ mapping,
                                                                       int* __restrict__ status, int ok, int bad) {
    const int v = blockIdx.x * BLOCK + threadIdx.x;
    if (v == 0) *status = (*flag != 0) ? bad : ok;
    if (v >= n_in) return;
    const int c = cid[v];
    if (c < -1 || c >= n_out) return;
    const int r = c >= 0 ? first[c] : -1;
    replace[v] = r;
    mapping[v] = (c >= 0 && r == v) ? c : -1;
}

inline int grid_for(long long n) { return (int)((n + BLOCK - 1) / BLOCK > 0 ? (n + BLOCK - 1) / BLOCK : 1); }

template <int VEC>
inline void launch_pool_forward(hipStream_t s, int mode, const float* x, int C, const int* off, const int* mem,
                                int n_out, const float* w, float* y, int* argmax) {
    const int g = grid_for((long long)n_out * (C / VEC));
    switch (mode) {
        case AVG: pool_forward_kernel<AVG, VEC><<<g, BLOCK, 0, s>>>(x, C, off, mem, n_out, w, y, argmax); break;
        case MAX: pool_forward_kernel<MAX, VEC><<<g, BLOCK, 0, s>>>(x, C, off, mem, n_out, w, y, argmax); break;
        case WEIGHTED: pool_forward_kernel<WEIGHTED, VEC><<<g, BLOCK, 0, s>>>(x, C, off, mem, n_out, w, y, argmax); break;
        default: pool_forward_kernel<SUM, VEC><<<g, BLOCK, 0, s>>>(x, C, off, mem, n_out, w, y, argmax); break;
    }
}

template <int VEC>
inline void launch_pool_backward(hipStream_t s, int mode, const float* gy, int n_in, int C, const int* cid,
                                 const int* off, const int* mem, const float* w, const int* argmax, float* gx) {
    const int g = grid_for((long long)n_in * (C / VEC));
    switch (mode) {
        case AVG: pool_backward_kernel<AVG, VEC><<<g, BLOCK, 0, s>>>(gy, n_in, C, cid, off, mem, w, argmax, gx); break;
        case MAX: pool_backward_kernel<MAX, VEC><<<g, BLOCK, 0, s>>>(gy, n_in, C, cid, off, mem, w, argmax, gx); break;
        case WEIGHTED:
            pool_backward_kernel<WEIGHTED, VEC><<<g, BLOCK, 0, s>>>(gy, n_in, C, cid, off, mem, w, argmax, gx);
            break;
        default: pool_backward_kernel<SUM, VEC><<<g, BLOCK, 0, s>>>(gy, n_in, C, cid, off, mem, w, argmax, gx); break;
    }
}

}  // namespace pool
