// picasso_pool_oracle.cpp -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
//
// Plain definitions of pooling and unpooling over the vertex clusters that
// the decimation records (Picasso paper, Sec. 3, paragraph "Pooling and
// unpooling": the clusters are the neighbourhoods; sum, average, max and
// weighted poolings; unpooling gives every vertex of a cluster the feature of
// the cluster's representative).  fp64 accumulation, written out as the
// definitions; it shares nothing with the HIP library.
//
// Readings where the paper gives no formula:
//  * weighted pooling = sum_v w_v x_v / sum_v w_v over the cluster (0 when the
//    weights of a cluster sum to 0);
//  * max pooling returns, per channel, the largest member value and the
//    lowest-index member that attains it; its backward pass routes the
//    gradient to that member only;
//  * backward passes are the adjoints of the forward passes with respect to
//    the features (the weights of weighted pooling are treated as constants);
//  * a cluster without members (cannot come out of the decimation) pools to 0.
//
// Pins: tests/test_pool_oracle_pins.py (hand-worked fixture, closed forms,
// adjointness of every backward pass against its forward pass, finite
// differences).
#include <cstdint>
#include <cstring>
#include <vector>

namespace {
constexpr int OK = 0, ERR_INVALID_ARG = -1, ERR_BAD_INDEX = -2;
enum { POOL_AVG = 0, POOL_MAX = 1, POOL_WEIGHTED = 2, POOL_SUM = 3 };

int check(const int32_t* cid, int n_in, int n_out, int C) {
    if (!cid || n_in < 0 || n_out < 0 || C < 1) return ERR_INVALID_ARG;
    for (int v = 0; v < n_in; ++v)
        if (cid[v] < 0 || cid[v] >= n_out) return ERR_BAD_INDEX;
    return OK;
}
}  // namespace

extern "C" {

// y [n_out, C]; argmax [n_out, C] (max pooling only, may be null): member index or -1.
int picasso_oracle_pool_forward(int mode, const float* x, int32_t n_in, int32_t C, const int32_t* cid, int32_t n_out,
                                const float* w, float* y, int32_t* argmax) {
    int st = check(cid, n_in, n_out, C);
    if (st != OK) return st;
    if (!x || !y || (mode == POOL_WEIGHTED && !w)) return ERR_INVALID_ARG;
    std::vector<double> acc((size_t)n_out * C, 0.0), wsum(n_out, 0.0);
    std::vector<int32_t> cnt(n_out, 0), arg((size_t)n_out * C, -1);
    for (int v = 0; v < n_in; ++v) {  // ascending member order
        const int c = cid[v];
        for (int k = 0; k < C; ++k) {
            const double xv = x[(size_t)v * C + k];
            double& a = acc[(size_t)c * C + k];
            if (mode == POOL_MAX) {
                if (cnt[c] == 0 || xv > a) {
                    a = xv;
                    arg[(size_t)c * C + k] = v;
                }
            } else if (mode == POOL_WEIGHTED) {
                a += (double)w[v] * xv;
            } else {
                a += xv;
            }
        }
        cnt[c] += 1;
        if (mode == POOL_WEIGHTED) wsum[c] += (double)w[v];
    }
    for (int c = 0; c < n_out; ++c)
        for (int k = 0; k < C; ++k) {
            double a = acc[(size_t)c * C + k];
            if (mode == POOL_AVG) a = cnt[c] ? a / cnt[c] : 0.0;
            if (mode == POOL_WEIGHTED) a = wsum[c] != 0.0 ? a / wsum[c] : 0.0;
            y[(size_t)c * C + k] = (float)a;
        }
    if (argmax && mode == POOL_MAX) std::memcpy(argmax, arg.data(), arg.size() * sizeof(int32_t));
    return OK;
}

// gx [n_in, C] = adjoint of the forward pass applied to gy [n_out, C].
int picasso_oracle_pool_backward(int mode, const float* gy, int32_t n_in, int32_t C, const int32_t* cid, int32_t n_out,
                                 const float* w, const int32_t* argmax, float* gx) {
    int st = check(cid, n_in, n_out, C);
    if (st != OK) return st;
    if (!gy || !gx || (mode == POOL_WEIGHTED && !w) || (mode == POOL_MAX && !argmax)) return ERR_INVALID_ARG;
    std::vector<double> wsum(n_out, 0.0);
    std::vector<int32_t> cnt(n_out, 0);
    for (int v = 0; v < n_in; ++v) {
        cnt[cid[v]] += 1;
        if (mode == POOL_WEIGHTED) wsum[cid[v]] += (double)w[v];
    }
    for (int v = 0; v < n_in; ++v) {
        const int c = cid[v];
        for (int k = 0; k < C; ++k) {
            const double g = gy[(size_t)c * C + k];
            double r;
            switch (mode) {
                case POOL_AVG: r = g / cnt[c]; break;
                case POOL_MAX: r = (argmax[(size_t)c * C + k] == v) ? g : 0.0; break;
                case POOL_WEIGHTED: r = wsum[c] != 0.0 ? g * (double)w[v] / wsum[c] : 0.0; break;
                default: r = g; break;
            }
            gx[(size_t)v * C + k] = (float)r;
        }
    }
    return OK;
}

// Unpooling: every vertex takes the feature of its cluster.
int picasso_oracle_unpool_forward(const float* y, int32_t n_in, int32_t C, const int32_t* cid, int32_t n_out, float* x) {
    int st = check(cid, n_in, n_out, C);
    if (st != OK) return st;
    if (!y || !x) return ERR_INVALID_ARG;
    for (int v = 0; v < n_in; ++v)
        for (int k = 0; k < C; ++k) x[(size_t)v * C + k] = y[(size_t)cid[v] * C + k];
    return OK;
}

// Its adjoint: the gradients of a cluster's vertices add up.
int picasso_oracle_unpool_backward(const float* gx, int32_t n_in, int32_t C, const int32_t* cid, int32_t n_out,
                                   float* gy) {
    return picasso_oracle_pool_forward(POOL_SUM, gx, n_in, C, cid, n_out, nullptr, gy, nullptr);
}

}  // extern "C"
