// picasso_conv_oracle.cpp -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
//
// Plain fp64 statements of the mesh convolutions of the Picasso paper
// (Sec. 4 "Mesh Convolution": vertex2facet with barycentric interpolation, its
// facet2facet variant for textured meshes, facet2vertex with Gaussian-mixture
// fuzzy coefficients; supplementary section
// "Backward propagations of different convolutions"), in their depth-wise
// form: one filter weight per channel (Sec. 4, last paragraph splits every
// convolution into a depth-wise and a channel-wise operation; the channel-wise
// one is an ordinary dense product and is not part of this file).  Written as
// the paper's formulas, loop by loop; shares nothing with the HIP library.
//
// Readings where the paper is silent or garbled:
//  * Interpolated points of a facet with level k >= 1 (Eq. "interpolate_num",
//    K = k (k + 1) / 2): the triangular lattice with k points per side,
//    barycentric coordinates (i, j, l) / (k - 1), i + j + l = k - 1, which
//    contains the three vertices (Fig. "v2v_conv" (a): "original and
//    interpolated points"); for k = 1 the single point is the centroid.
//  * The level formula is taken as printed, k = floor((A - A_min) / (A_max -
//    A_min)) * alpha + beta, the ratio being 0 when all areas are equal.
//    With the paper's alpha = beta = 1 a reading with alpha inside the floor
//    gives the same levels.  A_min, A_max run over the facets of one mesh.
//  * N(v) counts a facet once per corner at v (a facet that lists v twice
//    counts twice); a vertex without facets gets the zero feature.
//  * Fuzzy coefficients use the homogeneous diagonal covariance of the
//    paper's experiments: z_it = |n_i - mu_t|^2 / sigma_t^2, passed as
//    inv_var[t] = 1 / sigma_t^2.
//  * Backward passes: the supplementary's partial derivatives, chained with
//    the incoming gradient and summed over everything a quantity feeds;
//    d/d pi is added (needed when the covariances are learnable).
//
// Pins: tests/test_conv_oracle_pins.py.
#include <cmath>
#include <cstdint>
#include <vector>

namespace {
constexpr int OK = 0, ERR_INVALID_ARG = -1, ERR_BAD_INDEX = -2;

// barycentric coordinates of the K = k (k + 1) / 2 interpolated points of level k
void lattice(int k, std::vector<double>& xi) {
    xi.clear();
    if (k <= 1) {
        xi = {1.0 / 3.0, 1.0 / 3.0, 1.0 / 3.0};
        return;
    }
    for (int i = 0; i <= k - 1; ++i)
        for (int j = 0; i + j <= k - 1; ++j) {
            const int l = k - 1 - i - j;
            xi.push_back((double)i / (k - 1));
            xi.push_back((double)j / (k - 1));
            xi.push_back((double)l / (k - 1));
        }
}

int check_facets(const int32_t* facets, int32_t F, int32_t N) {
    for (int64_t i = 0; i < 3 * (int64_t)F; ++i)
        if (facets[i] < 0 || facets[i] >= N) return ERR_BAD_INDEX;
    return OK;
}
}  // namespace

extern "C" {

// Unit normal and area of every facet (Sec. 4, first paragraph); a facet of zero
// area gets the zero normal.  The area decides an integer (the level below), so
// this is computed in binary32, every operation rounded once, in the order
// written -- the precision and order the kernel uses.
int picasso_oracle_facet_geometry(const float* verts, int32_t N, const int32_t* facets, int32_t F, float* normals,
                                  float* areas) {
    if (!verts || !facets || !normals || !areas) return ERR_INVALID_ARG;
    if (check_facets(facets, F, N) != OK) return ERR_BAD_INDEX;
    for (int f = 0; f < F; ++f) {
        const float* p0 = verts + 3 * (size_t)facets[3 * f];
        const float* p1 = verts + 3 * (size_t)facets[3 * f + 1];
        const float* p2 = verts + 3 * (size_t)facets[3 * f + 2];
        const float ax = p1[0] - p0[0], ay = p1[1] - p0[1], az = p1[2] - p0[2];
        const float bx = p2[0] - p0[0], by = p2[1] - p0[1], bz = p2[2] - p0[2];
        const float nx = ay * bz - az * by;
        const float ny = az * bx - ax * bz;
        const float nz = ax * by - ay * bx;
        const float len = std::sqrt((nx * nx + ny * ny) + nz * nz);
        areas[f] = 0.5f * len;
        normals[3 * (size_t)f] = len > 0.0f ? nx / len : 0.0f;
        normals[3 * (size_t)f + 1] = len > 0.0f ? ny / len : 0.0f;
        normals[3 * (size_t)f + 2] = len > 0.0f ? nz / len : 0.0f;
    }
    return OK;
}

// Eq. "interpolate_num": level k of every facet from its area; foff[B+1] = facet
// offsets of the meshes of a batch (A_min, A_max are per mesh).  binary32 as above.
int picasso_oracle_facet_levels(const float* areas, int32_t B, const int32_t* foff, int32_t alpha, int32_t beta,
                                int32_t* level) {
    if (!areas || !foff || !level || B < 1 || alpha < 0 || beta < 1) return ERR_INVALID_ARG;
    for (int b = 0; b < B; ++b) {
        float amin = INFINITY, amax = -INFINITY;
        for (int f = foff[b]; f < foff[b + 1]; ++f) {
            if (areas[f] < amin) amin = areas[f];
            if (areas[f] > amax) amax = areas[f];
        }
        for (int f = foff[b]; f < foff[b + 1]; ++f) {
            const float ratio = amax > amin ? (areas[f] - amin) / (amax - amin) : 0.0f;
            level[f] = (int)std::floor(ratio) * alpha + beta;
        }
    }
    return OK;
}

// Fuzzy coefficients pi[F,T] of the facets from their normals (Sec. 4.2, the two
// equations for z_it and pi_it).
int picasso_oracle_fuzzy(const float* normals, int32_t F, const float* mu, const float* inv_var, int32_t T,
                         double* pi) {
    if (!normals || !mu || !inv_var || !pi || T < 1) return ERR_INVALID_ARG;
    std::vector<double> e(T);
    for (int f = 0; f < F; ++f) {
        double sum = 0.0;
        for (int t = 0; t < T; ++t) {
            double z = 0.0;
            for (int k = 0; k < 3; ++k) {
                const double d = (double)normals[3 * (size_t)f + k] - (double)mu[3 * t + k];
                z += d * d * (double)inv_var[t];
            }
            e[t] = std::exp(-z);
            sum += e[t];
        }
        for (int t = 0; t < T; ++t) pi[(size_t)f * T + t] = e[t] / sum;
    }
    return OK;
}

// Vertex2facet, depth-wise (Sec. 4.1): I_k = sum_s xi_ks I_s, W_k = sum_s xi_ks w_s,
// J = (1 / K) sum_k W_k I_k, per channel.  x [N,C], w [3,C], level [F], y [F,C].
int picasso_oracle_v2f_forward(const float* x, int32_t N, int32_t C, const int32_t* facets, int32_t F,
                               const int32_t* level, const float* w, double* y) {
    if (!x || !facets || !level || !w || !y || C < 1) return ERR_INVALID_ARG;
    if (check_facets(facets, F, N) != OK) return ERR_BAD_INDEX;
    std::vector<double> xi;
    for (int f = 0; f < F; ++f) {
        if (level[f] < 1) return ERR_INVALID_ARG;
        lattice(level[f], xi);
        const int K = (int)xi.size() / 3;
        for (int c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) {
                double Ik = 0.0, Wk = 0.0;
                for (int s = 0; s < 3; ++s) {
                    Ik += xi[3 * k + s] * (double)x[(size_t)facets[3 * f + s] * C + c];
                    Wk += xi[3 * k + s] * (double)w[s * C + c];
                }
                acc += Wk * Ik;
            }
            y[(size_t)f * C + c] = acc / K;
        }
    }
    return OK;
}

// Its backward pass (supplementary, vertex2facet kernel): dJ/dI_s = (1/K) sum_k
// xi_ks W_k, dJ/dw_s = (1/K) sum_k xi_ks I_k.  gy [F,C] in, gx [N,C] and gw [3,C] out.
int picasso_oracle_v2f_backward(const float* gy, const float* x, int32_t N, int32_t C, const int32_t* facets,
                                int32_t F, const int32_t* level, const float* w, double* gx, double* gw) {
    if (!gy || !x || !facets || !level || !w || !gx || !gw || C < 1) return ERR_INVALID_ARG;
    if (check_facets(facets, F, N) != OK) return ERR_BAD_INDEX;
    for (size_t i = 0; i < (size_t)N * C; ++i) gx[i] = 0.0;
    for (int i = 0; i < 3 * C; ++i) gw[i] = 0.0;
    std::vector<double> xi;
    for (int f = 0; f < F; ++f) {
        if (level[f] < 1) return ERR_INVALID_ARG;
        lattice(level[f], xi);
        const int K = (int)xi.size() / 3;
        for (int c = 0; c < C; ++c) {
            const double g = gy[(size_t)f * C + c];
            for (int s = 0; s < 3; ++s) {
                double dI = 0.0, dw = 0.0;
                for (int k = 0; k < K; ++k) {
                    double Ik = 0.0, Wk = 0.0;
                    for (int r = 0; r < 3; ++r) {
                        Ik += xi[3 * k + r] * (double)x[(size_t)facets[3 * f + r] * C + c];
                        Wk += xi[3 * k + r] * (double)w[r * C + c];
                    }
                    dI += xi[3 * k + s] * Wk;
                    dw += xi[3 * k + s] * Ik;
                }
                gx[(size_t)facets[3 * f + s] * C + c] += g * dI / K;
                gw[s * C + c] += g * dw / K;
            }
        }
    }
    return OK;
}

// Facet2vertex, depth-wise (Sec. 4.2, last equation): I_v = (1 / |N(v)|) sum_{f in
// N(v)} (sum_t pi_ft w_t) J_f per channel.  y [F,C], pi [F,T], w [T,C], x [N,C].
int picasso_oracle_f2v_forward(const float* y, int32_t F, int32_t C, const float* pi, int32_t T, const float* w,
                               const int32_t* facets, int32_t N, double* x) {
    if (!y || !pi || !w || !facets || !x || C < 1 || T < 1) return ERR_INVALID_ARG;
    if (check_facets(facets, F, N) != OK) return ERR_BAD_INDEX;
    std::vector<int> deg(N, 0);
    for (size_t i = 0; i < (size_t)N * C; ++i) x[i] = 0.0;
    for (int f = 0; f < F; ++f)
        for (int s = 0; s < 3; ++s) {
            const int v = facets[3 * f + s];
            ++deg[v];
            for (int c = 0; c < C; ++c) {
                double coef = 0.0;
                for (int t = 0; t < T; ++t) coef += (double)pi[(size_t)f * T + t] * (double)w[t * C + c];
                x[(size_t)v * C + c] += coef * (double)y[(size_t)f * C + c];
            }
        }
    for (int v = 0; v < N; ++v)
        if (deg[v] > 0)
            for (int c = 0; c < C; ++c) x[(size_t)v * C + c] /= deg[v];
    return OK;
}

// Its backward pass (supplementary, facet2vertex kernel): dI_v/dJ_f = coef_f / |N(v)|,
// dI_v/dw_t = (1 / |N(v)|) sum_f pi_ft J_f; and dI_v/dpi_ft = w_t J_f / |N(v)|.
// gx [N,C] in; gy [F,C], gw [T,C], gpi [F,T] (may be null) out.
int picasso_oracle_f2v_backward(const float* gx, const float* y, int32_t F, int32_t C, const float* pi, int32_t T,
                                const float* w, const int32_t* facets, int32_t N, double* gy, double* gw,
                                double* gpi) {
    if (!gx || !y || !pi || !w || !facets || !gy || !gw || C < 1 || T < 1) return ERR_INVALID_ARG;
    if (check_facets(facets, F, N) != OK) return ERR_BAD_INDEX;
    std::vector<int> deg(N, 0);
    for (int64_t i = 0; i < 3 * (int64_t)F; ++i) ++deg[facets[i]];
    for (size_t i = 0; i < (size_t)F * C; ++i) gy[i] = 0.0;
    for (int i = 0; i < T * C; ++i) gw[i] = 0.0;
    if (gpi)
        for (size_t i = 0; i < (size_t)F * T; ++i) gpi[i] = 0.0;
    for (int f = 0; f < F; ++f)
        for (int s = 0; s < 3; ++s) {
            const int v = facets[3 * f + s];
            for (int c = 0; c < C; ++c) {
                const double g = (double)gx[(size_t)v * C + c] / deg[v];
                double coef = 0.0;
                for (int t = 0; t < T; ++t) coef += (double)pi[(size_t)f * T + t] * (double)w[t * C + c];
                gy[(size_t)f * C + c] += g * coef;
                for (int t = 0; t < T; ++t) {
                    gw[t * C + c] += g * (double)pi[(size_t)f * T + t] * (double)y[(size_t)f * C + c];
                    if (gpi) gpi[(size_t)f * T + t] += g * (double)w[t * C + c] * (double)y[(size_t)f * C + c];
                }
            }
        }
    return OK;
}

// Facet2facet, depth-wise (Sec. 4.1, paragraph "Facet2Facet convolution"): every facet
// carries Gamma_f texture points with features of their own, so only the filter is
// interpolated: W_k = sum_s xi_ks w_s at the point's barycentric coordinates, and
// J_f = (1 / Gamma_f) sum_k W_k T_k as in the vertex2facet equation.  tex [P,C], bary [P,3],
// poff [F+1] (points of facet f = poff[f] .. poff[f+1]), w [3,C], y [F,C]; a facet without
// points gets 0.  The coordinates come with the rendered mesh (the paper does not say how
// the points are placed).
int picasso_oracle_f2f_forward(const float* tex, const float* bary, const int32_t* poff, int32_t F, int32_t C,
                               const float* w, double* y) {
    if (!tex || !bary || !poff || !w || !y || C < 1) return ERR_INVALID_ARG;
    for (int f = 0; f < F; ++f) {
        const int g = poff[f + 1] - poff[f];
        if (g < 0) return ERR_INVALID_ARG;
        for (int c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int k = poff[f]; k < poff[f + 1]; ++k) {
                double Wk = 0.0;
                for (int s = 0; s < 3; ++s) Wk += (double)bary[3 * (size_t)k + s] * (double)w[s * C + c];
                acc += Wk * (double)tex[(size_t)k * C + c];
            }
            y[(size_t)f * C + c] = g > 0 ? acc / g : 0.0;
        }
    }
    return OK;
}

// Its backward pass (the supplementary notes that it mirrors the vertex2facet one):
// dJ/dT_k = W_k / Gamma, dJ/dw_s = (1 / Gamma) sum_k xi_ks T_k.  gtex [P,C], gw [3,C].
int picasso_oracle_f2f_backward(const float* gy, const float* tex, const float* bary, const int32_t* poff, int32_t F,
                                int32_t C, const float* w, double* gtex, double* gw) {
    if (!gy || !tex || !bary || !poff || !w || !gtex || !gw || C < 1) return ERR_INVALID_ARG;
    for (int i = 0; i < 3 * C; ++i) gw[i] = 0.0;
    for (int f = 0; f < F; ++f) {
        const int g = poff[f + 1] - poff[f];
        if (g < 0) return ERR_INVALID_ARG;
        for (int k = poff[f]; k < poff[f + 1]; ++k)
            for (int c = 0; c < C; ++c) {
                double Wk = 0.0;
                for (int s = 0; s < 3; ++s) Wk += (double)bary[3 * (size_t)k + s] * (double)w[s * C + c];
                gtex[(size_t)k * C + c] = (double)gy[(size_t)f * C + c] * Wk / g;
                for (int s = 0; s < 3; ++s)
                    gw[s * C + c] += (double)gy[(size_t)f * C + c] * (double)bary[3 * (size_t)k + s] *
                                     (double)tex[(size_t)k * C + c] / g;
            }
    }
    return OK;
}

// Corners of the facet array at every vertex, ascending: offsets [N+1], corners [3F]
// (corner i = 3 f + s is vertex facets[i]).
int picasso_oracle_vertex_corner_csr(const int32_t* facets, int32_t F, int32_t N, int32_t* offsets, int32_t* corners) {
    if (!facets || !offsets || !corners) return ERR_INVALID_ARG;
    if (check_facets(facets, F, N) != OK) return ERR_BAD_INDEX;
    for (int v = 0; v <= N; ++v) offsets[v] = 0;
    for (int64_t i = 0; i < 3 * (int64_t)F; ++i) ++offsets[facets[i] + 1];
    for (int v = 0; v < N; ++v) offsets[v + 1] += offsets[v];
    std::vector<int32_t> fill(offsets, offsets + N);
    for (int64_t i = 0; i < 3 * (int64_t)F; ++i) corners[fill[facets[i]]++] = (int32_t)i;
    return OK;
}

}  // extern "C"
