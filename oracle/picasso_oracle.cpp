// picasso_oracle.cpp -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
//
// A plain, slow, single-threaded CPU statement of the round-based QEM mesh
// decimation of the Picasso paper (Sec. 3, Algorithm 2 "Fast GPU-accelerated
// mesh simplification"; supplementary section "Quadric error computation").
// It exists so that the HIP path can be compared against something written
// directly from the paper.  Only tests, the smoke check and the benchmark's
// cpu_baseline leg may call it.  It shares no code, header, table or helper
// with the HIP library.
//
// Build:  g++ -O2 -std=c++17 -ffp-contract=off -fPIC -shared
// (no fast-math, no FMA contraction: every + - * / sqrt below is one IEEE
//  binary32 operation rounded to nearest-even, in the order written).
//
// Readings of the paper taken here (the paper is silent or ambiguous on them):
//  * Alg. 2 line 11 (absorbing un-paired vertices into a neighbouring cluster)
//    is not applied: a round contracts disjoint vertex PAIRS only, so that the
//    vertex budget of lines 4-8 is met exactly.
//  * Several runs of the core algorithm (Sec. 3: "running the core algorithm
//    multiple times") carry the accumulated quadrics forward,
//    Q_C = sum of member vertex quadrics (supplementary, cluster quadric eq.);
//    facet quadrics are computed once from the input mesh.
//  * Contraction target = mean of the two current positions (supplementary,
//    Eq. "average_optimal" with |C| = 2), also used as the point at which the
//    pair's cost is evaluated.
//  * Facet quadrics are unweighted with unit normals; a facet with zero area or
//    a repeated index contributes the zero quadric.
//  * Ties in cost are broken by edge index; edge index = rank of (lo,hi) in
//    ascending lexicographic order.  Costs are compared through their
//    bit patterns mapped to an order-preserving unsigned key (-0 < +0).
//  * No consistency checks (Sec. 3, last paragraph).
//  * Facets that collapse (two equal indices) are dropped; of several facets
//    with the same unordered vertex triple the first in list order survives.
//  * The representative of a contracted pair is the smaller index; survivors
//    are renumbered in ascending order; every cluster stays an output vertex.
//
// Variant (off by default), entry points with the suffix _opts:
//  * placement = 1: the contraction target of a pair is the minimiser of its
//    summed quadric, -A^-1 b (supplementary, Eq. "inverse_optimal"), when A is
//    judged to have full rank by the reciprocal of its condition number, else the
//    mean as above.  The paper gives neither the way that number is computed
//    nor the threshold: taken here as the ratio of the smallest to the largest
//    pivot of A's L D L^T factorisation with diagonal pivoting (A is positive
//    semi-definite; a determinant-and-cofactor formula loses all accuracy on
//    the rank-1 matrices of flat regions), and a threshold the caller passes
//    (full rank iff ratio > threshold).  The system is solved with the same
//    factors.  The pair's cost (Alg. 2 line 2) is the quadric error at that
//    same target.
//  * absorb = 1: Alg. 2 line 11 is applied, under the vertex budget.  After
//    lines 5-10 the pairs are visited once more in the same ascending order; a
//    pair with one end in a cluster founded in lines 5-10 and the other end in
//    no cluster adds that end to that cluster, while n_r < N_r (every vertex
//    added is one more vertex removed, so the output still has exactly N
//    vertices whenever enough edges exist).  Only founders attract: a vertex
//    added by line 11 does not pull in its own neighbours (Fig. 2 (c) joins
//    each remaining point to a pair it touches).  A cluster is represented by
//    its founding pair's smaller index; its quadric and its mean position are
//    summed over its members in ascending index order.
//
//  * shuffle_seed != 0: the shuffle the paper inserts into the sorting of the
//    pairs (Sec. 3, footnote; Sec. 5, data augmentation) so that the decimated
//    mesh varies between epochs.  The paper does not say how; reading: pairs of
//    equal cost are visited in a seeded pseudo-random order instead of index
//    order, i.e. the order is ascending (cost key, tie(seed, index)) with tie a
//    bijection of the 32-bit integers; pairs of different cost keep their
//    order, so the result stays a greedy clustering by quadric cost.
//
// Pins: see tests/test_oracle_*.py (closed forms, brute force, invariants,
// hand-worked fixtures under tests/golden/).  The whole multi-round pipeline has
// no printed worked example in the paper (its Fig. 2 carries no numbers):
// beyond those pins, parity of the full pipeline is "parity unpinned".

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <map>
#include <set>
#include <array>
#include <utility>
#include <vector>

namespace {

constexpr int OK = 0;
constexpr int WARN_BUDGET_UNMET = 1;
constexpr int ERR_INVALID_ARG = -1;
constexpr int ERR_BAD_INDEX = -2;
constexpr int ERR_NONFINITE = -3;

// Quadric Q = (A, b, c) stored as a00 a01 a02 a11 a12 a22 b0 b1 b2 c.
struct Quadric {
    float q[10];
};

// Plane quadric of one facet: Q = (n n^T, d n, d^2), plane n.x + d = 0
// (supplementary, "Quadric error computation", first definition).
Quadric facet_quadric(const float* V, int i0, int i1, int i2) {
    Quadric Q;
    for (float& x : Q.q) x = 0.0f;
    if (i0 == i1 || i1 == i2 || i0 == i2) return Q;
    const float* p0 = V + 3 * (int64_t)i0;
    const float* p1 = V + 3 * (int64_t)i1;
    const float* p2 = V + 3 * (int64_t)i2;
    float ax = p1[0] - p0[0], ay = p1[1] - p0[1], az = p1[2] - p0[2];
    float bx = p2[0] - p0[0], by = p2[1] - p0[1], bz = p2[2] - p0[2];
    float nx = ay * bz - az * by;
    float ny = az * bx - ax * bz;
    float nz = ax * by - ay * bx;
    float len = std::sqrt((nx * nx + ny * ny) + nz * nz);
    if (len == 0.0f) return Q;
    nx = nx / len;
    ny = ny / len;
    nz = nz / len;
    float d = -((nx * p0[0] + ny * p0[1]) + nz * p0[2]);
    Q.q[0] = nx * nx;
    Q.q[1] = nx * ny;
    Q.q[2] = nx * nz;
    Q.q[3] = ny * ny;
    Q.q[4] = ny * nz;
    Q.q[5] = nz * nz;
    Q.q[6] = d * nx;
    Q.q[7] = d * ny;
    Q.q[8] = d * nz;
    Q.q[9] = d * d;
    return Q;
}

// Vertex quadric = sum of the quadrics of adjacent facets (supplementary,
// vertex quadric eq.), accumulated left to right from +0 in ascending
// (facet, corner) order.
void vertex_quadrics(const float* V, int N, const int32_t* F, int nF, std::vector<Quadric>& Qv) {
    Qv.assign(N, Quadric{});
    for (int v = 0; v < N; ++v)
        for (float& x : Qv[v].q) x = 0.0f;
    for (int f = 0; f < nF; ++f) {
        Quadric Qf = facet_quadric(V, F[3 * f], F[3 * f + 1], F[3 * f + 2]);
        for (int c = 0; c < 3; ++c) {
            Quadric& acc = Qv[F[3 * f + c]];
            for (int k = 0; k < 10; ++k) acc.q[k] = acc.q[k] + Qf.q[k];
        }
    }
}

// Candidate pairs = mesh edges only (Alg. 2 line 1): the distinct unordered
// sides of the current facets, ascending by (lo, hi).
void unique_edges(const int32_t* F, int nF, std::vector<std::pair<int32_t, int32_t>>& E) {
    E.clear();
    for (int f = 0; f < nF; ++f) {
        for (int c = 0; c < 3; ++c) {
            int32_t a = F[3 * f + c], b = F[3 * f + (c + 1) % 3];
            if (a == b) continue;
            E.emplace_back(std::min(a, b), std::max(a, b));
        }
    }
    std::sort(E.begin(), E.end());
    E.erase(std::unique(E.begin(), E.end()), E.end());
}

// Choices among the variants; the defaults are the path described at the top.
struct Opts {
    int placement = 0;        // 0: mean of the pair; 1: -A^-1 b where A has full rank, else the mean
    float rcond_min = 0.0f;   // full rank iff rcond > rcond_min
    int absorb = 0;           // 1: Alg. 2 line 11 under the budget
    uint64_t shuffle_seed = 0;  // != 0: equal costs in seeded pseudo-random order
};

// Seeded bijection of the 32-bit integers (every step is invertible: xor with a
// constant, multiplication by an odd number, xor with a right shift of itself,
// addition of a constant).  seed = 0 stands for "no shuffle": the identity.
uint32_t tie_break(uint64_t seed, uint32_t i) {
    if (seed == 0) return i;
    uint32_t x = i ^ (uint32_t)seed;
    x *= 0x9E3779B1u;
    x ^= x >> 15;
    x *= 0x85EBCA77u;
    x ^= x >> 13;
    x += (uint32_t)(seed >> 32);
    return x;
}

// The order in which Alg. 2 line 3 leaves the pairs: ascending (cost key, tie).
std::vector<int32_t> sorted_pairs(const std::vector<uint32_t>& key, uint64_t seed) {
    std::vector<int32_t> order(key.size());
    for (size_t i = 0; i < key.size(); ++i) order[i] = (int32_t)i;
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (key[a] != key[b]) return key[a] < key[b];
        return tie_break(seed, (uint32_t)a) < tie_break(seed, (uint32_t)b);
    });
    return order;
}

// Minimiser of the quadric s = (A, b, c): the solution of A x = -b
// (supplementary, Eq. "inverse_optimal").  A is a sum of plane quadrics n n^T,
// symmetric positive semi-definite, and is factored as P A P^T = L D L^T with
// diagonal pivoting (the largest remaining diagonal entry is eliminated
// next), so the pivots come out as d1 >= d2 >= d3 up to rounding.  The
// reciprocal condition number is estimated by d3 / d1 (for such a 3x3 matrix
// between 1 and 27 times lambda_min / lambda_max); A is taken to have full
// rank iff all pivots are positive and d3 > rcond_min * d1.  Returns false (x
// untouched) otherwise, or when a coordinate of x is not finite.
bool inverse_placement(const float* s, float rcond_min, float* x, float* rcond_out) {
    float a00 = s[0], a01 = s[1], a02 = s[2], a11 = s[3], a12 = s[4], a22 = s[5];
    float r0 = -s[6], r1 = -s[7], r2 = -s[8];
    if (rcond_out) *rcond_out = 0.0f;
    // first pivot: largest diagonal entry (the first of equal ones), moved to position 0
    int p = 0;
    float m = a00;
    if (a11 > m) { p = 1; m = a11; }
    if (a22 > m) { p = 2; m = a22; }
    if (p == 1) { std::swap(a00, a11); std::swap(a02, a12); std::swap(r0, r1); }
    if (p == 2) { std::swap(a00, a22); std::swap(a01, a12); std::swap(r0, r2); }
    const float d1 = a00;
    if (!(d1 > 0.0f)) return false;
    float l1 = a01 / d1, l2 = a02 / d1;
    // remaining 2x2 block, written so that it does not depend on which of the two axes comes first
    float s11 = a11 - (a01 * a01) / d1;
    float s12 = a12 - (a01 * a02) / d1;
    float s22 = a22 - (a02 * a02) / d1;
    // second pivot: larger diagonal entry of the remaining 2x2 block
    const bool swap12 = s22 > s11;
    if (swap12) { std::swap(s11, s22); std::swap(l1, l2); std::swap(r1, r2); }
    const float d2 = s11;
    if (!(d2 > 0.0f)) return false;
    const float l3 = s12 / d2;
    const float d3 = s22 - l3 * s12;
    if (!(d3 > 0.0f)) return false;
    if (rcond_out) *rcond_out = d3 / d1;
    if (!(d3 > rcond_min * d1)) return false;
    // L y = r, D z = y, L^T w = z
    const float y0 = r0;
    const float y1 = r1 - l1 * y0;
    const float y2 = (r2 - l2 * y0) - l3 * y1;
    float w2 = y2 / d3;
    float w1 = y1 / d2 - l3 * w2;
    float w0 = (y0 / d1 - l1 * w1) - l2 * w2;
    // undo the two exchanges, last one first
    if (swap12) std::swap(w1, w2);
    if (p == 1) std::swap(w0, w1);
    if (p == 2) std::swap(w0, w2);
    if (!std::isfinite(w0) || !std::isfinite(w1) || !std::isfinite(w2)) return false;
    x[0] = w0;
    x[1] = w1;
    x[2] = w2;
    return true;
}

// Contraction target of the pair (u, v) whose summed quadric is s: the mean of
// the two positions (supplementary, Eq. "average_optimal" with |C| = 2), or
// with placement = 1 the minimiser above wherever it is accepted.
void pair_target(const float* s, const float* pu, const float* pv, const Opts& o, float* t) {
    t[0] = (pu[0] + pv[0]) * 0.5f;
    t[1] = (pu[1] + pv[1]) * 0.5f;
    t[2] = (pu[2] + pv[2]) * 0.5f;
    if (o.placement == 1) inverse_placement(s, o.rcond_min, t, nullptr);
}

// Q(x) = x^T A x + 2 b^T x + c (supplementary, quadric error).
float quadric_error(const float* s, const float* x) {
    float mx = x[0], my = x[1], mz = x[2];
    float t0 = (s[0] * mx + s[1] * my) + s[2] * mz;
    float t1 = (s[1] * mx + s[3] * my) + s[4] * mz;
    float t2 = (s[2] * mx + s[4] * my) + s[5] * mz;
    float xAx = (mx * t0 + my * t1) + mz * t2;
    float bx = (s[6] * mx + s[7] * my) + s[8] * mz;
    return (xAx + 2.0f * bx) + s[9];
}

// Quadric error of the pair's summed quadric at the pair's contraction target
// (Alg. 2 line 2).
float pair_cost(const Quadric& Qu, const Quadric& Qv, const float* pu, const float* pv, const Opts& o = Opts()) {
    float s[10], t[3];
    for (int k = 0; k < 10; ++k) s[k] = Qu.q[k] + Qv.q[k];
    pair_target(s, pu, pv, o, t);
    return quadric_error(s, t);
}

// Unsigned key whose integer order is the numeric order of the floats
// (negative values: all bits flipped; others: sign bit set).
uint32_t cost_key(float c) {
    uint32_t u;
    std::memcpy(&u, &c, 4);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Alg. 2 lines 3-10: walk the pairs in ascending (key, index) order; a pair
// forms a new cluster iff neither end is in a cluster yet and fewer than
// n_remove pairs have been formed.
int greedy_pairs(const std::vector<std::pair<int32_t, int32_t>>& E, const std::vector<uint32_t>& key,
                 int N, int64_t n_remove, std::vector<uint8_t>& selected, uint64_t seed = 0) {
    const int nE = (int)E.size();
    const std::vector<int32_t> order = sorted_pairs(key, seed);
    std::vector<uint8_t> in_cluster(N, 0);
    selected.assign(nE, 0);
    int64_t n_r = 0;
    for (int r = 0; r < nE; ++r) {
        int e = order[r];
        int32_t u = E[e].first, v = E[e].second;
        if (!in_cluster[u] && !in_cluster[v] && n_r < n_remove) {
            selected[e] = 1;
            in_cluster[u] = in_cluster[v] = 1;
            ++n_r;
        }
    }
    return (int)n_r;
}

// Alg. 2 line 11 under the budget (see the header): second walk over the pairs
// in ascending (key, index) order.  founder[] marks the ends of the pairs formed
// in lines 5-10; via[w] receives the index of the pair that added w to a
// founder's cluster (-1 otherwise).  Returns the number of vertices added.
int absorb_remaining(const std::vector<std::pair<int32_t, int32_t>>& E, const std::vector<uint32_t>& key, int N,
                     int64_t n_remove, int64_t n_r, const std::vector<uint8_t>& selected,
                     std::vector<int32_t>& via, uint64_t seed = 0) {
    const int nE = (int)E.size();
    const std::vector<int32_t> order = sorted_pairs(key, seed);
    std::vector<uint8_t> founder(N, 0), in_cluster(N, 0);
    for (int e = 0; e < nE; ++e)
        if (selected[e]) founder[E[e].first] = founder[E[e].second] = in_cluster[E[e].first] = in_cluster[E[e].second] = 1;
    via.assign(N, -1);
    int added = 0;
    for (int r = 0; r < nE; ++r) {
        if (!(n_r < n_remove)) break;
        const int e = order[r];
        const int32_t u = E[e].first, v = E[e].second;
        int32_t w = -1;
        if (founder[u] && !in_cluster[v]) w = v;
        if (founder[v] && !in_cluster[u]) w = u;
        if (w < 0) continue;
        in_cluster[w] = 1;
        via[w] = e;
        ++n_r;
        ++added;
    }
    return added;
}

struct Mesh {
    std::vector<float> pos;       // [nv,3]
    std::vector<Quadric> Q;       // [nv]
    std::vector<int32_t> facets;  // [nf,3]
    int nv() const { return (int)Q.size(); }
    int nf() const { return (int)(facets.size() / 3); }
};

// One run of the core algorithm on the current mesh.  Returns the number of
// contracted pairs; label[] (one entry per ORIGINAL vertex) is updated.
int one_round(Mesh& M, int target_nv, std::vector<int32_t>& label, const Opts& o) {
    const int nv = M.nv();
    std::vector<std::pair<int32_t, int32_t>> E;
    unique_edges(M.facets.data(), M.nf(), E);
    std::vector<uint32_t> key(E.size());
    for (size_t e = 0; e < E.size(); ++e) {
        int32_t u = E[e].first, v = E[e].second;
        key[e] = cost_key(pair_cost(M.Q[u], M.Q[v], &M.pos[3 * (size_t)u], &M.pos[3 * (size_t)v], o));
    }
    std::vector<uint8_t> sel;
    int n_r = greedy_pairs(E, key, nv, (int64_t)nv - target_nv, sel, o.shuffle_seed);
    if (n_r == 0) return 0;

    // remap[w] = representative of w's cluster (the founding pair's smaller index)
    std::vector<int32_t> remap(nv);
    for (int w = 0; w < nv; ++w) remap[w] = w;
    for (size_t e = 0; e < E.size(); ++e)
        if (sel[e]) remap[E[e].second] = E[e].first;
    std::vector<std::vector<int32_t>> members;  // of the clusters line 11 enlarged, ascending; indexed by representative
    if (o.absorb) {
        std::vector<int32_t> via;
        n_r += absorb_remaining(E, key, nv, (int64_t)nv - target_nv, n_r, sel, via, o.shuffle_seed);
        std::vector<uint8_t> enlarged(nv, 0);
        for (int w = 0; w < nv; ++w) {
            if (via[w] < 0) continue;
            const int32_t a = E[via[w]].first, b = E[via[w]].second;
            remap[w] = remap[w == a ? b : a];
            enlarged[remap[w]] = 1;
        }
        members.resize(nv);
        for (int w = 0; w < nv; ++w)
            if (enlarged[remap[w]]) members[remap[w]].push_back(w);
    }

    // Alg. 2 lines 12-16: per cluster, summed quadric, target position, contract.
    for (size_t e = 0; e < E.size(); ++e) {
        if (!sel[e]) continue;
        int32_t u = E[e].first, v = E[e].second;  // u < v, u represents the pair
        if (members.empty() || members[u].empty()) {
            float t[3];
            for (int k = 0; k < 10; ++k) M.Q[u].q[k] = M.Q[u].q[k] + M.Q[v].q[k];
            pair_target(M.Q[u].q, &M.pos[3 * (size_t)u], &M.pos[3 * (size_t)v], o, t);
            for (int k = 0; k < 3; ++k) M.pos[3 * (size_t)u + k] = t[k];
            continue;
        }
        // a cluster that line 11 enlarged: members in ascending index order
        Quadric acc;
        float sum[3] = {0.0f, 0.0f, 0.0f};
        int cnt = 0;
        for (int32_t w : members[u]) {
            if (cnt == 0) {
                acc = M.Q[w];
                for (int k = 0; k < 3; ++k) sum[k] = M.pos[3 * (size_t)w + k];
            } else {
                for (int k = 0; k < 10; ++k) acc.q[k] = acc.q[k] + M.Q[w].q[k];
                for (int k = 0; k < 3; ++k) sum[k] = sum[k] + M.pos[3 * (size_t)w + k];
            }
            ++cnt;
        }
        float t[3] = {sum[0] / (float)cnt, sum[1] / (float)cnt, sum[2] / (float)cnt};
        if (o.placement == 1) inverse_placement(acc.q, o.rcond_min, t, nullptr);
        M.Q[u] = acc;
        for (int k = 0; k < 3; ++k) M.pos[3 * (size_t)u + k] = t[k];
    }

    // facets: re-index, drop collapsed ones and later copies of the same triple
    std::vector<int32_t> nf;
    nf.reserve(M.facets.size());
    std::set<std::array<int32_t, 3>> seen;
    for (int f = 0; f < M.nf(); ++f) {
        int32_t a = remap[M.facets[3 * f]], b = remap[M.facets[3 * f + 1]], c = remap[M.facets[3 * f + 2]];
        if (a == b || b == c || a == c) continue;
        std::array<int32_t, 3> t{a, b, c};
        std::sort(t.begin(), t.end());
        if (!seen.insert(t).second) continue;
        nf.push_back(a);
        nf.push_back(b);
        nf.push_back(c);
    }

    // survivors renumbered ascending
    std::vector<int32_t> newid(nv, -1);
    int cnt = 0;
    for (int w = 0; w < nv; ++w)
        if (remap[w] == w) newid[w] = cnt++;
    Mesh out;
    out.pos.resize(3 * (size_t)cnt);
    out.Q.resize(cnt);
    for (int w = 0; w < nv; ++w) {
        if (remap[w] != w) continue;
        for (int k = 0; k < 3; ++k) out.pos[3 * (size_t)newid[w] + k] = M.pos[3 * (size_t)w + k];
        out.Q[newid[w]] = M.Q[w];
    }
    out.facets.resize(nf.size());
    for (size_t i = 0; i < nf.size(); ++i) out.facets[i] = newid[nf[i]];
    for (int32_t& l : label) l = newid[remap[l]];
    M = std::move(out);
    return n_r;
}

int check_inputs(const float* verts, int32_t N, const int32_t* facets, int32_t F, int32_t target_nv) {
    if (!verts || N < 1 || F < 0 || (F > 0 && !facets) || target_nv < 1) return ERR_INVALID_ARG;
    for (int64_t i = 0; i < 3 * (int64_t)F; ++i)
        if (facets[i] < 0 || facets[i] >= N) return ERR_BAD_INDEX;
    for (int64_t i = 0; i < 3 * (int64_t)N; ++i)
        if (!std::isfinite(verts[i])) return ERR_NONFINITE;
    return OK;
}

int decimate(const float* verts, int32_t N, const int32_t* facets, int32_t F, int32_t target_nv, int32_t max_rounds,
             Mesh& M, std::vector<int32_t>& label, int32_t* rounds_out, const Opts& o = Opts()) {
    M.pos.assign(verts, verts + 3 * (size_t)N);
    M.facets.assign(facets, facets + 3 * (size_t)F);
    vertex_quadrics(verts, N, facets, F, M.Q);
    label.resize(N);
    for (int o = 0; o < N; ++o) label[o] = o;
    int rounds = 0, status = OK;
    while (M.nv() > target_nv && (max_rounds < 0 || rounds < max_rounds)) {
        if (one_round(M, target_nv, label, o) == 0) {
            status = WARN_BUDGET_UNMET;
            break;
        }
        ++rounds;
    }
    if (rounds_out) *rounds_out = rounds;
    return status;
}

}  // namespace

extern "C" {

// ---- stage-level entry points (used by the pin tests and by stage parity tests)

int picasso_oracle_facet_quadrics(const float* verts, int32_t N, const int32_t* facets, int32_t F, float* Qf) {
    (void)N;
    for (int f = 0; f < F; ++f) {
        Quadric Q = facet_quadric(verts, facets[3 * f], facets[3 * f + 1], facets[3 * f + 2]);
        std::memcpy(Qf + 10 * (size_t)f, Q.q, sizeof(Q.q));
    }
    return OK;
}

int picasso_oracle_vertex_quadrics(const float* verts, int32_t N, const int32_t* facets, int32_t F, float* Qv) {
    std::vector<Quadric> Q;
    vertex_quadrics(verts, N, facets, F, Q);
    for (int v = 0; v < N; ++v) std::memcpy(Qv + 10 * (size_t)v, Q[v].q, sizeof(Q[v].q));
    return OK;
}

// edges_out has room for 3*F pairs; returns the number of edges in *E.
int picasso_oracle_edges(const int32_t* facets, int32_t F, int32_t* edges_out, int32_t* E) {
    std::vector<std::pair<int32_t, int32_t>> Ed;
    unique_edges(facets, F, Ed);
    for (size_t e = 0; e < Ed.size(); ++e) {
        edges_out[2 * e] = Ed[e].first;
        edges_out[2 * e + 1] = Ed[e].second;
    }
    *E = (int32_t)Ed.size();
    return OK;
}

int picasso_oracle_edge_costs(const float* pos, const float* Q, const int32_t* edges, int32_t E, float* cost,
                              uint32_t* key) {
    for (int e = 0; e < E; ++e) {
        int32_t u = edges[2 * e], v = edges[2 * e + 1];
        Quadric Qu, Qv;
        std::memcpy(Qu.q, Q + 10 * (size_t)u, sizeof(Qu.q));
        std::memcpy(Qv.q, Q + 10 * (size_t)v, sizeof(Qv.q));
        float c = pair_cost(Qu, Qv, pos + 3 * (size_t)u, pos + 3 * (size_t)v);
        if (cost) cost[e] = c;
        if (key) key[e] = cost_key(c);
    }
    return OK;
}

uint32_t picasso_oracle_cost_key(float c) { return cost_key(c); }

// Greedy grouping of Alg. 2 lines 3-10 on an explicit edge list with explicit keys.
int picasso_oracle_select(const int32_t* edges, const uint32_t* key, int32_t E, int32_t N, int32_t n_remove,
                          uint8_t* selected) {
    std::vector<std::pair<int32_t, int32_t>> Ed(E);
    for (int e = 0; e < E; ++e) Ed[e] = {edges[2 * e], edges[2 * e + 1]};
    std::vector<uint32_t> k(key, key + E);
    std::vector<uint8_t> sel;
    int n = greedy_pairs(Ed, k, N, n_remove, sel);
    std::memcpy(selected, sel.data(), E);
    return n;
}

// ---- whole path

// max_rounds < 0: run until the budget is met.  All pointers are host memory.
// verts_out [N,3], facets_out [F,3], cluster_id [N] must have input capacity.
int picasso_oracle_decimate_rounds(const float* verts, int32_t N, const int32_t* facets, int32_t F, int32_t target_nv,
                                   int32_t max_rounds, float* verts_out, int32_t* facets_out, int32_t* cluster_id,
                                   int32_t* nv_out, int32_t* nf_out, int32_t* rounds_out, float* quadrics_out) {
    int st = check_inputs(verts, N, facets, F, target_nv);
    if (st < 0) return st;
    if (!verts_out || !facets_out || !cluster_id || !nv_out || !nf_out) return ERR_INVALID_ARG;
    Mesh M;
    std::vector<int32_t> label;
    st = decimate(verts, N, facets, F, target_nv, max_rounds, M, label, rounds_out);
    std::memcpy(verts_out, M.pos.data(), M.pos.size() * sizeof(float));
    std::memcpy(facets_out, M.facets.data(), M.facets.size() * sizeof(int32_t));
    std::memcpy(cluster_id, label.data(), label.size() * sizeof(int32_t));
    if (quadrics_out)
        for (int v = 0; v < M.nv(); ++v) std::memcpy(quadrics_out + 10 * (size_t)v, M.Q[v].q, 40);
    *nv_out = M.nv();
    *nf_out = M.nf();
    return st;
}

// ---- variants: placement (0 mean, 1 inverse with fallback) and its threshold

int picasso_oracle_pair_target(const float* quadric_sum, const float* pu, const float* pv, int32_t placement,
                               float rcond_min, float* target, float* rcond, int32_t* used_inverse) {
    Opts o;
    o.placement = placement;
    o.rcond_min = rcond_min;
    pair_target(quadric_sum, pu, pv, o, target);
    float x[3] = {0.0f, 0.0f, 0.0f};
    const bool ok = inverse_placement(quadric_sum, rcond_min, x, rcond);
    if (used_inverse) *used_inverse = (placement == 1 && ok) ? 1 : 0;
    return OK;
}

int picasso_oracle_edge_costs_opts(const float* pos, const float* Q, const int32_t* edges, int32_t E,
                                   int32_t placement, float rcond_min, float* cost, uint32_t* key) {
    Opts o;
    o.placement = placement;
    o.rcond_min = rcond_min;
    for (int e = 0; e < E; ++e) {
        int32_t u = edges[2 * e], v = edges[2 * e + 1];
        Quadric Qu, Qv;
        std::memcpy(Qu.q, Q + 10 * (size_t)u, sizeof(Qu.q));
        std::memcpy(Qv.q, Q + 10 * (size_t)v, sizeof(Qv.q));
        float c = pair_cost(Qu, Qv, pos + 3 * (size_t)u, pos + 3 * (size_t)v, o);
        if (cost) cost[e] = c;
        if (key) key[e] = cost_key(c);
    }
    return OK;
}

int picasso_oracle_decimate_opts(const float* verts, int32_t N, const int32_t* facets, int32_t F, int32_t target_nv,
                                 int32_t max_rounds, int32_t placement, float rcond_min, int32_t absorb,
                                 uint64_t shuffle_seed, float* verts_out, int32_t* facets_out, int32_t* cluster_id, int32_t* nv_out,
                                 int32_t* nf_out, int32_t* rounds_out, float* quadrics_out) {
    int st = check_inputs(verts, N, facets, F, target_nv);
    if (st < 0) return st;
    if (!verts_out || !facets_out || !cluster_id || !nv_out || !nf_out) return ERR_INVALID_ARG;
    if ((placement != 0 && placement != 1) || (absorb != 0 && absorb != 1)) return ERR_INVALID_ARG;
    Opts o;
    o.placement = placement;
    o.rcond_min = rcond_min;
    o.absorb = absorb;
    o.shuffle_seed = shuffle_seed;
    Mesh M;
    std::vector<int32_t> label;
    st = decimate(verts, N, facets, F, target_nv, max_rounds, M, label, rounds_out, o);
    std::memcpy(verts_out, M.pos.data(), M.pos.size() * sizeof(float));
    std::memcpy(facets_out, M.facets.data(), M.facets.size() * sizeof(int32_t));
    std::memcpy(cluster_id, label.data(), label.size() * sizeof(int32_t));
    if (quadrics_out)
        for (int v = 0; v < M.nv(); ++v) std::memcpy(quadrics_out + 10 * (size_t)v, M.Q[v].q, 40);
    *nv_out = M.nv();
    *nf_out = M.nf();
    return st;
}

// Alg. 2 lines 3-11 on an explicit edge list with explicit keys: selected[e] = 1
// for the pairs of lines 5-10, via[w] = index of the pair through which line 11
// added vertex w to a cluster (-1: not added).  Returns pairs + added vertices.
uint32_t picasso_oracle_tie_break(uint64_t seed, uint32_t i) { return tie_break(seed, i); }

// The same with the shuffle: pairs of equal key in the order of tie_break(seed, index).
int picasso_oracle_select_shuffled(const int32_t* edges, const uint32_t* key, int32_t E, int32_t N, int32_t n_remove,
                                   uint64_t seed, int32_t absorb, uint8_t* selected, int32_t* via) {
    std::vector<std::pair<int32_t, int32_t>> Ed(E);
    for (int e = 0; e < E; ++e) Ed[e] = {edges[2 * e], edges[2 * e + 1]};
    std::vector<uint32_t> k(key, key + E);
    std::vector<uint8_t> sel;
    int n = greedy_pairs(Ed, k, N, n_remove, sel, seed);
    std::vector<int32_t> v(N, -1);
    if (absorb) n += absorb_remaining(Ed, k, N, n_remove, n, sel, v, seed);
    std::memcpy(selected, sel.data(), E);
    std::memcpy(via, v.data(), sizeof(int32_t) * (size_t)N);
    return n;
}

int picasso_oracle_select_absorb(const int32_t* edges, const uint32_t* key, int32_t E, int32_t N, int32_t n_remove,
                                 uint8_t* selected, int32_t* via) {
    std::vector<std::pair<int32_t, int32_t>> Ed(E);
    for (int e = 0; e < E; ++e) Ed[e] = {edges[2 * e], edges[2 * e + 1]};
    std::vector<uint32_t> k(key, key + E);
    std::vector<uint8_t> sel;
    int n = greedy_pairs(Ed, k, N, n_remove, sel);
    std::vector<int32_t> v;
    n += absorb_remaining(Ed, k, N, n_remove, n, sel, v);
    std::memcpy(selected, sel.data(), E);
    std::memcpy(via, v.data(), sizeof(int32_t) * (size_t)N);
    return n;
}

// The two 1-D tensors of input-vertex length that Alg. 2 returns beside the mesh
// (Sec. 3, "Pooling and unpooling": the clustering and the degenerated-vertex
// information), derived from cluster_id.  The paper defers their definition to
// code it does not print; reading taken here: replace[v] = the representative of
// v's cluster as an INPUT vertex index, the cluster's smallest member;
// mapping[v] = the output index of v if v is that representative, -1 if v has
// degenerated into another vertex.  So cluster_id[v] == mapping[replace[v]].
// A vertex whose cluster was dropped (cluster id -1, see
// picasso_oracle_drop_unreferenced) gets -1 in both.
int picasso_oracle_replace_mapping(const int32_t* cluster_id, int32_t n_in, int32_t n_out, int32_t* replace,
                                   int32_t* mapping) {
    if (!cluster_id || n_in < 1 || n_out < 0 || !replace || !mapping) return ERR_INVALID_ARG;
    for (int v = 0; v < n_in; ++v)
        if (cluster_id[v] < -1 || cluster_id[v] >= n_out) return ERR_BAD_INDEX;
    std::vector<int32_t> first(n_out, -1);
    for (int v = 0; v < n_in; ++v)
        if (cluster_id[v] >= 0 && first[cluster_id[v]] < 0) first[cluster_id[v]] = v;
    for (int v = 0; v < n_in; ++v) {
        if (cluster_id[v] < 0) {  // the vertex's cluster has degenerated and was dropped: nothing represents it
            replace[v] = -1;
            mapping[v] = -1;
            continue;
        }
        replace[v] = first[cluster_id[v]];
        mapping[v] = (replace[v] == v) ? cluster_id[v] : -1;
    }
    return OK;
}

// Degenerated vertices removed (Sec. 3, "Pooling and unpooling": the mapping tensor carries the
// degenerated-vertex information; the paper leaves the definition to code it does not print).
// Reading: an output vertex that no output facet refers to has degenerated -- its cluster no longer
// touches the surface -- and is dropped from the output; the remaining output vertices keep their
// order and are renumbered; every input vertex of a dropped cluster gets cluster id -1.  Applied to
// the result of a decimation, in place: verts [sum nv_out, 3], facets [nf, 3], cluster_id [n_in], and
// the per-mesh vertex counts nv_out [B] of a batch (B = 1 for a single mesh).
int picasso_oracle_drop_unreferenced(float* verts, int32_t* facets, int32_t nf, int32_t* cluster_id, int32_t n_in,
                                     int32_t B, int32_t* nv_out) {
    if (!verts || (nf > 0 && !facets) || !cluster_id || B < 1 || !nv_out) return ERR_INVALID_ARG;
    int64_t nv = 0;
    for (int b = 0; b < B; ++b) nv += nv_out[b];
    std::vector<uint8_t> used((size_t)nv, 0);
    for (int64_t i = 0; i < 3 * (int64_t)nf; ++i) {
        if (facets[i] < 0 || facets[i] >= nv) return ERR_BAD_INDEX;
        used[facets[i]] = 1;
    }
    std::vector<int32_t> newid((size_t)nv, -1);
    int32_t kept = 0;
    int64_t v = 0;
    for (int b = 0; b < B; ++b) {
        int32_t kept_b = 0;
        for (int32_t k = 0; k < nv_out[b]; ++k, ++v) {
            if (!used[v]) continue;
            newid[v] = kept;
            for (int d = 0; d < 3; ++d) verts[3 * (size_t)kept + d] = verts[3 * (size_t)v + d];
            ++kept;
            ++kept_b;
        }
        nv_out[b] = kept_b;
    }
    for (int64_t i = 0; i < 3 * (int64_t)nf; ++i) facets[i] = newid[facets[i]];
    for (int32_t o = 0; o < n_in; ++o) {
        if (cluster_id[o] < 0 || cluster_id[o] >= nv) return ERR_BAD_INDEX;
        cluster_id[o] = newid[cluster_id[o]];
    }
    return OK;
}

int picasso_oracle_decimate(const float* verts, int32_t N, const int32_t* facets, int32_t F, int32_t target_nv,
                            float* verts_out, int32_t* facets_out, int32_t* cluster_id, int32_t* nv_out,
                            int32_t* nf_out) {
    return picasso_oracle_decimate_rounds(verts, N, facets, F, target_nv, -1, verts_out, facets_out, cluster_id,
                                          nv_out, nf_out, nullptr, nullptr);
}

// Concatenated meshes (Sec. 3: "mini-batches of concatenated meshes"): facet
// indices are global; every mesh is decimated on its own with its own budget.
// Outputs are concatenated in mesh order with global output indices.
// Returns the first error, else WARN_BUDGET_UNMET if any mesh fell short.
int picasso_oracle_decimate_batch(int32_t B, const float* verts, const int32_t* facets, const int32_t* nv_in,
                                  const int32_t* nf_in, const int32_t* target_nv, float* verts_out,
                                  int32_t* facets_out, int32_t* cluster_id, int32_t* nv_out, int32_t* nf_out) {
    if (B < 1 || !nv_in || !nf_in || !target_nv || !nv_out || !nf_out) return ERR_INVALID_ARG;
    int64_t v0 = 0, f0 = 0, vo = 0, fo = 0;
    int status = OK;
    for (int b = 0; b < B; ++b) {
        const int32_t N = nv_in[b], F = nf_in[b];
        if (N < 1 || F < 0) return ERR_INVALID_ARG;
        std::vector<int32_t> loc(3 * (size_t)F);
        for (int64_t i = 0; i < 3 * (int64_t)F; ++i) {
            int64_t g = facets[3 * f0 + i];
            if (g < v0 || g >= v0 + N) return ERR_BAD_INDEX;
            loc[i] = (int32_t)(g - v0);
        }
        std::vector<float> vout(3 * (size_t)N);
        std::vector<int32_t> fout(3 * (size_t)F), cid(N);
        int32_t nvo = 0, nfo = 0;
        int st = picasso_oracle_decimate(verts + 3 * v0, N, loc.data(), F, target_nv[b], vout.data(), fout.data(),
                                         cid.data(), &nvo, &nfo);
        if (st < 0) return st;
        if (st > 0) status = st;
        std::memcpy(verts_out + 3 * vo, vout.data(), 3 * (size_t)nvo * sizeof(float));
        for (int64_t i = 0; i < 3 * (int64_t)nfo; ++i) facets_out[3 * fo + i] = (int32_t)(fout[i] + vo);
        for (int i = 0; i < N; ++i) cluster_id[v0 + i] = (int32_t)(cid[i] + vo);
        nv_out[b] = nvo;
        nf_out[b] = nfo;
        v0 += N;
        f0 += F;
        vo += nvo;
        fo += nfo;
    }
    return status;
}

}  // extern "C"
