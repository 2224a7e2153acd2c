// picasso.hip -- host side of the library behind the C-ABI of include/picasso.h:
// the context and its workspace, the round loop of the decimation (Algorithm 2
// of the Picasso paper, Sec. 3; kernels in decimate_kernels.h), and the entry
// points, including those of pooling (pooling.h) and the mesh convolutions
// (conv.h).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <new>

#include "../../include/picasso.h"
#include "primitives.h"
#include "decimate_kernels.h"
#include "pooling.h"
#include "conv.h"

#pragma clang fp contract(off)

namespace {

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
constexpr int NF_ROUND_CAP = 64;  // rounds whose facet counts a call notes for the kernel-timing totals
struct StageRec { int round, stage, e0, e1; };

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
    SelectState* sel_state = nullptr;  // the budget step's radix select (one long run, see budget_step)
    int* mslots = nullptr;
    // pinned host staging
    // pinned host staging: read-back image of the header's front, then the upload image of the whole header
    int* h_pin = nullptr;
    int* h_pin_dev = nullptr;  // the same memory as the device addresses it
    size_t h_up_off = 0;
    size_t h_pin_ints = 0;
    size_t h_seq_off = 0;  // the word that kernels store a sequence number in for the host (a cache line of its own)
    int host_seq = 0;      // the last sequence number handed out
    int64_t opt_poll_us = 20000;  // for how long the host watches that word before it waits for the stream instead (0: not at all)
    int opt_ahead = 1;     // a round's contraction and facet kernels are queued before the host has looked
    int opt_trunc_width = 0;  // test hook: keys per lane of the per-mesh budget search (0: as the sizes need)
    int opt_drop_degenerated = 0;  // output vertices that no output facet refers to are dropped
    int opt_trunc_select = 1;      // a single mesh's long run in the budget step: 1 = radix select, 0 = sort
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
    int64_t kt_launches[PICASSO_KERNEL_COUNT] = {0};
    double kt_ms[PICASSO_KERNEL_COUNT] = {0.0}, kt_bytes[PICASSO_KERNEL_COUNT] = {0.0};
    // host mirrors of the per-mesh state of a decimate call (6 x max_meshes ints, allocated with the
    // context: the calls themselves allocate nothing, on the host either)
    int* h_mesh = nullptr;
    int nf_round[NF_ROUND_CAP];  // facets, vertices, distinct edges of each round of the current call
    int nv_round[NF_ROUND_CAP];
    int ne_round[NF_ROUND_CAP];
    int n_rounds_noted = 0;
    StageRec st_recs[PICASSO_STATS_ROUNDS * PICASSO_ST_COUNT + 2];
};

namespace {

constexpr int HDR_STATE_INTS = (int)(sizeof(State) / sizeof(int));
constexpr int SEQ_CHECK_WORD = 16;  // within the sequence word's 32-int area: the selection tail's copy of the number (a cache line further)

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
    x->sel_state = cv.take<SelectState>(1);
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
    int n_recs = 0;  // records in c->st_recs
    int open = -1;
    void begin(int round, int stage) {
        constexpr int cap = (int)(sizeof(c->st_recs) / sizeof(c->st_recs[0]));
        if (!on || n_recs >= cap || c->n_ev + 2 > (int)(sizeof(c->ev) / sizeof(c->ev[0]))) return;
        const StageRec r{round, stage, c->n_ev, c->n_ev + 1};
        c->n_ev += 2;
        (void)hipEventRecord(c->ev[r.e0], s);
        c->st_recs[n_recs] = r;
        open = n_recs++;
    }
    void end() {
        if (!on || open < 0) return;
        (void)hipEventRecord(c->ev[c->st_recs[open].e1], s);
        open = -1;
    }
    void collect(picasso_stats* stats) {
        if (!on || !stats) return;
        for (int i = 0; i < n_recs; ++i) {
            const StageRec& r = c->st_recs[i];
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, c->ev[r.e0], c->ev[r.e1]) == hipSuccess && r.round < PICASSO_STATS_ROUNDS)
                stats->ms_stage[r.round][r.stage] += ms;
        }
    }
};

// hipEvents around the launches made while this object lives, credited to `kernel` in round `round`
// (only in the calls that PICASSO_OPT_KERNEL_TIMING picks).
struct KernelBracket {
    picasso_ctx* c;
    hipStream_t s;
    bool on;
    KernelBracket(picasso_ctx* c_, hipStream_t s_, int kernel, int round, bool wanted = true) : c(c_), s(s_) {
        on = wanted && c->kt_this_call && round < 0xFF && c->kt.begin(s, (kernel << 8) | round);
    }
    ~KernelBracket() {
        if (on) c->kt.end(s);
    }
    KernelBracket(const KernelBracket&) = delete;
    KernelBracket& operator=(const KernelBracket&) = delete;
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

// `uq` (keys without values, bucket sorts only): the sort also does the count pass of the compaction
// that keeps one of every run of equal keys.
template <typename K, bool HAS_VAL, class Src = prim::ArrayKeys<K>>
int sort_by_vertex(hipStream_t s, K* k0, K* k1, u32* v0, u32* v1, const int* n_ptr, int n_max, int key_bits,
                   const prim::SortScratch& sc, u32* hist12, prim::LaunchTimer* lt = nullptr, int tag = 0,
                   bool counted = false, const Src* src = nullptr, const prim::UniqueCount<K>* uq = nullptr) {
    const int how = sort_by_vertex_path(n_max, key_bits);
    if (how == COUNT_SMALL)
        return prim::bucket_sort<K, HAS_VAL, Src>(s, k0, k1, v0, v1, n_ptr, n_max, key_bits, sc, lt, tag, counted,
                                                  hist12, src, uq);
    if (how == COUNT_LARGE)
        return prim::bucket_sort_large<K, HAS_VAL, Src>(s, k0, k1, v0, v1, n_ptr, n_max, key_bits, sc, hist12, lt, tag,
                                                        counted, src, uq);
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
    bool counted_firsts = false;  // the sort has left the unique step's tile counts
    if (H_ > 0) {
        const EdgeKeys src{c->fbuf[cur_], vbits_, sentinel_};  // (the counted sorts read the keys from here)
        // the bucket sorts also count, per tile of the compaction that follows, the keys that differ from
        // the key in front of them: the count pass of the unique step
        prim::UniqueCount<u64> uq;
        if (counted) {
            const int chunks = prim::compact_chunks_for(H_);
            uq.tilesum = c->tilesum;
            uq.tiles = prim::compact_tiles(H_, chunks);
            uq.tile_shift = ceil_log2((long long)BLOCK * chunks);
            uq.sentinel = sentinel_;
            counted_firsts = true;
        }
        int where = sort_by_vertex<u64, false, EdgeKeys>(st_, c->key64[0], c->key64[1], nullptr, nullptr, &c->st->nh,
                                                         H_, 2 * vbits_, c->sort_sc, c->hist12,
                                                         c->kt_this_call ? &c->kt : nullptr, round_, counted, &src,
                                                         counted ? &uq : nullptr);
        if (where < 0) return PICASSO_ERR_HIP;
        skeys = where ? c->key64[1] : c->key64[0];
    }
    if (!counted_firsts) {
        UniquePred up_{skeys, sentinel_};
        prim::compact_count(st_, up_, &c->st->nh, H_, c->tilesum);
    }
    *skeys_out = skeys;
    return PICASSO_OK;
}

constexpr int64_t OVERLAP_MIN_FACETS = 1 << 18;

// Bits of the incidence keys: vertex id above, facet id below.
inline int incidence_fbits(int F) { return ceil_log2(std::max(F, 1)); }
inline int incidence_key_bits(int N, int F) { return ceil_log2(N) + incidence_fbits(F); }

// Where init_kernel leaves the facets' planes for S0: the edge-key array, which nothing else uses
// before the first round's costs are computed (24 bytes per facet there, 16 needed).
inline float4* facet_planes(picasso_ctx* c) { return reinterpret_cast<float4*>(c->ekey); }

// The validating kernel, instantiated for the sort the incidence keys go to.
int launch_init(picasso_ctx* c, hipStream_t s, const float* d_verts, int N, const int32_t* d_facets, int F, int B,
                bool with_keys, HeaderInit init = HeaderInit{nullptr, 0, 0, 0, 0, 0, 0, 0}) {
    const int fbits = incidence_fbits(F), kb = incidence_key_bits(N, F);
    const int how = with_keys ? sort_by_vertex_path(3ll * F, kb) : COUNT_NONE;
    // only a sort that cannot make the keys itself (the plain LSD fallback) needs them written out
    u64* ikey = (with_keys && how == COUNT_NONE) ? c->s0_key[0] : nullptr;
    const int s0 = with_keys ? 1 : 0;
    float4* planes = with_keys ? facet_planes(c) : nullptr;
    const int grid = grid_for(std::max(N, F), 4096);
    if (how == COUNT_SMALL)
        init_kernel<COUNT_SMALL><<<grid, BLOCK, 0, s>>>(d_verts, N, d_facets, F, B, c->voff[0], c->foff, c->vrec[0],
                                                        c->cid, c->fbuf[0], ikey, fbits, prim::bucket_sort_low_bits(kb),
                                                        c->hist12_s0, c->st, c->hist12, s0, init, planes);
    else if (how == COUNT_LARGE)
        init_kernel<COUNT_LARGE><<<grid, BLOCK, 0, s>>>(d_verts, N, d_facets, F, B, c->voff[0], c->foff, c->vrec[0],
                                                        c->cid, c->fbuf[0], ikey, fbits,
                                                        kb - prim::BUCKET_LARGE_MSD_BITS, c->hist12_s0, c->st, c->hist12,
                                                        s0, init, planes);
    else
        init_kernel<COUNT_NONE><<<grid, BLOCK, 0, s>>>(d_verts, N, d_facets, F, B, c->voff[0], c->foff, c->vrec[0],
                                                       c->cid, c->fbuf[0], ikey, fbits, 0, nullptr, c->st, c->hist12,
                                                       s0, init, planes);
    return hipGetLastError() == hipSuccess ? PICASSO_OK : PICASSO_ERR_HIP;
}

// S0 on the incidence keys written by init_kernel (whose digit counts are in hist12_s0).
int run_vertex_quadrics(picasso_ctx* c, hipStream_t s, const float* d_verts, int N, int F) {
    const int H = 3 * F;
    const int fbits = incidence_fbits(F), kb = incidence_key_bits(N, F);
    if (F > 0) {
        const bool counted = sort_by_vertex_path(H, kb) != COUNT_NONE;
        const IncidenceKeys src{c->fbuf[0], fbits};  // (the counted sorts read the keys from here)
        int where = sort_by_vertex<u64, false, IncidenceKeys>(s, c->s0_key[0], c->s0_key[1], nullptr, nullptr,
                                                                  nullptr, H, kb, c->sort_sc_s0, c->hist12_s0,
                                                                  c->kt_this_call ? &c->kt : nullptr,
                                                                  PICASSO_KERNEL_SORT_INCIDENCE << 8, counted, &src);
        if (where < 0) return PICASSO_ERR_HIP;
        const u64* skey = where ? c->s0_key[1] : c->s0_key[0];
        const int tiles = (H + QR_TILE - 1) / QR_TILE;
        const KernelBracket timed(c, s, PICASSO_KERNEL_QUADRIC_ROWS, 0);
        quadric_rows_kernel<<<tiles, BLOCK, 0, s>>>(c->vrec[0], d_verts, N, facet_planes(c), skey, H, fbits,
                                                    c->hist12_s0);
    } else {
        quadric_rows_kernel<<<grid_for(N, 4096), BLOCK, 0, s>>>(c->vrec[0], d_verts, N, nullptr, nullptr, 0, 0,
                                                               c->hist12_s0);
    }
    return PICASSO_OK;
}

// Fills the pinned image of the header (State + per-mesh tables) and sends it with one copy.
// `by_kernel`: only the checks; the first kernel writes the header itself (a single mesh, see HeaderInit).
int upload_header(picasso_ctx* c, hipStream_t s, int B, const int32_t* nv_in, const int32_t* nf_in,
                  const int32_t* target, int64_t* N_out, int64_t* F_out, bool by_kernel = false) {
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
    if (!by_kernel) HIP_TRY(c, hipMemcpyAsync(c->hdr, img, sizeof(int) * total, hipMemcpyHostToDevice, s));
    return PICASSO_OK;
}

// The signal for the next kernel after which the host looks at the read-back area.
// (The number wraps around after 2^32 signals; only equality with the last one stored matters.)
HostSignal next_signal(picasso_ctx* c) {
    c->host_seq = (int)((unsigned)c->host_seq + 1u);
    return HostSignal{c->h_pin_dev + c->h_seq_off, c->host_seq};
}

// Waits until the kernel that was given `sig` has written its results to the pinned read-back
// area.  That kernel stores the sequence number after them (system-scope release), so the host
// watches the word: it sees it some microseconds before a stream synchronisation would return,
// and everything queued on the stream before that kernel is complete by then as well.  Falls back
// to the stream synchronisation when the word has not changed within the context's limit (20 ms
// unless set otherwise; 0 = do not watch at all), which also brings any launch error to light.
hipError_t wait_for_signal(picasso_ctx* c, hipStream_t s, const HostSignal& sig) {
    if (c->opt_poll_us > 0) {
        const int* word = c->h_pin + c->h_seq_off;
        const auto t0 = std::chrono::steady_clock::now();
        const auto limit = std::chrono::microseconds(c->opt_poll_us);
        const long check_every = c->opt_poll_us >= 1000 ? 1023 : 15;  // (the clock is read every so many looks)
        for (long spins = 1;; ++spins) {
            if (__atomic_load_n(word, __ATOMIC_ACQUIRE) == sig.seq) return hipSuccess;
            if ((spins & check_every) == 0 && std::chrono::steady_clock::now() - t0 > limit) break;
#if defined(__x86_64__)
            __builtin_ia32_pause();
#endif
        }
    }
    return hipStreamSynchronize(s);
}

// [State][matched][foff_out] brought to the pinned read-back area by a one-workgroup kernel that then
// tells the host; returns when the host has them (and everything queued before has been executed).
int read_header(picasso_ctx* c, hipStream_t s) {
    const HostSignal done = next_signal(c);
    publish_header_kernel<<<1, BLOCK, 0, s>>>(c->hdr, HDR_STATE_INTS + 2 * c->cap_b + 1, c->h_pin_dev, done);
    HIP_TRY(c, wait_for_signal(c, s, done));
    return PICASSO_OK;
}

int status_from_err_bits(int bits) {
    if (bits & ERR_BIT_INTERNAL) return PICASSO_ERR_INTERNAL;
    if (bits & ERR_BIT_BAD_INDEX) return PICASSO_ERR_BAD_INDEX;
    if (bits & ERR_BIT_NONFINITE) return PICASSO_ERR_NONFINITE;
    return PICASSO_OK;
}

// Budget step: among the edges `over` selects (the formed pairs, or the joining edges of line 11, of
// the meshes that have more of them than they may use: counts[b] > budgets[b]) each mesh keeps its
// budgets[b] first ones in ascending (cost key, tie-break) order; the others are released
// (release_edge<ABSORB>) and counts[] is clamped.  n_over = sum of those meshes' counts, seg_max
// their largest.
// `guarded` (per-mesh search only, i.e. seg_max <= the context's limit for it): queued behind the
// selection tail before the host has looked; ne, n_over and seg_max are then upper bounds and the
// kernels do nothing unless the tail finished the matching; `tell` is stored by the first of them.
template <bool ABSORB, class Over>
int budget_step(picasso_ctx* c, hipStream_t s, Over over, int B, int ne, int vbits, const MeshTab& mt,
                const TieBreak& tb, long long n_over, int seg_max, int* counts, int* budgets, bool guarded = false,
                HostSignal tell = HostSignal{nullptr, 0}) {
    if (guarded && seg_max > c->opt_trunc_block_max) return PICASSO_ERR_INVALID_ARG;
    if (seg_max <= c->opt_trunc_block_max) {
        const int* guard = guarded ? &c->st->go : nullptr;
        u32* tcost = reinterpret_cast<u32*>(c->key64[0]);
        TruncOutSplit to{c->ecost, tcost, c->val32[0]};
        // (`tell`: the first kernel also tells the host that the selection tail in front of it is done)
        SignalingPred<Over> first{over, tell};
        prim::compact(s, first, over, to, guarded ? &c->st->guard_ne : &c->st->ne, ne, c->tilesum, &c->st->trunc_n);
#define PICASSO_TRUNC_BLOCK(R)                                                                                       \
    do {                                                                                                             \
        if (tb.on)                                                                                                   \
            trunc_block_kernel<R, true><<<B, TRUNC_THREADS, 0, s>>>(tcost, c->val32[0], tb, counts, budgets, guard,   \
                                                                    c->st);                                          \
        else                                                                                                         \
            trunc_block_kernel<R, false><<<B, TRUNC_THREADS, 0, s>>>(tcost, c->val32[0], tb, counts, budgets, guard,  \
                                                                     c->st);                                         \
    } while (0)
        // keys per lane: what the largest mesh needs (or what the test hook says)
        const int width = c->opt_trunc_width ? c->opt_trunc_width : (seg_max + TRUNC_THREADS - 1) / TRUNC_THREADS;
        if (width <= 4) PICASSO_TRUNC_BLOCK(4);
        else if (width <= 8) PICASSO_TRUNC_BLOCK(8);
        else if (width <= 16) PICASSO_TRUNC_BLOCK(16);
        else PICASSO_TRUNC_BLOCK(32);
#undef PICASSO_TRUNC_BLOCK
        trunc_release_kernel<ABSORB><<<grid_for(n_over), BLOCK, 0, s>>>(tcost, c->val32[0], c->st, c->ekey, vbits,
                                                                        c->mate, B, counts, budgets, c->abid, guard);
        return PICASSO_OK;
    }
    if (B == 1 && !tb.on && c->opt_trunc_select) {
        // one long run, ties in edge order: no sort, the threshold key is found by three histogram passes
        u32* tcost = reinterpret_cast<u32*>(c->key64[0]);
        TruncOutSplit to{c->ecost, tcost, c->val32[0]};
        prim::compact(s, over, over, to, &c->st->ne, ne, c->tilesum, &c->st->trunc_n);
        SelectState* S = c->sel_state;
        constexpr int state_words = (int)(sizeof(SelectState) / sizeof(u32));
        prim::fill_u32_kernel<<<grid_for(state_words), BLOCK, 0, s>>>(reinterpret_cast<u32*>(S), state_words, 0u);
        const int hgrid = grid_for((n_over + SELECT_ITEMS - 1) / SELECT_ITEMS);
        trunc_select_hist_kernel<0><<<hgrid, BLOCK, 0, s>>>(tcost, c->st, S);
        trunc_select_pick_kernel<0><<<1, BLOCK, 0, s>>>(S, budgets);
        trunc_select_hist_kernel<1><<<hgrid, BLOCK, 0, s>>>(tcost, c->st, S);
        trunc_select_pick_kernel<1><<<1, BLOCK, 0, s>>>(S, budgets);
        trunc_select_hist_kernel<2><<<hgrid, BLOCK, 0, s>>>(tcost, c->st, S);
        trunc_select_pick_kernel<2><<<1, BLOCK, 0, s>>>(S, budgets);
        const SelectTiePred tie{tcost, S};
        const SelectFlagOut flag{tcost, S};
        prim::compact(s, tie, tie, flag, &c->st->trunc_n, (int)n_over, c->tilesum, nullptr);
        trunc_release_kernel<ABSORB><<<grid_for(n_over), BLOCK, 0, s>>>(tcost, c->val32[0], c->st, c->ekey, vbits,
                                                                        c->mate, B, counts, budgets, c->abid, nullptr);
        return hipGetLastError() == hipSuccess ? PICASSO_OK : PICASSO_ERR_HIP;
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
               const TieBreak& tb, const int* nrem, const int* h_matched, int* h_joined, const u64** akeys) {
    absorb_begin_kernel<<<grid_for(std::max(nv_total, B), 4096), BLOCK, 0, s>>>(c->abid, c->arep, c->acnt, c->st, cur, B, c->nrem,
                                                                              c->matched, c->arem, c->acand);
    absorb_bid_kernel<<<grid_for(std::max(ne, 1), 8192), BLOCK, 0, s>>>(c->ekey, c->ecost, c->st, vbits, c->mate, mt,
                                                                      c->arem, c->abid, tb);
    JoinPred jp{c->ekey, c->ecost, c->mate, c->abid, vbits, tb};
    JoinListOut jl{c->list};
    prim::compact(s, jp, jp, jl, &c->st->ne, ne, c->tilesum, &c->st->absorb_n);
    int* host_counts = c->h_pin_dev + HDR_STATE_INTS + c->cap_b;  // (the offsets' slots of the read-back area: free until the end)
    const HostSignal counted = next_signal(c);
    absorb_count_kernel<<<1, BLOCK, 0, s>>>(c->list, c->st, c->ekey, vbits, B, c->voff[cur], c->acand, host_counts,
                                            counted);
    HIP_TRY(c, wait_for_signal(c, s, counted));
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
    const bool header_by_kernel = B == 1;  // one mesh: no copy in front of the first kernel
    int rc = upload_header(c, s, B, nv_in, nf_in, target_nv, &N64, &F64, header_by_kernel);
    if (rc != PICASSO_OK) return rc;
    if (F64 > 0 && !d_facets) return PICASSO_ERR_INVALID_ARG;
    const int N = (int)N64, F = (int)F64;
    HeaderInit hinit{nullptr, 0, 0, 0, 0, 0, 0, 0};
    if (header_by_kernel)
        hinit = HeaderInit{c->hdr, HDR_STATE_INTS + 8 * c->cap_b + 3, (int)(c->voff[0] - c->hdr), (int)(c->foff - c->hdr),
                           (int)(c->target - c->hdr), N, F, target_nv[0]};

    c->n_ev = 0;
    c->kt.pool = c->kt_pool;
    c->kt.cap = (int)(sizeof(c->kt_pool) / sizeof(c->kt_pool[0]));
    c->kt.recs = c->kt_recs;
    c->kt.used = 0;
    c->kt.nrec = 0;
    c->kt_this_call = c->opt_kernel_timing > 0 && (c->kt_calls++ % c->opt_kernel_timing) == 0;
    struct TimingScope {  // (no brackets outside this call, however it ends)
        picasso_ctx* c;
        ~TimingScope() { c->kt_this_call = false; }
    } timing_scope{c};
    c->n_rounds_noted = 0;
    StageTimer tm{c, s, c->opt_stage_timing != 0 && stats != nullptr};
    if (stats) HIP_TRY(c, hipEventRecord(c->ev_total[0], s));  // (an event costs queue time: only when asked for)

    // host mirror of the per-mesh vertex counts
    int* const nvb = c->h_mesh;
    int* const stuck = nvb + c->max_meshes;
    int* const act = stuck + c->max_meshes;
    int* const nrem = act + c->max_meshes;
    int* const h_matched = nrem + c->max_meshes;
    int* const h_joined = h_matched + c->max_meshes;
    for (int b = 0; b < B; ++b) {
        nvb[b] = nv_in[b];
        stuck[b] = act[b] = nrem[b] = h_matched[b] = h_joined[b] = 0;
    }
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
    // costs are computed.  (Serial when stage times are being recorded, to keep them attributable, and in a
    // call whose kernels are bracketed by events: a bracketed kernel then has the chip to itself, and its
    // duration is its own.)
    // The fork and join cost about as much as a few small kernels, so small inputs stay on one stream.
    const u64* skeys = nullptr;
    const bool overlap = work && c->opt_overlap && c->side && !tm.on && !c->kt_this_call && F >= OVERLAP_MIN_FACETS;
    tm.begin(0, PICASSO_ST_QUADRICS);
    rc = launch_init(c, s, d_verts, N, d_facets, F, B, work, hinit);
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
        const KernelBracket timed(c, s, PICASSO_KERNEL_UNIQUE_COST, round);                                          \
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

        // The kernels after the selection.  `guarded`: queued behind the selection tail before the host
        // has looked; they then go by what the tail leaves in State (go, guard_nv, guard_nf) and do
        // nothing unless it finished the matching.
        auto issue_contract = [&](int nf_cap, int n_joined, const u64* akeys, bool guarded, HostSignal tell) {
            const int nxt = cur ^ 1;
            const int* guard = guarded ? &c->st->go : nullptr;
            const int* n_ptr = guarded ? &c->st->guard_nv : nullptr;
            AliveOut ao{c->newid};
            if (n_joined > 0) {
                AlivePredT<true> ap{c->mate, c->arep};
                prim::compact(s, ap, ap, ao, n_ptr, nv_total, c->tilesum, &c->st->nv[nxt]);
            } else {
                AlivePredT<false> ap{c->mate, nullptr};
                SignalingPred<AlivePredT<false>> first{ap, tell};  // (`tell.word` may be null: nothing to tell)
                prim::compact(s, first, ap, ao, n_ptr, nv_total, c->tilesum, &c->st->nv[nxt]);
            }
            const size_t hsize = next_pow2((size_t)2 * std::max(nf_cap, 1));
            const int cgrid = grid_for(std::max<long long>(nv_total, (long long)hsize), 8192);
#define PICASSO_CONTRACT(PLACE, ABSORB, RCOND)                                                                       \
    contract_kernel<PLACE, ABSORB><<<cgrid, BLOCK, 0, s>>>(c->vrec[cur], c->vrec[nxt], c->mate, c->newid, c->vmap,    \
                                                           c->st, cur, B, c->voff[cur], c->voff[nxt], c->htab,        \
                                                           (int)hsize, c->hist12, RCOND, c->arep, c->acnt, akeys,     \
                                                           vbits, guard)
            if (c->opt_placement == PLACE_INVERSE) {
                if (n_joined > 0) PICASSO_CONTRACT(PLACE_INVERSE, true, c->opt_rcond_min);
                else PICASSO_CONTRACT(PLACE_INVERSE, false, c->opt_rcond_min);
            } else {
                if (n_joined > 0) PICASSO_CONTRACT(PLACE_MEAN, true, 0.0f);
                else PICASSO_CONTRACT(PLACE_MEAN, false, 0.0f);
            }
#undef PICASSO_CONTRACT
        };
        auto issue_facets = [&](int nf_cap, bool guarded) {
            const int nxt = cur ^ 1;
            const size_t hsize = next_pow2((size_t)2 * std::max(nf_cap, 1));
            {
                const KernelBracket timed(c, s, PICASSO_KERNEL_FACET_INSERT, round);
                facet_insert_kernel<<<grid_for(std::max(nf_cap, N), 8192), BLOCK, 0, s>>>(
                    c->fbuf[cur], c->fmap, c->vmap, c->st, cur, c->htab, (u32)(hsize - 1), mt, c->voff[cur], c->cid, N,
                    c->fslot, guarded ? &c->st->go : nullptr);
            }
            FacetKeepPred kp{c->fslot, c->htab, c->keep};
            FlagPred fp{c->keep};
            FacetOut fo{c->fmap, c->fbuf[nxt]};
            prim::compact(s, kp, fp, fo, guarded ? &c->st->guard_nf : &c->st->nf[cur], nf_cap, c->tilesum, &c->st->nf[nxt]);
        };
        // Where no mesh can form more pairs than its budget allows (a matching pairs at most half the
        // vertices) and nothing else has to be decided after the selection, those kernels are queued
        // right behind the tail: the device does not idle while the host looks.
        // Where the budget will bind (a mesh has to stop below 40 % of its vertices; a matching on these
        // meshes pairs 85-95 % of them) and the per-mesh search can take every such mesh, the budget step
        // is queued there too, in front of them: it finds on the device which meshes are over their
        // budgets, and does nothing where none is.  In between (40-50 %) nothing is queued ahead.
        // Queued ahead, the kernels are sized by the facet bound of the round before (twice the hash
        // table to clear, twice the tiles), which costs more than the idling from about a million facets.
        constexpr int AHEAD_MAX_FACETS = 1 << 20;
        bool ahead_ok = !c->opt_absorb && !stats && c->opt_ahead && nf_bound <= AHEAD_MAX_FACETS;
        bool ahead_budget = false;
        long long over_bound = 0;  // pairs of the meshes that may exceed their budgets, at most
        int seg_bound = 0;         // ... of the largest of them
        if (ahead_ok) {
            bool likely = false;
            for (int b = 0; b < B; ++b)
                if (act[b] && 2ll * nrem[b] < nvb[b]) {
                    over_bound += nvb[b] / 2;
                    seg_bound = std::max(seg_bound, nvb[b] / 2);
                    likely |= 5ll * nrem[b] < 2ll * nvb[b];
                }
            ahead_budget = seg_bound > 0;
            if (ahead_budget && !(likely && seg_bound <= c->opt_trunc_block_max)) ahead_ok = false;
        }
        bool ahead = false;  // the kernels are queued and the tail has finished the matching

        // ---- S3: selection sub-rounds
        tm.begin(round, PICASSO_ST_SELECT);
        SelArgs sa;
        sa.cur = cur;
        sa.ekey = c->ekey;
        sa.ecost = c->ecost;
        for (int i = 0; i < 3; ++i) sa.vmin[i] = c->vmin[i];
        sa.mate = c->mate;
        sa.list = c->list;
        sa.lkey = c->key64[1];  // (the sort's arrays are free between the unique step and the budget step)
        sa.lcost = c->val32[1];
        sa.estate = c->estate;
        sa.st = c->st;
        sa.mt = mt;
        sa.vbits = vbits;
        sa.host_img = c->h_pin_dev;
        sa.publish_ints = HDR_STATE_INTS + B;
        sa.host_check = c->h_pin_dev + c->h_seq_off + SEQ_CHECK_WORD;
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
            // Below the sparse kernels' range the last of these sub-rounds has one lane per edge and as
            // many workgroups as the gather has tiles: it counts its surviving edges for the gather.
            // (wide == 0: so few edges that the tail takes them all from the start)
            const bool counts_live = wide > 0 && ne_bound < SPARSE_MIN_EDGES && prim::compact_chunks_for(ne_bound) == 1 &&
                                     grid_for(ne_bound, 1 << 16) == prim::compact_tiles(std::max(ne_bound, 1), 1);
            for (int j = 0; j < wide; ++j) {
                sa.tile_live = (counts_live && j == wide - 1) ? c->tilesum : nullptr;
                const int g4 = (ne_bound + BLOCK * 4 - 1) / (BLOCK * 4), g16 = (ne_bound + BLOCK * 16 - 1) / (BLOCK * 16);
                if (sel_k + j == 1 && ne_bound >= SPARSE_MIN_EDGES) {
                    if (tb.on) select_subround_sparse_kernel<4, true><<<g4, BLOCK, 0, s>>>(sa, sel_k + j);
                    else select_subround_sparse_kernel<4, false><<<g4, BLOCK, 0, s>>>(sa, sel_k + j);
                } else if (sel_k + j > 1 && ne_bound >= SPARSE_MIN_EDGES) {
                    if (tb.on) select_subround_sparse_kernel<16, true><<<g16, BLOCK, 0, s>>>(sa, sel_k + j);
                    else select_subround_sparse_kernel<16, false><<<g16, BLOCK, 0, s>>>(sa, sel_k + j);
                } else {
                    const KernelBracket timed(c, s, PICASSO_KERNEL_SUBROUND0, round, sel_k + j == 0);  // (the first only)
                    if (tb.on) select_subround_kernel<true><<<grid_for(ne_bound, 1 << 16), BLOCK, 0, s>>>(sa, sel_k + j);
                    else select_subround_kernel<false><<<grid_for(ne_bound, 1 << 16), BLOCK, 0, s>>>(sa, sel_k + j);
                }
            }
            sel_k += wide;
            LivePred lp{c->estate};
            LiveOut lo{c->list, c->ekey, c->ecost, c->key64[1], c->val32[1]};
            if (counts_live) prim::compact_scatter(s, lp, lo, &c->st->ne, ne_bound, c->tilesum, &c->st->live[0]);
            else prim::compact(s, lp, lp, lo, &c->st->ne, ne_bound, c->tilesum, &c->st->live[0]);
            // the kernel behind the tail tells the host that the tail's results are in the read-back area
            const HostSignal tail_done = next_signal(c);
            sa.host_seq = tail_done.seq;
            select_tail_kernel<<<1, TAIL_THREADS, 0, s>>>(sa);
            launched += wide + 3;
            const HostSignal nothing{nullptr, 0};
            if (ahead_ok) {
                if (ahead_budget) {
                    TruncPred tp{c->ekey, c->mate, mt, vbits};
                    rc = budget_step<false>(c, s, tp, B, ne_bound, vbits, mt, tb, over_bound, seg_bound, c->matched,
                                            c->nrem, true, tail_done);
                    if (rc != PICASSO_OK) return rc;
                }
                issue_contract(nf_bound, 0, nullptr, true, ahead_budget ? nothing : tail_done);
                issue_facets(nf_bound, true);
            } else {
                signal_kernel<<<1, 64, 0, s>>>(tail_done);
            }
            HIP_TRY(c, wait_for_signal(c, s, tail_done));  // [State][matched] are in the read-back area
            // The tail stored its counters at system scope and, after them, its own copy of the number
            // that the kernel behind it has just stored; should that copy not be there yet, what the
            // host would read is not to be trusted: wait for the stream, after which everything is.
            if (__atomic_load_n(c->h_pin + c->h_seq_off + SEQ_CHECK_WORD, __ATOMIC_ACQUIRE) != tail_done.seq) {
                HIP_TRY(c, hipStreamSynchronize(s));
                if (c->h_pin[c->h_seq_off + SEQ_CHECK_WORD] != tail_done.seq) {
                    snprintf(c->hip_err, sizeof(c->hip_err), "the selection's results did not reach host memory");
                    return PICASSO_ERR_HIP;
                }
            }
            if (!validated) {
                const int st_err = status_from_err_bits(hst->err);
                if (st_err != PICASSO_OK) {  // (the flags go back to zero for the next call, see HeaderInit)
                    prim::fill_u32_kernel<<<1, BLOCK, 0, s>>>(reinterpret_cast<u32*>(&c->st->err), 1, 0u);
                    return st_err;
                }
                validated = true;
            }
            if (hst->err & ERR_BIT_INTERNAL) {  // a kernel of the round before has refused its sizes
                prim::fill_u32_kernel<<<1, BLOCK, 0, s>>>(reinterpret_cast<u32*>(&c->st->err), 1, 0u);
                return PICASSO_ERR_INTERNAL;
            }
            sel_k = hst->sel_k;
            const int live = hst->live[0];
            if (live == 0) {
                ahead = ahead_ok;
                break;
            }
            live_est = live;
        }
        for (int b = 0; b < B; ++b) h_matched[b] = c->h_pin[HDR_STATE_INTS + b];
        nf_bound = std::min(nf_bound, hst->nf[cur]);
        if (c->n_rounds_noted < NF_ROUND_CAP) {
            c->nf_round[c->n_rounds_noted] = hst->nf[cur];
            c->nv_round[c->n_rounds_noted] = nv_total;
            c->ne_round[c->n_rounds_noted] = hst->ne;
            ++c->n_rounds_noted;
        }
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
        if (need_trunc && ahead && !ahead_budget) return PICASSO_ERR_HIP;  // (cannot happen: a matching pairs at most half the vertices)
        if (need_trunc && !ahead) {
            TruncPred tp{c->ekey, c->mate, mt, vbits};
            rc = budget_step<false>(c, s, tp, B, hst->ne, vbits, mt, tb, n_trunc, seg_max, c->matched, c->nrem);
            if (rc != PICASSO_OK) return rc;
        }

        // ---- Alg. 2 line 11 (option): un-paired vertices join a neighbouring pair's cluster while budget is left
        int n_joined = 0;
        const u64* akeys = nullptr;
        for (int b = 0; b < B; ++b) h_joined[b] = 0;
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

        // ---- S4 + S6: contraction and renumbering; S5: facets (already queued behind the tail, and run,
        // where `ahead` is set)
        const int nxt = cur ^ 1;
        if (!ahead) {
            tm.begin(round, PICASSO_ST_CONTRACT);
            issue_contract(nf_bound, n_joined, akeys, false, HostSignal{nullptr, 0});
            tm.end();
            tm.begin(round, PICASSO_ST_FACETS);
            issue_facets(nf_bound, false);
            tm.end();
        }

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

    const int out_grid = grid_for(std::max(std::max(N, 3 * nf_bound), 1), 8192);
    if (c->opt_drop_degenerated) {
        // output vertices that no output facet refers to are dropped: mark, number the others, copy out
        int* ref = c->mate;  // (free once the rounds are over)
        prim::fill_u32_kernel<<<grid_for(nv_total), BLOCK, 0, s>>>(reinterpret_cast<u32*>(ref), nv_total, 0u);
        mark_referenced_kernel<<<grid_for(std::max(3 * nf_bound, 1), 8192), BLOCK, 0, s>>>(c->fbuf[cur], c->st, cur, ref);
        const RefPred rp{ref};
        const RefOut ro{c->newid};
        prim::compact(s, rp, rp, ro, &c->st->nv[cur], nv_total, c->tilesum, &c->st->nv_kept);
        copy_out_kernel<true><<<out_grid, BLOCK, 0, s>>>(c->vrec[cur], c->fbuf[cur], c->cid, c->st, cur, N, d_verts_out,
                                                         d_facets_out, d_cluster_id, B, c->voff[cur], c->foff_out, ref,
                                                         c->newid, c->matched);
    } else {
        copy_out_kernel<false><<<out_grid, BLOCK, 0, s>>>(c->vrec[cur], c->fbuf[cur], c->cid, c->st, cur, N, d_verts_out,
                                                          d_facets_out, d_cluster_id, B, c->voff[cur], c->foff_out,
                                                          nullptr, nullptr, nullptr);
    }
    if (stats) HIP_TRY(c, hipEventRecord(c->ev_total[1], s));
    rc = read_header(c, s);
    if (rc != PICASSO_OK) return rc;
    if (hst->err & ERR_BIT_INTERNAL) return PICASSO_ERR_INTERNAL;  // (the publishing kernel has cleared the flag)
    // the events of the measurement options are read below; all were recorded before the last kernel,
    // so waiting for the last of them returns at once and leaves every one of them readable
    if (stats) HIP_TRY(c, hipEventSynchronize(c->ev_total[1]));
    else if (c->kt.nrec > 0) HIP_TRY(c, hipEventSynchronize(c->kt_pool[c->kt.recs[c->kt.nrec - 1].e1]));
    HIP_TRY(c, hipGetLastError());
    const int* h_foff = c->h_pin + HDR_STATE_INTS + c->cap_b;

    // the bracketed kernels: event times and the algorithmic bytes of their rounds (see picasso_timed_kernel)
    for (int i = 0; i < c->kt.nrec; ++i) {
        const prim::LaunchTimer::Rec& r = c->kt.recs[i];
        const int kernel = r.tag >> 8, rd = r.tag & 0xFF;
        float ms = 0.f;
        if (kernel < PICASSO_KERNEL_COUNT && rd < c->n_rounds_noted &&
            hipEventElapsedTime(&ms, c->kt_pool[r.e0], c->kt_pool[r.e1]) == hipSuccess) {
            const double nv = c->nv_round[rd], nf = c->nf_round[rd], ne = c->ne_round[rd], H = 3.0 * nf;
            double bytes = 0.0;
            switch (kernel) {
                case PICASSO_KERNEL_SORT: bytes = 16.0 * H; break;
                case PICASSO_KERNEL_UNIQUE_COST: bytes = 8.0 * H + 13.0 * ne + 72.0 * nv; break;
                case PICASSO_KERNEL_SUBROUND0: bytes = 14.0 * ne + 24.0 * nv; break;
                case PICASSO_KERNEL_FACET_INSERT: bytes = 32.0 * nf + 4.0 * nv + 8.0 * (double)N; break;
                case PICASSO_KERNEL_SORT_INCIDENCE: bytes = 48.0 * (double)F; break;
                default: bytes = 24.0 * (double)F + 16.0 * (double)F + 76.0 * (double)N; break;  // QUADRIC_ROWS
            }
            c->kt_launches[kernel] += 1;
            c->kt_ms[kernel] += ms;
            c->kt_bytes[kernel] += bytes;
        }
    }

    int warn = PICASSO_OK;
    for (int b = 0; b < B; ++b) {
        // (with degenerated vertices dropped, the last kernels have left the meshes' counts where the pair counts were)
        h_nv_out[b] = c->opt_drop_degenerated ? c->h_pin[HDR_STATE_INTS + b] : nvb[b];
        h_nf_out[b] = h_foff[b + 1] - h_foff[b];
        if (nvb[b] > target_nv[b] && (c->opt_max_rounds < 0 || stuck[b])) warn = PICASSO_WARN_BUDGET_UNMET;
    }
    if (stats) {
        stats->rounds = round;
        stats->nv_out = c->opt_drop_degenerated ? hst->nv_kept : hst->nv[cur];
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
    const int Q = vec4 ? C / 4 : C;  // channel packs; a stage-1 launch takes up to pool::BLOCK of them
    const size_t cap = (size_t)3 * (size_t)c->max_facets * sizeof(u64) / sizeof(float);  // floats in key64[0]
    const size_t per_group = (size_t)ROWS * C;
    if (per_group > cap) return PICASSO_ERR_WORKSPACE;
    const int R = pool::BLOCK / std::min(Q, pool::BLOCK);
    long long groups = std::min<long long>(1024, ((long long)n_rows + 4ll * R - 1) / (4ll * R));
    groups = std::max<long long>(1, std::min<long long>(groups, (long long)(cap / per_group)));
    const int chunk = (int)(((long long)n_rows + groups - 1) / groups);
    float* partial = reinterpret_cast<float*>(c->key64[0]);
    const size_t lds = (size_t)pool::BLOCK * ROWS * (vec4 ? 4 : 1) * sizeof(float);
    for (int q0 = 0; q0 < Q; q0 += pool::BLOCK) {
        const int qn = std::min(pool::BLOCK, Q - q0);
        if (vec4)
            conv::reduce_rows_stage1_kernel<ROWS, 4, Term><<<(int)groups, pool::BLOCK, lds, s>>>(term, n_rows, C, chunk, partial, q0, qn);
        else
            conv::reduce_rows_stage1_kernel<ROWS, 1, Term><<<(int)groups, pool::BLOCK, lds, s>>>(term, n_rows, C, chunk, partial, q0, qn);
    }
    conv::reduce_rows_stage2_kernel<<<pool::grid_for((long long)rows_used * C * 64), pool::BLOCK, 0, s>>>(
        partial, (int)groups, ROWS, rows_used, C, d_out);
    return PICASSO_OK;
}

}  // namespace

// Scratch of picasso_replace_mapping_static (the entry point for callers that cannot allocate):
// the smallest member of every cluster, then (a cache line further) the bad-index flag.  In host
// code this name is only a handle for hipGetSymbolAddress; kernels get the looked-up address.
static __device__ __align__(256) int scratch[PICASSO_STATIC_MAX_CLUSTERS + 64];

namespace {
constexpr int STATIC_MAX_DEVICES = 64;
std::atomic<int*> scratch_ptr[STATIC_MAX_DEVICES];  // per device: where its copy of `scratch` lies (null: not looked up yet)
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
    c->h_mesh = new (std::nothrow) int[6 * (size_t)max_meshes];
    if (!c->h_mesh) {
        (void)hipFree(c->ws);
        delete c;
        return PICASSO_ERR_HIP;
    }
    c->h_up_off = (size_t)HDR_STATE_INTS + 2 * (size_t)max_meshes + 16;
    c->h_seq_off = (c->h_up_off + HDR_STATE_INTS + 8 * (size_t)max_meshes + 16 + 31) / 32 * 32;
    c->h_pin_ints = c->h_seq_off + 32;
    // (mapped into the device's address space and coherent with it: kernels store there what the host reads while they run)
    if (hipHostMalloc((void**)&c->h_pin, c->h_pin_ints * sizeof(int), hipHostMallocMapped | hipHostMallocCoherent) != hipSuccess) {
        (void)hipFree(c->ws);
        delete[] c->h_mesh;
        delete c;
        return PICASSO_ERR_HIP;
    }
    memset(c->h_pin, 0, c->h_pin_ints * sizeof(int));
    // the incidence sort's digit counts start at zero; every S0 leaves them at zero again.  So do the
    // header's error flags (see HeaderInit).
    if (hipMemset(c->hist12_s0, 0, sizeof(u32) * 2 * prim::MSD_HIST_WORDS) != hipSuccess ||
        hipMemset(c->hdr, 0, sizeof(int) * (HDR_STATE_INTS + 8 * (size_t)max_meshes + 3)) != hipSuccess) {
        (void)hipHostFree(c->h_pin);
        (void)hipFree(c->ws);
        delete[] c->h_mesh;
        delete c;
        return PICASSO_ERR_HIP;
    }
    if (hipHostGetDevicePointer((void**)&c->h_pin_dev, c->h_pin, 0) != hipSuccess) {
        (void)hipHostFree(c->h_pin);
        (void)hipFree(c->ws);
        delete[] c->h_mesh;
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
    delete[] c->h_mesh;
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
        case PICASSO_OPT_HOST_POLL:
            if (value < 0 || value > 10000000) return PICASSO_ERR_INVALID_ARG;
            c->opt_poll_us = value == 1 ? 20000 : value;
            return PICASSO_OK;
        case PICASSO_OPT_LAUNCH_AHEAD:
            if (value != 0 && value != 1) return PICASSO_ERR_INVALID_ARG;
            c->opt_ahead = (int)value;
            return PICASSO_OK;
        case PICASSO_OPT_DROP_DEGENERATED:
            if (value != 0 && value != 1) return PICASSO_ERR_INVALID_ARG;
            c->opt_drop_degenerated = (int)value;
            return PICASSO_OK;
        case PICASSO_OPT_TRUNC_SELECT:
            if (value != 0 && value != 1) return PICASSO_ERR_INVALID_ARG;
            c->opt_trunc_select = (int)value;
            return PICASSO_OK;
        case PICASSO_OPT_TRUNC_WIDTH:
            if (value != 0 && value != 4 && value != 8 && value != 16 && value != 32) return PICASSO_ERR_INVALID_ARG;
            c->opt_trunc_width = (int)value;
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
        case PICASSO_ERR_INTERNAL: return "internal error: a kernel met sizes that its launch does not take";
        default: return "unknown status";
    }
}

const char* picasso_last_hip_error(picasso_ctx* c) { return c ? c->hip_err : ""; }

int picasso_kernel_timing(picasso_ctx* c, int kernel, int reset, int64_t* launches, double* ms_total,
                          double* bytes_total) {
    if (!c || kernel < 0 || kernel >= PICASSO_KERNEL_COUNT) return PICASSO_ERR_INVALID_ARG;
    if (launches) *launches = c->kt_launches[kernel];
    if (ms_total) *ms_total = c->kt_ms[kernel];
    if (bytes_total) *bytes_total = c->kt_bytes[kernel];
    if (reset) {
        c->kt_launches[kernel] = 0;
        c->kt_ms[kernel] = 0.0;
        c->kt_bytes[kernel] = 0.0;
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

int picasso_f2f_forward(picasso_ctx* c, void* stream, const float* d_tex, const float* d_bary, const int32_t* d_poff,
                        int32_t F, int32_t P, int32_t C, const float* d_w, float* d_y) {
    if (!c || !d_tex || !d_bary || !d_poff || F < 1 || P < 0 || C < 1 || !d_w || !d_y) return PICASSO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    if (conv_vec4(C, {d_tex, d_w, d_y}))
        conv::f2f_forward_kernel<4><<<pool::grid_for((long long)F * (C / 4)), pool::BLOCK, 0, s>>>(d_tex, d_bary, d_poff, F, P, C, d_w, d_y);
    else
        conv::f2f_forward_kernel<1><<<pool::grid_for((long long)F * C), pool::BLOCK, 0, s>>>(d_tex, d_bary, d_poff, F, P, C, d_w, d_y);
    HIP_TRY(c, hipGetLastError());
    return PICASSO_OK;
}

int picasso_f2f_backward(picasso_ctx* c, void* stream, const float* d_gy, const float* d_tex, const float* d_bary,
                         const int32_t* d_poff, int32_t F, int32_t P, int32_t C, const float* d_w, float* d_gtex,
                         float* d_gw) {
    if (!c || !d_gy || !d_tex || !d_bary || !d_poff || F < 1 || P < 0 || C < 1 || !d_w || (!d_gtex && !d_gw))
        return PICASSO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    const bool vec4 = conv_vec4(C, {d_gy, d_tex, d_w, d_gtex});
    if (d_gtex) {
        if (vec4)
            conv::f2f_backward_tex_kernel<4><<<pool::grid_for((long long)F * (C / 4)), pool::BLOCK, 0, s>>>(d_gy, d_bary, d_poff, F, P, C, d_w, d_gtex);
        else
            conv::f2f_backward_tex_kernel<1><<<pool::grid_for((long long)F * C), pool::BLOCK, 0, s>>>(d_gy, d_bary, d_poff, F, P, C, d_w, d_gtex);
    }
    if (d_gw) {
        conv::F2fWeightTerm term{d_gy, d_tex, d_bary, d_poff, C, P};
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
    const int grid = conv::xcd_grid((long long)N * (vec8 ? C / 8 : (vec4 ? C / 4 : C)));
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
    if (!c || !d_cluster_id || n_in < 1 || n_out < 0 || !d_replace || !d_mapping) return PICASSO_ERR_INVALID_ARG;
    if (n_out > c->max_verts) return PICASSO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(c, hipSetDevice(c->device));
    prim::fill_u32_kernel<<<1, BLOCK, 0, s>>>(reinterpret_cast<u32*>(&c->st->err), 1, 0u);
    if (n_out > 0)
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

int picasso_replace_mapping_static(int device, void* stream, const int32_t* d_cluster_id, int32_t n_in, int32_t n_out,
                                   int32_t* d_replace, int32_t* d_mapping, int32_t* d_status) {
    if (device < 0 || device >= STATIC_MAX_DEVICES || !d_cluster_id || n_in < 1 || n_out < 0 || !d_replace ||
        !d_mapping || !d_status)
        return PICASSO_ERR_INVALID_ARG;
    if (n_out > PICASSO_STATIC_MAX_CLUSTERS) return PICASSO_ERR_WORKSPACE;
    if (hipSetDevice(device) != hipSuccess) return PICASSO_ERR_HIP;
    // every device holds its own copy of the array at its own address: looked up once per device, with
    // that device current; from here on only that address is used, never the array's name
    int* ptr = scratch_ptr[device].load(std::memory_order_acquire);
    if (!ptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PICASSO_ERR_HIP;
        ptr = static_cast<int*>(p);
        scratch_ptr[device].store(ptr, std::memory_order_release);
    }
    hipStream_t s = (hipStream_t)stream;
    int* first = ptr;
    int* flag = ptr + PICASSO_STATIC_MAX_CLUSTERS;
    // the array keeps the last call's contents: what this call reads starts from its own fill
    // (a kernel, not a memset command, so that the call can be recorded into a graph)
    pool::static_begin_kernel<<<pool::grid_for(n_out), pool::BLOCK, 0, s>>>(first, n_out, flag);
    pool::cluster_first_kernel<<<pool::grid_for(n_in), pool::BLOCK, 0, s>>>(d_cluster_id, n_in, n_out, first, flag);
    pool::replace_mapping_status_kernel<<<pool::grid_for(n_in), pool::BLOCK, 0, s>>>(
        d_cluster_id, n_in, n_out, first, flag, d_replace, d_mapping, d_status, PICASSO_OK, PICASSO_ERR_BAD_INDEX);
    return hipGetLastError() == hipSuccess ? PICASSO_OK : PICASSO_ERR_HIP;
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
