// primitives.h -- wave64 device primitives for gfx950: block scans, a stable
// LSD radix sort (upsweep / row scan / downsweep per digit pass) and a
// flag-compaction "scan" built from two kernels.  No kernel here waits on
// another workgroup: all cross-workgroup ordering is by kernel boundaries.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include <stdint.h>

namespace prim {

typedef unsigned long long u64;
typedef uint32_t u32;

constexpr int BLOCK = 256;  // 4 wavefronts of 64 lanes
constexpr int WAVES = BLOCK / 64;

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }
__device__ __forceinline__ int wave_id() { return (int)(threadIdx.x >> 6); }
__device__ __forceinline__ u64 lanemask_lt() { return (1ull << lane_id()) - 1ull; }

// For a lane with `ok`: the lanes of its wave (itself included) that hold the same digit `d`, worked out
// for the first WAVE_DIGIT_PEEL distinct digits among the wave's lanes; a lane whose digit comes after
// those is left alone in its mask.  Lanes without `ok` get 0.  Keys in mesh order mostly bring one to
// three distinct leading digits into a wave, so one LDS atomic per digit (by the first lane of each
// mask, adding the mask's population) replaces up to 64 atomics on the same address.  By all lanes.
constexpr int WAVE_DIGIT_PEEL = 4;
__device__ __forceinline__ u64 wave_same_digit_lanes(bool ok, u32 d) {
    u64 rem = __ballot(ok);
    u64 mine = ok ? (1ull << lane_id()) : 0ull;
#pragma unroll
    for (int j = 0; j < WAVE_DIGIT_PEEL; ++j) {
        if (rem == 0) break;
        const int lead = __ffsll((long long)rem) - 1;
        const u32 d0 = (u32)__builtin_amdgcn_readlane((int)d, lead);
        const u64 m = __ballot(ok && d == d0);
        if (ok && d == d0) mine = m;
        rem &= ~m;
    }
    return mine;
}

// Reads a count that lives either on the device (n_ptr) or in the launch arguments.
__device__ __forceinline__ int load_count(const int* n_ptr, int n_host) { return n_ptr ? *n_ptr : n_host; }

// Exclusive prefix sum of one value per thread over a 256-thread block.
// `total` receives the block sum.  smem must hold WAVES words.  Contains barriers.
__device__ __forceinline__ u32 block_exclusive_scan(u32 v, u32* smem, u32& total) {
    const int lane = lane_id(), w = wave_id();
    u32 incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        u32 o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
    }
    __syncthreads();  // smem may still be in use by a previous call
    if (lane == 63) smem[w] = incl;
    __syncthreads();
    u32 woff = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
        u32 s = smem[i];
        if (i < w) woff += s;
        tot += s;
    }
    total = tot;
    return woff + incl - v;
}

__device__ __forceinline__ u32 block_sum(u32 v, u32* smem) {
    const int lane = lane_id(), w = wave_id();
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    __syncthreads();
    if (lane == 0) smem[w] = v;
    __syncthreads();
    u32 tot = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) tot += smem[i];
    return tot;
}

// ---------------------------------------------------------------------------
// Radix sort.  Tile = 4096 keys per workgroup.  Within a tile the order of the
// keys is (wave, item, lane), which equals their index order, so ranking by
// (digit, that order) keeps the sort stable.
// ---------------------------------------------------------------------------
// Keys per lane: 16 for large inputs, 4 when the input is small enough that
// 4096-key tiles would leave most compute units without a workgroup.
constexpr int SORT_ITEMS_BIG = 16;
constexpr int SORT_ITEMS_SMALL = 4;
constexpr int SORT_SMALL_MAX_TILES = 2048;

template <typename K>
__device__ __forceinline__ u32 digit_of(K k, int shift, u32 mask) {
    return (u32)(k >> shift) & mask;
}

// Stable ranks of a wave's keys among the wave's keys with the same digit.  digit[i] is the
// digit of the lane's i-th key (keys are ordered by (item, lane)); wrow[d] accumulates this
// wave's count of digit d and must be zero on entry.  On return rank[i] = number of the wave's
// earlier keys with the same digit.  Lanes that hold one digit are found with ballots; the first
// of them adds their number to wrow[d] with one LDS atomic, whose return value (the count left by
// the earlier items: LDS operations of a wave complete in order) it then hands to the others.
// Four items go through together so that four atomics are in flight instead of one.
constexpr int WAVE_RANK_MAX_BITS = 9;  // widest digit wave_rank_digits takes

template <int ITEMS>
__device__ __forceinline__ void wave_rank_digits(const u32 (&digit)[ITEMS], int items, int bits, u32* wrow,
                                                 u32 (&rank)[ITEMS]) {
    constexpr int GROUP = ITEMS < 4 ? ITEMS : 4;
    const u64 lt = lanemask_lt();
#pragma unroll
    for (int i0 = 0; i0 < ITEMS; i0 += GROUP) {
        if (i0 >= items) break;
        u32 below[GROUP], old[GROUP];
        int leader[GROUP];
#pragma unroll
        for (int j = 0; j < GROUP; ++j) {
            old[j] = 0;
            if (i0 + j < items) {
                const u32 d = digit[i0 + j];
                // lanes whose digit differs from this lane's in some bit: per bit, the ballot of the
                // bit XOR this lane's own bit spread over a word (unrolled; `bits` is wave-uniform)
                u32 dlo = 0, dhi = 0;
#pragma unroll
                for (int b = 0; b < WAVE_RANK_MAX_BITS; ++b) {
                    if (b < bits) {
                        const int own = (int)(d << (31 - b)) >> 31;  // 0 or -1
                        const u64 bal = __ballot(own != 0);
                        dlo |= (u32)bal ^ (u32)own;
                        dhi |= (u32)(bal >> 32) ^ (u32)own;
                    }
                }
                const u64 m = ~(((u64)dhi << 32) | dlo);  // lanes of this wave holding the same digit
                below[j] = (u32)__popcll(m & lt);
                leader[j] = __ffsll((long long)m) - 1;
                if (below[j] == 0) old[j] = atomicAdd(&wrow[d], (u32)__popcll(m));
            }
        }
#pragma unroll
        for (int j = 0; j < GROUP; ++j)
            if (i0 + j < items) rank[i0 + j] = (u32)__shfl((int)old[j], leader[j], 64) + below[j];
    }
}

// table[d * T + tile] = number of keys of this tile whose digit is d
template <typename K, int SORT_ITEMS>
__global__ __launch_bounds__(BLOCK) void radix_upsweep_kernel(const K* __restrict__ kin, const int* n_ptr, int n_host,
                                                              int T, u32* __restrict__ table, int shift, int bits) {
    constexpr int SORT_TILE = BLOCK * SORT_ITEMS;
    __shared__ u32 hist[WAVES][256];
    const int n = load_count(n_ptr, n_host);
    const int tile = blockIdx.x;
    const long long base = (long long)tile * SORT_TILE;
    if (base >= n) return;
    const int t = threadIdx.x, w = wave_id();
    const u32 R = 1u << bits, dmask = R - 1;
    for (int i = t; i < WAVES * 256; i += BLOCK) (&hist[0][0])[i] = 0;
    __syncthreads();
    // a digit narrower than 8 bits leaves room for 256/R copies of the histogram per wave:
    // lanes spread over the copies, so fewer of them meet on one LDS word
    const u32 copy = ((u32)lane_id() & ((256u >> bits) - 1u)) << bits;
#pragma unroll 4
    for (int i = 0; i < SORT_ITEMS; ++i) {
        long long idx = base + (long long)i * BLOCK + t;
        if (idx < n) atomicAdd(&hist[w][copy | digit_of<K>(kin[idx], shift, dmask)], 1u);
    }
    __syncthreads();
    if ((u32)t < R) {
        u32 sum = 0;
        for (u32 c = (u32)t; c < 256u; c += R) sum += hist[0][c] + hist[1][c] + hist[2][c] + hist[3][c];
        table[(size_t)t * T + tile] = sum;
    }
}

// One workgroup per digit: exclusive scan of its table row over the tiles in
// use; totals[d] = number of keys with digit d.
__global__ __launch_bounds__(BLOCK) void radix_scan_kernel(u32* __restrict__ table, u32* __restrict__ totals,
                                                           const int* n_ptr, int n_host, int T, int tile_keys) {
    __shared__ u32 smem[WAVES];
    const int n = load_count(n_ptr, n_host);
    const int tiles = (int)(((long long)n + tile_keys - 1) / tile_keys);
    u32* row = table + (size_t)blockIdx.x * T;
    const int t = threadIdx.x;
    u32 carry = 0;
    for (int c = 0; c < tiles; c += BLOCK) {
        const int i = c + t;
        u32 v = (i < tiles) ? row[i] : 0u;
        u32 tot;
        u32 ex = block_exclusive_scan(v, smem, tot);
        if (i < tiles) row[i] = carry + ex;
        carry += tot;
    }
    if (t == 0) totals[blockIdx.x] = carry;
}

template <typename K, bool HAS_VAL, int SORT_ITEMS>
__global__ __launch_bounds__(BLOCK) void radix_downsweep_kernel(const K* __restrict__ kin, K* __restrict__ kout,
                                                                const u32* __restrict__ vin, u32* __restrict__ vout,
                                                                const int* n_ptr, int n_host, int T,
                                                                const u32* __restrict__ table,
                                                                const u32* __restrict__ totals, int shift, int bits) {
    constexpr int SORT_TILE = BLOCK * SORT_ITEMS;
    __shared__ u32 wcnt[WAVES][256];
    __shared__ u32 tstart[256];
    __shared__ u32 gbase[256];
    __shared__ u32 smem[WAVES];
    __shared__ K skey[SORT_TILE];
    __shared__ u32 sval[HAS_VAL ? SORT_TILE : 1];

    const int n = load_count(n_ptr, n_host);
    const int tile = blockIdx.x;
    const long long base = (long long)tile * SORT_TILE;
    if (base >= n) return;
    const int t = threadIdx.x, w = wave_id(), lane = lane_id();
    const u32 R = 1u << bits, dmask = R - 1;

    for (int i = t; i < WAVES * 256; i += BLOCK) (&wcnt[0][0])[i] = 0;

    K key[SORT_ITEMS];
    u32 val[SORT_ITEMS];
    u32 rank[SORT_ITEMS];
#pragma unroll
    for (int i = 0; i < SORT_ITEMS; ++i) {
        long long idx = base + (long long)w * (64 * SORT_ITEMS) + i * 64 + lane;
        bool ok = idx < n;
        key[i] = ok ? kin[idx] : (K) ~(K)0;  // padding sorts last within the tile
        if (HAS_VAL) val[i] = ok ? vin[idx] : 0u;
    }
    __syncthreads();

    {
        u32 digit[SORT_ITEMS];
#pragma unroll
        for (int i = 0; i < SORT_ITEMS; ++i) digit[i] = digit_of<K>(key[i], shift, dmask);
        wave_rank_digits<SORT_ITEMS>(digit, SORT_ITEMS, bits, wcnt[w], rank);
    }
    __syncthreads();

    // per digit: wave counts -> exclusive offsets over waves, tile histogram
    u32 tot = 0;
    if ((u32)t < R) {
        u32 c0 = wcnt[0][t], c1 = wcnt[1][t], c2 = wcnt[2][t], c3 = wcnt[3][t];
        wcnt[0][t] = 0;
        wcnt[1][t] = c0;
        wcnt[2][t] = c0 + c1;
        wcnt[3][t] = c0 + c1 + c2;
        tot = c0 + c1 + c2 + c3;
    }
    u32 dummy;
    const u32 ex = block_exclusive_scan(tot, smem, dummy);
    const u32 gtot = ((u32)t < R) ? totals[t] : 0u;
    const u32 dbase = block_exclusive_scan(gtot, smem, dummy);
    if ((u32)t < R) {
        tstart[t] = ex;
        gbase[t] = dbase + table[(size_t)t * T + tile] - ex;
    }
    __syncthreads();

#pragma unroll
    for (int i = 0; i < SORT_ITEMS; ++i) {
        const u32 d = digit_of<K>(key[i], shift, dmask);
        const u32 p = tstart[d] + wcnt[w][d] + rank[i];
        skey[p] = key[i];
        if (HAS_VAL) sval[p] = val[i];
    }
    __syncthreads();

    const long long rem = (long long)n - base;
    const int nvalid = rem < SORT_TILE ? (int)rem : SORT_TILE;
    for (int q = t; q < nvalid; q += BLOCK) {
        const K k = skey[q];
        const u32 o = gbase[digit_of<K>(k, shift, dmask)] + (u32)q;
        kout[o] = k;
        if (HAS_VAL) vout[o] = sval[q];
    }
}

struct SortScratch {
    u32* table;   // [256 * T]
    u32* totals;  // [256]
    int T;        // row stride = tiles at capacity
};

// Optional hipEvent bracket around the launches of the sort's main streaming
// kernel (the per-bucket sort; the scatter passes when plain LSD is used), for
// the roofline measurement of the benchmark; `tag` travels to the record.
struct LaunchTimer {
    hipEvent_t* pool = nullptr;
    int cap = 0, used = 0;
    struct Rec { int e0, e1, tag; };
    Rec* recs = nullptr;
    int nrec = 0;
    bool begin(hipStream_t s, int tag) {
        if (!pool || used + 2 > cap) return false;
        recs[nrec] = Rec{used, used + 1, tag};
        (void)hipEventRecord(pool[used], s);
        used += 2;
        return true;
    }
    void end(hipStream_t s) {
        (void)hipEventRecord(pool[recs[nrec].e1], s);
        ++nrec;
    }
};

inline int sort_items_for(long long n_max) {
    return (n_max + BLOCK * SORT_ITEMS_SMALL - 1) / (BLOCK * SORT_ITEMS_SMALL) <= SORT_SMALL_MAX_TILES ? SORT_ITEMS_SMALL
                                                                                                      : SORT_ITEMS_BIG;
}
inline int sort_tiles(long long n, int items) { return (int)((n + (long long)BLOCK * items - 1) / ((long long)BLOCK * items)); }
// row stride of the tile table for inputs of up to n_cap keys
inline int sort_table_stride(long long n_cap) {
    const int big = sort_tiles(n_cap, SORT_ITEMS_BIG);
    return big > SORT_SMALL_MAX_TILES ? big : SORT_SMALL_MAX_TILES;
}

template <typename K, bool HAS_VAL, int ITEMS>
inline int radix_sort_impl(hipStream_t s, K* k0, K* k1, u32* v0, u32* v1, const int* n_ptr, int n_max, int key_bits,
                           const SortScratch& sc, LaunchTimer* lt, int tag) {
    const int passes = (key_bits + 7) / 8;
    const int per = (key_bits + passes - 1) / passes;
    const int tiles = sort_tiles(n_max, ITEMS);
    int cur = 0, shift = 0;
    for (int p = 0; p < passes; ++p) {
        const int bits = (key_bits - shift) < per ? (key_bits - shift) : per;
        K* kin = cur ? k1 : k0;
        K* kout = cur ? k0 : k1;
        u32* vin = cur ? v1 : v0;
        u32* vout = cur ? v0 : v1;
        radix_upsweep_kernel<K, ITEMS><<<tiles, BLOCK, 0, s>>>(kin, n_ptr, n_max, sc.T, sc.table, shift, bits);
        radix_scan_kernel<<<1 << bits, BLOCK, 0, s>>>(sc.table, sc.totals, n_ptr, n_max, sc.T, BLOCK * ITEMS);
        const bool timed = lt && lt->begin(s, tag);
        radix_downsweep_kernel<K, HAS_VAL, ITEMS>
            <<<tiles, BLOCK, 0, s>>>(kin, kout, vin, vout, n_ptr, n_max, sc.T, sc.table, sc.totals, shift, bits);
        if (timed) lt->end(s);
        shift += bits;
        cur ^= 1;
    }
    if (hipGetLastError() != hipSuccess) return -1;
    return cur;
}

// Sorts on key bits [0, key_bits).  Data ping-pongs between (k0,v0) and
// (k1,v1); returns 0 if the result is in (k0,v0), 1 if in (k1,v1), <0 on a
// launch error.  n_max bounds the device-side count for the grid size.
template <typename K, bool HAS_VAL>
inline int radix_sort(hipStream_t s, K* k0, K* k1, u32* v0, u32* v1, const int* n_ptr, int n_max, int key_bits,
                      const SortScratch& sc, LaunchTimer* lt = nullptr, int tag = 0) {
    if (n_max <= 0 || key_bits <= 0) return 0;
    if (sort_items_for(n_max) == SORT_ITEMS_SMALL)
        return radix_sort_impl<K, HAS_VAL, SORT_ITEMS_SMALL>(s, k0, k1, v0, v1, n_ptr, n_max, key_bits, sc, lt, tag);
    return radix_sort_impl<K, HAS_VAL, SORT_ITEMS_BIG>(s, k0, k1, v0, v1, n_ptr, n_max, key_bits, sc, lt, tag);
}

// ---------------------------------------------------------------------------
// Bucket sort for inputs of up to BUCKET_SORT_MAX_KEYS keys whose leading bits
// are spread evenly (vertex ids): one stable radix pass on the TOP 8 bits
// splits the keys into 256 buckets, then each bucket is sorted on the
// remaining bits by one workgroup entirely in LDS (register-staged LSD passes
// over a single LDS array).  Two sweeps over memory instead of one per 8 bits,
// and 4 launches instead of 3 per 8 bits.  A bucket that does not fit in LDS
// (a very uneven key distribution) is sorted by the same workgroup with a slow
// pass-by-pass LSD over global memory, so the result is always correct.
// ---------------------------------------------------------------------------
constexpr int BUCKET_THREADS_256 = 1024;  // 256 buckets: 8 keys per lane, up to 8192 keys of a bucket held in LDS
constexpr int BUCKET_THREADS_4096 = 512;  // 4096 buckets: up to 4096 keys (8 per lane), or 8192 key-value
                                          // pairs (16 per lane: vertex incidences run to ~6 per vertex and
                                          // vertex ids need not fill their bit range, so those buckets run fuller)
// keys without values (bucket_keys_kernel): lanes and keys per lane of a bucket's workgroup
constexpr int BUCKET_KEYS_THREADS_256 = 512, BUCKET_KEYS_ITEMS_256 = 16;   // 256 buckets: up to 8192 keys in LDS
constexpr int BUCKET_KEYS_THREADS_4096 = 256, BUCKET_KEYS_ITEMS_4096 = 16;  // 4096 buckets: up to 4096 keys in LDS
constexpr int BUCKET_MSD_BITS = 8;
constexpr long long BUCKET_SORT_MAX_KEYS = 1ll << 20;  // average bucket <= half of what LDS holds

template <int NW>
__device__ __forceinline__ u32 wide_block_exclusive_scan(u32 v, u32* smem, u32& total) {
    const int lane = lane_id(), w = wave_id();
    u32 incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        u32 o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
    }
    __syncthreads();
    if (lane == 63) smem[w] = incl;
    __syncthreads();
    u32 woff = 0, tot = 0;
    for (int i = 0; i < NW; ++i) {
        u32 x = smem[i];
        if (i < w) woff += x;
        tot += x;
    }
    total = tot;
    return woff + incl - v;
}

template <typename K>
__device__ __forceinline__ K coherent_load(const K* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Slow path for a bucket larger than BUCKET_CAP: stable LSD over global memory
// by this workgroup alone; wave 0 places the keys 64 at a time in order.
template <typename K, bool HAS_VAL, int BUCKET_THREADS>
__device__ void bucket_sort_oversize(K* a, K* b, u32* va, u32* vb, int cnt, int low_bits, u32* hist /*[256]*/,
                                     u32* smem) {
    constexpr int BUCKET_WAVES = BUCKET_THREADS / 64;
    // data starts in b (the partition pass wrote it there) and must end in a
    K* src = b;
    K* dst = a;
    u32* vsrc = vb;
    u32* vdst = va;
    const int passes = (low_bits + 7) / 8;
    const int per = (low_bits + passes - 1) / passes;
    const int t = threadIdx.x, lane = lane_id();
    int shift = 0;
    for (int p = 0; p < passes; ++p) {
        const int bits = (low_bits - shift) < per ? (low_bits - shift) : per;
        const u32 R = 1u << bits, dmask = R - 1;
        if (t < 256) hist[t] = 0;
        __syncthreads();
        for (int i = t; i < cnt; i += BUCKET_THREADS) atomicAdd(&hist[digit_of<K>(coherent_load(&src[i]), shift, dmask)], 1u);
        __syncthreads();
        u32 tot;
        const u32 c = (t < 256 && (u32)t < R) ? hist[t] : 0u;
        const u32 ex = wide_block_exclusive_scan<BUCKET_WAVES>(c, smem, tot);
        __syncthreads();
        if (t < 256) hist[t] = ex;  // running output position of each digit
        __syncthreads();
        if (t < 64) {
            for (int base = 0; base < cnt; base += 64) {
                const int i = base + lane;
                const bool ok = i < cnt;
                const K k = ok ? coherent_load(&src[i]) : (K)0;
                const u32 d = ok ? digit_of<K>(k, shift, dmask) : 0xFFFFFFFFu;
                u64 m = __ballot(ok);
                for (int bb = 0; bb < bits; ++bb) {
                    const bool bit = (d >> bb) & 1u;
                    const u64 bal = __ballot(bit);
                    m &= bit ? bal : ~bal;
                }
                if (ok) {
                    const u32 below = (u32)__popcll(m & lanemask_lt());
                    const u32 old = hist[d];
                    __builtin_amdgcn_wave_barrier();
                    if (below == 0) hist[d] = old + (u32)__popcll(m);
                    __builtin_amdgcn_wave_barrier();
                    dst[old + below] = k;
                    if (HAS_VAL) vdst[old + below] = coherent_load(&vsrc[i]);
                }
            }
        }
        __threadfence();
        __syncthreads();
        K* tk = src; src = dst; dst = tk;
        u32* tv = vsrc; vsrc = vdst; vdst = tv;
        shift += bits;
    }
    if (src != a) {  // an even number of passes left the result in b
        for (int i = t; i < cnt; i += BUCKET_THREADS) {
            a[i] = coherent_load(&src[i]);
            if (HAS_VAL) va[i] = coherent_load(&vsrc[i]);
        }
    }
}

// One workgroup per bucket.  kin/vin hold the keys partitioned by their top
// digit (bucket d occupies [start_d, start_d + totals[d])); the sorted bucket is
// written to the same range of kout/vout.  low_bits = key bits below the digit.
//
// The bucket is held in LDS.  One stable radix pass on the TOP (up to) 9 of the
// low bits splits it into up to 512 groups of keys that agree on all bits
// sorted so far; with vertex-pair keys a group is the handful of half-edges of
// one lower vertex.  Each group is then finished by one lane with a stable
// sort on the whole key (by counting ranks in registers for up to 16 keys,
// by insertion in place beyond), which for such groups costs far less than
// the two or three more radix passes over every key that the remaining bits
// would take (a radix pass spends one wave-wide ballot per key and bit).  If
// some group is long (keys crowded on few values of those 9 bits), the
// workgroup runs plain LSD radix passes over all the low bits instead.
constexpr int BUCKET_GROUP_BITS = 9;
constexpr int BUCKET_GROUP_MAX = 64;  // longest group the insertion sort is allowed

// Stable sort of the g <= G keys at [gs, gs + g) of an LDS array by one lane: the keys are read into
// registers together, each key's place is the number of keys that must precede it (G x G
// comparisons, none of which waits for memory), and the keys are written back to their places.
template <typename K, bool HAS_VAL, int G>
__device__ __forceinline__ void group_rank_sort(K* skey, u32* sval, int gs, int g) {
    K k[G];
    u32 v[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        k[j] = j < g ? skey[gs + j] : (K)0;
        v[j] = (HAS_VAL && j < g) ? sval[gs + j] : 0u;
    }
#pragma unroll
    for (int i = 0; i < G; ++i) {
        if (i < g) {
            int r = 0;
#pragma unroll
            for (int j = 0; j < G; ++j) r += (j < g && (k[j] < k[i] || (k[j] == k[i] && j < i))) ? 1 : 0;
            skey[gs + r] = k[i];
            if (HAS_VAL) sval[gs + r] = v[i];
        }
    }
}

// The same for keys without values (so that equal keys need no order among themselves): a bitonic
// sorting network over G registers, G a power of two, empty places filled with the largest key.
template <typename K, int G>
__device__ __forceinline__ void group_network_sort(K* skey, int gs, int g) {
    K k[G];
#pragma unroll
    for (int j = 0; j < G; ++j) k[j] = j < g ? skey[gs + j] : (K) ~(K)0;
#pragma unroll
    for (int size = 2; size <= G; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const int l = i ^ stride;
                if (l > i) {
                    const bool up = (i & size) == 0;
                    const K a = k[i], b = k[l];
                    const bool swap = up ? (a > b) : (a < b);
                    k[i] = swap ? b : a;
                    k[l] = swap ? a : b;
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < G; ++j)
        if (j < g) skey[gs + j] = k[j];
}

// LK = type of the keys while they are in LDS and registers.  All keys of a bucket agree above
// their low_bits bits, so 64-bit keys with low_bits <= 32 are kept as their low 32 bits (LK = u32:
// half the LDS, registers and comparison work) and get their common upper part back, bucket <<
// low_bits, on the way out.
template <typename K, bool HAS_VAL, int BUCKET_THREADS, int BUCKET_ITEMS, typename LK = K>
__device__ __forceinline__ void bucket_sort_one(const int bkt, K* __restrict__ kin, K* __restrict__ kout,
                                                u32* __restrict__ vin, u32* __restrict__ vout,
                                                const u32* __restrict__ totals, const u32* __restrict__ starts,
                                                int low_bits) {
    constexpr int BUCKET_WAVES = BUCKET_THREADS / 64;
    constexpr int BUCKET_CAP = BUCKET_THREADS * BUCKET_ITEMS;  // keys of one bucket held in LDS
    constexpr int RMAX = 1 << BUCKET_GROUP_BITS;
    static_assert(RMAX <= BUCKET_THREADS, "one thread per digit in the scans below");
    __shared__ LK skey[BUCKET_CAP];
    __shared__ u32 sval[HAS_VAL ? BUCKET_CAP : 1];
    __shared__ u32 wcnt[BUCKET_WAVES][RMAX];
    __shared__ u32 tstart[RMAX];
    __shared__ u32 smem[BUCKET_WAVES];
    const int t = threadIdx.x, w = wave_id(), lane = lane_id();

    // start of this bucket = sum of the counts of the buckets before it (given, or summed here)
    const int cnt = (int)totals[bkt];
    if (cnt == 0) return;
    u32 start;
    if (starts) {  // (the partition kernel has left them)
        start = starts[bkt];
    } else {
        u32 part = 0;
        for (int j = t; j < bkt; j += BUCKET_THREADS) part += totals[j];
        (void)wide_block_exclusive_scan<BUCKET_WAVES>(part, smem, start);
        __syncthreads();
    }
    if (cnt > BUCKET_CAP) {
        bucket_sort_oversize<K, HAS_VAL, BUCKET_THREADS>(kout + start, kin + start, HAS_VAL ? vout + start : nullptr,
                                         HAS_VAL ? vin + start : nullptr, cnt, low_bits, tstart, smem);
        return;
    }
    if (low_bits <= 0) {
        for (int i = t; i < cnt; i += BUCKET_THREADS) {
            kout[start + i] = kin[start + i];
            if (HAS_VAL) vout[start + i] = vin[start + i];
        }
        return;
    }
    kin += start;
    kout += start;
    if (HAS_VAL) {
        vin += start;
        vout += start;
    }

    const int items = (cnt + BUCKET_THREADS - 1) / BUCKET_THREADS;  // <= BUCKET_ITEMS, same for the whole workgroup

    // One stable pass on key bits [shift, shift + bits): the keys come from memory (FROM_MEMORY) or
    // from skey, in index order = (wave, item, lane), and land in skey/sval; tstart[d] = first
    // position of digit d afterwards.
    auto radix_pass = [&](auto from_memory, int shift, int bits) {
        constexpr bool FROM_MEMORY = decltype(from_memory)::value;
        const u32 R = 1u << bits, dmask = R - 1;
        for (int i = t; i < BUCKET_WAVES * RMAX; i += BUCKET_THREADS)
            if ((u32)(i & (RMAX - 1)) < R) (&wcnt[0][0])[i] = 0;
        LK key[BUCKET_ITEMS];
        u32 val[BUCKET_ITEMS];
        u32 rank[BUCKET_ITEMS];
        u32 digit[BUCKET_ITEMS];
#pragma unroll
        for (int i = 0; i < BUCKET_ITEMS; ++i) {
            key[i] = (LK) ~(LK)0;  // padding ranks last and is dropped
            val[i] = 0u;
            if (i < items) {
                const int idx = w * (64 * items) + i * 64 + lane;
                if (idx < cnt) {
                    key[i] = FROM_MEMORY ? (LK)kin[idx] : skey[idx];
                    if (HAS_VAL) val[i] = FROM_MEMORY ? vin[idx] : sval[idx];
                }
            }
            digit[i] = digit_of<LK>(key[i], shift, dmask);
        }
        __syncthreads();
        wave_rank_digits<BUCKET_ITEMS>(digit, items, bits, wcnt[w], rank);
        __syncthreads();
        u32 dtot = 0;
        if ((u32)t < R) {
            u32 run = 0;
            for (int ww = 0; ww < BUCKET_WAVES; ++ww) {
                const u32 c = wcnt[ww][t];
                wcnt[ww][t] = run;
                run += c;
            }
            dtot = run;
        }
        u32 dummy;
        const u32 dex = wide_block_exclusive_scan<BUCKET_WAVES>(dtot, smem, dummy);
        if ((u32)t < R) tstart[t] = dex;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < BUCKET_ITEMS; ++i) {
            if (i < items) {
                const u32 pos = tstart[digit[i]] + wcnt[w][digit[i]] + rank[i];
                if (pos < (u32)cnt) {
                    skey[pos] = key[i];
                    if (HAS_VAL) sval[pos] = val[i];
                }
            }
        }
        __syncthreads();
    };

    const int gbits = low_bits < BUCKET_GROUP_BITS ? low_bits : BUCKET_GROUP_BITS;
    const int rest = low_bits - gbits;
    radix_pass(std::true_type{}, rest, gbits);
    if (rest > 0) {
        // groups: positions [tstart[d], tstart[d + 1]) (the last one ends at cnt)
        const int ngroups = 1 << gbits;
        int gs = 0, ge = 0;
        if (t < ngroups) {
            gs = (int)tstart[t];
            ge = t + 1 < ngroups ? (int)tstart[t + 1] : cnt;
            if (ge > cnt) ge = cnt;
        }
        if (!__syncthreads_or(ge - gs > BUCKET_GROUP_MAX)) {
            const int g = ge - gs;
            if (g > 16) {  // one lane, in place: every step waits for LDS, so only for the rare long group
                for (int i = gs + 1; i < ge; ++i) {
                    const LK k = skey[i];
                    const u32 v = HAS_VAL ? sval[i] : 0u;
                    int j = i;
                    while (j > gs && skey[j - 1] > k) {
                        skey[j] = skey[j - 1];
                        if (HAS_VAL) sval[j] = sval[j - 1];
                        --j;
                    }
                    skey[j] = k;
                    if (HAS_VAL) sval[j] = v;
                }
            } else if (g > 8) {
                if constexpr (HAS_VAL) group_rank_sort<LK, true, 16>(skey, sval, gs, g);
                else group_network_sort<LK, 16>(skey, gs, g);
            } else if (g > 4) {
                if constexpr (HAS_VAL) group_rank_sort<LK, true, 8>(skey, sval, gs, g);
                else group_network_sort<LK, 8>(skey, gs, g);
            } else if (g > 1) {
                if constexpr (HAS_VAL) group_rank_sort<LK, true, 4>(skey, sval, gs, g);
                else group_network_sort<LK, 4>(skey, gs, g);
            }
            __syncthreads();
        } else {
            const int passes = (low_bits + 7) / 8;
            const int per = (low_bits + passes - 1) / passes;
            int shift = 0;
            for (int p = 0; p < passes; ++p) {
                const int bits = (low_bits - shift) < per ? (low_bits - shift) : per;
                radix_pass(std::false_type{}, shift, bits);
                shift += bits;
            }
        }
    }
    K upper = 0;
    if constexpr (sizeof(LK) < sizeof(K)) upper = (K)(u32)bkt << low_bits;
    for (int i = t; i < cnt; i += BUCKET_THREADS) {
        kout[i] = upper | (K)skey[i];
        if (HAS_VAL) vout[i] = sval[i];
    }
}

template <typename K, bool HAS_VAL, int BUCKET_THREADS, int BUCKET_ITEMS, typename LK = K>
__global__ __launch_bounds__(BUCKET_THREADS) void bucket_sort_kernel(K* __restrict__ kin, K* __restrict__ kout,
                                                                     u32* __restrict__ vin, u32* __restrict__ vout,
                                                                     const u32* __restrict__ totals, int nbuckets,
                                                                     int low_bits, const u32* __restrict__ starts = nullptr) {
    (void)nbuckets;
    bucket_sort_one<K, HAS_VAL, BUCKET_THREADS, BUCKET_ITEMS, LK>((int)blockIdx.x, kin, kout, vin, vout, totals, starts,
                                                                  low_bits);
}

// ---------------------------------------------------------------------------
// The per-bucket kernel for keys WITHOUT values (the sorts of the decimation path: incidence keys
// and edge keys).  Equal keys are indistinguishable, so nothing has to be stable:
//   1. the keys of the bucket are read once; each takes its place in its group (the keys that agree
//      on the top 9 of the bucket's low bits: with vertex-pair keys the half-edges of one lower
//      vertex) from one returning LDS atomic on the group's counter;
//   2. one scan of the (up to 512) group counters gives the groups' first positions;
//   3. one lane per group sorts its group on the whole key in registers with a sorting network of
//      minimal size for 4, 6, 8, 12 or 16 keys (a wave runs every size that occurs among its 64
//      groups, so the sizes are graded finely), by insertion up to 64 keys;
//   4. the bucket is written out in order; optionally (COUNT_UNIQUE) the kernel also does the count
//      pass of the compaction that keeps the first of every run of equal keys (the all-ones
//      `sentinel` not counted): it adds, per tile of 2^tile_shift positions of the whole output, the
//      number of such keys to tilesum[tile] (zero on entry), which is what tile_count_kernel would
//      leave there.
// A bucket with a group of more than 64 keys (a vertex of very high degree) is sorted as a whole by
// a bitonic network over the LDS array.  A bucket beyond the LDS capacity (uneven vertex numbering:
// up to 16 times the capacity) is sorted in parts, runs of whole groups that fit, each read out of the
// bucket by the workgroup; if it also has a group of more than 64 keys, or is larger still, it
// takes the slow global-memory route of bucket_sort_oversize.  Workgroups are small (256 lanes for the 4096-bucket
// sorts) so that eight of them share a compute unit and cover each other's barriers.
// ---------------------------------------------------------------------------
#define PRIM_CE(a, b)                       \
    {                                       \
        const K x_ = k[a], y_ = k[b];       \
        const bool s_ = y_ < x_;            \
        k[a] = s_ ? y_ : x_;                \
        k[b] = s_ ? x_ : y_;                \
    }

// Sorting networks of 5, 12, 19, 39 and 60 comparators (the smallest known for these sizes; each was
// checked on all 2^G inputs of zeros and ones).
template <typename K, int G>
__device__ __forceinline__ void network_sort_regs(K (&k)[G]) {
    if constexpr (G == 4) {
        PRIM_CE(0, 2) PRIM_CE(1, 3) PRIM_CE(0, 1) PRIM_CE(2, 3) PRIM_CE(1, 2)
    } else if constexpr (G == 6) {
        PRIM_CE(0, 5) PRIM_CE(1, 3) PRIM_CE(2, 4) PRIM_CE(1, 2) PRIM_CE(3, 4) PRIM_CE(0, 3) PRIM_CE(2, 5) PRIM_CE(0, 1)
        PRIM_CE(2, 3) PRIM_CE(4, 5) PRIM_CE(1, 2) PRIM_CE(3, 4)
    } else if constexpr (G == 8) {
        PRIM_CE(0, 2) PRIM_CE(1, 3) PRIM_CE(4, 6) PRIM_CE(5, 7) PRIM_CE(0, 4) PRIM_CE(1, 5) PRIM_CE(2, 6) PRIM_CE(3, 7)
        PRIM_CE(0, 1) PRIM_CE(2, 3) PRIM_CE(4, 5) PRIM_CE(6, 7) PRIM_CE(2, 4) PRIM_CE(3, 5) PRIM_CE(1, 4) PRIM_CE(3, 6)
        PRIM_CE(1, 2) PRIM_CE(3, 4) PRIM_CE(5, 6)
    } else if constexpr (G == 12) {
        PRIM_CE(0, 8) PRIM_CE(1, 7) PRIM_CE(2, 6) PRIM_CE(3, 11) PRIM_CE(4, 10) PRIM_CE(5, 9) PRIM_CE(0, 1) PRIM_CE(2, 5)
        PRIM_CE(3, 4) PRIM_CE(6, 9) PRIM_CE(7, 8) PRIM_CE(10, 11) PRIM_CE(0, 2) PRIM_CE(1, 6) PRIM_CE(5, 10) PRIM_CE(9, 11)
        PRIM_CE(0, 3) PRIM_CE(1, 2) PRIM_CE(4, 6) PRIM_CE(5, 7) PRIM_CE(8, 11) PRIM_CE(9, 10) PRIM_CE(1, 4) PRIM_CE(3, 5)
        PRIM_CE(6, 8) PRIM_CE(7, 10) PRIM_CE(1, 3) PRIM_CE(2, 5) PRIM_CE(6, 9) PRIM_CE(8, 10) PRIM_CE(2, 3) PRIM_CE(4, 5)
        PRIM_CE(6, 7) PRIM_CE(8, 9) PRIM_CE(4, 6) PRIM_CE(5, 7) PRIM_CE(3, 4) PRIM_CE(5, 6) PRIM_CE(7, 8)
    } else {
        static_assert(G == 16, "network sizes: 4, 6, 8, 12, 16");
        PRIM_CE(0, 13) PRIM_CE(1, 12) PRIM_CE(2, 15) PRIM_CE(3, 14) PRIM_CE(4, 8) PRIM_CE(5, 6) PRIM_CE(7, 11) PRIM_CE(9, 10)
        PRIM_CE(0, 5) PRIM_CE(1, 7) PRIM_CE(2, 9) PRIM_CE(3, 4) PRIM_CE(6, 13) PRIM_CE(8, 14) PRIM_CE(10, 15) PRIM_CE(11, 12)
        PRIM_CE(0, 1) PRIM_CE(2, 3) PRIM_CE(4, 5) PRIM_CE(6, 8) PRIM_CE(7, 9) PRIM_CE(10, 11) PRIM_CE(12, 13) PRIM_CE(14, 15)
        PRIM_CE(0, 2) PRIM_CE(1, 3) PRIM_CE(4, 10) PRIM_CE(5, 11) PRIM_CE(6, 7) PRIM_CE(8, 9) PRIM_CE(12, 14) PRIM_CE(13, 15)
        PRIM_CE(1, 2) PRIM_CE(3, 12) PRIM_CE(4, 6) PRIM_CE(5, 7) PRIM_CE(8, 10) PRIM_CE(9, 11) PRIM_CE(13, 14) PRIM_CE(1, 4)
        PRIM_CE(2, 6) PRIM_CE(5, 8) PRIM_CE(7, 10) PRIM_CE(9, 13) PRIM_CE(11, 14) PRIM_CE(2, 4) PRIM_CE(3, 6) PRIM_CE(9, 12)
        PRIM_CE(11, 13) PRIM_CE(3, 5) PRIM_CE(6, 8) PRIM_CE(7, 9) PRIM_CE(10, 12) PRIM_CE(3, 4) PRIM_CE(5, 6) PRIM_CE(7, 8)
        PRIM_CE(9, 10) PRIM_CE(11, 12) PRIM_CE(6, 7) PRIM_CE(8, 9)
    }
}
#undef PRIM_CE

// The g <= G keys at [gs, gs + g) of an LDS array sorted by one lane (empty places hold the largest key).
template <typename K, int G>
__device__ __forceinline__ void group_sort_lds(K* skey, int gs, int g) {
    K k[G];
#pragma unroll
    for (int j = 0; j < G; ++j) k[j] = j < g ? skey[gs + j] : (K) ~(K)0;
    network_sort_regs<K, G>(k);
#pragma unroll
    for (int j = 0; j < G; ++j)
        if (j < g) skey[gs + j] = k[j];
}

template <typename K, typename LK, int THREADS, int ITEMS, bool COUNT_UNIQUE>
__global__ __launch_bounds__(THREADS) void bucket_keys_kernel(K* __restrict__ kin, K* __restrict__ kout,
                                                              const u32* __restrict__ totals,
                                                              const u32* __restrict__ starts, int low_bits, K sentinel,
                                                              int* __restrict__ tilesum, int tile_shift) {
    constexpr int NW = THREADS / 64;
    constexpr int CAP = THREADS * ITEMS;
    constexpr int RMAX = 1 << BUCKET_GROUP_BITS;
    constexpr int PER = RMAX / THREADS > 0 ? RMAX / THREADS : 1;  // group counters per thread in the scan
    static_assert((CAP & (CAP - 1)) == 0, "the whole-bucket network pads to a power of two within the LDS array");
    static_assert(THREADS >= 64 && THREADS % 64 == 0 && (THREADS >= RMAX || RMAX % THREADS == 0), "whole counters per thread");
    __shared__ LK skey[CAP];
    __shared__ u32 gcnt[RMAX];
    __shared__ u32 gstart[RMAX + 1];
    __shared__ u32 smem[NW];
    __shared__ u32 nlong;
    constexpr int TALLY = (CAP >> 8) + 2;  // tiles (of at least 256 positions) that CAP consecutive positions can touch
    static_assert(TALLY <= THREADS, "one thread per tile of the tally");
    __shared__ int tcnt[COUNT_UNIQUE ? TALLY : 1];
    const int t = threadIdx.x, lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(wave_id());  // (in a scalar register: what follows from it is computed once per wave)
    const int bkt = (int)blockIdx.x;
    const int cnt = (int)totals[bkt];
    if (cnt == 0) return;
    const u32 start = starts[bkt];
    kin += start;
    kout += start;

    // By every lane of a wave together: the wave's lanes hold the output positions start + idx0 + lane
    // (idx0 the same in all lanes), `first` says whether a lane's key is the first of its run; the
    // counts go to the one or two tiles the 64 positions lie in: to the workgroup's tally in LDS
    // (`tally`), or straight to memory.
    const u32 tile0 = COUNT_UNIQUE ? start >> tile_shift : 0u;  // first tile this bucket's range touches
    auto count_firsts = [&](int idx0, bool first, int* tally) {
        const u64 bal = __ballot(first);
        if (bal == 0) return;
        const u32 p0 = start + (u32)idx0;
        const u32 tile_a = p0 >> tile_shift, tile_b = (p0 + 63u) >> tile_shift;
        const u32 in_a = ((tile_a + 1u) << tile_shift) - p0;  // positions of the wave that lie in its first tile
        const u64 mask_a = in_a >= 64u ? ~0ull : ((1ull << in_a) - 1ull);
        if (lane == 0) {
            const int ca = (int)__popcll(bal & mask_a), cb = (int)__popcll(bal & ~mask_a);
            if (tally) {
                if (ca) atomicAdd(&tally[tile_a - tile0], ca);
                if (cb) atomicAdd(&tally[tile_b - tile0], cb);
            } else {
                if (ca) atomicAdd(&tilesum[tile_a], ca);
                if (cb) atomicAdd(&tilesum[tile_b], cb);
            }
        }
    };

    const int gbits = low_bits < BUCKET_GROUP_BITS ? (low_bits > 0 ? low_bits : 0) : BUCKET_GROUP_BITS;
    const int rest = low_bits - gbits;
    const u32 R = 1u << gbits, dmask = R - 1;
    K upper = 0;  // what the keys of this bucket share above their low_bits bits
    if constexpr (sizeof(LK) < sizeof(K)) upper = (K)(u32)bkt << low_bits;

    // The groups g0 .. g1 - 1, whose keys lie at [gstart[g] - gstart[g0], ...) of the LDS array, each sorted on
    // the whole key: one lane per group of up to 16 keys (a sorting network), then a wave per longer group.
    // By the whole workgroup; no group may exceed 64 keys; uses gcnt (as the list of long groups) and nlong.
    auto sort_groups = [&](int g0, int g1) {
        const int lds0 = (int)gstart[g0];
        if (t == 0) nlong = 0;
        __syncthreads();
        for (int gi = g0 + t; gi < g1; gi += THREADS) {
            const int gs = (int)gstart[gi] - lds0;
            const int g = (int)gstart[gi + 1] - (int)gstart[gi];
            if (g > 16) {  // listed for the waves (the counters are no longer needed: the list goes there)
                gcnt[atomicAdd(&nlong, 1u)] = (u32)gi;
            } else if (g > 12) {
                group_sort_lds<LK, 16>(skey, gs, g);
            } else if (g > 8) {
                group_sort_lds<LK, 12>(skey, gs, g);
            } else if (g > 6) {
                group_sort_lds<LK, 8>(skey, gs, g);
            } else if (g > 4) {
                group_sort_lds<LK, 6>(skey, gs, g);
            } else if (g > 1) {
                group_sort_lds<LK, 4>(skey, gs, g);
            }
        }
        __syncthreads();
        // groups of 17 to 64 keys: a wave takes a group, one lane per key; a key's place is the number of
        // keys of the group that go before it (every lane reads the same address, one read after the
        // other with nothing waiting in between, where an insertion sort by one lane would wait for
        // LDS at every step)
        const int n_long = (int)nlong;
        if (n_long > 0) {
            for (int li = w; li < n_long; li += NW) {
                const int gi = (int)gcnt[li];
                const int gs = (int)gstart[gi] - lds0;
                const int g = (int)gstart[gi + 1] - (int)gstart[gi];
                const LK k = lane < g ? skey[gs + lane] : (LK)0;
                int r = 0;
                for (int i = 0; i < g; ++i) {
                    const LK o = skey[gs + i];
                    r += (o < k || (o == k && i < lane)) ? 1 : 0;
                }
                __builtin_amdgcn_wave_barrier();  // (a wave's LDS operations complete in order)
                if (lane < g) skey[gs + r] = k;
            }
            __syncthreads();
        }
    };

    if (cnt > CAP && low_bits > 0) {
        // More keys than the LDS array holds.  If no group is long, the bucket is sorted in parts: runs of
        // whole groups of at most CAP keys each, every part fetched from the bucket (which is read once per
        // part, and once more for the groups' sizes) and sorted like a bucket that fits.
        for (int i = t; i < (int)R; i += THREADS) gcnt[i] = 0;
        __syncthreads();
        // fn(key) for every key of the bucket; a thread's loads go out ITEMS at a time, so that a pass over
        // the bucket waits for memory once per CAP keys and not once per key of the thread
        auto for_each_key = [&](auto fn) {
            for (int base = 0; base < cnt; base += CAP) {
                LK kreg[ITEMS];
#pragma unroll
                for (int i = 0; i < ITEMS; ++i) {
                    const int idx = base + i * THREADS + t;
                    kreg[i] = idx < cnt ? (LK)kin[idx] : (LK)0;
                }
#pragma unroll
                for (int i = 0; i < ITEMS; ++i)
                    if (base + i * THREADS + t < cnt) fn(kreg[i]);
            }
        };
        for_each_key([&](LK k) { atomicAdd(&gcnt[digit_of<LK>(k, rest, dmask)], 1u); });
        __syncthreads();
        u32 c[PER], sum = 0, tot;
        int too_long = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const u32 d = (u32)(t * PER + j);
            c[j] = d < R ? gcnt[d] : 0u;
            sum += c[j];
            too_long |= c[j] > (u32)BUCKET_GROUP_MAX ? 1 : 0;
        }
        u32 run = wide_block_exclusive_scan<NW>(sum, smem, tot);
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const u32 d = (u32)(t * PER + j);
            if (d < R) gstart[d] = run;
            run += c[j];
        }
        if (t == 0) gstart[R] = (u32)cnt;
        if (!__syncthreads_or(too_long) && rest > 0 && cnt <= 16 * CAP) {
            for (int g0 = 0; g0 < (int)R;) {
                // the longest run of whole groups from g0 on with at most CAP keys (a group has at most 64
                // keys, so at least one fits): gstart ascends, the run's end is found by bisection
                int g1 = g0 + 1, g_hi = (int)R;
                const u32 part_end = gstart[g0] + (u32)CAP;
                while (g1 < g_hi) {
                    const int mid = (g1 + g_hi + 1) >> 1;
                    if (gstart[mid] <= part_end) g1 = mid;
                    else g_hi = mid - 1;
                }
                const int part0 = (int)gstart[g0], part_n = (int)gstart[g1] - part0;
                if (part_n > 0) {
                    for (int i = g0 + t; i < g1; i += THREADS) gcnt[i] = 0;
                    __syncthreads();
                    for_each_key([&](LK k) {
                        const int d = (int)digit_of<LK>(k, rest, dmask);
                        if (d >= g0 && d < g1) skey[gstart[d] - (u32)part0 + atomicAdd(&gcnt[d], 1u)] = k;
                    });
                    __syncthreads();
                    sort_groups(g0, g1);
                    for (int i0 = w * 64; i0 < part_n; i0 += THREADS) {  // (whole waves, for the ballot)
                        const int i = i0 + lane;
                        bool first = false;
                        if (i < part_n) {
                            const LK k = skey[i];
                            const K full = upper | (K)k;
                            kout[part0 + i] = full;
                            if constexpr (COUNT_UNIQUE) first = full != sentinel && (i == 0 || skey[i - 1] != k);
                        }
                        if constexpr (COUNT_UNIQUE) count_firsts(part0 + i0, first, nullptr);
                    }
                    __syncthreads();
                }
                g0 = g1;
            }
            return;
        }
    }
    if (cnt > CAP) {  // ... else pass by pass through global memory
        bucket_sort_oversize<K, false, THREADS>(kout, kin, nullptr, nullptr, cnt, low_bits, gcnt, smem);
        if constexpr (COUNT_UNIQUE) {
            __threadfence();
            __syncthreads();
            for (int i0 = w * 64; i0 < cnt; i0 += THREADS) {  // (whole waves, for the ballot)
                const int i = i0 + lane;
                bool first = false;
                if (i < cnt) {
                    const K k = coherent_load(&kout[i]);
                    first = k != sentinel && (i == 0 || coherent_load(&kout[i - 1]) != k);
                }
                count_firsts(i0, first, nullptr);
            }
        }
        return;
    }
    if (low_bits <= 0) {  // nothing below the bucket's digit: all keys equal
        for (int i = t; i < cnt; i += THREADS) kout[i] = kin[i];
        if constexpr (COUNT_UNIQUE) {
            if (w == 0) count_firsts(0, lane == 0 && kin[0] != sentinel, nullptr);
        }
        return;
    }

    for (int i = t; i < (int)R; i += THREADS) gcnt[i] = 0;
    if constexpr (COUNT_UNIQUE) {
        if (t < TALLY) tcnt[t] = 0;
    }
    const int items = (cnt + THREADS - 1) / THREADS;  // <= ITEMS, the same in every thread
    LK key[ITEMS];
    u32 pos[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        key[i] = (LK)0;
        pos[i] = 0;
        if (i < items) {
            const int idx = i * THREADS + t;
            if (idx < cnt) key[i] = (LK)kin[idx];
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i)
        if (i < items && i * THREADS + t < cnt) pos[i] = atomicAdd(&gcnt[digit_of<LK>(key[i], rest, dmask)], 1u);
    __syncthreads();
    u32 c[PER], sum = 0, tot;
    int too_long = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const u32 d = (u32)(t * PER + j);
        c[j] = d < R ? gcnt[d] : 0u;
        sum += c[j];
        too_long |= c[j] > (u32)BUCKET_GROUP_MAX ? 1 : 0;
    }
    u32 run = wide_block_exclusive_scan<NW>(sum, smem, tot);
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const u32 d = (u32)(t * PER + j);
        if (d < R) gstart[d] = run;
        run += c[j];
    }
    if (t == 0) gstart[R] = (u32)cnt;
    const int any_long = __syncthreads_or(too_long);
#pragma unroll
    for (int i = 0; i < ITEMS; ++i)
        if (i < items && i * THREADS + t < cnt) skey[gstart[digit_of<LK>(key[i], rest, dmask)] + pos[i]] = key[i];
    __syncthreads();
    if (rest > 0 && !any_long) {
        sort_groups(0, (int)R);
    } else if (rest > 0) {
        // some group is longer still: the whole bucket through a bitonic network, padded to a power of two
        int P = 64;
        while (P < cnt) P <<= 1;
        for (int i = cnt + t; i < P; i += THREADS) skey[i] = (LK) ~(LK)0;
        __syncthreads();
        for (int size = 2; size <= P; size <<= 1) {
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                for (int q = t; q < P / 2; q += THREADS) {
                    const int i = 2 * q - (q & (stride - 1)), l = i + stride;
                    const bool up = (i & size) == 0;
                    const LK a = skey[i], b = skey[l];
                    if ((a > b) == up) {
                        skey[i] = b;
                        skey[l] = a;
                    }
                }
                __syncthreads();
            }
        }
    }
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        if (i < items) {
            const int idx = i * THREADS + t;
            bool first = false;
            if (idx < cnt) {
                const LK k = skey[idx];
                const K full = upper | (K)k;
                kout[idx] = full;
                if constexpr (COUNT_UNIQUE) first = full != sentinel && (idx == 0 || skey[idx - 1] != k);
            }
            if constexpr (COUNT_UNIQUE) count_firsts(i * THREADS + w * 64, first, tcnt);
        }
    }
    if constexpr (COUNT_UNIQUE) {
        // A tile that lies wholly inside this bucket's range gets its count from this workgroup alone (a
        // plain store); the range's first and last tile may be shared with the neighbouring buckets.
        __syncthreads();
        const u32 last_tile = (start + (u32)cnt - 1u) >> tile_shift;
        if ((u32)t <= last_tile - tile0) {
            const u32 tile = tile0 + (u32)t;
            const int v = tcnt[t];
            const bool inside = (tile << tile_shift) >= start && ((tile + 1u) << tile_shift) <= start + (u32)cnt;
            if (inside) tilesum[tile] = v;
            else if (v) atomicAdd(&tilesum[tile], v);
        }
    }
}

// Launch of that kernel, one workgroup per bucket, with the narrowest in-LDS key type that holds low_bits
// bits.  tilesum == nullptr: no counting.
template <typename K, int THREADS, int ITEMS>
inline void launch_bucket_keys_kernel(int nbuckets, hipStream_t s, K* kin, K* kout, const u32* totals, int low_bits,
                                      const u32* starts, K sentinel = (K)0, int* tilesum = nullptr, int tile_shift = 0) {
    if constexpr (sizeof(K) == 8) {
        if (low_bits <= 32) {
            if (tilesum)
                bucket_keys_kernel<K, u32, THREADS, ITEMS, true><<<nbuckets, THREADS, 0, s>>>(kin, kout, totals, starts, low_bits, sentinel, tilesum, tile_shift);
            else
                bucket_keys_kernel<K, u32, THREADS, ITEMS, false><<<nbuckets, THREADS, 0, s>>>(kin, kout, totals, starts, low_bits, sentinel, tilesum, tile_shift);
            return;
        }
    }
    if (tilesum)
        bucket_keys_kernel<K, K, THREADS, ITEMS, true><<<nbuckets, THREADS, 0, s>>>(kin, kout, totals, starts, low_bits, sentinel, tilesum, tile_shift);
    else
        bucket_keys_kernel<K, K, THREADS, ITEMS, false><<<nbuckets, THREADS, 0, s>>>(kin, kout, totals, starts, low_bits, sentinel, tilesum, tile_shift);
}

// What a keys-only bucket sort may do for the compaction that follows it (see bucket_keys_kernel):
// the count pass of "keep the first of every run of equal keys, `sentinel` excepted" with tiles of
// 2^tile_shift positions; the partition kernel zeroes tilesum[0, tiles).  tilesum == nullptr: nothing.
template <typename K>
struct UniqueCount {
    int* tilesum = nullptr;
    int tile_shift = 0;
    int tiles = 0;
    K sentinel = (K)0;
};

// Histogram of the top RBITS-bit digit (bits [shift, shift + RBITS)) over the whole input, added
// to `hist` (which starts at zero); tiles of BLOCK * ITEMS keys.
template <typename K, int RBITS, int ITEMS>
__global__ __launch_bounds__(BLOCK) void msd_histogram_kernel(const K* __restrict__ kin, const int* n_ptr, int n_host,
                                                              u32* __restrict__ hist, int shift) {
    constexpr int R = 1 << RBITS;
    constexpr int TILE = BLOCK * ITEMS;
    __shared__ u32 h[R];
    const int n = load_count(n_ptr, n_host);
    const long long base = (long long)blockIdx.x * TILE;
    if (base >= n) return;
    const int t = threadIdx.x;
    for (int i = t; i < R; i += BLOCK) h[i] = 0;
    __syncthreads();
#pragma unroll 4
    for (int i = 0; i < ITEMS; ++i) {
        const long long idx = base + (long long)i * BLOCK + t;
        if (idx < n) atomicAdd(&h[digit_of<K>(kin[idx], shift, R - 1)], 1u);
    }
    __syncthreads();
    for (int i = t; i < R; i += BLOCK) {
        const u32 c = h[i];
        if (c) atomicAdd(&hist[i], c);
    }
}

// Partition of keys WITHOUT values by their top digit (bits [shift, shift + RBITS)) in one pass.
// hist[d] = number of keys with digit d over the whole input (so digit d owns the output range
// that starts at the sum of the counts before it; the first tile also writes these first
// positions to `starts`); cursor[d] = how much of that range is taken, zero at the start.  Every tile counts its keys per digit in LDS, takes its share of each
// digit's range with one returning atomic per digit it holds, and writes its keys there.  The
// order of the keys inside a digit's range depends on the order in which tiles arrive, so this is
// for sorts that then order each range on the whole key; with equal keys indistinguishable the
// final result does not depend on it.  The lanes of a wave whose keys share a digit (keys led by
// mesh indices bring few distinct digits into a wave) rank themselves with one LDS atomic.
// A key source gives key i of the input: an array, or a functor that makes the key on the fly (so
// that keys which are a cheap function of other data need not be written out and read back).
template <typename K>
struct ArrayKeys {
    const K* p;
    __device__ __forceinline__ K operator()(long long i) const { return p[i]; }
};

template <typename K, int RBITS, int ITEMS, class Src>
__global__ __launch_bounds__(BLOCK) void msd_scatter_kernel(Src kin, K* __restrict__ kout,
                                                            const int* n_ptr, int n_host, int shift,
                                                            const u32* __restrict__ hist, u32* __restrict__ cursor,
                                                            u32* __restrict__ starts, int* __restrict__ zero = nullptr,
                                                            int n_zero = 0) {
    constexpr int R = 1 << RBITS;
    constexpr int PER = R / BLOCK;  // digits per thread in the scan of the ranges' first positions
    // (an array that the kernel after this one adds to: zeroed here, by all workgroups together)
    for (int i = blockIdx.x * BLOCK + threadIdx.x; i < n_zero; i += gridDim.x * BLOCK) zero[i] = 0;
    static_assert(R % BLOCK == 0, "whole digits per thread");
    constexpr int TILE = BLOCK * ITEMS;
    __shared__ u32 h[R];  // per digit: this tile's count, then where the tile's keys of that digit go
    __shared__ u32 first[R + R / 32];  // (one unused word after every 32: a thread's PER consecutive digits, written by the scan
                                       // below, then fall into different banks from its neighbours')
    __shared__ u32 smem[WAVES];
    const int n = load_count(n_ptr, n_host);
    const long long base = (long long)blockIdx.x * TILE;
    if (base >= n) return;
    const int t = threadIdx.x, w = wave_id(), lane = lane_id();
    const u64 lt = lanemask_lt();
    for (int i = t; i < R; i += BLOCK) h[i] = 0;
    K key[ITEMS];
    u32 rk[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const long long idx = base + (long long)w * (64 * ITEMS) + i * 64 + lane;
        key[i] = idx < n ? kin(idx) : (K)0;
    }
    {   // first position of every digit's range
        u32 c[PER], sum = 0, tot;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            c[j] = hist[t * PER + j];
            sum += c[j];
        }
        u32 run = block_exclusive_scan(sum, smem, tot);
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            first[(t * PER + j) + ((t * PER + j) >> 5)] = run;
            if (blockIdx.x == 0) starts[t * PER + j] = run;  // for the kernel that sorts the ranges
            run += c[j];
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const long long idx = base + (long long)w * (64 * ITEMS) + i * 64 + lane;
        const bool ok = idx < n;
        const u32 d = digit_of<K>(key[i], shift, R - 1);
        // the lanes that share a digit rank themselves with one returning atomic, by the first of them
        const u64 same = wave_same_digit_lanes(ok, d);
        u32 b = 0;
        if (ok && (same & lt) == 0) b = atomicAdd(&h[d], (u32)__popcll(same));
        b = (u32)__shfl((int)b, ok ? __ffsll((long long)same) - 1 : lane, 64);
        rk[i] = b + (u32)__popcll(same & lt);
    }
    __syncthreads();
    for (int d = t; d < R; d += BLOCK) {
        const u32 c = h[d];
        if (c) h[d] = first[d + (d >> 5)] + atomicAdd(&cursor[d], c);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const long long idx = base + (long long)w * (64 * ITEMS) + i * 64 + lane;
        if (idx < n) {
            const u32 pos = h[digit_of<K>(key[i], shift, R - 1)] + rk[i];
            if (pos < (u32)n) kout[pos] = key[i];  // (always, when hist and cursor are as described)
        }
    }
}

// Keys without values are partitioned by msd_scatter_kernel, which works from a histogram of the
// top digit in msd_hist[0, R) and cursors in msd_hist[MSD_HIST_WORDS, MSD_HIST_WORDS + R), both
// zeroed beforehand; the ranges' first positions go to msd_hist[2 * MSD_HIST_WORDS, ...) (msd_hist
// holds 3 * MSD_HIST_WORDS words).  `counted`: the producer of the
// keys has already added the keys' digits to that (zeroed) histogram and left the cursors zero,
// so the histogram pass over the keys is skipped.
constexpr int MSD_HIST_WORDS = 4096;
inline int bucket_sort_msd_bits(int key_bits) { return key_bits < BUCKET_MSD_BITS ? key_bits : BUCKET_MSD_BITS; }
inline int bucket_sort_low_bits(int key_bits) { return key_bits - bucket_sort_msd_bits(key_bits); }

__global__ __launch_bounds__(BLOCK) void fill_u32_kernel(u32* __restrict__ p, int n, u32 v) {
    const int i = blockIdx.x * BLOCK + threadIdx.x;
    if (i < n) p[i] = v;
}

// `src`: where the keys come from when not from k0 (keys without values, `counted`); k0 then only
// receives the result.
template <typename K, bool HAS_VAL, class Src = ArrayKeys<K>>
inline int bucket_sort(hipStream_t s, K* k0, K* k1, u32* v0, u32* v1, const int* n_ptr, int n_max, int key_bits,
                       const SortScratch& sc, LaunchTimer* lt = nullptr, int tag = 0, bool counted = false,
                       u32* msd_hist = nullptr, const Src* src = nullptr, const UniqueCount<K>* uq = nullptr) {
    if (n_max <= 0 || key_bits <= 0) return 0;
    const int msd = bucket_sort_msd_bits(key_bits);
    const int low = key_bits - msd;
    const int tiles = sort_tiles(n_max, SORT_ITEMS_SMALL);
    if constexpr (!HAS_VAL) {
        if (msd == BUCKET_MSD_BITS && msd_hist) {
            // keys only: one unordered partition pass (msd_scatter_kernel), then each bucket is ordered on the whole key
            u32* cursor = msd_hist + MSD_HIST_WORDS;
            if (!counted) {
                fill_u32_kernel<<<2 * MSD_HIST_WORDS / BLOCK, BLOCK, 0, s>>>(msd_hist, 2 * MSD_HIST_WORDS, 0u);
                msd_histogram_kernel<K, BUCKET_MSD_BITS, SORT_ITEMS_SMALL><<<tiles, BLOCK, 0, s>>>(k0, n_ptr, n_max, msd_hist, low);
            }
            u32* starts = msd_hist + 2 * MSD_HIST_WORDS;
            const UniqueCount<K> none{};
            const UniqueCount<K>& u = uq ? *uq : none;
            if (src && counted)
                msd_scatter_kernel<K, BUCKET_MSD_BITS, SORT_ITEMS_SMALL, Src><<<tiles, BLOCK, 0, s>>>(*src, k1, n_ptr, n_max, low, msd_hist, cursor, starts, u.tilesum, u.tiles);
            else
                msd_scatter_kernel<K, BUCKET_MSD_BITS, SORT_ITEMS_SMALL, ArrayKeys<K>><<<tiles, BLOCK, 0, s>>>(ArrayKeys<K>{k0}, k1, n_ptr, n_max, low, msd_hist, cursor, starts, u.tilesum, u.tiles);
            const bool timed = lt && lt->begin(s, tag);
            launch_bucket_keys_kernel<K, BUCKET_KEYS_THREADS_256, BUCKET_KEYS_ITEMS_256>(1 << msd, s, k1, k0, msd_hist, low, starts, u.sentinel, u.tilesum, u.tile_shift);
            if (timed) lt->end(s);
            if (hipGetLastError() != hipSuccess) return -1;
            return 0;
        }
    }
    (void)counted;
    radix_upsweep_kernel<K, SORT_ITEMS_SMALL><<<tiles, BLOCK, 0, s>>>(k0, n_ptr, n_max, sc.T, sc.table, low, msd);
    radix_scan_kernel<<<1 << msd, BLOCK, 0, s>>>(sc.table, sc.totals, n_ptr, n_max, sc.T, BLOCK * SORT_ITEMS_SMALL);
    radix_downsweep_kernel<K, HAS_VAL, SORT_ITEMS_SMALL>
        <<<tiles, BLOCK, 0, s>>>(k0, k1, v0, v1, n_ptr, n_max, sc.T, sc.table, sc.totals, low, msd);
    const bool timed = lt && lt->begin(s, tag);
    bucket_sort_kernel<K, HAS_VAL, BUCKET_THREADS_256, 8>
        <<<1 << msd, BUCKET_THREADS_256, 0, s>>>(k1, k0, v1, v0, sc.totals, 1 << msd, low);
    if (timed) lt->end(s);
    if (hipGetLastError() != hipSuccess) return -1;
    return 0;
}

// Larger inputs (up to BUCKET_SORT_LARGE_MAX_KEYS): 4096 buckets on the top 12
// bits.  A single 12-bit partition pass would scatter about one key per digit
// and tile, so the partition is done as two stable 6-bit passes (low half
// first), and the bucket sizes come from a 12-bit histogram taken up front.
constexpr int BUCKET_LARGE_MSD_BITS = 12;
constexpr long long BUCKET_SORT_LARGE_MAX_KEYS = 1ll << 23;

// Histogram of the top 12-bit digit over the whole input (added to `hist`, which starts at zero),
// and from the same read of the keys the first partition pass's per-tile counts of the digit's
// low 6 bits (table[d6 * T + tile], what radix_upsweep_kernel would compute for bits
// [shift, shift + 6)).  Keys made from mesh indices often share their leading bits across a
// whole wave; such a wave counts itself with a single LDS atomic.
template <typename K>
__global__ __launch_bounds__(BLOCK) void top_digit_histogram_kernel(const K* __restrict__ kin, const int* n_ptr,
                                                                    int n_host, u32* __restrict__ hist, int shift, int T,
                                                                    u32* __restrict__ table) {
    constexpr int R = 1 << BUCKET_LARGE_MSD_BITS;
    constexpr int TILE = BLOCK * SORT_ITEMS_BIG;
    __shared__ u32 h[R];
    const int n = load_count(n_ptr, n_host);
    const long long base = (long long)blockIdx.x * TILE;
    if (base >= n) return;
    const int t = threadIdx.x;
    for (int i = t; i < R; i += BLOCK) h[i] = 0;
    __syncthreads();
#pragma unroll 4
    for (int i = 0; i < SORT_ITEMS_BIG; ++i) {
        const long long idx = base + (long long)i * BLOCK + t;
        const bool ok = idx < n;
        const u32 d = ok ? digit_of<K>(kin[idx], shift, R - 1) : 0u;
        const u64 on = __ballot(ok);
        if (on == 0) continue;
        const u32 d0 = (u32)__builtin_amdgcn_readfirstlane((int)d);  // (of the first lane with a key)
        if (__ballot(ok && d == d0) == on) {
            if (ok && (on & lanemask_lt()) == 0) atomicAdd(&h[d0], (u32)__popcll(on));
        } else if (ok) {
            atomicAdd(&h[d], 1u);
        }
    }
    __syncthreads();
    for (int i = t; i < R; i += BLOCK) {
        const u32 c = h[i];
        if (c) atomicAdd(&hist[i], c);
    }
    if (t < 64) {
        u32 sum = 0;
        for (int hi = 0; hi < 64; ++hi) sum += h[(hi << 6) | t];
        table[(size_t)t * T + blockIdx.x] = sum;
    }
}

// Result is in (k1, v1): returns 1 (keys with values), or in k0: returns 0 (keys only); <0 on a
// launch error.  hist12 holds 3 * MSD_HIST_WORDS words (counts, cursors, first positions).
template <typename K, bool HAS_VAL, class Src = ArrayKeys<K>>
inline int bucket_sort_large(hipStream_t s, K* k0, K* k1, u32* v0, u32* v1, const int* n_ptr, int n_max, int key_bits,
                             const SortScratch& sc, u32* hist12, LaunchTimer* lt = nullptr, int tag = 0,
                             bool counted = false, const Src* src = nullptr, const UniqueCount<K>* uq = nullptr) {
    constexpr int R = 1 << BUCKET_LARGE_MSD_BITS;
    const int low = key_bits - BUCKET_LARGE_MSD_BITS;
    const int tiles = sort_tiles(n_max, SORT_ITEMS_BIG);
    if constexpr (!HAS_VAL) {
        // keys only: one unordered partition pass (msd_scatter_kernel), then each bucket is ordered on the whole key
        u32* cursor = hist12 + MSD_HIST_WORDS;
        if (!counted) {
            fill_u32_kernel<<<2 * MSD_HIST_WORDS / BLOCK, BLOCK, 0, s>>>(hist12, 2 * MSD_HIST_WORDS, 0u);
            msd_histogram_kernel<K, BUCKET_LARGE_MSD_BITS, SORT_ITEMS_BIG><<<tiles, BLOCK, 0, s>>>(k0, n_ptr, n_max, hist12, low);
        }
        u32* starts = hist12 + 2 * MSD_HIST_WORDS;
        const UniqueCount<K> none{};
        const UniqueCount<K>& u = uq ? *uq : none;
        if (src && counted)
            msd_scatter_kernel<K, BUCKET_LARGE_MSD_BITS, SORT_ITEMS_BIG, Src><<<tiles, BLOCK, 0, s>>>(*src, k1, n_ptr, n_max, low, hist12, cursor, starts, u.tilesum, u.tiles);
        else
            msd_scatter_kernel<K, BUCKET_LARGE_MSD_BITS, SORT_ITEMS_BIG, ArrayKeys<K>><<<tiles, BLOCK, 0, s>>>(ArrayKeys<K>{k0}, k1, n_ptr, n_max, low, hist12, cursor, starts, u.tilesum, u.tiles);
        const bool timed = lt && lt->begin(s, tag);
        launch_bucket_keys_kernel<K, BUCKET_KEYS_THREADS_4096, BUCKET_KEYS_ITEMS_4096>(R, s, k1, k0, hist12, low, starts, u.sentinel, u.tilesum, u.tile_shift);
        if (timed) lt->end(s);
        if (hipGetLastError() != hipSuccess) return -1;
        return 0;
    }
    (void)counted;
    fill_u32_kernel<<<R / BLOCK, BLOCK, 0, s>>>(hist12, R, 0u);
    top_digit_histogram_kernel<K><<<tiles, BLOCK, 0, s>>>(k0, n_ptr, n_max, hist12, low, sc.T, sc.table);
    K* kin = k0;
    K* kout = k1;
    u32* vin = v0;
    u32* vout = v1;
    for (int half = 0; half < 2; ++half) {
        const int shift = low + 6 * half;
        if (half == 1)  // (the histogram kernel has left the first pass's counts)
            radix_upsweep_kernel<K, SORT_ITEMS_BIG><<<tiles, BLOCK, 0, s>>>(kin, n_ptr, n_max, sc.T, sc.table, shift, 6);
        radix_scan_kernel<<<64, BLOCK, 0, s>>>(sc.table, sc.totals, n_ptr, n_max, sc.T, BLOCK * SORT_ITEMS_BIG);
        radix_downsweep_kernel<K, HAS_VAL, SORT_ITEMS_BIG>
            <<<tiles, BLOCK, 0, s>>>(kin, kout, vin, vout, n_ptr, n_max, sc.T, sc.table, sc.totals, shift, 6);
        K* tk = kin; kin = kout; kout = tk;
        u32* tv = vin; vin = vout; vout = tv;
    }
    // after two passes the partitioned keys are back in (k0, v0)
    const bool timed = lt && lt->begin(s, tag);
    bucket_sort_kernel<K, HAS_VAL, BUCKET_THREADS_4096, (HAS_VAL ? 16 : 8)>
        <<<R, BUCKET_THREADS_4096, 0, s>>>(k0, k1, v0, v1, hist12, R, low);
    if (timed) lt->end(s);
    if (hipGetLastError() != hipSuccess) return -1;
    return 1;
}

// ---------------------------------------------------------------------------
// Flag compaction.  count kernel: tilesum[tile] = number of i in the tile with
// pred(i).  scatter kernel: calls out(i, rank) for every flagged i, rank = its
// position among flagged items in index order; writes the grand total.
// Tile = 256 x CHUNKS items (CHUNKS = 1, 4 or 16 per lane); wave w of a workgroup
// owns items [w * 64 * CHUNKS, (w + 1) * 64 * CHUNKS) of the tile.  As few items per
// lane as the tile limit allows: with one item per lane nothing in a lane waits
// for the item before it (measured: a limit of 8192 tiles instead of 2048 took
// 9 us off room115k, 29 us off scene1p2m, 21 us off the 16-mesh batch; 16384
// costs scene1p2m 30 us again, every workgroup of the scatter kernel adding up
// the sums of the tiles in front of it).
// ---------------------------------------------------------------------------
constexpr int COMPACT_MAX_SUMMED_TILES = 8192;  // beyond this the tile sums are scanned by a kernel of their own

inline int compact_chunks_for(long long n_max) {
    if ((n_max + BLOCK - 1) / BLOCK <= COMPACT_MAX_SUMMED_TILES) return 1;
    if ((n_max + 4 * BLOCK - 1) / (4 * BLOCK) <= COMPACT_MAX_SUMMED_TILES) return 4;
    return 16;
}
inline int compact_tiles(long long n, int chunks) {
    return (int)((n + (long long)BLOCK * chunks - 1) / ((long long)BLOCK * chunks));
}
// capacity of the tile-sum array for inputs of up to n_cap items
inline int compact_tilesum_capacity(long long n_cap) {
    const int big = compact_tiles(n_cap, 16);
    return (big > COMPACT_MAX_SUMMED_TILES ? big : COMPACT_MAX_SUMMED_TILES) + 1;
}

// A counting predicate may provide `void on_start() const`: one thread of the count kernel calls it
// before anything else, whatever the number of items (used to tell the host that the kernels in
// front of this one on the stream are done).
template <class P, class = void>
struct pred_has_on_start : std::false_type {};
template <class P>
struct pred_has_on_start<P, std::void_t<decltype(std::declval<const P&>().on_start())>> : std::true_type {};

template <class Pred, int CHUNKS>
__global__ __launch_bounds__(BLOCK) void tile_count_kernel(Pred pred, const int* n_ptr, int n_host,
                                                           int* __restrict__ tilesum) {
    constexpr int CTILE = BLOCK * CHUNKS;
    __shared__ u32 smem[WAVES];
    if constexpr (pred_has_on_start<Pred>::value) {
        if (blockIdx.x == 0 && threadIdx.x == 0) pred.on_start();
    }
    const int n = load_count(n_ptr, n_host);
    const long long base = (long long)blockIdx.x * CTILE;
    if (base >= n) return;
    const int w = wave_id(), lane = lane_id();
    u32 cnt = 0;
    for (int c = 0; c < CHUNKS; ++c) {
        const long long i = base + (long long)w * (64 * CHUNKS) + c * 64 + lane;
        const bool f = (i < n) && pred((int)i);
        cnt += (u32)__popcll(__ballot(f));
    }
    if (lane == 0) smem[w] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) tilesum[blockIdx.x] = (int)(smem[0] + smem[1] + smem[2] + smem[3]);
}

// In-place exclusive scan of a[0..T) by one workgroup (used when there are many tiles).
__global__ __launch_bounds__(BLOCK) void scan_tilesums_kernel(int* __restrict__ a, const int* n_ptr, int n_host,
                                                              int tile_items) {
    __shared__ u32 smem[WAVES];
    const int n = load_count(n_ptr, n_host);
    const int T = (int)(((long long)n + tile_items - 1) / tile_items);
    u32 carry = 0;
    for (int c = 0; c < T; c += BLOCK) {
        const int i = c + threadIdx.x;
        u32 v = i < T ? (u32)a[i] : 0u, tot;
        u32 ex = block_exclusive_scan(v, smem, tot);
        if (i < T) a[i] = (int)(carry + ex);
        carry += tot;
    }
}

// An output functor may declare `static constexpr bool WAVE_WIDE = true` and provide
// wave(i, in_range, flagged, pos), which all 64 lanes of a wave call together (so it may use
// cross-lane operations), in place of operator()(i, pos) called by the flagged lanes only.
template <class Out, class = void>
struct out_is_wave_wide : std::false_type {};
template <class Out>
struct out_is_wave_wide<Out, std::enable_if_t<Out::WAVE_WIDE>> : std::true_type {};

template <class Pred, class Out, int CHUNKS>
__global__ __launch_bounds__(BLOCK) void tile_scatter_kernel(Pred pred, Out out, const int* n_ptr, int n_host,
                                                             const int* __restrict__ tilesum, int prefixed,
                                                             int* __restrict__ total_out) {
    constexpr int CTILE = BLOCK * CHUNKS;
    __shared__ u32 smem[WAVES];
    const int n = load_count(n_ptr, n_host);
    if (n <= 0) {
        if (blockIdx.x == 0 && threadIdx.x == 0 && total_out) *total_out = 0;
        return;
    }
    const int tile = blockIdx.x;
    const long long base = (long long)tile * CTILE;
    if (base >= n) return;
    const int t = threadIdx.x, w = wave_id(), lane = lane_id();

    u32 tileoff;
    if (prefixed) {
        tileoff = (u32)tilesum[tile];
    } else {
        u32 part = 0;
        for (int j = t; j < tile; j += BLOCK) part += (u32)tilesum[j];
        tileoff = block_sum(part, smem);
    }

    u64 bal[CHUNKS];
    u32 cnt = 0;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
        const long long i = base + (long long)w * (64 * CHUNKS) + c * 64 + lane;
        const bool f = (i < n) && pred((int)i);
        bal[c] = __ballot(f);
        cnt += (u32)__popcll(bal[c]);
    }
    __syncthreads();
    if (lane == 0) smem[w] = cnt;
    __syncthreads();
    u32 woff = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
        if (i < w) woff += smem[i];
        tot += smem[i];
    }
    u32 run = tileoff + woff;
    const u64 lt = lanemask_lt();
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
        const long long i = base + (long long)w * (64 * CHUNKS) + c * 64 + lane;
        const bool f = ((bal[c] >> lane) & 1ull) != 0;
        const int pos = (int)(run + (u32)__popcll(bal[c] & lt));
        if constexpr (out_is_wave_wide<Out>::value) {
            out.wave((int)i, i < n, f, pos);  // every lane of the wave calls it
        } else {
            if (f) out((int)i, pos);
        }
        run += (u32)__popcll(bal[c]);
    }
    if (base + CTILE >= n && t == 0 && total_out) *total_out = (int)(tileoff + tot);
}

template <class PredCount, class PredScatter, class Out, int CHUNKS>
inline void compact_impl(hipStream_t s, PredCount pc, PredScatter ps, Out out, const int* n_ptr, int n_max,
                         int* tilesum, int* total_out) {
    const int tiles = compact_tiles(n_max > 0 ? n_max : 1, CHUNKS);
    tile_count_kernel<PredCount, CHUNKS><<<tiles, BLOCK, 0, s>>>(pc, n_ptr, n_max, tilesum);
    const int prefixed = tiles > COMPACT_MAX_SUMMED_TILES;
    if (prefixed) scan_tilesums_kernel<<<1, BLOCK, 0, s>>>(tilesum, n_ptr, n_max, BLOCK * CHUNKS);
    tile_scatter_kernel<PredScatter, Out, CHUNKS>
        <<<tiles, BLOCK, 0, s>>>(ps, out, n_ptr, n_max, tilesum, prefixed, total_out);
}

// The two halves of compact() on their own, for callers that put other work between them
// (or launch them on different streams).  Both must be given the same n_max.
template <class PredCount>
inline void compact_count(hipStream_t s, PredCount pc, const int* n_ptr, int n_max, int* tilesum) {
    const int tiles = compact_tiles(n_max > 0 ? n_max : 1, compact_chunks_for(n_max));
    switch (compact_chunks_for(n_max)) {
        case 1: tile_count_kernel<PredCount, 1><<<tiles, BLOCK, 0, s>>>(pc, n_ptr, n_max, tilesum); break;
        case 4: tile_count_kernel<PredCount, 4><<<tiles, BLOCK, 0, s>>>(pc, n_ptr, n_max, tilesum); break;
        default: tile_count_kernel<PredCount, 16><<<tiles, BLOCK, 0, s>>>(pc, n_ptr, n_max, tilesum);
    }
    if (tiles > COMPACT_MAX_SUMMED_TILES)
        scan_tilesums_kernel<<<1, BLOCK, 0, s>>>(tilesum, n_ptr, n_max, BLOCK * compact_chunks_for(n_max));
}

template <class PredScatter, class Out>
inline void compact_scatter(hipStream_t s, PredScatter ps, Out out, const int* n_ptr, int n_max, const int* tilesum,
                            int* total_out) {
    const int chunks = compact_chunks_for(n_max);
    const int tiles = compact_tiles(n_max > 0 ? n_max : 1, chunks);
    const int prefixed = tiles > COMPACT_MAX_SUMMED_TILES;
    switch (chunks) {
        case 1: tile_scatter_kernel<PredScatter, Out, 1><<<tiles, BLOCK, 0, s>>>(ps, out, n_ptr, n_max, tilesum, prefixed, total_out); break;
        case 4: tile_scatter_kernel<PredScatter, Out, 4><<<tiles, BLOCK, 0, s>>>(ps, out, n_ptr, n_max, tilesum, prefixed, total_out); break;
        default: tile_scatter_kernel<PredScatter, Out, 16><<<tiles, BLOCK, 0, s>>>(ps, out, n_ptr, n_max, tilesum, prefixed, total_out);
    }
}

// count pass may use a different functor (e.g. one that also stores the flag)
template <class PredCount, class PredScatter, class Out>
inline void compact(hipStream_t s, PredCount pc, PredScatter ps, Out out, const int* n_ptr, int n_max, int* tilesum,
                    int* total_out) {
    switch (compact_chunks_for(n_max)) {
        case 1: compact_impl<PredCount, PredScatter, Out, 1>(s, pc, ps, out, n_ptr, n_max, tilesum, total_out); break;
        case 4: compact_impl<PredCount, PredScatter, Out, 4>(s, pc, ps, out, n_ptr, n_max, tilesum, total_out); break;
        default: compact_impl<PredCount, PredScatter, Out, 16>(s, pc, ps, out, n_ptr, n_max, tilesum, total_out);
    }
}

}  // namespace prim
