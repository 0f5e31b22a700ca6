// Ordering a step's key lists (entities: heads | tails | corrupting ids; relations) by (id, position) inside blocks
// that ride along in another launch: the duplicate reduction of the update needs nothing but the ids for this, so the
// blocks can sit in whatever launch has room for them.  Shared by the gather / staging launch and the backward launch.
#pragma once
#include "kge_common.h"

namespace {

// One block size for both kinds of block in a launch: THREADS = 256 for short key lists, 1024 for long ones.  The
// rank blocks keep the whole key list in (dynamic) LDS, and every block of a launch is given the same amount; with
// a long list the blocks are large, so that the LDS of a gather block is spread over 16 row-gathering waves and
// does not limit how many of them a CU holds, and so that fewer blocks load the list.
constexpr int RANK_LONG_LIST = 6144;  // keys from which on the 1024-thread blocks are used (measured: lists of 2,200 and 4,096 keys are 4-5 us faster with the small brute-force blocks)
template <int THREADS> struct RankShape {
    static constexpr int R = THREADS == 256 ? 1 : 2;     // keys ranked by one 32-thread group
    static constexpr int ITEMS = (THREADS / 32) * R;     // keys ranked per block
    static constexpr int LOADS = THREADS == 256 ? 16 : 4;  // key loads in flight per thread
};

// Orders a key list by brute-force ranking: rank(i) = #{j : key_j < key_i} + #{j < i : key_j == key_i}.  The lists
// are a few thousand keys, so the n^2 comparisons, spread over n/8 (n/64) blocks that run beside the gather blocks of
// the same launch, cost less than one pass of a single-workgroup sort, need no other kernel and no other stream,
// and give exactly the order a stable sort by id would (equal ids in position order).  Every block holds the whole
// list in LDS.  A group of 32 threads ranks RANK_R consecutive keys: each thread scans every 32nd 16-byte chunk of
// the list and compares it with all RANK_R keys, so a chunk read from LDS serves 4 * RANK_R comparisons.  The tie
// rule costs nothing away from the group's own keys: for entries before them "key_j <= key_i" counts, i.e.
// key_j < key_i + 1, for entries after them key_j < key_i, so the scan is three loops over one comparison each.
template <int THREADS>
__device__ __forceinline__ void rank_block(const KeyList& l, int blk, uint32_t* keys) {
    constexpr int RANK_R = RankShape<THREADS>::R, RANK_ITEMS = RankShape<THREADS>::ITEMS;
    constexpr int RANK_LOADS = RankShape<THREADS>::LOADS, GATHER_THREADS = THREADS;
    const int tid = threadIdx.x, n = l.n;
    const int n4 = (n + 3) & ~3;  // the tail is padded with 0xffffffff, which is larger than any id
    // independent loads are issued before the first is used: one round of memory latency per 4096 keys
    const KeySources ks = key_sources(l);
    for (int base = 0; base < n4; base += RANK_LOADS * GATHER_THREADS) {
        int64_t raw[RANK_LOADS];
#pragma unroll
        for (int u = 0; u < RANK_LOADS; ++u) {
            const int i = base + u * GATHER_THREADS + tid;
            raw[u] = *key_address(l, ks, i < n ? i : 0);  // unconditional: all loads go out together
        }
#pragma unroll
        for (int u = 0; u < RANK_LOADS; ++u) {
            const int i = base + u * GATHER_THREADS + tid;
            if (i < n4) keys[i] = i < n ? clamp_key(l, raw[u]) : 0xffffffffu;
        }
    }
    __syncthreads();
    const int it0 = blk * RANK_ITEMS + (tid >> 5) * RANK_R, t = tid & 31;
    if (it0 >= n) return;
    uint32_t ki[RANK_R];
    int cnt[RANK_R];
#pragma unroll
    for (int r = 0; r < RANK_R; ++r) {
        ki[r] = keys[it0 + r < n4 ? it0 + r : n4 - 1];  // ids are below 2^31, so ki + 1 does not wrap for real keys
        cnt[r] = 0;
    }
    int j = 4 * t;
    // entries wholly before the group's keys: key_j <= key_i
#pragma unroll 2
    for (; j + 3 < it0; j += 128) {
        const uint4 kj = *reinterpret_cast<const uint4*>(keys + j);
#pragma unroll
        for (int r = 0; r < RANK_R; ++r) {
            const uint32_t thr = ki[r] + 1u;
            cnt[r] += (kj.x < thr) + (kj.y < thr) + (kj.z < thr) + (kj.w < thr);
        }
    }
    // the chunk(s) that hold the group's own keys: the full rule
    for (; j < it0 + RANK_R && j < n4; j += 128) {
        const uint4 kj = *reinterpret_cast<const uint4*>(keys + j);
        const uint32_t kv[4] = {kj.x, kj.y, kj.z, kj.w};
#pragma unroll
        for (int r = 0; r < RANK_R; ++r) {
#pragma unroll
            for (int e = 0; e < 4; ++e) cnt[r] += (kv[e] < ki[r] || (kv[e] == ki[r] && j + e < it0 + r)) ? 1 : 0;
        }
    }
    // entries after them: key_j < key_i
#pragma unroll 2
    for (; j < n4; j += 128) {
        const uint4 kj = *reinterpret_cast<const uint4*>(keys + j);
#pragma unroll
        for (int r = 0; r < RANK_R; ++r) cnt[r] += (kj.x < ki[r]) + (kj.y < ki[r]) + (kj.z < ki[r]) + (kj.w < ki[r]);
    }
    const int half = key_out_half(l);
#pragma unroll
    for (int r = 0; r < RANK_R; ++r) {
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) cnt[r] += __shfl_xor(cnt[r], o, 32);
        if (t == 0 && it0 + r < n) {
            l.key[half][cnt[r]] = ki[r];
            l.pos[half][cnt[r]] = (uint32_t)(it0 + r);
        }
    }
}

// Long lists (RANK_LONG_LIST keys and more): brute force would compare every key with every other (1.5e8 comparisons
// for 12,288 keys, which set the duration of the whole launch).  Here a block of 1024 threads ranks 1024 keys with
// work linear in the list.  The id range [0, n_ids) is cut into RANK_BUCKETS equal slices, so buckets are ordered
// like the ids they hold.  Every block (1) counts the keys per bucket with LDS atomics, (2) turns the counts into
// offsets, (3) drops one word per key into its bucket's stretch of LDS, in whatever order the atomics hand out:
// (id - first id of the bucket) << 14 | position, so that the words of a bucket compare like (id, position) pairs,
// and (4) ranks its own 1024 keys: offset of the key's bucket + the number of smaller words in that bucket.  The
// result does not depend on the order inside the buckets.  Needs positions below 2^14 (lists end at 14,336 keys) and
// buckets narrower than 2^18 ids (tables of up to 134 M rows; larger ones keep the brute-force blocks).
constexpr int RANK_BUCKETS = 512;
constexpr int RANK_POS_BITS = 14;
__host__ __device__ constexpr size_t bucketed_lds_words(int n) { return (size_t)n + 3 * RANK_BUCKETS + 16; }
inline bool bucketed_ranking_fits(int64_t n_ids) { return n_ids / RANK_BUCKETS + 2 < (1 << (32 - RANK_POS_BITS)); }

__device__ __forceinline__ void rank_block_bucketed(const KeyList& l, int blk, uint64_t bucket_mul, uint32_t* lds) {
    constexpr int T = 1024, MAXK = KGE_RANK_MAX_KEYS / T;  // keys per thread: position u * T + tid
    const int tid = threadIdx.x, n = l.n;
    uint32_t* word = lds;                               // [n] one word per key, bucket after bucket
    int* cnt = reinterpret_cast<int*>(lds + n);         // [RANK_BUCKETS]
    int* off = cnt + RANK_BUCKETS;                      // [RANK_BUCKETS] exclusive prefix of cnt
    uint32_t* first = reinterpret_cast<uint32_t*>(off + RANK_BUCKETS);  // [RANK_BUCKETS] smallest id of the bucket
    int* wave_tot = reinterpret_cast<int*>(first + RANK_BUCKETS);       // [8]
    if (tid < RANK_BUCKETS) {
        cnt[tid] = 0;
        // bucket(id) = (id * bucket_mul) >> 32 >= tid  <=>  id >= ceil((tid << 32) / bucket_mul)
        first[tid] = (uint32_t)((((uint64_t)tid << 32) + bucket_mul - 1) / bucket_mul);
    }
    const KeySources ks = key_sources(l);
    int64_t raw[MAXK];
#pragma unroll
    for (int u = 0; u < MAXK; ++u) {
        const int p = u * T + tid;
        raw[u] = *key_address(l, ks, p < n ? p : 0);
    }
    __syncthreads();
    uint32_t key[MAXK];
    int bucket[MAXK], slot[MAXK];
#pragma unroll
    for (int u = 0; u < MAXK; ++u) {
        key[u] = clamp_key(l, raw[u]);
        bucket[u] = (int)(((uint64_t)key[u] * bucket_mul) >> 32);
        slot[u] = u * T + tid < n ? atomicAdd(&cnt[bucket[u]], 1) : 0;
    }
    __syncthreads();
    if (tid < RANK_BUCKETS) {  // exclusive prefix over the bucket counts: scan inside the 8 waves, then across them
        const int c = cnt[tid];
        int inc = c;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(inc, o, 64);
            if ((tid & 63) >= o) inc += v;
        }
        if ((tid & 63) == 63) wave_tot[tid >> 6] = inc;
        off[tid] = inc - c;
    }
    __syncthreads();
    if (tid < RANK_BUCKETS) {
        int before = 0;
        for (int w = 0; w < (tid >> 6); ++w) before += wave_tot[w];
        off[tid] += before;
    }
    __syncthreads();
    uint32_t mine_word = 0;
    int mine_bucket = 0;
#pragma unroll
    for (int u = 0; u < MAXK; ++u) {
        const uint32_t wd = ((key[u] - first[bucket[u]]) << RANK_POS_BITS) | (uint32_t)(u * T + tid);
        if (u * T + tid < n) word[off[bucket[u]] + slot[u]] = wd;
        if (u == blk) { mine_word = wd; mine_bucket = bucket[u]; }  // this block ranks positions blk * T + tid
    }
    __syncthreads();
    const int mine = blk * T + tid;
    if (mine >= n) return;
    const int lo = off[mine_bucket], hi = lo + cnt[mine_bucket];
    int before = lo;
#pragma unroll 4
    for (int j = lo; j < hi; ++j) before += word[j] < mine_word ? 1 : 0;
    const int half = key_out_half(l);
    l.key[half][before] = (mine_word >> RANK_POS_BITS) + first[mine_bucket];
    l.pos[half][before] = (uint32_t)mine;
}

}  // namespace
