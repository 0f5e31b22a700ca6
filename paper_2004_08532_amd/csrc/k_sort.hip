// Duplicate reduction, part 1, for LONG key lists: sort the (row id, position) pairs of a mini-batch.
//
// A mini-batch touches few rows and may touch one row many times (paper Sec. 2); before the optimizer runs,
// all gradient rows of one embedding row have to be added up, so the key lists (2b + (b/g)k entity keys, b
// relation keys) are brought into (id, position) order.  Lists of up to KGE_RANK_MAX_KEYS keys are ordered by the
// rank blocks of the gather launch (k_gather.hip).  Longer lists are sorted here: ONE workgroup of 1024 threads per
// list, least-significant-digit radix sort, 8 bits per pass, over only as many bits as the table's row count
// needs, ping-ponging through global memory.  Within a pass every wavefront owns a contiguous slice of the list;
// equal digits inside a 64-key round are ranked with ballots, so the sort is stable and equal ids end up ordered
// by position.  Block 0 sorts the entity keys, block 1 the relation keys; the kernel runs on its own stream beside
// the forward/backward kernels.  This file also holds the export of distinct ids and counts (test hook).
#include "kge_common.h"

namespace {

constexpr int SORT_THREADS = 1024;
constexpr int SORT_WAVES = SORT_THREADS / 64;

__global__ __launch_bounds__(SORT_THREADS) void k_sort(KeyList ent, KeyList rel) {
    const KeyList& l = blockIdx.x == 0 ? ent : rel;
    __shared__ volatile uint32_t hist[SORT_WAVES][256];
    __shared__ uint32_t wave_tot[4];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n = l.n;
    const int per_wave = (((n + SORT_WAVES - 1) / SORT_WAVES) + 63) / 64 * 64;
    const int begin = min(n, w * per_wave), end = min(n, begin + per_wave);
    const uint64_t lt_mask = (1ull << lane) - 1ull;

    for (int pass = 0; pass < l.passes; ++pass) {
        const int shift = 8 * pass;
        const uint32_t* kin = pass == 0 ? nullptr : l.key[(pass - 1) & 1];
        const uint32_t* pin = pass == 0 ? nullptr : l.pos[(pass - 1) & 1];
        uint32_t* kout = l.key[pass & 1];
        uint32_t* pout = l.pos[pass & 1];

        for (int e = tid; e < SORT_WAVES * 256; e += SORT_THREADS) hist[e >> 8][e & 255] = 0;
        __syncthreads();

        // ---- per-wave digit counts
        for (int base = begin; base < end; base += 64) {
            const int idx = base + lane;
            const bool valid = idx < end;
            const uint32_t key = valid ? (pass == 0 ? fetch_key(l, idx) : kin[idx]) : 0u;
            const uint32_t d = (key >> shift) & 255u;
            uint64_t peers = __ballot(valid);
#pragma unroll
            for (int bit = 0; bit < 8; ++bit) {
                const bool one = (d >> bit) & 1u;
                const uint64_t bm = __ballot(valid && one);
                peers &= one ? bm : ~bm;
            }
            if (valid && (peers & lt_mask) == 0) hist[w][d] = hist[w][d] + (uint32_t)__popcll(peers);
        }
        __syncthreads();

        // ---- offsets: digit-major, wave-minor exclusive prefix
        uint32_t total = 0;
        if (tid < 256) {
            for (int ww = 0; ww < SORT_WAVES; ++ww) {
                const uint32_t v = hist[ww][tid];
                hist[ww][tid] = total;
                total += v;
            }
        }
        // exclusive scan of the 256 digit totals (threads 0..255 = waves 0..3)
        uint32_t incl = total;
        if (tid < 256) {
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t up = __shfl_up(incl, o, 64);
                if (lane >= o) incl += up;
            }
            if (lane == 63) wave_tot[w] = incl;
        }
        __syncthreads();
        if (tid < 256) {
            uint32_t off = incl - total;
            for (int ww = 0; ww < w; ++ww) off += wave_tot[ww];
            for (int ww = 0; ww < SORT_WAVES; ++ww) hist[ww][tid] = hist[ww][tid] + off;
        }
        __syncthreads();

        // ---- stable scatter
        for (int base = begin; base < end; base += 64) {
            const int idx = base + lane;
            const bool valid = idx < end;
            const uint32_t key = valid ? (pass == 0 ? fetch_key(l, idx) : kin[idx]) : 0u;
            const uint32_t pos = valid ? (pass == 0 ? (uint32_t)idx : pin[idx]) : 0u;
            const uint32_t d = (key >> shift) & 255u;
            uint64_t peers = __ballot(valid);
#pragma unroll
            for (int bit = 0; bit < 8; ++bit) {
                const bool one = (d >> bit) & 1u;
                const uint64_t bm = __ballot(valid && one);
                peers &= one ? bm : ~bm;
            }
            uint32_t dst = 0;
            if (valid) dst = hist[w][d] + (uint32_t)__popcll(peers & lt_mask);
            __builtin_amdgcn_wave_barrier();
            if (valid) {
                kout[dst] = key;
                pout[dst] = pos;
                if ((peers & lt_mask) == 0) hist[w][d] = hist[w][d] + (uint32_t)__popcll(peers);
            }
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();
    }
}

// Test hook: distinct ids and their multiplicities from a sorted key list (one workgroup).
__global__ __launch_bounds__(1024) void k_dedup_export(const uint32_t* keys, int n, int64_t* uniq, int32_t* count,
                                                       int64_t* n_unique) {
    __shared__ uint32_t wave_cnt[16];
    __shared__ uint32_t running;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (tid == 0) running = 0;
    __syncthreads();
    for (int base = 0; base < n; base += 1024) {
        const int p = base + tid;
        const bool is_head = p < n && (p == 0 || keys[p - 1] != keys[p]);
        const uint64_t bal = __ballot(is_head);
        const uint32_t in_wave = (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[w] = (uint32_t)__popcll(bal);
        __syncthreads();
        uint32_t off = running;
        for (int ww = 0; ww < w; ++ww) off += wave_cnt[ww];
        if (is_head) {
            const uint32_t key = keys[p];
            int q = p + 1;
            while (q < n && keys[q] == key) ++q;
            uniq[off + in_wave] = (int64_t)key;
            count[off + in_wave] = q - p;
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t s = running;
            for (int ww = 0; ww < 16; ++ww) s += wave_cnt[ww];
            running = s;
        }
        __syncthreads();
    }
    if (tid == 0) *n_unique = (int64_t)running;
}

int passes_for(int64_t n_ids) {
    int bits = 1;
    while (bits < 32 && (((int64_t)1) << bits) < n_ids) ++bits;
    return (bits + 7) / 8;
}

}  // namespace

void kge_make_key_lists(kge_ctx* c, const StepIds& ids, KeyList* ent, KeyList* rel) {
    KeyList e = {}, rl = {};
    const int b = ids.b, n_neg = ids.n_neg;
    e.src[0] = ids.h; e.src[1] = ids.t; e.src[2] = ids.neg;
    e.n_src[0] = b; e.n_src[1] = b; e.n_src[2] = n_neg;
    e.step_stride[0] = b; e.step_stride[1] = b; e.step_stride[2] = n_neg; e.step_ptr = ids.step_ptr;
    e.n = 2 * b + n_neg;
    e.passes = passes_for(c->cfg.num_entities);
    e.n_ids = c->cfg.num_entities;
    e.key[0] = c->ekey[0]; e.key[1] = c->ekey[1]; e.pos[0] = c->epos[0]; e.pos[1] = c->epos[1];
    rl.src[0] = ids.r; rl.src[1] = ids.r; rl.src[2] = ids.r;
    rl.n_src[0] = b; rl.n_src[1] = 0; rl.n_src[2] = 0;
    rl.step_stride[0] = b; rl.step_stride[1] = b; rl.step_stride[2] = b; rl.step_ptr = ids.step_ptr;
    rl.n = b;
    rl.passes = passes_for(c->cfg.num_relations);
    rl.n_ids = c->cfg.num_relations;
    rl.key[0] = c->rkey[0]; rl.key[1] = c->rkey[1]; rl.pos[0] = c->rpos[0]; rl.pos[1] = c->rpos[1];
    c->last_ent_keys = e.n;
    c->last_rel_keys = rl.n;
    *ent = e;
    *rel = rl;
}

// Radix sort of both key lists (lists too long for the rank path of the gather launch).
void kge_launch_sort(kge_ctx* c, const StepIds& ids, hipStream_t st) {
    KeyList e, rl;
    kge_make_key_lists(c, ids, &e, &rl);
    c->ebuf = (e.passes - 1) & 1;
    c->rbuf = (rl.passes - 1) & 1;
    KGE_LAUNCH(c, k_sort, dim3(2), dim3(SORT_THREADS), 0, st, e, rl);
}

void kge_launch_dedup_export(kge_ctx* c, int which, int64_t* uniq, int32_t* count, int64_t* n_unique,
                             hipStream_t st) {
    const uint32_t* keys = which == 0 ? c->ekey[c->ebuf] : c->rkey[c->rbuf];
    const int n = (int)(which == 0 ? c->last_ent_keys : c->last_rel_keys);
    hipLaunchKernelGGL(k_dedup_export, dim3(1), dim3(1024), 0, st, keys, n, uniq, count, n_unique);
}
