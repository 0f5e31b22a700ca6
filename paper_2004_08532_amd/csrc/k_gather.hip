// Row gather with fused positive forward (paper Sec. 3.1 step 2 and the first half of step 3).
//
// One wavefront per row.  A wave reads the rows it needs with 16-byte loads (a 1600-byte row is 100 such
// loads, lanes 0..63 then 0..35, so every request is a run of whole cache lines), forms
//     o_i = phi(a_i, r_i)   (Sec. 3.3: o = h + r for TransE; a*r, a*conj(r), rotations for the other models)
// scores the positive pair psi(o_i, c_i) (Table 1) with a shuffle reduction, and writes o_i once into the
// dense staging array that the chunked negative scoring reads.  Waves past the positives copy the k
// corrupting rows of every chunk into staging (the O(bkd/g) rows of Sec. 3.3) and compute |n|^2 for TransE-L2.
// In a training step the same launch carries extra blocks that bring the step's key lists into (id, position)
// order for the duplicate reduction (rank_block below): that work needs only the ids, so it rides along here.
#include "kge_common.h"

namespace {

struct GatherArgs {
    const float* E;
    const float* R;
    StepIds ids;
    int b, n_neg, D, Dr, bf16;
    float gamma;
    int64_t n_ent, n_rel;
    float* O;
    float* Nst;
    uint16_t* Obf;  // bf16 operands: o_i and the corrupting rows as the products read them (row pitch ld_bf);
    uint16_t* Nbf;  // Nst is then not written
    int ld_bf;
    float* fpos;
    float* pos_out;
    float* o_n2;
    float* n_n2;
    float* cpos;      // dL/df+_i = -sigmoid(-f+_i) / b
    float* inv_dpos;  // TransE-L2: 1 / |o_i - c_i| (0 if the distance is 0)
    float* row_loss;  // softplus(-f+_i) / b
    int32_t* rank_out;  // evaluation with ranks counted by the forward launch: set to 1 here (else null)
    int rank_blocks;         // blocks [0, rank_blocks) order the key lists, the others gather rows
    int ent_rank_blocks;     // the first ent_rank_blocks of them order the entity key list, the rest the relation keys
    uint64_t bucket_mul;     // long entity lists: bucket of an id = (id * bucket_mul) >> 32 (0: brute-force blocks)
    KeyList ent, rel;
};

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
#pragma unroll
    for (int r = 0; r < RANK_R; ++r) {
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) cnt[r] += __shfl_xor(cnt[r], o, 32);
        if (t == 0 && it0 + r < n) {
            l.key[0][cnt[r]] = ki[r];
            l.pos[0][cnt[r]] = (uint32_t)(it0 + r);
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
    // a bucket holds 24 words on average, the bucket of a hub entity hundreds, and the wave waits for its longest
    // scan: four words per LDS read once the position is a multiple of four
    int j = lo;
    for (; j < hi && (j & 3) != 0; ++j) before += word[j] < mine_word ? 1 : 0;
#pragma unroll 4
    for (; j + 3 < hi; j += 4) {
        const uint4 w4 = *reinterpret_cast<const uint4*>(word + j);
        before += (w4.x < mine_word) + (w4.y < mine_word) + (w4.z < mine_word) + (w4.w < mine_word);
    }
    for (; j < hi; ++j) before += word[j] < mine_word ? 1 : 0;
    l.key[0][before] = (mine_word >> RANK_POS_BITS) + first[mine_bucket];
    l.pos[0][before] = (uint32_t)mine;
}

__device__ __forceinline__ int64_t clamp_id(int64_t id, int64_t n) { return id < 0 ? 0 : (id >= n ? n - 1 : id); }

// four floats -> four bf16 (round to nearest even), stored as 8 bytes
__device__ __forceinline__ void st4_bf16(uint16_t* p, float x0, float x1, float x2, float x3) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 a, b;
    a[0] = (__bf16)x0; a[1] = (__bf16)x1; b[0] = (__bf16)x2; b[1] = (__bf16)x3;
    *reinterpret_cast<uint2*>(p) = make_uint2(__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, b));
}

// NV = 16-byte vectors per lane: ceil(D/4/64) for the real models, ceil(D/8/64) (re, im) pairs for the complex ones.
template <int MODEL, int NV, int THREADS>
__global__ __launch_bounds__(THREADS) void k_gather(GatherArgs a) {
    constexpr int ROWS_PER_BLOCK = THREADS / 64;
    extern __shared__ __attribute__((aligned(16))) uint32_t rank_keys[];  // (read 16 bytes at a time)
    // the rank blocks come first: they run longest and need nothing but the ids
    if ((int)blockIdx.x < a.rank_blocks) {
        const int rb = blockIdx.x;
        if (rb < a.ent_rank_blocks) {
            if (THREADS == 1024 && a.bucket_mul != 0) rank_block_bucketed(a.ent, rb, a.bucket_mul, rank_keys);
            else rank_block<THREADS>(a.ent, rb, rank_keys);
        } else {
            rank_block<THREADS>(a.rel, rb - a.ent_rank_blocks, rank_keys);
        }
        return;
    }
    const int lane = threadIdx.x & 63;
    const int row = (blockIdx.x - a.rank_blocks) * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    const int D = a.D;
    constexpr bool CPLX = (MODEL == KGE_COMPLEX || MODEL == KGE_ROTATE);
    const int nvec = CPLX ? D / 8 : D / 4;   // vectors (or re/im vector pairs) per row
    const int im_off = D / 2;                // float offset of the imaginary half

    if (row >= a.b + a.n_neg) return;
    const StepView sv = step_view(a.ids);

    if (row >= a.b) {  // ---- a corrupting row: copy it to staging
        const int j = row - a.b;
        const int64_t id = clamp_id(sv.neg[j], a.n_ent);
        const float* src = a.E + id * (int64_t)D;
        float* dst = a.Nst + (int64_t)j * D;
        float nn = 0.f;
        const int nv4 = D / 4;
        // every piece of the row is asked for before the first one is used (a load under a branch is waited for
        // where the branch ends: lanes past the row's end read its first piece instead)
        float4 xs[CPLX ? 2 * NV : NV];
#pragma unroll
        for (int it = 0; it < (CPLX ? 2 * NV : NV); ++it) xs[it] = ld4(src + 4 * (lane + it * 64 < nv4 ? lane + it * 64 : 0));
#pragma unroll
        for (int it = 0; it < (CPLX ? 2 * NV : NV); ++it) {
            const int v = lane + it * 64;
            if (v < nv4) {
                const float4 x = xs[it];
                float xv[4] = {x.x, x.y, x.z, x.w};
                if (a.bf16) {  // the product kernels round their operands to bf16: the norm is that of the rounded row
#pragma unroll
                    for (int e = 0; e < 4; ++e) xv[e] = round_bf16(xv[e]);
                }
                if (a.bf16) st4_bf16(a.Nbf + (int64_t)j * a.ld_bf + 4 * v, x.x, x.y, x.z, x.w);
                else st4(dst + 4 * v, x);
                nn += xv[0] * xv[0] + xv[1] * xv[1] + xv[2] * xv[2] + xv[3] * xv[3];
            }
        }
        if (MODEL == KGE_TRANSE_L2) {
            nn = wave_sum(nn);
            if (lane == 0) a.n_n2[j] = nn;
        }
        return;
    }

    // ---- a positive: rows a (kept entity), r, c (the entity that the negatives replace)
    if constexpr (MODEL == KGE_TRANSR) return;  // k_transr_phi has done the positives (they need the matrix)
    const int i = row;
    const int64_t hid = clamp_id(sv.h[i], a.n_ent), tid = clamp_id(sv.t[i], a.n_ent);
    const int64_t rid = clamp_id(sv.r[i], a.n_rel);
    const bool head = sv.side == KGE_NEG_HEAD;
    const float* pa = a.E + (head ? tid : hid) * (int64_t)D;
    const float* pc = a.E + (head ? hid : tid) * (int64_t)D;
    const float* pr = a.R + rid * (int64_t)a.Dr;
    float* po = a.O + (int64_t)i * D;
    float acc = 0.f, on = 0.f;

    // all loads first, as for the corrupting rows.  L1 .. L6: the (up to six) 16-byte pieces that piece v of o needs
    float4 L1[NV], L2[NV], L3[NV], L4[NV], L5[NV], L6[NV];
#pragma unroll
    for (int it = 0; it < NV; ++it) {
        const int vs = lane + it * 64 < nvec ? lane + it * 64 : 0;
        if constexpr (MODEL == KGE_RESCAL) {
            L1[it] = ld4(po + 4 * vs); L2[it] = ld4(pc + 4 * vs);
        } else if constexpr (!CPLX) {
            L1[it] = ld4(pa + 4 * vs); L2[it] = ld4(pr + 4 * vs); L3[it] = ld4(pc + 4 * vs);
        } else {
            L1[it] = ld4(pa + 4 * vs); L2[it] = ld4(pa + im_off + 4 * vs);
            L3[it] = ld4(pc + 4 * vs); L4[it] = ld4(pc + im_off + 4 * vs);
            L5[it] = ld4(pr + 4 * vs);
            if (MODEL != KGE_ROTATE) L6[it] = ld4(pr + im_off + 4 * vs);
        }
    }
#pragma unroll
    for (int it = 0; it < NV; ++it) {
        const int v = lane + it * 64;
        if (v >= nvec) continue;
        if constexpr (MODEL == KGE_RESCAL) {
            // o_i = M_r^T h or M_r t is already in staging (k_rescal); the positive's score is o . c
            const float4 Oo = L1[it], Cc = L2[it];
            acc += Oo.x * Cc.x + Oo.y * Cc.y + Oo.z * Cc.z + Oo.w * Cc.w;
            if (a.bf16) {
                const float n0 = round_bf16(Oo.x), n1 = round_bf16(Oo.y), n2 = round_bf16(Oo.z), n3 = round_bf16(Oo.w);
                on += n0 * n0 + n1 * n1 + n2 * n2 + n3 * n3;
            }
        } else if constexpr (!CPLX) {
            const float4 A = L1[it], Rr = L2[it], Cc = L3[it];
            const float av[4] = {A.x, A.y, A.z, A.w}, rv[4] = {Rr.x, Rr.y, Rr.z, Rr.w}, cv[4] = {Cc.x, Cc.y, Cc.z, Cc.w};
            float ov[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (MODEL == KGE_DISTMULT) ov[e] = av[e] * rv[e];
                else ov[e] = head ? av[e] - rv[e] : av[e] + rv[e];
            }
            st4(po + 4 * v, make_float4(ov[0], ov[1], ov[2], ov[3]));
            if (a.bf16) st4_bf16(a.Obf + (int64_t)i * a.ld_bf + 4 * v, ov[0], ov[1], ov[2], ov[3]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (MODEL == KGE_DISTMULT) acc += ov[e] * cv[e];
                else if (MODEL == KGE_TRANSE_L1) acc += fabsf(ov[e] - cv[e]);
                else { const float u = ov[e] - cv[e]; acc += u * u; }
            }
            if (MODEL == KGE_TRANSE_L2 || a.bf16) {
                float nv[4] = {ov[0], ov[1], ov[2], ov[3]};
                if (a.bf16) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) nv[e] = round_bf16(nv[e]);
                }
                on += nv[0] * nv[0] + nv[1] * nv[1] + nv[2] * nv[2] + nv[3] * nv[3];
            }
        } else {
            const float4 Are = L1[it], Aim = L2[it];
            const float4 Cre = L3[it], Cim = L4[it];
            const float are[4] = {Are.x, Are.y, Are.z, Are.w}, aim[4] = {Aim.x, Aim.y, Aim.z, Aim.w};
            const float cre[4] = {Cre.x, Cre.y, Cre.z, Cre.w}, cim[4] = {Cim.x, Cim.y, Cim.z, Cim.w};
            float rre[4], rim[4];
            if (MODEL == KGE_ROTATE) {
                const float4 Th = L5[it];
                const float th[4] = {Th.x, Th.y, Th.z, Th.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) sincosf(th[e], &rim[e], &rre[e]);
            } else {
                const float4 Rre = L5[it], Rim = L6[it];
                rre[0] = Rre.x; rre[1] = Rre.y; rre[2] = Rre.z; rre[3] = Rre.w;
                rim[0] = Rim.x; rim[1] = Rim.y; rim[2] = Rim.z; rim[3] = Rim.w;
            }
            float ore[4], oim[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float ri = head ? -rim[e] : rim[e];  // head corruption: o = t * conj(r)
                ore[e] = are[e] * rre[e] - aim[e] * ri;
                oim[e] = are[e] * ri + aim[e] * rre[e];
            }
            st4(po + 4 * v, make_float4(ore[0], ore[1], ore[2], ore[3]));
            st4(po + im_off + 4 * v, make_float4(oim[0], oim[1], oim[2], oim[3]));
            if (a.bf16) {
                st4_bf16(a.Obf + (int64_t)i * a.ld_bf + 4 * v, ore[0], ore[1], ore[2], ore[3]);
                st4_bf16(a.Obf + (int64_t)i * a.ld_bf + im_off + 4 * v, oim[0], oim[1], oim[2], oim[3]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (MODEL == KGE_COMPLEX) acc += ore[e] * cre[e] + oim[e] * cim[e];
                else {
                    const float qre = ore[e] - cre[e], qim = oim[e] - cim[e];
                    acc += sqrtf(qre * qre + qim * qim);
                }
            }
        }
    }
    acc = wave_sum(acc);
    if (MODEL == KGE_TRANSE_L2) on = wave_sum(on);
    if (lane == 0) {
        float f;
        if (MODEL == KGE_TRANSE_L2) f = a.gamma - sqrtf(acc);
        else if (MODEL == KGE_TRANSE_L1 || MODEL == KGE_ROTATE) f = a.gamma - acc;
        else f = acc;
        a.fpos[i] = f;
        if (a.pos_out) a.pos_out[i] = f;
        if (a.rank_out) a.rank_out[i] = 1;
        if (MODEL == KGE_TRANSE_L2) {
            a.o_n2[i] = on;
            a.inv_dpos[i] = acc > 0.f ? 1.f / sqrtf(acc) : 0.f;
        }
        // positive part of the logistic loss (Sec. 2, y = +1) and its derivative
        const float invb = 1.f / (float)a.b;
        const float e = expf(-fabsf(f));
        a.row_loss[i] = (fmaxf(-f, 0.f) + log1pf(e)) * invb;
        a.cpos[i] = -((f >= 0.f ? e : 1.f) / (1.f + e)) * invb;
    }
}

template <int MODEL, int THREADS>
void launch_nv(kge_ctx* c, const GatherArgs& a, int nv, dim3 grid, size_t lds, hipStream_t st) {
    switch (nv) {
    case 1: KGE_LAUNCH(c, (k_gather<MODEL, 1, THREADS>), grid, dim3(THREADS), lds, st, a); break;
    case 2: KGE_LAUNCH(c, (k_gather<MODEL, 2, THREADS>), grid, dim3(THREADS), lds, st, a); break;
    case 3: KGE_LAUNCH(c, (k_gather<MODEL, 3, THREADS>), grid, dim3(THREADS), lds, st, a); break;
    default: KGE_LAUNCH(c, (k_gather<MODEL, 4, THREADS>), grid, dim3(THREADS), lds, st, a); break;
    }
}

template <int THREADS>
void launch_model(kge_ctx* c, GatherArgs& a, int nv, int rows, bool with_keys, const StepIds& ids, hipStream_t st) {
    const int gather_blocks = (rows + THREADS / 64 - 1) / (THREADS / 64);
    a.ent_rank_blocks = 0;
    int rank_blocks = 0;
    size_t lds = 0;
    if (with_keys) {
        constexpr int ITEMS = RankShape<THREADS>::ITEMS;
        kge_make_key_lists(c, ids, &a.ent, &a.rel);
        a.bucket_mul = 0;
        if (THREADS == 1024 && bucketed_ranking_fits(a.ent.n_ids)) {  // long entity list: 1024 keys per block
            a.ent_rank_blocks = (a.ent.n + 1023) / 1024;
            a.bucket_mul = ((uint64_t)RANK_BUCKETS << 32) / (uint64_t)a.ent.n_ids;
            lds = sizeof(uint32_t) * bucketed_lds_words(a.ent.n);
            const size_t rel_lds = sizeof(uint32_t) * (size_t)((a.rel.n + 3) & ~3);
            if (rel_lds > lds) lds = rel_lds;
        } else {
            a.ent_rank_blocks = (a.ent.n + ITEMS - 1) / ITEMS;
            lds = sizeof(uint32_t) * (size_t)((a.ent.n + 3) & ~3);  // the entity list is the longer one
        }
        rank_blocks = a.ent_rank_blocks + (a.rel.n + ITEMS - 1) / ITEMS;
        c->ebuf = 0;
        c->rbuf = 0;
    }
    a.rank_blocks = rank_blocks;
    const dim3 grid(gather_blocks + rank_blocks);
    switch (c->cfg.model) {
    case KGE_TRANSE_L2: launch_nv<KGE_TRANSE_L2, THREADS>(c, a, nv, grid, lds, st); break;
    case KGE_TRANSE_L1: launch_nv<KGE_TRANSE_L1, THREADS>(c, a, nv, grid, lds, st); break;
    case KGE_DISTMULT: launch_nv<KGE_DISTMULT, THREADS>(c, a, nv, grid, lds, st); break;
    case KGE_COMPLEX: launch_nv<KGE_COMPLEX, THREADS>(c, a, nv, grid, lds, st); break;
    case KGE_RESCAL: launch_nv<KGE_RESCAL, THREADS>(c, a, nv, grid, lds, st); break;
    case KGE_TRANSR: launch_nv<KGE_TRANSR, THREADS>(c, a, nv, grid, lds, st); break;
    default: launch_nv<KGE_ROTATE, THREADS>(c, a, nv, grid, lds, st); break;
    }
}

}  // namespace

void kge_launch_gather(kge_ctx* c, const float* E, const float* R, const StepIds& ids, float gamma, float* pos_out,
                       bool with_keys, hipStream_t st) {
    GatherArgs a;
    const int b = ids.b, n_neg = ids.n_neg;
    a.E = E; a.R = R; a.ids = ids;
    a.b = b; a.n_neg = n_neg; a.D = c->cfg.ent_dim; a.Dr = c->cfg.rel_dim;
    a.bf16 = c->cfg.gemm_input;
    a.gamma = gamma; a.n_ent = c->cfg.num_entities; a.n_rel = c->cfg.num_relations;
    a.Obf = c->Obf; a.Nbf = c->Nbf; a.ld_bf = c->ld_bf;
    a.O = c->O; a.Nst = c->Nst; a.fpos = c->fpos; a.pos_out = pos_out; a.o_n2 = c->o_n2; a.n_n2 = c->n_n2;
    a.cpos = c->cpos; a.inv_dpos = c->inv_dpos; a.row_loss = c->row_loss; a.rank_out = c->rank_out;
    const int model = c->cfg.model;
    const bool cplx = model == KGE_COMPLEX || model == KGE_ROTATE;
    const int nvec = cplx ? a.D / 8 : a.D / 4;
    const int nv = (nvec + 63) / 64;
    if (with_keys && 2 * b + n_neg >= RANK_LONG_LIST) launch_model<1024>(c, a, nv, b + n_neg, with_keys, ids, st);
    else launch_model<256>(c, a, nv, b + n_neg, with_keys, ids, st);
}
