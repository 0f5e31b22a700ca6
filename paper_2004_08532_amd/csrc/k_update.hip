// Duplicate reduction, part 2, fused with the optimizer (paper Sec. 3.1 step 4): for every distinct row that the
// mini-batch touched, add up its gradient rows and apply Adagrad to that row of the global table, in place:
//     S += g^2 ;  theta -= lr * g / (sqrt(S) + eps)
// Table rows that are not in the batch are never touched.
//
// Work is cut by POSITION in the sorted key list, not by row id: every workgroup gets a tile of 4 consecutive
// sorted positions, and a run of equal keys (one distinct row) belongs to the tile in which it ENDS.  One row
// group of the workgroup (one thread per 16 bytes of a row: the "walkers") asks for the table / state rows of the
// runs that end in the tile and for the tile's gradient rows, then walks the tile in sorted order.  If the tile's
// first run began in an earlier tile (a row that occurs often: hub entities of degree-skewed graphs, frequent
// relations), the other waves of the workgroup (the "helpers") find where it began with one parallel look-back
// over the keys and add up those earlier gradient rows, split over their row groups, while the walkers' table
// rows are still on their way; the sums reach the walkers through LDS.  Positions of a run that goes on into the
// next tile are skipped: that tile's workgroup reads them.  One launch, no atomics on data, every sum has a fixed
// order, so the result is a function of the ids and the gradient rows alone.  Entity and relation rows go through
// the same launch; its last workgroup adds the loss terms in a fixed order and advances the device step counter.
#include "kge_common.h"

namespace {

constexpr int TILE_R = 4;   // sorted positions per workgroup (measured: 2, 3, 6, 8 and 16 are slower on every configuration)
constexpr int UPD_THREADS = 512;
constexpr int LOOKBACK_U = 16;  // gradient rows in flight per thread while summing the earlier part of a run

struct UpdateArgs {
    float* T[2];             // tables: entity, relation
    float* St[2];            // Adagrad accumulators
    const float* G[2];       // gradient rows, indexed by key position
    const uint32_t* key[2];  // sorted ids
    const uint32_t* pos[2];  // key position of each sorted entry
    int n[2];                // key list lengths
    int tiles[2];
    int D[2];
    float lr, eps;
    const float* row_loss;       // [b] per-positive loss terms
    const float* neg_loss_part;  // [n_loss_parts] negative-side loss sums of the backward launch (may be none)
    int n_loss_parts;
    int b;
    float* loss_out;        // direct mode: this step's scalar (may be null)
    StepBlock* blk;         // replay mode: the call's loss array and the running step, advanced here by the one
                            // thread that reads it
};

__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

// Workgroup barrier that orders LDS traffic only: global loads that are still in flight stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ROWWISE: the accumulator is one float per row, fed with the mean of the squared elements of the row's summed
// gradient:  S += mean_d g_d^2 ;  theta_d -= lr * g_d / (sqrt(S) + eps).
template <bool ROWWISE>
__global__ __launch_bounds__(UPD_THREADS) void k_update(UpdateArgs a) {
    int tile = blockIdx.x;
    const int tid = threadIdx.x;
    __shared__ __attribute__((aligned(16))) float4 red[UPD_THREADS];
    if (tile == a.tiles[0] + a.tiles[1]) {  // ---- loss: fixed-order tree over the b row terms
        float* part = reinterpret_cast<float*>(red);
        float s = 0.f;
        for (int i = tid; i < a.b; i += UPD_THREADS) s += a.row_loss[i];
        for (int i = tid; i < a.n_loss_parts; i += UPD_THREADS) s += a.neg_loss_part[i];
        part[tid] = s;
        __syncthreads();
        for (int o = UPD_THREADS / 2; o > 0; o >>= 1) {
            if (tid < o) part[tid] += part[tid + o];
            __syncthreads();
        }
        if (tid == 0) {
            if (a.blk) {
                const int64_t step = a.blk->step;
                float* out = a.blk->loss_out;
                if (out) out[step] = part[0];
                a.blk->step = step + 1;  // no other thread of this launch reads the counter
            } else if (a.loss_out) {
                a.loss_out[0] = part[0];
            }
        }
        return;
    }
    const int which = tile >= a.tiles[0];
    if (which) tile -= a.tiles[0];
    const int n = a.n[which], D = a.D[which], D4 = D / 4;
    const uint32_t* keys = a.key[which];
    const uint32_t* poss = a.pos[which];
    const int p0 = tile * TILE_R, p1 = min(p0 + TILE_R, n), cnt = p1 - p0;

    // keys p0-1 .. p1 and positions p0 .. p1-1 of this tile: the addresses are the same for every thread, and so is
    // everything computed from them below, so it all lives in scalar registers
    __shared__ int lookback;
    __shared__ uint32_t back_pos[UPD_THREADS];
    uint32_t key[TILE_R + 2], gpos[TILE_R];
#pragma unroll
    for (int j = 0; j < TILE_R + 2; ++j) {
        const int q = p0 - 1 + j;
        key[j] = __builtin_amdgcn_readfirstlane(keys[q < 0 ? 0 : (q < n ? q : n - 1)]);
    }
#pragma unroll
    for (int j = 0; j < TILE_R; ++j) gpos[j] = __builtin_amdgcn_readfirstlane(poss[p0 + j < n ? p0 + j : n - 1]);
    uint32_t last_key = key[1], next_key = key[2];  // key[cnt], key[cnt + 1]
#pragma unroll
    for (int j = 1; j < TILE_R; ++j) {
        if (j < cnt) { last_key = key[j + 1]; next_key = key[j + 2]; }
    }
    const bool starts_before = p0 > 0 && key[0] == key[1];
    const bool goes_on = p1 < n && last_key == next_key;

    // per position: is its run finished by this tile (need), and does a run end here (ends)
    bool ends[TILE_R], need[TILE_R];
#pragma unroll
    for (int j = 0; j < TILE_R; ++j) {
        need[j] = j < cnt && !(goes_on && key[j + 1] == last_key);
        ends[j] = need[j] && (j == cnt - 1 || key[j + 2] != key[j + 1]);
    }

    const float* G = a.G[which];
    float* Tb = a.T[which];
    float* Sb = a.St[which];
    const int lanes = D4;  // threads per row: one 16-byte column slice each (rows are at most 4 * 256 floats long)
    const int v = tid % lanes;
    // The first `walkers` threads (whole waves) hold the row group that walks the tile; the other waves only help
    // with a run that began before the tile (only if that run is finished here).
    const int walkers = (lanes + 63) & ~63;
    const bool look = starts_before && need[0];  // uniform

    if (tid >= walkers) {
        // ---- helper waves: the part of the tile's first run that lies before the tile
        // Look-back in chunks: helper thread i reads key and gradient-row position of sorted entry p0 - 1 - (base + i);
        // the first entry with another key ends the run.  The positions go to LDS, and the helpers, in row groups of
        // `lanes` threads, add up the gradient rows of the chunk, LOOKBACK_U rows per thread in flight.  The sums of
        // the row groups go to the walkers through LDS.
        if (!look) return;
        const int o = tid - walkers, n_look = UPD_THREADS - walkers;
        const int groups = n_look / lanes, grp = o / lanes;
        const bool active = grp < groups;
        if (o == 0) lookback = 1 << 30;
        float4 part = make_float4(0.f, 0.f, 0.f, 0.f);
        lds_barrier();  // (1)
        for (int base = 0;; base += n_look) {
            const int q = p0 - 1 - (base + o);
            const uint32_t kq = keys[q < 0 ? 0 : q], pq = poss[q < 0 ? 0 : q];
            const bool differs = q < 0 || kq != key[1];
            const unsigned long long bal = __ballot(differs);
            if ((tid & 63) == 0 && bal) atomicMin(&lookback, base + o + __builtin_ctzll(bal));  // one per wave
            back_pos[o] = pq;
            lds_barrier();  // (2)
            const int stop = lookback;                                          // first entry that is not in the run
            const int m = (stop < base + n_look ? stop : base + n_look) - base;  // run entries in this chunk
            if (active) {
                for (int i = grp; i < m; i += groups * LOOKBACK_U) {
                    float4 g[LOOKBACK_U];
#pragma unroll
                    for (int u = 0; u < LOOKBACK_U; ++u) {
                        const int ii = i + u * groups;
                        g[u] = ld4(G + (int64_t)back_pos[ii < m ? ii : i] * D + 4 * (o % lanes));
                    }
#pragma unroll
                    for (int u = 0; u < LOOKBACK_U; ++u) {
                        if (i + u * groups < m) part = add4(part, g[u]);
                    }
                }
            }
            if (stop < (1 << 30)) break;
            lds_barrier();  // (3) back_pos is overwritten by the next chunk
        }
        red[o] = part;
        lds_barrier();  // (4)
        return;
    }

    // ---- walker waves.  A wave gets its loads back in the order it issued them, and the table and state rows of the
    // runs that end here come from far away (random rows of a table that fills the memory): they are asked for
    // first, and while they travel the walkers only pass the helpers' barriers, which order LDS traffic and do not
    // wait for loads.
    const bool walker = tid < lanes;
    float4 x[TILE_R], s[TILE_R];
    float srow[TILE_R];
    if (walker) {
#pragma unroll
        for (int j = 0; j < TILE_R; ++j) {
            if (ends[j]) {
                x[j] = ld4(Tb + (int64_t)key[j + 1] * D + 4 * v);
                if (ROWWISE) srow[j] = Sb[key[j + 1]];
                else s[j] = ld4(Sb + (int64_t)key[j + 1] * D + 4 * v);
            }
        }
    }
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (look) {
        lds_barrier();  // (1)
        for (;;) {
            lds_barrier();  // (2)
            if (lookback < (1 << 30)) break;
            lds_barrier();  // (3)
        }
        lds_barrier();  // (4)
        if (walker) {
            const int groups = (UPD_THREADS - walkers) / lanes;
            for (int g2 = 0; g2 < groups; ++g2) acc = add4(acc, red[g2 * lanes + v]);
        }
    }
    // (row-wise state: the other lanes of the walker waves stay, with zeros, for the sums over the row below)
    if (!ROWWISE && !walker) return;

    float4 g[TILE_R];
#pragma unroll
    for (int j = 0; j < TILE_R; ++j) {
        g[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (need[j] && walker) g[j] = ld4(G + (int64_t)gpos[j] * D + 4 * v);
    }
    if (!ROWWISE) {
#pragma unroll
        for (int j = 0; j < TILE_R; ++j) {
            if (need[j]) acc = add4(acc, g[j]);
            if (ends[j]) {
                adagrad4(acc, x[j], s[j], a.lr, a.eps);
                st4(Sb + (int64_t)key[j + 1] * D + 4 * v, s[j]);
                st4(Tb + (int64_t)key[j + 1] * D + 4 * v, x[j]);
                acc = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
        return;
    }
    // Row-wise state.  First the summed gradient of every run that ends here (kept in g[j]) and, per walker wave, its
    // sum of squares; one barrier (the helper waves are gone by now, so it is among the walker waves only); then the
    // walker waves' sums are added in wave order to the mean square of the row and the update is applied.
    __shared__ float row_ss[TILE_R][UPD_THREADS / 64];
#pragma unroll
    for (int j = 0; j < TILE_R; ++j) {
        if (need[j]) acc = add4(acc, g[j]);
        if (ends[j]) {
            g[j] = acc;
            float ss = walker ? acc.x * acc.x + acc.y * acc.y + acc.z * acc.z + acc.w * acc.w : 0.f;
            ss = wave_sum(ss);
            if ((tid & 63) == 0) row_ss[j][tid >> 6] = ss;
            acc = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    lds_barrier();
    if (!walker) return;
#pragma unroll
    for (int j = 0; j < TILE_R; ++j) {
        if (ends[j]) {
            float tot = 0.f;
            for (int ww = 0; ww < walkers / 64; ++ww) tot += row_ss[j][ww];
            const float S_new = srow[j] + tot / (float)D;
            const float scale = a.lr * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(S_new) + a.eps);
            x[j].x -= scale * g[j].x; x[j].y -= scale * g[j].y; x[j].z -= scale * g[j].z; x[j].w -= scale * g[j].w;
            st4(Tb + (int64_t)key[j + 1] * D + 4 * v, x[j]);
            if (tid == 0) Sb[key[j + 1]] = S_new;
        }
    }
}

}  // namespace

void kge_launch_update(kge_ctx* c, float* E, float* SE, float* R, float* SR, const StepIds& ids, float lr,
                       int n_loss_parts, hipStream_t st) {
    UpdateArgs a;
    const int b = ids.b, n_ent_keys = 2 * ids.b + ids.n_neg, n_rel_keys = ids.b;
    float* loss_out = ids.loss_out;
    a.blk = ids.blk;
    a.T[0] = E; a.T[1] = R; a.St[0] = SE; a.St[1] = SR;
    a.G[0] = c->Gent; a.G[1] = c->Grel;
    a.key[0] = c->ekey[c->ebuf]; a.key[1] = c->rkey[c->rbuf];
    a.pos[0] = c->epos[c->ebuf]; a.pos[1] = c->rpos[c->rbuf];
    // (relation rows that hold D x D matrices have their own update kernels: k_rescal_update, k_transr_update)
    a.n[0] = n_ent_keys; a.n[1] = (c->cfg.model == KGE_RESCAL || c->cfg.model == KGE_TRANSR) ? 0 : n_rel_keys;
    a.tiles[0] = (n_ent_keys + TILE_R - 1) / TILE_R; a.tiles[1] = (a.n[1] + TILE_R - 1) / TILE_R;
    a.D[0] = c->cfg.ent_dim; a.D[1] = c->cfg.rel_dim;
    a.lr = lr; a.eps = c->eps; a.row_loss = c->row_loss; a.b = b; a.loss_out = loss_out;
    a.neg_loss_part = c->neg_loss_part; a.n_loss_parts = n_loss_parts;
    const int tiles = a.tiles[0] + a.tiles[1];
    if (c->cfg.adagrad_mode == 1) KGE_LAUNCH(c, k_update<true>, dim3(tiles + 1), dim3(UPD_THREADS), 0, st, a);
    else KGE_LAUNCH(c, k_update<false>, dim3(tiles + 1), dim3(UPD_THREADS), 0, st, a);
}
