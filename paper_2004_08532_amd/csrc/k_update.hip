// Duplicate reduction, part 2, fused with the optimizer (paper Sec. 3.1 step 4): for every distinct row that the
// mini-batch touched, add up its gradient rows and apply Adagrad to that row of the global table, in place:
//     S += g^2 ;  theta -= lr * g / (sqrt(S) + eps)
// Table rows that are not in the batch are never touched.
//
// Work is cut by POSITION in the sorted key list, not by row id, so a hub entity that occurs a hundred times in a
// batch (degree-skewed graphs) does not serialise one workgroup: k_update_tiles gives every workgroup a tile of 8
// consecutive sorted positions.  Its threads each own one 16-byte column slice; all 8 gradient-row loads and the
// table / state loads of the runs that lie wholly inside the tile are issued together, then the runs are summed in
// sorted order.  A run that lies inside the tile is finished on the spot.  A run that crosses a tile boundary
// leaves a partial sum per tile (the tile's first run in P_first, its last run in P_last), and k_update_fixup, in
// which the workgroup of the tile where such a run starts adds those partial sums in tile order, finishes it.
// No atomics, every sum has a fixed order, so the result is a function of the ids and the gradient rows alone.
// Entity and relation rows go through the same launches; the last workgroup of k_update_tiles adds the
// per-positive loss terms in a fixed order.
#include "kge_common.h"

namespace {

constexpr int TILE_R = 8;
constexpr int UPD_THREADS = 128;

struct UpdateArgs {
    float* T[2];             // tables: entity, relation
    float* St[2];            // Adagrad accumulators
    const float* G[2];       // gradient rows, indexed by key position
    const uint32_t* key[2];  // sorted ids
    const uint32_t* pos[2];  // key position of each sorted entry
    float* Pfirst[2];        // [tiles x D] partial sum of a tile's first run when it began in an earlier tile
    float* Plast[2];         // [tiles x D] partial sum of a tile's last run when it goes on in the next tile
    int n[2];                // key list lengths
    int tiles[2];
    int D[2];
    float lr, eps;
    const float* row_loss;       // [b] per-positive loss terms
    const float* neg_loss_part;  // [n_loss_parts] negative-side loss sums of the backward launch (may be none)
    int n_loss_parts;
    int b;
    float* loss_out;        // direct mode: this step's scalar; replay mode: one float per step
    int64_t* step_ptr;      // replay mode: which step is running; advanced by k_update_fixup
};

__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

// S += g^2 ; x -= lr * g / (sqrt(S) + eps), with the hardware square root and reciprocal (1 ulp each): the update
// is a step of size <= lr, so their 1e-7 relative error is far below the accuracy of g itself.
__device__ __forceinline__ float adagrad1(float g, float& s, float lr, float eps) {
    s = fmaf(g, g, s);
    return lr * g * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(s) + eps);
}
__device__ __forceinline__ void adagrad4(float4 g, float4& x, float4& s, float lr, float eps) {
    x.x -= adagrad1(g.x, s.x, lr, eps);
    x.y -= adagrad1(g.y, s.y, lr, eps);
    x.z -= adagrad1(g.z, s.z, lr, eps);
    x.w -= adagrad1(g.w, s.w, lr, eps);
}

__global__ __launch_bounds__(UPD_THREADS) void k_update_tiles(UpdateArgs a) {
    int tile = blockIdx.x;
    const int tid = threadIdx.x;
    if (tile == a.tiles[0] + a.tiles[1]) {  // ---- loss: fixed-order tree over the b row terms
        __shared__ float part[UPD_THREADS];
        float s = 0.f;
        for (int i = tid; i < a.b; i += UPD_THREADS) s += a.row_loss[i];
        for (int i = tid; i < a.n_loss_parts; i += UPD_THREADS) s += a.neg_loss_part[i];
        part[tid] = s;
        __syncthreads();
        for (int o = UPD_THREADS / 2; o > 0; o >>= 1) {
            if (tid < o) part[tid] += part[tid + o];
            __syncthreads();
        }
        if (tid == 0 && a.loss_out) a.loss_out[a.step_ptr ? *a.step_ptr : 0] = part[0];
        return;
    }
    const int which = tile >= a.tiles[0];
    if (which) tile -= a.tiles[0];
    const int n = a.n[which], D = a.D[which];
    const uint32_t* keys = a.key[which];
    const int p0 = tile * TILE_R, p1 = min(p0 + TILE_R, n), cnt = p1 - p0;

    // keys p0-1 .. p1 and positions p0 .. p1-1 of this tile, read once and shared
    __shared__ uint32_t sk[TILE_R + 2];
    __shared__ uint32_t sp[TILE_R];
    if (tid < TILE_R + 2) {
        const int q = p0 - 1 + tid;
        sk[tid] = (q >= 0 && q <= p1 && q < n) ? keys[q] : 0u;
    } else if (tid >= 64 && tid < 64 + TILE_R) {
        const int q = p0 + tid - 64;
        sp[tid - 64] = q < p1 ? a.pos[which][q] : 0u;
    }
    __syncthreads();
    // everything below is uniform over the workgroup: keep it in scalar registers
    uint32_t key[TILE_R + 2], gpos[TILE_R];
#pragma unroll
    for (int j = 0; j < TILE_R + 2; ++j) key[j] = __builtin_amdgcn_readfirstlane(sk[j]);
#pragma unroll
    for (int j = 0; j < TILE_R; ++j) gpos[j] = __builtin_amdgcn_readfirstlane(sp[j]);
    const bool starts_before = p0 > 0 && key[0] == key[1];
    const bool goes_on = p1 < n && __builtin_amdgcn_readfirstlane(sk[cnt]) == __builtin_amdgcn_readfirstlane(sk[cnt + 1]);

    // per position: does a run end here, and is that run wholly inside the tile
    bool ends[TILE_R], whole[TILE_R];
    {
        bool first_run = true;
#pragma unroll
        for (int j = 0; j < TILE_R; ++j) {
            ends[j] = j < cnt && (j == cnt - 1 || key[j + 2] != key[j + 1]);
            const bool cut_front = first_run && starts_before;
            const bool cut_back = j == cnt - 1 && goes_on;
            whole[j] = ends[j] && !cut_front && !cut_back;
            if (ends[j]) first_run = false;
        }
    }
    const float* G = a.G[which];
    float* Tb = a.T[which];
    float* Sb = a.St[which];

    for (int v = tid; v < D / 4; v += UPD_THREADS) {
        float4 g[TILE_R], x[TILE_R], s[TILE_R];
#pragma unroll
        for (int j = 0; j < TILE_R; ++j) {
            g[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (j < cnt) g[j] = ld4(G + (int64_t)gpos[j] * D + 4 * v);
        }
#pragma unroll
        for (int j = 0; j < TILE_R; ++j) {
            if (whole[j]) {
                x[j] = ld4(Tb + (int64_t)key[j + 1] * D + 4 * v);
                s[j] = ld4(Sb + (int64_t)key[j + 1] * D + 4 * v);
            }
        }
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        bool first_run = true;
#pragma unroll
        for (int j = 0; j < TILE_R; ++j) {
            if (j < cnt) acc = add4(acc, g[j]);
            if (ends[j]) {
                if (whole[j]) {
                    adagrad4(acc, x[j], s[j], a.lr, a.eps);
                    st4(Sb + (int64_t)key[j + 1] * D + 4 * v, s[j]);
                    st4(Tb + (int64_t)key[j + 1] * D + 4 * v, x[j]);
                } else if (first_run && starts_before) {
                    st4(a.Pfirst[which] + (int64_t)tile * D + 4 * v, acc);
                } else {
                    st4(a.Plast[which] + (int64_t)tile * D + 4 * v, acc);
                }
                acc = make_float4(0.f, 0.f, 0.f, 0.f);
                first_run = false;
            }
        }
    }
}

// Finishes the runs that cross tile boundaries.  The workgroup of the tile in which such a run STARTS owns it.
__global__ __launch_bounds__(UPD_THREADS) void k_update_fixup(UpdateArgs a) {
    int tile = blockIdx.x;
    const int tid = threadIdx.x;
    // last kernel of a step and the only one that does not read the step counter: advance it for the next step
    if (a.step_ptr && tile == 0 && tid == 0) *a.step_ptr = *a.step_ptr + 1;
    const int which = tile >= a.tiles[0];
    if (which) tile -= a.tiles[0];
    const int n = a.n[which], D = a.D[which];
    const uint32_t* keys = a.key[which];
    const int p0 = tile * TILE_R, p1 = min(p0 + TILE_R, n);
    if (p1 >= n) return;
    const uint32_t key = keys[p1 - 1];
    if (keys[p1] != key) return;  // the tile's last run ends with the tile
    // does the run begin in this tile?  (at most 8 keys back)
    int s = p1 - 1;
    while (s > p0 && keys[s - 1] == key) --s;
    if (s == p0 && p0 > 0 && keys[p0 - 1] == key) return;  // the run began in an earlier tile
    // tiles tile+1 .. tile+m start with this run.  Thread i looks at tile tile+1+i (and further ones in rounds of
    // 128): the run covers it completely and goes on iff its last key and the key after it are both `key`.
    __shared__ int first_stop;
    if (tid == 0) first_stop = 1 << 30;
    __syncthreads();
    int m = 0;
    for (int base = 0;; base += UPD_THREADS) {
        const int q = p1 + (base + tid) * TILE_R;  // first position of tile tile+1+base+tid
        bool stops = true;                         // does the run end inside (or before) that tile
        if (q < n && keys[q] == key) {
            const int e = min(q + TILE_R, n);
            stops = !(e < n && keys[e - 1] == key && keys[e] == key);
        }
        if (stops) atomicMin(&first_stop, base + tid);
        __syncthreads();
        const int fs = first_stop;
        if (fs < (1 << 30)) {
            // tile+1+fs is the last tile that holds part of the run, unless the run does not reach it at all
            const int q2 = p1 + fs * TILE_R;
            m = fs + ((q2 < n && keys[q2] == key) ? 1 : 0);
            break;
        }
        __syncthreads();
    }
    float* th = a.T[which] + (int64_t)key * D;
    float* st = a.St[which] + (int64_t)key * D;
    const float* Pf = a.Pfirst[which];
    for (int v = tid; v < D / 4; v += UPD_THREADS) {
        float4 x = ld4(th + 4 * v), sv = ld4(st + 4 * v);
        float4 g = ld4(a.Plast[which] + (int64_t)tile * D + 4 * v);
        int i = 1;
        for (; i + 3 <= m; i += 4) {
            const float4 g0 = ld4(Pf + (int64_t)(tile + i) * D + 4 * v);
            const float4 g1 = ld4(Pf + (int64_t)(tile + i + 1) * D + 4 * v);
            const float4 g2 = ld4(Pf + (int64_t)(tile + i + 2) * D + 4 * v);
            const float4 g3 = ld4(Pf + (int64_t)(tile + i + 3) * D + 4 * v);
            g = add4(g, add4(add4(g0, g1), add4(g2, g3)));
        }
        for (; i <= m; ++i) g = add4(g, ld4(Pf + (int64_t)(tile + i) * D + 4 * v));
        adagrad4(g, x, sv, a.lr, a.eps);
        st4(st + 4 * v, sv);
        st4(th + 4 * v, x);
    }
}

}  // namespace

void kge_launch_update(kge_ctx* c, float* E, float* SE, float* R, float* SR, const StepIds& ids, float lr,
                       int n_loss_parts, hipStream_t st) {
    UpdateArgs a;
    const int b = ids.b, n_ent_keys = 2 * ids.b + ids.n_neg, n_rel_keys = ids.b;
    float* loss_out = ids.loss_out;
    a.step_ptr = const_cast<int64_t*>(ids.step_ptr);
    a.T[0] = E; a.T[1] = R; a.St[0] = SE; a.St[1] = SR;
    a.G[0] = c->Gent; a.G[1] = c->Grel;
    a.key[0] = c->ekey[c->ebuf]; a.key[1] = c->rkey[c->rbuf];
    a.pos[0] = c->epos[c->ebuf]; a.pos[1] = c->rpos[c->rbuf];
    a.Pfirst[0] = c->Pfirst_e; a.Pfirst[1] = c->Pfirst_r; a.Plast[0] = c->Plast_e; a.Plast[1] = c->Plast_r;
    a.n[0] = n_ent_keys; a.n[1] = n_rel_keys;
    a.tiles[0] = (n_ent_keys + TILE_R - 1) / TILE_R; a.tiles[1] = (n_rel_keys + TILE_R - 1) / TILE_R;
    a.D[0] = c->cfg.ent_dim; a.D[1] = c->cfg.rel_dim;
    a.lr = lr; a.eps = c->eps; a.row_loss = c->row_loss; a.b = b; a.loss_out = loss_out;
    a.neg_loss_part = c->neg_loss_part; a.n_loss_parts = n_loss_parts;
    const int tiles = a.tiles[0] + a.tiles[1];
    hipLaunchKernelGGL(k_update_tiles, dim3(tiles + 1), dim3(UPD_THREADS), 0, st, a);
    hipLaunchKernelGGL(k_update_fixup, dim3(tiles), dim3(UPD_THREADS), 0, st, a);
}
