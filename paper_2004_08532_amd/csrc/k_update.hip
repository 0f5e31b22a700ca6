// Duplicate reduction, part 2, fused with the optimizer (paper Sec. 3.1 step 4): for every distinct row that the
// mini-batch touched, add up its gradient rows and apply Adagrad to that row of the global table, in place.
//
// One workgroup per position of the sorted key list; the workgroup whose position starts a run of equal ids
// owns that row, the others leave at once (no compaction pass, no atomics).  The owner's threads each take one
// 16-byte slice of the row, add the slice of every gradient row of the run in sorted order (four loads in
// flight), then read-modify-write the table and the state:  S += g^2 ; theta -= lr * g / (sqrt(S) + eps).
// Table rows that are not in the batch are never touched.  Entity and relation rows go through the same
// launch; its last workgroup adds the per-positive loss terms in a fixed order.
#include "kge_common.h"

namespace {

struct UpdateArgs {
    float* T[2];            // tables: entity, relation
    float* St[2];           // Adagrad accumulators
    const float* G[2];      // gradient rows, indexed by key position
    const uint32_t* key[2]; // sorted ids
    const uint32_t* pos[2]; // key position of each sorted entry
    int n[2];               // key list lengths
    int D[2];
    float lr, eps;
    const float* row_loss;
    int b;
    float* loss_out;
};

constexpr int UPD_THREADS = 128;

__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

__global__ __launch_bounds__(UPD_THREADS) void k_update(UpdateArgs a) {
    int p = blockIdx.x;
    const int tid = threadIdx.x;
    if (p == a.n[0] + a.n[1]) {  // ---- loss: fixed-order tree over the b row terms
        __shared__ float part[UPD_THREADS];
        float s = 0.f;
        for (int i = tid; i < a.b; i += UPD_THREADS) s += a.row_loss[i];
        part[tid] = s;
        __syncthreads();
        for (int o = UPD_THREADS / 2; o > 0; o >>= 1) {
            if (tid < o) part[tid] += part[tid + o];
            __syncthreads();
        }
        if (tid == 0 && a.loss_out) *a.loss_out = part[0];
        return;
    }
    const int which = p >= a.n[0];
    if (which) p -= a.n[0];
    const uint32_t* keys = a.key[which];
    const uint32_t key = keys[p];
    if (p > 0 && keys[p - 1] == key) return;  // not the first entry of its run
    const int n = a.n[which], D = a.D[which];
    int end = p + 1;
    while (end < n && keys[end] == key) ++end;
    const uint32_t* pos = a.pos[which];
    const float* G = a.G[which];
    float* th = a.T[which] + (int64_t)key * D;
    float* st = a.St[which] + (int64_t)key * D;

    for (int v = tid; v < D / 4; v += UPD_THREADS) {
        float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
        int q = p;
        for (; q + 4 <= end; q += 4) {
            const float4 g0 = ld4(G + (int64_t)pos[q] * D + 4 * v);
            const float4 g1 = ld4(G + (int64_t)pos[q + 1] * D + 4 * v);
            const float4 g2 = ld4(G + (int64_t)pos[q + 2] * D + 4 * v);
            const float4 g3 = ld4(G + (int64_t)pos[q + 3] * D + 4 * v);
            g = add4(g, add4(add4(g0, g1), add4(g2, g3)));
        }
        for (; q < end; ++q) g = add4(g, ld4(G + (int64_t)pos[q] * D + 4 * v));
        float4 x = ld4(th + 4 * v), s = ld4(st + 4 * v);
        s.x += g.x * g.x; s.y += g.y * g.y; s.z += g.z * g.z; s.w += g.w * g.w;
        x.x -= a.lr * g.x / (sqrtf(s.x) + a.eps);
        x.y -= a.lr * g.y / (sqrtf(s.y) + a.eps);
        x.z -= a.lr * g.z / (sqrtf(s.z) + a.eps);
        x.w -= a.lr * g.w / (sqrtf(s.w) + a.eps);
        st4(st + 4 * v, s);
        st4(th + 4 * v, x);
    }
}

}  // namespace

void kge_launch_update(kge_ctx* c, float* E, float* SE, float* R, float* SR, int n_ent_keys, int n_rel_keys,
                       float lr, int b, float* loss_out, hipStream_t st) {
    UpdateArgs a;
    a.T[0] = E; a.T[1] = R; a.St[0] = SE; a.St[1] = SR;
    a.G[0] = c->Gent; a.G[1] = c->Grel;
    a.key[0] = c->ekey[c->ebuf]; a.key[1] = c->rkey[c->rbuf];
    a.pos[0] = c->epos[c->ebuf]; a.pos[1] = c->rpos[c->rbuf];
    a.n[0] = n_ent_keys; a.n[1] = n_rel_keys;
    a.D[0] = c->cfg.ent_dim; a.D[1] = c->cfg.rel_dim;
    a.lr = lr; a.eps = c->eps; a.row_loss = c->row_loss; a.b = b; a.loss_out = loss_out;
    hipLaunchKernelGGL(k_update, dim3(n_ent_keys + n_rel_keys + 1), dim3(UPD_THREADS), 0, st, a);
}
