// RESCAL (Table 1 of the paper): f(h, r, t) = h^T M_r t, with M_r a D x D matrix kept as one relation row of D * D
// floats (row by row).  The split of Sec. 3.3 carries over: with the tail corrupted h^T M n = (M^T h) . n, with the
// head corrupted n^T M t = n . (M t), so with
//     o = M_r^T h   (tail corrupted)        o = M_r t   (head corrupted)
// every score of a positive against a replacement x is o . x, and negative scoring and its backward are the matrix
// products of DistMult.  What is particular to RESCAL is the matrix-vector product on either side of them:
//   k_rescal<false>  o_i from the kept entity and M_r                       (before the gather launch, which then
//                                                                            scores the positive from o_i)
//   k_rescal<true>   the chain rule: with go = dL/do_i (negatives' part from the backward product, plus the
//                    positive pair's dL/df+ * c), the kept entity gets M go (tail corrupted) or M^T go (head), the
//                    replaced entity dL/df+ * o, and the relation the outer product u w^T with (u, w) = (h, go)
//                    (tail) or (go, t) (head).  That would be a gradient row of D * D floats per positive; only its
//                    two factors are stored.
//   k_rescal_update  duplicate reduction and Adagrad for the relation matrices (Sec. 3.1 step 4): for every distinct
//                    relation of the step, dL/dM = sum over its positives of u w^T, formed straight from the factor
//                    rows (2 D floats per positive instead of D * D) and applied to the matrix in place.
// One workgroup per positive.  M is read once, row by row, every row as whole 16-byte loads; the two kinds of
// product are "row dots" (y_r = M[r, :] . v: a wave per row, shuffle reduction) and "column sums"
// (y = sum_r v_r M[r, :]: a thread per 16-byte column slice, rows dealt round-robin to thread groups whose partial
// sums are added in group order).  All sums have a fixed order.
#include "kge_common.h"

namespace {

constexpr int RT = 256;       // threads per workgroup
constexpr int MAX_D = 1024;   // entity rows are at most this long

struct RescalArgs {
    const float* E;
    const float* R;
    StepIds ids;
    int b, D;
    int64_t n_ent, n_rel;
    float* O;           // [b x D]  phi: written; chain: read
    const float* GO;    // [b x D]  chain: sum_j W_ij n_j
    const float* cpos;  // [b]      chain: dL/df+_i
    float* Gent;        // gradient rows in key order: heads | tails | corrupting rows
    float* GU;          // [b x D]  chain: left factor of the positive's matrix gradient
    float* GW;          // [b x D]  chain: right factor
};

__device__ __forceinline__ int64_t clamp_id(int64_t id, int64_t n) { return id < 0 ? 0 : (id >= n ? n - 1 : id); }

template <bool CHAIN>
__global__ __launch_bounds__(RT) void k_rescal(RescalArgs a) {
    __shared__ __attribute__((aligned(16))) float vec[MAX_D];  // the vector that multiplies M
    __shared__ __attribute__((aligned(16))) float res[MAX_D];  // the product
    __shared__ __attribute__((aligned(16))) float4 part[RT];   // column sums of the thread groups
    const int i = blockIdx.x, tid = threadIdx.x, D = a.D, lanes = D / 4;
    const StepView sv = step_view(a.ids);
    const bool head = sv.side == KGE_NEG_HEAD;
    const int64_t hid = clamp_id(sv.h[i], a.n_ent), tl = clamp_id(sv.t[i], a.n_ent);
    const int64_t rid = clamp_id(sv.r[i], a.n_rel);
    const float* pa = a.E + (head ? tl : hid) * (int64_t)D;  // the kept entity
    const float* pc = a.E + (head ? hid : tl) * (int64_t)D;  // the entity that the negatives replace
    const float* M = a.R + rid * (int64_t)D * D;
    const float cp = CHAIN ? a.cpos[i] : 0.f;

    for (int d = tid; d < D; d += RT) vec[d] = CHAIN ? a.GO[(int64_t)i * D + d] + cp * pc[d] : pa[d];
    __syncthreads();

    // phi: o = M^T a (tail corrupted: column sums) or M a (head: row dots); the chain rule needs the transposed one
    const bool rowdot = CHAIN ? !head : head;
    const int groups = RT / lanes, grp = tid / lanes, v = tid % lanes;  // column-slice ownership (lanes <= 256)
    if (rowdot) {
        const int w = tid >> 6, lane = tid & 63;
        float4 vv[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int q = lane + 64 * it;
            vv[it] = q < lanes ? ld4(vec + 4 * q) : f4(0.f);
        }
        if (lanes <= 64) {
            // one piece per lane: four rows per round, so that four loads are in flight (lanes past the row's end
            // read its first piece and add nothing)
            const float* Mc = M + (lane < lanes ? 4 * lane : 0);
            for (int r0 = w; r0 < D; r0 += 4 * (RT / 64)) {
                float4 m[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) m[u] = ld4(Mc + (int64_t)(r0 + u * (RT / 64) < D ? r0 + u * (RT / 64) : r0) * D);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    float s = lane < lanes ? m[u].x * vv[0].x + m[u].y * vv[0].y + m[u].z * vv[0].z + m[u].w * vv[0].w : 0.f;
                    s = wave_sum(s);
                    const int r = r0 + u * (RT / 64);
                    if (lane == 0 && r < D) res[r] = s;
                }
            }
        } else {
            for (int r = w; r < D; r += RT / 64) {
                const float* row = M + (int64_t)r * D;
                float s = 0.f;
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int q = lane + 64 * it;
                    if (q < lanes) {
                        const float4 m = ld4(row + 4 * q);
                        s += m.x * vv[it].x + m.y * vv[it].y + m.z * vv[it].z + m.w * vv[it].w;
                    }
                }
                s = wave_sum(s);
                if (lane == 0) res[r] = s;
            }
        }
    } else {
        float4 y = f4(0.f);
        if (grp < groups) {
            for (int r0 = grp; r0 < D; r0 += 4 * groups) {  // four rows per round, their loads in flight together
                float4 m[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) m[u] = ld4(M + (int64_t)(r0 + u * groups < D ? r0 + u * groups : r0) * D + 4 * v);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int r = r0 + u * groups;
                    const float s = r < D ? vec[r] : 0.f;
                    y.x += s * m[u].x; y.y += s * m[u].y; y.z += s * m[u].z; y.w += s * m[u].w;
                }
            }
        }
        part[tid] = y;
        __syncthreads();
        if (tid < lanes) {
            float4 t = part[tid];
            for (int g = 1; g < groups; ++g) {
                const float4 u = part[g * lanes + tid];
                t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
            }
            st4(res + 4 * tid, t);
        }
    }
    __syncthreads();

    if (!CHAIN) {
        for (int d = tid; d < D; d += RT) a.O[(int64_t)i * D + d] = res[d];
        return;
    }
    // key positions: heads 0 .. b-1, tails b .. 2b-1
    float* ga = a.Gent + (int64_t)(head ? a.b + i : i) * D;
    float* gc = a.Gent + (int64_t)(head ? i : a.b + i) * D;
    for (int d = tid; d < D; d += RT) {
        ga[d] = res[d];
        gc[d] = cp * a.O[(int64_t)i * D + d];
    }
    // dL/dM[r][c] = a_r go_c (tail corrupted, o = M^T a)  or  go_r a_c (head corrupted, o = M a): the factors
    for (int d = tid; d < D; d += RT) {
        a.GU[(int64_t)i * D + d] = head ? vec[d] : pa[d];
        a.GW[(int64_t)i * D + d] = head ? pa[d] : vec[d];
    }
}

struct RescalUpdArgs {
    float* T;             // relation table [n_rel x D*D]
    float* St;            // its Adagrad accumulator
    const uint32_t* key;  // sorted relation ids of the step
    const uint32_t* pos;  // position in the mini-batch of each sorted entry
    int n, D, rows_per_slab;
    const float* GU;
    const float* GW;
    float lr, eps;
};

// Workgroup (p, slab): if sorted position p is the last of its run of equal relation ids, it owns that relation in
// this step and updates `rows_per_slab` consecutive rows of its matrix (at most 1024 floats, a thread per 16 bytes):
// the matrix and state slices are asked for first; the run's start is found by a parallel look-back over the keys;
// then the outer products of the run's positives are summed in sorted order and Adagrad is applied.
__global__ __launch_bounds__(RT) void k_rescal_update(RescalUpdArgs a) {
    const int p = blockIdx.x, slab = blockIdx.y, tid = threadIdx.x;
    const uint32_t key = a.key[p];
    if (p + 1 < a.n && a.key[p + 1] == key) return;  // the run goes on (same decision in every thread)
    __shared__ int first_other;  // distance from p back to the nearest entry with another key
    __shared__ uint32_t lpos[RT];
    const int D = a.D, width = a.rows_per_slab * D, lanes = width / 4;
    const bool act = tid < lanes;
    const int e = act ? 4 * tid : 0, lrow = e / D, col = e - lrow * D;
    const int mrow = slab * a.rows_per_slab + lrow;
    const int64_t off = (int64_t)key * D * D + (int64_t)slab * width + e;
    float4 x = f4(0.f), s = f4(0.f);
    if (act) { x = ld4(a.T + off); s = ld4(a.St + off); }
    if (tid == 0) first_other = 1 << 30;
    __syncthreads();
    for (int base = 1;; base += RT) {
        const int q = p - (base + tid);
        const bool differs = q < 0 || a.key[q < 0 ? 0 : q] != key;
        const unsigned long long bal = __ballot(differs);
        if ((tid & 63) == 0 && bal) atomicMin(&first_other, base + tid + __builtin_ctzll(bal));
        __syncthreads();
        const bool found = first_other < (1 << 30);
        __syncthreads();  // everyone has read it before the next round may lower it
        if (found) break;
    }
    const int start = p - first_other + 1;
    float4 g = f4(0.f);
    for (int c0 = start; c0 <= p; c0 += RT) {
        __syncthreads();  // lpos is free again
        lpos[tid] = a.pos[c0 + tid <= p ? c0 + tid : p];
        __syncthreads();
        const int m = p - c0 + 1 < RT ? p - c0 + 1 : RT;
        if (act) {
            // (16 positives in flight per thread instead of 4 was measured slower: the registers cost more in
            // resident workgroups than the deeper queue gains on the few long runs)
#pragma unroll 4
            for (int j = 0; j < m; ++j) {
                const int64_t row = (int64_t)lpos[j] * D;
                const float u = a.GU[row + mrow];
                const float4 w = ld4(a.GW + row + col);
                g.x += u * w.x; g.y += u * w.y; g.z += u * w.z; g.w += u * w.w;
            }
        }
    }
    if (act) {
        adagrad4(g, x, s, a.lr, a.eps);
        st4(a.St + off, s);
        st4(a.T + off, x);
    }
}

RescalArgs make_args(kge_ctx* c, const float* E, const float* R, const StepIds& ids) {
    RescalArgs a;
    a.E = E; a.R = R; a.ids = ids; a.b = ids.b; a.D = c->cfg.ent_dim;
    a.n_ent = c->cfg.num_entities; a.n_rel = c->cfg.num_relations;
    a.O = c->O; a.GO = c->GO; a.cpos = c->cpos; a.Gent = c->Gent;
    a.GU = c->Grel; a.GW = c->Grel + (int64_t)ids.b * c->cfg.ent_dim;  // the relation-gradient area holds the factors
    return a;
}

}  // namespace

void kge_launch_rescal_phi(kge_ctx* c, const float* E, const float* R, const StepIds& ids, hipStream_t st) {
    const RescalArgs a = make_args(c, E, R, ids);
    KGE_LAUNCH(c, k_rescal<false>, dim3(ids.b), dim3(RT), 0, st, a);
}

void kge_launch_rescal_chain(kge_ctx* c, const float* E, const float* R, const StepIds& ids, hipStream_t st) {
    const RescalArgs a = make_args(c, E, R, ids);
    KGE_LAUNCH(c, k_rescal<true>, dim3(ids.b), dim3(RT), 0, st, a);
}

void kge_launch_rescal_update(kge_ctx* c, float* R, float* SR, const StepIds& ids, float lr, hipStream_t st) {
    RescalUpdArgs a;
    const int D = c->cfg.ent_dim;
    int rows = 1024 / D;  // matrix rows per workgroup: the largest divisor of D that keeps a slab within 1024 floats
    while (D % rows != 0) --rows;
    a.T = R; a.St = SR; a.key = c->rkey[c->rbuf]; a.pos = c->rpos[c->rbuf];
    a.n = ids.b; a.D = D; a.rows_per_slab = rows;
    a.GU = c->Grel; a.GW = c->Grel + (int64_t)ids.b * D;
    a.lr = lr; a.eps = c->eps;
    KGE_LAUNCH(c, k_rescal_update, dim3(ids.b, D / rows), dim3(RT), 0, st, a);
}
