// TransR (Table 1 of the paper): f(h, r, t) = gamma - |M_r h + r - M_r t|_2^2.  A relation row holds the translation r
// (D numbers) followed by the D x D projection M_r, row by row.
//
// With a the entity that is kept, x the one that is replaced (the true one for the positive, a corrupting one for a
// negative) and sigma = +1 (tail corrupted) or -1 (head corrupted):
//     o_i = M_i a_i + sigma r_i ,    P(x) = M_i x ,    f = gamma - |o_i - P(x)|^2
// so a positive's negatives need the chunk's corrupting rows projected with the positive's own matrix: batched products
// over the positives (k_gemm.hip).  Here are the steps around them, one workgroup per positive unless said otherwise:
//   k_transr_phi     o_i, p_i = M_i c_i, the positive's score and logistic-loss terms
//   k_transr_score   S_ij = gamma - |o_i - P_ij|^2 from the projections P_i = N_c M_i^T
//   (k_loss)         W = dL/df-
//   k_transr_dp      U_ij = dL/dP_ij = 2 W_ij (o_i - P_ij), in place over P; dL/do_i of the negatives = - sum_j U_ij
//   (product)        gradient rows of the corrupting entities: sum over the chunk's positives of U_i M_i
//   k_transr_chain   go = dL/do, gp = dL/dp -> kept entity M^T go, replaced entity M^T gp, translation sigma go,
//                    matrix += go a^T + gp c^T (on top of the negatives' share U_i^T N_c)
//   k_transr_update  duplicate reduction and Adagrad for the relation rows [r | M] (Sec. 3.1 step 4): the last sorted
//                    position of every run of equal relation ids sums the run's gradient rows, slab by slab
// All sums have a fixed order.
#include "kge_common.h"

namespace {

constexpr int RT = 256;
constexpr int MAX_D = 1024;

struct TransrArgs {
    const float* E;
    const float* R;
    StepIds ids;
    int b, D, k, g, ld_s;
    int64_t n_ent, n_rel, rel_dim;
    float gamma;
    float* O;        // [b x D]      o_i
    float* PP;       // [b x D]      p_i = M_i c_i
    float* P;        // [b x k x D]  projections, then U
    float* S;        // [b x ld_s]   scores, then W
    float* GO;       // [b x D]      dL/do_i from the negatives
    float* fpos;
    float* cpos;
    float* row_loss;
    float* Gent;     // gradient rows in key order: heads | tails | corrupting rows
    float* Gr;       // [b x D]      gradient of the translation
    float* GM;       // [b x D x D]  gradient of the matrix
};

__device__ __forceinline__ int64_t clamp_id(int64_t id, int64_t n) { return id < 0 ? 0 : (id >= n ? n - 1 : id); }

struct Rows {
    const float* a;  // kept entity
    const float* c;  // replaced entity
    const float* r;  // translation
    const float* M;  // projection
    float sigma;
    bool head;
};
__device__ __forceinline__ Rows rows_of(const TransrArgs& a, int i) {
    const StepView sv = step_view(a.ids);
    Rows x;
    x.head = sv.side == KGE_NEG_HEAD;
    const int64_t hid = clamp_id(sv.h[i], a.n_ent), tid = clamp_id(sv.t[i], a.n_ent);
    const int64_t rid = clamp_id(sv.r[i], a.n_rel);
    x.a = a.E + (x.head ? tid : hid) * (int64_t)a.D;
    x.c = a.E + (x.head ? hid : tid) * (int64_t)a.D;
    x.r = a.R + rid * a.rel_dim;
    x.M = x.r + a.D;
    x.sigma = x.head ? -1.f : 1.f;
    return x;
}

// y1 = M v1, y2 = M v2; v1, v2, y1, y2 in LDS.  Row dots: a group of SUB lanes (the power of two that holds the row's
// 16-byte pieces, at most a wave) per matrix row, four rows per round so that four loads are in flight, shuffle
// reductions inside the group.  Rows of more than 256 floats: a wave per row, up to four pieces per lane.
template <int SUB>
__device__ __forceinline__ void row_dots_short(const float* M, int D, const float* v1, const float* v2, float* y1, float* y2) {
    constexpr int GROUPS = RT / SUB;
    const int grp = threadIdx.x / SUB, ln = threadIdx.x % SUB, lanes = D / 4;
    const bool act = ln < lanes;
    const float4 a1 = act ? ld4(v1 + 4 * ln) : f4(0.f), a2 = act ? ld4(v2 + 4 * ln) : f4(0.f);
    const float* Mc = M + (act ? 4 * ln : 0);
    for (int r0 = grp; r0 < D; r0 += 4 * GROUPS) {
        float4 m[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) m[u] = ld4(Mc + (int64_t)(r0 + u * GROUPS < D ? r0 + u * GROUPS : r0) * D);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float s1 = act ? m[u].x * a1.x + m[u].y * a1.y + m[u].z * a1.z + m[u].w * a1.w : 0.f;
            float s2 = act ? m[u].x * a2.x + m[u].y * a2.y + m[u].z * a2.z + m[u].w * a2.w : 0.f;
#pragma unroll
            for (int o = SUB / 2; o > 0; o >>= 1) {
                s1 += __shfl_xor(s1, o, 64);
                s2 += __shfl_xor(s2, o, 64);
            }
            const int r = r0 + u * GROUPS;
            if (ln == 0 && r < D) { y1[r] = s1; y2[r] = s2; }
        }
    }
}

__device__ __forceinline__ void row_dots_long(const float* M, int D, const float* v1, const float* v2, float* y1, float* y2) {
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, lanes = D / 4;
    float4 a1[4], a2[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int q = lane + 64 * it;
        a1[it] = q < lanes ? ld4(v1 + 4 * q) : f4(0.f);
        a2[it] = q < lanes ? ld4(v2 + 4 * q) : f4(0.f);
    }
    for (int r = w; r < D; r += RT / 64) {
        const float* row = M + (int64_t)r * D;
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int q = lane + 64 * it;
            if (q < lanes) {
                const float4 m = ld4(row + 4 * q);
                s1 += m.x * a1[it].x + m.y * a1[it].y + m.z * a1[it].z + m.w * a1[it].w;
                s2 += m.x * a2[it].x + m.y * a2[it].y + m.z * a2[it].z + m.w * a2[it].w;
            }
        }
        s1 = wave_sum(s1);
        s2 = wave_sum(s2);
        if (lane == 0) { y1[r] = s1; y2[r] = s2; }
    }
}

__device__ __forceinline__ void row_dots(const float* M, int D, const float* v1, const float* v2, float* y1, float* y2) {
    const int lanes = D / 4;  // (the same for every thread)
    if (lanes <= 16) row_dots_short<16>(M, D, v1, v2, y1, y2);
    else if (lanes <= 32) row_dots_short<32>(M, D, v1, v2, y1, y2);
    else if (lanes <= 64) row_dots_short<64>(M, D, v1, v2, y1, y2);
    else row_dots_long(M, D, v1, v2, y1, y2);
}

__global__ __launch_bounds__(RT) void k_transr_phi(TransrArgs a, float* pos_out) {
    __shared__ __attribute__((aligned(16))) float va[MAX_D], vc[MAX_D], yo[MAX_D], yp[MAX_D];
    __shared__ float part[RT / 64];
    const int i = blockIdx.x, tid = threadIdx.x, D = a.D;
    const Rows x = rows_of(a, i);
    for (int d = tid; d < D; d += RT) { va[d] = x.a[d]; vc[d] = x.c[d]; }
    __syncthreads();
    row_dots(x.M, D, va, vc, yo, yp);
    __syncthreads();
    float ss = 0.f;
    for (int d = tid; d < D; d += RT) {
        const float o = yo[d] + x.sigma * x.r[d], p = yp[d];
        a.O[(int64_t)i * D + d] = o;
        a.PP[(int64_t)i * D + d] = p;
        ss += (o - p) * (o - p);
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) part[tid >> 6] = ss;
    __syncthreads();
    if (tid == 0) {
        float tot = 0.f;
        for (int w = 0; w < RT / 64; ++w) tot += part[w];
        const float f = a.gamma - tot;
        a.fpos[i] = f;
        if (pos_out) pos_out[i] = f;
        // positive part of the logistic loss (Sec. 2, y = +1) and its derivative
        const float invb = 1.f / (float)a.b;
        const float e = expf(-fabsf(f));
        a.row_loss[i] = (fmaxf(-f, 0.f) + log1pf(e)) * invb;
        a.cpos[i] = -((f >= 0.f ? e : 1.f) / (1.f + e)) * invb;
    }
}

// Workgroup per positive: S_ij = gamma - |o_i - P_ij|^2.  A row of D floats is D / 4 16-byte pieces; a group of SUB
// lanes (the power of two that holds them, at most a wave) takes one j at a time, so that short rows do not leave most
// of a wave idle, and works on four of its j in one round (four loads in flight, then four shuffle reductions).
template <int SUB>
__device__ __forceinline__ void transr_score_rows(const TransrArgs& a, float* out, int ld_out) {
    constexpr int GROUPS = RT / SUB;
    const int i = blockIdx.x, grp = threadIdx.x / SUB, ln = threadIdx.x % SUB, D = a.D, lanes = D / 4;
    const bool act = ln < lanes;
    const float4 ov = act ? ld4(a.O + (int64_t)i * D + 4 * ln) : f4(0.f);
    const float* P = a.P + (int64_t)i * a.k * D + (act ? 4 * ln : 0);
    for (int j0 = grp; j0 < a.k; j0 += 4 * GROUPS) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = j0 + u * GROUPS;
            v[u] = ld4(P + (int64_t)(j < a.k ? j : j0) * D);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float d0 = ov.x - v[u].x, d1 = ov.y - v[u].y, d2 = ov.z - v[u].z, d3 = ov.w - v[u].w;
            float ss = act ? d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3 : 0.f;
#pragma unroll
            for (int o = SUB / 2; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
            const int j = j0 + u * GROUPS;
            if (ln == 0 && j < a.k) out[(int64_t)i * ld_out + j] = a.gamma - ss;
        }
    }
}

// rows of more than 256 floats: a wave per j, up to four pieces per lane
__device__ __forceinline__ void transr_score_long_rows(const TransrArgs& a, float* out, int ld_out) {
    const int i = blockIdx.x, w = threadIdx.x >> 6, lane = threadIdx.x & 63, D = a.D, lanes = D / 4;
    const float* o = a.O + (int64_t)i * D;
    float4 ov[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) ov[it] = lane + 64 * it < lanes ? ld4(o + 4 * (lane + 64 * it)) : f4(0.f);
    for (int j = w; j < a.k; j += RT / 64) {
        const float* p = a.P + ((int64_t)i * a.k + j) * D;
        float ss = 0.f;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int q = lane + 64 * it;
            if (q < lanes) {
                const float4 v = ld4(p + 4 * q);
                const float d0 = ov[it].x - v.x, d1 = ov[it].y - v.y, d2 = ov[it].z - v.z, d3 = ov[it].w - v.w;
                ss += d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3;
            }
        }
        ss = wave_sum(ss);
        if (lane == 0) out[(int64_t)i * ld_out + j] = a.gamma - ss;
    }
}

__global__ __launch_bounds__(RT) void k_transr_score(TransrArgs a, float* out, int ld_out) {
    const int lanes = a.D / 4;  // (the same for every thread)
    if (lanes <= 16) transr_score_rows<16>(a, out, ld_out);
    else if (lanes <= 32) transr_score_rows<32>(a, out, ld_out);
    else if (lanes <= 64) transr_score_rows<64>(a, out, ld_out);
    else transr_score_long_rows(a, out, ld_out);
}

// Threads (group, 16 bytes of the row); the groups share out the rows they walk, four loads in flight each, and their
// sums meet in LDS in group order.
// U_ij = 2 W_ij (o_i - P_ij) over P_ij; GO_i = - sum_j U_ij
__global__ __launch_bounds__(RT) void k_transr_dp(TransrArgs a) {
    __shared__ __attribute__((aligned(16))) float4 part[RT];
    const int i = blockIdx.x, D = a.D, lanes = D / 4, groups = RT / lanes;
    const int grp = threadIdx.x / lanes, v = threadIdx.x % lanes;
    const float* W = a.S + (int64_t)i * a.ld_s;
    float4 go = f4(0.f);
    if (grp < groups) {
        const float4 o = ld4(a.O + (int64_t)i * D + 4 * v);
        float* P = a.P + (int64_t)i * a.k * D + 4 * v;
        for (int j0 = grp; j0 < a.k; j0 += 4 * groups) {
            float4 pv[4];
            float w2[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + u * groups < a.k ? j0 + u * groups : j0;
                pv[u] = ld4(P + (int64_t)j * D);
                w2[u] = 2.f * W[j];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + u * groups;
                if (j < a.k) {
                    const float4 q = make_float4(w2[u] * (o.x - pv[u].x), w2[u] * (o.y - pv[u].y), w2[u] * (o.z - pv[u].z),
                                                 w2[u] * (o.w - pv[u].w));
                    st4(P + (int64_t)j * D, q);
                    go.x -= q.x; go.y -= q.y; go.z -= q.z; go.w -= q.w;
                }
            }
        }
    }
    part[threadIdx.x] = go;
    __syncthreads();
    if (grp == 0) {
        float4 t = part[v];
        for (int g2 = 1; g2 < groups; ++g2) {
            const float4 q = part[g2 * lanes + v];
            t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w;
        }
        st4(a.GO + (int64_t)i * D + 4 * v, t);
    }
}

__global__ __launch_bounds__(RT) void k_transr_chain(TransrArgs a) {
    __shared__ __attribute__((aligned(16))) float go[MAX_D], gp[MAX_D];
    __shared__ __attribute__((aligned(16))) float4 part1[RT], part2[RT];
    const int i = blockIdx.x, tid = threadIdx.x, D = a.D, lanes = D / 4;
    const Rows x = rows_of(a, i);
    const float cp = a.cpos[i];
    for (int d = tid; d < D; d += RT) {
        const float q = a.O[(int64_t)i * D + d] - a.PP[(int64_t)i * D + d];
        const float g1 = a.GO[(int64_t)i * D + d] - 2.f * cp * q;  // df+/do = -2 (o - p)
        go[d] = g1;
        gp[d] = 2.f * cp * q;
        a.Gr[(int64_t)i * D + d] = x.sigma * g1;
    }
    __syncthreads();
    // M^T go and M^T gp (column sums: a thread per 16-byte column slice, rows dealt round-robin to thread groups),
    // and on the way, row by row, the outer products into the matrix gradient
    const int groups = RT / lanes, grp = tid / lanes, v = tid % lanes;
    float4 y1 = f4(0.f), y2 = f4(0.f);
    if (grp < groups) {
        const float4 av = ld4(x.a + 4 * v), cv = ld4(x.c + 4 * v);
        float* gm = a.GM + (int64_t)i * D * D;
        for (int r = grp; r < D; r += groups) {
            const float4 m = ld4(x.M + (int64_t)r * D + 4 * v);
            const float s1 = go[r], s2 = gp[r];
            y1.x += s1 * m.x; y1.y += s1 * m.y; y1.z += s1 * m.z; y1.w += s1 * m.w;
            y2.x += s2 * m.x; y2.y += s2 * m.y; y2.z += s2 * m.z; y2.w += s2 * m.w;
            float4 gv = ld4(gm + (int64_t)r * D + 4 * v);
            gv.x += s1 * av.x + s2 * cv.x; gv.y += s1 * av.y + s2 * cv.y;
            gv.z += s1 * av.z + s2 * cv.z; gv.w += s1 * av.w + s2 * cv.w;
            st4(gm + (int64_t)r * D + 4 * v, gv);
        }
    }
    part1[tid] = y1;
    part2[tid] = y2;
    __syncthreads();
    if (tid < lanes) {
        float4 t1 = part1[tid], t2 = part2[tid];
        for (int g = 1; g < groups; ++g) {
            const float4 u1 = part1[g * lanes + tid], u2 = part2[g * lanes + tid];
            t1.x += u1.x; t1.y += u1.y; t1.z += u1.z; t1.w += u1.w;
            t2.x += u2.x; t2.y += u2.y; t2.z += u2.z; t2.w += u2.w;
        }
        // key positions: heads 0 .. b-1, tails b .. 2b-1
        st4(a.Gent + (int64_t)(x.head ? a.b + i : i) * D + 4 * tid, t1);
        st4(a.Gent + (int64_t)(x.head ? i : a.b + i) * D + 4 * tid, t2);
    }
}

struct TransrUpdArgs {
    float* T;             // relation table [n_rel x (D + D*D)]
    float* St;            // its Adagrad accumulator
    const uint32_t* key;  // sorted relation ids of the step
    const uint32_t* pos;  // position in the mini-batch of each sorted entry
    int n, D, rows_per_slab;
    int64_t rel_dim;
    const float* Gr;
    const float* GM;
    float lr, eps;
};

// Workgroup (p, slab): slab 0 is the translation, slab s > 0 rows (s - 1) * rows_per_slab .. of the matrix.  If sorted
// position p is the last of its run of equal relation ids, the workgroup sums the run's gradient rows for its slab in
// sorted order and applies Adagrad.
__global__ __launch_bounds__(RT) void k_transr_update(TransrUpdArgs a) {
    const int p = blockIdx.x, slab = blockIdx.y, tid = threadIdx.x;
    const uint32_t key = a.key[p];
    if (p + 1 < a.n && a.key[p + 1] == key) return;  // the run goes on (same decision in every thread)
    __shared__ int first_other;
    __shared__ uint32_t lpos[RT];
    const int D = a.D;
    const int width = slab == 0 ? D : a.rows_per_slab * D, lanes = width / 4;
    const bool act = tid < lanes;
    const int e = act ? 4 * tid : 0;
    const int64_t in_row = slab == 0 ? e : (int64_t)D + (int64_t)(slab - 1) * a.rows_per_slab * D + e;
    const int64_t off = (int64_t)key * a.rel_dim + in_row;
    const float* G = slab == 0 ? a.Gr + e : a.GM + (int64_t)(slab - 1) * a.rows_per_slab * D + e;
    const int64_t g_stride = slab == 0 ? D : (int64_t)D * D;
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
        __syncthreads();
        if (found) break;
    }
    const int start = p - first_other + 1;
    float4 g = f4(0.f);
    for (int c0 = start; c0 <= p; c0 += RT) {
        __syncthreads();
        lpos[tid] = a.pos[c0 + tid <= p ? c0 + tid : p];
        __syncthreads();
        const int m = p - c0 + 1 < RT ? p - c0 + 1 : RT;
        if (act) {
#pragma unroll 4
            for (int j = 0; j < m; ++j) {
                const float4 t = ld4(G + (int64_t)lpos[j] * g_stride);
                g.x += t.x; g.y += t.y; g.z += t.z; g.w += t.w;
            }
        }
    }
    if (act) {
        adagrad4(g, x, s, a.lr, a.eps);
        st4(a.St + off, s);
        st4(a.T + off, x);
    }
}

TransrArgs make_args(kge_ctx* c, const float* E, const float* R, const StepIds& ids, int k, int gsz, float gamma) {
    TransrArgs a;
    const int D = c->cfg.ent_dim;
    a.E = E; a.R = R; a.ids = ids; a.b = ids.b; a.D = D; a.k = k; a.g = gsz; a.ld_s = c->ld_s;
    a.n_ent = c->cfg.num_entities; a.n_rel = c->cfg.num_relations; a.rel_dim = c->cfg.rel_dim;
    a.gamma = gamma;
    a.O = c->O; a.PP = c->PP; a.P = c->P3; a.S = c->S; a.GO = c->GO;
    a.fpos = c->fpos; a.cpos = c->cpos; a.row_loss = c->row_loss;
    a.Gent = c->Gent; a.Gr = c->Grel; a.GM = c->Grel + (int64_t)c->cfg.max_batch * D;
    return a;
}

}  // namespace

void kge_transr_phi(kge_ctx* c, const float* E, const float* R, const StepIds& ids, float gamma, float* pos_out,
                    hipStream_t st) {
    const TransrArgs a = make_args(c, E, R, ids, 0, 1, gamma);
    KGE_LAUNCH(c, k_transr_phi, dim3(ids.b), dim3(RT), 0, st, a, pos_out);
}

// negative scores from the projections (kge_gemm_transr_project has filled c->P3)
void kge_transr_score(kge_ctx* c, const StepIds& ids, int k, float gamma, float* out, int ld_out, hipStream_t st) {
    const TransrArgs a = make_args(c, nullptr, nullptr, ids, k, 1, gamma);
    KGE_LAUNCH(c, k_transr_score, dim3(ids.b), dim3(RT), 0, st, a, out, ld_out);
}

float* kge_transr_projections(kge_ctx* c) { return c->P3; }
float* kge_transr_matrix_grads(kge_ctx* c) { return c->Grel + (int64_t)c->cfg.max_batch * c->cfg.ent_dim; }

void kge_transr_dp(kge_ctx* c, const StepIds& ids, int k, hipStream_t st) {
    const TransrArgs a = make_args(c, nullptr, nullptr, ids, k, 1, 0.f);
    KGE_LAUNCH(c, k_transr_dp, dim3(ids.b), dim3(RT), 0, st, a);
}

void kge_transr_chain(kge_ctx* c, const float* E, const float* R, const StepIds& ids, hipStream_t st) {
    const TransrArgs a = make_args(c, E, R, ids, 0, 1, 0.f);
    KGE_LAUNCH(c, k_transr_chain, dim3(ids.b), dim3(RT), 0, st, a);
}

void kge_transr_update(kge_ctx* c, float* R, float* SR, const StepIds& ids, float lr, hipStream_t st) {
    TransrUpdArgs a;
    const int D = c->cfg.ent_dim;
    int rows = 1024 / D;  // matrix rows per workgroup: the largest divisor of D that keeps a slab within 1024 floats
    while (D % rows != 0) --rows;
    a.T = R; a.St = SR; a.key = c->rkey[c->rbuf]; a.pos = c->rpos[c->rbuf];
    a.n = ids.b; a.D = D; a.rows_per_slab = rows; a.rel_dim = c->cfg.rel_dim;
    a.Gr = c->Grel; a.GM = c->Grel + (int64_t)c->cfg.max_batch * D;
    a.lr = lr; a.eps = c->eps;
    KGE_LAUNCH(c, k_transr_update, dim3(ids.b, D / rows + 1), dim3(RT), 0, st, a);
}
