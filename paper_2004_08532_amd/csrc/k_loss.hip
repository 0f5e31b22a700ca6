// Logistic or pairwise ranking loss (paper Sec. 2) on the positive and negative scores, its derivatives, and the chain rule from
// dL/do back to the head / tail / relation rows (the back-propagation half of Sec. 3.1 step 3).
//
// k_loss: one wavefront per positive.  The k negative scores of the row are read by the 64 lanes, the optional
// softmax weights use shuffle reductions for the maximum and the sum, and the row leaves behind the
// coefficient matrix W that the backward products consume:
//     W_ij = w_ij * sigmoid(f-_ij) / b               (DistMult, ComplEx, RotatE, TransE-L1)
//     W_ij = w_ij * sigmoid(f-_ij) / (b * dist_ij)    (TransE-L2, so that dO = W N - rowsum(W) o)
// Ranking loss max(0, gamma - f+_i + f-_ij): sigmoid(f-_ij) is replaced by the indicator of a positive margin term,
// and dL/df+_i = -sum_j w_ij [term > 0] / b comes out of the same pass over the row.
// k_chain: one wavefront per positive.  Adds the positive pair's own term to dL/do, pushes it through
// o = phi(a, r) and writes the three gradient rows of the positive (kept entity, replaced entity, relation).
#include "kge_common.h"

namespace {

__device__ __forceinline__ float sigmoidf_(float x) {
    if (x >= 0.f) return 1.f / (1.f + expf(-x));
    const float e = expf(x);
    return e / (1.f + e);
}
__device__ __forceinline__ float softplusf_(float x) { return fmaxf(x, 0.f) + log1pf(expf(-fabsf(x))); }
// Both at once for a negative score, from one exponential, with the hardware exp2 / log2 / reciprocal (1 ulp each,
// about 1e-6 relative: the size of the rounding of the fp32 products that the results go into)
__device__ __forceinline__ void softplus_sigmoid(float f, float& sp, float& sg) {
    const float e = __builtin_amdgcn_exp2f(-fabsf(f) * 1.4426950408889634f);  // exp(-|f|) in (0, 1]
    sp = fmaxf(f, 0.f) + __builtin_amdgcn_logf(1.f + e) * 0.6931471805599453f;
    sg = (f >= 0.f ? 1.f : e) * __builtin_amdgcn_rcpf(1.f + e);
}

struct LossArgs {
    float* S;  // in: negative scores (distances when is_dist); out: W
    int ld_s, b, k;
    const float* fpos;
    float gamma, alpha;
    int is_dist;  // TransE-L2 training path: S holds distances, score = gamma - S
    int ranking;  // pairwise ranking loss instead of the logistic loss
    int bf16;
    float* cpos;
    float* row_loss;
};

// VPL: values per lane (the row's k scores live in registers: one pass over memory in, one out; all loads of a row
// are in flight together and every exponential is taken once).
template <int VPL>
__global__ __launch_bounds__(256) void k_loss(LossArgs a) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= a.b) return;
    float* s = a.S + (int64_t)i * a.ld_s;
    const float invb = 1.f / (float)a.b;
    const float fp = a.fpos[i];
    const int k = a.k;

    float raw[VPL], f[VPL], e[VPL];
#pragma unroll
    for (int u = 0; u < VPL; ++u) {
        const int j = lane + 64 * u;
        raw[u] = s[j < k ? j : 0];
    }
    float mx = -INFINITY, z = 1.f;
#pragma unroll
    for (int u = 0; u < VPL; ++u) {
        f[u] = a.is_dist ? a.gamma - raw[u] : raw[u];
        if (lane + 64 * u < k) mx = fmaxf(mx, a.alpha * f[u]);
    }
    if (a.alpha > 0.f) {
        mx = wave_max(mx);
        float zz = 0.f;
#pragma unroll
        for (int u = 0; u < VPL; ++u) {
            e[u] = a.bf16 ? expf(a.alpha * f[u] - mx) : __builtin_amdgcn_exp2f((a.alpha * f[u] - mx) * 1.4426950408889634f);
            if (lane + 64 * u < k) zz += e[u];
        }
        z = wave_sum(zz);
    }
    float li = 0.f, active = 0.f;
#pragma unroll
    for (int u = 0; u < VPL; ++u) {
        const int j = lane + 64 * u;
        if (j >= k) continue;
        const float w = a.alpha > 0.f ? e[u] / z : 1.f / (float)k;
        float coef;
        if (a.ranking) {
            const float m = a.gamma - fp + f[u];
            li += w * fmaxf(m, 0.f);
            coef = m > 0.f ? w * invb : 0.f;
            active += m > 0.f ? w : 0.f;
        } else if (a.bf16) {  // (W is rounded to bf16 afterwards: the library functions, so that no value sits on the fence)
            li += w * softplusf_(f[u]);
            coef = w * sigmoidf_(f[u]) * invb;
        } else {
            float sp, sg;
            softplus_sigmoid(f[u], sp, sg);
            li += w * sp;
            coef = w * sg * invb;
        }
        if (a.is_dist) coef = raw[u] > 0.f ? coef / raw[u] : 0.f;
        if (a.bf16) coef = round_bf16(coef);  // what the product kernels multiply with
        s[j] = coef;
    }
    li = wave_sum(li);
    if (a.ranking) active = wave_sum(active);
    if (lane == 0) {
        a.row_loss[i] = a.ranking ? li * invb : (softplusf_(-fp) + li) * invb;
        a.cpos[i] = a.ranking ? -active * invb : -sigmoidf_(-fp) * invb;
    }
}

// rows longer than 1024 scores: the same with three passes over memory
__global__ __launch_bounds__(256) void k_loss_long(LossArgs a) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= a.b) return;
    float* s = a.S + (int64_t)i * a.ld_s;
    const float invb = 1.f / (float)a.b;
    const float fp = a.fpos[i];
    const int k = a.k;

    float mx = -INFINITY, z = 1.f;
    if (a.alpha > 0.f) {
        for (int j = lane; j < k; j += 64) {
            const float f = a.is_dist ? a.gamma - s[j] : s[j];
            mx = fmaxf(mx, a.alpha * f);
        }
        mx = wave_max(mx);
        float zz = 0.f;
        for (int j = lane; j < k; j += 64) {
            const float f = a.is_dist ? a.gamma - s[j] : s[j];
            zz += expf(a.alpha * f - mx);
        }
        z = wave_sum(zz);
    }
    float li = 0.f, active = 0.f;
    for (int j = lane; j < k; j += 64) {
        const float raw = s[j];
        const float f = a.is_dist ? a.gamma - raw : raw;
        const float w = a.alpha > 0.f ? expf(a.alpha * f - mx) / z : 1.f / (float)k;
        float coef;
        if (a.ranking) {
            const float m = a.gamma - fp + f;
            li += w * fmaxf(m, 0.f);
            coef = m > 0.f ? w * invb : 0.f;
            active += m > 0.f ? w : 0.f;
        } else {
            li += w * softplusf_(f);
            coef = w * sigmoidf_(f) * invb;
        }
        if (a.is_dist) coef = raw > 0.f ? coef / raw : 0.f;
        if (a.bf16) coef = round_bf16(coef);
        s[j] = coef;
    }
    li = wave_sum(li);
    if (a.ranking) active = wave_sum(active);
    if (lane == 0) {
        a.row_loss[i] = a.ranking ? li * invb : (softplusf_(-fp) + li) * invb;
        a.cpos[i] = a.ranking ? -active * invb : -sigmoidf_(-fp) * invb;
    }
}

struct ChainArgs {
    const float* E;
    const float* R;
    StepIds ids;
    int b, D, Dr;
    int64_t n_ent, n_rel;
    const float* O;
    const float* GO;
    const float* cpos;
    float* Gent;
    float* Grel;
    // after the tiled backward of RotatE / TransE-L1: dL/do_i is the sum of go_parts rows go_stride floats apart, and
    // the workgroups from chain_blocks on add up the partial gradient rows of the corrupting entities
    int go_parts;
    int64_t go_stride;
    int chain_blocks;
    PartialRows rest;
};

// sum of `parts` (at most KGE_PAIR_MAX_PARTS) 16-byte pieces `stride` floats apart, in order; all of them are asked
// for before the first is added (a part that does not exist is read from part 0 and left out of the sum)
__device__ __forceinline__ float4 ld4_parts(const float* p, int parts, int64_t stride) {
    if (parts <= 1) return ld4(p);  // (the same for every thread)
    float4 v[KGE_PAIR_MAX_PARTS];
#pragma unroll
    for (int q = 0; q < KGE_PAIR_MAX_PARTS; ++q) v[q] = ld4(p + (q < parts ? q : 0) * stride);
    float4 s = v[0];
#pragma unroll
    for (int q = 1; q < KGE_PAIR_MAX_PARTS; ++q) {
        if (q < parts) { s.x += v[q].x; s.y += v[q].y; s.z += v[q].z; s.w += v[q].w; }
    }
    return s;
}

__device__ __forceinline__ int64_t clamp_id(int64_t id, int64_t n) { return id < 0 ? 0 : (id >= n ? n - 1 : id); }

template <int MODEL, int NV>
__global__ __launch_bounds__(256) void k_chain(ChainArgs a) {
    if ((int)blockIdx.x >= a.chain_blocks) {  // partial rows of the corrupting entities -> their gradient rows
        const int64_t step = (int64_t)(gridDim.x - a.chain_blocks) * 256;
        for (int64_t e = (int64_t)(blockIdx.x - a.chain_blocks) * 256 + threadIdx.x; e < a.rest.n4; e += step)
            st4(a.rest.out + 4 * e, ld4_parts(a.rest.src + 4 * e, a.rest.parts, a.rest.stride));
        return;
    }
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= a.b) return;
    constexpr bool CPLX = (MODEL == KGE_COMPLEX || MODEL == KGE_ROTATE);
    const int D = a.D;
    const int nvec = CPLX ? D / 8 : D / 4;
    const int im_off = D / 2;
    const StepView sv = step_view(a.ids);
    const bool head = sv.side == KGE_NEG_HEAD;
    const int64_t hid = clamp_id(sv.h[i], a.n_ent), tid = clamp_id(sv.t[i], a.n_ent);
    const int64_t rid = clamp_id(sv.r[i], a.n_rel);
    const float* pa = a.E + (head ? tid : hid) * (int64_t)D;
    const float* pc = a.E + (head ? hid : tid) * (int64_t)D;
    const float* pr = a.R + rid * (int64_t)a.Dr;
    const float* po = a.O + (int64_t)i * D;
    const float* pg = a.GO + (int64_t)i * D;
    // key positions: heads 0..b-1, tails b..2b-1
    float* ga = a.Gent + (int64_t)(head ? a.b + i : i) * D;
    float* gc = a.Gent + (int64_t)(head ? i : a.b + i) * D;
    float* gr = a.Grel + (int64_t)i * a.Dr;
    const float cp = a.cpos[i];

    if constexpr (!CPLX) {
        float4 Ov[NV], Cv[NV];
        float ss = 0.f;
#pragma unroll
        for (int it = 0; it < NV; ++it) {
            const int v = lane + it * 64;
            if (v < nvec) {
                Ov[it] = ld4(po + 4 * v);
                Cv[it] = ld4(pc + 4 * v);
                if (MODEL == KGE_TRANSE_L2) {
                    const float u0 = Ov[it].x - Cv[it].x, u1 = Ov[it].y - Cv[it].y, u2 = Ov[it].z - Cv[it].z,
                                u3 = Ov[it].w - Cv[it].w;
                    ss += u0 * u0 + u1 * u1 + u2 * u2 + u3 * u3;
                }
            }
        }
        float inv = 0.f;
        if (MODEL == KGE_TRANSE_L2) {
            ss = wave_sum(ss);
            inv = ss > 0.f ? 1.f / sqrtf(ss) : 0.f;
        }
#pragma unroll
        for (int it = 0; it < NV; ++it) {
            const int v = lane + it * 64;
            if (v >= nvec) continue;
            const float4 G = ld4_parts(pg + 4 * v, a.go_parts, a.go_stride);
            const float ov[4] = {Ov[it].x, Ov[it].y, Ov[it].z, Ov[it].w};
            const float cv[4] = {Cv[it].x, Cv[it].y, Cv[it].z, Cv[it].w};
            const float gv[4] = {G.x, G.y, G.z, G.w};
            float oa[4], oc[4], orl[4];
            if (MODEL == KGE_DISTMULT) {
                const float4 A = ld4(pa + 4 * v), Rr = ld4(pr + 4 * v);
                const float av[4] = {A.x, A.y, A.z, A.w}, rv[4] = {Rr.x, Rr.y, Rr.z, Rr.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float go = gv[e] + cp * cv[e];
                    oc[e] = cp * ov[e];
                    oa[e] = go * rv[e];
                    orl[e] = go * av[e];
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float u = ov[e] - cv[e];
                    const float dir = MODEL == KGE_TRANSE_L2 ? u * inv : (float)((u > 0.f) - (u < 0.f));
                    const float go = gv[e] - cp * dir;  // d psi / d o = -dir
                    oc[e] = cp * dir;
                    oa[e] = go;
                    orl[e] = head ? -go : go;
                }
            }
            st4(ga + 4 * v, make_float4(oa[0], oa[1], oa[2], oa[3]));
            st4(gc + 4 * v, make_float4(oc[0], oc[1], oc[2], oc[3]));
            st4(gr + 4 * v, make_float4(orl[0], orl[1], orl[2], orl[3]));
        }
    } else {
#pragma unroll
        for (int it = 0; it < NV; ++it) {
            const int v = lane + it * 64;
            if (v >= nvec) continue;
            const float4 Ore = ld4(po + 4 * v), Oim = ld4(po + im_off + 4 * v);
            const float4 Cre = ld4(pc + 4 * v), Cim = ld4(pc + im_off + 4 * v);
            const float4 Gre = ld4_parts(pg + 4 * v, a.go_parts, a.go_stride);
            const float4 Gim = ld4_parts(pg + im_off + 4 * v, a.go_parts, a.go_stride);
            const float4 Are = ld4(pa + 4 * v), Aim = ld4(pa + im_off + 4 * v);
            const float ore[4] = {Ore.x, Ore.y, Ore.z, Ore.w}, oim[4] = {Oim.x, Oim.y, Oim.z, Oim.w};
            const float cre[4] = {Cre.x, Cre.y, Cre.z, Cre.w}, cim[4] = {Cim.x, Cim.y, Cim.z, Cim.w};
            const float gre[4] = {Gre.x, Gre.y, Gre.z, Gre.w}, gim[4] = {Gim.x, Gim.y, Gim.z, Gim.w};
            const float are[4] = {Are.x, Are.y, Are.z, Are.w}, aim[4] = {Aim.x, Aim.y, Aim.z, Aim.w};
            float rre[4], rim[4];
            if (MODEL == KGE_ROTATE) {
                const float4 Th = ld4(pr + 4 * v);
                const float th[4] = {Th.x, Th.y, Th.z, Th.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) sincosf(th[e], &rim[e], &rre[e]);
            } else {
                const float4 Rre = ld4(pr + 4 * v), Rim = ld4(pr + im_off + 4 * v);
                rre[0] = Rre.x; rre[1] = Rre.y; rre[2] = Rre.z; rre[3] = Rre.w;
                rim[0] = Rim.x; rim[1] = Rim.y; rim[2] = Rim.z; rim[3] = Rim.w;
            }
            float oa_re[4], oa_im[4], oc_re[4], oc_im[4], or_a[4], or_b[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float g_re, g_im;
                if (MODEL == KGE_COMPLEX) {  // psi = o . c (real dot product of the [re|im] rows)
                    g_re = gre[e] + cp * cre[e];
                    g_im = gim[e] + cp * cim[e];
                    oc_re[e] = cp * ore[e];
                    oc_im[e] = cp * oim[e];
                } else {  // psi = gamma - sum |o - c|
                    const float q_re = ore[e] - cre[e], q_im = oim[e] - cim[e];
                    const float m2 = q_re * q_re + q_im * q_im;
                    const float invm = m2 > 0.f ? 1.f / sqrtf(m2) : 0.f;
                    const float e_re = q_re * invm, e_im = q_im * invm;
                    g_re = gre[e] - cp * e_re;
                    g_im = gim[e] - cp * e_im;
                    oc_re[e] = cp * e_re;
                    oc_im[e] = cp * e_im;
                }
                const float ri = head ? -rim[e] : rim[e];  // o = a * (rre + i ri)
                oa_re[e] = g_re * rre[e] + g_im * ri;      // g * conj(rre + i ri)
                oa_im[e] = g_im * rre[e] - g_re * ri;
                if (MODEL == KGE_COMPLEX) {
                    const float d_rre = g_re * are[e] + g_im * aim[e];
                    const float d_ri = -g_re * aim[e] + g_im * are[e];
                    or_a[e] = d_rre;
                    or_b[e] = head ? -d_ri : d_ri;
                } else {
                    const float d_th = -g_re * oim[e] + g_im * ore[e];  // do/dtheta = +i o (tail), -i o (head)
                    or_a[e] = head ? -d_th : d_th;
                }
            }
            st4(ga + 4 * v, make_float4(oa_re[0], oa_re[1], oa_re[2], oa_re[3]));
            st4(ga + im_off + 4 * v, make_float4(oa_im[0], oa_im[1], oa_im[2], oa_im[3]));
            st4(gc + 4 * v, make_float4(oc_re[0], oc_re[1], oc_re[2], oc_re[3]));
            st4(gc + im_off + 4 * v, make_float4(oc_im[0], oc_im[1], oc_im[2], oc_im[3]));
            st4(gr + 4 * v, make_float4(or_a[0], or_a[1], or_a[2], or_a[3]));
            if (MODEL == KGE_COMPLEX) st4(gr + im_off + 4 * v, make_float4(or_b[0], or_b[1], or_b[2], or_b[3]));
        }
    }
}

template <int MODEL>
void launch_chain_nv(kge_ctx* c, const ChainArgs& a, int nv, dim3 grid, hipStream_t st) {
    switch (nv) {
    case 1: KGE_LAUNCH(c, (k_chain<MODEL, 1>), grid, dim3(256), 0, st, a); break;
    case 2: KGE_LAUNCH(c, (k_chain<MODEL, 2>), grid, dim3(256), 0, st, a); break;
    case 3: KGE_LAUNCH(c, (k_chain<MODEL, 3>), grid, dim3(256), 0, st, a); break;
    default: KGE_LAUNCH(c, (k_chain<MODEL, 4>), grid, dim3(256), 0, st, a); break;
    }
}

}  // namespace

void kge_launch_loss(kge_ctx* c, int b, int k, float gamma, hipStream_t st) {
    LossArgs a;
    a.S = c->S; a.ld_s = c->ld_s; a.b = b; a.k = k; a.fpos = c->fpos; a.gamma = gamma;
    a.alpha = c->cfg.adv_temperature; a.is_dist = c->cfg.model == KGE_TRANSE_L2;
    a.bf16 = c->cfg.gemm_input; a.ranking = c->cfg.loss == KGE_LOSS_RANKING;
    a.cpos = c->cpos; a.row_loss = c->row_loss;
    const dim3 grid((b + 3) / 4);
    const int vpl = (k + 63) / 64;
    if (vpl <= 4) KGE_LAUNCH(c, k_loss<4>, grid, dim3(256), 0, st, a);
    else if (vpl <= 16) KGE_LAUNCH(c, k_loss<16>, grid, dim3(256), 0, st, a);
    else KGE_LAUNCH(c, k_loss_long, grid, dim3(256), 0, st, a);
}

void kge_launch_chain(kge_ctx* c, const float* E, const float* R, const StepIds& ids, hipStream_t st) {
    ChainArgs a;
    const int b = ids.b;
    a.E = E; a.R = R; a.ids = ids; a.b = b; a.D = c->cfg.ent_dim; a.Dr = c->cfg.rel_dim;
    a.n_ent = c->cfg.num_entities; a.n_rel = c->cfg.num_relations;
    a.O = c->O; a.GO = c->GO; a.cpos = c->cpos; a.Gent = c->Gent; a.Grel = c->Grel;
    a.go_parts = 1; a.go_stride = 0;
    if (c->go_partial.parts > 1) { a.GO = c->go_partial.src; a.go_parts = c->go_partial.parts; a.go_stride = c->go_partial.stride; }
    a.chain_blocks = (b + 3) / 4;
    a.rest = c->neg_partial;
    int rest_blocks = 0;  // 16 bytes per thread, up to four rounds
    if (a.rest.parts > 1) rest_blocks = (int)((a.rest.n4 + 1023) / 1024);
    const int model = c->cfg.model;
    const bool cplx = model == KGE_COMPLEX || model == KGE_ROTATE;
    const int nvec = cplx ? a.D / 8 : a.D / 4;
    const int nv = (nvec + 63) / 64;
    const dim3 grid(a.chain_blocks + rest_blocks);
    switch (model) {
    case KGE_TRANSE_L2: launch_chain_nv<KGE_TRANSE_L2>(c, a, nv, grid, st); break;
    case KGE_TRANSE_L1: launch_chain_nv<KGE_TRANSE_L1>(c, a, nv, grid, st); break;
    case KGE_DISTMULT: launch_chain_nv<KGE_DISTMULT>(c, a, nv, grid, st); break;
    case KGE_COMPLEX: launch_chain_nv<KGE_COMPLEX>(c, a, nv, grid, st); break;
    default: launch_chain_nv<KGE_ROTATE>(c, a, nv, grid, st); break;
    }
}
