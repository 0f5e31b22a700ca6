// Chunked negative scoring for the models whose pair function is not a bilinear form:
//     RotatE      psi(o, n) = gamma - sum_c |o_c - n_c|      (complex modulus per coordinate)
//     TransE-L1   psi(o, n) = gamma - sum_d |o_d - n_d|
// Sec. 3.3's grouping still applies (g positives share k corrupting rows, so each staged row is reused g or k
// times), but the g*k*D pair terms are an elementwise reduction with a square root or an absolute value in
// it, so they run on the vector ALUs, not on the matrix units.
//
// Forward: a workgroup owns a 32x32 tile of (positive, negative) pairs, stages 32 coordinates of both sides
// in LDS at a time, and each thread accumulates four pairs (one corrupting row against four positives).
// Backward: threads own coordinates instead of pairs, so the sums over j (for dL/do_i) and over i (for the
// gradient row of corrupting entity j) stay in registers: one kind of workgroup walks all k negatives for 8
// positives, the other walks all g positives for 8 negatives.  Nothing is accumulated with atomics.
#include "kge_common.h"

namespace {

constexpr int PT = 32;       // pair tile edge
constexpr int PCK = 32;      // coordinates staged per step
constexpr int PPITCH = 33;

struct PairArgs {
    const float* O;    // [b x D]
    const float* Nst;  // [C*k x D]
    float* S;          // forward: out [b x ld_s]; backward: W in
    int ld_s, g, k, D;
    float gamma;
    float* GO;         // [b x D]
    float* Gneg;       // [C*k x D] gradient rows of the corrupting entities
};

template <bool CPLX>
__global__ __launch_bounds__(256) void k_pair_fwd(PairArgs a) {
    __shared__ float Os[2][PT][PPITCH];
    __shared__ float Ns[2][PT][PPITCH];
    const int tid = threadIdx.x, tj = tid & 31, ti = tid >> 5;
    const int j0 = blockIdx.x * PT, i0 = blockIdx.y * PT, c = blockIdx.z;
    const int NC = CPLX ? a.D / 2 : a.D;  // coordinates
    const float* Oc = a.O + (int64_t)c * a.g * a.D;
    const float* Nc = a.Nst + (int64_t)c * a.k * a.D;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const int lr = tid >> 3, lc = 4 * (tid & 7);
    for (int c0 = 0; c0 < NC; c0 += PCK) {
        const bool cok = c0 + lc < NC;  // NC is a multiple of 4
#pragma unroll
        for (int part = 0; part < (CPLX ? 2 : 1); ++part) {
            float4 vo = make_float4(0.f, 0.f, 0.f, 0.f), vn = vo;
            if (cok && i0 + lr < a.g) vo = ld4(Oc + (int64_t)(i0 + lr) * a.D + part * NC + c0 + lc);
            if (cok && j0 + lr < a.k) vn = ld4(Nc + (int64_t)(j0 + lr) * a.D + part * NC + c0 + lc);
            Os[part][lr][lc] = vo.x; Os[part][lr][lc + 1] = vo.y; Os[part][lr][lc + 2] = vo.z; Os[part][lr][lc + 3] = vo.w;
            Ns[part][lr][lc] = vn.x; Ns[part][lr][lc + 1] = vn.y; Ns[part][lr][lc + 2] = vn.z; Ns[part][lr][lc + 3] = vn.w;
        }
        __syncthreads();
        // the 32 terms of this step are summed on their own and then added to the running total: the partial
        // sums stay small, which keeps the fp32 rounding of a 200- or 400-term sum near that of a pairwise sum
        float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int cc = 0; cc < PCK; ++cc) {
            const float n_re = Ns[0][tj][cc];
            const float n_im = CPLX ? Ns[1][tj][cc] : 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float q_re = Os[0][ti + 8 * s][cc] - n_re;
                if (CPLX) {
                    const float q_im = Os[1][ti + 8 * s][cc] - n_im;
                    part[s] += sqrtf(q_re * q_re + q_im * q_im);
                } else {
                    part[s] += fabsf(q_re);
                }
            }
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) acc[s] += part[s];
        __syncthreads();
    }
    // padded coordinates hold zeros on both sides and contribute |0 - 0| = 0
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int i = i0 + ti + 8 * s, j = j0 + tj;
        if (i < a.g && j < a.k) a.S[((int64_t)c * a.g + i) * a.ld_s + j] = a.gamma - acc[s];
    }
}

// direction of (o - n): unit complex number, or sign for real coordinates; 0 where o == n
template <bool CPLX>
__device__ __forceinline__ void direction(float q_re, float q_im, float& e_re, float& e_im) {
    if (CPLX) {
        const float m2 = q_re * q_re + q_im * q_im;
        const float inv = m2 > 0.f ? __builtin_amdgcn_rsqf(m2) : 0.f;
        e_re = q_re * inv;
        e_im = q_im * inv;
    } else {
        e_re = (float)((q_re > 0.f) - (q_re < 0.f));
        e_im = 0.f;
    }
}

constexpr int BT = 8;     // rows per backward workgroup
constexpr int BW = 256;   // coefficients staged per step

// blockIdx.x < n_i_tiles: dL/do for positives i0..i0+7 (sum over the chunk's k negatives)
// else               : gradient rows of negatives j0..j0+7 (sum over the chunk's g positives)
template <bool CPLX>
__global__ __launch_bounds__(256) void k_pair_bwd(PairArgs a, int n_i_tiles) {
    __shared__ float Ws[BW][BT];
    const int tid = threadIdx.x, c = blockIdx.y;
    const int NC = CPLX ? a.D / 2 : a.D;
    const float* Oc = a.O + (int64_t)c * a.g * a.D;
    const float* Nc = a.Nst + (int64_t)c * a.k * a.D;
    const float* Wc = a.S + (int64_t)c * a.g * a.ld_s;
    const bool for_o = (int)blockIdx.x < n_i_tiles;
    const int r0 = (for_o ? blockIdx.x : blockIdx.x - n_i_tiles) * BT;
    const int n_own = for_o ? a.g : a.k;      // rows on my side
    const int n_other = for_o ? a.k : a.g;    // rows I sum over
    const float* own = for_o ? Oc : Nc;
    const float* other = for_o ? Nc : Oc;
    const float sgn = for_o ? -1.f : 1.f;     // d psi/d o = -dir(o - n), d psi/d n = +dir(o - n)

    for (int cb = 0; cb < NC; cb += 256) {
        const int cc = cb + tid;
        const bool act = cc < NC;
        float x_re[BT], x_im[BT], g_re[BT], g_im[BT];
#pragma unroll
        for (int s = 0; s < BT; ++s) {
            const bool ok = act && r0 + s < n_own;
            x_re[s] = ok ? own[(int64_t)(r0 + s) * a.D + cc] : 0.f;
            x_im[s] = (ok && CPLX) ? own[(int64_t)(r0 + s) * a.D + NC + cc] : 0.f;
            g_re[s] = 0.f;
            g_im[s] = 0.f;
        }
        for (int m0 = 0; m0 < n_other; m0 += BW) {
            __syncthreads();
            // stage W[i][j] for my 8 rows against the next BW rows of the other side
            for (int e = tid; e < BW * BT; e += 256) {
                const int mm = e / BT, s = e % BT;
                float wv = 0.f;
                if (m0 + mm < n_other && r0 + s < n_own) {
                    const int i = for_o ? r0 + s : m0 + mm, j = for_o ? m0 + mm : r0 + s;
                    wv = Wc[(int64_t)i * a.ld_s + j];
                }
                Ws[mm][s] = wv;
            }
            __syncthreads();
            const int lim = min(BW, n_other - m0);
            if (act) {
                for (int mm = 0; mm < lim; ++mm) {
                    const float y_re = other[(int64_t)(m0 + mm) * a.D + cc];
                    const float y_im = CPLX ? other[(int64_t)(m0 + mm) * a.D + NC + cc] : 0.f;
#pragma unroll
                    for (int s = 0; s < BT; ++s) {
                        // o - n with o on my side (for_o) or on the other side
                        const float q_re = for_o ? x_re[s] - y_re : y_re - x_re[s];
                        const float q_im = for_o ? x_im[s] - y_im : y_im - x_im[s];
                        float e_re, e_im;
                        direction<CPLX>(q_re, q_im, e_re, e_im);
                        const float wv = Ws[mm][s] * sgn;
                        g_re[s] += wv * e_re;
                        if (CPLX) g_im[s] += wv * e_im;
                    }
                }
            }
        }
        float* dst = for_o ? a.GO + (int64_t)c * a.g * a.D : a.Gneg + (int64_t)c * a.k * a.D;
#pragma unroll
        for (int s = 0; s < BT; ++s) {
            if (act && r0 + s < n_own) {
                dst[(int64_t)(r0 + s) * a.D + cc] = g_re[s];
                if (CPLX) dst[(int64_t)(r0 + s) * a.D + NC + cc] = g_im[s];
            }
        }
    }
}

}  // namespace

void kge_pair_neg_score(kge_ctx* c, int b, int k, int gsz, float gamma, float* out, int ld_out, hipStream_t st) {
    PairArgs a = {};
    a.O = c->O; a.Nst = c->Nst; a.S = out; a.ld_s = ld_out; a.g = gsz; a.k = k; a.D = c->cfg.ent_dim; a.gamma = gamma;
    const dim3 grid((k + PT - 1) / PT, (gsz + PT - 1) / PT, b / gsz);
    if (c->cfg.model == KGE_ROTATE) KGE_LAUNCH(c, k_pair_fwd<true>, grid, dim3(256), 0, st, a);
    else KGE_LAUNCH(c, k_pair_fwd<false>, grid, dim3(256), 0, st, a);
}

void kge_pair_neg_backward(kge_ctx* c, int b, int k, int gsz, hipStream_t st) {
    PairArgs a = {};
    a.O = c->O; a.Nst = c->Nst; a.S = c->S; a.ld_s = c->ld_s; a.g = gsz; a.k = k; a.D = c->cfg.ent_dim;
    a.GO = c->GO; a.Gneg = c->Gent + (int64_t)2 * b * a.D;
    const int n_i_tiles = (gsz + BT - 1) / BT, n_j_tiles = (k + BT - 1) / BT;
    const dim3 grid(n_i_tiles + n_j_tiles, b / gsz);
    if (c->cfg.model == KGE_ROTATE) KGE_LAUNCH(c, k_pair_bwd<true>, grid, dim3(256), 0, st, a, n_i_tiles);
    else KGE_LAUNCH(c, k_pair_bwd<false>, grid, dim3(256), 0, st, a, n_i_tiles);
}
