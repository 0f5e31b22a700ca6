// Chunked negative scoring for the models whose pair function is not a bilinear form:
//     RotatE      psi(o, n) = gamma - sum_c |o_c - n_c|      (complex modulus per coordinate)
//     TransE-L1   psi(o, n) = gamma - sum_d |o_d - n_d|
// Sec. 3.3's grouping still applies (g positives share k corrupting rows, so each staged row is reused g or k
// times), but the g*k*D pair terms are an elementwise reduction with a square root or an absolute value in
// it, so they run on the vector ALUs, not on the matrix units.
//
// Forward: a workgroup owns a 32x32 tile of (positive, negative) pairs and stages 32 coordinates of both sides in
// LDS at a time; a thread accumulates a 2x2 block of pairs and reads four coordinates of a row with one 16-byte
// LDS load, so one load serves eight pair terms.  The modulus uses the hardware square root (1 ulp).
// Backward: threads own coordinates instead of pairs, so the sums over j (for dL/do_i) and over i (for the
// gradient row of corrupting entity j) stay in registers.  Both sums are made of the same terms
// W_ij dir(o_i - n_j) with opposite signs, and a term costs a reciprocal square root, so it should be formed once:
//   k_pair_bwd_tile  (chunks of up to 128 positives) a workgroup owns 16 positives x a range of negatives; a thread
//                    keeps its coordinate of the 16 o rows and of their 16 running sums in registers, walks the
//                    negatives that fall to its thread group, and adds every term to both sides.  What a workgroup
//                    can sum is partial (over its negatives for dL/do, over its 16 positives for a corrupting row):
//                    the partial rows go to a scratch area and the chain launch (k_chain) adds them in a fixed order.
//   k_pair_bwd       (longer chunks, where that would be too many partial rows) one kind of workgroup walks all k
//                    negatives for 8 positives, the other walks all g positives for 8 negatives, each forming every
//                    term for itself; a workgroup is two groups of threads with 4 rows each, so that rows of 200
//                    coordinates fill its wavefronts.
// Nothing is accumulated with atomics.
#include "kge_common.h"

namespace {

constexpr int PT = 32;       // pair tile edge
constexpr int PCK = 32;      // coordinates staged per step
constexpr int PPITCH = 36;   // floats per staged row: 16-byte aligned rows

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
__device__ __forceinline__ float pair_term(float o_re, float o_im, float n_re, float n_im) {
    const float q_re = o_re - n_re;
    if (!CPLX) return fabsf(q_re);
    const float q_im = o_im - n_im;
    return __builtin_amdgcn_sqrtf(q_re * q_re + q_im * q_im);
}

// 512 threads: both halves of the workgroup hold the same 2x2 blocks of pairs and take the groups of four coordinates of
// every staged step in turn (twice the waves for the same LDS traffic); their sums meet at the end.
template <bool CPLX>
__global__ __launch_bounds__(512) void k_pair_fwd(PairArgs a) {
    __shared__ __attribute__((aligned(16))) float Os[CPLX ? 2 : 1][PT][PPITCH];
    __shared__ __attribute__((aligned(16))) float Ns[CPLX ? 2 : 1][PT][PPITCH];
    __shared__ float halves[256][4];
    const int half = threadIdx.x >> 8, tid = threadIdx.x & 255;
    // pairs (ti + {0,16}, tj + {0,16}) of the tile: the 16 lanes with consecutive tj read consecutive staged rows,
    // which the row pitch spreads over all banks (rows 2 tj + {0,1} would fall on half of them)
    const int tj = tid & 15, ti = tid >> 4;
    const int j0 = blockIdx.x * PT, i0 = blockIdx.y * PT, c = blockIdx.z;
    const int NC = CPLX ? a.D / 2 : a.D;  // coordinates
    const float* Oc = a.O + (int64_t)c * a.g * a.D;
    const float* Nc = a.Nst + (int64_t)c * a.k * a.D;
    float acc[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
    const int lr = tid >> 3, lc = 4 * (tid & 7);
    // one thread stages one 16-byte piece per step (and per part): the first half of the workgroup the positives,
    // the second the negatives.  The piece for the next step is asked for before this step's arithmetic starts.
    const float* src = half == 0 ? Oc + (int64_t)(i0 + lr) * a.D : Nc + (int64_t)(j0 + lr) * a.D;
    const bool rok = half == 0 ? i0 + lr < a.g : j0 + lr < a.k;
    float (*dst)[PT][PPITCH] = half == 0 ? Os : Ns;
    float4 nxt[CPLX ? 2 : 1];
    auto fetch = [&](int c0) {
#pragma unroll
        for (int part = 0; part < (CPLX ? 2 : 1); ++part) {
            nxt[part] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (rok && c0 + lc < NC) nxt[part] = ld4(src + part * NC + c0 + lc);  // NC is a multiple of 4
        }
    };
    fetch(0);
    for (int c0 = 0; c0 < NC; c0 += PCK) {
#pragma unroll
        for (int part = 0; part < (CPLX ? 2 : 1); ++part) st4(&dst[part][lr][lc], nxt[part]);
        if (c0 + PCK < NC) fetch(c0 + PCK);
        __syncthreads();
        // the 32 terms of this step are summed on their own and then added to the running total: the partial
        // sums stay small, which keeps the fp32 rounding of a 200- or 400-term sum near that of a pairwise sum
        float part[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
#pragma unroll
        for (int cq = 0; cq < PCK / 2; cq += 4) {
            // groups of four coordinates go to the two halves in turn, so that a last step with few coordinates is
            // still shared; (NC is a multiple of 4) what lies past NC is padding
            const int cc = 2 * cq + 4 * half;
            if (c0 + cc >= NC) break;
            float o_re[2][4], o_im[2][4], n_re[2][4], n_im[2][4];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const float4 vo = ld4(&Os[0][ti + 16 * u][cc]), vn = ld4(&Ns[0][tj + 16 * u][cc]);
                o_re[u][0] = vo.x; o_re[u][1] = vo.y; o_re[u][2] = vo.z; o_re[u][3] = vo.w;
                n_re[u][0] = vn.x; n_re[u][1] = vn.y; n_re[u][2] = vn.z; n_re[u][3] = vn.w;
                if (CPLX) {
                    const float4 wo = ld4(&Os[CPLX ? 1 : 0][ti + 16 * u][cc]), wn = ld4(&Ns[CPLX ? 1 : 0][tj + 16 * u][cc]);
                    o_im[u][0] = wo.x; o_im[u][1] = wo.y; o_im[u][2] = wo.z; o_im[u][3] = wo.w;
                    n_im[u][0] = wn.x; n_im[u][1] = wn.y; n_im[u][2] = wn.z; n_im[u][3] = wn.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) { o_im[u][e] = 0.f; n_im[u][e] = 0.f; }
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
#pragma unroll
                    for (int q = 0; q < 2; ++q) part[u][q] += pair_term<CPLX>(o_re[u][e], o_im[u][e], n_re[q][e], n_im[q][e]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) { acc[u][0] += part[u][0]; acc[u][1] += part[u][1]; }
        __syncthreads();
    }
    // padded coordinates hold zeros on both sides and contribute |0 - 0| = 0
    if (half == 1) {
        halves[tid][0] = acc[0][0]; halves[tid][1] = acc[0][1]; halves[tid][2] = acc[1][0]; halves[tid][3] = acc[1][1];
    }
    __syncthreads();
    if (half == 1) return;
    acc[0][0] += halves[tid][0]; acc[0][1] += halves[tid][1]; acc[1][0] += halves[tid][2]; acc[1][1] += halves[tid][3];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int i = i0 + ti + 16 * u, j = j0 + tj + 16 * q;
            if (i < a.g && j < a.k) a.S[((int64_t)c * a.g + i) * a.ld_s + j] = a.gamma - acc[u][q];
        }
    }
}

constexpr int BT_MAX = 16;   // most rows per backward workgroup: two thread groups of up to 8 rows each
constexpr int BW = 128;      // coefficients staged per step and row

// blockIdx.x < n_i_tiles: dL/do for 2 BR_O positives (sum over the chunk's k negatives)
// else               : gradient rows of 2 BR_N negatives (sum over the chunk's g positives)
// Thread (group, coordinate): group 0 owns rows r0..r0+BR-1, group 1 the next BR; blockDim = 2 * coordinates per pass
// rounded up to whole waves.  A workgroup's running time goes with BR * (rows it sums over), so the side that sums
// over fewer rows takes 8 rows per thread and the other 4 when the chunk is lopsided (k >= 2g or g >= 2k): all
// workgroups of a launch then run about equally long.  d psi / d o = -dir(o - n), d psi / d n = +dir(o - n), dir = unit complex number (sign
// for real coordinates), 0 where o == n.
template <bool CPLX, bool FOR_O, int BR>
__device__ __forceinline__ void pair_bwd_rows(const PairArgs& a, int c, int r0, int cpp, float (*Ws)[BT_MAX]) {
    constexpr int BT = 2 * BR;
    const int tid = threadIdx.x;
    const int NC = CPLX ? a.D / 2 : a.D;
    const float* Oc = a.O + (int64_t)c * a.g * a.D;
    const float* Nc = a.Nst + (int64_t)c * a.k * a.D;
    const float* Wc = a.S + (int64_t)c * a.g * a.ld_s;
    const int n_own = FOR_O ? a.g : a.k;      // rows on my side
    const int n_other = FOR_O ? a.k : a.g;    // rows I sum over
    const float* own = FOR_O ? Oc : Nc;
    const float* other = FOR_O ? Nc : Oc;
    const int grp = tid >= cpp ? 1 : 0, lc = tid - grp * cpp;
    const int rg = r0 + grp * BR;             // first row of my group

    for (int cb = 0; cb < NC; cb += cpp) {
        const int cc = cb + lc;
        const bool act = lc < cpp && tid < 2 * cpp && cc < NC;
        const int ccs = act ? cc : 0;         // always a valid column
        float x_re[BR], x_im[BR], g_re[BR], g_im[BR];
#pragma unroll
        for (int s = 0; s < BR; ++s) {
            const bool ok = act && rg + s < n_own;
            x_re[s] = ok ? own[(int64_t)(rg + s) * a.D + cc] : 0.f;
            x_im[s] = (ok && CPLX) ? own[(int64_t)(rg + s) * a.D + NC + cc] : 0.f;
            g_re[s] = 0.f;
            g_im[s] = 0.f;
        }
        for (int m0 = 0; m0 < n_other; m0 += BW) {
            __syncthreads();
            // stage W[i][j] for the 8 rows of this workgroup against the next BW rows of the other side
            for (int e = tid; e < BW * BT; e += blockDim.x) {
                const int mm = FOR_O ? e % BW : e / BT, s = FOR_O ? e / BW : e % BT;  // lanes along the contiguous index
                float wv = 0.f;
                if (m0 + mm < n_other && r0 + s < n_own) {
                    const int i = FOR_O ? r0 + s : m0 + mm, j = FOR_O ? m0 + mm : r0 + s;
                    wv = Wc[(int64_t)i * a.ld_s + j];
                }
                Ws[mm][s] = FOR_O ? -wv : wv;
            }
            __syncthreads();
            const int lim = min(BW, n_other - m0);
            const float* yp = other + (int64_t)m0 * a.D + ccs;
            // eight rows of the other side per round, and the loads of the next round go out before this round is
            // worked on, so that the arithmetic of one round covers the latency of the next one's loads
            constexpr int RU = 8;
            float y_re[RU], y_im[RU];
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                const int row = u < lim ? u : lim - 1;
                y_re[u] = yp[(int64_t)row * a.D];
                y_im[u] = CPLX ? yp[(int64_t)row * a.D + NC] : 0.f;
            }
            for (int mm = 0; mm < lim; mm += RU) {
                float z_re[RU], z_im[RU];
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    const int row = mm + RU + u < lim ? mm + RU + u : lim - 1;
                    z_re[u] = yp[(int64_t)row * a.D];
                    z_im[u] = CPLX ? yp[(int64_t)row * a.D + NC] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    if (mm + u < lim) {
                        float wv[BR];
#pragma unroll
                        for (int s4 = 0; s4 < BR; s4 += 4) {
                            const float4 w4 = ld4(&Ws[mm + u][grp * BR + s4]);
                            wv[s4] = w4.x; wv[s4 + 1] = w4.y; wv[s4 + 2] = w4.z; wv[s4 + 3] = w4.w;
                        }
#pragma unroll
                        for (int s = 0; s < BR; ++s) {
                            // o - n with o on my side (FOR_O) or on the other side
                            const float q_re = FOR_O ? x_re[s] - y_re[u] : y_re[u] - x_re[s];
                            if (CPLX) {
                                const float q_im = FOR_O ? x_im[s] - y_im[u] : y_im[u] - x_im[s];
                                // w / |q|; q = 0 gives w * 2^63 * 0 = 0
                                const float t = wv[s] * __builtin_amdgcn_rsqf(fmaxf(q_re * q_re + q_im * q_im, 1e-38f));
                                g_re[s] = fmaf(t, q_re, g_re[s]);
                                g_im[s] = fmaf(t, q_im, g_im[s]);
                            } else {
                                g_re[s] += q_re > 0.f ? wv[s] : (q_re < 0.f ? -wv[s] : 0.f);
                            }
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < RU; ++u) { y_re[u] = z_re[u]; y_im[u] = z_im[u]; }
            }
        }
        float* dst = FOR_O ? a.GO + (int64_t)c * a.g * a.D : a.Gneg + (int64_t)c * a.k * a.D;
#pragma unroll
        for (int s = 0; s < BR; ++s) {
            if (act && rg + s < n_own) {
                dst[(int64_t)(rg + s) * a.D + cc] = g_re[s];
                if (CPLX) dst[(int64_t)(rg + s) * a.D + NC + cc] = g_im[s];
            }
        }
    }
}

template <bool CPLX, int BR_O, int BR_N>
__global__ __launch_bounds__(1024) void k_pair_bwd(PairArgs a, int n_i_tiles, int cpp) {
    __shared__ __attribute__((aligned(16))) float Ws[BW][BT_MAX];
    const int c = blockIdx.y;
    if ((int)blockIdx.x < n_i_tiles) pair_bwd_rows<CPLX, true, BR_O>(a, c, blockIdx.x * 2 * BR_O, cpp, Ws);
    else pair_bwd_rows<CPLX, false, BR_N>(a, c, (blockIdx.x - n_i_tiles) * 2 * BR_N, cpp, Ws);
}

// ---- the tile form of the backward
constexpr int TI = 16;          // positives per workgroup: their coordinate and running sum stay in registers
constexpr int NG = 5;           // thread groups per workgroup: 5 x 200 coordinates fill 16 wavefronts
constexpr int TJB = 8 * NG;     // negatives per staged block of W, dealt round-robin to the groups
constexpr int WPITCH = TI + 4;  // floats per staged row of W^T
constexpr int TILE_CPP = 1024 / NG;  // most coordinates per pass
constexpr int MAX_PARTS = KGE_PAIR_MAX_PARTS;  // most partial rows per gradient row

struct PairTileArgs {
    int n_i_tiles, tj;     // i-tiles per chunk; negatives per workgroup
    int cpp;               // coordinates per pass
    float* dstO;           // dL/do rows or their partial rows: [j-tile][b x D]
    float* dstN;           // gradient rows of the corrupting entities or their partial rows: [i-tile][C*k x D]
    int64_t strideO, strideN;  // floats between consecutive partials (0: the final rows are written directly)
};

// Thread (group, coordinate).  Held to 128 registers: 16 wavefronts per CU, four on every SIMD.
template <bool CPLX>
__global__ __launch_bounds__(1024) void k_pair_bwd_tile(PairArgs a, PairTileArgs t) {
    __shared__ __attribute__((aligned(16))) float Ws[TJB][WPITCH];  // W^T of the block: [negative][positive]
    __shared__ float2 Gs[TI][TILE_CPP];                             // another group's sums for dL/do
    const int tid = threadIdx.x, cpp = t.cpp;
    const int grp = tid / cpp, lc = tid - grp * cpp;
    const int it = blockIdx.x % t.n_i_tiles, jt = blockIdx.x / t.n_i_tiles, c = blockIdx.y;
    const int i0 = it * TI, jb0 = jt * t.tj, jb1 = min(jb0 + t.tj, a.k);
    const int NC = CPLX ? a.D / 2 : a.D;
    const float* Oc = a.O + (int64_t)c * a.g * a.D;
    const float* Nc = a.Nst + (int64_t)c * a.k * a.D;
    const float* Wc = a.S + (int64_t)c * a.g * a.ld_s;
    float* dN = t.dstN + it * t.strideN + (int64_t)c * a.k * a.D;
    float* dO = t.dstO + jt * t.strideO + (int64_t)c * a.g * a.D;

    for (int cb = 0; cb < NC; cb += cpp) {
        const int cc = cb + lc;
        const bool act = grp < NG && cc < NC;
        float x_re[TI], x_im[TI], g_re[TI], g_im[TI];
#pragma unroll
        for (int s = 0; s < TI; ++s) {
            const bool ok = act && i0 + s < a.g;
            x_re[s] = ok ? Oc[(int64_t)(i0 + s) * a.D + cc] : 0.f;
            x_im[s] = (ok && CPLX) ? Oc[(int64_t)(i0 + s) * a.D + NC + cc] : 0.f;
            g_re[s] = 0.f;
            g_im[s] = 0.f;
        }
        for (int j0 = jb0; j0 < jb1; j0 += TJB) {
            const int jn = min(TJB, jb1 - j0);  // negatives in this block
            __syncthreads();
            // W of the block, transposed; 0 for positives outside the chunk, so that such pairs add nothing
            for (int e = tid; e < jn * TI; e += blockDim.x) {
                const int jj = e % jn, ii = e / jn;
                Ws[jj][ii] = i0 + ii < a.g ? Wc[(int64_t)(i0 + ii) * a.ld_s + j0 + jj] : 0.f;
            }
            __syncthreads();
            if (grp >= jn || !act) continue;  // (the barriers above are outside of this)
            float y_re = Nc[(int64_t)(j0 + grp) * a.D + cc], y_im = CPLX ? Nc[(int64_t)(j0 + grp) * a.D + NC + cc] : 0.f;
            for (int jj = grp; jj < jn; jj += NG) {
                const int j = j0 + jj;
                const int jnx = jj + NG < jn ? j + NG : j;  // the next row is asked for before this one is worked on
                const float z_re = Nc[(int64_t)jnx * a.D + cc], z_im = CPLX ? Nc[(int64_t)jnx * a.D + NC + cc] : 0.f;
                float n_re = 0.f, n_im = 0.f;
#pragma unroll
                for (int s4 = 0; s4 < TI; s4 += 4) {
                    const float4 w4 = ld4(&Ws[jj][s4]);
                    const float wv[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int s = s4 + e;
                        const float q_re = x_re[s] - y_re;  // o - n
                        if (CPLX) {
                            const float q_im = x_im[s] - y_im;
                            // w / |q|; q = 0 gives a finite factor times 0
                            const float f = wv[e] * __builtin_amdgcn_rsqf(fmaf(q_im, q_im, fmaf(q_re, q_re, 1.2e-38f)));
                            g_re[s] = fmaf(-f, q_re, g_re[s]);
                            g_im[s] = fmaf(-f, q_im, g_im[s]);
                            n_re = fmaf(f, q_re, n_re);
                            n_im = fmaf(f, q_im, n_im);
                        } else {
                            const float v = q_re > 0.f ? wv[e] : (q_re < 0.f ? -wv[e] : 0.f);
                            g_re[s] -= v;
                            n_re += v;
                        }
                    }
                }
                dN[(int64_t)j * a.D + cc] = n_re;
                if (CPLX) dN[(int64_t)j * a.D + NC + cc] = n_im;
                y_re = z_re;
                y_im = z_im;
            }
        }
        // dL/do: the other groups' sums are added to the first group's, in group order
        for (int o = 1; o < NG; ++o) {
            __syncthreads();
            if (grp == o && act) {
#pragma unroll
                for (int s = 0; s < TI; ++s) Gs[s][lc] = make_float2(g_re[s], g_im[s]);
            }
            __syncthreads();
            if (grp == 0 && act) {
#pragma unroll
                for (int s = 0; s < TI; ++s) {
                    const float2 v = Gs[s][lc];
                    g_re[s] += v.x;
                    g_im[s] += v.y;
                }
            }
        }
        if (grp == 0 && act) {
#pragma unroll
            for (int s = 0; s < TI; ++s) {
                if (i0 + s < a.g) {
                    dO[(int64_t)(i0 + s) * a.D + cc] = g_re[s];
                    if (CPLX) dO[(int64_t)(i0 + s) * a.D + NC + cc] = g_im[s];
                }
            }
        }
    }
}

template <bool CPLX>
void launch_pair_bwd(kge_ctx* c, const PairArgs& a, int chunks, int cpp, dim3 block, hipStream_t st) {
    const int br_o = a.g >= 2 * a.k ? 8 : 4, br_n = a.k >= 2 * a.g ? 8 : 4;
    const int n_i_tiles = (a.g + 2 * br_o - 1) / (2 * br_o), n_j_tiles = (a.k + 2 * br_n - 1) / (2 * br_n);
    const dim3 grid(n_i_tiles + n_j_tiles, chunks);
    if (br_o == 8) KGE_LAUNCH(c, (k_pair_bwd<CPLX, 8, 4>), grid, block, 0, st, a, n_i_tiles, cpp);
    else if (br_n == 8) KGE_LAUNCH(c, (k_pair_bwd<CPLX, 4, 8>), grid, block, 0, st, a, n_i_tiles, cpp);
    else KGE_LAUNCH(c, (k_pair_bwd<CPLX, 4, 4>), grid, block, 0, st, a, n_i_tiles, cpp);
}

}  // namespace

void kge_pair_neg_score(kge_ctx* c, int b, int k, int gsz, float gamma, float* out, int ld_out, hipStream_t st) {
    PairArgs a = {};
    a.O = c->O; a.Nst = c->Nst; a.S = out; a.ld_s = ld_out; a.g = gsz; a.k = k; a.D = c->cfg.ent_dim; a.gamma = gamma;
    const dim3 grid((k + PT - 1) / PT, (gsz + PT - 1) / PT, b / gsz);
    if (c->cfg.model == KGE_ROTATE) KGE_LAUNCH(c, k_pair_fwd<true>, grid, dim3(512), 0, st, a);
    else KGE_LAUNCH(c, k_pair_fwd<false>, grid, dim3(512), 0, st, a);
}

void kge_pair_neg_backward(kge_ctx* c, int b, int k, int gsz, hipStream_t st) {
    PairArgs a = {};
    a.O = c->O; a.Nst = c->Nst; a.S = c->S; a.ld_s = c->ld_s; a.g = gsz; a.k = k; a.D = c->cfg.ent_dim;
    a.GO = c->GO; a.Gneg = c->Gent + (int64_t)2 * b * a.D;
    const int nc_all = c->cfg.model == KGE_ROTATE ? a.D / 2 : a.D;
    const int chunks = b / gsz, n_i_tiles = (gsz + TI - 1) / TI;
    if (n_i_tiles <= MAX_PARTS && c->pair_part_o) {
        // the tile form.  Enough workgroups for the chip, at most MAX_PARTS ranges of negatives per chunk
        int pj = (256 + chunks * n_i_tiles - 1) / (chunks * n_i_tiles);
        pj = pj > MAX_PARTS ? MAX_PARTS : pj;
        pj = pj > (k + NG - 1) / NG ? (k + NG - 1) / NG : pj;  // at least one negative per thread group
        PairTileArgs t;
        t.n_i_tiles = n_i_tiles;
        t.tj = (k + pj - 1) / pj;
        pj = (k + t.tj - 1) / t.tj;
        const int passes = (nc_all + TILE_CPP - 1) / TILE_CPP;
        t.cpp = (nc_all + passes - 1) / passes;
        const int64_t rows_o = (int64_t)b * a.D, rows_n = (int64_t)chunks * k * a.D;
        t.dstO = pj > 1 ? c->pair_part_o : a.GO;
        t.strideO = pj > 1 ? rows_o : 0;
        t.dstN = n_i_tiles > 1 ? c->pair_part_n : a.Gneg;
        t.strideN = n_i_tiles > 1 ? rows_n : 0;
        const dim3 grid(n_i_tiles * pj, chunks), block((NG * t.cpp + 63) / 64 * 64);
        if (c->cfg.model == KGE_ROTATE) KGE_LAUNCH(c, k_pair_bwd_tile<true>, grid, block, 0, st, a, t);
        else KGE_LAUNCH(c, k_pair_bwd_tile<false>, grid, block, 0, st, a, t);
        // the chain launch that follows adds up the partial rows
        c->go_partial = {c->pair_part_o, a.GO, pj, rows_o, rows_o / 4};
        c->neg_partial = {c->pair_part_n, a.Gneg, n_i_tiles, rows_n, rows_n / 4};
        return;
    }
    c->go_partial = {};
    c->neg_partial = {};
    // coordinates per pass: all of them if two thread groups of that size fit a workgroup, else 512
    const int nc = c->cfg.model == KGE_ROTATE ? a.D / 2 : a.D;
    const int cpp = nc <= 512 ? nc : 512;
    const dim3 block((2 * cpp + 63) / 64 * 64);
    if (c->cfg.model == KGE_ROTATE) launch_pair_bwd<true>(c, a, b / gsz, cpp, block, st);
    else launch_pair_bwd<false>(c, a, b / gsz, cpp, block, st);
}
