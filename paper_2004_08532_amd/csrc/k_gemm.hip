// Chunked negative scoring and its backward as batched fp32 matrix products on the MFMA units.
//
// Sec. 3.3 of the paper: inside one group of g positives that share k corrupting entities, the g*k pair
// scores are one dense contraction.  With O_c [g x D] the o-vectors of chunk c and N_c [k x D] its corrupting
// rows:
//     forward   S_c  = O_c N_c^T                (DistMult, ComplEx: the score itself;
//                                                TransE-L2: |o|^2 + |n|^2 - 2 S -> distance -> gamma - distance)
//     backward  dO_c = W_c N_c   [- rowsum(W) o  for TransE-L2]
//               dN_c = W_c^T O_c [- colsum(W) n  for TransE-L2]
// where W holds dL/df- (divided by the distance for TransE-L2).
//
// Kernel shape.  These products are small (0.16 GFLOP forward at b = 1000, k = 200, D = 400) and the chip has
// 1024 SIMDs, so a workgroup owns one 32x32 output tile and its NW wavefronts split the K dimension: wave w
// takes K-blocks w, w + NW, ... of 32.  Each wave stages its own 32x32 A and B blocks in a private LDS
// region (coalesced, branch-free 16-byte global loads that are all in flight together; no workgroup barrier in
// the main loop), feeds v_mfma_f32_32x32x2_f32, and the NW partial tiles are summed through LDS in a fixed
// order at the end, so results do not depend on scheduling.  Operands may be stored K-contiguous ("KC":
// [rows][K]) or row-contiguous ("MC": [K][rows]); both are read from memory as they lie.
//
// What is fused (uniform negative weights):
//   * W is then an elementwise function of the score, so the forward epilogue, which holds every score exactly
//     once, stores W instead of the score and adds up softplus(f-) for the loss value (no separate loss kernel).
//     (Forming W inside the backward tiles instead was measured: every element is then transformed in 26 tiles,
//     and those instructions, not memory, set the pace of the launch.)
//   * one backward launch computes dO and dN; their tiles run side by side; TransE-L2's rowsum(W) / colsum(W)
//     fall out of the operand fragments;
//   * for TransE-L2 and DistMult the chain rule from dL/do to the head, tail and relation gradient rows is
//     elementwise, so the dO epilogue writes those rows directly (no dL/do array, no separate chain kernel);
//     the rows it needs for that are fetched before the K loop starts.  ComplEx couples the real and the imaginary
//     part of a coordinate; its dO tiles take 16 real parts and their 16 imaginary parts as their 32 columns and do
//     the same.

#include "k_gemm_shared.h"

namespace {

constexpr int TILE = 32;
constexpr int KC_PITCH = 36;                 // floats; 16-byte aligned rows, conflict-free 128-bit reads
constexpr int REGION = TILE * KC_PITCH;      // floats per staged operand block

// Loads 32x32 blocks of one operand into registers (zero-filled outside the matrix).  The per-lane row pointers
// and edge masks are set up once.  Loads are branch-free: the four loads of a block are issued unconditionally
// (from a clamped, always valid address) and masked afterwards, so that all of them, and those of the other
// operand, are in flight together.
// KC: element (row, kk) at base[(r0 + row) * ld + k0 + kk]; lane covers row = lane/8 + 8*it, kk = 4*(lane%8)..+3
// MC: element (row, kk) at base[(k0 + kk) * ld + r0 + row]; lane covers kk = lane/8 + 8*it, row = 4*(lane%8)..+3
template <bool KC>
struct BlockLoader {
    const float* p[4];     // KC: start of the lane's row; MC: row (lane/8 + 8*it) of K-block 0 at the lane's column
    bool ok[4];            // KC: the lane's row exists
    const float* p0_safe;  // an address that is always valid to read 16 bytes from
    int minor, major0, ld, K;
    bool m1, m2, m3, any;  // MC: which of the lane's 4 consecutive rows exist
    __device__ __forceinline__ void init(const float* base, int ld_, int r0, int rows, int K_, int lane) {
        minor = 4 * (lane & 7);
        major0 = lane >> 3;
        ld = ld_;
        K = K_;
        p0_safe = base;
        if (KC) {
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int gr = r0 + major0 + 8 * it;
                ok[it] = gr < rows;
                p[it] = base + (int64_t)(ok[it] ? gr : 0) * ld;  // start of the row: always readable
            }
            any = true; m1 = m2 = m3 = true;
        } else {
            init_rows_at(base, r0 + minor, rows);
        }
    }
    // MC: the lane's four consecutive rows start at row gr of a range that ends before row lim
    __device__ __forceinline__ void init_rows_at(const float* base, int gr, int lim) {
        any = gr < lim; m1 = gr + 1 < lim; m2 = gr + 2 < lim; m3 = gr + 3 < lim;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            ok[it] = true;
            p[it] = base + (int64_t)(major0 + 8 * it) * ld + (any ? gr : 0);
        }
    }
    // shift: floats from the operand that init was given to the one that block kb is taken from (IND_CHUNK_SUM)
    __device__ __forceinline__ void issue(int kb, float4 (&reg)[4], int64_t shift = 0) const {
        const int k0 = kb * 32;
        if (KC) {
            const int gk = k0 + minor;
            const int koff = gk < K ? gk : 0;  // the first 16 bytes of a row are always there
#pragma unroll
            for (int it = 0; it < 4; ++it) reg[it] = ld4(p[it] + shift + koff);
        } else {
#pragma unroll
            for (int it = 0; it < 4; ++it)
                reg[it] = ld4(k0 + major0 + 8 * it < K ? p[it] + shift + (int64_t)k0 * ld : p0_safe);
        }
    }
    // validity of element e (0..3) of register it for K-block kb
    __device__ __forceinline__ bool valid(int kb, int it, int e) const {
        const int k0 = kb * 32;
        if (KC) return ok[it] && k0 + minor + e < K;
        const bool kin = k0 + major0 + 8 * it < K;
        return kin && (e == 0 ? any : (e == 1 ? m1 : (e == 2 ? m2 : m3)));
    }
    // Elements outside the matrix become 0.
    __device__ __forceinline__ void mask(int kb, float4 (&reg)[4]) const {
        const float fill = 0.f;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            reg[it].x = valid(kb, it, 0) ? reg[it].x : fill;
            reg[it].y = valid(kb, it, 1) ? reg[it].y : fill;
            reg[it].z = valid(kb, it, 2) ? reg[it].z : fill;
            reg[it].w = valid(kb, it, 3) ? reg[it].w : fill;
        }
    }
};

template <bool KC>
__device__ __forceinline__ void lds_store(float* region, int lane, const float4 (&reg)[4]) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int major = (lane >> 3) + 8 * it;
        const int minor = 4 * (lane & 7);
        st4(region + major * (KC ? KC_PITCH : TILE) + minor, reg[it]);
    }
}

// The four K-values a lane feeds to MFMAs t = 0..3 of K-octet q: kk = 8q + 4*(lane/32) + t, for row lane%32.
template <bool KC>
__device__ __forceinline__ void lds_frag(const float* region, int lane, int q, float (&f)[4]) {
    const int rw = lane & 31, kk = 8 * q + 4 * (lane >> 5);
    if (KC) {
        const float4 v = ld4(region + rw * KC_PITCH + kk);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) f[t] = region[(kk + t) * TILE + rw];
    }
}

// One 32x32 output tile: K loop, cross-wave sum, epilogue.
template <int NW, bool A_KC, bool B_KC, int EPI, bool IS_DO, int IND = IND_NONE>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, int tile, float (*lds)[2][REGION]) {
    constexpr bool CHAIN = EPI == EPI_CHAIN_L2 || EPI == EPI_CHAIN_DM || EPI == EPI_CHAIN_CX;
    constexpr bool CX = EPI == EPI_CHAIN_CX;
    constexpr bool WANT_ASUM = EPI == EPI_L2_DO || EPI == EPI_L2_DN || EPI == EPI_CHAIN_L2;
    constexpr bool IS_FWD = A_KC && B_KC;  // only the forward product has both operands K-contiguous
    constexpr int NE = TILE * TILE / (NW * 64);           // output elements per thread
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n0 = (tile % g.gx) * TILE, mt = (tile / g.gx) % g.gy, m0 = mt * TILE, c = tile / (g.gx * g.gy);
    const float* A = g.A + c * g.sA;
    const float* B = g.B + c * g.sB;
    if (IND == IND_CHUNK_REL) A = g.A + (c / g.ind_g) * g.sA;
    if (IND == IND_CHUNK_REL) {
        const StepView sv = step_view(g.ids);
        B = g.B + clamp_id(sv.r[c], g.n_rel) * g.sB + g.b_off;
    }
    if (IND == IND_ITEM_CHUNK) B = g.B + (c / g.ind_g) * g.sB;
    if (IND == IND_CHUNK_SUM) B = g.B + g.b_off;  // relation 0's matrix; a block is shifted to its positive's relation
    float* As = lds[w][0];
    float* Bs = lds[w][1];
    // ComplEx chain rule: the real and the imaginary part of a coordinate have to meet in one tile, so the tile's
    // 32 columns are 16 consecutive real parts (columns c0 .. of the [re | im] rows) and the 16 imaginary parts
    // that belong to them (columns N/2 + c0 ..); the tile index along N counts groups of 16 coordinates.
    const int c0 = CX ? (tile % g.gx) * (TILE / 2) : 0;
    auto col_of = [&](int j) { return CX ? (j < TILE / 2 ? c0 + j : g.N / 2 + c0 + j - TILE / 2) : n0 + j; };
    auto col_in = [&](int j) { return CX ? c0 + (j & (TILE / 2 - 1)) < g.N / 2 : n0 + j < g.N; };

    // ---- chain-rule epilogues: fetch what they need now, so that it arrives while the K loop runs
    float e_o[NE], e_c[NE], e_a[NE], e_r[NE], e_cp[NE], e_inv[NE];
    bool e_head = false;
    if (CHAIN) {
        const StepView sv = step_view(g.ids);
        e_head = sv.side == KGE_NEG_HEAD;
#pragma unroll
        for (int it = 0; it < NE; ++it) {
            const int e = threadIdx.x + it * NW * 64;
            const int gm = m0 + (e >> 5);
            const bool in = gm < g.M && col_in(e & 31);
            const int i = c * g.M + (in ? gm : 0);  // index of the positive in the mini-batch
            const int d = in ? col_of(e & 31) : 0;
            const int64_t hid = clamp_id(sv.h[i], g.n_ent), tid = clamp_id(sv.t[i], g.n_ent);
            const int64_t aid = e_head ? tid : hid, cid = e_head ? hid : tid;
            e_o[it] = g.X[(int64_t)i * g.ldx + d];
            e_c[it] = g.E[cid * g.D + d];
            e_cp[it] = g.cpos[i];
            e_a[it] = 0.f; e_r[it] = 0.f; e_inv[it] = 0.f;
            if (EPI == EPI_CHAIN_DM || CX) {
                const int64_t rid = clamp_id(sv.r[i], g.n_rel);
                e_a[it] = g.E[aid * g.D + d];
                e_r[it] = g.R[rid * g.D + d];
            } else {
                e_inv[it] = g.inv_dpos[i];
            }
        }
    }

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    float a_sum = 0.f;  // sum over this lane's K-values of A[m = lane%32][.]  (rowsum / colsum of W)

    const int nblk = (IND == IND_CHUNK_SUM ? g.ind_g : 1) * ((g.K + TILE - 1) / TILE);
    float4 ra[4], rb[4];
    BlockLoader<A_KC> la;
    BlockLoader<B_KC> lb;
    la.init(A, g.lda, m0, g.M, g.K, lane);
    lb.init(B, g.ldb, n0, g.N, g.K, lane);
    if (CX) {  // the lane's four columns lie inside one half of the tile, and inside one half of the row
        const int j = 4 * (lane & 7);
        lb.init_rows_at(B, col_of(j), col_in(j) ? (j < TILE / 2 ? g.N / 2 : g.N) : 0);
    }
    // IND_CHUNK_SUM: block kb is block kb % bpi of positive kb / bpi of the chunk; where its operands lie is looked up
    // (the positive's relation id) one round before its loads go out
    const int bpi = (g.K + TILE - 1) / TILE;
    const StepView sv_sum = IND == IND_CHUNK_SUM ? step_view(g.ids) : StepView();
    auto place = [&](int blk, int& kl, int64_t& sa, int64_t& sb) {
        kl = blk; sa = 0; sb = 0;
        if (IND == IND_CHUNK_SUM) {
            const int p = blk / bpi;
            kl = blk - p * bpi;
            sa = p * g.sA_item;
            sb = clamp_id(sv_sum.r[c * g.ind_g + p], g.n_rel) * g.sB;
        }
    };
    int kb = w, kl = 0, kl_n = 0;
    int64_t sa = 0, sb = 0, sa_n = 0, sb_n = 0;
    if (kb < nblk) {
        place(kb, kl, sa, sb);
        la.issue(kl, ra, sa);
        lb.issue(kl, rb, sb);
        if (kb + NW < nblk) place(kb + NW, kl_n, sa_n, sb_n);
    }
    while (kb < nblk) {
        la.mask(kl, ra);
        lb.mask(kl, rb);
        lds_store<A_KC>(As, lane, ra);
        lds_store<B_KC>(Bs, lane, rb);
        const int nxt = kb + NW;
        if (nxt < nblk) {  // next block's global loads fly while this block is multiplied
            la.issue(kl_n, ra, sa_n);
            lb.issue(kl_n, rb, sb_n);
            kl = kl_n;
            if (nxt + NW < nblk) place(nxt + NW, kl_n, sa_n, sb_n);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float fa[4], fb[4];
            lds_frag<A_KC>(As, lane, q, fa);
            lds_frag<B_KC>(Bs, lane, q, fb);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[t], fb[t], acc, 0, 0, 0);
                if (WANT_ASUM) a_sum += fa[t];
            }
        }
        __builtin_amdgcn_wave_barrier();
        kb = nxt;
    }

    // ---- sum the NW partial tiles (fixed order) and apply the epilogue
    // accumulator register v of lane l holds C[8*(v/4) + 4*(l/32) + v%4][l%32]
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        As[i * TILE + (lane & 31)] = acc[v];
    }
    if (WANT_ASUM) {
        a_sum += __shfl_xor(a_sum, 32, 64);
        if (lane < 32) Bs[lane] = a_sum;
    }
    __syncthreads();
    float* C = g.C + c * g.sC;
    float loss = 0.f;  // OUT_W: softplus(f-) of this thread's elements
#pragma unroll
    for (int it = 0; it < NE; ++it) {
        const int e = threadIdx.x + it * NW * 64;
        const int i = e >> 5, j = e & 31;
        const int gm = m0 + i, gn = n0 + j;
        if (IS_FWD && g.out_mode == OUT_RANK) {
            // evaluation: nothing is stored; rank_i = 1 + #{j : f-_ij > f+_i}.  The 32 consecutive lanes that hold the
            // row's columns of this tile count them and add the count to the row's rank (integer atomics, any order).
            const bool in = gm < g.M && gn < g.N;
            const int row = gm < g.M ? gm : 0, col = gn < g.N ? gn : 0;
            float f = 0.f;
#pragma unroll
            for (int ww = 0; ww < NW; ++ww) f += lds[ww][0][e];
            if (EPI == EPI_L2_FWD) {
                const float d2 = g.rowv[c * g.s_rowv + row] + g.colv[c * g.s_colv + col] - 2.f * f;
                f = g.gamma - sqrtf(fmaxf(d2, 0.f));
            }
            const unsigned long long m = __ballot(in && f > g.fpos[c * g.M + row]);
            const int cnt = __popcll(lane < 32 ? (m & 0xffffffffull) : (m >> 32));
            if ((lane & 31) == 0 && gm < g.M && cnt > 0) atomicAdd(&g.rank[c * g.M + gm], cnt);
            continue;
        }
        if (gm >= g.M || !col_in(j)) continue;  // (ComplEx: the two lanes of a coordinate stay or go together)
        const int bi = c * g.M + gm;  // index of the positive in the mini-batch (chain epilogues)
        float s = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) s += lds[ww][0][e];
        float rs = 0.f;
        if (WANT_ASUM) {
#pragma unroll
            for (int ww = 0; ww < NW; ++ww) rs += lds[ww][1][i];
        }
        if (EPI == EPI_PLAIN) {
            C[(int64_t)gm * g.ldc + gn] = (IS_FWD && g.out_mode == OUT_W) ? w_and_loss<true>(s, g.wk, loss) : s;
        } else if (EPI == EPI_L2_FWD) {
            const float d2 = g.rowv[c * g.s_rowv + gm] + g.colv[c * g.s_colv + gn] - 2.f * s;
            const float d = sqrtf(fmaxf(d2, 0.f));
            float out = g.out_mode == OUT_DIST ? d : g.gamma - d;
            if (g.out_mode == OUT_W) {  // W = w sigmoid(f) / |o - n|, 0 where the distance is 0
                const float coef = w_and_loss<true>(g.gamma - d, g.wk, loss);
                out = d > 0.f ? coef * __builtin_amdgcn_rcpf(d) : 0.f;
            }
            C[(int64_t)gm * g.ldc + gn] = out;
        } else if (EPI == EPI_L2_DO || EPI == EPI_L2_DN) {
            const float xv = g.X[c * g.sX + (int64_t)gm * g.ldx + gn];
            C[(int64_t)gm * g.ldc + gn] = s - rs * xv;
        } else if (EPI == EPI_CHAIN_L2) {
            // dL/do = W n - rowsum(W) o  +  dL/df+ * d(gamma - |o - c|)/do
            const float dir = (e_o[it] - e_c[it]) * e_inv[it];
            const float go = s - rs * e_o[it] - e_cp[it] * dir;
            g.Gent[(int64_t)(e_head ? g.b + bi : bi) * g.D + gn] = go;
            g.Gent[(int64_t)(e_head ? bi : g.b + bi) * g.D + gn] = e_cp[it] * dir;
            g.Grel[(int64_t)bi * g.D + gn] = e_head ? -go : go;
        } else if (CX) {
            // o = a (r_re + i r_i) with r_i = -r_im when the head is corrupted; psi = o . x over the [re | im] rows.
            // With go = dL/do: the kept entity gets go * conj(r_re + i r_i), the relation go * conj(a) (imaginary
            // part negated for the head side), the replaced entity dL/df+ * o.  The other part of the coordinate is
            // 16 lanes away.
            const bool im = j >= TILE / 2;
            const int d = col_of(j);
            const float go = s + e_cp[it] * e_c[it];
            const float go_p = __shfl_xor(go, TILE / 2, 64), r_p = __shfl_xor(e_r[it], TILE / 2, 64);
            const float a_p = __shfl_xor(e_a[it], TILE / 2, 64);
            const float sgn = e_head ? -1.f : 1.f;
            // re lane: g_re r_re + g_im r_i,  g_re a_re + g_im a_im
            // im lane: g_im r_re - g_re r_i,  sgn (g_im a_re - g_re a_im)
            const float ga = im ? go * r_p - go_p * (sgn * e_r[it]) : go * e_r[it] + go_p * (sgn * r_p);
            const float gr = im ? sgn * (go * a_p - go_p * e_a[it]) : go * e_a[it] + go_p * a_p;
            g.Gent[(int64_t)(e_head ? g.b + bi : bi) * g.D + d] = ga;
            g.Gent[(int64_t)(e_head ? bi : g.b + bi) * g.D + d] = e_cp[it] * e_o[it];
            g.Grel[(int64_t)bi * g.D + d] = gr;
        } else {  // EPI_CHAIN_DM: o = a * r, psi = o . x
            const float go = s + e_cp[it] * e_c[it];
            g.Gent[(int64_t)(e_head ? g.b + bi : bi) * g.D + gn] = go * e_r[it];
            g.Gent[(int64_t)(e_head ? bi : g.b + bi) * g.D + gn] = e_cp[it] * e_o[it];
            g.Grel[(int64_t)bi * g.D + gn] = go * e_a[it];
        }
    }
    if (IS_FWD && g.out_mode == OUT_W) {
        // negative part of the loss: this tile's sum of w softplus(f-), in a fixed order
        loss = wave_sum(loss);
        __syncthreads();  // the partial tiles in LDS have been read
        if (lane == 0) lds[w][1][0] = loss;
        __syncthreads();
        if (threadIdx.x == 0) {
            float t = 0.f;
#pragma unroll
            for (int ww = 0; ww < NW; ++ww) t += lds[ww][1][0];
            g.neg_loss_part[tile] = t * g.wk;
        }
    }
}

template <int NW, int EPI>
__global__ __launch_bounds__(NW * 64) void k_gemm_fwd(GemmArgs g) {
    __shared__ __attribute__((aligned(16))) float lds[NW][2][REGION];
    const int tile = xcd_tile(blockIdx.x >> 3, gridDim.x >> 3);
    if (tile >= g.tiles) return;
    gemm_tile<NW, true, true, EPI, false>(g, tile, lds);
}

// The tiles with the longer K loop first (dN: K is the chunk size; dO: K is the number of corrupting rows per chunk),
// then the others; each XCD gets its share of both.
// Held to 128 registers so that four waves fit on every SIMD (two 8-wave workgroups per CU): all tiles of the
// Freebase-scale step are then resident at once instead of running in two rounds.
template <int NW, int EPI_O, int EPI_N>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_gemm_bwd(GemmArgs gO, GemmArgs gN, int per_xcd_n, int per_xcd_o) {
    __shared__ __attribute__((aligned(16))) float lds[NW][2][REGION];
    const int per_xcd = per_xcd_n + per_xcd_o;
    int q = blockIdx.x >> 3;
    if (gO.K > gN.K) q = q < per_xcd_o ? q + per_xcd_n : q - per_xcd_o;  // dO tiles first
    if (q < per_xcd_n) {
        const int tile = xcd_tile(q, per_xcd_n);
        if (tile < gN.tiles) gemm_tile<NW, false, false, EPI_N, false>(gN, tile, lds);
    } else if (q < per_xcd) {
        const int tile = xcd_tile(q - per_xcd_n, per_xcd_o);
        if (tile < gO.tiles) gemm_tile<NW, true, false, EPI_O, true>(gO, tile, lds);
    }
}

// One plain product per batch item, operands found as IND says (the TransR products).
template <int NW, bool A_KC, bool B_KC, int IND>
__global__ __launch_bounds__(NW * 64) void k_gemm_one(GemmArgs g) {
    __shared__ __attribute__((aligned(16))) float lds[NW][2][REGION];
    const int tile = xcd_tile(blockIdx.x >> 3, gridDim.x >> 3);
    if (tile >= g.tiles) return;
    gemm_tile<NW, A_KC, B_KC, EPI_PLAIN, false, IND>(g, tile, lds);
}

// Number of K-splitting waves per tile.  With few tiles every K-block gets its own wave (one round of memory
// latency, all SIMDs of the CU busy); with thousands of tiles four waves per tile keep the cross-wave sum cheap.
int pick_nw(int tiles, int nblk, int cap) {
    if (tiles >= 1024) return 4;
    int nw = 4;
    while (nw < cap && nw < nblk) nw *= 2;
    return nw;
}

void set_tiling(GemmArgs& g, int chunks, bool coordinate_tiles = false) {
    g.gx = (g.N + TILE - 1) / TILE;
    if (coordinate_tiles) g.gx = (g.N / 2 + TILE / 2 - 1) / (TILE / 2);  // EPI_CHAIN_CX: 16 complex coordinates per tile
    g.gy = (g.M + TILE - 1) / TILE;
    g.tiles = g.gx * g.gy * chunks;
}

template <int EPI>
void launch_fwd(kge_ctx* c, GemmArgs g, int chunks, hipStream_t st) {
    set_tiling(g, chunks);
    const dim3 grid(8 * ((g.tiles + 7) / 8));
    const int nw = pick_nw(g.tiles, (g.K + TILE - 1) / TILE, 16);
    if (nw == 4) KGE_LAUNCH(c, (k_gemm_fwd<4, EPI>), grid, dim3(256), 0, st, g);
    else if (nw == 8) KGE_LAUNCH(c, (k_gemm_fwd<8, EPI>), grid, dim3(512), 0, st, g);
    else KGE_LAUNCH(c, (k_gemm_fwd<16, EPI>), grid, dim3(1024), 0, st, g);
}

template <bool A_KC, bool B_KC, int IND>
void launch_one(kge_ctx* c, GemmArgs g, int items, hipStream_t st) {
    set_tiling(g, items);
    g.out_mode = OUT_SCORE;
    const dim3 grid(8 * ((g.tiles + 7) / 8));
    const int nblk = (IND == IND_CHUNK_SUM ? g.ind_g : 1) * ((g.K + TILE - 1) / TILE);
    int nw = pick_nw(g.tiles, nblk, IND == IND_CHUNK_SUM ? 16 : 8);
    // thousands of tiles with a short K loop (rows of 100 floats are 4 K-blocks): one wave per tile, which multiplies
    // all the blocks between the tile's set-up and its epilogue, and sixteen tiles share a CU (measured on the
    // FB15k-sized TransR step: 113 us per product against 117 with two waves per tile and 134 with four)
    if (g.tiles >= 1024 && nblk <= 8) nw = 1;
    if (nw == 1) KGE_LAUNCH(c, (k_gemm_one<1, A_KC, B_KC, IND>), grid, dim3(64), 0, st, g);
    else if (nw == 4) KGE_LAUNCH(c, (k_gemm_one<4, A_KC, B_KC, IND>), grid, dim3(256), 0, st, g);
    else if (nw == 8) KGE_LAUNCH(c, (k_gemm_one<8, A_KC, B_KC, IND>), grid, dim3(512), 0, st, g);
    else KGE_LAUNCH(c, (k_gemm_one<16, A_KC, B_KC, IND>), grid, dim3(1024), 0, st, g);
}

template <int EPI_O, int EPI_N>
void launch_bwd(kge_ctx* c, GemmArgs gO, GemmArgs gN, int chunks, hipStream_t st) {
    set_tiling(gO, chunks, EPI_O == EPI_CHAIN_CX);
    set_tiling(gN, chunks);
    const int per_n = (gN.tiles + 7) / 8, per_o = (gO.tiles + 7) / 8;
    const dim3 grid(8 * (per_n + per_o));
    const int nblk = ((gO.K > gN.K ? gO.K : gN.K) + TILE - 1) / TILE;
    // at most 8 waves: 74 KB of LDS per workgroup, so two workgroups share a CU
    const int nw = pick_nw(gO.tiles + gN.tiles, nblk, 8);
    if (nw == 4) KGE_LAUNCH(c, (k_gemm_bwd<4, EPI_O, EPI_N>), grid, dim3(256), 0, st, gO, gN, per_n, per_o);
    else KGE_LAUNCH(c, (k_gemm_bwd<8, EPI_O, EPI_N>), grid, dim3(512), 0, st, gO, gN, per_n, per_o);
}

}  // namespace

// S_c = O_c N_c^T with the model's epilogue.  out_mode: 0 the scores (kge_score path); 1 what the loss kernel wants
// (TransE-L2: the distances, else the scores); 2 the backward coefficients W of uniformly weighted negatives, with
// the tiles' loss sums in neg_loss_part (training steps without a loss kernel); 3 nothing is stored, the ranks of the
// positives are counted into c->rank_out (only where kge_gemm_forward_can_rank says so).
void kge_gemm_neg_score(kge_ctx* c, int b, int k, int gsz, float gamma, float* out, int ld_out, int out_mode,
                        hipStream_t st) {
    const int D = c->cfg.ent_dim;
    GemmArgs g = {};
    g.A = c->O; g.B = c->Nst; g.C = out;
    g.M = gsz; g.N = k; g.K = D;
    g.lda = D; g.ldb = D; g.ldc = ld_out;
    g.sA = (int64_t)gsz * D; g.sB = (int64_t)k * D; g.sC = (int64_t)gsz * ld_out;
    g.rowv = c->o_n2; g.colv = c->n_n2; g.s_rowv = gsz; g.s_colv = k;
    g.gamma = gamma; g.out_mode = out_mode;
    g.wk = 1.f / ((float)k * (float)b); g.neg_loss_part = c->neg_loss_part;
    g.fpos = c->fpos; g.rank = c->rank_out;
    const int chunks = b / gsz;
    const bool bf = c->cfg.gemm_input == 1;
    const int epi = c->cfg.model == KGE_TRANSE_L2 ? EPI_L2_FWD : EPI_PLAIN;
    if (bf) {  // the operands as the gather launch rounded them
        g.A = reinterpret_cast<const float*>(c->Obf); g.B = reinterpret_cast<const float*>(c->Nbf);
        g.lda = c->ld_bf; g.ldb = c->ld_bf;
        g.sA = (int64_t)gsz * c->ld_bf; g.sB = (int64_t)k * c->ld_bf;
        kge_gemm_bf_forward(c, &g, epi, chunks, st);
    }
    else if (epi == EPI_L2_FWD) launch_fwd<EPI_L2_FWD>(c, g, chunks, st);
    else launch_fwd<EPI_PLAIN>(c, g, chunks, st);
}

// Evaluation: can the forward launch count the ranks itself (out_mode 3) instead of storing the scores?
bool kge_gemm_forward_can_rank(const kge_ctx* c) { return c->cfg.gemm_input == 0; }

// Logistic loss with uniform negative weights: the forward launch stores W and the loss sums, and no loss kernel
// runs.  (The ranking loss couples a positive with all of its negatives, so it always takes the loss kernel.)
bool kge_gemm_backward_forms_w(const kge_ctx* c) {
    return c->cfg.adv_temperature == 0.f && c->cfg.loss == KGE_LOSS_LOGISTIC;
}
bool kge_gemm_backward_does_chain(const kge_ctx* c) {
    return c->cfg.model == KGE_TRANSE_L2 || c->cfg.model == KGE_DISTMULT ||
           (c->cfg.model == KGE_COMPLEX && c->cfg.gemm_input == 0);
}
int kge_gemm_loss_parts(const kge_ctx* c, int b, int k, int gsz) {
    const int k_tiles = (k + TILE - 1) / TILE;
    return kge_gemm_backward_forms_w(c) ? (b / gsz) * ((gsz + TILE - 1) / TILE) * k_tiles : 0;
}

// dO_c = W_c N_c (- rowsum(W) o)  and  dN_c = W_c^T O_c (- colsum(W) n) in one launch.  dN goes straight into the
// gradient rows of the corrupting entities (key positions 2b ..); dO goes through the chain rule into the
// gradient rows of the positives (TransE-L2, DistMult, ComplEx with fp32 operands) or into GO for k_chain.
void kge_gemm_neg_backward(kge_ctx* c, const float* E, const float* R, const StepIds& ids, int k, int gsz, float gamma,
                           hipStream_t st) {
    const int D = c->cfg.ent_dim, b = ids.b;
    const int chunks = b / gsz;
    const int model = c->cfg.model;
    GemmArgs g = {};
    g.A = c->S; g.B = c->Nst; g.C = c->GO;
    g.M = gsz; g.N = D; g.K = k;
    g.lda = c->ld_s; g.ldb = D; g.ldc = D;
    g.sA = (int64_t)gsz * c->ld_s; g.sB = (int64_t)k * D; g.sC = (int64_t)gsz * D;
    g.X = c->O; g.ldx = D; g.sX = (int64_t)gsz * D;
    g.gamma = gamma;
    g.ids = ids; g.E = E; g.R = R; g.cpos = c->cpos; g.inv_dpos = c->inv_dpos; g.Gent = c->Gent; g.Grel = c->Grel;
    g.b = b; g.D = D; g.n_ent = c->cfg.num_entities; g.n_rel = c->cfg.num_relations;

    GemmArgs q = g;
    q.A = c->S; q.B = c->O; q.C = c->Gent + (int64_t)2 * b * D;
    q.M = k; q.N = D; q.K = gsz;
    q.lda = c->ld_s; q.ldb = D; q.ldc = D;
    q.sA = (int64_t)gsz * c->ld_s; q.sB = (int64_t)gsz * D; q.sC = (int64_t)k * D;
    q.X = c->Nst; q.ldx = D; q.sX = (int64_t)k * D;

    const bool bf = c->cfg.gemm_input == 1;
    if (bf) {  // N_c and O_c (the B operands) and the rows of the dN correction term as bf16
        g.B = reinterpret_cast<const float*>(c->Nbf); g.ldb = c->ld_bf; g.sB = (int64_t)k * c->ld_bf;
        q.B = reinterpret_cast<const float*>(c->Obf); q.ldb = c->ld_bf; q.sB = (int64_t)gsz * c->ld_bf;
        q.X = reinterpret_cast<const float*>(c->Nbf); q.ldx = c->ld_bf; q.sX = (int64_t)k * c->ld_bf;
    }
#define KGE_BWD(EO, EN)                                                     \
    do {                                                                    \
        if (bf) kge_gemm_bf_backward(c, &g, &q, EO, EN, chunks, st);        \
        else launch_bwd<EO, EN>(c, g, q, chunks, st);                \
    } while (0)
    if (model == KGE_TRANSE_L2) KGE_BWD(EPI_CHAIN_L2, EPI_L2_DN);
    else if (model == KGE_DISTMULT) KGE_BWD(EPI_CHAIN_DM, EPI_PLAIN);
    else if (model == KGE_COMPLEX && !bf) launch_bwd<EPI_CHAIN_CX, EPI_PLAIN>(c, g, q, chunks, st);
    else KGE_BWD(EPI_PLAIN, EPI_PLAIN);
#undef KGE_BWD
}

// ---- TransR: f = gamma - |M_r h + r - M_r t|^2 (Table 1).  Every positive i has its own projection matrix M_i (D x D,
// behind the D numbers of r in its relation row), so the products are batched over positives:
//   P_i = N_c M_i^T   [k x D]  projections of the chunk's corrupting rows              (forward)
//   sum_i U_i M_i     [k x D]  with U_i = dL/dP_i, over the chunk's positives i: one product per chunk whose K range
//                              is the concatenation of the positives' D values -> gradient rows of the negatives
//   G_i = U_i^T N_c   [D x D]  the negatives' share of dL/dM_i
void kge_gemm_transr_project(kge_ctx* c, const float* R, const StepIds& ids, int k, int gsz, float* P, hipStream_t st) {
    const int D = c->cfg.ent_dim;
    GemmArgs g = {};
    g.A = c->Nst; g.B = R; g.C = P;
    g.M = k; g.N = D; g.K = D; g.lda = D; g.ldb = D; g.ldc = D;
    g.sA = (int64_t)k * D; g.sB = c->cfg.rel_dim; g.sC = (int64_t)k * D;
    g.ids = ids; g.n_rel = c->cfg.num_relations; g.ind_g = gsz; g.b_off = D;
    launch_one<true, true, IND_CHUNK_REL>(c, g, ids.b, st);
}

// dL/dn for the corrupting rows of every chunk in one product per chunk: sum over the chunk's positives i of U_i M_i,
// i.e. the K range is the concatenation of the positives' D values; out = the gradient rows of the corrupting entities.
void kge_gemm_transr_back_project_sum(kge_ctx* c, const float* R, const StepIds& ids, int k, int gsz, const float* U,
                                      float* out, hipStream_t st) {
    const int D = c->cfg.ent_dim;
    GemmArgs g = {};
    g.A = U; g.B = R; g.C = out;
    g.M = k; g.N = D; g.K = D; g.lda = D; g.ldb = D; g.ldc = D;
    g.sA = (int64_t)gsz * k * D; g.sA_item = (int64_t)k * D; g.sB = c->cfg.rel_dim; g.sC = (int64_t)k * D;
    g.ids = ids; g.n_rel = c->cfg.num_relations; g.ind_g = gsz; g.b_off = D;
    launch_one<true, false, IND_CHUNK_SUM>(c, g, ids.b / gsz, st);
}

void kge_gemm_transr_matrix_grad(kge_ctx* c, const StepIds& ids, int k, int gsz, const float* U, float* GM,
                                 hipStream_t st) {
    const int D = c->cfg.ent_dim;
    GemmArgs g = {};
    g.A = U; g.B = c->Nst; g.C = GM;
    g.M = D; g.N = D; g.K = k; g.lda = D; g.ldb = D; g.ldc = D;
    g.sA = (int64_t)k * D; g.sB = (int64_t)k * D; g.sC = (int64_t)D * D;
    g.ids = ids; g.n_rel = c->cfg.num_relations; g.ind_g = gsz;
    launch_one<false, false, IND_ITEM_CHUNK>(c, g, ids.b, st);
}
