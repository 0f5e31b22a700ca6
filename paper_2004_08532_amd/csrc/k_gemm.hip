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
// region (coalesced 16-byte global loads, no workgroup barrier in the main loop), feeds
// v_mfma_f32_32x32x2_f32, and the NW partial tiles are summed through LDS in a fixed order at the end, so
// results do not depend on scheduling.  Operands may be stored K-contiguous ("KC": [rows][K]) or
// row-contiguous ("MC": [K][rows]); both are read from memory as they lie, no transposed copies are made.
#include "kge_common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

enum { EPI_PLAIN = 0, EPI_L2_FWD = 1, EPI_MINUS_ROWV_X = 2, EPI_MINUS_AROWSUM_X = 3 };

struct GemmArgs {
    const float* A;
    const float* B;
    float* C;
    int M, N, K;
    int lda, ldb, ldc;
    int64_t sA, sB, sC;  // chunk strides (floats)
    const float* rowv;   // indexed by m (per chunk stride s_rowv)
    const float* colv;   // indexed by n (per chunk stride s_colv)
    int64_t s_rowv, s_colv;
    const float* X;      // [M x ldx] correction operand
    int ldx;
    int64_t sX;
    float gamma;
    int store_dist;      // EPI_L2_FWD: store the distance instead of gamma - distance
    int gx, gy, tiles;   // tiles along N, along M, and in total (over all chunks); set by launch()
};

constexpr int TILE = 32;
constexpr int KC_PITCH = 36;                 // floats; 16-byte aligned rows, conflict-free 128-bit reads
constexpr int REGION = TILE * KC_PITCH;      // floats per staged operand block

// Loads 32x32 blocks of one operand into registers (zero-filled outside the matrix).  The per-lane row pointers
// and edge masks are set up once; a block load is then four 16-byte loads and a few selects.
// KC: element (row, kk) at base[(r0 + row) * ld + k0 + kk]; lane covers row = lane/8 + 8*it, kk = 4*(lane%8)..+3
// MC: element (row, kk) at base[(k0 + kk) * ld + r0 + row]; lane covers kk = lane/8 + 8*it, row = 4*(lane%8)..+3
template <bool KC>
struct BlockLoader {
    const float* p[4];  // KC: start of the lane's row; MC: row (lane/8 + 8*it) of K-block 0 at the lane's column
    bool ok[4];         // KC: the lane's row exists; MC: unused
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
            const int gr = r0 + minor;
            any = gr < rows; m1 = gr + 1 < rows; m2 = gr + 2 < rows; m3 = gr + 3 < rows;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                ok[it] = true;
                p[it] = base + (int64_t)(major0 + 8 * it) * ld + (any ? gr : 0);
            }
        }
    }
    // Branch-free: the four loads are issued unconditionally (from a clamped, always valid address) and masked
    // afterwards, so that all of them, and those of the other operand, are in flight together.
    __device__ __forceinline__ void load(int kb, float4 (&reg)[4]) const {
        const int k0 = kb * 32;
        if (KC) {
            const int gk = k0 + minor;
            const bool kin = gk < K;
            const int koff = kin ? gk : 0;  // the first 16 bytes of a row are always there
#pragma unroll
            for (int it = 0; it < 4; ++it) reg[it] = ld4(p[it] + koff);
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const bool v0 = ok[it] && kin;
                reg[it].x = v0 ? reg[it].x : 0.f;
                reg[it].y = (v0 && gk + 1 < K) ? reg[it].y : 0.f;
                reg[it].z = (v0 && gk + 2 < K) ? reg[it].z : 0.f;
                reg[it].w = (v0 && gk + 3 < K) ? reg[it].w : 0.f;
            }
        } else {
            bool kin[4];
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                kin[it] = k0 + major0 + 8 * it < K;
                reg[it] = ld4(kin[it] ? p[it] + (int64_t)k0 * ld : p0_safe);
            }
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const bool v0 = any && kin[it];
                reg[it].x = v0 ? reg[it].x : 0.f;
                reg[it].y = (v0 && m1) ? reg[it].y : 0.f;
                reg[it].z = (v0 && m2) ? reg[it].z : 0.f;
                reg[it].w = (v0 && m3) ? reg[it].w : 0.f;
            }
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

template <int NW, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(NW * 64) void k_gemm_f32(GemmArgs g) {
    __shared__ __attribute__((aligned(16))) float lds[NW][2][REGION];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // Workgroups are handed to the 8 XCDs round-robin by linear id, and every XCD has its own L2.  Give each XCD
    // a contiguous range of tiles (row-major, column tiles fastest) so that the tiles that share an A row-block
    // run on one XCD and re-read it from that L2 instead of from memory.
    const int per_xcd = gridDim.x >> 3;
    const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= g.tiles) return;
    const int n0 = (tile % g.gx) * TILE, m0 = ((tile / g.gx) % g.gy) * TILE, c = tile / (g.gx * g.gy);
    const float* A = g.A + c * g.sA;
    const float* B = g.B + c * g.sB;
    float* As = lds[w][0];
    float* Bs = lds[w][1];

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    float a_sum = 0.f;  // EPI_MINUS_AROWSUM_X: sum over this lane's K-values of A[m = lane%32][.]

    const int nblk = (g.K + TILE - 1) / TILE;
    float4 ra[4], rb[4];
    BlockLoader<A_KC> la;
    BlockLoader<B_KC> lb;
    la.init(A, g.lda, m0, g.M, g.K, lane);
    lb.init(B, g.ldb, n0, g.N, g.K, lane);
    int kb = w;
    if (kb < nblk) {
        la.load(kb, ra);
        lb.load(kb, rb);
    }
    while (kb < nblk) {
        lds_store<A_KC>(As, lane, ra);
        lds_store<B_KC>(Bs, lane, rb);
        const int nxt = kb + NW;
        if (nxt < nblk) {  // next block's global loads fly while this block is multiplied
            la.load(nxt, ra);
            lb.load(nxt, rb);
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
                if (EPI == EPI_MINUS_AROWSUM_X) a_sum += fa[t];
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
    if (EPI == EPI_MINUS_AROWSUM_X) {
        a_sum += __shfl_xor(a_sum, 32, 64);
        if (lane < 32) Bs[lane] = a_sum;
    }
    __syncthreads();
    float* C = g.C + c * g.sC;
    for (int e = threadIdx.x; e < TILE * TILE; e += NW * 64) {
        const int i = e >> 5, j = e & 31;
        const int gm = m0 + i, gn = n0 + j;
        if (gm >= g.M || gn >= g.N) continue;
        float s = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) s += lds[ww][0][e];
        float out = s;
        if (EPI == EPI_L2_FWD) {
            const float d2 = g.rowv[c * g.s_rowv + gm] + g.colv[c * g.s_colv + gn] - 2.f * s;
            const float d = sqrtf(fmaxf(d2, 0.f));
            out = g.store_dist ? d : g.gamma - d;
        } else if (EPI == EPI_MINUS_ROWV_X) {
            out = s - g.rowv[c * g.s_rowv + gm] * g.X[c * g.sX + (int64_t)gm * g.ldx + gn];
        } else if (EPI == EPI_MINUS_AROWSUM_X) {
            float rs = 0.f;
#pragma unroll
            for (int ww = 0; ww < NW; ++ww) rs += lds[ww][1][i];
            out = s - rs * g.X[c * g.sX + (int64_t)gm * g.ldx + gn];
        }
        C[(int64_t)gm * g.ldc + gn] = out;
    }
}

// Number of K-splitting waves per tile.  With few tiles every K-block gets its own wave (one round of memory
// latency, all SIMDs of the CU busy); with thousands of tiles four waves per tile keep the cross-wave sum cheap.
int pick_nw(int tiles, int nblk) {
    if (tiles >= 1024) return 4;
    int nw = 4;
    while (nw < 16 && nw < nblk) nw *= 2;
    return nw;
}

template <bool A_KC, bool B_KC, int EPI>
void launch(GemmArgs g, int chunks, hipStream_t st) {
    g.gx = (g.N + TILE - 1) / TILE;
    g.gy = (g.M + TILE - 1) / TILE;
    g.tiles = g.gx * g.gy * chunks;
    const dim3 grid(8 * ((g.tiles + 7) / 8));
    const int nblk = (g.K + TILE - 1) / TILE;
    const int nw = pick_nw(g.tiles, nblk);
    if (nw == 4) hipLaunchKernelGGL((k_gemm_f32<4, A_KC, B_KC, EPI>), grid, dim3(256), 0, st, g);
    else if (nw == 8) hipLaunchKernelGGL((k_gemm_f32<8, A_KC, B_KC, EPI>), grid, dim3(512), 0, st, g);
    else hipLaunchKernelGGL((k_gemm_f32<16, A_KC, B_KC, EPI>), grid, dim3(1024), 0, st, g);
}

}  // namespace

// S_c = O_c N_c^T with the model's epilogue.  dist_mode: TransE-L2 stores the distance (training path) instead
// of the score (kge_score path).
void kge_gemm_neg_score(kge_ctx* c, int b, int k, int gsz, float gamma, float* out, int ld_out, int dist_mode,
                        hipStream_t st) {
    const int D = c->cfg.ent_dim;
    GemmArgs g = {};
    g.A = c->O; g.B = c->Nst; g.C = out;
    g.M = gsz; g.N = k; g.K = D;
    g.lda = D; g.ldb = D; g.ldc = ld_out;
    g.sA = (int64_t)gsz * D; g.sB = (int64_t)k * D; g.sC = (int64_t)gsz * ld_out;
    g.rowv = c->o_n2; g.colv = c->n_n2; g.s_rowv = gsz; g.s_colv = k;
    g.gamma = gamma; g.store_dist = dist_mode;
    const int chunks = b / gsz;
    if (c->cfg.model == KGE_TRANSE_L2) launch<true, true, EPI_L2_FWD>(g, chunks, st);
    else launch<true, true, EPI_PLAIN>(g, chunks, st);
}

// dO_c = W_c N_c (- rowsum(W) o)  and  dN_c = W_c^T O_c (- colsum(W) n), the latter straight into the gradient
// rows of the corrupting entities (key positions 2b ..).
void kge_gemm_neg_backward(kge_ctx* c, int b, int k, int gsz, hipStream_t st) {
    const int D = c->cfg.ent_dim;
    const int chunks = b / gsz;
    const bool l2 = c->cfg.model == KGE_TRANSE_L2;
    GemmArgs g = {};
    g.A = c->S; g.B = c->Nst; g.C = c->GO;
    g.M = gsz; g.N = D; g.K = k;
    g.lda = c->ld_s; g.ldb = D; g.ldc = D;
    g.sA = (int64_t)gsz * c->ld_s; g.sB = (int64_t)k * D; g.sC = (int64_t)gsz * D;
    g.rowv = c->w_rowsum; g.s_rowv = gsz;
    g.X = c->O; g.ldx = D; g.sX = (int64_t)gsz * D;
    if (l2) launch<true, false, EPI_MINUS_ROWV_X>(g, chunks, st);
    else launch<true, false, EPI_PLAIN>(g, chunks, st);

    GemmArgs q = {};
    q.A = c->S; q.B = c->O; q.C = c->Gent + (int64_t)2 * b * D;
    q.M = k; q.N = D; q.K = gsz;
    q.lda = c->ld_s; q.ldb = D; q.ldc = D;
    q.sA = (int64_t)gsz * c->ld_s; q.sB = (int64_t)gsz * D; q.sC = (int64_t)k * D;
    q.X = c->Nst; q.ldx = D; q.sX = (int64_t)k * D;
    if (l2) launch<false, false, EPI_MINUS_AROWSUM_X>(q, chunks, st);
    else launch<false, false, EPI_PLAIN>(q, chunks, st);
}
