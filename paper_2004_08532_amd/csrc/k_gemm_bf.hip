// The chunked negative-scoring products (Sec. 3.3 of the paper) and their backward with bf16 operands and fp32
// accumulation: S_c = O_c N_c^T, dO_c = W_c N_c, dN_c = W_c^T O_c with the same epilogues as the fp32 path.
//
// Shapes here are the large ones (thousands of positives and corrupting rows per step), where a 32x32 tile per
// workgroup pulls every operand row from L2 into a CU once per 32 columns of output and spends as long on the
// cross-wave sum of its K split as on the product.  A workgroup therefore owns a 64x64 output tile over the whole K
// range (no split over K, no cross-wave sum, half the pulls per output); its four waves hold one 32x32 quarter each.  Per K block of 64 the 256 threads load the two 64x64 operand blocks (whole
// cache lines per request, the next two blocks in flight while this one is multiplied) and lay them out in LDS as
// bf16, K-contiguous whatever their
// orientation in memory, so that every v_mfma_f32_32x32x16_bf16 operand is one 16-byte LDS read.  The o rows and the
// corrupting rows arrive as bf16 (the gather launch rounds them once); the coefficients W are fp32 in memory and are
// rounded here (the hardware's round-to-nearest-even conversion, two values per instruction).  Operands that are
// stored with K along rows ("MC": N_c in dO, W_c and O_c in dN) are transposed on the way: a thread loads the same
// four columns of two adjacent K rows and packs the pairs.  LDS is double-buffered: one workgroup barrier per K
// block.
#include "k_gemm_shared.h"

namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int BT = 64;            // output tile edge
constexpr int BK = 64;            // K block
constexpr int PITCH = BK;         // bf16 per LDS row: 128 bytes, eight 16-byte groups, permuted per row (lds_word)
constexpr int PITCH_W = PITCH / 2;
constexpr int THREADS = 256;

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// Position (in 4-byte words) of word `word` of tile row `row` in LDS.  A row is 128 bytes, i.e. all 32 banks; its
// eight groups of four words (one 16-byte MFMA operand each) are permuted by (row mod 8) xor (row / 8 mod 8).  The
// first term spreads the 16-byte reads and writes of eight consecutive rows at one K position over the banks, the
// second the transposing 4-byte writes of the MC operands, which hit rows four apart.  Measured with the bank-conflict
// counter on the 'large' configuration: forward launch 0 conflict cycles (9.2e5 with rows of 144 bytes and a
// permutation by row / 8 alone), backward launch 7.5e5 (2.6e6).
__device__ __forceinline__ int lds_word(int row, int word) {
    return row * PITCH_W + (word ^ (4 * ((row & 7) ^ ((row >> 3) & 7))));
}

__device__ __forceinline__ void lds_barrier() {  // orders LDS traffic only: global loads stay in flight across it
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Stages 64 (rows) x 64 (K) blocks of one operand: fp32 in memory -> registers -> bf16 in LDS as [row][k].
// Element (row, kk) of the operand lies at base[row * ld + kk] (KC) or base[kk * ld + row] (MC).  Everything
// outside the matrix (rows >= R, kk >= K) becomes 0.  Loads are unconditional, from clamped addresses, and masked
// afterwards.  16-byte loads may run past R or K up to the next multiple of 4, which the row pitch covers.
template <bool KC>
struct Stager {
    const float* base;
    const float* p;  // MC: row 0 at the thread's first column
    const float* pr[4];  // KC: start of the thread's four rows
    int ld, K, R;
    int r;           // KC: the first of the thread's four rows in the tile (the others follow at + 16); MC: its first
                     // row (of 4 consecutive ones)
    int k;           // KC: first of its 4 K values; MC: first of its two K pairs (2 * kp; the second is 32 + 2 * kp)
    bool okr[4];
    bool full;       // all 64 rows of the tile lie inside the matrix
    struct Reg { float4 v[4]; };
    // A block that lies inside the matrix as a whole (the common case) is loaded and stored without the clamps and
    // masks: they cost several times the instructions of the copy itself.
    __device__ __forceinline__ bool inside(int kb) const { return full && kb * BK + BK <= K; }
    // KC: 16 consecutive lanes read 256 consecutive bytes of one row (whole cache lines per request)
    __device__ __forceinline__ void init(const float* base_, int ld_, int r0, int R_, int K_, int t) {
        base = base_; ld = ld_; K = K_; R = R_;
        full = r0 + BT <= R_;
        if (KC) {
            r = t >> 4;
            k = 4 * (t & 15);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                okr[q] = r0 + r + 16 * q < R;
                pr[q] = base + (int64_t)(okr[q] ? r0 + r + 16 * q : 0) * ld;
            }
            p = base;
        } else {
            r = 4 * (t & 15);
            k = 2 * (t >> 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) okr[e] = r0 + r + e < R;
            p = base + (okr[0] ? r0 + r : 0);
        }
    }
    __device__ __forceinline__ void issue(int kb, Reg& rg) const {
        float4 (&reg)[4] = rg.v;
        const int k0 = kb * BK + k;
        if (inside(kb)) {
            if (KC) {
#pragma unroll
                for (int q = 0; q < 4; ++q) reg[q] = ld4(pr[q] + k0);
            } else {
                const float* b = p + (int64_t)k0 * ld;
                reg[0] = ld4(b);
                reg[1] = ld4(b + ld);
                reg[2] = ld4(b + 32 * ld);
                reg[3] = ld4(b + 33 * ld);
            }
            return;
        }
        if (KC) {
#pragma unroll
            for (int q = 0; q < 4; ++q) reg[q] = ld4(pr[q] + (k0 < K ? k0 : 0));
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int kk = k0 + (q >> 1) * 32 + (q & 1);
                reg[q] = ld4(kk < K ? p + (int64_t)kk * ld : base);
            }
        }
    }
    __device__ __forceinline__ void store(int kb, const Reg& rg, __bf16* lds) const {
        const float4 (&reg)[4] = rg.v;
        const int k0 = kb * BK + k;
        if (inside(kb)) {
            uint32_t* l32 = reinterpret_cast<uint32_t*>(lds);
            if (KC) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<uint2*>(l32 + lds_word(r + 16 * q, k >> 1)) =
                        make_uint2(pack2(reg[q].x, reg[q].y), pack2(reg[q].z, reg[q].w));
            } else {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const float4 lo = reg[2 * h], hi = reg[2 * h + 1];
                    l32[lds_word(r + 0, (k >> 1) + 16 * h)] = pack2(lo.x, hi.x);
                    l32[lds_word(r + 1, (k >> 1) + 16 * h)] = pack2(lo.y, hi.y);
                    l32[lds_word(r + 2, (k >> 1) + 16 * h)] = pack2(lo.z, hi.z);
                    l32[lds_word(r + 3, (k >> 1) + 16 * h)] = pack2(lo.w, hi.w);
                }
            }
            return;
        }
        if (KC) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float v[4] = {reg[q].x, reg[q].y, reg[q].z, reg[q].w};
                float m[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) m[e] = (okr[q] && k0 + e < K) ? v[e] : 0.f;
                *reinterpret_cast<uint2*>(reinterpret_cast<uint32_t*>(lds) + lds_word(r + 16 * q, k >> 1)) =
                    make_uint2(pack2(m[0], m[1]), pack2(m[2], m[3]));
            }
        } else {
            uint32_t* l32 = reinterpret_cast<uint32_t*>(lds);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int kk = k0 + 32 * h;
                const float lo[4] = {reg[2 * h].x, reg[2 * h].y, reg[2 * h].z, reg[2 * h].w};
                const float hi[4] = {reg[2 * h + 1].x, reg[2 * h + 1].y, reg[2 * h + 1].z, reg[2 * h + 1].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float a = (okr[e] && kk < K) ? lo[e] : 0.f;
                    const float b = (okr[e] && kk + 1 < K) ? hi[e] : 0.f;
                    l32[lds_word(r + e, (k >> 1) + 16 * h)] = pack2(a, b);
                }
            }
        }
    }
};

// The same for an operand that the gather launch has already rounded to bf16 (the o rows and the corrupting rows; row
// pitch a multiple of 8 elements): half the bytes from L2, no conversion.  KC: 8 consecutive lanes read the 128 bytes
// that a row has in the K block and copy them; MC: 16 consecutive lanes read 128 consecutive bytes of one K row, and the
// 16-bit halves of two adjacent K rows are interleaved.
template <bool KC>
struct StagerBF {
    const uint16_t* base;
    const uint16_t* p;
    const uint16_t* pr[2];
    int ld, K, R, r, k;
    bool okr[4];
    bool full;
    struct Reg { uint4 v[2]; };  // KC: two rows x 8 K values; MC: (v[0].xy, v[0].zw, v[1].xy, v[1].zw) = 4 K rows x 4 columns
    __device__ __forceinline__ bool inside(int kb) const { return full && kb * BK + BK <= K; }
    __device__ __forceinline__ void init(const float* base_, int ld_, int r0, int R_, int K_, int t) {
        base = reinterpret_cast<const uint16_t*>(base_); ld = ld_; K = K_; R = R_;
        full = r0 + BT <= R_;
        if (KC) {
            r = t >> 3;
            k = 8 * (t & 7);
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                okr[q] = r0 + r + 32 * q < R;
                pr[q] = base + (int64_t)(okr[q] ? r0 + r + 32 * q : 0) * ld;
            }
            p = base;
        } else {
            r = 4 * (t & 15);
            k = 2 * (t >> 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) okr[e] = r0 + r + e < R;
            p = base + (okr[0] ? r0 + r : 0);
        }
    }
    __device__ __forceinline__ void issue(int kb, Reg& rg) const {
        const int k0 = kb * BK + k;
        if (inside(kb)) {
            if (KC) {
#pragma unroll
                for (int q = 0; q < 2; ++q) rg.v[q] = *reinterpret_cast<const uint4*>(pr[q] + k0);
            } else {
                const uint16_t* b = p + (int64_t)k0 * ld;
                const uint2 x0 = *reinterpret_cast<const uint2*>(b), x1 = *reinterpret_cast<const uint2*>(b + ld);
                const uint2 x2 = *reinterpret_cast<const uint2*>(b + 32 * ld);
                const uint2 x3 = *reinterpret_cast<const uint2*>(b + 33 * ld);
                rg.v[0] = make_uint4(x0.x, x0.y, x1.x, x1.y);
                rg.v[1] = make_uint4(x2.x, x2.y, x3.x, x3.y);
            }
            return;
        }
        if (KC) {
#pragma unroll
            for (int q = 0; q < 2; ++q) rg.v[q] = *reinterpret_cast<const uint4*>(pr[q] + (k0 < K ? k0 : 0));
        } else {
            uint2 x[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int kk = k0 + (q >> 1) * 32 + (q & 1);
                x[q] = *reinterpret_cast<const uint2*>(kk < K ? p + (int64_t)kk * ld : base);
            }
            rg.v[0] = make_uint4(x[0].x, x[0].y, x[1].x, x[1].y);
            rg.v[1] = make_uint4(x[2].x, x[2].y, x[3].x, x[3].y);
        }
    }
    __device__ __forceinline__ void store(int kb, const Reg& rg, __bf16* lds) const {
        const int k0 = kb * BK + k;
        if (inside(kb)) {
            uint32_t* l32 = reinterpret_cast<uint32_t*>(lds);
            if (KC) {
#pragma unroll
                for (int q = 0; q < 2; ++q) *reinterpret_cast<uint4*>(l32 + lds_word(r + 32 * q, k >> 1)) = rg.v[q];
            } else {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    // lo: K row kk, hi: K row kk + 1; each holds columns (0, 1) in .x / .z and (2, 3) in .y / .w
                    const uint32_t lo01 = rg.v[h].x, lo23 = rg.v[h].y, hi01 = rg.v[h].z, hi23 = rg.v[h].w;
                    l32[lds_word(r + 0, (k >> 1) + 16 * h)] = (lo01 & 0xffffu) | (hi01 << 16);
                    l32[lds_word(r + 1, (k >> 1) + 16 * h)] = (lo01 >> 16) | (hi01 & 0xffff0000u);
                    l32[lds_word(r + 2, (k >> 1) + 16 * h)] = (lo23 & 0xffffu) | (hi23 << 16);
                    l32[lds_word(r + 3, (k >> 1) + 16 * h)] = (lo23 >> 16) | (hi23 & 0xffff0000u);
                }
            }
            return;
        }
        if (KC) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                // K is a multiple of 4, so a pair of values is inside the matrix or outside as a whole
                uint4 w = rg.v[q];
                w.x = (okr[q] && k0 < K) ? w.x : 0u;
                w.y = (okr[q] && k0 + 2 < K) ? w.y : 0u;
                w.z = (okr[q] && k0 + 4 < K) ? w.z : 0u;
                w.w = (okr[q] && k0 + 6 < K) ? w.w : 0u;
                *reinterpret_cast<uint4*>(reinterpret_cast<uint32_t*>(lds) + lds_word(r + 32 * q, k >> 1)) = w;
            }
        } else {
            uint32_t* l32 = reinterpret_cast<uint32_t*>(lds);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int kk = k0 + 32 * h;
                // lo: K row kk, hi: K row kk + 1; each holds columns (0, 1) in .x / .z and (2, 3) in .y / .w
                const uint32_t lo01 = rg.v[h].x, lo23 = rg.v[h].y, hi01 = rg.v[h].z, hi23 = rg.v[h].w;
                const uint32_t lo[4] = {lo01 & 0xffffu, lo01 >> 16, lo23 & 0xffffu, lo23 >> 16};
                const uint32_t hi[4] = {hi01 << 16, hi01 & 0xffff0000u, hi23 << 16, hi23 & 0xffff0000u};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t a = (okr[e] && kk < K) ? lo[e] : 0u;
                    const uint32_t b = (okr[e] && kk + 1 < K) ? hi[e] : 0u;
                    l32[lds_word(r + e, (k >> 1) + 16 * h)] = a | b;
                }
            }
        }
    }
};

template <bool KC, bool SRC_BF> struct StagerSel { typedef Stager<KC> type; };
template <bool KC> struct StagerSel<KC, true> { typedef StagerBF<KC> type; };

// One 64x64 output tile.  EPI as in the fp32 path.  A_KC / B_KC: orientation of the operands in memory; A_BF / B_BF:
// the operand is stored as bf16 (g.A / g.B then point at 16-bit elements, strides and pitches counted in elements).
template <bool A_KC, bool B_KC, int EPI, bool A_BF, bool B_BF>
__device__ __forceinline__ void bf_tile(const GemmArgs& g, int tile, __bf16 (*lds)[2][BT * PITCH]) {
    constexpr bool CHAIN = EPI == EPI_CHAIN_L2 || EPI == EPI_CHAIN_DM;
    constexpr bool WANT_ASUM = EPI == EPI_L2_DN || EPI == EPI_CHAIN_L2;
    constexpr bool IS_FWD = A_KC && B_KC;
    static_assert(EPI != EPI_L2_DO, "with bf16 operands dL/do of TransE-L2 goes through the chain-rule epilogue");
    const int t = threadIdx.x, w = t >> 6, lane = t & 63;
    const int n0 = (tile % g.gx) * BT, mt = (tile / g.gx) % g.gy, m0 = mt * BT, c = tile / (g.gx * g.gy);
    // (a bf16 operand: the pointer is to 2-byte elements, chunk strides are counted in elements)
    const float* A = A_BF ? reinterpret_cast<const float*>(reinterpret_cast<const uint16_t*>(g.A) + c * g.sA) : g.A + c * g.sA;
    const float* B = B_BF ? reinterpret_cast<const float*>(reinterpret_cast<const uint16_t*>(g.B) + c * g.sB) : g.B + c * g.sB;
    const int wm = 32 * (w >> 1), wn = 32 * (w & 1);  // this wave's quarter of the tile

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    // sum over K of the rounded A[row wm + lane % 32][.], this lane's half of the K values.  (Taking the row sums from
    // a second MFMA against a matrix of ones instead was measured: the extra matrix instructions cost more than these
    // conversions and additions.)
    float a_sum = 0.f;

    typedef typename StagerSel<A_KC, A_BF>::type SA;
    typedef typename StagerSel<B_KC, B_BF>::type SB;
    SA sa;
    SB sb;
    sa.init(A, g.lda, m0, g.M, g.K, t);
    sb.init(B, g.ldb, n0, g.N, g.K, t);
    const int nblk = (g.K + BK - 1) / BK, last = nblk - 1;
    // Two K blocks of loads are in flight: while block kb is multiplied, kb + 1 is on its way in one register set
    // and kb + 2 in the other.  Blocks past the end are clamped to the last one (loaded again, never stored) rather
    // than branched around.  (Measured and slower: the K range split over two groups of waves that add their partial
    // tiles at the end; four blocks of loads in flight; all eight operand reads of a block issued before its first
    // matrix instruction.  The last two cost registers, and the launch loses more from fewer resident waves than it
    // gains.)
    typename SA::Reg ra0, ra1;
    typename SB::Reg rb0, rb1;
    sa.issue(0, ra0);
    sb.issue(0, rb0);
    sa.issue(1 < nblk ? 1 : last, ra1);
    sb.issue(1 < nblk ? 1 : last, rb1);
    auto multiply = [&](const __bf16* As, const __bf16* Bs) {
        // lane feeds row (column) lane % 32 of its quarter and K values 16 s + 8 (lane / 32) .. + 7 of MFMA s
        const uint32_t* a32 = reinterpret_cast<const uint32_t*>(As);
        const uint32_t* b32 = reinterpret_cast<const uint32_t*>(Bs);
        const int ra = wm + (lane & 31), rb = wn + (lane & 31), w0 = 4 * (lane >> 5);
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            const bf16x8 pa = *reinterpret_cast<const bf16x8*>(a32 + lds_word(ra, w0 + 8 * s));
            const bf16x8 pb = *reinterpret_cast<const bf16x8*>(b32 + lds_word(rb, w0 + 8 * s));
            if (WANT_ASUM && (w & 1) == 0) {  // the two waves of a row block hold the same A rows: one of them sums
#pragma unroll
                for (int e = 0; e < 8; ++e) a_sum += (float)pa[e];
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa, pb, acc, 0, 0, 0);
        }
    };
    for (int kb = 0; kb < nblk; kb += 2) {
        sa.store(kb, ra0, lds[0][0]);
        sb.store(kb, rb0, lds[0][1]);
        sa.issue(kb + 2 < nblk ? kb + 2 : last, ra0);
        sb.issue(kb + 2 < nblk ? kb + 2 : last, rb0);
        lds_barrier();
        multiply(lds[0][0], lds[0][1]);
        if (kb + 1 >= nblk) break;
        sa.store(kb + 1, ra1, lds[1][0]);
        sb.store(kb + 1, rb1, lds[1][1]);
        sa.issue(kb + 3 < nblk ? kb + 3 : last, ra1);
        sb.issue(kb + 3 < nblk ? kb + 3 : last, rb1);
        lds_barrier();
        multiply(lds[1][0], lds[1][1]);
    }

    // ---- epilogue, straight from the accumulators: register v of lane l holds C[8 (v/4) + 4 (l/32) + v%4][l%32]
    // of the wave's quarter
    float* rs_lds = reinterpret_cast<float*>(lds[0][0]) + 32 * (w >> 1);  // row sums of A for the quarter's 32 rows
    if (WANT_ASUM) {
        a_sum += __shfl_xor(a_sum, 32, 64);
        lds_barrier();  // every wave is done reading the operand blocks
        if (lane < 32 && (w & 1) == 0) rs_lds[lane] = a_sum;
        lds_barrier();
    }
    StepView sv;
    bool head = false;
    if (CHAIN) {
        sv = step_view(g.ids);
        head = sv.side == KGE_NEG_HEAD;
    }
    float* C = g.C + c * g.sC;
    float loss = 0.f;
    const int gn = n0 + wn + (lane & 31);
    const int gnc = gn < g.N ? gn : g.N - 1;
    // Everything the epilogue reads is fetched before its first store: a lane has 16 elements, and a load that follows
    // a store which may alias it cannot be moved up by the compiler, so loads written next to their stores would be 16
    // dependent round trips (table rows: to HBM) instead of one.  Addresses of elements outside the matrix are clamped.
    auto row_of = [&](int v) { return m0 + wm + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); };
    float in0[16], in1[16], in2[16], in3[16];
    if (EPI == EPI_L2_FWD) {
        const float cv = g.colv[c * g.s_colv + gnc];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int gm = row_of(v) < g.M ? row_of(v) : g.M - 1;
            in0[v] = g.rowv[c * g.s_rowv + gm] + cv;
        }
    } else if (EPI == EPI_L2_DN) {
        // the rows of the correction term are the bf16 rows that went into the products
        const uint16_t* xb = reinterpret_cast<const uint16_t*>(g.X) + c * g.sX + gnc;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int gm = row_of(v) < g.M ? row_of(v) : g.M - 1;
            in0[v] = __builtin_bit_cast(float, (uint32_t)xb[(int64_t)gm * g.ldx] << 16);
        }
    } else if (CHAIN) {
        int64_t cid[16], aid[16], rid[16];  // the replaced entity; DistMult: also the kept entity and the relation
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int bi = c * g.M + (row_of(v) < g.M ? row_of(v) : g.M - 1);
            const int64_t hid = clamp_id(sv.h[bi], g.n_ent), tid = clamp_id(sv.t[bi], g.n_ent);
            cid[v] = head ? hid : tid;
            aid[v] = head ? tid : hid;
            rid[v] = EPI == EPI_CHAIN_DM ? clamp_id(sv.r[bi], g.n_rel) : 0;
        }
        float in4[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int bi = c * g.M + (row_of(v) < g.M ? row_of(v) : g.M - 1);
            in0[v] = g.X[(int64_t)bi * g.ldx + gnc];   // o
            in1[v] = g.E[cid[v] * g.D + gnc];           // the replaced entity's row
            in2[v] = g.cpos[bi];                        // dL/df+
            if (EPI == EPI_CHAIN_L2) {
                in3[v] = g.inv_dpos[bi];
            } else {
                in3[v] = g.E[aid[v] * g.D + gnc];       // the kept entity's row
                in4[v] = g.R[rid[v] * g.D + gnc];       // the relation's row
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int gm = row_of(v);
            if (gm >= g.M || gn >= g.N) continue;
            const float s = acc[v];
            const float rs = WANT_ASUM ? rs_lds[8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)] : 0.f;
            const int bi = c * g.M + gm;  // index of the positive in the mini-batch
            const float e_o = in0[v], e_c = in1[v], e_cp = in2[v];
            float* ga = g.Gent + (int64_t)(head ? g.b + bi : bi) * g.D + gn;
            float* gc = g.Gent + (int64_t)(head ? bi : g.b + bi) * g.D + gn;
            float* gr = g.Grel + (int64_t)bi * g.D + gn;
            if (EPI == EPI_CHAIN_L2) {
                // dL/do = W n - rowsum(W) o  +  dL/df+ * d(gamma - |o - c|)/do
                const float dir = (e_o - e_c) * in3[v];
                const float go = s - rs * round_bf16(e_o) - e_cp * dir;
                *ga = go;
                *gc = e_cp * dir;
                *gr = head ? -go : go;
            } else {  // EPI_CHAIN_DM: o = a * r, psi = o . x
                const float go = s + e_cp * e_c;
                *ga = go * in4[v];
                *gc = e_cp * e_o;
                *gr = go * in3[v];
            }
        }
    }
    if (!CHAIN) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int gm = row_of(v);
            if (gm >= g.M || gn >= g.N) continue;
            const float s = acc[v];
            const float rs = WANT_ASUM ? rs_lds[8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)] : 0.f;
            if (EPI == EPI_PLAIN) {
                C[(int64_t)gm * g.ldc + gn] = (IS_FWD && g.out_mode == OUT_W) ? w_and_loss<false>(s, g.wk, loss) : s;
            } else if (EPI == EPI_L2_FWD) {
                const float d2 = in0[v] - 2.f * s;
                const float d = __builtin_amdgcn_sqrtf(fmaxf(d2, 0.f));  // 1 ulp
                float out = g.out_mode == OUT_DIST ? d : g.gamma - d;
                if (g.out_mode == OUT_W) {  // W = w sigmoid(f) / |o - n|, 0 where the distance is 0
                    const float coef = w_and_loss<false>(g.gamma - d, g.wk, loss);
                    out = d > 0.f ? coef * rcp_refined(d) : 0.f;
                }
                C[(int64_t)gm * g.ldc + gn] = out;
            } else {  // EPI_L2_DN
                C[(int64_t)gm * g.ldc + gn] = s - rs * in0[v];
            }
        }
    }
    if (IS_FWD && g.out_mode == OUT_W) {
        // negative part of the loss, one sum per 32x32 quarter that lies inside the matrix, indexed as the 32x32
        // tiling of the fp32 path indexes its tiles
        loss = wave_sum(loss);
        const int q_m = (m0 + wm) / 32, q_n = (n0 + wn) / 32;
        const int qx = (g.N + 31) / 32, qy = (g.M + 31) / 32;
        if (lane == 0 && m0 + wm < g.M && n0 + wn < g.N) g.neg_loss_part[(c * qy + q_m) * qx + q_n] = loss * g.wk;
    }
}

template <int EPI>
__global__ __launch_bounds__(THREADS) void k_gemm_bf_fwd(GemmArgs g) {
    __shared__ __attribute__((aligned(16))) __bf16 lds[2][2][BT * PITCH];  // [buffer][operand]
    const int tile = xcd_tile(blockIdx.x >> 3, gridDim.x >> 3);
    if (tile >= g.tiles) return;
    bf_tile<true, true, EPI, true, true>(g, tile, lds);
}

// dO tiles first: their K is the number of corrupting rows per chunk, the longer loop at these shapes
template <int EPI_O, int EPI_N>
__global__ __launch_bounds__(THREADS) void k_gemm_bf_bwd(GemmArgs gO, GemmArgs gN, int per_xcd_o, int per_xcd_n) {
    __shared__ __attribute__((aligned(16))) __bf16 lds[2][2][BT * PITCH];  // [buffer][operand]
    const int q = blockIdx.x >> 3;
    if (q < per_xcd_o) {
        const int tile = xcd_tile(q, per_xcd_o);
        if (tile < gO.tiles) bf_tile<true, false, EPI_O, false, true>(gO, tile, lds);
    } else {
        const int tile = xcd_tile(q - per_xcd_o, per_xcd_n);
        if (tile < gN.tiles) bf_tile<false, false, EPI_N, false, true>(gN, tile, lds);
    }
}

void set_tiling(GemmArgs& g, int chunks) {
    g.gx = (g.N + BT - 1) / BT;
    g.gy = (g.M + BT - 1) / BT;
    g.tiles = g.gx * g.gy * chunks;
}

template <int EPI_O, int EPI_N>
void launch_bwd(kge_ctx* c, GemmArgs gO, GemmArgs gN, int chunks, hipStream_t st) {
    set_tiling(gO, chunks);
    set_tiling(gN, chunks);
    const int per_o = (gO.tiles + 7) / 8, per_n = (gN.tiles + 7) / 8;
    KGE_LAUNCH(c, (k_gemm_bf_bwd<EPI_O, EPI_N>), dim3(8 * (per_o + per_n)), dim3(THREADS), 0, st, gO, gN, per_o, per_n);
}

}  // namespace

void kge_gemm_bf_forward(kge_ctx* c, const void* args, int epi, int chunks, hipStream_t st) {
    GemmArgs g = *static_cast<const GemmArgs*>(args);
    set_tiling(g, chunks);
    const dim3 grid(8 * ((g.tiles + 7) / 8));
    if (epi == EPI_L2_FWD) KGE_LAUNCH(c, k_gemm_bf_fwd<EPI_L2_FWD>, grid, dim3(THREADS), 0, st, g);
    else KGE_LAUNCH(c, k_gemm_bf_fwd<EPI_PLAIN>, grid, dim3(THREADS), 0, st, g);
}

void kge_gemm_bf_backward(kge_ctx* c, const void* args_o, const void* args_n, int epi_o, int epi_n, int chunks,
                          hipStream_t st) {
    const GemmArgs gO = *static_cast<const GemmArgs*>(args_o), gN = *static_cast<const GemmArgs*>(args_n);
    if (epi_o == EPI_CHAIN_L2 && epi_n == EPI_L2_DN) launch_bwd<EPI_CHAIN_L2, EPI_L2_DN>(c, gO, gN, chunks, st);
    else if (epi_o == EPI_CHAIN_DM && epi_n == EPI_PLAIN) launch_bwd<EPI_CHAIN_DM, EPI_PLAIN>(c, gO, gN, chunks, st);
    else launch_bwd<EPI_PLAIN, EPI_PLAIN>(c, gO, gN, chunks, st);
}
