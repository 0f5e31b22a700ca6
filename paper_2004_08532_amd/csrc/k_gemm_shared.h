// Shared by the two matrix-product sources (k_gemm.hip: fp32 operands, small tiles split over K; k_gemm_bf.hip:
// bf16 operands, 64x64 tiles): the argument block, the epilogue kinds and the helpers both use.
#pragma once
#include "kge_common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

enum { EPI_PLAIN = 0, EPI_L2_FWD = 1, EPI_L2_DO = 2, EPI_L2_DN = 3, EPI_CHAIN_L2 = 4, EPI_CHAIN_DM = 5, EPI_CHAIN_CX = 6 };
// what the forward launch leaves behind (see kge_gemm_neg_score); OUT_RANK: nothing but the ranks of the positives
enum { OUT_SCORE = 0, OUT_DIST = 1, OUT_W = 2, OUT_RANK = 3 };

struct GemmArgs {
    const float* A;
    const float* B;
    float* C;
    int M, N, K;
    int lda, ldb, ldc;
    int64_t sA, sB, sC;  // chunk strides (floats)
    const float* rowv;   // EPI_L2_FWD: |o|^2 per row (chunk stride s_rowv)
    const float* colv;   // EPI_L2_FWD: |n|^2 per column (chunk stride s_colv)
    int64_t s_rowv, s_colv;
    const float* X;      // [M x ldx] operand of the TransE-L2 correction term (o rows for dO, n rows for dN)
    int ldx;
    int64_t sX;
    float gamma;
    int out_mode;        // forward: OUT_SCORE, OUT_DIST (TransE-L2: the distance) or OUT_W (backward coefficients)
    int gx, gy, tiles;   // tiles along N, along M, and in total (over all chunks); set by the launchers
    // A-operand transform (uniform negative weights): W = wk * sigmoid(f) [/ distance]
    float wk;            // 1 / (k b)
    float* neg_loss_part;  // [forward tiles] OUT_W: sum of wk * softplus(f-) over the tile
    const float* fpos;     // OUT_RANK: scores of the positives
    int32_t* rank;         // OUT_RANK: [b], set to 1 beforehand; gets + #{j : f-_ij > f+_i}
    // chain-rule epilogues
    StepIds ids;
    const float* E;
    const float* R;
    const float* cpos;
    const float* inv_dpos;
    float* Gent;
    float* Grel;
    int b, D;
    int64_t n_ent, n_rel;
    // batches whose items are positives rather than chunks (TransR: every positive has its own projection matrix)
    int ind_g;       // positives per chunk: item i uses chunk i / ind_g of the operand that is stored per chunk
    int64_t sA_item; // IND_CHUNK_SUM: floats from one positive's A block to the next one's
    int64_t b_off;   // offset of the matrix inside a relation row
};
// how the operands of batch item i are found (IND of gemm_tile)
enum { IND_NONE = 0,      // A + i sA, B + i sB
       IND_CHUNK_REL = 1, // A + (i / ind_g) sA (per chunk), B + r_i sB + b_off (the positive's relation row)
       IND_ITEM_CHUNK = 2, // A + i sA,                       B + (i / ind_g) sB
       // batch item = chunk c; the K range is the concatenation, over the chunk's ind_g positives p, of their K values:
       // A + c sA + p sA_item, B + r_(c ind_g + p) sB + b_off; K counts one positive's share
       IND_CHUNK_SUM = 3
};

__device__ __forceinline__ int64_t clamp_id(int64_t id, int64_t n) { return id < 0 ? 0 : (id >= n ? n - 1 : id); }

// Backward coefficient of a negative score f with uniform weight wk: wk * sigmoid(f) = d/df [wk softplus(f)];
// adds softplus(f) to loss.  Runs once per score, in the forward epilogue.  FAST: the hardware exp2 / log2 /
// reciprocal (1 ulp each; about 1e-6 relative in W, the size of the rounding of the fp32 products W goes into).
// With bf16 operands W is rounded to bf16 afterwards, and which neighbour a value rounds to should not hinge on
// those last bits.  That path keeps the hardware functions (a library exp, log1p and two divisions per score cost
// about as much as the whole K loop of a 64x64 tile) and repairs what matters for W: the product |f| * log2(e) is
// split into its rounded value and the rounding error, so that the error of exp does not grow with |f|, and the
// reciprocal gets one Newton step.  W is then good to about 2 ulp; the loss term only needs 1e-5.
__device__ __forceinline__ float rcp_refined(float a) {
    const float r = __builtin_amdgcn_rcpf(a);
    return fmaf(fmaf(-a, r, 1.f), r, r);
}
template <bool FAST>
__device__ __forceinline__ float w_and_loss(float f, float wk, float& loss) {
    if (FAST) {
        const float e = __builtin_amdgcn_exp2f(-fabsf(f) * 1.4426950408889634f);  // exp(-|f|) in (0, 1]
        loss += fmaxf(f, 0.f) + __builtin_amdgcn_logf(1.f + e) * 0.6931471805599453f;
        return wk * ((f >= 0.f ? 1.f : e) * __builtin_amdgcn_rcpf(1.f + e));
    }
    const float x = -fabsf(f);
    const float y = x * 1.44269502162933349609375f;  // log2(e) rounded to fp32 ...
    const float yl = fmaf(x, 1.44269502162933349609375f, -y) + x * 1.92596299112661746e-8f;  // ... and what is lost
    float e = __builtin_amdgcn_exp2f(y);
    e = fmaf(e, yl * 0.6931471805599453f, e);  // e * 2^yl
    loss += fmaxf(f, 0.f) + __builtin_amdgcn_logf(1.f + e) * 0.6931471805599453f;
    return wk * ((f >= 0.f ? 1.f : e) * rcp_refined(1.f + e));
}

// Workgroups are handed to the 8 XCDs round-robin by linear id, and every XCD has its own L2.  Each XCD gets a
// contiguous range of tiles (row-major, column tiles fastest), so the tiles that share an A row-block run on one
// XCD and re-read it from that L2 instead of from memory.  q = index of the workgroup within its XCD.
__device__ __forceinline__ int xcd_tile(int q, int per_xcd) { return (blockIdx.x & 7) * per_xcd + q; }

}  // namespace

// bf16 operands (k_gemm_bf.hip): the same two launches on 64x64 tiles
void kge_gemm_bf_forward(kge_ctx* c, const void* args, int epi, int chunks, hipStream_t st);
void kge_gemm_bf_backward(kge_ctx* c, const void* args_o, const void* args_n, int epi_o, int epi_n, int chunks,
                          hipStream_t st);
