// Internal declarations shared by the HIP sources of libkge (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kge.h"

// ---------------------------------------------------------------------------------------------------------
// Context.  All device buffers are carved out of one allocation made in kge_create.
//
// Notation (paper Sec. 3.3): b positives per mini-batch, groups ("chunks") of g positives, C = b / g chunks,
// k corrupting entities per chunk, D floats per entity row.  For every positive i the library forms
//     o_i = phi(a_i, r_i)      a_i = the entity that is NOT corrupted (head for tail corruption, else tail)
// so that the score of (i, any replacement x) is psi(o_i, x); this is the split of Sec. 3.3
// (TransE: o = h + r, psi = gamma - |o - x|) carried over to the other models and to head corruption.
// ---------------------------------------------------------------------------------------------------------
struct kge_ctx {
    kge_config cfg;
    float eps;
    int ld_s;            // row pitch of S / W in floats (max_neg_per_chunk rounded up to 4)
    int max_neg_rows;    // max_chunks * max_neg_per_chunk
    int max_ent_keys;    // 2 * max_batch + max_neg_rows
    int ent_key_bits, rel_key_bits;

    void* ws_base;
    int64_t ws_bytes;

    float* O;        // [max_batch x D]      o_i
    float* Nst;      // [max_neg_rows x D]   gathered corrupting rows, chunk after chunk
    float* S;        // [max_batch x ld_s]   negative scores, then backward coefficients W
    float* GO;       // [max_batch x D]      dL/do_i
    float* Gent;     // [max_ent_keys x D]   gradient rows in key order: heads | tails | corrupting rows
    float* Grel;     // [max_batch x Dr]     gradient rows of the relations
    float* fpos;     // [max_batch]          positive scores
    float* o_n2;     // [max_batch]          |o_i|^2          (TransE-L2)
    float* n_n2;     // [max_neg_rows]       |n_j|^2          (TransE-L2)
    float* cpos;     // [max_batch]          dL/df+_i
    float* row_loss; // [max_batch]          loss terms of positive i, already divided by b
    float* w_rowsum; // [max_batch]          sum_j W_ij       (TransE-L2)
    uint16_t* Obf;   // bf16 copies of O, Nst, W (gemm_input = 1)
    uint16_t* Nbf;
    uint16_t* Wbf;
    uint32_t* ekey[2];  // entity sort ping-pong: keys
    uint32_t* epos[2];  //                        positions in the key list
    uint32_t* rkey[2];  // relation sort ping-pong
    uint32_t* rpos[2];
    int* flags;         // [0]: an id was out of range

    int ebuf, rbuf;                 // which ping-pong half holds the sorted result
    int64_t last_ent_keys, last_rel_keys;  // sizes of the last train step's key lists (0: none yet)
    hipStream_t side_stream;        // runs the key sort beside the forward/backward kernels
    hipEvent_t ev_fork, ev_join;
    bool prof_on;                   // kge_profile: bracket every kernel with events
    hipEvent_t prof_ev[KGE_PROF_SLOTS][2];
    double prof_ms[KGE_PROF_SLOTS];
    int64_t prof_steps;
    char err[512];
};

// ---------------------------------------------------------------------------------------------------------
// Host-side launchers (each in the source file named after its kernel group)
// ---------------------------------------------------------------------------------------------------------
// a1/a2: gather rows, o_i, positive scores, norms
void kge_launch_gather(kge_ctx* c, const float* E, const float* R, const int64_t* h, const int64_t* r,
                       const int64_t* t, int b, const int64_t* neg, int n_neg, int side, float gamma,
                       float* pos_out, hipStream_t st);
// a3: negative scores of every chunk into out[b x ld_out]: matrix-product models / elementwise-reduce models
void kge_gemm_neg_score(kge_ctx* c, int b, int k, int g, float gamma, float* out, int ld_out, int dist_mode,
                        hipStream_t st);
void kge_pair_neg_score(kge_ctx* c, int b, int k, int g, float gamma, float* out, int ld_out, hipStream_t st);
// a4: loss terms and backward coefficients (in place over S)
void kge_launch_loss(kge_ctx* c, int b, int k, float gamma, hipStream_t st);
// a5: dL/do and the gradient rows of the corrupting entities
void kge_gemm_neg_backward(kge_ctx* c, int b, int k, int g, hipStream_t st);
void kge_pair_neg_backward(kge_ctx* c, int b, int k, int g, hipStream_t st);
// a5: positive-pair term and chain rule through phi -> gradient rows of heads, tails and relations
void kge_launch_chain(kge_ctx* c, const float* E, const float* R, const int64_t* h, const int64_t* r,
                      const int64_t* t, int b, int side, float gamma, hipStream_t st);
// a6: sort (id, position) of the entity and relation key lists
void kge_launch_sort(kge_ctx* c, const int64_t* h, const int64_t* r, const int64_t* t, int b,
                     const int64_t* neg, int n_neg, hipStream_t st);
// a7: per distinct row, sum its gradient rows and apply Adagrad; also reduces the loss terms
void kge_launch_update(kge_ctx* c, float* E, float* SE, float* R, float* SR, int n_ent_keys, int n_rel_keys,
                       float lr, int b, float* loss_out, hipStream_t st);
// test hook: distinct ids and multiplicities from the sorted keys
void kge_launch_dedup_export(kge_ctx* c, int which, int64_t* uniq, int32_t* count, int64_t* n_unique,
                             hipStream_t st);

// ---------------------------------------------------------------------------------------------------------
// Device helpers
// ---------------------------------------------------------------------------------------------------------
#ifdef __HIPCC__
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ float4 f4(float x) { return make_float4(x, x, x, x); }

// round-to-nearest-even fp32 -> bf16 bits
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) return (uint16_t)(u >> 16);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
#endif
