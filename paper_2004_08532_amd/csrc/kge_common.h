// Internal declarations shared by the HIP sources of libkge (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kge.h"
#include <hip/hip_ext.h>

// ---------------------------------------------------------------------------------------------------------
// Context.  All device buffers are carved out of one allocation made in kge_create.
//
// Notation (paper Sec. 3.3): b positives per mini-batch, groups ("chunks") of g positives, C = b / g chunks,
// k corrupting entities per chunk, D floats per entity row.  For every positive i the library forms
//     o_i = phi(a_i, r_i)      a_i = the entity that is NOT corrupted (head for tail corruption, else tail)
// so that the score of (i, any replacement x) is psi(o_i, x); this is the split of Sec. 3.3
// (TransE: o = h + r, psi = gamma - |o - x|) carried over to the other models and to head corruption.
// ---------------------------------------------------------------------------------------------------------
// Gradient rows that exist as `parts` partial rows, `stride` floats apart, still to be added up (in order) into out.
struct PartialRows {
    const float* src;
    float* out;
    int parts;       // 0 or 1: nothing to add up
    int64_t stride;
    int64_t n4;      // 16-byte pieces per partial
};

struct StepBlock;

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
    uint16_t* Obf;   // bf16 operands only: o_i and the corrupting rows rounded to bf16, row pitch ld_bf (the products
    uint16_t* Nbf;   // read these; Nst is then not written)
    int ld_bf;       // D rounded up to 64 (rows of whole 128-byte lines)
    float* S;        // [max_batch x ld_s]   negative scores, then backward coefficients W
    float* PP;       // TransR: [max_batch x D] p_i = M_i c_i
    float* P3;       // TransR: [max_batch x max_neg_per_chunk x D] projections of the corrupting rows, then dL/dP
    float* GO;       // [max_batch x D]      dL/do_i
    float* pair_part_o;  // RotatE / TransE-L1: [KGE_PAIR_MAX_PARTS][max_batch x D] partial dL/do rows of the tiled backward
    PartialRows go_partial, neg_partial;  // what the last backward launch left for the chain launch to add up
    float* pair_part_n;  //                     [KGE_PAIR_MAX_PARTS][max_neg_rows x D] partial rows of the corrupting entities
    float* Gent;     // [max_ent_keys x D]   gradient rows in key order: heads | tails | corrupting rows
    float* Grel;     // [max_batch x Dr]     gradient rows of the relations
    float* fpos;     // [max_batch]          positive scores
    float* o_n2;     // [max_batch]          |o_i|^2          (TransE-L2)
    float* n_n2;     // [max_neg_rows]       |n_j|^2          (TransE-L2)
    float* cpos;     // [max_batch]          dL/df+_i
    float* row_loss; // [max_batch]          loss terms of positive i, already divided by b
    float* inv_dpos; // [max_batch]          1 / |o_i - c_i|  (TransE-L2)
    float* neg_loss_part;  // [forward tiles]  negative-side loss sums written by the forward launch
    uint32_t* ekey[2];  // entity sort ping-pong: keys
    uint32_t* epos[2];  //                        positions in the key list
    uint32_t* rkey[2];  // relation sort ping-pong
    uint32_t* rpos[2];
    int* flags;         // [0]: an id was out of range
    int32_t* rank_out;  // kge_rank: where the running call wants the ranks (the gather launch sets them to 1, the
                        // forward launch counts); null otherwise

    int ebuf, rbuf;                 // which ping-pong half holds the sorted result
    uint32_t* sort_counts;          // radix sort: digit counts / offsets, [slices of both lists][16 waves][256]
    int64_t last_ent_keys, last_rel_keys;  // sizes of the last train step's key lists (0: none yet)
    hipStream_t side_stream;        // runs the key sort beside the forward/backward kernels
    hipEvent_t ev_fork, ev_join;
    StepBlock* step_block;          // device: id arrays and step counter of the running kge_train_steps call
    int32_t* sides_dev;             // device: per-step sides of the running call, KGE_SIDES_CAP entries
    void* replay;                   // cached graphs of kge_train_steps (ReplayCache in kge_api.hip)
    int64_t graph_captures;         // how many times they were built
    bool prof_on;                   // kge_profile: bracket every kernel with events
    hipEvent_t prof_ev[KGE_PROF_SLOTS][2];
    double prof_ms[KGE_PROF_SLOTS];
    int64_t prof_steps;
    hipEvent_t launch_ev0, launch_ev1;  // set by a profiling scope: the next KGE_LAUNCH takes its own start/stop
                                        // timestamps into them
    char err[512];
};

// Kernel launch.  While profiling, the launch carries a start and a stop event that receive the dispatch's own
// begin / end timestamps (the ones a kernel trace shows), not the time at which a marker between kernels was
// processed.  One timed launch per profiling scope.
#define KGE_LAUNCH(c, kernel, grid, block, lds, st, ...)                                                            \
    do {                                                                                                            \
        if ((c)->launch_ev0) {                                                                                      \
            hipExtLaunchKernelGGL(kernel, grid, block, lds, st, (c)->launch_ev0, (c)->launch_ev1, 0, __VA_ARGS__);  \
            (c)->launch_ev0 = nullptr;                                                                              \
            (c)->launch_ev1 = nullptr;                                                                              \
        } else {                                                                                                    \
            hipLaunchKernelGGL(kernel, grid, block, lds, st, __VA_ARGS__);                                          \
        }                                                                                                           \
    } while (0)

// ---------------------------------------------------------------------------------------------------------
// The ids of one step, as the kernels receive them.
// Direct mode: blk == nullptr and h, r, t, neg point at this step's ids, side and loss_out are this step's.
// Replay mode (one captured HIP graph serves every step of every kge_train_steps call of the same shape): blk points
// at a block in the workspace that a one-thread kernel fills at the start of every call with the call's id arrays
// (ids of its step 0; consecutive steps lie b (n_neg) entries apart), its per-step sides (may be null: tail
// corruption throughout) and its loss array (one float per step, may be null), and whose step counter the last
// kernel of every step advances.  The graphs hold only the block's address, so new id arrays need no new capture.
// ---------------------------------------------------------------------------------------------------------
struct StepBlock {
    int64_t step;
    const int64_t* h;
    const int64_t* r;
    const int64_t* t;
    const int64_t* neg;
    const int32_t* sides;
    float* loss_out;
};

struct StepIds {
    const int64_t* h;
    const int64_t* r;
    const int64_t* t;
    const int64_t* neg;
    int b, n_neg, side;
    StepBlock* blk;
    float* loss_out;
};

// A key list of the duplicate reduction: the concatenation of up to three id arrays (entities: heads | tails |
// corrupting ids; relations: r), to be brought into (id, position) order.
struct KeyList {
    const int64_t* src[3];   // direct mode
    int n_src[3];
    const StepBlock* blk;    // replay mode: the arrays come from the block (which == 0: h | t | neg, 1: r)
    int which;
    int n;                   // total number of keys
    int passes;              // radix passes needed for ids < n_ids (8 bits each)
    int64_t n_ids;           // ids are clamped into [0, n_ids)
    uint32_t* key[2];        // sorted ids (ping-pong halves; the rank path writes half 0)
    uint32_t* pos[2];        // position in the key list of each sorted entry
};
void kge_make_key_lists(kge_ctx* c, const StepIds& ids, KeyList* ent, KeyList* rel);

// ---------------------------------------------------------------------------------------------------------
// Host-side launchers (each in the source file named after its kernel group)
// ---------------------------------------------------------------------------------------------------------
// a1/a2: gather rows, o_i, positive scores, norms
// with_keys: the same launch also brings the key lists into (id, position) order (lists of up to
// KGE_RANK_MAX_KEYS keys; longer lists go through kge_launch_sort)
void kge_launch_gather(kge_ctx* c, const float* E, const float* R, const StepIds& ids, float gamma, float* pos_out,
                       bool with_keys, hipStream_t st);
constexpr int KGE_SIDES_CAP = 65536;  // steps whose sides fit the workspace: longer kge_train_steps calls run in segments
constexpr int KGE_SORT_SLICE = 4096;  // keys per workgroup of the radix sort of long key lists
constexpr int KGE_PAIR_MAX_PARTS = 8;  // partial rows per gradient row in the tiled backward of RotatE / TransE-L1
constexpr int KGE_RANK_MAX_KEYS = 14336;  // 14 * 1024: positions fit 14 bits, the list and its tables fit 64 KB of LDS
// a3: negative scores of every chunk into out[b x ld_out]: matrix-product models / elementwise-reduce models
void kge_gemm_neg_score(kge_ctx* c, int b, int k, int g, float gamma, float* out, int ld_out, int dist_mode,
                        hipStream_t st);
void kge_pair_neg_score(kge_ctx* c, int b, int k, int g, float gamma, float* out, int ld_out, hipStream_t st);
// a4: loss terms and backward coefficients (in place over S)
void kge_launch_loss(kge_ctx* c, int b, int k, float gamma, hipStream_t st);
// a5: dL/do and the gradient rows of the corrupting entities
void kge_gemm_neg_backward(kge_ctx* c, const float* E, const float* R, const StepIds& ids, int k, int g, float gamma,
                           hipStream_t st);
bool kge_gemm_forward_can_rank(const kge_ctx* c);  // evaluation without storing the scores (fp32 products)
bool kge_gemm_backward_forms_w(const kge_ctx* c);     // the forward launch stores W and the loss sums (no k_loss)
bool kge_gemm_backward_does_chain(const kge_ctx* c);  // the backward launch writes the positives' gradient rows
int kge_gemm_loss_parts(const kge_ctx* c, int b, int k, int g);  // loss sums the forward launch leaves in neg_loss_part
void kge_pair_neg_backward(kge_ctx* c, int b, int k, int g, hipStream_t st);
// a5: positive-pair term and chain rule through phi -> gradient rows of heads, tails and relations
void kge_launch_chain(kge_ctx* c, const float* E, const float* R, const StepIds& ids, hipStream_t st);
// RESCAL: o_i from the kept entity and the relation's matrix (before the gather launch); chain rule through it
void kge_launch_rescal_phi(kge_ctx* c, const float* E, const float* R, const StepIds& ids, hipStream_t st);
void kge_launch_rescal_chain(kge_ctx* c, const float* E, const float* R, const StepIds& ids, hipStream_t st);
// RESCAL, a7 for the relation matrices: gradient of a distinct relation formed from the factor rows, then Adagrad
void kge_launch_rescal_update(kge_ctx* c, float* R, float* SR, const StepIds& ids, float lr, hipStream_t st);
// TransR: the steps around its batched products (k_transr.hip) and the products (k_gemm.hip)
void kge_transr_phi(kge_ctx* c, const float* E, const float* R, const StepIds& ids, float gamma, float* pos_out,
                    hipStream_t st);
void kge_transr_score(kge_ctx* c, const StepIds& ids, int k, float gamma, float* out, int ld_out, hipStream_t st);
void kge_transr_dp(kge_ctx* c, const StepIds& ids, int k, hipStream_t st);
void kge_transr_chain(kge_ctx* c, const float* E, const float* R, const StepIds& ids, hipStream_t st);
void kge_transr_update(kge_ctx* c, float* R, float* SR, const StepIds& ids, float lr, hipStream_t st);
float* kge_transr_projections(kge_ctx* c);
float* kge_transr_matrix_grads(kge_ctx* c);
void kge_gemm_transr_project(kge_ctx* c, const float* R, const StepIds& ids, int k, int g, float* P, hipStream_t st);
void kge_gemm_transr_back_project_sum(kge_ctx* c, const float* R, const StepIds& ids, int k, int g, const float* U,
                                      float* out, hipStream_t st);
void kge_gemm_transr_matrix_grad(kge_ctx* c, const StepIds& ids, int k, int g, const float* U, float* GM,
                                 hipStream_t st);
// a6: sort (id, position) of the entity and relation key lists
void kge_launch_sort(kge_ctx* c, const StepIds& ids, hipStream_t st);
// a7: per distinct row, sum its gradient rows and apply Adagrad; also reduces the loss terms
void kge_launch_update(kge_ctx* c, float* E, float* SE, float* R, float* SR, const StepIds& ids, float lr,
                       int n_loss_parts, hipStream_t st);
// evaluation: ranks of the positives among their negatives (from fpos and the scores in S), and the metrics
void kge_launch_rank(kge_ctx* c, int b, int k, int32_t* rank_out, hipStream_t st);
void kge_launch_rank_metrics(const int32_t* ranks, int64_t n, double* out, hipStream_t st);
// step 1: ids of a range of steps from the counter-based generator
int kge_sample_launch(const kge_sampler* s, int64_t first_step, int64_t n_steps, int64_t* h, int64_t* r, int64_t* t,
                      int64_t* neg, int32_t* sides, hipStream_t st);
// test hook: distinct ids and multiplicities from the sorted keys
void kge_launch_dedup_export(kge_ctx* c, int which, int64_t* uniq, int32_t* count, int64_t* n_unique,
                             hipStream_t st);

// ---------------------------------------------------------------------------------------------------------
// Device helpers
// ---------------------------------------------------------------------------------------------------------
#ifdef __HIPCC__
struct StepView {
    const int64_t* h;
    const int64_t* r;
    const int64_t* t;
    const int64_t* neg;
    int side;
    int64_t step;
};
__device__ __forceinline__ StepView step_view(const StepIds& s) {
    StepView v;
    if (s.blk) {
        const StepBlock* k = s.blk;  // uniform address: these are scalar loads of one cache line
        v.step = k->step;
        v.h = k->h + v.step * s.b;
        v.r = k->r + v.step * s.b;
        v.t = k->t + v.step * s.b;
        v.neg = k->neg + v.step * s.n_neg;
        const int32_t* sides = k->sides;
        v.side = sides ? sides[v.step] : KGE_NEG_TAIL;
    } else {
        v.step = 0;
        v.h = s.h; v.r = s.r; v.t = s.t; v.neg = s.neg;
        v.side = s.side;
    }
    return v;
}
// The (up to three) id arrays of a key list for the running step.
struct KeySources { const int64_t* p[3]; };
__device__ __forceinline__ KeySources key_sources(const KeyList& l) {
    KeySources s;
    if (l.blk) {
        const StepBlock* k = l.blk;
        const int64_t step = k->step;
        if (l.which == 0) {
            s.p[0] = k->h + step * l.n_src[0];
            s.p[1] = k->t + step * l.n_src[1];
            s.p[2] = k->neg + step * l.n_src[2];
        } else {
            s.p[0] = s.p[1] = s.p[2] = k->r + step * l.n_src[0];
        }
    } else {
        s.p[0] = l.src[0]; s.p[1] = l.src[1]; s.p[2] = l.src[2];
    }
    return s;
}
// Address of entry idx of a key list (branch-free, so that a thread can have many of these loads in flight).
__device__ __forceinline__ const int64_t* key_address(const KeyList& l, const KeySources& s, int idx) {
    const int a = l.n_src[0], ab = a + l.n_src[1];
    const int64_t* p0 = s.p[0] + idx;
    const int64_t* p1 = s.p[1] + (idx - a);
    const int64_t* p2 = s.p[2] + (idx - ab);
    return idx < a ? p0 : (idx < ab ? p1 : p2);
}
__device__ __forceinline__ uint32_t clamp_key(const KeyList& l, int64_t id) {
    id = id < 0 ? 0 : (id >= l.n_ids ? l.n_ids - 1 : id);
    return (uint32_t)id;
}
__device__ __forceinline__ uint32_t fetch_key(const KeyList& l, int idx) {
    return clamp_key(l, *key_address(l, key_sources(l), idx));
}
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

// Adagrad: S += g^2 ; x -= lr * g / (sqrt(S) + eps), with the hardware square root and reciprocal (1 ulp each): the
// update is a step of size <= lr, so their 1e-7 relative error is far below the accuracy of g itself.
__device__ __forceinline__ float adagrad1(float g, float& s, float lr, float eps) {
    s = fmaf(g, g, s);
    return lr * g * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(s) + eps);
}
__device__ __forceinline__ void adagrad4(float4 g, float4& x, float4& s, float lr, float eps) {
    x.x -= adagrad1(g.x, s.x, lr, eps);
    x.y -= adagrad1(g.y, s.y, lr, eps);
    x.z -= adagrad1(g.z, s.z, lr, eps);
    x.w -= adagrad1(g.w, s.w, lr, eps);
}

// fp32 -> bf16 -> fp32, round to nearest even (the hardware conversion of gfx950)
__device__ __forceinline__ float round_bf16(float x) { return (float)(__bf16)x; }
#endif
