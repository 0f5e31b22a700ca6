/*
 * kge.h -- C ABI of libkge: one mini-batch step of knowledge-graph-embedding training on one AMD MI355X.
 *
 * The step is steps 2-4 of the mini-batch loop of the DGL-KE paper (arXiv 2004.08532, Sec. 3.1): fetch the
 * embedding rows a mini-batch touches, run the forward and backward computation on them, and apply the
 * optimizer to exactly those rows of the global tables.  Positives and the jointly sampled corrupting entities
 * (Sec. 3.3) arrive as id arrays; they may be the caller's own or come from kge_sample_steps (step 1 of the loop).
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer on the context's device unless it is marked (host).  Tables,
 *     optimizer state, id arrays and outputs are owned by the caller and must stay alive and unmodified
 *     until the stream has finished the work the call enqueued.  The library owns only its workspace, which
 *     is allocated in kge_create and never grows; no other entry point allocates device memory (the first
 *     kge_train_steps call of a shape creates HIP graph objects, see there).
 *   - Calls that take a stream ENQUEUE work and return; they do not synchronise.
 *   - Return value: KGE_OK (0) or a negative kge_status.  When an error is detected on the host nothing has
 *     been enqueued and no caller memory has been touched.  No C++ exception crosses this boundary.
 *   - Tables are row-major, contiguous fp32, rows of ent_dim (rel_dim) floats, 16-byte aligned.
 *   - A context is bound to one device and is not re-entrant: use it from one thread and one stream at a
 *     time.
 */
#ifndef KGE_H
#define KGE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kge_ctx kge_ctx; /* opaque */

/* Score functions of Table 1 of the paper.  Distance models are used as f = gamma - distance; DistMult and
 * ComplEx ignore gamma.  TransE-L2 uses the un-squared norm (Table 1, Sec. 3.3).  RotatE is
 * gamma - sum_j |h_j r_j - t_j| over complex coordinates.  Rows of ComplEx / RotatE entities (and ComplEx
 * relations) are [real parts | imaginary parts]; a RotatE relation row holds ent_dim/2 phases in radians. */
typedef enum {
    KGE_TRANSE_L2 = 0,
    KGE_TRANSE_L1 = 1,
    KGE_DISTMULT = 2,
    KGE_COMPLEX = 3,
    KGE_ROTATE = 4,
    KGE_RESCAL = 5, /* h^T M_r t: a relation row is the ent_dim x ent_dim matrix M_r, row by row */
    KGE_TRANSR = 6  /* gamma - |M_r h + r - M_r t|^2 (squared, as Table 1 prints it): a relation row is the
                       translation r (ent_dim floats) followed by the ent_dim x ent_dim matrix M_r, row by row */
} kge_model;

/* Which entity of each positive is replaced to form its negatives (Sec. 2: only entities are corrupted). */
typedef enum { KGE_NEG_TAIL = 0, KGE_NEG_HEAD = 1 } kge_neg_side;

/* The two training losses of Sec. 2.  With b positives, k negatives per positive and weights w_ij (see
 * adv_temperature):
 *   logistic:  L = (1/b) sum_i [ log(1 + exp(-f+_i)) + sum_j w_ij log(1 + exp(f-_ij)) ]
 *   ranking:   L = (1/b) sum_i sum_j w_ij max(0, gamma - f+_i + f-_ij)      (gamma of the call is the margin; the
 *              gamma inside the distance scores cancels in f- - f+; sub-gradient 0 at the kink) */
typedef enum { KGE_LOSS_LOGISTIC = 0, KGE_LOSS_RANKING = 1 } kge_loss;

typedef enum {
    KGE_OK = 0,
    KGE_ERR_INVALID_ARG = -1, /* null pointer, size out of range, b not a multiple of chunk, bad enum   */
    KGE_ERR_UNSUPPORTED = -2, /* a combination this build does not implement                             */
    KGE_ERR_WORKSPACE = -3,   /* b, k or b/chunk exceed what the context was created for                 */
    KGE_ERR_DEVICE = -4,      /* a HIP call failed; kge_last_error has the text                          */
    KGE_ERR_INDEX_RANGE = -5  /* validate_indices found an id outside its table                          */
} kge_status;

typedef struct {
    int32_t model;             /* kge_model                                                               */
    int32_t device;            /* HIP device ordinal                                                      */
    int64_t num_entities;      /* rows of the entity table   (< 2^32)                                     */
    int64_t num_relations;     /* rows of the relation table (< 2^32)                                     */
    int32_t ent_dim;           /* floats per entity row: multiple of 4 (8 for ComplEx / RotatE), <= 1024  */
    int32_t rel_dim;           /* floats per relation row: ent_dim; ent_dim/2 for RotatE; ent_dim^2 for   */
                               /* RESCAL; ent_dim + ent_dim^2 for TransR                                  */
    int32_t max_batch;         /* largest b a call may pass                                               */
    int32_t max_neg_per_chunk; /* largest k                                                               */
    int32_t max_chunks;        /* largest b / chunk                                                       */
    int32_t gemm_input;        /* 0: fp32 operands; 1: bf16 operands, fp32 accumulation (GEMM models)     */
    int32_t adagrad_mode;      /* 0: element-wise state, same shape as the table; 1: one float per row    */
    float adagrad_eps;         /* added to sqrt(state); 0 selects the default 1e-10                       */
    float adv_temperature;     /* 0: negatives weigh 1/k each; > 0: softmax(temperature * score) weights  */
    int32_t validate_indices;  /* != 0: kge_train_step / kge_score range-check ids on the device and the  */
                               /* next kge_check_indices call reports the result                          */
    int32_t loss;              /* kge_loss                                                                */
} kge_config;

/* Create a context and its workspace on cfg->device.  (host) cfg, (host) out.  The workspace is sized from
 * max_batch, max_neg_per_chunk, max_chunks and ent_dim and stays allocated until kge_destroy; it holds what Sec. 3.1
 * step 2 fetches for one mini-batch (the rows, their gradients) and never the tables.  (Library lifecycle: the
 * paper has no passage for it.) */
int kge_create(const kge_config* cfg, kge_ctx** out);

/* Free the workspace and the context.  kge_destroy(NULL) does nothing.  The caller must have synchronised
 * every stream that still runs work of this context.  (Library lifecycle, no passage.) */
void kge_destroy(kge_ctx* ctx);

/*
 * One training step (Sec. 3.1 steps 2-4 with the negative sampling layout of Sec. 3.3).
 *
 *   ent [num_entities x ent_dim], ent_state (same shape; [num_entities] floats when adagrad_mode is 1): entity
 *   table and its Adagrad accumulator, updated in place; rel, rel_state likewise [num_relations x rel_dim].
 *   h, r, t [b]: int64 ids of the positive triples.
 *   neg [(b / chunk) * k]: int64 corrupting entity ids; positives chunk*c .. chunk*c + chunk - 1 share
 *   neg[c*k .. c*k + k - 1].  neg_side says whether they replace the tail or the head.
 *   Loss (Sec. 2, logistic loss with y = +1 on positives and -1 on negatives, unless cfg.loss selects the
 *   pairwise ranking loss, see kge_loss):
 *       L = (1/b) sum_i [ log(1 + exp(-f+_i)) + sum_j w_ij log(1 + exp(f-_ij)) ],
 *   w_ij = 1/k, or softmax_j(adv_temperature * f-_ij) held constant in the backward pass.
 *   Update: for every distinct row that occurs among h, t, neg (entities) or r (relations), with g the sum of
 *   all gradient contributions to that row:  state += g*g ; row -= lr * g / (sqrt(state) + eps), element by
 *   element (adagrad_mode 0), or with one accumulator for the whole row (adagrad_mode 1: the optimizer is not
 *   named in the paper; this variant keeps 1/ent_dim of the state):
 *   state += mean_d g_d^2 ; row -= lr * g / (sqrt(state) + eps).
 *   All reads of the tables use the values from before this step.  Rows that do not occur are not written.
 *   loss_out: device float, receives L; may be NULL.
 *
 * Requirements: b > 0, chunk > 0, b % chunk == 0, k > 0, and the workspace limits of kge_create.
 * Ids must lie inside their tables (a caller contract unless validate_indices is set).
 */
int kge_train_step(kge_ctx* ctx, float* ent, float* ent_state, float* rel, float* rel_state,
                   const int64_t* h, const int64_t* r, const int64_t* t, int64_t b,
                   const int64_t* neg, int64_t k, int64_t chunk, int32_t neg_side,
                   float gamma, float lr, void* hip_stream, float* loss_out);

/*
 * n_steps training steps in a row with ids staged on the device beforehand: step s uses h[s*b .. s*b + b - 1]
 * (r, t likewise) and neg[s*(b/chunk)*k ..].  neg_sides: (host) array of n_steps kge_neg_side values, or NULL for
 * tail corruption throughout.  loss_out: device float[n_steps] or NULL.  Same result as n_steps calls of
 * kge_train_step; exists so that a whole pass over pre-sampled mini-batches (Sec. 3.1 step 1 done ahead of time)
 * costs one call.  On a stream that can be captured (any stream but the legacy default stream) the steps are
 * replayed from HIP graphs that the context builds on the first call with a given combination of tables, b, k, chunk,
 * gamma and lr (that call creates graph objects) and keeps: the kernels find the id arrays, the sides and the loss
 * array of the running call through a block in the workspace, so later calls with other arrays replay the same
 * graphs and allocate nothing.  The call must not itself be made while the stream is being captured by the caller
 * (then, and on the default stream, and for fewer than 4 steps, it launches kernel by kernel).  The sides are copied
 * into a fixed part of the workspace; a call of more than 65,536 steps with sides runs in segments of that length.
 */
int kge_train_steps(kge_ctx* ctx, float* ent, float* ent_state, float* rel, float* rel_state,
                    const int64_t* h, const int64_t* r, const int64_t* t, int64_t b,
                    const int64_t* neg, int64_t k, int64_t chunk, const int32_t* neg_sides, int64_t n_steps,
                    float gamma, float lr, void* hip_stream, float* loss_out);

/*
 * Forward only: scores of the positives and of their chunked negatives (Table 1; Sec. 3.3 for the layout).
 * pos_out [b] receives f(h_i, r_i, t_i); neg_out [b*k], row-major with one row per positive, receives
 * f(h_i, r_i, n) (tail side) or f(n, r_i, t_i) (head side) for the k corrupting entities of i's chunk; either
 * may be NULL.  k may be 0 when neg_out is NULL.  Tables are not modified.
 */
int kge_score(kge_ctx* ctx, const float* ent, const float* rel,
              const int64_t* h, const int64_t* r, const int64_t* t, int64_t b,
              const int64_t* neg, int64_t k, int64_t chunk, int32_t neg_side, float gamma,
              void* hip_stream, float* pos_out, float* neg_out);

/*
 * kge_score for callers that cannot allocate device memory: code that runs while a stream is being captured into a
 * HIP graph, tight serving loops, harnesses that forbid hipMalloc.  There is no context: (host) cfg carries model,
 * device, num_entities, num_relations, ent_dim and rel_dim (gemm_input must be 0; the other fields are ignored), and
 * the staging that kge_score keeps in a context's workspace (the o rows, the gathered corrupting rows, norms) lives
 * in a fixed 8 MiB array inside the library's device image, of which every GPU that runs the library holds a copy
 * until the process ends.  The call makes no hipMalloc / hipFree and calls no allocating library routine; its first
 * use on a device looks the array's address up (and, like any first launch, loads the kernels), so make one call
 * before a capture begins.  Other arguments, outputs and results exactly as for kge_score.
 * Limits: TransE-L2, TransE-L1, DistMult, ComplEx, RotatE; 4 * ent_dim * (b + (b/chunk) * k) + 24 * (b + (b/chunk) * k)
 * bytes (each piece rounded up to 256) must fit the 8 MiB, else KGE_ERR_WORKSPACE and nothing is enqueued; ids are
 * clamped into their tables (no validate_indices).  Every call on a GPU uses that GPU's one array: calls that overlap
 * on one GPU, on whatever streams, race; calls on one stream are ordered.  Errors: kge_last_error(NULL) has the text.
 */
int kge_score_noalloc(const kge_config* cfg, const float* ent, const float* rel,
                      const int64_t* h, const int64_t* r, const int64_t* t, int64_t b,
                      const int64_t* neg, int64_t k, int64_t chunk, int32_t neg_side, float gamma,
                      void* hip_stream, float* pos_out, float* neg_out);

/*
 * Test hook for the duplicate reduction of the last kge_train_step on this context (Sec. 2: mini-batches
 * touch few rows, and one row may be touched many times).  which = 0: entity rows (the multiset
 * {h_i} + {t_i} + {neg}); which = 1: relation rows ({r_i}).  uniq_out receives the distinct ids in ascending
 * order, count_out their multiplicities, *n_unique_out how many there are; each output array must hold as
 * many elements as the multiset has (2b + (b/chunk)*k, or b).  Enqueues on hip_stream.
 */
int kge_get_dedup(kge_ctx* ctx, int32_t which, int64_t* uniq_out, int32_t* count_out, int64_t* n_unique_out,
                  void* hip_stream);

/* Synchronises hip_stream and returns KGE_ERR_INDEX_RANGE if any call since the last check saw an id outside
 * its table (contexts created with validate_indices), else KGE_OK; the flag is cleared by the call that reports it.
 * What the kernels do with such an id, validated or not: they clamp it into its table (an id below 0 becomes row 0,
 * an id of num_entities / num_relations or more becomes the last row), so nothing outside the tables is ever read
 * or written, and the call computes exactly what it would with the clamped ids: in a training step the clamped
 * row is read, takes the bad position's gradient and is updated.  A caller that must not train on such a batch
 * checks before it uses the tables again.  (No passage of the paper: input validation.) */
int kge_check_indices(kge_ctx* ctx, void* hip_stream);

/*
 * Per-kernel timing for measurement (the paper reports where time goes per phase, Sec. 6.1.3; this is the
 * library's counterpart).  kge_profile(ctx, 1) makes every following kge_train_step / kge_train_steps launch
 * each of its kernels with a start and a stop event that receive the dispatch's own begin / end timestamps (the
 * duration a kernel trace reports), and synchronise the stream after every step; kge_profile(ctx, 0) restores
 * normal asynchronous operation.  Either call clears the accumulated times.
 * kge_profile_read: (host) ms_out[KGE_PROF_SLOTS] receives the summed kernel times in milliseconds per slot,
 * (host) *steps_out the number of steps they cover.  kge_profile_slot_name: (host) static name of a slot.
 */
enum {
    KGE_PROF_GATHER = 0,   /* row gather + positive scores             */
    KGE_PROF_SCORE = 1,    /* chunked negative scoring                  */
    KGE_PROF_LOSS = 2,     /* loss and backward coefficients            */
    KGE_PROF_BACKWARD = 3, /* dL/do and gradient rows of the negatives  */
    KGE_PROF_CHAIN = 4,    /* chain rule to head / tail / relation rows */
    KGE_PROF_SORT = 5,     /* (id, position) sort, on its own stream    */
    KGE_PROF_UPDATE = 6,   /* segment sum + sparse Adagrad              */
    KGE_PROF_PHI = 7,      /* RESCAL: o = M_r^T h or M_r t              */
    KGE_PROF_REL_UPDATE = 8, /* RESCAL: update of the relation matrices */
    KGE_PROF_SLOTS = 9
};
int kge_profile(kge_ctx* ctx, int32_t enable);
int kge_profile_read(kge_ctx* ctx, double* ms_out, int64_t* steps_out);
const char* kge_profile_slot_name(int32_t slot);

/*
 * Link-prediction evaluation (paper Sec. 5: a test triple is ranked among the triples obtained by replacing its
 * tail, or its head, with sampled corrupting entities; no filtering).  Arguments as for kge_score; the k
 * corrupting entities of a chunk are the candidates of every positive of that chunk.
 *   rank_out[i] = 1 + #{ j : f-_ij > f+_i }   (device int32 [b]; ties with the positive do not count against it)
 * Scores are formed as in kge_score (fp32, or bf16 operands when the context says so) and live in the context's
 * workspace only.  Tables are not modified.
 * kge_rank_metrics: (device) metrics_out[5] = Hit@1, Hit@3, Hit@10 (shares of ranks <= 1, 3, 10), MR (mean rank),
 * MRR (mean reciprocal rank) of ranks[0 .. n-1] (device), as fp64; one kernel on the current device, counts are
 * exact integers, the reciprocal sum has a fixed order.
 */
int kge_rank(kge_ctx* ctx, const float* ent, const float* rel,
             const int64_t* h, const int64_t* r, const int64_t* t, int64_t b,
             const int64_t* neg, int64_t k, int64_t chunk, int32_t neg_side, float gamma,
             void* hip_stream, int32_t* rank_out);
int kge_rank_metrics(const int32_t* ranks, int64_t n, double* metrics_out, void* hip_stream);

/*
 * Step 1 of the mini-batch loop on the device (paper Sec. 3.1 step 1; Sec. 3.3 for the negatives): the ids of
 * n_steps consecutive steps, first_step .. first_step + n_steps - 1, in the layout kge_train_steps takes.
 * Every id is a function of (seed, step, position) alone, so steps can be generated in any order and any number
 * at a time; kge.h's counter-based generator is:
 *     key = mix(mix(mix(mix(seed + 0x9E3779B97F4A7C15 * tag) + step) + a) + j),  id = floor(key * n / 2^64),
 *     mix(z): z = (z ^ z >> 30) * 0xBF58476D1CE4E5B9; z = (z ^ z >> 27) * 0x94D049BB133111EB; z ^ z >> 31
 *   positives  (tag 1, a = 0, j = position in the batch, n = n_triples): the triple at that index of `triples`
 *              (drawn uniformly with replacement);
 *   negatives  slot j of chunk a: for j >= n_degree uniform over all entities (tag 2, n = num_entities); for
 *              j < n_degree (tag 3, n = batch) the tail -- the head when heads are corrupted -- of that position
 *              of the same mini-batch: degree-proportional sampling from the batch, as in Sec. 3.3.
 *   side       side_mode 0: tails corrupted in every step, 1: heads, 2: tails in even steps, heads in odd ones.
 * triples: (device) [n_triples x 3] int64 rows (h, r, t), 0 < n_triples < 2^32.
 * h, r, t: (device) [n_steps x batch]; neg: (device) [n_steps x n_chunks x neg_per_chunk] (may be NULL when
 * neg_per_chunk is 0); sides: (device) [n_steps] int32, may be NULL.  Enqueues one kernel on `stream` of the
 * current device and returns; errors (null pointers, sizes out of range) are reported before anything is enqueued
 * and kge_last_error(NULL) has the text.
 */
typedef struct {
    uint64_t seed;
    const int64_t* triples;
    int64_t n_triples;
    int64_t num_entities;
    int32_t batch;
    int32_t n_chunks;
    int32_t neg_per_chunk;
    int32_t n_degree;  /* 0 .. neg_per_chunk */
    int32_t side_mode; /* 0, 1, 2 */
} kge_sampler;
int kge_sample_steps(const kge_sampler* sampler, int64_t first_step, int64_t n_steps, int64_t* h, int64_t* r,
                     int64_t* t, int64_t* neg, int32_t* sides, void* stream);

/* (host) Text of the last error on this context ("" if none); valid until the next call on the context.
 * kge_last_error(NULL) returns the text of the last failed context-free call (kge_create, kge_sample_steps,
 * kge_rank_metrics, kge_score_noalloc) on this thread.  (Error reporting, no passage.) */
const char* kge_last_error(const kge_ctx* ctx);

/* Bytes of device workspace the context holds.  (No passage of the paper: library bookkeeping.) */
int64_t kge_workspace_bytes(const kge_ctx* ctx);

/* How many times kge_train_steps has built its HIP graphs on this context: once per combination of tables, b, k,
 * chunk, gamma and lr, never because the id, side or loss arrays changed.  (Measurement / test aid, no passage.) */
int64_t kge_graph_captures(const kge_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* KGE_H */
