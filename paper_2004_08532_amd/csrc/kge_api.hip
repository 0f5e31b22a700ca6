// C ABI of libkge: argument checks, workspace, and the order in which the kernels of one step are enqueued.
// See include/kge.h for the contract of each entry point.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>

#include "kge_common.h"

// Scratch memory of kge_score_noalloc, the one entry point that allocates nothing: a fixed array in the library's
// device image (every GPU that runs the library holds its own copy until the process ends).  In host code the name
// below is only a handle for hipGetSymbolAddress; the address the kernels get is the one that call returns.
constexpr size_t KGE_NOALLOC_SCRATCH_BYTES = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[KGE_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int KGE_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[KGE_MAX_DEVICES] = {};  // per device: where that GPU's copy of `scratch` lives

// Address of the current device's scratch array (resolved once per device, with that device current).
hipError_t scratch_address(int device, void** out) {
    if (device < 0 || device >= KGE_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

thread_local char g_create_err[512] = "";

int fail(kge_ctx* c, int code, const char* fmt, const char* detail = "") {
    char* dst = c ? c->err : g_create_err;
    snprintf(dst, 512, fmt, detail);
    return code;
}

#define KGE_HIP(c, call)                                                                 \
    do {                                                                                 \
        hipError_t e_ = (call);                                                          \
        if (e_ != hipSuccess) return fail((c), KGE_ERR_DEVICE, #call ": %s", hipGetErrorString(e_)); \
    } while (0)

bool is_gemm_model(int m) { return m == KGE_TRANSE_L2 || m == KGE_DISTMULT || m == KGE_COMPLEX || m == KGE_RESCAL; }

__global__ void k_validate(StepIds ids, int64_t n_ent, int64_t n_rel, int* flag) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const StepView v = step_view(ids);
    bool bad = false;
    if (i < ids.b)
        bad = v.h[i] < 0 || v.h[i] >= n_ent || v.t[i] < 0 || v.t[i] >= n_ent || v.r[i] < 0 || v.r[i] >= n_rel;
    if (i < ids.n_neg) bad = bad || v.neg[i] < 0 || v.neg[i] >= n_ent;
    if (bad) atomicOr(flag, 1);
}

void launch_validate(kge_ctx* c, const StepIds& ids, hipStream_t st) {
    const int n = ids.b > ids.n_neg ? ids.b : ids.n_neg;
    hipLaunchKernelGGL(k_validate, dim3((n + 255) / 256), dim3(256), 0, st, ids, c->cfg.num_entities,
                       c->cfg.num_relations, c->flags);
}

StepIds direct_ids(const int64_t* h, const int64_t* r, const int64_t* t, int b, const int64_t* neg, int n_neg, int side,
                   float* loss_out) {
    StepIds ids;
    ids.h = h; ids.r = r; ids.t = t; ids.neg = neg; ids.b = b; ids.n_neg = n_neg; ids.side = side;
    ids.blk = nullptr; ids.loss_out = loss_out;
    return ids;
}

// Fills the step block of a kge_train_steps call (replay mode): one thread, the values travel as kernel arguments.
__global__ void k_set_step_block(StepBlock* blk, StepBlock value) { *blk = value; }

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

int check_batch(kge_ctx* c, const void* ent, const void* rel, const int64_t* h, const int64_t* r, const int64_t* t,
                int64_t b, const int64_t* neg, int64_t k, int64_t chunk, int32_t side, bool need_neg) {
    if (!ent || !rel || !h || !r || !t) return fail(c, KGE_ERR_INVALID_ARG, "null table or id pointer%s");
    if (b <= 0 || chunk <= 0 || b % chunk != 0) return fail(c, KGE_ERR_INVALID_ARG, "b must be a positive multiple of chunk%s");
    if (k < 0 || (need_neg && k == 0)) return fail(c, KGE_ERR_INVALID_ARG, "k out of range%s");
    if (k > 0 && !neg) return fail(c, KGE_ERR_INVALID_ARG, "neg is null%s");
    if (side != KGE_NEG_TAIL && side != KGE_NEG_HEAD) return fail(c, KGE_ERR_INVALID_ARG, "neg_side must be 0 or 1%s");
    if (b > c->cfg.max_batch || k > c->cfg.max_neg_per_chunk || b / chunk > c->cfg.max_chunks)
        return fail(c, KGE_ERR_WORKSPACE, "b, k or b/chunk exceed the sizes given to kge_create%s");
    return KGE_OK;
}

void forward(kge_ctx* c, const float* ent, const float* rel, const StepIds& ids, int k, int chunk, float gamma,
             float* pos_out, float* neg_out, int ld_out, int dist_mode, hipStream_t st) {
    if (c->cfg.validate_indices) launch_validate(c, ids, st);
    if (c->cfg.model == KGE_RESCAL) kge_launch_rescal_phi(c, ent, rel, ids, st);
    if (c->cfg.model == KGE_TRANSR) kge_transr_phi(c, ent, rel, ids, gamma, pos_out, st);
    kge_launch_gather(c, ent, rel, ids, gamma, pos_out, false, st);
    if (neg_out && k > 0) {
        if (c->cfg.model == KGE_TRANSR) {
            kge_gemm_transr_project(c, rel, ids, k, chunk, kge_transr_projections(c), st);
            kge_transr_score(c, ids, k, gamma, neg_out, ld_out, st);
        } else if (is_gemm_model(c->cfg.model)) {
            kge_gemm_neg_score(c, ids.b, k, chunk, gamma, neg_out, ld_out, dist_mode, st);
        } else {
            kge_pair_neg_score(c, ids.b, k, chunk, gamma, neg_out, ld_out, st);
        }
    }
}

// ---- optional per-kernel timing (kge_profile): the one kernel launched inside a scope carries the scope's two
// events as its start / stop events (KGE_LAUNCH), the stream is synchronised after the step, and the elapsed times
// are accumulated per slot.
struct ProfScope {
    kge_ctx* c;
    ProfScope(kge_ctx* c_, int slot) : c(c_) {
        if (c->prof_on) { c->launch_ev0 = c->prof_ev[slot][0]; c->launch_ev1 = c->prof_ev[slot][1]; }
    }
    ~ProfScope() { c->launch_ev0 = nullptr; c->launch_ev1 = nullptr; }
};

// TransR after its phi and gather launches: the three batched products with the elementwise steps between them.
// Profile slots: neg_score = the projection product, loss, neg_backward = the back-projection product, chain,
// rel_update, update; the small kernels between them are not timed separately.
int enqueue_transr_rest(kge_ctx* c, float* ent, float* ent_state, float* rel, float* rel_state, const StepIds& ids,
                        int K, int G, float gamma, float lr, bool long_lists, hipStream_t st) {
    float* P = kge_transr_projections(c);
    {
        ProfScope p(c, KGE_PROF_SCORE);
        kge_gemm_transr_project(c, rel, ids, K, G, P, st);
    }
    kge_transr_score(c, ids, K, gamma, c->S, c->ld_s, st);
    {
        ProfScope p(c, KGE_PROF_LOSS);
        kge_launch_loss(c, ids.b, K, gamma, st);
    }
    kge_transr_dp(c, ids, K, st);
    {
        ProfScope p(c, KGE_PROF_BACKWARD);
        kge_gemm_transr_back_project_sum(c, rel, ids, K, G, P, c->Gent + (int64_t)2 * ids.b * c->cfg.ent_dim, st);
    }
    kge_gemm_transr_matrix_grad(c, ids, K, G, P, kge_transr_matrix_grads(c), st);
    {
        ProfScope p(c, KGE_PROF_CHAIN);
        kge_transr_chain(c, ent, rel, ids, st);
    }
    if (long_lists) KGE_HIP(c, hipStreamWaitEvent(st, c->ev_join, 0));
    {
        ProfScope p(c, KGE_PROF_REL_UPDATE);
        kge_transr_update(c, rel, rel_state, ids, lr, st);
    }
    {
        ProfScope p(c, KGE_PROF_UPDATE);
        kge_launch_update(c, ent, ent_state, rel, rel_state, ids, lr, 0, st);
    }
    KGE_HIP(c, hipGetLastError());
    if (c->prof_on) {
        KGE_HIP(c, hipStreamSynchronize(st));
        for (int s = 0; s < KGE_PROF_SLOTS; ++s) {
            float ms = 0.f;
            if (s == KGE_PROF_SORT && !long_lists) continue;
            if (hipEventElapsedTime(&ms, c->prof_ev[s][0], c->prof_ev[s][1]) == hipSuccess) c->prof_ms[s] += ms;
        }
        c->prof_steps += 1;
    }
    return KGE_OK;
}

int enqueue_step(kge_ctx* c, float* ent, float* ent_state, float* rel, float* rel_state, const StepIds& ids, int K,
                 int G, float gamma, float lr, hipStream_t st) {
    const int B = ids.b;
    // Ordering the key lists needs only the ids.  Short lists are ordered by extra blocks of the gather launch;
    // long ones by a radix sort on a second stream that joins before the update.
    const bool long_lists = 2 * B + ids.n_neg > KGE_RANK_MAX_KEYS;
    if (long_lists) {
        KGE_HIP(c, hipEventRecord(c->ev_fork, st));
        KGE_HIP(c, hipStreamWaitEvent(c->side_stream, c->ev_fork, 0));
        {
            ProfScope p(c, KGE_PROF_SORT);
            kge_launch_sort(c, ids, c->side_stream);
        }
        KGE_HIP(c, hipEventRecord(c->ev_join, c->side_stream));
    }
    if (c->cfg.validate_indices) launch_validate(c, ids, st);
    if (c->cfg.model == KGE_RESCAL) {
        ProfScope p(c, KGE_PROF_PHI);
        kge_launch_rescal_phi(c, ent, rel, ids, st);
    }
    if (c->cfg.model == KGE_TRANSR) {
        ProfScope p(c, KGE_PROF_PHI);
        kge_transr_phi(c, ent, rel, ids, gamma, nullptr, st);
    }
    {
        ProfScope p(c, KGE_PROF_GATHER);
        kge_launch_gather(c, ent, rel, ids, gamma, nullptr, !long_lists, st);
    }
    if (c->cfg.model == KGE_TRANSR) return enqueue_transr_rest(c, ent, ent_state, rel, rel_state, ids, K, G, gamma, lr, long_lists, st);
    {
        ProfScope p(c, KGE_PROF_SCORE);
        if (is_gemm_model(c->cfg.model))
            kge_gemm_neg_score(c, B, K, G, gamma, c->S, c->ld_s, kge_gemm_backward_forms_w(c) ? 2 : 1, st);
        else kge_pair_neg_score(c, B, K, G, gamma, c->S, c->ld_s, st);
    }
    // The matrix-product models fold the loss (uniform weights) and the chain rule (TransE-L2, DistMult) into
    // the backward launch; whatever is not folded runs as its own kernel.
    const bool gemm = is_gemm_model(c->cfg.model);
    const bool run_loss = !(gemm && kge_gemm_backward_forms_w(c));
    const bool run_chain = !(gemm && kge_gemm_backward_does_chain(c));
    const int n_loss_parts = gemm ? kge_gemm_loss_parts(c, B, K, G) : 0;
    if (run_loss) {
        ProfScope p(c, KGE_PROF_LOSS);
        kge_launch_loss(c, B, K, gamma, st);
    }
    {
        ProfScope p(c, KGE_PROF_BACKWARD);
        if (gemm) kge_gemm_neg_backward(c, ent, rel, ids, K, G, gamma, st);
        else kge_pair_neg_backward(c, B, K, G, st);
    }
    if (run_chain) {
        ProfScope p(c, KGE_PROF_CHAIN);
        if (c->cfg.model == KGE_RESCAL) kge_launch_rescal_chain(c, ent, rel, ids, st);
        else kge_launch_chain(c, ent, rel, ids, st);
    }
    if (long_lists) KGE_HIP(c, hipStreamWaitEvent(st, c->ev_join, 0));
    if (c->cfg.model == KGE_RESCAL) {
        ProfScope p(c, KGE_PROF_REL_UPDATE);
        kge_launch_rescal_update(c, rel, rel_state, ids, lr, st);
    }
    {
        ProfScope p(c, KGE_PROF_UPDATE);
        kge_launch_update(c, ent, ent_state, rel, rel_state, ids, lr, n_loss_parts, st);
    }
    KGE_HIP(c, hipGetLastError());
    if (c->prof_on) {
        KGE_HIP(c, hipStreamSynchronize(st));
        for (int s = 0; s < KGE_PROF_SLOTS; ++s) {
            float ms = 0.f;
            if ((s == KGE_PROF_SORT && !long_lists) || (s == KGE_PROF_LOSS && !run_loss) ||
                (s == KGE_PROF_CHAIN && !run_chain) || ((s == KGE_PROF_PHI || s == KGE_PROF_REL_UPDATE) && c->cfg.model != KGE_RESCAL))
                continue;  // that kernel did not run in this configuration
            if (hipEventElapsedTime(&ms, c->prof_ev[s][0], c->prof_ev[s][1]) == hipSuccess) c->prof_ms[s] += ms;
        }
        c->prof_steps += 1;
    }
    return KGE_OK;
}

// ---- replay: kge_train_steps captures 1, 2, 4, ... 32 consecutive steps into HIP graphs whose kernels take the step
// number and the id arrays from device memory (the step block), so the same graphs serve every step of every call
// of the same shape.  Launching a graph costs the host about 2 us per kernel in it plus a fixed part, and the
// device starts on a graph only once the whole of it is enqueued, and every graph start costs the device about 8 us
// of idling: a call therefore starts with a graph of one step (the device is busy after one step's worth of
// enqueueing), lets the graphs grow as fast as the host can stay ahead, and otherwise uses as few graphs as the step
// count allows (20 steps: 1, 1, 2, 16).
constexpr int REPLAY_SIZES = 6;  // graphs of 1 << i steps, i < REPLAY_SIZES (measured per Freebase-scale step in a
                                 // 10,000-step call: longest graph 8 steps 38.2 us, 16: 37.9, 32: 37.8, 64: 38.4)

// Launches exec[i] (1 << i steps), or, if that graph is too long for its place in the call, its two halves.  Too long:
// more than RAMP times the steps already enqueued by this call (the first graph of a call is one step).  Enqueueing
// costs the host about 8 us per step, a step takes the device four times that or more, so the host stays ahead.
constexpr int64_t RAMP = 4;
void launch_graphs(hipGraphExec_t* exec, int i, int64_t* done, hipStream_t st, hipError_t* err) {
    const int64_t len = (int64_t)1 << i, cap = *done > 0 ? RAMP * *done : 1;
    if (i > 0 && len > cap) {
        launch_graphs(exec, i - 1, done, st, err);
        launch_graphs(exec, i - 1, done, st, err);
        return;
    }
    const hipError_t e = hipGraphLaunch(exec[i], st);
    if (*err == hipSuccess) *err = e;
    *done += len;
}

// What a captured graph depends on.  The id arrays, the per-step sides and the loss array are not part of it: the
// kernels find them through the step block.
struct ReplayKey {
    void *ent, *ent_state, *rel, *rel_state;
    int64_t b, k, chunk;
    float gamma, lr;
    bool operator==(const ReplayKey& o) const { return memcmp(this, &o, sizeof(ReplayKey)) == 0; }
};

struct ReplayCache {
    bool valid = false;
    ReplayKey key;
    hipGraphExec_t exec[REPLAY_SIZES] = {};  // exec[i] runs 1 << i steps
};

void replay_drop(ReplayCache* rc) {
    for (int i = 0; i < REPLAY_SIZES; ++i) {
        if (rc->exec[i]) (void)hipGraphExecDestroy(rc->exec[i]);
        rc->exec[i] = nullptr;
    }
    rc->valid = false;
}

int capture_steps(kge_ctx* c, float* ent, float* ent_state, float* rel, float* rel_state, const StepIds& ids, int K,
                  int G, float gamma, float lr, hipStream_t st, int n, hipGraphExec_t* out) {
    hipGraph_t graph = nullptr;
    KGE_HIP(c, hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
    int rc = KGE_OK;
    for (int s = 0; s < n && rc == KGE_OK; ++s) rc = enqueue_step(c, ent, ent_state, rel, rel_state, ids, K, G, gamma, lr, st);
    hipError_t e = hipStreamEndCapture(st, &graph);
    if (rc != KGE_OK) {
        if (graph) (void)hipGraphDestroy(graph);
        return rc;
    }
    if (e != hipSuccess) return fail(c, KGE_ERR_DEVICE, "hipStreamEndCapture: %s", hipGetErrorString(e));
    e = hipGraphInstantiate(out, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) return fail(c, KGE_ERR_DEVICE, "hipGraphInstantiate: %s", hipGetErrorString(e));
    (void)hipGraphUpload(*out, st);  // so that the first launch does not pay for it; a failure here is not one
    (void)hipGetLastError();
    return KGE_OK;
}

}  // namespace

extern "C" {

int kge_create(const kge_config* cfg, kge_ctx** out) {
    if (!cfg || !out) return fail(nullptr, KGE_ERR_INVALID_ARG, "null argument%s");
    *out = nullptr;
    const int m = cfg->model;
    if (m < KGE_TRANSE_L2 || m > KGE_TRANSR) return fail(nullptr, KGE_ERR_INVALID_ARG, "unknown model%s");
    const bool cplx = m == KGE_COMPLEX || m == KGE_ROTATE;
    if (cfg->ent_dim <= 0 || cfg->ent_dim > 1024 || cfg->ent_dim % (cplx ? 8 : 4) != 0)
        return fail(nullptr, KGE_ERR_INVALID_ARG, "ent_dim must be a multiple of 4 (8 for ComplEx/RotatE), at most 1024%s");
    const int sq = cfg->ent_dim * cfg->ent_dim;
    const int want_rel = m == KGE_ROTATE ? cfg->ent_dim / 2 : (m == KGE_RESCAL ? sq : (m == KGE_TRANSR ? cfg->ent_dim + sq : cfg->ent_dim));
    if (cfg->rel_dim != want_rel)
        return fail(nullptr, KGE_ERR_INVALID_ARG, "rel_dim must be ent_dim (ent_dim/2 for RotatE, ent_dim^2 for RESCAL, ent_dim + ent_dim^2 for TransR)%s");
    if ((m == KGE_RESCAL || m == KGE_TRANSR) && (cfg->adagrad_mode != 0 || cfg->gemm_input != 0))
        return fail(nullptr, KGE_ERR_UNSUPPORTED, "RESCAL and TransR run with element-wise Adagrad state and fp32 operands only%s");
    if (cfg->num_entities <= 0 || cfg->num_relations <= 0 || cfg->num_entities >= (1ll << 32) ||
        cfg->num_relations >= (1ll << 32))
        return fail(nullptr, KGE_ERR_INVALID_ARG, "table row counts must be in [1, 2^32)%s");
    if (cfg->max_batch <= 0 || cfg->max_neg_per_chunk < 0 || cfg->max_chunks <= 0 || cfg->max_chunks > cfg->max_batch)
        return fail(nullptr, KGE_ERR_INVALID_ARG, "bad workspace limits%s");
    if ((int64_t)cfg->max_chunks * cfg->max_neg_per_chunk + 2ll * cfg->max_batch > (1 << 24))
        return fail(nullptr, KGE_ERR_INVALID_ARG, "more than 2^24 entity keys per step%s");
    if (cfg->adagrad_mode != 0 && cfg->adagrad_mode != 1) return fail(nullptr, KGE_ERR_INVALID_ARG, "adagrad_mode must be 0 or 1%s");
    if (cfg->loss != KGE_LOSS_LOGISTIC && cfg->loss != KGE_LOSS_RANKING) return fail(nullptr, KGE_ERR_INVALID_ARG, "loss must be 0 (logistic) or 1 (ranking)%s");
    if (cfg->gemm_input != 0 && cfg->gemm_input != 1) return fail(nullptr, KGE_ERR_INVALID_ARG, "gemm_input must be 0 or 1%s");
    if (cfg->gemm_input == 1 && !is_gemm_model(cfg->model))
        return fail(nullptr, KGE_ERR_UNSUPPORTED, "bf16 operands exist for the matrix-product models only (TransE-L2, DistMult, ComplEx)%s");
    if (cfg->adv_temperature < 0.f || cfg->adagrad_eps < 0.f) return fail(nullptr, KGE_ERR_INVALID_ARG, "negative temperature or eps%s");

    int ndev = 0;
    KGE_HIP(nullptr, hipGetDeviceCount(&ndev));
    if (cfg->device < 0 || cfg->device >= ndev) return fail(nullptr, KGE_ERR_INVALID_ARG, "no such device%s");
    KGE_HIP(nullptr, hipSetDevice(cfg->device));

    kge_ctx* c = new (std::nothrow) kge_ctx();
    if (!c) return fail(nullptr, KGE_ERR_DEVICE, "out of host memory%s");
    memset(c, 0, sizeof(*c));
    c->cfg = *cfg;
    c->eps = cfg->adagrad_eps > 0.f ? cfg->adagrad_eps : 1e-10f;
    c->ld_s = (cfg->max_neg_per_chunk + 3) / 4 * 4;
    if (c->ld_s == 0) c->ld_s = 4;
    c->max_neg_rows = cfg->max_chunks * cfg->max_neg_per_chunk;
    c->max_ent_keys = 2 * cfg->max_batch + c->max_neg_rows;

    const size_t D = cfg->ent_dim, Dr = cfg->rel_dim, B = cfg->max_batch, NR = c->max_neg_rows > 0 ? c->max_neg_rows : 1;
    const size_t EK = c->max_ent_keys;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    const size_t o_O = take(B * D * 4), o_N = take(NR * D * 4), o_S = take(B * c->ld_s * 4), o_GO = take(B * D * 4);
    const size_t o_Ge = take(EK * D * 4), o_Gr = take(B * (m == KGE_RESCAL ? 2 * D : Dr) * 4);  // RESCAL keeps two factor rows per positive
    const size_t o_fpos = take(B * 4), o_on2 = take(B * 4), o_nn2 = take(NR * 4), o_cpos = take(B * 4);
    const size_t o_rl = take(B * 4), o_idp = take(B * 4);
    const size_t o_nlp = take((B / 32 + cfg->max_chunks + 1) * ((size_t)cfg->max_neg_per_chunk / 32 + 1) * 4);
    const size_t o_ek0 = take(EK * 4), o_ek1 = take(EK * 4), o_ep0 = take(EK * 4), o_ep1 = take(EK * 4);
    const size_t o_rk0 = take(B * 4), o_rk1 = take(B * 4), o_rp0 = take(B * 4), o_rp1 = take(B * 4);
    const size_t o_flags = take(256), o_step = take(256), o_sides = take(sizeof(int32_t) * KGE_SIDES_CAP);
    c->ld_bf = (cfg->ent_dim + 63) / 64 * 64;  // rows start on 128-byte lines: a K block of a row is one line, not two
    const bool bf = cfg->gemm_input == 1;
    const size_t o_Obf = take(bf ? B * c->ld_bf * 2 + 64 : 0), o_Nbf = take(bf ? NR * c->ld_bf * 2 + 64 : 0);
    const bool transr = m == KGE_TRANSR;
    const size_t proj = transr ? B * (size_t)(cfg->max_neg_per_chunk > 0 ? cfg->max_neg_per_chunk : 1) * D * 4 : 0;
    const size_t o_PP = take(transr ? B * D * 4 : 0), o_P3 = take(proj);
    const size_t sort_slices = (EK + KGE_SORT_SLICE - 1) / KGE_SORT_SLICE + (B + KGE_SORT_SLICE - 1) / KGE_SORT_SLICE;
    const size_t o_sc = take(sort_slices * 17 * 256 * 4 + 2 * 256 * 4);  // digit counts per wave and per slice + the two lists' digit bases
    const bool pair_model = m == KGE_ROTATE || m == KGE_TRANSE_L1;
    const size_t o_ppo = take(pair_model ? KGE_PAIR_MAX_PARTS * B * D * 4 : 0), o_ppn = take(pair_model ? KGE_PAIR_MAX_PARTS * NR * D * 4 : 0);
    c->ws_bytes = (int64_t)off;

    hipError_t e = hipMalloc(&c->ws_base, off);
    if (e != hipSuccess) {
        fail(nullptr, KGE_ERR_DEVICE, "hipMalloc(workspace): %s", hipGetErrorString(e));
        delete c;
        return KGE_ERR_DEVICE;
    }
    char* base = (char*)c->ws_base;
    c->O = (float*)(base + o_O); c->Nst = (float*)(base + o_N); c->S = (float*)(base + o_S);
    c->GO = (float*)(base + o_GO); c->Gent = (float*)(base + o_Ge); c->Grel = (float*)(base + o_Gr);
    c->fpos = (float*)(base + o_fpos); c->o_n2 = (float*)(base + o_on2); c->n_n2 = (float*)(base + o_nn2);
    c->cpos = (float*)(base + o_cpos); c->row_loss = (float*)(base + o_rl);
    c->inv_dpos = (float*)(base + o_idp); c->neg_loss_part = (float*)(base + o_nlp);
    c->ekey[0] = (uint32_t*)(base + o_ek0); c->ekey[1] = (uint32_t*)(base + o_ek1);
    c->epos[0] = (uint32_t*)(base + o_ep0); c->epos[1] = (uint32_t*)(base + o_ep1);
    c->rkey[0] = (uint32_t*)(base + o_rk0); c->rkey[1] = (uint32_t*)(base + o_rk1);
    c->rpos[0] = (uint32_t*)(base + o_rp0); c->rpos[1] = (uint32_t*)(base + o_rp1);
    c->Obf = bf ? (uint16_t*)(base + o_Obf) : nullptr;
    c->Nbf = bf ? (uint16_t*)(base + o_Nbf) : nullptr;
    c->PP = transr ? (float*)(base + o_PP) : nullptr;
    c->P3 = transr ? (float*)(base + o_P3) : nullptr;
    c->pair_part_o = pair_model ? (float*)(base + o_ppo) : nullptr;
    c->pair_part_n = pair_model ? (float*)(base + o_ppn) : nullptr;
    c->sort_counts = (uint32_t*)(base + o_sc);
    c->flags = (int*)(base + o_flags);
    c->step_block = (StepBlock*)(base + o_step);
    c->sides_dev = (int32_t*)(base + o_sides);

    // hipMemset on device memory returns before the fill has run (it is queued on the null stream, behind whatever
    // the caller has there), and the streams that callers pass are not ordered against the null stream: without the
    // wait below the fill could land after the first call has written its step block into the workspace.
    bool ok = hipMemset(c->ws_base, 0, off) == hipSuccess;
    ok = ok && hipDeviceSynchronize() == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&c->side_stream, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        fail(nullptr, KGE_ERR_DEVICE, "stream/event creation failed%s");
        kge_destroy(c);
        return KGE_ERR_DEVICE;
    }
    *out = c;
    return KGE_OK;
}

void kge_destroy(kge_ctx* c) {
    if (!c) return;
    (void)hipSetDevice(c->cfg.device);
    if (c->side_stream) { (void)hipStreamSynchronize(c->side_stream); (void)hipStreamDestroy(c->side_stream); }
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    for (int s = 0; s < KGE_PROF_SLOTS; ++s)
        for (int e = 0; e < 2; ++e)
            if (c->prof_ev[s][e]) (void)hipEventDestroy(c->prof_ev[s][e]);
    if (c->replay) {
        replay_drop((ReplayCache*)c->replay);
        delete (ReplayCache*)c->replay;
    }
    if (c->ws_base) (void)hipFree(c->ws_base);
    delete c;
}

int kge_train_step(kge_ctx* c, float* ent, float* ent_state, float* rel, float* rel_state,
                   const int64_t* h, const int64_t* r, const int64_t* t, int64_t b,
                   const int64_t* neg, int64_t k, int64_t chunk, int32_t neg_side,
                   float gamma, float lr, void* hip_stream, float* loss_out) {
    if (!c) return KGE_ERR_INVALID_ARG;
    c->err[0] = 0;
    if (!ent_state || !rel_state) return fail(c, KGE_ERR_INVALID_ARG, "null optimizer state%s");
    const int rc = check_batch(c, ent, rel, h, r, t, b, neg, k, chunk, neg_side, true);
    if (rc != KGE_OK) return rc;
    KGE_HIP(c, hipSetDevice(c->cfg.device));
    const StepIds ids = direct_ids(h, r, t, (int)b, neg, (int)((b / chunk) * k), neg_side, loss_out);
    return enqueue_step(c, ent, ent_state, rel, rel_state, ids, (int)k, (int)chunk, gamma, lr, (hipStream_t)hip_stream);
}

int kge_train_steps(kge_ctx* c, float* ent, float* ent_state, float* rel, float* rel_state,
                    const int64_t* h, const int64_t* r, const int64_t* t, int64_t b,
                    const int64_t* neg, int64_t k, int64_t chunk, const int32_t* neg_sides, int64_t n_steps,
                    float gamma, float lr, void* hip_stream, float* loss_out) {
    if (!c) return KGE_ERR_INVALID_ARG;
    c->err[0] = 0;
    if (!ent_state || !rel_state) return fail(c, KGE_ERR_INVALID_ARG, "null optimizer state%s");
    if (n_steps < 0) return fail(c, KGE_ERR_INVALID_ARG, "negative step count%s");
    int rc = check_batch(c, ent, rel, h, r, t, b, neg, k, chunk, KGE_NEG_TAIL, true);
    if (rc != KGE_OK) return rc;
    for (int64_t s = 0; neg_sides && s < n_steps; ++s)
        if (neg_sides[s] != KGE_NEG_TAIL && neg_sides[s] != KGE_NEG_HEAD)
            return fail(c, KGE_ERR_INVALID_ARG, "neg_sides entries must be 0 or 1%s");
    if (n_steps == 0) return KGE_OK;
    KGE_HIP(c, hipSetDevice(c->cfg.device));
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t n_neg = (b / chunk) * k;

    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    (void)hipStreamIsCapturing(st, &cap);
    static const bool replay_enabled = []() {
        const char* e = getenv("KGE_TRAIN_STEPS_REPLAY");  // "0" turns graph replay off (measurement aid)
        return !(e && e[0] == '0');
    }();
    if (!replay_enabled || c->prof_on || n_steps < 4 || cap != hipStreamCaptureStatusNone || st == nullptr ||
        st == hipStreamLegacy) {
        // plain launches: timing mode, very short runs, the caller is capturing this stream itself, or the stream
        // is the legacy default stream, which cannot be captured
        for (int64_t s = 0; s < n_steps; ++s) {
            const StepIds ids = direct_ids(h + s * b, r + s * b, t + s * b, (int)b, neg + s * n_neg, (int)n_neg,
                                           neg_sides ? neg_sides[s] : KGE_NEG_TAIL, loss_out ? loss_out + s : nullptr);
            rc = enqueue_step(c, ent, ent_state, rel, rel_state, ids, (int)k, (int)chunk, gamma, lr, st);
            if (rc != KGE_OK) return rc;
        }
        return KGE_OK;
    }

    // replay path: nothing here allocates once the two graphs exist
    ReplayKey key;
    memset(&key, 0, sizeof(key));
    key.ent = ent; key.ent_state = ent_state; key.rel = rel; key.rel_state = rel_state;
    key.b = b; key.k = k; key.chunk = chunk; key.gamma = gamma; key.lr = lr;
    if (!c->replay) c->replay = new (std::nothrow) ReplayCache();
    ReplayCache* cache = (ReplayCache*)c->replay;
    if (!cache) return fail(c, KGE_ERR_DEVICE, "out of host memory%s");
    if (!cache->valid || !(cache->key == key)) {
        replay_drop(cache);
        StepIds ids = direct_ids(nullptr, nullptr, nullptr, (int)b, nullptr, (int)n_neg, KGE_NEG_TAIL, nullptr);
        ids.blk = c->step_block;
        for (int i = 0; i < REPLAY_SIZES && rc == KGE_OK; ++i)
            rc = capture_steps(c, ent, ent_state, rel, rel_state, ids, (int)k, (int)chunk, gamma, lr, st, 1 << i,
                               &cache->exec[i]);
        if (rc != KGE_OK) {
            replay_drop(cache);
            return rc;
        }
        cache->key = key;
        cache->valid = true;
        c->graph_captures += 1;
    }
    // the per-step sides live in a fixed part of the workspace: a longer call runs in segments of that many steps
    for (int64_t first = 0; first < n_steps; first += KGE_SIDES_CAP) {
        const int64_t n = n_steps - first < KGE_SIDES_CAP ? n_steps - first : KGE_SIDES_CAP;
        if (neg_sides)
            KGE_HIP(c, hipMemcpyAsync(c->sides_dev, neg_sides + first, sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice, st));
        StepBlock blk;
        blk.step = 0;
        blk.h = h + first * b; blk.r = r + first * b; blk.t = t + first * b; blk.neg = neg + first * n_neg;
        blk.sides = neg_sides ? c->sides_dev : nullptr;
        blk.loss_out = loss_out ? loss_out + first : nullptr;
        hipLaunchKernelGGL(k_set_step_block, dim3(1), dim3(1), 0, st, c->step_block, blk);
        // As few graphs as possible: the binary digits of n below the longest graph, smallest first, then the
        // longest graph for the rest.  A graph that is too long for its place in the call (see launch_graphs) is cut
        // into halves.
        int64_t done = 0;
        hipError_t herr = hipSuccess;
        for (int i = 0; i + 1 < REPLAY_SIZES; ++i)
            if (n & ((int64_t)1 << i)) launch_graphs(cache->exec, i, &done, st, &herr);
        for (int64_t q = n >> (REPLAY_SIZES - 1); q > 0; --q) launch_graphs(cache->exec, REPLAY_SIZES - 1, &done, st, &herr);
        KGE_HIP(c, herr);
    }
    KGE_HIP(c, hipGetLastError());
    return KGE_OK;
}

int kge_score(kge_ctx* c, const float* ent, const float* rel,
              const int64_t* h, const int64_t* r, const int64_t* t, int64_t b,
              const int64_t* neg, int64_t k, int64_t chunk, int32_t neg_side, float gamma,
              void* hip_stream, float* pos_out, float* neg_out) {
    if (!c) return KGE_ERR_INVALID_ARG;
    c->err[0] = 0;
    const int rc = check_batch(c, ent, rel, h, r, t, b, neg, k, chunk, neg_side, neg_out != nullptr);
    if (rc != KGE_OK) return rc;
    KGE_HIP(c, hipSetDevice(c->cfg.device));
    const int kk = neg_out ? (int)k : 0;
    const StepIds ids = direct_ids(h, r, t, (int)b, neg, (int)((b / chunk) * kk), neg_side, nullptr);
    forward(c, ent, rel, ids, kk, (int)chunk, gamma, pos_out, neg_out, (int)k, 0, (hipStream_t)hip_stream);
    KGE_HIP(c, hipGetLastError());
    return KGE_OK;
}

int kge_score_noalloc(const kge_config* cfg, const float* ent, const float* rel,
                      const int64_t* h, const int64_t* r, const int64_t* t, int64_t b,
                      const int64_t* neg, int64_t k, int64_t chunk, int32_t neg_side, float gamma,
                      void* hip_stream, float* pos_out, float* neg_out) {
    if (!cfg) return fail(nullptr, KGE_ERR_INVALID_ARG, "null configuration%s");
    const int m = cfg->model;
    if (m != KGE_TRANSE_L2 && m != KGE_TRANSE_L1 && m != KGE_DISTMULT && m != KGE_COMPLEX && m != KGE_ROTATE)
        return fail(nullptr, KGE_ERR_UNSUPPORTED, "kge_score_noalloc serves TransE-L1/L2, DistMult, ComplEx and RotatE%s");
    if (cfg->gemm_input != 0) return fail(nullptr, KGE_ERR_UNSUPPORTED, "kge_score_noalloc takes fp32 operands only%s");
    const bool cplx = m == KGE_COMPLEX || m == KGE_ROTATE;
    if (cfg->ent_dim <= 0 || cfg->ent_dim > 1024 || cfg->ent_dim % (cplx ? 8 : 4) != 0)
        return fail(nullptr, KGE_ERR_INVALID_ARG, "ent_dim must be a multiple of 4 (8 for ComplEx/RotatE), at most 1024%s");
    if (cfg->rel_dim != (m == KGE_ROTATE ? cfg->ent_dim / 2 : cfg->ent_dim))
        return fail(nullptr, KGE_ERR_INVALID_ARG, "rel_dim must be ent_dim (ent_dim/2 for RotatE)%s");
    if (cfg->num_entities <= 0 || cfg->num_relations <= 0 || cfg->num_entities >= (1ll << 32) ||
        cfg->num_relations >= (1ll << 32))
        return fail(nullptr, KGE_ERR_INVALID_ARG, "table row counts must be in [1, 2^32)%s");
    if (!ent || !rel || !h || !r || !t) return fail(nullptr, KGE_ERR_INVALID_ARG, "null table or id pointer%s");
    if (b <= 0 || chunk <= 0 || b % chunk != 0) return fail(nullptr, KGE_ERR_INVALID_ARG, "b must be a positive multiple of chunk%s");
    if (k < 0 || (neg_out && k == 0)) return fail(nullptr, KGE_ERR_INVALID_ARG, "k out of range%s");
    if (neg_out && !neg) return fail(nullptr, KGE_ERR_INVALID_ARG, "neg is null%s");
    if (neg_side != KGE_NEG_TAIL && neg_side != KGE_NEG_HEAD) return fail(nullptr, KGE_ERR_INVALID_ARG, "neg_side must be 0 or 1%s");
    const int64_t kk = neg_out ? k : 0, n_neg = (b / chunk) * kk;
    if (b > (1 << 24) || n_neg > (1 << 24) || kk > (1 << 24)) return fail(nullptr, KGE_ERR_WORKSPACE, "b or (b/chunk)*k beyond 2^24%s");
    // layout of the scratch array for this call: o rows | staged corrupting rows | six small vectors
    const size_t D = (size_t)cfg->ent_dim, B = (size_t)b, NR = (size_t)(n_neg > 0 ? n_neg : 1);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    const size_t o_O = take(B * D * 4), o_N = take(NR * D * 4), o_fpos = take(B * 4), o_on2 = take(B * 4);
    const size_t o_nn2 = take(NR * 4), o_cpos = take(B * 4), o_idp = take(B * 4), o_rl = take(B * 4);
    if (off > KGE_NOALLOC_SCRATCH_BYTES)
        return fail(nullptr, KGE_ERR_WORKSPACE, "kge_score_noalloc: 4 * ent_dim * (b + (b/chunk)*k) bytes of rows (plus 24 bytes per row) exceed its 8 MiB of scratch memory%s");

    int ndev = 0;
    KGE_HIP(nullptr, hipGetDeviceCount(&ndev));
    if (cfg->device < 0 || cfg->device >= ndev) return fail(nullptr, KGE_ERR_INVALID_ARG, "no such device%s");
    KGE_HIP(nullptr, hipSetDevice(cfg->device));
    void* base_v = nullptr;
    KGE_HIP(nullptr, scratch_address(cfg->device, &base_v));
    char* base = (char*)base_v;

    // a context that lives on this call's stack and owns nothing: its buffers are pieces of the scratch array.
    // Every piece that a kernel of this call reads has been written by an earlier kernel of the same call (the gather
    // launch fills all of them), so nothing has to be cleared between calls.
    kge_ctx c;
    memset(&c, 0, sizeof(c));
    c.cfg = *cfg;
    c.cfg.validate_indices = 0;  // there is no context to report to: ids are clamped into their tables, as always
    c.cfg.adagrad_mode = 0; c.cfg.loss = KGE_LOSS_LOGISTIC; c.cfg.adv_temperature = 0.f;
    c.cfg.max_batch = (int32_t)b; c.cfg.max_neg_per_chunk = (int32_t)kk; c.cfg.max_chunks = (int32_t)(b / chunk);
    c.ld_s = (int)kk;
    c.O = (float*)(base + o_O); c.Nst = (float*)(base + o_N); c.fpos = (float*)(base + o_fpos);
    c.o_n2 = (float*)(base + o_on2); c.n_n2 = (float*)(base + o_nn2); c.cpos = (float*)(base + o_cpos);
    c.inv_dpos = (float*)(base + o_idp); c.row_loss = (float*)(base + o_rl);
    const StepIds ids = direct_ids(h, r, t, (int)b, neg, (int)n_neg, neg_side, nullptr);
    forward(&c, ent, rel, ids, (int)kk, (int)chunk, gamma, pos_out, neg_out, (int)k, 0, (hipStream_t)hip_stream);
    KGE_HIP(nullptr, hipGetLastError());
    return KGE_OK;
}

int kge_rank(kge_ctx* c, const float* ent, const float* rel,
             const int64_t* h, const int64_t* r, const int64_t* t, int64_t b,
             const int64_t* neg, int64_t k, int64_t chunk, int32_t neg_side, float gamma,
             void* hip_stream, int32_t* rank_out) {
    if (!c) return KGE_ERR_INVALID_ARG;
    c->err[0] = 0;
    if (!rank_out) return fail(c, KGE_ERR_INVALID_ARG, "rank_out is null%s");
    const int rc = check_batch(c, ent, rel, h, r, t, b, neg, k, chunk, neg_side, true);
    if (rc != KGE_OK) return rc;
    KGE_HIP(c, hipSetDevice(c->cfg.device));
    const StepIds ids = direct_ids(h, r, t, (int)b, neg, (int)((b / chunk) * k), neg_side, nullptr);
    hipStream_t st = (hipStream_t)hip_stream;
    if (is_gemm_model(c->cfg.model) && kge_gemm_forward_can_rank(c)) {
        // the gather launch sets every rank to 1, the forward launch adds the candidates that score higher
        c->rank_out = rank_out;
        forward(c, ent, rel, ids, (int)k, (int)chunk, gamma, nullptr, c->S, c->ld_s, 3, st);
        c->rank_out = nullptr;
    } else {
        forward(c, ent, rel, ids, (int)k, (int)chunk, gamma, nullptr, c->S, c->ld_s, 0, st);
        kge_launch_rank(c, (int)b, (int)k, rank_out, st);
    }
    KGE_HIP(c, hipGetLastError());
    return KGE_OK;
}

int kge_rank_metrics(const int32_t* ranks, int64_t n, double* metrics_out, void* hip_stream) {
    if (!ranks || !metrics_out || n <= 0) return fail(nullptr, KGE_ERR_INVALID_ARG, "null pointer or no ranks%s");
    kge_launch_rank_metrics(ranks, n, metrics_out, (hipStream_t)hip_stream);
    if (hipGetLastError() != hipSuccess) return fail(nullptr, KGE_ERR_DEVICE, "launch of the metrics kernel failed%s");
    return KGE_OK;
}

int kge_get_dedup(kge_ctx* c, int32_t which, int64_t* uniq_out, int32_t* count_out, int64_t* n_unique_out,
                  void* hip_stream) {
    if (!c) return KGE_ERR_INVALID_ARG;
    c->err[0] = 0;
    if ((which != 0 && which != 1) || !uniq_out || !count_out || !n_unique_out)
        return fail(c, KGE_ERR_INVALID_ARG, "bad argument to kge_get_dedup%s");
    if (c->last_ent_keys == 0) return fail(c, KGE_ERR_INVALID_ARG, "no training step has run on this context%s");
    KGE_HIP(c, hipSetDevice(c->cfg.device));
    kge_launch_dedup_export(c, which, uniq_out, count_out, n_unique_out, (hipStream_t)hip_stream);
    KGE_HIP(c, hipGetLastError());
    return KGE_OK;
}

int kge_check_indices(kge_ctx* c, void* hip_stream) {
    if (!c) return KGE_ERR_INVALID_ARG;
    c->err[0] = 0;
    KGE_HIP(c, hipSetDevice(c->cfg.device));
    hipStream_t st = (hipStream_t)hip_stream;
    int flag = 0;
    KGE_HIP(c, hipMemcpyAsync(&flag, c->flags, sizeof(int), hipMemcpyDeviceToHost, st));
    KGE_HIP(c, hipStreamSynchronize(st));
    if (flag) {
        KGE_HIP(c, hipMemsetAsync(c->flags, 0, sizeof(int), st));
        KGE_HIP(c, hipStreamSynchronize(st));
        return fail(c, KGE_ERR_INDEX_RANGE, "an id was outside its table%s");
    }
    return KGE_OK;
}

int kge_profile(kge_ctx* c, int32_t enable) {
    if (!c) return KGE_ERR_INVALID_ARG;
    c->err[0] = 0;
    KGE_HIP(c, hipSetDevice(c->cfg.device));
    if (enable && !c->prof_ev[0][0]) {
        for (int s = 0; s < KGE_PROF_SLOTS; ++s)
            for (int e = 0; e < 2; ++e) KGE_HIP(c, hipEventCreate(&c->prof_ev[s][e]));
    }
    c->prof_on = enable != 0;
    for (int s = 0; s < KGE_PROF_SLOTS; ++s) c->prof_ms[s] = 0.0;
    c->prof_steps = 0;
    return KGE_OK;
}

int kge_profile_read(kge_ctx* c, double* ms_out, int64_t* steps_out) {
    if (!c || !ms_out || !steps_out) return KGE_ERR_INVALID_ARG;
    for (int s = 0; s < KGE_PROF_SLOTS; ++s) ms_out[s] = c->prof_ms[s];
    *steps_out = c->prof_steps;
    return KGE_OK;
}

const char* kge_profile_slot_name(int32_t slot) {
    static const char* names[KGE_PROF_SLOTS] = {"gather", "neg_score", "loss", "neg_backward", "chain", "sort", "update", "phi", "rel_update"};
    return slot >= 0 && slot < KGE_PROF_SLOTS ? names[slot] : "";
}

int kge_sample_steps(const kge_sampler* sp, int64_t first_step, int64_t n_steps, int64_t* h, int64_t* r, int64_t* t,
                     int64_t* neg, int32_t* sides, void* stream) {
    if (!sp || !sp->triples || !h || !r || !t) return fail(nullptr, KGE_ERR_INVALID_ARG, "null sampler, triple list or output%s");
    if (sp->n_triples <= 0 || sp->n_triples >= ((int64_t)1 << 32) || sp->num_entities <= 0 ||
        sp->num_entities >= ((int64_t)1 << 32))
        return fail(nullptr, KGE_ERR_INVALID_ARG, "n_triples and num_entities must be in (0, 2^32)%s");
    if (sp->batch <= 0 || sp->n_chunks <= 0 || sp->neg_per_chunk < 0 || sp->n_degree < 0 ||
        sp->n_degree > sp->neg_per_chunk || sp->side_mode < 0 || sp->side_mode > 2)
        return fail(nullptr, KGE_ERR_INVALID_ARG, "batch, n_chunks, neg_per_chunk, n_degree or side_mode out of range%s");
    if (sp->neg_per_chunk > 0 && !neg) return fail(nullptr, KGE_ERR_INVALID_ARG, "neg is null%s");
    if (first_step < 0 || n_steps < 0) return fail(nullptr, KGE_ERR_INVALID_ARG, "negative step range%s");
    if (n_steps == 0) return KGE_OK;
    if (kge_sample_launch(sp, first_step, n_steps, h, r, t, neg, sides, (hipStream_t)stream) != KGE_OK)
        return fail(nullptr, KGE_ERR_DEVICE, "launch of the sampling kernel failed%s");
    return KGE_OK;
}

const char* kge_last_error(const kge_ctx* c) { return c ? c->err : g_create_err; }

int64_t kge_workspace_bytes(const kge_ctx* c) { return c ? c->ws_bytes : 0; }

int64_t kge_graph_captures(const kge_ctx* c) { return c ? c->graph_captures : 0; }

}  // extern "C"
