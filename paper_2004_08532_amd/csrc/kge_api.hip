// C ABI of libkge: argument checks, workspace, and the order in which the kernels of one step are enqueued.
// See include/kge.h for the contract of each entry point.
#include <stdio.h>
#include <string.h>

#include <new>

#include "kge_common.h"

namespace {

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

bool is_gemm_model(int m) { return m == KGE_TRANSE_L2 || m == KGE_DISTMULT || m == KGE_COMPLEX; }

__global__ void k_validate(const int64_t* h, const int64_t* r, const int64_t* t, int b, const int64_t* neg, int n_neg,
                           int64_t n_ent, int64_t n_rel, int* flag) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    bool bad = false;
    if (i < b) bad = h[i] < 0 || h[i] >= n_ent || t[i] < 0 || t[i] >= n_ent || r[i] < 0 || r[i] >= n_rel;
    if (i < n_neg) bad = bad || neg[i] < 0 || neg[i] >= n_ent;
    if (bad) atomicOr(flag, 1);
}

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

void forward(kge_ctx* c, const float* ent, const float* rel, const int64_t* h, const int64_t* r, const int64_t* t,
             int b, const int64_t* neg, int k, int chunk, int side, float gamma, float* pos_out, float* neg_out,
             int ld_out, int dist_mode, hipStream_t st) {
    const int n_neg = (b / chunk) * k;
    if (c->cfg.validate_indices) {
        const int n = b > n_neg ? b : n_neg;
        hipLaunchKernelGGL(k_validate, dim3((n + 255) / 256), dim3(256), 0, st, h, r, t, b, neg, n_neg,
                           c->cfg.num_entities, c->cfg.num_relations, c->flags);
    }
    kge_launch_gather(c, ent, rel, h, r, t, b, neg, n_neg, side, gamma, pos_out, st);
    if (neg_out && k > 0) {
        if (is_gemm_model(c->cfg.model)) kge_gemm_neg_score(c, b, k, chunk, gamma, neg_out, ld_out, dist_mode, st);
        else kge_pair_neg_score(c, b, k, chunk, gamma, neg_out, ld_out, st);
    }
}

// ---- optional per-kernel timing (kge_profile): every kernel of a step is bracketed by events on the stream it
// runs on, the stream is synchronised after the step, and the elapsed times are accumulated per slot.
struct ProfScope {
    kge_ctx* c;
    int slot;
    hipStream_t st;
    ProfScope(kge_ctx* c_, int slot_, hipStream_t st_) : c(c_), slot(slot_), st(st_) {
        if (c->prof_on) (void)hipEventRecord(c->prof_ev[slot][0], st);
    }
    ~ProfScope() {
        if (c->prof_on) (void)hipEventRecord(c->prof_ev[slot][1], st);
    }
};

int enqueue_step(kge_ctx* c, float* ent, float* ent_state, float* rel, float* rel_state, const int64_t* h,
                 const int64_t* r, const int64_t* t, int B, const int64_t* neg, int K, int G, int side, float gamma,
                 float lr, hipStream_t st, float* loss_out) {
    const int n_neg = (B / G) * K;
    // the key sort needs only the ids: it runs beside the forward/backward kernels and joins before the update
    KGE_HIP(c, hipEventRecord(c->ev_fork, st));
    KGE_HIP(c, hipStreamWaitEvent(c->side_stream, c->ev_fork, 0));
    {
        ProfScope p(c, KGE_PROF_SORT, c->side_stream);
        kge_launch_sort(c, h, r, t, B, neg, n_neg, c->side_stream);
    }
    KGE_HIP(c, hipEventRecord(c->ev_join, c->side_stream));
    if (c->cfg.validate_indices) {
        const int n = B > n_neg ? B : n_neg;
        hipLaunchKernelGGL(k_validate, dim3((n + 255) / 256), dim3(256), 0, st, h, r, t, B, neg, n_neg,
                           c->cfg.num_entities, c->cfg.num_relations, c->flags);
    }
    {
        ProfScope p(c, KGE_PROF_GATHER, st);
        kge_launch_gather(c, ent, rel, h, r, t, B, neg, n_neg, side, gamma, nullptr, st);
    }
    {
        ProfScope p(c, KGE_PROF_SCORE, st);
        if (is_gemm_model(c->cfg.model)) kge_gemm_neg_score(c, B, K, G, gamma, c->S, c->ld_s, 1, st);
        else kge_pair_neg_score(c, B, K, G, gamma, c->S, c->ld_s, st);
    }
    {
        ProfScope p(c, KGE_PROF_LOSS, st);
        kge_launch_loss(c, B, K, gamma, st);
    }
    {
        ProfScope p(c, KGE_PROF_BACKWARD, st);
        if (is_gemm_model(c->cfg.model)) kge_gemm_neg_backward(c, B, K, G, st);
        else kge_pair_neg_backward(c, B, K, G, st);
    }
    {
        ProfScope p(c, KGE_PROF_CHAIN, st);
        kge_launch_chain(c, ent, rel, h, r, t, B, side, gamma, st);
    }
    KGE_HIP(c, hipStreamWaitEvent(st, c->ev_join, 0));
    {
        ProfScope p(c, KGE_PROF_UPDATE, st);
        kge_launch_update(c, ent, ent_state, rel, rel_state, 2 * B + n_neg, B, lr, B, loss_out, st);
    }
    KGE_HIP(c, hipGetLastError());
    if (c->prof_on) {
        KGE_HIP(c, hipStreamSynchronize(st));
        for (int s = 0; s < KGE_PROF_SLOTS; ++s) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, c->prof_ev[s][0], c->prof_ev[s][1]) == hipSuccess) c->prof_ms[s] += ms;
        }
        c->prof_steps += 1;
    }
    return KGE_OK;
}

}  // namespace

extern "C" {

int kge_create(const kge_config* cfg, kge_ctx** out) {
    if (!cfg || !out) return fail(nullptr, KGE_ERR_INVALID_ARG, "null argument%s");
    *out = nullptr;
    const int m = cfg->model;
    if (m < KGE_TRANSE_L2 || m > KGE_ROTATE) return fail(nullptr, KGE_ERR_INVALID_ARG, "unknown model%s");
    const bool cplx = m == KGE_COMPLEX || m == KGE_ROTATE;
    if (cfg->ent_dim <= 0 || cfg->ent_dim > 1024 || cfg->ent_dim % (cplx ? 8 : 4) != 0)
        return fail(nullptr, KGE_ERR_INVALID_ARG, "ent_dim must be a multiple of 4 (8 for ComplEx/RotatE), at most 1024%s");
    if (cfg->rel_dim != (m == KGE_ROTATE ? cfg->ent_dim / 2 : cfg->ent_dim))
        return fail(nullptr, KGE_ERR_INVALID_ARG, "rel_dim must be ent_dim (ent_dim/2 for RotatE)%s");
    if (cfg->num_entities <= 0 || cfg->num_relations <= 0 || cfg->num_entities >= (1ll << 32) ||
        cfg->num_relations >= (1ll << 32))
        return fail(nullptr, KGE_ERR_INVALID_ARG, "table row counts must be in [1, 2^32)%s");
    if (cfg->max_batch <= 0 || cfg->max_neg_per_chunk < 0 || cfg->max_chunks <= 0 || cfg->max_chunks > cfg->max_batch)
        return fail(nullptr, KGE_ERR_INVALID_ARG, "bad workspace limits%s");
    if ((int64_t)cfg->max_chunks * cfg->max_neg_per_chunk + 2ll * cfg->max_batch > (1 << 24))
        return fail(nullptr, KGE_ERR_INVALID_ARG, "more than 2^24 entity keys per step%s");
    if (cfg->adagrad_mode != 0) return fail(nullptr, KGE_ERR_UNSUPPORTED, "only element-wise Adagrad state is implemented%s");
    if (cfg->gemm_input != 0 && cfg->gemm_input != 1) return fail(nullptr, KGE_ERR_INVALID_ARG, "gemm_input must be 0 or 1%s");
    if (cfg->gemm_input == 1) return fail(nullptr, KGE_ERR_UNSUPPORTED, "bf16 operands are not implemented yet%s");
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
    const size_t o_Ge = take(EK * D * 4), o_Gr = take(B * Dr * 4);
    const size_t o_fpos = take(B * 4), o_on2 = take(B * 4), o_nn2 = take(NR * 4), o_cpos = take(B * 4);
    const size_t o_rl = take(B * 4), o_wrs = take(B * 4);
    const size_t o_ek0 = take(EK * 4), o_ek1 = take(EK * 4), o_ep0 = take(EK * 4), o_ep1 = take(EK * 4);
    const size_t o_rk0 = take(B * 4), o_rk1 = take(B * 4), o_rp0 = take(B * 4), o_rp1 = take(B * 4);
    const size_t o_flags = take(256);
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
    c->cpos = (float*)(base + o_cpos); c->row_loss = (float*)(base + o_rl); c->w_rowsum = (float*)(base + o_wrs);
    c->ekey[0] = (uint32_t*)(base + o_ek0); c->ekey[1] = (uint32_t*)(base + o_ek1);
    c->epos[0] = (uint32_t*)(base + o_ep0); c->epos[1] = (uint32_t*)(base + o_ep1);
    c->rkey[0] = (uint32_t*)(base + o_rk0); c->rkey[1] = (uint32_t*)(base + o_rk1);
    c->rpos[0] = (uint32_t*)(base + o_rp0); c->rpos[1] = (uint32_t*)(base + o_rp1);
    c->flags = (int*)(base + o_flags);

    bool ok = hipMemset(c->ws_base, 0, off) == hipSuccess;
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
    return enqueue_step(c, ent, ent_state, rel, rel_state, h, r, t, (int)b, neg, (int)k, (int)chunk, neg_side, gamma,
                        lr, (hipStream_t)hip_stream, loss_out);
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
    KGE_HIP(c, hipSetDevice(c->cfg.device));
    const int64_t n_neg = (b / chunk) * k;
    for (int64_t s = 0; s < n_steps; ++s) {
        rc = enqueue_step(c, ent, ent_state, rel, rel_state, h + s * b, r + s * b, t + s * b, (int)b, neg + s * n_neg,
                          (int)k, (int)chunk, neg_sides ? neg_sides[s] : KGE_NEG_TAIL, gamma, lr,
                          (hipStream_t)hip_stream, loss_out ? loss_out + s : nullptr);
        if (rc != KGE_OK) return rc;
    }
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
    forward(c, ent, rel, h, r, t, (int)b, neg, kk, (int)chunk, neg_side, gamma, pos_out, neg_out, (int)k, 0,
            (hipStream_t)hip_stream);
    KGE_HIP(c, hipGetLastError());
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
    static const char* names[KGE_PROF_SLOTS] = {"gather", "neg_score", "loss", "neg_backward", "chain", "sort", "update"};
    return slot >= 0 && slot < KGE_PROF_SLOTS ? names[slot] : "";
}

const char* kge_last_error(const kge_ctx* c) { return c ? c->err : g_create_err; }

int64_t kge_workspace_bytes(const kge_ctx* c) { return c ? c->ws_bytes : 0; }

}  // extern "C"
