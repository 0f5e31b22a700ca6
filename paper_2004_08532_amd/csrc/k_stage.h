// Staging of table rows for the staged-rows path of the training step (see kge_staged_path): one wavefront copies one
// row, by its position in the step's row list
//     [0, b) head rows | [b, 2b) tail rows | [2b, 2b + n_neg) corrupting rows | then b relation rows,
// the first three in the order of the entity key list, so that position p of that list is row p here.
#pragma once
#include "kge_common.h"

namespace {

struct StageArgs {
    const float* E;
    const float* R;
    float* Hs;
    float* Rs;
    float* Ts;
    float* Nst;
    int b, n_neg, D, Dr;
    int64_t n_ent, n_rel;
};

__device__ __forceinline__ int64_t stage_clamp(int64_t id, int64_t n) { return id < 0 ? 0 : (id >= n ? n - 1 : id); }

// Is id among the ascending keys[0 .. n)?  The whole wave asks for one id: 64 probes per round narrow the range by a
// factor of 64 (two dependent rounds for the few thousand keys of a step).
__device__ __forceinline__ bool wave_contains(const uint32_t* keys, int n, uint32_t id, int lane) {
    int lo = 0, len = n;  // if id is present it is in [lo, lo + len)
    while (len > 64) {
        const int stride = (len + 63) >> 6;
        const int idx = lo + lane * stride;
        const bool le = idx < lo + len && keys[idx] <= id;
        const unsigned long long m = __ballot(le);
        if (m == 0) return false;  // smaller than every key of the range
        const int nlo = lo + (__popcll(m) - 1) * stride;  // the keys are ascending: the lanes that say yes are the first ones
        len = min(stride, lo + len - nlo);
        lo = nlo;
    }
    const bool eq = lane < len && keys[lo + lane] == id;
    return __ballot(eq) != 0;
}

// Destination and source of row-list position p; returns the row length in floats (0: nothing to do).
// skip_e / skip_r: ascending key lists (n_skip_e / n_skip_r entries, may be null) of rows that somebody else stages.
__device__ __forceinline__ void stage_row(const StageArgs& a, const StepView& sv, int p, int lane,
                                          const uint32_t* skip_e, int n_skip_e, const uint32_t* skip_r, int n_skip_r) {
    const int nb = a.b, n_ent_rows = 2 * nb + a.n_neg;
    if (p >= n_ent_rows + nb) return;
    const float* src;
    float* dst;
    int len;
    if (p < n_ent_rows) {
        const int64_t raw = p < nb ? sv.h[p] : (p < 2 * nb ? sv.t[p - nb] : sv.neg[p - 2 * nb]);
        const int64_t id = stage_clamp(raw, a.n_ent);
        if (skip_e && wave_contains(skip_e, n_skip_e, (uint32_t)id, lane)) return;
        src = a.E + id * (int64_t)a.D;
        dst = p < nb ? a.Hs + (int64_t)p * a.D : (p < 2 * nb ? a.Ts + (int64_t)(p - nb) * a.D : a.Nst + (int64_t)(p - 2 * nb) * a.D);
        len = a.D;
    } else {
        const int i = p - n_ent_rows;
        const int64_t id = stage_clamp(sv.r[i], a.n_rel);
        if (skip_r && wave_contains(skip_r, n_skip_r, (uint32_t)id, lane)) return;
        src = a.R + id * (int64_t)a.Dr;
        dst = a.Rs + (int64_t)i * a.Dr;
        len = a.Dr;
    }
    const int n4 = len / 4;  // rows are at most 1024 floats: four 16-byte pieces per lane, all asked for before the first is used
    float4 x[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) x[it] = ld4(src + 4 * (lane + it * 64 < n4 ? lane + it * 64 : 0));
#pragma unroll
    for (int it = 0; it < 4; ++it)
        if (lane + it * 64 < n4) st4(dst + 4 * (lane + it * 64), x[it]);
}

}  // namespace
