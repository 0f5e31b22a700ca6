// Step 1 of the mini-batch loop (paper Sec. 3.1) on the device: positive triples and the jointly sampled
// corrupting entities of Sec. 3.3, for any range of steps at once, as id arrays that kge_train_steps consumes.
//
// Every id is a function of (seed, stream tag, step, chunk, slot) alone:
//     key = mix(mix(mix(mix(seed + GOLDEN * tag) + step) + a) + j),   id = floor(key * n / 2^64)
// with `mix` a 64-bit xor-shift / multiply finaliser, so any step can be generated without the ones before it and
// one launch fills thousands of steps.  Streams (tags):
//   1  positives: position j of the mini-batch = triple number floor(key * n_triples / 2^64) of the triple list
//   2  uniform corrupting entities: slot j of chunk a = entity floor(key * num_entities / 2^64)
//   3  degree-proportional corrupting entities (Sec. 3.3): slot j of chunk a = the tail (head, when heads are
//      corrupted) of position floor(key * b / 2^64) of the SAME mini-batch; entities are then drawn in proportion
//      to how often they occur in the batch
// Of the k slots of a chunk the first n_degree use stream 3, the others stream 2.
#include "kge_common.h"

namespace {

constexpr uint64_t GOLDEN = 0x9E3779B97F4A7C15ull;

__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// floor(key * n / 2^64)
__device__ __forceinline__ int64_t scale_to(uint64_t key, uint64_t n) { return (int64_t)__umul64hi(key, n); }

struct SampleArgs {
    kge_sampler s;
    uint64_t base[4];  // mix(seed + GOLDEN * tag) per tag, formed on the host
    int64_t first_step, n_steps;
    int64_t* h;
    int64_t* r;
    int64_t* t;
    int64_t* neg;
    int32_t* sides;
};

__device__ __forceinline__ int side_of(int mode, int64_t step) { return mode == 2 ? (int)(step & 1) : mode; }

__device__ __forceinline__ int64_t position(const SampleArgs& a, uint64_t zs, int64_t j) {
    // zs = mix(base[1] + step); positives use a = 0
    return scale_to(mix64(mix64(zs + 0) + (uint64_t)j), (uint64_t)a.s.n_triples);
}

__global__ __launch_bounds__(256) void k_sample(SampleArgs a) {
    const int b = a.s.batch, k = a.s.neg_per_chunk, per_step = b + a.s.n_chunks * k;
    const int64_t total = a.n_steps * per_step;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int64_t si = idx / per_step;
        const int item = (int)(idx - si * per_step);
        const int64_t step = a.first_step + si;
        const int side = side_of(a.s.side_mode, step);
        const uint64_t zpos = mix64(a.base[1] + (uint64_t)step);
        if (item < b) {
            const int64_t p = position(a, zpos, item);
            a.h[si * b + item] = a.s.triples[3 * p];
            a.r[si * b + item] = a.s.triples[3 * p + 1];
            a.t[si * b + item] = a.s.triples[3 * p + 2];
            if (item == 0 && a.sides) a.sides[si] = side;
        } else {
            const int q = item - b, c = q / k, j = q - c * k;
            int64_t id;
            if (j < a.s.n_degree) {
                const uint64_t key = mix64(mix64(mix64(a.base[3] + (uint64_t)step) + (uint64_t)c) + (uint64_t)j);
                const int64_t pick = scale_to(key, (uint64_t)b);
                const int64_t p = position(a, zpos, pick);
                id = a.s.triples[3 * p + (side == KGE_NEG_HEAD ? 0 : 2)];
            } else {
                const uint64_t key = mix64(mix64(mix64(a.base[2] + (uint64_t)step) + (uint64_t)c) + (uint64_t)j);
                id = scale_to(key, (uint64_t)a.s.num_entities);
            }
            a.neg[si * (int64_t)(a.s.n_chunks * k) + q] = id;
        }
    }
}

}  // namespace

int kge_sample_launch(const kge_sampler* s, int64_t first_step, int64_t n_steps, int64_t* h, int64_t* r, int64_t* t,
                      int64_t* neg, int32_t* sides, hipStream_t st) {
    SampleArgs a;
    a.s = *s;
    for (int tag = 0; tag < 4; ++tag) a.base[tag] = mix64(s->seed + GOLDEN * (uint64_t)tag);
    a.first_step = first_step; a.n_steps = n_steps;
    a.h = h; a.r = r; a.t = t; a.neg = neg; a.sides = sides;
    const int64_t total = n_steps * (int64_t)(s->batch + s->n_chunks * s->neg_per_chunk);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_sample, dim3((unsigned)blocks), dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? KGE_OK : KGE_ERR_DEVICE;
}
