// Link-prediction evaluation on top of the forward path (paper Sec. 5, evaluation protocol: a test triple is ranked
// among the triples obtained by replacing its tail (head) with sampled corrupting entities, no filtering).
//   rank_i = 1 + #{ j : f-_ij > f+_i }
// and from the ranks Hit@1, Hit@3, Hit@10 (share of ranks <= 1, 3, 10), MR (mean rank) and MRR (mean of 1/rank).
#include "kge_common.h"

namespace {

// one wave per positive: count the negatives of its row that score strictly higher
__global__ __launch_bounds__(256) void k_rank(const float* fpos, const float* S, int ld_s, int b, int k, int32_t* rank_out) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= b) return;
    const float fp = fpos[i];
    const float* s = S + (int64_t)i * ld_s;
    int cnt = 0;
    for (int j = lane; j < k; j += 64) cnt += s[j] > fp ? 1 : 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
    if (lane == 0) rank_out[i] = 1 + cnt;
}

// one block; integer sums are exact, the sum of reciprocals is a fixed-order tree in fp64
__global__ __launch_bounds__(1024) void k_rank_metrics(const int32_t* ranks, int64_t n, double* out) {
    __shared__ double s_rr[1024];
    __shared__ unsigned long long s_cnt[4][1024];
    const int tid = threadIdx.x;
    double rr = 0.0;
    unsigned long long h1 = 0, h3 = 0, h10 = 0, sum = 0;
    for (int64_t i = tid; i < n; i += 1024) {
        const int r = ranks[i];
        h1 += r <= 1; h3 += r <= 3; h10 += r <= 10; sum += (unsigned long long)r;
        rr += 1.0 / (double)r;
    }
    s_rr[tid] = rr; s_cnt[0][tid] = h1; s_cnt[1][tid] = h3; s_cnt[2][tid] = h10; s_cnt[3][tid] = sum;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if (tid < o) {
            s_rr[tid] += s_rr[tid + o];
#pragma unroll
            for (int q = 0; q < 4; ++q) s_cnt[q][tid] += s_cnt[q][tid + o];
        }
        __syncthreads();
    }
    if (tid == 0) {
        const double dn = n > 0 ? (double)n : 1.0;
        out[0] = (double)s_cnt[0][0] / dn;
        out[1] = (double)s_cnt[1][0] / dn;
        out[2] = (double)s_cnt[2][0] / dn;
        out[3] = (double)s_cnt[3][0] / dn;
        out[4] = s_rr[0] / dn;
    }
}

}  // namespace

void kge_launch_rank(kge_ctx* c, int b, int k, int32_t* rank_out, hipStream_t st) {
    hipLaunchKernelGGL(k_rank, dim3((b + 3) / 4), dim3(256), 0, st, c->fpos, c->S, c->ld_s, b, k, rank_out);
}

void kge_launch_rank_metrics(const int32_t* ranks, int64_t n, double* out, hipStream_t st) {
    hipLaunchKernelGGL(k_rank_metrics, dim3(1), dim3(1024), 0, st, ranks, n, out);
}
