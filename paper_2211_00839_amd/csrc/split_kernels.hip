// Class split of Algorithm 1 ("Split the ground set V into V_1..V_L according to
// class labels"): a stable counting sort of sample indices by label, so that
// inside every class the samples keep the caller's order.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "rcd_state.h"

namespace split {

constexpr int CHUNK = 1024;   // samples per chunk, one wave per chunk

// chunk_hist[chunk][l] = number of samples with label l in the chunk; flags bad labels.
// allow_unassigned: a label of -1 is not an error, the sample just belongs nowhere (worker shards of a
// partition that left samples over).
__global__ void __launch_bounds__(64)
k_hist(const int32_t *__restrict__ labels, long long N, int L, int32_t *__restrict__ chunk_hist, RcdPlan *plan,
       int allow_unassigned = 0)
{
    extern __shared__ int s_cnt[];
    const int lane = threadIdx.x;
    for (int l = lane; l < L; l += 64) s_cnt[l] = 0;
    __syncthreads();
    const long long base = (long long)blockIdx.x * CHUNK;
    int bad = 0;
    for (int g = 0; g < CHUNK / 64; ++g) {
        const long long i = base + g * 64 + lane;
        if (i < N) {
            const int lab = labels[i];
            if (lab >= 0 && lab < L) atomicAdd(&s_cnt[lab], 1);
            else if (!(allow_unassigned && lab == -1)) bad = 1;
        }
    }
    __syncthreads();
    for (int l = lane; l < L; l += 64) chunk_hist[(size_t)blockIdx.x * L + l] = s_cnt[l];
    if (bad) plan->bad = 1;
}

// Per class: exclusive prefix of chunk_hist over chunks (in place) and the class total.
__global__ void __launch_bounds__(256)
k_scan(int32_t *__restrict__ chunk_hist, int nchunks, int L, int32_t *__restrict__ class_count)
{
    const int l = blockIdx.x * 256 + threadIdx.x;
    if (l >= L) return;
    int run = 0;
    for (int c = 0; c < nchunks; ++c) {
        const int v = chunk_hist[(size_t)c * L + l];
        chunk_hist[(size_t)c * L + l] = run;
        run += v;
    }
    class_count[l] = run;
}

// idx[class_offset[l] + rank] = i, rank = number of earlier samples with label l.
__global__ void __launch_bounds__(64)
k_scatter(const int32_t *__restrict__ labels, long long N, int L, const int32_t *__restrict__ chunk_base,
          const int32_t *__restrict__ class_offset, int32_t *__restrict__ idx)
{
    extern __shared__ int s_cnt[];
    const int lane = threadIdx.x;
    for (int l = lane; l < L; l += 64) s_cnt[l] = chunk_base[(size_t)blockIdx.x * L + l] + class_offset[l];
    __syncthreads();
    const long long base = (long long)blockIdx.x * CHUNK;
    for (int g = 0; g < CHUNK / 64; ++g) {
        const long long i = base + g * 64 + lane;
        const int lab = i < N ? labels[i] : -1;
        unsigned long long todo = __ballot(lab >= 0 && lab < L);
        while (todo) {
            const int leader = __ffsll((long long)todo) - 1;
            const int l0 = __shfl(lab, leader);
            const unsigned long long same = __ballot(lab == l0);
            const int start = s_cnt[l0];
            __syncthreads();
            if (lab == l0) {
                const int rank = __popcll(same & ((1ull << lane) - 1ull));
                idx[start + rank] = (int32_t)i;
            }
            if (lane == leader) s_cnt[l0] = start + __popcll(same);
            __syncthreads();
            todo &= ~same;
        }
    }
}

} // namespace split
