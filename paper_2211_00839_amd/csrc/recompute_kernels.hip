// Gain sweep with the similarity recomputed on the fly, for classes whose S is
// not stored: every 256 x 128 tile of S = exp(-|x_j - x_v|^2 / (2 sigma^2)) is
// produced by the matrix cores from the feature rows (same main loop and same
// epilogue arithmetic as the similarity build, so the values are bit-identical
// to it) and consumed in registers by the facility-location gain of
// Algorithm 1's GreedyStep; S is never written.  Included by rcd_lib.hip after
// greedy_kernels.hip and similarity_kernels.hip.
#include <hip/hip_runtime.h>
#include "rcd_state.h"

namespace {

// One (class, 128-candidate tile, row chunk) item.  KS = blocks evaluated.
template <typename T, bool FAST, int KS>
__device__ __forceinline__ void recompute_body(const RcdClass &st, int tile, int chunk, unsigned char *lds,
                                               float *cur_s /* KS x 256 */, float *sq_s /* 256 */)
{
    using namespace sim;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int n = st.n, ld = st.ld, d = st.d, nneed = st.nneed;
    const long long ldx = st.ldx64;
    const T *__restrict__ X = reinterpret_cast<const T *>(st.X);
    const gci32 xi = (gci32)st.x_index;
    const gci32 perm = (gci32)st.perm;
    const gcf32 sq = (gcf32)st.sq;
    const bool vec_ok = FAST;

    int kb[KS];
#pragma unroll
    for (int i = 0; i < KS; ++i) kb[i] = st.need[i < nneed ? i : nneed - 1];

    // candidates of this tile: B operand rows, and for the epilogue the sample and norm of my two columns
    int brow[2];
    const T *gp[6];            // FAST: this lane's six chunk addresses of a stage (A part refreshed per row tile)
    int a_trow[6], a_chunk[6];
    if constexpr (FAST) {
#pragma unroll
        for (int u = 0; u < 6; ++u) {
            dma_slot(wave, u, lane, &a_trow[u], &a_chunk[u]);
            if (a_trow[u] >= BM) {
                int v = perm[tile * RCD_TILE_RC + a_trow[u] - BM];
                v = min(max(v, 0), n - 1);
                gp[u] = X + (size_t)(xi ? xi[v] : v) * ldx + a_chunk[u] * (CHUNK / (int)sizeof(T));
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            int v = perm[tile * RCD_TILE_RC + (tid >> 2) + 64 * u];
            v = min(max(v, 0), n - 1);
            brow[u] = xi ? xi[v] : v;
        }
    }
    int vcol[2];
    float sqv[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        int v = perm[tile * RCD_TILE_RC + wc * 64 + b * 32 + (lane & 31)];
        v = min(max(v, 0), n - 1);
        vcol[b] = v;
        sqv[b] = sq[v] * st.exp_scale;
    }
    const float exp_scale = st.exp_scale;
    const float scale2 = -2.f * exp_scale;

    float gsum[KS][2];
#pragma unroll
    for (int i = 0; i < KS; ++i) { gsum[i][0] = 0.f; gsum[i][1] = 0.f; }

    const int row_begin = chunk * st.rpc;
    const int row_end = min(n, row_begin + st.rpc);
    for (int i0 = row_begin; i0 < row_end; i0 += RCD_ROWS_RC) {
        // coverage values and norms of the 256 rows (rows past n: +inf coverage = no gain).
        // In the fast path they are staged after the main loop, in the LDS it has freed.
        auto stage_rows = [&]() {
            const int i = i0 + tid;
            sq_s[tid] = i < n ? sq[i] * exp_scale : 0.f;
#pragma unroll
            for (int k = 0; k < KS; ++k)
                cur_s[k * RCD_ROWS_RC + tid] = i < n ? ((gcf32)st.cur)[(size_t)kb[k] * ld + i] : __builtin_inff();
        };
        f32x16 acc[4][2];
        __syncthreads();       // the previous tile's epilogue is done with cur_s / sq_s
        if constexpr (FAST) {
#pragma unroll
            for (int u = 0; u < 6; ++u)
                if (a_trow[u] < BM) {
                    const int ai = min(i0 + a_trow[u], n - 1);
                    gp[u] = X + (size_t)(xi ? xi[ai] : ai) * ldx + a_chunk[u] * (CHUNK / (int)sizeof(T));
                }
            gram_mainloop_dma<T>(gp, d, lds, acc);   // ends with a barrier: the ring is free
            stage_rows();
            __syncthreads();
        } else {
            stage_rows();
            int arow[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int ai = min(i0 + (tid >> 2) + 64 * u, n - 1);
                arow[u] = xi ? xi[ai] : ai;
            }
            gram_mainloop<T, false>(X, ldx, d, vec_ok, arow, brow, lds, acc);   // ends with a barrier
        }

        // does any candidate of this tile sit among these 256 rows?  (its own similarity is exactly 1)
        const bool maybe_diag = __any((vcol[0] >= i0 && vcol[0] < i0 + RCD_ROWS_RC) ||
                                      (vcol[1] >= i0 && vcol[1] < i0 + RCD_ROWS_RC));
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int rl = wr * 128 + a * 32 + rq * 8 + (lane >> 5) * 4;   // 4 consecutive rows rl..rl+3
                const float4 sqi = *reinterpret_cast<const float4 *>(sq_s + rl);
                float s[2][4];
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const float q[4] = {sqi.x, sqi.y, sqi.z, sqi.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        s[b][e] = rbf_value(acc[a][b][rq * 4 + e], q[e], sqv[b], scale2);
                        if (maybe_diag && i0 + rl + e == vcol[b]) s[b][e] = 1.f;
                    }
                }
#pragma unroll
                for (int k = 0; k < KS; ++k) {
                    const float4 c = *reinterpret_cast<const float4 *>(cur_s + k * RCD_ROWS_RC + rl);
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        gsum[k][b] += clamp01(s[b][0] - c.x);
                        gsum[k][b] += clamp01(s[b][1] - c.y);
                        gsum[k][b] += clamp01(s[b][2] - c.z);
                        gsum[k][b] += clamp01(s[b][3] - c.w);
                    }
                }
            }
        }
    }

    // Reduce: the two half-waves hold the same columns over different rows, and so do
    // the waves wr = 0 and 1.  Fixed order: lower half + upper half, then wr 0 + wr 1.
    __syncthreads();
    float *red = cur_s;   // reuse: [wr 2][KS][128 columns]
#pragma unroll
    for (int k = 0; k < KS; ++k)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const float other = __shfl_xor(gsum[k][b], 32);
            const float tot = (lane < 32) ? gsum[k][b] + other : other + gsum[k][b];
            if (lane < 32) red[(wr * KS + k) * RCD_TILE_RC + wc * 64 + b * 32 + lane] = tot;
        }
    __syncthreads();
    const gf32 part = (gf32)st.part + (size_t)chunk * st.K * ld + (size_t)tile * RCD_TILE_RC;
    for (int e = tid; e < KS * RCD_TILE_RC; e += 256) {
        const int k = e / RCD_TILE_RC, c = e % RCD_TILE_RC;
        if (k < nneed) {
            const float v = red[(0 * KS + k) * RCD_TILE_RC + c] + red[(1 * KS + k) * RCD_TILE_RC + c];
            int kk = kb[0];
#pragma unroll
            for (int i = 0; i < KS; ++i)
                if (i == k) kk = kb[i];
            dev_store(part + (size_t)kk * ld + c, v);
        }
    }
}

} // namespace

template <typename T, bool FAST, bool FUSE>
__global__ void __launch_bounds__(256, 2)
rcd_k_round_rc(RcdClass *__restrict__ classes, RcdPlan *__restrict__ plans, int buf)
{
    // fast path: the coverage/norm staging area aliases the start of the (then idle) stage ring
    constexpr int ROWS_BYTES = (RCD_KMAX + 1) * RCD_ROWS_RC * 4;
    __shared__ __attribute__((aligned(16))) unsigned char lds[FAST ? sim::DMA_LDS_BYTES : 2 * sim::STAGE_BYTES + ROWS_BYTES];
    float *cur_s = reinterpret_cast<float *>(FAST ? lds : lds + 2 * sim::STAGE_BYTES);
    float *sq_s = cur_s + RCD_KMAX * RCD_ROWS_RC;
    static_assert(ROWS_BYTES <= sim::DMA_LDS_BYTES, "row staging area must fit in the stage ring");
    __shared__ StepShared sh;
    __shared__ int s_flag;
    const RcdPlan *plan = plans + buf;
    const int item = blockIdx.x;
    if (item >= plan->items) return;
    const int ncls = plans[0].ncls;
    const int32_t *prefix = plan_prefix(plans, buf);
    const int c = ncls > 1 ? find_class(prefix, ncls, item) : 0;
    RcdClass &st = classes[c];
    const int local = item - prefix[c];
    const int tiles = (st.nR + RCD_TILE_RC - 1) / RCD_TILE_RC;
    const int tile = local % tiles;
    const int chunk = local / tiles;
    const int nneed = st.nneed;
    if (nneed <= 1) recompute_body<T, FAST, 1>(st, tile, chunk, lds, cur_s, sq_s);
    else if (nneed == 2) recompute_body<T, FAST, 2>(st, tile, chunk, lds, cur_s, sq_s);
    else if (nneed <= 4) recompute_body<T, FAST, 4>(st, tile, chunk, lds, cur_s, sq_s);
    else if (nneed <= 8) recompute_body<T, FAST, 8>(st, tile, chunk, lds, cur_s, sq_s);
    else recompute_body<T, FAST, 16>(st, tile, chunk, lds, cur_s, sq_s);
    round_tail<256, RCD_TILE_RC, FUSE>(st, classes, plans, buf, tile, tiles, sh, &s_flag);
}

// Apply kernel of the recompute mode: there is no stored matrix, so the coverage
// update cur_js(j) = max(cur_js(j), S(j, v*)) recomputes the one similarity column
// it needs from the features: one wave per row j, fp32 accumulation, same
// clamp / exp2 arithmetic as the sweep's epilogue.  Row block 0 also moves the
// gains and perm entries and writes the caller's arrays.
template <typename T>
__global__ void __launch_bounds__(256)
rcd_k_apply_rc(RcdClass *__restrict__ classes, int round_no)
{
    RcdClass &st = classes[blockIdx.y];
    if (st.apply_round != round_no) return;
    const int nupd = st.nupd, npatch = st.npatch;
    const int n = st.n, ld = st.ld, K = st.K, d = st.d;
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    const T *X = reinterpret_cast<const T *>(st.X);
    if (j < n) {
        const T *xj = X + (size_t)(st.x_index ? st.x_index[j] : j) * st.ldx64;
        for (int i = 0; i < nupd; ++i) {
            const int v = st.uv[i];
            const T *xv = X + (size_t)(st.x_index ? st.x_index[v] : v) * st.ldx64;
            float dot = 0.f;
            for (int t = lane; t < d; t += 64) dot = fmaf(sim::to_f32(xj[t]), sim::to_f32(xv[t]), dot);
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) dot += __shfl_xor(dot, off);
            if (lane == 0) {
                const float s = (j == v) ? 1.f
                                         : sim::rbf_value(dot, st.sq[j] * st.exp_scale, st.sq[v] * st.exp_scale,
                                                          -2.f * st.exp_scale);
                float *c = st.cur + (size_t)st.ujs[i] * ld + j;
                if (s > *c) *c = s;
            }
        }
    }
    if (blockIdx.x == 0) {
        const int tid = threadIdx.x;
        for (int e = tid; e < npatch * (K + 1); e += 256) {
            const int i = e / (K + 1), k = e % (K + 1);
            const int dpos = st.ppos[i], spos = st.psrc[i];
            if (k < K) st.gain[(size_t)k * ld + dpos] = st.gain[(size_t)k * ld + spos];
            else st.perm[dpos] = st.perm[spos];
        }
        if (tid < nupd) {
            const int v = st.uv[tid];
            const int oi = st.out_index ? st.out_index[v] : v;
            st.assign_out[oi] = st.ujs[tid];
            if (st.order_out) st.order_out[oi] = st.ut[tid];
        }
    }
}
