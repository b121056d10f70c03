// Gain sweep with the similarity recomputed on the fly, for classes whose S is
// not stored: every tile of S = exp(-|x_j - x_v|^2 / (2 sigma^2)) (256 rows j x
// 256 candidates v on the fast path, 256 x 128 on the general one) is produced by
// the matrix cores from the feature rows (same main loops and same epilogue
// arithmetic as the similarity build, so the values are bit-identical to it) and
// consumed in registers by the facility-location gain of Algorithm 1's
// GreedyStep; S is never written.  Included by rcd_lib.hip after
// greedy_kernels.hip and similarity_kernels.hip.
#include <hip/hip_runtime.h>
#include "rcd_state.h"

// dynamic LDS of the fast sweep: the stage ring, then per row tile 256 coverage values per block, 256 norms
// and the 256 feature rows of the next row tile
#define RCD_RC_FAST_LDS (sim::pipe::LDS_BYTES + (RCD_KMAX + 2) * RCD_ROWS_RC * 4)

namespace {

// General path: one (class, 128-candidate tile, row chunk) item.  KS = blocks evaluated.
template <typename T, int KS>
__device__ __forceinline__ void recompute_body(const RcdClass &st, int tile, int chunk, unsigned char *lds,
                                               float *cur_s /* KS x 256 */, float *sq_s /* 256 */)
{
    using namespace sim;
    constexpr int TW = RCD_TILE_RC;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int n = st.n, ld = st.ld, d = st.d, nneed = st.nneed;
    const long long ldx = st.ldx64;
    const T *__restrict__ X = reinterpret_cast<const T *>(st.X);
    const gci32 xi = (gci32)st.x_index;
    const gci32 perm = (gci32)st.perm;
    const gcf32 sq = (gcf32)st.sq;
    const bool vec_ok = (reinterpret_cast<uintptr_t>(st.X) & 15) == 0 && ((ldx * (long long)sizeof(T)) % 16) == 0;

    int kb[KS];
#pragma unroll
    for (int i = 0; i < KS; ++i) kb[i] = st.need[i < nneed ? i : nneed - 1];

    // candidates of this tile: B operand rows, and for the epilogue the sample and norm of my two columns
    int brow[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        int v = perm[tile * TW + (tid >> 2) + 64 * u];
        v = min(max(v, 0), n - 1);
        brow[u] = xi ? xi[v] : v;
    }
    int vcol[2];
    float sqv[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        int v = perm[tile * TW + wc * 64 + b * 32 + (lane & 31)];
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
        f32x16 acc[4][2];
        __syncthreads();       // the previous tile's epilogue is done with cur_s / sq_s
        {
            // coverage values and norms of the 256 rows (rows past n: +inf coverage = no gain)
            const int i = i0 + tid;
            sq_s[tid] = i < n ? sq[i] * exp_scale : 0.f;
#pragma unroll
            for (int k = 0; k < KS; ++k)
                cur_s[k * RCD_ROWS_RC + tid] = i < n ? ((gcf32)st.cur)[(size_t)kb[k] * ld + i] : __builtin_inff();
        }
        int arow[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ai = min(i0 + (tid >> 2) + 64 * u, n - 1);
            arow[u] = xi ? xi[ai] : ai;
        }
        gram_mainloop<T>(X, ldx, d, vec_ok, arow, brow, lds, acc);   // ends with a barrier

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
            if (lane < 32) red[(wr * KS + k) * TW + wc * 64 + b * 32 + lane] = tot;
        }
    __syncthreads();
    const gf32 part = (gf32)st.part + (size_t)chunk * st.K * ld + (size_t)tile * TW;
    for (int e = tid; e < KS * TW; e += 256) {
        const int k = e / TW, c = e % TW;
        if (k < nneed) {
            const float v = red[(0 * KS + k) * TW + c] + red[(1 * KS + k) * TW + c];
            int kk = kb[0];
#pragma unroll
            for (int i = 0; i < KS; ++i)
                if (i == k) kk = kb[i];
            dev_store(part + (size_t)kk * ld + c, v);
        }
    }
}

// Fast path (feature rows 16-byte aligned and a multiple of 128 bytes long): one (class,
// 256-candidate tile, row chunk) item on the 256 x 256 pipeline of the similarity build.
// The candidates' rows (the x_j operand, fetched by waves 2 and 3) stay the same for the
// whole item; the x_i operand walks down the chunk's rows 256 at a time.
template <typename T, int KS>
__device__ __forceinline__ void recompute_body_fast(const RcdClass &st, int tile, int chunk, unsigned char *lds)
{
    using namespace sim;
    using namespace sim::pipe;
    constexpr int TW = RCD_TILE_FAST;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wc = wave & 1;
    const int n = st.n, ld = st.ld, nneed = st.nneed;
    const long long ldxb = st.ldx64 * (long long)sizeof(T);
    const unsigned char *__restrict__ X = reinterpret_cast<const unsigned char *>(st.X);
    const gci32 xi = (gci32)st.x_index;
    const gci32 perm = (gci32)st.perm;
    const gcf32 sq = (gcf32)st.sq;
    const int nstage = (int)(((long long)st.d * (int)sizeof(T)) / LINE);
    const long long row_bytes = (long long)nstage * LINE;

    int kb[KS];
#pragma unroll
    for (int i = 0; i < KS; ++i) kb[i] = st.need[i < nneed ? i : nneed - 1];

    Pipe<T> p;
    p.init(lds);
    const bool loads_rows = wave < 2;      // waves 0,1 fetch the x_i rows, waves 2,3 the candidates' rows
    // tile row my u-th load belongs to, 0..255 within its operand, and the byte offset of my
    // chunk inside that row's line (the swizzle only depends on u's parity and the lane)
    auto slot_row = [&](int u) { return ((wave & 1) * NLOAD + u) * 8 + (lane >> 3); };
    auto slot_chunk = [&](int u) { return ((lane & 7) ^ (((lane >> 4) + 4 * (u & 1)) & 7)) * CHUNK; };
    if (loads_rows) {
#pragma unroll
        for (int u = 0; u < NLOAD; ++u) {
            const int ai = min(chunk * st.rpc + slot_row(u), n - 1);
            p.gp[u] = X + (size_t)(xi ? xi[ai] : ai) * ldxb + slot_chunk(u);
        }
    } else {
#pragma unroll
        for (int u = 0; u < NLOAD; ++u) {
            int v = perm[tile * TW + slot_row(u)];
            v = min(max(v, 0), n - 1);
            p.gp[u] = X + (size_t)(xi ? xi[v] : v) * ldxb + slot_chunk(u);
        }
    }
    // for the epilogue: sample and pre-scaled norm of my four columns
    const float exp_scale = st.exp_scale;
    const float scale2 = -2.f * exp_scale;
    int vcol[4];
    float sqv[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        int v = perm[tile * TW + wc * 128 + b * 32 + (lane & 31)];
        v = min(max(v, 0), n - 1);
        vcol[b] = v;
        sqv[b] = sq[v] * exp_scale;
    }
    p.start(nstage);     // after every ordinary load above: waiting for those would wait for these too
    float gsum[KS][4];
#pragma unroll
    for (int i = 0; i < KS; ++i)
#pragma unroll
        for (int b = 0; b < 4; ++b) gsum[i][b] = 0.f;

    // Staging area behind the ring: of the current row tile the coverage values of the evaluated
    // blocks and the squared norms, and the feature rows of the next row tile.  Filled under the
    // k loop by 4-byte loads straight into LDS (a wave's 64 lanes land side by side).
    float *cur_s = reinterpret_cast<float *>(lds + LDS_BYTES);  // KS x 256
    float *sq_s = cur_s + RCD_KMAX * RCD_ROWS_RC;               // 256
    int *idx_s = reinterpret_cast<int *>(sq_s + RCD_ROWS_RC);   // 256
    const unsigned stage_dst = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds + LDS_BYTES +
                               wave * 256;

    const int row_begin = chunk * st.rpc;
    const int row_end = min(n, row_begin + st.rpc);
    for (int i0 = row_begin; i0 < row_end; i0 += RCD_ROWS_RC) {
        const bool more = i0 + RCD_ROWS_RC < row_end;
        const int my_row = i0 + tid;
        {
            const int r = min(my_row, n - 1);
#pragma unroll
            for (int k = 0; k < KS; ++k)
                load_dword_to_lds(st.cur + (size_t)kb[k] * ld + r, stage_dst + k * (RCD_ROWS_RC * 4));
            load_dword_to_lds(st.sq + r, stage_dst + RCD_KMAX * (RCD_ROWS_RC * 4));
            if (more && xi) load_dword_to_lds(st.x_index + min(my_row + RCD_ROWS_RC, n - 1), stage_dst + (RCD_KMAX + 1) * (RCD_ROWS_RC * 4));
        }

        f32x16 acc[4][4];
        p.run(nstage, acc);      // ends with every load landed and a barrier: the ring is free

        // rows past n: +inf coverage = no gain
        if (my_row >= n) {
#pragma unroll
            for (int k = 0; k < KS; ++k) cur_s[k * RCD_ROWS_RC + tid] = __builtin_inff();
        }
        // the next row tile's first stages travel while this one's epilogue runs
        if (more) {
            if (loads_rows) {
#pragma unroll
                for (int u = 0; u < NLOAD; ++u) {
                    const int t = slot_row(u);
                    const int row = xi ? idx_s[t] : min(i0 + RCD_ROWS_RC + t, n - 1);
                    p.gp[u] = X + (size_t)row * ldxb + slot_chunk(u);
                }
            } else {
#pragma unroll
                for (int u = 0; u < NLOAD; ++u) p.gp[u] -= row_bytes;      // back to the candidates' first stage
            }
            p.start(nstage);
        }
        __syncthreads();

        // does any candidate of this tile sit among these 256 rows?  (its own similarity is exactly 1)
        // dv[b]: where my column's own row sits relative to my first row of this row tile
        const int lane_row = wr * 128 + (lane >> 5) * 4;
        int dv[4];
        bool diag = false;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            dv[b] = vcol[b] - i0 - lane_row;
            diag |= vcol[b] >= i0 && vcol[b] < i0 + RCD_ROWS_RC;
        }
        const bool maybe_diag = __any(diag);
        // my rows are lane_row + 32 a + 8 rq + e: one base address per lane, the rest are constants
        const float *sq_lane = sq_s + lane_row;
        const float *cur_lane = cur_s + lane_row;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const float4 sqi = *reinterpret_cast<const float4 *>(sq_lane + (a * 32 + rq * 8));
                const float q[4] = {sqi.x * exp_scale, sqi.y * exp_scale, sqi.z * exp_scale, sqi.w * exp_scale};
                float s[4][4];
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        s[b][e] = rbf_value(acc_read(acc[a][b][rq * 4 + e]), q[e], sqv[b], scale2);
                        if (maybe_diag && dv[b] == a * 32 + rq * 8 + e) s[b][e] = 1.f;
                    }
#pragma unroll
                for (int k = 0; k < KS; ++k) {
                    const float4 c = *reinterpret_cast<const float4 *>(cur_lane + (k * RCD_ROWS_RC + a * 32 + rq * 8));
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        gsum[k][b] += clamp01(s[b][0] - c.x);
                        gsum[k][b] += clamp01(s[b][1] - c.y);
                        gsum[k][b] += clamp01(s[b][2] - c.z);
                        gsum[k][b] += clamp01(s[b][3] - c.w);
                    }
                }
                pin_schedule();
            }
        }
        __syncthreads();       // everyone is done with the staging area before the next row tile refills it
    }

    // Reduce: the two half-waves hold the same columns over different rows, and so do
    // the waves wr = 0 and 1.  Fixed order: lower half + upper half, then wr 0 + wr 1.
    float *red = reinterpret_cast<float *>(lds);   // [wr 2][KS][256 columns]
#pragma unroll
    for (int k = 0; k < KS; ++k)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const float other = __shfl_xor(gsum[k][b], 32);
            const float tot = (lane < 32) ? gsum[k][b] + other : other + gsum[k][b];
            if (lane < 32) red[(wr * KS + k) * TW + wc * 128 + b * 32 + lane] = tot;
        }
    __syncthreads();
    const gf32 part = (gf32)st.part + (size_t)chunk * st.K * ld + (size_t)tile * TW;
    for (int e = tid; e < KS * TW; e += 256) {
        const int k = e / TW, c = e % TW;
        if (k < nneed) {
            const float v = red[(0 * KS + k) * TW + c] + red[(1 * KS + k) * TW + c];
            int kk = kb[0];
#pragma unroll
            for (int i = 0; i < KS; ++i)
                if (i == k) kk = kb[i];
            dev_store(part + (size_t)kk * ld + c, v);
        }
    }
    __syncthreads();           // red is read before the caller's tail reuses the LDS
}

} // namespace

// General path: static LDS, two workgroups per compute unit.
template <typename T, bool FUSE>
__global__ void __launch_bounds__(256, 2)
rcd_k_round_rc(RcdClass *__restrict__ classes, RcdPlan *__restrict__ plans, int buf)
{
    constexpr int ROWS_BYTES = (RCD_KMAX + 1) * RCD_ROWS_RC * 4;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * sim::STAGE_BYTES + ROWS_BYTES];
    float *cur_s = reinterpret_cast<float *>(lds + 2 * sim::STAGE_BYTES);
    float *sq_s = cur_s + RCD_KMAX * RCD_ROWS_RC;
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
    if (nneed <= 1) recompute_body<T, 1>(st, tile, chunk, lds, cur_s, sq_s);
    else if (nneed == 2) recompute_body<T, 2>(st, tile, chunk, lds, cur_s, sq_s);
    else if (nneed <= 4) recompute_body<T, 4>(st, tile, chunk, lds, cur_s, sq_s);
    else if (nneed <= 8) recompute_body<T, 8>(st, tile, chunk, lds, cur_s, sq_s);
    else recompute_body<T, 16>(st, tile, chunk, lds, cur_s, sq_s);
    round_tail<256, RCD_TILE_RC, FUSE>(st, classes, plans, buf, tile, tiles, sh, &s_flag);
}

// Fast path: dynamic LDS of RCD_RC_FAST_LDS bytes (the stage ring, then the staging area of
// a row tile's coverage values and norms), one workgroup per compute unit.
template <typename T, bool FUSE>
__global__ void __launch_bounds__(256, 1)
rcd_k_round_rc_fast(RcdClass *__restrict__ classes, RcdPlan *__restrict__ plans, int buf)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    static_assert(2 * RCD_KMAX * RCD_TILE_FAST * 4 <= sim::pipe::STAGE, "reduction area must fit in one stage");
    static_assert(sizeof(StepShared) + 16 <= sim::pipe::STAGE, "step loop state must fit in one stage");
    StepShared &sh = *reinterpret_cast<StepShared *>(lds + sim::pipe::STAGE);   // second stage: free after the sweep
    int *s_flag = reinterpret_cast<int *>(lds + sim::pipe::STAGE + sizeof(StepShared));
    const RcdPlan *plan = plans + buf;
    const int item = blockIdx.x;
    if (item >= plan->items) return;
    const int ncls = plans[0].ncls;
    const int32_t *prefix = plan_prefix(plans, buf);
    const int c = ncls > 1 ? find_class(prefix, ncls, item) : 0;
    RcdClass &st = classes[c];
    const int local = item - prefix[c];
    const int tiles = (st.nR + RCD_TILE_FAST - 1) / RCD_TILE_FAST;
    const int tile = local % tiles;
    const int chunk = local / tiles;
    const int nneed = st.nneed;
    if (nneed <= 1) recompute_body_fast<T, 1>(st, tile, chunk, lds);
    else if (nneed == 2) recompute_body_fast<T, 2>(st, tile, chunk, lds);
    else if (nneed <= 4) recompute_body_fast<T, 4>(st, tile, chunk, lds);
    else if (nneed <= 8) recompute_body_fast<T, 8>(st, tile, chunk, lds);
    else recompute_body_fast<T, 16>(st, tile, chunk, lds);
    round_tail<256, RCD_TILE_FAST, FUSE>(st, classes, plans, buf, tile, tiles, sh, s_flag);
}

// Apply kernel of the recompute mode: there is no stored matrix, so the coverage
// update cur_js(j) = max(cur_js(j), S(j, v*)) rebuilds the similarity columns it needs
// from the features.  The sweep that follows subtracts these coverage values from tiles
// that the matrix cores produce, so the columns come from the matrix cores too, with the
// same products in the same order: k advances in 32-byte groups, lanes 0-31 of a group
// carry its first 16 bytes and lanes 32-63 the second, one 32x32x16 multiply per group
// (bf16) or four 32x32x2 ones (fp32), one accumulator per element, then the epilogue
// expression every similarity goes through.  An element of a matrix-core product depends
// only on its own row of each operand, so S(j, v*) here is the S(j, v*) of the sweep's
// tiles and of the similarity build, bit for bit (tested).
// One wave = 32 rows j x the samples taken this round (at most 16, one per block; the
// other columns of the 32 repeat the first and are dropped).  grid = (ceil(n / 128), classes).
// Row block 0 also moves the gains and perm entries and writes the caller's arrays.
template <typename T>
__global__ void __launch_bounds__(256)
rcd_k_apply_rc(RcdClass *__restrict__ classes, int round_no)
{
    using namespace sim;
    RcdClass &st = classes[blockIdx.y];
    if (st.apply_round != round_no) return;
    const int nupd = st.nupd, npatch = st.npatch;
    const int n = st.n, ld = st.ld, K = st.K, d = st.d;
    const int lane = threadIdx.x & 63;
    const int jbase = (blockIdx.x * 4 + (threadIdx.x >> 6)) * 32;
    if (jbase < n && nupd > 0) {
        const T *X = reinterpret_cast<const T *>(st.X);
        const long long ldx = st.ldx64;
        const bool vec_ok = (reinterpret_cast<uintptr_t>(st.X) & 15) == 0 && ((ldx * (long long)sizeof(T)) % 16) == 0;
        constexpr int EPC = CHUNK / (int)sizeof(T);      // elements in 16 bytes
        const int col = lane & 31;
        const int u = col < nupd ? col : 0;
        const int v = st.uv[u];
        const int jrow = min(jbase + col, n - 1);
        const int ra = st.x_index ? st.x_index[jrow] : jrow;   // x_i operand: row j
        const int rb = st.x_index ? st.x_index[v] : v;         // x_j operand: the taken sample
        const int half = (lane >> 5) * EPC;
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        // four 32-byte groups of k per trip (groups past d are zeros and add nothing)
        for (int k0 = 0; k0 < d; k0 += 8 * EPC) {
            uint4 fa[4], fb[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                fa[g] = load_chunk<T>(X, ldx, ra, k0 + g * 2 * EPC + half, d, vec_ok);
                fb[g] = load_chunk<T>(X, ldx, rb, k0 + g * 2 * EPC + half, d, vec_ok);
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if constexpr (sizeof(T) == 2) {
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[g]),
                                                                  __builtin_bit_cast(bf16x8, fb[g]), acc, 0, 0, 0);
                } else {
                    const f32x4 va = __builtin_bit_cast(f32x4, fa[g]);
                    const f32x4 vb = __builtin_bit_cast(f32x4, fb[g]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(va[e], vb[e], acc, 0, 0, 0);
                }
            }
        }
        // a lane holds column `col`, rows jbase + 8 (r / 4) + 4 (lane >> 5) + (r & 3)
        if (col < nupd) {
            const float exp_scale = st.exp_scale;
            const float scale2 = -2.f * exp_scale;
            const float sqv = st.sq[v] * exp_scale;
            float *cur = st.cur + (size_t)st.ujs[col] * ld;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = jbase + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (j < n) {
                    const float s = (j == v) ? 1.f : rbf_value(acc[r], st.sq[j] * exp_scale, sqv, scale2);
                    if (s > cur[j]) cur[j] = s;
                }
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
