// Kernels of the class greedy (Algorithm 1 of arXiv 2211.00839, inner while loop,
// with the facility-location function of Section 4) for gfx950.
//
// Data layout.  M is the class's similarity matrix, row j = covered sample j in
// the class's original order, column p = candidate perm[p].  Only the first nR
// columns are live: when a candidate is taken its column is overwritten by the
// last live column, so a sweep reads exactly n x nR entries.  Because S is
// symmetric, "row j, 256 consecutive candidates" is a contiguous 1 KB read and
// each lane owns its candidates' sums outright: cur_k(j) is wave-uniform and
// comes through scalar loads, and no cross-lane reduction exists anywhere in
// the sweep.
#include <hip/hip_runtime.h>
#include "rcd_state.h"

namespace {

// Pointers that arrive through a descriptor in memory are generic to the
// compiler; every one of them points to device global memory, and saying so
// lets it use global (and, for wave-uniform reads, scalar) loads.
#define RCD_GLOBAL __attribute__((address_space(1)))
typedef const float RCD_GLOBAL *gcf32;
typedef float RCD_GLOBAL *gf32;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef const f32x4 RCD_GLOBAL *gcf32x4;
typedef f32x4 RCD_GLOBAL *gf32x4;
// Memory that no thread writes while the kernel runs may be read through the
// constant address space, which lets wave-uniform reads use the scalar unit.
typedef const float __attribute__((address_space(4))) *ccf32;

__device__ __forceinline__ float clamp01(float x)
{
    // S in [0,1] and cur in [0,1] give S-cur in [-1,1]: max(0, S-cur) is the
    // subtraction with the hardware clamp-to-[0,1] output modifier, one VALU op.
    return __builtin_amdgcn_fmed3f(x, 0.0f, 1.0f);
}

__device__ __forceinline__ const int32_t *item_prefix(const RcdPlan *plan)
{
    return reinterpret_cast<const int32_t *>(plan + 1);
}
__device__ __forceinline__ const int32_t *tile_prefix(const RcdPlan *plan)
{
    return reinterpret_cast<const int32_t *>(plan + 1) + (plan->ncls + 1);
}

// largest c with prefix[c] <= item (prefix is non-decreasing, prefix[ncls] > item)
__device__ __forceinline__ int find_class(const int32_t *__restrict__ prefix, int ncls, int item)
{
    int lo = 0, hi = ncls;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (prefix[mid] <= item) lo = mid; else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------------------
// Gain sweep (GreedyStep's objective for every candidate and every stale block):
//   part[chunk][k][p] = sum_{j in chunk} max(0, M[j][p] - cur_k(j))
// One workgroup = 4 waves on one 256-column tile; wave w takes the w-th quarter
// of the chunk's rows.  KS = number of blocks evaluated (compile-time so the
// accumulators stay in registers).
// ---------------------------------------------------------------------------
template <int KS>
__device__ __forceinline__ void sweep_body(const RcdClass &st, int tile, int chunk, float4 *lds)
{
    const int lane = threadIdx.x & 63;
    // the wave index is the same in all 64 lanes: tell the compiler, so that row
    // counters and coverage addresses live in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ld = st.ld;
    const int rpw = st.rpc >> 2;
    const int row0 = chunk * st.rpc + wave * rpw;
    const int row1 = min(st.n, row0 + rpw);
    const int nneed = st.nneed;

    const gcf32 Mp = (gcf32)st.M + (size_t)tile * RCD_TILE + lane * 4;
    ccf32 cp[KS];
    int kb[KS];
#pragma unroll
    for (int i = 0; i < KS; ++i) {
        kb[i] = st.need[i < nneed ? i : nneed - 1];
        cp[i] = (ccf32)st.cur + (size_t)kb[i] * ld;
    }
    float4 acc[KS];
#pragma unroll
    for (int i = 0; i < KS; ++i) acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);

    int j = row0;
    for (; j + 4 <= row1; j += 4) {
        const f32x4 s0 = *(gcf32x4)(Mp + (size_t)(j + 0) * ld);
        const f32x4 s1 = *(gcf32x4)(Mp + (size_t)(j + 1) * ld);
        const f32x4 s2 = *(gcf32x4)(Mp + (size_t)(j + 2) * ld);
        const f32x4 s3 = *(gcf32x4)(Mp + (size_t)(j + 3) * ld);
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            const float c0 = cp[i][j], c1 = cp[i][j + 1], c2 = cp[i][j + 2], c3 = cp[i][j + 3];
            acc[i].x += clamp01(s0.x - c0); acc[i].y += clamp01(s0.y - c0);
            acc[i].z += clamp01(s0.z - c0); acc[i].w += clamp01(s0.w - c0);
            acc[i].x += clamp01(s1.x - c1); acc[i].y += clamp01(s1.y - c1);
            acc[i].z += clamp01(s1.z - c1); acc[i].w += clamp01(s1.w - c1);
            acc[i].x += clamp01(s2.x - c2); acc[i].y += clamp01(s2.y - c2);
            acc[i].z += clamp01(s2.z - c2); acc[i].w += clamp01(s2.w - c2);
            acc[i].x += clamp01(s3.x - c3); acc[i].y += clamp01(s3.y - c3);
            acc[i].z += clamp01(s3.z - c3); acc[i].w += clamp01(s3.w - c3);
        }
    }
    for (; j < row1; ++j) {
        const f32x4 s0 = *(gcf32x4)(Mp + (size_t)j * ld);
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            const float c0 = cp[i][j];
            acc[i].x += clamp01(s0.x - c0); acc[i].y += clamp01(s0.y - c0);
            acc[i].z += clamp01(s0.z - c0); acc[i].w += clamp01(s0.w - c0);
        }
    }

    // Add the four waves' sums in wave order, four blocks at a time.
    // lds is [wave 4][block-in-group 4][lane 64] float4 = 16 KB.
    const gf32 part = (gf32)st.part + (size_t)chunk * st.K * ld + (size_t)tile * RCD_TILE + lane * 4;
#pragma unroll
    for (int g0 = 0; g0 < KS; g0 += 4) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (g0 + i < KS) lds[(wave * 4 + i) * 64 + lane] = acc[g0 + i];
        __syncthreads();
        const int mine = g0 + wave;
        if (mine < KS && mine < nneed) {
            float4 a = lds[(0 * 4 + wave) * 64 + lane];
            const float4 b = lds[(1 * 4 + wave) * 64 + lane];
            const float4 c = lds[(2 * 4 + wave) * 64 + lane];
            const float4 e = lds[(3 * 4 + wave) * 64 + lane];
            a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
            a.x += c.x; a.y += c.y; a.z += c.z; a.w += c.w;
            a.x += e.x; a.y += e.y; a.z += e.z; a.w += e.w;
            int kmine = kb[0];
#pragma unroll
            for (int i = 0; i < KS; ++i)
                if (i == mine) kmine = kb[i];
            f32x4 out;
            out.x = a.x; out.y = a.y; out.z = a.z; out.w = a.w;
            *(gf32x4)(part + (size_t)kmine * ld) = out;
        }
        __syncthreads();
    }
}

} // namespace

extern "C" __global__ void __launch_bounds__(RCD_SWEEP_THREADS)
rcd_k_sweep(const RcdClass *__restrict__ classes, const RcdPlan *__restrict__ plan)
{
    __shared__ float4 lds[4 * 4 * 64];
    const int item = blockIdx.x;
    if (item >= plan->items) return;
    const int ncls = plan->ncls;
    const int32_t *__restrict__ prefix = item_prefix(plan);
    const int c = ncls > 1 ? find_class(prefix, ncls, item) : 0;
    const RcdClass &st = classes[c];
    const int local = item - prefix[c];
    const int tiles = (st.nR + RCD_TILE - 1) / RCD_TILE;
    const int tile = local % tiles;
    const int chunk = local / tiles;
    const int nneed = st.nneed;
    if (nneed <= 1) sweep_body<1>(st, tile, chunk, lds);
    else if (nneed == 2) sweep_body<2>(st, tile, chunk, lds);
    else if (nneed == 3) sweep_body<3>(st, tile, chunk, lds);
    else if (nneed == 4) sweep_body<4>(st, tile, chunk, lds);
    else if (nneed <= 6) sweep_body<6>(st, tile, chunk, lds);
    else if (nneed <= 8) sweep_body<8>(st, tile, chunk, lds);
    else if (nneed <= 12) sweep_body<12>(st, tile, chunk, lds);
    else sweep_body<16>(st, tile, chunk, lds);
}

// gain[k][p] = sum over row chunks, in chunk order, of part[chunk][k][p].
extern "C" __global__ void __launch_bounds__(RCD_TILE)
rcd_k_finalize(const RcdClass *__restrict__ classes, const RcdPlan *__restrict__ plan)
{
    const int item = blockIdx.x;
    if (item >= plan->tiles) return;
    const int ncls = plan->ncls;
    const int32_t *__restrict__ prefix = tile_prefix(plan);
    const int c = ncls > 1 ? find_class(prefix, ncls, item) : 0;
    const RcdClass &st = classes[c];
    const int tile = item - prefix[c];
    const int col = tile * RCD_TILE + threadIdx.x;
    const int ld = st.ld, K = st.K, C = st.C;
    for (int i = 0; i < st.nneed; ++i) {
        const int k = st.need[i];
        const float *__restrict__ p = st.part + (size_t)k * ld + col;
        float g = 0.f;
        for (int ch = 0; ch < C; ++ch) g += p[(size_t)ch * K * ld];
        st.gain[(size_t)k * ld + col] = g;
    }
}

// ---------------------------------------------------------------------------
// Steps kernel: one workgroup per class.  Repeats Algorithm 1's loop body
//   j* = argmin over non-full blocks of f (lowest index on ties)
//   v* = argmax over unassigned v of the gain for block j* (lowest index on ties)
//   A_j* += v*, R -= v*, coverage update cur_j*(j) = max(cur_j*(j), S(j, v*))
// for as long as block j*'s gain row is current.  A gain row stays current
// until its own block changes: taking a sample away from R only removes a
// column.  Ends by publishing which rows the next sweep has to rebuild.
// ---------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long pack_key(float g, int v)
{
    // g >= +0 so its bit pattern orders like its value; larger gain wins, then
    // the smaller original index.
    return ((unsigned long long)__float_as_uint(g) << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)v);
}

extern "C" __global__ void __launch_bounds__(RCD_STEP_THREADS)
rcd_k_steps(RcdClass *__restrict__ classes, RcdPlan *__restrict__ plan, int target_total)
{
    __shared__ double s_f[RCD_KMAX];
    __shared__ int s_cnt[RCD_KMAX], s_cap[RCD_KMAX], s_valid[RCD_KMAX];
    __shared__ unsigned long long s_wkey[RCD_STEP_THREADS / 64];
    __shared__ int s_wpos[RCD_STEP_THREADS / 64];
    __shared__ int s_last_arrival;

    RcdClass &st = classes[blockIdx.x];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    int done = st.done;

    if (!done) {
        const int K = st.K, n = st.n, ld = st.ld, total = st.total;
        if (tid < RCD_KMAX) {
            s_f[tid] = st.f[tid];
            s_cnt[tid] = st.cnt[tid];
            s_cap[tid] = st.cap[tid];
            s_valid[tid] = st.valid[tid];
        }
        __syncthreads();
        // the sweep + finalize that ran since the last call rebuilt these rows
        if (tid < st.nneed) s_valid[st.need[tid]] = 1;
        __syncthreads();

        int nR = st.nR, t = st.t;
        long long useful = 0;
        float *const M = st.M;
        int32_t *const perm = st.perm;

        for (;;) {
            if (t >= total) { done = 1; break; }
            int js = -1;
            double fbest = 0.0;
            for (int k = 0; k < K; ++k) {
                if (s_cnt[k] >= s_cap[k]) continue;
                const double fk = s_f[k];
                if (js < 0 || fk < fbest) { js = k; fbest = fk; }
            }
            if (js < 0) { done = 1; break; }
            if (!s_valid[js]) break;

            // masked argmax over the live columns
            const float *g = st.gain + (size_t)js * ld;
            unsigned long long best = 0ull;
            int bpos = -1;
            for (int p = tid; p < nR; p += RCD_STEP_THREADS) {
                const unsigned long long key = pack_key(g[p], perm[p]);
                if (key > best) { best = key; bpos = p; }
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const unsigned long long ok = __shfl_xor(best, off);
                const int op = __shfl_xor(bpos, off);
                if (ok > best) { best = ok; bpos = op; }
            }
            if (lane == 0) { s_wkey[wave] = best; s_wpos[wave] = bpos; }
            __syncthreads();
            best = s_wkey[0]; bpos = s_wpos[0];
#pragma unroll
            for (int w = 1; w < RCD_STEP_THREADS / 64; ++w) {
                const unsigned long long ok = s_wkey[w];
                if (ok > best) { best = ok; bpos = s_wpos[w]; }
            }
            const float gbest = __uint_as_float((unsigned)(best >> 32));
            const int vstar = (int)(0xFFFFFFFFu - (unsigned)(best & 0xFFFFFFFFull));
            const int pstar = bpos;
            const int last = nR - 1;

            // coverage update from column p*, then compaction: last live column -> p*
            float *cur = st.cur + (size_t)js * ld;
            for (int j = tid; j < n; j += RCD_STEP_THREADS) {
                float *row = M + (size_t)j * ld;
                const float s = row[pstar];
                if (s > cur[j]) cur[j] = s;
                if (pstar != last) row[pstar] = row[last];
            }
            if (pstar != last) {
                if (tid < K) st.gain[(size_t)tid * ld + pstar] = st.gain[(size_t)tid * ld + last];
                if (tid == 64) perm[pstar] = perm[last];
            }
            if (tid == 0) {
                const int oi = st.out_index ? st.out_index[vstar] : vstar;
                st.assign_out[oi] = js;
                if (st.order_out) st.order_out[oi] = t;
            }
            __syncthreads();   // everyone has read s_f/s_cnt/s_valid/s_wkey of this step
            if (tid == 0) {
                s_cnt[js] += 1;
                s_f[js] += (double)gbest;
                s_valid[js] = 0;
            }
            useful += nR;
            nR = last;
            ++t;
            __syncthreads();
        }

        // publish the state and what the next sweep must do
        if (tid == 0) {
            int nneed = 0;
            if (!done) {
                for (int k = 0; k < K; ++k)
                    if (s_cnt[k] < s_cap[k] && !s_valid[k]) st.need[nneed++] = k;
            }
            st.nneed = nneed;
            if (nneed > 0) {
                const int tiles = (nR + RCD_TILE - 1) / RCD_TILE;
                int C = (st.target_items + tiles - 1) / tiles;
                C = C < 1 ? 1 : (C > RCD_CMAX ? RCD_CMAX : C);
                int rpc = (n + C - 1) / C;
                rpc = (rpc + 15) & ~15;
                st.rpc = rpc;
                st.C = (n + rpc - 1) / rpc;
                st.stat_sweeps += 1;
                st.stat_entries += (long long)nR * n;
                st.stat_computed += (long long)nneed * nR;
            }
            st.stat_steps += t - st.t;
            st.stat_useful += useful;
            st.nR = nR;
            st.t = t;
            st.done = done;
            for (int k = 0; k < K; ++k) {
                st.f[k] = s_f[k];
                st.cnt[k] = s_cnt[k];
                st.valid[k] = s_valid[k];
            }
        }
    } else if (tid == 0) {
        st.nneed = 0;
    }

    // The last workgroup to get here lays out the next sweep over all classes.
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const int ticket = atomicAdd(&plan->arrive, 1);
        s_last_arrival = (ticket == (int)gridDim.x - 1);
    }
    __syncthreads();
    if (s_last_arrival && tid == 0) {
        __threadfence();
        int32_t *ip = reinterpret_cast<int32_t *>(plan + 1);
        int32_t *tp = ip + (plan->ncls + 1);
        int items = 0, tiles_total = 0, ndone = 0;
        const int ncls = plan->ncls;
        for (int c = 0; c < ncls; ++c) {
            const RcdClass &o = classes[c];
            const int nneed = __atomic_load_n(&o.nneed, __ATOMIC_RELAXED);
            ip[c] = items;
            tp[c] = tiles_total;
            if (nneed > 0) {
                const int tiles = (__atomic_load_n(&o.nR, __ATOMIC_RELAXED) + RCD_TILE - 1) / RCD_TILE;
                items += tiles * __atomic_load_n(&o.C, __ATOMIC_RELAXED);
                tiles_total += tiles;
            }
            ndone += __atomic_load_n(&o.done, __ATOMIC_RELAXED) ? 1 : 0;
        }
        ip[ncls] = items;
        tp[ncls] = tiles_total;
        plan->items = items;
        plan->tiles = tiles_total;
        plan->ndone = ndone;
        plan->arrive = 0;
    }
    (void)target_total;
}

// Initial state of a group of classes: cur = 0 (f of the empty set is 0),
// perm = identity, outputs = -1.  grid = (blocks, ncls).
extern "C" __global__ void rcd_k_init(const RcdClass *__restrict__ classes)
{
    const RcdClass &st = classes[blockIdx.y];
    const int stride = gridDim.x * blockDim.x;
    const int i0 = blockIdx.x * blockDim.x + threadIdx.x;
    const size_t ncur = (size_t)st.K * st.ld;
    for (size_t i = i0; i < ncur; i += stride) st.cur[i] = 0.f;
    for (int i = i0; i < st.ld; i += stride) st.perm[i] = i;
    for (int i = i0; i < st.n; i += stride) {
        const int oi = st.out_index ? st.out_index[i] : i;
        st.assign_out[oi] = -1;
        if (st.order_out) st.order_out[oi] = -1;
    }
}

// obj[c][k] = f(A_k) = sum_j cur_k(j), in double, fixed tree order.  grid = (K, ncls).
extern "C" __global__ void __launch_bounds__(256)
rcd_k_objective(const RcdClass *__restrict__ classes, double *__restrict__ obj, int Kstride)
{
    __shared__ double sh[256];
    const RcdClass &st = classes[blockIdx.y];
    const int k = blockIdx.x;
    if (k >= st.K) return;
    const float *cur = st.cur + (size_t)k * st.ld;
    double a = 0.0;
    for (int j = threadIdx.x; j < st.n; j += 256) a += (double)cur[j];
    sh[threadIdx.x] = a;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) obj[(size_t)blockIdx.y * Kstride + k] = sh[0];
}

// Copy a caller's S (n x n, pitch lds) into the working matrix (pitch ld) and
// flag entries outside [0,1] or NaN.  grid-stride over rows.
extern "C" __global__ void __launch_bounds__(256)
rcd_k_copy_check(const float *__restrict__ S, long long lds, float *__restrict__ M, int ld, int n,
                 RcdPlan *plan)
{
    int bad = 0;
    for (int j = blockIdx.x; j < n; j += gridDim.x) {
        const float *src = S + (size_t)j * lds;
        float *dst = M + (size_t)j * ld;
        for (int p = threadIdx.x; p < ld; p += 256) {
            float v = 0.f;
            if (p < n) {
                v = src[p];
                if (!(v >= 0.f && v <= 1.f)) bad = 1;
            }
            dst[p] = v;
        }
    }
    if (bad) plan->bad = 1;
}

// Test/benchmark helper behind rcd_gain_sweep: out[k][v] = gain[k][v] for v < n.
extern "C" __global__ void rcd_k_export_gains(const RcdClass *__restrict__ classes, float *__restrict__ out)
{
    const RcdClass &st = classes[0];
    const int v = blockIdx.x * blockDim.x + threadIdx.x;
    const int k = blockIdx.y;
    if (v < st.n) out[(size_t)k * st.n + v] = st.gain[(size_t)k * st.ld + v];
}

extern "C" __global__ void rcd_k_import_cur(const RcdClass *__restrict__ classes, const float *__restrict__ in)
{
    const RcdClass &st = classes[0];
    const int v = blockIdx.x * blockDim.x + threadIdx.x;
    const int k = blockIdx.y;
    if (v < st.n) st.cur[(size_t)k * st.ld + v] = in[(size_t)k * st.n + v];
}
