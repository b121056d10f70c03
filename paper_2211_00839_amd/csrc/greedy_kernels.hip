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

// Data handed from one workgroup to another inside a launch (sweep partials,
// finished gains, a class's published state) is written and read at device
// scope: such stores go through to memory and such loads do not hit another
// XCD's stale L2 lines, so no cache-wide write-back or invalidate is needed.
// The hand-over itself is "wait for my stores, barrier, bump a counter".
__device__ __forceinline__ void dev_store(float RCD_GLOBAL *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void dev_store(int32_t RCD_GLOBAL *p, int32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 16-byte device-scope store (one write-through transaction instead of four partial ones)
__device__ __forceinline__ void dev_store4(float RCD_GLOBAL *p, float x, float y, float z, float w)
{
    typedef float v4 __attribute__((ext_vector_type(4)));
    const v4 v = {x, y, z, w};
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ float dev_load(const float RCD_GLOBAL *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t dev_load(const int32_t RCD_GLOBAL *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_for_my_stores()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}
// true in exactly one workgroup: the one whose arrival completes `expected`
__device__ __forceinline__ bool arrive_last(int32_t *counter, int expected, int *s_flag)
{
    wait_for_my_stores();
    __syncthreads();
    if (threadIdx.x == 0)
        *s_flag = (__hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == expected - 1);
    __syncthreads();
    return *s_flag != 0;
}

__device__ __forceinline__ float clamp01(float x)
{
    // S in [0,1] and cur in [0,1] give S-cur in [-1,1]: max(0, S-cur) is the
    // subtraction with the hardware clamp-to-[0,1] output modifier, one VALU op.
    return __builtin_amdgcn_fmed3f(x, 0.0f, 1.0f);
}

// two plan headers, then two prefix arrays of ncls+1 entries
__device__ __forceinline__ int32_t *plan_prefix(RcdPlan *plans, int buf)
{
    return reinterpret_cast<int32_t *>(plans + 2) + (size_t)buf * (plans[0].ncls + 1);
}
__device__ __forceinline__ const int32_t *plan_prefix(const RcdPlan *plans, int buf)
{
    return reinterpret_cast<const int32_t *>(plans + 2) + (size_t)buf * (plans[0].ncls + 1);
}

// largest c with prefix[c] <= item (prefix is non-decreasing, prefix[ncls] > item).
// Up to 64 classes at a time: lane c reads prefix[c] and a ballot counts, one trip
// to memory instead of a chain of dependent ones.
__device__ __forceinline__ int find_class(const int32_t *prefix, int ncls, int item)
{
    const int lane = threadIdx.x & 63;
    int c = 0;
    for (int base = 0; base < ncls; base += 64) {
        const int i = base + lane;
        const bool le = i < ncls && prefix[i] <= item;
        const int cnt = __popcll(__ballot(le));
        if (cnt == 0) break;
        c = base + cnt - 1;
        if (cnt < 64) break;
    }
    return __builtin_amdgcn_readfirstlane(c);
}

// ---------------------------------------------------------------------------
// Gain sweep (GreedyStep's objective for every candidate and every stale block):
//   part[chunk][k][p] = sum_{j in chunk} max(0, M[j][p] - cur_k(j))
// One workgroup = 8 waves on one 256-column tile; wave w takes the w-th eighth
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
    const int rpw = st.rpc / RCD_SWEEP_WAVES;
    const int row0 = chunk * st.rpc + wave * rpw;
    const int row1 = min(st.n, row0 + rpw);
    const int nneed = st.nneed;

    // lanes whose four columns are all dead (past the last live candidate) re-read column 0
    // instead: one shared line per row rather than a wasted fetch of their own
    const int col0 = tile * RCD_TILE + lane * 4;
    const gcf32 Mp = (gcf32)st.M + (col0 < st.nR ? col0 : 0);
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

    // Add the waves' sums in wave order, four blocks at a time.
    // lds is [wave][block-in-group 4][lane 64] float4.
    const gf32 part = (gf32)st.part + (size_t)chunk * st.K * ld + (size_t)tile * RCD_TILE + lane * 4;
#pragma unroll
    for (int g0 = 0; g0 < KS; g0 += 4) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (g0 + i < KS) lds[(wave * 4 + i) * 64 + lane] = acc[g0 + i];
        __syncthreads();
        const int mine = g0 + wave;
        if (wave < 4 && mine < KS && mine < nneed) {
            float4 a = lds[(0 * 4 + wave) * 64 + lane];
#pragma unroll
            for (int w = 1; w < RCD_SWEEP_WAVES; ++w) {
                const float4 b = lds[(w * 4 + wave) * 64 + lane];
                a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
            }
            int kmine = kb[0];
#pragma unroll
            for (int i = 0; i < KS; ++i)
                if (i == mine) kmine = kb[i];
            const gf32 dst = part + (size_t)kmine * ld;
            dev_store4(dst, a.x, a.y, a.z, a.w);
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Greedy steps of one class, run by one workgroup of NT threads.  Repeats
// Algorithm 1's loop body
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

typedef const int32_t RCD_GLOBAL *gci32;
typedef int32_t RCD_GLOBAL *gi32;

struct StepShared {
    double f[RCD_KMAX];
    int cnt[RCD_KMAX], cap[RCD_KMAX], valid[RCD_KMAX];
    unsigned long long wkey[RCD_STEP_THREADS / 64];
    int wpos[RCD_STEP_THREADS / 64];
    // columns displaced during this call: live position ppos[i] now shows the
    // column that was at position psrc[i] when the call began
    int npatch, ppos[RCD_KMAX], psrc[RCD_KMAX];
    // the steps taken: block, column (position at the start of the call) that
    // was taken, sample, step index, gain
    int nupd, ujs[RCD_KMAX], usrc[RCD_KMAX], uv[RCD_KMAX], ut[RCD_KMAX];
};

// position at the start of the call of the column now shown at position p
__device__ __forceinline__ int effective_pos(const StepShared &sh, int npatch, int p)
{
    int e = p;
    for (int i = 0; i < npatch; ++i)
        if (sh.ppos[i] == p) e = sh.psrc[i];
    return e;
}

// Only the decisions are taken here, so that one step costs one trip to memory:
// argmin block, argmax column (gains and perm are read through the list of
// columns displaced so far, nothing of the matrix is touched), bookkeeping in
// LDS.  The consequences - coverage updates from the taken columns, moving the
// displaced columns, their gains and perm entries, the caller's output arrays -
// are applied by rcd_k_apply, which has the whole GPU for the strided column
// traffic.  A block is stepped at most once per call (its gains go stale), so
// a call takes at most K steps.
// SCOPED: the gains were written earlier in this same launch by other workgroups
// (fused round), so they are read at device scope; in its own launch plain loads do.
template <int NT, bool SCOPED>
__device__ __forceinline__ void class_steps(RcdClass &st, StepShared &sh)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    int done = st.done;
    if (done) {
        if (tid == 0) dev_store((gi32)&st.nneed, 0);
        return;
    }
    const int K = st.K, n = st.n, ld = st.ld, total = st.total;
    const long long tick0 = wall_clock64();
    __syncthreads();
    if (tid < RCD_KMAX) {
        sh.f[tid] = st.f[tid];
        sh.cnt[tid] = st.cnt[tid];
        sh.cap[tid] = st.cap[tid];
        sh.valid[tid] = st.valid[tid];
    }
    if (tid == 0) { sh.npatch = 0; sh.nupd = 0; }
    __syncthreads();
    // the sweep that ran since the last call rebuilt these rows
    if (tid < st.nneed) sh.valid[st.need[tid]] = 1;
    __syncthreads();

    const int nR0 = st.nR, t0 = st.t;
    int nR = nR0, t = t0;
    long long useful = 0;
    const gf32 M = (gf32)st.M;
    const gf32 gain = (gf32)st.gain;
    const gi32 perm = (gi32)st.perm;

    // ---- A. decide
    for (;;) {
        if (t >= total) { done = 1; break; }
        int js = -1;
        double fbest = 0.0;
        for (int k = 0; k < K; ++k) {
            if (sh.cnt[k] >= sh.cap[k]) continue;
            const double fk = sh.f[k];
            if (js < 0 || fk < fbest) { js = k; fbest = fk; }
        }
        if (js < 0) { done = 1; break; }
        if (!sh.valid[js]) break;

        const gcf32 g = (gcf32)gain + (size_t)js * ld;
        const int npatch = sh.npatch;
        unsigned long long best = 0ull;
        int bpos = -1;
        constexpr int UA = NT >= 1024 ? 8 : 12;   // loads in flight per thread and array
        for (int p0 = 0; p0 < nR; p0 += UA * NT) {
            float gv[UA];
            int pv[UA];
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                const int p = p0 + u * NT + tid;
                if (p < nR) {
                    const int e = npatch ? effective_pos(sh, npatch, p) : p;
                    gv[u] = SCOPED ? dev_load(g + e) : g[e];
                    pv[u] = perm[e];
                }
            }
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                const int p = p0 + u * NT + tid;
                if (p < nR) {
                    const unsigned long long key = pack_key(gv[u], pv[u]);
                    if (key > best) { best = key; bpos = p; }
                }
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const unsigned long long ok = __shfl_xor(best, off);
            const int op = __shfl_xor(bpos, off);
            if (ok > best) { best = ok; bpos = op; }
        }
        if (lane == 0) { sh.wkey[wave] = best; sh.wpos[wave] = bpos; }
        __syncthreads();
        best = sh.wkey[0]; bpos = sh.wpos[0];
#pragma unroll
        for (int w = 1; w < NT / 64; ++w) {
            const unsigned long long ok = sh.wkey[w];
            if (ok > best) { best = ok; bpos = sh.wpos[w]; }
        }
        const float gbest = __uint_as_float((unsigned)(best >> 32));
        const int vstar = (int)(0xFFFFFFFFu - (unsigned)(best & 0xFFFFFFFFull));
        const int pstar = bpos;
        const int last = nR - 1;
        __syncthreads();   // everyone has read sh.f/cnt/valid/wkey and the patch list of this step
        if (tid == 0) {
            const int np = sh.npatch;
            const int src_star = effective_pos(sh, np, pstar);
            const int src_last = effective_pos(sh, np, last);
            const int u = sh.nupd;
            sh.ujs[u] = js; sh.usrc[u] = src_star; sh.uv[u] = vstar; sh.ut[u] = t;
            sh.nupd = u + 1;
            // drop what the list said about the two positions, then: p* shows the last column
            int m = 0;
            for (int i = 0; i < np; ++i)
                if (sh.ppos[i] != pstar && sh.ppos[i] != last) { sh.ppos[m] = sh.ppos[i]; sh.psrc[m] = sh.psrc[i]; ++m; }
            if (pstar != last) { sh.ppos[m] = pstar; sh.psrc[m] = src_last; ++m; }
            sh.npatch = m;
            sh.cnt[js] += 1;
            sh.f[js] += (double)gbest;
            sh.valid[js] = 0;
        }
        useful += nR;
        nR = last;
        ++t;
        __syncthreads();
    }

    // ---- hand the steps taken and the displaced columns to the apply kernel
    if (tid < RCD_KMAX) {
        st.ujs[tid] = sh.ujs[tid];
        st.usrc[tid] = sh.usrc[tid];
        st.uv[tid] = sh.uv[tid];
        st.ut[tid] = sh.ut[tid];
        st.ppos[tid] = sh.ppos[tid];
        st.psrc[tid] = sh.psrc[tid];
    }
    // publish the state and what the next sweep must do
    if (tid == 0) {
        int nneed = 0;
        if (!done) {
            for (int k = 0; k < K; ++k)
                if (sh.cnt[k] < sh.cap[k] && !sh.valid[k]) st.need[nneed++] = k;
        }
        dev_store((gi32)&st.nneed, nneed);
        if (nneed > 0) {
            const int tiles = (nR + st.tw - 1) / st.tw;
            int C = (st.target_items + tiles - 1) / tiles;
            C = C < 1 ? 1 : (C > RCD_CMAX ? RCD_CMAX : C);
            int rpc = (n + C - 1) / C;
            rpc = (rpc + st.row_align - 1) / st.row_align * st.row_align;
            st.rpc = rpc;
            dev_store((gi32)&st.C, (n + rpc - 1) / rpc);
            st.stat_sweeps += 1;
            st.stat_entries += (long long)nR * n;
            st.stat_computed += (long long)nneed * nR;
        }
        st.stat_steps += t - t0;
        st.stat_useful += useful;
        st.stat_ticks += wall_clock64() - tick0;
        st.nupd = sh.nupd;
        st.npatch = sh.npatch;
        st.apply_round = st.apply_round + 1;
        dev_store((gi32)&st.nR, nR);
        st.t = t;
        dev_store((gi32)&st.done, done);
        for (int k = 0; k < K; ++k) {
            st.f[k] = sh.f[k];
            st.cnt[k] = sh.cnt[k];
            st.valid[k] = sh.valid[k];
        }
    }
}

// Lay out the next round's sweep over all classes into plan buffer `next` and
// retire buffer `cur_buf`.  Called by every thread of one workgroup (NT threads)
// after the last arrival: thread c reads class c's published state, a block scan
// turns the per-class workgroup counts into the prefix array.  scratch: NT/64 ints of LDS.
template <int NT>
__device__ __forceinline__ void write_plan(RcdClass *classes, RcdPlan *plans, int cur_buf, int next, int *scratch)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ncls = plans[0].ncls;
    int32_t *ip = plan_prefix(plans, next);
    int items = 0, ndone = 0, nactive = 0;
    for (int base = 0; base < ncls; base += NT) {
        const int c = base + tid;
        int it = 0, dn = 0, ac = 0;
        if (c < ncls) {
            const RcdClass &o = classes[c];
            const int nneed = dev_load((gci32)&o.nneed);
            const int nR = dev_load((gci32)&o.nR);
            const int C = dev_load((gci32)&o.C);
            dn = dev_load((gci32)&o.done) ? 1 : 0;
            if (nneed > 0) {
                it = ((nR + o.tw - 1) / o.tw) * C;
                ac = 1;
            }
        }
        int incl = it;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int v = __shfl_up(incl, off);
            if (lane >= off) incl += v;
        }
        __syncthreads();
        if (lane == 63) scratch[wave] = incl;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) {
            const int v = scratch[w];
            if (w < wave) before += v;
            total += v;
        }
        if (c < ncls) ip[c] = items + before + incl - it;
        items += total;
        ndone += __syncthreads_count(dn);
        nactive += __syncthreads_count(ac);
    }
    if (tid == 0) {
        ip[ncls] = items;
        plans[next].items = items;
        plans[next].nactive = nactive;
        plans[next].ndone = ndone;
        plans[next].arrive = 0;
        if (cur_buf >= 0) {
            // late workgroups of this launch only ever see "nothing to do" here
            plans[cur_buf].items = 0;
            plans[cur_buf].nactive = 0;
            plans[cur_buf].ndone = ndone;
        }
    }
}

// What follows a workgroup's sweep item (steps 2-4 of a round, see rcd_k_round).
// NT threads in the workgroup, TW columns per tile.
// FUSE = false stops after step 2: the step loops then run in their own launch (rcd_k_steps).
template <int NT, int TW, bool FUSE>
__device__ __forceinline__ void round_tail(RcdClass &st, RcdClass *classes, RcdPlan *plans, int buf, int tile,
                                           int tiles, StepShared &sh, int *s_flag)
{
    // ---- 2. last chunk of this tile?  then add the chunks' partial sums in order
    const int tid = threadIdx.x;
    const int C = st.C;
    const int nneed = st.nneed;
    if (!arrive_last(&st.tilecnt[tile], C, s_flag)) return;
    if (tid < TW) {
        const int ld = st.ld, K = st.K;
        const int col = tile * TW + tid;
        const gcf32 part = (gcf32)st.part + col;
        const size_t kstride = (size_t)K * ld;
        for (int i = 0; i < nneed; ++i) {
            const int k = st.need[i];
            const gcf32 p = part + (size_t)k * ld;
            float g = 0.f;
            int ch = 0;
            for (; ch + 8 <= C; ch += 8) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = dev_load(p + (size_t)(ch + u) * kstride);
#pragma unroll
                for (int u = 0; u < 8; ++u) g += v[u];
            }
            for (; ch < C; ++ch) g += dev_load(p + (size_t)ch * kstride);
            dev_store((gf32)st.gain + (size_t)k * ld + col, g);
        }
        if (tid == 0) st.tilecnt[tile] = 0;
    }
    if constexpr (!FUSE) return;
    // ---- 3. last tile of this class?  then run the class's greedy steps
    if (!arrive_last(&st.tiles_done, tiles, s_flag)) return;
    if (tid == 0) st.tiles_done = 0;
    class_steps<NT, true>(st, sh);
    // ---- 4. last active class of the group?  then lay out the next round
    if (arrive_last(&plans[buf].arrive, plans[buf].nactive, s_flag))
        write_plan<NT>(classes, plans, buf, buf ^ 1, reinterpret_cast<int *>(sh.wkey));
}

} // namespace

// Bootstrap (and the whole loop when there is nothing to sweep): one workgroup
// per class runs the steps and the last one to finish writes plan buffer 0.
extern "C" __global__ void __launch_bounds__(RCD_STEP_THREADS)
rcd_k_steps(RcdClass *__restrict__ classes, RcdPlan *__restrict__ plans)
{
    __shared__ StepShared sh;
    __shared__ int s_flag;
    class_steps<RCD_STEP_THREADS, false>(classes[blockIdx.x], sh);
    if (arrive_last(&plans[1].arrive, (int)gridDim.x, &s_flag)) {
        if (threadIdx.x == 0) plans[1].arrive = 0;
        write_plan<RCD_STEP_THREADS>(classes, plans, -1, 0, reinterpret_cast<int *>(sh.wkey));
    }
}

// One round for every class of the group, in a single launch (FUSE), or its
// first two parts (the host then launches rcd_k_steps for parts 3 and 4: with
// many classes in flight the sweep is bandwidth-bound and the step loop of the
// class that finishes last would only lengthen it):
//   1. sweep: every workgroup computes one (class, tile, row chunk) of partial gains
//   2. the workgroup that completes a tile adds its chunks in order -> gain
//   3. the workgroup that completes a class runs that class's greedy steps
//      (while other classes are still being swept)
//   4. the workgroup that completes the last class writes the next round's plan
// Completion is detected with arrival counters; nothing ever waits.  Launch r reads plan buffer r&1 and writes
// the other one.
// KCAP: no class of the group has more blocks than this (the host picks the
// smallest instance that fits, which keeps the register count, hence the
// occupancy, of small-K data sets independent of the K = 16 code).
template <int KCAP, bool FUSE>
__global__ void __launch_bounds__(RCD_SWEEP_THREADS)
rcd_k_round(RcdClass *__restrict__ classes, RcdPlan *__restrict__ plans, int buf)
{
    __shared__ float4 lds[RCD_SWEEP_WAVES * 4 * 64];
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
    const int tiles = (st.nR + RCD_TILE - 1) / RCD_TILE;
    const int tile = local % tiles;
    const int chunk = local / tiles;
    const int nneed = st.nneed;
    if (nneed <= 1) sweep_body<1>(st, tile, chunk, lds);
    else if (nneed == 2) sweep_body<2>(st, tile, chunk, lds);
    else if (nneed == 3) sweep_body<3>(st, tile, chunk, lds);
    else if (nneed == 4 || KCAP <= 4) sweep_body<4>(st, tile, chunk, lds);
    else if (nneed <= 6) sweep_body<6>(st, tile, chunk, lds);
    else if (nneed <= 8 || KCAP <= 8) sweep_body<8>(st, tile, chunk, lds);
    else if (nneed <= 12) sweep_body<12>(st, tile, chunk, lds);
    else sweep_body<16>(st, tile, chunk, lds);

    round_tail<RCD_SWEEP_THREADS, RCD_TILE, FUSE>(st, classes, plans, buf, tile, tiles, sh, &s_flag);
}

// Applies what the step loops of the last round decided.  grid = (row blocks, ncls),
// one thread per row j of the class:
//   coverage:  cur_js(j) = max(cur_js(j), S(j, v*)) for every step taken
//   compaction: the column at (dead) position psrc moves to live position ppos
// All loads come before the stores; sources of moves are dead positions that
// nothing writes, and the coverage reads use positions as they were before the
// moves, so the order inside a thread is all that matters.  Row block 0 also
// moves the gains and perm entries and writes the caller's arrays.
extern "C" __global__ void __launch_bounds__(256)
rcd_k_apply(RcdClass *__restrict__ classes, int round_no)
{
    RcdClass &st = classes[blockIdx.y];
    if (st.apply_round != round_no) return;
    const int nupd = st.nupd, npatch = st.npatch;
    const int n = st.n, ld = st.ld, K = st.K;
    const int j = blockIdx.x * 256 + threadIdx.x;
    const gf32 M = (gf32)st.M;
    if (j < n) {
        float sv[RCD_KMAX], cv[RCD_KMAX], mv[RCD_KMAX];
        const gf32 row = M + (size_t)j * ld;
#pragma unroll
        for (int i = 0; i < RCD_KMAX; ++i)
            if (i < nupd) {
                sv[i] = row[st.usrc[i]];
                cv[i] = ((gf32)st.cur)[(size_t)st.ujs[i] * ld + j];
            }
#pragma unroll
        for (int i = 0; i < RCD_KMAX; ++i)
            if (i < npatch) mv[i] = row[st.psrc[i]];
#pragma unroll
        for (int i = 0; i < RCD_KMAX; ++i)
            if (i < nupd && sv[i] > cv[i]) ((gf32)st.cur)[(size_t)st.ujs[i] * ld + j] = sv[i];
#pragma unroll
        for (int i = 0; i < RCD_KMAX; ++i)
            if (i < npatch) row[st.ppos[i]] = mv[i];
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
    for (int i = i0; i < st.ld / RCD_TILE_RC; i += stride) st.tilecnt[i] = 0;
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
