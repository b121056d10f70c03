// Kernels of the class greedy (Algorithm 1 of arXiv 2211.00839, inner while loop,
// with the facility-location function of Section 4) for gfx950.
//
// Data layout, stored similarity.  M[v][j] = S(j, v): row v holds candidate v's
// similarity to every sample j of the class, contiguous (for the symmetric matrix
// the similarity builder writes, M is simply S).  M is never written.  The
// unassigned candidates are the list perm[0 .. nR): a sweep streams exactly those
// nR rows, and taking a candidate moves the last list entry into its place.
// The recomputed mode (other file) shares the step loop and the arrival helpers.
#include <hip/hip_runtime.h>
#include <cstddef>
#include <type_traits>
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
// Gain sweep, stored similarity (GreedyStep's objective for every candidate and
// every stale block):
//   part[c][k][p] = sum_{j in chunk c} max(0, M[perm[p]][j] - cur_k(j))
// One wave streams one candidate's row (contiguous) at a time, with non-temporal loads
// (a row is not touched again before the next sweep, by which time the caches have turned
// over many times; a plain streaming read measures 6.2 TB/s on this chip, a non-temporal
// one 6.9); the workgroup's
// 16 waves share the coverage vectors of the evaluated blocks, staged in LDS for
// the chunk of j the pass covers.  A lane keeps one running sum per block, the
// wave adds its 64 lanes in a fixed order at the end of the row, and lane 0
// writes the result: no partial sums between workgroups, nothing to finalise.
// KS = number of blocks evaluated (compile-time so the sums stay in registers).
// The workgroup is the w-th of W that serve this class.
// ---------------------------------------------------------------------------
typedef const int32_t __attribute__((address_space(4))) *cci32;
typedef float __attribute__((address_space(3))) *lf32;
typedef const f32x4 __attribute__((address_space(3))) *lcf32x4;

// Sum over the 64 lanes, same value in every lane, fixed order:
// pairs, quads, halves of a 16-lane row, the row, then the four rows.
__device__ __forceinline__ float wave_sum(float v)
{
    int x;
    x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true);    // quad_perm 1,0,3,2
    v += __int_as_float(x);
    x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true);    // quad_perm 2,3,0,1
    v += __int_as_float(x);
    x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true);   // row_half_mirror
    v += __int_as_float(x);
    x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true);   // row_mirror
    v += __int_as_float(x);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (r0 + r1) + (r2 + r3);
}

template <int KS>
__device__ __forceinline__ void sweep_rows(const RcdClass &st, int w, int W, float *lds)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // the wave index is the same in all 64 lanes: tell the compiler, so that row
    // counters and row addresses live in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // the descriptor is the same for the whole workgroup: keep its fields in scalar registers
    const int ld = __builtin_amdgcn_readfirstlane(st.ld), nR = __builtin_amdgcn_readfirstlane(st.nR);
    const int K = __builtin_amdgcn_readfirstlane(st.K), nneed = __builtin_amdgcn_readfirstlane(st.nneed);
    const int JC = __builtin_amdgcn_readfirstlane(st.rpc), C = __builtin_amdgcn_readfirstlane(st.C);
    int kb[KS];
#pragma unroll
    for (int i = 0; i < KS; ++i) kb[i] = __builtin_amdgcn_readfirstlane(st.need[i < nneed ? i : nneed - 1]);
    const gcf32 M = (gcf32)st.M;
    const gcf32 cur = (gcf32)st.cur;
    const cci32 perm = (cci32)st.perm;
    const gf32 part = (gf32)st.part;
    const int stride = W * RCD_SWEEP_WAVES;
    const lf32 lcur = (lf32)lds;

    for (int c = 0; c < C; ++c) {
        const int j0 = c * JC;
        const int len = min(JC, ld - j0);   // a multiple of 256
        if (c > 0) __syncthreads();
        // (a plain loop over the slots: unrolled, the KS source pointers were kept in registers all at once
        // and the sixteen-slot variant spilled)
#pragma unroll 1
        for (int i = 0; i < KS; ++i) {
            const int k = __builtin_amdgcn_readfirstlane(st.need[i < nneed ? i : nneed - 1]);
            const gcf32 src = cur + (size_t)k * ld + j0;
            for (int e = tid * 4; e < len; e += RCD_SWEEP_THREADS * 4)
                *(f32x4 __attribute__((address_space(3))) *)(lcur + i * JC + e) = *(gcf32x4)(src + e);
        }
        __syncthreads();

        int p = w * RCD_SWEEP_WAVES + wave;
        int v = p < nR ? perm[p] : 0;
        while (p < nR) {
            const int pn = p + stride;
            const int vn = pn < nR ? perm[pn] : 0;   // next row's sample, fetched under this row's stream
            const gcf32 row = M + (size_t)v * ld + j0 + lane * 4;
            f32x4 acc[KS];
#pragma unroll
            for (int i = 0; i < KS; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
            int s = 0;
            // U row pieces of 1 KB in flight per wave (fewer when many blocks' sums fill the registers)
            constexpr int U = KS <= 8 ? 4 : 2;
            for (; s + 256 * U <= len; s += 256 * U) {
                f32x4 m[U];
#pragma unroll
                for (int u = 0; u < U; ++u) m[u] = __builtin_nontemporal_load((gcf32x4)(row + s + 256 * u));
#pragma unroll
                for (int i = 0; i < KS; ++i) {
                    const lcf32x4 cp = (lcf32x4)(lcur + i * JC + s + lane * 4);
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const f32x4 cc = cp[64 * u];
                        if constexpr (KS > 8) {
                            // one running sum per block, or sixteen blocks would not fit the registers
                            acc[i].x += (clamp01(m[u].x - cc.x) + clamp01(m[u].y - cc.y)) +
                                        (clamp01(m[u].z - cc.z) + clamp01(m[u].w - cc.w));
                        } else {
                            acc[i].x += clamp01(m[u].x - cc.x); acc[i].y += clamp01(m[u].y - cc.y);
                            acc[i].z += clamp01(m[u].z - cc.z); acc[i].w += clamp01(m[u].w - cc.w);
                        }
                    }
                }
            }
            if (s < len) {
                // the last, shorter batch (len is a multiple of 256): its pieces in flight together as well
                f32x4 m[U - 1];
#pragma unroll
                for (int u = 0; u < U - 1; ++u)
                    if (s + 256 * u < len) m[u] = __builtin_nontemporal_load((gcf32x4)(row + s + 256 * u));
#pragma unroll
                for (int u = 0; u < U - 1; ++u) {
                    if (s + 256 * u < len) {
#pragma unroll
                        for (int i = 0; i < KS; ++i) {
                            const f32x4 c0 = *(lcf32x4)(lcur + i * JC + s + 256 * u + lane * 4);
                            if constexpr (KS > 8) {
                                acc[i].x += (clamp01(m[u].x - c0.x) + clamp01(m[u].y - c0.y)) +
                                            (clamp01(m[u].z - c0.z) + clamp01(m[u].w - c0.w));
                            } else {
                                acc[i].x += clamp01(m[u].x - c0.x); acc[i].y += clamp01(m[u].y - c0.y);
                                acc[i].z += clamp01(m[u].z - c0.z); acc[i].w += clamp01(m[u].w - c0.w);
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < KS; ++i) {
                const float t = wave_sum((acc[i].x + acc[i].y) + (acc[i].z + acc[i].w));
                if (lane == 0 && i < nneed) part[((size_t)c * K + kb[i]) * ld + p] = t;
            }
            p = pn;
            v = vn;
        }
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

// ---------------------------------------------------------------------------
// Greedy steps of one class whose similarity is stored (M[v] = candidate v's row),
// one workgroup of NT threads.  Same loop as class_steps, arranged around trips
// to memory, of which a call makes three:
//   1. the class descriptor, copied to LDS;
//   2. the gain rows of every block that may step (current row, not full): each
//      thread scans its share of the candidates once and keeps its best per
//      block, one batched reduction leaves every block's argmax in LDS;
//      then the loop - argmin block, take that block's argmax, note the position
//      as removed - runs on LDS alone (if a block's argmax was taken by another
//      block earlier in the call, its row is scanned again without the removed
//      positions);
//   3. the consequences, all contiguous: coverage from the taken candidates' rows
//      of M, the last list entries (perm and every block's gains) moved into the
//      holes, the caller's arrays, the descriptor.
// The gain of a candidate is the sum of its chunk partials, as many as the sweep
// that built that block's row used.
// ---------------------------------------------------------------------------
struct RowsShared {
    RcdClass d;                                   // the descriptor, then the evolving copy
    unsigned long long wkey[RCD_KMAX][RCD_STEP_THREADS / 64];
    int wpos[RCD_KMAX][RCD_STEP_THREADS / 64];
    unsigned long long bkey[RCD_KMAX];            // argmax of block k's row: (gain bits, ~sample)
    int bpos[RCD_KMAX];
    int cand[RCD_KMAX], ncand;                    // blocks that may step in this call
    int removed[RCD_KMAX], nrem;                  // list positions taken in this call
    int hole[RCD_KMAX], src[RCD_KMAX], nmove;     // list compaction
};

// max over the wave of an unsigned value, same in every lane
__device__ __forceinline__ unsigned wave_max_u32(unsigned v)
{
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true));
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true));
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true));
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true));
    const unsigned r0 = __builtin_amdgcn_readlane((int)v, 0), r1 = __builtin_amdgcn_readlane((int)v, 16);
    const unsigned r2 = __builtin_amdgcn_readlane((int)v, 32), r3 = __builtin_amdgcn_readlane((int)v, 48);
    return max(max(r0, r1), max(r2, r3));
}

// wave-wide maximum of a packed key and the position that goes with it
__device__ __forceinline__ void wave_best(unsigned long long &key, int &pos)
{
    const unsigned hi = (unsigned)(key >> 32), lo = (unsigned)key;
    const unsigned mhi = wave_max_u32(hi);
    const unsigned mlo = wave_max_u32(hi == mhi ? lo : 0u);
    const unsigned long long who = __ballot(hi == mhi && lo == mlo);
    const int src = who ? __ffsll((long long)who) - 1 : 0;
    pos = __builtin_amdgcn_readlane(pos, src);
    key = ((unsigned long long)mhi << 32) | mlo;
}

// Algorithm 1's choice of the block: the non-full block of least f, lowest index on ties; -1 when every block is
// full.  d lives in LDS.  Lane k looks at block k (the lanes past RCD_KMAX repeat them), so the choice costs one
// trip to LDS and two wave reductions instead of a chain of K dependent reads; the result is the same in every
// lane and sits in a scalar register.  The least f is found as the largest order-preserving key of -f (-0 made +0).
__device__ __forceinline__ int least_open_block(const RcdClass &d, int K)
{
    static_assert((RCD_KMAX & (RCD_KMAX - 1)) == 0 && RCD_KMAX <= 64, "a lane per block");
    const int k = (int)(threadIdx.x & (RCD_KMAX - 1));
    const bool open = k < K && d.cnt[k] < d.cap[k];
    unsigned long long key = 0ull;               // below the key of any number
    if (open) {
        const unsigned long long b = (unsigned long long)__double_as_longlong(-d.f[k] + 0.0);
        key = (b >> 63) ? ~b : (b | 0x8000000000000000ull);
    }
    const unsigned hi = (unsigned)(key >> 32), lo = (unsigned)key;
    const unsigned mhi = wave_max_u32(hi);
    const unsigned mlo = wave_max_u32(hi == mhi ? lo : 0u);
    const unsigned long long who = __ballot(open && hi == mhi && lo == mlo);
    return who ? ((__ffsll((long long)who) - 1) & (RCD_KMAX - 1)) : -1;
}

template <int NT>
__device__ __forceinline__ void steps_rows(RcdClass &st, RcdPlan *plans, RowsShared &sh)
{
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // ---- trip 1: the descriptor
    {
        const gci32 g = (gci32)reinterpret_cast<const int32_t *>(&st);
        int32_t *l = reinterpret_cast<int32_t *>(&sh.d);
        for (int i = tid; i < (int)(sizeof(RcdClass) / 4); i += NT) l[i] = g[i];
    }
    __syncthreads();
    RcdClass &d = sh.d;
    if (d.done) {
        if (tid == 0) st.nneed = 0;
        return;
    }
    const long long tick0 = wall_clock64();
    // values that are the same in every lane are kept in scalar registers (uni), so that
    // addresses are "scalar base + lane offset" and the vector registers stay free for data
    auto uni = [](int x) { return __builtin_amdgcn_readfirstlane(x); };
    auto uni_ptr = [&](const void *q) {
        const unsigned long long a = reinterpret_cast<unsigned long long>(q);
        const unsigned lo = (unsigned)uni((int)(unsigned)a), hi = (unsigned)uni((int)(unsigned)(a >> 32));
        return ((unsigned long long)hi << 32) | lo;
    };
    const int K = uni(d.K), n = uni(d.n), ld = uni(d.ld), total = uni(d.total);
    const int nR0 = uni(d.nR), t0 = uni(d.t);
    const size_t cstride = (size_t)K * ld;
    const gcf32 part = (gcf32)reinterpret_cast<const float *>(uni_ptr(d.part));
    const gi32 perm = (gi32)reinterpret_cast<int32_t *>(uni_ptr(d.perm));
    // the sweep that ran since the last call rebuilt these rows
    if (tid < d.nneed) d.valid[d.need[tid]] = 1;
    __syncthreads();
    // the blocks that may step in this call, ascending (one lane per block and a ballot: a loop by one thread is a
    // chain of K dependent trips to LDS)
    static_assert(RCD_KMAX <= 64 && NW >= RCD_KMAX, "a lane per block, a wave per candidate block");
    if (tid < 64) {
        const bool c = tid < K && d.valid[tid] && d.cnt[tid] < d.cap[tid];
        const unsigned long long b = __ballot(c);
        if (c) sh.cand[__popcll(b & ((1ull << tid) - 1ull))] = tid;
        if (tid == 0) {
            sh.ncand = __popcll(b);
            sh.nrem = 0;
            sh.nmove = 0;
        }
    }
    __syncthreads();
    const int ncand = uni(sh.ncand);

    // ---- trip 2: every candidate block's argmax
    // scan of block k's row over the list positions not in removed[0 .. nrem)
    auto scan_row = [&](int k, int nrem, unsigned long long &best, int &bpos) {
        const gcf32 g = part + (size_t)k * ld;
        const int nchunk = uni(d.cblk[k]);
        constexpr int UA = 8;
        for (int p0 = 0; p0 < nR0; p0 += UA * NT) {
            float gv[UA];
            int pv[UA];
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                const int p = p0 + u * NT + tid;
                if (p < nR0) {
                    gv[u] = g[p];
                    pv[u] = perm[p];
                }
            }
            for (int c = 1; c < nchunk; ++c)
#pragma unroll
                for (int u = 0; u < UA; ++u) {
                    const int p = p0 + u * NT + tid;
                    if (p < nR0) gv[u] += g[c * cstride + p];
                }
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                const int p = p0 + u * NT + tid;
                if (p < nR0) {
                    bool gone = false;
                    for (int i = 0; i < nrem; ++i) gone |= sh.removed[i] == p;
                    const unsigned long long key = pack_key(gv[u], pv[u]);
                    if (!gone && key > best) { best = key; bpos = p; }
                }
            }
        }
    };
    // KC candidate blocks at once, from the i0-th on: KC x UB gains in flight per thread
    auto scan_all = [&](auto kc_tag, auto ub_tag, int i0) {
        constexpr int KC = decltype(kc_tag)::value, UB = decltype(ub_tag)::value;
        const int ncand = uni(sh.ncand) - i0;
        unsigned long long best[KC];
        int bpos[KC], kk[KC], nc[KC];
#pragma unroll
        for (int i = 0; i < KC; ++i) {
            best[i] = 0ull;
            bpos[i] = -1;
            kk[i] = uni(sh.cand[i < ncand ? i0 + i : 0]);
            nc[i] = uni(d.cblk[kk[i]]);
        }
        int ncmax = 1;
#pragma unroll
        for (int i = 0; i < KC; ++i) ncmax = max(ncmax, i < ncand ? nc[i] : 1);
        for (int p0 = 0; p0 < nR0; p0 += UB * NT) {
            float gv[KC][UB];
            int pv[UB];
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int p = p0 + u * NT + tid;
                if (p < nR0) {
                    pv[u] = perm[p];
#pragma unroll
                    for (int i = 0; i < KC; ++i)
                        if (i < ncand) gv[i][u] = part[(size_t)kk[i] * ld + p];
                }
            }
            // further chunk partials, if any block's row has them: kept out of the way of the
            // loads above, which must all be in flight together
            if (ncmax > 1) {
                for (int c = 1; c < ncmax; ++c)
#pragma unroll
                    for (int u = 0; u < UB; ++u) {
                        const int p = p0 + u * NT + tid;
#pragma unroll
                        for (int i = 0; i < KC; ++i)
                            if (p < nR0 && i < ncand && c < nc[i]) gv[i][u] += part[c * cstride + (size_t)kk[i] * ld + p];
                    }
            }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int p = p0 + u * NT + tid;
                if (p < nR0) {
#pragma unroll
                    for (int i = 0; i < KC; ++i)
                        if (i < ncand) {
                            const unsigned long long key = pack_key(gv[i][u], pv[u]);
                            if (key > best[i]) { best[i] = key; bpos[i] = p; }
                        }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < KC; ++i)
            if (i < ncand) {
                wave_best(best[i], bpos[i]);
                if (lane == 0) { sh.wkey[i0 + i][wave] = best[i]; sh.wpos[i0 + i][wave] = bpos[i]; }
            }
    };
    if (K <= 4) {
        if (ncand > 0) scan_all(std::integral_constant<int, 4>{}, std::integral_constant<int, 8>{}, 0);
    } else {
        for (int i0 = 0; i0 < ncand; i0 += 8) scan_all(std::integral_constant<int, 8>{}, std::integral_constant<int, 4>{}, i0);
    }
    __syncthreads();
    if (wave < ncand) {
        // wave i combines the waves' results for candidate block i, one per lane (largest key; equal keys name the
        // same sample or no sample, so which lane's position is taken does not matter)
        unsigned long long best = sh.wkey[wave][lane & (NW - 1)];
        int bpos = sh.wpos[wave][lane & (NW - 1)];
        wave_best(best, bpos);
        if (lane == 0) {
            sh.bkey[sh.cand[wave]] = best;
            sh.bpos[sh.cand[wave]] = bpos;
        }
    }
    __syncthreads();

    // ---- the loop (Algorithm 1's while body), on LDS
    int nR = nR0, t = t0, done = 0;
    long long useful = 0;
    for (;;) {
        if (t >= total) { done = 1; break; }
        const int js = least_open_block(d, K);
        if (js < 0) { done = 1; break; }
        if (!d.valid[js]) break;
        const int nrem = uni(sh.nrem);
        int pstar = sh.bpos[js];
        bool taken = false;
        for (int i = 0; i < nrem; ++i) taken |= sh.removed[i] == pstar;
        if (taken) {
            // another block took this block's best candidate earlier in the call
            unsigned long long best = 0ull;
            int bpos = -1;
            scan_row(js, nrem, best, bpos);
            wave_best(best, bpos);
            __syncthreads();   // everyone is past reading bkey/bpos/wkey of the previous step
            if (lane == 0) { sh.wkey[0][wave] = best; sh.wpos[0][wave] = bpos; }
            __syncthreads();
            if (tid == 0) {
                best = sh.wkey[0][0];
                bpos = sh.wpos[0][0];
                for (int w = 1; w < NW; ++w)
                    if (sh.wkey[0][w] > best) { best = sh.wkey[0][w]; bpos = sh.wpos[0][w]; }
                sh.bkey[js] = best;
                sh.bpos[js] = bpos;
            }
            __syncthreads();
            pstar = sh.bpos[js];
        }
        const unsigned long long key = sh.bkey[js];
        const float gbest = __uint_as_float((unsigned)(key >> 32));
        const int vstar = (int)(0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFull));
        __syncthreads();   // everyone has read the state this step was decided on
        if (tid == 0) {
            const int u = sh.nrem;
            sh.removed[u] = pstar;
            sh.nrem = u + 1;
            d.ujs[u] = js; d.uv[u] = vstar; d.ut[u] = t;
            d.cnt[js] += 1;
            d.f[js] += (double)gbest;
            d.valid[js] = 0;
        }
        useful += nR;
        nR -= 1;
        ++t;
        __syncthreads();
    }

    // ---- trip 3: consequences
    const int nupd = uni(sh.nrem);
    if (tid < 64) {
        // holes: removed positions below the new length, in the order they were taken; sources: the surviving
        // positions at or above it, ascending (as many as there are holes); the i-th hole is filled from the i-th
        // source.  Lane i holds the i-th removed position and looks at position nR + i; everything else is wave
        // operations (nupd <= K <= 64).
        const int mine = lane < nupd ? sh.removed[lane] : -1;
        bool gone = false;
        for (int q = 0; q < nupd; ++q) gone |= __builtin_amdgcn_readlane(mine, q) == nR + lane;
        const unsigned long long surv = __ballot(lane < nupd && !gone);
        const bool hole = lane < nupd && mine < nR;
        const unsigned long long holes = __ballot(hole);
        if (hole) {
            const int rank = __popcll(holes & ((1ull << lane) - 1ull));
            unsigned long long m = surv;
            for (int r = 0; r < rank; ++r) m &= m - 1ull;
            sh.hole[rank] = mine;
            sh.src[rank] = nR + (__ffsll((long long)m) - 1);
        }
        if (lane == 0) sh.nmove = __popcll(holes);
    }
    __syncthreads();
    const int nmove = uni(sh.nmove);
    {
        // coverage: cur_js(j) = max(cur_js(j), S(j, v*)); a block steps at most once per call,
        // so the updates touch different vectors and all loads can precede all stores
        const gcf32 M = (gcf32)reinterpret_cast<const float *>(uni_ptr(d.M));
        const gf32 cur = (gf32)reinterpret_cast<float *>(uni_ptr(d.cur));
        // two pieces of each vector per thread and trip: a class of up to 8192 samples needs one
        for (int u0 = 0; u0 < nupd; u0 += 4)
            for (int j0 = tid * 4; j0 < ld; j0 += NT * 8) {
                const int j1 = j0 + NT * 4;
                f32x4 m[2][4], c[2][4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (u0 + u < nupd) {
                        const gcf32 mr = M + (size_t)uni(d.uv[u0 + u]) * ld;
                        const gcf32 cr = cur + (size_t)uni(d.ujs[u0 + u]) * ld;
                        m[0][u] = *(gcf32x4)(mr + j0);
                        c[0][u] = *(gcf32x4)(cr + j0);
                        if (j1 < ld) {
                            m[1][u] = *(gcf32x4)(mr + j1);
                            c[1][u] = *(gcf32x4)(cr + j1);
                        }
                    }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (u0 + u < nupd) {
                        const gf32 cr = cur + (size_t)uni(d.ujs[u0 + u]) * ld;
                        f32x4 r;
                        r.x = fmaxf(c[0][u].x, m[0][u].x); r.y = fmaxf(c[0][u].y, m[0][u].y);
                        r.z = fmaxf(c[0][u].z, m[0][u].z); r.w = fmaxf(c[0][u].w, m[0][u].w);
                        *(gf32x4)(cr + j0) = r;
                        if (j1 < ld) {
                            r.x = fmaxf(c[1][u].x, m[1][u].x); r.y = fmaxf(c[1][u].y, m[1][u].y);
                            r.z = fmaxf(c[1][u].z, m[1][u].z); r.w = fmaxf(c[1][u].w, m[1][u].w);
                            *(gf32x4)(cr + j1) = r;
                        }
                    }
            }
        // list compaction: perm and every block's partial gains
        int cmax = 1;
        for (int k = 0; k < K; ++k) cmax = max(cmax, d.cblk[k]);
        const gf32 wpart = (gf32)reinterpret_cast<float *>(uni_ptr(d.part));
        for (int e = tid; e < nmove * K * cmax; e += NT) {
            const int i = e / (K * cmax), r = e % (K * cmax);   // r = chunk * K + block
            if (r / K < d.cblk[r % K]) wpart[(size_t)r * ld + sh.hole[i]] = wpart[(size_t)r * ld + sh.src[i]];
        }
        if (tid < nmove) perm[sh.hole[tid]] = perm[sh.src[tid]];
        if (tid < nupd) {
            const int v = d.uv[tid];
            const int oi = d.out_index ? d.out_index[v] : v;
            d.assign_out[oi] = d.ujs[tid];
            if (d.order_out) d.order_out[oi] = d.ut[tid];
        }
    }
    // every wave is done reading cblk[] (the compaction above) before thread 0 rewrites it
    __syncthreads();
    // ---- the descriptor: what the next sweep must do, the state, the counters
    if (tid < 64) {
        // the blocks whose gains the next sweep must produce, ascending (one lane per block again)
        const bool stale = !done && tid < K && d.cnt[tid] < d.cap[tid] && !d.valid[tid];
        const unsigned long long b = __ballot(stale);
        const int nneed = __popcll(b);
        // the coverage vectors of the evaluated blocks share the sweep workgroup's LDS:
        // the more blocks, the shorter the chunk of j one pass covers
        int jc = rcd_sweep_chunk(max(nneed, 1));
        jc = jc > ld ? ld : jc;
        const int C = (ld + jc - 1) / jc;
        if (stale) {
            d.need[__popcll(b & ((1ull << tid) - 1ull))] = tid;
            d.cblk[tid] = C;
        }
        if (tid == 0) {
            d.nneed = nneed;
            if (nneed > 0) {
                d.rpc = jc;
                d.C = C;
                d.stat_sweeps += 1;
                d.stat_entries += (long long)nR * n;
                d.stat_computed += (long long)nneed * nR;
            }
            d.stat_steps += t - t0;
            d.stat_useful += useful;
            d.nupd = nupd;
            d.npatch = nmove;
            d.apply_round += 1;
            d.nR = nR;
            d.t = t;
            d.done = done;
            d.stat_ticks += wall_clock64() - tick0;
            if (done) __hip_atomic_fetch_add(&plans[0].ndone, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
    {
        // everything from nR on changes; the fixed part in front of it stays as it is
        constexpr int first = (int)(offsetof(RcdClass, nR) / 4);
        gi32 g = (gi32)reinterpret_cast<int32_t *>(&st);
        const int32_t *l = reinterpret_cast<const int32_t *>(&sh.d);
        for (int i = first + tid; i < (int)(sizeof(RcdClass) / 4); i += NT) g[i] = l[i];
    }
}

// Stored similarity: one workgroup per class runs the class's steps; a round is
// the sweep launch and this one.  plans[0].ndone counts the finished classes.
extern "C" __global__ void __launch_bounds__(RCD_STEP_THREADS)
rcd_k_steps_rows(RcdClass *__restrict__ classes, RcdPlan *__restrict__ plans)
{
    __shared__ RowsShared sh;
    steps_rows<RCD_STEP_THREADS>(classes[blockIdx.x], plans, sh);
}

// Gain sweep of every class of a stored-similarity group.  The workgroups are dealt
// to the classes once, in proportion to their size (wgmap[b] = class, index among
// the class's workgroups, their count): a workgroup stays with one class, stages that
// class's coverage vectors once per pass and then only streams rows.
extern "C" __global__ void __launch_bounds__(RCD_SWEEP_THREADS)
rcd_k_sweep_rows(const RcdClass *__restrict__ classes, const RcdWg *__restrict__ wgmap)
{
    extern __shared__ __attribute__((aligned(16))) float lds_cur[];
    const RcdWg wg = wgmap[blockIdx.x];
    const RcdClass &st = classes[wg.cls];
    const int nneed = st.nneed;
    if (nneed <= 0 || st.done) return;
    // the variants are those rcd_sweep_slots() names: all KS slots of a variant are staged, so the
    // chunk length st.rpc was cut for KS slots, not for nneed
    if (nneed == 1) sweep_rows<1>(st, wg.w, wg.W, lds_cur);
    else if (nneed == 2) sweep_rows<2>(st, wg.w, wg.W, lds_cur);
    else if (nneed == 3) sweep_rows<3>(st, wg.w, wg.W, lds_cur);
    else if (nneed == 4) sweep_rows<4>(st, wg.w, wg.W, lds_cur);
    else if (nneed <= 6) sweep_rows<6>(st, wg.w, wg.W, lds_cur);
    else if (nneed <= 8) sweep_rows<8>(st, wg.w, wg.W, lds_cur);
    else if (nneed <= 12) sweep_rows<12>(st, wg.w, wg.W, lds_cur);
    else sweep_rows<16>(st, wg.w, wg.W, lds_cur);
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
    for (int i = i0; i < RCD_MW_INTS; i += stride) st.mwbuf[i] = 0;
    for (int i = i0; i < st.n && st.assign_out; i += stride) {
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

// Copy a caller's S (n x n, pitch lds) transposed into the working matrix (pitch ld):
// M[v][j] = S[j][v], so that candidate v's similarities to every j are one contiguous
// row whether or not S is symmetric; zero the pad columns; flag entries outside [0,1]
// or NaN.  grid = (ld/32, ceil(n/32)), 32 x 8 threads, one 32 x 32 tile through LDS.
extern "C" __global__ void __launch_bounds__(256)
rcd_k_copy_check(const float *__restrict__ S, long long lds, float *__restrict__ M, int ld, int n,
                 RcdPlan *plan)
{
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int jb = blockIdx.x * 32, vb = blockIdx.y * 32;
    int bad = 0;
    for (int r = ty; r < 32; r += 8) {
        const int j = jb + r, v = vb + tx;
        float x = 0.f;
        if (j < n && v < n) {
            x = S[(size_t)j * lds + v];
            if (!(x >= 0.f && x <= 1.f)) bad = 1;
        }
        tile[r][tx] = x;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int v = vb + r, j = jb + tx;
        if (v < n && j < ld) M[(size_t)v * ld + j] = tile[tx][r];
    }
    if (bad) plan->bad = 1;
}

// Test/benchmark helper behind rcd_gain_sweep: out[k][v] = gain[k][v] for v < n.
extern "C" __global__ void rcd_k_export_gains(const RcdClass *__restrict__ classes, float *__restrict__ out)
{
    const RcdClass &st = classes[0];
    const int v = blockIdx.x * blockDim.x + threadIdx.x;
    const int k = blockIdx.y;
    if (v < st.n) {
        float g = 0.f;
        for (int c = 0; c < st.C; ++c) g += st.part[((size_t)c * st.K + k) * st.ld + v];
        out[(size_t)k * st.n + v] = g;
    }
}

extern "C" __global__ void rcd_k_import_cur(const RcdClass *__restrict__ classes, const float *__restrict__ in)
{
    const RcdClass &st = classes[0];
    const int v = blockIdx.x * blockDim.x + threadIdx.x;
    const int k = blockIdx.y;
    if (v < st.n) st.cur[(size_t)k * st.ld + v] = in[(size_t)k * st.n + v];
}
