// Step loops of large classes run by several workgroups per class (gfx950).
//
// The step loops of the incremental-gain route and of the graph-cut function (Algorithm 1's inner
// while loop: argmin block, argmax sample, coverage / marginal-value update) are latency-bound, and
// with one workgroup per class a class of 50 000 samples pushes 2.3 MB per step through one compute
// unit.  Here W workgroups share a class.  Workgroup w owns the w-th slice of the class's samples,
// both as candidates v (its slice of every block's gains: scanned, updated and struck out by nobody
// else) and as rows j of the coverage vectors (its slice of cur_k).  What crosses workgroups in a
// step is small: each workgroup's best candidate (16 bytes), and for the incremental route the
// entries (j, old, new) of the coverage update, which every workgroup needs for its own candidates.
// Those go through device-scope stores and loads; the phases of a step are separated by an exchange
// among the class's W workgroups (every workgroup posts 16 bytes, and with them a list segment of up to three
// entries, and polls until it has read everybody's post for that exchange: see MwExchange), which is the step's
// barrier and carries its payload at once; longer segments are fetched from memory after the exchange.
//
// Every wait is bounded: a workgroup that has waited longer than `spin_ticks` (100 MHz ticks) raises
// plans[0].bad = 2 and every workgroup, seeing it, leaves its loop; the kernel always exits and the
// host reports the failure.  The host sizes the grid to what the device can hold at once (occupancy x
// compute units) and keeps such launches on one stream, so in normal operation a wait lasts microseconds.
//
// Results are those of the one-workgroup loops bit for bit: a gain is a per-candidate sum over the
// update list in list order (ascending j: the segments of workgroups 0, 1, ... in order), the argmax
// is the largest value with the lowest index wherever it sits, and f adds the same gains in the
// same order.  Included by rcd_lib.hip after incremental_kernels.hip.
#include <hip/hip_runtime.h>
#include "rcd_state.h"

namespace {

__device__ __forceinline__ float *inc_dnew(const RcdClass &st) { return st.part + 3 * (size_t)st.K * st.ld; }

// A pointer that is the same in every lane, moved into scalar registers (it then costs no vector register
// and addresses become "scalar base + lane offset").
template <typename P> __device__ __forceinline__ P *mw_uniform(P *q)
{
    const unsigned long long a = reinterpret_cast<unsigned long long>(q);
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)a);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32));
    return reinterpret_cast<P *>(((unsigned long long)hi << 32) | lo);
}

// An exchange among the W workgroups of a class: every workgroup posts three ints, then every workgroup
// has everybody's.  Also the barrier between the phases of a step (what a workgroup wrote with
// device-scope stores before posting is visible to whoever has read its post).
//
// A post is one 16-byte device-scope store {a, b, c, tag} into the workgroup's slot of the bank the
// exchange's number selects (two banks, used alternately: nobody can be two exchanges ahead of anybody,
// because completing one needs everybody's post for it).  tag = a hash of the exchange's number and of
// the three ints, never zero: a reader takes a slot only when its tag fits its contents and the current
// exchange, so a slot still holding an older post, a freshly zeroed one, or a (never observed) torn
// 16-byte read is simply read again.  No counter, no atomic: a store, then polls.
// An exchange "with entries" (the one that carries the lengths a of the list's segments) appends up to
// MW_INLINE more 16-byte pieces {j, old, new, tag} to the post, stored by the next lanes in the same instruction
// and each checked by its own tag: a workgroup whose segment has at most MW_INLINE entries sends them along, and
// nobody has to fetch that segment from memory afterwards (the usual case: 87 % of the steps of a 50 000-sample
// class have no longer segment).
// The exchange numbers of one partition call rise from launch to launch (epoch0 from the host).
// Every wait is bounded by `deadline`; when it runs out the flag *abort_flag is set to 2 and every
// workgroup that sees it gives up.
struct MwExchange {
    int32_t *banks;        // 2 x RCD_MW_MAX x 4 ints
    int32_t *abort_flag;   // plans[0].bad
    int W, w;
    unsigned epoch;
    long long deadline;
};

constexpr int MW_INLINE = 3;       // list entries that travel inside a post (a segment of at most this many does)

struct MwShared {
    int a[RCD_MW_MAX], b[RCD_MW_MAX], c[RCD_MW_MAX];
    int pre[RCD_MW_MAX + 1];
    int ok;
    int any_long;      // after an exchange of list segments: one of them is longer than MW_INLINE
    // my own first entries, staged by whoever found them, for my post
    int mj[MW_INLINE];
    float mo[MW_INLINE], mn[MW_INLINE];
};

__device__ __forceinline__ unsigned mw_tag(unsigned epoch, unsigned a, unsigned b, unsigned c)
{
    return ((epoch * 0x9E3779B1u) ^ a ^ ((b << 11) | (b >> 21)) ^ ((c << 22) | (c >> 10)) ^ 0xA5A5A5A5u) | 1u;
}

typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4 dev_load4(const int32_t *p)
{
    i32x4 v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(p) : "memory");
    return v;
}
// the four 16-byte pieces of a slot, requested together (one trip)
__device__ __forceinline__ void dev_load4x4(const int32_t *p, i32x4 &a, i32x4 &b, i32x4 &c, i32x4 &d)
{
    asm volatile("global_load_dwordx4 %0, %4, off sc1\n\t"
                 "global_load_dwordx4 %1, %4, off offset:16 sc1\n\t"
                 "global_load_dwordx4 %2, %4, off offset:32 sc1\n\t"
                 "global_load_dwordx4 %3, %4, off offset:48 sc1\n\t"
                 "s_waitcnt vmcnt(0)"
                 : "=&v"(a), "=&v"(b), "=&v"(c), "=&v"(d)
                 : "v"(p)
                 : "memory");
}
__device__ __forceinline__ void dev_store4i(int32_t *p, int a, int b, int c, int d)
{
    const i32x4 v = {a, b, c, d};
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}

// What the polling wave makes of the posts before it lets the workgroup go on (it has one post per lane in
// registers, so these are wave operations instead of loops over LDS by every thread):
//   MW_PLAIN  nothing: ms.a/b/c[0..W) hold the posts;
//   MW_BEST   (a, b) = a candidate's key, c = its sample: ms.a/b/c[0] hold the best of them (largest key, lowest
//             sample on ties);
//   MW_LIST   a = length of my list segment, which ms.mj/mo/mn hold and the post carries along when it has at most
//             MW_INLINE entries: ms.pre[i] = entries before workgroup i's, ms.pre[W] = all of them, ms.any_long =
//             some segment is longer than MW_INLINE (it has to be fetched), and the entries that came with the posts
//             are already in place in list_j/list_old/list_new (as far as list_cap reaches).
enum { MW_PLAIN = 0, MW_BEST = 1, MW_LIST = 2 };

// Every thread of the workgroup calls this with the same (a, b, c).
// publish: the workgroup has written memory that the others read after this exchange (a list segment longer than
// MW_INLINE); the post then waits for those stores.  Everything else a step writes is read back by the writing
// workgroup only.
template <int KIND>
__device__ __forceinline__ bool mw_exchange(MwExchange &x, MwShared &ms, int a, int b, int c, bool publish,
                                            int *list_j = nullptr, float *list_old = nullptr, float *list_new = nullptr,
                                            int list_cap = 0)
{
    const int tid = threadIdx.x;
    if (publish) wait_for_my_stores();      // what I wrote for the others has left this compute unit ...
    __syncthreads();                        // ... and so has what the rest of my workgroup wrote
    x.epoch += 1;
    const int mine_inline = KIND == MW_LIST && a <= MW_INLINE ? a : 0;
    int32_t *bank = x.banks + (x.epoch & 1u) * (MW_SLOT_INTS * RCD_MW_MAX);
    if (x.W > 1 && tid <= mine_inline) {
        // piece 0: the post proper; pieces 1..: my entries (their tags are tied to the exchange and to the piece)
        int p0 = a, p1 = b, p2 = c;
        if (tid > 0) { p0 = ms.mj[tid - 1]; p1 = __float_as_int(ms.mo[tid - 1]); p2 = __float_as_int(ms.mn[tid - 1]); }
        dev_store4i(bank + MW_SLOT_INTS * x.w + 4 * tid, p0, p1, p2,
                    (int)mw_tag(x.epoch + 0x01000000u * (unsigned)tid, (unsigned)p0, (unsigned)p1, (unsigned)p2));
    }
    if (tid < 64) {
        int ok = 0;
        i32x4 s = {0, 0, 0, 0};
        i32x4 e[MW_INLINE];
        for (;;) {
#pragma unroll
            for (int g = 0; g < MW_INLINE; ++g) e[g] = (i32x4){0, 0, 0, 0};
            s = (i32x4){0, 0, 0, 0};
            if (x.W == 1) {
                // alone: my post is the exchange
                if (tid == 0) {
                    s = (i32x4){a, b, c, 0};
#pragma unroll
                    for (int g = 0; g < MW_INLINE; ++g)
                        if (g < mine_inline) e[g] = (i32x4){ms.mj[g], __float_as_int(ms.mo[g]), __float_as_int(ms.mn[g]), 0};
                }
                ok = 1;
                break;
            }
            if (tid < x.W) {
                if (KIND == MW_LIST) dev_load4x4(bank + MW_SLOT_INTS * tid, s, e[0], e[1], e[2]);
                else s = dev_load4(bank + MW_SLOT_INTS * tid);
            }
            bool good = tid >= x.W || (unsigned)s.w == mw_tag(x.epoch, (unsigned)s.x, (unsigned)s.y, (unsigned)s.z);
            if (KIND == MW_LIST && tid < x.W && good && s.x <= MW_INLINE) {
#pragma unroll
                for (int g = 0; g < MW_INLINE; ++g)
                    if (g < s.x)
                        good = good && (unsigned)e[g].w == mw_tag(x.epoch + 0x01000000u * (unsigned)(g + 1), (unsigned)e[g].x,
                                                                   (unsigned)e[g].y, (unsigned)e[g].z);
            }
            if (__all(good)) {
                ok = 1;
                break;
            }
            if (__hip_atomic_load(x.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 2) break;
            if (wall_clock64() > x.deadline) {
                __hip_atomic_store(x.abort_flag, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        if (ok) {
            const bool have = tid < x.W;
            if (KIND == MW_PLAIN) {
                if (have) { ms.a[tid] = s.x; ms.b[tid] = s.y; ms.c[tid] = s.z; }
            } else if (KIND == MW_BEST) {
                unsigned long long key = have ? ((unsigned long long)(unsigned)s.x << 32) | (unsigned)s.y : 0ull;
                int bv = have ? s.z : 0x7fffffff;
                inc_wave_best(key, bv);
                if (tid == 0) { ms.a[0] = (int)(unsigned)(key >> 32); ms.b[0] = (int)(unsigned)key; ms.c[0] = bv; }
            } else {
                const int len = have ? s.x : 0;
                int incl = len;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const int up = __shfl_up(incl, off);
                    if (tid >= off) incl += up;
                }
                const int pre = incl - len;
                if (have) { ms.a[tid] = len; ms.pre[tid] = pre; }
                const unsigned long long lng = __ballot(have && len > MW_INLINE);
                if (tid == 63) { ms.pre[x.W] = incl; ms.any_long = lng != 0ull; }
                if (have && len <= MW_INLINE) {
#pragma unroll
                    for (int g = 0; g < MW_INLINE; ++g)
                        if (g < len && pre + g < list_cap) {
                            list_j[pre + g] = e[g].x;
                            list_old[pre + g] = __int_as_float(e[g].y);
                            list_new[pre + g] = __int_as_float(e[g].z);
                        }
                }
            }
        }
        if (tid == 0) ms.ok = ok;
    }
    __syncthreads();
    return ms.ok != 0;
}

// The class's best candidate from the workgroups' best: largest key, lowest sample on ties.
__device__ __forceinline__ bool mw_best_of_class(MwExchange &x, MwShared &ms, unsigned long long &key, int &bv)
{
    if (x.W == 1) return true;
    if (!mw_exchange<MW_BEST>(x, ms, (int)(unsigned)(key >> 32), (int)(unsigned)key, bv, false)) return false;
    key = ((unsigned long long)(unsigned)ms.a[0] << 32) | (unsigned)ms.b[0];
    bv = ms.c[0];
    return true;
}

} // namespace

// Greedy steps of the incremental-gain route, W workgroups of 1024 threads per class (wgmap[b] = class,
// index among the class's workgroups, their count).  Same loop and same limits as rcd_k_inc_steps.
// epoch0: exchanges done by this call's earlier launches (an upper bound; the numbers only have to rise).
extern "C" __global__ void __launch_bounds__(RCD_STEP_THREADS)
rcd_k_inc_steps_mw(RcdClass *__restrict__ classes, RcdPlan *__restrict__ plans, const RcdWg *__restrict__ wgmap,
                   int max_steps, int small_bytes, unsigned epoch0, long long spin_ticks)
{
    constexpr int NT = RCD_STEP_THREADS, NW = NT / 64;
    __shared__ IncShared sh;
    __shared__ MwShared ms;
    const RcdWg wg = wgmap[blockIdx.x];
    RcdClass &st = classes[wg.cls];
    const int w = wg.w, W = wg.W;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    {
        const gci32 g = (gci32)reinterpret_cast<const int32_t *>(&st);
        int32_t *l = reinterpret_cast<int32_t *>(&sh.d);
        for (int i = tid; i < (int)(sizeof(RcdClass) / 4); i += NT) l[i] = g[i];
    }
    __syncthreads();
    RcdClass &d = sh.d;
    if (d.done) {
        if (w == 0 && tid == 0) st.nneed = 0;
        return;
    }
    const long long tick0 = wall_clock64();
    MwExchange bar;
    bar.banks = mw_uniform(d.mwbuf) + MW_SLOT;
    bar.abort_flag = &plans[0].bad;
    bar.W = W;
    bar.w = w;
    bar.epoch = epoch0;
    bar.deadline = tick0 + spin_ticks;
    // everyone holds its copy of the descriptor before anyone may write it back
    if (!mw_exchange<MW_PLAIN>(bar, ms, 0, 0, 0, false)) return;

    const int K = d.K, n = d.n, ld = d.ld, total = d.total;
    if (tid < d.nneed) d.valid[d.need[tid]] = 1;      // the update launch brought these blocks' gains up to date
    __syncthreads();
    double *G = mw_uniform(inc_gains(d));
    int32_t *dlist = mw_uniform(inc_dlist(d));
    float *dold = mw_uniform(inc_dold(d)), *dnew = mw_uniform(inc_dnew(d));
    const gcf32 M = (gcf32)mw_uniform(d.M);
    float *cur_all = mw_uniform(d.cur);
    // my slice of the samples: candidates v and coverage rows j alike
    const int mwseg = __builtin_amdgcn_readfirstlane(d.mwseg);
    const int v0 = min(w * mwseg, ld), v1 = min(v0 + mwseg, ld), nv = max(min(v1, n) - v0, 0);
    const int seg = ((v1 - v0 + NW - 1) / NW + 255) / 256 * 256;      // j range of a wave inside the slice
    // lists up to this many rows are applied right here, every workgroup on its own candidates
    const long long row_bytes = (long long)ld * 4;
    const int small = (int)max(4LL, min((long long)INC_SMALL, (long long)small_bytes * W / row_bytes));
    int32_t *mwbuf = mw_uniform(d.mwbuf);

    int nR = d.nR, t = d.t, done = 0;
    const int t0 = t;
    bool alive = true;
    long long useful = 0, entries = 0, computed = 0, sweeps = 0;
    for (;;) {
        if (t >= total) { done = 1; break; }
        if (t - t0 >= max_steps) break;
        const int js = least_open_block(d, K);
        if (js < 0) { done = 1; break; }
        if (!d.valid[js]) break;

        // ---- argmax over my slice of the block's gains, then over the class
        double best = INC_LIVE_ABOVE;
        int bv = 0x7fffffff;
        inc_scan<NT>(G + (size_t)js * ld + v0, nv, tid, best, bv);
        if (bv != 0x7fffffff) bv += v0;
        unsigned long long key = inc_key(best);
        inc_wave_best(key, bv);
        if (lane == 0) { sh.wkey[wave] = key; sh.wv[wave] = bv; }
        __syncthreads();
        // every wave takes the waves' results one per lane and reduces them again: one read of LDS and three wave
        // reductions instead of a chain over NW entries
        static_assert((NW & (NW - 1)) == 0 && NW <= 64, "a lane per wave");
        key = sh.wkey[lane & (NW - 1)];
        bv = sh.wv[lane & (NW - 1)];
        inc_wave_best(key, bv);
        if (!mw_best_of_class(bar, ms, key, bv)) { alive = false; break; }
        best = inc_value(key);
        const int vstar = bv;
        if (vstar >= n) { done = 1; break; }          // no candidate left (cannot happen while t < total <= n)

        // ---- bookkeeping (every workgroup keeps the same copy of the state) and outputs (workgroup 0)
        __syncthreads();                              // everyone has read the block state this step was decided on
        int oi = vstar;              // asked for now, used at the end of the step (see rcd_k_inc_steps)
        if (tid == 0) {
            d.cnt[js] += 1;
            d.f[js] += best;
            if (w == 0 && d.out_index) oi = d.out_index[vstar];
        }
        if (tid < K && vstar >= v0 && vstar < v1) G[(size_t)tid * ld + vstar] = INC_TAKEN;

        // ---- coverage update on my rows j: cur_js(j) = max(cur_js(j), S(j, v*)); the changed j, ascending,
        //      with their old and new values, go to my segment of the block's list (at my slice's offset)
        const gcf32 row = M + (size_t)vstar * ld;
        float *cur = cur_all + (size_t)js * ld;
        const int j_begin = min(v0 + wave * seg, v1), j_end = min(j_begin + seg, v1);
        // A wave's range is at most two pieces of 256 when the slice is at most 8192 samples (the usual case):
        // both pieces of the row and of the coverage vector are fetched in one trip and kept for the write-out.
        const bool two = seg <= 512;
        f32x4 pm[2], pc[2];
        int cnt = 0;
        if (two) {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int s = j_begin + lane * 4 + p * 256;
                if (s < j_end) {
                    pm[p] = *(gcf32x4)(row + s);
                    pc[p] = *(const f32x4 *)(cur + s);
                } else {
                    pm[p] = (f32x4){0.f, 0.f, 0.f, 0.f};
                    pc[p] = (f32x4){0.f, 0.f, 0.f, 0.f};
                }
            }
#pragma unroll
            for (int p = 0; p < 2; ++p)
                cnt += (pm[p].x > pc[p].x) + (pm[p].y > pc[p].y) + (pm[p].z > pc[p].z) + (pm[p].w > pc[p].w);
        } else {
            for (int s = j_begin + lane * 4; s < j_end; s += 256) {
                const f32x4 m = *(gcf32x4)(row + s);
                const f32x4 c = *(const f32x4 *)(cur + s);
                cnt += (m.x > c.x) + (m.y > c.y) + (m.z > c.z) + (m.w > c.w);
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) cnt += __shfl_xor(cnt, off);
        if (lane == 0) sh.wcount[wave] = cnt;
        __syncthreads();
        int base = 0, mine = 0;
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int c = sh.wcount[i];
            if (i < wave) base += c;
            mine += c;
        }
        if (cnt > 0) {
            gi32 dl = (gi32)(dlist + (size_t)js * ld + v0);
            gf32 dol = (gf32)(dold + (size_t)js * ld + v0), dnw = (gf32)(dnew + (size_t)js * ld + v0);
            // one piece: its changed entries, in ascending j, appended at `base`; the piece's coverage raised
            auto write_piece = [&](int s, const f32x4 &m, const f32x4 &c) {
                const bool ch[4] = {m.x > c.x, m.y > c.y, m.z > c.z, m.w > c.w};
                const int here = ch[0] + ch[1] + ch[2] + ch[3];
                int incl = here;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const int up = __shfl_up(incl, off);
                    if (lane >= off) incl += up;
                }
                int pos = base + incl - here;
                const float mv[4] = {m.x, m.y, m.z, m.w}, cv[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (ch[q]) {
                        dev_store(dl + pos, s + q);
                        dev_store(dol + pos, cv[q]);
                        dev_store(dnw + pos, mv[q]);
                        if (pos < MW_INLINE) { ms.mj[pos] = s + q; ms.mo[pos] = cv[q]; ms.mn[pos] = mv[q]; }   // for my post
                        ++pos;
                    }
                if (here) {
                    f32x4 r;
                    r.x = fmaxf(c.x, m.x); r.y = fmaxf(c.y, m.y); r.z = fmaxf(c.z, m.z); r.w = fmaxf(c.w, m.w);
                    *(f32x4 *)(cur + s) = r;
                }
                base += __shfl(incl, 63);
            };
            if (two) {
#pragma unroll
                for (int p = 0; p < 2; ++p) write_piece(j_begin + lane * 4 + p * 256, pm[p], pc[p]);
            } else {
                for (int s = j_begin + lane * 4; s < j_end; s += 256) {
                    const f32x4 m = *(gcf32x4)(row + s);
                    const f32x4 c = *(const f32x4 *)(cur + s);
                    write_piece(s, m, c);
                }
            }
        }
        // ---- the whole list: every workgroup's segment, in order (the exchange carries the segment lengths)
        //      (a segment of at most MW_INLINE entries travels in the post itself: nobody reads it from memory in this
        //      launch, so the post does not wait for those stores)
        if (!mw_exchange<MW_LIST>(bar, ms, mine, 0, 0, mine > MW_INLINE, sh.sj, sh.sold, sh.snew, INC_SMALL)) { alive = false; break; }
        const int nd = ms.pre[W];
        entries += (long long)nd * n;
        computed += nR - 1;
        if (nd > small) {
            // long list: left to the update launch (which walks the segments), the block sits out until then
            if (tid == 0) {
                d.valid[js] = 0;
                d.dcount[js] = nd;
                mwbuf[MW_PEND + js * RCD_MW_MAX + w] = mine;
            }
            sweeps += 1;
        } else if (nd > 0) {
            // the entries that came with the posts are in sh.sj/sold/snew already; longer segments are fetched
            if (ms.any_long) {
                for (int e = tid; e < nd; e += NT) {
                    int i = 0;
                    while (e >= ms.pre[i + 1]) ++i;
                    if (ms.a[i] > MW_INLINE) {
                        const size_t at = (size_t)js * ld + (size_t)i * mwseg + (e - ms.pre[i]);
                        sh.sj[e] = dev_load((gci32)(dlist + at));
                        sh.sold[e] = dev_load((gcf32)(dold + at));
                        sh.snew[e] = dev_load((gcf32)(dnew + at));
                    }
                }
                __syncthreads();
            }
            double *gj = G + (size_t)js * ld;
            // A thread's candidates in a stretch of NT * 5 samples of the slice: four in a row at 4 tid, and sample
            // NT * 4 + tid (a slice a little over NT * 4 samples, the usual case, is then one stretch).
            for (int sb = v0; sb < v1; sb += NT * 5) {
                const int vv = sb + tid * 4;               // v1 - v0 is a multiple of 4: a piece is whole or absent
                const int vx = sb + NT * 4 + tid;
                const bool piece = vv < v1, single = vx < v1;
                if (!piece && !single) continue;
                // (what a thread has no use for is loaded from the stretch's first sample)
                const int pv = piece ? vv : sb, px = single ? vx : sb;
                double acc[4] = {0.0, 0.0, 0.0, 0.0}, accx = 0.0;
                // U rows of the list from e0 on, all requested before the first is used; past the list's end its last
                // row again (a register left undefined on some path would be kept alive around the whole step loop).
                // The list is taken eight rows at a time and its tail in the smallest of 1, 2, 4, 8 that holds it: most
                // lists are a row or two, and every load, wanted or not, costs the memory pipeline its turn.
                auto rows = [&](auto u_tag, int e0) {
                    constexpr int U = decltype(u_tag)::value;
                    f32x4 m[U];
                    float x[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const gcf32 r = M + (size_t)sh.sj[min(e0 + u, nd - 1)] * ld;
                        m[u] = *(gcf32x4)(r + pv);
                        x[u] = r[px];
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        if (e0 + u < nd) {
                            const float cn = sh.snew[e0 + u], co = sh.sold[e0 + u];
                            acc[0] += inc_term(m[u].x, cn, co);
                            acc[1] += inc_term(m[u].y, cn, co);
                            acc[2] += inc_term(m[u].z, cn, co);
                            acc[3] += inc_term(m[u].w, cn, co);
                            accx += inc_term(x[u], cn, co);
                        }
                };
                int e0 = 0;
                for (; nd - e0 > 4; e0 += 8) rows(std::integral_constant<int, 8>{}, e0);
                if (nd - e0 > 2) rows(std::integral_constant<int, 4>{}, e0);
                else if (nd - e0 == 2) rows(std::integral_constant<int, 2>{}, e0);
                else if (nd - e0 == 1) rows(std::integral_constant<int, 1>{}, e0);
                if (piece) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) gj[vv + c] += acc[c];
                }
                if (single) gj[vx] += accx;
            }
        }
        if (tid == 0 && w == 0) {
            d.assign_out[oi] = js;
            if (d.order_out) d.order_out[oi] = t;
        }
        useful += nR;
        nR -= 1;
        ++t;
        __syncthreads();           // the step's writes (gains, LDS state) are in place
    }
    if (!alive) return;            // a bounded wait ran out: plans[0].bad says so, nothing is written back

    // ---- the descriptor, by workgroup 0 (every workgroup holds the same copy)
    __syncthreads();
    if (w != 0) return;
    if (tid == 0) {
        int nneed = 0;
        if (!done)
            for (int k = 0; k < K; ++k)
                if (d.cnt[k] < d.cap[k] && !d.valid[k]) d.need[nneed++] = k;
        d.nneed = nneed;
        d.stat_sweeps += sweeps;
        d.stat_entries += entries;
        d.stat_computed += computed;
        d.stat_steps += t - t0;
        d.stat_useful += useful;
        d.nR = nR;
        d.t = t;
        d.done = done;
        d.stat_ticks += wall_clock64() - tick0;
        if (done) __hip_atomic_fetch_add(&plans[0].ndone, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    {
        constexpr int first = (int)(offsetof(RcdClass, nR) / 4);
        gi32 g = (gi32)reinterpret_cast<int32_t *>(&st);
        const int32_t *l = reinterpret_cast<const int32_t *>(&sh.d);
        for (int i = first + tid; i < (int)(sizeof(RcdClass) / 4); i += NT) g[i] = l[i];
    }
}

// Greedy steps with the graph-cut function, W workgroups per class: a step is a scan of my slice of
// the block's marginal values, one exchange of the workgroups' best candidates, and row v* of S taken
// off my slice.  One exchange per step.
extern "C" __global__ void __launch_bounds__(RCD_STEP_THREADS)
rcd_k_gc_steps_mw(RcdClass *__restrict__ classes, RcdPlan *__restrict__ plans, const RcdWg *__restrict__ wgmap,
                  int max_steps, unsigned epoch0, long long spin_ticks)
{
    constexpr int NT = RCD_STEP_THREADS, NW = NT / 64;
    __shared__ IncShared sh;
    __shared__ MwShared ms;
    const RcdWg wg = wgmap[blockIdx.x];
    RcdClass &st = classes[wg.cls];
    const int w = wg.w, W = wg.W;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    {
        const gci32 g = (gci32)reinterpret_cast<const int32_t *>(&st);
        int32_t *l = reinterpret_cast<int32_t *>(&sh.d);
        for (int i = tid; i < (int)(sizeof(RcdClass) / 4); i += NT) l[i] = g[i];
    }
    __syncthreads();
    RcdClass &d = sh.d;
    if (d.done) return;
    const long long tick0 = wall_clock64();
    MwExchange bar;
    bar.banks = mw_uniform(d.mwbuf) + MW_SLOT;
    bar.abort_flag = &plans[0].bad;
    bar.W = W;
    bar.w = w;
    bar.epoch = epoch0;
    bar.deadline = tick0 + spin_ticks;
    if (!mw_exchange<MW_PLAIN>(bar, ms, 0, 0, 0, false)) return;

    const int K = d.K, n = d.n, ld = d.ld, total = d.total;
    double *G = inc_gains(d);
    const gcf32 M = (gcf32)d.M;
    const int mwseg = d.mwseg;
    const int v0 = min(w * mwseg, ld), v1 = min(v0 + mwseg, ld), nv = max(min(v1, n) - v0, 0);
    int nR = d.nR, t = d.t, done = 0;
    const int t0 = t;
    bool alive = true;
    long long useful = 0;
    for (;;) {
        if (t >= total) { done = 1; break; }
        if (t - t0 >= max_steps) break;
        const int js = least_open_block(d, K);
        if (js < 0) { done = 1; break; }
        double *g = G + (size_t)js * ld;
        double best = INC_LIVE_ABOVE;
        int bv = 0x7fffffff;
        inc_scan<NT>(g + v0, nv, tid, best, bv);
        if (bv != 0x7fffffff) bv += v0;
        unsigned long long key = inc_key(best);
        inc_wave_best(key, bv);
        if (lane == 0) { sh.wkey[wave] = key; sh.wv[wave] = bv; }
        __syncthreads();
        // every wave takes the waves' results one per lane and reduces them again: one read of LDS and three wave
        // reductions instead of a chain over NW entries
        static_assert((NW & (NW - 1)) == 0 && NW <= 64, "a lane per wave");
        key = sh.wkey[lane & (NW - 1)];
        bv = sh.wv[lane & (NW - 1)];
        inc_wave_best(key, bv);
        if (!mw_best_of_class(bar, ms, key, bv)) { alive = false; break; }
        best = inc_value(key);
        const int vstar = bv;
        if (vstar >= n) { done = 1; break; }
        __syncthreads();                              // everyone has read the block state this step was decided on
        int oi = vstar;              // asked for now, used at the end of the step (see rcd_k_inc_steps)
        if (tid == 0) {
            d.cnt[js] += 1;
            d.f[js] += best;
            if (w == 0 && d.out_index) oi = d.out_index[vstar];
        }
        // ---- every marginal value of the block drops by 2 S(v, v*), on my slice
        const gcf32 row = M + (size_t)vstar * ld;
        for (int vv = v0 + tid * 4; vv < v1; vv += NT * 8) {
            // two pieces of four per thread and trip (a slice a little over NT * 4 samples is one round)
            const int vw = vv + NT * 4;
            const bool second = vw < v1;
            const f32x4 m0 = *(gcf32x4)(row + vv);
            f32x4 m1 = m0;
            double o0[4], o1[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) o0[c] = g[vv + c];
            if (second) {
                m1 = *(gcf32x4)(row + vw);
#pragma unroll
                for (int c = 0; c < 4; ++c) o1[c] = g[vw + c];
            }
            g[vv] = o0[0] - 2.0 * (double)m0.x;
            g[vv + 1] = o0[1] - 2.0 * (double)m0.y;
            g[vv + 2] = o0[2] - 2.0 * (double)m0.z;
            g[vv + 3] = o0[3] - 2.0 * (double)m0.w;
            if (second) {
                g[vw] = o1[0] - 2.0 * (double)m1.x;
                g[vw + 1] = o1[1] - 2.0 * (double)m1.y;
                g[vw + 2] = o1[2] - 2.0 * (double)m1.z;
                g[vw + 3] = o1[3] - 2.0 * (double)m1.w;
            }
        }
        // v* leaves every block's candidates: its owner strikes it out (in the served block, the thread that has
        // just updated that entry: its own earlier store to the same address)
        if (vstar >= v0 && vstar < v1) {
            if (((vstar - v0) >> 2) % NT == tid) g[vstar] = INC_TAKEN;
            if (tid < K && tid != js) G[(size_t)tid * ld + vstar] = INC_TAKEN;
        }
        if (tid == 0 && w == 0) {
            d.assign_out[oi] = js;
            if (d.order_out) d.order_out[oi] = t;
        }
        useful += nR;
        nR -= 1;
        ++t;
        __syncthreads();
    }
    if (!alive) return;
    __syncthreads();
    if (w != 0) return;
    if (tid == 0) {
        d.nneed = 0;
        d.stat_steps += t - t0;
        d.stat_useful += useful;
        d.stat_entries += (long long)(t - t0) * n;
        d.nR = nR;
        d.t = t;
        d.done = done;
        d.stat_ticks += wall_clock64() - tick0;
        if (done) __hip_atomic_fetch_add(&plans[0].ndone, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    {
        constexpr int first = (int)(offsetof(RcdClass, nR) / 4);
        gi32 gd = (gi32)reinterpret_cast<int32_t *>(&st);
        const int32_t *l = reinterpret_cast<const int32_t *>(&sh.d);
        for (int i = first + tid; i < (int)(sizeof(RcdClass) / 4); i += NT) gd[i] = l[i];
    }
}
