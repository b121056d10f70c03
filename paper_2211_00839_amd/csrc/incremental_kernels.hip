// Class greedy with incrementally maintained gains (stored similarity), for gfx950.
//
// Algorithm 1's loop is unchanged: j* = the non-full block of least f, v* = the unassigned
// sample of largest gain f(A_j* u {v}) - f(A_j*), lowest index on ties.  What changes is how a
// block's gains are kept current.  With the facility-location function of Section 4,
//     gain_k(v) = sum_j max(0, S(j,v) - cur_k(j)),     cur_k(j) = max_{a in A_k} S(j,a),
// taking v* into block k raises cur_k only on D = { j : S(j,v*) > cur_k(j) }, so
//     gain_k(v) += sum_{j in D} [ max(0, S(j,v) - new_j) - max(0, S(j,v) - old_j) ]      for every v.
// D is the whole class for a block's first sample and shrinks quickly after that (a dozen rows
// after a few hundred samples on mixture data), so a step reads |D| rows of S instead of one row
// per candidate.  The gains start as the column sums of S (all cur = 0).
//
// Precision.  A gain shrinks by five orders of magnitude over a run while being updated thousands
// of times, so the running values are kept in double: every term is a difference of two fp32 numbers
// taken in double, hence exact, and the sums are good to ~1e-13 relative.  Two candidates with
// identical columns go through identical operations in identical order, so exact ties stay exact
// and the lowest index wins them.
//
// Layout (inside the buffers every class owns; see inc_* below): gains G[k][v] in sample order
// (a taken sample's entries are set to a large negative sentinel), and per block the list of the
// changed j in ascending order with their old coverage values (the new ones are in cur).
// Included by rcd_lib.hip after greedy_kernels.hip.
#include <hip/hip_runtime.h>
#include "rcd_state.h"

namespace {

constexpr double INC_TAKEN = -1.0e300;      // gain entry of a sample that is no longer a candidate
constexpr double INC_LIVE_ABOVE = -1.0e299; // anything above this is a live candidate's gain
constexpr int INC_STAGE = 32;               // changed j a wave can hold back in LDS during that single pass
constexpr int INC_SMALL = 512;              // most rows of an update list that the step loop applies itself (LDS copy of the list)

__device__ __forceinline__ double *inc_gains(const RcdClass &st) { return reinterpret_cast<double *>(st.part); }
__device__ __forceinline__ float *inc_dold(const RcdClass &st) { return st.part + 2 * (size_t)st.K * st.ld; }
__device__ __forceinline__ int32_t *inc_dlist(const RcdClass &st) { return reinterpret_cast<int32_t *>(st.gain); }

// One term of the update, in double: max(0, s - new) - max(0, s - old) with old < new, written as
// -min(clamp(s - old, 0, 1), new - old) (s <= old: 0; old < s <= new: old - s; s > new: old - new; the upper
// clamp never bites because the similarities lie in [0, 1]).  Every kernel of this route takes its terms from here,
// so a gain is the same number whichever of them applied an update.
__device__ __forceinline__ double inc_term(float s, float new_c, float old_c)
{
    const double od = (double)old_c;
    const double w = (double)new_c - od;
    const double x = fmin(fmax((double)s - od, 0.0), 1.0);
    return -fmin(x, w);
}

constexpr int INC_FUSE_MAX = 8;             // most blocks whose pending lists one fused update pass applies

// Whether a class's pending lists are applied by rcd_k_inc_update_fused (one walk over the union of the lists'
// rows) instead of list by list: two to eight blocks wait, the byte-per-sample membership table fits lds_bytes,
// and the lists together hold at least pct percent of the class (then many rows are on several lists and the fused
// pass reads such a row once).  Both update kernels evaluate this on the same descriptor, so exactly one of
// them serves a class.  lds_bytes = 0 switches the fused pass off.
__device__ __forceinline__ bool inc_fused(const RcdClass &st, int lds_bytes, int pct)
{
    const int nneed = st.nneed;
    if (lds_bytes <= 0 || nneed < 2 || nneed > INC_FUSE_MAX || st.ld > lds_bytes) return false;
    long long tot = 0;
    for (int s = 0; s < nneed; ++s) tot += max(st.dcount[st.need[s]], 0);
    return tot * 100 >= (long long)pct * st.n;
}

__device__ __forceinline__ double wave_sum_f64(double a)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) a += __shfl_xor(a, off);   // partners add the same two numbers
    return a;
}

} // namespace

// Initial gains: G[k][v] = sum_j S(j,v) for every block (all coverage vectors are 0), one wave
// per candidate row of M, double accumulation in a fixed order.  grid = (ceil(max n / 4), ncls).
extern "C" __global__ void __launch_bounds__(256)
rcd_k_inc_init(const RcdClass *__restrict__ classes)
{
    const RcdClass &st = classes[blockIdx.y];
    const int lane = threadIdx.x & 63;
    const int v = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= st.n) return;
    const int ld = st.ld, K = st.K;
    const gcf32 row = (gcf32)st.M + (size_t)v * ld + lane * 4;
    double a = 0.0;
    for (int s = 0; s < ld; s += 256) {
        const f32x4 m = *(gcf32x4)(row + s);
        a += ((double)m.x + (double)m.y) + ((double)m.z + (double)m.w);
    }
    a = wave_sum_f64(a);
    if (lane < K) inc_gains(st)[(size_t)lane * ld + v] = a;
}

// Apply the pending update lists: for every class, every block with a pending list, every tile of
// 1024 samples v:  G[k][v] += sum over the list of the term above, added in list order.  Each of the
// workgroup's 4 waves takes 256 samples and walks the whole list, eight rows in flight; the four waves
// read neighbouring kilobytes of the same rows at about the same time.
// grid = (ceil(max ld / 1024), K, ncls).
extern "C" __global__ void __launch_bounds__(256)
rcd_k_inc_update(const RcdClass *__restrict__ classes, int fuse_lds_bytes, int fuse_pct)
{
    const RcdClass &st = classes[blockIdx.z];
    const int slot = blockIdx.y;
    if (st.done || slot >= st.nneed) return;
    if (inc_fused(st, fuse_lds_bytes, fuse_pct)) return;      // the fused pass serves this class
    const int k = st.need[slot];
    const int ld = st.ld;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int v0 = blockIdx.x * 1024 + wave * 256;
    if (st.dcount[k] <= 0 || v0 >= ld) return;
    const ccf32 cur = (ccf32)(st.cur + (size_t)k * ld);
    const gcf32 M = (gcf32)st.M + v0 + lane * 4;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    // The list is one run of dcount entries, or, when several workgroups share the class's step loop, one
    // segment per workgroup at the offset of its slice of the samples (ascending j across the segments).
    const int nseg = st.mw > 1 ? st.mw : 1;
    for (int sg = 0; sg < nseg; ++sg) {
        const int nd = st.mw > 1 ? st.mwbuf[MW_PEND + k * RCD_MW_MAX + sg] : st.dcount[k];
        const size_t off = (size_t)k * ld + (st.mw > 1 ? (size_t)sg * st.mwseg : 0);
        const cci32 dl = (cci32)(inc_dlist(st) + off);
        const ccf32 dold = (ccf32)(inc_dold(st) + off);
        int e = 0;
        constexpr int U = 8;      // rows in flight per wave
        for (; e + U <= nd; e += U) {
            f32x4 m[U];
            float cn[U], co[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = dl[e + u];
                cn[u] = cur[j];
                co[u] = dold[e + u];
                m[u] = __builtin_nontemporal_load((gcf32x4)(M + (size_t)j * ld));
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                acc[0] += inc_term(m[u].x, cn[u], co[u]);
                acc[1] += inc_term(m[u].y, cn[u], co[u]);
                acc[2] += inc_term(m[u].z, cn[u], co[u]);
                acc[3] += inc_term(m[u].w, cn[u], co[u]);
            }
        }
        for (; e < nd; ++e) {
            const int j = dl[e];
            const float cn = cur[j], co = dold[e];
            const f32x4 m = __builtin_nontemporal_load((gcf32x4)(M + (size_t)j * ld));
            acc[0] += inc_term(m.x, cn, co);
            acc[1] += inc_term(m.y, cn, co);
            acc[2] += inc_term(m.z, cn, co);
            acc[3] += inc_term(m.w, cn, co);
        }
    }
    double *g = inc_gains(st) + (size_t)k * ld + v0 + lane * 4;
#pragma unroll
    for (int c = 0; c < 4; ++c) g[c] += acc[c];
}

namespace {

__device__ __forceinline__ float inc_lane_value(float x, int l)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}

// U rows of one 64-row group (the lowest U set bits of `rows`, which has at least U): loads first, then every row's
// terms for the blocks it is listed for.  mb: this lane's row's membership byte; cnv/cov: per block, this lane's row's
// new and old coverage.
template <int U>
__device__ __forceinline__ void inc_fused_rows(unsigned long long &rows, unsigned mb, const float (&cnv)[INC_FUSE_MAX],
                                               const float (&cov)[INC_FUSE_MAX], gcf32 Mj0, int ld,
                                               double (&acc)[INC_FUSE_MAX][4])
{
    int bit[U];
    unsigned mk[U];
    f32x4 m[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        bit[u] = (int)__builtin_ctzll(rows);
        rows &= rows - 1ull;
        mk[u] = (unsigned)__builtin_amdgcn_readlane((int)mb, bit[u]);
        m[u] = __builtin_nontemporal_load((gcf32x4)(Mj0 + (size_t)bit[u] * ld));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int s = 0; s < INC_FUSE_MAX; ++s) {
            if ((mk[u] >> s) & 1u) {
                const float cn = inc_lane_value(cnv[s], bit[u]), co = inc_lane_value(cov[s], bit[u]);
                acc[s][0] += inc_term(m[u].x, cn, co);
                acc[s][1] += inc_term(m[u].y, cn, co);
                acc[s][2] += inc_term(m[u].z, cn, co);
                acc[s][3] += inc_term(m[u].w, cn, co);
            }
        }
    }
}

} // namespace

// The same update for a class whose pending lists overlap (inc_fused above): one walk over the samples j in
// ascending order, a row of S read once and its terms added to every block that lists j.  A block's gains
// receive the same terms in the same order as from rcd_k_inc_update, hence the same bits.
// The workgroup first marks, in a table of one byte per sample in LDS, which blocks list which j (bit s: block
// need[s]); then each of its 4 waves takes 256 samples v and walks the table 64 rows at a time: the group's
// coverage values (new from cur, old from the lists, whose entries are met in list order) are fetched one row
// per lane, the listed rows are read eight at a time.
// plans[1].fused counts the classes served.
// grid = (ceil(max ld / 1024), ceil(min(K, 8) / per_wg), ncls), dynamic LDS = lds_bytes >= ld of every class served.
extern "C" __global__ void __launch_bounds__(256)
rcd_k_inc_update_fused(const RcdClass *__restrict__ classes, RcdPlan *__restrict__ plans, int lds_bytes, int pct,
                       int per_wg)
{
    extern __shared__ unsigned int inc_member[];
    const RcdClass &st = classes[blockIdx.z];
    if (st.done || !inc_fused(st, lds_bytes, pct)) return;
    const int ld = st.ld;
    // this workgroup's share of the waiting blocks: need[s_base .. s_base + nmine)
    const int s_base = blockIdx.y * per_wg;
    const int nmine = min(per_wg, st.nneed - s_base);
    if ((int)blockIdx.x * 1024 >= ld || nmine <= 0) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // the host stops launching this kernel once a batch of rounds has gone by without a class for it
    if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0)
        __hip_atomic_fetch_add(&plans[1].fused, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool shared = st.mw > 1;
    const int nseg = shared ? st.mw : 1;
    const int seg_len = shared ? st.mwseg : ld;      // a list's segment sg holds the changed j of [sg seg_len, (sg+1) seg_len)
    for (int i = tid; i < ld / 4; i += 256) inc_member[i] = 0u;
    __syncthreads();
    for (int s = 0; s < nmine; ++s) {
        const int k = st.need[s_base + s];
        for (int sg = 0; sg < nseg; ++sg) {
            const int nd = shared ? st.mwbuf[MW_PEND + k * RCD_MW_MAX + sg] : st.dcount[k];
            const cci32 dl = (cci32)(inc_dlist(st) + (size_t)k * ld + (shared ? (size_t)sg * seg_len : 0));
            for (int e = tid; e < nd; e += 256) {
                const int j = dl[e];
                atomicOr(&inc_member[j >> 2], (1u << s) << ((j & 3) * 8));
            }
        }
    }
    __syncthreads();
    const int v0 = blockIdx.x * 1024 + wave * 256;
    if (v0 >= ld) return;

    const unsigned char *member = reinterpret_cast<const unsigned char *>(inc_member);
    const unsigned long long below = (1ull << lane) - 1ull;
    const gcf32 M = (gcf32)st.M + v0 + lane * 4;
    // per block: coverage vector, the list's old values, position in the list (slots past nmine repeat the last
    // block; their bit is never set)
    ccf32 curp[INC_FUSE_MAX], oldp[INC_FUSE_MAX];
    int pos[INC_FUSE_MAX];
#pragma unroll
    for (int s = 0; s < INC_FUSE_MAX; ++s) {
        const int k = st.need[s_base + min(s, nmine - 1)];
        curp[s] = (ccf32)(st.cur + (size_t)k * ld);
        oldp[s] = (ccf32)(inc_dold(st) + (size_t)k * ld);
        pos[s] = 0;
    }
    double acc[INC_FUSE_MAX][4];
#pragma unroll
    for (int s = 0; s < INC_FUSE_MAX; ++s)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[s][c] = 0.0;

    int next_seg = 0;
    for (int j0 = 0; j0 < ld; j0 += 64) {
        if (j0 == next_seg) {        // a new segment of every list starts at the offset of its slice
#pragma unroll
            for (int s = 0; s < INC_FUSE_MAX; ++s) pos[s] = shared ? j0 : 0;
            next_seg += seg_len;
        }
        const unsigned mb = member[j0 + lane];
        unsigned long long rows = __ballot(mb != 0u);
        if (rows == 0ull) continue;
        float cnv[INC_FUSE_MAX], cov[INC_FUSE_MAX];
#pragma unroll
        for (int s = 0; s < INC_FUSE_MAX; ++s) {
            const bool in = (mb >> s) & 1u;
            const unsigned long long bs = __ballot(in);
            const int e = pos[s] + __popcll(bs & below);
            cnv[s] = 0.0f;
            cov[s] = 0.0f;
            if (in) {
                cnv[s] = curp[s][j0 + lane];
                cov[s] = oldp[s][e];
            }
            pos[s] += __popcll(bs);
        }
        const gcf32 Mj0 = M + (size_t)j0 * ld;
        while (__popcll(rows) >= 8) inc_fused_rows<8>(rows, mb, cnv, cov, Mj0, ld, acc);
        if (__popcll(rows) >= 4) inc_fused_rows<4>(rows, mb, cnv, cov, Mj0, ld, acc);
        if (__popcll(rows) >= 2) inc_fused_rows<2>(rows, mb, cnv, cov, Mj0, ld, acc);
        if (rows != 0ull) inc_fused_rows<1>(rows, mb, cnv, cov, Mj0, ld, acc);
    }
#pragma unroll
    for (int s = 0; s < INC_FUSE_MAX; ++s) {
        if (s < nmine) {
            double *g = inc_gains(st) + (size_t)st.need[s_base + s] * ld + v0 + lane * 4;
#pragma unroll
            for (int c = 0; c < 4; ++c) g[c] += acc[s][c];
        }
    }
}

namespace {

struct IncShared {
    RcdClass d;
    unsigned long long wkey[RCD_STEP_THREADS / 64];
    int wv[RCD_STEP_THREADS / 64];
    int wcount[RCD_STEP_THREADS / 64];
    int sj[INC_SMALL];
    float sold[INC_SMALL], snew[INC_SMALL];
    // what a wave found in its j range during the single pass of a short coverage update
    int stj[RCD_STEP_THREADS / 64][INC_STAGE];
    float stold[RCD_STEP_THREADS / 64][INC_STAGE], stnew[RCD_STEP_THREADS / 64][INC_STAGE];
};

// Order-preserving 64-bit key of a double (no NaNs here; -0 is made +0 first so that equal values
// get equal keys), and back.
__device__ __forceinline__ unsigned long long inc_key(double x)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(x + 0.0);
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}
__device__ __forceinline__ double inc_value(unsigned long long k)
{
    return __longlong_as_double((long long)((k >> 63) ? (k & 0x7fffffffffffffffull) : ~k));
}

// better of two (key, sample) pairs: larger key, then the smaller sample index
__device__ __forceinline__ void inc_better(unsigned long long &k, int &v, unsigned long long ok, int ov)
{
    if (ok > k || (ok == k && ov < v)) { k = ok; v = ov; }
}

// The same over the wave, result in every lane: three maximum reductions on 32-bit halves (value high
// word, low word among those, complemented sample index among those), no trips through LDS.
__device__ __forceinline__ void inc_wave_best(unsigned long long &key, int &v)
{
    const unsigned hi = (unsigned)(key >> 32), lo = (unsigned)key;
    const unsigned mhi = wave_max_u32(hi);
    const unsigned mlo = wave_max_u32(hi == mhi ? lo : 0u);
    const unsigned mv = wave_max_u32(hi == mhi && lo == mlo ? ~(unsigned)v : 0u);
    key = ((unsigned long long)mhi << 32) | mlo;
    v = (int)~mv;
}

// One thread's share of the argmax scan over g[0..n): samples tid, tid + NT, ... in ascending order, the
// first maximum kept.  Eight loads are in flight at a time: taken one by one, every load is a full trip
// to L2 and the trips add up (five of them at n = 5000, forty-nine at n = 50 000).
template <int NT>
__device__ __forceinline__ void inc_scan(const double *__restrict__ g, int n, int tid, double &best, int &bv)
{
    constexpr int U = 8;
    int v = tid;
    for (; v + (U - 1) * NT < n; v += U * NT) {
        double x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = g[v + u * NT];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (x[u] > best) { best = x[u]; bv = v + u * NT; }
    }
    double x[U - 1];
#pragma unroll
    for (int u = 0; u < U - 1; ++u) x[u] = v + u * NT < n ? g[v + u * NT] : INC_TAKEN;
#pragma unroll
    for (int u = 0; u < U - 1; ++u)
        if (x[u] > best) { best = x[u]; bv = v + u * NT; }
}

} // namespace

// Greedy steps of one class, one workgroup of 1024 threads, for as long as the block that is next
// in turn has current gains.  A step: argmin block (LDS), argmax over that block's gains (one scan),
// bookkeeping, coverage update from row v* of M with the ordered list of changed j, and then either
// the gain update applied right here (short list) or the list left pending for rcd_k_inc_update
// (long list, more than small_bytes of rows; the block sits out until then, the others go on).  At most
// max_steps steps per call.
// plans[0].ndone counts finished classes.
extern "C" __global__ void __launch_bounds__(RCD_STEP_THREADS)
rcd_k_inc_steps(RcdClass *__restrict__ classes, RcdPlan *__restrict__ plans, int max_steps, int small_bytes)
{
    constexpr int NT = RCD_STEP_THREADS, NW = NT / 64;
    __shared__ IncShared sh;
    RcdClass &st = classes[blockIdx.x];
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
        if (tid == 0) st.nneed = 0;
        return;
    }
    const long long tick0 = wall_clock64();
    const int K = d.K, n = d.n, ld = d.ld, total = d.total;
    // the update launch that ran since the last call brought these blocks' gains up to date
    if (tid < d.nneed) d.valid[d.need[tid]] = 1;
    __syncthreads();
    double *G = inc_gains(d);
    int32_t *dlist = inc_dlist(d);
    float *dold = inc_dold(d);
    const gcf32 M = (gcf32)d.M;
    const int seg = ((ld + NW - 1) / NW + 255) / 256 * 256;     // j range of a wave in the coverage update
    // lists up to this many rows are applied right here: one workgroup reads a few MB in the time a
    // trip through the update launch takes, so the limit is a number of bytes
    const int small = max(4, min(INC_SMALL, small_bytes / (ld * 4)));

    int nR = d.nR, t = d.t, done = 0;
    const int t0 = t;
    long long useful = 0, entries = 0, computed = 0, sweeps = 0;
    for (;;) {
        if (t >= total) { done = 1; break; }
        if (t - t0 >= max_steps) break;      // a class that waits for the update launch waits for every class's call
        const int js = least_open_block(d, K);
        if (js < 0) { done = 1; break; }
        if (!d.valid[js]) break;

        // ---- argmax over the block's gains
        const double *g = G + (size_t)js * ld;
        double best = INC_LIVE_ABOVE;
        int bv = 0x7fffffff;
        inc_scan<NT>(g, n, tid, best, bv);
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
        best = inc_value(key);
        const int vstar = bv;
        if (vstar >= n) { done = 1; break; }          // no candidate left (cannot happen while t < total <= n)

        // ---- bookkeeping and outputs
        // (where v* goes in the caller's arrays is asked for now and used at the end of the step: the answer is a
        // trip to memory that the first wave would otherwise sit out before its share of the coverage update)
        int oi = vstar;
        if (tid == 0) {
            d.cnt[js] += 1;
            d.f[js] += best;
            if (d.out_index) oi = d.out_index[vstar];
        }
        if (tid < K) G[(size_t)tid * ld + vstar] = INC_TAKEN;

        // ---- coverage update cur_js(j) = max(cur_js(j), S(j, v*)) and the ordered list of changed j
        const gcf32 row = M + (size_t)vstar * ld;
        float *cur = d.cur + (size_t)js * ld;
        const int j_begin = wave * seg, j_end = min(ld, j_begin + seg);
        // One pass over the wave's range finds the changed j (ascending: pieces in order, lanes in order,
        // the four entries of a lane in order) and holds back the first INC_STAGE of them in LDS; most steps
        // change a handful of entries in all, and then this pass is the only one.
        int cnt = 0;               // the same in every lane of the wave
        const unsigned long long below = (1ull << lane) - 1ull;
        for (int s = j_begin + lane * 4; s < j_end; s += 256) {
            const f32x4 m = *(gcf32x4)(row + s);
            const f32x4 c = *(const f32x4 *)(cur + s);
            const bool ch[4] = {m.x > c.x, m.y > c.y, m.z > c.z, m.w > c.w};
            const unsigned long long b0 = __ballot(ch[0]), b1 = __ballot(ch[1]), b2 = __ballot(ch[2]), b3 = __ballot(ch[3]);
            if ((b0 | b1 | b2 | b3) == 0ull) continue;
            int pos = cnt + __popcll(b0 & below) + __popcll(b1 & below) + __popcll(b2 & below) + __popcll(b3 & below);
            const float mv[4] = {m.x, m.y, m.z, m.w}, cv[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (ch[q]) {
                    if (pos < INC_STAGE) { sh.stj[wave][pos] = s + q; sh.stold[wave][pos] = cv[q]; sh.stnew[wave][pos] = mv[q]; }
                    ++pos;
                }
            cnt += __popcll(b0) + __popcll(b1) + __popcll(b2) + __popcll(b3);
        }
        if (lane == 0) sh.wcount[wave] = cnt;      // last read before the barrier that ended the previous step
        __syncthreads();
        int base = 0, nd = 0;
        bool staged = true;        // every wave's entries fit what it held back
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const int c = sh.wcount[w];
            if (w < wave) base += c;
            nd += c;
            staged = staged && c <= INC_STAGE;
        }
        int32_t *dl = dlist + (size_t)js * ld;
        float *dol = dold + (size_t)js * ld;
        if (nd <= small && staged) {
            // short list, all of it in LDS already: put the waves' parts end to end and raise the coverage
            if (lane < cnt) {
                const int j = sh.stj[wave][lane];
                const float nw = sh.stnew[wave][lane];
                sh.sj[base + lane] = j;
                sh.sold[base + lane] = sh.stold[wave][lane];
                sh.snew[base + lane] = nw;
                cur[j] = nw;
            }
        } else
        for (int s = j_begin + lane * 4; s < j_end; s += 256) {
            const f32x4 m = *(gcf32x4)(row + s);
            const f32x4 c = *(const f32x4 *)(cur + s);
            const bool ch[4] = {m.x > c.x, m.y > c.y, m.z > c.z, m.w > c.w};
            const int mine = ch[0] + ch[1] + ch[2] + ch[3];
            int incl = mine;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            int pos = base + incl - mine;
            const float mv[4] = {m.x, m.y, m.z, m.w}, cv[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (ch[q]) {
                    dl[pos] = s + q;
                    dol[pos] = cv[q];
                    if (nd <= small) { sh.sj[pos] = s + q; sh.sold[pos] = cv[q]; sh.snew[pos] = mv[q]; }
                    ++pos;
                }
            if (mine) {
                f32x4 r;
                r.x = fmaxf(c.x, m.x); r.y = fmaxf(c.y, m.y); r.z = fmaxf(c.z, m.z); r.w = fmaxf(c.w, m.w);
                *(f32x4 *)(cur + s) = r;
            }
            base += __shfl(incl, 63);
        }
        entries += (long long)nd * n;
        computed += nR - 1;
        if (nd > small) {
            // long list: left to the update launch, the block sits out until then
            if (tid == 0) { d.valid[js] = 0; d.dcount[js] = nd; }
            sweeps += 1;
        } else if (nd > 0) {
            __syncthreads();       // the short list is complete in LDS
            double *gj = G + (size_t)js * ld;
            // A thread's candidates in a stretch of NT * 5 samples: four in a row at 4 tid, and sample NT * 4 + tid,
            // so that a class of up to 5120 samples is one stretch and a list of up to eight rows one trip to
            // memory (in stretches of NT * 4 the last 1024 samples of such a class cost every step a second trip).
            for (int sb = 0; sb < ld; sb += NT * 5) {
                const int vv = sb + tid * 4;               // ld is a multiple of 4: a piece is whole or absent
                const int vx = sb + NT * 4 + tid;
                const bool piece = vv < ld, single = vx < ld;
                if (!piece && !single) continue;
                // (what a thread has no use for is loaded from the stretch's first sample)
                const int pv = piece ? vv : sb, px = single ? vx : sb;
                double acc[4] = {0.0, 0.0, 0.0, 0.0}, accx = 0.0;
                // U rows of the list from e0 on, all requested before the first is used; past the list's end its last
                // row again (every register is defined on every path).  The list is taken eight rows at a time and
                // its tail in the smallest of 1, 2, 4, 8 that holds it: most lists are a row or two, and every load,
                // wanted or not, costs the compute unit's memory pipeline its turn.
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
        if (tid == 0) {
            d.assign_out[oi] = js;
            if (d.order_out) d.order_out[oi] = t;
        }
        useful += nR;
        nR -= 1;
        ++t;
        __syncthreads();           // the step's writes (gains, lists, LDS state) are in place
    }

    // ---- the descriptor: which blocks wait for the update launch, the state, the counters
    __syncthreads();
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

// ======================================================================================
// Graph cut, the second submodular function of Section 4:
//     f(A) = sum_{v in V_l \ A} sum_{v' in A} sim(v, v').
// With a symmetric S, f(A u {u}) - f(A) = colsum(u) - S(u,u) - 2 sum_{a in A} S(u,a): a block's
// marginal values start as the column sums without the diagonal and taking v* lowers every one of
// them by 2 S(v, v*), which is row v* of M.  So the gains are always current, a step is one scan
// and one row, and the whole class runs in the step loop below.  Same Algorithm 1, same tie
// rules; f is not monotone, marginal values go negative and the largest one is still taken (the
// quotas have to be met).  Gains are carried in double (sums of fp32 numbers taken in double are
// exact), so exact ties stay exact.  Uses the gain array of the incremental route.
// ======================================================================================

// G[k][v] = sum_j S(j,v) - S(v,v) for every block.  grid = (ceil(max n / 4), ncls).
extern "C" __global__ void __launch_bounds__(256)
rcd_k_gc_init(const RcdClass *__restrict__ classes)
{
    const RcdClass &st = classes[blockIdx.y];
    const int lane = threadIdx.x & 63;
    const int v = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= st.n) return;
    const int ld = st.ld, K = st.K;
    const gcf32 row = (gcf32)st.M + (size_t)v * ld + lane * 4;
    double a = 0.0;
    for (int s = 0; s < ld; s += 256) {
        const f32x4 m = *(gcf32x4)(row + s);
        a += ((double)m.x + (double)m.y) + ((double)m.z + (double)m.w);
    }
    // whole row first, diagonal off afterwards: two samples with identical rows get identical values
    a = wave_sum_f64(a) - (double)((gcf32)st.M)[(size_t)v * ld + v];
    if (lane < K) inc_gains(st)[(size_t)lane * ld + v] = a;
}

// Greedy steps of one class with the graph-cut function, one workgroup of 1024 threads, up to
// max_steps steps per call.  plans[0].ndone counts finished classes.
extern "C" __global__ void __launch_bounds__(RCD_STEP_THREADS)
rcd_k_gc_steps(RcdClass *__restrict__ classes, RcdPlan *__restrict__ plans, int max_steps)
{
    constexpr int NT = RCD_STEP_THREADS, NW = NT / 64;
    __shared__ IncShared sh;
    RcdClass &st = classes[blockIdx.x];
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
    const int K = d.K, n = d.n, ld = d.ld, total = d.total;
    double *G = inc_gains(d);
    const gcf32 M = (gcf32)d.M;
    int nR = d.nR, t = d.t, done = 0;
    const int t0 = t;
    long long useful = 0;
    for (;;) {
        if (t >= total) { done = 1; break; }
        if (t - t0 >= max_steps) break;
        const int js = least_open_block(d, K);
        if (js < 0) { done = 1; break; }
        // ---- argmax over the block's marginal values (they may be negative)
        double *g = G + (size_t)js * ld;
        double best = INC_LIVE_ABOVE;
        int bv = 0x7fffffff;
        inc_scan<NT>(g, n, tid, best, bv);
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
        best = inc_value(key);
        const int vstar = bv;
        if (vstar >= n) { done = 1; break; }
        // (every thread chose js from the block state before the barrier above: it may change now)
        int oi = vstar;              // asked for now, used at the end of the step (see rcd_k_inc_steps)
        if (tid == 0) {
            d.cnt[js] += 1;
            d.f[js] += best;
            if (d.out_index) oi = d.out_index[vstar];
        }
        // ---- every marginal value of the block drops by 2 S(v, v*); v* leaves every block's candidates
        const gcf32 row = M + (size_t)vstar * ld;
        constexpr int UB = 4;      // batches of four pieces per thread: their loads are in flight together
        for (int v0 = tid * 4; v0 < ld; v0 += UB * NT * 4) {
            f32x4 m[UB];
            double o[UB][4];
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int vu = v0 + u * NT * 4;
                if (vu < ld) {
                    m[u] = *(gcf32x4)(row + vu);
#pragma unroll
                    for (int c = 0; c < 4; ++c) o[u][c] = g[vu + c];
                }
            }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int vu = v0 + u * NT * 4;
                if (vu < ld) {
                    g[vu] = o[u][0] - 2.0 * (double)m[u].x;
                    g[vu + 1] = o[u][1] - 2.0 * (double)m[u].y;
                    g[vu + 2] = o[u][2] - 2.0 * (double)m[u].z;
                    g[vu + 3] = o[u][3] - 2.0 * (double)m[u].w;
                }
            }
        }
        // v* leaves every block's candidates; in the served block the thread that has just updated that
        // entry strikes it out (its own earlier store to the same address: no barrier in between is needed)
        if ((vstar >> 2) % NT == tid) g[vstar] = INC_TAKEN;
        if (tid < K && tid != js) G[(size_t)tid * ld + vstar] = INC_TAKEN;
        if (tid == 0) {
            d.assign_out[oi] = js;
            if (d.order_out) d.order_out[oi] = t;
        }
        useful += nR;
        nR -= 1;
        ++t;
        __syncthreads();
    }
    __syncthreads();
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

// obj[c][k] = f(A_k): the running sum of the accepted marginal values (exact to rounding in double).
// grid = (1, ncls), K threads.
extern "C" __global__ void rcd_k_gc_objective(const RcdClass *__restrict__ classes, double *__restrict__ obj, int Kstride)
{
    const RcdClass &st = classes[blockIdx.y];
    const int k = threadIdx.x;
    if (k < st.K) obj[(size_t)blockIdx.y * Kstride + k] = st.f[k];
}
