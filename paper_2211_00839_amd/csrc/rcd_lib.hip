// Host side of librcd: argument checks, workspace layout, class grouping and the
// round loop that drives the kernels.  One translation unit: the kernel files
// are included so that their launch stubs are local to this library.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>
#include <thread>

#include "../../include/rcd.h"
#include "rcd_state.h"
#include "greedy_kernels.hip"
#include "similarity_kernels.hip"
#include "split_kernels.hip"
#include "recompute_kernels.hip"
#include "incremental_kernels.hip"
#include "multi_wg_kernels.hip"

static_assert(RCD_KMAX == RCD_MAX_K, "public and internal block limits differ");

// every sweep variant's staged coverage (slots x chunk of j) stays inside the workgroup's LDS
constexpr bool sweep_chunks_fit()
{
    for (int k = 1; k <= RCD_KMAX; ++k)
        if (rcd_sweep_slots(k) < k || rcd_sweep_chunk(k) < RCD_TILE ||
            rcd_sweep_slots(k) * rcd_sweep_chunk(k) > RCD_SWEEP_LDS_FLOATS)
            return false;
    return true;
}
static_assert(sweep_chunks_fit(), "a stored-S sweep variant would stage past its LDS");

namespace {

thread_local char g_hip_err[320] = "";
thread_local int64_t g_stats[8] = {0, 0, 0, 0, 0, 0, 0, 0};
thread_local RcdPlan *g_pinned = nullptr;   // per lane 2 progress slots of 2 plan headers, pinned, never freed
// optional per-kernel timing (HIP events between the launches of a round)
thread_local int g_profile_on = 0;
thread_local double g_prof[8] = {0, 0, 0, 0, 0, 0, 0, 0};   // ms: steps, sweep, apply; rounds; similarity ms
thread_local std::vector<hipEvent_t> g_prof_ev[4];
thread_local hipStream_t g_side[4] = {nullptr, nullptr, nullptr, nullptr};   // created on first use, never destroyed

#define HIP_TRY(expr)                                                                      \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess) {                                                            \
            snprintf(g_hip_err, sizeof g_hip_err, "%s -> %s", #expr, hipGetErrorString(e_)); \
            return RCD_ERR_HIP;                                                            \
        }                                                                                  \
    } while (0)

#define RCD_TRY(expr)              \
    do {                           \
        int rc_ = (expr);          \
        if (rc_ != RCD_OK) return rc_; \
    } while (0)

inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
inline int pitch_of(int64_t n) { return (int)((std::max<int64_t>(n, 1) + RCD_TILE - 1) / RCD_TILE * RCD_TILE); }

int env_int(const char *name, int dflt, int lo, int hi)
{
    const char *s = getenv(name);
    if (!s || !*s) return dflt;
    long v = strtol(s, nullptr, 10);
    if (v < lo) v = lo;
    if (v > hi) v = hi;
    return (int)v;
}

struct Carver {
    char *base;
    size_t off, cap;
    bool fail;
    Carver(void *p, size_t bytes) : base((char *)p), off(0), cap(bytes), fail(false) {}
    template <typename T> T *take(size_t count)
    {
        const size_t b = up256(count * sizeof(T));
        if (off + b > cap) { fail = true; return nullptr; }
        T *p = reinterpret_cast<T *>(base + off);
        off += b;
        return p;
    }
};

size_t class_state_bytes(int64_t n, int K, bool stored)
{
    const size_t ld = (size_t)pitch_of(n);
    size_t b = 0;
    if (stored) b += up256((size_t)n * ld * 4);
    else b += up256((size_t)n * 4);              // squared row norms
    b += up256((size_t)K * ld * 4);              // cur
    b += up256((size_t)RCD_CMAX * K * ld * 4);   // part
    b += up256((size_t)K * ld * 4);              // gain
    b += up256(ld / RCD_TILE_RC * 4);            // tilecnt
    b += up256(ld * 4);                          // perm
    b += up256(RCD_MW_INTS * 4);                 // exchange area of the multi-workgroup step loops
    return b;
}

// Most classes a data-set call takes.
constexpr int RCD_MAX_CLASSES = 8192;

// Classes of a group may be dealt to this many lanes that advance side by side.
constexpr int RCD_MAX_LANES = 4;
// Progress records (and their events) a lane cycles through: batches in flight + 1 at most.
constexpr int RCD_SLOTS = 4;

size_t plan_area_bytes(int ncls) { return up256(2 * sizeof(RcdPlan) + 2 * (size_t)(ncls + 1) * 4); }

// Room for a lane's workgroup-to-class table of the stored-S sweep.
constexpr int RCD_MAX_SWEEP_WGS = 2048;
size_t wg_area_bytes(int ncls) { return up256((size_t)(RCD_MAX_SWEEP_WGS + ncls) * sizeof(RcdWg)); }

size_t group_fixed_bytes(int ncls, int K)
{
    return up256((size_t)ncls * sizeof(RcdClass)) + RCD_MAX_LANES * (plan_area_bytes(ncls) + wg_area_bytes(ncls)) +
           up256((size_t)ncls * K * sizeof(double));
}

struct Group {
    RcdClass *classes_dev = nullptr;
    RcdPlan *plan_dev = nullptr;                 // = plan_area[0]
    RcdPlan *plan_area[RCD_MAX_LANES] = {};      // one plan record per lane (only the owner of the workspace slice has them all)
    RcdWg *wgmap_dev = nullptr;                  // = wg_area[0]
    RcdWg *wg_area[RCD_MAX_LANES] = {};
    double *obj_dev = nullptr;
    std::vector<RcdClass> host;   // kept alive until the stream has consumed it
    int K = 0;
};

// Carve the state of one class out of the workspace and fill its descriptor.
bool carve_class(Carver &cv, RcdClass &c, int64_t n, int K, const int64_t *cap, bool stored)
{
    memset(&c, 0, sizeof c);
    const size_t ld = (size_t)pitch_of(n);
    c.n = (int)n;
    c.ld = (int)ld;
    c.K = K;
    if (stored) c.M = cv.take<float>((size_t)n * ld);
    else c.sq = cv.take<float>((size_t)n);
    c.tw = stored ? RCD_TILE : RCD_TILE_RC;
    c.row_align = RCD_ROWS_RC;
    c.cur = cv.take<float>((size_t)K * ld);
    c.part = cv.take<float>((size_t)RCD_CMAX * K * ld);
    c.gain = cv.take<float>((size_t)K * ld);
    c.tilecnt = cv.take<int32_t>(ld / RCD_TILE_RC);
    c.perm = cv.take<int32_t>(ld);
    c.mwbuf = cv.take<int32_t>(RCD_MW_INTS);
    int64_t total = 0;
    for (int k = 0; k < K; ++k) {
        c.cap[k] = (int)cap[k];
        total += cap[k];
    }
    c.total = (int)total;
    c.nR = (int)n;
    c.mode = stored ? RCD_MODE_STORED : RCD_MODE_RECOMPUTE;
    return !cv.fail;
}

int sweep_items_bound(const RcdClass &c)
{
    const int tiles0 = (c.n + c.tw - 1) / c.tw;
    return std::min(RCD_CMAX * tiles0, c.target_items + tiles0);
}

// Stored-S sweep evaluating nneed blocks: length of a chunk of j and number of chunks
// (the step loop applies the same rule on the device).
void stored_chunks(int ld, int nneed, int *C, int *jc)
{
    int len = std::min(rcd_sweep_chunk(nneed), ld);
    *jc = len;
    *C = (ld + len - 1) / len;
}

// Can a class of n samples and K blocks run in stored mode (chunk partials fit their buffer)?
bool stored_supported(int64_t n, int K)
{
    int C, jc;
    stored_chunks(pitch_of(n), K, &C, &jc);
    return C <= RCD_CMAX;
}

// Deal `total` sweep workgroups to the classes in proportion to their matrix sizes,
// at least one each.  Returns the table (class-major).
std::vector<RcdWg> deal_workgroups(const std::vector<RcdClass> &cls, int total)
{
    double sum = 0.0;
    for (const RcdClass &c : cls) sum += (double)c.n * c.n;
    std::vector<RcdWg> map;
    const int ncls = (int)cls.size();
    for (int i = 0; i < ncls; ++i) {
        const double share = sum > 0.0 ? (double)cls[i].n * cls[i].n / sum : 1.0 / ncls;
        int W = (int)std::lround(share * total);
        // no more workgroups than rows for their waves to take
        W = std::min(W, (cls[i].n + RCD_SWEEP_WAVES - 1) / RCD_SWEEP_WAVES);
        W = std::max(W, 1);
        for (int w = 0; w < W && (int)map.size() < RCD_MAX_SWEEP_WGS + i; ++w) map.push_back(RcdWg{i, w, W, 0});
    }
    // a class cut short by the table's capacity: its workgroups must know the real count
    std::vector<int> have(ncls, 0);
    for (const RcdWg &m : map) have[m.cls] += 1;
    for (RcdWg &m : map) m.W = have[m.cls];
    return map;
}

// What is set up once per device (kernel attributes are per device, and so is the address of a
// __device__ array): guarded by one mutex, since partition calls may come from several threads.
constexpr int RCD_MAX_DEVICES = 64;
struct DeviceSetup {
    int cus = 0;               // compute units; 0 = sweep kernel not set up yet
    bool fast_ready = false;   // the matrix-core kernels' LDS limit has been raised
    float *static_norms = nullptr;   // device address of g_static_norms on this device
};
std::mutex g_setup_mutex;
DeviceSetup g_dev[RCD_MAX_DEVICES];

// The current device's record, or null (and g_hip_err) if the device cannot be told.
DeviceSetup *device_setup()
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= RCD_MAX_DEVICES) {
        snprintf(g_hip_err, sizeof g_hip_err, "hipGetDevice -> %s", e != hipSuccess ? hipGetErrorString(e) : "device index beyond 63");
        return nullptr;
    }
    return &g_dev[dev];
}

int sweep_setup()
{
    DeviceSetup *ds = device_setup();
    if (!ds) return RCD_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    if (ds->cus == 0) {
        int dev = 0, cus = 0;
        HIP_TRY(hipGetDevice(&dev));
        HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(rcd_k_sweep_rows),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, RCD_SWEEP_LDS_FLOATS * 4));
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(rcd_k_inc_update_fused),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, RCD_INC_FUSE_LDS_MAX));
        ds->cus = std::max(cus, 1);
    }
    return RCD_OK;
}

// Compute units of the current device (after sweep_setup() succeeded; 256 if it has not run).
int cu_count()
{
    DeviceSetup *ds = device_setup();
    if (!ds) return 256;
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    return ds->cus > 0 ? ds->cus : 256;
}

// Scratch of rcd_similarity_static (the squared row norms its kernels pass from one launch to the
// next): a file-scope device array, so that the entry point needs no workspace and allocates nothing.
// Every device the library runs on holds its own copy, at its own address, until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress: the kernels are given the address
// that call returns for the current device, never the name.
} // namespace
static __device__ __align__(256) float g_static_norms[RCD_STATIC_MAX_N];
namespace {

// Device address of g_static_norms on the current device (looked up once per device).
int static_setup(float **norms)
{
    DeviceSetup *ds = device_setup();
    if (!ds) return RCD_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    if (!ds->static_norms) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_norms)));
        if (!ptr) {
            snprintf(g_hip_err, sizeof g_hip_err, "hipGetSymbolAddress(g_static_norms) returned no address");
            return RCD_ERR_HIP;
        }
        ds->static_norms = static_cast<float *>(ptr);
    }
    if (norms) *norms = ds->static_norms;
    return RCD_OK;
}

// Fast path of the matrix-core kernels: feature rows that can go straight from global memory
// into LDS a whole 128-byte line at a time.
bool rows_fit_fast_path(const void *X, int dt, int64_t d, int64_t ldx)
{
    const int64_t esz = dt == RCD_F32 ? 4 : 2;
    return (reinterpret_cast<uintptr_t>(X) & 15) == 0 && ((ldx * esz) % 16) == 0 && d * esz >= sim::pipe::LINE &&
           (d * esz) % sim::pipe::LINE == 0;
}

// The fast kernels use more LDS than a kernel may by default: raise their limit once.
int fast_setup()
{
    DeviceSetup *ds = device_setup();
    if (!ds) return RCD_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    if (!ds->fast_ready) {
        const void *sim_kernels[] = {reinterpret_cast<const void *>(&sim::k_gram_rbf_fast<float>),
                                     reinterpret_cast<const void *>(&sim::k_gram_rbf_fast<__bf16>),
                                     reinterpret_cast<const void *>(&sim::k_gram_rbf_fast<float, sim::EPI_RBF_MIRROR>),
                                     reinterpret_cast<const void *>(&sim::k_gram_rbf_fast<__bf16, sim::EPI_RBF_MIRROR>),
                                     reinterpret_cast<const void *>(&sim::k_gram_rbf_fast<float, sim::EPI_DISTANCE>),
                                     reinterpret_cast<const void *>(&sim::k_gram_rbf_fast<__bf16, sim::EPI_DISTANCE>)};
        for (const void *k : sim_kernels)
            HIP_TRY(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, sim::pipe::LDS_BYTES));
        const void *batch_kernels[] = {
            reinterpret_cast<const void *>(&sim::k_gram_rbf_fast_batch<float, sim::EPI_RBF>),
            reinterpret_cast<const void *>(&sim::k_gram_rbf_fast_batch<__bf16, sim::EPI_RBF>),
            reinterpret_cast<const void *>(&sim::k_gram_rbf_fast_batch<float, sim::EPI_RBF_MIRROR>),
            reinterpret_cast<const void *>(&sim::k_gram_rbf_fast_batch<__bf16, sim::EPI_RBF_MIRROR>)};
        for (const void *k : batch_kernels)
            HIP_TRY(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, sim::pipe::LDS_BYTES));
        const void *rc_kernels[] = {reinterpret_cast<const void *>(&rcd_k_round_rc_fast<float, true>),
                                    reinterpret_cast<const void *>(&rcd_k_round_rc_fast<float, false>),
                                    reinterpret_cast<const void *>(&rcd_k_round_rc_fast<__bf16, true>),
                                    reinterpret_cast<const void *>(&rcd_k_round_rc_fast<__bf16, false>)};
        for (const void *k : rc_kernels)
            HIP_TRY(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, RCD_RC_FAST_LDS));
        ds->fast_ready = true;
    }
    return RCD_OK;
}

int ensure_pinned()
{
    if (!g_pinned) {
        void *p = nullptr;
        HIP_TRY(hipHostMalloc(&p, RCD_MAX_LANES * RCD_SLOTS * 2 * sizeof(RcdPlan), hipHostMallocDefault));
        g_pinned = (RcdPlan *)p;
    }
    return RCD_OK;
}

// Streams of the library's own, for groups of classes that advance side by side.
int ensure_side_streams(int count)
{
    for (int i = 0; i < count && i < RCD_MAX_LANES; ++i)
        if (!g_side[i]) HIP_TRY(hipStreamCreateWithFlags(&g_side[i], hipStreamNonBlocking));
    return RCD_OK;
}

// Do the step loops of the incremental and graph-cut routes share a class among several workgroups?  From
// RCD_MW_MIN_N samples in the largest class on (0 switches it off): below that one workgroup's step is short
// enough that the barriers between the phases would cost more than they save.
bool multi_wg_wanted(int64_t max_n)
{
    const int min_n = env_int("RCD_MW_MIN_N", 16384, 0, 0x7fffffff);
    return min_n > 0 && max_n >= min_n;
}

// One group of classes on one stream.  The host keeps a few batches of rounds
// queued ahead of the device: start(), then enqueue_batch() while fewer than
// `depth` batches are unread and poll() to read the oldest one's progress record,
// until finished; then finish().  Several lanes can be driven in an interleaved
// way; each keeps to its own stream, descriptors, plans and progress slots.
struct Lane {
    Group *g = nullptr;
    hipStream_t stream = nullptr;
    int slot = 0;            // which pinned progress slots are this lane's
    int ncls = 0, rounds = 16, items_ub = 0, round_no = 0;
    bool recompute = false, fused = false, prof = false, finished = false;
    bool incremental = false;   // stored S with incrementally maintained gains
    bool graph_cut = false;     // graph-cut function: stored S, the step loop keeps its own gains current
    int gc_max_steps = 4096;    // steps per class and launch (bounds a launch's duration)
    // several workgroups per class for the step loops of large classes (incremental gains, graph cut)
    bool mw = false;
    int mw_wgs = 0;
    unsigned mw_epoch = 0;      // exchanges the earlier launches of this call may have used
    long long mw_spin_ticks = 200000000;   // bound of a grid-barrier wait, 100 MHz ticks (2 s)
    dim3 update_grid;
    int inc_small_bytes = 512 << 10;   // update lists up to this many bytes of rows are applied by the step loop itself
    int inc_fuse_lds = 0;              // LDS bytes of the fused update pass (its membership table); 0: no fused pass
    int inc_fuse_pct = 50;             // a class's lists are fused when together they hold this share of its samples
    int inc_fuse_seen = -1;            // plans[1].fused as of the last batch read back
    int inc_fuse_per_wg = 8;           // waiting blocks a workgroup of the fused pass serves
    int inc_max_steps = 64;     // steps per class and launch: a class that waits for the update launch waits for the whole lane
    void (*round_rc)(RcdClass *, RcdPlan *, int) = nullptr;
    size_t round_rc_lds = 0;   // dynamic LDS of the recompute sweep (fast path only)
    void (*apply_rc)(RcdClass *, int) = nullptr;
    int sweep_wgs = 0;       // stored S: workgroups of the sweep launch
    dim3 apply_rc_grid;
    hipEvent_t ev[RCD_SLOTS] = {};
    int64_t launches = 0, max_batches = 0;
    int64_t batch = 0;       // batches enqueued
    int64_t polled = 0;      // batches whose progress record has been read
    int64_t prof_done = 0;   // batches whose timing events have been read

    RcdPlan *pinned(int64_t b) const { return g_pinned + 2 * (RCD_SLOTS * slot + (int)(b % RCD_SLOTS)); }

    // The step loops of the incremental and graph-cut routes: one workgroup per class, or, for large classes,
    // several (a launch numbers its exchanges from where the launch before it may have stopped: one exchange at
    // the start, then two per step on the incremental route, one with the graph-cut function).
    void launch_inc_steps()
    {
        const unsigned epoch0 = mw_epoch;
        mw_epoch += 2u * (unsigned)inc_max_steps + 8u;
        (void)epoch0;
        if (mw)
            hipLaunchKernelGGL(rcd_k_inc_steps_mw, dim3(mw_wgs), dim3(RCD_STEP_THREADS), 0, stream, g->classes_dev,
                               g->plan_dev, (const RcdWg *)g->wgmap_dev, inc_max_steps, inc_small_bytes, epoch0,
                               mw_spin_ticks);
        else
            hipLaunchKernelGGL(rcd_k_inc_steps, dim3(ncls), dim3(RCD_STEP_THREADS), 0, stream, g->classes_dev,
                               g->plan_dev, inc_max_steps, inc_small_bytes);
    }
    void launch_gc_steps()
    {
        const unsigned epoch0 = mw_epoch;
        mw_epoch += (unsigned)gc_max_steps + 8u;
        (void)epoch0;
        if (mw)
            hipLaunchKernelGGL(rcd_k_gc_steps_mw, dim3(mw_wgs), dim3(RCD_STEP_THREADS), 0, stream, g->classes_dev,
                               g->plan_dev, (const RcdWg *)g->wgmap_dev, gc_max_steps, epoch0, mw_spin_ticks);
        else
            hipLaunchKernelGGL(rcd_k_gc_steps, dim3(ncls), dim3(RCD_STEP_THREADS), 0, stream, g->classes_dev,
                               g->plan_dev, gc_max_steps);
    }

    void launch_apply(int rn)
    {
        // stored S: the step loops apply their own decisions
        if (recompute) hipLaunchKernelGGL(apply_rc, apply_rc_grid, dim3(256), 0, stream, g->classes_dev, rn);
    }

    void read_events(int64_t b)
    {
        std::vector<hipEvent_t> &e = g_prof_ev[b % RCD_SLOTS];
        for (int r = 0; r < rounds; ++r) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, e[3 * r], e[3 * r + 1]) == hipSuccess) g_prof[1] += ms;
            if (hipEventElapsedTime(&ms, e[3 * r + 1], e[3 * r + 2]) == hipSuccess) g_prof[0] += ms;
            if (hipEventElapsedTime(&ms, e[3 * r + 2], e[3 * r + 3]) == hipSuccess) g_prof[2] += ms;
        }
        g_prof[3] += rounds;
    }

    // Upload the descriptors, reset the state, run the first step loop.
    // target_total: sweep workgroups per round this lane aims at.
    // sweep_target: workgroups the stored-S sweep launch aims at.
    int start(Group &group, hipStream_t s, int slot_, int target_total, int sweep_target, bool profile)
    {
        g = &group;
        stream = s;
        slot = slot_;
        prof = profile;
        ncls = (int)g->host.size();
        const int per_class = std::max(1, target_total / ncls);
        items_ub = 0;
        int max_n = 0;
        int64_t max_total = 0;
        for (RcdClass &c : g->host) {
            c.target_items = per_class;
            items_ub += sweep_items_bound(c);
            max_n = std::max(max_n, c.n);
            max_total = std::max<int64_t>(max_total, c.total);
        }
        rounds = env_int("RCD_ROUNDS_PER_BATCH", 16, 1, 1024);
        // every round takes at least one step in every unfinished class, so this
        // many batches (plus those queued ahead) always suffice; running past it means a defect, not work
        max_batches = (max_total + 2) / rounds + 3 + RCD_SLOTS;
        RcdPlan plan0;
        memset(&plan0, 0, sizeof plan0);
        plan0.ncls = ncls;
        // the validation kernels may already have raised plans[0].bad: keep it
        HIP_TRY(hipMemcpyAsync(&g->plan_dev[0].ncls, &plan0.ncls, sizeof(int32_t) * 5, hipMemcpyHostToDevice, stream));
        HIP_TRY(hipMemcpyAsync(&g->plan_dev[1], &plan0, sizeof plan0, hipMemcpyHostToDevice, stream));
        HIP_TRY(hipMemcpyAsync(g->classes_dev, g->host.data(), sizeof(RcdClass) * ncls, hipMemcpyHostToDevice, stream));
        hipLaunchKernelGGL(rcd_k_init, dim3(64, ncls), dim3(256), 0, stream, g->classes_dev);
        apply_rc_grid = dim3((unsigned)((max_n + 127) / 128), (unsigned)ncls);   // a wave takes 32 rows
        // a group is homogeneous: all stored, or all recomputed from the same X
        const RcdClass &first = g->host[0];
        recompute = first.mode == RCD_MODE_RECOMPUTE;
        graph_cut = first.objective == 1;
        incremental = !recompute && !graph_cut && first.incremental != 0;
        gc_max_steps = env_int("RCD_GC_STEPS", 4096, 1, 1 << 20);
        // classes that share a lane: a class that waits for the update launch waits for every class's call,
        // so a call is kept to about a third of a millisecond (a step takes about 7 ns per sample)
        const int shared_steps = std::min(32, std::max(4, 400000 / std::max(max_n, 1)));
        inc_max_steps = env_int("RCD_INC_STEPS", ncls > 1 ? shared_steps : 4096, 1, 1 << 20);
        inc_small_bytes = env_int("RCD_INC_SMALL_KB", 512, 1, 1 << 20) * 1024;
        mw = false;
        if ((graph_cut || incremental) && multi_wg_wanted(max_n)) {
            // Workgroups per class: what the device can hold at once, shared evenly, at most RCD_MW_MAX and no
            // more than one per RCD_MW_SLICE (2048) samples; classes too small to share keep one workgroup in the same launch.
            int per_cu = 0;
            const void *kfn = graph_cut ? reinterpret_cast<const void *>(rcd_k_gc_steps_mw)
                                        : reinterpret_cast<const void *>(rcd_k_inc_steps_mw);
            HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kfn, RCD_STEP_THREADS, 0));
            const int capacity = std::max(per_cu, 0) * cu_count();
            // (measured on one 50 000-sample class: graph cut 1418 ms with one workgroup, 260 / 236 / 228 / 225 ms with
            // 12 / 16 / 24 / 32; incremental gains 627 / 599 / 586 / 590 ms)
            const int w_max = std::min(env_int("RCD_MW_MAX_WGS", 24, 1, RCD_MW_MAX), capacity / std::max(ncls, 1));
            const int mw_slice = env_int("RCD_MW_SLICE", 2048, 256, 1 << 20) / 256 * 256;    // samples a workgroup owns, at least
            if (w_max >= 2) {
                std::vector<RcdWg> map;
                for (int i = 0; i < ncls; ++i) {
                    RcdClass &c = g->host[i];
                    int W = std::min(w_max, std::max(1, c.ld / mw_slice));
                    int seg = ((c.ld + W - 1) / W + 255) / 256 * 256;
                    W = (c.ld + seg - 1) / seg;               // no empty slice
                    c.mw = W;
                    c.mwseg = seg;
                    for (int w = 0; w < W; ++w) map.push_back(RcdWg{i, w, W, 0});
                }
                if ((int)map.size() <= capacity && (int)map.size() <= RCD_MAX_SWEEP_WGS) {
                    mw = true;
                    mw_wgs = (int)map.size();
                    mw_epoch = 0;
                    mw_spin_ticks = (long long)env_int("RCD_MW_SPIN_MS", 2000, 0, 60000) * 100000LL;
                    // a shared class steps about four times faster: four times the steps per call for the same wait
                    if (ncls > 1)
                        inc_max_steps = env_int("RCD_INC_STEPS", std::min(64, std::max(8, 1600000 / std::max(max_n, 1))), 1, 1 << 20);
                    // with many classes in the launch an update launch gives each class a small share of the memory
                    // bandwidth, and lists four times as long are better applied by the class's own workgroups
                    // (20 classes of 50 000: 1.92 -> 1.86 s; one class alone: 774 -> 875 ms, so not there)
                    if (ncls >= 4) inc_small_bytes = env_int("RCD_INC_SMALL_KB", 2048, 1, 1 << 20) * 1024;
                    HIP_TRY(hipMemcpyAsync(g->wgmap_dev, map.data(), sizeof(RcdWg) * map.size(), hipMemcpyHostToDevice, stream));
                    HIP_TRY(hipMemcpyAsync(g->classes_dev, g->host.data(), sizeof(RcdClass) * ncls, hipMemcpyHostToDevice, stream));
                } else {
                    for (RcdClass &c : g->host) { c.mw = 0; c.mwseg = 0; }
                }
            }
        }
        if (graph_cut) {
            // initial marginal values = column sums of S without the diagonal
            hipLaunchKernelGGL(rcd_k_gc_init, dim3((unsigned)((max_n + 3) / 4), (unsigned)ncls), dim3(256), 0, stream,
                               (const RcdClass *)g->classes_dev);
        } else if (incremental) {
            int max_ld = 0;
            for (const RcdClass &c : g->host) max_ld = std::max(max_ld, c.ld);
            update_grid = dim3((unsigned)((max_ld + 1023) / 1024), (unsigned)first.K, (unsigned)ncls);
            // Large classes: while the pending lists of a class overlap (the first rounds), one fused pass applies them
            // all.  Its table of one byte per sample must fit beside nothing else in LDS.
            const int fuse_min_n = env_int("RCD_INC_FUSE_MIN_N", 16384, 0, 1 << 30);
            inc_fuse_pct = env_int("RCD_INC_FUSE_PCT", 50, 1, 1000);
            inc_fuse_lds = 0;
            inc_fuse_seen = -1;
            if (fuse_min_n > 0 && max_n >= fuse_min_n && max_ld <= RCD_INC_FUSE_LDS_MAX && first.K >= 2) {
                RCD_TRY(sweep_setup());          // raises that kernel's LDS limit
                // A workgroup serves a tile of 1024 samples and up to eight waiting blocks.  With few classes that is too
                // few workgroups for the device (one class of 50 000: 49), so the blocks are dealt to several then, down
                // to two each; one block each is the list-by-list kernel's job.
                const int slots = std::min(first.K, 8);
                const int64_t tiles = (int64_t)update_grid.x * ncls;
                const int groups = (int)std::min<int64_t>(slots, std::max<int64_t>(1, (3 * (int64_t)cu_count() + tiles - 1) / tiles));
                inc_fuse_per_wg = env_int("RCD_INC_FUSE_BLOCKS", (slots + groups - 1) / groups, 1, 8);
                if (inc_fuse_per_wg >= 2) inc_fuse_lds = (max_ld + 1023) / 1024 * 1024;
            }
            // initial gains = column sums of S: every coverage vector is 0
            hipLaunchKernelGGL(rcd_k_inc_init, dim3((unsigned)((max_n + 3) / 4), (unsigned)ncls), dim3(256), 0, stream,
                               (const RcdClass *)g->classes_dev);
        } else if (!recompute) {
            RCD_TRY(sweep_setup());
            const std::vector<RcdWg> map = deal_workgroups(g->host, std::min(sweep_target, RCD_MAX_SWEEP_WGS));
            sweep_wgs = (int)map.size();
            // pageable source: the copy is staged before the call returns
            HIP_TRY(hipMemcpyAsync(g->wgmap_dev, map.data(), sizeof(RcdWg) * map.size(), hipMemcpyHostToDevice, stream));
        }
        // step loop number 1 (the bootstrap) and its apply; step loop r+2 follows round r's sweep
        if (graph_cut)
            launch_gc_steps();
        else if (recompute)
            hipLaunchKernelGGL(rcd_k_steps, dim3(ncls), dim3(RCD_STEP_THREADS), 0, stream, g->classes_dev, g->plan_dev);
        else if (incremental)
            launch_inc_steps();
        else
            hipLaunchKernelGGL(rcd_k_steps_rows, dim3(ncls), dim3(RCD_STEP_THREADS), 0, stream, g->classes_dev,
                               g->plan_dev);

        for (int i = 0; i < RCD_SLOTS; ++i) HIP_TRY(hipEventCreateWithFlags(&ev[i], hipEventDisableTiming));
        // One launch per round (sweep + step loops fused) pays off when few classes are in
        // flight; with many, the sweep is bandwidth-bound and the step loops get their own launch.
        fused = recompute && env_int("RCD_FUSED", ncls <= 2 ? 1 : 0, 0, 1) != 0;
        if (recompute) {
            const bool fast = first.tw == RCD_TILE_FAST;
            const bool f32 = first.dt == RCD_F32;
            if (fast) {
                RCD_TRY(fast_setup());
                round_rc_lds = RCD_RC_FAST_LDS;
                round_rc = f32 ? (fused ? rcd_k_round_rc_fast<float, true> : rcd_k_round_rc_fast<float, false>)
                               : (fused ? rcd_k_round_rc_fast<__bf16, true> : rcd_k_round_rc_fast<__bf16, false>);
            } else {
                round_rc_lds = 0;
                round_rc = f32 ? (fused ? rcd_k_round_rc<float, true> : rcd_k_round_rc<float, false>)
                               : (fused ? rcd_k_round_rc<__bf16, true> : rcd_k_round_rc<__bf16, false>);
            }
            apply_rc = f32 ? rcd_k_apply_rc<float> : rcd_k_apply_rc<__bf16>;
        }
        launches = 3;
        round_no = 0;
        launch_apply(1);
        if (prof) {
            for (int i = 0; i < RCD_SLOTS; ++i)
                while ((int)g_prof_ev[i].size() < 3 * rounds + 1) {
                    hipEvent_t e;
                    HIP_TRY(hipEventCreate(&e));
                    g_prof_ev[i].push_back(e);
                }
        }
        batch = 0;
        polled = 0;
        prof_done = 0;
        finished = false;
        return RCD_OK;
    }

    // One batch of rounds, then a copy of the progress record for the host.
    int enqueue_batch()
    {
        const int64_t b = batch;
        if (b > max_batches) {
            snprintf(g_hip_err, sizeof g_hip_err, "greedy made no progress within %lld batches", (long long)max_batches);
            return RCD_ERR_HIP;
        }
        std::vector<hipEvent_t> *pe = prof ? &g_prof_ev[b % RCD_SLOTS] : nullptr;
        if (pe) (void)hipEventRecord((*pe)[0], stream);
        for (int r = 0; r < rounds; ++r) {
            const int buf = fused ? (round_no & 1) : 0;
            if (graph_cut)
                ;   // nothing between the step loops: the gains are always current
            else if (recompute)
                hipLaunchKernelGGL(round_rc, dim3(items_ub), dim3(256), round_rc_lds, stream, g->classes_dev, g->plan_dev,
                                   buf);
            else if (incremental)
            {
                hipLaunchKernelGGL(rcd_k_inc_update, update_grid, dim3(256), 0, stream, (const RcdClass *)g->classes_dev,
                                   inc_fuse_lds, inc_fuse_pct);
                if (inc_fuse_lds > 0)
                    hipLaunchKernelGGL(rcd_k_inc_update_fused,
                                       dim3(update_grid.x, (unsigned)((std::min(g->K, 8) + inc_fuse_per_wg - 1) / inc_fuse_per_wg),
                                            update_grid.z),
                                       dim3(256), (size_t)inc_fuse_lds, stream, (const RcdClass *)g->classes_dev,
                                       g->plan_dev, inc_fuse_lds, inc_fuse_pct, inc_fuse_per_wg);
            }
            else
                hipLaunchKernelGGL(rcd_k_sweep_rows, dim3(sweep_wgs), dim3(RCD_SWEEP_THREADS),
                                   RCD_SWEEP_LDS_FLOATS * 4, stream, (const RcdClass *)g->classes_dev,
                                   (const RcdWg *)g->wgmap_dev);
            ++round_no;
            if (pe) (void)hipEventRecord((*pe)[3 * r + 1], stream);
            if (graph_cut)
                launch_gc_steps();
            else if (incremental)
                launch_inc_steps();
            else if (!recompute)
                hipLaunchKernelGGL(rcd_k_steps_rows, dim3(ncls), dim3(RCD_STEP_THREADS), 0, stream, g->classes_dev,
                                   g->plan_dev);
            else if (!fused)
                hipLaunchKernelGGL(rcd_k_steps, dim3(ncls), dim3(RCD_STEP_THREADS), 0, stream, g->classes_dev,
                                   g->plan_dev);
            if (pe) (void)hipEventRecord((*pe)[3 * r + 2], stream);
            launch_apply(round_no + 1);
            if (pe) (void)hipEventRecord((*pe)[3 * r + 3], stream);
        }
        launches += (graph_cut ? 1 : !recompute || fused ? 2 : 3) * (int64_t)rounds;
        hipError_t le = hipGetLastError();
        if (le != hipSuccess) {
            snprintf(g_hip_err, sizeof g_hip_err, "kernel launch -> %s", hipGetErrorString(le));
            return RCD_ERR_HIP;
        }
        hipError_t e1 = hipMemcpyAsync(pinned(b), g->plan_dev, 2 * sizeof(RcdPlan), hipMemcpyDeviceToHost, stream);
        hipError_t e2 = hipEventRecord(ev[b % RCD_SLOTS], stream);
        if (e1 != hipSuccess || e2 != hipSuccess) {
            snprintf(g_hip_err, sizeof g_hip_err, "progress readback -> %s",
                     hipGetErrorString(e1 != hipSuccess ? e1 : e2));
            return RCD_ERR_HIP;
        }
        batch = b + 1;
        return RCD_OK;
    }

    // Read the progress record of the oldest unread batch: waiting for it (block), or only
    // if it has already arrived.  *got says whether a record was read.
    int poll(bool block, bool *got)
    {
        *got = false;
        if (polled >= batch) return RCD_OK;
        hipEvent_t e = ev[polled % RCD_SLOTS];
        hipError_t q = block ? hipEventSynchronize(e) : hipEventQuery(e);
        if (q == hipErrorNotReady) return RCD_OK;
        if (q != hipSuccess) {
            snprintf(g_hip_err, sizeof g_hip_err, "waiting for a batch of rounds -> %s", hipGetErrorString(q));
            return RCD_ERR_HIP;
        }
        *got = true;
        if (prof) { read_events(polled); prof_done = polled + 1; }
        const RcdPlan *seen = pinned(polled);
        ++polled;
        if (seen[0].bad == 2) {
            finished = true;
            snprintf(g_hip_err, sizeof g_hip_err,
                     "a workgroup's bounded wait at a grid barrier of the multi-workgroup step loop ran out");
            return RCD_ERR_HIP;
        }
        if (seen[0].bad) { finished = true; return RCD_ERR_BAD_SIMILARITY; }
        if (std::max(seen[0].ndone, seen[1].ndone) >= ncls) finished = true;
        if (inc_fuse_lds > 0) {
            // the lists overlap in a run's first rounds only: after a batch in which no class took the fused pass the
            // launches to come leave it out (both update kernels get the same switch, so either serves a class)
            if (seen[1].fused == inc_fuse_seen) inc_fuse_lds = 0;
            inc_fuse_seen = seen[1].fused;
        }
        return RCD_OK;
    }

    // Drain the stream; on success compute the objectives and collect the counters.
    int finish(int rc)
    {
        hipError_t es = hipStreamSynchronize(stream);
        if (prof && es == hipSuccess && rc == RCD_OK)
            for (int64_t b = prof_done; b < batch; ++b) read_events(b);
        for (int i = 0; i < RCD_SLOTS; ++i) {
            if (ev[i]) (void)hipEventDestroy(ev[i]);
            ev[i] = nullptr;
        }
        if (rc != RCD_OK) return rc;
        if (es != hipSuccess) {
            snprintf(g_hip_err, sizeof g_hip_err, "hipStreamSynchronize -> %s", hipGetErrorString(es));
            return RCD_ERR_HIP;
        }
        if (graph_cut)
            hipLaunchKernelGGL(rcd_k_gc_objective, dim3(1, ncls), dim3(64), 0, stream, (const RcdClass *)g->classes_dev,
                               g->obj_dev, g->K);
        else
            hipLaunchKernelGGL(rcd_k_objective, dim3(g->K, ncls), dim3(256), 0, stream, (const RcdClass *)g->classes_dev,
                               g->obj_dev, g->K);
        HIP_TRY(hipMemcpyAsync(g->host.data(), g->classes_dev, sizeof(RcdClass) * ncls, hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipStreamSynchronize(stream));
        for (const RcdClass &c : g->host) {
            g_stats[0] += c.stat_steps;
            g_stats[1] += c.stat_sweeps;
            g_stats[2] += c.stat_entries;
            g_stats[3] += c.stat_useful;
            g_stats[5] += c.stat_computed;
            g_stats[6] += c.stat_ticks;
        }
        g_stats[4] += launches + 1;
        return RCD_OK;
    }
};

// Run every group to completion.  One group: on the caller's stream.  Several:
// each on a stream of the library's own, ordered after what the caller's stream
// holds so far; the host feeds them in turn, so that one group's step loops and
// coverage updates (latency-bound, a few workgroups) overlap the other groups'
// sweeps (bandwidth-bound, the whole chip).  Returns after all of them finished:
// work the caller enqueues afterwards is ordered behind them.  Fills each
// group's obj_dev and accumulates g_stats.
int run_groups(std::vector<Group> &groups, hipStream_t stream)
{
    const int nl = (int)groups.size();
    if (nl < 1) return RCD_OK;
    if (nl > RCD_MAX_LANES) return RCD_ERR_INVALID_ARG;
    RCD_TRY(ensure_pinned());
    const int target_total = env_int("RCD_TARGET_ITEMS", 2048, 1, 1 << 20);
    RCD_TRY(sweep_setup());
    // one workgroup of the stored-S sweep fills a compute unit (its LDS holds the coverage vectors);
    // two per unit, run one after the other, even out what the waves of the first leave uneven
    const int sweep_target = env_int("RCD_SWEEP_WGS", 2 * cu_count(), 1, RCD_MAX_SWEEP_WGS);
    std::vector<Lane> lanes(nl);
    int rc = RCD_OK;
    int started = 0;
    if (nl == 1) {
        rc = lanes[0].start(groups[0], stream, 0, target_total, sweep_target, g_profile_on != 0);
        started = 1;
    } else {
        RCD_TRY(ensure_side_streams(nl));
        hipEvent_t ready;
        HIP_TRY(hipEventCreateWithFlags(&ready, hipEventDisableTiming));
        hipError_t e = hipEventRecord(ready, stream);
        for (int i = 0; i < nl && e == hipSuccess; ++i) e = hipStreamWaitEvent(g_side[i], ready, 0);
        (void)hipEventDestroy(ready);
        if (e != hipSuccess) {
            snprintf(g_hip_err, sizeof g_hip_err, "stream fork -> %s", hipGetErrorString(e));
            return RCD_ERR_HIP;
        }
        const int per_lane = std::max(256, target_total * 2 / (nl + 1));
        for (int i = 0; i < nl && rc == RCD_OK; ++i) {
            rc = lanes[i].start(groups[i], g_side[i], i, per_lane, sweep_target, false);
            ++started;
        }
    }
    // One lane: one batch ahead, blocking waits.  Several: up to three batches queued per
    // lane, so that no lane runs dry while the host looks after another one; records are
    // read as they arrive.
    const int depth = nl == 1 ? 2 : RCD_SLOTS - 1;
    while (rc == RCD_OK) {
        bool any = false, progressed = false;
        for (int i = 0; i < nl && rc == RCD_OK; ++i) {
            Lane &ln = lanes[i];
            if (ln.finished) continue;
            any = true;
            while (rc == RCD_OK && ln.batch - ln.polled < depth) {
                rc = ln.enqueue_batch();
                progressed = true;
            }
            bool got = false;
            if (rc == RCD_OK) rc = ln.poll(nl == 1, &got);
            progressed |= got;
        }
        if (!any) break;
        if (!progressed) std::this_thread::yield();
    }
    // every started lane is drained, whatever happened, before the workspace is let go
    for (int i = 0; i < started; ++i) {
        const int r = lanes[i].finish(rc);
        if (rc == RCD_OK) rc = r;
    }
    return rc;
}

int run_group(Group &g, hipStream_t stream)
{
    std::vector<Group> one(1);
    one[0] = std::move(g);
    const int rc = run_groups(one, stream);
    g = std::move(one[0]);
    return rc;
}

bool carve_group_fixed(Carver &cv, Group &g, int ncls, int K)
{
    g.classes_dev = cv.take<RcdClass>((size_t)ncls);
    for (int i = 0; i < RCD_MAX_LANES; ++i)
        g.plan_area[i] = reinterpret_cast<RcdPlan *>(cv.take<char>(plan_area_bytes(ncls)));
    g.plan_dev = g.plan_area[0];
    for (int i = 0; i < RCD_MAX_LANES; ++i)
        g.wg_area[i] = reinterpret_cast<RcdWg *>(cv.take<char>(wg_area_bytes(ncls)));
    g.wgmap_dev = g.wg_area[0];
    g.obj_dev = cv.take<double>((size_t)ncls * K);
    g.K = K;
    return !cv.fail;
}

// The mirrored build is asked for (RCD_SIM_MIRROR = 2), or pays: tiles_in_flight = tiles of the full build
// that the launch holds.
bool mirror_wanted(int dt, int64_t d, int64_t tiles_in_flight)
{
    const int mode = env_int("RCD_SIM_MIRROR", 1, 0, 2);
    if (mode != 1) return mode == 2;
    return (dt == RCD_F32 ? 32 : 2) * d >= 2048 && sweep_setup() == RCD_OK && tiles_in_flight > cu_count();
}

int launch_similarity(const void *X, int dt, int64_t n, int64_t d, int64_t ldx, const int32_t *row_index,
                      float sigma2, float *S, int64_t ld_s, int ncols_pad, float *sq, hipStream_t stream)
{
    const float exp_scale = (float)(-1.4426950408889634 / (2.0 * (double)sigma2));
    const unsigned nblk = (unsigned)((n + 3) / 4);
    const bool fast = rows_fit_fast_path(X, dt, d, ldx);
    if (dt == RCD_F32)
        hipLaunchKernelGGL(sim::k_row_norms<float>, dim3(nblk), dim3(256), 0, stream, (const float *)X,
                           (long long)ldx, row_index, (int)n, (int)d, sq);
    else
        hipLaunchKernelGGL(sim::k_row_norms<__bf16>, dim3(nblk), dim3(256), 0, stream, (const __bf16 *)X,
                           (long long)ldx, row_index, (int)n, (int)d, sq);
    // Only the tiles on and above the diagonal, each also storing its transpose, when the output can take
    // 16-byte stores along its rows and the k loop is long enough to be worth it: the mirrored stores go out
    // in 16-byte pieces (about 2 TB/s against 2.7 for whole lines), so this pays once the matrix cores, not
    // the writes, bound a tile: from about 2048 matrix-core cycles per 256 x 256 tile and wave (measured:
    // fp32 d >= 96 and bf16 d >= 1024 gain, up to 1.9x and 1.6x; fp32 d = 64 is even, bf16 d = 512 loses),
    // and once the full build has more tiles than the chip has compute units (below that the mirrored
    // build only leaves more of them idle).
    // RCD_SIM_MIRROR: 0 never, 1 by that rule, 2 whenever the layout allows.
    const int64_t tm = (n + sim::pipe::TM - 1) / sim::pipe::TM;
    const bool mirror = fast && mirror_wanted(dt, d, tm * tm) &&
                        (ncols_pad + sim::pipe::TN - 1) / sim::pipe::TN == tm &&
                        (reinterpret_cast<uintptr_t>(S) & 15) == 0 && ld_s % 4 == 0;
    if (mirror) {
        RCD_TRY(fast_setup());
        const int64_t tiles = ((tm + 1) / 2) * (tm + 1);
        const dim3 grid((unsigned)((tiles + 7) / 8 * 8));
        if (dt == RCD_F32)
            hipLaunchKernelGGL((sim::k_gram_rbf_fast<float, sim::EPI_RBF_MIRROR>), grid, dim3(sim::THREADS),
                               sim::pipe::LDS_BYTES, stream, (const float *)X, (long long)ldx, row_index, (int)n, (int)d,
                               (const float *)sq, exp_scale, S, (long long)ld_s, ncols_pad, (double *)nullptr);
        else
            hipLaunchKernelGGL((sim::k_gram_rbf_fast<__bf16, sim::EPI_RBF_MIRROR>), grid, dim3(sim::THREADS),
                               sim::pipe::LDS_BYTES, stream, (const __bf16 *)X, (long long)ldx, row_index, (int)n, (int)d,
                               (const float *)sq, exp_scale, S, (long long)ld_s, ncols_pad, (double *)nullptr);
    } else if (fast) {
        RCD_TRY(fast_setup());
        const int64_t tiles = ((n + sim::pipe::TM - 1) / sim::pipe::TM) * ((ncols_pad + sim::pipe::TN - 1) / sim::pipe::TN);
        const dim3 grid((unsigned)((tiles + 7) / 8 * 8));
        if (dt == RCD_F32)
            hipLaunchKernelGGL(sim::k_gram_rbf_fast<float>, grid, dim3(sim::THREADS), sim::pipe::LDS_BYTES, stream,
                               (const float *)X, (long long)ldx, row_index, (int)n, (int)d, (const float *)sq,
                               exp_scale, S, (long long)ld_s, ncols_pad, (double *)nullptr);
        else
            hipLaunchKernelGGL(sim::k_gram_rbf_fast<__bf16>, grid, dim3(sim::THREADS), sim::pipe::LDS_BYTES, stream,
                               (const __bf16 *)X, (long long)ldx, row_index, (int)n, (int)d, (const float *)sq,
                               exp_scale, S, (long long)ld_s, ncols_pad, (double *)nullptr);
    } else {
        const dim3 grid((unsigned)((ncols_pad + sim::BN - 1) / sim::BN), (unsigned)((n + sim::BM - 1) / sim::BM));
        if (dt == RCD_F32)
            hipLaunchKernelGGL(sim::k_gram_rbf<float>, grid, dim3(sim::THREADS), 0, stream, (const float *)X,
                               (long long)ldx, row_index, (int)n, (int)d, (const float *)sq, exp_scale, S,
                               (long long)ld_s, ncols_pad, (double *)nullptr);
        else
            hipLaunchKernelGGL(sim::k_gram_rbf<__bf16>, grid, dim3(sim::THREADS), 0, stream, (const __bf16 *)X,
                               (long long)ldx, row_index, (int)n, (int)d, (const float *)sq, exp_scale, S,
                               (long long)ld_s, ncols_pad, (double *)nullptr);
    }
    HIP_TRY(hipGetLastError());
    return RCD_OK;
}

// Tiles of the pairwise-distance sum: the same Gram kernels with the distance epilogue.
void bandwidth_tiles(int64_t n, bool fast, int64_t *tiles_m, int64_t *tiles_n)
{
    if (fast) {
        *tiles_m = (n + sim::pipe::TM - 1) / sim::pipe::TM;
        *tiles_n = (n + sim::pipe::TN - 1) / sim::pipe::TN;
    } else {
        *tiles_m = (n + sim::BM - 1) / sim::BM;
        *tiles_n = (n + sim::BN - 1) / sim::BN;
    }
}

int launch_row_norms(const void *X, int dt, int64_t n, int64_t d, int64_t ldx, const int32_t *row_index, float *sq,
                     hipStream_t stream)
{
    const unsigned nblk = (unsigned)((n + 3) / 4);
    if (dt == RCD_F32)
        hipLaunchKernelGGL(sim::k_row_norms<float>, dim3(nblk), dim3(256), 0, stream, (const float *)X, (long long)ldx,
                           row_index, (int)n, (int)d, sq);
    else
        hipLaunchKernelGGL(sim::k_row_norms<__bf16>, dim3(nblk), dim3(256), 0, stream, (const __bf16 *)X,
                           (long long)ldx, row_index, (int)n, (int)d, sq);
    HIP_TRY(hipGetLastError());
    return RCD_OK;
}

// One class of a data set whose similarity matrix is to be built into its descriptor's M.
struct SimRequest {
    const int32_t *row_index;
    int64_t n;
    float *S;
    int64_t ld;
    float *sq;
};

// Similarity matrices of several classes over the same features.  Rows that fit the fast path: all the
// row norms in one launch and all the tiles in one launch per 64 classes, so that classes of a few tiles
// fill the chip together; otherwise one pair of launches per class.
int launch_similarity_batch(const void *X, int dt, int64_t d, int64_t ldx, float sigma2,
                            const std::vector<SimRequest> &req, hipStream_t stream)
{
    if (req.empty()) return RCD_OK;
    if (!rows_fit_fast_path(X, dt, d, ldx) || req.size() == 1 || env_int("RCD_SIM_BATCH", 1, 0, 1) == 0) {
        for (const SimRequest &q : req)
            RCD_TRY(launch_similarity(X, dt, q.n, d, ldx, q.row_index, sigma2, q.S, q.ld, (int)q.ld, q.sq, stream));
        return RCD_OK;
    }
    RCD_TRY(fast_setup());
    const float exp_scale = (float)(-1.4426950408889634 / (2.0 * (double)sigma2));
    int64_t all_tiles = 0;
    for (const SimRequest &q : req) {
        const int64_t tm = (q.n + sim::pipe::TM - 1) / sim::pipe::TM;
        all_tiles += tm * tm;
    }
    const bool mirror = mirror_wanted(dt, d, all_tiles);
    for (size_t first = 0; first < req.size(); first += sim::SIM_BATCH) {
        sim::SimBatch b;
        memset(&b, 0, sizeof b);
        b.njobs = (int)std::min<size_t>(sim::SIM_BATCH, req.size() - first);
        int64_t wgs = 0, row_wgs = 0;
        for (int j = 0; j < b.njobs; ++j) {
            const SimRequest &q = req[first + j];
            const int64_t tm = (q.n + sim::pipe::TM - 1) / sim::pipe::TM;
            const int64_t tiles = mirror ? ((tm + 1) / 2) * (tm + 1) : tm * ((q.ld + sim::pipe::TN - 1) / sim::pipe::TN);
            sim::SimJob &job = b.job[j];
            job.row_index = q.row_index;
            job.sq = q.sq;
            job.S = q.S;
            job.lds_out = q.ld;
            job.n = (int)q.n;
            job.ncols_pad = (int)q.ld;
            job.wg_begin = (int)wgs;
            job.wg_count = (int)((tiles + 7) / 8 * 8);
            job.row_wg_begin = (int)row_wgs;
            wgs += job.wg_count;
            row_wgs += (q.n + 3) / 4;
            if (wgs > 0x7fffffff || row_wgs > 0x7fffffff) return RCD_ERR_UNSUPPORTED;
        }
        if (dt == RCD_F32) {
            hipLaunchKernelGGL(sim::k_row_norms_batch<float>, dim3((unsigned)row_wgs), dim3(256), 0, stream,
                               (const float *)X, (long long)ldx, (int)d, b);
            if (mirror)
                hipLaunchKernelGGL((sim::k_gram_rbf_fast_batch<float, sim::EPI_RBF_MIRROR>), dim3((unsigned)wgs),
                                   dim3(sim::THREADS), sim::pipe::LDS_BYTES, stream, (const float *)X, (long long)ldx,
                                   (int)d, exp_scale, b);
            else
                hipLaunchKernelGGL((sim::k_gram_rbf_fast_batch<float, sim::EPI_RBF>), dim3((unsigned)wgs),
                                   dim3(sim::THREADS), sim::pipe::LDS_BYTES, stream, (const float *)X, (long long)ldx,
                                   (int)d, exp_scale, b);
        } else {
            hipLaunchKernelGGL(sim::k_row_norms_batch<__bf16>, dim3((unsigned)row_wgs), dim3(256), 0, stream,
                               (const __bf16 *)X, (long long)ldx, (int)d, b);
            if (mirror)
                hipLaunchKernelGGL((sim::k_gram_rbf_fast_batch<__bf16, sim::EPI_RBF_MIRROR>), dim3((unsigned)wgs),
                                   dim3(sim::THREADS), sim::pipe::LDS_BYTES, stream, (const __bf16 *)X, (long long)ldx,
                                   (int)d, exp_scale, b);
            else
                hipLaunchKernelGGL((sim::k_gram_rbf_fast_batch<__bf16, sim::EPI_RBF>), dim3((unsigned)wgs),
                                   dim3(sim::THREADS), sim::pipe::LDS_BYTES, stream, (const __bf16 *)X, (long long)ldx,
                                   (int)d, exp_scale, b);
        }
        HIP_TRY(hipGetLastError());
    }
    return RCD_OK;
}

void set_recompute_source(RcdClass &c, const void *X, int dt, int64_t d, int64_t ldx, const int32_t *x_index,
                          float sigma2)
{
    c.X = X;
    c.x_index = x_index;
    c.ldx64 = ldx;
    c.d = (int)d;
    c.ldx = (int)std::min<int64_t>(ldx, 0x7fffffff);
    c.dt = dt;
    c.exp_scale = (float)(-1.4426950408889634 / (2.0 * (double)sigma2));
    c.tw = rows_fit_fast_path(X, dt, d, ldx) ? RCD_TILE_FAST : RCD_TILE_RC;
}

int check_workspace(const void *ws, size_t have, size_t need)
{
    if (need == 0) return RCD_OK;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) != 0 || have < need) return RCD_ERR_WORKSPACE;
    return RCD_OK;
}

int check_common(int64_t n, int K)
{
    if (n < 0) return RCD_ERR_INVALID_ARG;
    if (K < 1) return RCD_ERR_INVALID_ARG;
    if (K > RCD_MAX_K) return RCD_ERR_UNSUPPORTED;
    if (n > (int64_t)0x7fffff00) return RCD_ERR_UNSUPPORTED;
    return RCD_OK;
}

void reset_stats() { memset(g_stats, 0, sizeof g_stats); }

} // namespace

// ===========================================================================
extern "C" {

const char *rcd_strerror(int status)
{
    switch (status) {
    case RCD_OK: return "ok";
    case RCD_ERR_INVALID_ARG: return "invalid argument";
    case RCD_ERR_BAD_LABEL: return "label outside [0, L)";
    case RCD_ERR_BAD_CAPACITY: return "bad capacity or quota";
    case RCD_ERR_UNSUPPORTED: return "unsupported size, dtype or mode";
    case RCD_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case RCD_ERR_HIP: return "HIP runtime error";
    case RCD_ERR_BAD_SIMILARITY: return "similarity outside [0, 1]";
    default: return "unknown status";
    }
}

const char *rcd_last_hip_error(void) { return g_hip_err; }

void rcd_last_stats(int64_t *out8_host)
{
    if (out8_host) memcpy(out8_host, g_stats, sizeof g_stats);
}

void rcd_profile(int enable)
{
    g_profile_on = enable ? 1 : 0;
    memset(g_prof, 0, sizeof g_prof);
}

void rcd_profile_read(double *out8_host)
{
    if (out8_host) memcpy(out8_host, g_prof, sizeof g_prof);
}

size_t rcd_similarity_workspace_bytes(int64_t n) { return n > 0 ? up256((size_t)n * 4) : 0; }

int rcd_similarity(const void *X_dev, int dt, int64_t n, int64_t d, int64_t ld_x,
                   const int32_t *row_index_dev, float sigma2, float *S_dev, int64_t ld_s,
                   void *workspace_dev, size_t workspace_bytes, void *stream)
{
    if (dt != RCD_F32 && dt != RCD_BF16) return RCD_ERR_UNSUPPORTED;
    if (n < 0 || d < 1 || ld_x < d || ld_s < n || !(sigma2 > 0.f) || !std::isfinite(sigma2)) return RCD_ERR_INVALID_ARG;
    if (n > (int64_t)0x7fffff00 || d > (int64_t)0x7fffff00) return RCD_ERR_UNSUPPORTED;
    if (n == 0) return RCD_OK;
    if (!X_dev || !S_dev) return RCD_ERR_INVALID_ARG;
    RCD_TRY(check_workspace(workspace_dev, workspace_bytes, rcd_similarity_workspace_bytes(n)));
    return launch_similarity(X_dev, dt, n, d, ld_x, row_index_dev, sigma2, S_dev, ld_s, (int)n,
                             (float *)workspace_dev, (hipStream_t)stream);
}

size_t rcd_bandwidth_workspace_bytes(int64_t n)
{
    if (n <= 0) return 0;
    // row norms, one double per tile (whichever path's tile list is longer), the total
    int64_t tm, tn, fm, fn;
    bandwidth_tiles(n, false, &tm, &tn);
    bandwidth_tiles(n, true, &fm, &fn);
    const int64_t slots = std::max(tm * tn, ((fm + 1) / 2) * (fm + 1));
    return up256((size_t)n * 4) + up256((size_t)slots * 8) + 256;
}

int rcd_bandwidth(const void *X_dev, int dt, int64_t n, int64_t d, int64_t ld_x, const int32_t *row_index_dev,
                  double *sigma_host, void *workspace_dev, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (dt != RCD_F32 && dt != RCD_BF16) return RCD_ERR_UNSUPPORTED;
    if (n < 0 || d < 1 || ld_x < d || !sigma_host) return RCD_ERR_INVALID_ARG;
    if (n > (int64_t)0x7fffff00 || d > (int64_t)0x7fffff00) return RCD_ERR_UNSUPPORTED;
    *sigma_host = 0.0;
    if (n == 0) return RCD_OK;
    if (!X_dev) return RCD_ERR_INVALID_ARG;
    RCD_TRY(check_workspace(workspace_dev, workspace_bytes, rcd_bandwidth_workspace_bytes(n)));
    Carver cv(workspace_dev, workspace_bytes);
    float *sq = cv.take<float>((size_t)n);
    const bool fast = rows_fit_fast_path(X_dev, dt, d, ld_x);
    int64_t tm, tn;
    bandwidth_tiles(n, fast, &tm, &tn);
    if (fast) {
        // the fast kernel walks the tiles on and above the diagonal, folded into a rectangle
        tn = tm + 1;
        tm = (tm + 1) / 2;
    }
    double *pair_sums = cv.take<double>((size_t)(tm * tn));
    double *total = cv.take<double>(1);
    if (cv.fail) return RCD_ERR_WORKSPACE;
    RCD_TRY(launch_row_norms(X_dev, dt, n, d, ld_x, row_index_dev, sq, stream));
    if (fast) {
        RCD_TRY(fast_setup());
        const dim3 grid((unsigned)((tm * tn + 7) / 8 * 8));
        if (dt == RCD_F32)
            hipLaunchKernelGGL((sim::k_gram_rbf_fast<float, sim::EPI_DISTANCE>), grid, dim3(sim::THREADS),
                               sim::pipe::LDS_BYTES, stream, (const float *)X_dev, (long long)ld_x, row_index_dev, (int)n,
                               (int)d, (const float *)sq, 1.f, (float *)nullptr, 0LL, (int)n, pair_sums);
        else
            hipLaunchKernelGGL((sim::k_gram_rbf_fast<__bf16, sim::EPI_DISTANCE>), grid, dim3(sim::THREADS),
                               sim::pipe::LDS_BYTES, stream, (const __bf16 *)X_dev, (long long)ld_x, row_index_dev, (int)n,
                               (int)d, (const float *)sq, 1.f, (float *)nullptr, 0LL, (int)n, pair_sums);
    } else {
        const dim3 grid((unsigned)tn, (unsigned)tm);
        if (dt == RCD_F32)
            hipLaunchKernelGGL((sim::k_gram_rbf<float, sim::EPI_DISTANCE>), grid, dim3(sim::THREADS), 0, stream,
                               (const float *)X_dev, (long long)ld_x, row_index_dev, (int)n, (int)d, (const float *)sq,
                               1.f, (float *)nullptr, 0LL, (int)n, pair_sums);
        else
            hipLaunchKernelGGL((sim::k_gram_rbf<__bf16, sim::EPI_DISTANCE>), grid, dim3(sim::THREADS), 0, stream,
                               (const __bf16 *)X_dev, (long long)ld_x, row_index_dev, (int)n, (int)d, (const float *)sq,
                               1.f, (float *)nullptr, 0LL, (int)n, pair_sums);
    }
    hipLaunchKernelGGL(sim::k_sum_doubles, dim3(1), dim3(1024), 0, stream, (const double *)pair_sums,
                       (long long)(tm * tn), total);
    HIP_TRY(hipGetLastError());
    double pairs = 0.0;
    HIP_TRY(hipMemcpyAsync(&pairs, total, sizeof pairs, hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    // every unordered pair was summed once; the n zero distances of a sample to itself add nothing
    *sigma_host = 2.0 * pairs / ((double)n * (double)n);
    return RCD_OK;
}

int rcd_quota(int64_t n_l, const int32_t *r_host, int K, int64_t *cap_host)
{
    if (n_l < 0 || K < 1 || !r_host || !cap_host) return RCD_ERR_INVALID_ARG;
    int64_t R = 0;
    for (int k = 0; k < K; ++k) {
        if (r_host[k] < 1) return RCD_ERR_BAD_CAPACITY;
        R += r_host[k];
    }
    int64_t given = 0;
    for (int k = 0; k < K; ++k) {
        // n_l * r_k fits in 128 bits trivially; keep to 64 by splitting the product
        cap_host[k] = (int64_t)(((__int128)n_l * r_host[k]) / R);
        given += cap_host[k];
    }
    // workers in the order (r descending, index ascending) receive the remainder
    std::vector<int> order(K);
    for (int k = 0; k < K; ++k) order[k] = k;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return r_host[a] > r_host[b]; });
    int64_t rem = n_l - given;
    for (int i = 0; i < K && rem > 0; ++i, --rem) cap_host[order[i]] += 1;
    return RCD_OK;
}

size_t rcd_worker_shards_workspace_bytes(int64_t N, int K)
{
    if (N <= 0 || K < 1) return 0;
    const size_t nchunks = (size_t)((N + split::CHUNK - 1) / split::CHUNK);
    return up256(nchunks * K * 4) + 2 * up256((size_t)K * 4) + up256(sizeof(RcdPlan));
}

int rcd_worker_shards(const int32_t *assign_dev, int64_t N, int K, int32_t *index_dev, int64_t *offset_host,
                      void *workspace_dev, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    RCD_TRY(check_common(N, K));
    if (!offset_host) return RCD_ERR_INVALID_ARG;
    for (int k = 0; k <= K; ++k) offset_host[k] = 0;
    if (N == 0) return RCD_OK;
    if (!assign_dev || !index_dev) return RCD_ERR_INVALID_ARG;
    RCD_TRY(check_workspace(workspace_dev, workspace_bytes, rcd_worker_shards_workspace_bytes(N, K)));
    // the class split's stable counting sort, keyed by worker instead of label
    const int nchunks = (int)((N + split::CHUNK - 1) / split::CHUNK);
    Carver cv(workspace_dev, workspace_bytes);
    int32_t *chunk_hist = cv.take<int32_t>((size_t)nchunks * K);
    int32_t *count_dev = cv.take<int32_t>((size_t)K);
    int32_t *offset_dev = cv.take<int32_t>((size_t)K);
    RcdPlan *flag = reinterpret_cast<RcdPlan *>(cv.take<char>(sizeof(RcdPlan)));
    if (cv.fail) return RCD_ERR_WORKSPACE;
    HIP_TRY(hipMemsetAsync(flag, 0, sizeof(RcdPlan), stream));
    hipLaunchKernelGGL(split::k_hist, dim3(nchunks), dim3(64), (size_t)K * 4, stream, assign_dev, (long long)N, K,
                       chunk_hist, flag, 1);
    hipLaunchKernelGGL(split::k_scan, dim3((K + 255) / 256), dim3(256), 0, stream, chunk_hist, nchunks, K, count_dev);
    HIP_TRY(hipGetLastError());
    std::vector<int32_t> count(K), offset(K);
    RcdPlan flag_host;
    HIP_TRY(hipMemcpyAsync(count.data(), count_dev, sizeof(int32_t) * K, hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipMemcpyAsync(&flag_host, flag, sizeof flag_host, hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    if (flag_host.bad) return RCD_ERR_BAD_LABEL;
    int32_t run = 0;
    for (int k = 0; k < K; ++k) {
        offset[k] = run;
        offset_host[k] = run;
        run += count[k];
    }
    offset_host[K] = run;
    HIP_TRY(hipMemcpyAsync(offset_dev, offset.data(), sizeof(int32_t) * K, hipMemcpyHostToDevice, stream));
    hipLaunchKernelGGL(split::k_scatter, dim3(nchunks), dim3(64), (size_t)K * 4, stream, assign_dev, (long long)N, K,
                       (const int32_t *)chunk_hist, (const int32_t *)offset_dev, index_dev);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(stream));
    return RCD_OK;
}

int rcd_batch_sizes(int64_t B, const int32_t *r_host, int K, int64_t *batch_host)
{
    if (B < 1 || K < 1 || !r_host || !batch_host) return RCD_ERR_INVALID_ARG;
    for (int k = 0; k < K; ++k)
        if (r_host[k] < 1) return RCD_ERR_BAD_CAPACITY;
    for (int k = 0; k < K; ++k) {
        // B r_k / r_1 to the nearest integer (halves up), never below 1
        const __int128 num = (__int128)B * r_host[k] * 2 + r_host[0];
        const int64_t q = (int64_t)(num / ((__int128)2 * r_host[0]));
        batch_host[k] = q < 1 ? 1 : q;
    }
    return RCD_OK;
}

size_t rcd_class_workspace_bytes(int64_t n, int K, int mode)
{
    if (n <= 0 || K < 1 || K > RCD_MAX_K) return 0;
    const bool stored = mode != RCD_MODE_RECOMPUTE;
    return group_fixed_bytes(1, K) + class_state_bytes(n, K, stored);
}

int rcd_dataset_workspace_bytes(int64_t N, int L, int64_t max_class_n, int K, int mode,
                                size_t *min_bytes, size_t *full_bytes)
{
    if (N < 0 || L < 1 || K < 1 || max_class_n < 0 || max_class_n > N) return RCD_ERR_INVALID_ARG;
    if (K > RCD_MAX_K) return RCD_ERR_UNSUPPORTED;
    const bool stored = mode != RCD_MODE_RECOMPUTE;
    const size_t nchunks = (size_t)((N + split::CHUNK - 1) / split::CHUNK);
    const size_t fixed = up256((size_t)N * 4) + 2 * up256((size_t)L * 4) + up256(nchunks * L * 4) + up256(sizeof(RcdPlan));
    const size_t one = class_state_bytes(max_class_n, K, stored) + up256((size_t)max_class_n * 4);
    if (min_bytes) *min_bytes = fixed + group_fixed_bytes(1, K) + one;
    // every class at most max_class_n and the sizes sum to N: the similarity
    // matrices together need at most ceil(N / max) classes of the largest size
    const size_t worst_classes = max_class_n > 0 ? (size_t)std::min<int64_t>(L, (N + max_class_n - 1) / max_class_n + 1) : 1;
    if (full_bytes) {
        size_t small = class_state_bytes(1, K, stored) + up256(4);
        *full_bytes = fixed + group_fixed_bytes(L, K) + worst_classes * one + (size_t)L * small;
    }
    return RCD_OK;
}

size_t rcd_workspace_bytes(int64_t N_or_n, int64_t max_class_n, int64_t d, int K, int dt, int mode)
{
    (void)d;    // features are read in place and S is fp32 whatever the feature type:
    (void)dt;   // neither enters the size
    if (N_or_n <= 0 || K < 1 || K > RCD_MAX_K || max_class_n < 0 || max_class_n > N_or_n) return 0;
    if (max_class_n == 0) return rcd_class_workspace_bytes(N_or_n, K, mode);
    // a data set: the smallest size that works whatever the number of classes
    const int L = (int)std::min<int64_t>(N_or_n, RCD_MAX_CLASSES);
    size_t mn = 0;
    if (rcd_dataset_workspace_bytes(N_or_n, L, max_class_n, K, mode, &mn, nullptr) != RCD_OK) return 0;
    return mn;
}

int rcd_init(void)
{
    RCD_TRY(sweep_setup());
    RCD_TRY(fast_setup());
    RCD_TRY(static_setup(nullptr));
    return RCD_OK;
}

void rcd_release(void)
{
    for (int i = 0; i < RCD_MAX_LANES; ++i)
        if (g_side[i]) {
            (void)hipStreamSynchronize(g_side[i]);
            (void)hipStreamDestroy(g_side[i]);
            g_side[i] = nullptr;
        }
    for (int i = 0; i < 4; ++i) {
        for (hipEvent_t e : g_prof_ev[i]) (void)hipEventDestroy(e);
        g_prof_ev[i].clear();
    }
    if (g_pinned) {
        (void)hipHostFree(g_pinned);
        g_pinned = nullptr;
    }
}

int rcd_similarity_static(const void *X_dev, int dt, int64_t n, int64_t d, int64_t ld_x,
                          const int32_t *row_index_dev, float sigma2, float *S_dev, int64_t ld_s, void *stream)
{
    if (dt != RCD_F32 && dt != RCD_BF16) return RCD_ERR_UNSUPPORTED;
    if (n < 0 || d < 1 || ld_x < d || ld_s < n || !(sigma2 > 0.f) || !std::isfinite(sigma2)) return RCD_ERR_INVALID_ARG;
    if (n > RCD_STATIC_MAX_N || d > (int64_t)0x7fffff00) return RCD_ERR_UNSUPPORTED;
    if (n == 0) return RCD_OK;
    if (!X_dev || !S_dev) return RCD_ERR_INVALID_ARG;
    float *norms = nullptr;
    RCD_TRY(static_setup(&norms));
    // the same launches as rcd_similarity, the squared row norms in this device's static array
    return launch_similarity(X_dev, dt, n, d, ld_x, row_index_dev, sigma2, S_dev, ld_s, (int)n, norms,
                             (hipStream_t)stream);
}

int rcd_gain_sweep(const float *S_dev, int64_t ld_s, int64_t n, int K, const float *cur_dev,
                   float *gains_dev, void *workspace_dev, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    RCD_TRY(check_common(n, K));
    if (n == 0) return RCD_OK;
    if (!S_dev || !cur_dev || !gains_dev || ld_s < n) return RCD_ERR_INVALID_ARG;
    if (!stored_supported(n, K)) return RCD_ERR_UNSUPPORTED;
    RCD_TRY(check_workspace(workspace_dev, workspace_bytes, rcd_class_workspace_bytes(n, K, RCD_MODE_STORED)));
    Carver cv(workspace_dev, workspace_bytes);
    Group g;
    if (!carve_group_fixed(cv, g, 1, K)) return RCD_ERR_WORKSPACE;
    g.host.resize(1);
    std::vector<int64_t> cap(K, 0);
    RcdClass &c = g.host[0];
    if (!carve_class(cv, c, n, K, cap.data(), true)) return RCD_ERR_WORKSPACE;
    c.assign_out = nullptr;
    c.nneed = K;
    for (int k = 0; k < K; ++k) c.need[k] = k;
    stored_chunks(c.ld, K, &c.C, &c.rpc);
    RCD_TRY(sweep_setup());
    const std::vector<RcdWg> map =
        deal_workgroups(g.host, env_int("RCD_SWEEP_WGS", 2 * cu_count(), 1, RCD_MAX_SWEEP_WGS));
    RcdPlan plan[2];
    memset(plan, 0, sizeof plan);
    plan[0].ncls = plan[1].ncls = 1;
    HIP_TRY(hipMemcpyAsync(g.plan_dev, plan, sizeof plan, hipMemcpyHostToDevice, stream));
    HIP_TRY(hipMemcpyAsync(g.classes_dev, g.host.data(), sizeof(RcdClass), hipMemcpyHostToDevice, stream));
    HIP_TRY(hipMemcpyAsync(g.wgmap_dev, map.data(), sizeof(RcdWg) * map.size(), hipMemcpyHostToDevice, stream));
    hipLaunchKernelGGL(rcd_k_copy_check, dim3((unsigned)(c.ld / 32), (unsigned)((n + 31) / 32)), dim3(256), 0, stream,
                       S_dev, (long long)ld_s, c.M, c.ld, c.n, g.plan_dev);
    hipLaunchKernelGGL(rcd_k_init, dim3(64, 1), dim3(256), 0, stream, (const RcdClass *)g.classes_dev);
    hipLaunchKernelGGL(rcd_k_import_cur, dim3((unsigned)((n + 255) / 256), K), dim3(256), 0, stream,
                       (const RcdClass *)g.classes_dev, cur_dev);
    hipLaunchKernelGGL(rcd_k_sweep_rows, dim3((unsigned)map.size()), dim3(RCD_SWEEP_THREADS), RCD_SWEEP_LDS_FLOATS * 4,
                       stream, (const RcdClass *)g.classes_dev, (const RcdWg *)g.wgmap_dev);
    hipLaunchKernelGGL(rcd_k_export_gains, dim3((unsigned)((n + 255) / 256), K), dim3(256), 0, stream,
                       (const RcdClass *)g.classes_dev, gains_dev);
    HIP_TRY(hipGetLastError());
    RcdPlan back;
    HIP_TRY(hipMemcpyAsync(&back, &g.plan_dev[0], sizeof back, hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    if (back.bad) return RCD_ERR_BAD_SIMILARITY;
    return RCD_OK;
}

// objective: 0 = facility location, 1 = graph cut (stored S only)
// incremental: stored S, facility location: gains kept current by update lists instead of sweeps
static int partition_class_impl(int objective, bool incremental, const float *S_dev, int64_t ld_s,
                                const void *X_dev, int dt, int64_t d, int64_t ld_x, float sigma2,
                                int64_t n, int K, const int64_t *cap_host,
                                int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                                void *workspace_dev, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    reset_stats();
    RCD_TRY(check_common(n, K));
    if (!cap_host || !obj_host) return RCD_ERR_INVALID_ARG;
    int64_t total = 0;
    for (int k = 0; k < K; ++k) {
        if (cap_host[k] < 0) return RCD_ERR_BAD_CAPACITY;
        total += cap_host[k];
    }
    if (total > n) return RCD_ERR_BAD_CAPACITY;
    for (int k = 0; k < K; ++k) obj_host[k] = 0.0;
    if (n == 0) return RCD_OK;
    if (!assign_dev) return RCD_ERR_INVALID_ARG;
    const bool stored = S_dev != nullptr;
    if (objective == 1 && !stored) return RCD_ERR_INVALID_ARG;
    if (stored) {
        if (ld_s < n) return RCD_ERR_INVALID_ARG;
        if (!stored_supported(n, K)) return RCD_ERR_UNSUPPORTED;
    } else {
        if (!X_dev || d < 1 || ld_x < d || !(sigma2 > 0.f)) return RCD_ERR_INVALID_ARG;
        if (dt != RCD_F32 && dt != RCD_BF16) return RCD_ERR_UNSUPPORTED;
        if (d > (int64_t)0x7fffff00) return RCD_ERR_UNSUPPORTED;
    }
    RCD_TRY(check_workspace(workspace_dev, workspace_bytes,
                            rcd_class_workspace_bytes(n, K, stored ? RCD_MODE_STORED : RCD_MODE_RECOMPUTE)));
    Carver cv(workspace_dev, workspace_bytes);
    Group g;
    if (!carve_group_fixed(cv, g, 1, K)) return RCD_ERR_WORKSPACE;
    g.host.resize(1);
    RcdClass &c = g.host[0];
    if (!carve_class(cv, c, n, K, cap_host, stored)) return RCD_ERR_WORKSPACE;
    c.assign_out = assign_dev;
    c.order_out = order_dev;
    c.objective = objective;
    c.incremental = stored && objective == 0 && incremental;
    if (c.incremental)
        for (int k = 0; k < K; ++k) c.valid[k] = 1;      // the initial gains (column sums) are current
    HIP_TRY(hipMemsetAsync(g.plan_dev, 0, 2 * sizeof(RcdPlan), stream));
    if (stored) {
        hipLaunchKernelGGL(rcd_k_copy_check, dim3((unsigned)(c.ld / 32), (unsigned)((n + 31) / 32)), dim3(256), 0,
                           stream, S_dev, (long long)ld_s, c.M, c.ld, c.n, g.plan_dev);
    } else {
        set_recompute_source(c, X_dev, dt, d, ld_x, nullptr, sigma2);
        RCD_TRY(launch_row_norms(X_dev, dt, n, d, ld_x, nullptr, c.sq, stream));
    }
    RCD_TRY(run_group(g, stream));
    HIP_TRY(hipMemcpy(obj_host, g.obj_dev, sizeof(double) * K, hipMemcpyDeviceToHost));
    return RCD_OK;
}

int rcd_partition_class(const float *S_dev, int64_t ld_s,
                        const void *X_dev, int dt, int64_t d, int64_t ld_x, float sigma2,
                        int64_t n, int K, const int64_t *cap_host,
                        int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                        void *workspace_dev, size_t workspace_bytes, void *stream)
{
    return partition_class_impl(0, false, S_dev, ld_s, X_dev, dt, d, ld_x, sigma2, n, K, cap_host, assign_dev,
                                order_dev, obj_host, workspace_dev, workspace_bytes, stream);
}

int rcd_partition_class_mode(const float *S_dev, int64_t ld_s,
                             const void *X_dev, int dt, int64_t d, int64_t ld_x, float sigma2,
                             int64_t n, int K, const int64_t *cap_host, int mode,
                             int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                             void *workspace_dev, size_t workspace_bytes, void *stream)
{
    switch (mode) {
    case RCD_MODE_AUTO:
        // like the data-set call: gains kept current whenever S is stored
        return partition_class_impl(0, S_dev != nullptr, S_dev, ld_s, X_dev, dt, d, ld_x, sigma2, n, K, cap_host,
                                    assign_dev, order_dev, obj_host, workspace_dev, workspace_bytes, stream);
    case RCD_MODE_STORED:
    case RCD_MODE_INCREMENTAL:
        if (!S_dev && n > 0) return RCD_ERR_INVALID_ARG;
        return partition_class_impl(0, mode == RCD_MODE_INCREMENTAL, S_dev, ld_s, nullptr, RCD_F32, 0, 0, 0.f, n, K,
                                    cap_host, assign_dev, order_dev, obj_host, workspace_dev, workspace_bytes, stream);
    case RCD_MODE_RECOMPUTE:
        if (!X_dev && n > 0) return RCD_ERR_INVALID_ARG;
        return partition_class_impl(0, false, nullptr, 0, X_dev, dt, d, ld_x, sigma2, n, K, cap_host, assign_dev,
                                    order_dev, obj_host, workspace_dev, workspace_bytes, stream);
    default:
        return RCD_ERR_UNSUPPORTED;
    }
}

int rcd_partition_class_graph_cut(const float *S_dev, int64_t ld_s, int64_t n, int K, const int64_t *cap_host,
                                  int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                                  void *workspace_dev, size_t workspace_bytes, void *stream)
{
    if (!S_dev && n > 0) return RCD_ERR_INVALID_ARG;
    return partition_class_impl(1, false, S_dev, ld_s, nullptr, RCD_F32, 0, 0, 0.f, n, K, cap_host, assign_dev,
                                order_dev, obj_host, workspace_dev, workspace_bytes, stream);
}

static int partition_dataset_impl(int objective, const void *X_dev, int dt, int64_t N, int64_t d, int64_t ld_x,
                                  const int32_t *labels_dev, int L, const int32_t *r_host, int K,
                                  float sigma2, int mode,
                                  int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                                  void *workspace_dev, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    reset_stats();
    RCD_TRY(check_common(N, K));
    if (L < 1 || !r_host || !obj_host) return RCD_ERR_INVALID_ARG;
    if (L > RCD_MAX_CLASSES) return RCD_ERR_UNSUPPORTED;
    if (dt != RCD_F32 && dt != RCD_BF16) return RCD_ERR_UNSUPPORTED;
    if (mode != RCD_MODE_AUTO && mode != RCD_MODE_STORED && mode != RCD_MODE_RECOMPUTE && mode != RCD_MODE_INCREMENTAL)
        return RCD_ERR_UNSUPPORTED;
    const bool incremental = objective == 0 && mode == RCD_MODE_INCREMENTAL;
    if (d < 1 || ld_x < d || !(sigma2 > 0.f) || !std::isfinite(sigma2)) return RCD_ERR_INVALID_ARG;
    for (int k = 0; k < K; ++k)
        if (r_host[k] < 1) return RCD_ERR_BAD_CAPACITY;
    for (size_t i = 0; i < (size_t)L * K; ++i) obj_host[i] = 0.0;
    if (N == 0) return RCD_OK;
    if (!X_dev || !labels_dev || !assign_dev) return RCD_ERR_INVALID_ARG;

    // ---- class split (stable counting sort of indices by label)
    const int nchunks = (int)((N + split::CHUNK - 1) / split::CHUNK);
    Carver cv(workspace_dev, workspace_bytes);
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255) != 0) return RCD_ERR_WORKSPACE;
    int32_t *idx = cv.take<int32_t>((size_t)N);
    int32_t *class_count = cv.take<int32_t>((size_t)L);
    int32_t *class_offset = cv.take<int32_t>((size_t)L);
    int32_t *chunk_hist = cv.take<int32_t>((size_t)nchunks * L);
    RcdPlan *flag = reinterpret_cast<RcdPlan *>(cv.take<char>(sizeof(RcdPlan)));
    if (cv.fail) return RCD_ERR_WORKSPACE;
    HIP_TRY(hipMemsetAsync(flag, 0, sizeof(RcdPlan), stream));
    hipLaunchKernelGGL(split::k_hist, dim3(nchunks), dim3(64), (size_t)L * 4, stream, labels_dev, (long long)N, L,
                       chunk_hist, flag, 0);
    hipLaunchKernelGGL(split::k_scan, dim3((L + 255) / 256), dim3(256), 0, stream, chunk_hist, nchunks, L,
                       class_count);
    HIP_TRY(hipGetLastError());
    std::vector<int32_t> count(L), offset(L);
    RcdPlan flag_host;
    HIP_TRY(hipMemcpyAsync(count.data(), class_count, sizeof(int32_t) * L, hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipMemcpyAsync(&flag_host, flag, sizeof flag_host, hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    if (flag_host.bad) return RCD_ERR_BAD_LABEL;
    int32_t run = 0;
    for (int l = 0; l < L; ++l) {
        offset[l] = run;
        run += count[l];
    }
    HIP_TRY(hipMemcpyAsync(class_offset, offset.data(), sizeof(int32_t) * L, hipMemcpyHostToDevice, stream));
    hipLaunchKernelGGL(split::k_scatter, dim3(nchunks), dim3(64), (size_t)L * 4, stream, labels_dev, (long long)N, L,
                       (const int32_t *)chunk_hist, (const int32_t *)class_offset, idx);
    HIP_TRY(hipGetLastError());

    // ---- quotas (same r for every class: the extras land on the same workers)
    std::vector<int64_t> cap((size_t)L * K);
    for (int l = 0; l < L; ++l) RCD_TRY(rcd_quota(count[l], r_host, K, cap.data() + (size_t)l * K));

    // ---- classes advance in groups that fit the workspace
    const size_t group_base = cv.off;
    int max_count = 0;
    for (int l = 0; l < L; ++l) max_count = std::max(max_count, count[l]);
    bool stored = mode != RCD_MODE_RECOMPUTE;
    if (mode == RCD_MODE_AUTO) {
        // stored if the largest class, alone, fits; else recompute everything
        const size_t need_one = group_base + group_fixed_bytes(1, K) + class_state_bytes(max_count, K, true) +
                                up256((size_t)max_count * 4);
        stored = need_one <= workspace_bytes && stored_supported(max_count, K);
    }
    // left to choose, the library keeps the gains current instead of sweeping: same decisions, far fewer bytes
    const bool auto_incremental = mode == RCD_MODE_AUTO && stored && objective == 0;
    if (stored && !stored_supported(max_count, K)) return RCD_ERR_UNSUPPORTED;
    int l0 = 0;
    while (l0 < L) {
        // how many consecutive classes fit?
        size_t need = 0;
        int l1 = l0, live = 0;
        while (l1 < L) {
            size_t add = 0;
            int live_next = live;
            if (count[l1] > 0) {
                add = class_state_bytes(count[l1], K, stored) + (stored ? up256((size_t)count[l1] * 4) : 0);
                live_next = live + 1;
            }
            if (group_base + group_fixed_bytes(std::max(live_next, 1), K) + need + add > workspace_bytes) break;
            need += add;
            live = live_next;
            ++l1;
        }
        if (l1 == l0) return RCD_ERR_WORKSPACE;   // not even one class fits
        if (live > 0) {
            Carver gc((char *)workspace_dev + group_base, workspace_bytes - group_base);
            Group g;
            if (!carve_group_fixed(gc, g, live, K)) return RCD_ERR_WORKSPACE;
            g.host.resize(live);
            std::vector<int> cls_of(live);
            int gi = 0;
            for (int i = 0; i < RCD_MAX_LANES; ++i)
                HIP_TRY(hipMemsetAsync(g.plan_area[i], 0, 2 * sizeof(RcdPlan), stream));
            hipEvent_t sim_ev[2] = {nullptr, nullptr};
            if (g_profile_on) {
                HIP_TRY(hipEventCreate(&sim_ev[0]));
                HIP_TRY(hipEventCreate(&sim_ev[1]));
                HIP_TRY(hipEventRecord(sim_ev[0], stream));
            }
            std::vector<SimRequest> sim_requests;
            for (int l = l0; l < l1; ++l) {
                if (count[l] == 0) continue;
                RcdClass &c = g.host[gi];
                if (!carve_class(gc, c, count[l], K, cap.data() + (size_t)l * K, stored)) return RCD_ERR_WORKSPACE;
                c.assign_out = assign_dev;
                c.order_out = order_dev;
                c.out_index = idx + offset[l];
                c.objective = objective;
                c.incremental = stored && (incremental || auto_incremental);
                if (c.incremental)
                    for (int k = 0; k < K; ++k) c.valid[k] = 1;      // the initial gains (column sums) are current
                if (stored) {
                    float *sq = gc.take<float>((size_t)count[l]);
                    if (gc.fail) return RCD_ERR_WORKSPACE;
                    sim_requests.push_back(SimRequest{idx + offset[l], count[l], c.M, c.ld, sq});
                } else {
                    set_recompute_source(c, X_dev, dt, d, ld_x, idx + offset[l], sigma2);
                    RCD_TRY(launch_row_norms(X_dev, dt, count[l], d, ld_x, idx + offset[l], c.sq, stream));
                }
                cls_of[gi++] = l;
            }
            RCD_TRY(launch_similarity_batch(X_dev, dt, d, ld_x, sigma2, sim_requests, stream));
            if (g_profile_on) HIP_TRY(hipEventRecord(sim_ev[1], stream));
            // Stored mode: deal the classes to a few lanes of about equal work (cost ~ n^3),
            // contiguous in the descriptor array.  A recomputed sweep keeps the matrix cores
            // busy for milliseconds per round, so there is nothing for a second lane to hide.
            int nl = 1;
            if (stored && !g_profile_on) nl = std::min(live, env_int("RCD_LANES", 2, 1, RCD_MAX_LANES));
            // step loops that share classes among workgroups wait for one another inside the kernel: such
            // launches stay on one stream, so that two of them never compete for the compute units
            if (stored && (objective == 1 || incremental || auto_incremental) && multi_wg_wanted(max_count)) nl = 1;
            std::vector<Group> lanes(nl);
            {
                std::vector<double> cum(live + 1, 0.0);
                for (int i = 0; i < live; ++i) {
                    const double n = (double)g.host[i].n;
                    cum[i + 1] = cum[i] + n * n * n + 1.0;
                }
                int a = 0;
                for (int i = 0; i < nl; ++i) {
                    int b = a + 1;   // at least one class per lane, and leave one for each lane after this
                    while (b < live - (nl - 1 - i) && cum[b] < cum[live] * (i + 1) / nl) ++b;
                    if (i == nl - 1) b = live;
                    Group &sub = lanes[i];
                    sub.classes_dev = g.classes_dev + a;
                    sub.plan_dev = sub.plan_area[0] = g.plan_area[i];
                    sub.wgmap_dev = sub.wg_area[0] = g.wg_area[i];
                    sub.obj_dev = g.obj_dev + (size_t)a * K;
                    sub.K = K;
                    sub.host.assign(g.host.begin() + a, g.host.begin() + b);
                    a = b;
                }
            }
            RCD_TRY(run_groups(lanes, stream));
            if (g_profile_on) {
                float ms = 0.f;
                if (hipEventElapsedTime(&ms, sim_ev[0], sim_ev[1]) == hipSuccess) g_prof[4] += ms;
                (void)hipEventDestroy(sim_ev[0]);
                (void)hipEventDestroy(sim_ev[1]);
            }
            std::vector<double> obj((size_t)live * K);
            HIP_TRY(hipMemcpy(obj.data(), g.obj_dev, sizeof(double) * obj.size(), hipMemcpyDeviceToHost));
            for (int i = 0; i < live; ++i)
                memcpy(obj_host + (size_t)cls_of[i] * K, obj.data() + (size_t)i * K, sizeof(double) * K);
        }
        l0 = l1;
    }
    HIP_TRY(hipStreamSynchronize(stream));
    return RCD_OK;
}

int rcd_partition_dataset(const void *X_dev, int dt, int64_t N, int64_t d, int64_t ld_x,
                          const int32_t *labels_dev, int L, const int32_t *r_host, int K,
                          float sigma2, int mode,
                          int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                          void *workspace_dev, size_t workspace_bytes, void *stream)
{
    return partition_dataset_impl(0, X_dev, dt, N, d, ld_x, labels_dev, L, r_host, K, sigma2, mode, assign_dev,
                                  order_dev, obj_host, workspace_dev, workspace_bytes, stream);
}

int rcd_partition_dataset_graph_cut(const void *X_dev, int dt, int64_t N, int64_t d, int64_t ld_x,
                                    const int32_t *labels_dev, int L, const int32_t *r_host, int K,
                                    float sigma2,
                                    int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                                    void *workspace_dev, size_t workspace_bytes, void *stream)
{
    return partition_dataset_impl(1, X_dev, dt, N, d, ld_x, labels_dev, L, r_host, K, sigma2, RCD_MODE_STORED,
                                  assign_dev, order_dev, obj_host, workspace_dev, workspace_bytes, stream);
}

} // extern "C"
