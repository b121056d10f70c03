/*
 * rcd.h - C ABI of the MI355X (gfx950) implementation of the ratio-constrained
 * submodular partitioner of RCD-SGD (arXiv 2211.00839, Algorithm 1, with the
 * facility-location function and Gaussian-kernel similarity of Section 4).
 *
 * Conventions for every entry point
 *   - `*_dev` arguments are device pointers (HIP global memory on the current
 *     device), `*_host` arguments are host pointers.  The caller owns every
 *     buffer, workspace included; the library keeps no pointer to a caller's
 *     buffer after a call returns, allocates no device memory and frees nothing
 *     of the caller's.
 *   - What the library does keep, until rcd_release() or the end of the process:
 *     per calling thread, one small pinned host buffer (progress records of the
 *     partition calls), up to four non-blocking streams of its own (the lanes on
 *     which groups of classes advance side by side) and the events of
 *     rcd_profile; per device, a record of one-time set-up (kernel attributes,
 *     the compute-unit count, the address of the static scratch array of
 *     rcd_similarity_static), guarded by a mutex.  Calls from different threads
 *     are independent as long as their buffers are.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *   - Inputs are never modified.  The return value is an rcd_status; on any
 *     value other than RCD_OK the contents of output buffers are unspecified.
 *     Everything that can be checked from the arguments is checked before the
 *     first launch.  The data-set calls learn the class sizes from the class
 *     split (their first three launches), so the part of their workspace
 *     requirement that depends on those sizes, a label outside [0, L) and a
 *     class too large for the mode are reported after the split and before
 *     anything else runs.  No exception or abort crosses the boundary.
 *   - Same inputs give byte-identical outputs (fixed reduction orders, no
 *     floating-point atomics).
 *   - Tuning: the partition and similarity calls read a few environment
 *     variables named RCD_* at each call (lanes, rounds per batch, workgroups
 *     per launch, steps per launch, the sizes from which large classes are
 *     shared among workgroups or their update lists fused, the bound of a
 *     wait between those workgroups).  They set launch shapes and thresholds
 *     only: none selects the algorithmic route (that is the `mode` argument),
 *     and every setting meets the contract stated at the entry point.  Unset,
 *     each has a measured default.
 *   - "lowest index" always means the lowest position in the caller's arrays.
 *   - Matrices are row-major with an explicit leading dimension in ELEMENTS.
 */
#ifndef RCD_H
#define RCD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RCD_MAX_K 16 /* largest number of workers (blocks) supported */

typedef enum {
    RCD_OK = 0,
    RCD_ERR_INVALID_ARG = 1,  /* null pointer, non-positive size, bad leading dimension, sigma2 <= 0 */
    RCD_ERR_BAD_LABEL = 2,    /* a label outside [0, L) */
    RCD_ERR_BAD_CAPACITY = 3, /* capacity < 1 (data set) / quota < 0 or sum of quotas > n (class) */
    RCD_ERR_UNSUPPORTED = 4,  /* K > RCD_MAX_K, unknown dtype or mode, size beyond 2^31-1 */
    RCD_ERR_WORKSPACE = 5,    /* workspace pointer null/misaligned or smaller than required */
    RCD_ERR_HIP = 6,          /* a HIP call failed; rcd_last_hip_error() has its text */
    RCD_ERR_BAD_SIMILARITY = 7 /* a similarity outside [0, 1] (or NaN) was found in a caller-supplied S */
} rcd_status;

typedef enum { RCD_F32 = 0, RCD_BF16 = 1 } rcd_dtype;

typedef enum {
    RCD_MODE_AUTO = 0,     /* RCD_MODE_INCREMENTAL if the workspace can hold at least one class's S, else
                              RCD_MODE_RECOMPUTE */
    RCD_MODE_STORED = 1,   /* build S per class once, stream it in every gain sweep */
    RCD_MODE_RECOMPUTE = 2, /* never store S: rebuild its tiles from X inside every gain sweep */
    RCD_MODE_INCREMENTAL = 3 /* stored S, and every block's gains are kept current from step to step:
                                taking v* into block k changes cur_k on D = {j : S(j,v*) > cur_k(j)} only, and
                                gain_k(v) moves by sum_{j in D} [max(0,S(j,v)-new_j) - max(0,S(j,v)-old_j)],
                                so a step reads |D| rows of S instead of one per candidate.  Same Algorithm 1,
                                same tie rules; gains are carried in double, where the sweeps of RCD_MODE_STORED
                                sum in fp32: the two routes take the same decisions except at steps whose two
                                best gains differ by less than fp32 rounding of a sum of n terms (inside the
                                1e-5 relative window either choice is a correct run of Algorithm 1). */
} rcd_mode;

/*
 * Similarity build.  Section 4 ("Gaussian kernel with L2 distance"):
 *     S[i*ld_s + j] = exp(-||x_i - x_j||^2 / (2*sigma2)),   0 <= i,j < n,
 * x_i = row i of X (n x d, leading dimension ld_x, dtype dt).  The squared
 * distance comes from the Gram matrix X X^T (matrix cores, fp32 accumulation)
 * and the squared row norms, clamped at 0; S is exactly symmetric and its
 * diagonal is exactly 1.0f.  row_index_dev (nullable, int32[n]) selects rows:
 * x_i = row row_index_dev[i] of X.  Asynchronous on `stream`.
 * Requirements: d >= 1, ld_x >= d, ld_s >= n.  Fastest when X is 16-byte aligned
 * and ld_x * sizeof(element) is a multiple of 16.
 * workspace: rcd_similarity_workspace_bytes(n) bytes (the squared row norms).
 */
int rcd_similarity(const void *X_dev, int dt, int64_t n, int64_t d, int64_t ld_x,
                   const int32_t *row_index_dev, float sigma2, float *S_dev, int64_t ld_s,
                   void *workspace_dev, size_t workspace_bytes, void *stream);
size_t rcd_similarity_workspace_bytes(int64_t n);

/*
 * Kernel bandwidth.  Section 4 sets the bandwidth of the Gaussian kernel to the mean
 * L2 distance over all ordered pairs of the set the similarity is built on:
 *     sigma = sum_{i,j < n} ||x_i - x_j||_2 / n^2
 * (the n zero distances of a sample to itself are part of the n^2).  x_i = row i of X,
 * or row row_index_dev[i] when row_index_dev is non-null, so the set can be the whole
 * data set or one class.  Distances come from the same Gram tiles as rcd_similarity
 * (matrix cores, fp32 accumulation, squared distance clamped at 0 before the root);
 * tile sums and their total are accumulated in double in a fixed order.
 * *sigma_host receives sigma (0 for n = 0); pass sigma*sigma as sigma2 elsewhere.
 * Synchronises `stream` before returning.
 * workspace: rcd_bandwidth_workspace_bytes(n) bytes.
 */
int rcd_bandwidth(const void *X_dev, int dt, int64_t n, int64_t d, int64_t ld_x,
                  const int32_t *row_index_dev, double *sigma_host,
                  void *workspace_dev, size_t workspace_bytes, void *stream);
size_t rcd_bandwidth_workspace_bytes(int64_t n);

/*
 * Quota rule.  Algorithm 1, constraint line: C_{l,j} = n_l * r_j / sum_j r_j,
 * made integral by floor; the remainder goes one each to the workers with the
 * largest r (lowest index first among equals), the same workers in every class.
 * Host only.  r_host[K] >= 1, cap_host[K] receives the quotas (sum = n_l).
 */
int rcd_quota(int64_t n_l, const int32_t *r_host, int K, int64_t *cap_host);

/*
 * One gain sweep (the GreedyStep of Algorithm 1 evaluated for every candidate
 * and every block at once, facility-location f of Section 4):
 *     gains[k*n + v] = sum_{j<n} max(0, S[j*ld_s + v] - cur[k*n + j])
 * for all k < K, v < n, accumulated in fp32 in a fixed order.  S must be
 * symmetric with entries in [0,1]; cur_dev is K x n (coverage vectors).
 * Exposed so that the kernel can be checked and timed on its own; the
 * partition entry points run the same kernel on their internal state.
 * Synchronises `stream` before returning.
 */
int rcd_gain_sweep(const float *S_dev, int64_t ld_s, int64_t n, int K, const float *cur_dev,
                   float *gains_dev, void *workspace_dev, size_t workspace_bytes, void *stream);

/*
 * One class of Algorithm 1 (its inner while loop):
 *   repeat until every quota is met: j* = the non-full block with the least
 *   f (lowest index on ties); v* = the unassigned sample with the largest
 *   f(A_j* u {v}) - f(A_j*) (lowest index on ties); give v* to j*.
 * Similarity source: S_dev (n x n, ld_s, symmetric, entries in [0,1]) if it is
 * non-null, otherwise X_dev/dt/d/ld_x/sigma2 and S is recomputed tile by tile
 * inside every sweep (never stored).
 *   cap_host[K]   quotas, each >= 0, sum <= n
 *   assign_dev[n] block of each sample, -1 if left over (sum of quotas < n)
 *   order_dev[n]  (nullable) step at which the sample was taken, -1 if never
 *   obj_host[K]   f(A_k) of the final blocks, evaluated from the coverage
 *                 vectors in double precision
 * Synchronises `stream` before returning.
 */
int rcd_partition_class(const float *S_dev, int64_t ld_s,
                        const void *X_dev, int dt, int64_t d, int64_t ld_x, float sigma2,
                        int64_t n, int K, const int64_t *cap_host,
                        int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                        void *workspace_dev, size_t workspace_bytes, void *stream);

/*
 * rcd_partition_class with the route as an argument (rcd_partition_class itself sweeps a stored S, or
 * recomputes when S_dev is null):
 *   RCD_MODE_STORED       S_dev required; one gain sweep over S per round
 *   RCD_MODE_INCREMENTAL  S_dev required; gains kept current from step to step
 *   RCD_MODE_RECOMPUTE    X_dev required (S_dev is ignored); S rebuilt tile by tile inside every sweep
 *   RCD_MODE_AUTO         RCD_MODE_INCREMENTAL if S_dev is non-null, else RCD_MODE_RECOMPUTE
 * Workspace: rcd_class_workspace_bytes(n, K, mode) (the stored and incremental routes need the same).
 * Everything else as for rcd_partition_class.
 */
int rcd_partition_class_mode(const float *S_dev, int64_t ld_s,
                             const void *X_dev, int dt, int64_t d, int64_t ld_x, float sigma2,
                             int64_t n, int K, const int64_t *cap_host, int mode,
                             int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                             void *workspace_dev, size_t workspace_bytes, void *stream);

/*
 * Whole data set (Algorithm 1, outer loop): split the samples by label keeping
 * their order, give every class the quotas of rcd_quota, run the class greedy
 * on every class (classes are advanced together, as many at a time as the
 * workspace holds), and join the per-class blocks.
 *   labels_dev[N] in [0, L);  r_host[K] integer capacities >= 1
 *   assign_dev[N] worker of each sample;  order_dev[N] (nullable) step index
 *   inside the sample's own class;  obj_host[L*K] row-major f(A_k^l).
 * Synchronises `stream` before returning.
 */
int rcd_partition_dataset(const void *X_dev, int dt, int64_t N, int64_t d, int64_t ld_x,
                          const int32_t *labels_dev, int L, const int32_t *r_host, int K,
                          float sigma2, int mode,
                          int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                          void *workspace_dev, size_t workspace_bytes, void *stream);

/*
 * The same two calls with the graph-cut function, the other submodular function
 * Section 4 names for Algorithm 1:
 *     f(A) = sum_{v in V_l \ A} sum_{a in A} S(v, a)
 * (the similarity mass between a block and the rest of its class).  Algorithm 1
 * itself, the quotas and both tie rules are unchanged.  f is submodular but not
 * monotone: a marginal value f(A u {v}) - f(A) = sum_{u != v} S(u,v) - 2 sum_{a in A} S(v,a)
 * can be negative, and the largest one is taken all the same, since the quotas
 * are constraints.  S must be symmetric (it is read by rows).  Marginal values are
 * carried in double from exact fp32 entries, so candidates that tie exactly in
 * exact arithmetic tie here.  S is always stored: the class call takes S_dev
 * (n x n, ld_s, entries in [0,1]), the data-set call builds S per class like
 * RCD_MODE_STORED.  Workspace: the RCD_MODE_STORED sizes.  obj_host receives
 * f(A_k) as the sum of the accepted marginal values.  Arguments, outputs, error
 * codes and synchronisation as for rcd_partition_class / rcd_partition_dataset.
 */
int rcd_partition_class_graph_cut(const float *S_dev, int64_t ld_s, int64_t n, int K, const int64_t *cap_host,
                                  int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                                  void *workspace_dev, size_t workspace_bytes, void *stream);
int rcd_partition_dataset_graph_cut(const void *X_dev, int dt, int64_t N, int64_t d, int64_t ld_x,
                                    const int32_t *labels_dev, int L, const int32_t *r_host, int K,
                                    float sigma2,
                                    int32_t *assign_dev, int32_t *order_dev, double *obj_host,
                                    void *workspace_dev, size_t workspace_bytes, void *stream);

/*
 * Hand-off to the training loop (Algorithm 2, initialisation: worker i imports its subset A_i
 * of the partition and runs with a batch size scaled by the capacity ratios).
 *
 * rcd_worker_shards: per-worker index lists from an assignment (stable counting sort by worker).
 *   assign_dev[N] in [0, K), or -1 for a sample given to nobody (skipped)
 *   index_dev[N]  receives the sample indices grouped by worker, ascending inside a worker:
 *                 worker k owns index_dev[offset_host[k] .. offset_host[k+1])
 *   offset_host[K+1]  offset_host[K] = number of assigned samples
 * A value outside [-1, K) gives RCD_ERR_BAD_LABEL.  Synchronises `stream` before returning.
 *
 * rcd_batch_sizes (host only): batch_host[k] = B * r_k / r_1 to the nearest integer (halves up,
 * at least 1), so that worker 1 runs batch B and every worker's batch is proportional to its
 * capacity.  The algorithm box prints the factor the other way round (r_1 / r_i); the text
 * says batch and shard are proportional to the processing speed and that all workers then
 * finish a round in the same time, which only this direction gives.
 */
int rcd_worker_shards(const int32_t *assign_dev, int64_t N, int K, int32_t *index_dev, int64_t *offset_host,
                      void *workspace_dev, size_t workspace_bytes, void *stream);
size_t rcd_worker_shards_workspace_bytes(int64_t N, int K);
int rcd_batch_sizes(int64_t B, const int32_t *r_host, int K, int64_t *batch_host);

/* Workspace sizes in bytes (multiples of 256; the pointer must be 256-byte aligned).
 * rcd_class_workspace_bytes: what rcd_partition_class / rcd_gain_sweep need for a
 *   class of n samples (stored mode includes a private n x ld copy of S).
 * rcd_dataset_workspace_bytes: `min` is enough to run one class of max_class_n at
 *   a time, `full` lets all L classes advance together (fastest). */
size_t rcd_class_workspace_bytes(int64_t n, int K, int mode);
int rcd_dataset_workspace_bytes(int64_t N, int L, int64_t max_class_n, int K, int mode,
                                size_t *min_bytes, size_t *full_bytes);
/* One query for both: max_class_n = 0 gives rcd_class_workspace_bytes(N_or_n, K, mode); max_class_n > 0
 * gives a size with which the data-set calls run N_or_n samples in classes of at most max_class_n
 * samples whatever the number of classes (one class at a time; rcd_dataset_workspace_bytes, which is
 * told L, also gives the size that lets all classes advance together).  d and dt do not enter: features
 * are read in place and S is fp32.  0 on arguments out of range. */
size_t rcd_workspace_bytes(int64_t N_or_n, int64_t max_class_n, int64_t d, int K, int dt, int mode);

/*
 * One-time set-up for the current device (kernel attributes, compute-unit count, address of the
 * static scratch array).  Optional: every entry point does what it needs on its first call; calling
 * this first keeps that work out of a timed or captured region.
 */
int rcd_init(void);
/*
 * Frees what the calling thread's earlier calls keep (pinned progress buffer, the library's own
 * streams, profiling events).  No call of this thread may be in flight.  Later calls set up again.
 */
void rcd_release(void);

/*
 * rcd_similarity for callers that can neither allocate nor pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the
 * workspace, same kernels, same bits in S; the squared row norms live in a static device array of
 * the library (RCD_STATIC_MAX_N floats = 256 KB on every device the library runs on, held until
 * the process ends), so n <= RCD_STATIC_MAX_N, beyond which RCD_ERR_UNSUPPORTED is returned and
 * nothing is launched.  Calls no allocating routine.  Asynchronous on `stream`.  Every call on a
 * device uses that device's one array (each call overwrites the entries it needs): two calls whose
 * kernels may overlap on one device, on different streams or from different threads, race.
 */
#define RCD_STATIC_MAX_N 65536
int rcd_similarity_static(const void *X_dev, int dt, int64_t n, int64_t d, int64_t ld_x,
                          const int32_t *row_index_dev, float sigma2, float *S_dev, int64_t ld_s, void *stream);

/* Static description of a status code. */
const char *rcd_strerror(int status);
/* Text of the HIP error behind the calling thread's last RCD_ERR_HIP ("" if none). */
const char *rcd_last_hip_error(void);

/*
 * Counters of the calling thread's last partition call (for benchmarks):
 *   out[0] greedy steps taken        out[1] gain sweeps that did work
 *   out[2] sum over those sweeps of (candidates x class size) = similarity
 *          entries streamed          out[3] sum over steps of candidates
 *          (gain evaluations Algorithm 1 consumes)
 *   out[4] kernel launches           out[5] sum over sweeps of blocks evaluated
 *          x candidates (gain evaluations computed)
 *   out[6] 10 ns ticks spent in the step loops, summed over classes   out[7] 0
 */
void rcd_last_stats(int64_t *out8_host);

/*
 * Per-kernel timing for benchmarks.  rcd_profile(1) makes the calling thread's
 * later partition calls put HIP events between the launches of every round
 * (on the caller's stream) and add up the elapsed times; rcd_profile(0) turns
 * it off; either call clears the sums.  rcd_profile_read: out[0] = ms spent in
 * the step-loop launches (0 when the step loops run fused into the sweep launch),
 * out[1] = ms in the gain-sweep launches, out[2] = ms in the apply launches,
 * out[3] = rounds timed, out[4] = ms of the similarity builds of
 * rcd_partition_dataset, out[5..7] = 0.
 */
void rcd_profile(int enable);
void rcd_profile_read(double *out8_host);

#ifdef __cplusplus
}
#endif
#endif /* RCD_H */
