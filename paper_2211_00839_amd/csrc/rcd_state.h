// Device-resident state of the class greedy (Algorithm 1, inner loop) shared by
// the host orchestration and the kernels.  One RcdClass per class that is being
// advanced; all classes of a group move in lock step, one "round" at a time:
//   sweep  - recomputes the gain rows that went stale
//   steps  - runs as many greedy steps as the current gain rows allow
// A round is one sweep launch and one step-loop launch (recompute mode can fuse the two: rcd_k_round_rc_fast).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define RCD_KMAX 16          // must equal RCD_MAX_K of the public header
#define RCD_TILE 256         // pitch granule of a stored matrix row (one wave reads 64 lanes x 4 floats at a time)
#define RCD_TILE_RC 128      // candidate columns per sweep tile when S is recomputed, general path
#define RCD_TILE_FAST 256    // the same on the fast path (aligned feature rows, a multiple of 128 bytes long)
#define RCD_ROWS_RC 256      // rows of one recomputed tile
#define RCD_CMAX 32          // most row chunks a class's sweep is split into
#define RCD_SWEEP_WAVES 16    // waves of a stored-S sweep workgroup: each streams one candidate row at a time
#define RCD_SWEEP_THREADS (64 * RCD_SWEEP_WAVES)
#define RCD_INC_FUSE_LDS_MAX (152 * 1024)   // most LDS the fused update pass of the incremental route may take (a byte per sample)
#define RCD_SWEEP_LDS_FLOATS 32768   // LDS of a stored-S sweep workgroup: coverage of the evaluated blocks, one chunk of j
#define RCD_STEP_THREADS 1024
#define RCD_MW_MAX 32        // most workgroups that share one class in the multi-workgroup step loops
#define RCD_MW_INTS 2048     // ints of a class's exchange area for those loops (layout: MW_* below)

// The stored-S sweep kernel exists for these numbers of evaluated blocks; a sweep of nneed blocks runs
// the smallest variant that holds them and stages that many coverage vectors (the spare slots repeat the
// last block), so the chunk of j one pass covers is cut for the variant's slots: slots x chunk floats
// never exceed the workgroup's LDS.
__host__ __device__ constexpr int rcd_sweep_slots(int nneed)
{
    return nneed <= 1 ? 1 : nneed <= 4 ? nneed : nneed <= 6 ? 6 : nneed <= 8 ? 8 : nneed <= 12 ? 12 : 16;
}
__host__ __device__ constexpr int rcd_sweep_chunk(int nneed)
{
    return (RCD_SWEEP_LDS_FLOATS / rcd_sweep_slots(nneed)) / 256 * 256;
}

struct RcdClass {
    // ---- fixed for the run
    float *M;            // stored S: n x ld, M[v][j] = S(j, v), read-only
    float *cur;          // K x ld coverage vectors cur_k(j) = max_{a in A_k} S(j,a)
    float *part;         // RCD_CMAX x K x ld partial gain sums per chunk (stored S: chunk of j; recompute: of rows)
    float *gain;         // K x ld finished gains, indexed by column position
    int32_t *perm;       // ld: class-local index of the candidate at list position (column) p
    int32_t *tilecnt;    // ld/RCD_TILE_RC arrival counters of the sweep's row chunks, per tile
    float *sq;           // recompute mode: squared norms of the class's rows
    int32_t *assign_out; // caller's arrays (global indexing through out_index)
    int32_t *order_out;  // nullable
    const int32_t *out_index; // nullable: position of local sample v in the caller's arrays
    int32_t *mwbuf;      // RCD_MW_INTS ints: what the workgroups of a multi-workgroup step loop exchange
    const void *X;       // recompute mode: features (rows picked through x_index)
    const int32_t *x_index; // nullable
    int64_t ldx64;
    int32_t n, ld, K, total;    // total = sum of quotas
    int32_t d, ldx, dt, mode;
    int32_t tw;          // sweep tile width in columns (recompute mode: RCD_TILE_FAST selects the fast path)
    int32_t row_align;   // rows per chunk are a multiple of this
    float exp_scale;     // -log2(e) / (2 sigma^2)
    int32_t target_items;       // sweep workgroups this class should be split into
    int32_t incremental;        // stored S: gains are kept current by update lists instead of sweeps
    int32_t objective;          // 0 = facility location, 1 = graph cut (stored S, its own step loop)
    int32_t mw, mwseg;          // workgroups that share this class's step loop (0 or 1: one) and the samples each owns
    // ---- evolving
    int32_t nR;          // unassigned samples = live columns
    int32_t t;           // steps taken
    int32_t done;
    int32_t nneed;       // blocks whose gains the next sweep must produce
    int32_t C, rpc;      // chunks of the next sweep and their length (recompute: rows; stored S: j's per pass)
    int32_t tiles_done;  // arrival counter of the sweep's finished tiles
    int32_t need[RCD_KMAX];
    int32_t cblk[RCD_KMAX];  // stored S: chunk partials that make up block k's current gain row
    int32_t cnt[RCD_KMAX];
    int32_t cap[RCD_KMAX];
    int32_t valid[RCD_KMAX];
    int32_t dcount[RCD_KMAX];   // incremental gains: length of block k's pending update list
    double f[RCD_KMAX];  // running f(A_k): sum of accepted gains
    // decisions of the last step loop, consumed by the apply kernel of the same round
    int32_t apply_round; // number of step loops run so far = round the lists belong to
    int32_t nupd, npatch;
    int32_t ujs[RCD_KMAX], usrc[RCD_KMAX], uv[RCD_KMAX], ut[RCD_KMAX];   // block, column position, sample, step
    int32_t ppos[RCD_KMAX], psrc[RCD_KMAX];   // live position <- dead position
    // ---- counters
    int64_t stat_steps, stat_sweeps, stat_entries, stat_useful, stat_computed;
    int64_t stat_ticks;  // 100 MHz ticks spent inside the step loops
};

// Exchange area of the multi-workgroup step loops, in ints from RcdClass::mwbuf (zeroed when a call starts).
enum {
    MW_SLOT = 16,                                // 2 banks x RCD_MW_MAX slots x 16 ints: a workgroup's post (four pieces
                                                 // of three ints and a tag: the post proper, then up to three list entries)
    MW_SLOT_INTS = 16,
    MW_PEND = MW_SLOT + 2 * MW_SLOT_INTS * RCD_MW_MAX,   // RCD_KMAX x RCD_MW_MAX: segment lengths of block k's pending list
    MW_END = MW_PEND + RCD_KMAX * RCD_MW_MAX
};
static_assert(MW_END <= RCD_MW_INTS, "exchange area too small");

// Work layout of one round.  Two of these are kept (launch r reads buffer r&1
// and writes the other), followed in memory by two int32 prefix[ncls+1] arrays:
// prefix[c] = first sweep workgroup of class c.
struct RcdPlan {
    int32_t ncls;        // classes in the group (buffer 0's copy is the one read)
    int32_t arrive;      // arrival counter of classes that finished their steps
    int32_t items;       // sweep workgroups with work this round
    int32_t nactive;     // classes with work this round
    int32_t ndone;       // classes finished
    int32_t bad;         // set by validation kernels (buffer 0 only)
    int32_t fused;       // incremental route: classes served by the fused update pass so far (buffer 1's copy counts)
    int32_t pad;
};

// Stored-S sweep: which class a workgroup serves, and as which of how many.
struct RcdWg {
    int32_t cls, w, W, pad;
};
