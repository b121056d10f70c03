/*
 * CPU oracle for the ratio-constrained submodular partitioner of RCD-SGD
 * (arXiv 2211.00839, Algorithm 1 with the facility-location function of
 * Section 4, item "Submodular functions").
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded,
 * double-precision statement of what the GPU library must compute.  It shares
 * no code, header, table or helper with the HIP path and nothing in the
 * product path may call it: only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark do.
 *
 * Conventions fixed where the paper is silent (each is a reading, not a quote):
 *   - Gaussian kernel:  sim(v,v') = exp(-||v-v'||^2 / (2 sigma^2)); sigma^2 is
 *     an argument (Section 4 names the kernel, prints no formula).
 *   - f(empty set) = 0, so the coverage vector starts at 0.
 *   - argmin over blocks and argmax over elements break exact ties towards the
 *     lowest index (Algorithm 1 allows any minimiser / maximiser).
 *   - the facility-location sum runs over every member of the class, the
 *     candidate itself and already assigned samples included.
 *   - real-valued quotas |V_l| r_j / sum r are turned into integers by floor,
 *     the remainder going one each to the workers of largest capacity
 *     (lowest index first among equals).
 *
 * Pins: see tests/test_oracle_*.py (closed forms, reduction to a sort,
 * reduction to the textbook cardinality-constrained greedy with its (1-1/e)
 * bound against exhaustive search, definition-level re-evaluation of every
 * gain, exact quota vectors, submodularity/monotonicity of f).
 * Parity unpinned by the paper: the choice among exact ties (lowest index is
 * this build's contract, the paper allows any).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* bf16 -> double is exact: a bf16 is the top half of an IEEE binary32. */
static double bf16_bits_to_double(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double elem_as_double(const void *X, int dtype, int64_t idx)
{
    if (dtype == ORACLE_BF16)
        return bf16_bits_to_double(((const uint16_t *)X)[idx]);
    return (double)((const float *)X)[idx];
}

/*
 * Similarity (Section 4, "Gaussian kernel with L2 distance").
 * Every (i,j) pair is computed on its own from coordinate differences; the
 * symmetric half is NOT copied, so symmetry of the output is a checkable fact.
 * The diagonal is the kernel at distance zero, i.e. exactly 1.
 * Outputs: S64 (n*n doubles) and/or S32 (n*n floats, S64 rounded to nearest);
 * either may be NULL.  Returns 0, or -1 on a bad argument.
 */
int oracle_similarity(const void *X, int dtype, int64_t n, int64_t d, int64_t ldx,
                      double sigma2, double *S64, float *S32)
{
    if (!X || n < 0 || d < 1 || ldx < d || !(sigma2 > 0.0))
        return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return -1;
    double *xi = (double *)malloc((size_t)d * sizeof(double));
    if (!xi)
        return -1;
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t t = 0; t < d; ++t)
            xi[t] = elem_as_double(X, dtype, i * ldx + t);
        for (int64_t j = 0; j < n; ++j) {
            double dist2 = 0.0;
            for (int64_t t = 0; t < d; ++t) {
                double diff = xi[t] - elem_as_double(X, dtype, j * ldx + t);
                dist2 += diff * diff;
            }
            double s = exp(-dist2 / (2.0 * sigma2));
            if (S64)
                S64[i * n + j] = s;
            if (S32)
                S32[i * n + j] = (float)s;
        }
    }
    free(xi);
    return 0;
}

/*
 * Quotas (Algorithm 1, the "Constraint C_{l,j}" line): C_{l,j} = n_l r_j / sum r.
 * Integer reading: floor, then +1 to the `rem` workers taken in the order
 * (r descending, index ascending).  cap[K] receives the result.
 */
int oracle_quota(int64_t n_l, const int64_t *r, int K, int64_t *cap)
{
    if (n_l < 0 || K < 1 || !r || !cap)
        return -1;
    int64_t R = 0;
    for (int k = 0; k < K; ++k) {
        if (r[k] < 1)
            return -1;
        R += r[k];
    }
    int64_t given = 0;
    for (int k = 0; k < K; ++k) {
        cap[k] = (n_l * r[k]) / R;
        given += cap[k];
    }
    int64_t rem = n_l - given;
    char *extra = (char *)calloc((size_t)K, 1);
    if (!extra)
        return -1;
    while (rem > 0) {
        int pick = -1;
        for (int k = 0; k < K; ++k) {
            if (extra[k])
                continue;
            if (pick < 0 || r[k] > r[pick])
                pick = k;
        }
        extra[pick] = 1;
        cap[pick] += 1;
        --rem;
    }
    free(extra);
    return 0;
}

/*
 * Facility-location value straight from its definition (Section 4):
 *   f(A) = sum over every v in the class of  max_{a in A} sim(v, a),
 * with f(empty) = 0.  members[m] lists A.
 */
double oracle_f(const float *S, int64_t lds, int64_t n, const int32_t *members, int64_t m)
{
    if (m <= 0)
        return 0.0;
    double total = 0.0;
    for (int64_t v = 0; v < n; ++v) {
        double best = (double)S[v * lds + members[0]];
        for (int64_t a = 1; a < m; ++a) {
            double s = (double)S[v * lds + members[a]];
            if (s > best)
                best = s;
        }
        total += best;
    }
    return total;
}

/* Marginal value of adding v to a block whose coverage vector is cov:
 * f(A u {v}) - f(A) = sum_j max(0, sim(j,v) - cov_j)  (incremental form of the
 * definition above; the equality is what tests/test_oracle_greedy.py pins). */
static double gain_of(const float *S, int64_t lds, int64_t n, const double *cov, int64_t v)
{
    double g = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        double diff = (double)S[j * lds + v] - cov[j];
        if (diff > 0.0)
            g += diff;
    }
    return g;
}

/* All gains of one block at the current state; entries of assigned samples
 * are set to -1.  Exposed so that kernel-level tests can compare whole rows. */
int oracle_gain_row(const float *S, int64_t lds, int64_t n, const double *cov,
                    const int32_t *assign, double *gains)
{
    if (!S || !cov || !gains || n < 0 || lds < n)
        return -1;
    for (int64_t v = 0; v < n; ++v)
        gains[v] = (assign && assign[v] >= 0) ? -1.0 : gain_of(S, lds, n, cov, v);
    return 0;
}

/*
 * One class of Algorithm 1 (the inner while loop) with the facility-location f.
 *   J = open blocks, R = unassigned samples.
 *   loop while R and J are non-empty:
 *       j* = block of J with the least f (lowest index among equals)
 *       if block j* can still take a sample (count below its quota):
 *            v* = GreedyStep: the unassigned v maximising f(A_j* u {v})
 *            A_j* += v*,  R -= v*
 *       else J -= j*
 * Outputs (all optional except assign):
 *   assign[n]  block of every sample, -1 if it was left over (sum cap < n)
 *   order[n]   step index at which the sample was taken, -1 if never
 *   obj[K]     f(A_k) re-evaluated from the definition at the end
 *   fsum[K]    the running sums of accepted gains (must equal obj)
 *   tr_block/tr_elem/tr_gain[steps]  the trace: block, element, gain per step
 * Returns the number of steps taken, or -1 on a bad argument.
 */
int64_t oracle_partition_class(const float *S, int64_t lds, int64_t n, int K, const int64_t *cap,
                               int32_t *assign, int32_t *order, double *obj, double *fsum,
                               int32_t *tr_block, int32_t *tr_elem, double *tr_gain)
{
    if (!S || !cap || !assign || n < 0 || K < 1 || lds < n)
        return -1;
    int64_t total_cap = 0;
    for (int k = 0; k < K; ++k) {
        if (cap[k] < 0)
            return -1;
        total_cap += cap[k];
    }
    if (total_cap > n)
        return -1;

    double *cov = (double *)calloc((size_t)K * (size_t)(n > 0 ? n : 1), sizeof(double));
    double *f = (double *)calloc((size_t)K, sizeof(double));
    int64_t *cnt = (int64_t *)calloc((size_t)K, sizeof(int64_t));
    char *open = (char *)malloc((size_t)K);
    if (!cov || !f || !cnt || !open) {
        free(cov); free(f); free(cnt); free(open);
        return -1;
    }
    memset(open, 1, (size_t)K);
    for (int64_t v = 0; v < n; ++v) {
        assign[v] = -1;
        if (order)
            order[v] = -1;
    }
    int64_t remaining = n;  /* |R| */
    int n_open = K;         /* |J| */
    int64_t t = 0;

    while (remaining > 0 && n_open > 0) {
        int js = -1;
        for (int k = 0; k < K; ++k) {
            if (!open[k])
                continue;
            if (js < 0 || f[k] < f[js])
                js = k;
        }
        if (cnt[js] < cap[js]) {
            const double *cj = cov + (size_t)js * (size_t)n;
            int64_t vs = -1;
            double best = 0.0;
            for (int64_t v = 0; v < n; ++v) {
                if (assign[v] >= 0)
                    continue;
                double g = gain_of(S, lds, n, cj, v);
                if (vs < 0 || g > best) {
                    best = g;
                    vs = v;
                }
            }
            assign[vs] = js;
            if (order)
                order[vs] = (int32_t)t;
            if (tr_block) tr_block[t] = js;
            if (tr_elem) tr_elem[t] = (int32_t)vs;
            if (tr_gain) tr_gain[t] = best;
            cnt[js] += 1;
            f[js] += best;
            double *cw = cov + (size_t)js * (size_t)n;
            for (int64_t j = 0; j < n; ++j) {
                double s = (double)S[j * lds + vs];
                if (s > cw[j])
                    cw[j] = s;
            }
            remaining -= 1;
            t += 1;
        } else {
            open[js] = 0;
            n_open -= 1;
        }
    }

    if (fsum)
        for (int k = 0; k < K; ++k)
            fsum[k] = f[k];
    if (obj) {
        int32_t *mem = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
        if (!mem) {
            free(cov); free(f); free(cnt); free(open);
            return -1;
        }
        for (int k = 0; k < K; ++k) {
            int64_t m = 0;
            for (int64_t v = 0; v < n; ++v)
                if (assign[v] == k)
                    mem[m++] = (int32_t)v;
            obj[k] = oracle_f(S, lds, n, mem, m);
        }
        free(mem);
    }
    free(cov); free(f); free(cnt); free(open);
    return t;
}

/*
 * Lock-step referee.  Replays a trace produced elsewhere (order[], assign[])
 * through Algorithm 1's state and, at every step t with check[t] != 0 (or at
 * all steps if check is NULL), asks what the oracle would have done from that
 * very state:
 *   - the block: accepted if it is the oracle's argmin, or its f is within
 *     rel_tol (relative to the larger magnitude) of the oracle's minimum;
 *   - the element: accepted if it is the oracle's argmax, or its oracle gain is
 *     within rel_tol relative of the oracle's best gain.
 * A block that is full, an element already taken, or a gap in order[] is a
 * hard failure.  stats[0]=steps checked, [1]=exact agreements,
 * [2]=accepted near-ties of the block, [3]=accepted near-ties of the element,
 * [4]=violations, [5]=first violating step (-1 if none).
 * worst[0] = largest accepted-or-not relative gap of the element choice,
 * worst[1] = same for the block choice.
 * Returns 0 if there is no violation, 1 if there is, -1 on a malformed trace.
 */
int oracle_lockstep(const float *S, int64_t lds, int64_t n, int K, const int64_t *cap,
                    const int32_t *order, const int32_t *assign, int64_t steps,
                    const uint8_t *check, double rel_tol, int64_t *stats, double *worst)
{
    if (!S || !cap || !order || !assign || !stats || n < 0 || K < 1 || steps < 0 || steps > n)
        return -1;
    int32_t *elem_at = (int32_t *)malloc((size_t)(steps > 0 ? steps : 1) * sizeof(int32_t));
    double *cov = (double *)calloc((size_t)K * (size_t)(n > 0 ? n : 1), sizeof(double));
    double *f = (double *)calloc((size_t)K, sizeof(double));
    int64_t *cnt = (int64_t *)calloc((size_t)K, sizeof(int64_t));
    char *taken = (char *)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!elem_at || !cov || !f || !cnt || !taken) {
        free(elem_at); free(cov); free(f); free(cnt); free(taken);
        return -1;
    }
    int rc = 0;
    for (int64_t t = 0; t < steps; ++t)
        elem_at[t] = -1;
    for (int64_t v = 0; v < n; ++v) {
        int32_t o = order[v];
        if (o < 0) {
            if (assign[v] >= 0) rc = -1;
            continue;
        }
        if (o >= steps || elem_at[o] >= 0 || assign[v] < 0 || assign[v] >= K) {
            rc = -1;
            continue;
        }
        elem_at[o] = (int32_t)v;
    }
    for (int64_t t = 0; t < steps; ++t)
        if (elem_at[t] < 0)
            rc = -1;
    for (int i = 0; i < 6; ++i)
        stats[i] = 0;
    stats[5] = -1;
    if (worst) {
        worst[0] = 0.0;
        worst[1] = 0.0;
    }
    if (rc != 0) {
        free(elem_at); free(cov); free(f); free(cnt); free(taken);
        return -1;
    }

    for (int64_t t = 0; t < steps; ++t) {
        int32_t v_ext = elem_at[t];
        int k_ext = assign[v_ext];
        double *ck = cov + (size_t)k_ext * (size_t)n;
        int violated = 0;
        if (cnt[k_ext] >= cap[k_ext])
            violated = 1; /* over quota: never acceptable */
        double g_ext = gain_of(S, lds, n, ck, v_ext);

        if (!violated && (!check || check[t])) {
            int near_block = 0, near_elem = 0;
            /* block choice */
            int js = -1;
            for (int k = 0; k < K; ++k) {
                if (cnt[k] >= cap[k])
                    continue;
                if (js < 0 || f[k] < f[js])
                    js = k;
            }
            if (js != k_ext) {
                double gap = fabs(f[k_ext] - f[js]);
                double scale = fmax(fabs(f[k_ext]), fabs(f[js]));
                double rel = scale > 0.0 ? gap / scale : 0.0;
                if (worst && rel > worst[1]) worst[1] = rel;
                if (rel <= rel_tol)
                    near_block = 1;
                else
                    violated = 1;
            }
            /* element choice, judged inside the block the trace used */
            int64_t vs = -1;
            double best = 0.0;
            for (int64_t v = 0; v < n; ++v) {
                if (taken[v])
                    continue;
                double g = gain_of(S, lds, n, ck, v);
                if (vs < 0 || g > best) {
                    best = g;
                    vs = v;
                }
            }
            if (vs != v_ext) {
                double rel = best > 0.0 ? (best - g_ext) / best : 0.0;
                if (worst && rel > worst[0]) worst[0] = rel;
                if (rel <= rel_tol)
                    near_elem = 1;
                else
                    violated = 1;
            }
            stats[0] += 1;
            if (!violated) {
                if (!near_block && !near_elem) stats[1] += 1;
                if (near_block) stats[2] += 1;
                if (near_elem) stats[3] += 1;
            }
        }
        if (violated) {
            stats[4] += 1;
            if (stats[5] < 0)
                stats[5] = t;
            rc = 1;
        }
        /* follow the trace */
        taken[v_ext] = 1;
        cnt[k_ext] += 1;
        f[k_ext] += g_ext;
        for (int64_t j = 0; j < n; ++j) {
            double s = (double)S[j * lds + v_ext];
            if (s > ck[j])
                ck[j] = s;
        }
    }
    free(elem_at); free(cov); free(f); free(cnt); free(taken);
    return rc;
}

/*
 * Exhaustive search over every way of giving exactly cap[k] samples to block k
 * (samples beyond sum cap stay unassigned).  For tiny n only.
 * best[0] = max over assignments of sum_k f(A_k); best[1] = max of min_k f(A_k).
 * Returns the number of complete assignments visited, -1 on a bad argument.
 */
struct bf_state {
    const float *S;
    int64_t lds, n;
    int K;
    const int64_t *cap;
    int64_t cnt[8];
    int32_t mem[8][16];
    double best_sum, best_min;
    int64_t visited;
};

static void bf_visit(struct bf_state *st, int64_t v, int64_t left_free)
{
    if (v == st->n) {
        double sum = 0.0, mn = 0.0;
        for (int k = 0; k < st->K; ++k) {
            double fk = oracle_f(st->S, st->lds, st->n, st->mem[k], st->cnt[k]);
            sum += fk;
            if (k == 0 || fk < mn)
                mn = fk;
        }
        if (st->visited == 0 || sum > st->best_sum) st->best_sum = sum;
        if (st->visited == 0 || mn > st->best_min) st->best_min = mn;
        st->visited += 1;
        return;
    }
    for (int k = 0; k < st->K; ++k) {
        if (st->cnt[k] >= st->cap[k])
            continue;
        st->mem[k][st->cnt[k]] = (int32_t)v;
        st->cnt[k] += 1;
        bf_visit(st, v + 1, left_free);
        st->cnt[k] -= 1;
    }
    if (left_free > 0)
        bf_visit(st, v + 1, left_free - 1);
}

int64_t oracle_bruteforce(const float *S, int64_t lds, int64_t n, int K, const int64_t *cap,
                          double *best)
{
    if (!S || !cap || !best || n < 1 || n > 16 || K < 1 || K > 8 || lds < n)
        return -1;
    struct bf_state st;
    memset(&st, 0, sizeof st);
    st.S = S; st.lds = lds; st.n = n; st.K = K; st.cap = cap;
    int64_t total = 0;
    for (int k = 0; k < K; ++k) {
        if (cap[k] < 0 || cap[k] > 16)
            return -1;
        total += cap[k];
    }
    if (total > n)
        return -1;
    bf_visit(&st, 0, n - total);
    best[0] = st.best_sum;
    best[1] = st.best_min;
    return st.visited;
}

/*
 * Whole data set (Algorithm 1, outer loop): split by label keeping the input
 * order inside each class, then per class: similarity, quotas, greedy; finally
 * join the per-class blocks.  labels in [0,L).  r[K] integer capacities >= 1.
 * assign[N], order[N] (step index inside the sample's own class), obj[L*K].
 * Returns 0, -1 on a bad argument.
 */
int oracle_partition_dataset(const void *X, int dtype, int64_t N, int64_t d, int64_t ldx,
                             const int32_t *labels, int L, const int64_t *r, int K, double sigma2,
                             int32_t *assign, int32_t *order, double *obj)
{
    if (!X || !labels || !r || !assign || N < 0 || L < 1 || K < 1 || d < 1 || ldx < d)
        return -1;
    for (int64_t i = 0; i < N; ++i)
        if (labels[i] < 0 || labels[i] >= L)
            return -1;
    size_t esz = dtype == ORACLE_BF16 ? 2 : 4;
    int64_t *cap = (int64_t *)malloc((size_t)K * sizeof(int64_t));
    int32_t *idx = (int32_t *)malloc((size_t)(N > 0 ? N : 1) * sizeof(int32_t));
    if (!cap || !idx) {
        free(cap); free(idx);
        return -1;
    }
    int rc = 0;
    for (int l = 0; l < L && rc == 0; ++l) {
        int64_t nl = 0;
        for (int64_t i = 0; i < N; ++i)
            if (labels[i] == l)
                idx[nl++] = (int32_t)i;
        if (oracle_quota(nl, r, K, cap) != 0) {
            rc = -1;
            break;
        }
        if (nl == 0) {
            if (obj)
                for (int k = 0; k < K; ++k)
                    obj[(size_t)l * K + k] = 0.0;
            continue;
        }
        char *Xl = (char *)malloc((size_t)nl * (size_t)d * esz);
        float *S = (float *)malloc((size_t)nl * (size_t)nl * sizeof(float));
        int32_t *a = (int32_t *)malloc((size_t)nl * sizeof(int32_t));
        int32_t *o = (int32_t *)malloc((size_t)nl * sizeof(int32_t));
        if (!Xl || !S || !a || !o) {
            rc = -1;
        } else {
            for (int64_t i = 0; i < nl; ++i)
                memcpy(Xl + (size_t)i * (size_t)d * esz,
                       (const char *)X + (size_t)idx[i] * (size_t)ldx * esz, (size_t)d * esz);
            if (oracle_similarity(Xl, dtype, nl, d, d, sigma2, NULL, S) != 0)
                rc = -1;
            else if (oracle_partition_class(S, nl, nl, K, cap, a, o,
                                            obj ? obj + (size_t)l * K : NULL, NULL,
                                            NULL, NULL, NULL) < 0)
                rc = -1;
            else
                for (int64_t i = 0; i < nl; ++i) {
                    assign[idx[i]] = a[i];
                    if (order)
                        order[idx[i]] = o[i];
                }
        }
        free(Xl); free(S); free(a); free(o);
    }
    free(cap); free(idx);
    return rc;
}

/* ======================================================================================
 * Graph cut, the paper's second submodular function (Section 4, "Submodular functions"):
 *   f(A) = sum over v in V_l \ A of  sum over v' in A of  sim(v, v').
 * V_l \ A is every class member outside A, samples given to other blocks included.
 * Algorithm 1 is unchanged (argmin-f block, GreedyStep = the unassigned v of largest
 * f(A u {v}) - f(A), lowest index on ties, a block leaves J once its quota is met).
 * f is not monotone: a marginal value can be negative, and the sample with the largest one
 * is still taken, because the quotas have to be met (Algorithm 1 has no sign test).
 * Readings: f(empty) = 0 (empty sum).  oracle_f_gc evaluates the definition with sim used as
 * printed, S[v][a] = sim(v, a) with v outside A and a inside, on any S.  Section 4's similarity is
 * a function of the distance between two samples, hence symmetric; the greedy and its referee
 * below take that as a precondition: they return -2 for an S that is not exactly symmetric, and
 * read sim(v, u) as S[u][v].
 * ====================================================================================== */

/* f(A) from the definition; members[m] lists A. */
double oracle_f_gc(const float *S, int64_t lds, int64_t n, const int32_t *members, int64_t m)
{
    if (m <= 0)
        return 0.0;
    char *in = (char *)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!in)
        return 0.0;
    for (int64_t a = 0; a < m; ++a)
        in[members[a]] = 1;
    double total = 0.0;
    for (int64_t v = 0; v < n; ++v) {
        if (in[v])
            continue;
        for (int64_t a = 0; a < m; ++a)
            total += (double)S[v * lds + members[a]];
    }
    free(in);
    return total;
}

/* 1 if S[i][j] == S[j][i] for all i, j < n, else 0. */
static int is_symmetric(const float *S, int64_t lds, int64_t n)
{
    /* every pair once, walked in 64 x 64 squares so that a 50 000 x 50 000 matrix stays in cache */
    for (int64_t i0 = 0; i0 < n; i0 += 64)
        for (int64_t j0 = i0; j0 < n; j0 += 64)
            for (int64_t i = i0; i < i0 + 64 && i < n; ++i)
                for (int64_t j = (j0 > i ? j0 : i + 1); j < j0 + 64 && j < n; ++j)
                    if (S[i * lds + j] != S[j * lds + i])
                        return 0;
    return 1;
}

/* f(A u {u}) - f(A) for the block whose members are the v with assign[v] == k:
 * u leaves V \ A, so its own terms sum_{a in A} sim(u, a) go, and u enters A, so the
 * terms sum_{v outside A, v != u} sim(v, u) come in.  (tests pin this against the
 * definition above evaluated twice.)  S is symmetric here (checked by the two callers),
 * so sim(v, u) = S[v][u] = S[u][v] and both sums walk row u. */
static double gain_of_gc(const float *S, int64_t lds, int64_t n, const int32_t *assign, int k, int64_t u)
{
    double g = 0.0;
    for (int64_t v = 0; v < n; ++v) {
        if (v == u)
            continue;
        if (assign[v] == k)
            g -= (double)S[u * lds + v];
        else
            g += (double)S[u * lds + v];
    }
    return g;
}

/* Same contract as oracle_partition_class, with the graph-cut f. */
int64_t oracle_partition_class_gc(const float *S, int64_t lds, int64_t n, int K, const int64_t *cap,
                                  int32_t *assign, int32_t *order, double *obj, double *fsum,
                                  int32_t *tr_block, int32_t *tr_elem, double *tr_gain)
{
    if (!S || !cap || !assign || n < 0 || K < 1 || lds < n)
        return -1;
    int64_t total_cap = 0;
    for (int k = 0; k < K; ++k) {
        if (cap[k] < 0)
            return -1;
        total_cap += cap[k];
    }
    if (total_cap > n)
        return -1;
    if (!is_symmetric(S, lds, n))
        return -2;
    double *f = (double *)calloc((size_t)K, sizeof(double));
    int64_t *cnt = (int64_t *)calloc((size_t)K, sizeof(int64_t));
    char *open = (char *)malloc((size_t)K);
    if (!f || !cnt || !open) {
        free(f); free(cnt); free(open);
        return -1;
    }
    memset(open, 1, (size_t)K);
    for (int64_t v = 0; v < n; ++v) {
        assign[v] = -1;
        if (order)
            order[v] = -1;
    }
    int64_t remaining = n;
    int n_open = K;
    int64_t t = 0;
    while (remaining > 0 && n_open > 0) {
        int js = -1;
        for (int k = 0; k < K; ++k) {
            if (!open[k])
                continue;
            if (js < 0 || f[k] < f[js])
                js = k;
        }
        if (cnt[js] < cap[js]) {
            int64_t vs = -1;
            double best = 0.0;
            for (int64_t v = 0; v < n; ++v) {
                if (assign[v] >= 0)
                    continue;
                double g = gain_of_gc(S, lds, n, assign, js, v);
                if (vs < 0 || g > best) {
                    best = g;
                    vs = v;
                }
            }
            assign[vs] = js;
            if (order)
                order[vs] = (int32_t)t;
            if (tr_block) tr_block[t] = js;
            if (tr_elem) tr_elem[t] = (int32_t)vs;
            if (tr_gain) tr_gain[t] = best;
            cnt[js] += 1;
            f[js] += best;
            remaining -= 1;
            t += 1;
        } else {
            open[js] = 0;
            n_open -= 1;
        }
    }
    if (fsum)
        for (int k = 0; k < K; ++k)
            fsum[k] = f[k];
    if (obj) {
        int32_t *mem = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
        if (!mem) {
            free(f); free(cnt); free(open);
            return -1;
        }
        for (int k = 0; k < K; ++k) {
            int64_t m = 0;
            for (int64_t v = 0; v < n; ++v)
                if (assign[v] == k)
                    mem[m++] = (int32_t)v;
            obj[k] = oracle_f_gc(S, lds, n, mem, m);
        }
        free(mem);
    }
    free(f); free(cnt); free(open);
    return t;
}

/* Lock-step referee for the graph-cut f: same contract and statistics as oracle_lockstep.
 * Marginal values can be negative or zero, so the element gap is taken relative to the
 * larger magnitude of the two values compared.  A marginal value here is a difference of two
 * sums of similarities, so when the trace was made on a slightly different S (entries off by
 * e each) its values are off by up to n*e however small they are themselves: abs_tol (>= 0,
 * 0 for a trace made on this very S) widens the element window by that absolute amount: a step
 * whose sample is not the referee's is accepted when the referee's best marginal value exceeds
 * the marginal value of the sample taken by at most abs_tol.  Returns -2 for an S that is not
 * symmetric. */
int oracle_lockstep_gc(const float *S, int64_t lds, int64_t n, int K, const int64_t *cap,
                       const int32_t *order, const int32_t *assign, int64_t steps,
                       const uint8_t *check, double rel_tol, double abs_tol, int64_t *stats, double *worst)
{
    if (!S || !cap || !order || !assign || !stats || n < 0 || K < 1 || steps < 0 || steps > n)
        return -1;
    if (!is_symmetric(S, lds, n))
        return -2;
    int32_t *elem_at = (int32_t *)malloc((size_t)(steps > 0 ? steps : 1) * sizeof(int32_t));
    int32_t *state = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));   /* block so far, -1 */
    double *f = (double *)calloc((size_t)K, sizeof(double));
    int64_t *cnt = (int64_t *)calloc((size_t)K, sizeof(int64_t));
    if (!elem_at || !state || !f || !cnt) {
        free(elem_at); free(state); free(f); free(cnt);
        return -1;
    }
    int rc = 0;
    for (int64_t t = 0; t < steps; ++t)
        elem_at[t] = -1;
    for (int64_t v = 0; v < n; ++v) {
        state[v] = -1;
        int32_t o = order[v];
        if (o < 0) {
            if (assign[v] >= 0) rc = -1;
            continue;
        }
        if (o >= steps || elem_at[o] >= 0 || assign[v] < 0 || assign[v] >= K) {
            rc = -1;
            continue;
        }
        elem_at[o] = (int32_t)v;
    }
    for (int64_t t = 0; t < steps; ++t)
        if (elem_at[t] < 0)
            rc = -1;
    for (int i = 0; i < 6; ++i)
        stats[i] = 0;
    stats[5] = -1;
    if (worst) {
        worst[0] = 0.0;
        worst[1] = 0.0;
    }
    if (rc != 0) {
        free(elem_at); free(state); free(f); free(cnt);
        return -1;
    }
    for (int64_t t = 0; t < steps; ++t) {
        int32_t v_ext = elem_at[t];
        int k_ext = assign[v_ext];
        int violated = 0;
        if (cnt[k_ext] >= cap[k_ext])
            violated = 1;
        double g_ext = gain_of_gc(S, lds, n, state, k_ext, v_ext);
        if (!violated && (!check || check[t])) {
            int near_block = 0, near_elem = 0;
            int js = -1;
            for (int k = 0; k < K; ++k) {
                if (cnt[k] >= cap[k])
                    continue;
                if (js < 0 || f[k] < f[js])
                    js = k;
            }
            if (js != k_ext) {
                double gap = fabs(f[k_ext] - f[js]);
                double scale = fmax(fabs(f[k_ext]), fabs(f[js]));
                double rel = scale > 0.0 ? gap / scale : 0.0;
                if (worst && rel > worst[1]) worst[1] = rel;
                if (rel <= rel_tol)
                    near_block = 1;
                else
                    violated = 1;
            }
            int64_t vs = -1;
            double best = 0.0;
            for (int64_t v = 0; v < n; ++v) {
                if (state[v] >= 0)
                    continue;
                double g = gain_of_gc(S, lds, n, state, k_ext, v);
                if (vs < 0 || g > best) {
                    best = g;
                    vs = v;
                }
            }
            if (vs != v_ext) {
                double scale = fmax(fabs(best), fabs(g_ext));
                double rel = scale > 0.0 ? (best - g_ext) / scale : 0.0;
                if (worst && rel > worst[0]) worst[0] = rel;
                if (rel <= rel_tol || best - g_ext <= abs_tol)
                    near_elem = 1;
                else
                    violated = 1;
            }
            stats[0] += 1;
            if (!violated) {
                if (!near_block && !near_elem) stats[1] += 1;
                if (near_block) stats[2] += 1;
                if (near_elem) stats[3] += 1;
            }
        }
        if (violated) {
            stats[4] += 1;
            if (stats[5] < 0)
                stats[5] = t;
            rc = 1;
        }
        state[v_ext] = k_ext;
        cnt[k_ext] += 1;
        f[k_ext] += g_ext;
    }
    free(elem_at); free(state); free(f); free(cnt);
    return rc;
}

/* ======================================================================================
 * Bandwidth of the Gaussian kernel (Section 4, "Submodular functions"): the paper sets
 *   sigma = sum over v, v' in V of ||v - v'||_2  /  n^2,
 * the mean L2 distance over all n^2 ordered pairs of the set the similarity is built on,
 * the n pairs of a sample with itself (distance 0) included in the count.
 * Readings: n = |V| (the formula's n is the size of the set summed over, not the worker
 * index n of Algorithm 1); the distance is not squared; V is whatever row set the caller
 * passes (the whole data set, or one class).
 * Every ordered pair is computed on its own from coordinate differences.
 * Returns sigma, or -1 on a bad argument; 0 for an empty set.
 * ====================================================================================== */
double oracle_bandwidth(const void *X, int dtype, int64_t n, int64_t d, int64_t ldx)
{
    if (n < 0 || d < 1 || ldx < d || (n > 0 && !X))
        return -1.0;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return -1.0;
    if (n == 0)
        return 0.0;
    double total = 0.0;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double dist2 = 0.0;
            for (int64_t t = 0; t < d; ++t) {
                double diff = elem_as_double(X, dtype, i * ldx + t) - elem_as_double(X, dtype, j * ldx + t);
                dist2 += diff * diff;
            }
            total += sqrt(dist2);
        }
    return total / ((double)n * (double)n);
}

/* ======================================================================================
 * Hand-off to Algorithm 2 (its initialisation line: worker i imports its subset A_i, and
 * runs with a batch size set from the capacity ratios).
 * ====================================================================================== */

/* Worker k's list = the samples with assign == k in ascending order; the lists are laid
 * end to end in index[], offset[k] .. offset[k+1] delimiting list k (offset has K+1 entries).
 * Samples with assign == -1 belong to no list.  Returns 0, or -1 on a bad argument or an
 * assignment outside [-1, K). */
int oracle_worker_shards(const int32_t *assign, int64_t N, int K, int32_t *index, int64_t *offset)
{
    if (N < 0 || K < 1 || !offset || (N > 0 && (!assign || !index)))
        return -1;
    for (int64_t i = 0; i < N; ++i)
        if (assign[i] < -1 || assign[i] >= K)
            return -1;
    int64_t at = 0;
    for (int k = 0; k < K; ++k) {
        offset[k] = at;
        for (int64_t i = 0; i < N; ++i)
            if (assign[i] == k)
                index[at++] = (int32_t)i;
    }
    offset[K] = at;
    return 0;
}

/* Batch sizes.  The text after Algorithm 2 says a worker's batch size, like its shard, is
 * proportional to its processing speed, so that all workers finish their local iterations in
 * the same time; the algorithm box prints the factor as r_1 / r_i, which would do the
 * opposite.  Reading taken: batch_i = B r_i / r_1 (worker 1 runs B), to the nearest integer
 * with halves rounded up, and never less than 1. */
int oracle_batch_sizes(int64_t B, const int64_t *r, int K, int64_t *batch)
{
    if (B < 1 || K < 1 || !r || !batch)
        return -1;
    for (int k = 0; k < K; ++k)
        if (r[k] < 1)
            return -1;
    for (int k = 0; k < K; ++k) {
        double exact = (double)B * (double)r[k] / (double)r[0];
        int64_t q = (int64_t)floor(exact + 0.5);
        batch[k] = q < 1 ? 1 : q;
    }
    return 0;
}
