/*
 * CPU oracle for the one-device TA-MoE hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision restatement of what the paper
 * "TA-MoE: Topology-Aware Large Scale Mixture-of-Expert Training" defines for
 * one device i of an expert-parallel MoE layer.  Scalar loops, no BLAS, no
 * blocking, no fusion.  It exists so that the HIP library can be checked
 * against something independent: it shares no source, header, table or helper
 * with the HIP path and nothing in the product may call it.  Only the tests,
 * the smoke check and the benchmark's "cpu_baseline" leg use it.
 *
 * Notation (Section 3.1 "MoE Model Structure"): N experts, P devices,
 * E = N/P experts per device (device j holds experts jE .. (j+1)E-1), S tokens
 * on this device, k experts selected per token, hidden size d.  c[e] is the
 * number of (token, choice) pairs of this device that selected expert e,
 * G(x) the softmax gate vector, m[e] the mean of G(x)[e] over the S tokens.
 *
 * The only parallelism is an OpenMP "parallel for" over tokens on loops whose
 * iterations are independent (used by the benchmark's all-cores timing); the
 * arithmetic of each iteration is unchanged by it.
 *
 * Every function below is pinned by tests/test_oracle_*.py against closed
 * forms, invariants, brute force, library routines and the worked numbers of
 * the paper's Table 1.  Not pinned ("parity unpinned"): none of the exported
 * functions, but two of them restate a reading rather than a definition
 * of the paper, and their pins are the paper's single example plus invariants:
 * the merge of asymmetric trees in orc_tree_levels and the arc choice of
 * orc_ring_table.  Global (cross-device) capacity is not implemented.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_F32 0
#define ORC_BF16 1
#define ORC_F16 2

static int g_threads = 1;

void orc_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_num_procs();
#else
    return 1;
#endif
}

/* ---- storage types ------------------------------------------------------ */

static size_t elem_size(int dtype) { return dtype == ORC_F32 ? 4u : 2u; }

/* exact value of an IEEE half-precision bit pattern (1 sign, 5 exponent, 10 fraction bits) */
static double half_value(uint16_t h)
{
    int sign = h >> 15, ex = (h >> 10) & 31, frac = h & 1023;
    double v;
    if (ex == 31)
        v = frac ? NAN : INFINITY;
    else if (ex == 0)
        v = ldexp((double)frac, -24);               /* subnormal: frac * 2^-24 */
    else
        v = ldexp(1.0 + (double)frac / 1024.0, ex - 15);
    return sign ? -v : v;
}

/* nearest half-precision value (11 significand bits), ties to even, straight from double */
static uint16_t round_to_f16(double v)
{
    uint16_t sign = (uint16_t)(signbit(v) ? 0x8000u : 0u);
    if (isnan(v))
        return (uint16_t)0x7E00u;
    double a = fabs(v);
    if (a == 0.0)
        return sign;
    if (isinf(v))
        return (uint16_t)(sign | 0x7C00u);
    int ex;
    (void)frexp(a, &ex);
    int e = ex - 1;                 /* floor(log2 a) */
    if (e < -14)
        e = -14;                    /* subnormal range shares the spacing of the smallest normal */
    double ulp = ldexp(1.0, e - 10);
    double q = nearbyint(a / ulp);  /* to nearest, ties to even; q <= 2048 */
    double r = q * ulp;
    if (r >= 65520.0)               /* halfway between the largest finite value and 2^16 rounds to infinity */
        return (uint16_t)(sign | 0x7C00u);
    if (r < ldexp(1.0, -14))        /* subnormal (or zero): the fraction field is r / 2^-24 */
        return (uint16_t)(sign | (uint16_t)(r / ldexp(1.0, -24)));
    int re;
    double f = frexp(r, &re);       /* r = f * 2^re, f in [0.5, 1) */
    int biased = re - 1 + 15;
    int frac = (int)((f * 2.0 - 1.0) * 1024.0);
    return (uint16_t)(sign | (uint16_t)(biased << 10) | (uint16_t)frac);
}

/* exact value of element i of a float32 / bfloat16 / half-precision buffer */
static double load_elem(const void *buf, int dtype, int64_t i)
{
    if (dtype == ORC_F32)
        return (double)((const float *)buf)[i];
    if (dtype == ORC_F16)
        return half_value(((const uint16_t *)buf)[i]);
    uint32_t bits = (uint32_t)((const uint16_t *)buf)[i] << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

/* nearest bfloat16 (8 significand bits), ties to even, straight from double:
 * no intermediate float rounding */
static uint16_t round_to_bf16(double v)
{
    if (v == 0.0 || isnan(v)) {
        uint16_t z = (uint16_t)(signbit(v) ? 0x8000u : 0u);
        return isnan(v) ? (uint16_t)0x7FC0u : z;
    }
    if (isinf(v))
        return (uint16_t)(v > 0 ? 0x7F80u : 0xFF80u);
    int ex;
    (void)frexp(fabs(v), &ex); /* |v| = f * 2^ex, f in [0.5, 1) => |v| in [2^(ex-1), 2^ex) */
    int e = ex - 1;            /* floor(log2 |v|) */
    if (e < -126)
        e = -126;              /* subnormal range shares the spacing of the smallest normal */
    double ulp = ldexp(1.0, e - 7);
    double q = nearbyint(v / ulp); /* default rounding mode: to nearest, ties to even */
    double r = q * ulp;            /* representable in bfloat16 unless it overflowed */
    float f = (float)r;            /* exact */
    if (isinf(f) || fabs(r) >= ldexp(1.0, 128))
        return (uint16_t)(v > 0 ? 0x7F80u : 0xFF80u);
    uint32_t bits;
    memcpy(&bits, &f, 4);
    return (uint16_t)(bits >> 16);
}

static void store_elem(void *buf, int dtype, int64_t i, double v)
{
    if (dtype == ORC_F32)
        ((float *)buf)[i] = (float)v;
    else if (dtype == ORC_F16)
        ((uint16_t *)buf)[i] = round_to_f16(v);
    else
        ((uint16_t *)buf)[i] = round_to_bf16(v);
}

/* exported so the roundings and the half-precision decoding can be pinned by tests */
uint16_t orc_round_to_bf16(double v) { return round_to_bf16(v); }
uint16_t orc_round_to_f16(double v) { return round_to_f16(v); }
double orc_half_value(uint16_t h) { return half_value(h); }

/* ---- setup: communication model, target pattern, penalty ----------------- */

/*
 * Per-level smoothing of a profiled inverse-bandwidth table (Section 4.2
 * "Model Optimization", the alpha_l / beta_l definition and the hierarchical
 * matrix that follows it).  level[i*P+j] labels the tree level of the pair
 * (i, j).  beta_l is the mean of beta_ij over the pairs i < j on level l (the
 * paper's printed pair count only equals the real one on the deepest level;
 * the mean over the actual pairs is what "eliminate the noise of profiling"
 * needs).  A level that occurs only on the diagonal (self transfers) has no
 * pair i < j; its value is the mean of those diagonal entries.
 * beta_hat_ij = beta_{level(i,j)}.  Returns 0, or 1 on a bad level label.
 */
int orc_smooth_beta(const double *beta, const int32_t *level, int P, double *beta_hat)
{
    int n_levels = 0;
    for (int q = 0; q < P * P; ++q) {
        if (level[q] < 0)
            return 1;
        if (level[q] + 1 > n_levels)
            n_levels = level[q] + 1;
    }
    double *sum = (double *)calloc((size_t)n_levels, sizeof(double));
    double *cnt = (double *)calloc((size_t)n_levels, sizeof(double));
    double *dsum = (double *)calloc((size_t)n_levels, sizeof(double));
    double *dcnt = (double *)calloc((size_t)n_levels, sizeof(double));
    for (int i = 0; i < P; ++i) {
        for (int j = i + 1; j < P; ++j) {
            int l = level[i * P + j];
            sum[l] += beta[i * P + j];
            cnt[l] += 1.0;
        }
        int l = level[i * P + i];
        dsum[l] += beta[i * P + i];
        dcnt[l] += 1.0;
    }
    for (int i = 0; i < P; ++i) {
        for (int j = 0; j < P; ++j) {
            int l = level[i * P + j];
            beta_hat[i * P + j] = cnt[l] > 0.0 ? sum[l] / cnt[l] : dsum[l] / dcnt[l];
        }
    }
    free(sum); free(cnt); free(dsum); free(dcnt);
    return 0;
}

/*
 * Target dispatch pattern of device `rank` (Section 4.2, the closed-form
 * solution of the min-max problem after the latency term is dropped):
 *   c_hat[e] = k*S / ( E * (sum_j 1/beta_hat[rank][j]) * beta_hat[rank][floor(e/E)] )
 * The sum runs over all P devices, j = rank included.
 */
void orc_target_pattern(const double *beta_hat, int P, int N, int rank, int k, int64_t S,
                        double *c_hat)
{
    int E = N / P;
    const double *row = beta_hat + (size_t)rank * P;
    double Z = 0.0;
    for (int j = 0; j < P; ++j)
        Z += 1.0 / row[j];
    for (int e = 0; e < N; ++e)
        c_hat[e] = (double)k * (double)S / ((double)E * Z * row[e / E]);
}

/* Penalty weights (Section 4.3 "Routing Strategy"): p = Norm(1 / c_hat) with Norm = divide
 * by the sum, so that sum_e p[e] = 1 (the reading under which the N*P factor of the loss
 * keeps the magnitude of the loss: homogeneous network => N * p[e] = 1). */
void orc_penalty(const double *c_hat, int N, double *p)
{
    double tot = 0.0;
    for (int e = 0; e < N; ++e)
        tot += 1.0 / c_hat[e];
    for (int e = 0; e < N; ++e)
        p[e] = (1.0 / c_hat[e]) / tot;
}

/*
 * Softmax-type Norm of the penalty (Section 4.3, the sentence after the penalty
 * equation: normalisations that enlarge the penalty of slow transfers, such as
 * softmax, are admissible too).  The paper gives no scale for the softmax
 * argument; here it is explicit: r[e] = (1/c_hat[e]) / mean_e'(1/c_hat[e'])
 * (the inverse pattern in units of its mean), p[e] = exp(tau*r[e]) / sum_e'
 * exp(tau*r[e']).  tau = 0 gives the uniform weight 1/N.
 */
void orc_penalty_softmax(const double *c_hat, int N, double tau, double *p)
{
    double tot = 0.0;
    for (int e = 0; e < N; ++e)
        tot += 1.0 / c_hat[e];
    double mean = tot / (double)N;
    double zmax = -INFINITY;
    for (int e = 0; e < N; ++e) {
        p[e] = tau * ((1.0 / c_hat[e]) / mean);
        if (p[e] > zmax)
            zmax = p[e];
    }
    double den = 0.0;
    for (int e = 0; e < N; ++e) {
        p[e] = exp(p[e] - zmax);
        den += p[e];
    }
    for (int e = 0; e < N; ++e)
        p[e] /= den;
}

/*
 * Local capacity per expert (Section 3.1, last paragraph, and Section 4.3,
 * the paragraph on DeepSpeed-MoE): mode 0 is the uniform capacity at the
 * load-balanced target, ceil(cf * k*S/N); mode 1 makes it proportional to
 * the target pattern, ceil(cf * c_hat[e]).  A product that is an integer up
 * to 1e-9 is taken as that integer.
 */
void orc_capacity(const double *c_hat, int N, int k, int64_t S, double cf, int mode, int32_t *cap)
{
    for (int e = 0; e < N; ++e) {
        double v = mode == 0 ? cf * (double)k * (double)S / (double)N : cf * c_hat[e];
        cap[e] = (int32_t)ceil(v - 1e-9);
    }
}

/*
 * Value of the exchange objective (Section 4.1 "Communication Model"): the slowest of the
 * P*P peer deliveries, max_{i,j} ( alpha_ij + beta_ij * sum_{e on device j} c[i][e] * bytes ),
 * bytes = d*b per token row.  alpha may be NULL (zero latency).  c is [P][N].
 */
double orc_exchange_cost(const double *alpha, const double *beta, const double *c, int P, int N,
                         double bytes_per_row)
{
    int E = N / P;
    double worst = -INFINITY;
    for (int i = 0; i < P; ++i) {
        for (int j = 0; j < P; ++j) {
            double rows = 0.0;
            for (int e = E * j; e <= E * (j + 1) - 1; ++e)
                rows += c[(size_t)i * N + e];
            double t = (alpha ? alpha[i * P + j] : 0.0) + beta[i * P + j] * rows * bytes_per_row;
            if (t > worst)
                worst = t;
        }
    }
    return worst;
}

/* ---- topology front-end (host-side setup, Sections 3.2 and 4.2) ---------- */

/*
 * Target pattern with the latency term kept: the row problem of Section 4.1 / 4.2 for one
 * sender,  min over v >= 0 with sum_j v[j] = k*S of  max_j ( alpha[j] + beta[j] * bytes * v[j] ),
 * v[j] = rows sent to device j, shared equally by the E experts of the device.  The optimum
 * fills the links up to a common completion time T: v[j] = max(0, (T - alpha[j]) / (beta[j] *
 * bytes)); a link whose latency alone exceeds T carries nothing.  T is found by bisection on the
 * monotone function sum_j v[j](T) - k*S.  With alpha == NULL (or all zero) this is the closed form
 * of Section 4.2.  The column constraint (every expert receives k*S/E rows in total) is not
 * imposed, exactly as in the closed form, where it holds by the symmetry of the table.
 * Returns T.
 */
double orc_minmax_pattern(const double *alpha, const double *beta, int P, int N, int k, int64_t S,
                          double bytes, double *c_hat)
{
    int E = N / P;
    double total = (double)k * (double)S;
    double lo = INFINITY, hi = -INFINITY;
    for (int j = 0; j < P; ++j) {
        double a = alpha ? alpha[j] : 0.0;
        if (a < lo)
            lo = a;
        if (a + beta[j] * bytes * total > hi)
            hi = a + beta[j] * bytes * total;
    }
    for (int it = 0; it < 400; ++it) {
        double T = 0.5 * (lo + hi);
        double rows = 0.0;
        for (int j = 0; j < P; ++j) {
            double a = alpha ? alpha[j] : 0.0;
            if (T > a)
                rows += (T - a) / (beta[j] * bytes);
        }
        if (rows < total)
            lo = T;
        else
            hi = T;
    }
    double T = 0.5 * (lo + hi);
    for (int e = 0; e < N; ++e) {
        int j = e / E;
        double a = alpha ? alpha[j] : 0.0;
        double v = T > a ? (T - a) / (beta[j] * bytes) : 0.0;
        c_hat[e] = v / (double)E;
    }
    return T;
}

/*
 * Pairwise tables of a ring (Section 3.2: adjacent devices are joined by links whose bandwidths
 * may differ; other pairs hop through the devices between them and the slowest link on the way
 * dominates).  link q joins devices q and (q+1) mod P.  For a pair the two arcs are compared:
 * the arc with the smaller bottleneck max(beta of its links) is taken, on a tie the one with
 * fewer hops, then the ascending one.  beta[i][j] = that bottleneck, alpha[i][j] = sum of the
 * arc's link latencies, level[i][j] = its hop count; the diagonal takes self_beta, self_alpha
 * and level 0.  alpha_link and alpha may be NULL.
 */
void orc_ring_table(const double *beta_link, const double *alpha_link, int P, double self_beta,
                    double self_alpha, double *beta, double *alpha, int32_t *level)
{
    for (int i = 0; i < P; ++i) {
        for (int j = 0; j < P; ++j) {
            if (i == j) {
                beta[i * P + j] = self_beta;
                if (alpha)
                    alpha[i * P + j] = self_alpha;
                level[i * P + j] = 0;
                continue;
            }
            double b_up = 0.0, a_up = 0.0, b_dn = 0.0, a_dn = 0.0;
            int h_up = 0, h_dn = 0;
            for (int q = i; q != j; q = (q + 1) % P) {            /* ascending arc: links i .. j-1 */
                if (beta_link[q] > b_up)
                    b_up = beta_link[q];
                a_up += alpha_link ? alpha_link[q] : 0.0;
                h_up += 1;
            }
            for (int q = j; q != i; q = (q + 1) % P) {            /* the other way round: links j .. i-1 */
                if (beta_link[q] > b_dn)
                    b_dn = beta_link[q];
                a_dn += alpha_link ? alpha_link[q] : 0.0;
                h_dn += 1;
            }
            int up = b_up < b_dn || (b_up == b_dn && h_up <= h_dn);
            beta[i * P + j] = up ? b_up : b_dn;
            if (alpha)
                alpha[i * P + j] = up ? a_up : a_dn;
            level[i * P + j] = up ? h_up : h_dn;
        }
    }
}

/*
 * Tree topologies in the nested-list notation of Section 3.2 (elements of one sub-list hang off
 * one switch).  An integer n is a switch with n devices; a list is a switch that joins its
 * elements.  "[2,2]" is the two-layer symmetric tree of the paper's figure, "[[2,2],[2]]" its
 * three-layer asymmetric one.  Devices are numbered from left to right.
 *
 * Nodes live in flat arrays; a list's children are chained through `next`.
 */
#define ORC_MAX_NODES 4096
typedef struct {
    int n_dev[ORC_MAX_NODES];   /* > 0: a switch with that many devices; 0: a list */
    int base[ORC_MAX_NODES];    /* device switch: number of its first device in the tree as given */
    int seen;                   /* devices read so far */
    int first[ORC_MAX_NODES];   /* first child of a list, -1 if none */
    int next[ORC_MAX_NODES];    /* next sibling, -1 at the end */
    int used;
    const char *s;              /* parse position */
    int bad;
} orc_tree;

static void skip_blank(orc_tree *t)
{
    while (*t->s == ' ' || *t->s == '\t')
        t->s++;
}

static int parse_element(orc_tree *t)
{
    skip_blank(t);
    if (t->used >= ORC_MAX_NODES) {
        t->bad = 1;
        return -1;
    }
    int me = t->used++;
    t->first[me] = -1;
    t->next[me] = -1;
    t->n_dev[me] = 0;
    if (*t->s >= '0' && *t->s <= '9') {
        long v = 0;
        while (*t->s >= '0' && *t->s <= '9' && v < 100000)
            v = v * 10 + (*t->s++ - '0');
        if (v <= 0 || v >= 100000)
            t->bad = 1;
        t->n_dev[me] = (int)v;
        t->base[me] = t->seen;
        t->seen += (int)v;
        return me;
    }
    if (*t->s != '[') {
        t->bad = 1;
        return me;
    }
    t->s++;
    int last = -1;
    for (;;) {
        int c = parse_element(t);
        if (t->bad)
            return me;
        if (last < 0)
            t->first[me] = c;
        else
            t->next[last] = c;
        last = c;
        skip_blank(t);
        if (*t->s == ',') {
            t->s++;
            continue;
        }
        if (*t->s == ']') {
            t->s++;
            return me;
        }
        t->bad = 1;
        return me;
    }
}

static int tree_height(const orc_tree *t, int v)
{
    if (t->n_dev[v] > 0)
        return 1;
    int h = 0;
    for (int c = t->first[v]; c >= 0; c = t->next[c]) {
        int hc = tree_height(t, c);
        if (hc > h)
            h = hc;
    }
    return h + 1;
}

static int child_count(const orc_tree *t, int v)
{
    int n = 0;
    for (int c = t->first[v]; c >= 0; c = t->next[c])
        n++;
    return n;
}

/*
 * Merge of an asymmetric tree (Section 4.2, last paragraph: for fairness among the experts the
 * separate nodes are merged into the close symmetric sub-trees; [[2,2],[2]] becomes [[2,2,2]]).
 * The paper gives that one example and the aim: a symmetric tree, on which the second constraint of
 * Section 4.1 (every expert receives k*S/E rows) holds for the closed-form pattern again.
 * Reading taken here, one pass from the leaves up; at a list whose elements are all lists:
 *   - the reference size is the largest member count among the elements as they stand when the list
 *     is reached; elements of that size are the full sub-trees, smaller ones the separate nodes;
 *   - the separate nodes are taken from left to right; each hands all its members to one full
 *     sub-tree of its own height and disappears.  Of the candidates it takes the one that has been
 *     given the fewest members so far, then the one nearest to it in the list, then the left one;
 *   - nothing is looked at twice: the reference and the set of full sub-trees stay what they were.
 * Spreading the members evenly makes the list symmetric whenever the separate nodes can be shared
 * out equally; when they cannot ([[2,2],[2,2],[2]] -> [[2,2],[2,2,2]]) the tree stays asymmetric and
 * keeps its layers rather than collapsing into one switch.
 */
typedef struct {
    int taken, dist, pos;                 /* order of preference among the full sub-trees */
} orc_merge_key;

static int key_before(orc_merge_key a, orc_merge_key b)
{
    if (a.taken != b.taken)
        return a.taken < b.taken;
    if (a.dist != b.dist)
        return a.dist < b.dist;
    return a.pos < b.pos;
}

static void merge_list(orc_tree *t, int v)
{
    int kids[512], size0[512], high[512], taken[512], gone[512];
    int n = 0, ref = 0;
    for (int c = t->first[v]; c >= 0; c = t->next[c]) {
        if (t->n_dev[c] > 0 || n >= 512)
            return;                       /* a device switch among the elements: nothing to merge */
        kids[n++] = c;
    }
    for (int i = 0; i < n; ++i) {
        size0[i] = child_count(t, kids[i]);
        high[i] = tree_height(t, kids[i]);
        taken[i] = 0;
        gone[i] = 0;
        if (size0[i] > ref)
            ref = size0[i];
    }
    for (int i = 0; i < n; ++i) {
        if (size0[i] == ref)
            continue;
        int target = -1;
        orc_merge_key best = {0, 0, 0};
        for (int j = 0; j < n; ++j) {
            if (size0[j] != ref || high[j] != high[i])
                continue;
            orc_merge_key key = {taken[j], j > i ? j - i : i - j, j};
            if (target < 0 || key_before(key, best)) {
                target = j;
                best = key;
            }
        }
        if (target < 0)
            continue;
        int tail = t->first[kids[target]];
        while (t->next[tail] >= 0)
            tail = t->next[tail];
        t->next[tail] = t->first[kids[i]];     /* members go to the end of the target's list */
        t->first[kids[i]] = -1;
        taken[target] += size0[i];
        gone[i] = 1;
    }
    int last = -1;
    t->first[v] = -1;
    for (int i = 0; i < n; ++i) {
        if (gone[i])
            continue;
        if (last < 0)
            t->first[v] = kids[i];
        else
            t->next[last] = kids[i];
        t->next[kids[i]] = -1;
        last = kids[i];
    }
}

static void merge_tree(orc_tree *t, int v)
{
    if (t->n_dev[v] > 0)
        return;
    for (int c = t->first[v]; c >= 0; c = t->next[c])
        merge_tree(t, c);
    merge_list(t, v);
}

static int count_devices(const orc_tree *t, int v)
{
    if (t->n_dev[v] > 0)
        return t->n_dev[v];
    int n = 0;
    for (int c = t->first[v]; c >= 0; c = t->next[c])
        n += count_devices(t, c);
    return n;
}

/* numbers (as given) of the devices below v, left to right in the tree as it stands; returns how many */
static int devices_below(const orc_tree *t, int v, int32_t *out)
{
    if (t->n_dev[v] > 0) {
        for (int q = 0; q < t->n_dev[v]; ++q)
            out[q] = t->base[v] + q;
        return t->n_dev[v];
    }
    int n = 0;
    for (int c = t->first[v]; c >= 0; c = t->next[c])
        n += devices_below(t, c, out + n);
    return n;
}

/* level labels of all pairs with both devices below v; dev: room for the device numbers below v */
static void label_pairs(const orc_tree *t, int v, int P, int32_t *level, int32_t *dev)
{
    int h = tree_height(t, v);
    int n = devices_below(t, v, dev);
    /* every pair below v gets v's height first; deeper switches overwrite their own pairs */
    for (int a = 0; a < n; ++a)
        for (int b = 0; b < n; ++b)
            level[dev[a] * P + dev[b]] = a == b ? 0 : h;
    if (t->n_dev[v] > 0)
        return;
    for (int c = t->first[v]; c >= 0; c = t->next[c])
        label_pairs(t, c, P, level, dev);
}

static int print_tree(const orc_tree *t, int v, char *out, int len, int pos)
{
    if (t->n_dev[v] > 0) {
        char buf[16];
        int m = 0, x = t->n_dev[v];
        while (x > 0) {
            buf[m++] = (char)('0' + x % 10);
            x /= 10;
        }
        while (m > 0 && pos < len - 1)
            out[pos++] = buf[--m];
        return pos;
    }
    if (pos < len - 1)
        out[pos++] = '[';
    for (int c = t->first[v]; c >= 0; c = t->next[c]) {
        pos = print_tree(t, c, out, len, pos);
        if (t->next[c] >= 0 && pos < len - 1)
            out[pos++] = ',';
    }
    if (pos < len - 1)
        out[pos++] = ']';
    return pos;
}

/*
 * Level table of a tree topology: level[i][j] = height of the lowest switch that joins devices i
 * and j (1: the same device switch, 2: one layer up, ...), 0 on the diagonal.  Devices keep the
 * numbers they have in the tree as given (left to right), also when the merge (merge != 0, see
 * merge_list) moves their switch elsewhere.  `text_out` (may be NULL) receives the notation of the
 * tree that was labelled and `order_out` (may be NULL, room for max_P) the device numbers in the
 * order in which that tree lists them.  Returns the number of devices P, -1 on a syntax error,
 * -2 if P > max_P.
 */
int orc_tree_levels(const char *text, int merge, int max_P, int32_t *level, char *text_out,
                    int text_len, int32_t *order_out)
{
    orc_tree *t = (orc_tree *)malloc(sizeof(orc_tree));
    t->used = 0;
    t->seen = 0;
    t->s = text;
    t->bad = 0;
    int root = parse_element(t);
    skip_blank(t);
    if (t->bad || *t->s != '\0') {
        free(t);
        return -1;
    }
    if (merge)
        merge_tree(t, root);
    int P = count_devices(t, root);
    if (P > max_P) {
        free(t);
        return -2;
    }
    int32_t *dev = (int32_t *)malloc(sizeof(int32_t) * (size_t)P);
    label_pairs(t, root, P, level, dev);
    if (order_out != NULL)
        devices_below(t, root, order_out);
    free(dev);
    if (text_out != NULL && text_len > 0) {
        int pos = print_tree(t, root, text_out, text_len, 0);
        text_out[pos] = '\0';
    }
    free(t);
    return P;
}

/* ---- gate: scores, softmax, top-k ---------------------------------------- */

/* Gate scores (Section 3.1, first paragraph): logits[t][e] = sum_q x[t][q] * W[e][q]. */
void orc_logits(const void *x, const void *w, int dtype, int64_t S, int d, int N, double *logits)
{
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t t = 0; t < S; ++t) {
        for (int e = 0; e < N; ++e) {
            double acc = 0.0;
            for (int q = 0; q < d; ++q)
                acc += load_elem(x, dtype, t * d + q) * load_elem(w, dtype, (int64_t)e * d + q);
            logits[t * N + e] = acc;
        }
    }
}

/* Softmax over the N experts of each token (Section 3.1): the gate vector G(x). */
void orc_softmax(const double *logits, int64_t S, int N, double *G)
{
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t t = 0; t < S; ++t) {
        const double *l = logits + t * N;
        double mx = l[0];
        for (int e = 1; e < N; ++e)
            if (l[e] > mx)
                mx = l[e];
        double den = 0.0;
        for (int e = 0; e < N; ++e)
            den += exp(l[e] - mx);
        for (int e = 0; e < N; ++e)
            G[t * N + e] = exp(l[e] - mx) / den;
    }
}

/*
 * Top-k selection (Section 3.1: only the experts with the top k scores process the sample).
 * Selection is on the scores; equal scores go to the lower expert index; the k choices are
 * listed best first.  The combine weight of a choice is its softmax value, not renormalised.
 */
void orc_topk(const double *logits, const double *G, int64_t S, int N, int k,
              int32_t *idx, double *wgt)
{
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t t = 0; t < S; ++t) {
        const double *l = logits + t * N;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < N; ++e) {
                int taken = 0;
                for (int jj = 0; jj < j; ++jj)
                    if (idx[t * k + jj] == e)
                        taken = 1;
                if (taken)
                    continue;
                if (best < 0 || l[e] > l[best])
                    best = e; /* strict '>' keeps the lowest index among equals */
            }
            idx[t * k + j] = best;
            wgt[t * k + j] = G[t * N + best];
        }
    }
}

/*
 * Load statistics of this device before any capacity pruning (Section 3.1 and the merged
 * per-device delivery of Section 4.1): c_expert[e] = number of (t, j) with idx[t][j] = e,
 * c_device[j] = sum of c_expert over the experts of device j, m[e] = (1/S) sum_t G[t][e].
 */
void orc_counts(const int32_t *idx, const double *G, int64_t S, int N, int P, int k,
                int32_t *c_expert, int32_t *c_device, double *m)
{
    int E = N / P;
    for (int e = 0; e < N; ++e)
        c_expert[e] = 0;
    for (int64_t t = 0; t < S; ++t)
        for (int j = 0; j < k; ++j)
            c_expert[idx[t * k + j]] += 1;
    for (int j = 0; j < P; ++j) {
        c_device[j] = 0;
        for (int e = E * j; e <= E * (j + 1) - 1; ++e)
            c_device[j] += c_expert[e];
    }
    for (int e = 0; e < N; ++e) {
        double s = 0.0;
        for (int64_t t = 0; t < S; ++t)
            s += G[t * N + e];
        m[e] = s / (double)S;
    }
}

/* Load-balance loss (Section 3.1): l_aux = sum_e m[e] * (c[e] / S). */
double orc_l_aux(const double *m, const int32_t *c, int N, int64_t S)
{
    double l = 0.0;
    for (int e = 0; e < N; ++e)
        l += m[e] * ((double)c[e] / (double)S);
    return l;
}

/* Topology-aware loss (Section 4.3): l_topo = N*P * sum_e p[e] * m[e] * c[e] / S. */
double orc_l_topo(const double *p, const double *m, const int32_t *c, int N, int P, int64_t S)
{
    double l = 0.0;
    for (int e = 0; e < N; ++e)
        l += p[e] * m[e] * (double)c[e] / (double)S;
    return (double)N * (double)P * l;
}

/*
 * Combine weights renormalised over a token's k selected experts (a variant of the weighting
 * G(x)_e of Section 3.1 in which the k weights of a token sum to one):
 *   out[t][j] = wgt[t][j] / sum_j' wgt[t][j'].
 */
void orc_renorm_topk(const double *wgt, int64_t S, int k, double *out)
{
    for (int64_t t = 0; t < S; ++t) {
        double s = 0.0;
        for (int j = 0; j < k; ++j)
            s += wgt[t * k + j];
        for (int j = 0; j < k; ++j)
            out[t * k + j] = wgt[t * k + j] / s;
    }
}

/* Its transpose for a gradient d_out that arrives at the renormalised weights:
 *   d_wgt[t][i] = d_out[t][i] / s - (sum_j d_out[t][j] * wgt[t][j]) / s^2,  s = sum_j wgt[t][j]. */
void orc_renorm_topk_bwd(const double *wgt, const double *d_out, int64_t S, int k, double *d_wgt)
{
    for (int64_t t = 0; t < S; ++t) {
        double s = 0.0, dot = 0.0;
        for (int j = 0; j < k; ++j) {
            s += wgt[t * k + j];
            dot += d_out[t * k + j] * wgt[t * k + j];
        }
        for (int i = 0; i < k; ++i)
            d_wgt[t * k + i] = d_out[t * k + i] / s - dot / (s * s);
    }
}

/* ---- capacity-limited dispatch and combine ------------------------------- */

/*
 * Capacity pruning and send-buffer positions (Section 3.1 local capacity c_ie <= C_ie;
 * Section 4.1 chunks for one device merged into one delivery; Section 4.3 variable sizes
 * instead of zero padding).  The (token, choice) pairs are visited choice-major: every first
 * choice in token order, then every second choice, ...  The pair's position among the pairs of
 * its expert is pos; it is kept iff pos < cap[e].  kept[e] = min(c[e], cap[e]); the send buffer
 * lists the kept rows expert by expert (hence device by device), off[e] = sum of kept[e'] for
 * e' < e, slot = off[e] + pos, or -1 for a dropped pair.  send_count_dev[j] is the number of
 * rows bound for device j.  Returns K = off[N], the number of rows in the send buffer.
 */
int64_t orc_slots(const int32_t *idx, const int32_t *cap, int64_t S, int N, int P, int k,
                  int32_t *slot, int32_t *kept, int32_t *off, int32_t *send_count_dev)
{
    int E = N / P;
    int32_t *counter = (int32_t *)calloc((size_t)N, sizeof(int32_t));
    int32_t *pos = (int32_t *)malloc((size_t)S * k * sizeof(int32_t));
    for (int j = 0; j < k; ++j) {
        for (int64_t t = 0; t < S; ++t) {
            int e = idx[t * k + j];
            pos[t * k + j] = counter[e];
            counter[e] += 1;
        }
    }
    for (int e = 0; e < N; ++e)
        kept[e] = counter[e] < cap[e] ? counter[e] : cap[e];
    off[0] = 0;
    for (int e = 0; e < N; ++e)
        off[e + 1] = off[e] + kept[e];
    for (int64_t t = 0; t < S; ++t) {
        for (int j = 0; j < k; ++j) {
            int e = idx[t * k + j];
            slot[t * k + j] = pos[t * k + j] < cap[e] ? off[e] + pos[t * k + j] : -1;
        }
    }
    for (int j = 0; j < P; ++j) {
        send_count_dev[j] = 0;
        for (int e = E * j; e <= E * (j + 1) - 1; ++e)
            send_count_dev[j] += kept[e];
    }
    free(counter);
    free(pos);
    return (int64_t)off[N];
}

/*
 * Fixed-size zero-padded layout (Section 4.3, last paragraph: the layout of DeepSpeed-MoE that
 * the variable chunk sizes replace; Section 3.1: local capacity).  Every expert owns C rows of
 * the buffer whether it fills them or not: slot = e*C + pos for a pair with pos < min(cap[e], C)
 * (cap may be NULL: the limit is C alone), -1 otherwise; kept[e] = min(c[e], cap[e], C).  Rows
 * e*C + kept[e] .. (e+1)*C - 1 stay zero.  The pair order is that of orc_slots.
 */
void orc_slots_padded(const int32_t *idx, const int32_t *cap, int64_t S, int N, int k, int C,
                      int32_t *slot, int32_t *kept)
{
    int32_t *counter = (int32_t *)calloc((size_t)N, sizeof(int32_t));
    for (int j = 0; j < k; ++j) {
        for (int64_t t = 0; t < S; ++t) {
            int e = idx[t * k + j];
            int32_t lim = cap != NULL && cap[e] < C ? cap[e] : C;
            slot[t * k + j] = counter[e] < lim ? e * C + counter[e] : -1;
            counter[e] += 1;
        }
    }
    for (int e = 0; e < N; ++e) {
        int32_t lim = cap != NULL && cap[e] < C ? cap[e] : C;
        kept[e] = counter[e] < lim ? counter[e] : lim;
    }
    free(counter);
}

/* Scatter (Section 3.1: dispatched data of shape [k*S, d], [c_ie, d] per expert): a bit copy
 * send[slot[t][j]][:] = x[t][:] for every kept pair. */
void orc_scatter(const void *x, int dtype, const int32_t *slot, int64_t S, int d, int k, void *send)
{
    size_t row = (size_t)d * elem_size(dtype);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t t = 0; t < S; ++t) {
        for (int j = 0; j < k; ++j) {
            int32_t s = slot[t * k + j];
            if (s >= 0)
                memcpy((char *)send + (size_t)s * row, (const char *)x + (size_t)t * row, row);
        }
    }
}

/*
 * Combine (Section 3.1: the layer output y aggregates the computed results): recv holds the
 * expert outputs in the row order of the send buffer;
 *   y[t][:] = sum over kept choices j (ascending) of wgt[t][j] * recv[slot[t][j]][:],
 * a zero row if every choice of the token was dropped.  y_exact (may be NULL) receives the
 * double result, y (may be NULL) the result rounded once to the storage type.
 */
void orc_combine(const void *recv, int dtype, const int32_t *slot, const double *wgt,
                 int64_t S, int d, int k, double *y_exact, void *y)
{
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t t = 0; t < S; ++t) {
        for (int q = 0; q < d; ++q) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j) {
                int32_t s = slot[t * k + j];
                if (s >= 0)
                    acc += wgt[t * k + j] * load_elem(recv, dtype, (int64_t)s * d + q);
            }
            if (y_exact)
                y_exact[t * d + q] = acc;
            if (y)
                store_elem(y, dtype, t * d + q, acc);
        }
    }
}

/* ---- backward of the path (for training: the auxiliary loss is added to the train loss,
 * Section 3.1 / Section 4.3, so its gradient and the transposes of the row movers are needed) -- */

/*
 * Gradient with respect to the gate scores, for fixed routing (the counts c and the selected
 * indices do not depend on the scores differentiably):
 *   L = sum_{t,j} dwgt[t][j] * G[t][idx[t][j]]  +  loss_scale * l_topo,
 *   l_topo = N*P * sum_e p[e] * m[e] * c[e] / S,   m[e] = (1/S) sum_t G[t][e]   (Section 4.3).
 * With u[t][e] = sum_j dwgt[t][j] * [idx[t][j] == e] + loss_scale * N*P*p[e]*c[e]/S^2 the softmax
 * Jacobian dG_i/dl_e = G_i (delta_ie - G_e) gives
 *   dlogits[t][e] = G[t][e] * ( u[t][e] - sum_e' u[t][e'] * G[t][e'] ).
 * p == NULL stands for the load-balance loss l_aux of Section 3.1 (weights 1, no N*P factor).
 */
void orc_gate_bwd(const double *logits, const int32_t *idx, const double *dwgt, const double *p,
                  const int32_t *c, double loss_scale, int64_t S, int N, int P, int k, double *dlogits)
{
    double *G = (double *)malloc((size_t)S * N * sizeof(double));
    orc_softmax(logits, S, N, G);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t t = 0; t < S; ++t) {
        double ubar = 0.0;
        for (int e = 0; e < N; ++e) {
            double u = loss_scale * (p ? (double)N * (double)P * p[e] : 1.0) * (double)c[e]
                       / ((double)S * (double)S);
            for (int j = 0; j < k; ++j)
                if (idx[t * k + j] == e)
                    u += dwgt[t * k + j];
            dlogits[t * N + e] = u; /* u for now */
            ubar += u * G[t * N + e];
        }
        for (int e = 0; e < N; ++e)
            dlogits[t * N + e] = G[t * N + e] * (dlogits[t * N + e] - ubar);
    }
    free(G);
}

/*
 * Backward of the combine y[t] = sum_j wgt[t][j] * recv[slot[t][j]]:
 *   drecv[slot[t][j]][:] = wgt[t][j] * dy[t][:]          for every kept pair (rows that no slot
 *                                                         names stay zero),
 *   dwgt[t][j] = sum_q dy[t][q] * recv[slot[t][j]][q]    for a kept pair, 0 for a dropped one.
 * drecv_exact (may be NULL) is the double result, drecv (may be NULL) the result rounded once
 * to the storage type.
 */
void orc_combine_bwd(const void *dy, const void *recv, int dtype, const int32_t *slot,
                     const double *wgt, int64_t S, int64_t K, int d, int k,
                     double *drecv_exact, void *drecv, double *dwgt)
{
    if (drecv_exact)
        memset(drecv_exact, 0, (size_t)K * d * sizeof(double));
    if (drecv)
        memset(drecv, 0, (size_t)K * d * elem_size(dtype));
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t t = 0; t < S; ++t) {
        for (int j = 0; j < k; ++j) {
            int32_t s = slot[t * k + j];
            double dot = 0.0;
            if (s >= 0) {
                for (int q = 0; q < d; ++q) {
                    double g = load_elem(dy, dtype, t * d + q);
                    double v = wgt[t * k + j] * g;
                    if (drecv_exact)
                        drecv_exact[(int64_t)s * d + q] = v;
                    if (drecv)
                        store_elem(drecv, dtype, (int64_t)s * d + q, v);
                    dot += g * load_elem(recv, dtype, (int64_t)s * d + q);
                }
            }
            dwgt[t * k + j] = dot;
        }
    }
}

/*
 * Backward of the scatter send[slot[t][j]] = x[t]: the transpose adds the rows back,
 *   dx[t][:] = sum over kept j of dsend[slot[t][j]][:].
 */
void orc_dispatch_bwd(const void *dsend, int dtype, const int32_t *slot, int64_t S, int d, int k,
                      double *dx_exact, void *dx)
{
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t t = 0; t < S; ++t) {
        for (int q = 0; q < d; ++q) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j) {
                int32_t s = slot[t * k + j];
                if (s >= 0)
                    acc += load_elem(dsend, dtype, (int64_t)s * d + q);
            }
            if (dx_exact)
                dx_exact[t * d + q] = acc;
            if (dx)
                store_elem(dx, dtype, t * d + q, acc);
        }
    }
}

/* ---- receive side: rows of the exchange regrouped per local expert --------------------------- */

/*
 * After the global exchange (Section 3.1: each expert receives a combined batch of tokens) this
 * device holds one chunk per source device s = 0..P-1, in that order; inside a chunk the rows are
 * grouped by local expert e = 0..E-1 (the sender's buffer lists rows expert by expert), cnt[s][e]
 * rows each (the c_se of Section 3.1 after capacity).  The experts need one batch each:
 *   expert-major layout = for e = 0..E-1, for s = 0..P-1: the cnt[s][e] rows of (s, e).
 * to_expert_major != 0 converts source-major -> expert-major, 0 converts back (for the return
 * exchange).  expert_offset[e] (E+1 entries, may be NULL) = first row of expert e's batch.
 * Returns the number of rows R.
 */
int64_t orc_regroup(const void *in, int dtype, const int32_t *cnt, int P, int E, int d,
                    int to_expert_major, void *out, int32_t *expert_offset)
{
    size_t row = (size_t)d * elem_size(dtype);
    int64_t src_pos = 0; /* position in the source-major buffer */
    for (int s = 0; s < P; ++s) {
        for (int e = 0; e < E; ++e) {
            /* position of segment (s, e) in the expert-major buffer */
            int64_t em_pos = 0;
            for (int ee = 0; ee < E; ++ee)
                for (int ss = 0; ss < P; ++ss)
                    if (ee < e || (ee == e && ss < s))
                        em_pos += cnt[ss * E + ee];
            for (int32_t r = 0; r < cnt[s * E + e]; ++r) {
                if (to_expert_major)
                    memcpy((char *)out + (size_t)(em_pos + r) * row, (const char *)in + (size_t)(src_pos + r) * row, row);
                else
                    memcpy((char *)out + (size_t)(src_pos + r) * row, (const char *)in + (size_t)(em_pos + r) * row, row);
            }
            src_pos += cnt[s * E + e];
        }
    }
    if (expert_offset) {
        int64_t acc = 0;
        for (int e = 0; e < E; ++e) {
            expert_offset[e] = (int32_t)acc;
            for (int s = 0; s < P; ++s)
                acc += cnt[s * E + e];
        }
        expert_offset[E] = (int32_t)acc;
    }
    return src_pos;
}
