/*
 * CPU oracle for the WAGMA-SGD per-iteration hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
 * reference that the GPU library is checked against.  It shares no code,
 * header, table or constant generator with the HIP library, and only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * Every function follows the paper (arXiv 2005.00124) in the paper's own
 * order and notation:
 *   - oracle_grouping_unionfind : Algorithm 1 (dynamic grouping), literally,
 *                                 with a union-find over the P processes.
 *   - oracle_member_table       : the butterfly phases of Section 3.3 (the
 *                                 text after Algorithm 1) turned into an
 *                                 ordered member list per group.
 *   - oracle_step_f32 / _f64    : Algorithm 2 lines 6-17 for one iteration t
 *                                 on P model replicas held as P rows, as
 *                                 printed (functions of their own).
 *   - oracle_step_lag_f32/_f64  : the same iteration when some processes are
 *                                 still computing an earlier step and take
 *                                 part only through their send buffer
 *                                 (Section 4, the execution snapshot;
 *                                 Assumption 1, item 3).
 *   - oracle_stale_mask         : the seeded stand-in for "which processes
 *                                 are late in iteration t" (not in the paper;
 *                                 a counter-based integer hash).
 *   - oracle_lag_states/_masks  : who is on time, late or still computing when
 *                                 every process runs its steps back to back
 *                                 and the first to finish activates the
 *                                 group allreduce (Section 3.2).
 *
 * Readings of the paper taken here (each is also pinned by a CPU test):
 *   - Algorithm 1 line 6: the mask of a phase is 1 << shift, built afresh in
 *     every phase (the printed "mask <<= shift" would accumulate; only the
 *     afresh reading reproduces the printed P=8,S=4 groups of iteration 1).
 *   - Algorithm 2 line 8: iteration t is a global one iff (t+1) mod tau == 0;
 *     tau == 0 means "never".
 *   - U() in Algorithm 2 line 6 is heavy-ball momentum SGD:
 *       m' = mu*m + g,  w' = w - lr*m'   (each one fused multiply-add).
 *   - The sum inside a group is taken in butterfly-phase order: a balanced
 *     pairwise tree over the member list, first phase = adjacent members.
 *     The global sum is the same tree over ranks 0..P-1.
 *   - 1/S and 1/P are exact powers of two (a multiply); 1/(S+1) is a true
 *     IEEE division applied after the addition W_sum + W'.
 *   - The send buffer ("pub") of every process holds W' of the last
 *     iteration: pub <- W' at the end of every iteration, global ones too.
 *   - A process that is still computing when a group allreduce runs (lateness
 *     deeper than one iteration) contributes its send buffer once more and is
 *     otherwise left alone in that iteration: no local update, no gradient
 *     read, send buffer not refreshed; the sum that lands in its receive
 *     buffer is overwritten by a later one before it looks.  A global
 *     iteration waits for everybody, so nobody is late or absent in it.
 *
 * Parity unpinned: where the paper is silent the reading above is a choice; the
 * pins fix the arithmetic of the choice (hand values, brute force), nothing in
 * the paper fixes the choice itself.  These are: what the send buffer holds
 * after a global iteration and before the first iteration (the caller sets
 * it); what a process that is still computing does in an iteration
 * (oracle_step_lag_*) and the clock model that says who is in time, late or
 * still computing (oracle_lag_states, oracle_lag_masks); and the three seeded
 * lateness generators, which stand in for physical lateness.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC ... -lm
 * (no contraction, no fast-math, no flush-to-zero: IEEE fp32 throughout).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)
#define ORACLE_ENOMEM (-2)

/* log2 of a power of two, or -1. */
static int exact_log2(int64_t x)
{
    int l = 0;
    if (x < 1)
        return -1;
    while ((x & 1) == 0) {
        x >>= 1;
        ++l;
    }
    return x == 1 ? l : -1;
}

static int uf_find(int32_t *parent, int p)
{
    while (parent[p] != p)
        p = parent[p];
    return p;
}

/*
 * Algorithm 1 as a union-find over the P ranks.  All ranks begin in sets of
 * one.  Iteration t runs log2(S) butterfly phases; the first works on address
 * bit (t * log2 S) mod log2 P and each later one on the next bit, cyclically.
 * A phase on bit b joins the sets of every two ranks that differ in bit b only.
 * rep[p] receives the smallest member of p's set, which names the group.
 */
int oracle_grouping_unionfind(int P, int S, int64_t t, int32_t *rep)
{
    int log2_P = exact_log2(P);
    int log2_S = exact_log2(S);
    if (log2_P < 0 || log2_S < 0 || S > P || t < 0 || !rep)
        return ORACLE_EINVAL;

    int32_t *parent = (int32_t *)malloc(sizeof(int32_t) * (size_t)P);
    if (!parent)
        return ORACLE_ENOMEM;
    for (int p = 0; p < P; ++p)
        parent[p] = p;

    int bit = log2_P > 0 ? (int)((t * (int64_t)log2_S) % log2_P) : 0;
    for (int phase = 0; phase < log2_S; ++phase) {
        for (int p = 0; p < P; ++p) {
            int partner = p ^ (1 << bit); /* the rank p exchanges with in this phase */
            int root_a = uf_find(parent, p);
            int root_b = uf_find(parent, partner);
            /* the smaller root stays on top, so a set's root is its smallest member */
            if (root_a < root_b)
                parent[root_b] = root_a;
            else if (root_b < root_a)
                parent[root_a] = root_b;
        }
        bit = (bit + 1) % log2_P;
    }
    for (int p = 0; p < P; ++p)
        rep[p] = uf_find(parent, p);
    free(parent);
    return ORACLE_OK;
}

/*
 * The bit positions of the butterfly phases executed in iteration t, in the
 * order Algorithm 1 visits them.  bits[] must hold log2(S) entries.
 */
static void phase_bits(int log2_P, int log2_S, int64_t t, int *bits)
{
    int bit = 0;
    if (log2_P > 0)
        bit = (int)((t * (int64_t)log2_S) % log2_P);
    for (int r = 0; r < log2_S; ++r) {
        bits[r] = bit;
        bit = (bit + 1) % log2_P;
    }
}

/*
 * Ordered member list of every group in iteration t.
 * table[k*S + e] = rank of member e of the k-th group.  Groups are listed by
 * ascending smallest member.  Inside a group, member e differs from the
 * smallest member in exactly the phase bits selected by the binary digits of
 * e: digit r of e switches the bit of phase r.  So members e and e^1 are the
 * pair that exchanges in the first phase, e and e^2 in the second, and so on:
 * a balanced pairwise sum over e = 0..S-1 is the butterfly's own order.
 */
int oracle_member_table(int P, int S, int64_t t, int32_t *table)
{
    int log2_P = exact_log2(P);
    int log2_S = exact_log2(S);
    int bits[32];
    if (log2_P < 0 || log2_S < 0 || S > P || t < 0 || !table)
        return ORACLE_EINVAL;
    phase_bits(log2_P, log2_S, t, bits);

    int all_bits = 0;
    for (int r = 0; r < log2_S; ++r)
        all_bits |= 1 << bits[r];

    int k = 0;
    for (int base = 0; base < P; ++base) {
        if (base & all_bits)
            continue; /* not the smallest member of its group */
        for (int e = 0; e < S; ++e) {
            int p = base;
            for (int r = 0; r < log2_S; ++r)
                if ((e >> r) & 1)
                    p |= 1 << bits[r];
            table[k * S + e] = p;
        }
        ++k;
    }
    return k == P / S ? ORACLE_OK : ORACLE_EINVAL;
}

/* Is iteration t one that ends in the global average (Algorithm 2 line 8)? */
int oracle_is_global_iteration(int tau, int64_t t)
{
    return tau > 0 && ((t + 1) % tau) == 0;
}

/* Balanced pairwise sum of count = 2^k values, adjacent pairs first. */
static float tree_sum_f32(const float *c, int count)
{
    if (count == 1)
        return c[0];
    float left = tree_sum_f32(c, count / 2);
    float right = tree_sum_f32(c + count / 2, count / 2);
    return left + right;
}

static double tree_sum_f64(const double *c, int count)
{
    if (count == 1)
        return c[0];
    double left = tree_sum_f64(c, count / 2);
    double right = tree_sum_f64(c + count / 2, count / 2);
    return left + right;
}

static int mask_bit(const uint64_t *stale_mask, int p)
{
    if (!stale_mask)
        return 0;
    return (int)((stale_mask[p >> 6] >> (p & 63)) & 1u);
}

/*
 * Algorithm 2, lines 6-17, as printed: one iteration t for all P replicas, in
 * which every process finishes its local step inside the iteration (nobody is
 * still computing an earlier one).  w, g, m, pub: P rows of ld floats, n used
 * columns; w, m, pub are updated in place, g is read only.  stale_mask: bit p
 * set = process p is late (NULL = nobody).  fixed_groups != 0: the groups of
 * iteration 0 in every group iteration (the second ablation of Section 6.2).
 * Written out on its own so that it can be read against the paper
 * without the third state; a CPU test pins oracle_step_lag_f32(busy_mask = NULL)
 * to it bit for bit.
 */
int oracle_step_f32(int P, int S, int64_t n, int64_t ld, int tau, int64_t t,
                    float *w, const float *g, float *m, float *pub,
                    const uint64_t *stale_mask, float lr, float mu, int fixed_groups)
{
    if (exact_log2(P) < 0 || exact_log2(S) < 0 || S > P || n < 1 || ld < n ||
        tau < 0 || t < 0 || !w || !g || !m || !pub)
        return ORACLE_EINVAL;

    int32_t *table = (int32_t *)malloc(sizeof(int32_t) * (size_t)P);
    float *w_prime = (float *)malloc(sizeof(float) * (size_t)P);
    float *contrib = (float *)malloc(sizeof(float) * (size_t)P);
    if (!table || !w_prime || !contrib) {
        free(table);
        free(w_prime);
        free(contrib);
        return ORACLE_ENOMEM;
    }
    int global = oracle_is_global_iteration(tau, t);
    if (!global)
        oracle_member_table(P, S, fixed_groups ? 0 : t, table);

    for (int64_t j = 0; j < n; ++j) {
        /* lines 6-7: W' = W + U(G, W, t), heavy-ball momentum */
        for (int i = 0; i < P; ++i) {
            int64_t at = (int64_t)i * ld + j;
            float m_new = fmaf(mu, m[at], g[at]);
            w_prime[i] = fmaf(-lr, m_new, w[at]);
            m[at] = m_new;
        }
        if (global) {
            /* lines 15-16: W_{t+1} = (1/P) * sum over all processes of W' */
            float avg = tree_sum_f32(w_prime, P) * (1.0f / (float)P);
            for (int i = 0; i < P; ++i)
                w[(int64_t)i * ld + j] = avg;
        } else {
            for (int k = 0; k < P / S; ++k) {
                const int32_t *member = table + (int64_t)k * S;
                /* line 9: W_sum; a late process is represented by its send buffer */
                for (int e = 0; e < S; ++e) {
                    int p = member[e];
                    contrib[e] = mask_bit(stale_mask, p) ? pub[(int64_t)p * ld + j] : w_prime[p];
                }
                float w_sum = tree_sum_f32(contrib, S);
                for (int e = 0; e < S; ++e) {
                    int p = member[e];
                    if (!mask_bit(stale_mask, p))
                        w[(int64_t)p * ld + j] = w_sum * (1.0f / (float)S);            /* lines 10-11 */
                    else
                        w[(int64_t)p * ld + j] = (w_sum + w_prime[p]) / (float)(S + 1); /* lines 12-13 */
                }
            }
        }
        /* Section 4: the send buffer is refreshed with W' */
        for (int i = 0; i < P; ++i)
            pub[(int64_t)i * ld + j] = w_prime[i];
    }
    free(table);
    free(w_prime);
    free(contrib);
    return ORACLE_OK;
}

/* The same in fp64 (the shadow that bounds the rounding of the fp32 path). */
int oracle_step_f64(int P, int S, int64_t n, int64_t ld, int tau, int64_t t,
                    double *w, const double *g, double *m, double *pub,
                    const uint64_t *stale_mask, double lr, double mu, int fixed_groups)
{
    if (exact_log2(P) < 0 || exact_log2(S) < 0 || S > P || n < 1 || ld < n ||
        tau < 0 || t < 0 || !w || !g || !m || !pub)
        return ORACLE_EINVAL;

    int32_t *table = (int32_t *)malloc(sizeof(int32_t) * (size_t)P);
    double *w_prime = (double *)malloc(sizeof(double) * (size_t)P);
    double *contrib = (double *)malloc(sizeof(double) * (size_t)P);
    if (!table || !w_prime || !contrib) {
        free(table);
        free(w_prime);
        free(contrib);
        return ORACLE_ENOMEM;
    }
    int global = oracle_is_global_iteration(tau, t);
    if (!global)
        oracle_member_table(P, S, fixed_groups ? 0 : t, table);

    for (int64_t j = 0; j < n; ++j) {
        for (int i = 0; i < P; ++i) {
            int64_t at = (int64_t)i * ld + j;
            double m_new = mu * m[at] + g[at];
            w_prime[i] = w[at] - lr * m_new;
            m[at] = m_new;
        }
        if (global) {
            double avg = tree_sum_f64(w_prime, P) / (double)P;
            for (int i = 0; i < P; ++i)
                w[(int64_t)i * ld + j] = avg;
        } else {
            for (int k = 0; k < P / S; ++k) {
                const int32_t *member = table + (int64_t)k * S;
                for (int e = 0; e < S; ++e) {
                    int p = member[e];
                    contrib[e] = mask_bit(stale_mask, p) ? pub[(int64_t)p * ld + j] : w_prime[p];
                }
                double w_sum = tree_sum_f64(contrib, S);
                for (int e = 0; e < S; ++e) {
                    int p = member[e];
                    if (!mask_bit(stale_mask, p))
                        w[(int64_t)p * ld + j] = w_sum / (double)S;
                    else
                        w[(int64_t)p * ld + j] = (w_sum + w_prime[p]) / (double)(S + 1);
                }
            }
        }
        for (int i = 0; i < P; ++i)
            pub[(int64_t)i * ld + j] = w_prime[i];
    }
    free(table);
    free(w_prime);
    free(contrib);
    return ORACLE_OK;
}

/*
 * The iteration of oracle_step_f32 with a third state beside "in time" and
 * "late": a process that is still computing an earlier step when this
 * iteration's group allreduce runs (the execution snapshot of Section 4,
 * carried beyond one iteration).
 * w, g, m, pub: P rows of ld floats, n used columns.  w, m, pub are updated
 * in place; g is read only.  stale_mask: bit p set = process p is late in
 * this iteration (NULL = nobody): it contributes its send buffer, finishes its
 * local step afterwards and averages the group's sum with its own W' (lines
 * 12-13).  busy_mask: bit p set = process p is still computing (NULL =
 * nobody): it contributes its send buffer again and nothing of it changes.
 * busy wins over late.  Both masks are ignored in a global iteration, which
 * every process enters after the same number of steps.
 * fixed_groups != 0 is the paper's second ablation (Section 6.2): group model
 * averaging without the dynamic grouping strategy, i.e. the groups of
 * iteration 0 in every group iteration.
 */
int oracle_step_lag_f32(int P, int S, int64_t n, int64_t ld, int tau, int64_t t,
                        float *w, const float *g, float *m, float *pub,
                        const uint64_t *stale_mask, const uint64_t *busy_mask,
                        float lr, float mu, int fixed_groups)
{
    if (exact_log2(P) < 0 || exact_log2(S) < 0 || S > P || n < 1 || ld < n ||
        tau < 0 || t < 0 || !w || !g || !m || !pub)
        return ORACLE_EINVAL;

    int32_t *table = (int32_t *)malloc(sizeof(int32_t) * (size_t)P);
    float *w_prime = (float *)malloc(sizeof(float) * (size_t)P);
    float *contrib = (float *)malloc(sizeof(float) * (size_t)P);
    if (!table || !w_prime || !contrib) {
        free(table);
        free(w_prime);
        free(contrib);
        return ORACLE_ENOMEM;
    }
    int global = oracle_is_global_iteration(tau, t);
    if (!global)
        oracle_member_table(P, S, fixed_groups ? 0 : t, table);

    for (int64_t j = 0; j < n; ++j) {
        /* lines 6-7: local update of every replica that finishes a step in this iteration */
        for (int i = 0; i < P; ++i) {
            if (!global && mask_bit(busy_mask, i))
                continue; /* still computing: nothing of this process changes */
            int64_t at = (int64_t)i * ld + j;
            float m_new = fmaf(mu, m[at], g[at]);
            w_prime[i] = fmaf(-lr, m_new, w[at]);
            m[at] = m_new;
        }
        if (global) {
            /* lines 15-16: everybody contributes W', staleness ignored */
            float sum = tree_sum_f32(w_prime, P);
            float avg = sum * (1.0f / (float)P);
            for (int i = 0; i < P; ++i)
                w[(int64_t)i * ld + j] = avg;
        } else {
            /* lines 9-14 */
            for (int k = 0; k < P / S; ++k) {
                const int32_t *member = table + (int64_t)k * S;
                for (int e = 0; e < S; ++e) {
                    int p = member[e];
                    contrib[e] = (mask_bit(stale_mask, p) || mask_bit(busy_mask, p))
                                     ? pub[(int64_t)p * ld + j] /* send buffer */
                                     : w_prime[p];
                }
                float w_sum = tree_sum_f32(contrib, S);
                for (int e = 0; e < S; ++e) {
                    int p = member[e];
                    int64_t at = (int64_t)p * ld + j;
                    if (mask_bit(busy_mask, p))
                        continue; /* the sum waits in its receive buffer, unread */
                    if (!mask_bit(stale_mask, p))
                        w[at] = w_sum * (1.0f / (float)S);
                    else
                        w[at] = (w_sum + w_prime[p]) / (float)(S + 1);
                }
            }
        }
        /* the send buffer now holds this iteration's locally updated model */
        for (int i = 0; i < P; ++i)
            if (global || !mask_bit(busy_mask, i))
                pub[(int64_t)i * ld + j] = w_prime[i];
    }
    free(table);
    free(w_prime);
    free(contrib);
    return ORACLE_OK;
}

/* The same iteration carried in fp64 (a shadow used to bound rounding). */
int oracle_step_lag_f64(int P, int S, int64_t n, int64_t ld, int tau, int64_t t,
                        double *w, const double *g, double *m, double *pub,
                        const uint64_t *stale_mask, const uint64_t *busy_mask,
                        double lr, double mu, int fixed_groups)
{
    if (exact_log2(P) < 0 || exact_log2(S) < 0 || S > P || n < 1 || ld < n ||
        tau < 0 || t < 0 || !w || !g || !m || !pub)
        return ORACLE_EINVAL;

    int32_t *table = (int32_t *)malloc(sizeof(int32_t) * (size_t)P);
    double *w_prime = (double *)malloc(sizeof(double) * (size_t)P);
    double *contrib = (double *)malloc(sizeof(double) * (size_t)P);
    if (!table || !w_prime || !contrib) {
        free(table);
        free(w_prime);
        free(contrib);
        return ORACLE_ENOMEM;
    }
    int global = oracle_is_global_iteration(tau, t);
    if (!global)
        oracle_member_table(P, S, fixed_groups ? 0 : t, table);

    for (int64_t j = 0; j < n; ++j) {
        for (int i = 0; i < P; ++i) {
            if (!global && mask_bit(busy_mask, i))
                continue;
            int64_t at = (int64_t)i * ld + j;
            double m_new = mu * m[at] + g[at];
            w_prime[i] = w[at] - lr * m_new;
            m[at] = m_new;
        }
        if (global) {
            double avg = tree_sum_f64(w_prime, P) / (double)P;
            for (int i = 0; i < P; ++i)
                w[(int64_t)i * ld + j] = avg;
        } else {
            for (int k = 0; k < P / S; ++k) {
                const int32_t *member = table + (int64_t)k * S;
                for (int e = 0; e < S; ++e) {
                    int p = member[e];
                    contrib[e] = (mask_bit(stale_mask, p) || mask_bit(busy_mask, p))
                                     ? pub[(int64_t)p * ld + j]
                                     : w_prime[p];
                }
                double w_sum = tree_sum_f64(contrib, S);
                for (int e = 0; e < S; ++e) {
                    int p = member[e];
                    int64_t at = (int64_t)p * ld + j;
                    if (mask_bit(busy_mask, p))
                        continue;
                    if (!mask_bit(stale_mask, p))
                        w[at] = w_sum / (double)S;
                    else
                        w[at] = (w_sum + w_prime[p]) / (double)(S + 1);
                }
            }
        }
        for (int i = 0; i < P; ++i)
            if (global || !mask_bit(busy_mask, i))
                pub[(int64_t)i * ld + j] = w_prime[i];
    }
    free(table);
    free(w_prime);
    free(contrib);
    return ORACLE_OK;
}

/*
 * Seeded lateness: process p is late in iteration t iff the upper 32 bits of
 * a 64-bit integer hash of (seed, t, p) fall below `threshold`
 * (threshold = floor(q * 2^32) for a late probability q).  Integer only, so
 * any two implementations agree bit for bit.
 * The hash is two rounds of the public splitmix64 output function
 * (Steele, Lea, Flood 2014; Vigna's splitmix64.c), keyed by t and then p.
 */
static uint64_t splitmix_finish(uint64_t z)
{
    z ^= z >> 30;
    z *= UINT64_C(0xBF58476D1CE4E5B9);
    z ^= z >> 27;
    z *= UINT64_C(0x94D049BB133111EB);
    z ^= z >> 31;
    return z;
}

int oracle_stale_mask(uint64_t seed, int64_t t, int P, uint32_t threshold,
                      uint64_t *mask_words)
{
    if (P < 1 || t < 0 || !mask_words)
        return ORACLE_EINVAL;
    int words = (P + 63) / 64;
    for (int k = 0; k < words; ++k)
        mask_words[k] = 0;
    uint64_t per_iter =
        splitmix_finish(seed + UINT64_C(0x9E3779B97F4A7C15) * ((uint64_t)t + 1u));
    for (int p = 0; p < P; ++p) {
        uint64_t h = splitmix_finish(
            per_iter + UINT64_C(0xD1B54A32D192ED03) * ((uint64_t)p + 1u));
        if ((uint32_t)(h >> 32) < threshold)
            mask_words[p >> 6] |= UINT64_C(1) << (p & 63);
    }
    return ORACLE_OK;
}

/*
 * Lateness as the paper's image-classification experiment injects it
 * (Section 6.2): in every training step `count` randomly selected processes
 * are delayed (the paper selects two).  Draw j of iteration t is the top
 * log2(P) bits of a hash of (seed, t, j); draws that repeat a process already
 * selected are skipped.  P must be a power of two.
 */
int oracle_straggler_mask(uint64_t seed, int64_t t, int P, int count, uint64_t *mask_words)
{
    int bits = exact_log2(P);
    if (bits < 0 || t < 0 || count < 0 || count > P || !mask_words)
        return ORACLE_EINVAL;
    for (int k = 0; k < (P + 63) / 64; ++k)
        mask_words[k] = 0;
    uint64_t per_iter =
        splitmix_finish((seed ^ UINT64_C(0x5354524147474C52)) + UINT64_C(0x9E3779B97F4A7C15) * ((uint64_t)t + 1u));
    int chosen = 0;
    for (uint64_t j = 0; chosen < count; ++j) {
        uint64_t h = splitmix_finish(per_iter + UINT64_C(0xD1B54A32D192ED03) * (j + 1u));
        int p = bits == 0 ? 0 : (int)(h >> (64 - bits));
        if ((mask_words[p >> 6] >> (p & 63)) & 1u)
            continue;
        mask_words[p >> 6] |= UINT64_C(1) << (p & 63);
        ++chosen;
    }
    return ORACLE_OK;
}

/*
 * Lateness from simulated step times, shaped like the reinforcement-learning
 * workload of Section 6.4 (iteration times from 1.7 s to 43.5 s, median below
 * 2 s): nine steps in sixteen take between 1.7 s and 2 s, the others one of 16
 * geometrically spaced times from 2 s to 43.5 s.  The process that finishes
 * first is the activator (Section 3.2) and is never late; any other process is
 * late iff it finishes more than tolerance_ms after the activator.
 * step_ms, if not NULL, receives the P step times.
 */
static const uint32_t oracle_tail_ms[16] = {2000, 2456, 3016, 3703, 4548, 5585, 6858, 8422,
                                            10342, 12700, 15595, 19151, 23517, 28879, 35463, 43500};

int oracle_clock_mask(uint64_t seed, int64_t t, int P, uint32_t tolerance_ms,
                      uint64_t *mask_words, uint32_t *step_ms)
{
    if (P < 1 || t < 0 || !mask_words)
        return ORACLE_EINVAL;
    uint32_t *ms = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)P);
    if (!ms)
        return ORACLE_ENOMEM;
    uint64_t per_iter =
        splitmix_finish((seed ^ UINT64_C(0x434C4F434B4D534B)) + UINT64_C(0x9E3779B97F4A7C15) * ((uint64_t)t + 1u));
    uint32_t fastest = UINT32_MAX;
    for (int p = 0; p < P; ++p) {
        uint64_t h = splitmix_finish(per_iter + UINT64_C(0xD1B54A32D192ED03) * ((uint64_t)p + 1u));
        if ((h >> 60) < 9u)
            ms[p] = 1700u + (uint32_t)((h >> 32) & 0xFFu) * 300u / 256u; /* 1700 .. 1999 */
        else
            ms[p] = oracle_tail_ms[(h >> 56) & 15u];
        if (ms[p] < fastest)
            fastest = ms[p];
    }
    for (int k = 0; k < (P + 63) / 64; ++k)
        mask_words[k] = 0;
    for (int p = 0; p < P; ++p) {
        if ((uint64_t)ms[p] > (uint64_t)fastest + tolerance_ms)
            mask_words[p >> 6] |= UINT64_C(1) << (p & 63);
        if (step_ms)
            step_ms[p] = ms[p];
    }
    free(ms);
    return ORACLE_OK;
}

/*
 * Lateness deeper than one iteration.  Between two global iterations nobody
 * waits for anybody (Section 3.2): every process runs its local steps back to
 * back, and group allreduce number k is activated by the first process that
 * finishes a step begun for it.  The allreduce takes the models as they stand
 * tolerance_ms after the activation and hands the sum back at that moment.
 * In iteration k a process is
 *   ORACLE_FRESH  it finished the step it had begun for allreduce k in time:
 *                 it contributes W', receives the average and begins its next
 *                 step when the allreduce is done;
 *   ORACLE_LATE   it finishes a step after allreduce k has taken its send
 *                 buffer and before allreduce k+1 takes it again: it averages
 *                 the sum of allreduce k with its W' (Algorithm 2 lines 12-13)
 *                 and begins its next step, for allreduce k+1, straight away;
 *   ORACLE_BUSY   it is still computing when allreduce k+1 runs.
 * A step begun for allreduce k by process p lasts step_ms[k][p] (a process that
 * is busy in iteration k never uses its entry of row k).
 *
 * step_ms: K+1 rows of P times, row 0 = the first iteration of the window (the
 * iteration after a global one), every time above tolerance_ms.
 * states: K rows of P.
 */
enum { ORACLE_FRESH = 0, ORACLE_LATE = 1, ORACLE_BUSY = 2 };

int oracle_lag_states(int P, int K, const uint32_t *step_ms, uint32_t tolerance_ms, uint8_t *states)
{
    if (P < 1 || K < 0 || !step_ms || !states)
        return ORACLE_EINVAL;
    for (int64_t i = 0; i < (int64_t)(K + 1) * P; ++i)
        if (step_ms[i] <= tolerance_ms)
            return ORACLE_EINVAL;
    int64_t *finish = (int64_t *)malloc(sizeof(int64_t) * (size_t)P); /* end of the current step */
    int *begun_for = (int *)malloc(sizeof(int) * (size_t)P);          /* allreduce it was begun for */
    if (!finish || !begun_for) {
        free(finish);
        free(begun_for);
        return ORACLE_ENOMEM;
    }
    for (int p = 0; p < P; ++p) {
        finish[p] = step_ms[p];
        begun_for[p] = 0;
    }
    for (int k = 0; k < K; ++k) {
        uint8_t *state = states + (int64_t)k * P;
        const uint32_t *next_ms = step_ms + (int64_t)(k + 1) * P;
        /* the activator: first to finish a step begun for allreduce k */
        int64_t activated = INT64_MAX;
        for (int p = 0; p < P; ++p)
            if (begun_for[p] == k && finish[p] < activated)
                activated = finish[p];
        int64_t taken = activated + tolerance_ms; /* when allreduce k reads the models */
        /* earliest moment allreduce k+1 can be activated, as far as known */
        int64_t next_activated = INT64_MAX;
        for (int p = 0; p < P; ++p) {
            state[p] = ORACLE_BUSY; /* until shown otherwise below */
            if (begun_for[p] == k && finish[p] <= taken) {
                state[p] = ORACLE_FRESH;
                begun_for[p] = k + 1;
                finish[p] = taken + next_ms[p];
                if (finish[p] < next_activated)
                    next_activated = finish[p];
            }
        }
        /* the others in the order in which they finish: one that ends its step before
           allreduce k+1 reads the models is late in k, and its next step may itself
           activate allreduce k+1 */
        for (;;) {
            int first = -1;
            for (int p = 0; p < P; ++p)
                if (state[p] == ORACLE_BUSY && begun_for[p] <= k &&
                    (first < 0 || finish[p] < finish[first]))
                    first = p;
            if (first < 0 || finish[first] > next_activated + tolerance_ms)
                break;
            state[first] = ORACLE_LATE;
            begun_for[first] = k + 1;
            finish[first] += next_ms[first];
            if (finish[first] < next_activated)
                next_activated = finish[first];
        }
    }
    free(finish);
    free(begun_for);
    return ORACLE_OK;
}

/* the step time of process p for a step begun in iteration t (as in oracle_clock_mask) */
static uint32_t clock_step_ms(uint64_t seed, int64_t t, int p)
{
    uint64_t per_iter =
        splitmix_finish((seed ^ UINT64_C(0x434C4F434B4D534B)) + UINT64_C(0x9E3779B97F4A7C15) * ((uint64_t)t + 1u));
    uint64_t h = splitmix_finish(per_iter + UINT64_C(0xD1B54A32D192ED03) * ((uint64_t)p + 1u));
    if ((h >> 60) < 9u)
        return 1700u + (uint32_t)((h >> 32) & 0xFFu) * 300u / 256u;
    return oracle_tail_ms[(h >> 56) & 15u];
}

/*
 * The two masks of iteration t under the step times of oracle_clock_mask.  The
 * clocks restart after every global iteration (Algorithm 2 lines 15-16: there
 * everybody waits); with tau == 0 they restart every `window` iterations
 * instead, which bounds the staleness as Assumption 1 item 3 asks.  In a global
 * iteration both masks are empty.
 */
int oracle_lag_masks(uint64_t seed, int64_t t, int P, int tau, int window, uint32_t tolerance_ms,
                     uint64_t *late_words, uint64_t *busy_words)
{
    if (P < 1 || t < 0 || tau < 0 || (tau == 0 && window < 1) || tolerance_ms >= 1700u ||
        !late_words || !busy_words)
        return ORACLE_EINVAL;
    for (int k = 0; k < (P + 63) / 64; ++k)
        late_words[k] = busy_words[k] = 0;
    if (oracle_is_global_iteration(tau, t))
        return ORACLE_OK;
    int64_t length = tau > 0 ? tau : window;
    int64_t first = t / length * length;
    int K = (int)(t - first) + 1;
    uint32_t *ms = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(K + 1) * (size_t)P);
    uint8_t *states = (uint8_t *)malloc((size_t)K * (size_t)P);
    if (!ms || !states) {
        free(ms);
        free(states);
        return ORACLE_ENOMEM;
    }
    for (int k = 0; k <= K; ++k)
        for (int p = 0; p < P; ++p)
            ms[(int64_t)k * P + p] = clock_step_ms(seed, first + k, p);
    int rc = oracle_lag_states(P, K, ms, tolerance_ms, states);
    if (rc == ORACLE_OK) {
        for (int p = 0; p < P; ++p) {
            uint8_t s = states[(int64_t)(K - 1) * P + p];
            if (s == ORACLE_LATE)
                late_words[p >> 6] |= UINT64_C(1) << (p & 63);
            else if (s == ORACLE_BUSY)
                busy_words[p >> 6] |= UINT64_C(1) << (p & 63);
        }
    }
    free(ms);
    free(states);
    return rc;
}
