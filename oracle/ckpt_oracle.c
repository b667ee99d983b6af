/*
 * CPU oracle for the activation-checkpoint dynamic program.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * solver computes; the tests, the smoke check and the benchmark's cpu_baseline
 * leg are its only callers.  It shares no code, header, table or constant with
 * the GPU library and the GPU library never calls it.
 *
 * What it computes: C_BP(s, t, m) of the paper's Theorem (Section "Activation
 * Checkpoint Solver / Modeling"), the optimal time of a persistent schedule
 * that back-propagates through stages s..t with m memory slots, for every
 * 1 <= s <= t <= L and every m in 0..M, plus the candidate that attains it.
 *
 * Readings taken where the paper leaves a choice:
 *   - u_f and u_b arrive with the communication times of Table 2 already added,
 *     o_f and o_b with the communication overheads already added.
 *   - "infinity" is the sentinel 2^30; a value is min(2^30, exact sum), so any
 *     infeasible operand makes the candidate infeasible.
 *   - a negative memory argument means infeasible.
 *   - candidates are numbered k = s for C_all (also the only candidate when
 *     s == t) and k = s' in s+1..t for C_ck(s, s', t, m); the recorded choice is
 *     the smallest k that attains the minimum, 0 when the cell is infeasible.
 *   - m ranges over 0..M inclusive.
 *
 * Layout of the outputs (one chain): cost[((s-1)*L + (t-1))*(M+1) + m], same for
 * choice; entries with s > t are left untouched.
 *
 * Parity pins (tests/test_oracle_*.py): hand-derived L=3 example, brute force
 * over every persistent schedule for L <= 6 through an independent operation
 * simulator, the unlimited-memory closed form, monotonicity in m, the
 * infeasibility bound, an independent scalar minimum-memory recursion.  The
 * m_null gate, which no schedule-level check can see when every omega_abar is
 * at least its omega_a (it is then implied by the feasibility of the
 * operands), is pinned by the peak of the forward sweep F_ck^s,
 * F_null^{s+1..t-1} run through that same simulator.
 *
 * Outside the model: an omega_abar below its omega_a contradicts the paper's
 * "abar contains a"; the Theorem is then no longer the optimum over
 * persistent schedules (the brute force shows counter-examples), so there is
 * nothing to be exact against.  The functions below still evaluate the printed
 * formulas on such inputs; the GPU library flags them as a violated
 * precondition.
 */
#include <stdint.h>
#include <stdlib.h>

#define ORACLE_INF ((int64_t)1 << 30)

static int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }

/* Stage arrays are 1-based in the paper; uf[k-1] holds u_f^k and so on.
 * wa and wd are indexed 0..L directly. */
typedef struct {
    int L, M;
    const int32_t *uf, *ub, *wa, *wab, *wd, *of, *ob;
    int32_t *cost;
    int16_t *choice;
} chain_t;

static size_t cell(const chain_t *c, int s, int t, int m) {
    return ((size_t)(s - 1) * c->L + (size_t)(t - 1)) * ((size_t)c->M + 1) + (size_t)m;
}

/* C_BP(s, t, mm) with the convention that a negative budget is infeasible. */
static int64_t lookup(const chain_t *c, int s, int t, int64_t mm) {
    if (mm < 0) return ORACLE_INF;
    return c->cost[cell(c, s, t, (int)mm)];
}

/* m_all^{s,t}: memory needed to run F_all^s (with delta^t resident) and later B^s. */
static int64_t m_all(const chain_t *c, int s, int t) {
    int64_t fwd = (int64_t)c->wd[t] + c->wab[s - 1] + c->of[s - 1];
    int64_t bwd = (int64_t)c->wd[s] + c->wab[s - 1] + c->ob[s - 1];
    return max64(fwd, bwd);
}

/* m_null^{s,t}: memory needed to run F_ck^s and then F_null^j for s+1 <= j < t. */
static int64_t m_null(const chain_t *c, int s, int t) {
    int64_t need = (int64_t)c->wa[s] + c->of[s - 1];
    for (int j = s + 1; j < t; ++j)
        need = max64(need, (int64_t)c->wa[j - 1] + c->wa[j] + c->of[j - 1]);
    return (int64_t)c->wd[t] + need;
}

static void solve_cell_row(const chain_t *c, int s, int t) {
    const int64_t need_all = m_all(c, s, t);
    const int64_t need_null = (t > s) ? m_null(c, s, t) : 0;
    for (int m = 0; m <= c->M; ++m) {
        int64_t best = ORACLE_INF;
        int pick = 0;
        if (s == t) {
            if (m >= need_all) {
                int64_t v = (int64_t)c->uf[s - 1] + c->ub[s - 1];
                if (v > ORACLE_INF) v = ORACLE_INF;
                if (v < best) { best = v; pick = s; }
            }
        } else {
            /* C_2: keep everything of stage s (F_all^s), recurse on s+1..t, then B^s. */
            if (m >= need_all) {
                int64_t v = (int64_t)c->uf[s - 1] + c->ub[s - 1]
                          + lookup(c, s + 1, t, (int64_t)m - c->wab[s - 1]);
                if (v > ORACLE_INF) v = ORACLE_INF;
                if (v < best) { best = v; pick = s; }
            }
            /* C_1: checkpoint a^{s-1}, run forward to a^{s'-1}, solve s'..t, then s..s'-1. */
            if (m >= need_null) {
                int64_t fwd = 0;
                for (int sp = s + 1; sp <= t; ++sp) {
                    fwd += c->uf[sp - 2]; /* sum_{k=s}^{s'-1} u_f^k */
                    int64_t v = fwd + lookup(c, sp, t, (int64_t)m - c->wa[sp - 1])
                              + lookup(c, s, sp - 1, m);
                    if (v > ORACLE_INF) v = ORACLE_INF;
                    if (v < best) { best = v; pick = sp; }
                }
            }
        }
        c->cost[cell(c, s, t, m)] = (int32_t)best;
        c->choice[cell(c, s, t, m)] = (int16_t)pick;
    }
}

/*
 * Fill the table of one chain.  Returns 0, or -1 on a bad argument.
 * nthreads > 1 spreads the independent rows of one segment length over OpenMP
 * threads; the arithmetic of a row is the same either way.
 */
int oracle_solve_chain(int L, int M, const int32_t *uf, const int32_t *ub, const int32_t *wa,
                       const int32_t *wab, const int32_t *wd, const int32_t *of, const int32_t *ob,
                       int32_t *cost, int16_t *choice, int nthreads) {
    if (L < 1 || M < 0 || !uf || !ub || !wa || !wab || !wd || !of || !ob || !cost || !choice) return -1;
    chain_t c = {L, M, uf, ub, wa, wab, wd, of, ob, cost, choice};
    (void)nthreads;
    for (int d = 0; d < L; ++d) {
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
#endif
        for (int s = 1; s <= L - d; ++s) solve_cell_row(&c, s, s + d);
    }
    return 0;
}

/* The two thresholds, exported so that tests can look at them. */
int64_t oracle_m_all(int L, const int32_t *wa, const int32_t *wab, const int32_t *wd, const int32_t *of,
                     const int32_t *ob, int s, int t) {
    chain_t c = {L, 0, 0, 0, wa, wab, wd, of, ob, 0, 0};
    return m_all(&c, s, t);
}

int64_t oracle_m_null(int L, const int32_t *wa, const int32_t *wab, const int32_t *wd, const int32_t *of,
                      const int32_t *ob, int s, int t) {
    chain_t c = {L, 0, 0, 0, wa, wab, wd, of, ob, 0, 0};
    return m_null(&c, s, t);
}

int oracle_max_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
