/*
 * tictac_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, single-threaded CPU implementation of the scheduling math of
 * "TicTac: Accelerating Distributed Deep Learning with Communication
 * Scheduling" (arXiv 1803.03288), written from the paper's definitions.  It is
 * the yardstick the GPU library is compared with and shares no code with it.
 * Only the tests, the smoke check and the benchmark's CPU-baseline leg may
 * call it; the library never does.
 *
 * What follows which passage
 *   oracle_find_dependencies   Sec. 4.1 "Communication Dependency (op.dep)"
 *   oracle_update_properties   Sec. 4.1 Algorithm 1 (op.M, recv.P, recv.M+)
 *   oracle_tic                 Sec. 4.2 Algorithm 2 with the General Time Oracle
 *   oracle_tac                 Sec. 4.3: pairwise rule of Case 1, tie-break of
 *                              Case 2, selection loop of Algorithm 3
 *   oracle_simulate            Sec. 3.1 (resources, priorities), Sec. 3.2
 *                              (makespan bounds U and L, Scheduling Efficiency E,
 *                              Speedup S), Sec. 5.1 (one transfer at a time per
 *                              channel, transfers released in priority order)
 *   oracle_simulate_channels   the same with one channel per parameter server
 *                              (Sec. 4.1, 5.1)
 *   oracle_simulate_sends      the same with send ops on an uplink (Sec. 2.2)
 *   oracle_straggler           Sec. 6 "Straggler Effect"
 *   oracle_time_oracle_min     Sec. 5 "Time Oracle"
 *   oracle_order_search        Sec. 3.1 (the best order is NP-hard to find) and
 *                              Sec. 4.3 (the comparator is an approximation): a
 *                              climb through proposed exchanges, measured by
 *                              oracle_simulate
 *
 * Readings where the paper is silent or inconsistent (each is restated at the
 * function that uses it):
 *   - recv.dep contains the recv itself, so that recv.M = Time(recv) as the text
 *     under Algorithm 1 says.
 *   - The comparator follows the derived pairwise rule (Case 1): A goes before B
 *     when min{P_B, M_A} < min{P_A, M_B}.  The printed comparator listing has
 *     the two min-terms the other way round, which contradicts that derivation
 *     and the toy example of Sec. 2.2; comparator_mode = 1 selects the printed
 *     form so that a test can show it fails those pins.
 *   - "Find the minimum op wrt Comparator" is an ascending-index linear scan
 *     that keeps the current best and replaces it only when the candidate
 *     strictly precedes it.
 *   - M+ stays +infinity when no op has two or more outstanding dependencies
 *     including the recv; TIC reports INT32_MAX for it.          parity unpinned
 *   - E := 1 and S := 0 when U == L (nothing to schedule); S := 0 when L == 0.
 *                                                                parity unpinned
 *   - One compute resource running one op at a time and one channel with one
 *     active transfer; all transfers are requested at t = 0 and served
 *     back-to-back in the given order; a ready compute op is started as soon as
 *     the device is idle (the pick among several ready ops is by a caller-given
 *     key, lowest first; the makespan does not depend on it).
 *
 * Bitsets: row v of dep has W = ceil(R/64) 64-bit words; recv i is bit (i & 63)
 * of word (i >> 6).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_CYCLE (-1)
#define ORACLE_ERR_ARG (-2)
#define ORACLE_ERR_MEM (-3)
#define ORACLE_PRIO_INF INT32_MAX

static int n_words(int R) { return (R + 63) / 64; }
static int bit_get(const uint64_t *row, int i) { return (int)((row[i >> 6] >> (i & 63)) & 1u); }
static void bit_set(uint64_t *row, int i) { row[i >> 6] |= (uint64_t)1 << (i & 63); }

/* recv index of every op (-1 for a compute op) */
static int32_t *recv_index_of_op(int n, int R, const int32_t *recv_ids)
{
    int32_t *ri = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    if (!ri) return NULL;
    for (int v = 0; v < n; ++v) ri[v] = -1;
    for (int i = 0; i < R; ++i) ri[recv_ids[i]] = i;
    return ri;
}

/* ------------------------------------------------------------------------
 * Sec. 4.1, Communication Dependency: op.dep is the set of recv ops that the
 * op depends on directly or transitively, found by a depth-first post-order
 * traversal: an op is finished after all of its predecessors, and its set is
 * then its own recv (if it is one) united with the sets of its predecessors.
 * dep: [n][W], written entirely.
 * ---------------------------------------------------------------------- */
int oracle_find_dependencies(int n, const int32_t *row_ptr, const int32_t *col_idx, int R,
                             const int32_t *recv_ids, uint64_t *dep)
{
    const int W = n_words(R);
    if (n < 0 || R < 0) return ORACLE_ERR_ARG;
    int32_t *ri = recv_index_of_op(n, R, recv_ids);
    uint8_t *state = (uint8_t *)calloc((size_t)(n > 0 ? n : 1), 1);   /* 0 new, 1 open, 2 done */
    int32_t *stack = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    int32_t *next = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    if (!ri || !state || !stack || !next) { free(ri); free(state); free(stack); free(next); return ORACLE_ERR_MEM; }
    memset(dep, 0, (size_t)n * (size_t)W * sizeof(uint64_t));
    int rc = ORACLE_OK;
    for (int root = 0; root < n && rc == ORACLE_OK; ++root) {
        if (state[root]) continue;
        int top = 0;
        stack[0] = root; state[root] = 1; next[root] = row_ptr[root];
        while (top >= 0) {
            int v = stack[top];
            if (next[v] < row_ptr[v + 1]) {
                int u = col_idx[next[v]++];
                if (state[u] == 0) { state[u] = 1; next[u] = row_ptr[u]; stack[++top] = u; }
                else if (state[u] == 1) { rc = ORACLE_ERR_CYCLE; break; }
            } else {
                uint64_t *dv = dep + (size_t)v * W;
                if (ri[v] >= 0) bit_set(dv, ri[v]);
                for (int e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
                    const uint64_t *du = dep + (size_t)col_idx[e] * W;
                    for (int w = 0; w < W; ++w) dv[w] |= du[w];
                }
                state[v] = 2; --top;
            }
        }
    }
    free(ri); free(state); free(stack); free(next);
    return rc;
}

/* op.dep as a sorted list of recv indices per op (the same sets as the bitset
 * rows, in a form that is cheap to walk): set v is idx[ptr[v] .. ptr[v+1]). */
typedef struct { int64_t *ptr; int32_t *idx; } depsets_t;

static int depsets_build(int n, int R, int W, const uint64_t *dep, depsets_t *s)
{
    s->ptr = (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
    if (!s->ptr) return ORACLE_ERR_MEM;
    int64_t total = 0;
    for (int v = 0; v < n; ++v) {
        s->ptr[v] = total;
        for (int i = 0; i < R; ++i) total += bit_get(dep + (size_t)v * W, i);
    }
    s->ptr[n] = total;
    s->idx = (int32_t *)malloc((size_t)(total > 0 ? total : 1) * sizeof(int32_t));
    if (!s->idx) { free(s->ptr); return ORACLE_ERR_MEM; }
    int64_t k = 0;
    for (int v = 0; v < n; ++v)
        for (int i = 0; i < R; ++i)
            if (bit_get(dep + (size_t)v * W, i)) s->idx[k++] = i;
    return ORACLE_OK;
}
static void depsets_free(depsets_t *s) { free(s->ptr); free(s->idx); }

/* ------------------------------------------------------------------------
 * Sec. 4.1, Algorithm 1 (property update) for the outstanding set `alive`.
 *   time  [n]  Time(op) by op id
 *   alive [R]  1 = recv i is outstanding
 *   M     [n]  out: sum of Time(r) over r in op.dep that are outstanding,
 *              added in ascending recv index
 *   P     [R]  out (outstanding recvs only; others left 0)
 *   Mplus [R]  out (outstanding recvs only; others left +inf)
 * The third loop runs over the ops that are not outstanding recvs, in
 * ascending op id.
 * ---------------------------------------------------------------------- */
static void update_properties(int n, int R, const depsets_t *s, const int32_t *ri,
                              const double *time, const int32_t *recv_ids, const uint8_t *alive,
                              double *M, double *P, double *Mplus)
{
    for (int v = 0; v < n; ++v) {
        double m = 0.0;
        for (int64_t k = s->ptr[v]; k < s->ptr[v + 1]; ++k) {
            int i = s->idx[k];
            if (alive[i]) m += time[recv_ids[i]];
        }
        M[v] = m;
    }
    for (int i = 0; i < R; ++i) { P[i] = 0.0; Mplus[i] = HUGE_VAL; }
    for (int v = 0; v < n; ++v) {
        if (ri[v] >= 0 && alive[ri[v]]) continue;          /* op in R: skipped */
        int cnt = 0;                                       /* |op.dep intersect R| */
        for (int64_t k = s->ptr[v]; k < s->ptr[v + 1]; ++k) cnt += alive[s->idx[k]];
        if (cnt == 1) {
            for (int64_t k = s->ptr[v]; k < s->ptr[v + 1]; ++k)
                if (alive[s->idx[k]]) P[s->idx[k]] += time[v];
        } else if (cnt > 1) {
            for (int64_t k = s->ptr[v]; k < s->ptr[v + 1]; ++k) {
                int i = s->idx[k];
                if (alive[i] && M[v] < Mplus[i]) Mplus[i] = M[v];
            }
        }
    }
}

int oracle_update_properties(int n, int R, const uint64_t *dep, const int32_t *recv_ids,
                             const double *time, const uint8_t *alive, double *M, double *P,
                             double *Mplus)
{
    int32_t *ri = recv_index_of_op(n, R, recv_ids);
    depsets_t s;
    if (!ri) return ORACLE_ERR_MEM;
    if (depsets_build(n, R, n_words(R), dep, &s) != ORACLE_OK) { free(ri); return ORACLE_ERR_MEM; }
    update_properties(n, R, &s, ri, time, recv_ids, alive, M, P, Mplus);
    depsets_free(&s);
    free(ri);
    return ORACLE_OK;
}

/* stable ordering of recv indices by an integer key; rank = inverse */
static void order_by_key(int R, const int32_t *key, int32_t *order, int32_t *rank)
{
    for (int i = 0; i < R; ++i) {
        int r = 0;
        for (int j = 0; j < R; ++j)
            if (key[j] < key[i] || (key[j] == key[i] && j < i)) ++r;
        rank[i] = r;
        order[r] = i;
    }
}

/* ------------------------------------------------------------------------
 * Sec. 4.2, Algorithm 2 (TIC): Algorithm 1 with every recv outstanding and the
 * General Time Oracle (recv = 1, anything else = 0), in integer arithmetic;
 * priority(recv) = recv.M+.  A recv with no multi-dependency consumer keeps
 * M+ = infinity, reported as INT32_MAX.
 *   prio [R] raw M+; order [R] recv indices by (prio, index); rank [R] inverse.
 * ---------------------------------------------------------------------- */
int oracle_tic(int n, int R, const uint64_t *dep, const int32_t *recv_ids, int32_t *prio,
               int32_t *order, int32_t *rank)
{
    const int W = n_words(R);
    int32_t *ri = recv_index_of_op(n, R, recv_ids);
    if (!ri) return ORACLE_ERR_MEM;
    for (int i = 0; i < R; ++i) prio[i] = ORACLE_PRIO_INF;
    for (int v = 0; v < n; ++v) {
        if (ri[v] >= 0) continue;                         /* every recv is outstanding */
        const uint64_t *dv = dep + (size_t)v * W;
        int32_t m = 0;                                    /* op.M = number of recvs in op.dep */
        for (int i = 0; i < R; ++i) m += bit_get(dv, i);
        if (m > 1)
            for (int i = 0; i < R; ++i)
                if (bit_get(dv, i) && m < prio[i]) prio[i] = m;
    }
    order_by_key(R, prio, order, rank);
    free(ri);
    return ORACLE_OK;
}

/* Sec. 4.3.  Does recv a go before recv b?
 * mode 0: Case 1's derived rule, min{P_b, M_a} < min{P_a, M_b}, and on equality
 *         Case 2's tie-break, smaller M+ first.
 * mode 1: the comparator as its listing prints it (min-terms exchanged); kept
 *         only so that a test can show that it contradicts the pins. */
static int precedes(int a, int b, const double *P, const double *Mrecv, const double *Mplus, int mode)
{
    double x, y;
    if (mode == 0) { x = fmin(P[b], Mrecv[a]); y = fmin(P[a], Mrecv[b]); }
    else           { x = fmin(P[a], Mrecv[b]); y = fmin(P[b], Mrecv[a]); }
    if (x != y) return x < y;
    return Mplus[a] < Mplus[b];
}

/* ------------------------------------------------------------------------
 * Sec. 4.3, Algorithm 3 (TAC) for B timing samples.
 *   op_time [B][N]: column j = j-th compute op in ascending op id
 *   recv_time [B][R]: column i = recv i
 *   alive0: NULL, or [B][R] with 1 = recv i of sample b is still outstanding when the
 *           loop starts.  Algorithm 3 starts with every recv in R; its loop body (the
 *           property update of Algorithm 1 on the current R, then the choice of the
 *           minimum) depends on nothing but the current R, so starting from a smaller R
 *           yields the rounds that follow a prefix which removed the other recvs.
 *   max_rounds < 0: run until R is empty; otherwise stop after that many selections
 *                   (remaining order entries and ranks are -1)
 *   order [B][R] step -> recv (steps counted from the start set); rank [B][R] recv -> step;
 *   sel_P, sel_Mplus [B][R] (may be NULL): P and M+ of each recv in the round in
 *   which it was selected.
 * Every round recomputes Algorithm 1 from scratch over the whole graph.
 * ---------------------------------------------------------------------- */
int oracle_tac(int n, int R, const uint64_t *dep, const int32_t *recv_ids, int B, const double *op_time,
               const double *recv_time, const uint8_t *alive0, int max_rounds, int comparator_mode,
               int32_t *order, int32_t *rank, double *sel_P, double *sel_Mplus)
{
    const int N = n - R;
    int32_t *ri = recv_index_of_op(n, R, recv_ids);
    depsets_t s;
    if (depsets_build(n, R, n_words(R), dep, &s) != ORACLE_OK) { free(ri); return ORACLE_ERR_MEM; }
    double *time = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    double *M = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    double *P = (double *)malloc((size_t)(R > 0 ? R : 1) * sizeof(double));
    double *Mplus = (double *)malloc((size_t)(R > 0 ? R : 1) * sizeof(double));
    double *Mrecv = (double *)malloc((size_t)(R > 0 ? R : 1) * sizeof(double));
    uint8_t *alive = (uint8_t *)malloc((size_t)(R > 0 ? R : 1));
    if (!ri || !time || !M || !P || !Mplus || !Mrecv || !alive) {
        free(ri); free(time); free(M); free(P); free(Mplus); free(Mrecv); free(alive);
        depsets_free(&s);
        return ORACLE_ERR_MEM;
    }
    for (int b = 0; b < B; ++b) {
        const double *ot = op_time + (size_t)b * N, *rt = recv_time + (size_t)b * R;
        int32_t *ord = order + (size_t)b * R, *rk = rank + (size_t)b * R;
        int j = 0, outstanding = 0;
        for (int v = 0; v < n; ++v) time[v] = (ri[v] >= 0) ? rt[ri[v]] : ot[j++];
        for (int i = 0; i < R; ++i) {
            alive[i] = alive0 ? (alive0[(size_t)b * R + i] != 0) : 1;
            outstanding += alive[i];
            ord[i] = -1; rk[i] = -1;
        }
        const int rounds = (max_rounds < 0 || max_rounds > outstanding) ? outstanding : max_rounds;
        for (int step = 0; step < rounds; ++step) {
            update_properties(n, R, &s, ri, time, recv_ids, alive, M, P, Mplus);
            for (int i = 0; i < R; ++i) Mrecv[i] = M[recv_ids[i]];   /* = Time(recv i) while outstanding */
            int best = -1;
            for (int i = 0; i < R; ++i) {
                if (!alive[i]) continue;
                if (best < 0) best = i;
                else if (precedes(i, best, P, Mrecv, Mplus, comparator_mode)) best = i;
            }
            ord[step] = best; rk[best] = step;
            if (sel_P) sel_P[(size_t)b * R + best] = P[best];
            if (sel_Mplus) sel_Mplus[(size_t)b * R + best] = Mplus[best];
            alive[best] = 0;
        }
    }
    free(ri); free(time); free(M); free(P); free(Mplus); free(Mrecv); free(alive);
    depsets_free(&s);
    return ORACLE_OK;
}

/* a binary min-heap of (key, op) used as the ready-to-execute queue */
typedef struct { int32_t *key, *op; int len; } heap_t;
static void heap_push(heap_t *h, int32_t key, int32_t op)
{
    int i = h->len++;
    while (i > 0) {
        int p = (i - 1) / 2;
        if (h->key[p] <= key) break;
        h->key[i] = h->key[p]; h->op[i] = h->op[p]; i = p;
    }
    h->key[i] = key; h->op[i] = op;
}
static int32_t heap_pop(heap_t *h)
{
    int32_t top = h->op[0];
    int32_t key = h->key[--h->len], op = h->op[h->len];
    int i = 0;
    for (;;) {
        int c = 2 * i + 1;
        if (c >= h->len) break;
        if (c + 1 < h->len && h->key[c + 1] < h->key[c]) ++c;
        if (h->key[c] >= key) break;
        h->key[i] = h->key[c]; h->op[i] = h->op[c]; i = c;
    }
    if (h->len > 0) { h->key[i] = key; h->op[i] = op; }
    return top;
}

/* ------------------------------------------------------------------------
 * One iteration under a transfer order, for B timing samples (Sec. 3.1, 3.2, 5.1).
 * Two resources: the channel serves the recvs back-to-back from t = 0 in
 * `order` (one active transfer at a time); the compute device runs one op at a
 * time and, whenever it is idle and some op is ready (all predecessors
 * finished), starts the ready op with the lowest pick_key at once.
 *   order: [R] shared (order_stride = 0) or [B][R] (order_stride = R)
 *   pick_key [n] by op id, or NULL for the op id itself
 *   makespan = finish time of the last op (recvs included)
 *   U = sum of all times; L = max(sum of compute times, sum of recv times)
 *   E = (U - m) / (U - L), 1 when U == L;  S = (U - L) / L, 0 when U == L or L == 0
 *   U_out, L_out, S_out may be NULL.
 * ---------------------------------------------------------------------- */
int oracle_simulate(int n, const int32_t *row_ptr, const int32_t *col_idx, int R, const int32_t *recv_ids,
                    int B, const int32_t *order, int order_stride, const double *op_time,
                    const double *recv_time, const int32_t *pick_key, double *makespan, double *eff,
                    double *U_out, double *L_out, double *S_out)
{
    const int N = n - R;
    const size_t n1 = (size_t)(n > 0 ? n : 1);
    int32_t *ri = recv_index_of_op(n, R, recv_ids);
    /* successor lists */
    int32_t *sptr = (int32_t *)calloc(n1 + 1, sizeof(int32_t));
    int32_t *sidx = (int32_t *)malloc((size_t)(row_ptr[n] > 0 ? row_ptr[n] : 1) * sizeof(int32_t));
    int32_t *fill = (int32_t *)malloc(n1 * sizeof(int32_t));
    int32_t *waiting = (int32_t *)malloc(n1 * sizeof(int32_t));
    double *time = (double *)malloc(n1 * sizeof(double));
    heap_t h = { (int32_t *)malloc(n1 * sizeof(int32_t)), (int32_t *)malloc(n1 * sizeof(int32_t)), 0 };
    if (!ri || !sptr || !sidx || !fill || !waiting || !time || !h.key || !h.op) return ORACLE_ERR_MEM;
    for (int v = 0; v < n; ++v)
        for (int e = row_ptr[v]; e < row_ptr[v + 1]; ++e) sptr[col_idx[e] + 1]++;
    for (int v = 0; v < n; ++v) sptr[v + 1] += sptr[v];
    for (int v = 0; v < n; ++v) fill[v] = sptr[v];
    for (int v = 0; v < n; ++v)
        for (int e = row_ptr[v]; e < row_ptr[v + 1]; ++e) sidx[fill[col_idx[e]]++] = v;

    int rc = ORACLE_OK;
    for (int b = 0; b < B && rc == ORACLE_OK; ++b) {
        const double *ot = op_time + (size_t)b * N, *rt = recv_time + (size_t)b * R;
        const int32_t *ord = order + (size_t)b * order_stride;
        int j = 0;
        double sum_c = 0.0, sum_r = 0.0;
        for (int v = 0; v < n; ++v) {
            if (ri[v] >= 0) { time[v] = rt[ri[v]]; sum_r += time[v]; }
            else { time[v] = ot[j++]; sum_c += time[v]; }
            waiting[v] = row_ptr[v + 1] - row_ptr[v];
        }
        h.len = 0;
        for (int v = 0; v < n; ++v)
            if (ri[v] < 0 && waiting[v] == 0) heap_push(&h, pick_key ? pick_key[v] : v, v);

        double now = 0.0, m = 0.0;
        int k = 0;                   /* next transfer to complete */
        double net_end = (R > 0) ? rt[ord[0]] : 0.0;
        int running = -1;
        double run_end = 0.0;
        int finished = 0;
        while (finished < n) {
            int acted = 0;
            /* completions at the current time */
            while (k < R && net_end <= now) {
                int v = recv_ids[ord[k]];
                if (net_end > m) m = net_end;
                for (int e = sptr[v]; e < sptr[v + 1]; ++e)
                    if (--waiting[sidx[e]] == 0) heap_push(&h, pick_key ? pick_key[sidx[e]] : sidx[e], sidx[e]);
                ++finished; ++k; acted = 1;
                if (k < R) net_end = net_end + rt[ord[k]];
            }
            if (running >= 0 && run_end <= now) {
                int v = running;
                if (run_end > m) m = run_end;
                for (int e = sptr[v]; e < sptr[v + 1]; ++e)
                    if (--waiting[sidx[e]] == 0) heap_push(&h, pick_key ? pick_key[sidx[e]] : sidx[e], sidx[e]);
                running = -1; ++finished; acted = 1;
            }
            if (running < 0 && h.len > 0) {
                running = heap_pop(&h);
                run_end = now + time[running];
                acted = 1;
            }
            if (acted) continue;     /* something may complete or start at this same instant */
            /* advance to the next completion */
            double nxt = HUGE_VAL;
            if (k < R) nxt = net_end;
            if (running >= 0 && run_end < nxt) nxt = run_end;
            if (nxt == HUGE_VAL) { rc = ORACLE_ERR_CYCLE; break; }   /* ops left that can never start */
            now = nxt;
        }
        double U = sum_c + sum_r;
        double L = sum_c > sum_r ? sum_c : sum_r;
        makespan[b] = m;
        eff[b] = (U == L) ? 1.0 : (U - m) / (U - L);
        if (U_out) U_out[b] = U;
        if (L_out) L_out[b] = L;
        if (S_out) S_out[b] = (U == L || L == 0.0) ? 0.0 : (U - L) / L;
    }
    free(ri); free(sptr); free(sidx); free(fill); free(waiting); free(time); free(h.key); free(h.op);
    return rc;
}

/* ------------------------------------------------------------------------
 * The iteration with send ops (Sec. 2.2: in the worker's graph the recv ops are roots and the
 * send ops are leaves; they carry results back to the parameter servers).  The paper orders
 * the recvs only and gives the sends no model of their own; the reading taken here:
 *   - a send is a leaf of the graph whose time is a transfer time on the uplink, a third
 *     resource beside the compute device and the (downlink) channel of oracle_simulate,
 *     with one active transfer at a time (Sec. 5.1's rule for a channel);
 *   - a send is requested at the instant its last predecessor finishes, and the uplink
 *     serves requests first come first served (requests of one instant by op id);
 *   - the compute device runs the other compute ops as in oracle_simulate, and since the
 *     finish times of single ops now matter, so does its pick among several ready ops:
 *     the lowest op id (pick_key NULL) or the lowest pick_key;
 *   - makespan = finish of the last op, sends included; U = sum of all times;
 *     L = max(sum of compute times without the sends, sum of recv times, sum of send times)
 *     (Eq. 2: one term per resource); E and S from them as in oracle_simulate.
 *   send_ids [n_send]: op ids; every one must be a compute op without successors.
 *   op_time holds a send's transfer time in the send's column.
 * ---------------------------------------------------------------------- */
int oracle_simulate_sends(int n, const int32_t *row_ptr, const int32_t *col_idx, int R, const int32_t *recv_ids,
                          int n_send, const int32_t *send_ids, int B, const int32_t *order, int order_stride,
                          const double *op_time, const double *recv_time, const int32_t *pick_key,
                          double *makespan, double *eff, double *U_out, double *L_out, double *S_out)
{
    const int N = n - R;
    const size_t n1 = (size_t)(n > 0 ? n : 1);
    int32_t *ri = recv_index_of_op(n, R, recv_ids);
    int32_t *sptr = (int32_t *)calloc(n1 + 1, sizeof(int32_t));
    int32_t *sidx = (int32_t *)malloc((size_t)(row_ptr[n] > 0 ? row_ptr[n] : 1) * sizeof(int32_t));
    int32_t *fill = (int32_t *)malloc(n1 * sizeof(int32_t));
    int32_t *waiting = (int32_t *)malloc(n1 * sizeof(int32_t));
    uint8_t *is_send = (uint8_t *)calloc(n1, 1);
    int32_t *queue = (int32_t *)malloc(n1 * sizeof(int32_t));       /* requests to the uplink, in service order */
    int32_t *fresh = (int32_t *)malloc(n1 * sizeof(int32_t));       /* sends requested at the current instant */
    double *time = (double *)malloc(n1 * sizeof(double));
    heap_t h = { (int32_t *)malloc(n1 * sizeof(int32_t)), (int32_t *)malloc(n1 * sizeof(int32_t)), 0 };
    if (!ri || !sptr || !sidx || !fill || !waiting || !is_send || !queue || !fresh || !time || !h.key || !h.op)
        return ORACLE_ERR_MEM;
    for (int v = 0; v < n; ++v)
        for (int e = row_ptr[v]; e < row_ptr[v + 1]; ++e) sptr[col_idx[e] + 1]++;
    for (int v = 0; v < n; ++v) sptr[v + 1] += sptr[v];
    for (int v = 0; v < n; ++v) fill[v] = sptr[v];
    for (int v = 0; v < n; ++v)
        for (int e = row_ptr[v]; e < row_ptr[v + 1]; ++e) sidx[fill[col_idx[e]]++] = v;
    for (int i = 0; i < n_send; ++i) {
        const int v = send_ids[i];
        if (v < 0 || v >= n || ri[v] >= 0 || is_send[v] || sptr[v + 1] != sptr[v]) return ORACLE_ERR_ARG;
        is_send[v] = 1;
    }

    int rc = ORACLE_OK;
    for (int b = 0; b < B && rc == ORACLE_OK; ++b) {
        const double *ot = op_time + (size_t)b * N, *rt = recv_time + (size_t)b * R;
        const int32_t *ord = order + (size_t)b * order_stride;
        int j = 0;
        double sum_c = 0.0, sum_r = 0.0, sum_s = 0.0;
        for (int v = 0; v < n; ++v) {
            if (ri[v] >= 0) { time[v] = rt[ri[v]]; sum_r += time[v]; }
            else {
                time[v] = ot[j++];
                if (is_send[v]) sum_s += time[v]; else sum_c += time[v];
            }
            waiting[v] = row_ptr[v + 1] - row_ptr[v];
        }
        h.len = 0;
        int q_head = 0, q_tail = 0, n_fresh = 0;
        for (int v = 0; v < n; ++v) {
            if (ri[v] >= 0 || waiting[v] != 0) continue;
            if (is_send[v]) fresh[n_fresh++] = v;                   /* a send without predecessors: requested at 0 */
            else heap_push(&h, pick_key ? pick_key[v] : v, v);
        }

        double now = 0.0, m = 0.0;
        int k = 0;
        double net_end = (R > 0) ? rt[ord[0]] : 0.0;
        int running = -1, sending = -1;
        double run_end = 0.0, send_end = 0.0;
        int finished = 0;
        while (finished < n) {
            int acted = 0;
            /* completions at the current time: their successors become ready, sends among them are requested */
            while (k < R && net_end <= now) {
                int v = recv_ids[ord[k]];
                if (net_end > m) m = net_end;
                for (int e = sptr[v]; e < sptr[v + 1]; ++e) {
                    const int s2 = sidx[e];
                    if (--waiting[s2] == 0) {
                        if (is_send[s2]) fresh[n_fresh++] = s2;
                        else heap_push(&h, pick_key ? pick_key[s2] : s2, s2);
                    }
                }
                ++finished; ++k; acted = 1;
                if (k < R) net_end = net_end + rt[ord[k]];
            }
            if (running >= 0 && run_end <= now) {
                int v = running;
                if (run_end > m) m = run_end;
                for (int e = sptr[v]; e < sptr[v + 1]; ++e) {
                    const int s2 = sidx[e];
                    if (--waiting[s2] == 0) {
                        if (is_send[s2]) fresh[n_fresh++] = s2;
                        else heap_push(&h, pick_key ? pick_key[s2] : s2, s2);
                    }
                }
                running = -1; ++finished; acted = 1;
            }
            if (sending >= 0 && send_end <= now) {
                if (send_end > m) m = send_end;
                sending = -1; ++finished; acted = 1;
            }
            if (running < 0 && h.len > 0) {
                running = heap_pop(&h);
                run_end = now + time[running];
                acted = 1;
            }
            if (acted) continue;     /* something may complete or start at this same instant */
            /* the instant is over: its requests join the queue by op id, and an idle uplink starts the next one */
            if (n_fresh > 0) {
                for (int a = 1; a < n_fresh; ++a) {                 /* insertion sort by op id */
                    const int v = fresh[a];
                    int c = a;
                    while (c > 0 && fresh[c - 1] > v) { fresh[c] = fresh[c - 1]; --c; }
                    fresh[c] = v;
                }
                for (int a = 0; a < n_fresh; ++a) queue[q_tail++] = fresh[a];
                n_fresh = 0;
            }
            if (sending < 0 && q_head < q_tail) {
                sending = queue[q_head++];
                send_end = now + time[sending];
                continue;            /* a send of zero time completes at this instant */
            }
            /* advance to the next completion */
            double nxt = HUGE_VAL;
            if (k < R) nxt = net_end;
            if (running >= 0 && run_end < nxt) nxt = run_end;
            if (sending >= 0 && send_end < nxt) nxt = send_end;
            if (nxt == HUGE_VAL) { rc = ORACLE_ERR_CYCLE; break; }   /* ops left that can never start */
            now = nxt;
        }
        double U = sum_c + sum_r + sum_s;
        double L = sum_c > sum_r ? sum_c : sum_r;
        if (sum_s > L) L = sum_s;
        makespan[b] = m;
        eff[b] = (U == L) ? 1.0 : (U - m) / (U - L);
        if (U_out) U_out[b] = U;
        if (L_out) L_out[b] = L;
        if (S_out) S_out[b] = (U == L || L == 0.0) ? 0.0 : (U - L) / L;
    }
    free(ri); free(sptr); free(sidx); free(fill); free(waiting); free(is_send); free(queue); free(fresh);
    free(time); free(h.key); free(h.op);
    return rc;
}

/* ------------------------------------------------------------------------
 * The same iteration with several channels (Sec. 4.1: a device has one channel per
 * parameter server it talks to; Sec. 5.1: each channel carries one transfer at a time, in
 * priority order).  Recv i uses channel channel_of_recv[i]; every channel serves its own
 * recvs back-to-back from t = 0, in the order in which they appear in `order`, and the
 * channels run side by side.  The compute device is as in oracle_simulate.
 *   L = max(sum of compute times, largest per-channel sum of recv times)   (Eq. 2: one
 *   term per resource); everything else as in oracle_simulate.
 * ---------------------------------------------------------------------- */
int oracle_simulate_channels(int n, const int32_t *row_ptr, const int32_t *col_idx, int R,
                             const int32_t *recv_ids, int n_channels, const int32_t *channel_of_recv,
                             int B, const int32_t *order, int order_stride, const double *op_time,
                             const double *recv_time, double *makespan, double *eff,
                             double *U_out, double *L_out, double *S_out)
{
    if (n_channels < 1) return ORACLE_ERR_ARG;
    for (int i = 0; i < R; ++i)
        if (channel_of_recv[i] < 0 || channel_of_recv[i] >= n_channels) return ORACLE_ERR_ARG;
    const int N = n - R, C = n_channels;
    const size_t n1 = (size_t)(n > 0 ? n : 1), r1 = (size_t)(R > 0 ? R : 1);
    int32_t *ri = recv_index_of_op(n, R, recv_ids);
    int32_t *sptr = (int32_t *)calloc(n1 + 1, sizeof(int32_t));
    int32_t *sidx = (int32_t *)malloc((size_t)(row_ptr[n] > 0 ? row_ptr[n] : 1) * sizeof(int32_t));
    int32_t *fill = (int32_t *)malloc(n1 * sizeof(int32_t));
    int32_t *waiting = (int32_t *)malloc(n1 * sizeof(int32_t));
    double *time = (double *)malloc(n1 * sizeof(double));
    heap_t h = { (int32_t *)malloc(n1 * sizeof(int32_t)), (int32_t *)malloc(n1 * sizeof(int32_t)), 0 };
    /* per channel: its queue of recv indices (a slice of `queue`), the next one to complete,
       the completion time of the transfer in progress, the sum of its transfer times */
    int32_t *queue = (int32_t *)malloc(r1 * sizeof(int32_t));
    int32_t *qbeg = (int32_t *)malloc(((size_t)C + 1) * sizeof(int32_t));
    int32_t *qnext = (int32_t *)malloc((size_t)C * sizeof(int32_t));
    double *qend = (double *)malloc((size_t)C * sizeof(double));
    double *qsum = (double *)malloc((size_t)C * sizeof(double));
    if (!ri || !sptr || !sidx || !fill || !waiting || !time || !h.key || !h.op || !queue || !qbeg || !qnext ||
        !qend || !qsum)
        return ORACLE_ERR_MEM;
    for (int v = 0; v < n; ++v)
        for (int e = row_ptr[v]; e < row_ptr[v + 1]; ++e) sptr[col_idx[e] + 1]++;
    for (int v = 0; v < n; ++v) sptr[v + 1] += sptr[v];
    for (int v = 0; v < n; ++v) fill[v] = sptr[v];
    for (int v = 0; v < n; ++v)
        for (int e = row_ptr[v]; e < row_ptr[v + 1]; ++e) sidx[fill[col_idx[e]]++] = v;

    int rc = ORACLE_OK;
    for (int b = 0; b < B && rc == ORACLE_OK; ++b) {
        const double *ot = op_time + (size_t)b * N, *rt = recv_time + (size_t)b * R;
        const int32_t *ord = order + (size_t)b * order_stride;
        int j = 0;
        double sum_c = 0.0, sum_r = 0.0;
        for (int v = 0; v < n; ++v) {
            if (ri[v] >= 0) { time[v] = rt[ri[v]]; sum_r += time[v]; }
            else { time[v] = ot[j++]; sum_c += time[v]; }
            waiting[v] = row_ptr[v + 1] - row_ptr[v];
        }
        /* the queues: channel c takes its recvs in the order of `ord` */
        int pos = 0;
        for (int c = 0; c < C; ++c) {
            qbeg[c] = pos;
            qsum[c] = 0.0;
            for (int k = 0; k < R; ++k)
                if (channel_of_recv[ord[k]] == c) { queue[pos++] = ord[k]; qsum[c] += rt[ord[k]]; }
            qnext[c] = qbeg[c];
            qend[c] = (pos > qbeg[c]) ? rt[queue[qbeg[c]]] : 0.0;
        }
        qbeg[C] = pos;
        h.len = 0;
        for (int v = 0; v < n; ++v)
            if (ri[v] < 0 && waiting[v] == 0) heap_push(&h, v, v);

        double now = 0.0, m = 0.0;
        int running = -1;
        double run_end = 0.0;
        int finished = 0;
        while (finished < n) {
            int acted = 0;
            for (int c = 0; c < C; ++c)
                while (qnext[c] < qbeg[c + 1] && qend[c] <= now) {
                    int v = recv_ids[queue[qnext[c]]];
                    if (qend[c] > m) m = qend[c];
                    for (int e = sptr[v]; e < sptr[v + 1]; ++e)
                        if (--waiting[sidx[e]] == 0) heap_push(&h, sidx[e], sidx[e]);
                    ++finished; ++qnext[c]; acted = 1;
                    if (qnext[c] < qbeg[c + 1]) qend[c] = qend[c] + rt[queue[qnext[c]]];
                }
            if (running >= 0 && run_end <= now) {
                int v = running;
                if (run_end > m) m = run_end;
                for (int e = sptr[v]; e < sptr[v + 1]; ++e)
                    if (--waiting[sidx[e]] == 0) heap_push(&h, sidx[e], sidx[e]);
                running = -1; ++finished; acted = 1;
            }
            if (running < 0 && h.len > 0) {
                running = heap_pop(&h);
                run_end = now + time[running];
                acted = 1;
            }
            if (acted) continue;
            double nxt = HUGE_VAL;
            for (int c = 0; c < C; ++c)
                if (qnext[c] < qbeg[c + 1] && qend[c] < nxt) nxt = qend[c];
            if (running >= 0 && run_end < nxt) nxt = run_end;
            if (nxt == HUGE_VAL) { rc = ORACLE_ERR_CYCLE; break; }
            now = nxt;
        }
        double U = sum_c + sum_r;
        double L = sum_c;
        for (int c = 0; c < C; ++c) if (qsum[c] > L) L = qsum[c];
        makespan[b] = m;
        eff[b] = (U == L) ? 1.0 : (U - m) / (U - L);
        if (U_out) U_out[b] = U;
        if (L_out) L_out[b] = L;
        if (S_out) S_out[b] = (U == L || L == 0.0) ? 0.0 : (U - L) / L;
    }
    free(ri); free(sptr); free(sidx); free(fill); free(waiting); free(time); free(h.key); free(h.op);
    free(queue); free(qbeg); free(qnext); free(qend); free(qsum);
    return rc;
}

/* ---------------------------------------------------------------------------
 * Straggler effect (Sec. 6, "Straggler Effect"): workers that run one synchronous
 * iteration together all wait for the slowest; the effect is the longest wait of any
 * worker as a fraction of the iteration time.  Here the workers of group g are the w
 * consecutive samples g*w .. g*w + w - 1 with makespans m_i:
 *     iteration time T = max m_i,  longest wait = T - min m_i,  effect = (T - min m_i) / T,
 * 0 when T == 0.  Groups: B / w (whole groups only).
 * ------------------------------------------------------------------------- */
int oracle_straggler(int B, int w, const double *makespan, double *out)
{
    if (B < 0 || w < 1) return -2;
    if (B > 0 && (!makespan || !out)) return -1;
    for (int g = 0; g < B / w; ++g) {
        double mx = makespan[(size_t)g * w], mn = mx;
        for (int i = 1; i < w; ++i) {
            const double m = makespan[(size_t)g * w + i];
            if (m > mx) mx = m;
            if (m < mn) mn = m;
        }
        out[g] = mx > 0.0 ? (mx - mn) / mx : 0.0;
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Time oracle estimator (Sec. 5, "Time Oracle"): every op is measured in several runs and
 * the smallest measurement is taken as its time.  runs [n_runs][n] -> time [n].
 * ------------------------------------------------------------------------- */
int oracle_time_oracle_min(int n_runs, long long n, const double *runs, double *time)
{
    if (n_runs < 1 || n < 0) return -2;
    if (n > 0 && (!runs || !time)) return -1;
    for (long long i = 0; i < n; ++i) {
        double m = runs[i];
        for (int k = 1; k < n_runs; ++k)
            if (runs[(size_t)k * (size_t)n + (size_t)i] < m) m = runs[(size_t)k * (size_t)n + (size_t)i];
        time[i] = m;
    }
    return 0;
}


/* ---------------------------------------------------------------------------
 * Order search with the iteration of oracle_simulate as its measure (Sec. 3.1: the best
 * order is a job-shop problem and NP-hard, so TIC and TAC are heuristics; Sec. 4.3: the
 * comparator extends the two-recv rule by an induction that need not hold in general).  To
 * see how far a heuristic order is from a better one, every sample climbs from its start
 * order through a list of proposed exchanges that the caller draws:
 *     cur = start order, m_cur = makespan(cur)
 *     for each move (a, b), in the order given:
 *         positions a and b of cur are exchanged; m = makespan of that order
 *         if m < m_cur the exchange is kept (m_cur = m), else it is undone
 * A move with a == b or a position outside 0 .. R-1 changes nothing.  The moves are the same
 * for every sample.
 *   order  [R] shared (order_stride = 0) or [B][R] (order_stride = R): the start orders
 *   moves  [n_moves][2]
 *   best_order [B][R], best_makespan [B]: the order a sample ends with and its makespan
 *   start_makespan [B], n_accepted [B]: may be NULL
 * ------------------------------------------------------------------------- */
int oracle_order_search(int n, const int32_t *row_ptr, const int32_t *col_idx, int R, const int32_t *recv_ids,
                        int B, const int32_t *order, int order_stride, int n_moves, const int32_t *moves,
                        const double *op_time, const double *recv_time, int32_t *best_order,
                        double *best_makespan, double *start_makespan, int32_t *n_accepted)
{
    if (B < 0 || n_moves < 0) return ORACLE_ERR_ARG;
    const int N = n - R;
    int rc = ORACLE_OK;
    for (int b = 0; b < B && rc == ORACLE_OK; ++b) {
        const double *ot = op_time + (size_t)b * N, *rt = recv_time + (size_t)b * R;
        int32_t *cur = best_order + (size_t)b * R;
        for (int k = 0; k < R; ++k) cur[k] = order[(size_t)b * order_stride + k];
        double m_cur, e;
        rc = oracle_simulate(n, row_ptr, col_idx, R, recv_ids, 1, cur, 0, ot, rt, NULL, &m_cur, &e, NULL, NULL, NULL);
        if (rc != ORACLE_OK) break;
        if (start_makespan) start_makespan[b] = m_cur;
        int acc = 0;
        for (int i = 0; i < n_moves && rc == ORACLE_OK; ++i) {
            const int pa = moves[2 * i], pb = moves[2 * i + 1];
            if (pa < 0 || pa >= R || pb < 0 || pb >= R || pa == pb) continue;
            int32_t x = cur[pa]; cur[pa] = cur[pb]; cur[pb] = x;
            double m;
            rc = oracle_simulate(n, row_ptr, col_idx, R, recv_ids, 1, cur, 0, ot, rt, NULL, &m, &e, NULL, NULL, NULL);
            if (rc == ORACLE_OK && m < m_cur) { m_cur = m; ++acc; }
            else { x = cur[pa]; cur[pa] = cur[pb]; cur[pb] = x; }
        }
        best_makespan[b] = m_cur;
        if (n_accepted) n_accepted[b] = acc;
    }
    return rc;
}
