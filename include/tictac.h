/*
 * tictac.h -- C ABI of libtictac: the scheduling math of "TicTac: Accelerating
 * Distributed Deep Learning with Communication Scheduling" (arXiv 1803.03288)
 * as hand-written HIP kernels for gfx950 (MI355X).
 *
 * Given the worker's computational DAG, whose communication ops (recv) are its
 * roots (Sec. 2.2), and a time oracle Time(op) (Sec. 3.1), the library computes
 *   1. op.dep, the set of recvs every op depends on       (Sec. 4.1)
 *   2. the timing-independent priorities, TIC              (Sec. 4.2, Algorithm 2)
 *   3. the timing-aware order, TAC, for a batch of
 *      timing samples                                      (Sec. 4.3, Algorithm 3)
 *   4. makespan, its bounds, Scheduling Efficiency and
 *      Speedup of an iteration under a transfer order,
 *      for a batch of timing samples                       (Sec. 3.2, Eq. 1-4)
 *   5. the same with several channels side by side         (Sec. 4.1, 5.1)
 *   6. the straggler effect of groups of workers           (Sec. 6)
 *   7. the time oracle estimate from measured runs         (Sec. 5)
 *   8. a search for better orders by proposed exchanges,
 *      measured by 4                                       (Sec. 3.1, 4.3)
 * 3 and 4 also take the timing samples as float32 arrays (tictac_simulate_f32,
 * tictac_tac_simulate_f32).
 *
 * Conventions
 *   - "host" pointers are ordinary memory, "device" pointers are HIP device
 *     memory of the current device.  The library never takes ownership of a
 *     caller's buffer; it only uses it for the duration of the stream-ordered
 *     call.  Everything a tictac_dag owns is released by tictac_dag_free.
 *   - Ops are numbered 0..n_ops-1 in any order.  recv i is the op recv_ids[i];
 *     bit i of a dependency bitset (bit i & 63 of 64-bit word i >> 6) stands
 *     for it.  W = ceil(n_recv / 64) words per bitset.
 *   - N = n_ops - n_recv compute ops.  Column j of an op_time row is the j-th
 *     compute op in ascending op id; column i of a recv_time row is recv i.
 *     Times are float64 seconds, finite and >= 0 (not checked on the device).
 *   - Every function returns TICTAC_OK (0) or a negative tictac_status; on an
 *     error nothing is written to the outputs and tictac_last_error() holds a
 *     message.  No exception or abort crosses this boundary.
 *   - Calls taking a stream are asynchronous on it unless stated otherwise.
 *     Calls on the same tictac_dag must not overlap in time on different
 *     streams (the handle owns one scratch workspace).
 */
#ifndef TICTAC_H
#define TICTAC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tictac_status {
    TICTAC_OK = 0,
    TICTAC_ERR_NULL = -1,          /* a required pointer is NULL */
    TICTAC_ERR_BAD_CSR = -2,       /* row_ptr not monotone from 0, or an id out of range, or negative size */
    TICTAC_ERR_CYCLE = -3,         /* the graph is not acyclic */
    TICTAC_ERR_RECV_NOT_ROOT = -4, /* a recv op has predecessors (Sec. 2.2: recvs are roots) */
    TICTAC_ERR_DUP_RECV = -5,      /* recv_ids holds an op twice */
    TICTAC_ERR_BAD_ORDER = -6,     /* order_stride is neither 0 nor n_recv, a channel index is out of range, or an order is no permutation */
    TICTAC_ERR_HIP = -7,           /* a HIP runtime call failed */
    TICTAC_ERR_NO_MEM = -8,        /* host or device allocation failed */
    TICTAC_ERR_UNSUPPORTED = -9    /* size beyond what the kernels are built for */
} tictac_status;

/* TIC priority of a recv that no multi-dependency op consumes (M+ = +infinity). */
#define TICTAC_PRIO_INF INT32_MAX

typedef struct tictac_dag tictac_dag; /* opaque; owns device copies of the graph, op.dep and derived tables */
typedef void *tictac_stream;          /* a hipStream_t; NULL = the default stream */

/*
 * Sec. 4.1, Communication Dependency.  Validates the graph, uploads it, and
 * computes dep[v] = ({i} if v is recv i) U (union of dep[u] over predecessors u)
 * for every op on the device.
 *   pred_row_ptr [n_ops+1], pred_col_idx [E]  host: predecessors of op v are
 *       pred_col_idx[pred_row_ptr[v] .. pred_row_ptr[v+1])
 *   recv_ids [n_recv]                         host
 *   *out receives a new handle (free with tictac_dag_free).
 * Synchronises with the stream before returning (the handle is complete).
 * n_recv = 0 and n_ops = 0 are valid.
 */
int tictac_build_deps(int32_t n_ops, const int32_t *pred_row_ptr, const int32_t *pred_col_idx,
                      int32_t n_recv, const int32_t *recv_ids, tictac_stream stream, tictac_dag **out);

/* Sizes of a handle; any output pointer may be NULL.  n_levels = length of the
 * longest path, in ops.  n_classes = number of distinct dep sets among the compute
 * ops (ops with the same set form the unit the TAC and simulation kernels work on). */
int tictac_dag_info(const tictac_dag *dag, int32_t *n_ops, int32_t *n_recv, int32_t *words,
                    int32_t *n_levels, int32_t *n_classes);

/* Borrowed device pointer to op.dep: uint64 [n_ops][W], row-major, row = op id.
 * Valid until tictac_dag_free.  NULL when n_ops * W == 0. */
int tictac_dag_deps(const tictac_dag *dag, const uint64_t **dep_device);

/* Copies op.dep ([n_ops][W], as above) into a caller-owned device buffer, asynchronously
 * on the stream. */
int tictac_dag_copy_deps(const tictac_dag *dag, uint64_t *dst_device, tictac_stream stream);

/* Runs the propagation kernel again on the handle's graph, overwriting op.dep with the
 * same values (for timing the kernel without the host-side part of tictac_build_deps).
 * Asynchronous on the stream. */
int tictac_dag_recompute_deps(tictac_dag *dag, tictac_stream stream);

/* The same for n_dags handles at once (Sec. 4.1, the propagation of tictac_build_deps).  One graph is a
 * chain of dependent levels and leaves most of the chip idle; handles of graphs of one shape (as several
 * handles of one graph are) are propagated side by side by a single launch, any others one after the
 * other.  Every handle's op.dep is overwritten with the same values.  Asynchronous on the stream; the
 * handles must not be used by other calls meanwhile. */
int tictac_dag_recompute_deps_batch(tictac_dag *const *dags, int32_t n_dags, tictac_stream stream);

/* Sec. 3.2 takes the transfer order as a permutation of the recvs.  tictac_simulate, tictac_simulate_f32,
 * tictac_simulate_channels and tictac_order_search are asynchronous and cannot return what only the device
 * sees, so each of them first checks, on the device, every order it is given (each entry in 0 .. n_recv-1,
 * none twice) and raises a flag of the handle when one fails; the outputs of such a sample are unspecified
 * (entries out of range are skipped, nothing is read or written out of bounds).  This call waits for the
 * stream, returns TICTAC_ERR_BAD_ORDER when the flag was raised since the last such call, TICTAC_OK otherwise,
 * and lowers the flag. */
int tictac_dag_check_orders(tictac_dag *dag, tictac_stream stream);

int tictac_dag_free(tictac_dag *dag);

/*
 * Sec. 4.2, Algorithm 2 (TIC): the property update of Algorithm 1 with every recv
 * outstanding and the General Time Oracle (recv = 1, others = 0), in integers.
 *   prio  [n_recv] device: M+ of each recv = the smallest |op.dep| over compute ops
 *         whose dep holds the recv and at least one more; TICTAC_PRIO_INF if none
 *   order [n_recv] device: recv indices sorted by (prio, index)   (may be NULL)
 *   rank  [n_recv] device: inverse of order = the number of transfers that go
 *         before recv i, the normalised priority of Sec. 5.1      (may be NULL)
 */
int tictac_tic_priority(const tictac_dag *dag, int32_t *prio, int32_t *order, int32_t *rank,
                        tictac_stream stream);

/*
 * Sec. 4.3, Algorithm 3 (TAC) for B timing samples.  Per sample: all recvs start
 * outstanding; n_recv times, the properties M, P, M+ of Algorithm 1 are taken for
 * the outstanding set, the recv that is minimal under the comparator is selected
 * (ascending-index scan that replaces the current best only by a recv that strictly
 * precedes it; A precedes B when min{P_B, M_A} < min{P_A, M_B}, and when those are
 * equal, when M+_A < M+_B) and removed.
 *   op_time [B][N], recv_time [B][n_recv]   device, row-major
 *   order [B][n_recv] device: step -> recv index
 *   rank  [B][n_recv] device: recv index -> step            (may be NULL)
 *   sel_P, sel_Mplus [B][n_recv] device: P and M+ of each recv in the round that
 *         selected it (+infinity when no M+ exists)          (each may be NULL)
 * B = 0 is valid.
 */
int tictac_tac_priority(const tictac_dag *dag, int32_t B, const double *op_time, const double *recv_time,
                        int32_t *order, int32_t *rank, double *sel_P, double *sel_Mplus,
                        tictac_stream stream);

/*
 * Sec. 3.2: one iteration under a transfer order, for B timing samples.  One
 * channel serves the recvs back to back from t = 0 in the given order (Sec. 5.1:
 * one active transfer per channel, released in priority order); one compute
 * device runs one op at a time and never idles while an op is ready.
 *   order: device, recv indices.  order_stride = 0: one order [n_recv] for every
 *          sample; order_stride = n_recv: order [B][n_recv].  Must be a
 *          permutation of 0..n_recv-1 (checked on the device: tictac_dag_check_orders).
 *   makespan [B] device: finish time of the last op
 *   eff      [B] device: E = (U - m) / (U - L) (Eq. 3); 1 when U == L
 *   U, L, S  [B] device, each may be NULL: U = sum of all times (Eq. 1),
 *          L = max(sum of compute times, sum of transfer times) (Eq. 2),
 *          S = (U - L) / L (Eq. 4); 0 when U == L or L == 0
 */
int tictac_simulate(const tictac_dag *dag, int32_t B, const int32_t *order, int32_t order_stride,
                    const double *op_time, const double *recv_time, double *makespan, double *eff,
                    double *U, double *L, double *S, tictac_stream stream);

/*
 * Algorithm 3 followed by the iteration under the order it produced, in one pass
 * over the timing samples (each op_time row is read once).  Outputs as in
 * tictac_tac_priority and tictac_simulate; order must not be NULL, every other
 * output may be.
 */
int tictac_tac_simulate(const tictac_dag *dag, int32_t B, const double *op_time, const double *recv_time,
                        int32_t *order, int32_t *rank, double *sel_P, double *sel_Mplus,
                        double *makespan, double *eff, double *U, double *L, double *S,
                        tictac_stream stream);

/*
 * tictac_tac_simulate for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The call allocates nothing, neither on the
 * first call nor later: the one flag per sample that its kernels pass between them lives in an array
 * that is part of the library itself (4 MiB per GPU, held until the process ends).
 *   - at most 2^20 samples per call, and only graphs that the wave-per-sample kernels serve (at
 *     most 384 recvs and 512 classes of compute ops with identical dependency sets); anything else:
 *     TICTAC_ERR_UNSUPPORTED and nothing is written;
 *   - every call on one GPU uses the same array, so calls that overlap in time on one GPU (on
 *     different streams or from different threads) race; calls on one stream do not;
 *   - no per-round outputs (sel_P, sel_Mplus); everything else as in tictac_tac_simulate, and the
 *     results are the same.
 */
int tictac_tac_simulate_noalloc(const tictac_dag *dag, int32_t B, const double *op_time, const double *recv_time,
                                int32_t *order, int32_t *rank, double *makespan, double *eff, double *U, double *L,
                                double *S, tictac_stream stream);

/*
 * The two calls above with the timing arrays stored as float32 (half the bytes of the pass over
 * the samples).  Every value is converted to float64 when it is loaded and all sums and
 * comparisons are float64, so the results are those of the float64 calls on the converted values:
 * orders are the TAC orders of the rounded times, and makespans differ from those of unrounded
 * float64 times by the rounding of the inputs (below 1e-6 relative; the float32 bound is 1e-3).
 *   op_time [B][N], recv_time [B][n_recv]   device, float32, row-major
 * Everything else as in tictac_simulate and tictac_tac_simulate (outputs are float64).
 */
int tictac_simulate_f32(const tictac_dag *dag, int32_t B, const int32_t *order, int32_t order_stride,
                        const float *op_time, const float *recv_time, double *makespan, double *eff,
                        double *U, double *L, double *S, tictac_stream stream);
int tictac_tac_simulate_f32(const tictac_dag *dag, int32_t B, const float *op_time, const float *recv_time,
                            int32_t *order, int32_t *rank, double *sel_P, double *sel_Mplus,
                            double *makespan, double *eff, double *U, double *L, double *S,
                            tictac_stream stream);

/*
 * tictac_simulate with several channels (Sec. 4.1: a device has one channel per parameter
 * server it talks to; Sec. 5.1: every channel carries one transfer at a time, in priority
 * order).  Recv i uses channel channel_of_recv[i]; every channel serves its own recvs back to
 * back from t = 0, in the order in which they appear in `order`, and the channels run side
 * by side.  L counts every channel as a resource: L = max(sum of compute times, largest
 * per-channel sum of transfer times).  Everything else as in tictac_simulate.
 *   n_channels       1 .. 64
 *   channel_of_recv  HOST, [n_recv], values in 0 .. n_channels-1 (TICTAC_ERR_BAD_ORDER otherwise)
 * Graphs with more than 512 recvs or more than 512 classes of compute ops with identical
 * dependency sets: TICTAC_ERR_UNSUPPORTED.
 */
int tictac_simulate_channels(const tictac_dag *dag, int32_t B, int32_t n_channels, const int32_t *channel_of_recv,
                             const int32_t *order, int32_t order_stride, const double *op_time,
                             const double *recv_time, double *makespan, double *eff, double *U, double *L,
                             double *S, tictac_stream stream);

/*
 * Sec. 2.2: in the worker's graph the recv ops are the roots and the send ops the leaves (they carry results
 * back to the parameter servers).  One iteration under a transfer order as in tictac_simulate, with the ops
 * send_ids as sends: a send's time (its column of op_time) is a transfer time on the uplink, a third
 * resource beside the compute device and the channel of the recvs, which carries one transfer at a time
 * (Sec. 5.1) and serves the sends first come first served, a send being requested at the instant its last
 * predecessor finishes.  The finish times of single compute ops matter here, so the pick of the compute
 * device is part of the definition: whenever it is idle it starts the ready compute op of lowest op id.
 *   send_ids  HOST, [n_send] op ids: compute ops without successors, each once (TICTAC_ERR_BAD_CSR
 *             otherwise).  n_send = 0 gives the results of tictac_simulate.  The tables for a send set are
 *             built at the first call with it (the call then waits for the stream once).
 *   makespan  finish of the last op, sends included;  U = sum of all times (Eq. 1);
 *   L = max(compute times without the sends, transfer times of the recvs, transfer times of the sends)
 *   (Eq. 2: one term per resource);  E, S from them (Eq. 3, 4).  U, L, S may be NULL.
 * Orders are checked as for tictac_simulate (tictac_dag_check_orders).  Graphs whose per-sample state
 * (2 bytes per op, 12 per recv) exceeds the LDS of a compute unit: TICTAC_ERR_UNSUPPORTED.  B = 0 is valid.
 */
int tictac_simulate_sends(const tictac_dag *dag, int32_t B, int32_t n_send, const int32_t *send_ids,
                          const int32_t *order, int32_t order_stride, const double *op_time,
                          const double *recv_time, double *makespan, double *eff, double *U, double *L, double *S,
                          tictac_stream stream);

/*
 * Sec. 6, "Straggler Effect": workers that run one synchronous iteration together wait
 * for the slowest one; the effect is the longest wait of any worker as a fraction of the
 * iteration time.  The workers of group g are the w consecutive samples g*w .. g*w+w-1:
 *     straggler[g] = (max m_i - min m_i) / max m_i   over the group, 0 when the maximum is 0.
 *   makespan  [B]      device (as written by tictac_simulate / tictac_tac_simulate)
 *   straggler [B / w]  device; only whole groups are formed, trailing samples are not used
 * w >= 1 (TICTAC_ERR_UNSUPPORTED otherwise); B = 0 is valid.
 */
int tictac_straggler_effect(int32_t B, int32_t w, const double *makespan, double *straggler,
                            tictac_stream stream);

/*
 * Sec. 5, "Time Oracle": every op is measured in several runs and the smallest measurement
 * is taken as its time.
 *   runs [n_runs][n]  device, row-major (one row per measured run; n may be a whole batch
 *                     of timing rows, B * N or B * n_recv values)
 *   time [n]          device
 * n_runs >= 1 and n >= 0 (TICTAC_ERR_UNSUPPORTED otherwise); NaN measurements are ignored
 * where another run has a number.
 */
int tictac_time_oracle_min(int32_t n_runs, int64_t n, const double *runs, double *time, tictac_stream stream);

/*
 * Order search with the iteration of tictac_simulate as its measure.  Sec. 3.1: finding the best
 * order is a job-shop problem and NP-hard, TIC and TAC are heuristics; Sec. 4.3: the comparator
 * extends the two-recv rule by an induction that need not hold in general.  Every sample climbs
 * from its start order through the proposed exchanges, which are the same for all samples:
 *     cur = start order, m_cur = makespan(cur)
 *     for every move (a, b), in the order given: exchange positions a and b of cur and take the
 *     makespan m of that order; keep the exchange when m < m_cur (then m_cur = m), else undo it.
 * A move with a == b or with a position outside 0 .. n_recv-1 is skipped.
 *   order  device, start orders: order_stride = 0: one order [n_recv] for every sample;
 *          order_stride = n_recv: [B][n_recv].  Must be permutations (checked on the device: tictac_dag_check_orders).
 *   moves  device, int32 [n_moves][2]; n_moves >= 0
 *   best_order     [B][n_recv] device: the order every sample ends with
 *   best_makespan  [B] device: its makespan, equal to what tictac_simulate gives for it
 *   start_makespan [B] device, may be NULL: makespan of the start order
 *   n_accepted     [B] device, may be NULL: number of exchanges that were kept
 * Graphs without a recv, with more than 512 recvs or with more than 512 classes of compute ops
 * with identical dependency sets: TICTAC_ERR_UNSUPPORTED.  B = 0 is valid.
 */
int tictac_order_search(const tictac_dag *dag, int32_t B, const int32_t *order, int32_t order_stride,
                        int32_t n_moves, const int32_t *moves, const double *op_time, const double *recv_time,
                        int32_t *best_order, double *best_makespan, double *start_makespan, int32_t *n_accepted,
                        tictac_stream stream);

/* Message of the last error on the calling thread; valid until its next call. */
const char *tictac_last_error(void);

/* Library version, "major.minor". */
const char *tictac_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TICTAC_H */
