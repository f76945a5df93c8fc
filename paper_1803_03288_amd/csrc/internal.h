// Internal declarations of libtictac (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "tictac.h"

namespace tictac {

constexpr int kK1Rpt = 4;             // positions per thread group and chunk of the node kernel

void set_error(const char *fmt, ...);

// Everything a handle owns.  Device arrays are sized exactly; empty ones are NULL.
struct Dag {
    int32_t n = 0, R = 0, W = 0, N = 0, E = 0;
    int32_t n_levels = 0;
    int32_t max_level_width = 0;
    int device = 0;

    int32_t *d_recv_of_op = nullptr;// [n]  recv index or -1

    // Condensed graph used by the propagation.  A compute op whose only predecessor is a
    // compute op has that op's dep; every other compute op is a *node*.  Nodes are sorted
    // by level (longest path counted in nodes) into positions 0..M-1.
    int32_t M = 0;                  // number of nodes
    int32_t n_node_levels = 0;
    int32_t max_node_level_width = 0;
    struct NodeRec {                // 32 bytes, one per position
        int32_t in[6];              // first inputs: q >= 0 node position, ~i < 0 recv i, INT32_MIN none
        int32_t op;                 // op id of the node
        int32_t ovf_beg;            // -1, or: ovf_idx[ovf_beg] further inputs follow at ovf_idx[ovf_beg + 1 ..]
    };
    NodeRec *d_nodes = nullptr;     // [M]
    int32_t *d_ovf_idx = nullptr;   // inputs beyond the fourth
    int32_t *d_nlvl_ptr = nullptr;  // [n_node_levels + 1] positions of each level
    // launch shape of the node kernel and its chunks of consecutive levels (at most 4 k1_threads / k1_wc
    // positions and 64 levels each): chunk_end[lv] = first level after the chunk that starts at lv
    int32_t k1_wc = 0, k1_threads = 0;
    int32_t *d_chunk_end = nullptr; // [n_node_levels]
    // The same nodes decoded for the chunked kernel, which keeps the rows of the last k1_ring
    // positions (a power of two) in an LDS ring of k1_wc words per row, plus one all-zero row
    // after it.  A node with at most four node inputs, all of them still in the ring when its
    // level is computed, and at most two recv inputs, is "fast": in[] are byte offsets of its
    // input rows in the ring (unused: the zero row), rcv[] its recv indices (-1 none).  Any
    // other node has only zero rows and -1 here, and all its inputs (in the encoding of
    // NodeRec::in) at fovf[ovf + 1 ..], fovf[ovf] of them.
    struct FastRec {                // 32 bytes, one per position
        int32_t in[4];
        int32_t rcv[2];
        int32_t op;                 // op id of the node
        int32_t ovf;                // -1 for a fast node
    };
    int32_t k1_ring = 0;
    bool k1_wave = false;       // narrow levels, everything in LDS: one wave per slice, k1_ring = M rows, no ring
    FastRec *d_frecs = nullptr;     // [M] (not built when a level is wider than one pass)
    int32_t *d_fovf = nullptr;
    int32_t fovf_len = 0;
    // Level-major form of the same records for graphs whose levels fill most of a pass: level l
    // owns the slots l * P .. l * P + P - 1 (P = k1_threads / k1_wc), slot l * P + j holds the j-th node
    // of the level, the others a record with op = -1.  Positions, ring offsets and the input
    // lists (lfovf) count slots.  Not built (NULL) when the padding would cost too much or the
    // graph takes another kernel.
    FastRec *d_lrecs = nullptr;     // [n_node_levels * P]
    int32_t *d_lfovf = nullptr;
    int32_t lfovf_len = 0;
    int32_t k1_lring = 0;           // slots held in LDS (a power of two, at least 16 levels)
    // The level-major records of the kernel with 64-byte slices (four lanes per slot, P = k1_threads / 4):
    // ring slots of up to four input rows in 16-bit halves (unused: the zero row, slot k1_lring), two recv indices
    // likewise (0xffff none), the op id (-1: no node in the slot; -2: a copy node, which hands a row on inside the
    // ring and stores nothing).  Any other node: in01 = 0xffffffff and in23 = the start of its list in lfovf.
    struct QuadRec {                // 16 bytes, one per slot
        uint32_t in01, in23, rcv01;
        int32_t op;
    };
    int32_t k1_q_ring = 0, k1_q_threads = 0;   // slots held in LDS (0: no such records), threads of a workgroup
    QuadRec *d_qrecs = nullptr;     // [n_node_levels * P]
    int32_t *d_qfovf = nullptr;     // the lists of the other nodes, as lfovf
    int32_t qfovf_len = 0;
    uint64_t *d_k1_q_sink = nullptr;    // [slices * k1_q_threads][2]
    int32_t *d_q_copied = nullptr;  // [n_q_copied][2] the copied rows (see d_copied) that found no free slot of these records
    int32_t n_q_copied = 0;
    uint64_t *d_k1_sink = nullptr;  // [slices * k1_threads] one word per thread: where a thread without a node stores
    int32_t *d_op_of_col = nullptr; // [N] op id of every op_time column
    int32_t *d_cls_first_op = nullptr;  // [C] (graphs grouped on the device) the op whose row is the class's
    int32_t *d_bad_order = nullptr; // one flag: an order handed to a simulation or a search was no permutation
    // the ops whose rows are copies, as pairs (op, ~i for recv i or the op id of the node whose row it has)
    int32_t *d_copied = nullptr;    // [n_copied][2]
    int32_t n_copied = 0;
    // op.dep
    uint64_t *d_dep = nullptr;      // [n][W]

    // classes of compute ops with identical dep rows (rows with no recv: class 0 if any)
    int32_t C = 0;                  // number of classes (after splitting long ones)
    int32_t C_distinct = 0;         // number of distinct non-empty rows
    int32_t Cpad = 0;               // C rounded up to a multiple of 64
    int64_t cls_nnz = 0;            // total number of set bits over class rows
    uint64_t *d_cls_dep = nullptr;  // [C][W]
    uint64_t *d_cls_depT = nullptr; // [W][Cpad]
    int32_t *d_cls_cnt0 = nullptr;  // [C]   |dep| of the class
    int32_t *d_cls_isum = nullptr;  // [C]   sum of the recv indices in dep of the class (R <= 1024 only)
    int32_t *d_cls_ptr = nullptr;   // [C+1] members of class c: cls_cols[cls_ptr[c] .. cls_ptr[c+1])
    int32_t *d_cls_cols = nullptr;  // [N]   op_time columns, grouped by class
    int32_t *d_col_cls = nullptr;   // [N]   class of every op_time column
    // every class row as runs of consecutive recv indices [lo, hi): row c = runs run_ptr[c] .. run_ptr[c+1])
    int32_t *d_run_ptr = nullptr;   // [C+1]
    int32_t *d_run_lo = nullptr;    // [n_runs]
    int32_t *d_run_hi = nullptr;    // [n_runs]
    int32_t max_members = 0;        // largest class (ops)

    // Tables of the bit-sliced TAC kernel (graphs with many classes; NULL / 0 otherwise).  Classes are
    // taken 64 at a time ("class words"): bit c & 63 of word c >> 6 stands for class c.
    int32_t CW = 0, CWpad = 0;      // class words, and the row length of the tables below
    uint64_t *d_colbits = nullptr;  // [R][CWpad]   which classes hold recv r
    uint64_t *d_planes0 = nullptr;  // [13][CWpad]  bit j of |dep| of every class (bit-sliced counts)
    uint64_t *d_live0 = nullptr;    // [CWpad]      classes with |dep| >= 2
    // "parents" of a class: up to two classes of predecessor ops whose dep is a strict subset with at
    // least two recvs.  ndom0 holds the number of parents, two bits per class (class word w: bits of
    // words 2w and 2w+1); crec lists the children of every class (the classes that name it as parent).
    uint64_t *d_ndom0 = nullptr;    // [CWpad][2]
    int32_t *d_cls_par = nullptr;   // [C][2] the parents (-1: none)
    int4 *d_crec = nullptr;         // [C] {n_children, child, child, child}; more than three: w = offset of children 2.. in child_ovf
    int32_t *d_child_ovf = nullptr;
    int32_t *d_single_ptr = nullptr;// [R+1] classes whose dep is {r}: single_cls[single_ptr[r] .. single_ptr[r+1]), ascending
    int32_t *d_single_cls = nullptr;
    int32_t *d_empty_cls = nullptr; // classes with an empty dep
    int32_t n_empty_cls = 0;

    // scratch owned by the handle (grown on demand, stream-ordered use)
    // the two allocations that hold every array above (graph tables + dep; class tables)
    void *d_graph_block = nullptr, *d_class_block = nullptr;
    void *d_work = nullptr;
    int32_t *d_chan = nullptr;      // [R] channel table of the last several-channel simulation
    std::vector<int32_t> h_chan;    // its host copy
    // The graph as given (predecessor lists), kept for the tables of the iteration with send ops, which are
    // built for the send set of the last such call (one device block; see k6_sends.hip for the arrays).
    std::vector<int32_t> h_row_ptr, h_col_idx, h_recv_ids, h_send_ids;
    bool send_tables_built = false;
    void *d_send_block = nullptr;
    int4 *d_send_rec = nullptr, *d_send_succ = nullptr;
    int32_t *d_send_free = nullptr, *d_send_recv_ids = nullptr;
    uint16_t *d_send_indeg = nullptr;
    uint32_t *d_send_ready0 = nullptr;
    uint8_t *d_send_col_kind = nullptr;
    int32_t n_send_free = 0;
    size_t work_bytes = 0;
};

hipError_t ensure_workspace(Dag *d, size_t bytes);

// Number of compute units of a device and the number of workgroups of a kernel that fit one,
// asked of the runtime once and remembered (the queries cost microseconds on every launch
// otherwise).  The occupancy is remembered per (kernel, threads, dynamic LDS bytes).
int device_cu_count(int device);
// hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes), asked of the runtime only when
// `bytes` exceeds what has already been set for the kernel on the current device
hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes);
hipError_t cached_blocks_per_cu(int *per_cu, const void *kernel, int threads, size_t lds);

// ---- kernel launchers (each returns the HIP status of its launches) ----

// op.dep for every op (Sec. 4.1)
hipError_t launch_propagate(const Dag &d, hipStream_t s);
// the same for G graphs of one launch shape in one launch; staging: device memory of propagate_batch_staging_bytes(G)
size_t propagate_batch_staging_bytes(int G);
hipError_t launch_propagate_batch(Dag *const *ds, int G, void *staging, hipStream_t s);

// TIC (Sec. 4.2): prio always; order / rank when not NULL
hipError_t launch_tic(const Dag &d, int32_t *prio, int32_t *order, int32_t *rank, int32_t *scratch_prio,
                      hipStream_t s);

struct TacArgs {
    int32_t B;
    const void *op_time, *recv_time;    // float64, or float32 when f32 is set (converted on load; the arithmetic is float64)
    int32_t *order, *rank;
    double *sel_P, *sel_Mplus;
    // fused simulation outputs; all NULL = TAC only
    bool simulate;
    double *makespan, *eff, *U, *L, *S;
    bool f32 = false;
    // when not NULL: one flag per sample in memory that the caller provides, and nothing may be allocated:
    // graphs whose kernels need more per-call memory than that are refused (hipErrorNotSupported)
    int32_t *ext_flags = nullptr;
};
hipError_t launch_tac(Dag &d, const TacArgs &a, hipStream_t s);
// LDS bytes of the general TAC kernel with the per-sample state in LDS; graphs for which this is at most
// 40 KB (and at most 1024 classes) run it with one wave per sample
inline size_t tac_lds_state_bytes(int32_t R, int32_t W, int32_t C)
{
    return ((size_t)R * 2 + (R + 1) + 16 + (size_t)W * 2) * 8 + (size_t)C * 16 + (size_t)R * 8 + (size_t)C * 4;
}
inline bool tac_small_graph(int32_t R, int32_t W, int32_t C) { return tac_lds_state_bytes(R, W, C) <= 40 * 1024 && C <= 1024; }
// bit-sliced variant for graphs with many classes (tables above); the same contract as launch_tac_reg
bool tac_sliced_fits(const Dag &d);
// (flags: the first flag_bytes of the handle's workspace, which the launcher grows as needed)
hipError_t launch_tac_sliced(Dag &d, const TacArgs &a, size_t flag_bytes, int32_t **flags_out, hipStream_t s);
// device-side construction of colbits, planes0 and live0 from cls_dep and cls_cnt0
hipError_t launch_sliced_tables(const Dag &d, hipStream_t s);
// register-resident variant for graphs with few classes; returns hipErrorNotSupported when
// the graph does not fit it.  Samples it cannot order (a transfer time of zero) are marked
// in flags[b] = 1 for the general kernel.
hipError_t launch_tac_reg(Dag &d, const TacArgs &a, int32_t *flags, hipStream_t s);

struct SimArgs {
    int32_t B;
    const int32_t *order;
    int32_t order_stride;
    const void *op_time, *recv_time;    // float64, or float32 when f32 is set
    double *makespan, *eff, *U, *L, *S;
    bool f32 = false;
};
// raises *d.d_bad_order when a row of `order` (B rows, or one when order_stride = 0) is no permutation of 0 .. R-1
// Class grouping on the device, for graphs whose rows are too many to bring back to the host:
//   launch_row_digests: per compute op (op_of_col[j]) a 128-bit hash of its row, its number of set bits and its
//   lowest set bit (-1 none), as int32[8] per op: h0 lo, h0 hi, h1 lo, h1 hi, count, lowest, 0, 0;
//   launch_class_rows: cls_dep[c] = dep[first_op[c]] for every class, its transpose cls_depT (columns C..Cpad-1
//   zero), and *mismatch is raised when the row of a compute op differs from the row of its class (two different
//   rows with one hash: the caller then groups on the host)
hipError_t launch_row_digests(const Dag &d, const int32_t *op_of_col, int32_t *digest, hipStream_t s);
hipError_t launch_class_rows(const Dag &d, const int32_t *op_of_col, const int32_t *first_op, int32_t *mismatch,
                             hipStream_t s);
hipError_t launch_check_orders(Dag &d, int32_t B, const int32_t *order, int32_t order_stride, hipStream_t s);
hipError_t launch_simulate(Dag &d, const SimArgs &a, hipStream_t s);
// (needs the tables d_send_*; hipErrorNotSupported when the per-sample state does not fit LDS)
hipError_t launch_simulate_sends(Dag &d, const SimArgs &a, hipStream_t s);
hipError_t launch_simulate_channels(Dag &d, const SimArgs &a, int32_t n_channels, const int32_t *chan, hipStream_t s);
hipError_t launch_time_oracle_min(int32_t n_runs, int64_t n, const double *runs, double *time, hipStream_t s);
hipError_t launch_straggler(int32_t B, int32_t w, const double *makespan, double *out, hipStream_t s);

// order search (Sec. 3.1, 4.3): a climb through proposed exchanges of two positions
struct SearchArgs {
    int32_t B;
    const int32_t *order;
    int32_t order_stride;       // 0 (one start order) or R
    int32_t n_moves;
    const int32_t *moves;       // [n_moves][2]
    const double *op_time, *recv_time;
    int32_t *best_order;
    double *best_makespan, *start_makespan;
    int32_t *n_accepted;
};
// hipErrorNotSupported: the graph is outside what the kernel handles
hipError_t launch_order_search(Dag &d, const SearchArgs &a, hipStream_t s);

}  // namespace tictac
