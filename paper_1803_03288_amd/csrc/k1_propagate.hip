// Dependency-bitset propagation (Sec. 4.1, Communication Dependency):
//   dep[v] = ({i} if v is recv i) | OR over predecessors u of dep[u].
//
// The host condenses the graph first: a compute op whose only predecessor is a compute op
// has exactly that op's set, so only the remaining ops ("nodes": joins, ops fed by a recv,
// roots) are computed by the level-ordered kernel; every other row is a copy made by a
// fully parallel second kernel.
//
// Node kernel.  Bit columns are independent, so the words of a row are split into slices of
// WC consecutive words and every workgroup owns one slice of all nodes: it walks the node
// levels in order and only ever reads words it wrote itself, so one workgroup barrier per
// level is the only synchronisation and no two workgroups communicate.  Nodes are stored in
// level order ("positions"); the slice of the most recent RING positions is kept in an LDS
// ring, so that inputs from recent levels cost an LDS read and only long edges go to
// memory.
#include "device_utils.h"
#include <algorithm>

#include "internal.h"

namespace tictac {

using NodeRec = Dag::NodeRec;

struct PropParams {
    int32_t n_levels, W, M, ring;       // ring: positions held in LDS (power of two)
    const NodeRec *nodes;
    const int32_t *ovf_idx;
    const Dag::FastRec *frecs;          // the chunked kernel's form of the nodes
    const int32_t *fovf;
    int32_t fovf_lds;                   // > 0: that many entries of fovf (all of them) are copied to LDS
    const int32_t *nlvl_ptr;
    uint64_t *dep;
};

// Levels are short (a few hundred nodes), so a level costs about one trip to memory unless
// the node records are fetched well ahead.  The WC threads that share a node take turns:
// the thread with word index (lv + 1) % WC hands the record of level lv + 1 to its
// neighbours through LDS just before the barrier of level lv, and then starts the load of
// the record of level lv + 1 + WC, which has WC levels to arrive.  Level boundaries are kept
// in an LDS window that is refilled every LVL_CHUNK levels.
constexpr int LVL_CHUNK = 512;

// Workgroup barrier that waits for this wave's LDS traffic only.  The per-level barrier must
// not wait for the global stores of the level (a trip to memory per level); rows that have
// left the LDS ring are read from memory only after a barrier that did drain the stores.
// Slice of the row words that a workgroup owns.  Consecutive workgroups are placed on
// different XCDs (eight of them, each with an L2 of its own); when the number of slices is a
// multiple of eight, the slices are dealt so that every XCD gets a run of adjacent slices
// and the narrow stores of one row meet in one L2 before they are written back.
__device__ __forceinline__ int slice_of(int b, int n) { return (n & 7) == 0 ? (b & 7) * (n >> 3) + (b >> 3) : b; }
__device__ __forceinline__ int slice_of_block() { return slice_of(blockIdx.x, gridDim.x); }

// Accesses that are stated to be to device memory.  A pointer that a kernel reads from a record in memory (not from
// its own arguments) could point anywhere as far as the compiler knows, and an access through it becomes a generic one,
// which counts as an LDS operation too: the LDS-only waits before the barriers would then wait for memory.
typedef int tt_i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int4 load_device_16(const void *q)
{
    const tt_i32x4 v = *(const __attribute__((address_space(1))) tt_i32x4 *)q;
    return make_int4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_device_8(void *q, uint64_t v) { *(__attribute__((address_space(1))) uint64_t *)q = v; }
__device__ __forceinline__ uint64_t load_device_8(const void *q) { return *(const __attribute__((address_space(1))) uint64_t *)q; }
__device__ __forceinline__ int32_t load_device_4(const void *q) { return *(const __attribute__((address_space(1))) int32_t *)q; }

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void drain_barrier() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int WC>
__global__ void __launch_bounds__(1024)
propagate_nodes_wide(const PropParams p)
{
    extern __shared__ uint64_t ring[];                  // [ring][WC], then records, then level bounds
    const int W = p.W;
    const int w = threadIdx.x % WC;                     // word of the slice
    const int gw = slice_of_block() * WC + w;           // word of the row
    const int sub = threadIdx.x / WC;                   // node within a pass over a level
    const int per_pass = blockDim.x / WC;
    const uint32_t rmask = (uint32_t)p.ring - 1u;
    int4 *recbuf = reinterpret_cast<int4 *>(ring + (size_t)p.ring * WC);     // [2][per_pass][2]
    int32_t *lvl = reinterpret_cast<int32_t *>(recbuf + 4 * per_pass);      // [LVL_CHUNK + WC + 3]
    const int L = p.n_levels;

    // bounds of level x (valid for base <= x <= base + LVL_CHUNK + WC + 1, clamped to L)
    int base = 0;
    auto fill_bounds = [&](int b0) {
        for (int i = threadIdx.x; i < LVL_CHUNK + WC + 3; i += blockDim.x) lvl[i] = p.nlvl_ptr[min(b0 + i, L)];
    };
    fill_bounds(0);
    __syncthreads();

    // records in flight: this thread holds the record of its node (sub) of level `held_lv`
    int4 ha = make_int4(0, 0, 0, 0), hb = ha;
    bool held_ok = false;
    auto start_load = [&](int lv) {                      // record of node `sub` of level lv
        held_ok = false;
        if (lv < L) {
            const int pos = lvl[lv - base] + sub;
            if (pos < lvl[lv + 1 - base]) {
                const int4 *q = reinterpret_cast<const int4 *>(p.nodes + pos);
                ha = q[0]; hb = q[1];
                held_ok = true;
            }
        }
    };
    // prologue: thread w holds level (w == 0 ? WC : w); level 0 is read directly
    start_load(w == 0 ? WC : w);
    if (w == 0 && L > 0) {                               // level 0 goes through the record buffer too
        const int pos = lvl[0] + sub;
        if (pos < lvl[1]) {
            const int4 *q = reinterpret_cast<const int4 *>(p.nodes + pos);
            recbuf[(0 * per_pass + sub) * 2] = q[0];
            recbuf[(0 * per_pass + sub) * 2 + 1] = q[1];
        }
    }
    __syncthreads();

    int drained = 0;                                    // rows of positions < drained are in memory
    for (int lv = 0; lv < L; ++lv) {
        const int beg = lvl[lv - base], end = lvl[lv + 1 - base];
        const int safe_from = end - p.ring;             // positions >= safe_from are still in the ring
        // (positions < safe_from are < drained: see the end of the loop body)
        for (int pos = beg + sub; pos < end; pos += per_pass) {
            int4 a, b;
            if (pos == beg + sub) {
                a = recbuf[((lv & 1) * per_pass + sub) * 2];
                b = recbuf[((lv & 1) * per_pass + sub) * 2 + 1];
            } else {                                     // levels wider than one pass: fetched on demand
                const int4 *q = reinterpret_cast<const int4 *>(p.nodes + pos);
                a = q[0]; b = q[1];
            }
            const int in[6] = {a.x, a.y, a.z, a.w, b.x, b.y};
            const int op = b.z, ovf_beg = b.w;
            uint64_t val = 0;
            if (gw < W) {
#pragma unroll
                for (int j = 0; j < 6; ++j) {
                    const int x = in[j];
                    if (x == INT32_MIN) continue;
                    if (x < 0) {
                        const int i = ~x;
                        if ((i >> 6) == gw) val |= 1ull << (i & 63);
                    } else if (x >= safe_from) {
                        val |= ring[((uint32_t)x & rmask) * WC + w];
                    } else {
                        val |= p.dep[(size_t)p.nodes[x].op * W + gw];
                    }
                }
                const int ovf_cnt = ovf_beg >= 0 ? p.ovf_idx[ovf_beg] : 0;
                for (int e = 1; e <= ovf_cnt; ++e) {
                    const int x = p.ovf_idx[ovf_beg + e];
                    if (x < 0) {
                        const int i = ~x;
                        if ((i >> 6) == gw) val |= 1ull << (i & 63);
                    } else if (x >= safe_from) {
                        val |= ring[((uint32_t)x & rmask) * WC + w];
                    } else {
                        val |= p.dep[(size_t)p.nodes[x].op * W + gw];
                    }
                }
                p.dep[(size_t)op * W + gw] = val;
            }
            ring[((uint32_t)pos & rmask) * WC + w] = val;
        }
        // hand over the record of level lv + 1 and start on level lv + 1 + WC
        if (w == (lv + 1) % WC) {
            if (held_ok) {
                recbuf[(((lv + 1) & 1) * per_pass + sub) * 2] = ha;
                recbuf[(((lv + 1) & 1) * per_pass + sub) * 2 + 1] = hb;
            }
            start_load(lv + 1 + WC);
        }
        // the next level reads from memory the positions below (its end - ring): if some of
        // them were stored since the last drain, wait for all stores before the barrier
        const int next_safe = lvl[min(lv + 2, L) - base] - p.ring;
        if (next_safe > drained) {                       // uniform over the workgroup
            drain_barrier();
            drained = end;
        } else {
            lds_barrier();
        }
        if (lv + 1 - base == LVL_CHUNK) {                // slide the window of level bounds
            base += LVL_CHUNK;
            fill_bounds(base);
            __syncthreads();
        }
    }
}

// Main node kernel, for graphs whose widest level fits one pass of the workgroup (one
// thread per node and word).  Nothing on the per-level path touches memory:
//   * levels are processed in chunks made by the host (at most RPT positions per thread
//     group, at most 64 levels).  The records of a chunk sit in LDS.  At a chunk boundary a
//     thread writes the records it requested two boundaries earlier into the other LDS
//     buffer, stores the words it computed in the chunk just finished, and requests the
//     records of the third chunk ahead; so loads have two chunks to complete, stores one,
//     and the barrier between two levels waits for LDS only;
//   * the wait at a boundary covers everything but the latest request, hence the stores of
//     the previous boundary: the rows of a chunk are in memory two chunks later.  The ring
//     holds at least two chunks (or every node), hence any input that has left the ring is
//     in memory.
constexpr int WIN_LEVELS = 512;                 // levels per refill of the bounds window
constexpr int WIN_MARGIN = 330;                 // one chunk past the window and four chunks ahead (64 levels each), and slack
constexpr int RPT = kK1Rpt;                     // positions per thread group and chunk

template <int WC>
__global__ void __launch_bounds__(1024)
propagate_nodes(const PropParams p, const int32_t *__restrict__ chunk_end)
{
    extern __shared__ uint64_t ring[];                  // [ring][WC], records [2][CH], level windows
    const int W = p.W, L = p.n_levels;
    const int w = threadIdx.x % WC;
    const int gw = slice_of_block() * WC + w;
    const int sub = threadIdx.x / WC;
    const int per_pass = blockDim.x / WC;
    const int CH = RPT * per_pass;                      // most positions of a chunk
    const uint32_t rmask = (uint32_t)p.ring - 1u;
    // row p.ring of the ring is all zero; two rows are reserved so that what follows stays 16-byte aligned
    int4 *recbuf = reinterpret_cast<int4 *>(ring + (size_t)(p.ring + 2) * WC);  // [2][CH][2]
    if (threadIdx.x < 2 * WC) ring[(size_t)p.ring * WC + threadIdx.x] = 0;
    int32_t *lvl = reinterpret_cast<int32_t *>(recbuf + (size_t)4 * CH);        // [WIN_LEVELS + WIN_MARGIN]
    int32_t *cend = lvl + WIN_LEVELS + WIN_MARGIN;                               // [WIN_LEVELS + WIN_MARGIN]
    int32_t *fov = cend + WIN_LEVELS + WIN_MARGIN;                               // [fovf_lds] input lists of the other nodes
    for (int i = threadIdx.x; i < p.fovf_lds; i += blockDim.x) fov[i] = p.fovf[i];

    int base = 0;
    auto fill_window = [&](int b0) {
        for (int i = threadIdx.x; i < WIN_LEVELS + WIN_MARGIN; i += blockDim.x) {
            lvl[i] = p.nlvl_ptr[min(b0 + i, L)];
            cend[i] = b0 + i < L ? chunk_end[b0 + i] : L;
        }
    };
    fill_window(0);
    __syncthreads();
    if (L == 0) return;

    // chunk c: levels [L0, L1), positions [c0, c1); chunks c+1, c+2: [L1, L2), [L2, L3)
    int L0 = 0, L1 = cend[0];
    int c0 = lvl[0], c1 = lvl[L1];
    int L2 = L1 < L ? cend[L1] : L1;
    int c2 = lvl[L2];
    int L3 = L2 < L ? cend[L2] : L2;
    int c3 = lvl[L3];
    // Records in flight, two register sets used in turn: at the boundary after chunk c one set
    // holds the records of chunk c+1 (requested two boundaries earlier) and is refilled with
    // the request for chunk c+3.  A request is always 2 RPT loads (addresses clamped), so
    // "at most 2 RPT memory operations outstanding" means: everything before the latest
    // request has completed.
    static_assert(RPT == 4, "the s_waitcnt below is written for 2 * RPT = 8 loads per request");
    int4 a0_0, a0_1, a0_2, a0_3, b0_0, b0_1, b0_2, b0_3, a1_0, a1_1, a1_2, a1_3, b1_0, b1_1, b1_2, b1_3;
    // (macros rather than functions taking the sets by reference: the sets must stay in registers)
#define K1_REQ1(sa, sb, from, j)                                                          \
    {                                                                                     \
        const int i_ = min((from) + sub + (j) * per_pass, p.M - 1);                       \
        const int4 *q_ = reinterpret_cast<const int4 *>(p.frecs + i_);                    \
        sa##_##j = q_[0]; sb##_##j = q_[1];                                               \
    }
#define K1_REQUEST(sa, sb, from) K1_REQ1(sa, sb, from, 0) K1_REQ1(sa, sb, from, 1) K1_REQ1(sa, sb, from, 2) K1_REQ1(sa, sb, from, 3)
#define K1_PUT1(sa, sb, j)                                                                \
    {                                                                                     \
        const int i_ = sub + (j) * per_pass;                                              \
        if (w == 0 && c1 + i_ < c2) { other[(size_t)i_ * 2] = sa##_##j; other[(size_t)i_ * 2 + 1] = sb##_##j; } \
    }
    // prologue: records of chunk 0 straight into buffer 0, chunks 1 and 2 requested
    for (int j = 0; j < RPT; ++j) {
        const int i = sub + j * per_pass;
        if (w == 0 && c0 + i < c1) {
            const int4 *q = reinterpret_cast<const int4 *>(p.frecs + c0 + i);
            recbuf[(size_t)i * 2] = q[0];
            recbuf[(size_t)i * 2 + 1] = q[1];
        }
    }
    K1_REQUEST(a0, b0, c1)
    K1_REQUEST(a1, b1, c2)
    __syncthreads();

    int cur = 0;
#define K1_RUN_CHUNK(sa, sb)                                                                        \
    {                                                                                               \
        const int4 *rec = recbuf + (size_t)cur * 2 * CH;                                            \
        /* A level is at most per_pass wide, so a thread group meets at most one of its positions */\
        /* c0 + sub + j per_pass per level, in ascending j.  The record of the next one is read */  \
        /* from LDS a level ahead; so is the upper bound of the next level. */                      \
        int mypos = c0 + sub;                                                                       \
        int4 ra = make_int4(0, 0, 0, 0), rb = ra;                                                   \
        if (mypos < c1) { ra = rec[(size_t)(mypos - c0) * 2]; rb = rec[(size_t)(mypos - c0) * 2 + 1]; }\
        int end_next = lvl[L0 + 1 - base];                                                          \
        for (int lv = L0; lv < L1; ++lv) {                                                          \
            const int end = end_next;                                                               \
            if (lv + 1 < L1) end_next = lvl[lv + 2 - base];                                         \
            if (mypos < end) {                                                                      \
                /* a fast node: four rows of the ring (unused inputs read the zero row after it) */ \
                /* and the bits of up to two recvs */                                               \
                const char *rbase = reinterpret_cast<const char *>(ring) + w * 8;                   \
                const uint64_t v0 = *reinterpret_cast<const uint64_t *>(rbase + ra.x);              \
                const uint64_t v1 = *reinterpret_cast<const uint64_t *>(rbase + ra.y);              \
                const uint64_t v2 = *reinterpret_cast<const uint64_t *>(rbase + ra.z);              \
                const uint64_t v3 = *reinterpret_cast<const uint64_t *>(rbase + ra.w);              \
                uint64_t bits = (rb.x >> 6) == gw ? 1ull << (rb.x & 63) : 0ull;                     \
                bits |= (rb.y >> 6) == gw ? 1ull << (rb.y & 63) : 0ull;                             \
                uint64_t val = bits | v0 | v1 | v2 | v3;                                            \
                const int ovf_beg = rb.w;                                                           \
                if (ovf_beg >= 0 && gw < W) {                 /* any other node (rare): all inputs from its list */\
                    const int safe_from = max(end - p.ring, 0);   /* older positions: read from memory */\
                    const bool in_lds = p.fovf_lds > 0;                                             \
                    const int ovf_cnt = in_lds ? fov[ovf_beg] : p.fovf[ovf_beg];                    \
                    for (int e = 1; e <= ovf_cnt; ++e) {                                            \
                        const int x = in_lds ? fov[ovf_beg + e] : p.fovf[ovf_beg + e];              \
                        if (x < 0) {                                                                \
                            const int i = ~x;                                                       \
                            if ((i >> 6) == gw) val |= 1ull << (i & 63);                            \
                        } else if (x >= safe_from) {                                                \
                            val |= ring[((uint32_t)x & rmask) * WC + w];                            \
                        } else {                                                                    \
                            val |= p.dep[(size_t)p.frecs[x].op * W + gw];                           \
                        }                                                                           \
                    }                                                                               \
                }                                                                                   \
                if (gw >= W) val = 0;                                                               \
                ring[((uint32_t)mypos & rmask) * WC + w] = val;                                     \
                mypos += per_pass;                                                                  \
                if (mypos < c1) { ra = rec[(size_t)(mypos - c0) * 2]; rb = rec[(size_t)(mypos - c0) * 2 + 1]; }\
            }                                                                                       \
            if (lv + 1 < L1) lds_barrier();                                                         \
        }                                                                                           \
        /* ---- chunk boundary ---- */                                                              \
        /* everything issued before the latest request is complete after this: the records in */    \
        /* (sa, sb), and the stores of the chunk before this one */                                 \
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");                                            \
        /* records of chunk c+1 into the other buffer */                                            \
        int4 *other = recbuf + (size_t)(cur ^ 1) * 2 * CH;                                          \
K1_PUT1(sa, sb, 0) K1_PUT1(sa, sb, 1) K1_PUT1(sa, sb, 2) K1_PUT1(sa, sb, 3)                         \
        /* words of chunk c to memory (each thread stores what it computed itself) */               \
_Pragma("unroll")                                                                                   \
        for (int j = 0; j < RPT; ++j) {                                                             \
            const int pos = c0 + sub + j * per_pass;                                                \
            if (pos < c1 && gw < W) {                                                               \
                const int op = reinterpret_cast<const int32_t *>(rec + (size_t)(pos - c0) * 2 + 1)[2];\
                p.dep[(size_t)op * W + gw] = ring[((uint32_t)pos & rmask) * WC + w];                \
            }                                                                                       \
        }                                                                                           \
        /* request the records of chunk c+3 */                                                      \
        const int L4 = L3 < L ? cend[L3 - base] : L3;                                               \
        const int c4 = lvl[L4 - base];                                                              \
        K1_REQUEST(sa, sb, c3)                                                                      \
        lds_barrier();                                                                              \
        cur ^= 1;                                                                                   \
        L0 = L1; L1 = L2; L2 = L3; L3 = L4; c0 = c1; c1 = c2; c2 = c3; c3 = c4;                     \
        if (L0 < L && L0 - base >= WIN_LEVELS) {         /* slide the windows (uniform) */          \
            base = L0;                                                                              \
            fill_window(base);                                                                      \
            __syncthreads();                                                                        \
        }                                                                                           \
    }
    while (L0 < L) {
        K1_RUN_CHUNK(a0, b0)
        if (L0 >= L) break;
        K1_RUN_CHUNK(a1, b1)
    }
#undef K1_RUN_CHUNK
#undef K1_REQUEST
}

// Narrow graphs (no level wider than 64 / WC nodes, all rows of the slice and all records in LDS; the
// host narrows the slice until they fit): one wave per slice and no barrier at all.  The LDS
// operations of a wave are carried out in the order in which they are issued, so a row written at one
// level can be read by another lane at the next without a wait in between; the record of the next
// level's node is read from LDS a level ahead, which leaves one LDS round trip per level: the reads of
// the input rows.  Rows go to memory as they are computed and are never read back here.
// Table of n elements from memory to LDS by one wave, eight loads in flight per lane (a load per trip to memory
// would make the copy as long as the propagation itself).
// (keep_loaded: the value is in its registers at this point of the program, so the load that brings it is
// issued before; without it the compiler moves every load down to the store that uses it, behind that store's test)
__device__ __forceinline__ void keep_loaded(int32_t &x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void keep_loaded(int4 &v) { asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w)); }
template <typename T>
__device__ __forceinline__ void copy_to_lds(T *dst, const T *__restrict__ src, int n, int lane)
{
    for (int i0 = 0; i0 < n; i0 += 8 * 64) {
        T v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = i0 + j * 64 + lane;
            v[j] = src[min(i, n - 1)];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) keep_loaded(v[j]);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = i0 + j * 64 + lane;
            if (i < n) dst[i] = v[j];
        }
    }
}

template <int WC>
__global__ void __launch_bounds__(64)
propagate_nodes_wave(const PropParams p)
{
    extern __shared__ uint64_t ring[];          // rows [ring + 2][WC] (the last two all zero), records [M][2], level bounds [L + 1], input lists
    const int W = p.W, L = p.n_levels, M = p.M;
    const int w = threadIdx.x % WC, sub = threadIdx.x / WC;
    const int gw = slice_of_block() * WC + w;
    int4 *recs = reinterpret_cast<int4 *>(ring + ((((size_t)p.ring + 2) * WC + 1) & ~(size_t)1));   // 16-byte aligned
    int32_t *lvl = reinterpret_cast<int32_t *>(recs + (size_t)2 * M);
    int32_t *fov = lvl + (L + 1);
    if (threadIdx.x < 2 * WC) ring[(size_t)p.ring * WC + threadIdx.x] = 0;
    copy_to_lds(recs, reinterpret_cast<const int4 *>(p.frecs), 2 * M, threadIdx.x);
    copy_to_lds(lvl, p.nlvl_ptr, L + 1, threadIdx.x);
    copy_to_lds(fov, p.fovf, p.fovf_lds, threadIdx.x);
    __syncthreads();
    if (L == 0) return;

    // A level in straight-line code.  A lane without a node at the level works on the record of some other
    // node (the index is clamped), reads rows that exist, and writes its result to the spare row after the zero
    // row; nothing is branched on but the two rare kinds of node (recv inputs, inputs in a list).  Two register
    // sets for the records, used in turn, so that nothing is moved between levels.
    int beg = lvl[0], end = lvl[1], end2 = lvl[min(2, L)];
    char *rbase = reinterpret_cast<char *>(ring) + w * 8;
    const int spare = (p.ring + 1) * WC * 8;
    int4 ra0, rb0, ra1, rb1;
    {
        const int q = min(beg + sub, M - 1);
        ra0 = recs[(size_t)q * 2]; rb0 = recs[(size_t)q * 2 + 1];
    }
#define K1W_LEVEL(ra, rb, na, nb, lvx)                                                              \
    {                                                                                               \
        const int pos = beg + sub;                                                                  \
        const bool valid = pos < end;                                                               \
        const uint64_t v0 = *reinterpret_cast<const uint64_t *>(rbase + ra.x);                      \
        const uint64_t v1 = *reinterpret_cast<const uint64_t *>(rbase + ra.y);                      \
        const uint64_t v2 = *reinterpret_cast<const uint64_t *>(rbase + ra.z);                      \
        const uint64_t v3 = *reinterpret_cast<const uint64_t *>(rbase + ra.w);                      \
        /* the record of the next level's node and the bound after it, a level ahead */             \
        const int q = min(end + sub, M - 1);                                                        \
        na = recs[(size_t)q * 2]; nb = recs[(size_t)q * 2 + 1];                                     \
        const int end3 = lvl[min((lvx) + 3, L)];                                                      \
        uint64_t val = (v0 | v1) | (v2 | v3);                                                       \
        if (__ballot(valid && (rb.x & rb.w) != -1) != 0ull) {    /* a recv input or a list */        \
            if (rb.x >= 0 && (rb.x >> 6) == gw) val |= 1ull << (rb.x & 63);                         \
            if (rb.y >= 0 && (rb.y >> 6) == gw) val |= 1ull << (rb.y & 63);                         \
            if (valid && rb.w >= 0) {               /* all inputs from the list (every row is in LDS) */ \
                const int cnt = fov[rb.w];                                                          \
                for (int e = 1; e <= cnt; ++e) {                                                    \
                    const int x = fov[rb.w + e];                                                    \
                    if (x < 0) {                                                                    \
                        const int i = ~x;                                                           \
                        if ((i >> 6) == gw) val |= 1ull << (i & 63);                                \
                    } else {                                                                        \
                        val |= ring[(size_t)x * WC + w];                                            \
                    }                                                                               \
                }                                                                                   \
            }                                                                                       \
        }                                                                                           \
        if (gw >= W) val = 0;                                                                       \
        *reinterpret_cast<uint64_t *>(rbase + (valid ? pos * (WC * 8) : spare)) = val;              \
        if (valid && gw < W) p.dep[(size_t)rb.z * W + gw] = val;                                    \
        wave_sync();                                                                                \
        beg = end; end = end2; end2 = end3;                                                         \
    }
    for (int lv = 0; lv < L; lv += 2) {
        K1W_LEVEL(ra0, rb0, ra1, rb1, lv)
        if (lv + 1 >= L) break;
        K1W_LEVEL(ra1, rb1, ra0, rb0, lv + 1)
    }
#undef K1W_LEVEL
}

// Level-major records (see internal.h): thread group j of the workgroup takes slot l * P + j at
// level l, so a level needs no bounds and no bookkeeping of positions, and the records need no
// staging in LDS: every thread reads its own record straight from memory, eight levels ahead,
// into eight register sets used in turn.  A level is then: the reads of the input rows from the
// ring, the OR, the write of the row to the ring and to memory, one barrier.  Memory
// operations of a wave complete in the order in which they were issued, and a level issues at
// exactly two loads (the record of eight levels on) and one store (a thread without a node stores
// a zero to a word of its own), so "at most twenty-one outstanding" before the barrier of a level
// means that this wave's stores of seven levels ago and earlier are in memory, and that the record
// of the next level has arrived; the ring holds at least sixteen levels, hence a row that has left
// the ring can be read from memory.
// all inputs of a node that does not fit a record, from its list (in LDS when fov is not NULL):
// recv bits, rows still in the ring (slots from safe_from on), older rows from memory.  The
// arguments are passed one by one: a kernel whose parameter block has its address taken reads
// every pointer of it through generic loads, which wait for LDS and memory alike.
__device__ __noinline__ uint64_t other_inputs(const int32_t *lfovf, const int32_t *fov, const uint64_t *ring,
                                              const Dag::FastRec *lrecs, uint64_t *dep, int W, int beg,
                                              int safe_from, uint32_t rmask, int WC, int w, int gw)
{
    const int32_t *list = fov ? fov : lfovf;
    const int cnt = list[beg];
    uint64_t val = 0;
    for (int e = 1; e <= cnt; ++e) {
        const int x = list[beg + e];
        if (x < 0) {
            const int i = ~x;
            if ((i >> 6) == gw) val |= 1ull << (i & 63);
        } else if (x >= safe_from) {
            val |= ring[((uint32_t)x & rmask) * WC + w];
        } else {
            val |= __hip_atomic_load(&dep[(size_t)lrecs[x].op * W + gw], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    return val;
}

struct LevelParams {
    int32_t n_levels, W, P, ring;       // P slots per level; ring: slots held in LDS (power of two)
    const Dag::FastRec *lrecs;          // [n_levels * P]
    const int32_t *lfovf;
    int32_t lfovf_lds;                  // > 0: that many entries of lfovf (all of them) are copied to LDS
    uint64_t *dep;
    uint64_t *sink;                     // [gridDim.x * blockDim.x]
};

#define KL_EACH(F) F(0) F(1) F(2) F(3) F(4) F(5) F(6) F(7)

// `block` of `n_blocks`: which slice of the graph this workgroup takes (its index in a launch for one graph;
// in a launch for several graphs, its index among the workgroups of its graph)
template <int WC>
__device__ __forceinline__ void propagate_levels_body(const LevelParams &p, uint64_t *ring, int block, int n_blocks)
{
    const int W = p.W, L = p.n_levels, P = p.P;
    const int w = threadIdx.x % WC, sub = threadIdx.x / WC;
    const int gw = slice_of(block, n_blocks) * WC + w;
    const uint32_t rmask = (uint32_t)p.ring - 1u;
    int32_t *fov = reinterpret_cast<int32_t *>(ring + (size_t)(p.ring + 2) * WC);
    if (threadIdx.x < 2 * WC) ring[(size_t)p.ring * WC + threadIdx.x] = 0;
    for (int i = threadIdx.x; i < p.lfovf_lds; i += blockDim.x) fov[i] = load_device_4(p.lfovf + i);
    __syncthreads();
    if (L == 0) return;

    // record of level l for this thread group (levels past the end: the last level again, never used)
#define KL_LOAD(a, b, l)                                                                  \
    {                                                                                     \
        const int4 *q_ = reinterpret_cast<const int4 *>(p.lrecs + (size_t)min((l), L - 1) * P + sub); \
        a = load_device_16(q_); b = load_device_16(q_ + 1);                               \
    }
#define KL_DECL(i) int4 a##i, b##i; KL_LOAD(a##i, b##i, i)
    KL_EACH(KL_DECL)

    uint64_t *const sink = p.sink + (size_t)block * blockDim.x + threadIdx.x;
    const char *const rbase = reinterpret_cast<const char *>(ring) + w * 8;
    uint32_t slot = (uint32_t)sub;              // the slot of this thread group at the level being computed
    // (the next record of a set is requested after the last use of the set, into the same registers)
#define KL_STEP(i)                                                                        \
    {                                                                                     \
        const int l = lbase + i;                                                          \
        uint64_t val = 0;                                                                 \
        uint64_t *dst = sink;               /* past the last level and without a node: a zero to the sink */ \
        if (l < L && b##i.z >= 0) {                                                       \
            const uint64_t v0 = *reinterpret_cast<const uint64_t *>(rbase + a##i.x);      \
            const uint64_t v1 = *reinterpret_cast<const uint64_t *>(rbase + a##i.y);      \
            const uint64_t v2 = *reinterpret_cast<const uint64_t *>(rbase + a##i.z);      \
            const uint64_t v3 = *reinterpret_cast<const uint64_t *>(rbase + a##i.w);      \
            uint64_t bits = (b##i.x >> 6) == gw ? 1ull << (b##i.x & 63) : 0ull;           \
            bits |= (b##i.y >> 6) == gw ? 1ull << (b##i.y & 63) : 0ull;                   \
            val = bits | v0 | v1 | v2 | v3;                                               \
            if (b##i.w >= 0 && gw < W)                                                    \
                val |= other_inputs(p.lfovf, p.lfovf_lds > 0 ? fov : nullptr, ring, p.lrecs, p.dep, W, b##i.w, \
                                    (l + 1) * P - p.ring, rmask, WC, w, gw);              \
            if (gw >= W) val = 0;                                                         \
            ring[(slot & rmask) * WC + w] = val;                                          \
            if (gw < W) dst = &p.dep[(size_t)b##i.z * W + gw];                            \
        }                                                                                 \
        store_device_8(dst, val);                                                         \
        slot += (uint32_t)P;                                                              \
        asm volatile("" : "+v"(slot));   /* (else one register per unrolled level holds its slot) */ \
        KL_LOAD(a##i, b##i, l + 8)                                                        \
        asm volatile("s_waitcnt vmcnt(21)" ::: "memory");                                 \
        lds_barrier();                                                                    \
    }
    // (32 levels per trip of the loop: the compiler drains every outstanding load and store at the
    // head of a loop that carries loaded registers round, which should be rare)
    for (int l0 = 0; l0 < L; l0 += 32) {
        { const int lbase = l0;      KL_EACH(KL_STEP) }
        { const int lbase = l0 + 8;  KL_EACH(KL_STEP) }
        { const int lbase = l0 + 16; KL_EACH(KL_STEP) }
        { const int lbase = l0 + 24; KL_EACH(KL_STEP) }
    }
#undef KL_STEP
#undef KL_DECL
#undef KL_LOAD
}

template <int WC>
__global__ void __launch_bounds__(1024)
propagate_levels(const LevelParams p)
{
    extern __shared__ uint64_t ring[];          // rows [ring + 2][WC] (the last two all zero), then the input lists
    propagate_levels_body<WC>(p, ring, blockIdx.x, gridDim.x);
}

// Several graphs of one launch shape in one launch: workgroup b takes slice b % blocks_per of graph b / blocks_per.
// (One graph is a chain of dependent levels and cannot fill the chip; independent graphs side by side can.)
template <int WC>
__global__ void __launch_bounds__(1024)
propagate_levels_batch(const LevelParams *__restrict__ ps, int blocks_per)
{
    extern __shared__ uint64_t ring[];
    const int g = blockIdx.x / blocks_per;
    const LevelParams p = ps[g];
    propagate_levels_body<WC>(p, ring, blockIdx.x - g * blocks_per, blocks_per);
}

// ---- the level-major kernel with 64-byte slices ----
// For wide rows (a multiple of eight words).  A workgroup takes a slice of eight consecutive words (64 bytes) of
// every row, and four adjacent lanes take one slot of a level, 16 bytes each: the four lanes' store of a row is one
// 64-byte piece, their reads of an input row one 64-byte stretch of LDS, and they share the slot's record.  An
// eighth of the workgroups, of the record traffic and of the store requests of one-word slices for the same bytes.
// The ring then holds fewer levels (2048 slots in 128 KB); the host gives a row that is needed after it has left
// the ring a copy node some levels later (see the build of the records), so a level still reads LDS only.
// The records are 16 bytes (see internal.h): a level issues exactly one 16-byte load and one 16-byte store per thread.
typedef unsigned long long tt_u64x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_device_16(void *q, tt_u64x2 v) { *(__attribute__((address_space(1))) tt_u64x2 *)q = v; }

// words gw, gw + 1 of all inputs of a node that does not fit a record (see other_inputs)
__device__ __noinline__ tt_u64x2 other_inputs_q(const int32_t *lfovf, const int32_t *fov, const uint64_t *ring,
                                                const Dag::QuadRec *qrecs, uint64_t *dep, int W, int beg, int safe_from,
                                                uint32_t rmask, int row_words, int word_in_slice, int gw)
{
    const int32_t *list = fov ? fov : lfovf;
    const int cnt = list[beg];
    tt_u64x2 val = {0ull, 0ull};
    for (int e = 1; e <= cnt; ++e) {
        const int x = list[beg + e];
        if (x < 0) {
            const int i = ~x;
            if ((i >> 6) == gw) val.x |= 1ull << (i & 63);
            if ((i >> 6) == gw + 1) val.y |= 1ull << (i & 63);
        } else if (x >= safe_from) {
            val |= *reinterpret_cast<const tt_u64x2 *>(ring + ((uint32_t)x & rmask) * row_words + word_in_slice);
        } else {
            const uint64_t *q = &dep[(size_t)qrecs[x].op * W + gw];
            val.x |= __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            val.y |= __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    return val;
}

struct QuadParams {
    int32_t n_levels, W, P, ring;       // P slots per level; ring: slots held in LDS (power of two)
    const Dag::QuadRec *qrecs;          // [n_levels * P]
    const int32_t *lfovf;
    int32_t lfovf_lds;                  // > 0: that many entries of lfovf (all of them) are copied to LDS
    uint64_t *dep;
    uint64_t *sink;                     // [gridDim.x * blockDim.x][2]
};

// QC lanes per slot (4: 64-byte slices, 2: 32-byte slices)
template <int QC>
__device__ __forceinline__ void propagate_levels_q_body(const QuadParams &p, uint64_t *ring, int block, int n_blocks)
{
    constexpr int RW = 2 * QC;                  // words of a row in the ring
    constexpr int SH = QC == 4 ? 6 : 5;         // log2 of the bytes of a row in the ring
    const int W = p.W, L = p.n_levels, P = p.P;
    const int sub = threadIdx.x / QC, qd = threadIdx.x % QC;
    const int gw = slice_of(block, n_blocks) * RW + qd * 2;      // first of this thread's two words of the row
    const uint32_t rmask = (uint32_t)p.ring - 1u;
    int32_t *fov = reinterpret_cast<int32_t *>(ring + (size_t)(p.ring + 2) * RW);
    if (threadIdx.x < 2 * RW) ring[(size_t)p.ring * RW + threadIdx.x] = 0;
    for (int i = threadIdx.x; i < p.lfovf_lds; i += blockDim.x) fov[i] = load_device_4(p.lfovf + i);
    __syncthreads();
    if (L == 0) return;

#define KQ_LOAD(a, l) a = load_device_16(p.qrecs + (size_t)min((l), L - 1) * P + sub);
#define KQ_DECL(i) int4 a##i; KQ_LOAD(a##i, i)
    KL_EACH(KQ_DECL)

    uint64_t *const sink = p.sink + ((size_t)block * blockDim.x + threadIdx.x) * 2;
    const char *const rb = reinterpret_cast<const char *>(ring) + qd * 16;
    uint32_t slot = (uint32_t)sub;              // the slot of these four lanes at the level being computed
#define KQ_BIT(r)                                                                         \
    {                                                                                     \
        const int wi_ = (int)((r) >> 6) - gw;          /* no recv: r = 0xffff, word 1023, which no row here has */ \
        const uint64_t bit_ = 1ull << ((r) & 63);                                         \
        val.x |= wi_ == 0 ? bit_ : 0ull;                                                  \
        val.y |= wi_ == 1 ? bit_ : 0ull;                                                  \
    }
    // (a level issues exactly one 16-byte load and one 16-byte store per thread: "at most fourteen outstanding")
#define KQ_STEP(i)                                                                        \
    {                                                                                     \
        const int l = lbase + i;                                                          \
        tt_u64x2 val = {0ull, 0ull};                                                      \
        uint64_t *dst = sink;               /* past the last level, no node, a copy: to the sink */ \
        if (l < L && a##i.w != -1) {                                                      \
            const uint32_t i01 = (uint32_t)a##i.x, i23 = (uint32_t)a##i.y, r01 = (uint32_t)a##i.z; \
            if (i01 != 0xffffffffu) {                                                     \
                val = *reinterpret_cast<const tt_u64x2 *>(rb + ((i01 & 0xffffu) << SH)) | \
                      *reinterpret_cast<const tt_u64x2 *>(rb + ((i01 >> 16) << SH)) |     \
                      *reinterpret_cast<const tt_u64x2 *>(rb + ((i23 & 0xffffu) << SH)) | \
                      *reinterpret_cast<const tt_u64x2 *>(rb + ((i23 >> 16) << SH));      \
                KQ_BIT(r01 & 0xffffu)                                                     \
                KQ_BIT(r01 >> 16)                                                         \
            } else {                                                                      \
                val = other_inputs_q(p.lfovf, p.lfovf_lds > 0 ? fov : nullptr, ring, p.qrecs, p.dep, W, (int)i23, \
                                     (l + 1) * P - p.ring, rmask, RW, qd * 2, gw);        \
            }                                                                             \
            *reinterpret_cast<tt_u64x2 *>(ring + (slot & rmask) * RW + qd * 2) = val;     \
            if (a##i.w >= 0) dst = &p.dep[(size_t)a##i.w * W + gw];                       \
        }                                                                                 \
        store_device_16(dst, val);                                                        \
        slot += (uint32_t)P;                                                              \
        asm volatile("" : "+v"(slot));   /* (else one register per unrolled level holds its slot) */ \
        KQ_LOAD(a##i, l + 8)                                                              \
        asm volatile("s_waitcnt vmcnt(14)" ::: "memory");                                 \
        lds_barrier();                                                                    \
    }
    for (int l0 = 0; l0 < L; l0 += 32) {
        { const int lbase = l0;      KL_EACH(KQ_STEP) }
        { const int lbase = l0 + 8;  KL_EACH(KQ_STEP) }
        { const int lbase = l0 + 16; KL_EACH(KQ_STEP) }
        { const int lbase = l0 + 24; KL_EACH(KQ_STEP) }
    }
#undef KQ_STEP
#undef KQ_BIT
#undef KQ_DECL
#undef KQ_LOAD
}

template <int QC>
__global__ void __launch_bounds__(256 * QC)
propagate_levels_q_batch(const QuadParams *__restrict__ ps, int blocks_per)
{
    extern __shared__ uint64_t ring[];          // rows [ring + 2][2 QC] (the last two all zero), then the input lists
    // Workgroup b runs on XCD b % 8.  The workgroups are renumbered so that every XCD gets a run of consecutive
    // numbers, hence whole graphs where it can: the slices of a row then meet in one L2 and leave it as whole
    // lines, and the eight slices of a graph read its records through one L2.
    const int n = gridDim.x;
    const int v = (n & 7) == 0 ? (blockIdx.x & 7) * (n >> 3) + (blockIdx.x >> 3) : (int)blockIdx.x;
    const int g = v / blocks_per;
    const QuadParams p = ps[g];
    propagate_levels_q_body<QC>(p, ring, v - g * blocks_per, 1);
}

// rows that are copies: a recv's single bit, or the row of the node an op collapses onto.  `copied`: the ops
// with such rows, as pairs (op, ~i for recv i or the op id of the node whose row it has).
__device__ __forceinline__ void expand_word(int32_t n_copied, int32_t W, const int32_t *copied, uint64_t *dep, size_t idx)
{
    if (idx >= (size_t)n_copied * W) return;
    const int e = (int)(idx / W), w = (int)(idx % W);
    const int v = load_device_4(copied + 2 * e), s = load_device_4(copied + 2 * e + 1);
    uint64_t val;
    if (s < 0) {
        const int i = ~s;
        val = (i >> 6) == w ? 1ull << (i & 63) : 0ull;
    } else {
        val = load_device_8(dep + (size_t)s * W + w);
    }
    store_device_8(dep + (size_t)v * W + w, val);
}

__global__ void __launch_bounds__(256)
expand_rows(int32_t n_copied, int32_t W, const int32_t *__restrict__ copied, uint64_t *dep)
{
    expand_word(n_copied, W, copied, dep, (size_t)blockIdx.x * blockDim.x + threadIdx.x);
}

// the same for several graphs: blockIdx.y = graph
struct ExpandParams {
    int32_t n_copied, W;
    const int32_t *copied;
    uint64_t *dep;
};
__global__ void __launch_bounds__(256)
expand_rows_batch(const ExpandParams *__restrict__ ps)
{
    const ExpandParams p = ps[blockIdx.y];
    expand_word(p.n_copied, p.W, p.copied, p.dep, (size_t)blockIdx.x * blockDim.x + threadIdx.x);
}

static bool level_params(const Dag &d, int WC, LevelParams *q, size_t *lds)
{
    if (!d.d_lrecs || !d.d_k1_sink || d.k1_wc != WC) return false;
    q->n_levels = d.n_node_levels; q->W = d.W; q->P = d.k1_threads / WC; q->ring = d.k1_lring;
    q->lrecs = d.d_lrecs; q->lfovf = d.d_lfovf; q->dep = d.d_dep; q->sink = d.d_k1_sink;
    q->lfovf_lds = d.lfovf_len <= 4096 ? d.lfovf_len : 0;
    *lds = (size_t)(d.k1_lring + 2) * WC * 8 + (size_t)q->lfovf_lds * 4;
    return *lds <= 150 * 1024;
}

static bool quad_params(const Dag &d, int QC, QuadParams *q, size_t *lds)
{
    // (k1_q_threads is four lanes per slot; QC lanes per slot need a multiple of 64 threads as well)
    const int threads = d.k1_q_threads / 4 * QC;
    if (d.k1_q_ring <= 0 || !d.d_qrecs || !d.d_k1_q_sink || d.W % 8 != 0 || threads % 64 != 0 || threads > 256 * QC)
        return false;
    q->n_levels = d.n_node_levels; q->W = d.W; q->P = d.k1_q_threads / 4; q->ring = d.k1_q_ring;
    q->qrecs = d.d_qrecs; q->lfovf = d.d_qfovf; q->dep = d.d_dep; q->sink = d.d_k1_q_sink;
    q->lfovf_lds = d.qfovf_len <= 4096 ? d.qfovf_len : 0;
    *lds = (size_t)(d.k1_q_ring + 2) * QC * 16 + (size_t)q->lfovf_lds * 4;
    return *lds <= 150 * 1024;
}

// Propagation for G graphs that all take the level-major kernel with one launch shape (as G handles of one
// graph do): one launch of the node kernel, one of the copies.  `staging`: device memory for G parameter records
// of each kind (filled here, stream-ordered).  hipErrorNotSupported when the graphs do not fit that description.
template <int WC>
static hipError_t launch_levels_batch(Dag *const *ds, int G, void *staging, hipStream_t s)
{
    std::vector<LevelParams> lp(G);
    std::vector<ExpandParams> ep(G);
    size_t lds0 = 0;
    int32_t most_copied = 0;
    for (int g = 0; g < G; ++g) {
        size_t lds = 0;
        if (!level_params(*ds[g], WC, &lp[g], &lds)) return hipErrorNotSupported;
        if (g == 0) lds0 = lds;
        if (lds != lds0 || ds[g]->k1_threads != ds[0]->k1_threads || ds[g]->W != ds[0]->W || ds[g]->n != ds[0]->n)
            return hipErrorNotSupported;
        ep[g] = ExpandParams{ds[g]->n_copied, ds[g]->W, ds[g]->d_copied, ds[g]->d_dep};
        most_copied = std::max(most_copied, ds[g]->n_copied);
    }
    LevelParams *d_lp = static_cast<LevelParams *>(staging);
    ExpandParams *d_ep = reinterpret_cast<ExpandParams *>(d_lp + G);
    hipError_t e = hipMemcpyAsync(d_lp, lp.data(), sizeof(LevelParams) * G, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return e;
    e = hipMemcpyAsync(d_ep, ep.data(), sizeof(ExpandParams) * G, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return e;
    if (lds0 > 48 * 1024) {
        e = ensure_dynamic_lds(reinterpret_cast<const void *>(propagate_levels_batch<WC>), lds0);
        if (e != hipSuccess) return e;
    }
    const Dag &d0 = *ds[0];
    const int blocks_per = (d0.W + WC - 1) / WC;
    hipLaunchKernelGGL(propagate_levels_batch<WC>, dim3(blocks_per * G), dim3(d0.k1_threads), lds0, s, d_lp, blocks_per);
    const size_t total = (size_t)most_copied * d0.W;
    if (total) hipLaunchKernelGGL(expand_rows_batch, dim3((unsigned)((total + 255) / 256), G), dim3(256), 0, s, d_ep);
    return hipGetLastError();
}

// the same for graphs that take the kernel with 64-byte (QC = 4) or 32-byte (QC = 2) slices
template <int QC>
static hipError_t launch_quad_batch(Dag *const *ds, int G, void *staging, hipStream_t s)
{
    std::vector<QuadParams> lp(G);
    std::vector<ExpandParams> ep(G);
    size_t lds0 = 0;
    int32_t most_copied = 0;
    for (int g = 0; g < G; ++g) {
        size_t lds = 0;
        if (!quad_params(*ds[g], QC, &lp[g], &lds)) return hipErrorNotSupported;
        if (g == 0) lds0 = lds;
        if (lds != lds0 || ds[g]->k1_q_threads != ds[0]->k1_q_threads || ds[g]->W != ds[0]->W || ds[g]->n != ds[0]->n)
            return hipErrorNotSupported;
        ep[g] = ExpandParams{ds[g]->n_q_copied, ds[g]->W, ds[g]->d_q_copied, ds[g]->d_dep};
        most_copied = std::max(most_copied, ds[g]->n_q_copied);
    }
    QuadParams *d_lp = static_cast<QuadParams *>(staging);
    ExpandParams *d_ep = reinterpret_cast<ExpandParams *>(d_lp + G);
    hipError_t e = hipMemcpyAsync(d_lp, lp.data(), sizeof(QuadParams) * G, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return e;
    e = hipMemcpyAsync(d_ep, ep.data(), sizeof(ExpandParams) * G, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return e;
    if (lds0 > 48 * 1024) {
        e = ensure_dynamic_lds(reinterpret_cast<const void *>(propagate_levels_q_batch<QC>), lds0);
        if (e != hipSuccess) return e;
    }
    const Dag &d0 = *ds[0];
    const int blocks_per = d0.W / (2 * QC);
    hipLaunchKernelGGL(propagate_levels_q_batch<QC>, dim3(blocks_per * G), dim3(d0.k1_q_threads / 4 * QC), lds0, s, d_lp,
                       blocks_per);
    const size_t total = (size_t)most_copied * d0.W;
    if (total) hipLaunchKernelGGL(expand_rows_batch, dim3((unsigned)((total + 255) / 256), G), dim3(256), 0, s, d_ep);
    return hipGetLastError();
}

size_t propagate_batch_staging_bytes(int G)
{
    return (std::max(sizeof(LevelParams), sizeof(QuadParams)) + sizeof(ExpandParams)) * (size_t)G;
}

hipError_t launch_propagate_batch(Dag *const *ds, int G, void *staging, hipStream_t s)
{
    if (G <= 0) return hipSuccess;
    if (ds[0]->n == 0 || ds[0]->W == 0 || ds[0]->M == 0) return hipErrorNotSupported;
    // (32-byte slices, QC = 2, were measured too: as fast up to sixteen graphs, a third slower from 32 on)
    if (G >= 2 && ds[0]->k1_q_ring > 0) return launch_quad_batch<4>(ds, G, staging, s);
    if (ds[0]->k1_wc == 1) return launch_levels_batch<1>(ds, G, staging, s);
    if (ds[0]->k1_wc == 2) return launch_levels_batch<2>(ds, G, staging, s);
    return launch_levels_batch<4>(ds, G, staging, s);
}

template <int WC>
static hipError_t launch_nodes(const Dag &d, hipStream_t s)
{
    PropParams p;
    p.n_levels = d.n_node_levels; p.W = d.W; p.M = d.M;
    p.nodes = d.d_nodes; p.ovf_idx = d.d_ovf_idx; p.nlvl_ptr = d.d_nlvl_ptr; p.dep = d.d_dep;
    p.frecs = d.d_frecs; p.fovf = d.d_fovf;
    p.fovf_lds = d.fovf_len <= 4096 ? d.fovf_len : 0;
    const int threads = d.k1_threads;
    const int per_pass = threads / WC;
    const int blocks = (d.W + WC - 1) / WC;
    const bool wide = d.max_node_level_width > per_pass;
    if (!wide && !d.d_frecs && !d.d_lrecs) return hipErrorInvalidValue;
    if (d.d_lrecs) {
        // level-major records: no staging, no chunks
        LevelParams q;
        size_t lds_l = 0;
        if (!level_params(d, WC, &q, &lds_l)) return hipErrorInvalidValue;
        if (lds_l > 48 * 1024) {
            hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(propagate_levels<WC>), lds_l);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(propagate_levels<WC>, dim3(blocks), dim3(threads), lds_l, s, q);
        return hipGetLastError();
    }
    const int ring = d.k1_ring;
    p.ring = ring;
    // one wave per slice when no level is wider than a wave and everything fits in LDS (decided when the records were made)
    if (d.k1_wave) {
        const size_t lds_w = ((((size_t)ring + 2) * WC + 1) & ~(size_t)1) * 8 + (size_t)d.M * 32 +
                             (size_t)(d.n_node_levels + 1) * 4 + (size_t)p.fovf_lds * 4;
        if (wide || threads != 64 || ring != d.M || lds_w > 150 * 1024 || (d.fovf_len > 0 && p.fovf_lds == 0))
            return hipErrorInvalidValue;
        if (lds_w > 48 * 1024) {
            hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(propagate_nodes_wave<WC>), lds_w);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(propagate_nodes_wave<WC>, dim3(blocks), dim3(64), lds_w, s, p);
        return hipGetLastError();
    }
    size_t lds = (size_t)ring * WC * 8;
    if (wide) lds += (size_t)4 * per_pass * 16 + (size_t)(LVL_CHUNK + WC + 3) * 4;
    else lds += (size_t)2 * WC * 8 + (size_t)4 * RPT * per_pass * 16 + (size_t)2 * (WIN_LEVELS + WIN_MARGIN) * 4 +
                (size_t)p.fovf_lds * 4;
    if (lds > 150 * 1024) return hipErrorInvalidValue;
    const void *kern = wide ? reinterpret_cast<const void *>(propagate_nodes_wide<WC>)
                            : reinterpret_cast<const void *>(propagate_nodes<WC>);
    if (lds > 48 * 1024) {
        hipError_t e = ensure_dynamic_lds(kern, lds);
        if (e != hipSuccess) return e;
    }
    if (wide)
        hipLaunchKernelGGL(propagate_nodes_wide<WC>, dim3(blocks), dim3(threads), lds, s, p);
    else
        hipLaunchKernelGGL(propagate_nodes<WC>, dim3(blocks), dim3(threads), lds, s, p, d.d_chunk_end);
    return hipGetLastError();
}

hipError_t launch_propagate(const Dag &d, hipStream_t s)
{
    if (d.n == 0 || d.W == 0) return hipSuccess;
    hipError_t e = hipSuccess;
    if (d.M > 0) {
        if (d.k1_wc == 1) e = launch_nodes<1>(d, s);
        else if (d.k1_wc == 2) e = launch_nodes<2>(d, s);
        else e = launch_nodes<4>(d, s);
        if (e != hipSuccess) return e;
    }
    const size_t total = (size_t)d.n_copied * d.W;
    if (total)
        hipLaunchKernelGGL(expand_rows, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, d.n_copied, d.W, d.d_copied, d.d_dep);
    return hipGetLastError();
}

}  // namespace tictac
