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
#include "internal.h"

namespace tictac {

using NodeRec = Dag::NodeRec;

struct PropParams {
    int32_t n_levels, W, M, ring;       // ring: positions held in LDS (power of two)
    const NodeRec *nodes;
    const int32_t *ovf_idx;
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
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void drain_barrier() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int WC>
__global__ void __launch_bounds__(1024)
propagate_nodes(const PropParams p)
{
    extern __shared__ uint64_t ring[];                  // [ring][WC], then records, then level bounds
    const int W = p.W;
    const int w = threadIdx.x % WC;                     // word of the slice
    const int gw = blockIdx.x * WC + w;                 // word of the row
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

// rows that are copies: a recv's single bit, or the row of the node an op collapses onto
__global__ void __launch_bounds__(256)
expand_rows(int32_t n, int32_t W, const int32_t *__restrict__ src, uint64_t *dep)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)n * W) return;
    const int v = (int)(idx / W), w = (int)(idx % W);
    const int s = src[v];
    if (s < 0) {
        const int i = ~s;
        dep[idx] = (i >> 6) == w ? 1ull << (i & 63) : 0ull;
    } else if (s != v) {
        dep[idx] = dep[(size_t)s * W + w];
    }
}

template <int WC>
static hipError_t launch_nodes(const Dag &d, hipStream_t s)
{
    PropParams p;
    p.n_levels = d.n_node_levels; p.W = d.W; p.M = d.M;
    p.nodes = d.d_nodes; p.ovf_idx = d.d_ovf_idx; p.nlvl_ptr = d.d_nlvl_ptr; p.dep = d.d_dep;
    // ring: the largest power of two of positions within 96 KB, no larger than needed
    int ring = 64;
    while (ring < d.M && (size_t)ring * 2 * WC * 8 <= 96 * 1024) ring *= 2;
    p.ring = ring;
    int threads = d.max_node_level_width * WC;
    threads = threads < 64 ? 64 : (threads > 1024 ? 1024 : (threads + 63) / 64 * 64);
    const size_t lds = (size_t)ring * WC * 8 + (size_t)4 * (threads / WC) * 16 + (size_t)(LVL_CHUNK + WC + 3) * 4;
    // threads must be a multiple of WC so that a thread keeps its word: 64 | threads and WC | 64
    auto kern = propagate_nodes<WC>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const int blocks = (d.W + WC - 1) / WC;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), lds, s, p);
    return hipGetLastError();
}

hipError_t launch_propagate(const Dag &d, hipStream_t s)
{
    if (d.n == 0 || d.W == 0) return hipSuccess;
    hipError_t e = hipSuccess;
    if (d.M > 0) {
        if (d.W <= 1) e = launch_nodes<1>(d, s);
        else if (d.W <= 2) e = launch_nodes<2>(d, s);
        else e = launch_nodes<4>(d, s);
        if (e != hipSuccess) return e;
    }
    const size_t total = (size_t)d.n * d.W;
    hipLaunchKernelGGL(expand_rows, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, d.n, d.W, d.d_src, d.d_dep);
    return hipGetLastError();
}

}  // namespace tictac
