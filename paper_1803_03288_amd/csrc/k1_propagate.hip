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
// memory.  The record of a thread's first node of the next level is loaded one level ahead.
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

__device__ __forceinline__ NodeRec load_rec(const NodeRec *p)
{
    const int4 *q = reinterpret_cast<const int4 *>(p);
    const int4 a = q[0], b = q[1];
    NodeRec r;
    r.in[0] = a.x; r.in[1] = a.y; r.in[2] = a.z; r.in[3] = a.w;
    r.op = b.x; r.ovf_beg = b.y; r.ovf_cnt = b.z; r.pad = b.w;
    return r;
}

template <int WC>
__global__ void __launch_bounds__(1024)
propagate_nodes(const PropParams p)
{
    extern __shared__ uint64_t ring[];                  // [ring][WC]
    const int W = p.W;
    const int w = threadIdx.x % WC;                     // word of the slice
    const int gw = blockIdx.x * WC + w;                 // word of the row
    const int sub = threadIdx.x / WC;                   // node within a pass over a level
    const int per_pass = blockDim.x / WC;
    const uint32_t rmask = (uint32_t)p.ring - 1u;

    int beg = p.nlvl_ptr[0], end = p.n_levels > 0 ? p.nlvl_ptr[1] : 0;
    NodeRec cur;
    if (beg + sub < end) cur = load_rec(p.nodes + beg + sub);
    for (int lv = 0; lv < p.n_levels; ++lv) {
        // the record this thread needs first at the next level
        const int nbeg = end, nend = lv + 1 < p.n_levels ? p.nlvl_ptr[lv + 2] : end;
        NodeRec nxt;
        if (lv + 1 < p.n_levels && nbeg + sub < nend) nxt = load_rec(p.nodes + nbeg + sub);

        const int safe_from = end - p.ring;             // positions >= safe_from are still in the ring
        for (int pos = beg + sub; pos < end; pos += per_pass) {
            const NodeRec rec = (pos == beg + sub) ? cur : load_rec(p.nodes + pos);
            uint64_t val = 0;
            if (gw < W) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int x = rec.in[j];
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
                for (int e = 0; e < rec.ovf_cnt; ++e) {
                    const int x = p.ovf_idx[rec.ovf_beg + e];
                    if (x < 0) {
                        const int i = ~x;
                        if ((i >> 6) == gw) val |= 1ull << (i & 63);
                    } else if (x >= safe_from) {
                        val |= ring[((uint32_t)x & rmask) * WC + w];
                    } else {
                        val |= p.dep[(size_t)p.nodes[x].op * W + gw];
                    }
                }
                p.dep[(size_t)rec.op * W + gw] = val;
            }
            ring[((uint32_t)pos & rmask) * WC + w] = val;
        }
        __syncthreads();   // orders the ring and this workgroup's global writes before later reads
        beg = nbeg; end = nend; cur = nxt;
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
    // ring: the largest power of two of positions within 128 KB, no larger than needed
    int ring = 64;
    while (ring < d.M && (size_t)ring * 2 * WC * 8 <= 128 * 1024) ring *= 2;
    p.ring = ring;
    const size_t lds = (size_t)ring * WC * 8;
    int threads = d.max_node_level_width * WC;
    threads = threads < 64 ? 64 : (threads > 1024 ? 1024 : (threads + 63) / 64 * 64);
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
        else if (d.W <= 4) e = launch_nodes<4>(d, s);
        else e = launch_nodes<8>(d, s);
        if (e != hipSuccess) return e;
    }
    const size_t total = (size_t)d.n * d.W;
    hipLaunchKernelGGL(expand_rows, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, d.n, d.W, d.d_src, d.d_dep);
    return hipGetLastError();
}

}  // namespace tictac
