// Dependency-bitset propagation (Sec. 4.1, Communication Dependency):
//   dep[v] = ({i} if v is recv i) | OR over predecessors u of dep[u].
//
// Bit columns are independent of each other, so the words of a row are split into
// slices of WC consecutive words and every workgroup owns one slice for all ops.  A
// workgroup walks the levels of the DAG (level = longest path from a root) in order
// and only ever reads words that it wrote itself at an earlier level, so a
// workgroup barrier per level is the only synchronisation and no two workgroups
// communicate.
#include "internal.h"

namespace tictac {

template <int WC>
__global__ void __launch_bounds__(1024)
propagate_levels(int32_t n_levels, int32_t W, const int32_t *__restrict__ lvl_ptr,
                 const int32_t *__restrict__ lvl_ops, const int32_t *__restrict__ row_ptr,
                 const int32_t *__restrict__ col_idx, const int32_t *__restrict__ recv_of_op,
                 uint64_t *dep)
{
    const int32_t w0 = blockIdx.x * WC;
    for (int32_t lv = 0; lv < n_levels; ++lv) {
        const int32_t beg = lvl_ptr[lv], cnt = lvl_ptr[lv + 1] - beg;
        for (int32_t item = threadIdx.x; item < cnt * WC; item += blockDim.x) {
            const int32_t k = item / WC, w = w0 + item % WC;
            if (w >= W) continue;
            const int32_t v = lvl_ops[beg + k];
            const int32_t ri = recv_of_op[v];
            uint64_t val = (ri >= 0 && (ri >> 6) == w) ? (uint64_t)1 << (ri & 63) : 0;
            for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e)
                val |= dep[(size_t)col_idx[e] * W + w];
            dep[(size_t)v * W + w] = val;
        }
        __syncthreads();   // also orders this workgroup's global writes before its later reads
    }
}

hipError_t launch_propagate(const Dag &d, hipStream_t s)
{
    if (d.n == 0 || d.W == 0) return hipSuccess;
    constexpr int WC = 8;
    const int blocks = (d.W + WC - 1) / WC;
    int threads = d.max_level_width * WC;
    threads = threads < 64 ? 64 : (threads > 1024 ? 1024 : (threads + 63) / 64 * 64);
    hipLaunchKernelGGL(propagate_levels<WC>, dim3(blocks), dim3(threads), 0, s, d.n_levels, d.W, d.d_lvl_ptr,
                       d.d_lvl_ops, d.d_row_ptr, d.d_col_idx, d.d_recv_of_op, d.d_dep);
    return hipGetLastError();
}

}  // namespace tictac
