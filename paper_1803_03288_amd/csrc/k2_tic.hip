// TIC (Sec. 4.2, Algorithm 2): with every recv outstanding and the General Time Oracle
// (recv = 1, others = 0), op.M = |op.dep|, every P is 0 and
//   priority(recv i) = M+ = min{ |dep[v]| : v a compute op, i in dep[v], |dep[v]| > 1 }.
// Integer arithmetic throughout, so the result does not depend on the order of the
// min-updates.
#include "internal.h"

namespace tictac {

__global__ void fill_i32(int32_t *p, int32_t n, int32_t value)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

// One wave per row at a time: popcount of the row, then a min-update of every recv in it.
// USE_LDS: the block keeps its own copy of prio in LDS and merges it at the end.
template <bool USE_LDS>
__global__ void __launch_bounds__(256)
tic_min_kernel(int32_t n, int32_t R, int32_t W, const uint64_t *__restrict__ dep,
               const int32_t *__restrict__ recv_of_op, int32_t rows_per_block, int32_t *prio)
{
    extern __shared__ int32_t prio_l[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    if (USE_LDS) {
        for (int32_t i = threadIdx.x; i < R; i += blockDim.x) prio_l[i] = TICTAC_PRIO_INF;
        __syncthreads();
    }
    int32_t *target = USE_LDS ? prio_l : prio;
    const int32_t v0 = blockIdx.x * rows_per_block;
    const int32_t v1 = min(n, v0 + rows_per_block);
    for (int32_t v = v0 + wave; v < v1; v += n_waves) {
        if (recv_of_op[v] >= 0) continue;                 // wave-uniform
        const uint64_t *row = dep + (size_t)v * W;
        int32_t cnt = 0;
        for (int32_t w = lane; w < W; w += 64) cnt += __popcll(row[w]);
        for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off);
        if (cnt <= 1) continue;                           // wave-uniform
        for (int32_t w = lane; w < W; w += 64) {
            uint64_t x = row[w];
            while (x) {
                const int b = __builtin_ctzll(x);
                x &= x - 1;
                atomicMin(&target[w * 64 + b], cnt);
            }
        }
    }
    if (USE_LDS) {
        __syncthreads();
        for (int32_t i = threadIdx.x; i < R; i += blockDim.x)
            if (prio_l[i] != TICTAC_PRIO_INF) atomicMin(&prio[i], prio_l[i]);
    }
}

// rank[i] = number of recvs j with (prio[j], j) < (prio[i], i); order[rank[i]] = i.
__global__ void __launch_bounds__(256)
tic_rank_kernel(int32_t R, const int32_t *__restrict__ prio, int32_t *order, int32_t *rank)
{
    __shared__ int32_t tile[1024];
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const int32_t pi = (i < R) ? prio[i] : 0;
    int32_t r = 0;
    for (int32_t j0 = 0; j0 < R; j0 += 1024) {
        const int32_t m = min(1024, R - j0);
        __syncthreads();
        for (int32_t j = threadIdx.x; j < m; j += blockDim.x) tile[j] = prio[j0 + j];
        __syncthreads();
        if (i < R)
            for (int32_t j = 0; j < m; ++j) {
                const int32_t pj = tile[j];
                r += (pj < pi) || (pj == pi && (j0 + j) < i);
            }
    }
    if (i < R) {
        if (rank) rank[i] = r;
        if (order) order[r] = i;
    }
}

// Small graphs in one launch of one workgroup: thread i owns recv i, takes the minimum of
// |dep| over the classes (compute ops with identical rows) whose row holds i, and ranks
// itself by counting.  depT is the transposed class table [W][Cpad].  When the table and the
// class sizes fit (lds_words > 0: W * Cpad words, then C counts), the workgroup first copies them
// to LDS with all its threads, so that the loop over the classes does not wait on memory.
__global__ void __launch_bounds__(1024)
tic_small_kernel(int32_t R, int32_t C, int32_t Cpad, int32_t lds_words, const uint64_t *__restrict__ depT,
                 const int32_t *__restrict__ cnt0, int32_t *prio, int32_t *order, int32_t *rank)
{
    extern __shared__ uint64_t tic_table[];         // [lds_words] depT, then [C] counts
    __shared__ int32_t tile[1024];
    const int32_t i = threadIdx.x;
    if (lds_words > 0) {
        int32_t *cnt_l = reinterpret_cast<int32_t *>(tic_table + lds_words);
        for (int32_t x = i; x < lds_words; x += blockDim.x) tic_table[x] = depT[x];
        for (int32_t c = i; c < C; c += blockDim.x) cnt_l[c] = cnt0[c];
        __syncthreads();
    }
    int32_t m = TICTAC_PRIO_INF;
    if (i < R) {
        const int sh = i & 63;
        if (lds_words > 0) {
            const uint64_t *col = tic_table + (size_t)(i >> 6) * Cpad;
            const int32_t *cnt_l = reinterpret_cast<const int32_t *>(tic_table + lds_words);
#pragma unroll 4
            for (int32_t c = 0; c < C; ++c) {
                const int32_t k = cnt_l[c];
                if (((col[c] >> sh) & 1ull) && k > 1) m = min(m, k);
            }
        } else {
            const uint64_t *col = depT + (size_t)(i >> 6) * Cpad;   // the same word for the 64 lanes of a wave
#pragma unroll 8
            for (int32_t c = 0; c < C; ++c) {
                const int32_t k = cnt0[c];
                if (((col[c] >> sh) & 1ull) && k > 1) m = min(m, k);
            }
        }
        prio[i] = m;
    }
    tile[i] = m;
    __syncthreads();
    if (i < R && (order || rank)) {
        int32_t r = 0;
        for (int32_t j = 0; j < R; ++j) {
            const int32_t pj = tile[j];
            r += (pj < m) || (pj == m && j < i);
        }
        if (rank) rank[i] = r;
        if (order) order[r] = i;
    }
}

hipError_t launch_tic(const Dag &d, int32_t *prio, int32_t *order, int32_t *rank, int32_t *, hipStream_t s)
{
    const int32_t R = d.R;
    if (R == 0) return hipSuccess;
    if (R <= 1024 && d.C <= 8192 && d.d_cls_depT && d.d_cls_cnt0) {
        int threads = (R + 63) / 64 * 64;
        const size_t words = (size_t)d.W * d.Cpad;
        const size_t lds = words * 8 + (size_t)d.C * 4;
        const bool in_lds = lds <= 40 * 1024;
        if (in_lds && threads < 256) threads = 256;     // more threads for the copy
        hipLaunchKernelGGL(tic_small_kernel, dim3(1), dim3(threads), in_lds ? lds : 0, s, R, d.C, d.Cpad,
                           in_lds ? (int32_t)words : 0, d.d_cls_depT, d.d_cls_cnt0, prio, order, rank);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(fill_i32, dim3((R + 255) / 256), dim3(256), 0, s, prio, R, (int32_t)TICTAC_PRIO_INF);
    if (d.n > 0) {
        const int32_t rows_per_block = d.n <= 4096 ? 32 : 128;
        const int blocks = (d.n + rows_per_block - 1) / rows_per_block;
        const size_t lds = (size_t)R * sizeof(int32_t);
        if (lds <= 48 * 1024)
            hipLaunchKernelGGL(tic_min_kernel<true>, dim3(blocks), dim3(256), lds, s, d.n, R, d.W, d.d_dep,
                               d.d_recv_of_op, rows_per_block, prio);
        else
            hipLaunchKernelGGL(tic_min_kernel<false>, dim3(blocks), dim3(256), 0, s, d.n, R, d.W, d.d_dep,
                               d.d_recv_of_op, rows_per_block, prio);
    }
    if (order || rank)
        hipLaunchKernelGGL(tic_rank_kernel, dim3((R + 255) / 256), dim3(256), 0, s, R, prio, order, rank);
    return hipGetLastError();
}

}  // namespace tictac
