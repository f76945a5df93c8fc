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

// ---- class grouping on the device (see internal.h) ----
__device__ __forceinline__ uint64_t mix64(uint64_t h, uint64_t x, uint64_t k)
{
    h ^= x + k + (h << 6) + (h >> 2);
    return h * 0xFF51AFD7ED558CCDull;
}

// one wave per compute op: lanes take words lane, lane + 64, ...; the two hashes mix the words in index order, so
// they are formed by lane 0 from the words gathered through LDS-free cross-lane reads, 64 words at a time
__global__ void __launch_bounds__(256)
row_digest_kernel(int32_t N, int32_t W, const int32_t *__restrict__ op_of_col, const uint64_t *__restrict__ dep,
                  int32_t *__restrict__ digest)
{
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= N) return;
    const uint64_t *row = dep + (size_t)op_of_col[j] * W;
    uint64_t h0 = 0x9E3779B97F4A7C15ull, h1 = 0xC2B2AE3D27D4EB4Full;
    int cnt = 0, lowest = -1;
    for (int w0 = 0; w0 < W; w0 += 64) {
        const uint64_t x = w0 + lane < W ? row[w0 + lane] : 0ull;
        cnt += __builtin_popcountll(x);
        const uint64_t has = __ballot(x != 0ull);
        if (lowest < 0 && has != 0ull) {
            const int l = __builtin_ctzll(has);
            const uint64_t xl = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(x >> 32), l) << 32) |
                                (uint32_t)__builtin_amdgcn_readlane((int)x, l);
            lowest = (w0 + l) * 64 + __builtin_ctzll(xl);
        }
        // position-dependent contribution of every word, combined by a sum: independent of the order of the lanes
        const uint64_t k = (uint64_t)(w0 + lane) * 0x9E3779B97F4A7C15ull;
        uint64_t a = mix64(0x243F6A8885A308D3ull ^ k, x, 0x9E3779B97F4A7C15ull);
        uint64_t b = mix64(0x13198A2E03707344ull + k, x ^ (x >> 29), 0xA4093822299F31D0ull);
        a ^= a >> 32; b ^= b >> 31;
        if (x == 0ull) { a = 0; b = 0; }            // (rows are sparse; an absent word adds nothing)
        for (int off = 32; off > 0; off >>= 1) {
            a += ((uint64_t)(uint32_t)__shfl_xor((int)(a >> 32), off) << 32) | (uint32_t)__shfl_xor((int)a, off);
            b += ((uint64_t)(uint32_t)__shfl_xor((int)(b >> 32), off) << 32) | (uint32_t)__shfl_xor((int)b, off);
        }
        h0 = mix64(h0, a, 0x9E3779B97F4A7C15ull);
        h1 = mix64(h1, b, 0x452821E638D01377ull);
    }
    for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off);
    if (lane == 0) {
        int32_t *o = digest + (size_t)j * 8;
        o[0] = (int32_t)h0; o[1] = (int32_t)(h0 >> 32); o[2] = (int32_t)h1; o[3] = (int32_t)(h1 >> 32);
        o[4] = cnt; o[5] = lowest; o[6] = 0; o[7] = 0;
    }
}

hipError_t launch_row_digests(const Dag &d, const int32_t *op_of_col, int32_t *digest, hipStream_t s)
{
    if (d.N == 0) return hipSuccess;
    hipLaunchKernelGGL(row_digest_kernel, dim3((d.N + 3) / 4), dim3(256), 0, s, d.N, d.W, op_of_col, d.d_dep, digest);
    return hipGetLastError();
}

// thread per (class, word): the class's row from its first op, into cls_dep and cls_depT
__global__ void __launch_bounds__(256)
class_rows_kernel(int32_t C, int32_t Cpad, int32_t W, const int32_t *__restrict__ first_op,
                  const uint64_t *__restrict__ dep, uint64_t *__restrict__ cls_dep, uint64_t *__restrict__ cls_depT)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)Cpad * W) return;
    const int c = (int)(idx / W), w = (int)(idx % W);
    const uint64_t x = c < C ? dep[(size_t)first_op[c] * W + w] : 0ull;
    if (c < C) cls_dep[idx] = x;
    cls_depT[(size_t)w * Cpad + c] = x;
}

// thread per (compute op, word): the op's row against the row of its class
__global__ void __launch_bounds__(256)
class_check_kernel(int32_t N, int32_t W, const int32_t *__restrict__ op_of_col, const int32_t *__restrict__ col_cls,
                   const uint64_t *__restrict__ dep, const uint64_t *__restrict__ cls_dep, int32_t *mismatch)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)N * W) return;
    const int j = (int)(idx / W), w = (int)(idx % W);
    if (dep[(size_t)op_of_col[j] * W + w] != cls_dep[(size_t)col_cls[j] * W + w]) atomicOr(mismatch, 1);
}

hipError_t launch_class_rows(const Dag &d, const int32_t *op_of_col, const int32_t *first_op, int32_t *mismatch,
                             hipStream_t s)
{
    if (d.C == 0 || d.W == 0) return hipSuccess;
    const size_t total = (size_t)d.Cpad * d.W;
    hipLaunchKernelGGL(class_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, d.C, d.Cpad, d.W,
                       first_op, d.d_dep, d.d_cls_dep, d.d_cls_depT);
    const size_t all = (size_t)d.N * d.W;
    hipLaunchKernelGGL(class_check_kernel, dim3((unsigned)((all + 255) / 256)), dim3(256), 0, s, d.N, d.W, op_of_col,
                       d.d_col_cls, d.d_dep, d.d_cls_dep, mismatch);
    return hipGetLastError();
}

}  // namespace tictac
