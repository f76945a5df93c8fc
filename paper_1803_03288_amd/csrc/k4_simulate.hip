// One iteration under a transfer order, for a batch of timing samples (Sec. 3.2; channel
// model of Sec. 5.1).  One workgroup per sample.
//
// The channel never waits (recvs are roots and are all requested at t = 0), so the k-th
// transfer of the order ends at F_k = sum of the first k transfer times.  A compute op
// can start once the last of the recvs it depends on has arrived, i.e. after
// kappa = max position of dep[op] in the order (0 if it depends on no recv); ops of a
// class (identical dep) share kappa.  A device that never idles while an op is ready
// finishes the work released up to transfer k at
//     busy_0 = A_0,   busy_k = max(busy_{k-1}, F_k) + A_k,
// A_k = total time of the classes with kappa = k, whatever ready op it picks first
// (a predecessor of a released op was released no later).  makespan = max(busy_R, F_R).
#include "device_utils.h"
#include "internal.h"

namespace tictac {

struct SimKernelParams {
    int32_t B, R, W, C, N;
    const uint64_t *cls_dep;    // [C][W]
    const int32_t *cls_ptr;     // [C+1]
    const int32_t *cls_cols;    // [N]
    const int32_t *order;       // [R] or [B][R]
    int32_t order_stride;
    const int32_t *kappa;       // [C] for a shared order, else NULL
    const double *op_time, *recv_time;
    double *makespan, *eff, *U, *L, *S;
};

// 1-based position of every recv in an order shared by all samples
__global__ void __launch_bounds__(256)
position_kernel(int32_t R, const int32_t *__restrict__ order, int32_t *pos /*[R]*/)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k < R && (unsigned)order[k] < (unsigned)R) pos[order[k]] = k + 1;
}

// kappa of every class under that order
__global__ void __launch_bounds__(256)
kappa_kernel(int32_t W, int32_t C, const uint64_t *__restrict__ cls_dep, const int32_t *__restrict__ pos,
             int32_t *kappa /*[C]*/)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    int kap = 0;
    const uint64_t *row = cls_dep + (size_t)c * W;
    for (int w = 0; w < W; ++w) {
        uint64_t x = row[w];
        while (x) {
            kap = max(kap, pos[w * 64 + __builtin_ctzll(x)]);
            x &= x - 1;
        }
    }
    kappa[c] = kap;
}

template <int BS>
__global__ void __launch_bounds__(BS)
simulate_kernel(const SimKernelParams p)
{
    extern __shared__ double smem[];
    const int R = p.R, W = p.W, C = p.C, N = p.N;
    const int tid = threadIdx.x;
    double *Fs = smem;                  // [R+1] F_k
    double *A = Fs + (R + 1);           // [R+1] A_k
    double *red = A + (R + 1);          // [16]
    int32_t *pos = reinterpret_cast<int32_t *>(red + 16);   // [R] 1-based position of recv r

    for (int b = blockIdx.x; b < p.B; b += gridDim.x) {
        const double *rt = p.recv_time + (size_t)b * R;
        const double *ot = p.op_time + (size_t)b * N;
        const int32_t *ord = p.order + (size_t)b * p.order_stride;
        __syncthreads();
        for (int k = tid; k < R; k += BS) {
            const int r = ord[k];
            const bool ok = (unsigned)r < (unsigned)R;   // an invalid entry is skipped, never dereferenced
            if (ok) pos[r] = k + 1;
            Fs[k + 1] = ok ? rt[r] : 0.0;   // transfer time of the k-th transfer, summed below
        }
        for (int k = tid; k <= R; k += BS) A[k] = 0.0;
        if (tid == 0) Fs[0] = 0.0;
        __syncthreads();

        double ct_sum = 0.0;
        for (int c0 = 0; c0 < C; c0 += BS) {
            const int c = c0 + tid;
            const bool valid = c < C;
            double s = 0.0;
            int kap = 0;
            if (valid) {
                for (int m = p.cls_ptr[c]; m < p.cls_ptr[c + 1]; ++m) s += ot[p.cls_cols[m]];
                if (p.kappa) {
                    kap = p.kappa[c];
                } else {
                    const uint64_t *row = p.cls_dep + (size_t)c * W;
                    for (int w = 0; w < W; ++w) {
                        uint64_t x = row[w];
                        while (x) {
                            kap = max(kap, pos[w * 64 + __builtin_ctzll(x)]);
                            x &= x - 1;
                        }
                    }
                }
                ct_sum += s;
            }
            lds_scatter_add<BS>(A, kap, s, valid);
        }
        const double sum_c = block_sum_f64<BS>(ct_sum, red);
        __syncthreads();
        if (tid == 0) {
            double F = 0.0, busy = A[0];
            for (int k = 1; k <= R; ++k) {
                F += Fs[k];
                busy = fmax(busy, F) + A[k];
            }
            const double m = fmax(busy, F);
            const double U = sum_c + F;
            const double L = fmax(sum_c, F);
            p.makespan[b] = m;
            p.eff[b] = (U == L) ? 1.0 : (U - m) / (U - L);
            if (p.U) p.U[b] = U;
            if (p.L) p.L[b] = L;
            if (p.S) p.S[b] = (U == L || L == 0.0) ? 0.0 : (U - L) / L;
        }
    }
}

template <int BS>
static hipError_t launch_sim_t(const SimKernelParams &p, int grid, size_t lds, hipStream_t s)
{
    auto kern = simulate_kernel<BS>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(BS), lds, s, p);
    return hipGetLastError();
}

hipError_t launch_simulate(Dag &d, const SimArgs &a, hipStream_t s)
{
    if (a.B == 0) return hipSuccess;
    SimKernelParams p{};
    p.B = a.B; p.R = d.R; p.W = d.W; p.C = d.C; p.N = d.N;
    p.cls_dep = d.d_cls_dep; p.cls_ptr = d.d_cls_ptr; p.cls_cols = d.d_cls_cols;
    p.order = a.order; p.order_stride = a.order_stride; p.kappa = nullptr;
    p.op_time = a.op_time; p.recv_time = a.recv_time;
    p.makespan = a.makespan; p.eff = a.eff; p.U = a.U; p.L = a.L; p.S = a.S;
    if (a.order_stride == 0 && d.R > 0 && d.C > 0) {
        hipError_t e = ensure_workspace(&d, ((size_t)d.R + d.C) * sizeof(int32_t));
        if (e != hipSuccess) return e;
        int32_t *pos = static_cast<int32_t *>(d.d_work);
        int32_t *kappa = pos + d.R;
        hipLaunchKernelGGL(position_kernel, dim3((d.R + 255) / 256), dim3(256), 0, s, d.R, a.order, pos);
        hipLaunchKernelGGL(kappa_kernel, dim3((d.C + 255) / 256), dim3(256), 0, s, d.W, d.C, d.d_cls_dep, pos, kappa);
        p.kappa = kappa;
    }
    const size_t lds = ((size_t)(d.R + 1) * 2 + 16) * 8 + (size_t)d.R * 4;
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    if (d.C <= 2048 && lds <= 40 * 1024) {
        const int grid = a.B < 256 * 16 ? a.B : 256 * 16;
        return launch_sim_t<64>(p, grid, lds, s);
    }
    const int grid = a.B < 256 * 2 ? a.B : 256 * 2;
    return launch_sim_t<1024>(p, grid, lds, s);
}

}  // namespace tictac
