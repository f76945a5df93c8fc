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
#include <algorithm>

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
    const void *op_time, *recv_time;    // float64, or float32 when f32 is set
    int32_t f32;
    double *makespan, *eff, *U, *L, *S;
};

// 1-based position of every recv in an order shared by all samples (one workgroup; 0 for a recv that an
// invalid order leaves out, so that every position read later is in 0 .. R)
__global__ void __launch_bounds__(256)
position_kernel(int32_t R, const int32_t *__restrict__ order, int32_t *pos /*[R]*/)
{
    for (int k = threadIdx.x; k < R; k += 256) pos[k] = 0;
    __syncthreads();
    for (int k = threadIdx.x; k < R; k += 256)
        if ((unsigned)order[k] < (unsigned)R) pos[order[k]] = k + 1;
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
        const TimeRow rt = time_row(p.recv_time, (size_t)b * R, p.f32 != 0);
        const TimeRow ot = time_row(p.op_time, (size_t)b * N, p.f32 != 0);
        const int32_t *ord = p.order + (size_t)b * p.order_stride;
        __syncthreads();
        for (int k = tid; k < R; k += BS) pos[k] = 0;   // (a recv that an invalid order leaves out: position 0)
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

// The same computation with one wavefront per sample, for graphs with at most 8 classes per
// lane and at most 512 recvs.  Lane l owns the classes l, l + 64, ... and the positions l,
// l + 64, ... of the order; a workgroup is four independent waves.  Per sample: the transfer
// times and the order are requested first, into registers, then the op_time row is read once,
// coalesced, every run of columns of one class adding itself to the total of its class in LDS
// (so one trip to memory per sample is waited for, not three); kappa of a class is the maximum of the positions of its recvs, taken run by run of
// consecutive recv indices from a sparse table of range maxima over the position array (or read
// from a table when all samples share one order); then A by kappa, and
//     makespan = max over k of F_k + (A_k + ... + A_R),   F_0 = 0,
// which is the recurrence above unrolled.
struct SimWaveParams {
    int32_t B, R, C, N, n_waves, wave_bytes, levels;
    const int32_t *col_cls;     // [N] class of every op_time column
    const int32_t *run_ptr;     // [C+1] runs [run_lo, run_hi) of consecutive recv indices of the class rows
    const int32_t *run_lo, *run_hi;
    const int32_t *order;
    int32_t order_stride;
    const int32_t *kappa;       // [C] for a shared order, else NULL
    const void *op_time, *recv_time;    // float64, or float32 when f32 is set
    int32_t f32;
    double *makespan, *eff, *U, *L, *S;
};

constexpr int kSimWaves = 4;

#define SW_EACH_K(F) F(0) F(1) F(2) F(3) F(4) F(5) F(6) F(7)

template <int KT>
__global__ void __launch_bounds__(64 * kSimWaves, KT <= 3 ? 5 : (KT <= 4 ? 4 : 2))
simulate_wave_kernel(const SimWaveParams p)
{
    extern __shared__ double smem[];
    const int R = p.R, C = p.C, N = p.N;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    char *mine = reinterpret_cast<char *>(smem) + (size_t)wave * p.wave_bytes;
    double *t = reinterpret_cast<double *>(mine);           // [R]   Time(recv)
    double *F = t + R;                                      // [R]   F[k-1] = end of the k-th transfer
    double *A = F + R;                                      // [R+1] class time by kappa
    double *csum = F;                                       // [64 KT] class totals while they are summed (spans F and A)
    uint16_t *pos = reinterpret_cast<uint16_t *>(A + (R + 1));   // [levels][R] range maxima of the 1-based positions

    // Per class slot, fixed for the launch: kappa from the table when all samples share one order,
    // else the first two runs of the class row (lo | hi << 16; longer rows read the rest from memory).
#define SW_RUNS(k)                                                                        \
    int rb_##k = 0, re_##k = 0;                                                           \
    unsigned ra_##k = 0, rc_##k = 0;                                                      \
    if constexpr (k < KT) {                                                               \
        const int c = k * 64 + lane;                                                      \
        if (c < C) {                                                                      \
            if (p.kappa) {                                                                \
                ra_##k = (unsigned)p.kappa[c];                                            \
            } else {                                                                      \
                rb_##k = p.run_ptr[c];                                                    \
                re_##k = p.run_ptr[c + 1];                                                \
                if (re_##k > rb_##k) ra_##k = (unsigned)p.run_lo[rb_##k] | ((unsigned)p.run_hi[rb_##k] << 16);              \
                if (re_##k > rb_##k + 1) rc_##k = (unsigned)p.run_lo[rb_##k + 1] | ((unsigned)p.run_hi[rb_##k + 1] << 16);  \
            }                                                                             \
        }                                                                                 \
    }
    SW_EACH_K(SW_RUNS)

    const int gwave = blockIdx.x * kSimWaves + wave;
    for (int b = gwave; b < p.B; b += p.n_waves) {
        const TimeRow rt = time_row(p.recv_time, (size_t)b * R, p.f32 != 0);
        const TimeRow ot = time_row(p.op_time, (size_t)b * N, p.f32 != 0);
        const int32_t *ord = p.order + (size_t)b * p.order_stride;
        wave_sync();                        // LDS of the previous sample is no longer read

        // ---- everything the sample reads from memory is requested here: the transfer times and
        // the order into registers (position slot q: r = q * 64 + lane), then the op_time row ----
#define SW_REQUEST(q)                                                                     \
        double rt_##q = 0.0;                                                              \
        int or_##q = -1;                                                                  \
        if constexpr (q < KT) {                                                           \
            if (q * 64 + lane < R) { rt_##q = rt[q * 64 + lane]; or_##q = ord[q * 64 + lane]; } \
        }
        SW_EACH_K(SW_REQUEST)
        for (int c = lane; c < 64 * KT; c += 64) csum[c] = 0.0;
        wave_sync();
        class_totals(csum, ot, p.col_cls, N, lane);
        wave_sync();
#define SW_DECL(k) double ct_##k = 0.0; int kap_##k = 0;
        SW_EACH_K(SW_DECL)
#define SW_TOTAL(k) if constexpr (k < KT) { ct_##k = csum[k * 64 + lane]; }
        SW_EACH_K(SW_TOTAL)
#define SW_TIMES(q) if constexpr (q < KT) { if (q * 64 + lane < R) { t[q * 64 + lane] = rt_##q; pos[q * 64 + lane] = 0; } }
        SW_EACH_K(SW_TIMES)
        wave_sync();

        // ---- positions, F ----
        double fc = 0.0;
#define SW_PLACE(q)                                                                       \
        if constexpr (q < KT) {                                                           \
            if (q * 64 < R) {                                                             \
                const int s = q * 64 + lane;                                              \
                const int r = or_##q;                                                     \
                const bool ok = (unsigned)r < (unsigned)R;  /* an invalid entry is skipped, never dereferenced */ \
                if (ok) pos[r] = (uint16_t)(s + 1);                                       \
                const double x = ok ? t[r] : 0.0;                                         \
                const double inc = wave_incl_scan_f64_dpp(x);                             \
                if (s < R) F[s] = fc + inc;                                               \
                fc += lane63_f64(inc);                                                    \
            }                                                                             \
        }
        SW_EACH_K(SW_PLACE)
        const double Ftot = fc;
        for (int j = lane; j <= R; j += 64) A[j] = 0.0;
        wave_sync();

        // ---- kappa ----
        if (p.kappa) {
#define SW_KAPPA_TABLE(k) if constexpr (k < KT) { kap_##k = (int)ra_##k; }
            SW_EACH_K(SW_KAPPA_TABLE)
        } else {
            // level j of the table: maximum over [i, min(i + 2^j, R))
            for (int j = 1; j < p.levels; ++j) {
                const uint16_t *prev = pos + (size_t)(j - 1) * R;
                uint16_t *cur = pos + (size_t)j * R;
                const int h = 1 << (j - 1);
                for (int i = lane; i < R; i += 64) cur[i] = max(prev[i], prev[min(i + h, R - 1)]);
                wave_sync();
            }
#define SW_RANGE_MAX(lo, hi)                                                              \
                    {                                                                     \
                        const int j_ = 31 - __builtin_clz((hi) - (lo));                   \
                        const uint16_t *lv_ = pos + (size_t)j_ * R;                       \
                        m = max(m, max((int)lv_[lo], (int)lv_[(hi) - (1 << j_)]));        \
                    }
#define SW_KAPPA_RUNS(k)                                                                  \
            if constexpr (k < KT) {                                                       \
                if (k * 64 + lane < C) {                                                  \
                    int m = 0;                                                            \
                    if (re_##k > rb_##k) SW_RANGE_MAX((int)(ra_##k & 0xffffu), (int)(ra_##k >> 16))          \
                    if (re_##k > rb_##k + 1) SW_RANGE_MAX((int)(rc_##k & 0xffffu), (int)(rc_##k >> 16))      \
                    for (int q = rb_##k + 2; q < re_##k; ++q) {                           \
                        const int lo = p.run_lo[q], hi = p.run_hi[q];                     \
                        SW_RANGE_MAX(lo, hi)                                              \
                    }                                                                     \
                    kap_##k = m;                                                          \
                }                                                                         \
            }
            SW_EACH_K(SW_KAPPA_RUNS)
        }

        // ---- A by kappa, suffix sums, makespan ----
        double ct_sum = 0.0;
#define SW_RELEASE(k) if constexpr (k < KT) { if (k * 64 + lane < C) atomicAdd(&A[kap_##k], ct_##k); ct_sum += ct_##k; }
        SW_EACH_K(SW_RELEASE)
        wave_sync();
        const double sum_c = wave_sum_f64_dpp(ct_sum);
        double sfx = 0.0, mloc = sum_c;                   // k = 0: F_0 + S_0 = all class time
        for (int base = ((R - 1) / 64) * 64; base >= 0; base -= 64) {
            const int k = base + lane + 1;                // 1 <= k <= R handled here
            const double x = k <= R ? A[k] : 0.0;
            const double inc = wave_incl_scan_f64_dpp(x);
            const double tot = lane63_f64(inc);
            if (k <= R) mloc = fmax(mloc, F[k - 1] + (sfx + (tot - inc + x)));
            sfx += tot;
        }
        const double m = wave_max_f64_dpp(mloc);
        if (lane == 0) {
            const double U = sum_c + Ftot;
            const double L = fmax(sum_c, Ftot);
            p.makespan[b] = m;
            p.eff[b] = (U == L) ? 1.0 : (U - m) / (U - L);
            if (p.U) p.U[b] = U;
            if (p.L) p.L[b] = L;
            if (p.S) p.S[b] = (U == L || L == 0.0) ? 0.0 : (U - L) / L;
        }
    }
}

template <int KT>
static hipError_t launch_sim_wave(SimWaveParams &p, const Dag &d, hipStream_t s)
{
    int levels = 1;
    while ((1 << levels) <= d.R) ++levels;            // floor(log2 R) + 1 levels of the table
    p.levels = levels;
    size_t wave_bytes = ((size_t)3 * d.R + 1) * 8 + (size_t)levels * d.R * 2;
    wave_bytes = (wave_bytes + 15) & ~(size_t)15;
    const size_t lds = wave_bytes * kSimWaves;
    if (lds > 150 * 1024) return hipErrorNotSupported;     // 160 KB of LDS per compute unit
    p.wave_bytes = (int32_t)wave_bytes;
    hipError_t e;
    if (lds > 48 * 1024) {
        e = ensure_dynamic_lds(reinterpret_cast<const void *>(simulate_wave_kernel<KT>), lds);
        if (e != hipSuccess) return e;
    }
    int per_cu = 0;
    e = cached_blocks_per_cu(&per_cu, reinterpret_cast<const void *>(simulate_wave_kernel<KT>), 64 * kSimWaves, lds);
    if (e != hipSuccess) return e;
    if (per_cu < 1) per_cu = 1;
    const int n_cu = device_cu_count(d.device);
    int grid = per_cu * n_cu;
    const int need = (p.B + kSimWaves - 1) / kSimWaves;
    if (grid > need) grid = need;
    p.n_waves = grid * kSimWaves;
    hipLaunchKernelGGL((simulate_wave_kernel<KT>), dim3(grid), dim3(64 * kSimWaves), lds, s, p);
    return hipGetLastError();
}

// hipErrorNotSupported: the graph is outside what the wave kernel handles
static hipError_t try_simulate_wave(const Dag &d, const SimArgs &a, const int32_t *kappa, hipStream_t s)
{
    const int K = std::max((d.C + 63) / 64, (d.R + 63) / 64);   // slots per lane: classes, and positions of the order
    const int KT = K;                                 // the instantiation that is launched below
    // (the class totals are summed in the space of F and A: one double per class slot must fit)
    if (d.R == 0 || d.R > 512 || d.C == 0 || K > 8 || !d.d_col_cls || !d.d_run_ptr || (size_t)64 * KT > 2 * (size_t)d.R + 1)
        return hipErrorNotSupported;
    SimWaveParams p{};
    p.B = a.B; p.R = d.R; p.C = d.C; p.N = d.N;
    p.col_cls = d.d_col_cls; p.run_ptr = d.d_run_ptr; p.run_lo = d.d_run_lo; p.run_hi = d.d_run_hi;
    p.order = a.order; p.order_stride = a.order_stride; p.kappa = kappa;
    p.op_time = a.op_time; p.recv_time = a.recv_time; p.f32 = a.f32 ? 1 : 0;
    p.makespan = a.makespan; p.eff = a.eff; p.U = a.U; p.L = a.L; p.S = a.S;
    if (K <= 1) return launch_sim_wave<1>(p, d, s);
    if (K <= 2) return launch_sim_wave<2>(p, d, s);
    if (K <= 3) return launch_sim_wave<3>(p, d, s);
    if (K <= 4) return launch_sim_wave<4>(p, d, s);
    if (K <= 5) return launch_sim_wave<5>(p, d, s);
    if (K <= 6) return launch_sim_wave<6>(p, d, s);
    if (K <= 7) return launch_sim_wave<7>(p, d, s);
    return launch_sim_wave<8>(p, d, s);
}

template <int BS>
static hipError_t launch_sim_t(const SimKernelParams &p, int grid, size_t lds, hipStream_t s)
{
    auto kern = simulate_kernel<BS>;
    if (lds > 48 * 1024) {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(BS), lds, s, p);
    return hipGetLastError();
}

// Several channels (Sec. 4.1: one per parameter server; Sec. 5.1: one transfer at a time per
// channel).  Recv i uses channel chan[i]; every channel serves its recvs back to back from
// t = 0 in the order in which they appear in the given order.  The channels never wait (recvs
// are roots), so recv r arrives at the sum of the transfer times queued up to and including it
// on its channel; a class is released when the last recv of its row has arrived (rho); and a
// device that never idles while an op is ready finishes at
//     max( latest arrival,  max over classes c of  rho_c + sum of the times of the classes with rho >= rho_c ).
// One wave per sample: arrivals by one wave scan per channel, rho by range maxima over the
// arrival array (runs of the class rows; lane l owns classes l, l + 64, ...), the last step by ranking the
// release dates among the arrivals: on one channel the arrivals increase along the order, so the number of
// arrivals up to rho is one binary search per channel; the class times are added up by that rank and one
// suffix sum over the ranks gives the second term for every class.
struct SimChanParams {
    int32_t B, R, C, N, n_waves, wave_bytes, levels, n_channels, chan_bytes;
    int32_t nb, x_doubles;      // blocks of four recvs; doubles shared by the transfer times and the table of block maxima
    const int32_t *col_cls, *run_ptr, *run_lo, *run_hi;
    const int32_t *chan;        // [R] channel of every recv, 0 <= chan < n_channels <= 64
    const int32_t *order;
    int32_t order_stride;
    const void *op_time, *recv_time;    // float64, or float32 when f32 is set
    int32_t f32;
    double *makespan, *eff, *U, *L, *S;
};

// (three waves per SIMD: 168 registers per lane; with a cap of 128 the kernel spills and is slower)
template <int KT>
__global__ void __launch_bounds__(256, 3)
simulate_channels_kernel(const SimChanParams p)
{
    extern __shared__ double smem[];
    const int R = p.R, C = p.C, N = p.N;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t *chan_l = reinterpret_cast<int32_t *>(smem);    // [R] channel of every recv, shared by the waves
    int32_t *coff = chan_l + R;             // [64] where the arrivals of a channel start in `lists`
    int32_t *clen = coff + 64;              // [64] recvs of a channel
    double *mine = reinterpret_cast<double *>(reinterpret_cast<char *>(smem) + p.chan_bytes + (size_t)wave * p.wave_bytes);
    const int Rp = (R + 3) & ~3, nb = p.nb;
    double *arr = mine;                     // [Rp] arrival of recv r, zero beyond R
    double *t = arr + Rp;                   // [R]  Time(recv), until the arrivals are known; then
    double *tab = t;                        // [levels][nb] level j: maxima of the arrivals over the blocks [i, i + 2^j) of four recvs
    double *csum = t + p.x_doubles;         // [64 KT] the class totals while they are summed; then
    double *lists = csum;                   // [R] the arrivals channel by channel, in the order's sequence
    for (int r = threadIdx.x; r < R; r += blockDim.x) chan_l[r] = p.chan[r];
    __syncthreads();
    if (wave == 0) {
        int n_mine = 0;                     // lane c: recvs of channel c
        for (int r = 0; r < R; ++r) n_mine += chan_l[r] == lane;
        int incl = n_mine;
        for (int off = 1; off < 64; off <<= 1) {
            const int v = __shfl_up(incl, off);
            if (lane >= off) incl += v;
        }
        coff[lane] = incl - n_mine;
        clen[lane] = n_mine;
    }
    __syncthreads();
    const uint64_t lanes_below = (1ull << lane) - 1ull;
    // the first two runs of every class row (lo | hi << 16), fixed for the launch; longer rows read the rest
#define SC_RUNS(k)                                                                        \
    int rb_##k = 0, re_##k = 0;                                                           \
    unsigned ra_##k = 0, rc_##k = 0;                                                      \
    if constexpr (k < KT) {                                                               \
        const int c = k * 64 + lane;                                                      \
        if (c < C) {                                                                      \
            rb_##k = p.run_ptr[c];                                                        \
            re_##k = p.run_ptr[c + 1];                                                    \
            if (re_##k > rb_##k) ra_##k = (unsigned)p.run_lo[rb_##k] | ((unsigned)p.run_hi[rb_##k] << 16);              \
            if (re_##k > rb_##k + 1) rc_##k = (unsigned)p.run_lo[rb_##k + 1] | ((unsigned)p.run_hi[rb_##k + 1] << 16);  \
        }                                                                                 \
    }
    SW_EACH_K(SC_RUNS)

    const int gwave = blockIdx.x * (blockDim.x >> 6) + wave;
    for (int b = gwave; b < p.B; b += p.n_waves) {
        const TimeRow rt = time_row(p.recv_time, (size_t)b * R, p.f32 != 0);
        const TimeRow ot = time_row(p.op_time, (size_t)b * N, p.f32 != 0);
        const int32_t *ord = p.order + (size_t)b * p.order_stride;
        wave_sync();

        // ---- transfer times and the order are requested first, into registers (position slot q:
        // q * 64 + lane), then the op_time row ----
#define SC_REQUEST(q)                                                                     \
        double rt_##q = 0.0;                                                              \
        int or_##q = -1;                                                                  \
        if constexpr (q < KT) {                                                           \
            if (q * 64 + lane < R) { rt_##q = rt[q * 64 + lane]; or_##q = ord[q * 64 + lane]; } \
        }
        SW_EACH_K(SC_REQUEST)
        for (int c = lane; c < 64 * KT; c += 64) csum[c] = 0.0;
        wave_sync();
        class_totals(csum, ot, p.col_cls, N, lane);
        wave_sync();
#define SC_DECL(k) double ct_##k = 0.0, rho_##k = 0.0;
        SW_EACH_K(SC_DECL)
#define SC_TOTAL(k) if constexpr (k < KT) { ct_##k = csum[k * 64 + lane]; }
        SW_EACH_K(SC_TOTAL)
#define SC_TIMES(q) if constexpr (q < KT) { if (q * 64 + lane < R) { t[q * 64 + lane] = rt_##q; arr[q * 64 + lane] = 0.0; } }
        SW_EACH_K(SC_TIMES)
        if (R + lane < Rp) arr[R + lane] = 0.0;
        wave_sync();

        // ---- arrivals: per channel, prefix sums over the positions of the order ----
        double carry = 0.0;                 // lane c: time queued on channel c so far
        int queued = 0;                     // lane c: recvs queued on channel c so far
        double sum_r = 0.0;
#define SC_ARRIVE(q)                                                                      \
        if constexpr (q < KT) {                                                           \
            if (q * 64 < R) {                                                             \
                const int r = or_##q;                                                     \
                const bool ok = (unsigned)r < (unsigned)R;  /* an invalid entry is skipped, never dereferenced */ \
                const int cl = ok ? chan_l[r] : -1;                                       \
                const double x = ok ? t[r] : 0.0;                                         \
                double a = 0.0;                                                           \
                int nth = 0;                        /* this recv is the nth of its channel */ \
                for (int c = 0; c < p.n_channels; ++c) {                                  \
                    const double inc = wave_incl_scan_f64_dpp(cl == c ? x : 0.0);         \
                    const double before = readlane_f64(carry, c);                         \
                    if (cl == c) a = before + inc;                                        \
                    if (lane == c) carry += lane63_f64(inc);                              \
                    const uint64_t on_c = __ballot(cl == c);                              \
                    const int n_before = __builtin_amdgcn_readlane(queued, c);            \
                    if (cl == c) nth = n_before + __popcll(on_c & lanes_below);           \
                    if (lane == c) queued += __popcll(on_c);                              \
                }                                                                         \
                if (ok) {                                                                 \
                    arr[r] = a;                                                           \
                    /* (an order that is no permutation cannot write past the channel's share) */ \
                    if (nth < clen[cl]) lists[coff[cl] + nth] = a;                        \
                }                                                                         \
                sum_r += x;                                                               \
            }                                                                             \
        }
        SW_EACH_K(SC_ARRIVE)
        sum_r = wave_sum_f64_dpp(sum_r);
        const double last_arrival = wave_max_f64_dpp(lane < p.n_channels ? carry : 0.0);   // = largest channel sum
        wave_sync();

        // ---- rho of every class: maximum arrival over the runs of its row ----
        // A run [lo, hi) is at most three recvs, whole blocks of four, and at most three recvs: the blocks are
        // looked up in a table of maxima over 2^j blocks (two reads), the recvs at the ends are read one by one.
        for (int i = lane; i < nb; i += 64) {
            const double2 x = *reinterpret_cast<const double2 *>(arr + 4 * i), y = *reinterpret_cast<const double2 *>(arr + 4 * i + 2);
            tab[i] = fmax(fmax(x.x, x.y), fmax(y.x, y.y));
        }
        wave_sync();
        for (int j = 1; j < p.levels; ++j) {
            const double *prev = tab + (size_t)(j - 1) * nb;
            double *cur = tab + (size_t)j * nb;
            const int h = 1 << (j - 1);
            for (int i = lane; i < nb; i += 64) cur[i] = fmax(prev[i], prev[min(i + h, nb - 1)]);
            wave_sync();
        }
#define SC_RANGE_MAX(lo, hi)                                                              \
                {                                                                         \
                    const int lo_ = (lo), hi_ = (hi);                                     \
                    const int b_lo = (lo_ + 3) >> 2, b_hi = hi_ >> 2;                     \
                    const int e1 = min(4 * b_lo, hi_), s2 = max(4 * b_hi, e1);            \
                    _Pragma("unroll")                                                     \
                    for (int u = 0; u < 3; ++u) {                                         \
                        if (lo_ + u < e1) m = fmax(m, arr[lo_ + u]);                      \
                        if (s2 + u < hi_) m = fmax(m, arr[s2 + u]);                       \
                    }                                                                     \
                    if (b_lo < b_hi) {                                                    \
                        const int j_ = 31 - __builtin_clz(b_hi - b_lo);                   \
                        const double *lv_ = tab + (size_t)j_ * nb;                        \
                        m = fmax(m, fmax(lv_[b_lo], lv_[b_hi - (1 << j_)]));              \
                    }                                                                     \
                }
#define SC_RHO(k)                                                                         \
        if constexpr (k < KT) {                                                           \
            const int c = k * 64 + lane;                                                  \
            if (c < C) {                                                                  \
                double m = 0.0;                                                           \
                if (re_##k > rb_##k) SC_RANGE_MAX((int)(ra_##k & 0xffffu), (int)(ra_##k >> 16))         \
                if (re_##k > rb_##k + 1) SC_RANGE_MAX((int)(rc_##k & 0xffffu), (int)(rc_##k >> 16))     \
                for (int q = rb_##k + 2; q < re_##k; ++q) {                               \
                    const int lo = p.run_lo[q], hi = p.run_hi[q];                         \
                    SC_RANGE_MAX(lo, hi)                                                  \
                }                                                                         \
                rho_##k = m;                                                              \
            }                                                                             \
        }
        SW_EACH_K(SC_RHO)
        wave_sync();

        // ---- the compute device: makespan = max over classes of (release date + time of the classes released
        // then or later) ----
        double mloc = last_arrival, ct_sum = 0.0;
        {
            // the rank of a release date is the number of arrivals up to it, one branch-free binary
            // search per channel (release dates are arrivals, so a later release date has a higher rank and equal
            // ones the same); the class times are added up by rank, a suffix sum over the ranks follows
            double *A = arr;                // [R + 1] by rank (the arrivals and the table are not read any more)
            for (int j = lane; j <= R; j += 64) A[j] = 0.0;
#define SC_RANK_DECL(k) int rank_##k = 0, pos_##k = 0;
            SW_EACH_K(SC_RANK_DECL)
            for (int c = 0; c < p.n_channels; ++c) {
                const int len = min(__builtin_amdgcn_readlane(queued, c), clen[c]);
                if (len == 0) continue;
                const double *lc = lists + coff[c];
#define SC_RANK_ZERO(k) pos_##k = 0;
                SW_EACH_K(SC_RANK_ZERO)
                for (int step = 1 << (31 - __builtin_clz(len)); step > 0; step >>= 1) {
#define SC_RANK_STEP(k)                                                                   \
                    if constexpr (k < KT) {                                               \
                        const int np = pos_##k + step;                                    \
                        const double v = lc[min(np, len) - 1];                            \
                        if (np <= len && v <= rho_##k) pos_##k = np;                      \
                    }
                    SW_EACH_K(SC_RANK_STEP)
                }
#define SC_RANK_ADD(k) rank_##k += pos_##k;
                SW_EACH_K(SC_RANK_ADD)
            }
            wave_sync();
#define SC_RANK_SUM(k) if constexpr (k < KT) { if (k * 64 + lane < C) atomicAdd(&A[rank_##k], ct_##k); ct_sum += ct_##k; }
            SW_EACH_K(SC_RANK_SUM)
            wave_sync();
            double sfx = 0.0;
            for (int base = (R / 64) * 64; base >= 0; base -= 64) {
                const int j = base + lane;
                const double x = j <= R ? A[j] : 0.0;
                const double inc = wave_incl_scan_f64_dpp(x);
                const double tot = lane63_f64(inc);
                if (j <= R) A[j] = sfx + (tot - inc + x);           // this rank and every later one
                sfx += tot;
            }
            wave_sync();
#define SC_RANK_MAX(k) if constexpr (k < KT) { if (k * 64 + lane < C) mloc = fmax(mloc, rho_##k + A[rank_##k]); }
            SW_EACH_K(SC_RANK_MAX)
        }
        const double m = wave_max_f64_dpp(mloc);
        const double sum_c = wave_sum_f64_dpp(ct_sum);
        if (lane == 0) {
            const double U = sum_c + sum_r;
            const double L = fmax(sum_c, last_arrival);
            p.makespan[b] = m;
            p.eff[b] = (U == L) ? 1.0 : (U - m) / (U - L);
            if (p.U) p.U[b] = U;
            if (p.L) p.L[b] = L;
            if (p.S) p.S[b] = (U == L || L == 0.0) ? 0.0 : (U - L) / L;
        }
    }
}

template <int KT>
static hipError_t launch_sim_chan(SimChanParams &p, const Dag &d, hipStream_t s)
{
    const int nb = (d.R + 3) / 4;
    int levels = 1;
    while ((1 << levels) <= nb) ++levels;             // floor(log2 nb) + 1 levels of the table of block maxima
    p.levels = levels;
    p.nb = nb;
    // the transfer times, later the table; at least one double beyond the padded arrivals for the sums by rank
    const size_t x_doubles = (std::max((size_t)d.R, (size_t)levels * nb) + 2) & ~(size_t)1;
    p.x_doubles = (int32_t)x_doubles;
    // after those: the class totals, then the arrivals by channel
    const size_t extra = std::max((size_t)64 * KT, ((size_t)d.R + 1) & ~(size_t)1);
    const size_t wave_bytes = ((size_t)4 * nb + x_doubles + extra) * 8;       // a multiple of 16
    int waves = 4;
    while (waves > 1 && wave_bytes * waves > 40 * 1024) waves >>= 1;
    const size_t chan_bytes = (((size_t)d.R + 128) * 4 + 15) & ~(size_t)15;
    const size_t lds = chan_bytes + wave_bytes * waves;
    if (lds > 150 * 1024) return hipErrorNotSupported;     // 160 KB of LDS per compute unit
    p.wave_bytes = (int32_t)wave_bytes;
    p.chan_bytes = (int32_t)chan_bytes;
    hipError_t e;
    if (lds > 48 * 1024) {
        e = ensure_dynamic_lds(reinterpret_cast<const void *>(simulate_channels_kernel<KT>), lds);
        if (e != hipSuccess) return e;
    }
    int per_cu = 0;
    e = cached_blocks_per_cu(&per_cu, reinterpret_cast<const void *>(simulate_channels_kernel<KT>), 64 * waves, lds);
    if (e != hipSuccess) return e;
    if (per_cu < 1) per_cu = 1;
    const int n_cu = device_cu_count(d.device);
    int grid = per_cu * n_cu;
    const int need = (p.B + waves - 1) / waves;
    if (grid > need) grid = need;
    p.n_waves = grid * waves;
    hipLaunchKernelGGL((simulate_channels_kernel<KT>), dim3(grid), dim3(64 * waves), lds, s, p);
    return hipGetLastError();
}

hipError_t launch_simulate_channels(Dag &d, const SimArgs &a, int32_t n_channels, const int32_t *chan, hipStream_t s)
{
    if (a.B == 0) return hipSuccess;
    const int K = std::max((d.C + 63) / 64, (d.R + 63) / 64);   // slots per lane: classes, and positions of the order
    const int KT = K < 1 ? 1 : K;
    if (d.R == 0 || d.R > 512 || K > 8 || n_channels > 64 || (d.C > 0 && (!d.d_col_cls || !d.d_run_ptr))) return hipErrorNotSupported;
    SimChanParams p{};
    p.B = a.B; p.R = d.R; p.C = d.C; p.N = d.N; p.n_channels = n_channels;
    p.col_cls = d.d_col_cls; p.run_ptr = d.d_run_ptr; p.run_lo = d.d_run_lo; p.run_hi = d.d_run_hi;
    p.chan = chan; p.order = a.order; p.order_stride = a.order_stride;
    p.op_time = a.op_time; p.recv_time = a.recv_time; p.f32 = a.f32 ? 1 : 0;
    p.makespan = a.makespan; p.eff = a.eff; p.U = a.U; p.L = a.L; p.S = a.S;
    switch (KT) {
    case 1: return launch_sim_chan<1>(p, d, s);
    case 2: return launch_sim_chan<2>(p, d, s);
    case 3: return launch_sim_chan<3>(p, d, s);
    case 4: return launch_sim_chan<4>(p, d, s);
    case 5: return launch_sim_chan<5>(p, d, s);
    case 6: return launch_sim_chan<6>(p, d, s);
    case 7: return launch_sim_chan<7>(p, d, s);
    default: return launch_sim_chan<8>(p, d, s);
    }
}

// Straggler effect of groups of w consecutive samples (Sec. 6): (max - min) / max of their
// makespans.  A group is spread over the lanes of one wave (w > 4) or handled by one thread.
__global__ void __launch_bounds__(256)
straggler_kernel(int32_t n_groups, int32_t w, const double *__restrict__ makespan, double *__restrict__ out)
{
    if (w <= 4) {
        const int g = blockIdx.x * blockDim.x + threadIdx.x;
        if (g >= n_groups) return;
        double mx = makespan[(size_t)g * w], mn = mx;
        for (int i = 1; i < w; ++i) {
            const double m = makespan[(size_t)g * w + i];
            mx = fmax(mx, m);
            mn = fmin(mn, m);
        }
        out[g] = mx > 0.0 ? (mx - mn) / mx : 0.0;
        return;
    }
    const int lane = threadIdx.x & 63;
    const int g = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);     // wave-uniform
    if (g >= n_groups) return;
    double mx = -TT_INF, mn = TT_INF;
    for (int i = lane; i < w; i += 64) {
        const double m = makespan[(size_t)g * w + i];
        mx = fmax(mx, m);
        mn = fmin(mn, m);
    }
    mx = wave_max_f64_dpp(mx);
    mn = wave_min_f64_dpp(mn);
    if (lane == 0) out[g] = mx > 0.0 ? (mx - mn) / mx : 0.0;
}

hipError_t launch_straggler(int32_t B, int32_t w, const double *makespan, double *out, hipStream_t s)
{
    const int32_t n_groups = B / w;
    if (n_groups == 0) return hipSuccess;
    const int per_block = w <= 4 ? 256 : 4;
    hipLaunchKernelGGL(straggler_kernel, dim3((n_groups + per_block - 1) / per_block), dim3(256), 0, s,
                       n_groups, w, makespan, out);
    return hipGetLastError();
}

// Time oracle estimator (Sec. 5): time[i] = minimum over the measured runs of runs[k][i].
// A streaming kernel: every element is read once per run; two doubles per lane and load.
__global__ void __launch_bounds__(256)
time_oracle_min_kernel(int32_t n_runs, int64_t n, bool pairs_ok, const double *__restrict__ runs,
                       double *__restrict__ time)
{
    const int64_t n2 = n >> 1;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    if (pairs_ok) {
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n2; i += stride) {
            double2 m = reinterpret_cast<const double2 *>(runs)[i];
            for (int k = 1; k < n_runs; ++k) {
                const double2 x = reinterpret_cast<const double2 *>(runs + (size_t)k * n)[i];
                m.x = fmin(m.x, x.x);
                m.y = fmin(m.y, x.y);
            }
            reinterpret_cast<double2 *>(time)[i] = m;
        }
    } else {
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
            double m = runs[i];
            for (int k = 1; k < n_runs; ++k) m = fmin(m, runs[(size_t)k * n + i]);
            time[i] = m;
        }
    }
}

hipError_t launch_time_oracle_min(int32_t n_runs, int64_t n, const double *runs, double *time, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    // pairs when every row starts on a 16-byte boundary
    const bool pairs_ok = (n & 1) == 0 && ((reinterpret_cast<uintptr_t>(runs) | reinterpret_cast<uintptr_t>(time)) & 15) == 0;
    const int64_t work = pairs_ok ? n / 2 : n;
    int64_t blocks = (work + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;          // 32 workgroups per compute unit, grid-stride beyond
    hipLaunchKernelGGL(time_oracle_min_kernel, dim3((unsigned)blocks), dim3(256), 0, s, n_runs, n, pairs_ok, runs, time);
    return hipGetLastError();
}

hipError_t launch_simulate(Dag &d, const SimArgs &a, hipStream_t s)
{
    if (a.B == 0) return hipSuccess;
    SimKernelParams p{};
    p.B = a.B; p.R = d.R; p.W = d.W; p.C = d.C; p.N = d.N;
    p.cls_dep = d.d_cls_dep; p.cls_ptr = d.d_cls_ptr; p.cls_cols = d.d_cls_cols;
    p.order = a.order; p.order_stride = a.order_stride; p.kappa = nullptr;
    p.op_time = a.op_time; p.recv_time = a.recv_time; p.f32 = a.f32 ? 1 : 0;
    p.makespan = a.makespan; p.eff = a.eff; p.U = a.U; p.L = a.L; p.S = a.S;
    if (a.order_stride == 0 && d.R > 0 && d.C > 0) {
        hipError_t e = ensure_workspace(&d, ((size_t)d.R + d.C) * sizeof(int32_t));
        if (e != hipSuccess) return e;
        int32_t *pos = static_cast<int32_t *>(d.d_work);
        int32_t *kappa = pos + d.R;
        hipLaunchKernelGGL(position_kernel, dim3(1), dim3(256), 0, s, d.R, a.order, pos);
        hipLaunchKernelGGL(kappa_kernel, dim3((d.C + 255) / 256), dim3(256), 0, s, d.W, d.C, d.d_cls_dep, pos, kappa);
        p.kappa = kappa;
    }
    {
        const hipError_t e = try_simulate_wave(d, a, p.kappa, s);
        if (e != hipErrorNotSupported) return e;
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

// ---- orders given by the caller ----
// One wave per order: every entry in 0 .. R-1 and none twice (a bit per recv in LDS), else the flag is raised.
// The simulations and the search skip entries out of range themselves; what they return for such a row is unspecified.
__global__ void __launch_bounds__(256)
check_orders_kernel(int32_t R, int32_t rows, const int32_t *__restrict__ order, int32_t stride, int32_t *flag)
{
    extern __shared__ uint32_t seen_all[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, words = (R + 31) >> 5;
    uint32_t *seen = seen_all + (size_t)wave * words;
    bool bad = false;
    for (int b = blockIdx.x * 4 + wave; b < rows; b += gridDim.x * 4) {
        const int32_t *ord = order + (size_t)b * stride;
        for (int i = lane; i < words; i += 64) seen[i] = 0;
        wave_sync();
        for (int k = lane; k < R; k += 64) {
            const int r = ord[k];
            if ((unsigned)r >= (unsigned)R) { bad = true; continue; }
            const uint32_t bit = 1u << (r & 31);
            if (atomicOr(&seen[r >> 5], bit) & bit) bad = true;
        }
        wave_sync();
    }
    if (bad) atomicOr(flag, 1);
}

hipError_t launch_check_orders(Dag &d, int32_t B, const int32_t *order, int32_t order_stride, hipStream_t s)
{
    if (d.R <= 0 || B <= 0 || !order) return hipSuccess;
    if (!d.d_bad_order) return hipErrorInvalidValue;
    const int rows = order_stride == 0 ? 1 : B;
    const size_t lds = (size_t)4 * ((d.R + 31) / 32) * 4;
    if (lds > 48 * 1024) return hipErrorInvalidValue;
    const int blocks = std::min((rows + 3) / 4, 8 * device_cu_count(d.device));
    hipLaunchKernelGGL(check_orders_kernel, dim3(blocks), dim3(256), lds, s, d.R, rows, order, order_stride, d.d_bad_order);
    return hipGetLastError();
}

}  // namespace tictac
