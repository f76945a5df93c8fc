// TAC (Sec. 4.3, Algorithm 3) with the iteration under its order (Sec. 3.2), one wavefront
// per timing sample, for graphs whose classes fit the register file: lane l owns the
// classes l, l + 64, ... (KT per lane) and keeps their dependency rows, outstanding
// counts, M and class times in VGPRs for the whole selection loop.  The bitsets of
// outstanding recvs and of Q = {outstanding recvs with P > 0} are wave-uniform values
// (scalar registers); LDS holds the per-recv arrays (Time, P) and the order built so far.
// Per round nothing is read from global memory.
//
// The algorithm is the one described at the top of k3_tac.hip (incremental Algorithm 1,
// selection by the scan over Q or by the minimum of M over classes with two or more
// outstanding recvs).  Differences in how it is carried out:
//   * the op_time row is staged into LDS by coalesced loads and the class totals are
//     gathered from there;
//   * M of a class is initialised from prefix sums T of the transfer times:
//     sum over the runs [lo, hi) of consecutive recv indices of its row of T[hi] - T[lo];
//   * the outstanding count of a class and the sum of the indices of its outstanding
//     recvs share one register; when the count reaches 1 the index sum *is* the last
//     outstanding recv, to whose P the class time is added (LDS atomic issued by the
//     owning lane; lanes of one instruction and successive instructions are served in a
//     fixed order, so the result is reproducible).  Q gets that recv's bit when the class
//     time is positive (P only grows while the recv is outstanding);
//   * a class whose count reaches 0 after k transfers adds its time to A[k]; the makespan
//     is formed after the loop as max_k (F_k + S_k), F_k the end of the k-th transfer,
//     S_k = A[k] + A[k+1] + ...  (the closed form of the work-conserving device described
//     in k4_simulate.hip);
//   * blocks of 64 classes whose counts are all 0 are skipped (classes are numbered by
//     their first op, so on layered models they finish roughly in order);
//   * a sample with a transfer time of zero is not handled here: it is flagged for the
//     general kernel, which takes the literal path for it.
#include <type_traits>

#include "device_utils.h"
#include "internal.h"

namespace tictac {

struct TacRegParams {
    int32_t B, R, W, C, N;
    const uint64_t *cls_dep;    // [C][W]
    const int32_t *cls_cnt0;    // [C]
    const int32_t *cls_isum;    // [C]   sum of the recv indices of the row
    const int32_t *cls_ptr;     // [C+1]
    const int32_t *cls_cols;    // [N]
    const int32_t *run_ptr;     // [C+1]
    const int32_t *run_lo, *run_hi;
    const double *op_time, *recv_time;
    int32_t *order, *rank;
    int32_t simulate;
    double *makespan, *eff, *U, *L, *S;
    int32_t *flags;             // [B] 1 = left to the general kernel
    int32_t xlen;               // doubles in the staging / simulation region of LDS
};

// calls f(std::integral_constant<int, i>) for the i in [I, IN) equal to the (wave-uniform) index
template <int I, int IN, class F>
__device__ __forceinline__ void dispatch_index(int idx, F &&f)
{
    if constexpr (I < IN) {
        if (idx == I) f(std::integral_constant<int, I>{});
        else dispatch_index<I + 1, IN>(idx, f);
    }
}

template <int WT>
__device__ __forceinline__ int first_alive(const uint32_t (&row)[2 * WT], const uint64_t (&alive)[WT])
{
    int r = INT32_MAX;
#pragma unroll
    for (int j = WT - 1; j >= 0; --j) {
        const uint64_t x = (((uint64_t)row[2 * j + 1] << 32) | row[2 * j]) & alive[j];
        if (x) r = j * 64 + __builtin_ctzll(x);
    }
    return r;
}

// does the row hold recv q?  (AND with a one-hot mask per word: no element of the register
// array is selected by a run-time index)
template <int WT>
__device__ __forceinline__ bool row_has(const uint32_t (&row)[2 * WT], int q)
{
    uint32_t acc = 0;
#pragma unroll
    for (int j = 0; j < 2 * WT; ++j) {
        const uint32_t mask = ((q >> 5) == j) ? (1u << (q & 31)) : 0u;
        acc |= row[j] & mask;
    }
    return acc != 0;
}

template <int KT, int WT, bool STAGE>
__global__ void __launch_bounds__(64)
tac_reg_kernel(const TacRegParams p)
{
    extern __shared__ double smem[];
    const int R = p.R, W = p.W, C = p.C, N = p.N;
    const int lane = threadIdx.x;

    double *t = smem;                       // [R]    Time(recv)
    double *P = t + R;                      // [R+1]  P; before the loop: prefix sums T
    double *X = P + (R + 1);                // [xlen] op_time row, later A [R+1] and F [R+1]
    int32_t *ordl = reinterpret_cast<int32_t *>(X + p.xlen);                     // [R]
    double *A = X, *Fs = X + (R + 1);

    // ---- per-lane tables, the same for every sample ----
    // packed0 = (|row| << 20) + sum of the recv indices of the row.  The running value
    // `packed` loses (1 << 20) + r when recv r of the row is removed, so its upper bits are
    // the outstanding count and, once that count is 1, its lower 20 bits are the index of
    // the last outstanding recv of the class.
    constexpr int CNT1 = 1 << 20;
    uint32_t row[KT][2 * WT];
    int packed0[KT];
#pragma unroll
    for (int k = 0; k < KT; ++k) {
        const int c = k * 64 + lane;
#pragma unroll
        for (int j = 0; j < WT; ++j) {
            const uint64_t x = (c < C && j < W) ? p.cls_dep[(size_t)c * W + j] : 0ull;
            row[k][2 * j] = (uint32_t)x;
            row[k][2 * j + 1] = (uint32_t)(x >> 32);
        }
        packed0[k] = c < C ? p.cls_cnt0[c] * CNT1 + p.cls_isum[c] : 0;
    }

    for (int b = blockIdx.x; b < p.B; b += gridDim.x) {
        const double *rt = p.recv_time + (size_t)b * R;
        const double *ot = p.op_time + (size_t)b * N;
        __syncthreads();                    // LDS of the previous sample is no longer read

        // ---- a. transfer times, their prefix sums, and the op_time row ----
        bool zero_seen = false;
        double carry = 0.0;
        for (int base = 0; base < R; base += 64) {
            const int r = base + lane;
            const double x = r < R ? rt[r] : 0.0;
            if (r < R) { t[r] = x; zero_seen |= !(x > 0.0); }
            const double inc = wave_incl_scan_f64(x);
            if (r < R) P[r + 1] = carry + inc;
            carry += __shfl(inc, 63);
        }
        if (lane == 0) P[0] = 0.0;
        const bool skip = __ballot(zero_seen) != 0ull;
        if (lane == 0) p.flags[b] = skip ? 1 : 0;
        if (skip) continue;
        if (STAGE)
            for (int j = lane; j < N; j += 64) X[j] = ot[j];
        __syncthreads();

        // ---- b. class totals and initial M ----
        double ct[KT], M[KT];
        int packed[KT];
        double ct_sum = 0.0;
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            const int c = k * 64 + lane;
            double s = 0.0, Mk = 0.0;
            if (c < C) {
                const int mend = p.cls_ptr[c + 1], rend = p.run_ptr[c + 1];
                for (int m = p.cls_ptr[c]; m < mend; ++m) s += STAGE ? X[p.cls_cols[m]] : ot[p.cls_cols[m]];
                for (int q = p.run_ptr[c]; q < rend; ++q) Mk += P[p.run_hi[q]] - P[p.run_lo[q]];
            }
            ct[k] = s; M[k] = Mk; packed[k] = packed0[k];
            ct_sum += s;
        }
        __syncthreads();                    // T and the staged row are consumed

        // ---- c. P, A; the wave-uniform bitsets of outstanding recvs and of Q ----
        for (int r = lane; r < R; r += 64) P[r] = 0.0;
        if (p.simulate)
            for (int j = lane; j <= R; j += 64) A[j] = 0.0;
        if (p.simulate && lane == 0) Fs[0] = 0.0;
        uint64_t alive[WT], Q[WT];
#pragma unroll
        for (int j = 0; j < WT; ++j) {
            const int nbits = R - j * 64;
            alive[j] = nbits >= 64 ? ~0ull : (nbits > 0 ? ((1ull << nbits) - 1ull) : 0ull);
            Q[j] = 0ull;
        }
        __syncthreads();
        uint32_t live = 0;                  // bit k: some class of block k still has outstanding recvs
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            const bool one = (unsigned)(packed[k] - CNT1) < (unsigned)CNT1;      // count == 1
            if (one) atomicAdd(&P[packed[k] & (CNT1 - 1)], ct[k]);
            uint64_t qm = __ballot(one && ct[k] > 0.0);
            while (qm) {
                const int l = __builtin_ctzll(qm);
                qm &= qm - 1;
                const int sole = __builtin_amdgcn_readlane(packed[k], l) & (CNT1 - 1);
#pragma unroll
                for (int j = 0; j < WT; ++j)
                    if (j == (sole >> 6)) Q[j] |= 1ull << (sole & 63);
            }
            if (p.simulate && packed[k] < CNT1 && k * 64 + lane < C) atomicAdd(&A[0], ct[k]);
            if (__ballot(packed[k] >= CNT1)) live |= 1u << k;
        }

        // ---- d. selection loop ----
        double F = 0.0;
        for (int step = 0; step < R; ++step) {
            int nq = 0;
#pragma unroll
            for (int j = 0; j < WT; ++j) nq += __builtin_popcountll(Q[j]);
            int best = INT32_MAX;
            if (nq == 1) {
#pragma unroll
                for (int j = WT - 1; j >= 0; --j)
                    if (Q[j]) best = j * 64 + __builtin_ctzll(Q[j]);
            } else if (nq == 0) {
                // every outstanding recv has P = 0: lowest index among those of minimal M+
                double lmin = TT_INF;
#pragma unroll
                for (int k = 0; k < KT; ++k)
                    if (packed[k] >= 2 * CNT1) lmin = fmin(lmin, M[k]);
                const double g = wave_min_f64(lmin);
                int cand = INT32_MAX;
                if (g != TT_INF) {
#pragma unroll
                    for (int k = 0; k < KT; ++k)
                        if (packed[k] >= 2 * CNT1 && M[k] == g) cand = min(cand, first_alive<WT>(row[k], alive));
                }
                best = wave_min_i32(cand);            // INT32_MAX when no M+ exists: fixed up below
            } else {
                // ascending scan over Q with the comparator
                double mp_best = -1.0;
                best = -1;
                __syncthreads();                      // P of this round is complete
#pragma unroll
                for (int j = 0; j < WT; ++j) {
                    uint64_t x = Q[j];
                    while (x) {
                        const int a = j * 64 + __builtin_ctzll(x);
                        x &= x - 1;
                        if (best < 0) { best = a; continue; }
                        const double xa = fmin(P[best], t[a]);
                        const double ya = fmin(P[a], t[best]);
                        bool prec;
                        double mp_a = -1.0;
                        if (xa != ya) {
                            prec = xa < ya;
                        } else {
                            double v = TT_INF, u = TT_INF;
#pragma unroll
                            for (int k = 0; k < KT; ++k) {
                                if (packed[k] >= 2 * CNT1 && row_has<WT>(row[k], a)) v = fmin(v, M[k]);
                                if (packed[k] >= 2 * CNT1 && row_has<WT>(row[k], best)) u = fmin(u, M[k]);
                            }
                            mp_a = wave_min_f64(v);
                            if (mp_best < 0.0) mp_best = wave_min_f64(u);
                            prec = mp_a < mp_best;
                        }
                        if (prec) { best = a; mp_best = mp_a; }
                    }
                }
            }
            best = __builtin_amdgcn_readfirstlane(best);
            if ((unsigned)best >= (unsigned)R) {      // no M+ exists: the lowest outstanding recv
#pragma unroll
                for (int j = WT - 1; j >= 0; --j)
                    if (alive[j]) best = j * 64 + __builtin_ctzll(alive[j]);
            }
            const double tb = t[best];
            F += tb;
            const int bw = best >> 6;
            const uint64_t bbit = 1ull << (best & 63);
#pragma unroll
            for (int j = 0; j < WT; ++j)
                if (j == bw) { alive[j] &= ~bbit; Q[j] &= ~bbit; }
            if (lane == 0) {
                ordl[step] = best;
                if (p.simulate) Fs[step + 1] = F;
            }

            // ---- incremental property update ----
            const int sh = best & 31;
            const int delta = CNT1 + best;
            const long long tb_bits = __double_as_longlong(tb);
            dispatch_index<0, 2 * WT>(best >> 5, [&](auto hc) {      // wave-uniform branch on the word half
                constexpr int hh = decltype(hc)::value;
#pragma unroll
                for (int k = 0; k < KT; ++k) {
                    if (!(live & (1u << k))) continue;               // wave-uniform
                    const int mask = __builtin_amdgcn_sbfe(row[k][hh], sh, 1);     // 0 or -1
                    packed[k] += __mul24(mask, delta);
                    M[k] -= __longlong_as_double(tb_bits & (long long)mask);
                    const bool ev = mask != 0 && (unsigned)packed[k] < (unsigned)(2 * CNT1);
                    if (__ballot(ev)) {
                        const bool hit0 = ev && packed[k] < CNT1;
                        const bool hit1 = ev && !hit0;
                        if (hit1) atomicAdd(&P[packed[k] & (CNT1 - 1)], ct[k]);
                        uint64_t qm = __ballot(hit1 && ct[k] > 0.0);
                        while (qm) {
                            const int l = __builtin_ctzll(qm);
                            qm &= qm - 1;
                            const int sole = __builtin_amdgcn_readlane(packed[k], l) & (CNT1 - 1);
#pragma unroll
                            for (int j = 0; j < WT; ++j)
                                if (j == (sole >> 6)) Q[j] |= 1ull << (sole & 63);
                        }
                        if (__ballot(hit0)) {
                            if (p.simulate && hit0) atomicAdd(&A[step + 1], ct[k]);
                            if (__ballot(packed[k] >= CNT1) == 0ull) live &= ~(1u << k);
                        }
                    }
                }
            });
        }
        __syncthreads();

        // ---- e. outputs ----
        for (int s = lane; s < R; s += 64) {
            const int r = ordl[s];
            p.order[(size_t)b * R + s] = r;
            if (p.rank) p.rank[(size_t)b * R + r] = s;
        }
        if (p.simulate) {
            // makespan = max over k of F_k + (time of the classes released after k or more transfers)
            double sfx = 0.0, mloc = 0.0;
            for (int base = (R / 64) * 64; base >= 0; base -= 64) {
                const int j = base + 63 - lane;              // descending index along the lanes
                const double x = j <= R ? A[j] : 0.0;
                const double inc = wave_incl_scan_f64(x);    // sum of A over indices >= j of this chunk
                if (j <= R) mloc = fmax(mloc, Fs[j] + (sfx + inc));
                sfx += __shfl(inc, 63);
            }
            const double m = wave_max_f64(mloc);
            const double sum_c = wave_sum_f64(ct_sum);
            if (lane == 0) {
                const double U = sum_c + F;
                const double L = fmax(sum_c, F);
                if (p.makespan) p.makespan[b] = m;
                if (p.eff) p.eff[b] = (U == L) ? 1.0 : (U - m) / (U - L);
                if (p.U) p.U[b] = U;
                if (p.L) p.L[b] = L;
                if (p.S) p.S[b] = (U == L || L == 0.0) ? 0.0 : (U - L) / L;
            }
        }
    }
}

template <int KT, int WT>
static hipError_t launch_reg_t(const TacRegParams &p, bool stage, int grid, size_t lds, hipStream_t s)
{
    if (stage)
        hipLaunchKernelGGL((tac_reg_kernel<KT, WT, true>), dim3(grid), dim3(64), lds, s, p);
    else
        hipLaunchKernelGGL((tac_reg_kernel<KT, WT, false>), dim3(grid), dim3(64), lds, s, p);
    return hipGetLastError();
}

template <int KT>
static hipError_t launch_reg_k(const TacRegParams &p, int W, bool stage, int grid, size_t lds, hipStream_t s)
{
    if (W <= 1) return launch_reg_t<KT, 1>(p, stage, grid, lds, s);
    if (W <= 2) return launch_reg_t<KT, 2>(p, stage, grid, lds, s);
    if (W <= 3) return launch_reg_t<KT, 3>(p, stage, grid, lds, s);
    if (W <= 4) return launch_reg_t<KT, 4>(p, stage, grid, lds, s);
    return launch_reg_t<KT, 6>(p, stage, grid, lds, s);
}

hipError_t launch_tac_reg(Dag &d, const TacArgs &a, int32_t *flags, hipStream_t s)
{
    if (d.R == 0 || d.W > 6 || d.C > 8 * 64 || a.sel_P || a.sel_Mplus) return hipErrorNotSupported;
    TacRegParams p{};
    p.B = a.B; p.R = d.R; p.W = d.W; p.C = d.C; p.N = d.N;
    p.cls_dep = d.d_cls_dep; p.cls_cnt0 = d.d_cls_cnt0; p.cls_isum = d.d_cls_isum;
    p.cls_ptr = d.d_cls_ptr; p.cls_cols = d.d_cls_cols;
    p.run_ptr = d.d_run_ptr; p.run_lo = d.d_run_lo; p.run_hi = d.d_run_hi;
    p.op_time = a.op_time; p.recv_time = a.recv_time;
    p.order = a.order; p.rank = a.rank;
    p.simulate = a.simulate ? 1 : 0;
    p.makespan = a.makespan; p.eff = a.eff; p.U = a.U; p.L = a.L; p.S = a.S;
    p.flags = flags;
    const bool stage = (size_t)d.N * 8 <= 16 * 1024;
    const int sim_len = a.simulate ? 2 * (d.R + 1) : 0;
    p.xlen = std::max(stage ? d.N : 0, sim_len);
    const size_t lds = ((size_t)d.R + (d.R + 1) + p.xlen) * 8 + (size_t)d.R * 4;
    if (lds > 60 * 1024) return hipErrorNotSupported;
    const int grid = a.B < 256 * 16 ? a.B : 256 * 16;
    const int K = (d.C + 63) / 64;
    if (K <= 1) return launch_reg_k<1>(p, d.W, stage, grid, lds, s);
    if (K <= 2) return launch_reg_k<2>(p, d.W, stage, grid, lds, s);
    if (K <= 4) return launch_reg_k<4>(p, d.W, stage, grid, lds, s);
    return launch_reg_k<8>(p, d.W, stage, grid, lds, s);
}

}  // namespace tictac
