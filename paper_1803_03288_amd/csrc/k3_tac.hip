// TAC (Sec. 4.3, Algorithm 3) for a batch of timing samples, optionally followed by the
// iteration under the order it produces (Sec. 3.2).  One workgroup per sample.
//
// The selection loop of Algorithm 3 recomputes the properties of Algorithm 1 from
// scratch in every round.  Here they are maintained incrementally, on classes of compute
// ops with identical dependency sets (only the total time of a class matters to
// Algorithm 1):
//   cnt[c] = |dep[c] ∩ R|,  M[c] = sum of Time(r) over dep[c] ∩ R   (R = outstanding recvs)
//   P[r]   = sum of the class times with cnt = 1 whose remaining recv is r
//   M+[r]  = min of M[c] over the classes with cnt >= 2 that hold r
// Removing recv r* touches the classes that hold r*: cnt -= 1, M -= Time(r*); a class
// reaching cnt = 1 adds its time to P of its last recv; a class reaching cnt = 0 is
// released to the compute device at that moment (used by the fused simulation).
//
// Minimum under the comparator.  A precedes B when x = min{P_B, M_A} < y = min{P_A, M_B},
// and when x == y, when M+_A < M+_B; the minimum is taken by an ascending-index scan that
// replaces the current best only by a recv that strictly precedes it.  When every
// transfer time of the sample is positive:
//   * a recv with P > 0 precedes every recv with P = 0 and is never replaced by one, so if
//     Q = {r outstanding : P[r] > 0} is not empty the scan over all outstanding recvs gives
//     the same result as the scan over Q alone (done literally, in ascending index);
//   * if Q is empty every pair ties on x == y == 0 and the scan returns the lowest index
//     among the recvs of minimal M+.  min M+ = g = min of M[c] over classes with cnt >= 2,
//     and the recvs attaining it are the outstanding members of the classes with
//     cnt >= 2 and M[c] == g.
// A sample with a transfer time of zero takes the literal path: M+ of every outstanding
// recv is formed and the ascending scan runs over all of them.
#include "device_utils.h"
#include "internal.h"

namespace tictac {

struct TacKernelParams {
    int32_t B, R, W, C, Cpad, N;
    const uint64_t *cls_dep;    // [C][W]
    const uint64_t *cls_depT;   // [W][Cpad]
    const int32_t *cls_cnt0;    // [C]
    const int32_t *cls_ptr;     // [C+1]
    const int32_t *cls_cols;    // [N]
    const void *op_time, *recv_time;    // float64, or float32 when f32 is set
    int32_t f32;
    int32_t *order, *rank;
    double *sel_P, *sel_Mplus;
    int32_t simulate;
    double *makespan, *eff, *U, *L, *S;
    // per-workgroup state in global memory (GSTATE kernels): ct, M [C] f64, Mp [R] f64, cnt [C] i32
    char *gstate;
    size_t gstate_stride;
    // when not NULL, only the samples with only_flagged[b] != 0 are processed
    const int32_t *only_flagged;
};

// M+ values of the literal path are produced by atomics of other threads; when they live
// in global memory they are read past the per-CU cache.
template <bool GSTATE>
__device__ __forceinline__ double load_mp(const double *q)
{
    if (GSTATE) return __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *q;
}

__device__ __forceinline__ int row_lowest_alive(const uint64_t *__restrict__ row, const uint64_t *alive, int W)
{
    for (int w = 0; w < W; ++w) {
        const uint64_t x = row[w] & alive[w];
        if (x) return w * 64 + __builtin_ctzll(x);
    }
    return INT32_MAX;
}

template <int BS, bool GSTATE>
__global__ void __launch_bounds__(BS)
tac_kernel(const TacKernelParams p)
{
    extern __shared__ double smem[];
    const int R = p.R, W = p.W, C = p.C, N = p.N;
    const int tid = threadIdx.x;

    // ---- LDS carve-up ----
    double *t = smem;                   // [R]   Time(recv)
    double *P = t + R;                  // [R]
    double *A = P + R;                  // [R+1] class time released after k transfers
    double *red = A + (R + 1);          // [16]  reduction scratch
    uint64_t *alive = reinterpret_cast<uint64_t *>(red + 16);   // [W]
    uint64_t *Q = alive + W;                                     // [W]
    double *tail = reinterpret_cast<double *>(Q + W);
    double *ct, *M, *Mp;
    int32_t *cnt;
    if (GSTATE) {
        char *g = p.gstate + (size_t)blockIdx.x * p.gstate_stride;
        ct = reinterpret_cast<double *>(g);
        M = ct + C;
        Mp = M + C;
        cnt = reinterpret_cast<int32_t *>(Mp + R);
    } else {
        ct = tail;
        M = ct + C;
        Mp = M + C;                     // [R] M+ of every recv (literal path only)
        cnt = reinterpret_cast<int32_t *>(Mp + R);
    }

    if (p.only_flagged) {
        // as a rule no sample of the workgroup is flagged: its threads look at one flag each and leave
        int any = 0;
        for (long long b = blockIdx.x + (long long)tid * gridDim.x; b < p.B; b += (long long)BS * gridDim.x)
            any |= p.only_flagged[b];
        if (!__syncthreads_or(any)) return;
    }
    for (int b = blockIdx.x; b < p.B; b += gridDim.x) {
        if (p.only_flagged && p.only_flagged[b] == 0) continue;   // uniform over the workgroup
        const TimeRow rt = time_row(p.recv_time, (size_t)b * R, p.f32 != 0);
        const TimeRow ot = time_row(p.op_time, (size_t)b * N, p.f32 != 0);
        __syncthreads();   // previous sample's LDS fully consumed

        // ---- per-sample init ----
        int zero_seen = 0;
        for (int r = tid; r < R; r += BS) {
            const double x = rt[r];
            t[r] = x;
            P[r] = 0.0;
            zero_seen |= !(x > 0.0);
        }
        for (int k = tid; k <= R; k += BS) A[k] = 0.0;
        for (int w = tid; w < W; w += BS) {
            const int nbits = R - w * 64;
            alive[w] = nbits >= 64 ? ~0ull : ((1ull << nbits) - 1ull);
            Q[w] = 0ull;
        }
        __syncthreads();
        const bool literal = __syncthreads_or(zero_seen) != 0;

        double lmin = TT_INF;          // min M over this thread's classes with cnt >= 2
        double ct_sum = 0.0;
        for (int c0 = 0; c0 < C; c0 += BS) {
            const int c = c0 + tid;
            const bool valid = c < C;
            double s = 0.0;
            int n = 0, sole = 0;
            if (valid) {
                for (int m = p.cls_ptr[c]; m < p.cls_ptr[c + 1]; ++m) s += ot[p.cls_cols[m]];
                double Mc = 0.0;
                const uint64_t *row = p.cls_dep + (size_t)c * W;
                for (int w = 0; w < W; ++w) {
                    uint64_t x = row[w];
                    while (x) {
                        Mc += t[w * 64 + __builtin_ctzll(x)];
                        x &= x - 1;
                    }
                }
                n = p.cls_cnt0[c];
                ct[c] = s; M[c] = Mc; cnt[c] = n;
                ct_sum += s;
                if (n >= 2) lmin = fmin(lmin, Mc);
                if (n == 1) sole = row_lowest_alive(row, alive, W);
            }
            lds_scatter_add<BS>(P, sole, s, valid && n == 1 && sole < R);
            lds_scatter_add<BS>(A, 0, s, valid && n == 0);
        }
        __syncthreads();
        for (int r = tid; r < R; r += BS)
            if (P[r] > 0.0) atomicOr((unsigned long long *)&Q[r >> 6], 1ull << (r & 63));
        __syncthreads();

        double F = 0.0;                 // finish time of the transfers selected so far
        double busy = A[0];             // the compute device is busy until here
        for (int step = 0; step < R; ++step) {
            // ================= selection =================
            int best = -1;
            double selP = 0.0, selM = TT_INF;
            if (!literal) {
                bool q_any = false;
                for (int w = 0; w < W && !q_any; ++w) q_any = Q[w] != 0ull;
                if (q_any) {
                    double mp_best = -1.0;                 // M+ of best, < 0 = not formed yet
                    for (int w = 0; w < W; ++w) {
                        uint64_t x = Q[w];
                        while (x) {
                            const int q = w * 64 + __builtin_ctzll(x);
                            x &= x - 1;
                            if (best < 0) { best = q; continue; }
                            const double xa = fmin(P[best], t[q]);     // min{P_B, M_A}, A = q, B = best
                            const double ya = fmin(P[q], t[best]);     // min{P_A, M_B}
                            bool prec;
                            double mp_q = -1.0;
                            if (xa != ya) {
                                prec = xa < ya;
                            } else {
                                // tie: M+ of both (block reductions, uniform control flow)
                                double v = TT_INF;
                                for (int c = tid; c < C; c += BS)
                                    if (cnt[c] >= 2 && ((p.cls_depT[(size_t)(q >> 6) * p.Cpad + c] >> (q & 63)) & 1ull))
                                        v = fmin(v, M[c]);
                                mp_q = block_min_f64<BS>(v, red);
                                if (mp_best < 0.0) {
                                    double u = TT_INF;
                                    for (int c = tid; c < C; c += BS)
                                        if (cnt[c] >= 2 && ((p.cls_depT[(size_t)(best >> 6) * p.Cpad + c] >> (best & 63)) & 1ull))
                                            u = fmin(u, M[c]);
                                    mp_best = block_min_f64<BS>(u, red);
                                }
                                prec = mp_q < mp_best;
                            }
                            if (prec) { best = q; mp_best = mp_q; }
                        }
                    }
                    selP = P[best];
                    if (p.sel_Mplus) {
                        if (mp_best < 0.0) {
                            double u = TT_INF;
                            for (int c = tid; c < C; c += BS)
                                if (cnt[c] >= 2 && ((p.cls_depT[(size_t)(best >> 6) * p.Cpad + c] >> (best & 63)) & 1ull))
                                    u = fmin(u, M[c]);
                            mp_best = block_min_f64<BS>(u, red);
                        }
                        selM = mp_best;
                    }
                } else {
                    const double g = block_min_f64<BS>(lmin, red);
                    int cand = INT32_MAX;
                    if (g == TT_INF) {
                        if (tid == 0) cand = row_lowest_alive(alive, alive, W);
                    } else {
                        for (int c = tid; c < C; c += BS)
                            if (cnt[c] >= 2 && M[c] == g)
                                cand = min(cand, row_lowest_alive(p.cls_dep + (size_t)c * W, alive, W));
                    }
                    best = block_min_i32<BS>(cand, red);
                    selM = g;
                }
            } else {
                // ---- literal path: M+ of every outstanding recv, then the ascending scan ----
                for (int r = tid; r < R; r += BS) Mp[r] = TT_INF;
                __syncthreads();
                for (int c = tid; c < C; c += BS) {
                    if (cnt[c] < 2) continue;
                    const uint64_t *row = p.cls_dep + (size_t)c * W;
                    // M of the class as Algorithm 1 forms it: the sum over its outstanding recvs in
                    // ascending index.  (The running M[c] is kept by subtraction; with transfer times of
                    // zero outstanding, its rounding residue can be negative or positive where the
                    // fresh sum is exactly 0, which would change both the minimum and exact ties.)
                    double Mc = 0.0;
                    for (int w = 0; w < W; ++w) {
                        uint64_t x = row[w] & alive[w];
                        while (x) {
                            Mc += t[w * 64 + __builtin_ctzll(x)];
                            x &= x - 1;
                        }
                    }
                    const unsigned long long mbits = (unsigned long long)__double_as_longlong(Mc);
                    for (int w = 0; w < W; ++w) {
                        uint64_t x = row[w] & alive[w];
                        while (x) {
                            // times are >= 0, so the bit patterns of the doubles order like the values
                            atomicMin((unsigned long long *)&Mp[w * 64 + __builtin_ctzll(x)], mbits);
                            x &= x - 1;
                        }
                    }
                }
                __syncthreads();
                for (int w = 0; w < W; ++w) {
                    uint64_t x = alive[w];
                    while (x) {
                        const int j = w * 64 + __builtin_ctzll(x);
                        x &= x - 1;
                        if (best < 0) { best = j; continue; }
                        const double xa = fmin(P[best], t[j]);
                        const double ya = fmin(P[j], t[best]);
                        const bool prec = (xa != ya) ? (xa < ya) : (load_mp<GSTATE>(&Mp[j]) < load_mp<GSTATE>(&Mp[best]));
                        if (prec) best = j;
                    }
                }
                selP = P[best];
                selM = load_mp<GSTATE>(&Mp[best]);
            }

            // ================= record and remove =================
            // (never taken when the bookkeeping above is consistent; keeps every index in range)
            if ((unsigned)best >= (unsigned)R) best = row_lowest_alive(alive, alive, W);
            const double tb = t[best];
            if (tid == 0) {
                p.order[(size_t)b * R + step] = best;
                if (p.rank) p.rank[(size_t)b * R + best] = step;
                if (p.sel_P) p.sel_P[(size_t)b * R + best] = selP;
                if (p.sel_Mplus) p.sel_Mplus[(size_t)b * R + best] = selM;
            }
            F += tb;
            __syncthreads();           // every thread has finished reading alive / Q / P of this round
            if (tid == 0) {
                alive[best >> 6] &= ~(1ull << (best & 63));
                Q[best >> 6] &= ~(1ull << (best & 63));
            }
            __syncthreads();

            // ================= incremental property update =================
            lmin = TT_INF;
            const uint64_t *col = p.cls_depT + (size_t)(best >> 6) * p.Cpad;
            const int bit = best & 63;
            for (int c0 = 0; c0 < C; c0 += BS) {
                const int c = c0 + tid;
                const bool valid = c < C;
                bool hit1 = false, hit0 = false;
                int sole = 0;
                double s = 0.0;
                if (valid) {
                    int n = cnt[c];
                    double Mc = M[c];
                    if ((col[c] >> bit) & 1ull) {
                        n -= 1;
                        Mc -= tb;
                        cnt[c] = n;
                        M[c] = Mc;
                        if (n == 1) {
                            sole = row_lowest_alive(p.cls_dep + (size_t)c * W, alive, W);
                            hit1 = sole < R;
                            s = ct[c];
                        } else if (n == 0) {
                            hit0 = true;
                            s = ct[c];
                        }
                    }
                    if (n >= 2) lmin = fmin(lmin, Mc);
                }
                // P of the last outstanding recv of the class, and its membership in Q
                if (BS == 64) {
                    unsigned long long m = __ballot(hit1);
                    while (m) {
                        const int l = __builtin_ctzll(m);
                        m &= m - 1;
                        const int i = __shfl(sole, l);
                        const double x = __shfl(s, l);
                        if (tid == 0) {
                            const double np = P[i] + x;
                            P[i] = np;
                            if (np > 0.0) Q[i >> 6] |= 1ull << (i & 63);
                        }
                    }
                } else if (hit1) {
                    const double old = atomicAdd(&P[sole], s);
                    if (old + s > 0.0) atomicOr((unsigned long long *)&Q[sole >> 6], 1ull << (sole & 63));
                }
                if (p.simulate) lds_scatter_add<BS>(A, step + 1, s, hit0);
            }
            __syncthreads();
            if (p.simulate) busy = fmax(busy, F) + A[step + 1];   // released classes run after the transfer
        }

        // ================= iteration metrics (Sec. 3.2) =================
        if (p.simulate) {
            const double sum_c = block_sum_f64<BS>(ct_sum, red);
            if (tid == 0) {
                const double m = fmax(busy, F);
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

static size_t tac_lds_bytes(const Dag &d, bool gstate)
{
    if (!gstate) return tac_lds_state_bytes(d.R, d.W, d.C);
    return ((size_t)d.R * 2 + (d.R + 1) + 16 + (size_t)d.W * 2) * 8;
}

static size_t tac_gstate_bytes(const Dag &d)
{
    size_t b = (size_t)d.C * 16 + (size_t)d.R * 8 + (size_t)d.C * 4;
    return (b + 255) / 256 * 256;
}

template <int BS, bool GSTATE>
static hipError_t launch_tac_t(Dag &d, TacKernelParams &p, int grid, size_t lds, hipStream_t s)
{
    auto kern = tac_kernel<BS, GSTATE>;
    if (lds > 48 * 1024) {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(BS), lds, s, p);
    return hipGetLastError();
}

hipError_t launch_tac(Dag &d, const TacArgs &a, hipStream_t s)
{
    if (a.B == 0) return hipSuccess;
    if (d.R == 0) {
        // nothing to order; the iteration is the compute ops back to back
        if (!a.simulate) return hipSuccess;
        SimArgs sa{a.B, nullptr, 0, a.op_time, a.recv_time, a.makespan, a.eff, a.U, a.L, a.S};
        sa.f32 = a.f32;
        return launch_simulate(d, sa, s);
    }
    TacKernelParams p{};
    p.B = a.B; p.R = d.R; p.W = d.W; p.C = d.C; p.Cpad = d.Cpad; p.N = d.N;
    p.cls_dep = d.d_cls_dep; p.cls_depT = d.d_cls_depT; p.cls_cnt0 = d.d_cls_cnt0;
    p.cls_ptr = d.d_cls_ptr; p.cls_cols = d.d_cls_cols;
    p.op_time = a.op_time; p.recv_time = a.recv_time; p.f32 = a.f32 ? 1 : 0;
    p.order = a.order; p.rank = a.rank; p.sel_P = a.sel_P; p.sel_Mplus = a.sel_Mplus;
    p.simulate = a.simulate ? 1 : 0;
    p.makespan = a.makespan; p.eff = a.eff; p.U = a.U; p.L = a.L; p.S = a.S;
    p.only_flagged = nullptr;

    // graphs with few classes: register-resident kernel; graphs with many: bit-sliced kernel; then the
    // general kernel for the samples either of them flagged (those with a transfer time of zero).
    // The handle's workspace: one flag per sample first, the state of the running kernel after them.
    const size_t flag_bytes = ((size_t)a.B * sizeof(int32_t) + 255) & ~(size_t)255;
    const size_t lds_small = tac_lds_bytes(d, false);
    const bool small = tac_small_graph(d.R, d.W, d.C);              // one wave per sample, state in LDS
    const bool gstate = lds_small > 150 * 1024;                     // state in global memory
    const int gstate_grid = a.B < 256 ? a.B : 256;
    const size_t gstate_bytes = gstate ? tac_gstate_bytes(d) * (size_t)gstate_grid : 0;
    if (a.ext_flags) {
        // the caller's flags, no workspace: the register-resident kernel, then the one-wave kernel with its
        // state in LDS for the samples that were flagged
        if (a.sel_P || a.sel_Mplus || !small || !(d.C <= 8 * 64 && d.W <= 6)) return hipErrorNotSupported;
        const hipError_t e = launch_tac_reg(d, a, a.ext_flags, s);
        if (e != hipSuccess) return e;
        p.only_flagged = a.ext_flags;
        const int grid = a.B < 256 * 16 ? a.B : 256 * 16;
        return launch_tac_t<64, false>(d, p, grid, lds_small, s);
    }
    if (!a.sel_P && !a.sel_Mplus && d.C <= 8 * 64 && d.W <= 6) {
        hipError_t e = ensure_workspace(&d, flag_bytes + gstate_bytes);
        if (e != hipSuccess) return e;
        int32_t *flags = static_cast<int32_t *>(d.d_work);
        e = launch_tac_reg(d, a, flags, s);
        if (e == hipSuccess) p.only_flagged = flags;
        else if (e != hipErrorNotSupported) return e;
    }
    if (!p.only_flagged && !a.sel_P && !a.sel_Mplus && !small && tac_sliced_fits(d)) {
        // (sized first for the general kernel's pass over the flagged samples, so that the block is not replaced
        // between the two launches)
        hipError_t e = ensure_workspace(&d, flag_bytes + gstate_bytes);
        if (e != hipSuccess) return e;
        int32_t *flags = nullptr;
        e = launch_tac_sliced(d, a, flag_bytes, &flags, s);
        if (e == hipSuccess) p.only_flagged = flags;
        else if (e != hipErrorNotSupported) return e;
    }

    if (small) {
        const int grid = a.B < 256 * 16 ? a.B : 256 * 16;
        return launch_tac_t<64, false>(d, p, grid, lds_small, s);
    }
    if (!gstate) {
        const int grid = a.B < 256 * 2 ? a.B : 256 * 2;
        return launch_tac_t<256, false>(d, p, grid, lds_small, s);
    }
    // state in global memory, one large workgroup per sample
    const size_t lds = tac_lds_bytes(d, true);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    p.gstate_stride = tac_gstate_bytes(d);
    hipError_t e = ensure_workspace(&d, flag_bytes + gstate_bytes);
    if (e != hipSuccess) return e;
    if (p.only_flagged) p.only_flagged = static_cast<int32_t *>(d.d_work);   // (the block did not move: it was sized for this)
    p.gstate = static_cast<char *>(d.d_work) + flag_bytes;
    return launch_tac_t<1024, true>(d, p, gstate_grid, lds, s);
}

}  // namespace tictac
