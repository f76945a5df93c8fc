// TAC (Sec. 4.3, Algorithm 3) with the iteration under its order (Sec. 3.2) for graphs with many
// classes of compute ops (thousands of distinct dependency sets, up to 4096 recvs).  One workgroup
// per timing sample: a control wave that selects, and up to fifteen worker waves that keep the
// properties of Algorithm 1 up to date.
//
// The selection loop of Algorithm 3 takes the properties of Algorithm 1 afresh in every round; as in
// the other TAC kernels they are maintained incrementally, on classes (ops with one dependency set
// count as one op with their total time).  What is specific to this kernel:
//   * |dep(c) ∩ R|, the number of outstanding recvs of a class, is the only per-class quantity that
//     every round touches.  The counts of 64 classes are kept bit-sliced in the registers of one
//     lane (plane j holds bit j of the 64 counts), so removing a recv from all classes that hold it
//     is a ripple-borrow over the planes with the 64-bit column of that recv as the borrow-in, and
//     "which classes just fell to one outstanding recv" is one more bitwise expression.  Nothing
//     per class is read from or written to memory in a round, only the column (8 bytes per lane).
//   * A class that falls to one outstanding recv is an event: its last recv is found from its row
//     and the outstanding set, and (class, recv, class time) goes to the control wave through a
//     list in LDS.  The control wave adds the class times to P in a fixed order (ascending class
//     for one recv), so the sums do not depend on which wave was first.
//   * M of a class is needed only when no outstanding recv has P > 0 (then the recv of lowest index
//     among those of minimal M+ is selected: the minimum of M over the classes with two or more
//     outstanding recvs) or when the comparator ties.  It is then formed afresh, as the sum of the
//     outstanding transfer times of the row, and only for the classes that can attain the minimum:
//     dep(u) ⊆ dep(v) along every edge u -> v, so M(u) <= M(v), and when both have two or more
//     outstanding recvs and the sums are equal the outstanding recvs are the same (times are
//     positive here).  A class one of whose "parents" (classes of predecessor ops with a strictly
//     smaller dep) still has two or more outstanding recvs is therefore left out; the number of
//     such parents per class is kept in memory (two bits per class) and decremented at the
//     parents' events.  On layered graphs a few hundred of tens of thousands of classes remain.
//   * A class is released to the compute device when its last recv is selected, and P of that recv
//     at its selection is exactly the time released then, so the closed form of the iteration
//     (k4_simulate.hip) needs nothing but the order and the values of P at selection.
//   * A sample with a transfer time of zero is flagged for the general kernel (k3_tac.hip), which
//     takes the literal path for it.
#include "device_utils.h"
#include "internal.h"

namespace tictac {

constexpr int kPlanes = 13;             // bit planes of a count: up to 8191 recvs in a dep
constexpr int kEvPerWave = 16;          // events of one round and worker wave kept in LDS; further ones go to memory
constexpr int kWorkersMax = 15;         // worker waves per workgroup, next to the control wave

enum : int { REQ_DONE = 0, REQ_QEMPTY = 1, REQ_MPLUS = 2, REQ_FLUSH = 3 };
enum : int { CT_REQ = 1, CT_BEST = 2, CT_R1 = 3, CT_R2 = 4, CT_CIDX = 5, CT_WORDS = 16 };

struct SlicedParams {
    int32_t B, R, W, C, CW, CWpad, N;
    const uint64_t *cls_dep;        // [C][W]
    const int32_t *cls_ptr, *cls_cols;
    const uint64_t *colbits;        // [R][CWpad]
    const uint64_t *planes0;        // [kPlanes][CWpad]
    const uint64_t *live0;          // [CWpad]
    const uint64_t *ndom0;          // [CWpad][2]
    const int2 *cls_par;            // [C] parents of every class (-1: none)
    const int4 *crec;               // [C]
    const int32_t *child_ovf;
    const int32_t *single_ptr, *single_cls;
    const int32_t *empty_cls;
    int32_t n_empty;
    const void *op_time, *recv_time;
    int32_t f32;
    int32_t *order, *rank;
    int32_t simulate;
    double *makespan, *eff, *U, *L, *S;
    int32_t *flags;                 // [B] 1 = left to the general kernel
    char *scratch;                  // per workgroup: class times [C] f64, parent counts [CWpad][2] u64, spilled events [C] int2,
                                    // the classes with two or more outstanding recvs [CWpad] u64 (written when a tie needs them)
    size_t scratch_stride;
};

struct EvEntry {                    // 16 bytes: a class that fell to one outstanding recv, that recv, the class time
    int32_t cls;
    int32_t sole;
    double ct;
};

__device__ __forceinline__ void lds_only_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void wait_memory() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ uint64_t readlane_u64(uint64_t v, int l)     // l wave-uniform
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
    return ((uint64_t)hi << 32) | lo;
}

// A value that is the same in every lane, moved to scalar registers: what is computed from it is
// known to be uniform, and branches on it are scalar branches.
__device__ __forceinline__ double uniform_f64(double v)
{
    return __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(v)), __builtin_amdgcn_readfirstlane(__double2loint(v)));
}
__device__ __forceinline__ uint64_t uniform_u64(uint64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ int wave_sum_i32_dpp(int v)
{
    v += dpp_i32<0x111, 0xf>(0, v);
    v += dpp_i32<0x112, 0xf>(0, v);
    v += dpp_i32<0x114, 0xf>(0, v);
    v += dpp_i32<0x118, 0xf>(0, v);
    v += dpp_i32<0x142, 0xa>(0, v);
    v += dpp_i32<0x143, 0xc>(0, v);
    return __builtin_amdgcn_readlane(v, 63);
}

// the even bits of x (bit 2i -> bit i), x having no odd bit set
__device__ __forceinline__ uint32_t even_bits(uint64_t x)
{
    x = (x | (x >> 1)) & 0x3333333333333333ull;
    x = (x | (x >> 2)) & 0x0f0f0f0f0f0f0f0full;
    x = (x | (x >> 4)) & 0x00ff00ff00ff00ffull;
    x = (x | (x >> 8)) & 0x0000ffff0000ffffull;
    x = (x | (x >> 16)) & 0x00000000ffffffffull;
    return (uint32_t)x;
}

// M of class c, the sum of the outstanding transfer times of its row, and its lowest outstanding recv.
// Called by a whole wave; lane w takes word w of the row and the partial sums are added in lane order.
__device__ __forceinline__ void class_M(const uint64_t *__restrict__ row, const uint64_t *alive, const double *t,
                                        int W, int lane, double &M, int &low)
{
    uint64_t x = lane < W ? (row[lane] & alive[lane]) : 0ull;
    int lo = x ? lane * 64 + __builtin_ctzll(x) : INT32_MAX;
    double s = 0.0;
    while (x) {
        s += t[lane * 64 + __builtin_ctzll(x)];
        x &= x - 1;
    }
    M = wave_sum_f64_dpp(s);
    low = wave_min_i32_dpp(lo);
}

template <int KW>
__global__ void __launch_bounds__(64 * (kWorkersMax + 1))
tac_sliced_kernel(const SlicedParams p)
{
    extern __shared__ double smem[];
    const int R = p.R, W = p.W, C = p.C, N = p.N, CW = p.CW, CWpad = p.CWpad;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // in a scalar register: branches on it are uniform
    const int NT = blockDim.x, NWT = NT - 64;       // threads, worker threads
    const int n_waves = NT >> 6;

    // ---- LDS ----
    double *t = smem;                               // [R]      Time(recv)
    double *P = t + R;                              // [R + 1]  P of Algorithm 1; P of a selected recv stays as it was at selection
    double *cbase = P + (R + 1);                    // [64]     end of the transfers before each chunk of 64 steps
    double *A0 = cbase + 64;                        // [1]      time of the classes that depend on no recv
    unsigned long long *cmin = reinterpret_cast<unsigned long long *>(A0 + 1);     // [2]  minima of M (bit patterns)
    // (R + R + 1 + 64 + 1 + 2 doubles: a multiple of 16 bytes)
    EvEntry *ev = reinterpret_cast<EvEntry *>(cmin + 2);                            // [kWorkersMax][kEvPerWave]
    uint64_t *alive = reinterpret_cast<uint64_t *>(ev + kWorkersMax * kEvPerWave);  // [W]
    uint64_t *Qb = alive + W;                                                       // [W] outstanding recvs with P > 0
    int32_t *ctrl = reinterpret_cast<int32_t *>(Qb + W);                            // [CT_WORDS]
    int32_t *evcnt = ctrl + CT_WORDS;                                               // [16] events of the round, per worker wave
    uint16_t *ordl = reinterpret_cast<uint16_t *>(evcnt + 16);                      // [R] the order so far
    uint16_t *stage = ordl + R + (R & 1);                                           // [64] members of Q of the chunk being scanned

    // ---- per-workgroup memory ----
    char *scr = p.scratch + (size_t)blockIdx.x * p.scratch_stride;
    double *ct = reinterpret_cast<double *>(scr);                                   // [C]
    uint64_t *ndom = reinterpret_cast<uint64_t *>(ct + C);                          // [CWpad][2]
    // events beyond kEvPerWave of one wave and round, (class, recv): a region per worker wave, as large as the
    // number of its classes
    int2 *spill = reinterpret_cast<int2 *>(ndom + (size_t)2 * CWpad);              // [kWorkersMax][64 * 64 * KW]
    uint64_t *live_pub = reinterpret_cast<uint64_t *>(spill + (size_t)kWorkersMax * 4096 * KW);     // [CWpad]
    constexpr int kSpillPerWave = 4096 * KW;
    uint32_t *ndom32 = reinterpret_cast<uint32_t *>(ndom);

    // ---- worker state: KW class words per lane ----
    uint64_t pl[kPlanes][KW];
    uint64_t live[KW];
    int cwk[KW];
    // consecutive class words go to different waves: classes are numbered along the graph, and the classes
    // that fall to one recv in a round are neighbours, whose events are then handled by many waves at once
    const int n_workers = n_waves - 1;
#pragma unroll
    for (int k = 0; k < KW; ++k) cwk[k] = lane * n_workers + (wave - 1) + k * NWT;

    for (int b = blockIdx.x; b < p.B; b += gridDim.x) {
        const TimeRow rt = time_row(p.recv_time, (size_t)b * R, p.f32 != 0);
        const TimeRow ot = time_row(p.op_time, (size_t)b * N, p.f32 != 0);
        __syncthreads();                    // the previous sample is finished with LDS and with its memory

        // ---- transfer times; samples with a zero among them are left to the general kernel ----
        int zero_seen = 0;
        for (int r = tid; r < R; r += NT) {
            const double x = rt[r];
            t[r] = x;
            zero_seen |= !(x > 0.0);
        }
        if (tid < CT_WORDS) { ctrl[tid] = 0; evcnt[tid] = 0; }
        const bool literal = __syncthreads_or(zero_seen) != 0;
        if (tid == 0) p.flags[b] = literal ? 1 : 0;
        if (literal) continue;              // uniform over the workgroup

        // ---- class times, parent counts ----
        for (int c = tid; c < C; c += NT) {
            double s = 0.0;
            const int mend = p.cls_ptr[c + 1];
            for (int m = p.cls_ptr[c]; m < mend; ++m) s += ot[p.cls_cols[m]];
            ct[c] = s;
        }
        for (int i = tid; i < 2 * CWpad; i += NT) ndom[i] = p.ndom0[i];
        __syncthreads();
        // P of a recv starts as the time of the classes that depend on it alone (ascending class)
        for (int r = tid; r < R; r += NT) {
            double s = 0.0;
            const int jend = p.single_ptr[r + 1];
            for (int j = p.single_ptr[r]; j < jend; ++j) s += ct[p.single_cls[j]];
            P[r] = s;
        }
        if (tid == 0) {
            double s = 0.0;
            for (int j = 0; j < p.n_empty; ++j) s += ct[p.empty_cls[j]];
            *A0 = s;
            P[R] = 0.0;
        }
        __syncthreads();
        for (int w = wave; w < W; w += n_waves) {
            const int r = w * 64 + lane;
            const uint64_t a_ = __ballot(r < R);
            const uint64_t q_ = __ballot(r < R && P[r < R ? r : 0] > 0.0);
            if (lane == 0) { alive[w] = a_; Qb[w] = q_; }
        }

        // ================= selection loop =================
        // The control wave and the worker waves run loops of their own (so that neither carries the other's
        // registers) that meet at the same workgroup barriers: one when the events of a round are in the list,
        // one when the control wave has posted what it needs next (a request to the workers, or the selection).
        if (wave == 0) {
            // What the control wave asks of the workers: it posts the request, and both sides pass the same
            // barriers while it is served (REQ_QEMPTY has two more inside).
#define TS_REQUEST(code)                                                                  \
            {                                                                             \
                if (lane == 0) ctrl[CT_REQ] = (code);                                     \
                lds_only_barrier();                                                       \
                if ((code) == REQ_FLUSH) wait_memory();                                   \
                if ((code) == REQ_QEMPTY) { wait_memory(); lds_only_barrier(); lds_only_barrier(); } \
                if ((code) == REQ_MPLUS) { wait_memory(); lds_only_barrier(); }           \
                lds_only_barrier();                                                       \
            }
            for (int step = 0; step < R; ++step) {
                lds_only_barrier();         // the events of the previous round are in the list

                // ---- the events of the previous round: class times into P, new members of Q ----
                // Every worker wave has left its events in a region of its own, in an order that depends on
                // nothing but the state of the round.  They are taken wave by wave, 64 at a time: the events of a
                // chunk that name one recv add their class times to its P one after the other, in list order, so
                // the sums do not depend on which wave was first.
                const int cnt_w = lane < n_workers ? evcnt[lane] : 0;
                int incl_w = cnt_w;
                incl_w += dpp_i32<0x111, 0xf>(0, incl_w);
                incl_w += dpp_i32<0x112, 0xf>(0, incl_w);
                incl_w += dpp_i32<0x114, 0xf>(0, incl_w);
                incl_w += dpp_i32<0x118, 0xf>(0, incl_w);          // (at most fifteen workers: the first row of lanes)
                const int n = __builtin_amdgcn_readlane(incl_w, 15);
                if (wave_max_i32_dpp(cnt_w) > kEvPerWave) TS_REQUEST(REQ_FLUSH)   // entries in memory: wait until they have arrived
                for (int base = 0; base < n; base += 64) {      // (no event: nothing to do)
                    const int pos = base + lane;
                    const int m = min(64, n - base);
                    // the wave whose region holds position pos, and the offset in it
                    int wv = 0, off = 0;
                    for (int v = 0; v < n_workers; ++v) {
                        const int end_v = __builtin_amdgcn_readlane(incl_w, v), cnt_v = __builtin_amdgcn_readlane(cnt_w, v);
                        if (pos < end_v && pos >= end_v - cnt_v) { wv = v; off = pos - (end_v - cnt_v); }
                    }
                    int sole = -1;
                    double x = 0.0;
                    if (lane < m) {
                        if (off < kEvPerWave) {
                            sole = ev[wv * kEvPerWave + off].sole;
                            x = ev[wv * kEvPerWave + off].ct;
                        } else {
                            const int2 q = spill[(size_t)wv * kSpillPerWave + off - kEvPerWave];
                            sole = q.y;
                            x = ct[q.x];
                        }
                    }
                    int rank = 0;                   // earlier events of the chunk with the same recv
                    for (int i = 0; i < m; ++i) {
                        const int si = __builtin_amdgcn_readlane(sole, i);
                        rank += (si == sole && i < lane) ? 1 : 0;
                    }
                    const int maxrank = wave_max_i32_dpp(lane < m ? rank : 0);
                    for (int j = 0; j <= maxrank; ++j) {
                        if (lane < m && rank == j) P[sole] += x;
                        wave_sync();
                    }
                    if (lane < m && P[sole] > 0.0) atomicOr((unsigned long long *)&Qb[sole >> 6], 1ull << (sole & 63));
                    wave_sync();
                }

                // ---- the selection ----
                const uint64_t q_l = lane < W ? Qb[lane] : 0ull;
                const int cnt_l = __builtin_popcountll(q_l);
                const int nq = wave_sum_i32_dpp(cnt_l);
                int best;
                if (nq == 0) {
                    // no outstanding recv has P > 0: the recv of lowest index among those of minimal M+
                    if (lane == 0) {
                        cmin[0] = (unsigned long long)__double_as_longlong(TT_INF);
                        ctrl[CT_CIDX] = INT32_MAX;
                    }
                    TS_REQUEST(REQ_QEMPTY)
                    const unsigned long long g = uniform_u64(cmin[0]);
                    if (g == (unsigned long long)__double_as_longlong(TT_INF)) {
                        // no class with two outstanding recvs: every M+ is infinite, the lowest outstanding recv
                        const uint64_t a_l = lane < W ? alive[lane] : 0ull;
                        const uint64_t nzl = __ballot(a_l != 0ull);
                        const int L = nzl ? __builtin_ctzll(nzl) : 0;
                        best = L * 64 + __builtin_ctzll(readlane_u64(a_l, L) | (1ull << 63));
                    } else {
                        best = __builtin_amdgcn_readfirstlane(ctrl[CT_CIDX]);
                    }
                } else if (nq == 1) {
                    const uint64_t nzl = __ballot(q_l != 0ull);
                    const int L = __builtin_ctzll(nzl);
                    best = L * 64 + __builtin_ctzll(readlane_u64(q_l, L));
                } else {
                    // ascending scan over Q with the comparator.  Rank of this lane's first member of Q:
                    int incl = cnt_l;
                    incl += dpp_i32<0x111, 0xf>(0, incl);
                    incl += dpp_i32<0x112, 0xf>(0, incl);
                    incl += dpp_i32<0x114, 0xf>(0, incl);
                    incl += dpp_i32<0x118, 0xf>(0, incl);
                    incl += dpp_i32<0x142, 0xa>(0, incl);
                    incl += dpp_i32<0x143, 0xc>(0, incl);
                    const int first_rank = incl - cnt_l;
                    // best so far and its P and Time, the same in every lane (kept in vector registers and
                    // updated by selects, so that a step of the scan has no branch but the test for a tie)
                    int s_best = -1;
                    double s_Pb = 0.0, s_tb = 0.0, s_mpb = 0.0;
                    int s_mpb_ok = 0;
                    bool scanned = false;
                    if (nq <= 64) {
                        // One member of Q per lane.  The scan replaces its best so far by the first later member
                        // that precedes it: all later members are compared with the best at once, and the scan
                        // jumps to the first that precedes it, until none does.  A tie met before that is left to
                        // the loop below.
                        {
                            int rk = first_rank;
                            uint64_t x = q_l;
                            while (x) {
                                stage[rk] = (uint16_t)(lane * 64 + __builtin_ctzll(x));
                                x &= x - 1;
                                ++rk;
                            }
                        }
                        wave_sync();
                        const int a_l = lane < nq ? (int)stage[lane] : 0;
                        const double P_l = P[a_l], t_l = t[a_l];
                        wave_sync();
                        int cur = 0;
                        for (;;) {
                            const double Pc = readlane_f64(P_l, cur), tc = readlane_f64(t_l, cur);
                            const double xa = fmin(Pc, t_l);                // min{P_B, M_A}: A = this lane's member, B = the best
                            const double ya = fmin(P_l, tc);                // min{P_A, M_B}
                            const bool later = lane > cur && lane < nq;
                            const uint64_t lt = __ballot(later && xa < ya), eq = __ballot(later && xa == ya);
                            const int first_lt = lt ? __builtin_ctzll(lt) : 64, first_eq = eq ? __builtin_ctzll(eq) : 64;
                            if (first_eq < first_lt) break;                 // a tie comes first
                            if (first_lt == 64) { scanned = true; break; }
                            cur = first_lt;
                        }
                        if (scanned) s_best = __builtin_amdgcn_readlane(a_l, cur);
                    }
                    for (int base = 0; base < nq && !scanned; base += 64) {
                        // members base .. base + 63 of Q into the staging list, then one member per lane
                        {
                            int rk = first_rank;
                            uint64_t x = q_l;
                            while (x) {
                                if (rk >= base && rk < base + 64) stage[rk - base] = (uint16_t)(lane * 64 + __builtin_ctzll(x));
                                x &= x - 1;
                                ++rk;
                            }
                        }
                        wave_sync();
                        const int m = min(64, nq - base);
                        const int a_l = lane < m ? (int)stage[lane] : 0;
                        const double P_l = P[a_l], t_l = t[a_l];
                        wave_sync();
                        for (int j = 0; j < m; ++j) {
                            const int a = __builtin_amdgcn_readlane(a_l, j);
                            const double Pa = readlane_f64(P_l, j), ta = readlane_f64(t_l, j);
                            const bool first = s_best < 0;
                            const double xa = fmin(s_Pb, ta);               // min{P_B, M_A}, A = a, B = best
                            const double ya = fmin(Pa, s_tb);               // min{P_A, M_B}
                            bool take = first || xa < ya;
                            if (__builtin_amdgcn_readfirstlane((int)(!first && xa == ya))) {
                                // a tie of the comparator: M+ of both decides (Case 2); M+ of the best so far is
                                // kept until the best changes
                                if (lane == 0) {
                                    cmin[0] = (unsigned long long)__double_as_longlong(TT_INF);
                                    cmin[1] = (unsigned long long)__double_as_longlong(TT_INF);
                                    ctrl[CT_R1] = a;
                                    ctrl[CT_R2] = s_mpb_ok ? -1 : s_best;
                                }
                                TS_REQUEST(REQ_MPLUS)
                                const double mp_a = __longlong_as_double((long long)uniform_u64(cmin[0]));
                                if (!s_mpb_ok) s_mpb = __longlong_as_double((long long)uniform_u64(cmin[1]));
                                s_mpb_ok = 1;
                                take = mp_a < s_mpb;
                                if (take) s_mpb = mp_a;
                            } else if (take) {
                                s_mpb_ok = 0;
                            }
                            s_best = take ? a : s_best;
                            s_Pb = take ? Pa : s_Pb;
                            s_tb = take ? ta : s_tb;
                        }
                    }
                    best = __builtin_amdgcn_readfirstlane(s_best);
                }

                // ---- record the selection and remove the recv ----
                if ((unsigned)best >= (unsigned)R) {        // never taken when the bookkeeping is consistent; keeps indices in range
                    const uint64_t a_l = lane < W ? alive[lane] : 0ull;
                    const uint64_t nzl = __ballot(a_l != 0ull);
                    const int L = nzl ? __builtin_ctzll(nzl) : 0;
                    best = nzl ? L * 64 + __builtin_ctzll(readlane_u64(a_l, L) | (1ull << 63)) : 0;
                    if ((unsigned)best >= (unsigned)R) best = 0;
                }
                if (lane == 0) {
                    ctrl[CT_BEST] = best;
                    ctrl[CT_REQ] = REQ_DONE;
                    ordl[step] = (uint16_t)best;
                    alive[best >> 6] &= ~(1ull << (best & 63));
                    Qb[best >> 6] &= ~(1ull << (best & 63));
                }
                lds_only_barrier();
            }
#undef TS_REQUEST
        } else {
#pragma unroll
            for (int k = 0; k < KW; ++k) {
                const bool in = cwk[k] < CW;
                live[k] = in ? p.live0[cwk[k]] : 0ull;
#pragma unroll
                for (int j = 0; j < kPlanes; ++j) pl[j][k] = in ? p.planes0[(size_t)j * CWpad + cwk[k]] : 0ull;
            }
            for (int step = 0; step < R; ++step) {
                lds_only_barrier();
                for (;;) {
                    lds_only_barrier();
                    const int req = __builtin_amdgcn_readfirstlane(ctrl[CT_REQ]);
                    if (req == REQ_DONE) break;
                    if (req == REQ_FLUSH) {
                        wait_memory();
                    } else if (req == REQ_QEMPTY) {
                        // parent counts are decremented by atomics that are not waited for: wait now
                        wait_memory();
                        lds_only_barrier();
                        double lm = TT_INF;
                        int li = INT32_MAX;
                        if (wave >= 1) {
    #pragma unroll
                            for (int k = 0; k < KW; ++k) {
                                uint64_t cand = 0ull;
                                if (live[k] != 0ull) {
                                    const uint64_t lo = __hip_atomic_load(&ndom[(size_t)2 * cwk[k]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                    const uint64_t hi = __hip_atomic_load(&ndom[(size_t)2 * cwk[k] + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                    const uint64_t nz = (uint64_t)even_bits((lo | (lo >> 1)) & 0x5555555555555555ull) |
                                                        ((uint64_t)even_bits((hi | (hi >> 1)) & 0x5555555555555555ull) << 32);
                                    cand = live[k] & ~nz;
                                }
                                uint64_t bal = __ballot(cand != 0ull);
                                while (bal) {
                                    const int L = __builtin_ctzll(bal);
                                    bal &= bal - 1;
                                    uint64_t mL = readlane_u64(cand, L);
                                    const int cwL = __builtin_amdgcn_readlane(cwk[k], L);
                                    while (mL) {
                                        const int c = cwL * 64 + __builtin_ctzll(mL);
                                        mL &= mL - 1;
                                        double M;
                                        int low;
                                        class_M(p.cls_dep + (size_t)c * W, alive, t, W, lane, M, low);
                                        if (M < lm || (M == lm && low < li)) { lm = M; li = low; }
                                    }
                                }
                            }
                            if (lane == 0 && li != INT32_MAX) atomicMin(&cmin[0], (unsigned long long)__double_as_longlong(lm));
                        }
                        lds_only_barrier();
                        if (wave >= 1 && lane == 0 && li != INT32_MAX && (unsigned long long)__double_as_longlong(lm) == cmin[0])
                            atomicMin(&ctrl[CT_CIDX], li);
                    } else {
                        // REQ_MPLUS: M+ of one or two recvs = the minimum of M over the classes with two or more
                        // outstanding recvs that hold the recv.  As for the minimum over all classes, a class with
                        // a parent that holds the recv and still has two outstanding recvs cannot be the only one
                        // to attain it; the workers first publish which classes those are.
#pragma unroll
                        for (int k = 0; k < KW; ++k)
                            if (cwk[k] < CW) live_pub[cwk[k]] = live[k];
                        wait_memory();
                        lds_only_barrier();
#pragma unroll
                        for (int which = 0; which < 2; ++which) {
                            const int r = __builtin_amdgcn_readfirstlane(ctrl[which == 0 ? CT_R1 : CT_R2]);
                            if (r < 0) continue;
                            const uint64_t *colr = p.colbits + (size_t)r * CWpad;
                            double lm = TT_INF;
                            bool any = false;
#pragma unroll
                            for (int k = 0; k < KW; ++k) {
                                uint64_t set = 0ull;
                                if (live[k] != 0ull) {
                                    uint64_t x = live[k] & colr[cwk[k]];
                                    while (x) {
                                        const int bit = __builtin_ctzll(x);
                                        x &= x - 1;
                                        const int2 pr = p.cls_par[cwk[k] * 64 + bit];
                                        bool dom = false;
                                        if (pr.x >= 0)
                                            dom = ((__hip_atomic_load(&live_pub[pr.x >> 6], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) &
                                                    colr[pr.x >> 6]) >> (pr.x & 63)) & 1ull;
                                        if (!dom && pr.y >= 0)
                                            dom = ((__hip_atomic_load(&live_pub[pr.y >> 6], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) &
                                                    colr[pr.y >> 6]) >> (pr.y & 63)) & 1ull;
                                        if (!dom) set |= 1ull << bit;
                                    }
                                }
                                uint64_t bal = __ballot(set != 0ull);
                                while (bal) {
                                    const int L = __builtin_ctzll(bal);
                                    bal &= bal - 1;
                                    uint64_t mL = readlane_u64(set, L);
                                    const int cwL = __builtin_amdgcn_readlane(cwk[k], L);
                                    while (mL) {
                                        const int c = cwL * 64 + __builtin_ctzll(mL);
                                        mL &= mL - 1;
                                        double M;
                                        int low;
                                        class_M(p.cls_dep + (size_t)c * W, alive, t, W, lane, M, low);
                                        lm = fmin(lm, M);
                                        any = true;
                                    }
                                }
                            }
                            if (lane == 0 && any) atomicMin(&cmin[which], (unsigned long long)__double_as_longlong(lm));
                        }
                    }
                    lds_only_barrier();
                }
                const int best = __builtin_amdgcn_readfirstlane(ctrl[CT_BEST]);

                // ================= the counts of the classes that hold `best`; events =================
                int my_events = 0;              // events of this wave in this round (uniform)
                uint64_t anyl = 0ull;
#pragma unroll
                for (int k = 0; k < KW; ++k) anyl |= live[k];
                if (__ballot(anyl != 0ull) != 0ull) {           // uniform: some class of this wave still has two recvs outstanding
                    uint64_t col[KW], evw[KW];
#pragma unroll
                    for (int k = 0; k < KW; ++k)
                        col[k] = live[k] != 0ull ? p.colbits[(size_t)best * CWpad + cwk[k]] : 0ull;
#pragma unroll
                    for (int k = 0; k < KW; ++k) {
                        const uint64_t m = col[k] & live[k];
                        uint64_t borrow = m;
#pragma unroll
                        for (int j = 0; j < kPlanes; ++j) {
                            // plane ^= borrow; borrow &= plane (the borrow goes on where the bit was 0), on the two
                            // halves, in place: written out so that every plane keeps its registers
                            uint32_t plo = (uint32_t)pl[j][k], phi = (uint32_t)(pl[j][k] >> 32);
                            uint32_t blo = (uint32_t)borrow, bhi = (uint32_t)(borrow >> 32);
                            asm volatile("v_xor_b32 %0, %0, %1\n\tv_and_b32 %1, %1, %0" : "+v"(plo), "+v"(blo));
                            asm volatile("v_xor_b32 %0, %0, %1\n\tv_and_b32 %1, %1, %0" : "+v"(phi), "+v"(bhi));
                            pl[j][k] = ((uint64_t)phi << 32) | plo;
                            borrow = ((uint64_t)bhi << 32) | blo;
                        }
                        uint64_t hi = pl[1][k];
#pragma unroll
                        for (int j = 2; j < kPlanes; ++j) hi |= pl[j][k];
                        evw[k] = m & pl[0][k] & ~hi;            // the count is now exactly one
                        live[k] &= ~evw[k];
                    }
#pragma unroll
                    for (int k = 0; k < KW; ++k) {
                        uint64_t mine = evw[k];
                        uint64_t bal = __ballot(mine != 0ull);
                        while (bal) {
                            // up to four events at a time, so that their trips to memory overlap
                            int c0 = 0, c1 = 0, c2 = 0, c3 = 0, nb = 0;
                            while (nb < 4 && bal) {
                                const int L = __builtin_ctzll(bal);
                                const uint64_t mL = readlane_u64(mine, L);
                                const int c = __builtin_amdgcn_readlane(cwk[k], L) * 64 + __builtin_ctzll(mL);
                                if (nb == 0) c0 = c; else if (nb == 1) c1 = c; else if (nb == 2) c2 = c; else c3 = c;
                                ++nb;
                                const uint64_t rest = mL & (mL - 1);
                                if (lane == L) mine = rest;
                                if (!rest) bal &= bal - 1;
                            }
                            const int myc = lane == 0 ? c0 : (lane == 1 ? c1 : (lane == 2 ? c2 : c3));
                            double ctv = 0.0;
                            int4 rec = make_int4(0, 0, 0, 0);
                            if (lane < nb) { ctv = ct[myc]; rec = p.crec[myc]; }
                            uint64_t x0 = 0ull, x1 = 0ull, x2 = 0ull, x3 = 0ull;
                            if (lane < W) {
                                x0 = p.cls_dep[(size_t)c0 * W + lane];
                                if (nb > 1) x1 = p.cls_dep[(size_t)c1 * W + lane];
                                if (nb > 2) x2 = p.cls_dep[(size_t)c2 * W + lane];
                                if (nb > 3) x3 = p.cls_dep[(size_t)c3 * W + lane];
                                const uint64_t al = alive[lane];
                                x0 &= al; x1 &= al; x2 &= al; x3 &= al;
                            }
                            // the one outstanding recv of each class
                            int mysole = 0;
#define TS_SOLE(e, x)                                                                     \
                            if (nb > e) {                                                 \
                                const uint64_t sb_ = __ballot(x != 0ull);                 \
                                const int S_ = sb_ ? __builtin_ctzll(sb_) : 0;            \
                                const uint64_t xs_ = readlane_u64(x, S_);                 \
                                const int so_ = xs_ ? S_ * 64 + __builtin_ctzll(xs_) : 0; \
                                if (lane == e) mysole = so_;                              \
                            }
                            TS_SOLE(0, x0) TS_SOLE(1, x1) TS_SOLE(2, x2) TS_SOLE(3, x3)
#undef TS_SOLE
                            if (lane < nb) {
                                const int idx = my_events + lane;
                                if (idx < kEvPerWave) {
                                    EvEntry *q = ev + (wave - 1) * kEvPerWave + idx;
                                    q->cls = myc;
                                    q->sole = mysole;
                                    q->ct = ctv;
                                } else {
                                    spill[(size_t)(wave - 1) * kSpillPerWave + idx - kEvPerWave] = make_int2(myc, mysole);
                                }
                                // this class no longer keeps its children out of the minimum of M
                                const int nch = rec.x;
                                for (int q = 0; q < nch; ++q) {
                                    int v;
                                    if (nch <= 3) v = q == 0 ? rec.y : (q == 1 ? rec.z : rec.w);
                                    else v = q == 0 ? rec.y : (q == 1 ? rec.z : p.child_ovf[rec.w + q - 2]);
                                    __hip_atomic_fetch_sub(&ndom32[v >> 4], 1u << ((v & 15) * 2), __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT);
                                }
                            }
                            my_events += nb;
                        }
                    }
                }
                if (lane == 0) evcnt[wave - 1] = my_events;
            }
        }

        // ================= outputs; iteration metrics (Sec. 3.2), by the control wave =================
        // (the order goes to memory here and not round by round: a store in flight would be waited for by
        // the next wait for a load of the control wave)
        if (wave == 0) {
            wave_sync();
            for (int s_ = lane; s_ < R; s_ += 64) {
                const int r = ordl[s_];
                p.order[(size_t)b * R + s_] = r;
                if (p.rank) p.rank[(size_t)b * R + r] = s_;
            }
        }
        if (p.simulate && wave == 0) {
            wave_sync();
            // P of a recv at its selection = time of the classes released by it; F_k = end of the k-th transfer
            const int n_chunks = (R + 63) / 64;
            double fc = 0.0;
            for (int ch = 0; ch < n_chunks; ++ch) {
                const int s = ch * 64 + lane;
                const double x = s < R ? t[ordl[s]] : 0.0;
                if (lane == 0) cbase[ch] = fc;
                fc += wave_sum_f64_dpp(x);
            }
            const double F = fc;
            wave_sync();
            double sfx = 0.0, mloc = -TT_INF;
            for (int ch = n_chunks - 1; ch >= 0; --ch) {
                const int s = ch * 64 + lane;                           // step s = transfer k = s + 1
                const int r = s < R ? (int)ordl[s] : 0;
                const double x = s < R ? t[r] : 0.0;
                const double a = s < R ? P[r] : 0.0;
                const double fk = cbase[ch] + wave_incl_scan_f64_dpp(x);
                const double inc = wave_incl_scan_f64_dpp(a);
                const double tot = lane63_f64(inc);
                if (s < R) mloc = fmax(mloc, fk + (sfx + (tot - inc + a)));
                sfx += tot;
            }
            const double sum_c = *A0 + sfx;
            mloc = fmax(mloc, sum_c);                                   // k = 0: nothing transferred yet, all compute time ahead
            const double m = fmax(wave_max_f64_dpp(mloc), F);
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

// ---- tables (built once per graph, on the device) ----

// colbits[r][cw]: one wave per (word w of the rows, class word cw) transposes a 64 x 64 block of bits
__global__ void __launch_bounds__(256)
sliced_colbits_kernel(int32_t R, int32_t W, int32_t C, int32_t CWpad, const uint64_t *__restrict__ cls_dep,
                      uint64_t *__restrict__ colbits)
{
    const int lane = threadIdx.x & 63;
    const long long gw = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (gw >= (long long)W * CWpad) return;             // uniform over the wave
    const int w = (int)(gw % W), cw = (int)(gw / W);
    const int c = cw * 64 + lane;
    const uint64_t x = c < C ? cls_dep[(size_t)c * W + w] : 0ull;
    uint64_t mine = 0ull;
    for (int i = 0; i < 64; ++i) {
        const uint64_t bal = __ballot((x >> i) & 1ull);
        if (lane == i) mine = bal;
    }
    const int r = w * 64 + lane;
    if (r < R) colbits[(size_t)r * CWpad + cw] = mine;
}

__global__ void __launch_bounds__(256)
sliced_planes_kernel(int32_t C, int32_t CWpad, const int32_t *__restrict__ cls_cnt0, uint64_t *__restrict__ planes0,
                     uint64_t *__restrict__ live0)
{
    const int lane = threadIdx.x & 63;
    const int cw = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (cw >= CWpad) return;
    const int c = cw * 64 + lane;
    const int cnt = c < C ? cls_cnt0[c] : 0;
    for (int j = 0; j < kPlanes; ++j) {
        const uint64_t bal = __ballot((cnt >> j) & 1);
        if (lane == 0) planes0[(size_t)j * CWpad + cw] = bal;
    }
    const uint64_t lv = __ballot(cnt >= 2);
    if (lane == 0) live0[cw] = lv;
}

hipError_t launch_sliced_tables(const Dag &d, hipStream_t s)
{
    if (!d.d_colbits) return hipSuccess;
    const long long waves = (long long)d.W * d.CWpad;
    hipLaunchKernelGGL(sliced_colbits_kernel, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s, d.R, d.W, d.C, d.CWpad,
                       d.d_cls_dep, d.d_colbits);
    hipLaunchKernelGGL(sliced_planes_kernel, dim3((unsigned)((d.CWpad + 3) / 4)), dim3(256), 0, s, d.C, d.CWpad, d.d_cls_cnt0,
                       d.d_planes0, d.d_live0);
    return hipGetLastError();
}

bool tac_sliced_fits(const Dag &d)
{
    return d.d_colbits != nullptr;
}

static size_t sliced_lds_bytes(const Dag &d)
{
    size_t b = ((size_t)2 * d.R + 68) * 8 + (size_t)kWorkersMax * kEvPerWave * sizeof(EvEntry) + (size_t)2 * d.W * 8 + (CT_WORDS + 16) * 4;
    b += ((size_t)d.R + (d.R & 1) + 64) * 2;
    return (b + 15) & ~(size_t)15;
}

static size_t tac_sliced_scratch_stride(const Dag &d, int KW)
{
    const size_t b = (size_t)d.C * 8 + (size_t)d.CWpad * 16 + (size_t)kWorkersMax * 4096 * KW * 8 + (size_t)d.CWpad * 8;
    return (b + 255) & ~(size_t)255;
}

template <int KW>
static hipError_t launch_sliced_k(SlicedParams &p, Dag &d, const TacArgs &a, size_t flag_bytes, int32_t **flags_out,
                                  hipStream_t s)
{
    int workers = (d.CW + KW * 64 - 1) / (KW * 64);
    if (workers < 1) workers = 1;
    if (workers > kWorkersMax) return hipErrorNotSupported;
    const int threads = 64 * (workers + 1);
    const size_t lds = sliced_lds_bytes(d);
    if (lds > 150 * 1024) return hipErrorNotSupported;
    hipError_t e;
    if (lds > 48 * 1024) {
        e = ensure_dynamic_lds(reinterpret_cast<const void *>(tac_sliced_kernel<KW>), lds);
        if (e != hipSuccess) return e;
    }
    int per_cu = 0;
    e = cached_blocks_per_cu(&per_cu, reinterpret_cast<const void *>(tac_sliced_kernel<KW>), threads, lds);
    if (e != hipSuccess) return e;
    if (per_cu < 1) per_cu = 1;
    int grid = per_cu * device_cu_count(d.device);
    if (grid > a.B) grid = a.B;
    p.scratch_stride = tac_sliced_scratch_stride(d, KW);
    e = ensure_workspace(&d, flag_bytes + p.scratch_stride * (size_t)grid);
    if (e != hipSuccess) return e;
    p.flags = static_cast<int32_t *>(d.d_work);
    p.scratch = static_cast<char *>(d.d_work) + flag_bytes;
    *flags_out = p.flags;
    hipLaunchKernelGGL((tac_sliced_kernel<KW>), dim3(grid), dim3(threads), lds, s, p);
    return hipGetLastError();
}

hipError_t launch_tac_sliced(Dag &d, const TacArgs &a, size_t flag_bytes, int32_t **flags_out, hipStream_t s)
{
    if (!tac_sliced_fits(d) || a.sel_P || a.sel_Mplus) return hipErrorNotSupported;
    SlicedParams p{};
    p.B = a.B; p.R = d.R; p.W = d.W; p.C = d.C; p.CW = d.CW; p.CWpad = d.CWpad; p.N = d.N;
    p.cls_dep = d.d_cls_dep; p.cls_ptr = d.d_cls_ptr; p.cls_cols = d.d_cls_cols;
    p.colbits = d.d_colbits; p.planes0 = d.d_planes0; p.live0 = d.d_live0; p.ndom0 = d.d_ndom0;
    p.cls_par = reinterpret_cast<const int2 *>(d.d_cls_par);
    p.crec = d.d_crec; p.child_ovf = d.d_child_ovf;
    p.single_ptr = d.d_single_ptr; p.single_cls = d.d_single_cls;
    p.empty_cls = d.d_empty_cls; p.n_empty = d.n_empty_cls;
    p.op_time = a.op_time; p.recv_time = a.recv_time; p.f32 = a.f32 ? 1 : 0;
    p.order = a.order; p.rank = a.rank;
    p.simulate = a.simulate ? 1 : 0;
    p.makespan = a.makespan; p.eff = a.eff; p.U = a.U; p.L = a.L; p.S = a.S;
    const int per_lane = (d.CW + kWorkersMax * 64 - 1) / (kWorkersMax * 64);
    if (per_lane <= 1) return launch_sliced_k<1>(p, d, a, flag_bytes, flags_out, s);
    if (per_lane <= 2) return launch_sliced_k<2>(p, d, a, flag_bytes, flags_out, s);
    if (per_lane <= 3) return launch_sliced_k<3>(p, d, a, flag_bytes, flags_out, s);
    if (per_lane <= 4) return launch_sliced_k<4>(p, d, a, flag_bytes, flags_out, s);
    return hipErrorNotSupported;
}

}  // namespace tictac
