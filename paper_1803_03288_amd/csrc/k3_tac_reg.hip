// TAC (Sec. 4.3, Algorithm 3) with the iteration under its order (Sec. 3.2), one wavefront
// per timing sample, for graphs with few classes (at most 8 per lane).  A workgroup is a few
// independent waves that share one read-only LDS copy of the class rows; lane l of a wave
// owns the classes l, l + 64, ... and keeps their outstanding counts and class times in
// VGPRs for the whole selection loop.  Per round nothing is read from global memory.
//
// The algorithm is the one described at the top of k3_tac.hip (incremental Algorithm 1;
// selection by the scan over Q = {outstanding recvs with P > 0}, or by the minimum of M over
// classes with two or more outstanding recvs when Q is empty).  How it is carried out here:
//   * a round is bound by instruction issue (the scalar unit first), so it is kept short: the
//     row bits of the selected recv come from one LDS read per lane, the per-class update is
//     branch-free, and whatever is wave-uniform stays in scalar registers;
//   * one register per class holds (count - 2) << 20 | sum of the indices of its outstanding
//     recvs.  It goes negative when the count falls below 2 (the only moments at which
//     anything else has to happen), and once the count is 1 the index sum *is* the last
//     outstanding recv of the class, to whose P the class time is then added: the class
//     "points" at that recv;
//   * Q, the set of recvs pointed at by a class with a positive time, is tracked by the number
//     of pointers and the targets of the latest two of them (one pointer: its target is the
//     member of Q, the common case on layered models; two pointers at two recvs: one
//     comparison).  With many classes per lane the latest four targets are kept: with three or
//     four pointers at distinct recvs the scan over Q is a sorting network on scalars and two or
//     three comparisons in straight-line code, and the members that stay are known afterwards.
//     Only the general path enumerates Q, from the class registers;
//   * M of a class is needed only when Q is empty or the comparator ties.  It is formed at the
//     first such round as the sum of the transfer times over the runs of consecutive recv
//     indices of its row and brought up to date from the order built so far; rounds that do
//     not need it do not touch it;
//   * the class totals of a sample are formed by one coalesced pass over its op_time row,
//     each column adding itself to its class's total in LDS;
//   * a class is released when the recv it pointed at (its last one) is selected, so its release
//     position kappa is that recv's position in the finished order; after the loop the class
//     times are added up by kappa and the makespan is max_k (F_k + S_k), F_k
//     the end of the k-th transfer, S_k the time of the classes with kappa >= k (the closed
//     form of the work-conserving device described in k4_simulate.hip);
//   * a sample with a transfer time of zero is not handled here: it is flagged for the
//     general kernel, which takes the literal path for it.
// LDS atomics of one wave are served in issue order and lane order, so the sums they form
// are reproducible from run to run.
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
    const int32_t *col_cls;     // [N]   class of every op_time column; NULL: gather by member lists
    const int32_t *run_ptr;     // [C+1]
    const int32_t *run_lo, *run_hi;
    const void *op_time, *recv_time;    // float64, or float32 when f32 is set
    int32_t f32;
    int32_t *order, *rank;
    int32_t simulate;
    double *makespan, *eff, *U, *L, *S;
    int32_t *flags;             // [B] 1 = left to the general kernel
    int32_t wave_doubles;       // LDS doubles per wave
    int32_t n_waves;            // total waves of the grid
};

// Waves per workgroup.  The class rows in LDS are shared by the workgroup, so with many classes
// per lane (large rows, many registers) one large workgroup per compute unit leaves the most
// LDS to the per-wave arrays; sixteen waves cap the registers at 128 per lane, four waves per SIMD.
constexpr int kRegWavesMax = 16;
constexpr int reg_waves(int KT) { return KT <= 4 ? 4 : kRegWavesMax; }
// Words per lane in the LDS table of class rows: the KT words of a lane sit next to each other,
// with one word of padding when KT is even, so that the lanes of a wave reading their k-th word
// fall into different banks (an even stride puts every 32 / gcd(stride, 32)-th lane on one bank).
constexpr int row_stride(int KT) { return (KT % 2 == 0) ? KT + 1 : KT; }
constexpr int CNT1 = 1 << 20;          // one unit of the outstanding count in `packed`
constexpr int IDX_MASK = CNT1 - 1;

// lowest outstanding recv of class (lane, k); rows: [2W][64][row_stride(KT)] halves, alive: [2W] halves in LDS
template <int KT>
__device__ __forceinline__ int first_alive(const uint32_t *rows, const uint32_t *alive, int W, int lane, int k)
{
    for (int h = 0; h < 2 * W; ++h) {
        const uint32_t x = rows[(h * 64 + lane) * row_stride(KT) + k] & alive[h];
        if (x) return h * 32 + __builtin_ctz(x);
    }
    return INT32_MAX;
}

// The per-class state is kept in individually named scalars (not arrays), so that every
// class stays in its own registers across the branches of the loop.  K(F) applies F to the
// class slots 0..7; a slot beyond KT compiles to nothing.
#define TT_EACH_K(F) F(0) F(1) F(2) F(3) F(4) F(5) F(6) F(7)

template <int KT>
__global__ void __launch_bounds__(64 * reg_waves(KT), (KT <= 3 ? 6 : (KT <= 4 ? 5 : 1)))
tac_reg_kernel(const TacRegParams p)
{
    extern __shared__ double smem[];
    const int R = p.R, W = p.W, C = p.C, N = p.N;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // ---- LDS: class rows shared by the workgroup, then one private region per wave ----
    constexpr int KS = row_stride(KT);
    uint32_t *rows = reinterpret_cast<uint32_t *>(smem);            // [2W][64][KS]
    const int rows_doubles = (2 * W * 64 * KS + 1) / 2;
    double *mine = smem + rows_doubles + (size_t)wave * p.wave_doubles;
    double *t = mine;                       // [R+1]  Time(recv); after the loop: class time by release position
    double *P = t + (R + 1);                // [R+1]  P; after the loop: positions, then the ends of the transfers
    int32_t *ordl = reinterpret_cast<int32_t *>(P + (R + 1));       // [R] order built so far
    uint32_t *aliveh = reinterpret_cast<uint32_t *>(ordl + R);      // [2W] outstanding recvs

    for (int idx = threadIdx.x; idx < 2 * W * 64 * KS; idx += blockDim.x) {
        const int h = idx / (64 * KS), rem = idx % (64 * KS);
        const int l = rem / KS, k = rem % KS;
        const int c = k * 64 + l;
        const uint64_t x = (k < KT && c < C) ? p.cls_dep[(size_t)c * W + (h >> 1)] : 0ull;
        rows[idx] = (h & 1) ? (uint32_t)(x >> 32) : (uint32_t)x;
    }
    __syncthreads();                        // the only workgroup barrier

    // ---- wave-uniform bounds of the member loops of the class slots ----
#define TT_DECL_CONST(k) int mmax_##k = 0;
    TT_EACH_K(TT_DECL_CONST)
#define TT_INIT_CONST(k)                                                                  \
    if constexpr (k < KT) {                                                               \
        const int c = k * 64 + lane;                                                      \
        int mx = c < C ? p.cls_ptr[c + 1] - p.cls_ptr[c] : 0;                             \
        for (int off = 32; off > 0; off >>= 1) mx = max(mx, __shfl_xor(mx, off));         \
        mmax_##k = __builtin_amdgcn_readfirstlane(mx);                                    \
    }
    TT_EACH_K(TT_INIT_CONST)

    const uint32_t *rows_lane = rows + lane * KS;      // this lane's KT words of half-row 0
    double *csum = P;                                  // [64 KT] class totals while they are summed (spans P, ordl, aliveh)

    const int gwave = blockIdx.x * (blockDim.x >> 6) + wave;
    for (int b = gwave; b < p.B; b += p.n_waves) {
        const TimeRow rt = time_row(p.recv_time, (size_t)b * R, p.f32 != 0);
        const TimeRow ot = time_row(p.op_time, (size_t)b * N, p.f32 != 0);
        wave_sync();                        // LDS of the previous sample is no longer read

        // ---- a. transfer times ----
        bool zero_seen = false;
        for (int r = lane; r < R; r += 64) {
            const double x = rt[r];
            t[r] = x;
            zero_seen |= !(x > 0.0);
        }
        const bool skip = __ballot(zero_seen) != 0ull;
        if (lane == 0) p.flags[b] = skip ? 1 : 0;
        if (skip) continue;

        // ---- b. class totals ----
#define TT_DECL_STATE(k) int pk_##k = -2 * CNT1, sole_##k = -1, mk_##k = 0; double M_##k = 0.0, ct_##k = 0.0;
        TT_EACH_K(TT_DECL_STATE)
        if (p.col_cls) {
            // the row is read once; every column (run of columns) adds itself to the total of its class
            for (int c = lane; c < 64 * KT; c += 64) csum[c] = 0.0;
            wave_sync();
            class_totals(csum, ot, p.col_cls, N, lane);
            wave_sync();
#define TT_READ_TOTAL(k) if constexpr (k < KT) { ct_##k = csum[k * 64 + lane]; }
            TT_EACH_K(TT_READ_TOTAL)
            wave_sync();
        } else {
#define TT_GATHER_TOTAL(k)                                                                \
            if constexpr (k < KT) {                                                       \
                const int c = k * 64 + lane;                                              \
                double s = 0.0;                                                           \
                if (c < C) {                                                              \
                    const int mbeg = p.cls_ptr[c], mcnt = p.cls_ptr[c + 1] - mbeg;        \
                    _Pragma("unroll 4")                                                   \
                    for (int m = 0; m < mmax_##k; ++m)                                    \
                        if (m < mcnt) s += ot[p.cls_cols[mbeg + m]];                      \
                }                                                                         \
                ct_##k = s;                                                               \
            }
            TT_EACH_K(TT_GATHER_TOTAL)
        }
#define TT_INIT_STATE(k)                                                                  \
        if constexpr (k < KT) {                                                           \
            const int c = k * 64 + lane;                                                  \
            if (c < C) pk_##k = (p.cls_cnt0[c] - 2) * CNT1 + p.cls_isum[c];               \
        }
        TT_EACH_K(TT_INIT_STATE)

        // ---- c. P, the bitsets of outstanding recvs and of Q ----
        for (int r = lane; r < R; r += 64) P[r] = 0.0;
        wave_sync();
        // A class with exactly one outstanding recv left and a positive time "points" at that
        // recv; Q is the set of recvs pointed at (the outstanding recvs with P > 0).  Tracked
        // wave-uniformly: the number of pointers and the targets of the latest ones, q0 the newest.
        // While there are no more pointers than tracked targets, Q is known without looking at
        // the classes.
        int qm = 0, q0 = 0, q1 = 0, q2 = 0, q3 = 0;
        // (four targets only where classes are many: graphs with few classes rarely have more than two
        // members in Q, and the forced rounds are measurably slower with the two extra values)
        constexpr bool kFour = KT >= 4;
        int m_sync = -1;                    // M_k is current up to this step; -1: not formed yet
        // lane 4 i + j: bit offsets of member i and of member j in the packed scalars of the scan over three or four
        const int pair_shift = 10 * min((lane >> 2) & 3, 2) | (10 * max((lane & 3) - 1, 0)) << 8;
        int32_t *ord_next = ordl;           // where the next selected recv is recorded

        // outstanding recvs as 32-bit halves in LDS, rebuilt from the order so far on the rare
        // path that needs them by index
        auto publish_alive = [&](int upto) {
            for (int h = lane; h < 2 * W; h += 64) {
                const int nbits = min(32, max(0, R - 32 * h));
                aliveh[h] = nbits >= 32 ? 0xffffffffu : ((1u << nbits) - 1u);
            }
            wave_sync();
            for (int s_ = lane; s_ < upto; s_ += 64) {
                const int r_ = ordl[s_];
                atomicAnd(&aliveh[r_ >> 5], ~(1u << (r_ & 31)));
            }
            wave_sync();
        };

        // M of the classes is only needed when Q is empty or the comparator ties, so its
        // updates are deferred: formed as the sum of the transfer times over the runs [lo, hi)
        // of consecutive recv indices of the class row, and then brought up to `upto` by the
        // subtractions of the rounds since m_sync, in their order.  ordl holds those rounds.
#define TT_M_FORM(k)                                                                      \
        if constexpr (k < KT) {                                                           \
            const int c = k * 64 + lane;                                                  \
            double Mk = 0.0;                                                              \
            if (c < C) {                                                                  \
                const int rend = p.run_ptr[c + 1];                                        \
                for (int q = p.run_ptr[c]; q < rend; ++q) {                               \
                    const int hi_ = p.run_hi[q];                                          \
                    for (int r_ = p.run_lo[q]; r_ < hi_; ++r_) Mk += t[r_];               \
                }                                                                         \
            }                                                                             \
            M_##k = Mk;                                                                   \
        }
#define TT_M_SUB(k)                                                                       \
        if constexpr (k < KT) {                                                           \
            const int m_ = __builtin_amdgcn_sbfe(rbm[k], shm, 1);                         \
            M_##k -= __hiloint2double(thi & m_, tlo & m_);                                \
        }
#define TT_ENSURE_M(upto)                                                                 \
        {                                                                                 \
            if (m_sync < 0) {                                                             \
                TT_EACH_K(TT_M_FORM)                                                      \
                m_sync = 0;                                                               \
            }                                                                             \
            for (int s0 = m_sync; s0 < (upto); s0 += 64) {                                \
                const int n_ = min(64, (upto) - s0);                                      \
                const int r_l = lane < n_ ? ordl[s0 + lane] : 0;                          \
                const double t_l = t[r_l];                                                \
                for (int i = 0; i < n_; ++i) {                                            \
                    const int r_ = __builtin_amdgcn_readlane(r_l, i);                     \
                    const int tlo = __builtin_amdgcn_readlane(__double2loint(t_l), i);    \
                    const int thi = __builtin_amdgcn_readlane(__double2hiint(t_l), i);    \
                    const uint32_t *rbm = rows_lane + (r_ >> 5) * (64 * KS);              \
                    const int shm = r_ & 31;                                              \
                    TT_EACH_K(TT_M_SUB)                                                   \
                }                                                                         \
            }                                                                             \
            m_sync = (upto);                                                              \
        }

        // A class that fell to one outstanding recv: its time goes to P of that recv, and with a
        // positive time it becomes a pointer.
#define TT_PUSH_Q(target)                                                                 \
                qm += 1;                                                                  \
                if constexpr (kFour) { q3 = q2; q2 = q1; }                                \
                q1 = q0;                                                                  \
                q0 = (target);
#define TT_POINTER(k)                                                                     \
            {                                                                             \
                const int l = __builtin_ctzll(nm);                                        \
                nm ^= 1ull << l;                                                          \
                const int sole = __builtin_amdgcn_readlane(sole_##k, l);                  \
                TT_PUSH_Q(sole)                                                           \
            }
#define TT_TO_P(k, hit1, hm)     /* hm: the ballot of hit1 */                            \
        {                                                                                 \
            if (hit1) {                                                                   \
                sole_##k = pk_##k & IDX_MASK;       /* the class is released when this recv is */ \
                atomicAdd(&P[sole_##k], ct_##k);                                          \
            }                                                                             \
            uint64_t nm = (hm) & ctpos_##k;               /* positive class time: a pointer */ \
            if (nm) {                                     /* one, as a rule */            \
                TT_POINTER(k)                                                             \
                while (nm) TT_POINTER(k)                                                  \
            }                                                                             \
        }
        // lanes whose class k has a positive time (wave-uniform masks, fixed for the sample)
#define TT_CTPOS(k) const uint64_t ctpos_##k = (k < KT) ? __ballot(ct_##k > 0.0) : 0ull;
        TT_EACH_K(TT_CTPOS)
#define TT_INIT_P(k)                                                                      \
        if constexpr (k < KT) {                                                           \
            const bool one = pk_##k < 0 && pk_##k >= -CNT1;                               \
            const uint64_t hm1 = __builtin_amdgcn_ballot_w64(one);                        \
            TT_TO_P(k, one, hm1)                                                          \
        }
        TT_EACH_K(TT_INIT_P)

        // ---- d. selection loop ----
        // What a round does once `best` is chosen: record it, and the straight-line
        // incremental update of every class; then, where a class fell to one outstanding recv,
        // that class's time goes to P of that recv.
#define TT_UPDATE(k)                                                                      \
            if constexpr (k < KT) {                                                       \
                mk_##k = __builtin_amdgcn_sbfe(row_##k, best, 1); /* 0 or -1; the bit offset is best mod 32 */ \
                __builtin_assume(mk_##k >= -1 && mk_##k <= 0);                            \
                pk_##k += mk_##k * delta;           /* both fit 24 bits: one multiply-add */ \
                hmax = max(hmax, (uint32_t)(pk_##k & mk_##k));   /* count fell to 1: top 12 bits all set */ \
            }
#define TT_EVENT(k)                                                                       \
            if constexpr (k < KT) {                                                       \
                const bool hit1 = (uint32_t)(pk_##k & mk_##k) >= (uint32_t)-CNT1;         \
                const uint64_t hm_ = __builtin_amdgcn_ballot_w64(hit1);                   \
                if (hm_ != 0ull) TT_TO_P(k, hit1, hm_)                                    \
            }
        // (with many class slots all words of the row are requested before the first is used: one LDS round trip
        // instead of one per read, which is what the compiler schedules by itself)
#define TT_ROW_LOAD(k) uint32_t row_##k = 0; if constexpr (k < KT) { row_##k = rb[k]; }
#define TT_ROW_KEEP(k) if constexpr (k < KT && KT >= 4) { asm volatile("" : "+v"(row_##k)); }
#define TT_APPLY()                                                                        \
            {                                                                             \
                *ord_next++ = best;                     /* every lane writes the same value */ \
                const uint32_t *rb = rows_lane + (best >> 5) * (64 * KS);                 \
                const int delta = CNT1 + (best & IDX_MASK);    /* the mask tells the compiler it fits 24 bits */ \
                uint32_t hmax = 0;                                                        \
                TT_EACH_K(TT_ROW_LOAD)                                                    \
                TT_EACH_K(TT_ROW_KEEP)                                                    \
                TT_EACH_K(TT_UPDATE)                                                      \
                if (__ballot(hmax >= (uint32_t)-CNT1) != 0ull) { TT_EACH_K(TT_EVENT) }    \
                ++step;                                                                   \
            }
#define TT_UNIFORM_Q()                                                                    \
            {                                                                             \
                qm = __builtin_amdgcn_readfirstlane(qm);                                  \
                q0 = __builtin_amdgcn_readfirstlane(q0);                                  \
                q1 = __builtin_amdgcn_readfirstlane(q1);                                  \
                if constexpr (kFour) {                                                    \
                    q2 = __builtin_amdgcn_readfirstlane(q2);                              \
                    q3 = __builtin_amdgcn_readfirstlane(q3);                              \
                }                                                                         \
            }
        // pointers counted afresh from the class registers (after a round that removed an
        // unknown number of them)
#define TT_RECOUNT(k)                                                                     \
            if constexpr (k < KT) {                                                       \
                uint64_t nm = __ballot((uint32_t)pk_##k >= (uint32_t)-CNT1) & ctpos_##k;    \
                while (nm) {                                                              \
                    const int l = __builtin_ctzll(nm);                                    \
                    nm ^= 1ull << l;                                                      \
                    const int sole = __builtin_amdgcn_readlane(sole_##k, l);              \
                    TT_PUSH_Q(sole)                                                       \
                }                                                                         \
            }
        int step = 0;
        TT_UNIFORM_Q()
        while (step < R) {
            // One pointer: its target precedes every recv with P = 0 and is selected; its
            // pointers (all of them) are gone with it.  These rounds form the inner loop; M of the
            // classes is not touched in it.
            while (qm == 1) {
                const int best = q0;
                qm = 0;
                TT_APPLY()
                TT_UNIFORM_Q()
            }
            if (step >= R) break;
            if (qm == 2) {
                if (q0 == q1) { qm = 1; continue; }      // two pointers at one recv: |Q| = 1 as well
                // two pointers at two recvs a < b: Q = {a, b}, and the scan is one comparison:
                // b precedes a when min{P_a, Time(b)} < min{P_b, Time(a)}.  A tie is left to
                // the general path below.
                const int a_ = min(q0, q1), b_ = max(q0, q1);
                const double xa = fmin(P[a_], t[b_]);
                const double ya = fmin(P[b_], t[a_]);
                if (__ballot(xa != ya) != 0ull) {               // (the same in every lane)
                    const int best = __ballot(xa < ya) != 0ull ? b_ : a_;
                    qm = 1; q0 = a_ + b_ - best;
                    TT_APPLY()
                    TT_UNIFORM_Q()
                    continue;
                }
            }
            if (kFour && (qm == 3 || qm == 4)) {
                // Three or four pointers, all of them tracked.  When their targets are distinct, Q is these
                // recvs and the ascending scan is two or three comparisons in straight-line code; those that
                // stay are known, nothing is counted again.  Anything else (two pointers at one recv, a tie in
                // a comparison) is left to the paths below.
                const bool four = qm == 4;
                int m0 = q0, m1 = q1, m2 = q2, m3 = four ? q3 : INT32_MAX;
                { const int lo = min(m0, m1), hi = max(m0, m1); m0 = lo; m1 = hi; }
                { const int lo = min(m2, m3), hi = max(m2, m3); m2 = lo; m3 = hi; }
                { const int lo = min(m0, m2), hi = max(m0, m2); m0 = lo; m2 = hi; }
                { const int lo = min(m1, m3), hi = max(m1, m3); m1 = lo; m3 = hi; }
                { const int lo = min(m1, m2), hi = max(m1, m2); m1 = lo; m2 = hi; }
                if (m0 != m1 && m1 != m2 && m2 != m3) {
                    // Lane 4 i + j (i < j) evaluates the comparator for the members i and j: j precedes i when
                    // min{P_i, Time(j)} < min{P_j, Time(i)}.  Its members come out of two scalars that hold three
                    // members of ten bits each (0, 1, 2 for i; 1, 2, 3 for j; with three members the fourth is a copy
                    // of the third).  The scan then walks over the outcomes in scalar code.
                    const int m3r = four ? m3 : m2;
                    const int pack_i = m0 | m1 << 10 | m2 << 20, pack_j = m1 | m2 << 10 | m3r << 20;
                    const int mi = __builtin_amdgcn_ubfe(pack_i, pair_shift & 31, 10);
                    const int mj = __builtin_amdgcn_ubfe(pack_j, pair_shift >> 8, 10);
                    const double xi = fmin(P[mi], t[mj]), yi = fmin(P[mj], t[mi]);
                    const uint64_t lt = __ballot(xi < yi), eq = __ballot(xi == yi);
                    int bi = (int)(lt >> 1) & 1;                                 // members 0 and 1: lane 1
                    uint64_t looked = 1ull << 1;
                    looked |= 1ull << (4 * bi + 2);
                    if ((lt >> (4 * bi + 2)) & 1) bi = 2;
                    if (four) {
                        looked |= 1ull << (4 * bi + 3);
                        if ((lt >> (4 * bi + 3)) & 1) bi = 3;
                    }
                    if ((eq & looked) == 0ull) {                                // no tie in a comparison that was made
                        const int best = bi == 0 ? m0 : (bi == 1 ? m1 : (bi == 2 ? m2 : m3));
                        // the members that stay, in ascending order
                        qm -= 1;
                        q0 = best == m0 ? m1 : m0;
                        q1 = (best == m0 || best == m1) ? m2 : m1;
                        q2 = best == m3 ? m2 : m3;
                        TT_APPLY()
                        TT_UNIFORM_Q()
                        continue;
                    }
                }
            }
            if (qm >= 2 && q0 == q1 && (!kFour || (q1 == q2 && (qm == 3 || q2 == q3)))) {
                // the latest pointers aim at one recv; with more pointers than tracked targets, look at
                // all of them to be sure
                uint64_t other_target = 0;
                if (qm > (kFour ? 4 : 2)) {
#define TT_SAME(k)                                                                        \
                    if constexpr (k < KT)                                                 \
                        other_target |= __ballot((uint32_t)pk_##k >= (uint32_t)-CNT1 && sole_##k != q0) & ctpos_##k;
                    TT_EACH_K(TT_SAME)
                }
                if (other_target == 0) {
                    // several pointers at one recv: |Q| = 1 as well
                    const int best = q0;
                    qm = 0;
                    TT_APPLY()
                    TT_UNIFORM_Q()
                    continue;
                }
            }
            int best;
            wave_sync();                    // the order so far is in ordl for the paths that read it
            m_sync = __builtin_amdgcn_readfirstlane(m_sync);
            if (qm == 0) {
                // every outstanding recv has P = 0: lowest index among those of minimal M+
                TT_ENSURE_M(step)
                publish_alive(step);
                double lmin = TT_INF;
#define TT_LMIN(k) if constexpr (k < KT) { if (pk_##k >= 0) lmin = fmin(lmin, M_##k); }
                TT_EACH_K(TT_LMIN)
                const double g = wave_min_f64_dpp(lmin);
                int cand = INT32_MAX;
                if (g != TT_INF) {
#define TT_CAND(k) if constexpr (k < KT) { if (pk_##k >= 0 && M_##k == g) cand = min(cand, first_alive<KT>(rows, aliveh, W, lane, k)); }
                    TT_EACH_K(TT_CAND)
                }
                best = wave_min_i32_dpp(cand);            // INT32_MAX when no M+ exists: fixed up below
                if ((unsigned)best >= (unsigned)R) {  // no M+ exists: the lowest outstanding recv
                    for (int h = 2 * W - 1; h >= 0; --h) {
                        const uint32_t x = aliveh[h];
                        if (x) best = h * 32 + __builtin_ctz(x);
                    }
                }
            } else {
                // ascending scan over Q with the comparator
                double mp_best = -1.0;
                best = -1;
                // Q from the pointers: bit j of lane l stands for recv 64 j + l
                uint32_t qbits_l = 0;
#define TT_QBITS(k)                                                                       \
                if constexpr (k < KT) {                                                   \
                    uint64_t nm = __ballot((uint32_t)pk_##k >= (uint32_t)-CNT1) & ctpos_##k; \
                    while (nm) {                                                          \
                        const int l = __builtin_ctzll(nm);                                \
                        nm ^= 1ull << l;                                                  \
                        const int sole = __builtin_amdgcn_readlane(sole_##k, l);          \
                        qbits_l |= (uint32_t)(lane == (sole & 63)) << (sole >> 6);        \
                    }                                                                     \
                }
                TT_EACH_K(TT_QBITS)
                for (int j = 0; j < W; ++j) {
                    uint64_t x = __ballot((qbits_l >> j) & 1u);
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
                            TT_ENSURE_M(step)
                            double v = TT_INF, u = TT_INF;
#define TT_MPLUS(k)                                                                       \
                            if constexpr (k < KT) {                                   \
                                const uint32_t ra = rows[((a >> 5) * 64 + lane) * KS + k] >> (a & 31);       \
                                const uint32_t rb2 = rows[((best >> 5) * 64 + lane) * KS + k] >> (best & 31); \
                                if (pk_##k >= 0 && (ra & 1u)) v = fmin(v, M_##k);     \
                                if (pk_##k >= 0 && (rb2 & 1u)) u = fmin(u, M_##k);    \
                            }
                            TT_EACH_K(TT_MPLUS)
                            mp_a = wave_min_f64_dpp(v);
                            if (mp_best < 0.0) mp_best = wave_min_f64_dpp(u);
                            prec = mp_a < mp_best;
                        }
                        if (prec) { best = a; mp_best = mp_a; }
                    }
                }
            }
            best = __builtin_amdgcn_readfirstlane(best);
            TT_APPLY()
            qm = 0;
            TT_EACH_K(TT_RECOUNT)
            TT_UNIFORM_Q()
        }
        wave_sync();

        // ---- e. outputs ----
        for (int s = lane; s < R; s += 64) {
            const int r = ordl[s];
            p.order[(size_t)b * R + s] = r;
            if (p.rank) p.rank[(size_t)b * R + r] = s;
        }
        if (p.simulate) {
            // A class is released by its last recv, the one it pointed at once its count had fallen
            // to one: kappa = 1-based position of that recv in the order, 0 for a class without recvs.
            int32_t *posl = reinterpret_cast<int32_t *>(P);        // [R] recv -> step (P is free now)
            for (int s = lane; s < R; s += 64) posl[ordl[s]] = s;
            wave_sync();
#define TT_KAPPA(k) const int kap_##k = (k < KT && sole_##k >= 0) ? posl[sole_##k] + 1 : 0;
            TT_EACH_K(TT_KAPPA)
            wave_sync();
            // F_k into P[k - 1]: prefix sums of the transfer times in TAC order
            double fc = 0.0;
            for (int base = 0; base < R; base += 64) {
                const int s = base + lane;
                const double x = s < R ? t[ordl[s]] : 0.0;
                const double inc = wave_incl_scan_f64_dpp(x);
                if (s < R) P[s] = fc + inc;
                fc += lane63_f64(inc);
            }
            const double F = fc;
            wave_sync();
            // A[k] = time of the classes released after k transfers (in the space of t, which is
            // not read any more); makespan = max over k of F_k + (A[k] + ... + A[R]), with F_0 = 0.
            double *A = t;
            for (int j = lane; j <= R; j += 64) A[j] = 0.0;
            wave_sync();
#define TT_RELEASE(k) if constexpr (k < KT) { if (k * 64 + lane < C) atomicAdd(&A[kap_##k], ct_##k); }
            TT_EACH_K(TT_RELEASE)
            wave_sync();
            double ct_sum = 0.0;
#define TT_TOTAL(k) if constexpr (k < KT) { ct_sum += ct_##k; }
            TT_EACH_K(TT_TOTAL)
            const double sum_c = wave_sum_f64_dpp(ct_sum);
            double sfx = 0.0, mloc = sum_c;               // k = 0: F_0 + S_0 = all class time
            for (int base = ((R - 1) / 64) * 64; base >= 0; base -= 64) {
                const int k = base + lane + 1;            // 1 <= k <= R handled here
                const double x = k <= R ? A[k] : 0.0;
                const double inc = wave_incl_scan_f64_dpp(x);
                const double tot = lane63_f64(inc);
                if (k <= R) mloc = fmax(mloc, P[k - 1] + (sfx + (tot - inc + x)));
                sfx += tot;
            }
            const double m = wave_max_f64_dpp(mloc);
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

template <int KT>
static hipError_t launch_reg_k(TacRegParams &p, const Dag &d, hipStream_t s)
{
    // LDS: shared rows + per wave t [R+1], P [R+1], ordl [R] i32, outstanding set [2W] u32
    const size_t rows_doubles = ((size_t)2 * d.W * 64 * row_stride(KT) + 1) / 2;
    const size_t per_wave = 2 * ((size_t)d.R + 1) + ((size_t)d.R + 2 * d.W + 1) / 2 + 1;
    // as many waves as LDS allows, at most reg_waves(KT)
    int waves = reg_waves(KT);
    while (waves > 4 && (rows_doubles + per_wave * waves) * 8 > 150 * 1024) --waves;
    const size_t lds = (rows_doubles + per_wave * waves) * 8;
    if (lds > (waves > 4 ? 150 : 80) * 1024) return hipErrorNotSupported;
    p.wave_doubles = (int32_t)per_wave;
    // the class totals are summed in the space of P, ordl and the outstanding set when that holds
    // one double per class slot
    p.col_cls = (size_t)64 * KT <= (size_t)d.R + 1 + ((size_t)d.R + 2 * d.W) / 2 ? d.d_col_cls : nullptr;
    int per_cu = 0;
    hipError_t e;
    if (lds > 48 * 1024) {
        e = ensure_dynamic_lds(reinterpret_cast<const void *>(tac_reg_kernel<KT>), lds);
        if (e != hipSuccess) return e;
    }
    e = cached_blocks_per_cu(&per_cu, reinterpret_cast<const void *>(tac_reg_kernel<KT>), 64 * waves, lds);
    if (e != hipSuccess) return e;
    if (per_cu < 1) per_cu = 1;
    const int n_cu = device_cu_count(d.device);
    int grid = per_cu * n_cu;                       // one resident set of workgroups, no tail
    const int need = (p.B + waves - 1) / waves;
    if (grid > need) grid = need;
    p.n_waves = grid * waves;
    hipLaunchKernelGGL((tac_reg_kernel<KT>), dim3(grid), dim3(64 * waves), lds, s, p);
    return hipGetLastError();
}

hipError_t launch_tac_reg(Dag &d, const TacArgs &a, int32_t *flags, hipStream_t s)
{
    if (d.R == 0 || d.R > 1024 || d.C > 8 * 64 || a.sel_P || a.sel_Mplus || !d.d_cls_isum || !d.d_run_ptr)
        return hipErrorNotSupported;
    TacRegParams p{};
    p.B = a.B; p.R = d.R; p.W = d.W; p.C = d.C; p.N = d.N;
    p.cls_dep = d.d_cls_dep; p.cls_cnt0 = d.d_cls_cnt0; p.cls_isum = d.d_cls_isum;
    p.cls_ptr = d.d_cls_ptr; p.cls_cols = d.d_cls_cols;
    p.run_ptr = d.d_run_ptr; p.run_lo = d.d_run_lo; p.run_hi = d.d_run_hi;
    p.op_time = a.op_time; p.recv_time = a.recv_time; p.f32 = a.f32 ? 1 : 0;
    p.order = a.order; p.rank = a.rank;
    p.simulate = a.simulate ? 1 : 0;
    p.makespan = a.makespan; p.eff = a.eff; p.U = a.U; p.L = a.L; p.S = a.S;
    p.flags = flags;
    const int K = (d.C + 63) / 64;
    if (K <= 1) return launch_reg_k<1>(p, d, s);
    if (K <= 2) return launch_reg_k<2>(p, d, s);
    if (K <= 3) return launch_reg_k<3>(p, d, s);
    if (K <= 4) return launch_reg_k<4>(p, d, s);
    if (K <= 5) return launch_reg_k<5>(p, d, s);
    if (K <= 6) return launch_reg_k<6>(p, d, s);
    if (K <= 7) return launch_reg_k<7>(p, d, s);
    return launch_reg_k<8>(p, d, s);
}

}  // namespace tictac
