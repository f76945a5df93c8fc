// Order search with the simulated iteration as its measure.  Finding the best transfer order is
// a job-shop problem and NP-hard (Sec. 3.1), and the comparator of TAC extends a two-recv rule by
// an induction that need not hold in general (Sec. 4.3); climbing from a heuristic order through
// proposed exchanges shows how far it is from a better one.
//
// Per timing sample:  cur = start order, m_cur = makespan(cur); for every move (a, b) in the
// order given: exchange positions a and b of cur, m = makespan of that order; keep the exchange
// when m < m_cur, else undo it.  A move with a == b or a position outside 0 .. R-1 is skipped.
//
// The makespan of an order is the one of the single-channel simulation: F_k = end of the k-th
// transfer (prefix sums over the order), kappa of a class = last position among the recvs of its
// row, A_k = class time released by transfer k, makespan = max_k (F_k + sum_{k' >= k} A_k').
//
// One wave per sample.  The op_time row is read once (class totals); after that a move touches
// registers and LDS only.  Lane l owns classes l, l + 64, ... (their totals and kappa) and the
// positions l, l + 64, ... of the order (the transfer time at that position).  A move changes
// kappa of few classes: when the recv at the earlier position (x) and the one at the later
// position (y) change places, a class with x in its row gets max(kappa, later position); a class
// with y and without x whose kappa was y's position needs its maximum taken again, which the whole
// wave does over the row (one recv per lane and word); every other class keeps its kappa.  A and
// the two scans are then formed afresh from the registers, so every makespan is the one a full
// evaluation of that order gives.
//
// Most moves are turned down without that evaluation.  Let k* be a position where the current
// makespan is attained, m_cur = F_k* + S_k* (S_k = class time with kappa >= k).  The makespan after
// the move is at least F'_k* + S'_k*.  Exchanging positions lo < hi leaves F_k and S_k as they are
// for k <= lo and for k > hi + 1, so a move with k* outside lo + 1 .. hi + 1 cannot help (decided
// for 64 moves at a time, one per lane).  Otherwise F_k* changes by Time(y) - Time(x) when k* <= hi, S_k* gains the
// classes with x whose kappa was below k* and loses at most the classes that need their maximum
// taken again; when that sum is not negative the move cannot help either (one wave sum, no LDS
// write).  Only the remaining moves are evaluated.
#include "device_utils.h"
#include "internal.h"

namespace tictac {

struct SearchParams {
    int32_t B, R, C, N, W, n_waves, wave_bytes, levels, n_moves, fa_len, rows_bytes;
    const int32_t *col_cls;     // [N] class of every op_time column
    const uint64_t *cls_dep;    // [C][W] class rows
    const int32_t *run_ptr;     // [C+1] runs [run_lo, run_hi) of consecutive recv indices of the class rows
    const int32_t *run_lo, *run_hi;
    const int32_t *order;       // start orders
    int32_t order_stride;
    const int32_t *moves;       // [n_moves][2]
    const double *op_time, *recv_time;
    int32_t *best_order;        // [B][R]
    double *best_makespan;      // [B]
    double *start_makespan;     // [B] or NULL
    int32_t *n_accepted;        // [B] or NULL
};

constexpr int kSearchWaves = 4;

#define OS_EACH(F) F(0) F(1) F(2) F(3) F(4) F(5) F(6) F(7)

// T slots per lane, for classes (64 T >= C) and for positions (64 T >= R)
template <int T>
__global__ void __launch_bounds__(64 * kSearchWaves)
order_search_kernel(const SearchParams p)
{
    extern __shared__ double smem[];
    const int R = p.R, C = p.C, N = p.N, W = p.W;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t *rows = reinterpret_cast<const uint64_t *>(smem);          // [C][W], shared by the waves
    char *mine = reinterpret_cast<char *>(smem) + p.rows_bytes + (size_t)wave * p.wave_bytes;
    double *t = reinterpret_cast<double *>(mine);           // [R]   Time(recv)
    double *A = t + R;                                      // [R+1] class time by kappa
    double *csum = t;                                       // [64 T] class totals while they are summed (fa_len doubles from t on)
    uint16_t *ordl = reinterpret_cast<uint16_t *>(t + p.fa_len);     // [R] the order being tried
    uint16_t *pos = ordl + R + (R & 1);                     // [levels][R] level 0: 1-based position of every recv;
                                                            // level j: maxima over [i, min(i + 2^j, R)) (start order only)
    {
        uint64_t *rw = reinterpret_cast<uint64_t *>(smem);
        for (int i = threadIdx.x; i < C * W; i += blockDim.x) rw[i] = p.cls_dep[i];
    }
    __syncthreads();

    const int gwave = blockIdx.x * kSearchWaves + wave;
    for (int b = gwave; b < p.B; b += p.n_waves) {
        const double *rt = p.recv_time + (size_t)b * R;
        const double *ot = p.op_time + (size_t)b * N;
        const int32_t *ord = p.order + (size_t)b * p.order_stride;
        wave_sync();                        // LDS of the previous sample is no longer read

        // ---- class totals ----
        for (int c = lane; c < 64 * T; c += 64) csum[c] = 0.0;
        wave_sync();
        class_totals(csum, ot, p.col_cls, N, lane);
        wave_sync();
#define OS_DECL(k) double ct_##k = 0.0, xs_##k = 0.0; int kap_##k = 0, kn_##k = 0;
        OS_EACH(OS_DECL)
#define OS_TOTAL(k) if constexpr (k < T) { ct_##k = csum[k * 64 + lane]; }
        OS_EACH(OS_TOTAL)
        double ct_sum = 0.0;
#define OS_SUM(k) if constexpr (k < T) { ct_sum += ct_##k; }
        OS_EACH(OS_SUM)
        const double sum_c = wave_sum_f64_dpp(ct_sum);
        wave_sync();

        // ---- transfer times, start order, positions ----
        for (int r = lane; r < R; r += 64) {
            t[r] = rt[r];
            pos[r] = 0;
            const int o = ord[r];
            ordl[r] = (uint16_t)((unsigned)o < (unsigned)R ? o : 0);     // an invalid entry is never used as an index
        }
        wave_sync();
#define OS_PLACE(k)                                                                       \
        if constexpr (k < T) {                                                            \
            const int s = k * 64 + lane;                                                  \
            if (s < R) {                                                                  \
                const int r = ordl[s];                                                    \
                pos[r] = (uint16_t)(s + 1);                                               \
                xs_##k = t[r];                                                            \
            }                                                                             \
        }
        OS_EACH(OS_PLACE)
        wave_sync();

        // ---- kappa of the start order: range maxima over the runs of every class row ----
        for (int j = 1; j < p.levels; ++j) {
            const uint16_t *prev = pos + (size_t)(j - 1) * R;
            uint16_t *cur = pos + (size_t)j * R;
            const int h = 1 << (j - 1);
            for (int i = lane; i < R; i += 64) cur[i] = max(prev[i], prev[min(i + h, R - 1)]);
            wave_sync();
        }
#define OS_KAPPA0(k)                                                                      \
        if constexpr (k < T) {                                                            \
            const int c = k * 64 + lane;                                                  \
            if (c < C) {                                                                  \
                const int rend = p.run_ptr[c + 1];                                        \
                int m = 0;                                                                \
                for (int q = p.run_ptr[c]; q < rend; ++q) {                               \
                    const int lo = p.run_lo[q], hi = p.run_hi[q];                         \
                    const int j = 31 - __builtin_clz(hi - lo);                            \
                    const uint16_t *lv = pos + (size_t)j * R;                             \
                    m = max(m, max((int)lv[lo], (int)lv[hi - (1 << j)]));                 \
                }                                                                         \
                kn_##k = m;                                                               \
            }                                                                             \
        }
        OS_EACH(OS_KAPPA0)

        double m_cur = 0.0;
        int n_acc = 0;
        int kstar = 0;                      // a position where the current makespan is attained
        // 64 moves at a time, one per lane: the moves that k* rules out are dropped by one ballot
        int base = -64;                     // first move of the chunk in mv_lo / mv_hi
        int mv_lo = 0, mv_hi = -1;          // lane i: the positions of move base + i; mv_hi < 0: not an exchange
        unsigned long long todo = 0;        // moves of the chunk that are still to be looked at
        bool first = true;                  // the start order is evaluated before any move
        for (;;) {
            int lo = 0, hi = 0, x = 0, y = 0, cur = 0;
            if (!first) {
                while (todo == 0) {
                    base += 64;
                    if (base >= p.n_moves) break;
                    const int i = base + lane;
                    const int pa = i < p.n_moves ? p.moves[2 * i] : -1;
                    const int pb = i < p.n_moves ? p.moves[2 * i + 1] : -1;
                    const bool ok = (unsigned)pa < (unsigned)R && (unsigned)pb < (unsigned)R && pa != pb;
                    mv_lo = min(pa, pb);
                    mv_hi = ok ? max(pa, pb) : -1;
                    todo = __ballot(mv_hi >= 0 && kstar > mv_lo && kstar <= mv_hi + 1);
                }
                if (todo == 0) break;       // no move left
                cur = __builtin_ctzll(todo);
                todo &= todo - 1;
                lo = __builtin_amdgcn_readlane(mv_lo, cur);
                hi = __builtin_amdgcn_readlane(mv_hi, cur);
                x = __builtin_amdgcn_readfirstlane((int)ordl[lo]);      // moves from lo to hi
                y = __builtin_amdgcn_readfirstlane((int)ordl[hi]);      // moves from hi to lo
                const double tx = t[x], ty = t[y];
                // which classes hold x, which hold y
                const int wx = x >> 6, wy = y >> 6;
                const uint64_t bx = (uint64_t)1 << (x & 63), by = (uint64_t)1 << (y & 63);
                double dsum = 0.0;          // change of S at k*: classes gained, classes that may be lost
                bool moved = false;
#define OS_MEMBER(k)                                                                      \
                bool redo_##k = false;                                                    \
                if constexpr (k < T) {                                                    \
                    kn_##k = kap_##k;                                                     \
                    const int c = k * 64 + lane;                                          \
                    if (c < C) {                                                          \
                        const bool has_x = (rows[(size_t)c * W + wx] & bx) != 0;          \
                        const bool has_y = (rows[(size_t)c * W + wy] & by) != 0;          \
                        if (has_x) kn_##k = max(kap_##k, hi + 1);                         \
                        redo_##k = has_y && !has_x && kap_##k == hi + 1;                  \
                        if (has_x && kap_##k < kstar) { dsum += ct_##k; moved = true; }   \
                        if (redo_##k) { dsum -= ct_##k; moved = true; }                   \
                    }                                                                     \
                }
                OS_EACH(OS_MEMBER)
                double d = kstar <= hi ? ty - tx : 0.0;
                if (__ballot(moved)) d += wave_sum_f64_dpp(dsum);
                // (the comparison is the same in every lane; taking it from the first one tells the compiler so)
                if (__builtin_amdgcn_readfirstlane((int)(d >= 0.0))) continue;     // F'_k* + S'_k* >= m_cur: the move cannot help
                wave_sync();
                if (lane == 0) {
                    ordl[lo] = (uint16_t)y; ordl[hi] = (uint16_t)x;
                    pos[x] = (uint16_t)(hi + 1); pos[y] = (uint16_t)(lo + 1);
                }
                wave_sync();
                // classes that lose their last recv: the maximum over the row again, by the whole wave
#define OS_REDO(k)                                                                        \
                if constexpr (k < T) {                                                    \
                    unsigned long long todo = __ballot(redo_##k);                         \
                    while (todo) {                                                        \
                        const int l = __builtin_ctzll(todo);                              \
                        todo &= todo - 1;                                                 \
                        const uint64_t *row = rows + (size_t)(k * 64 + l) * W;            \
                        int v = 0;                                                        \
                        for (int w = 0; w < W; ++w)                                       \
                            if ((row[w] >> lane) & 1) v = max(v, (int)pos[w * 64 + lane]);\
                        v = wave_max_i32_dpp(v);                                          \
                        if (lane == l) kn_##k = v;                                        \
                    }                                                                     \
                }
                OS_EACH(OS_REDO)
                // the transfer times at the two positions change places
#define OS_SWAP_X(k, to_lo, to_hi)                                                        \
                if constexpr (k < T) {                                                    \
                    if (k * 64 + lane == lo) xs_##k = to_lo;                              \
                    if (k * 64 + lane == hi) xs_##k = to_hi;                              \
                }
#define OS_SWAP_FWD(k) OS_SWAP_X(k, ty, tx)
                OS_EACH(OS_SWAP_FWD)
            }

            // ---- A by kappa; F; suffix sums of A; makespan ----
            for (int j = lane; j <= R; j += 64) A[j] = 0.0;
            wave_sync();
#define OS_RELEASE(k) if constexpr (k < T) { if (k * 64 + lane < C) atomicAdd(&A[kn_##k], ct_##k); }
            OS_EACH(OS_RELEASE)
            double fc = 0.0;
#define OS_F(k)                                                                           \
            double F_##k = 0.0;                                                           \
            if constexpr (k < T) {                                                        \
                if (k * 64 < R) {                                                         \
                    const double inc = wave_incl_scan_f64_dpp(xs_##k);                    \
                    F_##k = fc + inc;                                                     \
                    fc += lane63_f64(inc);                                                \
                }                                                                         \
            }
            OS_EACH(OS_F)
            wave_sync();
            double sfx = 0.0, mloc = sum_c;                   // k = 0: F_0 + S_0 = all class time
            int kb = 0;                                       // where this lane's maximum is attained
#define OS_SUFFIX(kk)                                                                     \
            if constexpr (7 - kk < T) {                                                   \
                constexpr int j = 7 - kk;                                                 \
                if (j * 64 < R) {                                                         \
                    const int k = j * 64 + lane + 1;          /* 1 <= k <= R handled here */ \
                    const double a = k <= R ? A[k] : 0.0;                                 \
                    const double inc = wave_incl_scan_f64_dpp(a);                         \
                    const double tot = lane63_f64(inc);                                   \
                    const double cand = OS_F_OF(j) + (sfx + (tot - inc + a));             \
                    if (k <= R && cand > mloc) { mloc = cand; kb = k; }                   \
                    sfx += tot;                                                           \
                }                                                                         \
            }
#define OS_F_OF(j) (j == 0 ? F_0 : j == 1 ? F_1 : j == 2 ? F_2 : j == 3 ? F_3 : j == 4 ? F_4 : j == 5 ? F_5 : j == 6 ? F_6 : F_7)
            OS_EACH(OS_SUFFIX)
            const double m = wave_max_f64_dpp(mloc);

#define OS_KEEP(k) if constexpr (k < T) { kap_##k = kn_##k; }
            if (first || __builtin_amdgcn_readfirstlane((int)(m < m_cur))) {
                m_cur = m;
                const unsigned long long at = __ballot(mloc == m);
                kstar = at ? __builtin_amdgcn_readlane(kb, __builtin_ctzll(at)) : 0;
                OS_EACH(OS_KEEP)
                if (first) {
                    if (lane == 0 && p.start_makespan) p.start_makespan[b] = m;
                    first = false;
                } else {
                    ++n_acc;
                    // the moves after this one, under the new k*
                    const unsigned long long later = cur == 63 ? 0ull : ~0ull << (cur + 1);
                    todo = __ballot(mv_hi >= 0 && kstar > mv_lo && kstar <= mv_hi + 1) & later;
                }
            } else {
                const double tx = t[x], ty = t[y];
#define OS_SWAP_BACK(k) OS_SWAP_X(k, tx, ty)
                OS_EACH(OS_SWAP_BACK)
                wave_sync();
                if (lane == 0) {
                    ordl[lo] = (uint16_t)x; ordl[hi] = (uint16_t)y;
                    pos[x] = (uint16_t)(lo + 1); pos[y] = (uint16_t)(hi + 1);
                }
                wave_sync();
            }
        }

        for (int s = lane; s < R; s += 64) p.best_order[(size_t)b * R + s] = ordl[s];
        if (lane == 0) {
            p.best_makespan[b] = m_cur;
            if (p.n_accepted) p.n_accepted[b] = n_acc;
        }
    }
}

template <int T>
static hipError_t launch_search_t(SearchParams &p, const Dag &d, hipStream_t s)
{
    int levels = 1;
    while ((1 << levels) <= d.R) ++levels;            // floor(log2 R) + 1 levels of the table
    p.levels = levels;
    const size_t fa = (size_t)2 * d.R + 1 > (size_t)64 * T ? (size_t)2 * d.R + 1 : (size_t)64 * T;
    p.fa_len = (int32_t)fa;
    size_t wave_bytes = fa * 8 + ((size_t)d.R + (d.R & 1)) * 2 + (size_t)levels * d.R * 2;
    wave_bytes = (wave_bytes + 15) & ~(size_t)15;
    const size_t rows_bytes = (((size_t)d.C * d.W * 8) + 15) & ~(size_t)15;
    const size_t lds = rows_bytes + wave_bytes * kSearchWaves;
    if (lds > 150 * 1024) return hipErrorNotSupported;     // 160 KB of LDS per compute unit
    p.wave_bytes = (int32_t)wave_bytes;
    p.rows_bytes = (int32_t)rows_bytes;
    hipError_t e;
    if (lds > 48 * 1024) {
        e = ensure_dynamic_lds(reinterpret_cast<const void *>(order_search_kernel<T>), lds);
        if (e != hipSuccess) return e;
    }
    int per_cu = 0;
    e = cached_blocks_per_cu(&per_cu, reinterpret_cast<const void *>(order_search_kernel<T>), 64 * kSearchWaves, lds);
    if (e != hipSuccess) return e;
    if (per_cu < 1) per_cu = 1;
    const int n_cu = device_cu_count(d.device);
    int grid = per_cu * n_cu;
    const int need = (p.B + kSearchWaves - 1) / kSearchWaves;
    if (grid > need) grid = need;
    p.n_waves = grid * kSearchWaves;
    hipLaunchKernelGGL((order_search_kernel<T>), dim3(grid), dim3(64 * kSearchWaves), lds, s, p);
    return hipGetLastError();
}

hipError_t launch_order_search(Dag &d, const SearchArgs &a, hipStream_t s)
{
    const int KC = (d.C + 63) / 64, KR = (d.R + 63) / 64;
    const int K = KC > KR ? KC : KR;
    if (d.R == 0 || d.R > 512 || d.C == 0 || K > 8 || !d.d_col_cls || !d.d_cls_dep || !d.d_run_ptr) return hipErrorNotSupported;
    SearchParams p{};
    p.B = a.B; p.R = d.R; p.C = d.C; p.N = d.N; p.W = d.W; p.n_moves = a.n_moves;
    p.col_cls = d.d_col_cls; p.cls_dep = d.d_cls_dep;
    p.run_ptr = d.d_run_ptr; p.run_lo = d.d_run_lo; p.run_hi = d.d_run_hi;
    p.order = a.order; p.order_stride = a.order_stride; p.moves = a.moves;
    p.op_time = a.op_time; p.recv_time = a.recv_time;
    p.best_order = a.best_order; p.best_makespan = a.best_makespan;
    p.start_makespan = a.start_makespan; p.n_accepted = a.n_accepted;
    if (K <= 1) return launch_search_t<1>(p, d, s);
    if (K <= 2) return launch_search_t<2>(p, d, s);
    if (K <= 3) return launch_search_t<3>(p, d, s);
    if (K <= 4) return launch_search_t<4>(p, d, s);
    if (K <= 5) return launch_search_t<5>(p, d, s);
    if (K <= 6) return launch_search_t<6>(p, d, s);
    if (K <= 7) return launch_search_t<7>(p, d, s);
    return launch_search_t<8>(p, d, s);
}

}  // namespace tictac
