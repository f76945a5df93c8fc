// One iteration with send ops (Sec. 2.2: in the worker's graph the recv ops are roots and the send ops
// leaves), for a batch of timing samples.  Three resources: the channel that serves the recvs back to back
// in the given order (Sec. 5.1), the compute device, and an uplink that carries the sends one at a time,
// first come first served, a send being requested when its last predecessor finishes.
//
// With sends the finish times of single compute ops matter, so the closed form over classes of
// k4_simulate.hip does not apply: the compute device is followed op by op.  It takes, whenever it is
// idle, the ready op of lowest id.  One wavefront per sample:
//   * the downlink needs no events: the k-th transfer ends at F_k, a prefix sum;
//   * the device is a loop over the compute ops in the order in which it runs them.  A step: the lowest set
//     bit of the ready set (a bitmap in LDS, one word per lane and pass), the op's record (successor list,
//     column of its time), finish = start + Time(op); then the transfers that end up to `finish` release
//     their successors, then the op releases its own.  Releasing: one lane per successor decrements its
//     count of unfinished predecessors (LDS, returning atomics); a count that reaches zero sets the ready
//     bit, or, for a send, requests the uplink;
//   * the uplink needs no queue: requests arrive in non-decreasing time (the steps above are taken in
//     time order), and for the requests of one instant only the sum of their times matters, so
//     busy = max(busy, instant) + sum; the last send ends at the final value of busy.
// A step reads from device memory the op's time and its successor list.  Both addresses come with the list entry
// through which the op was released (the lane that released it keeps them), so an op released by the op before it,
// the common case on chains, costs one trip to memory; any other op costs a second one for its record.  The
// per-sample state in LDS is 2 bytes per op plus a bit per op plus 12 bytes per recv.
#include <algorithm>

#include "device_utils.h"
#include "internal.h"

namespace tictac {

struct SendSimParams {
    int32_t B, n, R, N;
    const int4 *rec;                // [n] per op: successors from succ[x] on (-1: none), column of its time (z; -1 recv), w: 1 = send
    const int4 *succ;               // [E + 64] x: successor op id, top bit set on the last of a list; y, z, w: that op's
                                    // column, start of its successors and send flag (as in rec)
    const uint16_t *indeg;          // [n] number of predecessors
    const uint32_t *ready0;         // [ceil(n / 32)] compute ops (not sends) without predecessors
    const int32_t *send0;           // [n_send0] columns of the sends without predecessors (requested at 0)
    int32_t n_send0;
    const uint8_t *col_kind;        // [N] 1 = the column is a send's
    const int32_t *recv_ids;        // [R]
    const int32_t *order;
    int32_t order_stride;
    const double *op_time, *recv_time;
    double *makespan, *eff, *U, *L, *S;
    int32_t wave_bytes, n_waves;
};

__device__ __forceinline__ double uniform(double v)
{
    return __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(v)),
                            __builtin_amdgcn_readfirstlane(__double2loint(v)));
}

__global__ void __launch_bounds__(256)
simulate_sends_kernel(const SendSimParams p)
{
    extern __shared__ double smem[];
    const int n = p.n, R = p.R, N = p.N;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_words = (n + 31) >> 5;
    char *mine = reinterpret_cast<char *>(smem) + (size_t)wave * p.wave_bytes;
    double *F = reinterpret_cast<double *>(mine);                               // [R] end of the k-th transfer
    int32_t *rop = reinterpret_cast<int32_t *>(F + R);                          // [R] where the successors of the k-th recv start
    uint32_t *rdy = reinterpret_cast<uint32_t *>(rop + R);                      // [n_words]
    uint16_t *waiting = reinterpret_cast<uint16_t *>(rdy + n_words);            // [n] (padded to a multiple of two)

    const int gwave = blockIdx.x * (blockDim.x >> 6) + wave;
    for (int b = gwave; b < p.B; b += p.n_waves) {
        const double *ot = p.op_time + (size_t)b * N;
        const double *rt = p.recv_time + (size_t)b * R;
        const int32_t *ord = p.order + (size_t)b * p.order_stride;
        wave_sync();

        // ---- the downlink: ends of the transfers in the given order; sums of the three resources ----
        double fc = 0.0;
        for (int base = 0; base < R; base += 64) {
            const int k = base + lane;
            int r = k < R ? ord[k] : 0;
            const bool ok = k < R && (unsigned)r < (unsigned)R;     // an invalid entry is skipped, never dereferenced
            if (!ok) r = 0;
            const double x = ok ? rt[r] : 0.0;
            const double inc = wave_incl_scan_f64_dpp(x);
            if (k < R) { F[k] = fc + inc; rop[k] = ok ? p.rec[p.recv_ids[r]].x : -1; }
            fc += lane63_f64(inc);
        }
        const double sum_r = fc;
        double sc = 0.0, ss = 0.0;
        for (int j = lane; j < N; j += 64) {
            const double x = ot[j];
            if (p.col_kind[j]) ss += x; else sc += x;
        }
        const double sum_c = wave_sum_f64_dpp(sc), sum_s = wave_sum_f64_dpp(ss);

        // ---- state of the sample ----
        for (int w = lane; w < n_words; w += 64) rdy[w] = p.ready0[w];
        for (int v = lane; v < n; v += 64) waiting[v] = p.indeg[v];
        double up_busy = 0.0, m = 0.0;
        {
            double s0 = 0.0;                                        // sends without predecessors: requested at 0
            for (int i = lane; i < p.n_send0; i += 64) s0 += ot[p.send0[i]];
            s0 = wave_sum_f64_dpp(s0);
            if (p.n_send0 > 0) { up_busy = s0; m = s0; }
        }
        wave_sync();

        // What the lane knows of the op it released last: id, column of its time, start of its successors.
        int held_op = -1, held_col = 0, held_beg = 0;
        // the successors listed from succ[beg] on are released at time `at`
        auto release = [&](int beg, double at) {
            if (beg < 0) return;
            double sent = 0.0;
            bool any_send = false;
            for (int base = beg;; base += 64) {
                const int4 se = p.succ[base + lane];
                const uint64_t ends = __ballot(se.x < 0);
                const int n_here = ends ? __builtin_ctzll(ends) + 1 : 64;   // entries of this list among the 64 read
                if (lane < n_here) {
                    const int s2 = se.x & 0x7fffffff;
                    // (16-bit counters: the atomic works on the 32-bit word that holds the counter)
                    uint32_t *word = reinterpret_cast<uint32_t *>(waiting) + (s2 >> 1);
                    const int sh = (s2 & 1) * 16;
                    const uint32_t old = atomicSub(word, 1u << sh);
                    if (((old >> sh) & 0xffffu) == 1u) {
                        if (se.w) { sent += ot[se.y]; any_send = true; }
                        else {
                            atomicOr(&rdy[s2 >> 5], 1u << (s2 & 31));
                            held_op = s2; held_col = se.y; held_beg = se.z;
                        }
                    }
                }
                if (ends) break;
            }
            if (__ballot(any_send) != 0ull) {
                up_busy = fmax(up_busy, at) + wave_sum_f64_dpp(sent);
                m = fmax(m, up_busy);
            }
        };

        // ---- the compute device, op by op ----
        double t_dev = 0.0;
        int k = 0;                                                  // transfers released so far
        for (;;) {
            wave_sync();
            int v = -1;
            for (int w0 = 0; w0 < n_words; w0 += 64) {
                const uint32_t x = w0 + lane < n_words ? rdy[w0 + lane] : 0u;
                const uint64_t has = __ballot(x != 0u);
                if (has != 0ull) {
                    const int l = __builtin_ctzll(has);
                    const uint32_t xw = (uint32_t)__builtin_amdgcn_readlane((int)x, l);
                    v = ((w0 + l) << 5) + __builtin_ctz(xw);
                    break;
                }
            }
            if (v < 0) {
                if (k >= R) break;                                  // nothing ready and no transfer left
                // the device idles until the next transfer ends
                const double at = uniform(F[k]);
                t_dev = fmax(t_dev, at);
                release(__builtin_amdgcn_readfirstlane(rop[k]), at);
                ++k;
                continue;
            }
            int v_col, v_beg;
            const uint64_t holders = __ballot(held_op == v);
            if (holders) {
                const int l = __builtin_ctzll(holders);
                v_col = __builtin_amdgcn_readlane(held_col, l);
                v_beg = __builtin_amdgcn_readlane(held_beg, l);
            } else {
                const int4 rv = p.rec[v];
                v_col = __builtin_amdgcn_readfirstlane(rv.z);
                v_beg = __builtin_amdgcn_readfirstlane(rv.x);
            }
            const double finish = t_dev + uniform(ot[v_col]);
            if (lane == 0) rdy[v >> 5] &= ~(1u << (v & 31));
            // transfers that end while the op runs release their successors first (requests to the uplink
            // are served in the order of their instants)
            while (k < R && uniform(F[k]) <= finish) {
                release(__builtin_amdgcn_readfirstlane(rop[k]), uniform(F[k]));
                ++k;
            }
            release(v_beg, finish);
            t_dev = finish;
            m = fmax(m, finish);
        }
        if (R > 0) m = fmax(m, uniform(F[R - 1]));

        if (lane == 0) {
            const double U = sum_c + sum_r + sum_s;
            const double L = fmax(fmax(sum_c, sum_r), sum_s);
            p.makespan[b] = m;
            p.eff[b] = (U == L) ? 1.0 : (U - m) / (U - L);
            if (p.U) p.U[b] = U;
            if (p.L) p.L[b] = L;
            if (p.S) p.S[b] = (U == L || L == 0.0) ? 0.0 : (U - L) / L;
        }
    }
}

hipError_t launch_simulate_sends(Dag &d, const SimArgs &a, hipStream_t s)
{
    if (a.B == 0) return hipSuccess;
    if (!d.d_send_rec || d.n > 65535 * 2) return hipErrorNotSupported;
    SendSimParams p{};
    p.B = a.B; p.n = d.n; p.R = d.R; p.N = d.N;
    p.rec = d.d_send_rec; p.succ = d.d_send_succ; p.indeg = d.d_send_indeg; p.ready0 = d.d_send_ready0;
    p.send0 = d.d_send_free; p.n_send0 = d.n_send_free; p.col_kind = d.d_send_col_kind;
    p.recv_ids = d.d_send_recv_ids;
    p.order = a.order; p.order_stride = a.order_stride;
    p.op_time = static_cast<const double *>(a.op_time); p.recv_time = static_cast<const double *>(a.recv_time);
    p.makespan = a.makespan; p.eff = a.eff; p.U = a.U; p.L = a.L; p.S = a.S;
    const size_t n_words = ((size_t)d.n + 31) / 32;
    size_t per_wave = (size_t)d.R * 12 + n_words * 4 + (((size_t)d.n + 1) & ~(size_t)1) * 2;
    per_wave = (per_wave + 15) & ~(size_t)15;
    int waves = 4;
    while (waves > 1 && per_wave * waves > 150 * 1024) --waves;
    if (per_wave * waves > 150 * 1024) return hipErrorNotSupported;
    const size_t lds = per_wave * waves;
    p.wave_bytes = (int32_t)per_wave;
    if (lds > 48 * 1024) {
        const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(simulate_sends_kernel), lds);
        if (e != hipSuccess) return e;
    }
    int per_cu = 0;
    hipError_t e = cached_blocks_per_cu(&per_cu, reinterpret_cast<const void *>(simulate_sends_kernel), 64 * waves, lds);
    if (e != hipSuccess) return e;
    if (per_cu < 1) per_cu = 1;
    int grid = per_cu * device_cu_count(d.device);
    const int need = (a.B + waves - 1) / waves;
    if (grid > need) grid = need;
    p.n_waves = grid * waves;
    hipLaunchKernelGGL(simulate_sends_kernel, dim3(grid), dim3(64 * waves), lds, s, p);
    return hipGetLastError();
}

}  // namespace tictac
