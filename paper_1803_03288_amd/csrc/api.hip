// C ABI of libtictac: argument checks, graph validation and levelling, grouping of
// compute ops into classes of identical dependency sets, and the calls into the
// kernel launchers.  All arithmetic of the method runs in the kernels.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <numeric>
#include <unordered_map>

#include "internal.h"

namespace tictac {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

#define HIP_TRY(expr)                                                                        \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess) {                                                              \
            set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return TICTAC_ERR_HIP;                                                           \
        }                                                                                    \
    } while (0)

// Pinned host memory for the transfers of tictac_build_deps: one block per calling thread,
// grown on demand and kept until the thread's next larger request (pinning costs milliseconds,
// and copies from or to pageable memory are staged by the runtime and take three to four
// times as long).  NULL when the request is empty, beyond the cap, or cannot be pinned: the
// caller then copies from or to its own pageable memory.  The block is free again once the
// stream has been synchronised, which tictac_build_deps does before it returns.
static thread_local void *g_stage = nullptr;
static thread_local size_t g_stage_bytes = 0;
constexpr size_t kStageMax = (size_t)96 << 20;

static void *stage(size_t bytes)
{
    if (bytes == 0 || bytes > kStageMax) return nullptr;
    if (bytes <= g_stage_bytes) return g_stage;
    if (g_stage) {
        (void)hipHostFree(g_stage);
        g_stage = nullptr;
        g_stage_bytes = 0;
    }
    const size_t want = (bytes + ((size_t)1 << 20) - 1) & ~(((size_t)1 << 20) - 1);
    void *q = nullptr;
    if (hipHostMalloc(&q, want, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_stage = q;
    g_stage_bytes = want;
    return q;
}

// Collects host arrays (and device-only reservations) into one device block: one
// allocation and one host-to-device copy instead of one of each per array.
struct Packer {
    std::vector<char> host;
    struct Fix { void **dst; size_t off; };
    std::vector<Fix> fixes;
    size_t device_only = 0;

    static size_t align(size_t x) { return (x + 255) & ~(size_t)255; }

    template <typename T>
    void add(T **dst, const std::vector<T> &src)
    {
        *dst = nullptr;
        if (src.empty()) return;
        const size_t off = align(host.size());
        host.resize(off + src.size() * sizeof(T));
        memcpy(host.data() + off, src.data(), src.size() * sizeof(T));
        fixes.push_back({reinterpret_cast<void **>(dst), off});
    }
    // space after the copied part that only kernels write; call after the last add()
    template <typename T>
    void reserve(T **dst, size_t bytes)
    {
        *dst = nullptr;
        if (!bytes) return;
        fixes.push_back({reinterpret_cast<void **>(dst), align(host.size()) + device_only});
        device_only += align(bytes);
    }
    hipError_t commit(void **block, hipStream_t s)
    {
        *block = nullptr;
        const size_t total = align(host.size()) + device_only;
        if (!total) return hipSuccess;
        hipError_t e = hipMalloc(block, total);
        if (e != hipSuccess) return e;
        for (const Fix &f : fixes) *f.dst = static_cast<char *>(*block) + f.off;
        if (host.empty()) return hipSuccess;
        const void *src = host.data();
        if (void *st = stage(host.size())) {
            memcpy(st, host.data(), host.size());
            src = st;
        }
        return hipMemcpyAsync(*block, src, host.size(), hipMemcpyHostToDevice, s);
    }
};

int device_cu_count(int device)
{
    static thread_local int known_device = -1, known_count = 0;
    if (device == known_device) return known_count;
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        n = 256;
    }
    known_device = device;
    known_count = n;
    return n;
}

hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes)
{
    // (one table for the process: the attribute belongs to the kernel on a device, not to a thread)
    struct Entry { int device; const void *kernel; size_t bytes; };
    static std::vector<Entry> known;
    static std::mutex mutex;
    int device = 0;
    hipError_t err = hipGetDevice(&device);
    if (err != hipSuccess) return err;
    std::lock_guard<std::mutex> lock(mutex);
    for (Entry &e : known)
        if (e.kernel == kernel && e.device == device) {
            if (bytes <= e.bytes) return hipSuccess;
            err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (err == hipSuccess) e.bytes = bytes;
            return err;
        }
    err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (err == hipSuccess) known.push_back({device, kernel, bytes});
    return err;
}

hipError_t cached_blocks_per_cu(int *per_cu, const void *kernel, int threads, size_t lds)
{
    struct Entry { const void *kernel; int threads; size_t lds; int per_cu; };
    static thread_local std::vector<Entry> known;
    for (const Entry &e : known)
        if (e.kernel == kernel && e.threads == threads && e.lds == lds) { *per_cu = e.per_cu; return hipSuccess; }
    int n = 0;
    const hipError_t err = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, threads, lds);
    if (err != hipSuccess) return err;
    if (n < 1) n = 1;
    if (known.size() < 256) known.push_back({kernel, threads, lds, n});
    *per_cu = n;
    return hipSuccess;
}

hipError_t ensure_workspace(Dag *d, size_t bytes)
{
    if (bytes <= d->work_bytes) return hipSuccess;
    if (d->d_work) {
        hipError_t e = hipFree(d->d_work);   // synchronises: earlier users of the old block are done
        d->d_work = nullptr;
        d->work_bytes = 0;
        if (e != hipSuccess) return e;
    }
    size_t want = bytes + bytes / 8;
    hipError_t e = hipMalloc(&d->d_work, want);
    if (e != hipSuccess) return e;
    d->work_bytes = want;
    return hipSuccess;
}

// Device copy of a channel table [R].  A table equal to the one already there is not sent
// again; a new one is copied synchronously after the work queued on the stream (which may
// still read the old table) has finished.
static hipError_t ensure_chan_table(Dag *d, const int32_t *chan, hipStream_t s)
{
    const size_t bytes = (size_t)d->R * sizeof(int32_t);
    if (d->d_chan && d->h_chan.size() == (size_t)d->R && memcmp(d->h_chan.data(), chan, bytes) == 0)
        return hipSuccess;
    hipError_t e;
    if (!d->d_chan) {
        e = hipMalloc((void **)&d->d_chan, bytes);
        if (e != hipSuccess) return e;
    }
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return e;
    d->h_chan.clear();
    e = hipMemcpy(d->d_chan, chan, bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) return e;
    d->h_chan.assign(chan, chan + d->R);
    return hipSuccess;
}

static void free_dag(Dag *d)
{
    if (!d) return;
    void *ptrs[] = {d->d_graph_block, d->d_class_block, d->d_work, d->d_chan, d->d_send_block};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    delete d;
}

// Groups the compute ops by identical dependency rows.  `rows` holds the rows of the
// compute ops in op_time column order.  Classes are numbered by their first member;
// a class with more than `max_members` ops is split into consecutive pieces (the
// pieces have the same row, which every kernel handles like distinct classes).
static void group_classes(const std::vector<uint64_t> &rows, int32_t N, int32_t W, int32_t max_members,
                          std::vector<uint64_t> &cls_dep, std::vector<int32_t> &cls_ptr,
                          std::vector<int32_t> &cls_cols, int32_t &n_distinct)
{
    // open-addressing table from row hash to the distinct row's number; scanning the ops in
    // ascending order numbers the distinct rows by first member and keeps members ascending
    size_t cap = 16;
    while (cap < (size_t)N * 2) cap <<= 1;
    std::vector<int32_t> slot(cap, -1);
    std::vector<int32_t> first;                 // first member of every distinct row
    std::vector<int32_t> cls_of(N), count;
    for (int32_t j = 0; j < N; ++j) {
        uint64_t h = 0x9E3779B97F4A7C15ull;
        for (int32_t w = 0; w < W; ++w) {
            h ^= rows[(size_t)j * W + w] + 0x9E3779B97F4A7C15ull + (h << 6) + (h >> 2);
            h *= 0xFF51AFD7ED558CCDull;
        }
        size_t q = (h ^ (h >> 29)) & (cap - 1);
        for (;;) {
            const int32_t c = slot[q];
            if (c < 0) {
                slot[q] = (int32_t)first.size();
                cls_of[j] = (int32_t)first.size();
                first.push_back(j);
                count.push_back(1);
                break;
            }
            if (W == 0 || memcmp(&rows[(size_t)first[c] * W], &rows[(size_t)j * W], (size_t)W * 8) == 0) {
                cls_of[j] = c;
                ++count[c];
                break;
            }
            q = (q + 1) & (cap - 1);
        }
    }
    n_distinct = (int32_t)first.size();
    // members of every distinct row, ascending (counting sort by row number)
    std::vector<int32_t> start(n_distinct + 1, 0);
    for (int32_t c = 0; c < n_distinct; ++c) start[c + 1] = start[c] + count[c];
    std::vector<int32_t> members(N), fill(start.begin(), start.end() - 1);
    for (int32_t j = 0; j < N; ++j) members[fill[cls_of[j]]++] = j;
    cls_dep.clear(); cls_ptr.clear(); cls_cols.clear();
    cls_ptr.push_back(0);
    for (int32_t c = 0; c < n_distinct; ++c)
        for (int32_t k = start[c]; k < start[c + 1]; k += max_members) {
            const int32_t e = std::min(start[c + 1], k + max_members);
            for (int32_t m = k; m < e; ++m) cls_cols.push_back(members[m]);
            cls_ptr.push_back((int32_t)cls_cols.size());
            for (int32_t w = 0; w < W; ++w) cls_dep.push_back(rows[(size_t)first[c] * W + w]);
        }
}

// The same grouping from per-op digests (int32[8] per op: a 128-bit hash of the row in the first four words, the
// number of set bits in the fifth): ops with equal digests form a class.  first_col: the first member of every
// class (piece), whose row is the row of the class.
static void group_digests(const int32_t *digest, int32_t N, int32_t max_members, std::vector<int32_t> &cls_ptr,
                          std::vector<int32_t> &cls_cols, std::vector<int32_t> &first_col, int32_t &n_distinct)
{
    size_t cap = 16;
    while (cap < (size_t)N * 2) cap <<= 1;
    std::vector<int32_t> slot(cap, -1), first, cls_of(N), count;
    for (int32_t j = 0; j < N; ++j) {
        const int32_t *g = digest + (size_t)j * 8;
        size_t q = ((uint32_t)g[0] ^ ((size_t)(uint32_t)g[1] << 17) ^ ((size_t)(uint32_t)g[3] << 33)) & (cap - 1);
        for (;;) {
            const int32_t c = slot[q];
            if (c < 0) {
                slot[q] = (int32_t)first.size();
                cls_of[j] = (int32_t)first.size();
                first.push_back(j);
                count.push_back(1);
                break;
            }
            if (memcmp(digest + (size_t)first[c] * 8, g, 5 * sizeof(int32_t)) == 0) {
                cls_of[j] = c;
                ++count[c];
                break;
            }
            q = (q + 1) & (cap - 1);
        }
    }
    n_distinct = (int32_t)first.size();
    std::vector<int32_t> start(n_distinct + 1, 0);
    for (int32_t c = 0; c < n_distinct; ++c) start[c + 1] = start[c] + count[c];
    std::vector<int32_t> members(N), fill(start.begin(), start.end() - 1);
    for (int32_t j = 0; j < N; ++j) members[fill[cls_of[j]]++] = j;
    cls_ptr.assign(1, 0); cls_cols.clear(); first_col.clear();
    for (int32_t c = 0; c < n_distinct; ++c)
        for (int32_t k = start[c]; k < start[c + 1]; k += max_members) {
            const int32_t e = std::min(start[c + 1], k + max_members);
            for (int32_t m = k; m < e; ++m) cls_cols.push_back(members[m]);
            cls_ptr.push_back((int32_t)cls_cols.size());
            first_col.push_back(first[c]);
        }
}

static int build(int32_t n, const int32_t *row_ptr, const int32_t *col_idx, int32_t R, const int32_t *recv_ids,
                 hipStream_t s, Dag *d)
{
    // ---- validation (host) ----
    if (n < 0 || R < 0 || R > n) { set_error("bad sizes: n_ops=%d n_recv=%d", n, R); return TICTAC_ERR_BAD_CSR; }
    if (!row_ptr) { set_error("pred_row_ptr is NULL"); return TICTAC_ERR_NULL; }
    if (R > 0 && !recv_ids) { set_error("recv_ids is NULL"); return TICTAC_ERR_NULL; }
    if (row_ptr[0] != 0) { set_error("pred_row_ptr[0] != 0"); return TICTAC_ERR_BAD_CSR; }
    for (int32_t v = 0; v < n; ++v)
        if (row_ptr[v + 1] < row_ptr[v]) { set_error("pred_row_ptr decreases at op %d", v); return TICTAC_ERR_BAD_CSR; }
    const int32_t E = row_ptr[n];
    if (E > 0 && !col_idx) { set_error("pred_col_idx is NULL"); return TICTAC_ERR_NULL; }
    for (int32_t e = 0; e < E; ++e)
        if (col_idx[e] < 0 || col_idx[e] >= n) { set_error("pred_col_idx[%d]=%d out of range", e, col_idx[e]); return TICTAC_ERR_BAD_CSR; }
    std::vector<int32_t> recv_of_op(n, -1);
    for (int32_t i = 0; i < R; ++i) {
        int32_t v = recv_ids[i];
        if (v < 0 || v >= n) { set_error("recv_ids[%d]=%d out of range", i, v); return TICTAC_ERR_BAD_CSR; }
        if (recv_of_op[v] >= 0) { set_error("op %d listed twice in recv_ids", v); return TICTAC_ERR_DUP_RECV; }
        recv_of_op[v] = i;
    }
    for (int32_t i = 0; i < R; ++i) {
        int32_t v = recv_ids[i];
        if (row_ptr[v + 1] != row_ptr[v]) { set_error("recv %d (op %d) has predecessors", i, v); return TICTAC_ERR_RECV_NOT_ROOT; }
    }
    // ---- levels = longest path from a root (Kahn) ----
    std::vector<int32_t> sptr(n + 1, 0), sidx(E), waiting(n), level(n, 0), queue;
    for (int32_t e = 0; e < E; ++e) sptr[col_idx[e] + 1]++;
    for (int32_t v = 0; v < n; ++v) sptr[v + 1] += sptr[v];
    {
        std::vector<int32_t> fill(sptr.begin(), sptr.end() - 1);
        for (int32_t v = 0; v < n; ++v)
            for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) sidx[fill[col_idx[e]]++] = v;
    }
    queue.reserve(n);
    for (int32_t v = 0; v < n; ++v) {
        waiting[v] = row_ptr[v + 1] - row_ptr[v];
        if (waiting[v] == 0) queue.push_back(v);
    }
    int32_t n_levels = 0;
    for (size_t q = 0; q < queue.size(); ++q) {
        int32_t u = queue[q];
        n_levels = std::max(n_levels, level[u] + 1);
        for (int32_t e = sptr[u]; e < sptr[u + 1]; ++e) {
            int32_t v = sidx[e];
            level[v] = std::max(level[v], level[u] + 1);
            if (--waiting[v] == 0) queue.push_back(v);
        }
    }
    if ((int32_t)queue.size() != n) { set_error("the graph has a cycle"); return TICTAC_ERR_CYCLE; }
    std::vector<int32_t> comp_col(n, -1);
    {
        int32_t j = 0;
        for (int32_t v = 0; v < n; ++v)
            if (recv_of_op[v] < 0) comp_col[v] = j++;
    }

    // ---- condensed graph: chains of single-predecessor compute ops collapse onto their head ----
    // rep[v] = the node whose dep op v has (itself if v is a node); recvs are not nodes, they
    // enter a node as single bits.
    std::vector<int32_t> rep(n, -1), node_level(n, 0);
    std::vector<int32_t> node_in, node_in_ptr(1, 0);     // inputs of node k: node_in[node_in_ptr[k] .. node_in_ptr[k + 1])
    node_in.reserve(E);
    std::vector<int32_t> node_ops;                       // in topological order
    std::vector<int32_t> node_index(n, -1);              // op -> index into node_ops
    std::vector<int32_t> tmp;
    for (int32_t v : queue) {
        if (recv_of_op[v] >= 0) continue;
        tmp.assign(col_idx + row_ptr[v], col_idx + row_ptr[v + 1]);
        std::sort(tmp.begin(), tmp.end());
        tmp.erase(std::unique(tmp.begin(), tmp.end()), tmp.end());
        if (tmp.size() == 1 && recv_of_op[tmp[0]] < 0) { rep[v] = rep[tmp[0]]; continue; }
        rep[v] = v;
        node_index[v] = (int32_t)node_ops.size();
        node_ops.push_back(v);
        const size_t first = node_in.size();             // ~i for recv i, else index of the input node
        for (int32_t u : tmp) {
            if (recv_of_op[u] >= 0) node_in.push_back(~recv_of_op[u]);
            else node_in.push_back(node_index[rep[u]]);
        }
        std::sort(node_in.begin() + first, node_in.end());
        node_in.erase(std::unique(node_in.begin() + first, node_in.end()), node_in.end());
        node_in_ptr.push_back((int32_t)node_in.size());
    }
    const int32_t M = (int32_t)node_ops.size();
    // Nodes are grouped by the level of their op in the full graph (an input of a node lies on a
    // strictly lower level, and close to it, which keeps inputs inside the kernel's LDS ring);
    // levels without nodes are dropped.
    int32_t n_node_levels = 0;
    {
        std::vector<int32_t> used(n_levels + 1, 0);
        for (int32_t v : node_ops) used[level[v]] = 1;
        for (int32_t l = 0; l < n_levels; ++l) { const int32_t u = used[l]; used[l] = n_node_levels; n_node_levels += u; }
        for (int32_t v : node_ops) node_level[v] = used[level[v]];
    }
    std::vector<int32_t> nlvl_ptr(n_node_levels + 1, 0), pos_of_index(M);
    for (int32_t v : node_ops) nlvl_ptr[node_level[v] + 1]++;
    int32_t max_width = 0;
    for (int32_t l = 0; l < n_node_levels; ++l) { max_width = std::max(max_width, nlvl_ptr[l + 1]); nlvl_ptr[l + 1] += nlvl_ptr[l]; }
    {
        std::vector<int32_t> fill(nlvl_ptr.begin(), nlvl_ptr.end() - 1);
        for (int32_t k = 0; k < M; ++k) pos_of_index[k] = fill[node_level[node_ops[k]]]++;
    }
    std::vector<Dag::NodeRec> nodes(M);
    std::vector<int32_t> ovf_idx;
    for (int32_t k = 0; k < M; ++k) {
        Dag::NodeRec &r = nodes[pos_of_index[k]];
        r.op = node_ops[k];
        r.ovf_beg = -1;
        for (int j = 0; j < 6; ++j) r.in[j] = INT32_MIN;
        int j = 0;
        for (int32_t e = node_in_ptr[k]; e < node_in_ptr[k + 1]; ++e) {
            const int32_t x = node_in[e];
            const int32_t y = x < 0 ? x : pos_of_index[x];
            if (j < 6) {
                r.in[j] = y;
            } else {
                if (r.ovf_beg < 0) { r.ovf_beg = (int32_t)ovf_idx.size(); ovf_idx.push_back(0); }
                ovf_idx.push_back(y);
                ovf_idx[r.ovf_beg]++;
            }
            ++j;
        }
    }
    std::vector<int32_t> src(n);
    for (int32_t v = 0; v < n; ++v) src[v] = recv_of_op[v] >= 0 ? ~recv_of_op[v] : rep[v];

    d->n = n; d->R = R; d->W = (R + 63) / 64; d->N = n - R; d->E = E;
    d->h_row_ptr.assign(row_ptr, row_ptr + n + 1);
    d->h_col_idx.assign(col_idx, col_idx + E);
    d->h_recv_ids.assign(recv_ids, recv_ids + R);
    d->n_levels = n_levels;
    d->M = M; d->n_node_levels = n_node_levels; d->max_node_level_width = max_width;
    HIP_TRY(hipGetDevice(&d->device));

    // ---- upload and propagate ----
    // the ops whose rows are copies (of a recv's single bit, or of the row of the node the op collapses onto)
    std::vector<int32_t> copied;
    for (int32_t v = 0; v < n; ++v)
        if (src[v] != v) { copied.push_back(v); copied.push_back(src[v]); }
    d->n_copied = (int32_t)(copied.size() / 2);
    Packer graph;
    graph.add(&d->d_recv_of_op, recv_of_op);
    graph.add(&d->d_nodes, nodes);
    graph.add(&d->d_ovf_idx, ovf_idx);
    graph.add(&d->d_nlvl_ptr, nlvl_ptr);
    {
        // words per workgroup slice, threads, and the chunks of levels of the node kernel
        // a workgroup's LDS traffic per level grows with its slice, so wide bitsets get many narrow slices
        d->k1_wc = d->W <= 1 ? 1 : (d->W <= 2 ? 2 : (d->W >= 16 ? 1 : 4));
        // Graphs with narrow levels take a level per LDS round trip when one wave holds every row of its slice,
        // every record and the input lists of the nodes that fit no record in LDS (propagate_nodes_wave); the
        // slice is narrowed until that fits.
        size_t list_entries = 0;
        for (int32_t q = 0; q < M; ++q) {
            const Dag::NodeRec &r = nodes[q];
            int nn = 0, nr = 0;
            for (int j = 0; j < 6; ++j) if (r.in[j] != INT32_MIN) (r.in[j] < 0 ? nr : nn) += 1;
            if (r.ovf_beg >= 0)
                for (int32_t e = 1; e <= ovf_idx[r.ovf_beg]; ++e) (ovf_idx[r.ovf_beg + e] < 0 ? nr : nn) += 1;
            if (nn > 4 || nr > 2) list_entries += 1 + (size_t)nn + nr;
        }
        d->k1_wave = false;
        for (int wc = d->k1_wc; wc >= 1 && max_width <= 64 && list_entries <= 4096 && M > 0; wc >>= 1) {
            if (max_width * wc <= 64 &&
                ((size_t)(M + 2) * wc + 1) * 8 + (size_t)M * 32 + (size_t)(n_node_levels + 1) * 4 + list_entries * 4 <= 150 * 1024) {
                d->k1_wc = wc;
                d->k1_wave = true;
                break;
            }
        }
        int threads = max_width * d->k1_wc;
        threads = threads < 64 ? 64 : (threads > 1024 ? 1024 : (threads + 63) / 64 * 64);
        d->k1_threads = threads;
        const int32_t per_pass = threads / d->k1_wc;
        std::vector<int32_t> chunk_end(n_node_levels, 0);
        for (int32_t l0 = 0; l0 < n_node_levels;) {
            int32_t l1 = l0 + 1;
            while (l1 < n_node_levels && l1 - l0 < 64 && nlvl_ptr[l1 + 1] - nlvl_ptr[l0] <= 4 * per_pass) ++l1;
            chunk_end[l0] = l1;
            l0 = l1;
        }
        graph.add(&d->d_chunk_end, chunk_end);
        // the LDS ring: a power of two of positions, at least two chunks (or all nodes), at most 64 KB beyond that
        int32_t ring = 64;
        while (ring < M && (ring < 2 * kK1Rpt * per_pass || (size_t)ring * 2 * d->k1_wc * 8 <= 64 * 1024)) ring *= 2;
        if (d->k1_wave) ring = M;                   // every row stays: no ring, positions are used as they are
        d->k1_ring = ring;
        // level-major records (see internal.h): when a workgroup has more than one wave, the padding at
        // most quadruples the records, and sixteen levels of slots fit the ring: at most 64 KB, and 32 KB for
        // one-word slices (many narrow workgroups: four of them then share a compute unit when several
        // graphs are propagated by one launch)
        int32_t lring = 0;
        if (max_width <= per_pass && threads > 64 && (int64_t)n_node_levels * per_pass <= (int64_t)4 * M + 8192) {
            const size_t ring_cap = d->k1_wc == 1 ? 32 * 1024 : 64 * 1024;
            lring = 64;
            while ((size_t)lring * 2 * d->k1_wc * 8 <= ring_cap && lring < n_node_levels * per_pass) lring *= 2;
            if (lring < 16 * per_pass && lring < n_node_levels * per_pass) lring = 0;
        }
        d->k1_lring = lring;
        // Rows of a multiple of eight words, levels of at most 256 nodes: also the records of the kernel with
        // 64-byte slices (four lanes per slot, or two with 32-byte slices; P slots per level, a multiple of 32 so that the
        // slots of a wave are whole; 2048 slots in the ring), which the propagation of several graphs by one launch takes.
        int32_t q_slots = (max_width + 31) / 32 * 32, q_ring = 0;
        if (q_slots < 32) q_slots = 32;
        if (d->k1_wc == 1 && d->W % 8 == 0 && d->W <= 1016 && max_width <= 256 && M > 0 &&
            (int64_t)n_node_levels * q_slots <= (int64_t)4 * M + 8192) {
            q_ring = 2048;
            while (q_ring > 64 && q_ring / 2 >= n_node_levels * q_slots) q_ring /= 2;
            if (q_ring < 4 * q_slots && q_ring < n_node_levels * q_slots) q_ring = 0;
        }
        d->k1_q_ring = q_ring;
        d->k1_q_threads = q_ring > 0 ? 4 * q_slots : 0;
        // Level-major records, of either kind.  While level l is computed the ring holds the slots from
        // (l + 1) * P - ring on.  With 64-byte slices that is few levels, and a row that a later level needs is
        // handed on by copy nodes (op = -2: one input, the row goes to the ring only) in free slots of the levels
        // between, each within reach of the one before; the copies of a row form one chain, which the consumers,
        // taken level by level, extend.
        auto level_major = [&](bool quad, int32_t P, int32_t lring, std::vector<Dag::FastRec> &lrecs,
                               std::vector<Dag::QuadRec> &qrecs, std::vector<int32_t> &lfovf, std::vector<int32_t> &left) {
            const int32_t row_bytes = d->k1_wc * 8, zero_row = lring * row_bytes;
            std::vector<int32_t> slot_of(M);            // position -> slot
            for (int32_t l = 0; l < n_node_levels; ++l)
                for (int32_t q = nlvl_ptr[l]; q < nlvl_ptr[l + 1]; ++q) slot_of[q] = l * P + (q - nlvl_ptr[l]);
            if (quad) {
                const uint32_t zero2 = (uint32_t)lring | (uint32_t)lring << 16;
                qrecs.assign((size_t)n_node_levels * P, Dag::QuadRec{zero2, zero2, 0xffffffffu, -1});
            } else {
                Dag::FastRec none;
                for (int j = 0; j < 4; ++j) none.in[j] = zero_row;
                none.rcv[0] = none.rcv[1] = -1;
                none.op = -1;
                none.ovf = -1;
                lrecs.assign((size_t)n_node_levels * P, none);
            }
            const int32_t reach = lring / P - 1;        // a row of level x is in the ring up to level x + reach
            std::vector<int32_t> used(n_node_levels);
            for (int32_t l = 0; l < n_node_levels; ++l) used[l] = nlvl_ptr[l + 1] - nlvl_ptr[l];
            std::unordered_map<int32_t, std::vector<int32_t>> chain;       // slot of a row -> slots of its copies
            auto within_reach = [&](int32_t slot, int32_t l) -> int32_t {   // the slot to read at level l, or -1
                if ((int64_t)slot >= (int64_t)(l + 1) * P - lring) return slot;
                if (!quad || reach < 1 || l - slot / P > 8 * reach) return -1;
                std::vector<int32_t> &ch = chain[slot];
                int32_t cur = ch.empty() ? slot : ch.back();
                while (l - cur / P > reach) {
                    int32_t t = cur / P + reach;
                    while (t > cur / P && used[t] >= P) --t;
                    if (t == cur / P) return -1;
                    const int32_t c = t * P + used[t]++;
                    qrecs[c].in01 = (uint32_t)(cur & (lring - 1)) | (uint32_t)lring << 16;
                    qrecs[c].op = -2;
                    ch.push_back(c);
                    cur = c;
                }
                return cur;
            };
            std::vector<int32_t> src_slot;
            for (int32_t l = 0; l < n_node_levels; ++l)
                for (int32_t q = nlvl_ptr[l]; q < nlvl_ptr[l + 1]; ++q) {
                    const Dag::NodeRec &r = nodes[q];
                    tmp.clear();
                    for (int j = 0; j < 6; ++j) if (r.in[j] != INT32_MIN) tmp.push_back(r.in[j]);
                    if (r.ovf_beg >= 0)
                        for (int32_t e = 1; e <= ovf_idx[r.ovf_beg]; ++e) tmp.push_back(ovf_idx[r.ovf_beg + e]);
                    int nn = 0, nr = 0;
                    for (int32_t &x : tmp) {
                        if (x < 0) { ++nr; continue; }
                        ++nn;
                        x = slot_of[x];
                    }
                    // (copies are made only for a node that then fits a record)
                    bool resident = nn <= 4 && nr <= 2;
                    src_slot.clear();
                    if (resident)
                        for (int32_t x : tmp) {
                            if (x < 0) continue;
                            const int32_t c = within_reach(x, l);
                            if (c < 0) { resident = false; break; }
                            src_slot.push_back(c);
                        }
                    if (quad) {
                        Dag::QuadRec &f = qrecs[slot_of[q]];
                        f.op = r.op;
                        if (resident) {
                            uint32_t in[4] = {(uint32_t)lring, (uint32_t)lring, (uint32_t)lring, (uint32_t)lring};
                            uint32_t rc[2] = {0xffffu, 0xffffu};
                            int a = 0, b = 0;
                            for (int32_t x : tmp) if (x < 0) rc[b++] = (uint32_t)~x;
                            for (int32_t c : src_slot) in[a++] = (uint32_t)(c & (lring - 1));
                            f.in01 = in[0] | in[1] << 16;
                            f.in23 = in[2] | in[3] << 16;
                            f.rcv01 = rc[0] | rc[1] << 16;
                        } else {
                            f.in01 = 0xffffffffu;
                            f.in23 = (uint32_t)lfovf.size();
                        }
                    } else {
                        Dag::FastRec &f = lrecs[slot_of[q]];
                        f.op = r.op;
                        if (resident) {
                            int a = 0, b = 0;
                            for (int32_t x : tmp) if (x < 0) f.rcv[b++] = ~x;
                            for (int32_t c : src_slot) f.in[a++] = (c & (lring - 1)) * row_bytes;
                        } else {
                            f.ovf = (int32_t)lfovf.size();
                        }
                    }
                    if (!resident) {
                        lfovf.push_back((int32_t)tmp.size());
                        lfovf.insert(lfovf.end(), tmp.begin(), tmp.end());
                    }
                }
            if (!quad) return;
            // The copied rows ride along in slots that are still free: a recv's row anywhere (no input, one recv
            // bit), the copy of a node's row at a level within reach of the node or of one of its copy nodes, as
            // a node with that one input and the op's own id.  What finds no slot stays on the list `left`.
            std::vector<int32_t> slot_of_op(n, -1);
            for (int32_t q = 0; q < M; ++q) slot_of_op[nodes[q].op] = slot_of[q];
            const uint32_t zero2 = (uint32_t)lring | (uint32_t)lring << 16;
            int32_t cursor = 0;
            for (size_t e = 0; e + 1 < copied.size(); e += 2) {
                const int32_t v = copied[e], sv = copied[e + 1];
                int32_t c = -1;
                if (sv < 0) {
                    while (cursor < n_node_levels && used[cursor] >= P) ++cursor;
                    if (cursor < n_node_levels) {
                        c = cursor * P + used[cursor]++;
                        qrecs[c] = Dag::QuadRec{zero2, zero2, (uint32_t)~sv | 0xffff0000u, v};
                    }
                } else if (slot_of_op[sv] >= 0 && reach >= 1) {
                    const int32_t base = slot_of_op[sv];
                    auto it = chain.find(base);
                    const size_t n_cand = 1 + (it == chain.end() ? 0 : it->second.size());
                    for (size_t k = 0; k < n_cand && c < 0; ++k) {
                        const int32_t from = k == 0 ? base : it->second[k - 1];
                        for (int32_t t = from / P + 1; t <= from / P + reach && t < n_node_levels; ++t)
                            if (used[t] < P) {
                                c = t * P + used[t]++;
                                qrecs[c] = Dag::QuadRec{(uint32_t)(from & (lring - 1)) | (uint32_t)lring << 16, zero2,
                                                        0xffffffffu, v};
                                break;
                            }
                    }
                }
                if (c < 0) { left.push_back(v); left.push_back(sv); }
            }
        };
        if (q_ring > 0) {
            std::vector<Dag::FastRec> unused;
            std::vector<Dag::QuadRec> qrecs;
            std::vector<int32_t> qfovf;
            std::vector<int32_t> left;
            level_major(true, q_slots, q_ring, unused, qrecs, qfovf, left);
            graph.add(&d->d_qrecs, qrecs);
            graph.add(&d->d_qfovf, qfovf);
            graph.add(&d->d_q_copied, left);
            d->qfovf_len = (int32_t)qfovf.size();
            d->n_q_copied = (int32_t)(left.size() / 2);
        }
        if (lring > 0) {
            std::vector<Dag::FastRec> lrecs;
            std::vector<Dag::QuadRec> unused;
            std::vector<int32_t> lfovf;
            std::vector<int32_t> none_left;
            level_major(false, per_pass, lring, lrecs, unused, lfovf, none_left);
            graph.add(&d->d_lrecs, lrecs);
            graph.add(&d->d_lfovf, lfovf);
            d->lfovf_len = (int32_t)lfovf.size();
        } else if (max_width <= per_pass) {
            const int32_t row_bytes = d->k1_wc * 8, zero_row = ring * row_bytes;
            std::vector<Dag::FastRec> frecs(M);
            std::vector<int32_t> fovf;
            for (int32_t l = 0; l < n_node_levels; ++l)
                for (int32_t q = nlvl_ptr[l]; q < nlvl_ptr[l + 1]; ++q) {
                    const Dag::NodeRec &r = nodes[q];
                    Dag::FastRec &f = frecs[q];
                    tmp.clear();
                    for (int j = 0; j < 6; ++j) if (r.in[j] != INT32_MIN) tmp.push_back(r.in[j]);
                    if (r.ovf_beg >= 0)
                        for (int32_t e = 1; e <= ovf_idx[r.ovf_beg]; ++e) tmp.push_back(ovf_idx[r.ovf_beg + e]);
                    int nn = 0, nr = 0;
                    bool resident = true;       // every node input is in the ring while level l is computed
                    for (int32_t x : tmp) {
                        if (x < 0) { ++nr; continue; }
                        ++nn;
                        resident = resident && x >= nlvl_ptr[l + 1] - ring;
                    }
                    f.op = r.op;
                    f.ovf = -1;
                    for (int j = 0; j < 4; ++j) f.in[j] = zero_row;
                    f.rcv[0] = f.rcv[1] = -1;
                    if (nn <= 4 && nr <= 2 && resident) {
                        int a = 0, b = 0;
                        for (int32_t x : tmp) {
                            if (x < 0) f.rcv[b++] = ~x;
                            else f.in[a++] = (d->k1_wave ? x : (x & (ring - 1))) * row_bytes;
                        }
                    } else {
                        f.ovf = (int32_t)fovf.size();
                        fovf.push_back((int32_t)tmp.size());
                        fovf.insert(fovf.end(), tmp.begin(), tmp.end());
                    }
                }
            graph.add(&d->d_frecs, frecs);
            graph.add(&d->d_fovf, fovf);
            d->fovf_len = (int32_t)fovf.size();
        }
    }
    graph.add(&d->d_copied, copied);
    std::vector<int32_t> op_of_col(d->N);
    for (int32_t v = 0; v < n; ++v)
        if (comp_col[v] >= 0) op_of_col[comp_col[v]] = v;
    graph.add(&d->d_op_of_col, op_of_col);
    const size_t dep_words = (size_t)n * d->W;
    graph.reserve(&d->d_dep, dep_words * 8);
    if (d->k1_lring > 0)
        graph.reserve(&d->d_k1_sink, (size_t)((d->W + d->k1_wc - 1) / d->k1_wc) * d->k1_threads * 8);
    if (d->k1_q_ring > 0) graph.reserve(&d->d_k1_q_sink, (size_t)(d->W / 8) * d->k1_q_threads * 16);
    graph.reserve(&d->d_bad_order, 256);
    // (sized for the copy back of the rows as well, so that the block is not replaced while a copy is under way)
    (void)stage(std::max(graph.host.size(), dep_words * 8));
    HIP_TRY(graph.commit(&d->d_graph_block, s));
    HIP_TRY(hipMemsetAsync(d->d_bad_order, 0, 256, s));
    if (dep_words) HIP_TRY(launch_propagate(*d, s));

    // ---- classes of identical rows among the compute ops (a lambda: done again on the host when the device's
    // grouping cannot be used; returns a status, or 1 for "again, from the rows") ----
    auto classes = [&](const bool on_device) -> int {
    // Large graphs (8 MB of rows or more) are grouped without bringing the rows to the host: the device hashes
    // every row (128 bits, with the number of set bits and the lowest one), the host groups the hashes, and the
    // device forms the class rows and checks every op's row against its class (on a mismatch, which two
    // different rows with one hash would cause, everything below is done again from the rows themselves).
    std::vector<uint64_t> rows, cls_dep, depT;
    std::vector<int32_t> cls_ptr, cls_cols, cnt0, first_op, lowest;
    // only classes far larger than a lane's fair share of the ops are split
    const int32_t max_members = std::min(256, std::max(16, (d->N + 63) / 64));
    if (on_device) {
        HIP_TRY(ensure_workspace(d, (size_t)d->N * 32));
        int32_t *d_digest = static_cast<int32_t *>(d->d_work);
        HIP_TRY(launch_row_digests(*d, d->d_op_of_col, d_digest, s));
        std::vector<int32_t> pageable;
        int32_t *dg = static_cast<int32_t *>(stage((size_t)d->N * 32));
        if (!dg) {
            pageable.resize((size_t)d->N * 8);
            dg = pageable.data();
        }
        HIP_TRY(hipMemcpyAsync(dg, d_digest, (size_t)d->N * 32, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        std::vector<int32_t> first_col;
        group_digests(dg, d->N, max_members, cls_ptr, cls_cols, first_col, d->C_distinct);
        d->C = (int32_t)cls_ptr.size() - 1;
        d->Cpad = (d->C + 63) / 64 * 64;
        if (d->R <= 1024 && d->C <= 512) return 1;      // the small-graph kernels want tables made from the rows
        cnt0.resize(d->C); first_op.resize(d->C); lowest.resize(d->C);
        for (int32_t c = 0; c < d->C; ++c) {
            cnt0[c] = dg[(size_t)first_col[c] * 8 + 4];
            lowest[c] = dg[(size_t)first_col[c] * 8 + 5];
            first_op[c] = op_of_col[first_col[c]];
        }
    } else {
        rows.resize((size_t)d->N * d->W);
        if (!rows.empty()) {
            std::vector<uint64_t> pageable;
            uint64_t *all = static_cast<uint64_t *>(stage(dep_words * 8));   // stream order: after the copy of the graph block out of it
            if (!all) {
                pageable.resize(dep_words);
                all = pageable.data();
            }
            HIP_TRY(hipMemcpyAsync(all, d->d_dep, dep_words * 8, hipMemcpyDeviceToHost, s));
            HIP_TRY(hipStreamSynchronize(s));
            for (int32_t v = 0; v < n; ++v)
                if (comp_col[v] >= 0)
                    memcpy(&rows[(size_t)comp_col[v] * d->W], &all[(size_t)v * d->W], (size_t)d->W * 8);
        }
        group_classes(rows, d->N, d->W, max_members, cls_dep, cls_ptr, cls_cols, d->C_distinct);
        d->C = (int32_t)cls_ptr.size() - 1;
        d->Cpad = (d->C + 63) / 64 * 64;
        cnt0.assign(d->C, 0);
        depT.assign((size_t)d->W * d->Cpad, 0);
        // (the transpose in blocks of 16 classes: the block of rows stays in cache and every word row
        // of depT receives 128 consecutive bytes at a time)
        for (int32_t c0 = 0; c0 < d->C; c0 += 16) {
            const int32_t c1 = std::min(d->C, c0 + 16);
            for (int32_t w = 0; w < d->W; ++w) {
                uint64_t *dst = &depT[(size_t)w * d->Cpad];
                for (int32_t c = c0; c < c1; ++c) {
                    const uint64_t x = cls_dep[(size_t)c * d->W + w];
                    cnt0[c] += __builtin_popcountll(x);
                    dst[c] = x;
                }
            }
        }
    }
    d->cls_nnz = 0;
    for (int32_t c = 0; c < d->C; ++c) d->cls_nnz += cnt0[c];
    // runs [lo, hi) of consecutive recv indices of every class row, and the sum of its indices
    // (only the kernels for graphs with at most 1 024 recvs and 512 classes use them)
    const bool want_runs = !on_device && d->R <= 1024 && d->C <= 512;
    std::vector<int32_t> run_ptr, run_lo, run_hi, isum;
    if (want_runs) {
        run_ptr.assign(1, 0);
        isum.assign(d->C, 0);
    }
    for (int32_t c = 0; want_runs && c < d->C; ++c) {
        const uint64_t *row = &cls_dep[(size_t)c * d->W];
        int32_t i = 0;
        int64_t sum = 0;
        while (i < d->R) {
            // next set bit at or after i
            int32_t w = i >> 6;
            uint64_t x = row[w] & (~0ull << (i & 63));
            while (!x && ++w < d->W) x = row[w];
            if (!x) break;
            const int32_t lo = w * 64 + __builtin_ctzll(x);
            // next clear bit after lo
            w = lo >> 6;
            uint64_t y = ~row[w] & (~0ull << (lo & 63));
            while (!y && ++w < d->W) y = ~row[w];
            const int32_t hi = y ? std::min(d->R, w * 64 + __builtin_ctzll(y)) : d->R;
            run_lo.push_back(lo);
            run_hi.push_back(hi);
            sum += (int64_t)(lo + hi - 1) * (hi - lo) / 2;
            i = hi;
        }
        run_ptr.push_back((int32_t)run_lo.size());
        isum[c] = (int32_t)sum;
    }
    Packer cls;
    cls.host.reserve((cls_dep.size() + depT.size()) * 8 +
                     (isum.size() + run_ptr.size() + 2 * run_lo.size() + cnt0.size() + cls_ptr.size() + cls_cols.size() +
                      (size_t)d->N) * 4 + 16 * 256);
    cls.add(&d->d_cls_isum, isum);      // index sums stay below 2^20 (nothing when the runs are not built)
    d->max_members = 0;
    for (int32_t c = 0; c < d->C; ++c) d->max_members = std::max(d->max_members, cls_ptr[c + 1] - cls_ptr[c]);
    cls.add(&d->d_run_ptr, run_ptr);
    cls.add(&d->d_run_lo, run_lo);
    cls.add(&d->d_run_hi, run_hi);
    if (!on_device) {
        cls.add(&d->d_cls_dep, cls_dep);
        cls.add(&d->d_cls_depT, depT);
    } else {
        cls.add(&d->d_cls_first_op, first_op);
    }
    cls.add(&d->d_cls_cnt0, cnt0);
    cls.add(&d->d_cls_ptr, cls_ptr);
    cls.add(&d->d_cls_cols, cls_cols);
    std::vector<int32_t> col_cls(d->N, 0);
    for (int32_t c = 0; c < d->C; ++c)
        for (int32_t m = cls_ptr[c]; m < cls_ptr[c + 1]; ++m) col_cls[cls_cols[m]] = c;
    cls.add(&d->d_col_cls, col_cls);

    // ---- tables of the bit-sliced TAC kernel (see internal.h), for graphs with many classes ----
    const int32_t CW = (d->C + 63) / 64;
    const bool want_sliced = d->R >= 1 && d->W <= 64 && CW <= 15 * 64 * 4 && !(d->C <= 8 * 64 && d->W <= 6) &&
                             !tac_small_graph(d->R, d->W, d->C);
    if (want_sliced) {
        d->CW = CW;
        d->CWpad = (CW + 15) / 16 * 16;
        // parents: among the classes of the compute predecessors of an op, those with a strictly smaller dep
        // that holds two recvs or more; the two largest are kept
        std::vector<int32_t> par((size_t)d->C * 2, -1);
        for (int32_t v = 0; v < n; ++v) {
            if (comp_col[v] < 0) continue;
            const int32_t cv = col_cls[comp_col[v]];
            for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
                const int32_t u = col_idx[e];
                if (comp_col[u] < 0) continue;
                const int32_t cu = col_cls[comp_col[u]];
                if (cnt0[cu] < 2 || cnt0[cu] >= cnt0[cv]) continue;
                int32_t *pv = &par[(size_t)cv * 2];
                if (pv[0] == cu || pv[1] == cu) continue;
                if (pv[0] < 0 || cnt0[cu] > cnt0[pv[0]]) { pv[1] = pv[0]; pv[0] = cu; }
                else if (pv[1] < 0 || cnt0[cu] > cnt0[pv[1]]) pv[1] = cu;
            }
        }
        std::vector<uint64_t> ndom0((size_t)d->CWpad * 2, 0);
        std::vector<int32_t> nchild(d->C, 0);
        for (int32_t c = 0; c < d->C; ++c)
            for (int j = 0; j < 2; ++j) {
                const int32_t u = par[(size_t)c * 2 + j];
                if (u < 0) continue;
                ndom0[(size_t)c >> 5] += 1ull << ((c & 31) * 2);
                ++nchild[u];
            }
        std::vector<int32_t> cptr(d->C + 1, 0);
        for (int32_t c = 0; c < d->C; ++c) cptr[c + 1] = cptr[c] + nchild[c];
        std::vector<int32_t> cidx(cptr[d->C]), cfill(cptr.begin(), cptr.end() - 1);
        for (int32_t c = 0; c < d->C; ++c)
            for (int j = 0; j < 2; ++j) {
                const int32_t u = par[(size_t)c * 2 + j];
                if (u >= 0) cidx[cfill[u]++] = c;
            }
        std::vector<int4> crec(d->C);
        std::vector<int32_t> child_ovf;
        for (int32_t c = 0; c < d->C; ++c) {
            const int32_t nc = nchild[c], *ch = cidx.data() + cptr[c];
            int4 r = make_int4(nc, -1, -1, -1);
            if (nc >= 1) r.y = ch[0];
            if (nc >= 2) r.z = ch[1];
            if (nc == 3) r.w = ch[2];
            if (nc > 3) {
                r.w = (int32_t)child_ovf.size();
                child_ovf.insert(child_ovf.end(), ch + 2, ch + nc);
            }
            crec[c] = r;
        }
        // classes that depend on one recv (by recv, ascending class) and on none
        std::vector<int32_t> single_ptr(d->R + 1, 0), single_cls, empty_cls, first_recv(d->C, -1);
        for (int32_t c = 0; c < d->C; ++c) {
            if (cnt0[c] == 0) empty_cls.push_back(c);
            if (cnt0[c] != 1) continue;
            if (on_device) first_recv[c] = lowest[c];
            for (int32_t w = 0; !on_device && w < d->W; ++w)
                if (const uint64_t x = cls_dep[(size_t)c * d->W + w]) { first_recv[c] = w * 64 + __builtin_ctzll(x); break; }
            single_ptr[first_recv[c] + 1]++;
        }
        for (int32_t r = 0; r < d->R; ++r) single_ptr[r + 1] += single_ptr[r];
        single_cls.resize(single_ptr[d->R]);
        {
            std::vector<int32_t> fill(single_ptr.begin(), single_ptr.end() - 1);
            for (int32_t c = 0; c < d->C; ++c)
                if (cnt0[c] == 1) single_cls[fill[first_recv[c]]++] = c;
        }
        d->n_empty_cls = (int32_t)empty_cls.size();
        cls.add(&d->d_ndom0, ndom0);
        cls.add(&d->d_cls_par, par);
        cls.add(&d->d_crec, crec);
        cls.add(&d->d_child_ovf, child_ovf);
        cls.add(&d->d_single_ptr, single_ptr);
        cls.add(&d->d_single_cls, single_cls);
        cls.add(&d->d_empty_cls, empty_cls);
        cls.reserve(&d->d_colbits, (size_t)d->R * d->CWpad * 8);
        cls.reserve(&d->d_planes0, (size_t)13 * d->CWpad * 8);
        cls.reserve(&d->d_live0, (size_t)d->CWpad * 8);
    }
    if (on_device) {
        cls.reserve(&d->d_cls_dep, (size_t)d->C * d->W * 8);
        cls.reserve(&d->d_cls_depT, (size_t)d->W * d->Cpad * 8);
    }
    HIP_TRY(cls.commit(&d->d_class_block, s));
    int32_t *mismatch = d->d_bad_order + 1;         // (a second word of the zeroed flag block)
    if (on_device) HIP_TRY(launch_class_rows(*d, d->d_op_of_col, d->d_cls_first_op, mismatch, s));
    if (want_sliced) HIP_TRY(launch_sliced_tables(*d, s));
    int32_t differs = 0;
    if (on_device) HIP_TRY(hipMemcpyAsync(&differs, mismatch, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));   // host vectors go out of scope; the handle is complete
    if (differs) {
        HIP_TRY(hipMemsetAsync(mismatch, 0, sizeof(int32_t), s));
        return 1;
    }
    return TICTAC_OK;
    };
    int rc = classes(dep_words * 8 >= ((size_t)8 << 20) && d->N > 0 && !getenv("TICTAC_GROUP_ON_HOST"));
    if (rc == 1) {
        if (d->d_class_block) { HIP_TRY(hipStreamSynchronize(s)); (void)hipFree(d->d_class_block); d->d_class_block = nullptr; }
        rc = classes(false);
    }
    return rc;
}

}  // namespace tictac

using namespace tictac;

extern "C" {

int tictac_build_deps(int32_t n_ops, const int32_t *pred_row_ptr, const int32_t *pred_col_idx, int32_t n_recv,
                      const int32_t *recv_ids, tictac_stream stream, tictac_dag **out)
{
    if (!out) { set_error("out is NULL"); return TICTAC_ERR_NULL; }
    Dag *d = new (std::nothrow) Dag();
    if (!d) { set_error("out of host memory"); return TICTAC_ERR_NO_MEM; }
    int rc;
    try {
        rc = build(n_ops, pred_row_ptr, pred_col_idx, n_recv, recv_ids, (hipStream_t)stream, d);
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        rc = TICTAC_ERR_NO_MEM;
    }
    if (rc != TICTAC_OK) { free_dag(d); return rc; }
    *out = reinterpret_cast<tictac_dag *>(d);
    return TICTAC_OK;
}

int tictac_dag_info(const tictac_dag *dag, int32_t *n_ops, int32_t *n_recv, int32_t *words, int32_t *n_levels,
                    int32_t *n_classes)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    const Dag *d = reinterpret_cast<const Dag *>(dag);
    if (n_ops) *n_ops = d->n;
    if (n_recv) *n_recv = d->R;
    if (words) *words = d->W;
    if (n_levels) *n_levels = d->n_levels;
    if (n_classes) *n_classes = d->C_distinct;
    return TICTAC_OK;
}

int tictac_dag_deps(const tictac_dag *dag, const uint64_t **dep_device)
{
    if (!dag || !dep_device) { set_error("NULL argument"); return TICTAC_ERR_NULL; }
    *dep_device = reinterpret_cast<const Dag *>(dag)->d_dep;
    return TICTAC_OK;
}

int tictac_dag_copy_deps(const tictac_dag *dag, uint64_t *dst_device, tictac_stream stream)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    const Dag *d = reinterpret_cast<const Dag *>(dag);
    const size_t bytes = (size_t)d->n * d->W * 8;
    if (bytes == 0) return TICTAC_OK;
    if (!dst_device) { set_error("dst_device is NULL"); return TICTAC_ERR_NULL; }
    HIP_TRY(hipMemcpyAsync(dst_device, d->d_dep, bytes, hipMemcpyDeviceToDevice, (hipStream_t)stream));
    return TICTAC_OK;
}

int tictac_dag_recompute_deps(tictac_dag *dag, tictac_stream stream)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    Dag *d = reinterpret_cast<Dag *>(dag);
    HIP_TRY(launch_propagate(*d, (hipStream_t)stream));
    return TICTAC_OK;
}

int tictac_dag_recompute_deps_batch(tictac_dag *const *dags, int32_t n_dags, tictac_stream stream)
{
    if (n_dags < 0) { set_error("n_dags = %d is negative", n_dags); return TICTAC_ERR_UNSUPPORTED; }
    if (n_dags == 0) return TICTAC_OK;
    if (!dags) { set_error("dags is NULL"); return TICTAC_ERR_NULL; }
    for (int32_t g = 0; g < n_dags; ++g)
        if (!dags[g]) { set_error("dags[%d] is NULL", g); return TICTAC_ERR_NULL; }
    Dag *const *ds = reinterpret_cast<Dag *const *>(dags);
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(ensure_workspace(ds[0], propagate_batch_staging_bytes(n_dags)));
    const hipError_t e = launch_propagate_batch(ds, n_dags, ds[0]->d_work, s);
    if (e == hipErrorNotSupported) {
        // graphs of different shapes, or graphs that take another propagation kernel: one after the other
        for (int32_t g = 0; g < n_dags; ++g) HIP_TRY(launch_propagate(*ds[g], s));
        return TICTAC_OK;
    }
    HIP_TRY(e);
    return TICTAC_OK;
}

int tictac_dag_free(tictac_dag *dag)
{
    if (!dag) return TICTAC_OK;
    free_dag(reinterpret_cast<Dag *>(dag));
    return TICTAC_OK;
}

int tictac_tic_priority(const tictac_dag *dag, int32_t *prio, int32_t *order, int32_t *rank, tictac_stream stream)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    const Dag *d = reinterpret_cast<const Dag *>(dag);
    if (d->R == 0) return TICTAC_OK;
    if (!prio) { set_error("prio is NULL"); return TICTAC_ERR_NULL; }
    HIP_TRY(launch_tic(*d, prio, order, rank, nullptr, (hipStream_t)stream));
    return TICTAC_OK;
}

static int check_batch(const Dag *d, int32_t B, const void *op_time, const void *recv_time)
{
    if (B < 0) { set_error("B = %d", B); return TICTAC_ERR_BAD_CSR; }
    if (B > 0 && d->N > 0 && !op_time) { set_error("op_time is NULL"); return TICTAC_ERR_NULL; }
    if (B > 0 && d->R > 0 && !recv_time) { set_error("recv_time is NULL"); return TICTAC_ERR_NULL; }
    return TICTAC_OK;
}

int tictac_tac_priority(const tictac_dag *dag, int32_t B, const double *op_time, const double *recv_time,
                        int32_t *order, int32_t *rank, double *sel_P, double *sel_Mplus, tictac_stream stream)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    Dag *d = const_cast<Dag *>(reinterpret_cast<const Dag *>(dag));
    int rc = check_batch(d, B, op_time, recv_time);
    if (rc != TICTAC_OK) return rc;
    if (B == 0 || d->R == 0) return TICTAC_OK;
    if (!order) { set_error("order is NULL"); return TICTAC_ERR_NULL; }
    TacArgs a{B, op_time, recv_time, order, rank, sel_P, sel_Mplus, false, nullptr, nullptr, nullptr, nullptr, nullptr};
    HIP_TRY(launch_tac(*d, a, (hipStream_t)stream));
    return TICTAC_OK;
}

static int tac_simulate_any(const tictac_dag *dag, int32_t B, const void *op_time, const void *recv_time, bool f32,
                            int32_t *order, int32_t *rank, double *sel_P, double *sel_Mplus, double *makespan,
                            double *eff, double *U, double *L, double *S, tictac_stream stream)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    Dag *d = const_cast<Dag *>(reinterpret_cast<const Dag *>(dag));
    int rc = check_batch(d, B, op_time, recv_time);
    if (rc != TICTAC_OK) return rc;
    if (B == 0) return TICTAC_OK;
    if (d->R > 0 && !order) { set_error("order is NULL"); return TICTAC_ERR_NULL; }
    TacArgs a{B, op_time, recv_time, order, rank, sel_P, sel_Mplus, true, makespan, eff, U, L, S};
    a.f32 = f32;
    HIP_TRY(launch_tac(*d, a, (hipStream_t)stream));
    return TICTAC_OK;
}

// ---- the entry point that allocates nothing ----
// Per-call memory of tictac_tac_simulate_noalloc: one flag per sample ("left to the general kernel").  The
// array exists once per GPU for as long as the library is loaded; every call on a GPU uses it.
constexpr int32_t kNoallocMaxB = 1 << 20;
static __device__ __align__(256) int32_t scratch[kNoallocMaxB];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];         // device address of `scratch` on every device, 0 = not asked yet
static std::mutex g_scratch_mutex;

// the device address of the array on the current device (asked of the runtime once per device)
static hipError_t scratch_address(int32_t **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *q = nullptr;
        e = hipGetSymbolAddress(&q, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = q;
    }
    *out = static_cast<int32_t *>(g_scratch_ptr[dev]);
    return hipSuccess;
}

int tictac_tac_simulate_noalloc(const tictac_dag *dag, int32_t B, const double *op_time, const double *recv_time,
                                int32_t *order, int32_t *rank, double *makespan, double *eff, double *U, double *L,
                                double *S, tictac_stream stream)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    Dag *d = const_cast<Dag *>(reinterpret_cast<const Dag *>(dag));
    int rc = check_batch(d, B, op_time, recv_time);
    if (rc != TICTAC_OK) return rc;
    if (B > kNoallocMaxB) {
        set_error("B = %d: tictac_tac_simulate_noalloc takes at most %d samples per call", B, kNoallocMaxB);
        return TICTAC_ERR_UNSUPPORTED;
    }
    if (B == 0) return TICTAC_OK;
    if (d->R > 0 && !order) { set_error("order is NULL"); return TICTAC_ERR_NULL; }
    int32_t *flags = nullptr;
    HIP_TRY(scratch_address(&flags));
    TacArgs a{B, op_time, recv_time, order, rank, nullptr, nullptr, true, makespan, eff, U, L, S};
    a.ext_flags = flags;
    const hipError_t e = launch_tac(*d, a, (hipStream_t)stream);
    if (e == hipErrorNotSupported) {
        set_error("%d recvs, %d classes: tictac_tac_simulate_noalloc serves graphs with at most 512 classes of compute ops, "
                  "384 recvs and per-sample state that fits the local memory of a compute unit", d->R, d->C);
        return TICTAC_ERR_UNSUPPORTED;
    }
    HIP_TRY(e);
    return TICTAC_OK;
}

int tictac_tac_simulate(const tictac_dag *dag, int32_t B, const double *op_time, const double *recv_time,
                        int32_t *order, int32_t *rank, double *sel_P, double *sel_Mplus, double *makespan,
                        double *eff, double *U, double *L, double *S, tictac_stream stream)
{
    return tac_simulate_any(dag, B, op_time, recv_time, false, order, rank, sel_P, sel_Mplus, makespan, eff, U, L, S,
                            stream);
}

int tictac_tac_simulate_f32(const tictac_dag *dag, int32_t B, const float *op_time, const float *recv_time,
                            int32_t *order, int32_t *rank, double *sel_P, double *sel_Mplus, double *makespan,
                            double *eff, double *U, double *L, double *S, tictac_stream stream)
{
    return tac_simulate_any(dag, B, op_time, recv_time, true, order, rank, sel_P, sel_Mplus, makespan, eff, U, L, S,
                            stream);
}

static int simulate_any(const tictac_dag *dag, int32_t B, const int32_t *order, int32_t order_stride,
                        const void *op_time, const void *recv_time, bool f32, double *makespan, double *eff, double *U,
                        double *L, double *S, tictac_stream stream)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    Dag *d = const_cast<Dag *>(reinterpret_cast<const Dag *>(dag));
    int rc = check_batch(d, B, op_time, recv_time);
    if (rc != TICTAC_OK) return rc;
    if (order_stride != 0 && order_stride != d->R) {
        set_error("order_stride = %d, expected 0 or n_recv = %d", order_stride, d->R);
        return TICTAC_ERR_BAD_ORDER;
    }
    if (B == 0) return TICTAC_OK;
    if (d->R > 0 && !order) { set_error("order is NULL"); return TICTAC_ERR_NULL; }
    if (!makespan || !eff) { set_error("makespan or eff is NULL"); return TICTAC_ERR_NULL; }
    SimArgs a{B, order, order_stride, op_time, recv_time, makespan, eff, U, L, S};
    a.f32 = f32;
    HIP_TRY(launch_check_orders(*d, B, order, order_stride, (hipStream_t)stream));
    HIP_TRY(launch_simulate(*d, a, (hipStream_t)stream));
    return TICTAC_OK;
}

int tictac_simulate(const tictac_dag *dag, int32_t B, const int32_t *order, int32_t order_stride,
                    const double *op_time, const double *recv_time, double *makespan, double *eff, double *U,
                    double *L, double *S, tictac_stream stream)
{
    return simulate_any(dag, B, order, order_stride, op_time, recv_time, false, makespan, eff, U, L, S, stream);
}

int tictac_simulate_f32(const tictac_dag *dag, int32_t B, const int32_t *order, int32_t order_stride,
                        const float *op_time, const float *recv_time, double *makespan, double *eff, double *U,
                        double *L, double *S, tictac_stream stream)
{
    return simulate_any(dag, B, order, order_stride, op_time, recv_time, true, makespan, eff, U, L, S, stream);
}

int tictac_simulate_channels(const tictac_dag *dag, int32_t B, int32_t n_channels, const int32_t *channel_of_recv,
                             const int32_t *order, int32_t order_stride, const double *op_time,
                             const double *recv_time, double *makespan, double *eff, double *U, double *L,
                             double *S, tictac_stream stream)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    Dag *d = const_cast<Dag *>(reinterpret_cast<const Dag *>(dag));
    int rc = check_batch(d, B, op_time, recv_time);
    if (rc != TICTAC_OK) return rc;
    if (n_channels < 1 || n_channels > 64) {
        set_error("n_channels = %d, expected 1 .. 64", n_channels);
        return TICTAC_ERR_UNSUPPORTED;
    }
    if (order_stride != 0 && order_stride != d->R) {
        set_error("order_stride = %d, expected 0 or n_recv = %d", order_stride, d->R);
        return TICTAC_ERR_BAD_ORDER;
    }
    if (d->R > 0 && !channel_of_recv) { set_error("channel_of_recv is NULL"); return TICTAC_ERR_NULL; }
    for (int32_t i = 0; i < d->R; ++i)
        if (channel_of_recv[i] < 0 || channel_of_recv[i] >= n_channels) {
            set_error("channel_of_recv[%d] = %d is outside 0 .. %d", i, channel_of_recv[i], n_channels - 1);
            return TICTAC_ERR_BAD_ORDER;
        }
    if (B == 0) return TICTAC_OK;
    if (d->R > 0 && !order) { set_error("order is NULL"); return TICTAC_ERR_NULL; }
    if (!makespan || !eff) { set_error("makespan or eff is NULL"); return TICTAC_ERR_NULL; }
    SimArgs a{B, order, order_stride, op_time, recv_time, makespan, eff, U, L, S};
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(launch_check_orders(*d, B, order, order_stride, s));
    if (d->R == 0) {                      // no transfers: the channels play no role
        HIP_TRY(launch_simulate(*d, a, s));
        return TICTAC_OK;
    }
    if (d->R > 512 || d->C > 512) {
        set_error("%d recvs and %d classes: the several-channel simulation handles at most 512 of each", d->R, d->C);
        return TICTAC_ERR_UNSUPPORTED;
    }
    // the channel table goes to the device through a staging block of the handle
    HIP_TRY(ensure_chan_table(d, channel_of_recv, s));
    const hipError_t e = launch_simulate_channels(*d, a, n_channels, d->d_chan, s);
    if (e == hipErrorNotSupported) {
        set_error("graph outside what the several-channel simulation handles");
        return TICTAC_ERR_UNSUPPORTED;
    }
    HIP_TRY(e);
    return TICTAC_OK;
}

int tictac_dag_check_orders(tictac_dag *dag, tictac_stream stream)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    Dag *d = reinterpret_cast<Dag *>(dag);
    if (!d->d_bad_order) return TICTAC_OK;
    hipStream_t s = (hipStream_t)stream;
    int32_t raised = 0;
    HIP_TRY(hipMemcpyAsync(&raised, d->d_bad_order, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (raised == 0) return TICTAC_OK;
    HIP_TRY(hipMemsetAsync(d->d_bad_order, 0, sizeof(int32_t), s));
    set_error("an order given since the last check was no permutation of 0 .. n_recv-1");
    return TICTAC_ERR_BAD_ORDER;
}

// Tables of the iteration with send ops for the given send set (kept until another set is given).
// TICTAC_OK, or the status to return (the error text is set).
static int ensure_send_tables(Dag *d, int32_t n_send, const int32_t *send_ids, hipStream_t s)
{
    if (d->send_tables_built && d->h_send_ids.size() == (size_t)n_send &&
        (n_send == 0 || memcmp(d->h_send_ids.data(), send_ids, (size_t)n_send * sizeof(int32_t)) == 0))
        return TICTAC_OK;
    const int32_t n = d->n, E = d->E;
    std::vector<int32_t> recv_of_op(n, -1), col_of_op(n, -1), n_succ(n, 0);
    for (int32_t i = 0; i < d->R; ++i) recv_of_op[d->h_recv_ids[i]] = i;
    for (int32_t v = 0, j = 0; v < n; ++v)
        if (recv_of_op[v] < 0) col_of_op[v] = j++;
    for (int32_t e = 0; e < E; ++e) n_succ[d->h_col_idx[e]]++;
    std::vector<uint8_t> is_send(n, 0);
    for (int32_t i = 0; i < n_send; ++i) {
        const int32_t v = send_ids[i];
        if (v < 0 || v >= n) { set_error("send_ids[%d] = %d is no op id", i, v); return TICTAC_ERR_BAD_CSR; }
        if (recv_of_op[v] >= 0) { set_error("send_ids[%d] = %d is a recv op", i, v); return TICTAC_ERR_BAD_CSR; }
        if (is_send[v]) { set_error("send_ids holds op %d twice", v); return TICTAC_ERR_BAD_CSR; }
        if (n_succ[v] != 0) {
            set_error("send op %d has successors (Sec. 2.2: the send ops are leaves)", v);
            return TICTAC_ERR_BAD_CSR;
        }
        is_send[v] = 1;
    }
    // rec[v]: where the successors of v start in succ (-1: none), the column of its time (-1: a recv), 1 for a send.
    // succ[e]: a successor (the top bit marks the last one of its list), and what running that successor needs, so
    // that an op released by the op before it is run without a read of rec: its column, where its own successors
    // start, 1 for a send.  64 entries of padding: a wave reads 64 entries at a time.
    std::vector<int4> rec(n), succ((size_t)E + 64, make_int4(0, 0, 0, 0));
    std::vector<int32_t> fill(n), send_free;
    std::vector<uint16_t> indeg(n);
    std::vector<uint32_t> ready0(((size_t)n + 31) / 32, 0u);
    std::vector<uint8_t> col_kind(d->N > 0 ? d->N : 1, 0);
    int32_t at = 0;
    for (int32_t v = 0; v < n; ++v) {
        rec[v] = make_int4(n_succ[v] > 0 ? at : -1, 0, col_of_op[v], is_send[v]);
        fill[v] = at;
        at += n_succ[v];
        const int32_t deg = d->h_row_ptr[v + 1] - d->h_row_ptr[v];
        if (deg > 65535) { set_error("op %d has %d predecessors, more than 65535", v, deg); return TICTAC_ERR_UNSUPPORTED; }
        indeg[v] = (uint16_t)deg;
        if (recv_of_op[v] < 0 && deg == 0) {
            if (is_send[v]) send_free.push_back(col_of_op[v]);
            else ready0[v >> 5] |= 1u << (v & 31);
        }
        if (is_send[v]) col_kind[col_of_op[v]] = 1;
    }
    for (int32_t v = 0; v < n; ++v)
        for (int32_t e = d->h_row_ptr[v]; e < d->h_row_ptr[v + 1]; ++e) {
            const int32_t u = d->h_col_idx[e], at_u = fill[u]++;
            const bool last = at_u + 1 == rec[u].x + n_succ[u];
            succ[at_u] = make_int4(last ? (int32_t)((uint32_t)v | 0x80000000u) : v, rec[v].z, rec[v].x, rec[v].w);
        }

    Packer tables;
    tables.add(&d->d_send_rec, rec);
    tables.add(&d->d_send_succ, succ);
    tables.add(&d->d_send_indeg, indeg);
    tables.add(&d->d_send_ready0, ready0);
    tables.add(&d->d_send_free, send_free);
    tables.add(&d->d_send_col_kind, col_kind);
    tables.add(&d->d_send_recv_ids, d->h_recv_ids);
    d->n_send_free = (int32_t)send_free.size();
    d->send_tables_built = false;
    HIP_TRY(hipStreamSynchronize(s));               // no kernel reads the old tables any more
    if (d->d_send_block) { (void)hipFree(d->d_send_block); d->d_send_block = nullptr; }
    HIP_TRY(tables.commit(&d->d_send_block, s));
    HIP_TRY(hipStreamSynchronize(s));               // the copy came out of `tables`, which ends here
    d->h_send_ids.assign(send_ids, send_ids + n_send);
    d->send_tables_built = true;
    return TICTAC_OK;
}

int tictac_simulate_sends(const tictac_dag *dag, int32_t B, int32_t n_send, const int32_t *send_ids,
                          const int32_t *order, int32_t order_stride, const double *op_time,
                          const double *recv_time, double *makespan, double *eff, double *U, double *L, double *S,
                          tictac_stream stream)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    Dag *d = const_cast<Dag *>(reinterpret_cast<const Dag *>(dag));
    int rc = check_batch(d, B, op_time, recv_time);
    if (rc != TICTAC_OK) return rc;
    if (n_send < 0) { set_error("n_send = %d is negative", n_send); return TICTAC_ERR_BAD_CSR; }
    if (n_send > 0 && !send_ids) { set_error("send_ids is NULL"); return TICTAC_ERR_NULL; }
    if (order_stride != 0 && order_stride != d->R) {
        set_error("order_stride = %d, expected 0 or n_recv = %d", order_stride, d->R);
        return TICTAC_ERR_BAD_ORDER;
    }
    hipStream_t s = (hipStream_t)stream;
    rc = ensure_send_tables(d, n_send, send_ids, s);
    if (rc != TICTAC_OK) return rc;
    if (B == 0) return TICTAC_OK;
    if (d->R > 0 && !order) { set_error("order is NULL"); return TICTAC_ERR_NULL; }
    if (!makespan || !eff) { set_error("makespan or eff is NULL"); return TICTAC_ERR_NULL; }
    if (d->n == 0) {
        SimArgs a0{B, order, order_stride, op_time, recv_time, makespan, eff, U, L, S};
        HIP_TRY(launch_simulate(*d, a0, s));        // the empty graph: nothing to send
        return TICTAC_OK;
    }
    SimArgs a{B, order, order_stride, op_time, recv_time, makespan, eff, U, L, S};
    HIP_TRY(launch_check_orders(*d, B, order, order_stride, s));
    const hipError_t e = launch_simulate_sends(*d, a, s);
    if (e == hipErrorNotSupported) {
        set_error("%d ops and %d recvs: the per-sample state of the iteration with send ops does not fit LDS", d->n, d->R);
        return TICTAC_ERR_UNSUPPORTED;
    }
    HIP_TRY(e);
    return TICTAC_OK;
}

int tictac_straggler_effect(int32_t B, int32_t w, const double *makespan, double *straggler, tictac_stream stream)
{
    if (B < 0) { set_error("B = %d is negative", B); return TICTAC_ERR_UNSUPPORTED; }
    if (w < 1) { set_error("w = %d, expected at least 1", w); return TICTAC_ERR_UNSUPPORTED; }
    if (B / w == 0) return TICTAC_OK;
    if (!makespan || !straggler) { set_error("makespan or straggler is NULL"); return TICTAC_ERR_NULL; }
    HIP_TRY(launch_straggler(B, w, makespan, straggler, (hipStream_t)stream));
    return TICTAC_OK;
}

int tictac_time_oracle_min(int32_t n_runs, int64_t n, const double *runs, double *time, tictac_stream stream)
{
    if (n_runs < 1) { set_error("n_runs = %d, expected at least 1", n_runs); return TICTAC_ERR_UNSUPPORTED; }
    if (n < 0) { set_error("n is negative"); return TICTAC_ERR_UNSUPPORTED; }
    if (n == 0) return TICTAC_OK;
    if (!runs || !time) { set_error("runs or time is NULL"); return TICTAC_ERR_NULL; }
    HIP_TRY(launch_time_oracle_min(n_runs, n, runs, time, (hipStream_t)stream));
    return TICTAC_OK;
}

int tictac_order_search(const tictac_dag *dag, int32_t B, const int32_t *order, int32_t order_stride,
                        int32_t n_moves, const int32_t *moves, const double *op_time, const double *recv_time,
                        int32_t *best_order, double *best_makespan, double *start_makespan, int32_t *n_accepted,
                        tictac_stream stream)
{
    if (!dag) { set_error("dag is NULL"); return TICTAC_ERR_NULL; }
    Dag *d = const_cast<Dag *>(reinterpret_cast<const Dag *>(dag));
    int rc = check_batch(d, B, op_time, recv_time);
    if (rc != TICTAC_OK) return rc;
    if (n_moves < 0) { set_error("n_moves = %d is negative", n_moves); return TICTAC_ERR_UNSUPPORTED; }
    if (order_stride != 0 && order_stride != d->R) {
        set_error("order_stride = %d, expected 0 or n_recv = %d", order_stride, d->R);
        return TICTAC_ERR_BAD_ORDER;
    }
    if (d->R == 0) { set_error("the graph has no recv: there is nothing to order"); return TICTAC_ERR_UNSUPPORTED; }
    if (d->R > 512 || d->C > 512) {
        set_error("%d recvs and %d classes: the order search handles at most 512 of each", d->R, d->C);
        return TICTAC_ERR_UNSUPPORTED;
    }
    if (B == 0) return TICTAC_OK;
    if (!order) { set_error("order is NULL"); return TICTAC_ERR_NULL; }
    if (n_moves > 0 && !moves) { set_error("moves is NULL"); return TICTAC_ERR_NULL; }
    if (!best_order || !best_makespan) { set_error("best_order or best_makespan is NULL"); return TICTAC_ERR_NULL; }
    SearchArgs a{B, order, order_stride, n_moves, moves, op_time, recv_time, best_order, best_makespan,
                 start_makespan, n_accepted};
    HIP_TRY(launch_check_orders(*d, B, order, order_stride, (hipStream_t)stream));
    const hipError_t e = launch_order_search(*d, a, (hipStream_t)stream);
    if (e == hipErrorNotSupported) {
        set_error("graph outside what the order search handles");
        return TICTAC_ERR_UNSUPPORTED;
    }
    HIP_TRY(e);
    return TICTAC_OK;
}

const char *tictac_last_error(void) { return g_err; }

const char *tictac_version(void) { return "0.1"; }

}  // extern "C"
