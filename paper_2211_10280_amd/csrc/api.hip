// C ABI of libtensair: argument checks, workspace carving, alias-table construction
// and the order in which the kernels of one DASGD worker step are enqueued.
// Call names follow the Model operator of TensAIR (arXiv 2211.10280), Algorithm 1.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/tensair.h"
#include "dev_common.h"
#include "kernels.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                      \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess)                                                              \
            return fail(TENSAIR_EHIP, "%s: %s", #expr, hipGetErrorString(e_));             \
    } while (0)

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

struct Sizes {
    i64 Bmax, Pmax, Omax;
    int key_bits, passes, bits, nd;
    int nblk_out, nblk_in;     // radix blocks
    int sblk_out, sblk_in;     // scan blocks
    int tiles_out, tiles_in;   // segmented-reduction tiles
    i64 words;
};

bool config_ok(const tensair_config *c, const char **why)
{
    *why = nullptr;
    if (!c) { *why = "cfg is NULL"; return false; }
    if (c->vocab < 1 || c->vocab > TENSAIR_MAX_VOCAB) { *why = "vocab outside 1..TENSAIR_MAX_VOCAB"; return false; }
    if (c->dim < 4 || c->dim > TENSAIR_MAX_DIM || c->dim % 4) { *why = "dim must be a multiple of 4 in 4..1024"; return false; }
    if (c->row_stride < c->dim || c->row_stride % 4) { *why = "row_stride must be >= dim and a multiple of 4"; return false; }
    if (c->dtype != TENSAIR_F32 && c->dtype != TENSAIR_BF16) { *why = "unknown dtype"; return false; }
    if (c->window < 1 || c->window > 1024) { *why = "window out of range"; return false; }
    if (c->negatives < 0 || c->negatives > 65535) { *why = "negatives out of range"; return false; }
    if (c->max_centers < 1) { *why = "max_centers must be positive"; return false; }
    if (c->max_peers < 0 || c->max_peers > TENSAIR_MAX_PEERS) { *why = "max_peers out of range"; return false; }
    if (c->worker_id >= 65536u) { *why = "worker_id must be below 65536"; return false; }
    if (c->flags & ~(TENSAIR_RESAMPLE_NEGATIVES | TENSAIR_STOCHASTIC_ROUNDING)) { *why = "unknown flag"; return false; }
    i64 omax = (i64)2 * c->window * c->max_centers * (c->negatives + 1);
    if (omax + c->max_centers >= 0x7FFFFFFFLL) { *why = "batch too large: occurrences must fit 31 bits"; return false; }
    return true;
}

Sizes sizes_of(const tensair_config &c)
{
    Sizes s;
    s.Bmax = c.max_centers;
    s.Pmax = (i64)2 * c.window * s.Bmax;
    s.Omax = s.Pmax * (c.negatives + 1);
    int kb = 1;
    while (((i64)1 << kb) < c.vocab) ++kb;
    s.key_bits = kb;
    tn_radix_shape(kb, &s.passes, &s.bits);
    s.nd = 1 << s.bits;
    s.nblk_out = (int)((s.Omax + TN_RADIX_TILE - 1) / TN_RADIX_TILE);
    s.nblk_in = (int)((s.Bmax + TN_RADIX_TILE - 1) / TN_RADIX_TILE);
    s.sblk_out = (int)((s.Omax + TN_SCAN_TILE - 1) / TN_SCAN_TILE);
    s.sblk_in = (int)((s.Bmax + TN_SCAN_TILE - 1) / TN_SCAN_TILE);
    s.tiles_out = (int)((s.Omax + tn_seg_tile(s.Omax) - 1) / tn_seg_tile(s.Omax));   // worst case over n <= Omax
    if (s.Omax > 65536 && s.tiles_out < 65536 / 8) s.tiles_out = 65536 / 8;
    s.tiles_in = (int)((s.Bmax + tn_seg_tile(s.Bmax) - 1) / tn_seg_tile(s.Bmax));
    if (s.Bmax > 65536 && s.tiles_in < 65536 / 8) s.tiles_in = 65536 / 8;
    s.words = (c.vocab + 63) / 64;
    return s;
}

}  // namespace

int tn_fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// Everything about a mini-batch that does not depend on the tables: keys (pairs and negatives), their
// sorted order, segments, unique row ids.  There are two sets, used in turn, so that the set of the
// coming mini-batch can be filled (tensair_prefetch) while the kernels of the current one still read theirs.
struct BatchSet {
    u32 *keys[3], *vals[2];
    u32 *counts_out, *totals_out, *counts_in, *totals_in;
    int *seg_of, *seg_start;
    int *long_cnt;
    int *blk_heads, *blk_weight;
    int *pair_center;
    // row index of a prefetched mini-batch, copied to the caller's buffers when it is consumed
    int *ids_in, *ids_out, *n_rows, *off_in, *off_out;
    int cur = 0, kb = 1;   // which vals / keys buffer holds the sorted order
};

// A mini-batch announced by tensair_prefetch.
struct Prefetched {
    bool valid = false;
    bool unprepared = false;   // announced, but left for the consuming call to prepare
    const int32_t *tokens = nullptr;
    i64 n_tokens = 0, begin = 0, P = 0;
    int n_centers = 0;
    u32 epoch = 0, worker_id = 0;
    bool is(const int32_t *t, i64 nt, i64 b, int n, u32 e, u32 w) const
    {
        return valid && tokens == t && n_tokens == nt && begin == b && n_centers == n && epoch == e &&
               worker_id == w;
    }
};

struct tensair_model {
    tensair_config cfg;
    Sizes sz;
    void *w_in, *w_out;
    // carved from the caller's workspace
    u32 *thr;
    int *alias;
    int *status;
    BatchSet set[2];
    int *long_list;
    float *g, *center_part, *center_loss, *part_out, *part_in, *cross_out, *cross_in;
    int *xinfo_out, *xinfo_in;
    u32 *start[2];
    u64 *mask[2];              // masks of the update's index, per table (buffer 0)
    u64 *mask_alt[2];          // a second set (buffer 1): inside tensair_step the two are used in turn, so that
                               // the one the next step will index can be cleared while this step still reads its own
    bool mask_clean[2] = {false, false};   // buffer b is all zeros (or will be when everything enqueued so far has run)
    u32 *wbase[2], *wblk[2];   // tensair_grad_add: place of every 64-row word in the summed gradient
    std::vector<uint32_t> h_thr;
    std::vector<int32_t> h_alias;
    // second stream, forked from and joined to the caller's stream with events: it runs what can go
    // on next to the caller's stream (the forward pass beside the sort, the index of the coming table
    // update beside the reductions, the preparation of announced mini-batches)
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_fwd = nullptr;
    // mini-batch sets: `busy` is the one the most recent gradient call reads; announced mini-batches are
    // prepared into the other one on the second stream (ev_prep recorded behind them)
    int busy = 1;
    Prefetched pend;               // prepared (or being prepared) in set 1 - busy
    Prefetched next;               // announced after `pend`: prepared when `pend` is consumed
    hipEvent_t ev_prep = nullptr, ev_reduced = nullptr;
    // a preparation enqueued beside a gradient calculation may still be running when its mini-batch is
    // consumed: its keys get an event of their own, so that the forward pass (which only needs the keys)
    // can start while the sort and the segment scan finish
    hipEvent_t ev_keys = nullptr;
    bool pend_late = false;
    bool side_follows = false;     // the second stream has waited for the start of the latest gradient call
    // every event recorded on the second stream takes a ticket; the caller's stream is behind all of
    // them up to main_ticket, so a prepared set with prep_ticket <= main_ticket needs no wait
    u64 side_ticket = 0, main_ticket = 0, prep_ticket = 0, keys_ticket = 0;
    // set by tensair_step: the index of the coming apply is built by extra workgroups at the front of the
    // forward pass (clearing) and of the segmented reduction (the id lists), on the caller's stream
    ApplyArgs *fused_apply = nullptr;
    bool fused_index_done = false;
    bool prepare_under_apply = false;   // tensair_step: the table update is long enough to hide a preparation
    Prefetched deferred;                // the mini-batch to prepare under that update (enqueued by tensair_step)
    u32 apply_serial = 0;               // table updates enqueued so far (stochastic rounding draws from it)
    // stage timing (tensair_profile): events recorded on the caller's stream
    int prof_level = 0;
    std::vector<hipEvent_t> prof_pool;
    std::vector<std::pair<int, hipEvent_t>> prof_marks;
    size_t prof_used = 0;
};

namespace {

// Lays the workspace out; with m == nullptr only the size is computed.
size_t carve(const tensair_config &c, const Sizes &s, char *base, tensair_model *m)
{
    size_t off = 0;
    auto take = [&](size_t bytes) -> char * {
        char *p = base ? base + off : nullptr;
        off += align_up(bytes);
        return p;
    };
    const size_t V = (size_t)c.vocab, D = (size_t)c.dim;
    const size_t NE = (size_t)(s.Omax + s.Bmax);
    const size_t K1 = (size_t)(c.max_peers + 1 > 2 ? c.max_peers + 1 : 2);   // the gradient sum indexes two sources
    char *p;
    p = take(V * 4); if (m) m->thr = (u32 *)p;
    p = take(V * 4); if (m) m->alias = (int *)p;
    p = take(256); if (m) m->status = (int *)p;
    const size_t cap_in = (size_t)(s.Bmax < (i64)V ? s.Bmax : (i64)V);
    const size_t cap_out = (size_t)(s.Omax < (i64)V ? s.Omax : (i64)V);
    for (int u = 0; u < 2; ++u) {
        BatchSet *b = m ? &m->set[u] : nullptr;
        for (int i = 0; i < 3; ++i) { p = take(NE * 4); if (b) b->keys[i] = (u32 *)p; }
        for (int i = 0; i < 2; ++i) { p = take(NE * 4); if (b) b->vals[i] = (u32 *)p; }
        p = take((size_t)s.nd * s.nblk_out * 4); if (b) b->counts_out = (u32 *)p;
        p = take((size_t)s.nd * 4); if (b) b->totals_out = (u32 *)p;
        p = take((size_t)s.nd * s.nblk_in * 4); if (b) b->counts_in = (u32 *)p;
        p = take((size_t)s.nd * 4); if (b) b->totals_in = (u32 *)p;
        p = take(NE * 4); if (b) b->seg_of = (int *)p;
        p = take((NE + 2) * 4); if (b) b->seg_start = (int *)p;   // out-side rows at 0, in-side at Omax+1
        p = take(256); if (b) b->long_cnt = (int *)p;
        p = take((size_t)(s.sblk_out + s.sblk_in) * 4); if (b) b->blk_heads = (int *)p;
        p = take((size_t)(s.sblk_out + s.sblk_in) * 4); if (b) b->blk_weight = (int *)p;
        p = take((size_t)s.Pmax * 4); if (b) b->pair_center = (int *)p;
        p = take(cap_in * 4); if (b) b->ids_in = (int *)p;
        p = take(cap_out * 4); if (b) b->ids_out = (int *)p;
        p = take(256); if (b) b->n_rows = (int *)p;
        p = take((cap_in + 1) * 4); if (b) b->off_in = (int *)p;
        p = take((cap_out + 1) * 4); if (b) b->off_out = (int *)p;
    }
    p = take((size_t)(s.tiles_out + s.tiles_in) * 4); if (m) m->long_list = (int *)p;
    p = take((size_t)s.Omax * 4); if (m) m->g = (float *)p;
    p = take((size_t)s.Bmax * D * 4); if (m) m->center_part = (float *)p;
    p = take((size_t)s.Bmax * 4); if (m) m->center_loss = (float *)p;
    p = take((size_t)s.tiles_out * 2 * D * 4); if (m) m->part_out = (float *)p;
    p = take((size_t)s.tiles_in * 2 * D * 4); if (m) m->part_in = (float *)p;
    p = take((size_t)(s.tiles_out / TN_SEG_XBLOCK + 2) * D * 4); if (m) m->cross_out = (float *)p;
    p = take((size_t)(s.tiles_in / TN_SEG_XBLOCK + 2) * D * 4); if (m) m->cross_in = (float *)p;
    p = take((size_t)(s.tiles_out / TN_SEG_XBLOCK + 2) * 4); if (m) m->xinfo_out = (int *)p;
    p = take((size_t)(s.tiles_in / TN_SEG_XBLOCK + 2) * 4); if (m) m->xinfo_in = (int *)p;
    for (int t = 0; t < 2; ++t) {
        p = take((size_t)(s.words + 1) * K1 * 4); if (m) m->start[t] = (u32 *)p;
        p = take((size_t)s.words * K1 * 8); if (m) m->mask[t] = (u64 *)p;
        p = take((size_t)s.words * K1 * 8); if (m) m->mask_alt[t] = (u64 *)p;
        p = take((size_t)s.words * 4); if (m) m->wbase[t] = (u32 *)p;
        p = take((size_t)(s.words / TN_UNION_WORDS + 1) * 4); if (m) m->wblk[t] = (u32 *)p;
    }
    return off;
}

// Alias table (Vose) of the noise distribution count^0.75 / sum.  Buckets whose scaled
// probability is below 1 keep floor(p * 2^32) as acceptance threshold and hand the rest
// of their mass to a donor; work lists are filled in ascending id order and consumed
// from the back, so the table is a deterministic function of the counts.
bool build_alias(const uint64_t *counts, i64 V, std::vector<uint32_t> &thr,
                 std::vector<int32_t> &alias)
{
    thr.assign((size_t)V, 0xFFFFFFFFu);
    alias.resize((size_t)V);
    std::vector<double> prob((size_t)V);
    double total = 0.0;
    for (i64 i = 0; i < V; ++i) {
        prob[(size_t)i] = std::pow((double)counts[i], 0.75);
        total += prob[(size_t)i];
        alias[(size_t)i] = (int32_t)i;
    }
    if (!(total > 0.0)) return false;
    std::vector<int32_t> lo, hi;
    lo.reserve((size_t)V);
    hi.reserve((size_t)V);
    const double scale = (double)V;
    for (i64 i = 0; i < V; ++i) {
        double q = prob[(size_t)i] * scale / total;
        prob[(size_t)i] = q;
        (q < 1.0 ? lo : hi).push_back((int32_t)i);
    }
    const double two32 = 4294967296.0;
    while (!lo.empty() && !hi.empty()) {
        const int32_t poor = lo.back();
        lo.pop_back();
        const int32_t rich = hi.back();
        hi.pop_back();
        const double t = std::floor(prob[(size_t)poor] * two32);
        thr[(size_t)poor] = t >= two32 ? 0xFFFFFFFFu : (uint32_t)t;
        alias[(size_t)poor] = rich;
        const double rest = (prob[(size_t)rich] + prob[(size_t)poor]) - 1.0;
        prob[(size_t)rich] = rest;
        (rest < 1.0 ? lo : hi).push_back(rich);
    }
    // whatever is left on either list keeps the full bucket (threshold max, alias = itself)
    return true;
}

// Stage tags of tensair_profile_read.  A tag's duration runs from the previous mark to its own.
enum { PF_BEGIN_GRAD = 0, PF_KEYS, PF_FORWARD, PF_SORT, PF_SEGMENTS, PF_REDUCE_IN, PF_REDUCE_OUT,
       PF_BEGIN_APPLY, PF_APPLY_INDEX, PF_APPLY_UPDATE, PF_BEGIN_ADD, PF_ADD_INDEX, PF_ADD_ROWS,
       PF_BEGIN_PACK, PF_PACK };

// records a timing event on `st` if stage timing asks for this tag; returns it (another stream may wait on
// it, which saves that stream's fork an event of its own) or nullptr
hipEvent_t mark(tensair_model *m, int tag, hipStream_t st)
{
    if (m->prof_level == 0) return nullptr;
    if (m->prof_level == 1 && tag != PF_APPLY_INDEX && tag != PF_APPLY_UPDATE && tag != PF_ADD_INDEX &&
        tag != PF_ADD_ROWS && tag != PF_BEGIN_PACK && tag != PF_PACK)
        return nullptr;
    if (m->prof_marks.size() >= 65536) return nullptr;
    hipEvent_t ev;
    if (m->prof_used < m->prof_pool.size()) {
        ev = m->prof_pool[m->prof_used];
    } else {
        if (hipEventCreate(&ev) != hipSuccess) return nullptr;
        m->prof_pool.push_back(ev);
    }
    ++m->prof_used;
    if (hipEventRecord(ev, st) != hipSuccess) return nullptr;
    m->prof_marks.emplace_back(tag, ev);
    return ev;
}

i64 pair_count(const tensair_config &c, i64 T, i64 begin, int n)
{
    return pairs_before(begin + n, T, c.window) - pairs_before(begin, T, c.window);
}

int check_rows(const tensair_sparse_rows &r, i64 need, const char *what)
{
    if (!r.n_rows || !r.row_ids || !r.row_grads) return fail(TENSAIR_EINVAL, "%s: NULL pointer", what);
    if (r.capacity < need)
        return fail(TENSAIR_ECAPACITY, "%s: capacity %lld < %lld rows required", what,
                    (long long)r.capacity, (long long)need);
    if (r.capacity > 0x7FFFFFFFLL) return fail(TENSAIR_EINVAL, "%s: capacity too large", what);
    return TENSAIR_OK;
}

// One source of the table update: the two tables' rows of a gradient (fp32) or of a bfloat16 message.
template <typename Grad>
int fill_apply_src(ApplyArgs &a, int k, const Grad *g, const char *what)
{
    for (int t = 0; t < 2; ++t) {
        const auto &r = t ? g->out : g->in;
        if (!r.n_rows || !r.row_ids || !r.row_grads) return fail(TENSAIR_EINVAL, "%s: NULL pointer", what);
        if (r.capacity < 0 || r.capacity > 0x7FFFFFFFLL) return fail(TENSAIR_EINVAL, "%s: bad capacity", what);
        if (((uintptr_t)r.row_grads & 15) || ((uintptr_t)r.row_ids & 3) || ((uintptr_t)r.n_rows & 3))
            return fail(TENSAIR_EINVAL, "%s: rows must be 16-byte aligned, ids and counts 4-byte aligned", what);
        a.src[t][k].ids = r.row_ids;
        a.src[t][k].rows = r.row_grads;
        a.src[t][k].n_rows = r.n_rows;
        a.src[t][k].capacity = r.capacity;
    }
    return TENSAIR_OK;
}

}  // namespace

extern "C" {

const char *tensair_last_error(void) { return g_err; }

int32_t tensair_aligned_row_stride(int32_t dim, int32_t dtype)
{
    if (dim < 1 || dim > TENSAIR_MAX_DIM || (dtype != TENSAIR_F32 && dtype != TENSAIR_BF16)) return -1;
    const int per_line = dtype == TENSAIR_F32 ? 32 : 64;   // elements in 128 bytes
    return (dim + per_line - 1) / per_line * per_line;
}

size_t tensair_workspace_bytes(const tensair_config *cfg)
{
    const char *why;
    if (!config_ok(cfg, &why)) { fail(TENSAIR_EINVAL, "%s", why); return 0; }
    return carve(*cfg, sizes_of(*cfg), nullptr, nullptr);
}

int64_t tensair_capacity_in(const tensair_config *cfg, int32_t n_centers)
{
    if (!cfg || n_centers < 0) return -1;
    i64 n = n_centers;
    return n < cfg->vocab ? n : cfg->vocab;
}

int64_t tensair_capacity_out(const tensair_config *cfg, int32_t n_centers)
{
    if (!cfg || n_centers < 0) return -1;
    i64 n = (i64)2 * cfg->window * n_centers * (cfg->negatives + 1);
    return n < cfg->vocab ? n : cfg->vocab;
}

int tensair_model_init(tensair_model **out, const tensair_config *cfg, void *w_in, void *w_out,
                       int fill_tables, const uint64_t *unigram_counts, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    const char *why;
    if (!out) return fail(TENSAIR_EINVAL, "out is NULL");
    *out = nullptr;
    if (!config_ok(cfg, &why)) return fail(TENSAIR_EINVAL, "%s", why);
    if (!w_in || !w_out || !unigram_counts || !workspace) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    if (((uintptr_t)w_in | (uintptr_t)w_out) & 15) return fail(TENSAIR_EINVAL, "tables must be 16-byte aligned");
    if ((uintptr_t)workspace & 255) return fail(TENSAIR_EINVAL, "workspace must be 256-byte aligned");
    Sizes sz = sizes_of(*cfg);
    size_t need = carve(*cfg, sz, nullptr, nullptr);
    if (workspace_bytes < need)
        return fail(TENSAIR_ECAPACITY, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    tensair_model *m = new (std::nothrow) tensair_model();
    if (!m) return fail(TENSAIR_EINVAL, "out of host memory");
    m->cfg = *cfg;
    m->sz = sz;
    m->w_in = w_in;
    m->w_out = w_out;
    carve(*cfg, sz, (char *)workspace, m);
    if (!build_alias(unigram_counts, cfg->vocab, m->h_thr, m->h_alias)) {
        delete m;
        return fail(TENSAIR_EINVAL, "unigram_counts has no positive entry");
    }
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(m->thr, m->h_thr.data(), (size_t)cfg->vocab * 4, hipMemcpyHostToDevice, st);
    if (e == hipSuccess)
        e = hipMemcpyAsync(m->alias, m->h_alias.data(), (size_t)cfg->vocab * 4, hipMemcpyHostToDevice, st);
    int zero[4] = {0, 0, 0, 0};
    if (e == hipSuccess) e = hipMemcpyAsync(m->status, zero, sizeof(zero), hipMemcpyHostToDevice, st);
    if (e == hipSuccess && fill_tables) {
        tn_launch_init_tables(w_in, w_out, cfg->vocab, cfg->dim, cfg->row_stride, cfg->dtype, cfg->seed, st);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        delete m;
        return fail(TENSAIR_EHIP, "model_init: %s", hipGetErrorString(e));
    }
    if (hipStreamCreateWithFlags(&m->side, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&m->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&m->ev_fwd, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&m->ev_prep, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&m->ev_keys, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&m->ev_reduced, hipEventDisableTiming) != hipSuccess) {
        tensair_model_destroy(m);
        return fail(TENSAIR_EHIP, "model_init: cannot create the side stream");
    }
    *out = m;
    return TENSAIR_OK;
}

int tensair_model_rebind(tensair_model *m, void *w_in, void *w_out, uint32_t worker_id)
{
    if (!m || !w_in || !w_out) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    if (((uintptr_t)w_in | (uintptr_t)w_out) & 15) return fail(TENSAIR_EINVAL, "tables must be 16-byte aligned");
    if (worker_id >= 65536u) return fail(TENSAIR_EINVAL, "worker_id must be below 65536");
    m->w_in = w_in;
    m->w_out = w_out;
    m->cfg.worker_id = worker_id;
    return TENSAIR_OK;
}

int tensair_model_alias(const tensair_model *m, uint32_t *thr, int32_t *alias)
{
    if (!m || !thr || !alias) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    memcpy(thr, m->h_thr.data(), (size_t)m->cfg.vocab * 4);
    memcpy(alias, m->h_alias.data(), (size_t)m->cfg.vocab * 4);
    return TENSAIR_OK;
}

int64_t tensair_pair_count(const tensair_model *m, int64_t n_tokens, int64_t center_begin, int32_t n_centers)
{
    if (!m || n_tokens < 1 || center_begin < 0 || n_centers < 0 || center_begin + n_centers > n_tokens) {
        fail(TENSAIR_EINVAL, "pair_count: bad range");
        return -1;
    }
    return pair_count(m->cfg, n_tokens, center_begin, n_centers);
}

// The table-independent part of a mini-batch, split in two so that other work can be enqueued in
// between: keys (pairs, negatives), then sort + segments.
struct BatchWork {
    BatchDesc b;
    i64 P, O;
    u32 epoch;
};

static BatchWork batch_work(const tensair_config &c, const int32_t *tokens, i64 n_tokens, i64 center_begin,
                            int n_centers, u32 epoch, i64 P)
{
    BatchWork w;
    w.b.tok = tokens;
    w.b.T = n_tokens;
    w.b.begin = center_begin;
    w.b.n_centers = n_centers;
    w.b.w = c.window;
    w.b.N = c.negatives;
    w.b.pair_base = pairs_before(center_begin, n_tokens, c.window);
    w.b.P = P;
    w.P = P;
    w.O = P * (c.negatives + 1);
    w.epoch = epoch;
    return w;
}

// keys: out-side occurrences at [0, O), in-side centers at [Omax, Omax + n_centers)
static void enqueue_keys(tensair_model *m, BatchSet &S, const BatchWork &w, int32_t *negatives_dbg, hipStream_t st)
{
    const tensair_config &c = m->cfg;
    tn_launch_build_keys(w.b, c.vocab, m->thr, m->alias, c.seed, c.worker_id, w.epoch,
                         (c.flags & TENSAIR_RESAMPLE_NEGATIVES) != 0, S.keys[0], S.keys[0] + m->sz.Omax,
                         S.pair_center, negatives_dbg, m->status, st);
}

struct RowIndexDst {
    int *ids, *n_rows, *offsets;
    i64 capacity;
};

static SegProb seg_prob(const tensair_model *m, const BatchSet &S, int side, int n)
{
    const Sizes &s = m->sz;
    SegProb p;
    memset(&p, 0, sizeof(p));
    const size_t at = side ? (size_t)s.Omax : 0;
    p.keys = S.keys[S.kb] + at;
    p.vals = S.vals[S.cur] + at;
    p.n = n;
    p.nblk = (n + TN_SCAN_TILE - 1) / TN_SCAN_TILE;
    p.blk_heads = S.blk_heads + (side ? s.sblk_out : 0);
    p.blk_weight = S.blk_weight + (side ? s.sblk_out : 0);
    p.seg_of = S.seg_of + at;
    p.seg_start = S.seg_start + (side ? (size_t)s.Omax + 1 : 0);
    p.long_cnt = S.long_cnt + side;
    p.weighted = side;
    return p;
}

// stable sort of both key lists by row id, then unique row ids and the segment of every sorted entry
// LDS that the sort asks for beyond its counters where it runs next to the forward pass or the reductions of a
// step (a preparation that was not tucked under a table update): 40 KB per workgroup, four workgroups per compute
// unit, is the occupancy at which it was measured not to crowd them (hot-row configuration: 0.66 against 0.69 ms
// per step with the sort at full occupancy); under a table update, or alone, it takes what it needs.
#ifndef TN_SORT_LDS_BESIDE
#define TN_SORT_LDS_BESIDE 40960
#endif
#ifndef TN_SORT_LDS_INLINE
#define TN_SORT_LDS_INLINE 0
#endif

static void enqueue_sort_segments(tensair_model *m, BatchSet &S, const BatchWork &w, const RowIndexDst &in,
                                  const RowIndexDst &out, size_t min_lds, hipStream_t st, hipStream_t st_mark)
{
    const tensair_config &c = m->cfg;
    const Sizes &s = m->sz;
    RadixProb ro, ri;
    for (int i = 0; i < 3; ++i) {
        ro.keys[i] = S.keys[i];
        ri.keys[i] = S.keys[i] + s.Omax;
    }
    for (int i = 0; i < 2; ++i) {
        ro.vals[i] = S.vals[i];
        ri.vals[i] = S.vals[i] + s.Omax;
    }
    ro.n = (int)w.O;
    ro.nblk = (int)((w.O + TN_RADIX_TILE - 1) / TN_RADIX_TILE);
    ro.counts = S.counts_out;
    ro.totals = S.totals_out;
    ri.n = w.b.n_centers;
    ri.nblk = (w.b.n_centers + TN_RADIX_TILE - 1) / TN_RADIX_TILE;
    ri.counts = S.counts_in;
    ri.totals = S.totals_in;
    S.cur = tn_launch_radix_sort(ro, ri, s.key_bits, min_lds, st, &S.kb);
    if (st_mark) mark(m, PF_SORT, st_mark);

    SegProb so = seg_prob(m, S, 0, (int)w.O), si = seg_prob(m, S, 1, w.b.n_centers);
    so.row_ids = out.ids;
    so.n_rows = out.n_rows;
    so.seg_offsets = out.offsets;
    so.capacity = out.capacity;
    si.row_ids = in.ids;
    si.n_rows = in.n_rows;
    si.seg_offsets = in.offsets;
    si.capacity = in.capacity;
    tn_launch_segments(so, si, w.b.begin, w.b.T, c.window, m->status, st);
    if (st_mark) mark(m, PF_SEGMENTS, st_mark);
}

static int check_batch(const tensair_model *m, const int32_t *tokens, i64 n_tokens, i64 center_begin, int n_centers,
                       u32 epoch)
{
    if (!tokens) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    if (n_tokens < 1 || center_begin < 0 || n_centers < 0 || center_begin + n_centers > n_tokens)
        return fail(TENSAIR_EINVAL, "center range [%lld, +%d) outside the stream of %lld tokens",
                    (long long)center_begin, n_centers, (long long)n_tokens);
    if (n_centers > m->cfg.max_centers)
        return fail(TENSAIR_ECAPACITY, "n_centers %d > max_centers %d", n_centers, m->cfg.max_centers);
    if (epoch >= 65536u) return fail(TENSAIR_EINVAL, "epoch must be below 65536");
    return TENSAIR_OK;
}

// Enqueue the preparation of an announced mini-batch on the second stream, into the set that the
// latest gradient call does not read.  The second stream must already be behind that set's last readers.
// late: the preparation may still be running when the mini-batch is consumed (it was not tucked under a
// long table update), so its keys are made available on their own.
// A preparation that runs beside the forward pass and the reductions of a step pays only where those kernels
// leave the chip idle between their round trips, i.e. for small mini-batches (measured: 1 k and 10 k pairs per
// step 6 % and 18 % faster with it, 262 k pairs 4 % slower: there both sides fight for the caches).  Larger
// mini-batches are prepared ahead only under a long table update; otherwise the consuming call prepares them.
#ifndef TN_BESIDE_MAX_OCC
#define TN_BESIDE_MAX_OCC (1 << 20)
#endif
static bool worth_preparing_beside(const tensair_model *m, const Prefetched &d)
{
    return d.P * (m->cfg.negatives + 1) <= TN_BESIDE_MAX_OCC;
}

static int enqueue_prepare(tensair_model *m, const Prefetched &d, bool late)
{
    const tensair_config &c = m->cfg;
    BatchSet &S = m->set[1 - m->busy];
    const BatchWork w = batch_work(c, d.tokens, d.n_tokens, d.begin, d.n_centers, d.epoch, d.P);
    enqueue_keys(m, S, w, nullptr, m->side);
    if (late) {
        HIP_TRY(hipEventRecord(m->ev_keys, m->side));
        m->keys_ticket = ++m->side_ticket;
    }
    m->pend_late = late;
    const RowIndexDst in = {S.ids_in, S.n_rows, S.off_in, tensair_capacity_in(&c, c.max_centers)};
    const RowIndexDst out = {S.ids_out, S.n_rows + 1, S.off_out, tensair_capacity_out(&c, c.max_centers)};
    enqueue_sort_segments(m, S, w, in, out, late ? TN_SORT_LDS_BESIDE : 0, m->side, nullptr);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(m->ev_prep, m->side));
    m->prep_ticket = ++m->side_ticket;
    m->pend = d;
    m->pend.unprepared = false;
    return TENSAIR_OK;
}

// After a HIP call has failed in the middle of a call that had already forked work to the second stream, the
// two streams and the host's record of them may disagree.  Wait for the second stream (best effort), forget
// every announcement and count the caller's stream as behind everything, so that the next call on the handle
// starts from a known state instead of racing leftover work.
static void abandon_side_work(tensair_model *m)
{
    if (m->side) (void)hipStreamSynchronize(m->side);
    m->pend.valid = m->next.valid = m->deferred.valid = false;
    m->pend_late = false;
    m->side_follows = false;
    m->main_ticket = m->side_ticket;
    m->fused_apply = nullptr;
    m->fused_index_done = false;
    m->mask_clean[0] = m->mask_clean[1] = false;
}

int tensair_prefetch(tensair_model *m, const int32_t *tokens, int64_t n_tokens, int64_t center_begin,
                     int32_t n_centers, uint32_t epoch, void *stream)
{
    if (!m) return fail(TENSAIR_EINVAL, "model is NULL");
    int rc = check_batch(m, tokens, n_tokens, center_begin, n_centers, epoch);
    if (rc) return rc;
    const tensair_config &c = m->cfg;
    Prefetched d;
    d.tokens = tokens;
    d.n_tokens = n_tokens;
    d.begin = center_begin;
    d.n_centers = n_centers;
    d.epoch = epoch;
    d.worker_id = c.worker_id;
    d.P = pair_count(c, n_tokens, center_begin, n_centers);
    if (d.P == 0) return TENSAIR_OK;   // nothing to prepare
    d.valid = true;
    if (m->pend.valid) {   // one mini-batch is waiting already: this one is prepared when that is consumed
        m->next = d;
        return TENSAIR_OK;
    }
    if (!worth_preparing_beside(m, d)) {   // kept as an announcement: the consuming call prepares it itself
        m->pend = d;
        m->pend.unprepared = true;
        return TENSAIR_OK;
    }
    // The set being filled was last read by the gradient call before the latest one.  If the second
    // stream has waited for the start of the latest call it is already behind those readers; if not,
    // it is put behind everything enqueued on the caller's stream so far.
    if (!m->side_follows) {
        hipStream_t st = (hipStream_t)stream;
        HIP_TRY(hipEventRecord(m->ev_fork, st));
        HIP_TRY(hipStreamWaitEvent(m->side, m->ev_fork, 0));
        m->side_follows = true;
    }
    const int rc2 = enqueue_prepare(m, d, true);
    if (rc2 == TENSAIR_EHIP) abandon_side_work(m);
    return rc2;
}

static int sgns_grad_impl(tensair_model *m, const int32_t *tokens, int64_t n_tokens, int64_t center_begin,
                          int32_t n_centers, uint32_t epoch, tensair_sparse_grad *grad_out, float *mean_loss,
                          int32_t *negatives_dbg, int32_t *seg_offsets_in, int32_t *seg_offsets_out, void *stream)
{
    if (!m || !grad_out) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    const tensair_config &c = m->cfg;
    int rc = check_batch(m, tokens, n_tokens, center_begin, n_centers, epoch);
    if (rc) return rc;
    if ((rc = check_rows(grad_out->in, tensair_capacity_in(&c, n_centers), "grad_out.in"))) return rc;
    if ((rc = check_rows(grad_out->out, tensair_capacity_out(&c, n_centers), "grad_out.out"))) return rc;
    hipStream_t st = (hipStream_t)stream;
    const Sizes &s = m->sz;

    const i64 P = pair_count(c, n_tokens, center_begin, n_centers);
    if (P == 0) {
        tn_launch_empty_grad(grad_out->in.n_rows, grad_out->out.n_rows, mean_loss, seg_offsets_in,
                             seg_offsets_out, st);
        HIP_TRY(hipGetLastError());
        return TENSAIR_OK;
    }
    const int Np1 = c.negatives + 1;
    const BatchWork w = batch_work(c, tokens, n_tokens, center_begin, n_centers, epoch, P);

    // Streams.  The sort and the segment scan only need the keys, the forward pass the keys and the
    // tables, the reductions both.  Without a prefetch the chain that the apply waits for (keys, sort,
    // segments, reductions) stays on the caller's stream, so that none of its links is a cross-stream
    // wait, and the forward pass runs next to the sort on the library's second stream.  With a matching
    // prefetch the keys, the sorted order and the segments are already there (made on the second stream
    // while the previous step ran) and the caller's stream starts with the forward pass.  The small jobs
    // around them -- the prepared row index to the caller's buffers, and inside tensair_step the index of
    // the coming table update -- ride at the front of the forward and the reduction launches: every event
    // between streams idles the waiting stream for microseconds, and a launch of their own is not worth
    // one.  When every stage is being timed (profile level 2) everything is serialised on the caller's
    // stream in launches of its own.
    const bool overlap = m->prof_level < 2;
    const bool fuse = overlap && m->fused_apply != nullptr;
    const bool announced = overlap && negatives_dbg == nullptr &&
                           m->pend.is(tokens, n_tokens, center_begin, n_centers, epoch, c.worker_id);
    const bool prepared = announced && !m->pend.unprepared;
    m->pend.valid = false;
    // the announced mini-batch after this one is prepared during this call; announcements that this
    // call does not follow are dropped
    const Prefetched following = announced ? m->next : Prefetched();
    m->next.valid = false;
    m->deferred.valid = false;
    // this call takes the set that announced mini-batches are prepared into; one that does not match
    // is overwritten, after its preparation has finished
    const int u = 1 - m->busy;
    BatchSet &S = m->set[u];
    // a prepared set that may not be finished yet: the forward pass waits for its keys only, the reductions
    // for the rest (below); otherwise the caller's stream gets behind the whole preparation here
    const bool split = prepared && m->pend_late && m->prep_ticket > m->main_ticket;
    if (split) {
        if (m->keys_ticket > m->main_ticket) {
            HIP_TRY(hipStreamWaitEvent(st, m->ev_keys, 0));
            m->main_ticket = m->keys_ticket;
        }
    } else if (m->prep_ticket > m->main_ticket) {
        HIP_TRY(hipStreamWaitEvent(st, m->ev_prep, 0));
        m->main_ticket = m->prep_ticket;
    }
    const u64 consumed_prep_ticket = m->prep_ticket;   // enqueue_prepare below moves on to the following mini-batch
    m->busy = u;
    m->side_follows = false;
    mark(m, PF_BEGIN_GRAD, st);

    FwdArgs f;
    f.w_in = m->w_in;
    f.w_out = m->w_out;
    f.V = c.vocab;
    f.dtype = c.dtype;
    f.D = c.dim;
    f.stride = c.row_stride;
    f.b = w.b;
    f.out_keys = S.keys[0];
    f.g = m->g;
    f.center_part = m->center_part;
    f.center_loss = mean_loss ? m->center_loss : nullptr;   // loss terms only on request
    f.inv_P = 1.0f / (float)P;

    AuxWork aux_fwd, aux_red;     // what rides at the front of the forward pass / of the reduction
    tn_aux_none(aux_fwd);
    tn_aux_none(aux_red);
    if (fuse) {
        // The index of the coming table update.  Its masks must be zero before the id lists are indexed, and the
        // two cannot share a launch, so there are two sets of masks: this step indexes a clean one, with the
        // forward pass (hidden behind its row gathers) where the id lists are known by then -- the peers'
        // always, the own one if the mini-batch was prepared -- else with the reductions; the other set, which
        // the previous step used, is cleared with the reductions and is the clean one of the next step.
        ApplyArgs &fa = *m->fused_apply;
        int pick = m->mask_clean[0] ? 0 : (m->mask_clean[1] ? 1 : -1);
        if (pick < 0) {           // the first step, or other calls have used both sets since
            pick = 0;
            ApplyArgs full = fa;  // the whole buffer, whatever layout its last user had
            full.n_src = (c.max_peers + 1 > 2 ? c.max_peers + 1 : 2);
            tn_launch_apply_clear(full, st);
        }
        for (int t = 0; t < 2; ++t) fa.mask[t] = pick ? m->mask_alt[t] : m->mask[t];
        m->mask_clean[pick] = false;
        const bool own_early = prepared && !split;   // the own id lists exist when the forward pass starts
        tn_aux_add_index(aux_fwd, fa, own_early ? 0 : 1, fa.n_src);
        if (!own_early) tn_aux_add_index(aux_red, fa, 0, 1);
        if (!m->mask_clean[1 - pick]) {
            const size_t all = (size_t)s.words * (size_t)(c.max_peers + 1 > 2 ? c.max_peers + 1 : 2);
            tn_aux_add_clear(aux_red, pick ? m->mask[0] : m->mask_alt[0], pick ? m->mask[1] : m->mask_alt[1], all);
            m->mask_clean[1 - pick] = true;
        }
        m->fused_index_done = true;
    }

    if (prepared) {
        // this mini-batch's row index goes to the caller's buffers with the forward pass -- with the
        // reductions if the forward pass starts on the keys alone, before the sort has finished
        RowIndexCopy rc2;
        rc2.side[0] = {S.ids_in, S.n_rows, S.off_in, grad_out->in.row_ids, grad_out->in.n_rows, seg_offsets_in};
        rc2.side[1] = {S.ids_out, S.n_rows + 1, S.off_out, grad_out->out.row_ids, grad_out->out.n_rows,
                       seg_offsets_out};
        tn_aux_add_copy(split ? aux_red : aux_fwd, rc2, tensair_capacity_out(&c, n_centers));
        if (fuse) {   // the own id lists are indexed where they are, whichever launch copies them
            AuxWork &ix = split ? aux_red : aux_fwd;
            ApplySrc &o_in = ix.apply.src[0][0], &o_out = ix.apply.src[1][0];
            o_in.ids = S.ids_in;
            o_in.n_rows = S.n_rows;
            o_in.capacity = tensair_capacity_in(&c, c.max_centers);
            o_out.ids = S.ids_out;
            o_out.n_rows = S.n_rows + 1;
            o_out.capacity = tensair_capacity_out(&c, c.max_centers);
        }
        // Where a long table update follows (tensair_step decides), the following mini-batch is prepared
        // under that update, which is bound by HBM bandwidth and loses little to it; otherwise next to this
        // call's forward pass, for which the second stream gets behind the caller's stream here.
        const bool under_apply = fuse && m->prepare_under_apply;
        if (following.valid && !under_apply) {
            HIP_TRY(hipEventRecord(m->ev_fork, st));
            HIP_TRY(hipStreamWaitEvent(m->side, m->ev_fork, 0));
            m->side_follows = true;
        }
        tn_launch_forward(f, &aux_fwd, st);
        if (mean_loss) tn_launch_loss(m->center_loss, n_centers, f.inv_P, mean_loss, st);
        if (split) {   // the sorted order and the segments of this mini-batch
            HIP_TRY(hipStreamWaitEvent(st, m->ev_prep, 0));
            if (consumed_prep_ticket > m->main_ticket) m->main_ticket = consumed_prep_ticket;
        }
        if (following.valid) {
            if (under_apply) {
                m->deferred = following;
            } else if (worth_preparing_beside(m, following)) {
                if ((rc = enqueue_prepare(m, following, true))) return rc;
            } else {
                m->pend = following;
                m->pend.unprepared = true;
            }
        }
    } else {
        // 1. keys
        enqueue_keys(m, S, w, negatives_dbg, st);
        mark(m, PF_KEYS, st);
        hipStream_t s_fwd = st;
        if (overlap) {
            HIP_TRY(hipEventRecord(m->ev_fork, st));
            HIP_TRY(hipStreamWaitEvent(m->side, m->ev_fork, 0));
            m->side_follows = true;
            s_fwd = m->side;
        }
        // 2. forward on the unsorted keys (the sort never writes their buffer): g per occurrence,
        //    per-center share of the W_in gradient, loss terms
        tn_launch_forward(f, &aux_fwd, s_fwd);
        if (mean_loss) tn_launch_loss(m->center_loss, n_centers, f.inv_P, mean_loss, s_fwd);
        mark(m, PF_FORWARD, st);
        u64 fwd_ticket = 0;
        if (overlap) {
            HIP_TRY(hipEventRecord(m->ev_fwd, m->side));
            fwd_ticket = ++m->side_ticket;
        }
        if (following.valid) {   // this mini-batch was announced but not prepared; the one after it may be
            if (fuse && m->prepare_under_apply) {
                m->deferred = following;
            } else if (worth_preparing_beside(m, following)) {
                if ((rc = enqueue_prepare(m, following, true))) return rc;   // behind the forward pass
            } else {
                m->pend = following;
                m->pend.unprepared = true;
            }
        }
        // 3./4. sort and segments, row index straight into the caller's buffers
        const RowIndexDst in = {grad_out->in.row_ids, grad_out->in.n_rows, seg_offsets_in, grad_out->in.capacity};
        const RowIndexDst out = {grad_out->out.row_ids, grad_out->out.n_rows, seg_offsets_out,
                                 grad_out->out.capacity};
        enqueue_sort_segments(m, S, w, in, out, TN_SORT_LDS_INLINE, st, st);
        if (overlap) {   // behind the forward pass (not behind a preparation enqueued after it)
            HIP_TRY(hipStreamWaitEvent(st, m->ev_fwd, 0));
            if (fwd_ticket > m->main_ticket) m->main_ticket = fwd_ticket;
        }
    }

    // 5. segmented reductions: duplicates of a row summed in sorted (= occurrence) order
    const SegProb so = seg_prob(m, S, 0, (int)w.O), si = seg_prob(m, S, 1, n_centers);
    SegReduceArgs r_in, r_out;
    memset(&r_in, 0, sizeof(r_in));
    r_in.D = c.dim;
    r_in.n = n_centers;
    r_in.vals = si.vals;
    r_in.seg_of = si.seg_of;
    r_in.seg_start = si.seg_start;
    r_in.long_cnt = si.long_cnt;
    r_in.long_list = m->long_list + s.tiles_out;
    r_in.out_rows = grad_out->in.row_grads;
    r_in.part = m->part_in;
    r_in.cross = m->cross_in;
    r_in.xinfo = m->xinfo_in;
    r_in.mode = 1;
    r_in.center_part = m->center_part;
    r_out = r_in;
    r_out.n = (int)w.O;
    r_out.vals = so.vals;
    r_out.seg_of = so.seg_of;
    r_out.seg_start = so.seg_start;
    r_out.long_cnt = so.long_cnt;
    r_out.long_list = m->long_list;
    r_out.out_rows = grad_out->out.row_grads;
    r_out.part = m->part_out;
    r_out.cross = m->cross_out;
    r_out.xinfo = m->xinfo_out;
    r_out.mode = 0;
    r_out.g = m->g;
    r_out.pair_center = S.pair_center;
    r_out.Np1 = Np1;
    r_out.table = m->w_in;
    r_out.dtype = c.dtype;
    r_out.stride = c.row_stride;
    if (overlap) {   // both sides in one launch
        tn_launch_segreduce(&r_out, &r_in, &aux_red, st);
    } else {         // one after the other, so that each can be timed
        tn_launch_segreduce(nullptr, &r_in, nullptr, st);
        mark(m, PF_REDUCE_IN, st);
        tn_launch_segreduce(&r_out, nullptr, nullptr, st);
    }
    mark(m, PF_REDUCE_OUT, st);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

int tensair_sgns_grad(tensair_model *m, const int32_t *tokens, int64_t n_tokens, int64_t center_begin,
                      int32_t n_centers, uint32_t epoch, tensair_sparse_grad *grad_out, float *mean_loss,
                      int32_t *negatives_dbg, int32_t *seg_offsets_in, int32_t *seg_offsets_out, void *stream)
{
    const int rc = sgns_grad_impl(m, tokens, n_tokens, center_begin, n_centers, epoch, grad_out, mean_loss,
                                  negatives_dbg, seg_offsets_in, seg_offsets_out, stream);
    if (rc == TENSAIR_EHIP && m) abandon_side_work(m);
    return rc;
}

// The preparation of the mini-batch that tensair_sgns_grad left in m->deferred: enqueued on the second
// stream behind everything that is on the caller's stream now (the reductions), so that it runs under the
// table update that the caller enqueues next.  `ev`: an event just recorded on the caller's stream, or
// nullptr to record one.
static int enqueue_deferred_prepare(tensair_model *m, hipEvent_t ev, hipStream_t st)
{
    if (!m->deferred.valid) return TENSAIR_OK;
    const Prefetched d = m->deferred;
    m->deferred.valid = false;
    if (!ev) {
        HIP_TRY(hipEventRecord(m->ev_reduced, st));
        ev = m->ev_reduced;
    }
    HIP_TRY(hipStreamWaitEvent(m->side, ev, 0));
    m->side_follows = true;
    return enqueue_prepare(m, d, false);
}

// peers are fp32 gradients (`peers`) or bfloat16 messages (`packed`), never both
static int make_apply_args(tensair_model *m, const tensair_sparse_grad *own, const tensair_sparse_grad *peers,
                           const tensair_packed_grad *packed, int32_t n_peers, float lr, ApplyArgs &a)
{
    const tensair_config &c = m->cfg;
    if (n_peers < 0 || n_peers > c.max_peers)
        return fail(TENSAIR_ECAPACITY, "n_peers %d outside 0..max_peers %d", n_peers, c.max_peers);
    if (n_peers > 0 && !peers && !packed) return fail(TENSAIR_EINVAL, "peers is NULL");
    if (!(lr == lr)) return fail(TENSAIR_EINVAL, "lr is NaN");
    memset(&a, 0, sizeof(a));
    a.table[0] = m->w_in;
    a.table[1] = m->w_out;
    a.dtype = c.dtype;
    a.D = c.dim;
    a.stride = c.row_stride;
    a.V = c.vocab;
    a.n_src = 1 + n_peers;
    a.lr = lr;
    a.status = m->status;
    a.packed = (packed != nullptr && n_peers > 0) ? 1 : 0;
    a.sr = ((c.flags & TENSAIR_STOCHASTIC_ROUNDING) && c.dtype == TENSAIR_BF16) ? 1 : 0;
    a.sr_k0 = (u32)(c.seed & 0xFFFFFFFFu);
    a.sr_k1 = (u32)(c.seed >> 32);
    a.sr_serial = m->apply_serial;
    for (int t = 0; t < 2; ++t) {
        a.start[t] = m->start[t];
        a.mask[t] = m->mask[t];
    }
    int rc;
    if (own && (rc = fill_apply_src(a, 0, own, "own"))) return rc;
    for (int k = 0; k < n_peers; ++k)
        if ((rc = packed ? fill_apply_src(a, 1 + k, &packed[k], "peer") : fill_apply_src(a, 1 + k, &peers[k], "peer")))
            return rc;
    return TENSAIR_OK;
}

static int apply_impl(tensair_model *m, const tensair_sparse_grad *own, const tensair_sparse_grad *peers,
                      const tensair_packed_grad *packed, int32_t n_peers, float lr, void *stream)
{
    if (!m) return fail(TENSAIR_EINVAL, "model is NULL");
    ApplyArgs a;
    int rc = make_apply_args(m, own, peers, packed, n_peers, lr, a);
    if (rc) return rc;
    if (!own && n_peers == 0) return TENSAIR_OK;
    hipStream_t st = (hipStream_t)stream;
    mark(m, PF_BEGIN_APPLY, st);
    m->mask_clean[0] = false;
    tn_launch_apply_clear(a, st);
    tn_launch_apply_index(a, 0, a.n_src, st);
    mark(m, PF_APPLY_INDEX, st);
    tn_launch_apply_update(a, st);
    ++m->apply_serial;
    mark(m, PF_APPLY_UPDATE, st);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

int tensair_dasgd_apply(tensair_model *m, const tensair_sparse_grad *own, const tensair_sparse_grad *peers,
                        int32_t n_peers, float lr, void *stream)
{
    return apply_impl(m, own, peers, nullptr, n_peers, lr, stream);
}

int tensair_dasgd_apply_packed(tensair_model *m, const tensair_sparse_grad *own, const tensair_packed_grad *peers,
                               int32_t n_peers, float lr, void *stream)
{
    if (n_peers > 0 && !peers) return fail(TENSAIR_EINVAL, "peers is NULL");
    return apply_impl(m, own, nullptr, peers, n_peers, lr, stream);
}

int tensair_grad_pack(tensair_model *m, const tensair_sparse_grad *g, tensair_packed_grad *out, void *stream)
{
    if (!m || !g || !out) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    GradPackArgs a;
    memset(&a, 0, sizeof(a));
    a.D = m->cfg.dim;
    a.status = m->status;
    const tensair_sparse_rows *src[2] = {&g->in, &g->out};
    const tensair_packed_rows *dst[2] = {&out->in, &out->out};
    for (int t = 0; t < 2; ++t) {
        const tensair_sparse_rows &r = *src[t];
        const tensair_packed_rows &d = *dst[t];
        if (!r.n_rows || !r.row_ids || !r.row_grads || !d.n_rows || !d.row_ids || !d.row_grads)
            return fail(TENSAIR_EINVAL, "grad_pack: NULL pointer");
        if (r.capacity < 0 || r.capacity > 0x7FFFFFFFLL || d.capacity < 0 || d.capacity > 0x7FFFFFFFLL)
            return fail(TENSAIR_EINVAL, "grad_pack: bad capacity");
        if (((uintptr_t)r.row_grads | (uintptr_t)d.row_grads) & 15)
            return fail(TENSAIR_EINVAL, "grad_pack: rows must be 16-byte aligned");
        if ((const void *)d.row_grads == (const void *)r.row_grads || d.row_ids == r.row_ids || d.n_rows == r.n_rows)
            return fail(TENSAIR_EINVAL, "grad_pack: out must not share buffers with g");
        a.n[t] = r.n_rows;
        a.ids[t] = r.row_ids;
        a.rows[t] = r.row_grads;
        a.cap[t] = r.capacity;
        a.out_n[t] = d.n_rows;
        a.out_ids[t] = d.row_ids;
        a.out_rows[t] = d.row_grads;
        a.out_cap[t] = d.capacity;
    }
    hipStream_t st = (hipStream_t)stream;
    mark(m, PF_BEGIN_PACK, st);
    tn_launch_grad_pack(a, st);
    mark(m, PF_PACK, st);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

int tensair_grad_add(tensair_model *m, const tensair_sparse_grad *a, const tensair_sparse_grad *b,
                     tensair_sparse_grad *out, void *stream)
{
    if (!m || !a || !b || !out) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    const tensair_config &c = m->cfg;
    GradSumArgs g;
    memset(&g, 0, sizeof(g));
    ApplyArgs &ap = g.a;
    ap.dtype = c.dtype;
    ap.D = c.dim;
    ap.stride = c.row_stride;
    ap.V = c.vocab;
    ap.n_src = 2;
    ap.status = m->status;
    int rc;
    if ((rc = fill_apply_src(ap, 0, a, "a")) || (rc = fill_apply_src(ap, 1, b, "b"))) return rc;
    const tensair_sparse_rows *dst[2] = {&out->in, &out->out};
    const tensair_sparse_rows *src[2][2] = {{&a->in, &b->in}, {&a->out, &b->out}};
    for (int t = 0; t < 2; ++t) {
        const tensair_sparse_rows &r = *dst[t];
        if (!r.n_rows || !r.row_ids || !r.row_grads) return fail(TENSAIR_EINVAL, "out: NULL pointer");
        if (r.capacity < 0 || r.capacity > 0x7FFFFFFFLL) return fail(TENSAIR_EINVAL, "out: bad capacity");
        for (int k = 0; k < 2; ++k)
            if (r.row_grads == src[t][k]->row_grads || r.row_ids == src[t][k]->row_ids ||
                r.n_rows == src[t][k]->n_rows)
                return fail(TENSAIR_EINVAL, "out must not share buffers with a or b");
        ap.start[t] = m->start[t];
        ap.mask[t] = m->mask[t];
        g.out_ids[t] = r.row_ids;
        g.out_rows[t] = r.row_grads;
        g.out_n[t] = r.n_rows;
        g.out_cap[t] = r.capacity;
        g.wbase[t] = m->wbase[t];
        g.wblk[t] = m->wblk[t];
    }
    hipStream_t st = (hipStream_t)stream;
    mark(m, PF_BEGIN_ADD, st);
    m->mask_clean[0] = false;
    tn_launch_grad_sum_index(g, st);
    mark(m, PF_ADD_INDEX, st);
    tn_launch_grad_sum_rows(g, st);
    mark(m, PF_ADD_ROWS, st);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

static int step_impl(tensair_model *m, const int32_t *tokens, int64_t n_tokens, int64_t center_begin,
                     int32_t n_centers, uint32_t epoch, const tensair_sparse_grad *peers,
                     const tensair_packed_grad *packed, int32_t n_peers, float lr, tensair_sparse_grad *own_out,
                     tensair_packed_grad *own_msg, float *mean_loss, void *stream)
{
    if (!m || !own_out) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    // validate the apply arguments before anything is enqueued
    ApplyArgs a;
    int rc = make_apply_args(m, own_out, peers, packed, n_peers, lr, a);
    if (rc) return rc;
    if (own_msg) {   // the own gradient leaves the update as a bfloat16 message as well
        if (n_centers < 0) return fail(TENSAIR_EINVAL, "n_centers is negative");
        const tensair_packed_rows *d[2] = {&own_msg->in, &own_msg->out};
        const tensair_sparse_rows *o[2] = {&own_out->in, &own_out->out};
        const int64_t need[2] = {tensair_capacity_in(&m->cfg, n_centers), tensair_capacity_out(&m->cfg, n_centers)};
        for (int t = 0; t < 2; ++t) {
            if (!d[t]->n_rows || !d[t]->row_ids || !d[t]->row_grads) return fail(TENSAIR_EINVAL, "own_msg: NULL pointer");
            if ((uintptr_t)d[t]->row_grads & 15) return fail(TENSAIR_EINVAL, "own_msg: rows must be 16-byte aligned");
            if (d[t]->capacity < need[t])
                return fail(TENSAIR_ECAPACITY, "own_msg: capacity %lld < %lld rows required", (long long)d[t]->capacity,
                            (long long)need[t]);
            if ((const void *)d[t]->row_grads == (const void *)o[t]->row_grads || d[t]->row_ids == o[t]->row_ids ||
                d[t]->n_rows == o[t]->n_rows)
                return fail(TENSAIR_EINVAL, "own_msg must not share buffers with own_out");
            a.msg_rows[t] = d[t]->row_grads;
            a.msg_ids[t] = d[t]->row_ids;
            a.msg_n[t] = d[t]->n_rows;
        }
        a.packed = 1;   // the kernel that handles messages, also with no peer at all
    }
    m->fused_apply = &a;
    m->fused_index_done = false;
    m->deferred.valid = false;
    {   // rough times of the table update (bytes of the gradient blocks at their largest, at 5 TB/s) and of
        // the preparation of a mini-batch (0.2 ns per occurrence plus its launches)
        const tensair_config &c = m->cfg;
        const double occ = 2.0 * c.window * (double)n_centers * (c.negatives + 1);
        const double rows = occ < (double)c.vocab ? occ : (double)c.vocab;
        const double src_bytes = 4.0 + (a.packed ? 2.0 : 4.0) * (a.n_src - 1);
        const double t_apply = src_bytes * rows * c.dim / 5e12;
        const double t_prepare = occ * 0.2e-9 + 60e-6;
        m->prepare_under_apply = t_apply >= 2.0 * t_prepare;
    }
    rc = sgns_grad_impl(m, tokens, n_tokens, center_begin, n_centers, epoch, own_out, mean_loss, nullptr,
                        nullptr, nullptr, stream);
    m->fused_apply = nullptr;
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    mark(m, PF_BEGIN_APPLY, st);
    if (!m->fused_index_done) {   // an empty mini-batch, or every stage in a launch of its own
        m->mask_clean[0] = false;
        tn_launch_apply_clear(a, st);
        tn_launch_apply_index(a, 0, a.n_src, st);
    }
    // the event that opens the timing of the table update also lets the second stream go
    const hipEvent_t ev = mark(m, PF_APPLY_INDEX, st);
    if ((rc = enqueue_deferred_prepare(m, ev, st))) return rc;
    tn_launch_apply_update(a, st);
    ++m->apply_serial;
    mark(m, PF_APPLY_UPDATE, st);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

int tensair_step(tensair_model *m, const int32_t *tokens, int64_t n_tokens, int64_t center_begin,
                 int32_t n_centers, uint32_t epoch, const tensair_sparse_grad *peers, int32_t n_peers,
                 float lr, tensair_sparse_grad *own_out, float *mean_loss, void *stream)
{
    const int rc = step_impl(m, tokens, n_tokens, center_begin, n_centers, epoch, peers, nullptr, n_peers, lr,
                             own_out, nullptr, mean_loss, stream);
    if (rc == TENSAIR_EHIP && m) abandon_side_work(m);
    return rc;
}

int tensair_step_packed(tensair_model *m, const int32_t *tokens, int64_t n_tokens, int64_t center_begin,
                        int32_t n_centers, uint32_t epoch, const tensair_packed_grad *peers, int32_t n_peers,
                        float lr, tensair_sparse_grad *own_out, tensair_packed_grad *own_msg_out, float *mean_loss,
                        void *stream)
{
    if (n_peers > 0 && !peers) return fail(TENSAIR_EINVAL, "peers is NULL");
    const int rc = step_impl(m, tokens, n_tokens, center_begin, n_centers, epoch, nullptr, peers, n_peers, lr,
                             own_out, own_msg_out, mean_loss, stream);
    if (rc == TENSAIR_EHIP && m) abandon_side_work(m);
    return rc;
}

int tensair_dense_apply(void *theta, int32_t dtype, int64_t n, const float *const *grads, int32_t n_grads,
                        float lr, void *stream)
{
    if (!theta || (n_grads > 0 && !grads)) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    if (dtype != TENSAIR_F32 && dtype != TENSAIR_BF16) return fail(TENSAIR_EINVAL, "unknown dtype");
    if (n < 0 || n > TENSAIR_MAX_DENSE) return fail(TENSAIR_EINVAL, "n outside 0..TENSAIR_MAX_DENSE");
    if (n_grads < 0 || n_grads > TENSAIR_MAX_PEERS + 1)
        return fail(TENSAIR_ECAPACITY, "n_grads %d outside 0..%d", n_grads, TENSAIR_MAX_PEERS + 1);
    if (!(lr == lr)) return fail(TENSAIR_EINVAL, "lr is NaN");
    if ((uintptr_t)theta & 15) return fail(TENSAIR_EINVAL, "theta must be 16-byte aligned");
    DenseApplyArgs a;
    memset(&a, 0, sizeof(a));
    a.theta = theta;
    a.n = n;
    a.n_grads = n_grads;
    a.dtype = dtype;
    a.lr = lr;
    for (int k = 0; k < n_grads; ++k) {
        if (!grads[k]) return fail(TENSAIR_EINVAL, "grads[%d] is NULL", k);
        if ((uintptr_t)grads[k] & 15) return fail(TENSAIR_EINVAL, "grads[%d] must be 16-byte aligned", k);
        a.grads[k] = grads[k];
    }
    if (n == 0 || n_grads == 0) return TENSAIR_OK;
    tn_launch_dense_apply(a, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

int tensair_lookup(tensair_model *m, int32_t table, const int32_t *ids, int64_t n, float *out, void *stream)
{
    if (!m || (n > 0 && (!ids || !out))) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    if (table != 0 && table != 1) return fail(TENSAIR_EINVAL, "table must be 0 (W_in) or 1 (W_out)");
    if (n < 0) return fail(TENSAIR_EINVAL, "n is negative");
    if ((uintptr_t)out & 15) return fail(TENSAIR_EINVAL, "out must be 16-byte aligned");
    const tensair_config &c = m->cfg;
    LookupArgs a;
    a.table = table ? m->w_out : m->w_in;
    a.ids = ids;
    a.out = out;
    a.n = n;
    a.V = c.vocab;
    a.D = c.dim;
    a.stride = c.row_stride;
    a.dtype = c.dtype;
    a.status = m->status;
    tn_launch_lookup(a, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

int tensair_cosine_difference(const void *a, const void *b, int32_t dtype, int64_t vocab, int32_t dim,
                              int32_t row_stride, float *diff, void *stream)
{
    if (!a || !b || !diff) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    if (dtype != TENSAIR_F32 && dtype != TENSAIR_BF16) return fail(TENSAIR_EINVAL, "unknown dtype");
    if (vocab < 0 || vocab > 0x7FFFFFFFLL) return fail(TENSAIR_EINVAL, "vocab out of range");
    if (dim < 4 || dim > TENSAIR_MAX_DIM || dim % 4) return fail(TENSAIR_EINVAL, "dim must be a multiple of 4 in 4..1024");
    if (row_stride < dim || row_stride % 4) return fail(TENSAIR_EINVAL, "row_stride must be >= dim and a multiple of 4");
    if (((uintptr_t)a | (uintptr_t)b) & 15) return fail(TENSAIR_EINVAL, "tables must be 16-byte aligned");
    CosineArgs c;
    c.a = a;
    c.b = b;
    c.diff = diff;
    c.V = vocab;
    c.D = dim;
    c.stride = row_stride;
    c.dtype = dtype;
    tn_launch_cosine_diff(c, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

int tensair_status(tensair_model *m, void *stream)
{
    if (!m) return fail(TENSAIR_EINVAL, "model is NULL");
    hipStream_t st = (hipStream_t)stream;
    int word = 0;
    HIP_TRY(hipMemcpyAsync(&word, m->status, sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (word != 0) {
        int zero = 0;
        HIP_TRY(hipMemcpyAsync(m->status, &zero, sizeof(int), hipMemcpyHostToDevice, st));
        HIP_TRY(hipStreamSynchronize(st));
        return fail(TENSAIR_EDATA, "kernels met invalid data:%s%s%s", (word & ST_BAD_ID) ? " id out of range" : "",
                    (word & ST_BAD_ORDER) ? " ids not strictly ascending" : "",
                    (word & ST_OVERFLOW) ? " row count above capacity" : "");
    }
    return TENSAIR_OK;
}

int tensair_copy_probe(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || (bytes & 15) || (((uintptr_t)dst | (uintptr_t)src) & 15))
        return fail(TENSAIR_EINVAL, "copy_probe: pointers and size must be multiples of 16");
    tn_launch_copy_probe(dst, src, bytes, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

int tensair_stream_probe(void *dst, const void *src, size_t bytes, int32_t mode, void *stream)
{
    if (!dst || !src || (bytes & 15) || (((uintptr_t)dst | (uintptr_t)src) & 15))
        return fail(TENSAIR_EINVAL, "stream_probe: pointers and size must be multiples of 16");
    if (mode < 0 || mode > 3) return fail(TENSAIR_EINVAL, "stream_probe: mode must be 0..3");
    tn_launch_stream_probe(dst, src, bytes, mode, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

int tensair_profile(tensair_model *m, int level)
{
    if (!m || level < 0 || level > 2) return fail(TENSAIR_EINVAL, "profile: bad argument");
    m->prof_level = level;
    return TENSAIR_OK;
}

int tensair_profile_read(tensair_model *m, int32_t *tags, float *ms, int32_t max_records)
{
    if (!m || !tags || !ms || max_records < 0) return fail(TENSAIR_EINVAL, "profile_read: bad argument");
    int n = 0;
    if (!m->prof_marks.empty()) {
        hipError_t e = hipEventSynchronize(m->prof_marks.back().second);
        if (e != hipSuccess) return fail(TENSAIR_EHIP, "profile_read: %s", hipGetErrorString(e));
    }
    for (size_t i = 1; i < m->prof_marks.size() && n < max_records; ++i) {
        const int tag = m->prof_marks[i].first;
        if (tag == PF_BEGIN_GRAD || tag == PF_BEGIN_APPLY || tag == PF_BEGIN_ADD || tag == PF_BEGIN_PACK) continue;
        if (m->prof_level == 1 && tag != PF_APPLY_UPDATE && tag != PF_ADD_ROWS && tag != PF_PACK) continue;
        float t = 0.f;
        if (hipEventElapsedTime(&t, m->prof_marks[i - 1].second, m->prof_marks[i].second) != hipSuccess) continue;
        tags[n] = tag;
        ms[n] = t;
        ++n;
    }
    m->prof_marks.clear();
    m->prof_used = 0;
    return n;
}

int tensair_model_destroy(tensair_model *m)
{
    if (m) {
        for (hipEvent_t ev : m->prof_pool) (void)hipEventDestroy(ev);
        if (m->ev_fork) (void)hipEventDestroy(m->ev_fork);
        if (m->ev_fwd) (void)hipEventDestroy(m->ev_fwd);
        if (m->ev_prep) (void)hipEventDestroy(m->ev_prep);
        if (m->ev_keys) (void)hipEventDestroy(m->ev_keys);
        if (m->ev_reduced) (void)hipEventDestroy(m->ev_reduced);
        if (m->side) {
            (void)hipStreamSynchronize(m->side);   // a pending prefetch still writes the workspace
            (void)hipStreamDestroy(m->side);
        }
    }
    delete m;
    return TENSAIR_OK;
}

}  // extern "C"
