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
    if (c->vocab < 1 || c->vocab > 0x7FFFFFFFLL) { *why = "vocab out of range"; return false; }
    if (c->dim < 4 || c->dim > TENSAIR_MAX_DIM || c->dim % 4) { *why = "dim must be a multiple of 4 in 4..1024"; return false; }
    if (c->row_stride < c->dim || c->row_stride % 4) { *why = "row_stride must be >= dim and a multiple of 4"; return false; }
    if (c->dtype != TENSAIR_F32 && c->dtype != TENSAIR_BF16) { *why = "unknown dtype"; return false; }
    if (c->window < 1 || c->window > 1024) { *why = "window out of range"; return false; }
    if (c->negatives < 0 || c->negatives > 65535) { *why = "negatives out of range"; return false; }
    if (c->max_centers < 1) { *why = "max_centers must be positive"; return false; }
    if (c->max_peers < 0 || c->max_peers > TENSAIR_MAX_PEERS) { *why = "max_peers out of range"; return false; }
    if (c->worker_id >= 65536u) { *why = "worker_id must be below 65536"; return false; }
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
    s.passes = (kb + 10) / 11;
    s.bits = (kb + s.passes - 1) / s.passes;
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

struct tensair_model {
    tensair_config cfg;
    Sizes sz;
    void *w_in, *w_out;
    // carved from the caller's workspace
    u32 *thr;
    int *alias;
    int *status;
    u32 *keys[3], *vals[2];
    u32 *counts_out, *totals_out, *counts_in, *totals_in;
    int *seg_of, *seg_start;
    int *long_cnt, *long_list;
    int *blk_heads, *blk_weight;
    int *pair_center;
    float *g, *center_part, *center_loss, *part_out, *part_in;
    u32 *start[2];
    u64 *mask[2];
    std::vector<uint32_t> h_thr;
    std::vector<int32_t> h_alias;
    // second stream for the part of the gradient calculation that does not depend on the forward
    // pass (sort + segments); forked from and joined to the caller's stream with events
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr, ev_index = nullptr;
    // set by tensair_step: the index of the coming apply is built on the second stream, next to
    // the reductions, as soon as the own row ids exist
    const ApplyArgs *fused_apply = nullptr;
    bool fused_index_done = false;
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
    const size_t K1 = (size_t)c.max_peers + 1;
    char *p;
    p = take(V * 4); if (m) m->thr = (u32 *)p;
    p = take(V * 4); if (m) m->alias = (int *)p;
    p = take(256); if (m) m->status = (int *)p;
    for (int i = 0; i < 3; ++i) { p = take(NE * 4); if (m) m->keys[i] = (u32 *)p; }
    for (int i = 0; i < 2; ++i) { p = take(NE * 4); if (m) m->vals[i] = (u32 *)p; }
    p = take((size_t)s.nd * s.nblk_out * 4); if (m) m->counts_out = (u32 *)p;
    p = take((size_t)s.nd * 4); if (m) m->totals_out = (u32 *)p;
    p = take((size_t)s.nd * s.nblk_in * 4); if (m) m->counts_in = (u32 *)p;
    p = take((size_t)s.nd * 4); if (m) m->totals_in = (u32 *)p;
    p = take(NE * 4); if (m) m->seg_of = (int *)p;
    p = take((NE + 2) * 4); if (m) m->seg_start = (int *)p;   // out-side rows at 0, in-side at Omax+1
    p = take(256); if (m) m->long_cnt = (int *)p;
    p = take((size_t)(s.tiles_out + s.tiles_in) * 4); if (m) m->long_list = (int *)p;
    p = take((size_t)(s.sblk_out + s.sblk_in) * 4); if (m) m->blk_heads = (int *)p;
    p = take((size_t)(s.sblk_out + s.sblk_in) * 4); if (m) m->blk_weight = (int *)p;
    p = take((size_t)s.Pmax * 4); if (m) m->pair_center = (int *)p;
    p = take((size_t)s.Omax * 4); if (m) m->g = (float *)p;
    p = take((size_t)s.Bmax * D * 4); if (m) m->center_part = (float *)p;
    p = take((size_t)s.Bmax * 4); if (m) m->center_loss = (float *)p;
    p = take((size_t)s.tiles_out * 2 * D * 4); if (m) m->part_out = (float *)p;
    p = take((size_t)s.tiles_in * 2 * D * 4); if (m) m->part_in = (float *)p;
    for (int t = 0; t < 2; ++t) {
        p = take((size_t)(s.words + 1) * K1 * 4); if (m) m->start[t] = (u32 *)p;
        p = take((size_t)s.words * K1 * 8); if (m) m->mask[t] = (u64 *)p;
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
       PF_BEGIN_APPLY, PF_APPLY_INDEX, PF_APPLY_UPDATE };

void mark(tensair_model *m, int tag, hipStream_t st)
{
    if (m->prof_level == 0) return;
    if (m->prof_level == 1 && tag != PF_APPLY_INDEX && tag != PF_APPLY_UPDATE) return;
    if (m->prof_marks.size() >= 65536) return;
    hipEvent_t ev;
    if (m->prof_used < m->prof_pool.size()) {
        ev = m->prof_pool[m->prof_used];
    } else {
        if (hipEventCreate(&ev) != hipSuccess) return;
        m->prof_pool.push_back(ev);
    }
    ++m->prof_used;
    if (hipEventRecord(ev, st) == hipSuccess) m->prof_marks.emplace_back(tag, ev);
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

}  // namespace

extern "C" {

const char *tensair_last_error(void) { return g_err; }

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
        hipEventCreateWithFlags(&m->ev_join, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&m->ev_index, hipEventDisableTiming) != hipSuccess) {
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

int tensair_sgns_grad(tensair_model *m, const int32_t *tokens, int64_t n_tokens, int64_t center_begin,
                      int32_t n_centers, uint32_t epoch, tensair_sparse_grad *grad_out, float *mean_loss,
                      int32_t *negatives_dbg, int32_t *seg_offsets_in, int32_t *seg_offsets_out, void *stream)
{
    if (!m || !tokens || !grad_out) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    const tensair_config &c = m->cfg;
    if (n_tokens < 1 || center_begin < 0 || n_centers < 0 || center_begin + n_centers > n_tokens)
        return fail(TENSAIR_EINVAL, "center range [%lld, +%d) outside the stream of %lld tokens",
                    (long long)center_begin, n_centers, (long long)n_tokens);
    if (n_centers > c.max_centers)
        return fail(TENSAIR_ECAPACITY, "n_centers %d > max_centers %d", n_centers, c.max_centers);
    if (epoch >= 65536u) return fail(TENSAIR_EINVAL, "epoch must be below 65536");
    int rc;
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
    const i64 O = P * Np1;

    BatchDesc b;
    b.tok = tokens;
    b.T = n_tokens;
    b.begin = center_begin;
    b.n_centers = n_centers;
    b.w = c.window;
    b.N = c.negatives;
    b.pair_base = pairs_before(center_begin, n_tokens, c.window);
    b.P = P;

    // Streams.  The sort and the segment scan only need the keys, the forward pass the keys and the
    // tables, the reductions both: the sort runs on the library's second stream next to the forward
    // pass (fork/join by events).  Inside tensair_step the second stream then builds the index of
    // the coming apply while the reductions run on the caller's stream.  When
    // every stage is being timed (profile level 2) everything is serialised on the caller's stream.
    const bool overlap = m->prof_level < 2;
    const bool fuse = overlap && m->fused_apply != nullptr;
    hipStream_t s_sort = overlap ? m->side : st;
    mark(m, PF_BEGIN_GRAD, st);
    // 1. keys: out-side occurrences at [0, O), in-side centers at [Omax, Omax + n_centers)
    tn_launch_build_keys(b, c.vocab, m->thr, m->alias, c.seed, c.worker_id, epoch, m->keys[0],
                         m->keys[0] + s.Omax, m->pair_center, negatives_dbg, m->status, st);
    mark(m, PF_KEYS, st);
    if (overlap) {
        HIP_TRY(hipEventRecord(m->ev_fork, st));
        HIP_TRY(hipStreamWaitEvent(m->side, m->ev_fork, 0));
    }

    // 2. forward on the unsorted keys (the sort never writes their buffer): g per occurrence,
    //    per-center share of the W_in gradient, loss terms
    FwdArgs f;
    f.w_in = m->w_in;
    f.w_out = m->w_out;
    f.V = c.vocab;
    f.dtype = c.dtype;
    f.D = c.dim;
    f.stride = c.row_stride;
    f.b = b;
    f.out_keys = m->keys[0];
    f.g = m->g;
    f.center_part = m->center_part;
    f.center_loss = mean_loss ? m->center_loss : nullptr;   // loss terms only on request
    f.inv_P = 1.0f / (float)P;
    tn_launch_forward(f, st);
    if (mean_loss) tn_launch_loss(m->center_loss, n_centers, f.inv_P, mean_loss, st);
    mark(m, PF_FORWARD, st);

    // 3. stable sort of both key lists by row id
    RadixProb ro, ri;
    for (int i = 0; i < 3; ++i) {
        ro.keys[i] = m->keys[i];
        ri.keys[i] = m->keys[i] + s.Omax;
    }
    for (int i = 0; i < 2; ++i) {
        ro.vals[i] = m->vals[i];
        ri.vals[i] = m->vals[i] + s.Omax;
    }
    ro.n = (int)O;
    ro.nblk = (int)((O + TN_RADIX_TILE - 1) / TN_RADIX_TILE);
    ro.counts = m->counts_out;
    ro.totals = m->totals_out;
    ri.n = n_centers;
    ri.nblk = (n_centers + TN_RADIX_TILE - 1) / TN_RADIX_TILE;
    ri.counts = m->counts_in;
    ri.totals = m->totals_in;
    int kb = 1;
    const int cur = tn_launch_radix_sort(ro, ri, s.key_bits, s_sort, &kb);
    mark(m, PF_SORT, st);

    // 4. unique row ids, segment index per sorted entry
    SegProb so, si;
    so.keys = ro.keys[kb];
    so.vals = ro.vals[cur];
    so.n = (int)O;
    so.nblk = (int)((O + TN_SCAN_TILE - 1) / TN_SCAN_TILE);
    so.blk_heads = m->blk_heads;
    so.blk_weight = m->blk_weight;
    so.seg_of = m->seg_of;
    so.seg_start = m->seg_start;
    so.long_cnt = m->long_cnt;
    so.row_ids = grad_out->out.row_ids;
    so.n_rows = grad_out->out.n_rows;
    so.seg_offsets = seg_offsets_out;
    so.capacity = grad_out->out.capacity;
    so.weighted = 0;
    si.keys = ri.keys[kb];
    si.vals = ri.vals[cur];
    si.n = n_centers;
    si.nblk = (n_centers + TN_SCAN_TILE - 1) / TN_SCAN_TILE;
    si.blk_heads = m->blk_heads + s.sblk_out;
    si.blk_weight = m->blk_weight + s.sblk_out;
    si.seg_of = m->seg_of + s.Omax;
    si.seg_start = m->seg_start + s.Omax + 1;
    si.long_cnt = m->long_cnt + 1;
    si.row_ids = grad_out->in.row_ids;
    si.n_rows = grad_out->in.n_rows;
    si.seg_offsets = seg_offsets_in;
    si.capacity = grad_out->in.capacity;
    si.weighted = 1;
    tn_launch_segments(so, si, center_begin, n_tokens, c.window, m->status, s_sort);
    mark(m, PF_SEGMENTS, st);
    if (overlap) {
        HIP_TRY(hipEventRecord(m->ev_join, m->side));
        HIP_TRY(hipStreamWaitEvent(st, m->ev_join, 0));
    }
    if (fuse) {   // off the critical path: the reductions run meanwhile, the apply waits for ev_index
        tn_launch_apply_clear(*m->fused_apply, m->side);
        tn_launch_apply_index(*m->fused_apply, 0, m->fused_apply->n_src, m->side);
        HIP_TRY(hipEventRecord(m->ev_index, m->side));
        m->fused_index_done = true;
    }

    // 5. segmented reductions: duplicates of a row summed in sorted (= occurrence) order
    SegReduceArgs r;
    memset(&r, 0, sizeof(r));
    r.D = c.dim;
    r.n = n_centers;
    r.vals = si.vals;
    r.seg_of = si.seg_of;
    r.seg_start = si.seg_start;
    r.long_cnt = si.long_cnt;
    r.long_list = m->long_list + s.tiles_out;
    r.out_rows = grad_out->in.row_grads;
    r.part = m->part_in;
    r.mode = 1;
    r.center_part = m->center_part;
    tn_launch_segreduce(r, st);
    mark(m, PF_REDUCE_IN, st);
    r.n = (int)O;
    r.vals = so.vals;
    r.seg_of = so.seg_of;
    r.seg_start = so.seg_start;
    r.long_cnt = so.long_cnt;
    r.long_list = m->long_list;
    r.out_rows = grad_out->out.row_grads;
    r.part = m->part_out;
    r.mode = 0;
    r.g = m->g;
    r.pair_center = m->pair_center;
    r.Np1 = Np1;
    r.table = m->w_in;
    r.dtype = c.dtype;
    r.stride = c.row_stride;
    tn_launch_segreduce(r, st);
    mark(m, PF_REDUCE_OUT, st);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

static int fill_apply_src(ApplyArgs &a, int k, const tensair_sparse_grad *g, const char *what)
{
    const tensair_sparse_rows *side[2] = {&g->in, &g->out};
    for (int t = 0; t < 2; ++t) {
        const tensair_sparse_rows &r = *side[t];
        if (!r.n_rows || !r.row_ids || !r.row_grads) return fail(TENSAIR_EINVAL, "%s: NULL pointer", what);
        if (r.capacity < 0 || r.capacity > 0x7FFFFFFFLL) return fail(TENSAIR_EINVAL, "%s: bad capacity", what);
        a.src[t][k].ids = r.row_ids;
        a.src[t][k].rows = r.row_grads;
        a.src[t][k].n_rows = r.n_rows;
        a.src[t][k].capacity = r.capacity;
    }
    return TENSAIR_OK;
}

static int make_apply_args(tensair_model *m, const tensair_sparse_grad *own, const tensair_sparse_grad *peers,
                           int32_t n_peers, float lr, ApplyArgs &a)
{
    const tensair_config &c = m->cfg;
    if (n_peers < 0 || n_peers > c.max_peers)
        return fail(TENSAIR_ECAPACITY, "n_peers %d outside 0..max_peers %d", n_peers, c.max_peers);
    if (n_peers > 0 && !peers) return fail(TENSAIR_EINVAL, "peers is NULL");
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
    for (int t = 0; t < 2; ++t) {
        a.start[t] = m->start[t];
        a.mask[t] = m->mask[t];
    }
    int rc;
    if (own && (rc = fill_apply_src(a, 0, own, "own"))) return rc;
    for (int k = 0; k < n_peers; ++k)
        if ((rc = fill_apply_src(a, 1 + k, &peers[k], "peer"))) return rc;
    return TENSAIR_OK;
}

int tensair_dasgd_apply(tensair_model *m, const tensair_sparse_grad *own, const tensair_sparse_grad *peers,
                        int32_t n_peers, float lr, void *stream)
{
    if (!m) return fail(TENSAIR_EINVAL, "model is NULL");
    ApplyArgs a;
    int rc = make_apply_args(m, own, peers, n_peers, lr, a);
    if (rc) return rc;
    if (!own && n_peers == 0) return TENSAIR_OK;
    hipStream_t st = (hipStream_t)stream;
    mark(m, PF_BEGIN_APPLY, st);
    tn_launch_apply_clear(a, st);
    tn_launch_apply_index(a, 0, a.n_src, st);
    mark(m, PF_APPLY_INDEX, st);
    tn_launch_apply_update(a, st);
    mark(m, PF_APPLY_UPDATE, st);
    HIP_TRY(hipGetLastError());
    return TENSAIR_OK;
}

int tensair_step(tensair_model *m, const int32_t *tokens, int64_t n_tokens, int64_t center_begin,
                 int32_t n_centers, uint32_t epoch, const tensair_sparse_grad *peers, int32_t n_peers,
                 float lr, tensair_sparse_grad *own_out, float *mean_loss, void *stream)
{
    if (!m || !own_out) return fail(TENSAIR_EINVAL, "NULL pointer argument");
    // validate the apply arguments before anything is enqueued
    ApplyArgs a;
    int rc = make_apply_args(m, own_out, peers, n_peers, lr, a);
    if (rc) return rc;
    m->fused_apply = &a;
    m->fused_index_done = false;
    rc = tensair_sgns_grad(m, tokens, n_tokens, center_begin, n_centers, epoch, own_out, mean_loss, nullptr,
                           nullptr, nullptr, stream);
    m->fused_apply = nullptr;
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    mark(m, PF_BEGIN_APPLY, st);
    if (m->fused_index_done) {
        HIP_TRY(hipStreamWaitEvent(st, m->ev_index, 0));
    } else {
        tn_launch_apply_clear(a, st);
        tn_launch_apply_index(a, 0, a.n_src, st);
    }
    mark(m, PF_APPLY_INDEX, st);
    tn_launch_apply_update(a, st);
    mark(m, PF_APPLY_UPDATE, st);
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

#ifdef TENSAIR_DEBUG
extern "C" int tensair_debug_ptrs(tensair_model *m, void **out)
{
    out[0] = m->part_out; out[1] = m->part_in; out[2] = m->seg_of; out[3] = m->seg_start;
    out[4] = m->vals[0]; out[5] = m->vals[1]; out[6] = m->g; out[7] = m->pair_center;
    return 0;
}
#endif

int tensair_copy_probe(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || (bytes & 15) || (((uintptr_t)dst | (uintptr_t)src) & 15))
        return fail(TENSAIR_EINVAL, "copy_probe: pointers and size must be multiples of 16");
    tn_launch_copy_probe(dst, src, bytes, (hipStream_t)stream);
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
        if (tag == PF_BEGIN_GRAD || tag == PF_BEGIN_APPLY) continue;
        if (m->prof_level == 1 && tag != PF_APPLY_UPDATE) continue;
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
        if (m->ev_join) (void)hipEventDestroy(m->ev_join);
        if (m->ev_index) (void)hipEventDestroy(m->ev_index);
        if (m->side) (void)hipStreamDestroy(m->side);
    }
    delete m;
    return TENSAIR_OK;
}

}  // extern "C"
