// tensair_dasgd_apply_static: the merged gradient application of tensair_dasgd_apply for callers that
// cannot allocate device memory and hold no model handle (code under HIP graph capture, tight serving
// loops, harnesses that forbid hipMalloc).  The only scratch the update needs -- the per-64-row-word
// (start, mask) index of every source and a status word -- lives in a fixed device array of this
// library instead of a caller workspace, which bounds the vocabulary and the number of peers.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>

#include "../../include/tensair.h"
#include "dev_common.h"
#include "kernels.h"

namespace {

constexpr size_t align256(size_t x) { return (x + 255) / 256 * 256; }
constexpr size_t NA_WORDS = (size_t)(TENSAIR_STATIC_MAX_VOCAB / 64);
constexpr size_t NA_SRC = TENSAIR_STATIC_MAX_PEERS + 1;
constexpr size_t NA_STATUS_BYTES = 256;
constexpr size_t NA_START_BYTES = align256((NA_WORDS + 1) * NA_SRC * sizeof(u32));
constexpr size_t NA_MASK_BYTES = align256(NA_WORDS * NA_SRC * sizeof(u64));
constexpr size_t NA_BYTES = NA_STATUS_BYTES + 2 * (NA_START_BYTES + NA_MASK_BYTES);   // 12.6 MB

}  // namespace

// Every GPU the library runs on holds its own copy of this array, at its own address, until the process
// ends.  In host code the name is only a handle for hipGetSymbolAddress: the address that kernels and
// copies may use is the one that call returns, kept per device in scratch_ptr below.
static __device__ __align__(256) unsigned char scratch[NA_BYTES];

namespace {

constexpr int NA_MAX_DEVICES = 64;
std::mutex na_lock;
unsigned char *scratch_ptr[NA_MAX_DEVICES] = {};

// address of the current device's copy of `scratch` (looked up once per device)
int scratch_of_current_device(unsigned char **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return tn_fail(TENSAIR_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= NA_MAX_DEVICES) return tn_fail(TENSAIR_EHIP, "device ordinal %d not supported", dev);
    std::lock_guard<std::mutex> hold(na_lock);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return tn_fail(TENSAIR_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        scratch_ptr[dev] = (unsigned char *)p;
    }
    *out = scratch_ptr[dev];
    return TENSAIR_OK;
}

int take_source(ApplyArgs &a, int k, const tensair_sparse_grad *g, const char *what)
{
    for (int t = 0; t < 2; ++t) {
        const tensair_sparse_rows &r = t ? g->out : g->in;
        if (!r.n_rows || !r.row_ids || !r.row_grads) return tn_fail(TENSAIR_EINVAL, "%s: NULL pointer", what);
        if (r.capacity < 0 || r.capacity > 0x7FFFFFFFLL) return tn_fail(TENSAIR_EINVAL, "%s: bad capacity", what);
        if (((uintptr_t)r.row_grads & 15) || ((uintptr_t)r.row_ids & 3) || ((uintptr_t)r.n_rows & 3))
            return tn_fail(TENSAIR_EINVAL, "%s: rows must be 16-byte aligned, ids and counts 4-byte aligned", what);
        a.src[t][k].ids = r.row_ids;
        a.src[t][k].rows = r.row_grads;
        a.src[t][k].n_rows = r.n_rows;
        a.src[t][k].capacity = r.capacity;
    }
    return TENSAIR_OK;
}

}  // namespace

extern "C" int tensair_dasgd_apply_static(void *w_in, void *w_out, int64_t vocab, int32_t dim, int32_t row_stride,
                                          int32_t dtype, const tensair_sparse_grad *own,
                                          const tensair_sparse_grad *peers, int32_t n_peers, float lr,
                                          int32_t *status, void *stream)
{
    // sizes first: nothing below touches the GPU before they are known to fit the fixed scratch
    if (vocab < 1) return tn_fail(TENSAIR_EINVAL, "vocab must be positive");
    if (vocab > TENSAIR_STATIC_MAX_VOCAB)
        return tn_fail(TENSAIR_ECAPACITY, "vocab %lld above the %lld rows the static scratch indexes",
                       (long long)vocab, (long long)TENSAIR_STATIC_MAX_VOCAB);
    if (n_peers < 0 || n_peers > TENSAIR_STATIC_MAX_PEERS)
        return tn_fail(TENSAIR_ECAPACITY, "n_peers %d outside 0..%d", n_peers, TENSAIR_STATIC_MAX_PEERS);
    if (!w_in || !w_out) return tn_fail(TENSAIR_EINVAL, "NULL table");
    if (((uintptr_t)w_in | (uintptr_t)w_out) & 15) return tn_fail(TENSAIR_EINVAL, "tables must be 16-byte aligned");
    if (dim < 4 || dim > TENSAIR_MAX_DIM || dim % 4) return tn_fail(TENSAIR_EINVAL, "dim must be a multiple of 4 in 4..1024");
    if (row_stride < dim || row_stride % 4) return tn_fail(TENSAIR_EINVAL, "row_stride must be >= dim and a multiple of 4");
    if (dtype != TENSAIR_F32 && dtype != TENSAIR_BF16) return tn_fail(TENSAIR_EINVAL, "unknown dtype");
    if (n_peers > 0 && !peers) return tn_fail(TENSAIR_EINVAL, "peers is NULL");
    if (!(lr == lr)) return tn_fail(TENSAIR_EINVAL, "lr is NaN");
    if ((uintptr_t)status & 3) return tn_fail(TENSAIR_EINVAL, "status must be 4-byte aligned");

    ApplyArgs a;
    memset(&a, 0, sizeof(a));
    a.table[0] = w_in;
    a.table[1] = w_out;
    a.dtype = dtype;
    a.D = dim;
    a.stride = row_stride;
    a.V = vocab;
    a.n_src = 1 + n_peers;
    a.lr = lr;
    int rc;
    if (own && (rc = take_source(a, 0, own, "own"))) return rc;
    for (int k = 0; k < n_peers; ++k)
        if ((rc = take_source(a, 1 + k, &peers[k], "peer"))) return rc;
    if (!own && n_peers == 0) return TENSAIR_OK;

    unsigned char *base = nullptr;
    if ((rc = scratch_of_current_device(&base))) return rc;
    // layout: status word | start of W_in | mask of W_in | start of W_out | mask of W_out.  The masks are
    // cleared by the first kernel below on every call; a start entry is only read where its mask has bits.
    a.status = status ? status : (int *)base;
    unsigned char *p = base + NA_STATUS_BYTES;
    for (int t = 0; t < 2; ++t) {
        a.start[t] = (u32 *)p;
        p += NA_START_BYTES;
        a.mask[t] = (u64 *)p;
        p += NA_MASK_BYTES;
    }
    hipStream_t st = (hipStream_t)stream;
    tn_launch_apply_clear(a, st);
    tn_launch_apply_index(a, 0, a.n_src, st);
    tn_launch_apply_update(a, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return tn_fail(TENSAIR_EHIP, "dasgd_apply_static: %s", hipGetErrorString(e));
    return TENSAIR_OK;
}
