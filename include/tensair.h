/*
 * libtensair -- one DASGD worker's training step on a skip-gram/negative-sampling
 * word-embedding model, for AMD MI355X (gfx950).
 *
 * The calls follow the Model operator of TensAIR (arXiv 2211.10280), Algorithm 1:
 *   Model(tfModel, maxBuffer)            -> tensair_model_init
 *   calculate_gradient(model, minibatch) -> tensair_sgns_grad      (gradient calculation, Section 2.2)
 *   apply_gradient(model, gradient)      -> tensair_dasgd_apply    (gradient application, Eq. 1)
 *   train(minibatch) incl. peer messages -> tensair_step
 *   a mini-batch waiting in the operator's input queue -> tensair_prefetch (optional)
 *   gradients += gradient (the buffer sent every maxGradBuffer steps) -> tensair_grad_add
 *   apply_gradient for a dense model                 -> tensair_dense_apply
 *   predict(msg) for an embedding model              -> tensair_lookup
 *   cosine difference of two embedding tables (Section 4.4) -> tensair_cosine_difference
 *   a gradient message with bfloat16 rows (a variant beyond the paper) -> tensair_grad_pack,
 *       tensair_dasgd_apply_packed, tensair_step_packed
 *
 * Conventions for every call
 *   - Plain C ABI.  Pointers marked DEVICE point to GPU memory owned by the caller;
 *     pointers marked HOST point to host memory.  The library allocates no device
 *     memory: everything it needs lives in the caller's workspace.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  The results
 *     of every call are complete on it (the library forks part of the work to a stream of
 *     its own and joins it again); use one stream for all calls on a model.  No call waits
 *     for the GPU except tensair_status, tensair_model_destroy and tensair_model_init
 *     (which uploads the alias table).  Sizes that depend on the data
 *     (number of unique rows) stay on the device.
 *   - Return value: TENSAIR_OK or a negative tensair_status code; host-detectable
 *     argument errors are reported before anything is launched;
 *     tensair_last_error() gives a thread-local message.
 *   - A model handle keeps host-side state between calls (announced mini-batches, the order of
 *     work on the library's stream): calls on one handle must not overlap in time on the host;
 *     different handles are independent.
 *   - Data errors seen by kernels (a peer gradient whose ids are out of range or not
 *     strictly ascending) never fault: the offending rows are skipped, a device
 *     status word is set, and tensair_status() reports TENSAIR_EDATA.
 */
#ifndef TENSAIR_H
#define TENSAIR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tensair_model tensair_model; /* opaque host handle */

enum { TENSAIR_F32 = 0, TENSAIR_BF16 = 1 }; /* table element type (gradients are always fp32) */

enum {
    TENSAIR_OK = 0,
    TENSAIR_EINVAL = -1,    /* bad argument (null, non-positive size, unsupported shape) */
    TENSAIR_ECAPACITY = -2, /* a caller buffer or the workspace is too small */
    TENSAIR_EHIP = -3,      /* a HIP runtime call failed */
    TENSAIR_EDATA = -4      /* kernels met invalid row ids */
};

#define TENSAIR_MAX_DIM 1024  /* dim must be a multiple of 4, 4..1024 */
#define TENSAIR_MAX_PEERS 31
/* Largest sizes that one launch of the update kernels covers (2^32 threads): a model of at most
 * TENSAIR_MAX_VOCAB rows, a dense parameter vector of at most TENSAIR_MAX_DENSE elements. */
#define TENSAIR_MAX_VOCAB 268435392LL      /* 2^28 - 64 */
#define TENSAIR_MAX_DENSE 8589934592LL     /* 2^33 */

typedef struct {
    int64_t vocab;       /* V, 1 .. TENSAIR_MAX_VOCAB */
    int32_t dim;         /* D, multiple of 4 */
    int32_t row_stride;  /* elements between consecutive table rows, >= dim, multiple of 4 */
    int32_t dtype;       /* TENSAIR_F32 | TENSAIR_BF16 */
    int32_t window;      /* w >= 1: contexts at offsets -w..-1, +1..+w, clipped to the stream */
    int32_t negatives;   /* N >= 0 negatives per (center, context) pair */
    int32_t max_centers; /* largest mini-batch (center positions) a call may pass */
    int32_t max_peers;   /* largest number of peer gradients a call may pass, <= TENSAIR_MAX_PEERS */
    uint32_t worker_id;  /* < 65536; enters the negative-sampling counter (peers differ by it) */
    uint64_t seed;       /* key of the counter-based generator (negatives and table init) */
    uint32_t flags;      /* 0, or TENSAIR_RESAMPLE_NEGATIVES | TENSAIR_STOCHASTIC_ROUNDING */
} tensair_config;

/* A variant the paper leaves open (it does not say what happens to a negative that equals the pair's
 * center or context word; by default it is kept and the row receives both contributions): with this
 * flag such a negative is drawn once more, from words 2 and 3 of the same Philox block (bucket by
 * multiply-high of word 2, word 3 against the threshold), and the second draw is kept whatever it
 * is.  Still a pure function of the counter, with fixed shapes. */
#define TENSAIR_RESAMPLE_NEGATIVES 1u

/* Another variant the paper leaves open (it does not say how a low-precision table is rounded; by
 * default round-to-nearest-even, which drops every update below half a unit in the last place): with
 * this flag the table update of a bf16 model (tensair_dasgd_apply, tensair_step and their _packed
 * forms) rounds stochastically.  The new value W[r] - lr * sum, in fp32, gets 16 random bits added
 * to its bit pattern below the bfloat16 mantissa and is truncated, so it goes up with probability
 * (discarded bits)/2^16 and its expectation is the fp32 value; infinities and NaN are kept.  The
 * bits of element i = r*dim + col are the low half of word (i mod 4) of Philox4x32-10(counter =
 * (i/4 low, i/4 high, serial, 'SRND' + table), key = seed), table = 0 for W_in, 1 for W_out; serial
 * counts the table updates enqueued on this model handle since tensair_model_init, from 0 (calls
 * that update nothing do not count).  Reproducible for a given sequence of calls.  No effect on
 * fp32 tables. */
#define TENSAIR_STOCHASTIC_ROUNDING 2u

/* One table's sparse gradient: the rows a mini-batch touches (Section 4, "Sparse vs.
 * Dense Models").  All pointers DEVICE, caller-owned.  row_ids[0..*n_rows) is strictly
 * ascending; row_grads is [capacity][dim] fp32, dense rows, no padding. */
typedef struct {
    int64_t capacity;  /* rows allocated in row_ids / row_grads */
    int32_t *n_rows;   /* device scalar: written by tensair_sgns_grad, read by tensair_dasgd_apply */
    int32_t *row_ids;
    float *row_grads;
} tensair_sparse_rows;

/* Gradient of one mini-batch: `in` = rows of W_in (centers), `out` = rows of W_out
 * (contexts and negatives).  This is the payload of a gradient message of Algorithm 1. */
typedef struct {
    tensair_sparse_rows in, out;
} tensair_sparse_grad;

/* The same message with its rows rounded to bfloat16: half the bytes on the wire and in the
 * receiver's gradient application.  Same layout; row_grads is [capacity][dim] bfloat16 bits, 16-byte
 * aligned.  Written by tensair_grad_pack, read by tensair_dasgd_apply_packed / tensair_step_packed. */
typedef struct {
    int64_t capacity;
    int32_t *n_rows;
    int32_t *row_ids;
    uint16_t *row_grads;
} tensair_packed_rows;

typedef struct {
    tensair_packed_rows in, out;
} tensair_packed_grad;

/* The row pitch (in elements) at which every table row starts on a 128-byte line: the smallest multiple
 * of 128 bytes that holds dim elements of dtype (dim 300 in fp32: 320).  Any row_stride >= dim that is a
 * multiple of 4 is accepted; with this one a row shares no cache line with its neighbours, which the table
 * update measurably likes (the padding columns are never read or written).  Returns -1 for a bad argument. */
int32_t tensair_aligned_row_stride(int32_t dim, int32_t dtype);

/* Bytes of DEVICE workspace tensair_model_init needs for `cfg` (0 if cfg is invalid). */
size_t tensair_workspace_bytes(const tensair_config *cfg);

/* Rows a tensair_sparse_grad must hold for a batch of `n_centers`:
 * in: min(V, n_centers); out: min(V, 2*w*n_centers*(N+1)). */
int64_t tensair_capacity_in(const tensair_config *cfg, int32_t n_centers);
int64_t tensair_capacity_out(const tensair_config *cfg, int32_t n_centers);

/* Constructor of Algorithm 1's Model: binds the two embedding tables
 * (DEVICE, [vocab][row_stride] of cfg->dtype, 16-byte aligned, caller-owned).
 * fill_tables = 1: a fresh model, W_in ~ U(-0.5/D, 0.5/D) from cfg->seed, W_out = 0
 * (padding columns zeroed); 0: adopt the contents (a pre-trained model).
 * unigram_counts: HOST [vocab] occurrence counts; the noise distribution is
 * count^0.75 / sum, stored as an alias table in the workspace.
 * workspace: DEVICE, 256-byte aligned, >= tensair_workspace_bytes(cfg), and kept alive
 * and untouched by the caller until tensair_model_destroy.
 * Waits for the upload of the alias table on `stream` before returning. */
int tensair_model_init(tensair_model **out, const tensair_config *cfg, void *w_in, void *w_out,
                       int fill_tables, const uint64_t *unigram_counts, void *workspace,
                       size_t workspace_bytes, void *stream);

/* Point the model at other tables of the same shape and type (e.g. an older snapshot,
 * which is how a stale peer of Section 3.1 is reproduced) and change the worker id. */
int tensair_model_rebind(tensair_model *m, void *w_in, void *w_out, uint32_t worker_id);

/* Copy the alias table to HOST arrays thr[vocab], alias[vocab].  A draw (b, r) with
 * bucket b and 32-bit uniform r yields b if r < thr[b], else alias[b]. */
int tensair_model_alias(const tensair_model *m, uint32_t *thr, int32_t *alias);

/* Number of (center, context) pairs of the mini-batch of center positions
 * [center_begin, center_begin + n_centers) in a stream of n_tokens (host arithmetic). */
int64_t tensair_pair_count(const tensair_model *m, int64_t n_tokens, int64_t center_begin,
                           int32_t n_centers);

/* calculate_gradient of Algorithm 1 for one mini-batch, on the tables as they stand.
 * tokens: DEVICE int32[n_tokens], ids in [0, vocab).  The mini-batch is the run of
 * center positions [center_begin, center_begin+n_centers), n_centers <= max_centers.
 * Pairs are enumerated center-ascending, offsets -w..-1,+1..+w; each pair draws N
 * negatives from Philox4x32-10(counter = (position lo, position hi, q*65536+slot,
 * worker_id + 65536*epoch), key = seed): word 0 picks the bucket by multiply-high,
 * word 1 is compared with the bucket's threshold.  Per pair and j in {context,
 * negatives}: s = <W_in[c], W_out[j]>, g = (sigmoid(s) - label)/P; Gin[c] += g W_out[j],
 * Gout[j] += g W_in[c] (fp32 accumulation in a fixed order, duplicates summed by
 * sort and segmented reduction, no atomics).
 * grad_out: capacities >= tensair_capacity_in/out(n_centers); receives n_rows, the
 * ascending unique row ids and the summed rows.
 * Optional DEVICE outputs (NULL to skip): mean_loss float[1] (mean over the P pairs);
 * negatives_dbg int32[P][N]; seg_offsets_in int32[U_in+1] / seg_offsets_out
 * int32[U_out+1] = number of occurrences with a smaller id (in: one per pair; out: N+1
 * per pair: context, then negatives), last entry = total. */
int tensair_sgns_grad(tensair_model *m, const int32_t *tokens, int64_t n_tokens,
                      int64_t center_begin, int32_t n_centers, uint32_t epoch,
                      tensair_sparse_grad *grad_out, float *mean_loss, int32_t *negatives_dbg,
                      int32_t *seg_offsets_in, int32_t *seg_offsets_out, void *stream);

/* apply_gradient of Algorithm 1 / Eq. 1 for the own gradient and n_peers received
 * gradients at once: for every row r in the union of their row ids,
 * W[r] <- W[r] - lr * (own[r] + peer_1[r] + ... + peer_K[r]), the sum taken in fp32 in
 * that order, one rounding on store (round-to-nearest-even for bf16 tables).  Rows
 * outside the union are not written.  own may be NULL (peers only).  peers: HOST array
 * of n_peers structs (device pointers inside), n_peers <= max_peers.  Each source's ids
 * must be strictly ascending and in range (else TENSAIR_EDATA via tensair_status). */
int tensair_dasgd_apply(tensair_model *m, const tensair_sparse_grad *own,
                        const tensair_sparse_grad *peers, int32_t n_peers, float lr, void *stream);

/* "gradients += gradient" of Algorithm 1, train(): the sum of two sparse gradients, which is how
 * a Model instance keeps the gradients it has computed and not yet sent (the buffer is broadcast
 * every maxGradBuffer steps and starts again from an empty gradient, *n_rows = 0).
 * out lists the union of the row ids of a and b, ascending; a row that only one of them has is
 * copied, a row that both have is a's row plus b's row in fp32 (one rounding).  A listed row
 * stays listed even if it sums to zero.  out must not share buffers with a or b.  If the union
 * has more rows than out's capacity the result is cut off there and tensair_status reports
 * TENSAIR_EDATA; min(vocab, a.capacity + b.capacity) always suffices.  Ids out of range or not
 * ascending in a or b are reported the same way (such rows are skipped, nothing faults).
 * Uses the same index scratch as tensair_dasgd_apply: calls on one model must be on one stream. */
int tensair_grad_add(tensair_model *m, const tensair_sparse_grad *a, const tensair_sparse_grad *b,
                     tensair_sparse_grad *out, void *stream);

/* apply_gradient of Algorithm 1 / Eq. 1 for a dense model (Section 4, "Sparse vs. Dense Models":
 * every variable receives gradient), for the own gradient and the gradients received from peers
 * at once: theta[i] <- theta[i] - lr * (grads[0][i] + ... + grads[n_grads-1][i]), the sum taken
 * in fp32 in that order, one rounding on store (round-to-nearest-even for bf16).
 * theta: DEVICE [n] of dtype, 16-byte aligned, n <= TENSAIR_MAX_DENSE.  grads: HOST array of n_grads DEVICE pointers to
 * fp32 [n] blocks, each 16-byte aligned, n_grads <= TENSAIR_MAX_PEERS + 1.  Needs no model handle. */
int tensair_dense_apply(void *theta, int32_t dtype, int64_t n, const float *const *grads, int32_t n_grads,
                        float lr, void *stream);

/* predict of Algorithm 1 for an embedding model: the vectors of n words.  table: 0 = W_in (the
 * word vectors), 1 = W_out.  ids: DEVICE int32[n]; out: DEVICE fp32 [n][dim], 16-byte aligned
 * (bf16 tables are widened, padding columns dropped).  An id outside [0, vocab) yields a row of
 * zeros and TENSAIR_EDATA from tensair_status. */
int tensair_lookup(tensair_model *m, int32_t table, const int32_t *ids, int64_t n, float *out, void *stream);

/* Section 4.4: how far training has moved every word, diff[r] = 1 - cos(a[r], b[r]) for two tables
 * of the same shape and type (DEVICE, [vocab][row_stride], 16-byte aligned); diff: DEVICE fp32
 * [vocab].  A row that is zero in both tables has difference 0, one that is zero in only one has 1.
 * Needs no model handle. */
int tensair_cosine_difference(const void *a, const void *b, int32_t dtype, int64_t vocab, int32_t dim,
                              int32_t row_stride, float *diff, void *stream);

/* train() of Algorithm 1 for one mini-batch plus the peer gradients that arrived:
 * tensair_sgns_grad into own_out on the current tables, then tensair_dasgd_apply of
 * own_out and the peers (Section 3.1: the own gradient is computed before the
 * received ones are applied).  own_out stays valid afterwards (it is what the worker
 * would broadcast). */
int tensair_step(tensair_model *m, const int32_t *tokens, int64_t n_tokens, int64_t center_begin,
                 int32_t n_centers, uint32_t epoch, const tensair_sparse_grad *peers,
                 int32_t n_peers, float lr, tensair_sparse_grad *own_out, float *mean_loss,
                 void *stream);

/* A variant the paper leaves open.  Section 4.3 finds that with more than three GPUs Word2Vec training
 * is limited by gradient application, which is not distributed, and every gradient message of
 * Algorithm 1 is broadcast to all other instances; the paper's remedy is maxGradBuffer.  Sending
 * the rows as bfloat16 halves both costs at the price of one rounding per element:
 * tensair_grad_pack turns a gradient into such a message -- *n_rows and the row ids are copied,
 * every element of the rows is rounded to the nearest bfloat16, ties to even (NaN becomes 0x7FC0,
 * values beyond the largest finite bfloat16 become infinity).  out needs capacities >= g's row counts
 * (else the message is cut off there and tensair_status reports TENSAIR_EDATA) and must not share
 * buffers with g.
 * tensair_dasgd_apply_packed is tensair_dasgd_apply with the peers' gradients given as such
 * messages: W[r] <- W[r] - lr * (own[r] + widen(peer_1[r]) + ... + widen(peer_K[r])), the own
 * gradient still fp32, the sum in fp32 in that order, one rounding on store.
 * tensair_step_packed is tensair_step with packed peers.  own_out stays fp32; with own_msg_out (NULL to
 * skip; capacities >= tensair_capacity_in/out(n_centers), no buffer shared with own_out) the own
 * gradient is also written as such a message, bit for bit what tensair_grad_pack makes of own_out,
 * while its rows pass through the table update -- the message this worker sends, at the cost of
 * its bytes alone. */
int tensair_grad_pack(tensair_model *m, const tensair_sparse_grad *g, tensair_packed_grad *out, void *stream);
int tensair_dasgd_apply_packed(tensair_model *m, const tensair_sparse_grad *own,
                               const tensair_packed_grad *peers, int32_t n_peers, float lr, void *stream);
int tensair_step_packed(tensair_model *m, const int32_t *tokens, int64_t n_tokens, int64_t center_begin,
                        int32_t n_centers, uint32_t epoch, const tensair_packed_grad *peers,
                        int32_t n_peers, float lr, tensair_sparse_grad *own_out,
                        tensair_packed_grad *own_msg_out, float *mean_loss, void *stream);

/* Announces a coming mini-batch, so that the part of its tensair_sgns_grad / tensair_step
 * call that does not depend on the tables -- pair enumeration, negatives, sort by row id,
 * segments, unique row ids -- is prepared ahead of time on the library's own stream, next to
 * whatever the caller's stream is doing (in TensAIR's dataflow, Section 3, mini-batches queue
 * up at the Model operator: the coming ones are known while the current one trains).
 * Up to two announcements are kept, in order.  When the first is prepared is the library's choice: at
 * once if the mini-batch is small (up to 2^20 context and negative occurrences: its sort is bound by
 * latency and fits beside whatever runs), else by the gradient call that consumes it.  A second one is
 * prepared during the gradient call that consumes the first -- under that call's table update if
 * tensair_step expects a long one, else beside its forward pass if small; a third replaces the second.
 * A gradient call on this model uses the
 * prepared data if its (tokens, n_tokens, center_begin, n_centers, epoch) and the model's
 * worker id are those of the oldest announcement -- its results are then bit-identical to
 * those of a call without prefetch -- and otherwise drops every announcement.
 * A mini-batch without pairs is not recorded.
 * Ordering: the preparation may start as soon as everything enqueued on `stream` before
 * the START of the most recent gradient call on this model has finished (before this call,
 * if the library's stream has not followed that call), so the token range must be ready by
 * then and must stay unchanged until the consuming call has run.
 * Same argument checks and error codes as tensair_sgns_grad. */
int tensair_prefetch(tensair_model *m, const int32_t *tokens, int64_t n_tokens, int64_t center_begin,
                     int32_t n_centers, uint32_t epoch, void *stream);

/* Waits for `stream`, then returns TENSAIR_OK, TENSAIR_EDATA (and clears the device
 * status word) or TENSAIR_EHIP. */
int tensair_status(tensair_model *m, void *stream);

/* Stage timing with HIP events on the caller's stream (a measurement aid, not part of the
 * method).  level 0: off (default); 1: one pair of events around the table-update kernel of
 * tensair_dasgd_apply / tensair_step; 2: an event after every stage of the step.
 * tensair_profile_read waits for the last recorded event, writes up to max_records
 * (tag, milliseconds) records since the previous read and returns their number (negative =
 * error).  Tags: 1 keys+negatives, 2 forward, 3 sort, 4 segments, 5 reduce W_in side,
 * 6 reduce W_out side, 8 apply index, 9 apply table update, 11 index and scan of
 * tensair_grad_add, 12 its row kernel (level 1 also brackets that one), 14 the kernel of
 * tensair_grad_pack (level 1 too); a tag's time runs from
 * the previous event to its own.  At most 65536 events are kept between reads. */
int tensair_profile(tensair_model *m, int level);
int tensair_profile_read(tensair_model *m, int32_t *tags, float *ms, int32_t max_records);

/* Measurement aid: one plain copy kernel, dst[0..bytes) = src[0..bytes) (DEVICE, 16-byte
 * aligned, bytes a multiple of 16, no overlap).  Reads `bytes` and writes `bytes`: the
 * streaming-bandwidth ceiling of the box and the calibration of its HBM byte counters. */
int tensair_copy_probe(void *dst, const void *src, size_t bytes, void *stream);

/* Measurement aid: streaming kernels with other mixes of reads and writes over `bytes` (DEVICE, 16-byte
 * aligned, a multiple of 16, no overlap), the ceilings that kernels of the same mix are set against.
 * mode 0: the plain copy of tensair_copy_probe; 1: the same copy around the caches (non-temporal loads and
 * stores); 2: read only -- src is read, dst receives one 16-byte chunk per workgroup (at most 256 KiB);
 * 3: three reads per write -- dst[i] = src[i] + src[n + i] + src[2n + i] over fp32 elements, src holding
 * 3 * bytes, around the caches (the read share of a table update that merges several gradient blocks). */
int tensair_stream_probe(void *dst, const void *src, size_t bytes, int32_t mode, void *stream);

/* tensair_dasgd_apply for callers that cannot allocate device memory and hold no model handle: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same update, same
 * kernels: W[r] <- W[r] - lr * (own[r] + peer_1[r] + ... + peer_K[r]) for every row in the union of the
 * sources' row ids, fp32 sum in that order, one rounding on store (round-to-nearest-even for bf16).
 * The tables are passed directly (DEVICE, [vocab][row_stride] of dtype, 16-byte aligned); own may be
 * NULL; peers: HOST array of n_peers structs.  The index scratch of the update (12.6 MB) is a fixed
 * device array inside the library instead of a workspace, which limits the call to
 * vocab <= TENSAIR_STATIC_MAX_VOCAB and n_peers <= TENSAIR_STATIC_MAX_PEERS: larger sizes are refused
 * with TENSAIR_ECAPACITY before anything is enqueued.  The call allocates nothing (no hipMalloc, no
 * hipFree, no allocating library routine) and does not wait for the GPU; the device of `stream` must
 * be the current device.  Every GPU holds one copy of the scratch, shared by all calls on that GPU:
 * the call clears what it needs itself, and calls that overlap in time on one GPU (two streams, two
 * threads) race -- keep them on one stream.
 * status: DEVICE int32 or NULL.  Data errors seen by the kernels (ids out of range or not strictly
 * ascending, a row count above its capacity) never fault; the offending rows are skipped and the bits
 * 1 (bad id), 2 (bad order), 4 (overflow) are OR-ed into *status, which the caller clears and reads. */
#define TENSAIR_STATIC_MAX_VOCAB 2097152 /* 2^21 rows per table */
#define TENSAIR_STATIC_MAX_PEERS 15
int tensair_dasgd_apply_static(void *w_in, void *w_out, int64_t vocab, int32_t dim, int32_t row_stride,
                               int32_t dtype, const tensair_sparse_grad *own,
                               const tensair_sparse_grad *peers, int32_t n_peers, float lr,
                               int32_t *status, void *stream);

/* Waits for the library's own stream (a pending prefetch), then frees the host handle. */
int tensair_model_destroy(tensair_model *m);

const char *tensair_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TENSAIR_H */
