// Host-callable launchers of the HIP kernels (one per pipeline stage).  All of them only
// enqueue work on `st`; none synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32;
typedef uint64_t u64;
typedef int64_t i64;

#define TN_MAX_SRC 32     // own + up to 31 peers
#define TN_MAX_BLOCKS ((1 << 24) - 1)   // workgroups of 256 threads that one launch may have (2^32 threads in all)
// sorted entries per wave in the segmented reduction: small problems get small tiles so that
// enough waves exist to hide the latency of the row loads
static inline int tn_seg_tile(i64 n) { return n <= 65536 ? 8 : 32; }
#define TN_RADIX_TILE 2048  // keys per block in a radix pass (256 threads x 8)
#define TN_RADIX_MAX_BITS 11  // widest digit of a radix pass
#ifndef TN_RADIX_WIDE_KEYS
#define TN_RADIX_WIDE_KEYS 16 // keys with more bits than this are sorted in digits of at most TN_RADIX_NARROW bits
#endif
#ifndef TN_RADIX_NARROW
#define TN_RADIX_NARROW 8
#endif
// Number of passes and digit width for keys of `key_bits` bits.  A pass scatters every key to the place of its
// digit; with d-bit digits a block of TN_RADIX_TILE keys writes runs of about TN_RADIX_TILE / 2^d neighbouring
// keys, and runs of two (11-bit digits) cost the memory system far more than their bytes when the sort shares the
// chip with a bandwidth-bound kernel.  Large vocabularies therefore take one pass more with narrower digits
// (measured at 20 and 21 key bits: the step 0.6 % and 2 % faster); small ones keep the fewest passes.
static inline void tn_radix_shape(int key_bits, int *passes, int *bits)
{
    if (key_bits < 1) key_bits = 1;
    const int widest = key_bits > TN_RADIX_WIDE_KEYS ? TN_RADIX_NARROW : TN_RADIX_MAX_BITS;
    *passes = (key_bits + widest - 1) / widest;
    *bits = (key_bits + *passes - 1) / *passes;
}
#define TN_SCAN_TILE 2048   // entries per block in the head scan
#define TN_SEG_XBLOCK 256    // tiles of the segmented reduction per block of partials
#define TN_SEG_CROSS_MIN 16384  // problems with more tiles than this get partials per block of tiles

// ---- stage 0: table initialisation
void tn_launch_init_tables(void *w_in, void *w_out, i64 V, int D, int stride, int dtype, u64 seed,
                           hipStream_t st);

// ---- stage 1: pair enumeration, negative sampling, sort keys
struct BatchDesc {
    const int *tok;   // DEVICE int32[T]
    i64 T;
    i64 begin;        // first center position
    int n_centers;
    int w, N;
    i64 pair_base;    // pairs_before(begin)
    i64 P;            // pairs in the batch
};
// resample: a negative equal to the pair's center or context word is drawn once more (words 2, 3)
void tn_launch_build_keys(const BatchDesc &b, i64 V, const u32 *thr, const int *alias, u64 seed,
                          u32 worker, u32 epoch, bool resample, u32 *out_keys, u32 *in_keys,
                          int *pair_center, int *neg_dbg, int *status, hipStream_t st);

// ---- stage 2: stable LSD radix sort of (key, value) for two independent problems at once
struct RadixProb {
    u32 *keys[3];   // input in keys[0], which is never written (other work may still read it);
                    // the passes go 0 -> 1 -> 2 -> 1 -> ...
    u32 *vals[2];   // values, ping-pong; the first pass writes the entry index (input order) itself
    int n;
    int nblk;       // ceil(n / TN_RADIX_TILE)
    u32 *counts;    // [2^bits][nblk] scratch
    u32 *totals;    // [2^bits] scratch
};
// returns which vals buffer (0/1) holds the sorted values; *key_buf = which keys buffer (1/2)
// min_lds_bytes: LDS to request per workgroup beyond what the counters need (0 = none): holds the occupancy of
// the sort down where it runs next to a kernel that it should not crowd
int tn_launch_radix_sort(RadixProb p0, RadixProb p1, int key_bits, size_t min_lds_bytes, hipStream_t st, int *key_buf);

// ---- stage 3: unique ids, segment index of every sorted entry, weighted segment offsets
struct SegProb {
    const u32 *keys;      // sorted keys
    const u32 *vals;      // sorted values
    int n;
    int nblk;             // ceil(n / TN_SCAN_TILE)
    int *blk_heads;       // [nblk] scratch
    int *blk_weight;      // [nblk] scratch
    int *seg_of;          // [n] out: row index (0..U-1) of every sorted entry
    int *seg_start;       // [U+1] out: index of the first sorted entry of every row, then n
    int *long_cnt;        // [1] zeroed here: the segmented reduction counts its long rows in it
    int *row_ids;         // [capacity] out
    int *n_rows;          // [1] out
    int *seg_offsets;     // [U+1] out or NULL
    i64 capacity;
    int weighted;         // 0: every entry weighs 1; 1: entry = center index, weighs its pair count
};
void tn_launch_segments(SegProb p0, SegProb p1, i64 begin, i64 T, int w, int *status, hipStream_t st);

// row ids / row count / segment offsets of a prepared mini-batch -> the consuming call's buffers
struct RowIndexCopy {
    struct Side {
        const int *src_ids, *src_n, *src_off;   // src_off [U+1]
        int *dst_ids, *dst_n, *dst_off;         // dst_off may be NULL
    } side[2];
};
void tn_launch_copy_row_index(const RowIndexCopy &c, i64 max_rows, hipStream_t st);

// ---- stage 4: forward pass and per-center partial of the W_in gradient
struct FwdArgs {
    const void *w_in, *w_out;
    i64 V;
    int dtype, D, stride;
    BatchDesc b;
    const u32 *out_keys;   // unsorted out-side keys [P][N+1]
    float *g;              // [P][N+1] out: (sigmoid - label)/P per occurrence
    float *center_part;    // [n_centers][D] out
    float *center_loss;    // [n_centers] out (sum of the loss terms, not yet divided by P)
    float inv_P;
};
struct AuxWork;
void tn_launch_forward(const FwdArgs &a, const AuxWork *aux, hipStream_t st);   // aux may be NULL

// ---- stage 5: segmented reduction of rows (duplicates summed in sorted order)
struct SegReduceArgs {
    int n;                 // sorted entries
    const u32 *vals;       // sorted values
    const int *seg_of;     // row index per sorted entry
    const int *seg_start;  // first sorted entry of every row; [U] = n
    float *out_rows;       // [U][D]
    float *part;           // [ntiles][2][D] scratch for rows that cross tile borders
    float *cross;          // [ceil(ntiles / TN_SEG_XBLOCK)][D] scratch: partials of long rows per block of tiles
                           // (the launcher clears the pointer for problems of at most TN_SEG_CROSS_MIN tiles)
    int *long_cnt;         // [1] number of long rows found (zeroed by the segment scan)
    int *long_list;        // [ntiles] tiles in which a long row begins, in no particular order
    int *xinfo;            // [ceil(ntiles / TN_SEG_XBLOCK)] scratch: does a long row cross the block's border
    int D;
    // source of the contribution of an entry:
    //  mode 0 (out-side): value = occurrence index o; row = g[o] * W_in[pair_center[o/(N+1)]]
    //  mode 1 (in-side):  value = center index i;     row = center_part[i]
    int mode;
    const float *g;
    const int *pair_center;
    int Np1;
    const void *table;
    int dtype, stride;
    const float *center_part;
};
// the W_out-side and the W_in-side problem of a mini-batch in one launch (either may be NULL)
void tn_launch_segreduce(const SegReduceArgs *out, const SegReduceArgs *in, const AuxWork *aux, hipStream_t st);

void tn_launch_loss(const float *center_loss, int n_centers, float inv_P, float *mean_loss,
                    hipStream_t st);
void tn_launch_empty_grad(int *n_in, int *n_out, float *mean_loss, int *seg_in, int *seg_out,
                          hipStream_t st);

// ---- stage 6/7: DASGD merge and table update
struct ApplySrc {
    const int *ids;
    const void *rows;        // [capacity][D] fp32; bfloat16 for the sources 1.. of a call with packed peers
    const int *n_rows;
    i64 capacity;
};
struct ApplyArgs {
    void *table[2];          // W_in, W_out
    int dtype, D, stride;
    i64 V;
    int n_src;               // own + peers actually passed
    ApplySrc src[2][TN_MAX_SRC];
    u32 *start[2];           // [words+1][n_src]
    u64 *mask[2];            // [words][n_src]
    float lr;
    int *status;
    int packed;              // 1: the peers' rows (sources 1..) are bfloat16 messages, the own gradient's fp32
    // packed peers only, optional (NULL to skip): the own gradient is also written out as a bfloat16 message
    // while its rows pass through the update (ids, count and rounded rows; capacity checked on the host)
    unsigned short *msg_rows[2];
    int *msg_ids[2], *msg_n[2];
    // stochastic rounding of bf16 tables (a variant): key and serial number of this update
    int sr;
    u32 sr_k0, sr_k1, sr_serial;
};
// Small jobs that ride at the front of the grid of the forward pass or of the segmented reduction
// (workgroups [0, total) of that launch): clearing the masks of the table update's index, copying a
// prepared mini-batch's row index to the caller's buffers, indexing the sources [k_begin, k_end) of the
// coming table update.  Clearing and indexing must not share a launch (the index needs cleared masks).
struct AuxWork {
    int total;               // clear_blocks + 2 * copy_blocks + 2 * (k_end - k_begin) * index_blocks
    int clear_blocks;
    u64 *clear_mask[2];      // masks to zero (both tables), clear_n entries each -- not necessarily apply's
    size_t clear_n;
    int copy_blocks;         // per table
    RowIndexCopy copy;
    int index_blocks;        // per (source, table)
    int k_begin, k_end;
    ApplyArgs apply;
};
void tn_aux_none(AuxWork &x);
void tn_aux_add_clear(AuxWork &x, u64 *mask_in, u64 *mask_out, size_t n);
void tn_aux_add_copy(AuxWork &x, const RowIndexCopy &c, i64 max_rows);
void tn_aux_add_index(AuxWork &x, const ApplyArgs &a, int k_begin, int k_end);

void tn_launch_apply_clear(const ApplyArgs &a, hipStream_t st);
void tn_launch_apply_index(const ApplyArgs &a, int k_begin, int k_end, hipStream_t st);
void tn_launch_apply_update(const ApplyArgs &a, hipStream_t st);

// ---- sum of sparse gradients: out = src_0 + src_1 + ... on the union of their rows
struct GradSumArgs {
    ApplyArgs a;             // sources, index arrays, V, D (tables, lr unused)
    int *out_ids[2];         // [capacity] ascending
    float *out_rows[2];      // [capacity][D]
    int *out_n[2];           // [1]
    i64 out_cap[2];
    u32 *wbase[2];           // [words] scratch: rows of the union before each 64-row word
    u32 *wblk[2];            // [ceil(words / TN_UNION_WORDS)] scratch: rows of the union per block of words
};
#define TN_UNION_WORDS 1024  // vocabulary words per workgroup in the union scan (256 threads x 4)
void tn_launch_grad_sum_index(const GradSumArgs &g, hipStream_t st);   // index + scan
void tn_launch_grad_sum_rows(const GradSumArgs &g, hipStream_t st);    // the rows themselves

// ---- a sparse gradient as a bfloat16 message: row counts and ids copied, rows rounded to nearest even
struct GradPackArgs {
    const int *n[2], *ids[2];
    const float *rows[2];
    int *out_n[2], *out_ids[2];
    unsigned short *out_rows[2];
    i64 cap[2], out_cap[2];
    int D;
    int *status;
};
void tn_launch_grad_pack(const GradPackArgs &a, hipStream_t st);

// ---- dense-model apply, embedding lookup, cosine difference between two tables
struct DenseApplyArgs {
    void *theta;                       // [n] f32 or bf16
    const float *grads[TN_MAX_SRC];    // n_grads blocks of [n] fp32
    i64 n;
    int n_grads, dtype;
    float lr;
};
void tn_launch_dense_apply(const DenseApplyArgs &a, hipStream_t st);
struct LookupArgs {
    const void *table;
    const int *ids;
    float *out;       // [n][D]
    i64 n, V;
    int D, stride, dtype;
    int *status;
};
void tn_launch_lookup(const LookupArgs &a, hipStream_t st);
struct CosineArgs {
    const void *a, *b;
    float *diff;      // [V]
    i64 V;
    int D, stride, dtype;
};
void tn_launch_cosine_diff(const CosineArgs &a, hipStream_t st);

// ---- measurement aid: plain copy of `bytes` (multiple of 16)
void tn_launch_copy_probe(void *dst, const void *src, size_t bytes, hipStream_t st);
// mode 0 plain copy, 1 copy around the caches, 2 read only, 3 three reads per write (src holds 3 * bytes)
void tn_launch_stream_probe(void *dst, const void *src, size_t bytes, int mode, hipStream_t st);

// ---- host-side helpers shared by the files that hold C-ABI entry points
// records the thread-local message of tensair_last_error and returns `code`
int tn_fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
