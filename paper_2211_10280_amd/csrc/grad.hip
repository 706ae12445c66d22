// Gradient calculation of one mini-batch (calculate_gradient of Algorithm 1; the "GC"
// term of Eq. 1 in TensAIR, arXiv 2211.10280, Section 2.2) for a skip-gram model with
// negative sampling: per pair (c, x) and j in {x, negatives},
//   s = <W_in[c], W_out[j]>,  g = (sigmoid(s) - label)/P,
//   Gin[c] += g W_out[j],     Gout[j] += g W_in[c].
//
// Two passes, both free of atomics:
//   forward   one workgroup per center position: the center row stays in registers, the
//             context/negative rows are gathered once, g is stored per occurrence and the
//             center's share of Gin is combined across waves through LDS;
//   segreduce the occurrences sorted by row id are cut into fixed tiles (64, or 8 for small lists); a wave sums
//             its tile in sorted order, writes rows that lie inside the tile directly and
//             rows that cross a tile border as partials, which a second kernel chains in
//             tile order.  Load balance is therefore independent of how hot a row is.
#include "dev_common.h"
#include "kernels.h"

#ifndef FWD_UNROLL
#define FWD_UNROLL 2   // measured: 2 rows in flight per wave beat 4 and 8 (occupancy matters more)
#endif
#ifndef SEG_UNROLL
#define SEG_UNROLL 4
#endif

// ---------------------------------------------------------------- forward
// LOSS: also accumulate the loss terms (only when the caller asked for the mean loss).
template <typename T, int ITERS, bool LOSS>
__global__ void __launch_bounds__(BLOCK) k_forward(FwdArgs a)
{
    __shared__ float red[WAVES_PER_BLOCK][ITERS * WAVE * 4];
    __shared__ float lred[WAVES_PER_BLOCK];
    const int i = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const int C4 = a.D >> 2;
    const BatchDesc &b = a.b;
    const i64 p = b.begin + i;
    const T *w_in = (const T *)a.w_in;
    const T *w_out = (const T *)a.w_out;
    const int Np1 = b.N + 1;

    int c = b.tok[p];
    if ((u32)c >= (u32)a.V) c = 0;   // flagged by the key kernel; stay in range
    i64 left = p < b.w ? p : b.w;
    i64 right = (b.T - 1 - p) < b.w ? (b.T - 1 - p) : b.w;
    const int ntasks = (int)(left + right) * Np1;
    const i64 occ0 = (pairs_before(p, b.T, b.w) - b.pair_base) * Np1;

    float4 v[ITERS], acc[ITERS];
    load_row<T, ITERS>(v, w_in + (size_t)c * a.stride, C4, lane);
    zero_row<ITERS>(acc);
    float loss = 0.f;   // per-lane partial (lanes 0..FWD_UNROLL-1 carry it)

    // wave `wave` takes tasks wave, wave+4, ...; FWD_UNROLL rows are in flight at a time.  The
    // dot products are reduced one by one, then lane x evaluates the sigmoid of task x, so the
    // transcendental code runs once per group instead of once per task.
    for (int t0 = wave; t0 < ntasks; t0 += WAVES_PER_BLOCK * FWD_UNROLL) {
        float4 u[FWD_UNROLL][ITERS];
#pragma unroll
        for (int x = 0; x < FWD_UNROLL; ++x) {
            int t = t0 + x * WAVES_PER_BLOCK;
            if (t < ntasks) {
                u32 j = a.out_keys[occ0 + t];
                load_row<T, ITERS>(u[x], w_out + (size_t)j * a.stride, C4, lane);
            } else {
                zero_row<ITERS>(u[x]);
            }
        }
        float s_l = 0.f;
#pragma unroll
        for (int x = 0; x < FWD_UNROLL; ++x) {
            float s = wave_sum_dpp(dot_partial<ITERS>(v, u[x]));
            s_l = (lane == x) ? s : s_l;
        }
        const int t_l = t0 + lane * WAVES_PER_BLOCK;
        const bool live = (lane < FWD_UNROLL) && (t_l < ntasks);
        const bool pos = (t_l % Np1) == 0;
        // sigmoid(s) - label without cancellation: label 1: -1/(1+e^s), label 0: 1/(1+e^-s)
        const float z = pos ? s_l : -s_l;
        float gg = 1.0f / (1.0f + expf(z));
        gg = pos ? -gg : gg;
        const float g_l = live ? gg * a.inv_P : 0.f;
        if (live) a.g[occ0 + t_l] = g_l;
        if (LOSS) {
            // loss term: softplus(-s) for the context, softplus(s) for a negative
            const float y = -z;
            if (live) loss += fmaxf(y, 0.f) + log1pf(expf(-fabsf(y)));
        }
#pragma unroll
        for (int x = 0; x < FWD_UNROLL; ++x) axpy_row<ITERS>(acc, rd_lane(g_l, x), u[x]);
    }
    // combine the four waves in a fixed order
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int e = (lane + WAVE * it) * 4;
        red[wave][e + 0] = acc[it].x;
        red[wave][e + 1] = acc[it].y;
        red[wave][e + 2] = acc[it].z;
        red[wave][e + 3] = acc[it].w;
    }
    if (LOSS) {
        loss = wave_sum_dpp(loss);
        if (lane == 0) lred[wave] = loss;
    }
    __syncthreads();
    float *dst = a.center_part + (size_t)i * a.D;
    for (int e = threadIdx.x; e < a.D; e += BLOCK) {
        float s = red[0][e];
#pragma unroll
        for (int w = 1; w < WAVES_PER_BLOCK; ++w) s += red[w][e];
        dst[e] = s;
    }
    if (LOSS && threadIdx.x == 0) {
        float s = lred[0];
#pragma unroll
        for (int w = 1; w < WAVES_PER_BLOCK; ++w) s += lred[w];
        a.center_loss[i] = s;
    }
}

template <typename T, bool LOSS>
static void launch_forward_t(const FwdArgs &a, hipStream_t st)
{
    int C4 = a.D / 4;
    int iters = (C4 + WAVE - 1) / WAVE;
    dim3 grid(a.b.n_centers), blk(BLOCK);
    switch (iters) {
    case 1: hipLaunchKernelGGL((k_forward<T, 1, LOSS>), grid, blk, 0, st, a); break;
    case 2: hipLaunchKernelGGL((k_forward<T, 2, LOSS>), grid, blk, 0, st, a); break;
    case 3: hipLaunchKernelGGL((k_forward<T, 3, LOSS>), grid, blk, 0, st, a); break;
    default: hipLaunchKernelGGL((k_forward<T, 4, LOSS>), grid, blk, 0, st, a); break;
    }
}

void tn_launch_forward(const FwdArgs &a, hipStream_t st)
{
    const bool loss = a.center_loss != nullptr;
    if (a.dtype == 0) loss ? launch_forward_t<float, true>(a, st) : launch_forward_t<float, false>(a, st);
    else loss ? launch_forward_t<bf16_t, true>(a, st) : launch_forward_t<bf16_t, false>(a, st);
}

// ---------------------------------------------------------------- segmented reduction
// Contribution of sorted entry e: scale * row, both fetched by the wave.
template <typename T, int ITERS, int MODE>
__device__ __forceinline__ void entry_source(const SegReduceArgs &a, u32 val, const T *&row,
                                             float &scale)
{
    if (MODE == 0) {
        int c = a.pair_center[val / (u32)a.Np1];
        row = (const T *)a.table + (size_t)c * a.stride;
        scale = a.g[val];
    } else {
        row = (const T *)a.center_part + (size_t)val * a.D;
        scale = 1.0f;
    }
}

// One wave per tile of TILE (<= 64) sorted entries.  A row whose entries all lie in the
// tile is written to out_rows; the leading row if it continues from the previous tile
// goes to part[tile][0], the trailing row if it continues into the next tile goes to
// part[tile][1] (a row covering the whole tile and both borders counts as leading).
template <typename T, int ITERS, int MODE, int TILE>
__global__ void __launch_bounds__(BLOCK) k_segreduce(SegReduceArgs a)
{
    const int tile = blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    const int lane = lane_id();
    const int t0 = tile * TILE;
    if (t0 >= a.n) return;
    const int cnt = min(TILE, a.n - t0);
    const int C4 = a.D >> 2;

    // lane l holds the metadata of entry t0 + l
    int seg_l = -1;
    u32 val_l = 0;
    if (lane < cnt) {
        seg_l = a.seg_of[t0 + lane];
        val_l = a.vals[t0 + lane];
    }
    const T *row_l = nullptr;
    float scale_l = 0.f;
    if (lane < cnt) entry_source<T, ITERS, MODE>(a, val_l, row_l, scale_l);
    const int seg_before = (t0 > 0) ? a.seg_of[t0 - 1] : -1;
    const int seg_after = (t0 + cnt < a.n) ? a.seg_of[t0 + cnt] : -2;

    int cur = rd_lane(seg_l, 0);
    bool open_left = (cur == seg_before);   // current row started in an earlier tile
    float4 acc[ITERS];
    zero_row<ITERS>(acc);
    float *part = a.part + (size_t)tile * 2 * a.D;

    for (int e0 = 0; e0 < cnt; e0 += SEG_UNROLL) {
        float4 r[SEG_UNROLL][ITERS];
        float sc[SEG_UNROLL];
        int sg[SEG_UNROLL];
#pragma unroll
        for (int x = 0; x < SEG_UNROLL; ++x) {
            int e = e0 + x;
            if (e < cnt) {
                sg[x] = rd_lane(seg_l, e);
                sc[x] = rd_lane(scale_l, e);
                const T *row = (const T *)rd_lane64((u64)row_l, e);
                load_row<T, ITERS>(r[x], row, C4, lane);
            }
        }
#pragma unroll
        for (int x = 0; x < SEG_UNROLL; ++x) {
            int e = e0 + x;
            if (e < cnt) {
                if (sg[x] != cur) {   // the row `cur` ends inside this tile
                    float *dst = open_left ? part : a.out_rows + (size_t)cur * a.D;
                    store_row<float, ITERS>(dst, acc, C4, lane);
                    zero_row<ITERS>(acc);
                    open_left = false;
                    cur = sg[x];
                }
                axpy_row<ITERS>(acc, sc[x], r[x]);
            }
        }
    }
    {
        bool open_right = (cur == seg_after);
        float *dst = open_left ? part : (open_right ? part + a.D : a.out_rows + (size_t)cur * a.D);
        store_row<float, ITERS>(dst, acc, C4, lane);
    }
}

// Chains the partials of rows that cross tile borders, in tile order.  One workgroup
// per tile; it acts only if the tile's trailing row continues into the next tile and
// started inside this tile (so every such row is owned by exactly one workgroup).
template <int ITERS, int TILE>
__global__ void __launch_bounds__(BLOCK) k_segfixup(SegReduceArgs a)
{
    __shared__ float red[WAVES_PER_BLOCK][ITERS * WAVE * 4];
    __shared__ int s_len;
    const int tile = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const int t0 = tile * TILE;
    const int t1 = min(a.n, t0 + TILE);
    if (t1 >= a.n) return;                        // last tile: nothing continues
    const int row = a.seg_of[t1 - 1];
    if (a.seg_of[t1] != row) return;              // trailing row ends at the border
    const bool started_before = (t0 > 0) && (a.seg_of[t0 - 1] == row) && (a.seg_of[t0] == row);
    if (started_before) return;                   // owned by the tile where the row starts
    // the chain: part[tile][1], then part[t][0] for t = tile+1 .. last tile holding `row`;
    // the entries are sorted, so the end of the row is found by bisection
    if (threadIdx.x == 0) {
        int lo = t1, hi = a.n;   // first index in [t1, n) whose row index exceeds `row`
        while (lo < hi) {
            int mid = lo + ((hi - lo) >> 1);
            if (a.seg_of[mid] <= row) lo = mid + 1;
            else hi = mid;
        }
        s_len = (lo - 1) / TILE - tile;   // number of leading partials to add
    }
    __syncthreads();
    const int len = s_len;
    const int C4 = a.D >> 2;
    float4 acc[ITERS];
    zero_row<ITERS>(acc);
    if (wave == 0) load_row<float, ITERS>(acc, a.part + ((size_t)tile * 2 + 1) * a.D, C4, lane);
    // wave w adds the leading partials of tiles tile+1+w, tile+1+w+4, ...
    for (int j0 = wave; j0 < len; j0 += WAVES_PER_BLOCK * SEG_UNROLL) {
        float4 r[SEG_UNROLL][ITERS];
#pragma unroll
        for (int x = 0; x < SEG_UNROLL; ++x) {
            int j = j0 + x * WAVES_PER_BLOCK;
            if (j < len) load_row<float, ITERS>(r[x], a.part + (size_t)(tile + 1 + j) * 2 * a.D, C4, lane);
        }
#pragma unroll
        for (int x = 0; x < SEG_UNROLL; ++x) {
            int j = j0 + x * WAVES_PER_BLOCK;
            if (j < len) add_row<ITERS>(acc, r[x]);
        }
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int e = (lane + WAVE * it) * 4;
        red[wave][e + 0] = acc[it].x;
        red[wave][e + 1] = acc[it].y;
        red[wave][e + 2] = acc[it].z;
        red[wave][e + 3] = acc[it].w;
    }
    __syncthreads();
    float *dst = a.out_rows + (size_t)row * a.D;
    for (int e = threadIdx.x; e < a.D; e += BLOCK) {
        float s = red[0][e];
#pragma unroll
        for (int w = 1; w < WAVES_PER_BLOCK; ++w) s += red[w][e];
        dst[e] = s;
    }
}

template <typename T, int MODE, int ITERS, int TILE>
static void launch_segreduce_i(const SegReduceArgs &a, hipStream_t st)
{
    int ntiles = (a.n + TILE - 1) / TILE;
    dim3 grid((ntiles + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK), blk(BLOCK);
    hipLaunchKernelGGL((k_segreduce<T, ITERS, MODE, TILE>), grid, blk, 0, st, a);
    if (ntiles > 1) hipLaunchKernelGGL((k_segfixup<ITERS, TILE>), dim3(ntiles - 1), blk, 0, st, a);
}

template <typename T, int MODE>
static void launch_segreduce_t(const SegReduceArgs &a, hipStream_t st)
{
    int C4 = a.D / 4;
    int iters = (C4 + WAVE - 1) / WAVE;
    const bool small = tn_seg_tile(a.n) == 8;
    switch (iters) {
    case 1: small ? launch_segreduce_i<T, MODE, 1, 8>(a, st) : launch_segreduce_i<T, MODE, 1, 64>(a, st); break;
    case 2: small ? launch_segreduce_i<T, MODE, 2, 8>(a, st) : launch_segreduce_i<T, MODE, 2, 64>(a, st); break;
    case 3: small ? launch_segreduce_i<T, MODE, 3, 8>(a, st) : launch_segreduce_i<T, MODE, 3, 64>(a, st); break;
    default: small ? launch_segreduce_i<T, MODE, 4, 8>(a, st) : launch_segreduce_i<T, MODE, 4, 64>(a, st); break;
    }
}

void tn_launch_segreduce(const SegReduceArgs &a, hipStream_t st)
{
    if (a.n <= 0) return;
    if (a.mode == 1) launch_segreduce_t<float, 1>(a, st);
    else if (a.dtype == 0) launch_segreduce_t<float, 0>(a, st);
    else launch_segreduce_t<bf16_t, 0>(a, st);
}

// ---------------------------------------------------------------- loss and the empty batch
__global__ void __launch_bounds__(BLOCK) k_loss(const float *center_loss, int n, float inv_P,
                                                float *mean_loss)
{
    __shared__ float sm[WAVES_PER_BLOCK];
    float s = 0.f;
    for (int i = threadIdx.x; i < n; i += BLOCK) s += center_loss[i];
    s = wave_sum(s);
    if (lane_id() == 0) sm[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = sm[0];
#pragma unroll
        for (int w = 1; w < WAVES_PER_BLOCK; ++w) t += sm[w];
        *mean_loss = t * inv_P;
    }
}

void tn_launch_loss(const float *center_loss, int n_centers, float inv_P, float *mean_loss,
                    hipStream_t st)
{
    hipLaunchKernelGGL(k_loss, dim3(1), dim3(BLOCK), 0, st, center_loss, n_centers, inv_P, mean_loss);
}

__global__ void k_empty_grad(int *n_in, int *n_out, float *mean_loss, int *seg_in, int *seg_out)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        *n_in = 0;
        *n_out = 0;
        if (mean_loss) *mean_loss = 0.f;
        if (seg_in) seg_in[0] = 0;
        if (seg_out) seg_out[0] = 0;
    }
}

void tn_launch_empty_grad(int *n_in, int *n_out, float *mean_loss, int *seg_in, int *seg_out,
                          hipStream_t st)
{
    hipLaunchKernelGGL(k_empty_grad, dim3(1), dim3(WAVE), 0, st, n_in, n_out, mean_loss, seg_in, seg_out);
}
