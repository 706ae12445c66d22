// Streaming operations around the worker step (TensAIR, arXiv 2211.10280):
//   k_dense_apply   apply_gradient of Algorithm 1 / Eq. 1 for a dense model (Section 4, "Sparse vs.
//                   Dense Models": every variable receives gradient): theta <- theta - alpha * sum_k g_k
//                   for the own gradient and the gradients received from peers, one pass, one rounding
//   k_lookup        predict of Algorithm 1 for an embedding model: the vectors of the given words
//   k_cosine_diff   Section 4.4: 1 - cos between the embeddings of every word in two tables
//   k_grad_pack     a sparse gradient turned into a bfloat16 message (a variant beyond the paper, aimed
//                   at what Section 4.3 names as the limit of Word2Vec scaling: gradient application
//                   and the network)
// All are bound by HBM bandwidth: every byte is touched once, loads are 16 bytes per lane.
#include "dev_common.h"
#include "kernels.h"

// ---------------------------------------------------------------- dense apply
// a thread takes one chunk of 4 elements; the gradients of the chunk are loaded DENSE_INFLIGHT
// sources at a time and summed in source order
#define DENSE_INFLIGHT 4
// STREAM: all accesses around the caches, for models far larger than them (+9 % at 300 M parameters)
template <typename T, bool STREAM>
__global__ void __launch_bounds__(BLOCK) k_dense_apply(DenseApplyArgs a)
{
    const i64 n4 = a.n >> 2;
    const float neg_lr = -a.lr;
    T *theta = (T *)a.theta;
    // one chunk per thread, consecutive workgroups consecutive chunks: the K+2 streams then advance
    // through memory together (a grid-stride loop over a fixed grid was 12 % slower)
    const i64 c = (i64)blockIdx.x * BLOCK + threadIdx.x;
    if (c < n4) {
        // theta stays as loaded (bf16 not yet widened) until the gradients' loads are out
        const typename Raw4<T>::type wr = STREAM ? ldraw_s(theta + 4 * c) : ldraw(theta + 4 * c);
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k0 = 0; k0 < a.n_grads; k0 += DENSE_INFLIGHT) {
            float4 x[DENSE_INFLIGHT];
#pragma unroll
            for (int j = 0; j < DENSE_INFLIGHT; ++j)
                x[j] = (k0 + j >= a.n_grads) ? make_float4(0.f, 0.f, 0.f, 0.f)
                       : (STREAM ? ld4s(a.grads[k0 + j] + 4 * c) : ld4(a.grads[k0 + j] + 4 * c));
#pragma unroll
            for (int j = 0; j < DENSE_INFLIGHT; ++j) {
                acc.x += x[j].x;
                acc.y += x[j].y;
                acc.z += x[j].z;
                acc.w += x[j].w;
            }
        }
        float4 w = widen4(wr);
        w.x = fmaf(neg_lr, acc.x, w.x);
        w.y = fmaf(neg_lr, acc.y, w.y);
        w.z = fmaf(neg_lr, acc.z, w.z);
        w.w = fmaf(neg_lr, acc.w, w.w);
        if (STREAM) st4s(theta + 4 * c, w);
        else st4(theta + 4 * c, w);
    }
    // the last n mod 4 elements, one thread each
    const i64 tail0 = n4 << 2;
    const i64 t = tail0 + (i64)blockIdx.x * BLOCK + threadIdx.x;
    if (blockIdx.x == 0 && t < a.n) {
        float acc = 0.f;
        for (int k = 0; k < a.n_grads; ++k) acc += a.grads[k][t];
        if (sizeof(T) == 4) {
            float *p = (float *)a.theta + t;
            *p = fmaf(neg_lr, acc, *p);
        } else {
            bf16_t *p = (bf16_t *)a.theta + t;
            *p = f32_to_bf16(fmaf(neg_lr, acc, bf16_to_f32(*p)));
        }
    }
}

void tn_launch_dense_apply(const DenseApplyArgs &a, hipStream_t st)
{
    const i64 n4 = a.n >> 2;
    i64 want = (n4 + BLOCK - 1) / BLOCK;
    if (want < 1) want = 1;
    const int blocks = (int)want;
    const bool stream = a.n * (a.dtype == 0 ? 4 : 2) + (i64)a.n_grads * a.n * 4 > ((i64)1 << 30);
    if (a.dtype == 0) {
        if (stream) hipLaunchKernelGGL((k_dense_apply<float, true>), dim3(blocks), dim3(BLOCK), 0, st, a);
        else hipLaunchKernelGGL((k_dense_apply<float, false>), dim3(blocks), dim3(BLOCK), 0, st, a);
    } else {
        if (stream) hipLaunchKernelGGL((k_dense_apply<bf16_t, true>), dim3(blocks), dim3(BLOCK), 0, st, a);
        else hipLaunchKernelGGL((k_dense_apply<bf16_t, false>), dim3(blocks), dim3(BLOCK), 0, st, a);
    }
}

// ---------------------------------------------------------------- lookup
// one wave per requested word: its row, widened to fp32, padding dropped; an id out of range yields
// a row of zeros and sets the status word
template <typename T, int ITERS>
__global__ void __launch_bounds__(BLOCK) k_lookup(LookupArgs a)
{
    const int lane = lane_id();
    const int C4 = a.D >> 2;
    const i64 nw = (i64)gridDim.x * WAVES_PER_BLOCK;
    for (i64 i = (i64)blockIdx.x * WAVES_PER_BLOCK + uniform((int)(threadIdx.x >> 6)); i < a.n; i += nw) {
        const int id = a.ids[i];
        float4 r[ITERS];
        if ((u32)id < (u32)a.V) {
            load_row<T, ITERS>(r, (const T *)a.table + (size_t)id * a.stride, C4, lane);
        } else {
            zero_row<ITERS>(r);
            if (lane == 0) atomicOr(a.status, ST_BAD_ID);
        }
        store_row_s<float, ITERS>(a.out + (size_t)i * a.D, r, C4, lane);
    }
}

template <typename T>
static void launch_lookup_t(const LookupArgs &a, hipStream_t st)
{
    const int iters = (a.D / 4 + WAVE - 1) / WAVE;
    i64 want = (a.n + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    const int blocks = (int)(want > TN_MAX_BLOCKS ? TN_MAX_BLOCKS : want);
    switch (iters) {
    case 1: hipLaunchKernelGGL((k_lookup<T, 1>), dim3(blocks), dim3(BLOCK), 0, st, a); break;
    case 2: hipLaunchKernelGGL((k_lookup<T, 2>), dim3(blocks), dim3(BLOCK), 0, st, a); break;
    case 3: hipLaunchKernelGGL((k_lookup<T, 3>), dim3(blocks), dim3(BLOCK), 0, st, a); break;
    default: hipLaunchKernelGGL((k_lookup<T, 4>), dim3(blocks), dim3(BLOCK), 0, st, a); break;
    }
}

void tn_launch_lookup(const LookupArgs &a, hipStream_t st)
{
    if (a.n <= 0) return;
    if (a.dtype == 0) launch_lookup_t<float>(a, st);
    else launch_lookup_t<bf16_t>(a, st);
}

// ---------------------------------------------------------------- cosine difference
// one wave per row: the three sums <a,b>, <a,a>, <b,b> reduced across the wave, then
// 1 - <a,b> / sqrt(<a,a> <b,b>); a row that is zero in both tables gives 0, in one of them 1
template <typename T, int ITERS>
__global__ void __launch_bounds__(BLOCK) k_cosine_diff(CosineArgs a)
{
    const int lane = lane_id();
    const int C4 = a.D >> 2;
    const i64 nw = (i64)gridDim.x * WAVES_PER_BLOCK;
    for (i64 r = (i64)blockIdx.x * WAVES_PER_BLOCK + uniform((int)(threadIdx.x >> 6)); r < a.V; r += nw) {
        typename Raw4<T>::type xr[ITERS], yr[ITERS];
        load_row_raw<T, ITERS, 1>(xr, (const T *)a.a + (size_t)r * a.stride, C4, lane);   // read once
        load_row_raw<T, ITERS, 1>(yr, (const T *)a.b + (size_t)r * a.stride, C4, lane);
        float4 x[ITERS], y[ITERS];
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            x[it] = widen4(xr[it]);
            y[it] = widen4(yr[it]);
        }
        const float dot = wave_sum_dpp(dot_partial<ITERS>(x, y));
        const float na = wave_sum_dpp(dot_partial<ITERS>(x, x));
        const float nb = wave_sum_dpp(dot_partial<ITERS>(y, y));
        float d;
        if (na > 0.f && nb > 0.f) d = 1.0f - dot / (sqrtf(na) * sqrtf(nb));
        else d = (na == 0.f && nb == 0.f) ? 0.f : 1.f;
        if (lane == 0) a.diff[r] = d;
    }
}

template <typename T>
static void launch_cosine_t(const CosineArgs &a, hipStream_t st)
{
    const int iters = (a.D / 4 + WAVE - 1) / WAVE;
    i64 want = (a.V + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    const int blocks = (int)(want > TN_MAX_BLOCKS ? TN_MAX_BLOCKS : want);
    switch (iters) {
    case 1: hipLaunchKernelGGL((k_cosine_diff<T, 1>), dim3(blocks), dim3(BLOCK), 0, st, a); break;
    case 2: hipLaunchKernelGGL((k_cosine_diff<T, 2>), dim3(blocks), dim3(BLOCK), 0, st, a); break;
    case 3: hipLaunchKernelGGL((k_cosine_diff<T, 3>), dim3(blocks), dim3(BLOCK), 0, st, a); break;
    default: hipLaunchKernelGGL((k_cosine_diff<T, 4>), dim3(blocks), dim3(BLOCK), 0, st, a); break;
    }
}

void tn_launch_cosine_diff(const CosineArgs &a, hipStream_t st)
{
    if (a.V <= 0) return;
    if (a.dtype == 0) launch_cosine_t<float>(a, st);
    else launch_cosine_t<bf16_t>(a, st);
}

// ---------------------------------------------------------------- gradient message in bfloat16
// grid (blocks, 2 tables).  The rows of a sparse gradient are dense, [n][D], so the conversion is flat: a
// workgroup rounds PACK_CHUNKS * 256 consecutive chunks of 4 elements (to nearest even), a thread one
// chunk of every 256, all its loads issued before the first store; the row ids are copied by the threads
// whose chunk index is below n.  The launch covers the capacity (n is only known on the device);
// workgroups beyond the n rows that are there leave at once.
#define PACK_CHUNKS 4
__global__ void __launch_bounds__(BLOCK) k_grad_pack(GradPackArgs a)
{
    const int tb = blockIdx.y;
    i64 n = *a.n[tb];
    if (n < 0) n = 0;
    bool over = false;
    if (n > a.cap[tb]) {   // the source claims more rows than it holds
        n = a.cap[tb];
        over = true;
    }
    if (n > a.out_cap[tb]) {
        n = a.out_cap[tb];
        over = true;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *a.out_n[tb] = (int)n;
        if (over) atomicOr(a.status, ST_OVERFLOW);
    }
    const i64 chunks = n * (a.D >> 2);
    const i64 step = (i64)gridDim.x * BLOCK * PACK_CHUNKS;
    // one pass unless the gradient is larger than the largest grid
    for (i64 base = (i64)blockIdx.x * BLOCK * PACK_CHUNKS + threadIdx.x; base < chunks; base += step) {
        float4 v[PACK_CHUNKS];
#pragma unroll
        for (int j = 0; j < PACK_CHUNKS; ++j) {
            const i64 c = base + (i64)j * BLOCK;
            v[j] = (c < chunks) ? ld4s(a.rows[tb] + 4 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int j = 0; j < PACK_CHUNKS; ++j) {
            const i64 c = base + (i64)j * BLOCK;
            if (c < n) a.out_ids[tb][c] = a.ids[tb][c];
            if (c < chunks) st4s(a.out_rows[tb] + 4 * c, v[j]);
        }
    }
}

void tn_launch_grad_pack(const GradPackArgs &a, hipStream_t st)
{
    i64 chunks = 1;
    for (int tb = 0; tb < 2; ++tb) {
        const i64 rows = a.cap[tb] < a.out_cap[tb] ? a.cap[tb] : a.out_cap[tb];
        if (rows * (a.D >> 2) > chunks) chunks = rows * (a.D >> 2);
    }
    i64 want = (chunks + BLOCK * PACK_CHUNKS - 1) / (BLOCK * PACK_CHUNKS);
    const int blocks = (int)(want > (1 << 22) ? (1 << 22) : want);
    hipLaunchKernelGGL(k_grad_pack, dim3(blocks, 2), dim3(BLOCK), 0, st, a);
}
