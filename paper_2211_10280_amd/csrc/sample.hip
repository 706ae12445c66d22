// Table initialisation, pair enumeration and Philox/alias negative sampling.
//
// TensAIR (arXiv 2211.10280) trains "a default skip-gram model" (Section 4.4) from
// freshly initialised or pre-trained weights (abstract); the mini-batch is an encoded
// message (Section 3, "Stream Processing").  Here the message is a run of center
// positions of a token stream; the (center, context) pairs and their negatives are
// derived on the GPU as pure functions of position, so no pair list crosses the ABI.
#include "dev_common.h"
#include "kernels.h"

// ---------------------------------------------------------------- init
// Element i = row*D + col of W_in takes word (i mod 4) of Philox(counter = (i/4 lo, i/4 hi,
// 0, 'INIT'), key = seed); u = top 24 bits * 2^-24; value = (u - 0.5) * (1/D) in fp32
// (each operation exactly rounded).  W_out and all padding columns are zero.
template <typename T>
__global__ void k_init_tables(T *w_in, T *w_out, i64 V, int D, int stride, u32 k0, u32 k1,
                              float invD)
{
    i64 total = V * (i64)stride;
    for (i64 at = (i64)blockIdx.x * blockDim.x + threadIdx.x; at < total;
         at += (i64)gridDim.x * blockDim.x) {
        i64 r = at / stride;
        int c = (int)(at - r * stride);
        float val = 0.f;
        if (c < D) {
            u64 i = (u64)r * (u64)D + (u64)c;
            u64 blk = i >> 2;
            philox_out o = philox4x32_10((u32)blk, (u32)(blk >> 32), 0u, 0x494E4954u, k0, k1);
            u32 wsel = (u32)(i & 3);
            u32 x = wsel == 0 ? o.r0 : wsel == 1 ? o.r1 : wsel == 2 ? o.r2 : o.r3;
            float u = (float)(x >> 8) * 0x1p-24f;
            val = __fmul_rn(__fsub_rn(u, 0.5f), invD);
        }
        if constexpr (sizeof(T) == 4) {
            w_in[at] = val;
            w_out[at] = 0.f;
        } else {
            w_in[at] = f32_to_bf16(val);
            w_out[at] = (bf16_t)0;
        }
    }
}

void tn_launch_init_tables(void *w_in, void *w_out, i64 V, int D, int stride, int dtype, u64 seed,
                           hipStream_t st)
{
    i64 total = V * (i64)stride;
    int blocks = (int)((total + BLOCK * 8 - 1) / (BLOCK * 8));
    if (blocks > 65536) blocks = 65536;
    if (blocks < 1) blocks = 1;
    u32 k0 = (u32)(seed & 0xFFFFFFFFu), k1 = (u32)(seed >> 32);
    const float invD = 1.0f / (float)D;  // host division: exactly rounded
    if (dtype == 0)
        hipLaunchKernelGGL(k_init_tables<float>, dim3(blocks), dim3(BLOCK), 0, st, (float *)w_in,
                           (float *)w_out, V, D, stride, k0, k1, invD);
    else
        hipLaunchKernelGGL(k_init_tables<bf16_t>, dim3(blocks), dim3(BLOCK), 0, st, (bf16_t *)w_in,
                           (bf16_t *)w_out, V, D, stride, k0, k1, invD);
}

// ---------------------------------------------------------------- keys
// One thread per (center i, offset index q, slot k): slot 0 is the context, slots 1..N
// are the negatives.  Writes the out-side key list [pair][N+1] (pair-major, the order of
// the occurrence list), the in-side key of every center, and the center token of every pair.
__global__ void k_build_keys(BatchDesc b, i64 V, const u32 *__restrict__ thr,
                             const int *__restrict__ alias, u32 k0, u32 k1, u32 ctr3, int resample,
                             u32 *__restrict__ out_keys, u32 *__restrict__ in_keys,
                             int *__restrict__ pair_center, int *__restrict__ neg_dbg,
                             int *__restrict__ status)
{
    const int Np1 = b.N + 1;
    const i64 per_center = (i64)2 * b.w * Np1;
    const i64 total = (i64)b.n_centers * per_center;
    i64 t = (i64)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    int i = (int)(t / per_center);
    int rem = (int)(t - (i64)i * per_center);
    int q = rem / Np1;
    int k = rem - q * Np1;
    i64 p = b.begin + i;
    int c = b.tok[p];
    if ((u32)c >= (u32)V) {  // invalid token: keep every later access in range, flag it
        c = 0;
        atomicOr(status, ST_BAD_ID);
    }
    if (rem == 0) in_keys[i] = (u32)c;
    i64 left = p < b.w ? p : b.w;
    i64 right = (b.T - 1 - p) < b.w ? (b.T - 1 - p) : b.w;
    i64 rank;
    i64 o;
    if (q < b.w) {
        if (q < b.w - left) return;
        rank = q - (b.w - left);
        o = (i64)q - b.w;
    } else {
        if (q - b.w >= right) return;
        rank = left + (q - b.w);
        o = (i64)q - b.w + 1;
    }
    i64 pair = pairs_before(p, b.T, b.w) - b.pair_base + rank;
    int ctx = b.tok[p + o];
    if ((u32)ctx >= (u32)V) {
        ctx = 0;
        atomicOr(status, ST_BAD_ID);
    }
    int id;
    if (k == 0) {
        id = ctx;
        pair_center[pair] = c;
    } else {
        philox_out r = philox4x32_10((u32)((u64)p & 0xFFFFFFFFu), (u32)((u64)p >> 32),
                                     (u32)q * 65536u + (u32)(k - 1), ctr3, k0, k1);
        u32 bkt = (u32)(((u64)r.r0 * (u64)V) >> 32);
        id = (r.r1 < thr[bkt]) ? (int)bkt : alias[bkt];
        if (resample && (id == c || id == ctx)) {   // the variant: one more draw from the block's other two words
            bkt = (u32)(((u64)r.r2 * (u64)V) >> 32);
            id = (r.r3 < thr[bkt]) ? (int)bkt : alias[bkt];
        }
        if (neg_dbg) neg_dbg[pair * b.N + (k - 1)] = id;
    }
    out_keys[pair * Np1 + k] = (u32)id;
}

void tn_launch_build_keys(const BatchDesc &b, i64 V, const u32 *thr, const int *alias, u64 seed,
                          u32 worker, u32 epoch, bool resample, u32 *out_keys, u32 *in_keys,
                          int *pair_center, int *neg_dbg, int *status, hipStream_t st)
{
    i64 total = (i64)b.n_centers * 2 * b.w * (b.N + 1);
    int blocks = (int)((total + BLOCK - 1) / BLOCK);
    hipLaunchKernelGGL(k_build_keys, dim3(blocks), dim3(BLOCK), 0, st, b, V, thr, alias,
                       (u32)(seed & 0xFFFFFFFFu), (u32)(seed >> 32), worker + 65536u * epoch,
                       resample ? 1 : 0, out_keys, in_keys, pair_center, neg_dbg, status);
}
