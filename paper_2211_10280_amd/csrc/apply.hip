// Gradient application (apply_gradient of Algorithm 1; the "GA" part of Eq. 1 in TensAIR,
// arXiv 2211.10280, Section 2.2) for the own sparse gradient and the K gradients received
// from peers, merged into one pass over the union of their rows:
//     W[r] <- W[r] - lr * (g_0[r] + g_1[r] + ... + g_K[r])
// The paper reports that this step, not the gradient calculation, limits Word2Vec
// scaling (Section 4.3), so it is organised to move every byte once:
//
//   k_apply_index  each source's id list is strictly ascending, so for every 64-row word
//                  of the vocabulary the source's rows in that word are a contiguous run
//                  [start, start + popcount(mask)).  One pass over each id list writes
//                  start[word][k] and mask[word][k] (no atomics, no sort of the union).
//   k_apply        one wave owns 16 consecutive vocabulary rows: lane k holds source k's
//                  (start, mask); rows present in any source are visited in ascending order,
//                  their source rows are streamed (all loads of a row issued together),
//                  summed in source order and applied with one fused multiply-add.  A row
//                  is written by exactly one wave: no write conflicts, fixed order of additions.
#include "dev_common.h"
#include "kernels.h"

#define APPLY_G 16                 // rows per wave
#define APPLY_GPW (64 / APPLY_G)   // waves per 64-row word
#define APPLY_CHUNK 16             // consecutive workgroups kept on one XCD

// ---------------------------------------------------------------- index
// grid: (blocks, n_src, 2 tables).  Virtual thread i in [0, U] of source k:
//   i <  U: if ids[i] opens a new word, fill the gap words before it and build its own word;
//   i == U: fill the words after the last id (covers U = 0).
__global__ void __launch_bounds__(BLOCK) k_apply_index(ApplyArgs a)
{
    const int k = blockIdx.y, tb = blockIdx.z;
    const ApplySrc &s = a.src[tb][k];
    if (s.ids == nullptr) return;
    int U = *s.n_rows;
    if (U < 0) U = 0;
    if ((i64)U > s.capacity) { U = (int)s.capacity; if (threadIdx.x == 0 && blockIdx.x == 0) atomicOr(a.status, ST_OVERFLOW); }
    const int words = (int)((a.V + 63) >> 6);
    const int ns = a.n_src;
    u32 *start = a.start[tb];
    u64 *mask = a.mask[tb];
    for (int i = blockIdx.x * BLOCK + threadIdx.x; i <= U; i += gridDim.x * BLOCK) {
        int wprev = -1;
        if (i > 0) {
            int idp = s.ids[i - 1];
            if ((u32)idp >= (u32)a.V) idp = (int)a.V - 1;
            wprev = idp >> 6;
        }
        if (i == U) {
            for (int w = wprev + 1; w <= words; ++w) {
                start[(size_t)w * ns + k] = (u32)U;
                if (w < words) mask[(size_t)w * ns + k] = 0ull;
            }
            continue;
        }
        int id = s.ids[i];
        if ((u32)id >= (u32)a.V) {
            atomicOr(a.status, ST_BAD_ID);
            id = (int)a.V - 1;
        }
        if (i > 0 && id <= s.ids[i - 1]) atomicOr(a.status, ST_BAD_ORDER);
        const int w = id >> 6;
        if (w == wprev) continue;   // not the first id of its word
        for (int g = wprev + 1; g < w; ++g) {
            start[(size_t)g * ns + k] = (u32)i;
            mask[(size_t)g * ns + k] = 0ull;
        }
        u64 m = 0;
        for (int j = i; j < U; ++j) {
            int idj = s.ids[j];
            if ((u32)idj >= (u32)a.V) idj = (int)a.V - 1;
            if ((idj >> 6) != w) break;
            m |= 1ull << (idj & 63);
        }
        start[(size_t)w * ns + k] = (u32)i;
        mask[(size_t)w * ns + k] = m;
    }
}

// ---------------------------------------------------------------- apply
template <typename T, int ITERS>
__global__ void __launch_bounds__(BLOCK) k_apply(ApplyArgs a, int nblocks)
{
    // keep runs of APPLY_CHUNK consecutive workgroups on one XCD (workgroups are dealt
    // round-robin to the 8 XCDs), so that neighbouring rows -- which share cache lines when
    // the row size is not a multiple of the line -- meet in the same L2
    int bid = blockIdx.x;
    {
        const int per_round = 8 * APPLY_CHUNK;
        int full = (nblocks / per_round) * per_round;
        if (bid < full) {
            int round = bid / per_round, r = bid - round * per_round;
            int xcd = r & 7, slot = r >> 3;
            bid = round * per_round + xcd * APPLY_CHUNK + slot;
        }
    }
    const int tb = blockIdx.y;
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const int gw = bid * WAVES_PER_BLOCK + wave;
    const int word = gw / APPLY_GPW, sub = gw - word * APPLY_GPW;
    const int words = (int)((a.V + 63) >> 6);
    if (word >= words) return;
    const int ns = a.n_src;
    const int C4 = a.D >> 2;

    // lane k < ns: source k's rows inside this wave's 16-row group
    u32 m = 0, st = 0;
    int U = 0;
    u64 rows_ptr = 0;
    if (lane < ns) {
        const ApplySrc &s = a.src[tb][lane];
        if (s.ids != nullptr) {
            u64 mk = a.mask[tb][(size_t)word * ns + lane];
            st = a.start[tb][(size_t)word * ns + lane];
            const int lo = sub * APPLY_G;
            st += (u32)__popcll(mk & ((1ull << lo) - 1ull));
            m = (u32)(mk >> lo) & ((1u << APPLY_G) - 1u);
            U = *s.n_rows;
            if ((i64)U > s.capacity) U = (int)s.capacity;
            rows_ptr = (u64)s.rows;
        }
    }
    u32 um = (u32)uniform((int)wave_or(m));
    T *table = (T *)a.table[tb];
    const float neg_lr = -a.lr;
    const i64 row0 = (i64)word * 64 + sub * APPLY_G;

    while (um) {
        const int b = __builtin_ctz(um);
        um &= um - 1u;
        const i64 r = row0 + b;
        if (r >= a.V) break;   // only reachable with a corrupt index (flagged input)
        // per lane: position of row r in its source (if present and in bounds)
        const u32 pos = st + (u32)__popc(m & ((1u << b) - 1u));
        const bool ok = ((m >> b) & 1u) && (pos < (u32)U);
        u64 S = __ballot(ok);
        T *wrow = table + (size_t)r * a.stride;
        float4 w[ITERS], acc[ITERS];
        load_row<T, ITERS>(w, wrow, C4, lane);
        zero_row<ITERS>(acc);
        while (S) {
            float4 x[4][ITERS];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (S) {
                    const int k = (int)__builtin_ctzll(S);
                    S &= S - 1ull;
                    const float *src = (const float *)rd_lane64(rows_ptr, k) +
                                       (size_t)(u32)rd_lane((int)pos, k) * a.D;
                    load_row<float, ITERS>(x[j], src, C4, lane);
                } else {
                    zero_row<ITERS>(x[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) add_row<ITERS>(acc, x[j]);
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            w[it].x = fmaf(neg_lr, acc[it].x, w[it].x);
            w[it].y = fmaf(neg_lr, acc[it].y, w[it].y);
            w[it].z = fmaf(neg_lr, acc[it].z, w[it].z);
            w[it].w = fmaf(neg_lr, acc[it].w, w[it].w);
        }
        store_row<T, ITERS>(wrow, w, C4, lane);
    }
}

template <typename T>
static void launch_apply_t(const ApplyArgs &a, hipStream_t st)
{
    const int words = (int)((a.V + 63) >> 6);
    const i64 nwaves = (i64)words * APPLY_GPW;
    const int nblocks = (int)((nwaves + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    const int iters = (a.D / 4 + WAVE - 1) / WAVE;
    dim3 grid(nblocks, 2), blk(BLOCK);
    switch (iters) {
    case 1: hipLaunchKernelGGL((k_apply<T, 1>), grid, blk, 0, st, a, nblocks); break;
    case 2: hipLaunchKernelGGL((k_apply<T, 2>), grid, blk, 0, st, a, nblocks); break;
    case 3: hipLaunchKernelGGL((k_apply<T, 3>), grid, blk, 0, st, a, nblocks); break;
    default: hipLaunchKernelGGL((k_apply<T, 4>), grid, blk, 0, st, a, nblocks); break;
    }
}

void tn_launch_apply_index(const ApplyArgs &a, hipStream_t st)
{
    // enough blocks to cover the largest possible id list, grid-strided
    i64 maxcap = 1;
    for (int tb = 0; tb < 2; ++tb)
        for (int k = 0; k < a.n_src; ++k)
            if (a.src[tb][k].ids && a.src[tb][k].capacity > maxcap) maxcap = a.src[tb][k].capacity;
    i64 want = (maxcap + 1 + BLOCK - 1) / BLOCK;
    int blocks = (int)(want > 1024 ? 1024 : want);
    hipLaunchKernelGGL(k_apply_index, dim3(blocks, a.n_src, 2), dim3(BLOCK), 0, st, a);
}

void tn_launch_apply_update(const ApplyArgs &a, hipStream_t st)
{
    if (a.dtype == 0) launch_apply_t<float>(a, st);
    else launch_apply_t<bf16_t>(a, st);
}
