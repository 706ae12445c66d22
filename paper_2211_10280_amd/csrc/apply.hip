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
//                  start[word][k] and mask[word][k]; a wave combines the bits of the ids it
//                  holds with a segmented OR, so only words that straddle two waves need an
//                  (integer, order-independent) atomic.  No sort of the union is needed.
//   k_apply        one wave owns G consecutive vocabulary rows of both tables: a lane holds one
//                  source's (start, mask); rows present in any source are visited in ascending order,
//                  their source rows are streamed (all loads of a row issued together),
//                  summed in source order and applied with one fused multiply-add.  A row
//                  is written by exactly one wave: no write conflicts, fixed order of additions.
//
// Measured and rejected: splitting the update into the rows the own gradient does not touch (which
// could run next to the gradient calculation) and the rows it touches.  The two halves read every
// peer block with holes, lose 20 % of the bandwidth between them, and the gradient calculation is
// itself bound by memory traffic, so nothing was gained by the overlap.

#include <string.h>

#include <type_traits>

#include "aux_dev.h"
#include "dev_common.h"
#include "kernels.h"

#ifndef APPLY_CHUNK
#define APPLY_CHUNK 16   // consecutive workgroups kept on one XCD
#endif

// ---------------------------------------------------------------- index
// (the work itself is in aux_dev.h: inside tensair_step it rides at the front of other launches)
__global__ void __launch_bounds__(BLOCK) k_apply_clear(u64 *m0, u64 *m1, size_t n)
{
    aux_clear_masks(m0, m1, n, (int)blockIdx.x);
}

// grid: (blocks, sources, 2 tables); every wave takes 64 consecutive ids of source k0 + blockIdx.y.
__global__ void __launch_bounds__(BLOCK) k_apply_index(ApplyArgs a, int k0)
{
    aux_index_source(a, k0 + (int)blockIdx.y, (int)blockIdx.z, (int)blockIdx.x, (int)gridDim.x);
}

// ---------------------------------------------------------------- apply
#ifndef APPLY_G
#define APPLY_G 4   // vocabulary rows per wave (measured: 16 -> 4 rows gains 4 %)
#endif
#ifndef GRADSUM_G
#define GRADSUM_G 8   // vocabulary rows per wave in the sum of two gradients (4 / 8 / 16 / 32: 0.213 / 0.185 / 0.186 / 0.206 ms)
#endif
#ifndef APPLY_G_SPARSE
#define APPLY_G_SPARSE 16   // the same where few of the vocabulary's rows are touched
#endif

// Stochastic rounding of one fp32 value to bfloat16: 16 random bits are added below the bfloat16 mantissa
// and the sum is truncated, so the value goes up with probability (discarded bits)/2^16; infinities and
// NaN are kept.
__device__ __forceinline__ u32 sr_bf16(float f, u32 rnd)
{
    const u32 u = __float_as_uint(f);
    if ((u & 0x7F800000u) == 0x7F800000u) return (u >> 16) | ((u & 0xFFFFu) ? 0x40u : 0u);
    return (u + (rnd & 0xFFFFu)) >> 16;
}
struct SrArgs {
    int on;
    u32 k0, k1, serial, tag;   // Philox key, counter words 2 and 3 ('SRND' + table)
};

// Sum of the sources of one row (bits of S, ascending: own first, then peers), W <- W - lr * sum.
// lane 32*tb + k holds the position `pos` of the row in source k and that source's row pointer.
// STREAM: the accesses go around the caches (non-temporal), for tables far larger than the caches.  Of a
// table row only the cache lines it fills completely are loaded that way: a row of 1200 bytes shares its
// first and last line with its neighbours, and with those two lines loaded through the caches the
// neighbour (mostly touched too, by the next wave) finds them there (measured: update 0.728 -> 0.685 ms;
// the same treatment of the stores, or of the gradient rows, gains less or loses).
// PACKED: the peers' rows are bfloat16 messages.  The own row (lane `own`) is fp32 and is loaded ahead of
// the loop, so that every load inside the loop has the same type and no branch separates them.
// (Measured on bf16 rows: widened right after each load the update ran 0.77 ms where the fp32 messages
// take 0.69 ms -- every load was followed by a wait for its data.)
template <typename T, int ITERS, bool STREAM, bool PACKED>
__device__ __forceinline__ void update_row(T *wrow, u64 S, u64 rows_ptr, u32 pos, int D, int C4, int lane,
                                           float neg_lr, int own, u64 chunk0, const SrArgs &sr, bf16_t *msg_row)
{
    typedef typename std::conditional<PACKED, bf16_t, float>::type G;
    // table row and source rows stay as loaded (bf16 not yet widened) until every load of the batch is out
    typename Raw4<T>::type wraw[ITERS];
    float4 acc[ITERS];
    load_row_raw<T, ITERS, STREAM ? 2 : 0>(wraw, wrow, C4, lane);
    zero_row<ITERS>(acc);
    float4 x0[ITERS];
    bool own_pending = PACKED;
    if (PACKED) {
        if ((S >> own) & 1ull) {
            const float *src = (const float *)rd_lane64(rows_ptr, own) + (size_t)(u32)rd_lane((int)pos, own) * D;
            load_row_raw<float, ITERS, STREAM ? 1 : 0>(x0, src, C4, lane);
        } else {
            zero_row<ITERS>(x0);
        }
        S &= ~(1ull << own);
    }
    while (S || own_pending) {
        typename Raw4<G>::type x[4][ITERS];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (S) {
                const int k = (int)__builtin_ctzll(S);
                S &= S - 1ull;
                const G *src = (const G *)rd_lane64(rows_ptr, k) + (size_t)(u32)rd_lane((int)pos, k) * D;
                load_row_raw<G, ITERS, STREAM ? 1 : 0>(x[j], src, C4, lane);
            } else {
                zero_row_raw<ITERS>(x[j]);
            }
        }
        if (PACKED && own_pending) add_row<ITERS>(acc, x0);   // the own row first, once the peers' loads are out
        own_pending = false;
#pragma unroll
        for (int j = 0; j < 4; ++j) add_row_raw<ITERS>(acc, x[j]);
    }
    // the own row on its way out as a bfloat16 message (its load has long arrived by now)
    if (PACKED && msg_row != nullptr) store_row_s<bf16_t, ITERS>(msg_row, x0, C4, lane);
    float4 w[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        w[it] = widen4(wraw[it]);
        w[it].x = fmaf(neg_lr, acc[it].x, w[it].x);
        w[it].y = fmaf(neg_lr, acc[it].y, w[it].y);
        w[it].z = fmaf(neg_lr, acc[it].z, w[it].z);
        w[it].w = fmaf(neg_lr, acc[it].w, w[it].w);
    }
    if constexpr (sizeof(T) == 2) {
        if (sr.on) {
            // the variant: element i = row*D + col takes the low half of word (i mod 4) of
            // Philox(counter = (i/4 low, i/4 high, serial, 'SRND' + table), key = seed); chunk0 = row*D/4
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int c = lane + WAVE * it;
                if (c < C4) {
                    const u64 blk = chunk0 + (u64)c;
                    const philox_out o = philox4x32_10((u32)blk, (u32)(blk >> 32), sr.serial, sr.tag, sr.k0, sr.k1);
                    v2u p;
                    p.x = sr_bf16(w[it].x, o.r0) | (sr_bf16(w[it].y, o.r1) << 16);
                    p.y = sr_bf16(w[it].z, o.r2) | (sr_bf16(w[it].w, o.r3) << 16);
                    if (STREAM) __builtin_nontemporal_store(p, (GLOBAL_AS v2u *)(wrow + 4 * c));
                    else *reinterpret_cast<v2u *>(wrow + 4 * c) = p;
                }
            }
            return;
        }
    }
    if (STREAM) store_row_s<T, ITERS>(wrow, w, C4, lane);
    else store_row<T, ITERS>(wrow, w, C4, lane);
}

// occupancy cap, so that the kernels of the second stream (the preparation of the next mini-batch) find wave
// slots next to this one; measured with table rows on 128-byte lines: 5 / 6 / 7 / 8 waves per SIMD give a step of
// 0.846 / 0.836 / 0.823 / 0.828 ms at a million words, and no difference at two million (3.46-3.49 ms)
#ifndef APPLY_MAX_WAVES
#define APPLY_MAX_WAVES 7
#endif
template <typename T, int ITERS, int G, bool STREAM, bool PACKED>
__global__ void __launch_bounds__(BLOCK) __attribute__((amdgpu_waves_per_eu(1, APPLY_MAX_WAVES)))
k_apply(ApplyArgs a, int nblocks)
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
    constexpr int GPW = 64 / G;
    const int wave = uniform((int)(threadIdx.x >> 6)), lane = lane_id();
    const int gw = bid * WAVES_PER_BLOCK + wave;
    const int word = gw / GPW, sub = gw - word * GPW;
    const int words = (int)((a.V + 63) >> 6);
    if (word >= words) return;
    const int ns = a.n_src;
    const int C4 = a.D >> 2;

    // lanes 0..31 hold W_in's sources, lanes 32..63 W_out's: lane 32*tb + k has source k's rows
    // inside this wave's group of rows of table tb
    u64 m = 0;
    u32 st = 0;
    int U = 0;
    u64 rows_ptr = 0;
    {
        const int tb = lane >> 5, k = lane & 31;
        if (k < ns) {
            const ApplySrc &s = a.src[tb][k];
            if (s.ids != nullptr) {
                u64 mk = a.mask[tb][idx_at(words, k, word)];
                st = a.start[tb][idx_at(words, k, word)];
                const int lo = sub * G;
                st += (u32)__popcll(mk & ((1ull << lo) - 1ull));
                m = (G == 64) ? mk : ((mk >> lo) & ((1ull << (G & 63)) - 1ull));
                U = *s.n_rows;
                if ((i64)U > s.capacity) U = (int)s.capacity;
                rows_ptr = (u64)s.rows;
                if (PACKED && k == 0 && gw == 0 && a.msg_n[tb] != nullptr) *a.msg_n[tb] = U < 0 ? 0 : U;
            }
        }
    }
    const float neg_lr = -a.lr;
    const i64 row0 = (i64)word * 64 + sub * G;

#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const bool mine = (lane >> 5) == tb;
        u64 um;
        {
            u32 lo32 = (u32)uniform((int)wave_or(mine ? (u32)m : 0u));
            u32 hi32 = (G > 32) ? (u32)uniform((int)wave_or(mine ? (u32)(m >> 32) : 0u)) : 0u;
            um = ((u64)hi32 << 32) | lo32;
        }
        T *table = (T *)a.table[tb];
        while (um) {
            const int b = (int)__builtin_ctzll(um);
            um &= um - 1ull;
            const i64 r = row0 + b;
            if (r >= a.V) break;   // only reachable with a corrupt index (flagged input)
            // per lane: position of row r in its source (if present and in bounds)
            const u32 pos = st + (u32)__popcll(m & ((1ull << b) - 1ull));
            const bool ok = mine && ((m >> b) & 1ull) && (pos < (u32)U);
            const u64 S = __ballot(ok);   // bit 32*tb + k: source k has row r
            const SrArgs sr = {a.sr, a.sr_k0, a.sr_k1, a.sr_serial, 0x53524E44u + (u32)tb};
            bf16_t *msg_row = nullptr;
            if (PACKED && a.msg_rows[tb] != nullptr && ((S >> (32 * tb)) & 1ull)) {
                const u32 at = (u32)rd_lane((int)pos, 32 * tb);          // place of row r in the own gradient
                msg_row = (bf16_t *)a.msg_rows[tb] + (size_t)at * a.D;
                if (lane == 32 * tb) a.msg_ids[tb][at] = (int)r;
            }
            update_row<T, ITERS, STREAM, PACKED>(table + (size_t)r * a.stride, S, rows_ptr, pos, a.D, C4, lane, neg_lr,
                                                 32 * tb, (u64)r * (u64)C4, sr, msg_row);
        }
    }
}

// The same update for rows of at most 32 chunks (D <= 128).  A whole wave per row would leave most of its lanes
// without a chunk, and the update's rate follows the number of row loads a wave issues, not their width
// (measured at a million words and 7 peers with whole-wave rows: 4.1 TB/s at D = 128 and 1.5 TB/s at D = 32 against
// 5.9 TB/s at D = 256; update 0.36 and 0.25 ms, with this kernel 0.31 and 0.09 ms).  Here a wave updates 64/SUB
// rows at a time, one per group of SUB lanes: each pass takes the next rows of the wave's share that any source
// has, the lanes that hold the sources' (start, mask) hand every group its row's positions through lane
// shuffles, and a group walks its own row's sources, four loads in flight, in source order -- every row is
// summed exactly as in k_apply.  ROWS: vocabulary rows per group and wave (more where few rows are touched, see
// launch_apply_sub).  Gradient messages in bfloat16 (PACKED) stay with k_apply.
#ifndef APPLY_SUB_ROWS
#define APPLY_SUB_ROWS 4   // rows per group of lanes and wave
#endif
template <typename T, int SUB, int ROWS, bool STREAM>
__global__ void __launch_bounds__(BLOCK) __attribute__((amdgpu_waves_per_eu(1, APPLY_MAX_WAVES)))
k_apply_sub(ApplyArgs a, int nblocks)
{
    constexpr int RPW = WAVE / SUB;   // rows in one pass of a wave
    constexpr int G = (ROWS * RPW > 32) ? 32 : ROWS * RPW;   // vocabulary rows per wave
    constexpr int GPW = 64 / G;
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
    const int wave = uniform((int)(threadIdx.x >> 6)), lane = lane_id();
    const int gw = bid * WAVES_PER_BLOCK + wave;
    const int word = gw / GPW, sub = gw - word * GPW;
    const int words = (int)((a.V + 63) >> 6);
    if (word >= words) return;
    const int ns = a.n_src;
    const int C4 = a.D >> 2;
    const int slot = lane / SUB, sl = lane - slot * SUB;   // group of the lane, chunk of the row it holds

    // lane 32*tb + k: source k's rows inside this wave's share of table tb, as in k_apply
    u32 m = 0, st = 0;
    int U = 0;
    u64 rows_ptr = 0;
    {
        const int tb = lane >> 5, k = lane & 31;
        if (k < ns) {
            const ApplySrc &s = a.src[tb][k];
            if (s.ids != nullptr) {
                const u64 mk = a.mask[tb][idx_at(words, k, word)];
                const int lo = sub * G;
                st = a.start[tb][idx_at(words, k, word)] + (u32)__popcll(mk & ((1ull << lo) - 1ull));
                m = (u32)((mk >> lo) & ((1ull << G) - 1ull));
                U = *s.n_rows;
                if ((i64)U > s.capacity) U = (int)s.capacity;
                rows_ptr = (u64)s.rows;
            }
        }
    }
    const int ptr_lo = (int)(u32)rows_ptr, ptr_hi = (int)(u32)(rows_ptr >> 32);
    const float neg_lr = -a.lr;
    const i64 row0 = (i64)word * 64 + sub * G;

#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const bool mine = (lane >> 5) == tb;
        u32 um = (u32)uniform((int)wave_or(mine ? m : 0u));
        T *table = (T *)a.table[tb];
        while (um) {
            // the next RPW rows: lane 32*tb + k works out source k's position of each, group s keeps row s
            int pos_s[RPW];
            u32 S_my = 0;
            int b_my = -1;
#pragma unroll
            for (int s = 0; s < RPW; ++s) {
                pos_s[s] = 0;
                if (um) {
                    const int b = (int)__builtin_ctz(um);
                    um &= um - 1u;
                    if (row0 + b >= a.V) {   // only reachable with a corrupt index (flagged input)
                        um = 0;
                    } else {
                        const u32 pos = st + (u32)__popc(m & ((1u << b) - 1u));
                        const bool ok = mine && ((m >> b) & 1u) && (pos < (u32)U);
                        const u64 S = __ballot(ok);
                        pos_s[s] = (int)pos;
                        if (slot == s) {
                            S_my = (u32)(S >> (32 * tb));
                            b_my = b;
                        }
                    }
                }
            }
            const bool act = (b_my >= 0) && (sl < C4);
            const i64 r = row0 + (b_my >= 0 ? b_my : 0);
            T *wrow = table + (size_t)r * a.stride;
            T *wp = wrow + 4 * sl;
            typename Raw4<T>::type wraw;
            zero_raw(wraw);
            bool around = STREAM;
            if (STREAM) {   // a 128-byte line shared with the neighbouring rows goes through the caches
                const uintptr_t lo = (uintptr_t)wrow, hi = lo + (size_t)C4 * 4 * sizeof(T);
                const uintptr_t line = (uintptr_t)wp & ~(uintptr_t)127;
                around = line >= lo && line + 128 <= hi;
            }
            if (act) {
                if (around) wraw = ldraw_s(wp);
                else wraw = ldraw(wp);
            }
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            u32 S_it = S_my;
            while (__ballot(S_it != 0u)) {
                float4 x[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool valid = S_it != 0u;
                    const int k = valid ? (int)__builtin_ctz(S_it) : 0;
                    S_it &= S_it - 1u;
                    const int from = 32 * tb + k;
                    int pos = 0;
#pragma unroll
                    for (int s = 0; s < RPW; ++s) {
                        const int v = __shfl(pos_s[s], from, WAVE);
                        pos = (slot == s) ? v : pos;
                    }
                    const u64 ptr = ((u64)(u32)__shfl(ptr_hi, from, WAVE) << 32) | (u64)(u32)__shfl(ptr_lo, from, WAVE);
                    x[j] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (valid && act) {
                        const float *src = (const float *)ptr + (size_t)(u32)pos * a.D + 4 * sl;
                        x[j] = STREAM ? ld4s(src) : ld4(src);
                    }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc.x += x[j].x;
                    acc.y += x[j].y;
                    acc.z += x[j].z;
                    acc.w += x[j].w;
                }
            }
            float4 w = widen4(wraw);
            w.x = fmaf(neg_lr, acc.x, w.x);
            w.y = fmaf(neg_lr, acc.y, w.y);
            w.z = fmaf(neg_lr, acc.z, w.z);
            w.w = fmaf(neg_lr, acc.w, w.w);
            if (!act) continue;
            if constexpr (sizeof(T) == 2) {
                if (a.sr) {   // the variant: the same draw per element as in update_row
                    const u64 blk = (u64)r * (u64)C4 + (u64)sl;
                    const philox_out o = philox4x32_10((u32)blk, (u32)(blk >> 32), a.sr_serial, 0x53524E44u + (u32)tb,
                                                       a.sr_k0, a.sr_k1);
                    v2u p;
                    p.x = sr_bf16(w.x, o.r0) | (sr_bf16(w.y, o.r1) << 16);
                    p.y = sr_bf16(w.z, o.r2) | (sr_bf16(w.w, o.r3) << 16);
                    if (STREAM) __builtin_nontemporal_store(p, (GLOBAL_AS v2u *)wp);
                    else *reinterpret_cast<v2u *>(wp) = p;
                    continue;
                }
            }
            if (STREAM) st4s(wp, w);
            else st4(wp, w);
        }
    }
}

template <typename T, int SUB, int ROWS, bool STREAM>
static void launch_apply_sub_r(const ApplyArgs &a, hipStream_t st)
{
    const int words = (int)((a.V + 63) >> 6);
    constexpr int G = (ROWS * (WAVE / SUB) > 32) ? 32 : ROWS * (WAVE / SUB);
    const i64 nwaves = (i64)words * (64 / G);
    const int nblocks = (int)((nwaves + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    hipLaunchKernelGGL((k_apply_sub<T, SUB, ROWS, STREAM>), dim3(nblocks), dim3(BLOCK), 0, st, a, nblocks);
}

// few of the vocabulary's rows touched, going by the sources' capacities (see launch_apply_t)
static bool sparse_union(const ApplyArgs &a)
{
    i64 cap = 0;
    for (int k = 0; k < a.n_src; ++k)
        if (a.src[1][k].ids != nullptr) cap += a.src[1][k].capacity;
    return 4 * cap < 3 * a.V;
}

// 4 rows per group of lanes and wave, or 32 rows per wave where few rows are touched (8 M words, D = 128, bf16:
// update 0.67 -> 0.42 ms; 16 M words, D = 64: 0.58 -> 0.40 ms)
template <typename T, int SUB, bool STREAM>
static void launch_apply_sub(const ApplyArgs &a, hipStream_t st)
{
    if (SUB > 8 && sparse_union(a)) launch_apply_sub_r<T, SUB, 16, STREAM>(a, st);
    else launch_apply_sub_r<T, SUB, APPLY_SUB_ROWS, STREAM>(a, st);
}

template <typename T, int G, bool STREAM, bool PACKED>
static void launch_apply_g(const ApplyArgs &a, hipStream_t st)
{
    const int iters = (a.D / 4 + WAVE - 1) / WAVE;
    const int words = (int)((a.V + 63) >> 6);
    const i64 nwaves = (i64)words * (64 / G);
    const int nblocks = (int)((nwaves + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    dim3 grid(nblocks), blk(BLOCK);
    switch (iters) {
    case 1: hipLaunchKernelGGL((k_apply<T, 1, G, STREAM, PACKED>), grid, blk, 0, st, a, nblocks); break;
    case 2: hipLaunchKernelGGL((k_apply<T, 2, G, STREAM, PACKED>), grid, blk, 0, st, a, nblocks); break;
    case 3: hipLaunchKernelGGL((k_apply<T, 3, G, STREAM, PACKED>), grid, blk, 0, st, a, nblocks); break;
    default: hipLaunchKernelGGL((k_apply<T, 4, G, STREAM, PACKED>), grid, blk, 0, st, a, nblocks); break;
    }
}

// Rows per wave.  Where most vocabulary rows are touched, 4 rows per wave are best (16: -4 % at a million words and
// 7 peers, two thirds of the rows touched); where few are, most waves of such a grid find nothing, and 16 rows per
// wave win (same gradients, update at 2 / 4 / 8 million words: 0.85 / 1.11 / 1.49 ms with 4 rows, 0.86 / 1.01 / 1.16 ms
// with 16, 64 rows no better).  How many rows the union has is only known on the device; the sources' capacities
// bound it, and below three quarters of a row of capacity per vocabulary row the sparse shape is taken.
template <typename T, bool STREAM, bool PACKED>
static void launch_apply_t(const ApplyArgs &a, hipStream_t st)
{
    if (sparse_union(a)) launch_apply_g<T, APPLY_G_SPARSE, STREAM, PACKED>(a, st);
    else launch_apply_g<T, APPLY_G, STREAM, PACKED>(a, st);
}

template <typename T, bool STREAM>
static void launch_apply_p(const ApplyArgs &a, hipStream_t st)
{
    const int C4 = a.D / 4;
    if (a.packed) launch_apply_t<T, STREAM, true>(a, st);
    else if (C4 > 32) launch_apply_t<T, STREAM, false>(a, st);
    else if (C4 > 16) launch_apply_sub<T, 32, STREAM>(a, st);
    else if (C4 > 8) launch_apply_sub<T, 16, STREAM>(a, st);
    else launch_apply_sub<T, 8, STREAM>(a, st);
}

static int index_blocks_for(const ApplyArgs &a, int k_begin, int k_end)
{
    // enough waves to cover the largest possible id list, grid-strided
    i64 maxcap = 1;
    for (int tb = 0; tb < 2; ++tb)
        for (int k = k_begin; k < k_end; ++k)
            if (a.src[tb][k].ids && a.src[tb][k].capacity > maxcap) maxcap = a.src[tb][k].capacity;
    i64 want = (maxcap + BLOCK * AUX_INDEX_UNROLL - 1) / (BLOCK * AUX_INDEX_UNROLL);
    return (int)(want > 2048 ? 2048 : want);
}

#ifndef AUX_COPY_BLOCKS
#define AUX_COPY_BLOCKS 32
#endif
#ifndef AUX_INDEX_BLOCKS
#define AUX_INDEX_BLOCKS 256
#endif
void tn_aux_none(AuxWork &x) { memset(&x, 0, sizeof(x)); }

void tn_aux_add_clear(AuxWork &x, u64 *mask_in, u64 *mask_out, size_t n)
{
    x.clear_mask[0] = mask_in;
    x.clear_mask[1] = mask_out;
    x.clear_n = n;
    x.clear_blocks = (int)((x.clear_n + BLOCK - 1) / BLOCK);
    x.total = x.clear_blocks + 2 * x.copy_blocks + 2 * (x.k_end - x.k_begin) * x.index_blocks;
}

void tn_aux_add_copy(AuxWork &x, const RowIndexCopy &c, i64 max_rows)
{
    x.copy = c;
    i64 want = (max_rows + 1 + BLOCK - 1) / BLOCK;
    x.copy_blocks = (int)(want > AUX_COPY_BLOCKS ? AUX_COPY_BLOCKS : want);
    x.total = x.clear_blocks + 2 * x.copy_blocks + 2 * (x.k_end - x.k_begin) * x.index_blocks;
}

void tn_aux_add_index(AuxWork &x, const ApplyArgs &a, int k_begin, int k_end)
{
    if (k_end <= k_begin) return;
    x.apply = a;
    x.k_begin = k_begin;
    x.k_end = k_end;
    // few workgroups per id list, each striding over it: riding in front of another kernel's grid, every
    // workgroup that finds nothing to do still delays that kernel's own
    x.index_blocks = index_blocks_for(a, k_begin, k_end);
    if (x.index_blocks > AUX_INDEX_BLOCKS) x.index_blocks = AUX_INDEX_BLOCKS;
    x.total = x.clear_blocks + 2 * x.copy_blocks + 2 * (x.k_end - x.k_begin) * x.index_blocks;
}

void tn_launch_apply_clear(const ApplyArgs &a, hipStream_t st)
{
    const size_t words = (size_t)((a.V + 63) >> 6);
    const size_t n = words * (size_t)a.n_src;
    hipLaunchKernelGGL(k_apply_clear, dim3((unsigned)((n + BLOCK - 1) / BLOCK)), dim3(BLOCK), 0, st,
                       a.mask[0], a.mask[1], n);
}

// index of the sources k_begin .. k_end-1 (the masks must have been cleared)
void tn_launch_apply_index(const ApplyArgs &a, int k_begin, int k_end, hipStream_t st)
{
    if (k_end <= k_begin) return;
    const int blocks = index_blocks_for(a, k_begin, k_end);
    hipLaunchKernelGGL(k_apply_index, dim3(blocks, k_end - k_begin, 2), dim3(BLOCK), 0, st, a, k_begin);
}

void tn_launch_apply_update(const ApplyArgs &a, hipStream_t st)
{
    // Tables that dwarf the caches (256 MB memory-side, 32 MB of L2) are updated around them: a row
    // touched here is not touched again before megabytes of others have passed, and what the gradient
    // calculation left in the caches (the frequent rows, which its next pass reads again) survives the
    // update.  Measured at a 2 x 1.2 GB model: step 0.953 -> 0.930 ms.  Small tables stay cached.
    const i64 elem = a.dtype == 0 ? 4 : 2;
    const bool stream = 2 * a.V * (i64)a.stride * elem > ((i64)1 << 30);
    if (a.dtype == 0) stream ? launch_apply_p<float, true>(a, st) : launch_apply_p<float, false>(a, st);
    else stream ? launch_apply_p<bf16_t, true>(a, st) : launch_apply_p<bf16_t, false>(a, st);
}

// ---------------------------------------------------------------- sum of sparse gradients
// Algorithm 1 keeps the gradients a Model instance has computed and not yet sent in a buffer
// ("gradients += gradient") and broadcasts the buffer every maxGradBuffer steps.  In the sparse form
// that sum lists the union of the rows: a row one source has is taken over, a row several have is
// added in source order (fp32, one rounding per addition).  The same per-word index as for the table
// update tells where every source's rows are; a scan over the popcounts of the united masks gives each
// 64-row word its place in the output, so ids come out ascending without any sort or merge.
#define UNION_WPT (TN_UNION_WORDS / BLOCK)

__device__ __forceinline__ u64 united_mask(const u64 *mask, size_t words, size_t word, int ns)
{
    u64 u = 0;
    for (int k = 0; k < ns; ++k) u |= mask[idx_at((i64)words, k, (i64)word)];
    return u;
}

// block-wide exclusive scan of one int per thread; total = block total
__device__ __forceinline__ int block_scan1(int x, int &total, int *sm)
{
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int incl = (int)wave_incl_scan((u32)x, lane);
    if (lane == WAVE - 1) sm[wave] = incl;
    __syncthreads();
    int off = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < WAVES_PER_BLOCK; ++w) {
        if (w < wave) off += sm[w];
        total += sm[w];
    }
    __syncthreads();
    return off + incl - x;
}

// grid (blocks, 2 tables): rows of the union inside each block of TN_UNION_WORDS words
__global__ void __launch_bounds__(BLOCK) k_union_count(GradSumArgs g)
{
    __shared__ int sm[WAVES_PER_BLOCK];
    const int tb = blockIdx.y, ns = g.a.n_src;
    const size_t words = (size_t)((g.a.V + 63) >> 6);
    const size_t w0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * UNION_WPT;
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < UNION_WPT; ++j)
        if (w0 + j < words) cnt += __popcll(united_mask(g.a.mask[tb], words, w0 + j, ns));
    int total;
    block_scan1(cnt, total, sm);
    if (threadIdx.x == 0) g.wblk[tb][blockIdx.x] = (u32)total;
}

// grid (blocks, 2 tables): place of every word in the output; the last block writes the row count
__global__ void __launch_bounds__(BLOCK) k_union_offsets(GradSumArgs g)
{
    __shared__ int sm[WAVES_PER_BLOCK];
    const int tb = blockIdx.y, ns = g.a.n_src;
    const size_t words = (size_t)((g.a.V + 63) >> 6);
    int before = 0;
    for (int j = threadIdx.x; j < (int)blockIdx.x; j += BLOCK) before += (int)g.wblk[tb][j];
    int prefix;
    block_scan1(before, prefix, sm);   // prefix = rows of the union in all earlier blocks
    const size_t w0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * UNION_WPT;
    int c[UNION_WPT];
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < UNION_WPT; ++j) {
        c[j] = (w0 + j < words) ? __popcll(united_mask(g.a.mask[tb], words, w0 + j, ns)) : 0;
        cnt += c[j];
    }
    int total;
    int run = prefix + block_scan1(cnt, total, sm);
#pragma unroll
    for (int j = 0; j < UNION_WPT; ++j) {
        if (w0 + j < words) g.wbase[tb][w0 + j] = (u32)run;
        run += c[j];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        i64 U = (i64)prefix + total;
        if (U > g.out_cap[tb]) {
            U = g.out_cap[tb];
            atomicOr(g.a.status, ST_OVERFLOW);
        }
        *g.out_n[tb] = (int)U;
    }
}

// one wave per G consecutive vocabulary rows of both tables, as in k_apply
template <int ITERS, int G>
__global__ void __launch_bounds__(BLOCK) k_grad_sum(GradSumArgs g, int nblocks)
{
    const ApplyArgs &a = g.a;
    constexpr int GPW = 64 / G;
    const int wave = uniform((int)(threadIdx.x >> 6)), lane = lane_id();
    const int gw = blockIdx.x * WAVES_PER_BLOCK + wave;
    const int word = gw / GPW, sub = gw - word * GPW;
    const int words = (int)((a.V + 63) >> 6);
    if (word >= words) return;
    const int ns = a.n_src;
    const int C4 = a.D >> 2;
    const int lo = sub * G;

    u64 mk = 0;
    u32 st = 0;
    int U = 0;
    u64 rows_ptr = 0;
    {
        const int tb = lane >> 5, k = lane & 31;
        if (k < ns) {
            const ApplySrc &s = a.src[tb][k];
            if (s.ids != nullptr) {
                mk = a.mask[tb][idx_at(words, k, word)];
                st = a.start[tb][idx_at(words, k, word)];
                U = *s.n_rows;
                if ((i64)U > s.capacity) U = (int)s.capacity;
                rows_ptr = (u64)s.rows;
            }
        }
    }
    const i64 row0 = (i64)word * 64;
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const bool mine = (lane >> 5) == tb;
        // rows of the word that any source has
        const u32 ulo = (u32)uniform((int)wave_or(mine ? (u32)mk : 0u));
        const u32 uhi = (u32)uniform((int)wave_or(mine ? (u32)(mk >> 32) : 0u));
        const u64 uw = ((u64)uhi << 32) | ulo;
        u64 um = (G == 64) ? uw : ((uw >> lo) & ((1ull << (G & 63)) - 1ull));
        const u32 base = g.wbase[tb][word];
        while (um) {
            const int b = lo + (int)__builtin_ctzll(um);
            um &= um - 1ull;
            const i64 r = row0 + b;
            const i64 dst = (i64)base + __popcll(uw & ((1ull << b) - 1ull));
            if (r >= a.V || dst >= g.out_cap[tb]) break;   // corrupt index or overflow (both flagged)
            const u32 pos = st + (u32)__popcll(mk & ((1ull << b) - 1ull));
            const bool ok = mine && ((mk >> b) & 1ull) && (pos < (u32)U);
            u64 S = __ballot(ok);
            float4 acc[ITERS];
            zero_row<ITERS>(acc);
            while (S) {
                float4 x[4][ITERS];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (S) {
                        const int k = (int)__builtin_ctzll(S);
                        S &= S - 1ull;
                        const float *src = (const float *)rd_lane64(rows_ptr, k) + (size_t)(u32)rd_lane((int)pos, k) * a.D;
                        load_row_s<float, ITERS>(x[j], src, C4, lane);   // read once: around the caches
                    } else {
                        zero_row<ITERS>(x[j]);
                    }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) add_row<ITERS>(acc, x[j]);
            }
            store_row_s<float, ITERS>(g.out_rows[tb] + (size_t)dst * a.D, acc, C4, lane);
            if (lane == 0) g.out_ids[tb][dst] = (int)r;
        }
    }
}

// index of the sources and place of every word in the output
void tn_launch_grad_sum_index(const GradSumArgs &g, hipStream_t st)
{
    const ApplyArgs &a = g.a;
    tn_launch_apply_clear(a, st);
    tn_launch_apply_index(a, 0, a.n_src, st);
    const int words = (int)((a.V + 63) >> 6);
    const int sblocks = (words + TN_UNION_WORDS - 1) / TN_UNION_WORDS;
    hipLaunchKernelGGL(k_union_count, dim3(sblocks, 2), dim3(BLOCK), 0, st, g);
    hipLaunchKernelGGL(k_union_offsets, dim3(sblocks, 2), dim3(BLOCK), 0, st, g);
}

void tn_launch_grad_sum_rows(const GradSumArgs &g, hipStream_t st)
{
    const ApplyArgs &a = g.a;
    const int words = (int)((a.V + 63) >> 6);
    const int iters = (a.D / 4 + WAVE - 1) / WAVE;
    const i64 nwaves = (i64)words * (64 / GRADSUM_G);
    const int nblocks = (int)((nwaves + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    dim3 grid(nblocks), blk(BLOCK);
    switch (iters) {
    case 1: hipLaunchKernelGGL((k_grad_sum<1, GRADSUM_G>), grid, blk, 0, st, g, nblocks); break;
    case 2: hipLaunchKernelGGL((k_grad_sum<2, GRADSUM_G>), grid, blk, 0, st, g, nblocks); break;
    case 3: hipLaunchKernelGGL((k_grad_sum<3, GRADSUM_G>), grid, blk, 0, st, g, nblocks); break;
    default: hipLaunchKernelGGL((k_grad_sum<4, GRADSUM_G>), grid, blk, 0, st, g, nblocks); break;
    }
}
