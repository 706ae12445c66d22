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
#include <cstdlib>

#include "dev_common.h"
#include "kernels.h"

#define APPLY_CHUNK 16   // consecutive workgroups kept on one XCD

// ---------------------------------------------------------------- index
__global__ void __launch_bounds__(BLOCK) k_apply_clear(u64 *m0, u64 *m1, size_t n)
{
    size_t i = (size_t)blockIdx.x * BLOCK + threadIdx.x;
    if (i < n) {
        m0[i] = 0ull;
        m1[i] = 0ull;
    }
}

// grid: (blocks, n_src, 2 tables); every wave takes 64 consecutive ids of source k.
__global__ void __launch_bounds__(BLOCK) k_apply_index(ApplyArgs a)
{
    const int k = blockIdx.y, tb = blockIdx.z;
    const ApplySrc &s = a.src[tb][k];
    if (s.ids == nullptr) return;
    int U = *s.n_rows;
    if (U < 0) U = 0;
    if ((i64)U > s.capacity) {
        U = (int)s.capacity;
        if (threadIdx.x == 0 && blockIdx.x == 0) atomicOr(a.status, ST_OVERFLOW);
    }
    const int ns = a.n_src;
    u32 *start = a.start[tb];
    u64 *mask = a.mask[tb];
    const int lane = lane_id();
    const int V = (int)a.V;
    // wave-uniform trip count: every lane takes part in the shuffles
    for (int base = (blockIdx.x * WAVES_PER_BLOCK + uniform((int)(threadIdx.x >> 6))) * WAVE; base < U;
         base += gridDim.x * BLOCK) {
        const int i = base + lane;
        const bool valid = i < U;
        int id = valid ? s.ids[i] : 0;
        int prev = (valid && i > 0) ? s.ids[i - 1] : -1;
        int next = (i + 1 < U) ? s.ids[i + 1] : -1;
        if (valid) {
            if ((u32)id >= (u32)V) {
                atomicOr(a.status, ST_BAD_ID);
                id = V - 1;
            }
            if (id <= prev) atomicOr(a.status, ST_BAD_ORDER);
        }
        if ((u32)prev >= (u32)V) prev = (prev < 0) ? -64 : V - 1;
        if ((u32)next >= (u32)V) next = (next < 0) ? -64 : V - 1;
        const int w = valid ? (id >> 6) : -2 - lane;          // invalid lanes: unique keys
        const bool head = valid && ((prev >> 6) != w);        // first id of its word
        if (head) start[(size_t)w * ns + k] = (u32)i;
        // segmented inclusive OR over lanes with equal w (equal keys are contiguous)
        u64 m = valid ? (1ull << (id & 63)) : 0ull;
#pragma unroll
        for (int o = 1; o < WAVE; o <<= 1) {
            u64 m2 = (u64)__shfl_up((unsigned long long)m, o, WAVE);
            int w2 = __shfl_up(w, o, WAVE);
            if (lane >= o && w2 == w) m |= m2;
        }
        const int w_dn = __shfl_down(w, 1, WAVE);
        const bool tail = valid && (lane == WAVE - 1 || w_dn != w);   // last lane of its run
        const int w0 = __shfl(w, 0, WAVE);
        const int head0 = __shfl((int)head, 0, WAVE);
        if (tail) {
            const bool open_left = (w == w0) && !head0;               // run began in an earlier wave
            const bool open_right = (lane == WAVE - 1) && ((next >> 6) == w);
            if (open_left || open_right)
                atomicOr((unsigned long long *)&mask[(size_t)w * ns + k], (unsigned long long)m);
            else
                mask[(size_t)w * ns + k] = m;
        }
    }
}

// ---------------------------------------------------------------- apply
// G  rows per wave (16, 32 or 64); NT 1: streaming (non-temporal, global) loads and stores
template <typename T, int ITERS, int G, int NT>
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
                u64 mk = a.mask[tb][(size_t)word * ns + k];
                st = a.start[tb][(size_t)word * ns + k];
                const int lo = sub * G;
                st += (u32)__popcll(mk & ((1ull << lo) - 1ull));
                m = (G == 64) ? mk : ((mk >> lo) & ((1ull << (G & 63)) - 1ull));
                U = *s.n_rows;
                if ((i64)U > s.capacity) U = (int)s.capacity;
                rows_ptr = (u64)s.rows;
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
            u64 S = __ballot(ok);   // bit 32*tb + k: source k has row r
            T *wrow = table + (size_t)r * a.stride;
            float4 w[ITERS], acc[ITERS];
            if (NT == 2) zero_row<ITERS>(w);
            else if (NT == 1) load_row_s<T, ITERS>(w, wrow, C4, lane);
            else load_row<T, ITERS>(w, wrow, C4, lane);
            zero_row<ITERS>(acc);
            if (NT == 3) S = 0;
            while (S) {
                float4 x[4][ITERS];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (S) {
                        const int k = (int)__builtin_ctzll(S);   // ascending: own first, then peers
                        S &= S - 1ull;
                        const float *src = (const float *)rd_lane64(rows_ptr, k) +
                                           (size_t)(u32)rd_lane((int)pos, k) * a.D;
                        if (NT) load_row_s<float, ITERS>(x[j], src, C4, lane);
                        else load_row<float, ITERS>(x[j], src, C4, lane);
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
            if (NT == 2) { if (w[0].x == 1234.5678f) store_row<T, ITERS>(wrow, w, C4, lane); }
            else if (NT == 1) store_row_s<T, ITERS>(wrow, w, C4, lane);
            else store_row<T, ITERS>(wrow, w, C4, lane);
        }
    }
}

// Persistent form: a fixed number of resident waves stride over the groups of G rows, so that at
// any moment the rows in flight across the chip are neighbours in memory (a narrow front through
// the tables and through every gradient block, which is what keeps HBM pages open); the
// (start, mask) words of the next group are fetched while the current rows are processed.
template <typename T, int ITERS, int G>
__global__ void __launch_bounds__(BLOCK) k_apply_persist(ApplyArgs a, int ngroups)
{
    const int wave = uniform((int)(threadIdx.x >> 6)), lane = lane_id();
    const int nblocks = gridDim.x;
    const int nwaves = nblocks * WAVES_PER_BLOCK;
    // workgroups are dealt round-robin to the 8 XCDs: give every XCD a contiguous share of each
    // front, so rows that share a cache line meet in the same L2
    int gw;
    {
        const int b = blockIdx.x;
        const int per = nblocks >> 3;
        if ((nblocks & 7) == 0) gw = ((b & 7) * per + (b >> 3)) * WAVES_PER_BLOCK + wave;
        else gw = b * WAVES_PER_BLOCK + wave;
    }
    const int ns = a.n_src;
    const int C4 = a.D >> 2;
    const int tb_l = lane >> 5, k_l = lane & 31;
    bool have = false;
    int U = 0;
    u64 rows_ptr = 0;
    const u64 *mask_l = a.mask[tb_l];
    const u32 *start_l = a.start[tb_l];
    if (k_l < ns) {
        const ApplySrc &s = a.src[tb_l][k_l];
        if (s.ids != nullptr) {
            have = true;
            U = *s.n_rows;
            if ((i64)U > s.capacity) U = (int)s.capacity;
            rows_ptr = (u64)s.rows;
        }
    }
    const float neg_lr = -a.lr;
    constexpr int GPW = 64 / G;
    u64 mk_n = 0;
    u32 st_n = 0;
    if (have && gw < ngroups) {
        const size_t at = (size_t)(gw / GPW) * ns + k_l;
        mk_n = mask_l[at];
        st_n = start_l[at];
    }
    for (int g = gw; g < ngroups; g += nwaves) {
        const u64 mk = mk_n;
        u32 st = st_n;
        const int gn = g + nwaves;
        if (have && gn < ngroups) {
            const size_t at = (size_t)(gn / GPW) * ns + k_l;
            mk_n = mask_l[at];
            st_n = start_l[at];
        }
        const int word = g / GPW, lo = (g - word * GPW) * G;
        st += (u32)__popcll(mk & ((1ull << lo) - 1ull));
        const u64 m = (G == 64) ? mk : ((mk >> lo) & ((1ull << (G & 63)) - 1ull));
        const i64 row0 = (i64)word * 64 + lo;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            const bool mine = tb_l == tb;
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
                const u32 pos = st + (u32)__popcll(m & ((1ull << b) - 1ull));
                const bool ok = mine && ((m >> b) & 1ull) && (pos < (u32)U);
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
                            const int k = (int)__builtin_ctzll(S);   // ascending: own first, then peers
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
    }
}

template <typename T, int ITERS, int G>
static void launch_apply_persist_i(const ApplyArgs &a, hipStream_t st)
{
    static int blocks_per_cu = 0, cus = 0;
    if (blocks_per_cu == 0) {
        int dev = 0;
        (void)hipGetDevice(&dev);
        hipDeviceProp_t prop;
        (void)hipGetDeviceProperties(&prop, dev);
        cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_apply_persist<T, ITERS, G>, BLOCK, 0) != hipSuccess || occ < 1)
            occ = 4;
        blocks_per_cu = occ;
    }
    const int words = (int)((a.V + 63) >> 6);
    const i64 ngroups = (i64)words * (64 / G);
    int mult = 1;
    if (const char *e = getenv("TENSAIR_APPLY_OCC")) mult = atoi(e);
    i64 nblocks = (i64)cus * (mult > 0 ? (blocks_per_cu < mult ? blocks_per_cu : mult) : blocks_per_cu);
    const i64 need = (ngroups + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    if (nblocks > need) nblocks = need;
    hipLaunchKernelGGL((k_apply_persist<T, ITERS, G>), dim3((unsigned)nblocks), dim3(BLOCK), 0, st, a, (int)ngroups);
}

template <typename T, int G>
static void launch_apply_persist_t(const ApplyArgs &a, hipStream_t st)
{
    const int iters = (a.D / 4 + WAVE - 1) / WAVE;
    switch (iters) {
    case 1: launch_apply_persist_i<T, 1, G>(a, st); break;
    case 2: launch_apply_persist_i<T, 2, G>(a, st); break;
    case 3: launch_apply_persist_i<T, 3, G>(a, st); break;
    default: launch_apply_persist_i<T, 4, G>(a, st); break;
    }
}

template <typename T, int G, int NT>
static void launch_apply_t(const ApplyArgs &a, hipStream_t st)
{
    const int words = (int)((a.V + 63) >> 6);
    const i64 nwaves = (i64)words * (64 / G);
    const int nblocks = (int)((nwaves + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    const int iters = (a.D / 4 + WAVE - 1) / WAVE;
    dim3 grid(nblocks), blk(BLOCK);
    switch (iters) {
    case 1: hipLaunchKernelGGL((k_apply<T, 1, G, NT>), grid, blk, 0, st, a, nblocks); break;
    case 2: hipLaunchKernelGGL((k_apply<T, 2, G, NT>), grid, blk, 0, st, a, nblocks); break;
    case 3: hipLaunchKernelGGL((k_apply<T, 3, G, NT>), grid, blk, 0, st, a, nblocks); break;
    default: hipLaunchKernelGGL((k_apply<T, 4, G, NT>), grid, blk, 0, st, a, nblocks); break;
    }
}

void tn_launch_apply_index(const ApplyArgs &a, hipStream_t st)
{
    const size_t words = (size_t)((a.V + 63) >> 6);
    const size_t n = words * (size_t)a.n_src;
    hipLaunchKernelGGL(k_apply_clear, dim3((unsigned)((n + BLOCK - 1) / BLOCK)), dim3(BLOCK), 0, st,
                       a.mask[0], a.mask[1], n);
    // enough waves to cover the largest possible id list, grid-strided
    i64 maxcap = 1;
    for (int tb = 0; tb < 2; ++tb)
        for (int k = 0; k < a.n_src; ++k)
            if (a.src[tb][k].ids && a.src[tb][k].capacity > maxcap) maxcap = a.src[tb][k].capacity;
    i64 want = (maxcap + BLOCK - 1) / BLOCK;
    int blocks = (int)(want > 2048 ? 2048 : want);
    hipLaunchKernelGGL(k_apply_index, dim3(blocks, a.n_src, 2), dim3(BLOCK), 0, st, a);
}

void tn_launch_apply_update(const ApplyArgs &a, hipStream_t st)
{
    static int variant = -1;
    if (variant < 0) {
        const char *e = getenv("TENSAIR_APPLY_VARIANT");
        variant = e ? atoi(e) : 0;
    }
    const int g = variant / 10, nt = variant % 10;
    if (a.dtype == 0) {
        if (g == 0 && nt == 2) launch_apply_t<float, 16, 2>(a, st);
        else if (g == 0 && nt == 3) launch_apply_t<float, 16, 3>(a, st);
        else if (g == 0 && nt == 0) launch_apply_t<float, 16, 0>(a, st);
        else if (g == 0) launch_apply_t<float, 16, 1>(a, st);
        else if (g == 1 && nt == 0) launch_apply_t<float, 32, 0>(a, st);
        else if (g == 1) launch_apply_t<float, 32, 1>(a, st);
        else if (g == 2 && nt == 0) launch_apply_t<float, 64, 0>(a, st);
        else if (g == 2) launch_apply_t<float, 64, 1>(a, st);
        else if (g == 3) launch_apply_t<float, 8, 0>(a, st);
        else if (g == 4) launch_apply_t<float, 4, 0>(a, st);
        else if (g == 5) launch_apply_t<float, 2, 0>(a, st);
        else if (g == 6) launch_apply_t<float, 1, 0>(a, st);
        else if (g == 7) launch_apply_persist_t<float, 1>(a, st);
        else if (g == 8) launch_apply_persist_t<float, 2>(a, st);
        else if (g == 9) launch_apply_persist_t<float, 4>(a, st);
        else launch_apply_persist_t<float, 8>(a, st);
    } else {
        launch_apply_t<bf16_t, 16, 0>(a, st);
    }
}
