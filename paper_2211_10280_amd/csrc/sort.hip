// Stable LSD radix sort of (row id, entry) pairs and the derivation of unique row ids
// and segments from the sorted list.
//
// The sparse gradient of a mini-batch touches only a small part of the model (TensAIR,
// arXiv 2211.10280, Section 4 "Sparse vs. Dense Models"); rows touched more than once
// (frequent words) must be summed.  Sorting the occurrences by row id turns every row
// into one contiguous segment, so the later reduction and the table update are free of
// write conflicts and need no floating-point atomics; stability fixes the order of
// the additions inside a segment.  All of this is integer work and bit-exact.
#include "aux_dev.h"
#include "dev_common.h"
#include "kernels.h"

#define RADIX_MAX_BITS TN_RADIX_MAX_BITS
#define RADIX_MAX_ND (1 << RADIX_MAX_BITS)
#define RADIX_IPT (TN_RADIX_TILE / BLOCK)   // keys per thread

struct RadixPass {
    const u32 *kin[2];
    u32 *kout[2];
    const u32 *vin[2];
    u32 *vout[2];
    int n[2];
    int nblk[2];
    u32 *counts[2];
    u32 *totals[2];
    int shift, bits, first;
};

// per-block digit histogram: counts[d][b]
// Dynamic LDS of the radix kernels: as many counters as the pass has digits.  The launcher may ask for more than
// that to hold the kernels' occupancy down next to a kernel that should not be disturbed.
extern __shared__ u32 radix_lds[];

__global__ void __launch_bounds__(BLOCK) k_radix_hist(RadixPass a)
{
    u32 *h = radix_lds;                                  // [nd]
    int b = blockIdx.x, pr = 0;
    if (b >= a.nblk[0]) { b -= a.nblk[0]; pr = 1; }
    const int nd = 1 << a.bits;
    const u32 dmask = (u32)nd - 1u;
    for (int d = threadIdx.x; d < nd; d += BLOCK) h[d] = 0;
    __syncthreads();
    const u32 *kin = a.kin[pr];
    const int n = a.n[pr];
    const int base = b * TN_RADIX_TILE;
#pragma unroll
    for (int j = 0; j < RADIX_IPT; ++j) {
        int idx = base + j * BLOCK + threadIdx.x;
        if (idx < n) atomicAdd(&h[(kin[idx] >> a.shift) & dmask], 1u);
    }
    __syncthreads();
    u32 *counts = a.counts[pr];
    const int nblk = a.nblk[pr];
    for (int d = threadIdx.x; d < nd; d += BLOCK) counts[(size_t)d * nblk + b] = h[d];
}

// one wave per digit: exclusive scan of that digit's counts over the blocks, plus the total
__global__ void __launch_bounds__(BLOCK) k_radix_rowscan(RadixPass a)
{
    const int pr = blockIdx.y;
    const int nd = 1 << a.bits;
    const int d = blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    const int lane = lane_id();
    if (d >= nd) return;
    const int nblk = a.nblk[pr];
    u32 *row = a.counts[pr] + (size_t)d * nblk;
    u32 carry = 0;
    for (int base = 0; base < nblk; base += WAVE) {
        int i = base + lane;
        u32 x = (i < nblk) ? row[i] : 0u;
        u32 incl = wave_incl_scan(x, lane);
        if (i < nblk) row[i] = carry + incl - x;
        carry += (u32)__shfl((int)incl, WAVE - 1, WAVE);
    }
    if (lane == 0) a.totals[pr][d] = carry;
}

// rank every key inside its block (stable), add the global base of its digit, scatter
__global__ void __launch_bounds__(BLOCK) k_radix_scatter(RadixPass a)
{
    __shared__ u32 wsum[WAVES_PER_BLOCK];
    int b = blockIdx.x, pr = 0;
    if (b >= a.nblk[0]) { b -= a.nblk[0]; pr = 1; }
    const int nd = 1 << a.bits;
    u32 *dbase = radix_lds;                              // [nd] global exclusive base of every digit
    u32 *whp = radix_lds + nd;                           // [WAVES_PER_BLOCK][nd] per-wave digit counters -> bases
    const u32 dmask = (u32)nd - 1u;
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const int n = a.n[pr], nblk = a.nblk[pr];

    for (int d = threadIdx.x; d < nd; d += BLOCK) {
#pragma unroll
        for (int w = 0; w < WAVES_PER_BLOCK; ++w) whp[w * nd + d] = 0;
    }
    // exclusive scan of the digit totals (nd <= 2048 = 256 threads x 8)
    {
        const int per = (nd + BLOCK - 1) / BLOCK;   // 1..8
        const u32 *tot = a.totals[pr];
        u32 loc[8];
        u32 s = 0;
        for (int j = 0; j < per; ++j) {
            int d = threadIdx.x * per + j;
            loc[j] = (d < nd) ? tot[d] : 0u;
            s += loc[j];
        }
        u32 incl = wave_incl_scan(s, lane);
        if (lane == WAVE - 1) wsum[wave] = incl;
        __syncthreads();
        u32 off = 0;
        for (int w = 0; w < wave; ++w) off += wsum[w];
        u32 run = off + incl - s;
        for (int j = 0; j < per; ++j) {
            int d = threadIdx.x * per + j;
            if (d < nd) dbase[d] = run;
            run += loc[j];
        }
    }
    __syncthreads();

    // wave `wave` owns the contiguous keys [wbase, wbase + IPT*64) of the block's tile
    const u32 *kin = a.kin[pr];
    const int wbase = b * TN_RADIX_TILE + wave * (RADIX_IPT * WAVE);
    u32 key[RADIX_IPT];
    u32 loc[RADIX_IPT];
    const u64 lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int it = 0; it < RADIX_IPT; ++it) {
        int idx = wbase + it * WAVE + lane;
        bool valid = idx < n;
        key[it] = valid ? kin[idx] : 0u;
        u32 d = (key[it] >> a.shift) & dmask;
        u64 m = __ballot(valid);
        for (int bit = 0; bit < a.bits; ++bit) {
            bool on = (d >> bit) & 1u;
            u64 bal = __ballot(valid && on);
            m &= on ? bal : ~bal;
        }
        u32 rank = (u32)__popcll(m & lt);
        u32 cnt = (u32)__popcll(m);
        u32 old = 0;
        if (valid) old = whp[wave * nd + d];
        if (valid && rank == 0) whp[wave * nd + d] = old + cnt;
        loc[it] = old + rank;
    }
    __syncthreads();
    // turn the per-wave counters into bases: global digit base + this block's offset inside
    // the digit + the counts of the lower waves
    {
        const u32 *counts = a.counts[pr];
        for (int d = threadIdx.x; d < nd; d += BLOCK) {
            u32 run = dbase[d] + counts[(size_t)d * nblk + b];
#pragma unroll
            for (int w = 0; w < WAVES_PER_BLOCK; ++w) {
                u32 c = whp[w * nd + d];
                whp[w * nd + d] = run;
                run += c;
            }
        }
    }
    __syncthreads();
    u32 *kout = a.kout[pr];
    u32 *vout = a.vout[pr];
    const u32 *vin = a.vin[pr];
#pragma unroll
    for (int it = 0; it < RADIX_IPT; ++it) {
        int idx = wbase + it * WAVE + lane;
        if (idx < n) {
            u32 d = (key[it] >> a.shift) & dmask;
            u32 pos = whp[wave * nd + d] + loc[it];
            kout[pos] = key[it];
            vout[pos] = a.first ? (u32)idx : vin[idx];
        }
    }
}

int tn_launch_radix_sort(RadixProb p0, RadixProb p1, int key_bits, size_t min_lds_bytes, hipStream_t st, int *key_buf)
{
    int passes, bits;
    tn_radix_shape(key_bits, &passes, &bits);
    RadixProb p[2] = {p0, p1};
    int cur = 0;    // vals buffer holding the current order
    int kin = 0;    // keys buffer holding the current order
    for (int pass = 0; pass < passes; ++pass) {
        const int kout = (kin == 1) ? 2 : 1;
        RadixPass a;
        for (int i = 0; i < 2; ++i) {
            a.kin[i] = p[i].keys[kin];
            a.kout[i] = p[i].keys[kout];
            a.vin[i] = p[i].vals[cur];
            a.vout[i] = p[i].vals[cur ^ 1];
            a.n[i] = p[i].n;
            a.nblk[i] = p[i].nblk;
            a.counts[i] = p[i].counts;
            a.totals[i] = p[i].totals;
        }
        a.shift = pass * bits;
        a.bits = bits;
        a.first = (pass == 0);
        int nblk = a.nblk[0] + a.nblk[1];
        int nd = 1 << bits;
        size_t lds_hist = (size_t)nd * 4, lds_scatter = (size_t)nd * 4 * (1 + WAVES_PER_BLOCK);
        if (lds_hist < min_lds_bytes) lds_hist = min_lds_bytes;
        if (lds_scatter < min_lds_bytes) lds_scatter = min_lds_bytes;
        hipLaunchKernelGGL(k_radix_hist, dim3(nblk), dim3(BLOCK), lds_hist, st, a);
        hipLaunchKernelGGL(k_radix_rowscan, dim3((nd + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK, 2),
                           dim3(BLOCK), 0, st, a);
        hipLaunchKernelGGL(k_radix_scatter, dim3(nblk), dim3(BLOCK), lds_scatter, st, a);
        cur ^= 1;
        kin = kout;
    }
    *key_buf = kin;
    return cur;
}

// ---------------------------------------------------------------- segments
#define SCAN_IPT (TN_SCAN_TILE / BLOCK)

struct SegPass {
    SegProb p[2];
    i64 begin, T;
    int w;
    int *status;
};

__device__ __forceinline__ int entry_weight(const SegProb &p, const SegPass &a, int i)
{
    if (!p.weighted) return 1;
    i64 pos = a.begin + (i64)p.vals[i];
    i64 left = pos < a.w ? pos : a.w;
    i64 right = (a.T - 1 - pos) < a.w ? (a.T - 1 - pos) : a.w;
    return (int)(left + right);
}

// block-wide exclusive scan of a pair of ints (one pair per thread); tot = block totals
__device__ __forceinline__ void block_scan2(int a, int b, int &ea, int &eb, int &ta, int &tb,
                                            int (*sm)[WAVES_PER_BLOCK])
{
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    int ia = (int)wave_incl_scan((u32)a, lane);
    int ib = (int)wave_incl_scan((u32)b, lane);
    if (lane == WAVE - 1) { sm[0][wave] = ia; sm[1][wave] = ib; }
    __syncthreads();
    int oa = 0, ob = 0;
    ta = 0; tb = 0;
#pragma unroll
    for (int w = 0; w < WAVES_PER_BLOCK; ++w) {
        if (w < wave) { oa += sm[0][w]; ob += sm[1][w]; }
        ta += sm[0][w]; tb += sm[1][w];
    }
    ea = oa + ia - a;
    eb = ob + ib - b;
    __syncthreads();
}

__global__ void __launch_bounds__(BLOCK) k_head_count(SegPass a)
{
    __shared__ int sm[2][WAVES_PER_BLOCK];
    int b = blockIdx.x, pr = 0;
    if (b >= a.p[0].nblk) { b -= a.p[0].nblk; pr = 1; }
    const SegProb &p = a.p[pr];
    int heads = 0, weight = 0;
    const int base = b * TN_SCAN_TILE + threadIdx.x * SCAN_IPT;
    u32 prev = (base > 0 && base <= p.n) ? p.keys[base - 1] : 0u;
#pragma unroll
    for (int j = 0; j < SCAN_IPT; ++j) {
        int i = base + j;
        if (i < p.n) {
            u32 k = p.keys[i];
            heads += (i == 0 || k != prev) ? 1 : 0;
            weight += entry_weight(p, a, i);
            prev = k;
        }
    }
    int ea, eb, ta, tb;
    block_scan2(heads, weight, ea, eb, ta, tb, sm);
    if (threadIdx.x == 0) { p.blk_heads[b] = ta; p.blk_weight[b] = tb; }
}

__global__ void __launch_bounds__(BLOCK) k_seg_assign(SegPass a)
{
    __shared__ int sm[2][WAVES_PER_BLOCK];
    int b = blockIdx.x, pr = 0;
    if (b >= a.p[0].nblk) { b -= a.p[0].nblk; pr = 1; }
    const SegProb &p = a.p[pr];
    if (b == 0 && threadIdx.x == 0) *p.long_cnt = 0;
    // heads / weight of all earlier blocks
    int ph = 0, pw = 0;
    for (int j = threadIdx.x; j < b; j += BLOCK) { ph += p.blk_heads[j]; pw += p.blk_weight[j]; }
    int e0, e1, pre_h, pre_w;
    block_scan2(ph, pw, e0, e1, pre_h, pre_w, sm);

    const int base = b * TN_SCAN_TILE + threadIdx.x * SCAN_IPT;
    u32 key[SCAN_IPT];
    int hd[SCAN_IPT], wt[SCAN_IPT];
    int heads = 0, weight = 0;
    u32 prev = (base > 0 && base <= p.n) ? p.keys[base - 1] : 0u;
#pragma unroll
    for (int j = 0; j < SCAN_IPT; ++j) {
        int i = base + j;
        hd[j] = 0; wt[j] = 0; key[j] = 0;
        if (i < p.n) {
            key[j] = p.keys[i];
            hd[j] = (i == 0 || key[j] != prev) ? 1 : 0;
            wt[j] = entry_weight(p, a, i);
            prev = key[j];
            heads += hd[j];
            weight += wt[j];
        }
    }
    int eh, ew, th, tw;
    block_scan2(heads, weight, eh, ew, th, tw, sm);
    int run_h = pre_h + eh, run_w = pre_w + ew;
#pragma unroll
    for (int j = 0; j < SCAN_IPT; ++j) {
        int i = base + j;
        if (i < p.n) {
            run_h += hd[j];
            int seg = run_h - 1;
            p.seg_of[i] = seg;
            if (hd[j]) p.seg_start[seg] = i;
            if (hd[j]) {
                if ((i64)seg < p.capacity) {
                    p.row_ids[seg] = (int)key[j];
                    if (p.seg_offsets) p.seg_offsets[seg] = run_w;
                } else {
                    atomicOr(a.status, ST_OVERFLOW);
                }
            }
            run_w += wt[j];
            if (i == p.n - 1) {
                p.seg_start[seg + 1] = p.n;
                int U = seg + 1;
                if ((i64)U > p.capacity) U = (int)p.capacity;
                *p.n_rows = U;
                if (p.seg_offsets && (i64)(seg + 1) <= p.capacity) p.seg_offsets[seg + 1] = run_w;
            }
        }
    }
}

void tn_launch_segments(SegProb p0, SegProb p1, i64 begin, i64 T, int w, int *status, hipStream_t st)
{
    SegPass a;
    a.p[0] = p0;
    a.p[1] = p1;
    a.begin = begin;
    a.T = T;
    a.w = w;
    a.status = status;
    int nblk = p0.nblk + p1.nblk;
    hipLaunchKernelGGL(k_head_count, dim3(nblk), dim3(BLOCK), 0, st, a);
    hipLaunchKernelGGL(k_seg_assign, dim3(nblk), dim3(BLOCK), 0, st, a);
}

// ---------------------------------------------------------------- hand-over of prepared row ids
// Row ids, row count and segment offsets of a mini-batch whose sort ran ahead of time sit in the
// workspace; this copies them into the buffers of the call that consumes them.
__global__ void __launch_bounds__(BLOCK) k_copy_row_index(RowIndexCopy c)
{
    aux_copy_row_index(c.side[blockIdx.y], (int)blockIdx.x, (int)gridDim.x);
}

void tn_launch_copy_row_index(const RowIndexCopy &c, i64 max_rows, hipStream_t st)
{
    i64 want = (max_rows + 1 + BLOCK - 1) / BLOCK;
    int blocks = (int)(want > 1024 ? 1024 : want);
    hipLaunchKernelGGL(k_copy_row_index, dim3(blocks, 2), dim3(BLOCK), 0, st, c);
}
