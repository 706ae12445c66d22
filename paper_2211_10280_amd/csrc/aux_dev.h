// Small integer jobs of a worker step -- clearing and building the per-word index of the table update,
// handing a prepared mini-batch's row index to the caller's buffers -- as device functions, so that they
// can run either as kernels of their own or as extra workgroups at the front of the grid of a kernel that
// is launched at that point of the step anyway (the forward pass, the segmented reduction): there they
// cost neither a launch nor a stream of their own nor the events that tie streams together.
#pragma once
#include "dev_common.h"
#include "kernels.h"

#ifndef AUX_INDEX_UNROLL
#define AUX_INDEX_UNROLL 4
#endif

// masks of both tables to zero; `block` of ceil(n / BLOCK) workgroups
__device__ __forceinline__ void aux_clear_masks(u64 *m0, u64 *m1, size_t n, int block)
{
    const size_t i = (size_t)block * BLOCK + threadIdx.x;
    if (i < n) {
        m0[i] = 0ull;
        m1[i] = 0ull;
    }
}

// Index of source k of table tb: each source's id list is strictly ascending, so for every 64-row word of
// the vocabulary the source's rows in that word are a contiguous run [start, start + popcount(mask)).
// Both arrays are laid out source by source ([k][word], see idx_at), so that a list's entries, which
// ascend with its ids, land next to each other.  The list is cut into runs of 64 consecutive ids, one per
// wave and trip; a word whose ids straddle two runs belongs to the run that holds its first id, which looks
// at the next run's ids for the rest of it (a word has at most 64 ids), while the next run leaves the ids
// of that word alone.  Every (word, source) entry is therefore written once, with plain stores: the masks
// only have to be zero beforehand for the words in which the source has no id.  `nblocks` workgroups
// stride over the list; a wave issues the loads of AUX_INDEX_UNROLL runs before it looks at any of them
// (the work per id is a few instructions, what counts is the number of round trips to memory).
__device__ __forceinline__ void aux_index_source(const ApplyArgs &a, int k, int tb, int block, int nblocks)
{
    const ApplySrc &s = a.src[tb][k];
    if (s.ids == nullptr) return;
    int U = *s.n_rows;
    if (U < 0) U = 0;
    if ((i64)U > s.capacity) {
        U = (int)s.capacity;
        if (threadIdx.x == 0 && block == 0) atomicOr(a.status, ST_OVERFLOW);
    }
    U = uniform(U);   // the same in every lane; said so, the loops below are scalar control flow
    const i64 words = (a.V + 63) >> 6;
    u32 *start = a.start[tb];
    u64 *mask = a.mask[tb];
    const int lane = lane_id();
    const int V = (int)a.V;
    // the trip count is wave-uniform: every lane takes part in the shuffles
    for (int base = (block * WAVES_PER_BLOCK + uniform((int)(threadIdx.x >> 6))) * (WAVE * AUX_INDEX_UNROLL); base < U;
         base += nblocks * (BLOCK * AUX_INDEX_UNROLL)) {
        int id_j[AUX_INDEX_UNROLL], prev_j[AUX_INDEX_UNROLL], ext_j[AUX_INDEX_UNROLL];
#pragma unroll
        for (int j = 0; j < AUX_INDEX_UNROLL; ++j) {
            const int i = base + j * WAVE + lane;
            id_j[j] = (i < U) ? s.ids[i] : 0;
            prev_j[j] = (i < U && i > 0) ? s.ids[i - 1] : -1;
            ext_j[j] = (i + WAVE < U) ? s.ids[i + WAVE] : -1;      // the same lane of the next run
        }
#pragma unroll
        for (int j = 0; j < AUX_INDEX_UNROLL; ++j) {
            const int run0 = base + j * WAVE;                       // wave-uniform
            if (run0 >= U) break;
            const int i = run0 + lane;
            const bool valid = i < U;
            int id = id_j[j], prev = prev_j[j], ext = ext_j[j];
            if (valid) {
                if ((u32)id >= (u32)V) {
                    atomicOr(a.status, ST_BAD_ID);
                    id = V - 1;
                }
                if (id <= prev) atomicOr(a.status, ST_BAD_ORDER);
            }
            if ((u32)prev >= (u32)V) prev = (prev < 0) ? -64 : V - 1;
            const bool ext_valid = (i + WAVE < U);
            if (ext_valid && (u32)ext >= (u32)V) ext = V - 1;       // as its own run will see it
            const int w = valid ? (id >> 6) : -2 - lane;            // invalid lanes: unique keys
            const bool head = valid && ((prev >> 6) != w);          // first id of its word
            if (head) start[idx_at(words, k, w)] = (u32)i;
            // ids at the front of the run that continue the previous run's last word belong to that run
            const int w_before = __shfl(prev >> 6, 0, WAVE);        // word of the id just before the run (-1: none)
            const bool foreign = valid && (w == w_before);
            // segmented inclusive OR over lanes with equal w (equal keys are contiguous)
            u64 m = valid ? (1ull << (id & 63)) : 0ull;
#pragma unroll
            for (int o = 1; o < WAVE; o <<= 1) {
                u64 m2 = (u64)__shfl_up((unsigned long long)m, o, WAVE);
                int w2 = __shfl_up(w, o, WAVE);
                if (lane >= o && w2 == w) m |= m2;
            }
            // the rest of the run's last word, from the next run
            const int w_last = __shfl(w, WAVE - 1, WAVE);           // < 0 if the run is not full
            const bool more = ext_valid && w_last >= 0 && (ext >> 6) == w_last;
            const u64 bit = more ? (1ull << (ext & 63)) : 0ull;
            const u64 m_ext = ((u64)wave_or((u32)(bit >> 32)) << 32) | (u64)wave_or((u32)bit);
            const int w_dn = __shfl_down(w, 1, WAVE);
            const bool tail = valid && (lane == WAVE - 1 || w_dn != w);   // last lane of its word within the run
            if (tail && !foreign) mask[idx_at(words, k, w)] = (lane == WAVE - 1) ? (m | m_ext) : m;
        }
    }
}

// row ids / row count / segment offsets of one table of a prepared mini-batch -> the consuming call's buffers
__device__ __forceinline__ void aux_copy_row_index(const RowIndexCopy::Side &s, int block, int nblocks)
{
    const int U = *s.src_n;
    if (block == 0 && threadIdx.x == 0) *s.dst_n = U;
    for (int i = block * BLOCK + threadIdx.x; i <= U; i += nblocks * BLOCK) {
        if (i < U) s.dst_ids[i] = s.src_ids[i];
        if (s.dst_off) s.dst_off[i] = s.src_off[i];
    }
}

// The jobs that ride at the front of a launch (see AuxWork): workgroup b of x.total.
__device__ __forceinline__ void aux_block(const AuxWork &x, int b)
{
    if (b < x.clear_blocks) {
        aux_clear_masks(x.clear_mask[0], x.clear_mask[1], x.clear_n, b);
        return;
    }
    b -= x.clear_blocks;
    if (b < 2 * x.copy_blocks) {
        const int side = b / x.copy_blocks;
        aux_copy_row_index(x.copy.side[side], b - side * x.copy_blocks, x.copy_blocks);
        return;
    }
    b -= 2 * x.copy_blocks;
    // index: jobs (source, table), index_blocks workgroups each
    const int job = b / x.index_blocks, blk = b - job * x.index_blocks;
    const int nk = x.k_end - x.k_begin;
    const int tb = job / nk, k = x.k_begin + (job - tb * nk);
    aux_index_source(x.apply, k, tb, blk, x.index_blocks);
}
