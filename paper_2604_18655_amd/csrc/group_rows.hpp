// Stable grouping of rows by adapter inside one workgroup, results in LDS.
#pragma once
#include "common.hpp"

namespace mlora {

struct GroupLds {
    int count[MLORA_MAX_ADAPTERS + 1];            // histogram, then running write offsets
    unsigned short perm[MLORA_MAX_ROWS];
    unsigned short seg_adapter[MLORA_MAX_ADAPTERS];
    unsigned short seg_start[MLORA_MAX_ADAPTERS + 1];
    int n_seg;
    int bad;                                      // an index was outside [-1, n_adapters)
};

// The same results for at most 64 rows (one wave's worth): at most 64 segments.
struct GroupLds64 {
    unsigned short perm[64];
    unsigned short seg_adapter[64];
    unsigned short seg_start[65];
    int n_seg;
    int bad;
};

// Rows without adapter (-1, or an out-of-range index) go to bucket n_adapters, which sorts last.
__device__ inline int bucket_of(int a, int n_adapters, bool &bad)
{
    bad = (a < -1) || (a >= n_adapters);
    return (a < 0 || a >= n_adapters) ? n_adapters : a;
}

// M <= 64: one wave, one row per lane, no LDS traffic until the results are written.  The
// position of a row in the sorted order is (#rows in a smaller bucket) + (#earlier rows in the
// same bucket); both sets are built as lane masks from one ballot per bit of the bucket id.
template <class G>
__device__ inline void group_rows_wave(const int *row_adapter, int M, int n_adapters, G &g)
{
    const int lane = threadIdx.x & 63;
    const unsigned long long below = (1ull << lane) - 1ull;
    const bool valid = lane < M;
    bool bad = false;
    int bucket = 0;
    if (valid) bucket = bucket_of(row_adapter[lane], n_adapters, bad);
    const unsigned long long vmask = __ballot(valid);
    unsigned long long eq = vmask, lt = 0;
    const int nbits = 32 - __clz(n_adapters);      // buckets 0..n_adapters
    for (int bit = nbits - 1; bit >= 0; --bit) {
        const bool set = (bucket >> bit) & 1;
        const unsigned long long bal = __ballot(valid && set);
        if (set) { lt |= eq & ~bal; eq &= bal; }
        else     { eq &= ~bal; }
    }
    const int rank = __popcll(eq & below);
    const int smaller = __popcll(lt);
    const bool has_adapter = valid && bucket < n_adapters;
    const bool first = has_adapter && rank == 0;
    const unsigned long long first_mask = __ballot(first);
    if (valid) g.perm[smaller + rank] = (unsigned short)lane;
    if (first) {
        const int idx = __popcll(first_mask & lt);
        g.seg_adapter[idx] = (unsigned short)bucket;
        g.seg_start[idx] = (unsigned short)smaller;
    }
    const int n_seg = __popcll(first_mask);
    const int with_adapter = __popcll(__ballot(has_adapter));
    const unsigned long long any_bad = __ballot(bad);
    if (lane == 0) {
        g.seg_start[n_seg] = (unsigned short)with_adapter;
        g.n_seg = n_seg;
        g.bad = any_bad != 0;
    }
}

// Any M: counting sort with the histogram in LDS; wave 0 scans it and scatters the rows in
// ascending order, 64 at a time.
__device__ inline void group_rows_counting(const int *row_adapter, int M, int n_adapters, GroupLds &g)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthreads = blockDim.x;
    for (int b = tid; b <= n_adapters; b += nthreads) g.count[b] = 0;
    if (tid == 0) g.bad = 0;
    __syncthreads();
    for (int m = tid; m < M; m += nthreads) {
        bool bad;
        const int b = bucket_of(row_adapter[m], n_adapters, bad);
        if (bad) g.bad = 1;
        atomicAdd(&g.count[b], 1);
    }
    __syncthreads();
    if (wave == 0) {
        volatile int *cnt = g.count;
        const unsigned long long below = (1ull << lane) - 1ull;
        // exclusive scan of the histogram, 64 buckets at a time; non-empty adapters become segments
        int carry = 0, nseg = 0;
        for (int base = 0; base <= n_adapters; base += 64) {
            const int b = base + lane;
            const int c = (b <= n_adapters) ? cnt[b] : 0;
            int incl = c;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int v = __shfl_up(incl, d);
                if (lane >= d) incl += v;
            }
            const int excl = incl - c + carry;
            const bool is_seg = (b < n_adapters) && (c > 0);
            const unsigned long long mask = __ballot(is_seg);
            if (b <= n_adapters) cnt[b] = excl;
            if (is_seg) {
                const int idx = nseg + __popcll(mask & below);
                g.seg_adapter[idx] = (unsigned short)b;
                g.seg_start[idx] = (unsigned short)excl;
            }
            carry += __shfl(incl, 63);
            nseg += __popcll(mask);
        }
        if (lane == 0) {
            g.seg_start[nseg] = (unsigned short)cnt[n_adapters];   // rows that carry an adapter
            g.n_seg = nseg;
        }
        // stable scatter: within a chunk each distinct bucket is served in turn and its rows
        // keep their lane order
        for (int base = 0; base < M; base += 64) {
            const int m = base + lane;
            const bool valid = m < M;
            int bucket = 0;
            if (valid) {
                bool bad;
                bucket = bucket_of(row_adapter[m], n_adapters, bad);
            }
            unsigned long long remaining = __ballot(valid);
            while (remaining) {
                const int leader = __ffsll((long long)remaining) - 1;
                const int bl = __builtin_amdgcn_readlane(bucket, leader);
                const bool mine = valid && bucket == bl;
                const unsigned long long same = __ballot(mine);
                const int off = cnt[bl];
                if (mine) g.perm[off + __popcll(same & below)] = (unsigned short)m;
                if (lane == leader) cnt[bl] = off + __popcll(same);
                remaining &= ~same;
            }
        }
    }
}

// Called by all threads of a block, M <= 64.  On return g holds the permutation and the segments.
__device__ inline void group_rows_lds64(const int *row_adapter, int M, int n_adapters, GroupLds64 &g)
{
    if ((threadIdx.x >> 6) == 0) group_rows_wave(row_adapter, M, n_adapters, g);
    __syncthreads();
}

// Called by all threads of a block.  On return g holds the permutation and the segments.
__device__ inline void group_rows_lds(const int *row_adapter, int M, int n_adapters, GroupLds &g)
{
    if (M <= 64) {
        if ((threadIdx.x >> 6) == 0) group_rows_wave(row_adapter, M, n_adapters, g);
    } else {
        group_rows_counting(row_adapter, M, n_adapters, g);
    }
    __syncthreads();
}

}  // namespace mlora
