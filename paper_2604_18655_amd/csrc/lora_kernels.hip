// Row grouping (stable counting sort by adapter, staged in LDS) and the LoRA shrink step
// t[m] = A[a(m)] . x[m], done per adapter segment so that each A[a] is streamed once.
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

// Rows without adapter (-1, or an out-of-range index) go to bucket n_adapters, which sorts last.
__device__ inline int bucket_of(int a, int n_adapters, bool &bad)
{
    bad = (a < -1) || (a >= n_adapters);
    return (a < 0 || a >= n_adapters) ? n_adapters : a;
}

// Called by all 256 threads of a block.  On return g holds the permutation and the segments.
__device__ void group_rows_lds(const int *row_adapter, int M, int n_adapters, GroupLds &g)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int b = tid; b <= n_adapters; b += 256) g.count[b] = 0;
    if (tid == 0) g.bad = 0;
    __syncthreads();
    for (int m = tid; m < M; m += 256) {
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
        // stable scatter: rows in ascending order, 64 at a time; within a chunk each distinct
        // bucket is served in turn and its rows keep their lane order
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
                const int bl = __shfl(bucket, leader);
                const bool mine = valid && bucket == bl;
                const unsigned long long same = __ballot(mine);
                const int off = cnt[bl];
                if (mine) g.perm[off + __popcll(same & below)] = (unsigned short)m;
                if (lane == leader) cnt[bl] = off + __popcll(same);
                remaining &= ~same;
            }
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(256) void group_rows_kernel(const int *row_adapter, int M,
                                                        int n_adapters, int *perm,
                                                        int *seg_adapter, int *seg_start,
                                                        int *n_seg)
{
    __shared__ GroupLds g;
    group_rows_lds(row_adapter, M, n_adapters, g);
    const int tid = threadIdx.x;
    for (int m = tid; m < M; m += 256) perm[m] = g.perm[m];
    for (int s = tid; s < g.n_seg; s += 256) seg_adapter[s] = g.seg_adapter[s];
    for (int s = tid; s <= g.n_seg; s += 256) seg_start[s] = g.seg_start[s];
    if (tid == 0) *n_seg = g.bad ? -1 : g.n_seg;
}

// One block = one (projection, 16-row tile of a segment, block of 16 ranks, K chunk); its four
// waves split the chunk's k-steps, each accumulating a 16x16 tile with MFMA (A operand: the
// tile's rows of x, B operand: 16 rows of A[adapter]); the four partial tiles are added in
// LDS in a fixed order and written to t_part[chunk][row][rank].
__global__ __launch_bounds__(256) void group_shrink_kernel(const LayerArgs a)
{
    __shared__ GroupLds g;
    __shared__ float red[4][256];

    int pi = 0;
    for (int i = 1; i < a.n_proj; ++i)
        if ((int)blockIdx.x >= a.p[i].shrink_begin) pi = i;
    const ProjArgs &P = a.p[pi];
    const int local = (int)blockIdx.x - P.shrink_begin;
    const int jblocks = P.r16 / 16;
    const int kc = local % P.kch;
    const int jb = (local / P.kch) % jblocks;
    const int ti = local / (P.kch * jblocks);

    group_rows_lds(a.row_adapter, a.M, P.n_adapters, g);

    // locate row tile ti among the segments (16 rows per tile, tiles never straddle segments)
    int seg = -1, first = 0, tiles_before = 0;
    for (int s = 0; s < g.n_seg; ++s) {
        const int len = (int)g.seg_start[s + 1] - (int)g.seg_start[s];
        const int nt = (len + 15) / 16;
        if (ti < tiles_before + nt) {
            seg = s;
            first = (int)g.seg_start[s] + 16 * (ti - tiles_before);
            break;
        }
        tiles_before += nt;
    }
    if (seg < 0) return;                                   // uniform over the block
    const int adapter = g.seg_adapter[seg];
    const int rows_here = min(16, (int)g.seg_start[seg + 1] - first);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;

    // k-steps of this block, then of this wave (balanced splits)
    const int nks = P.K / KSTEP;
    const int q = nks / P.kch, r = nks % P.kch;
    const int blk_beg = kc * q + min(kc, r), blk_cnt = q + (kc < r ? 1 : 0);
    const int wq_ = blk_cnt / 4, wr = blk_cnt % 4;
    const int my_beg = blk_beg + wave * wq_ + min(wave, wr), my_cnt = wq_ + (wave < wr ? 1 : 0);

    const int row = (l16 < rows_here) ? (int)g.perm[first + l16] : -1;
    const int j = jb * 16 + l16;
    const bool j_ok = j < P.rank;
    const uint16_t *xp = P.x + (size_t)(row < 0 ? 0 : row) * P.K + 8 * lq + (size_t)my_beg * KSTEP;
    const uint16_t *ap = P.lora_a + ((size_t)adapter * P.rank + (j_ok ? j : 0)) * P.K + 8 * lq +
                         (size_t)my_beg * KSTEP;
    const uint4 zero = make_uint4(0, 0, 0, 0);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    int s = 0;
    for (; s + 4 <= my_cnt; s += 4) {
        uint4 xa[4], ab[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            xa[u] = row >= 0 ? *reinterpret_cast<const uint4 *>(xp + (size_t)(s + u) * KSTEP) : zero;
            ab[u] = j_ok ? *reinterpret_cast<const uint4 *>(ap + (size_t)(s + u) * KSTEP) : zero;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = mfma16(xa[u], ab[u], acc);
    }
    for (; s < my_cnt; ++s) {
        const uint4 xa = row >= 0 ? *reinterpret_cast<const uint4 *>(xp + (size_t)s * KSTEP) : zero;
        const uint4 ab = j_ok ? *reinterpret_cast<const uint4 *>(ap + (size_t)s * KSTEP) : zero;
        acc = mfma16(xa, ab, acc);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) red[wave][e * 64 + lane] = acc[e];
    __syncthreads();
    {
        // thread (e, lane) owns tile row 4*(lane/16) + e and rank column lane%16
        const int e = wave;
        const int i = 4 * lq + e;
        const float v = ((red[0][e * 64 + lane] + red[1][e * 64 + lane]) + red[2][e * 64 + lane]) +
                        red[3][e * 64 + lane];
        if (i < rows_here) {
            const int m = g.perm[first + i];
            P.t_part[((size_t)kc * a.M + m) * P.r16 + jb * 16 + l16] = v;
        }
    }
}

hipError_t launch_group_rows(const int *row_adapter, int M, int n_adapters, int *perm,
                             int *seg_adapter, int *seg_start, int *n_seg, hipStream_t s)
{
    group_rows_kernel<<<dim3(1), dim3(256), 0, s>>>(row_adapter, M, n_adapters, perm, seg_adapter,
                                                    seg_start, n_seg);
    return hipGetLastError();
}

hipError_t launch_shrink(const LayerArgs &a, int n_blocks, hipStream_t s)
{
    group_shrink_kernel<<<dim3((unsigned)n_blocks), dim3(256), 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace mlora
