// The layer step: one launch.
//
// Base product.  A block of four waves owns one K unit of one tile of 64 output columns for one
// chunk of rows (16, 32 or 64 of them: three kernels, below).  Packed codes come straight from
// HBM with one 128-bit load per lane and k-step, the rows of x and the fp16 scales from L2;
// every code dword becomes four bf16 pairs with 7 integer ops and feeds 16x16x32 bf16 MFMAs
// whose A operand is a block of rows of x.  Scales multiply fp32 results, so the codes enter
// the matrix unit exactly.  What several waves add up is added in a fixed order.
//
// Long projections are cut into several K units per tile: units 1.. leave fp32 partial tiles in
// the workspace; unit 0 (the finishing block) adds them in order, adds the LoRA term
// alpha * B[a(m)][n] . t[m] and stores y.
//
// Order inside the launch.  The grid holds the shrink blocks first, then the split-K blocks,
// then the finishing blocks.  A finishing block streams its weights without waiting for
// anything; only before its epilogue does it wait (bounded spin on counters in the workspace)
// until the shrink blocks of its projection and the split-K blocks of its tile have signalled
// completion.  Blocks are dispatched in index order, producers never wait, so every wait
// ends; if one nevertheless runs out, the block sets the workspace status word and goes on.
//
// LoRA shrink, t[m] = A[a(m)] . x[m] in K chunks, MFMA (A operand: rows of x, B operand: 16 rank
// rows of A[adapter]); the partial sums go to t_part[chunk][row][rank].  Up to 16 rows: a block
// per (row, 16 ranks, K chunk).  More rows: the rows of a chunk of 64 are grouped by adapter
// and cut into tiles of 16, and a block's waves each take whole tiles.
#include <type_traits>

#include "group_rows.hpp"

namespace mlora {

// ------------------------------------------------------------------------------------------
// completion counters
// ------------------------------------------------------------------------------------------
// Data one block hands to another inside a launch (split-K partial tiles, the shrink step's t)
// is written and read with agent-scope accesses: they go through to memory and are re-fetched
// from it, so no cache of a compute unit or of a die ever holds a stale copy of it, and no
// cache-wide write-back or invalidate (which every fence at that scope costs) is needed.
__device__ __forceinline__ void store_shared(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_shared(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The same for 16 bytes at a time (the wide kernel's partial tiles: 64 KiB per block and unit).
// There is no 128-bit atomic type, so these are the plain 128-bit instructions with the cache
// policy of the 32-bit ones above (sc1), written out.  The compiler does not know that the load
// is in flight: shared16_wait (vmcnt(0)) must stand between a batch of loads and the first use.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_shared16(float *p, f32x4_t v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ f32x4_t load_shared16(const float *p)
{
    f32x4_t v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=&v"(v) : "v"(p) : "memory");
    return v;
}
__device__ __forceinline__ void shared16_wait(f32x4_t (&v)[8])
{
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7])
                 :
                 : "memory");
}
__device__ __forceinline__ void shared16_wait(f32x4_t (&v)[16])
{
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]),
                   "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]), "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])
                 :
                 : "memory");
}
// 16-byte loads of such data that the compiler can see (and so schedule, and wait for, by
// itself): buffer loads with the same cache policy (sc1, bit 4 of the policy argument) through a
// descriptor over `bytes` bytes at `base` (raw buffer, no stride; accesses past the end return 0).
// `base` and `bytes` must be the same for every lane of a wave.
typedef unsigned int u32x4_v __attribute__((vector_size(16)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t shared_buffer(const float *base, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ f32x4_t load_shared16(__amdgpu_buffer_rsrc_t rsrc, int byte_offset)
{
    return __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_offset, 0, 16));
}

// The hardware keeps the order "data, then counter" on the producer's side (the wait for the
// stores' acknowledgements below) and "counter, then data" on the consumer's (a wave's loads are
// issued in program order, and these go through to memory).  The compiler must keep it too:
// relaxed accesses to different addresses may be reordered, so a compiler-only fence (no
// instruction, no cache action) stands between the data accesses and the counter access.
__device__ __forceinline__ void compiler_fence() { __atomic_signal_fence(__ATOMIC_SEQ_CST); }

// all threads of the block, after their store_shared calls: wait until the own stores have been
// acknowledged, meet, then count the block as done in `copies` counter lines
__device__ __forceinline__ void signal_done(unsigned *counter, int copies)
{
    compiler_fence();
    __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): every store of this wave has completed
    __syncthreads();
    if ((int)threadIdx.x < copies) atomicAdd(counter + threadIdx.x * CTR_STRIDE, 1u);
}

// Wait until *counter has reached expected, polling at most `limit` times; false if the wait ran
// out (limit 0: at once).  Reads of what the counter guards must come after this call: the
// fence keeps the compiler from moving them up.
__device__ __forceinline__ bool wait_count(unsigned *counter, unsigned expected, int limit)
{
    bool ok = false;
    for (int i = 0; i < limit; ++i) {
        if (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= expected) { ok = true; break; }
        __builtin_amdgcn_s_sleep(1);
    }
    compiler_fence();
    return ok;
}

// ------------------------------------------------------------------------------------------
// base product
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float half_bits_lo(uint32_t v) { return half_bits_to_float((uint16_t)(v & 0xFFFFu)); }
__device__ __forceinline__ float half_bits_hi(uint32_t v) { return half_bits_to_float((uint16_t)(v >> 16)); }

// 8 packed codes -> 8 bf16 values code + 24 (4 dwords)
__device__ __forceinline__ uint4 expand_codes(uint32_t w, uint32_t mask, uint32_t bias)
{
    uint4 o;
    o.x = (w & mask) | bias;
    o.y = (__builtin_amdgcn_alignbit(w, w, 4) & mask) | bias;
    o.z = (__builtin_amdgcn_alignbit(w, w, 8) & mask) | bias;
    o.w = (__builtin_amdgcn_alignbit(w, w, 12) & mask) | bias;
    return o;
}

// (a native vector type: copies of HIP's uint4 struct from global to LDS would be lowered to
// memcpy through a private array instead of going through registers)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------
// A wave works through its inputs in rounds of R k-steps.  All operands of a round (R KiB of
// packed codes, the rows of x, the scales) are staged in a wave-private LDS buffer, and the
// math of a round is a ROLLED loop over its scale groups that reads everything back from
// LDS.  The loop is the point of the design: code that runs once is fetched at about 10
// cycles per instruction (instruction-cache misses), a loop body only on its first pass.
//
// The loads run ahead of the math as a register pipeline: two register sets hold the codes
// and scales of the next two rounds (they come from HBM: far), one set the rows of x of the
// next round (from L2: near).  A set goes to LDS as soon as its turn comes and is requested
// again at once, so a wave has 2*R KiB of codes in flight while it computes.
// ------------------------------------------------------------------------------------------
template <int XR, int R>
struct RoundLds {
    static constexpr int W_BYTES = R * 1024;
    static constexpr int SEG = R * 64;                         // bytes of one row of x in a round
    static constexpr int XROW = SEG + 16;                      // +16: rows 4 banks apart
    static constexpr int X_BYTES = XR * XROW;
    static constexpr int SC_BYTES = 1024;                      // up to 8 groups x 128 bytes
    static constexpr int NXL = XR * SEG / 1024;                // wave-wide loads for the rows of x
    static constexpr int BYTES = W_BYTES + X_BYTES + SC_BYTES; // per wave
};

template <int R>
struct RoundW {
    u32x4 w[R];                                  // packed codes
    u32x4 sc;                                    // the round's scale groups (up to 8 x 128 bytes)
};

template <int XR, int R>
struct RoundX {
    u32x4 x[RoundLds<XR, R>::NXL];
};

// Request the codes and scales of one round: k-steps [ks, ks + R) of the tile.  A request past
// the wave's range (!in) becomes a read of the tile's first 16 bytes by every lane: all loads
// stay unconditional, so the waits the compiler derives stay exact.
template <int R>
__device__ __forceinline__ void round_issue_w(RoundW<R> &rw, const uint4 *codes_tile, const uint2 *scales_tile,
                                              int spg, int ks, bool in, int lane)
{
    const u32x4 *wp = reinterpret_cast<const u32x4 *>(codes_tile) + (in ? (size_t)ks * 64 + lane : 0);
#pragma unroll
    for (int i = 0; i < R; ++i) rw.w[i] = __builtin_nontemporal_load(wp + (in ? i * 64 : 0));   // (read once)
    // the round's groups are contiguous: 128 bytes each, lane l takes bytes 16*l.. (past the
    // round's last group the blob's slack keeps the read in bounds)
    // (R / spg groups of 128 bytes: the lanes beyond them re-read the first 16 bytes)
    const bool mine = lane < (R / spg) * 8;
    rw.sc = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(scales_tile) +
                                       (in ? (size_t)(ks / spg) * 8 + (mine ? lane : 0) : 0));
}

// Request the rows of x (clamped to the chunk's rows and to K) of one round.
template <int XR, int R>
__device__ __forceinline__ void round_issue_x(RoundX<XR, R> &rx, const uint16_t *x, int K, int m0, int rows_here,
                                              int ks, bool in, int lane)
{
    using L = RoundLds<XR, R>;
    // (one uniform base and a 32-bit offset per load: eight 64-bit addresses would cost registers)
    const unsigned char *xb = reinterpret_cast<const unsigned char *>(x + (size_t)m0 * K);
#pragma unroll
    for (int i = 0; i < L::NXL; ++i) {
        const int byte = i * 1024 + lane * 16;
        const int row = min(byte / L::SEG, rows_here - 1);
        const int k = min(ks * KSTEP + (byte % L::SEG) / 2, K - 8);
        const unsigned off = in ? ((unsigned)row * (unsigned)K + (unsigned)k) * 2u : 0u;
        rx.x[i] = *reinterpret_cast<const u32x4 *>(xb + off);
    }
}

template <int XR, int R>
__device__ __forceinline__ void round_to_lds(const RoundW<R> &rw, const RoundX<XR, R> &rx, unsigned char *buf, int lane)
{
    using L = RoundLds<XR, R>;
#pragma unroll
    for (int i = 0; i < R; ++i) *reinterpret_cast<u32x4 *>(buf + i * 1024 + lane * 16) = rw.w[i];
#pragma unroll
    for (int i = 0; i < L::NXL; ++i) {
        const int byte = i * 1024 + lane * 16;
        *reinterpret_cast<u32x4 *>(buf + L::W_BYTES + (byte / L::SEG) * L::XROW + byte % L::SEG) = rx.x[i];
    }
    *reinterpret_cast<u32x4 *>(buf + L::W_BYTES + L::X_BYTES + lane * 16) = rw.sc;
}

// Math of one round: n_steps (a multiple of 4) k-steps starting at the front of the buffer.
// One loop pass = one scale group = SPG k-steps.
template <int MB, int XR, int R, int SPG>
__device__ __forceinline__ void round_compute(f32x4 (&acc)[MB][4], const unsigned char *buf,
                                              int n_steps, int rows_here, uint32_t mask,
                                              uint32_t bias, int lane)
{
    using L = RoundLds<XR, R>;
    const int l16 = lane & 15, lq = lane >> 4;
    const uint4 neg24 = make_uint4(0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u);
    const unsigned char *wl = buf + lane * 16;
    const unsigned char *xl[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
        xl[mb] = buf + L::W_BYTES + min(mb * 16 + l16, rows_here - 1) * L::XROW + 16 * lq;
    const unsigned char *sl = buf + L::W_BYTES + L::X_BYTES + l16 * 8;
#pragma nounroll
    for (int g = 0; g < n_steps / SPG; ++g) {
        uint4 xf[MB][SPG], wf[SPG];
#pragma unroll
        for (int s = 0; s < SPG; ++s) {
            wf[s] = *reinterpret_cast<const uint4 *>(wl + (g * SPG + s) * 1024);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                xf[mb][s] = *reinterpret_cast<const uint4 *>(xl[mb] + (g * SPG + s) * 64);
        }
        const uint2 sv = *reinterpret_cast<const uint2 *>(sl + g * 128);
        // -24 * sum of x over the group's inputs: cancels the offset of the stored codes
        f32x4 corr[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            corr[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < SPG; ++s) corr[mb] = mfma16(xf[mb][s], neg24, corr[mb]);
        }
        f32x4 d[MB][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) d[mb][j] = corr[mb];
#pragma unroll
            for (int s = 0; s < SPG; ++s) {
                const uint32_t wj = j == 0 ? wf[s].x : j == 1 ? wf[s].y : j == 2 ? wf[s].z : wf[s].w;
                const uint4 wb = expand_codes(wj, mask, bias);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) d[mb][j] = mfma16(xf[mb][s], wb, d[mb][j]);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float sj = j == 0 ? half_bits_lo(sv.x) : j == 1 ? half_bits_hi(sv.x)
                           : j == 2 ? half_bits_lo(sv.y) : half_bits_hi(sv.y);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[mb][j][e] = fmaf(d[mb][j][e], sj, acc[mb][j][e]);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Decode shapes (at most 16 rows per chunk): a wave has at most 16 k-steps, so there is no
// steady state to speak of and the K loop is a register pipeline instead of rounds.  The rows
// of x for the wave's whole range go to a wave-private LDS buffer once; the packed codes stay
// in registers, four k-steps deep, and each k-step's register is refilled as soon as it has
// been consumed.  Little state per wave (4 KiB of codes in flight, under 128 registers) lets
// four blocks share a compute unit, so every block of a decoder layer is resident at once and
// the bytes in flight come from the number of waves rather than from the depth of each.
// ------------------------------------------------------------------------------------------
template <int XR>
struct StreamLds {
    static constexpr int XSTEPS = UNIT_SUPER_STEPS;            // k-steps per wave: (16 super-steps x 4) / 4 waves
    static constexpr int XROW = XSTEPS * 64 + 16;              // bytes of a row of x; +16: rows 4 banks apart
    static constexpr int BYTES = XR * XROW;                    // per wave
};

// Codes and scales of one super-step (four k-steps); a wave keeps two of them in flight.
struct StreamRegs {
    u32x4 w[4];
    uint2 sc[4];                                               // one per scale group of the super-step
};

// Request super-step `ss` of the wave (wp0/sp0 = the wave's first chunk / first group WITHOUT the
// lane's offset).  A request past the wave's range (ss >= n_ss) becomes one 16-byte read of the
// first chunk by all lanes: every load stays unconditional, so the waits the compiler derives
// stay exact, and the useless ones cost next to nothing.
__device__ __forceinline__ void stream_request(StreamRegs &r, const u32x4 *wp0, const uint2 *sp0, int ss, int n_ss,
                                               int gs, int lane)
{
    const bool in = ss < n_ss;
    const u32x4 *wn = wp0 + (in ? (size_t)ss * 256 + lane : 0);
    const uint2 *sn = sp0 + (in ? (size_t)ss * gs * 16 + (lane & 15) : 0);
#pragma unroll
    for (int u = 0; u < 4; ++u) r.w[u] = __builtin_nontemporal_load(wn + (in ? u * 64 : 0));
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        // (the scales' type is HIP's struct, which the builtin does not take: read as two words)
        const unsigned long long v = __builtin_nontemporal_load(
            reinterpret_cast<const unsigned long long *>(sn + (in ? min(g, gs - 1) * 16 : 0)));
        r.sc[g] = make_uint2((unsigned)v, (unsigned)(v >> 32));
    }
}

// The math of one super-step; xs = this lane's row of x in LDS at the super-step's first k-step.
template <int SPG>
__device__ __forceinline__ void stream_math(f32x4 (&acc)[4], const StreamRegs &r, const unsigned char *xs,
                                            uint32_t mask, uint32_t bias)
{
    constexpr int GS = 4 / SPG;                                // scale groups per super-step
    const uint4 neg24 = make_uint4(0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u);
#pragma unroll
    for (int g = 0; g < GS; ++g) {
        uint4 xa[SPG];
        f32x4 corr = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < SPG; ++t) {
            xa[t] = *reinterpret_cast<const uint4 *>(xs + (g * SPG + t) * 64);
            corr = mfma16(xa[t], neg24, corr);                 // -24 * sum of x: cancels the code offset
        }
        f32x4 d[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            d[j] = corr;
#pragma unroll
            for (int t = 0; t < SPG; ++t) {
                const u32x4 wv = r.w[g * SPG + t];
                const uint32_t wj = j == 0 ? wv.x : j == 1 ? wv.y : j == 2 ? wv.z : wv.w;
                d[j] = mfma16(xa[t], expand_codes(wj, mask, bias), d[j]);
            }
        }
        const uint2 sv = r.sc[g];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float sj = j == 0 ? half_bits_lo(sv.x) : j == 1 ? half_bits_hi(sv.x)
                           : j == 2 ? half_bits_lo(sv.y) : half_bits_hi(sv.y);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[j][e] = fmaf(d[j][e], sj, acc[j][e]);
        }
    }
}

// n_ss super-steps (at most 4), two per pass: set A holds the even ones, set B the odd ones, and
// each set is requested again (two super-steps ahead) as soon as it has been consumed.  xl = this
// lane's row of x in LDS (+ 16 * (lane/16)).  During the last pass the wave also reads the two
// completion counters its epilogue depends on (poll_s, poll_p; before that, and for a wave that
// depends on nothing, a dummy address): if they are complete by then, the epilogue need not wait
// for a poll of its own.
template <int SPG>
__device__ __forceinline__ void stream_loop(f32x4 (&acc)[4], StreamRegs &ra, StreamRegs &rb, const u32x4 *wp0,
                                            const uint2 *sp0, int n_ss, const unsigned char *xl, uint32_t mask,
                                            uint32_t bias, int lane, const unsigned *poll_s, const unsigned *poll_p,
                                            unsigned &seen_s, unsigned &seen_p)
{
    constexpr int GS = 4 / SPG;
    const unsigned *dummy = reinterpret_cast<const unsigned *>(wp0);
#pragma nounroll
    for (int ss = 0; ss < n_ss; ss += 2) {
        const bool last = ss + 2 >= n_ss;
        seen_s = __hip_atomic_load(last ? poll_s : dummy, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        seen_p = __hip_atomic_load(last ? poll_p : dummy, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        stream_math<SPG>(acc, ra, xl + ss * 256, mask, bias);
        stream_request(ra, wp0, sp0, ss + 2, n_ss, GS, lane);
        if (ss + 1 < n_ss) stream_math<SPG>(acc, rb, xl + (ss + 1) * 256, mask, bias);
        stream_request(rb, wp0, sp0, ss + 3, n_ss, GS, lane);
    }
}

// Loads the epilogue needs that do not depend on other blocks, requested ahead of their use (all
// unconditional; a thread with nothing to fetch re-reads a valid address).  The N outputs of a
// thread lie in one row, 16 columns apart, so their rows of B differ by a fixed stride.
template <int N, int MBR, int FR>
struct EpiPrefetch {
    static constexpr int H = FR / 16;        // entries of t per thread and row block
    const uint16_t *bad[MBR];                // B of each row's adapter (or a safe address)
    int brank[MBR];                          // rank (0 with the safe address: every offset is 0)
    int n0, nlast;                           // column of output 0; last valid column
    // entries of t this thread sums: row t_ml + 16 * i, rank indices t_jj + 16 * h
    const float *tp[MBR][H];                 // the entry in t_part[0] (or a safe address)
    size_t tstride[MBR][H];                  // distance between K chunks of t_part (0 with the safe address)
    int kch, t_ml, t_jj;
    bool t_mine[MBR][H];
    uint4 b[N > 0 ? N : 1][FR / 8];
    __device__ __forceinline__ void issue()
    {
        // (global, not generic, loads: a generic load also counts as an LDS access, and every
        // later wait for LDS would wait for these as well)
        using G = const __attribute__((address_space(1))) u32x4;
#pragma unroll
        for (int q = 0; q < N; ++q) {
            const int mb = q >> 2;
            // the address passes through an empty asm: without it the compiler hoists these loads
            // to the top of the kernel and then spills their results across the whole K loop
            if ((q & 3) == 0) asm volatile("" : "+v"(bad[mb]));
            const uint16_t *row = bad[mb] + (unsigned)(min(n0 + 16 * (q & 3), nlast) * brank[mb]);
#pragma unroll
            for (int c = 0; c < FR / 8; ++c)     // (pieces past the rank re-read the first one)
                b[q][c] = __builtin_bit_cast(uint4, *(G *)(row + (brank[mb] > 8 * c ? 8 * c : 0)));
        }
    }
};

// sum over the 16 lanes of a row of lanes (DPP rotations, fixed order); every lane gets the result
__device__ __forceinline__ float row_sum16(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xF, 0xF, false));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x124, 0xF, 0xF, false));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x122, 0xF, 0xF, false));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x121, 0xF, 0xF, false));
    return v;
}

// Outputs of a fused call: the four values a lane holds of one row, columns 16 * j + l16 of a
// tile (so (v[0], v[2]) and (v[1], v[3]) are the pairs 32 columns apart), go through the
// projection's EpiArgs and are stored one by one.  The 16 lanes that differ in l16 only hold the
// same row and reach these calls together (m does not depend on l16): they share the sums over a
// row.  What the output stage reads from memory is fetched by fused_fetch, which a caller may
// issue well before the values are there (the loads then overlap what else it waits for).
struct FusedOperands {
    float scale_or_sum;            // row_scale[m], or this lane's share of the sums of squares
    float cs[2], sn[2];            // rotary cosines and sines of the lane's two pairs
    float res[4];                  // residual of the lane's four (SwiGLU: two) outputs
};

__device__ __forceinline__ FusedOperands fused_fetch(const LayerArgs &a, const ProjArgs &P, int pi, int m, int tile, int l16)
{
    FusedOperands f;
    const EpiArgs &E = a.epi[pi];
    const int mm = min(m, a.M - 1);                        // (rows past the end fetch a valid row and store nothing)
    f.scale_or_sum = 1.0f;
    if (E.row_scale) f.scale_or_sum = E.row_scale[mm];
    if (E.sq_in) {
        float sum = 0.f;
        for (int p = l16; p < E.sq_parts; p += 16) sum += E.sq_in[(size_t)mm * E.sq_parts + p];
        f.scale_or_sum = sum;
    }
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
        f.cs[jj] = 1.0f;
        f.sn[jj] = 0.0f;
        if (E.pair_op == PAIR_ROPE) {
            f.cs[jj] = E.rope_cos[(size_t)mm * 32 + 16 * jj + l16];
            f.sn[jj] = E.rope_sin[(size_t)mm * 32 + 16 * jj + l16];
        }
    }
    const int n_out = E.pair_op == PAIR_SWIGLU ? P.N >> 1 : P.N;
    const int n0 = tile * (E.pair_op == PAIR_SWIGLU ? TILE_N / 2 : TILE_N) + l16;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f.res[j] = 0.0f;
        if (E.residual && (E.pair_op != PAIR_SWIGLU || j < 2))
            f.res[j] = bf16_bits_to_float(E.residual[(size_t)mm * n_out + min(n0 + 16 * j, n_out - 1)]);
    }
    return f;
}

__device__ __forceinline__ void fused_store(const LayerArgs &a, const ProjArgs &P, int pi, int m, int tile, int l16,
                                            const FusedOperands &f, float (&v)[4])
{
    if (m >= a.M) return;
    const EpiArgs &E = a.epi[pi];
    float rs = f.scale_or_sum;
    if (E.sq_in) rs = 1.0f / sqrtf(row_sum16(f.scale_or_sum) / (float)P.K + E.sq_eps);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] *= rs;
    const int N = P.N;
    float sq = 0.f;                                        // squares of what this lane stores
    auto put = [&](size_t at, float o) {
        if (a.y_fp32) {
            reinterpret_cast<float *>(P.y)[at] = o;
        } else {
            const uint16_t h = float_to_bf16_bits(o);
            reinterpret_cast<uint16_t *>(P.y)[at] = h;
            o = bf16_bits_to_float(h);
        }
        sq = fmaf(o, o, sq);
    };
    if (E.pair_op == PAIR_SWIGLU) {
        const int n_out = N >> 1;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int n = tile * (TILE_N / 2) + 16 * jj + l16;
            const float g = v[jj];
            if (n < n_out) put((size_t)m * n_out + n, g / (1.0f + expf(-g)) * v[jj + 2] + f.res[jj]);
        }
    } else {
        if (E.pair_op == PAIR_ROPE) {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const float x0 = v[jj], x1 = v[jj + 2];
                v[jj] = x0 * f.cs[jj] - x1 * f.sn[jj];
                v[jj + 2] = x1 * f.cs[jj] + x0 * f.sn[jj];
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = tile * TILE_N + 16 * j + l16;
            if (n < N) put((size_t)m * N + n, v[j] + f.res[j]);
        }
    }
    if (E.sq_out) {
        sq = row_sum16(sq);
        if (l16 == 0) E.sq_out[(size_t)m * tiles_n(N) + tile] = sq;
    }
}

__device__ __forceinline__ void store_fused(const LayerArgs &a, const ProjArgs &P, int pi, int m, int tile, int l16,
                                            float (&v)[4])
{
    const FusedOperands f = fused_fetch(a, P, pi, m, tile, l16);
    fused_store(a, P, pi, m, tile, l16, f, v);
}

// the epilogue prefetch covers ranks up to this: 16 in the kernels for up to 16 rows (their register
// budget), 32 where a chunk has 32 rows (the prefetch there starts once the K loop's registers are free)
template <int MB> constexpr int fast_rank() { return MB == 1 ? 16 : 32; }

// LDS of a base block: the per-wave staging buffers, the per-wave partial tiles (red) and
// alpha * t of the chunk's rows.  Decode shapes: a wave's partial tile lies over its OWN staging
// buffer and t has room of its own, so a wave that is done with its K loop need not wait for the
// others before it writes either.  Above 16 rows red and t lie over the staging buffers of all
// waves and the block meets first.
template <int MB, int XR, int WAVES, int R>
struct BaseLds {
    static constexpr bool PRIVATE = MB == 1;
    static constexpr int WAVE_STAGE = PRIVATE ? StreamLds<XR>::BYTES : RoundLds<XR, R>::BYTES;
    static constexpr int STAGE_BYTES = WAVES * WAVE_STAGE;
    static constexpr int RED_WAVE = MB * 1024 * 4;             // bytes of one wave's partial tile
    static constexpr int TS_STRIDE = MLORA_MAX_RANK + 4;
    static constexpr int TS_BYTES = (PRIVATE ? XR : 16 * MB) * TS_STRIDE * 4;
    static constexpr int T_AT = PRIVATE ? STAGE_BYTES : WAVES * RED_WAVE;
    static constexpr int BYTES = T_AT + TS_BYTES > STAGE_BYTES ? T_AT + TS_BYTES : STAGE_BYTES;
    static_assert(!PRIVATE || WAVE_STAGE >= RED_WAVE, "a wave's partial tile must fit its own staging buffer");
    unsigned char *base;
    __device__ unsigned char *stage(int wave) const { return base + wave * WAVE_STAGE; }
    __device__ float *red(int wave) const
    {
        return reinterpret_cast<float *>(base + wave * (PRIVATE ? WAVE_STAGE : RED_WAVE));
    }
    __device__ float *t_row(int ml) const { return reinterpret_cast<float *>(base + T_AT) + ml * TS_STRIDE; }
};

__device__ __forceinline__ float dot8(uint4 b8, const float *t, float l)
{
    l = fmaf(bf16_bits_to_float(b8.x & 0xFFFFu), t[0], l);
    l = fmaf(bf16_bits_to_float(b8.x >> 16), t[1], l);
    l = fmaf(bf16_bits_to_float(b8.y & 0xFFFFu), t[2], l);
    l = fmaf(bf16_bits_to_float(b8.y >> 16), t[3], l);
    l = fmaf(bf16_bits_to_float(b8.z & 0xFFFFu), t[4], l);
    l = fmaf(bf16_bits_to_float(b8.z >> 16), t[5], l);
    l = fmaf(bf16_bits_to_float(b8.w & 0xFFFFu), t[6], l);
    l = fmaf(bf16_bits_to_float(b8.w >> 16), t[7], l);
    return l;
}

// ku == 0: finish the tile (add split-K partials, LoRA term, store y); ku > 0: leave a partial.
// WAVES (= 4) waves split the unit's super-steps.  In the MFMA result layout lane l holds, for
// row block mb and column block j, the rows 16*mb + 4*(l/16) + e (e = 0..3) of column 16*j + l%16;
// thread (wave w, lane l) finishes e = w of every (mb, j): EPT = 4*MB outputs that lie in MB rows
// (one adapter each), 16 columns apart.
template <int MB, int XR, int WAVES, int R, int FR>
__device__ __forceinline__ void base_unit(const LayerArgs &a, const ProjArgs &P, int pi, int tile, int ku,
                                 int m0, const BaseLds<MB, XR, WAVES, R> &lds)
{
    constexpr int ROWS = 16 * MB;
    constexpr int NT = 64 * WAVES;
    constexpr int EPT = MB * 16 / WAVES;
    const int K = P.K, N = P.N, M = a.M;
    int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int l16 = lane & 15, lq = lane >> 4;
    // the units of a split projection form the longest chain of the launch: they go first
    // wherever they share a SIMD with other waves
    if (P.ksplit > 1) __builtin_amdgcn_s_setprio(2);

    // super-steps of this K unit, then of this wave (balanced splits)
    const int nss = K / SUPER_K;
    const int uq = P.unit_q, ur = P.unit_r;
    const int unit_beg = ku * uq + min(ku, ur), unit_cnt = uq + (ku < ur ? 1 : 0);
    const int q = unit_cnt / WAVES, r = unit_cnt % WAVES;
    const int my_cnt = q + (wave < r ? 1 : 0);
    // a wave without work still issues (valid) loads: point it at the unit's first super-step
    const int my_beg = my_cnt > 0 ? unit_beg + wave * q + min(wave, r) : unit_beg;

    const int ksteps = K / KSTEP;
    const int ngroups = ksteps >> P.spg_shift;
    const uint4 *codes_tile = P.codes + (size_t)tile * ksteps * 64;
    const uint2 *scales_tile = P.scales + (size_t)tile * ngroups * 16;

    // what this thread will finish, and the adapter of each of its rows
    const bool lora = (ku == 0) && (a.row_adapter != nullptr) && (P.n_adapters > 0);
    const int rows_here = min(ROWS, M - m0);
    constexpr bool PREFETCH = EPT <= 8;                    // more outputs per thread: too many registers
    // (ranks up to FR: the entries of t of a chunk number at most MB * FR / 16 per thread)
    const bool fast = PREFETCH && lora && P.rank <= FR;
    // element qq of this thread: tile row and column (cheap to recompute, so not kept live)
    static_assert(WAVES == 4, "one wave per element of an MFMA result register");
    auto elem_ml = [&](int qq) { return (qq >> 2) * 16 + 4 * lq + wave; };
    auto elem_col = [&](int qq) { return 16 * (qq & 3) + l16; };
    const int *ra_safe = lora ? a.row_adapter : reinterpret_cast<const int *>(P.codes);
    const int ra_last = lora ? M - 1 : 0;
    int ad_raw[MB];                                        // as loaded, one per row of this thread
    auto elem_ad = [&](int qq) {
        const int v = ad_raw[qq >> 2];
        return (lora && m0 + elem_ml(qq) < M && v >= 0 && v < P.n_adapters) ? v : -1;
    };

    f32x4 acc[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[mb][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // epilogue operands fetched while the last round is being computed: the rows of B of this
    // thread's outputs (ranks up to FR) and its entries of t
    EpiPrefetch<PREFETCH ? EPT : 0, MB, FR> pf;
    constexpr int TH = FR / 16;
    auto prefetch_setup = [&]() {
        pf.t_ml = tid >> 4;
        pf.t_jj = tid & 15;
        pf.n0 = tile * TILE_N + l16;
        pf.nlast = N - 1;
        pf.kch = P.kch;
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            const int ad = elem_ad(4 * i);
            const bool ok = fast && ad >= 0;
            pf.bad[i] = ok ? P.lora_b + (size_t)ad * N * P.rank : reinterpret_cast<const uint16_t *>(P.codes);
            pf.brank[i] = ok ? P.rank : 0;
#pragma unroll
            for (int h = 0; h < TH; ++h) {
                pf.t_mine[i][h] = fast && pf.t_ml + 16 * i < rows_here && pf.t_jj + 16 * h < P.r16;
                pf.tp[i][h] = pf.t_mine[i][h] ? P.t_part + (size_t)(m0 + pf.t_ml + 16 * i) * P.r16 + pf.t_jj + 16 * h
                                              : reinterpret_cast<const float *>(P.codes);
                pf.tstride[i][h] = pf.t_mine[i][h] ? (size_t)M * P.r16 : 0;
            }
        }
    };
    // alpha * t of this thread's entries -> LDS: the K-chunk partials of the shrink step, all
    // requested at once and summed in fixed order
    auto t_entries_to_lds = [&]() {
        constexpr int E = MB * TH;                         // entries of this thread: (row block i, half h) = e / TH, e % TH
        float ts[E];
        if (pf.kch <= 4) {
            float tv[E][4];
#pragma unroll
            for (int e = 0; e < E; ++e)
#pragma unroll
                for (int kc = 0; kc < 4; ++kc)
                    tv[e][kc] = load_shared(pf.tp[e / TH][e % TH] + (size_t)min(kc, pf.kch - 1) * pf.tstride[e / TH][e % TH]);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                ts[e] = 0.f;
#pragma unroll
                for (int kc = 0; kc < 4; ++kc) ts[e] += kc < pf.kch ? tv[e][kc] : 0.f;
            }
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e) {
                float tv[MAX_KCHUNKS];
#pragma unroll
                for (int kc = 0; kc < MAX_KCHUNKS; ++kc)
                    tv[kc] = load_shared(pf.tp[e / TH][e % TH] + (size_t)min(kc, pf.kch - 1) * pf.tstride[e / TH][e % TH]);
                ts[e] = 0.f;
#pragma unroll
                for (int kc = 0; kc < MAX_KCHUNKS; ++kc) ts[e] += kc < pf.kch ? tv[kc] : 0.f;
            }
        }
#pragma unroll
        for (int e = 0; e < E; ++e)
            if (pf.t_mine[e / TH][e % TH]) lds.t_row(pf.t_ml + 16 * (e / TH))[pf.t_jj + 16 * (e % TH)] = ts[e] * P.alpha;
    };

    // the two constants of expand_codes arrive as kernel arguments so that they live in
    // registers and each field pair costs one and-or instead of an and plus an or with literals
    const uint32_t mask = a.code_mask;
    uint32_t bias = a.code_bias;
    asm volatile("" : "+v"(bias));      // pin to a vector register (one scalar operand per op)

    // counters this block depends on (or signals): see common.hpp
    const int tiles = tiles_n(N);
    const int chunk = m0 / ROWS, chunks = a.m_pad / ROWS;
    const int fin = tile * chunks + chunk;                 // this finishing block among its projection's
    const int copies = P.ctr_copies;                       // copies of the shrink counter in use (a power of two)
    unsigned *const sctr = a.ctrl + shrink_ctr(pi, fin & (copies - 1));
    unsigned *const pctr = a.ctrl + P.part_ctr + fin * CTR_STRIDE;
    const bool need_s = lora, need_p = ku == 0 && P.ksplit > 1;
    unsigned seen_s = 0, seen_p = 0;                       // what an early look at them showed

    unsigned char *buf = lds.stage(wave);
    const int ks_first = my_beg * 4, ks_total = my_cnt * 4;
    const int rows_x = min(rows_here, XR);
    if constexpr (MB == 1) {
        // decode shapes: rows of x of the wave's whole range -> LDS, then the register pipeline
        using L = StreamLds<XR>;
        u32x4 xr[XR];
        const int kx = min(ks_first * KSTEP + lane * 8, K - 8);
#pragma unroll
        for (int i = 0; i < XR; ++i)
            xr[i] = *reinterpret_cast<const u32x4 *>(P.x + (size_t)(m0 + min(i, rows_x - 1)) * K + kx);
        // adapters of this thread's rows: requested here (unconditionally), decoded below
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) ad_raw[mb] = ra_safe[min(m0 + elem_ml(4 * mb), ra_last)];
        const u32x4 *wp = reinterpret_cast<const u32x4 *>(codes_tile) + (size_t)ks_first * 64;
        const uint2 *sp = scales_tile + (size_t)(ks_first >> P.spg_shift) * 16;
        const unsigned char *xl = buf + min(l16, rows_x - 1) * L::XROW + 16 * lq;
        StreamRegs sa, sb;
        // an idle wave requests (and ignores) the unit's first super-step
        stream_request(sa, wp, sp, 0, max(my_cnt, 1), 4 >> P.spg_shift, lane);
        stream_request(sb, wp, sp, 1, my_cnt, 4 >> P.spg_shift, lane);
        __builtin_amdgcn_sched_barrier(0);                     // (the requests stay ahead of the wait for x)
#pragma unroll
        for (int i = 0; i < XR; ++i) *reinterpret_cast<u32x4 *>(buf + lane * 16 + i * L::XROW) = xr[i];
        const unsigned *dummy = reinterpret_cast<const unsigned *>(wp);
        const unsigned *poll_s = need_s ? sctr : dummy, *poll_p = need_p ? pctr : dummy;
        if (P.spg == 1)      stream_loop<1>(acc[0], sa, sb, wp, sp, my_cnt, xl, mask, bias, lane, poll_s, poll_p, seen_s, seen_p);
        else if (P.spg == 2) stream_loop<2>(acc[0], sa, sb, wp, sp, my_cnt, xl, mask, bias, lane, poll_s, poll_p, seen_s, seen_p);
        else                 stream_loop<4>(acc[0], sa, sb, wp, sp, my_cnt, xl, mask, bias, lane, poll_s, poll_p, seen_s, seen_p);
        // Everything below derives its indices afresh from the thread id: values shared with the
        // code above the loop would have to live across it, in registers the loop needs.
        asm volatile("" : "+v"(tid));
        lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
        // rows of B: in flight during what follows.  (The empty asm keeps the decoding of the
        // adapter index, and with it state that would live across the loop, behind the loop.)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) asm volatile("" : "+v"(ad_raw[mb]));
        prefetch_setup();
        pf.issue();
    } else {
        // K loop, two rounds per pass.  An idle wave (my_cnt == 0) still requests one round at a
        // valid place and computes nothing.
        const int nr = ks_total / R;                           // rounds of this wave
        RoundW<R> wa, wb;
        RoundX<XR, R> xr;
        round_issue_w<R>(wa, codes_tile, scales_tile, P.spg, ks_first, true, lane);
        round_issue_w<R>(wb, codes_tile, scales_tile, P.spg, ks_first + R, 1 < nr, lane);
        round_issue_x<XR, R>(xr, P.x, K, m0, rows_x, ks_first, true, lane);
        // (keeps all of these requests ahead of the first wait)
        __builtin_amdgcn_sched_barrier(0);
        auto compute = [&](int n) {
            if (P.spg == 1)      round_compute<MB, XR, R, 1>(acc, buf, n, rows_x, mask, bias, lane);
            else if (P.spg == 2) round_compute<MB, XR, R, 2>(acc, buf, n, rows_x, mask, bias, lane);
            else                 round_compute<MB, XR, R, 4>(acc, buf, n, rows_x, mask, bias, lane);
        };
#pragma nounroll
        for (int r0 = 0; r0 < max(nr, 1); r0 += 2) {
            round_to_lds<XR, R>(wa, xr, buf, lane);
            round_issue_w<R>(wa, codes_tile, scales_tile, P.spg, ks_first + (r0 + 2) * R, r0 + 2 < nr, lane);
            round_issue_x<XR, R>(xr, P.x, K, m0, rows_x, ks_first + (r0 + 1) * R, r0 + 1 < nr, lane);
            // (the scheduler would otherwise sink the requests below the math to save registers)
            __builtin_amdgcn_sched_barrier(0);
            compute(r0 < nr ? R : 0);
            round_to_lds<XR, R>(wb, xr, buf, lane);
            round_issue_w<R>(wb, codes_tile, scales_tile, P.spg, ks_first + (r0 + 3) * R, r0 + 3 < nr, lane);
            round_issue_x<XR, R>(xr, P.x, K, m0, rows_x, ks_first + (r0 + 2) * R, r0 + 2 < nr, lane);
            __builtin_amdgcn_sched_barrier(0);
            compute(r0 + 1 < nr ? R : 0);
        }
        // Everything below derives its indices afresh from the thread id: values shared with the
        // code above the loop would have to live across it, in registers the loop needs.
        asm volatile("" : "+v"(tid));
        lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
        // adapters of this thread's rows, then their rows of B: requested once the rounds'
        // registers are free
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) ad_raw[mb] = ra_safe[min(m0 + elem_ml(4 * mb), ra_last)];
        prefetch_setup();
        pf.issue();
    }

    // Above 16 rows the partial tiles and t lie over the staging buffers of all waves: meet first.
    if constexpr (!BaseLds<MB, XR, WAVES, R>::PRIVATE) __syncthreads();
    // What the epilogue reads from other blocks.  Every wave makes sure of it for itself (all
    // lanes poll the same word), unless the look during its last super-step already showed it.
    // A wave whose wait runs out sets the workspace's status word and stores NaN in place of its
    // outputs: a call that went wrong must not look like one that went right.
    bool poisoned = false;
    {
        const int limit = a.spin_limit;
        bool ok = true;
        if (need_s && (limit == 0 || seen_s < (unsigned)P.n_shrink_blocks)) ok = wait_count(sctr, (unsigned)P.n_shrink_blocks, limit);
        if (need_p && (limit == 0 || seen_p < (unsigned)(P.ksplit - 1))) ok = wait_count(pctr, (unsigned)(P.ksplit - 1), limit) && ok;
        compiler_fence();
        if (!ok && lane == 0) atomicOr(a.status, 1u);
        poisoned = !ok;
    }
    const float nan_f = __uint_as_float(0x7FC00000u);

    // partial tiles -> LDS: element (mb, j, e) of lane l at red_at(mb, e, l) + j, so that the thread
    // that finishes e of every j reads four of them at once
    auto red_at = [](int mb, int e, int l) { return ((mb * 4 + e) * 64 + l) * 4; };
    {
        float *red = lds.red(wave);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                *reinterpret_cast<f32x4 *>(red + red_at(mb, e, lane)) =
                    f32x4{acc[mb][0][e], acc[mb][1][e], acc[mb][2][e], acc[mb][3][e]};
    }

    constexpr int PU = 7;                                  // split-K units (beside the block's own) the short way out adds
    // The common decode case gets a short, nearly branch-free way out (code that runs once per
    // launch is paid for by the instruction fetch, so its length is its cost): a finishing block
    // whose LoRA term, if any, was prefetched above and whose K has at most PU + 1 units.
    const bool lean = PREFETCH && ku == 0 && (!lora || fast) && P.ksplit <= PU + 1;
    if (lean) {
        if constexpr (PREFETCH) {
            // a fused call's operands of the output stage: on their way while t and the partial
            // tiles are fetched
            FusedOperands fo[MB];
            if (a.fused) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) fo[mb] = fused_fetch(a, P, pi, m0 + elem_ml(4 * mb), tile, l16);
            }
            if (lora) t_entries_to_lds();
            float pv[EPT][PU];
            if (P.ksplit > 1) {
                const size_t ustride = (size_t)tiles * a.m_pad * TILE_N;
#pragma unroll
                for (int qq = 0; qq < EPT; ++qq) {
                    const int m = min(m0 + elem_ml(qq), M - 1);
                    const float *src = P.partial + ((size_t)tile * a.m_pad + m) * TILE_N + elem_col(qq);
#pragma unroll
                    for (int u = 0; u < 3; ++u) pv[qq][u] = load_shared(src + (size_t)min(u, P.ksplit - 2) * ustride);
                }
                // (more than four units: K above 8192; the common case does not pay for these loads)
                if (PU > 3 && P.ksplit > 4) {
#pragma unroll
                    for (int qq = 0; qq < EPT; ++qq) {
                        const int m = min(m0 + elem_ml(qq), M - 1);
                        const float *src = P.partial + ((size_t)tile * a.m_pad + m) * TILE_N + elem_col(qq);
#pragma unroll
                        for (int u = 3; u < PU; ++u) pv[qq][u] = load_shared(src + (size_t)min(u, P.ksplit - 2) * ustride);
                    }
                } else {
#pragma unroll
                    for (int qq = 0; qq < EPT; ++qq)
#pragma unroll
                        for (int u = 3; u < PU; ++u) pv[qq][u] = 0.f;
                }
            }
            __syncthreads();
            const int n0 = tile * TILE_N + l16;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                f32x4 v = *reinterpret_cast<const f32x4 *>(lds.red(0) + red_at(mb, wave, lane));
#pragma unroll
                for (int w = 1; w < WAVES; ++w)
                    v += *reinterpret_cast<const f32x4 *>(lds.red(w) + red_at(mb, wave, lane));
                if (P.ksplit > 1) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int u = 0; u < PU; ++u) v[j] += u + 1 < P.ksplit ? pv[4 * mb + j][u] : 0.f;
                }
                if (lora) {
                    // (entries of a row of t past the rank are not written and not used)
                    float t[FR];
                    const f32x4 *tr = reinterpret_cast<const f32x4 *>(lds.t_row(elem_ml(4 * mb)));
#pragma unroll
                    for (int i = 0; i < FR / 4; ++i) {
                        const f32x4 tq = tr[i];
                        t[4 * i] = tq[0]; t[4 * i + 1] = tq[1]; t[4 * i + 2] = tq[2]; t[4 * i + 3] = tq[3];
                    }
                    const bool mine = elem_ad(4 * mb) >= 0;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float l = dot8(pf.b[4 * mb + j][0], t, 0.f);
#pragma unroll
                        for (int c = 1; c < FR / 8; ++c)
                            if (P.rank > 8 * c) l = dot8(pf.b[4 * mb + j][c], t + 8 * c, l);
                        v[j] += mine ? l : 0.f;
                    }
                }
                const int m = m0 + elem_ml(4 * mb);
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = poisoned ? nan_f : v[j];
                if (a.fused) {
                    float vv[4] = {v[0], v[1], v[2], v[3]};
                    fused_store(a, P, pi, m, tile, l16, fo[mb], vv);
                } else if (m < M) {
                    if (a.y_fp32) {
                        float *yp = reinterpret_cast<float *>(P.y) + (size_t)m * N + n0;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (n0 + 16 * j < N) yp[16 * j] = v[j];
                    } else {
                        uint16_t *yp = reinterpret_cast<uint16_t *>(P.y) + (size_t)m * N + n0;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (n0 + 16 * j < N) yp[16 * j] = float_to_bf16_bits(v[j]);
                    }
                }
            }
        }
    } else {
        // split-K partials of this thread's outputs: all requested at once (a thread with nothing to
        // add re-reads a valid address), consumed after the reduction below
        constexpr int PU = 3;
        float pv[EPT][PU];
#pragma unroll
        for (int qq = 0; qq < EPT; ++qq)
#pragma unroll
            for (int u = 0; u < PU; ++u) {
                const int m = m0 + elem_ml(qq);
                const bool ok = ku == 0 && u + 1 < P.ksplit && m < M;
                const float *src = ok ? P.partial + (((size_t)u * tiles + tile) * a.m_pad + m) * TILE_N + elem_col(qq)
                                      : reinterpret_cast<const float *>(P.codes);
                pv[qq][u] = load_shared(src);
            }
        // t[m] = alpha * sum of the shrink step's K-chunk partials (fixed order)
        if (fast) {
            t_entries_to_lds();
        } else if (lora && MB == 1) {
            // (the kernels for up to 16 rows keep this path short: it is rare there, and its size
            // costs the common path instruction fetches)
            for (int idx = tid; idx < rows_here * P.r16; idx += NT) {
                const int ml = idx / P.r16, jj = idx % P.r16;
                const int ad = a.row_adapter[m0 + ml];
                float v = 0.f;
                if (ad >= 0 && ad < P.n_adapters)
                    for (int kc = 0; kc < P.kch; ++kc)
                        v += load_shared(P.t_part + ((size_t)kc * M + (m0 + ml)) * P.r16 + jj);
                lds.t_row(ml)[jj] = v * P.alpha;
            }
        } else if (lora) {
            // four entries of t per thread and four K chunks at a time: 16 loads in flight instead of
            // one after another (a rank of 32 at 32 rows is four entries per thread, each the sum
            // of up to 16 partials)
            for (int i0 = 0; i0 < rows_here * P.r16; i0 += 4 * NT) {
                float v[4] = {0.f, 0.f, 0.f, 0.f};
                bool live[4];
                const float *src[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = i0 + q * NT + tid;
                    const int ml = min(idx / P.r16, rows_here - 1), jj = idx % P.r16;
                    const int ad = a.row_adapter[m0 + ml];
                    live[q] = idx < rows_here * P.r16 && ad >= 0 && ad < P.n_adapters;
                    src[q] = live[q] ? P.t_part + (size_t)(m0 + ml) * P.r16 + jj : P.t_part;
                }
                for (int kc0 = 0; kc0 < P.kch; kc0 += 4) {
                    float pv[4][4];
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            pv[q][c] = load_shared(src[q] + (live[q] ? (size_t)min(kc0 + c, P.kch - 1) * M * P.r16 : 0));
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (kc0 + c < P.kch) v[q] += pv[q][c];
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = i0 + q * NT + tid;
                    if (idx < rows_here * P.r16) lds.t_row(idx / P.r16)[idx % P.r16] = live[q] ? v[q] * P.alpha : 0.f;
                }
            }
        }
        __syncthreads();

        float fv[EPT];                                     // a fused call's outputs, stored after the loop
#pragma unroll
        for (int qq = 0; qq < EPT; ++qq) fv[qq] = 0.f;
        // ranks above 16: B[a(m)][n] . t[m] of this thread's outputs, the rows of B fetched 32 ranks
        // of four outputs at a time (16 loads in flight), summed in rank order
        float ll[EPT];
#pragma unroll
        for (int qq = 0; qq < EPT; ++qq) ll[qq] = 0.f;
        if (MB == 2 && lora && !fast && ku == 0) {
            for (int jj0 = 0; jj0 < P.rank; jj0 += 32) {
#pragma unroll
                for (int h = 0; h < EPT; h += 4) {
                    uint4 bq[4][4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int ad = elem_ad(h + q);
                        const int n = min(tile * TILE_N + elem_col(h + q), N - 1);
                        const uint16_t *brow = P.lora_b + ((size_t)max(ad, 0) * N + n) * P.rank;
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            bq[q][c] = *reinterpret_cast<const uint4 *>(brow + min(jj0 + 8 * c, P.rank - 8));
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const bool mine = elem_ad(h + q) >= 0;
                        const float *tr = lds.t_row(elem_ml(h + q));
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (mine && jj0 + 8 * c < P.rank) ll[h + q] = dot8(bq[q][c], tr + jj0 + 8 * c, ll[h + q]);
                    }
                }
            }
        }
#pragma unroll
        for (int qq = 0; qq < EPT; ++qq) {
            const int off = red_at(qq >> 2, wave, lane) + (qq & 3);
            float v = lds.red(0)[off];
#pragma unroll
            for (int w = 1; w < WAVES; ++w) v += lds.red(w)[off];
            const int ml = elem_ml(qq), col = elem_col(qq);
            const int m = m0 + ml;
            const int n = tile * TILE_N + col;
            if (ku > 0) {
                store_shared(P.partial + (((size_t)(ku - 1) * tiles + tile) * a.m_pad + m) * TILE_N + col, v);
                continue;
            }
            if (m < M && n < N) {
#pragma unroll
                for (int u = 0; u < PU; ++u)
                    if (u + 1 < P.ksplit) v += pv[qq][u];
                for (int u = PU + 1; u < P.ksplit; ++u)
                    v += load_shared(P.partial + (((size_t)(u - 1) * tiles + tile) * a.m_pad + m) * TILE_N + col);
                const int ad = elem_ad(qq);
                if (ad >= 0) {
                    float l = 0.f;
                    if (fast) {
                        if constexpr (PREFETCH) {
                            l = dot8(pf.b[qq][0], lds.t_row(ml), l);
#pragma unroll
                            for (int c = 1; c < FR / 8; ++c)
                                if (P.rank > 8 * c) l = dot8(pf.b[qq][c], lds.t_row(ml) + 8 * c, l);
                        }
                    } else if (MB == 2) {
                        l = ll[qq];
                    } else {
                        const uint16_t *brow = P.lora_b + ((size_t)ad * N + n) * P.rank;
                        for (int jj = 0; jj < P.rank; jj += 8)
                            l = dot8(*reinterpret_cast<const uint4 *>(brow + jj), lds.t_row(ml) + jj, l);
                    }
                    v += l;
                }
                v = poisoned ? nan_f : v;
                if (a.fused) fv[qq] = v;
                else if (a.y_fp32) reinterpret_cast<float *>(P.y)[(size_t)m * N + n] = v;
                else reinterpret_cast<uint16_t *>(P.y)[(size_t)m * N + n] = float_to_bf16_bits(v);
            }
        }
        if (a.fused && ku == 0) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                float vv[4] = {fv[4 * mb], fv[4 * mb + 1], fv[4 * mb + 2], fv[4 * mb + 3]};
                store_fused(a, P, pi, m0 + elem_ml(4 * mb), tile, l16, vv);
            }
        }
    }
    if (ku > 0) signal_done(pctr, 1);
    // Counters go back to zero for the next call: a tile's split-K counter once every wave has
    // passed it (the barrier above), a copy of the shrink counter by the last block that used it.
    if (tid == 0 && need_p) __hip_atomic_store(pctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid == 0 && need_s) {
        const int users = (P.n_finish_blocks >> (31 - __clz(copies))) + ((fin & (copies - 1)) < (P.n_finish_blocks & (copies - 1)) ? 1 : 0);
        if (atomicAdd(sctr + 1, 1u) + 1u == (unsigned)users) {
            __hip_atomic_store(sctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(sctr + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// ------------------------------------------------------------------------------------------
// LoRA shrink
// ------------------------------------------------------------------------------------------
// Rows of x and rank rows of A are both K elements apart, a power of two as a rule: a request
// that takes 16 bytes from each of 16 such rows (an MFMA fragment read directly) lands in one
// memory channel and holds up every other wave of its compute unit.  So both are read in
// contiguous runs (4 rows x 256 bytes per instruction) and turned into fragments through a
// wave-private LDS buffer, four k-steps at a time.
//
// Grouped shrink (more than 16 rows per call).  A block = (chunk of 64 rows, share of the
// chunk's row tiles, 16 ranks, chunk of K).  Wave 0 groups the chunk's rows by adapter (a few
// ballots) and every segment is cut into tiles of 16 rows; the block's four waves then take the
// tiles of the block's share in turn, each wave working through the whole K chunk of its tile on
// its own: no reduction across waves, and few, long-lived blocks, which leaves the compute
// units to the base blocks from the start of the launch (the blocks of a launch are placed in
// grid order, so many short shrink blocks in front would hold every base block back).
struct ShrinkLds {
    static constexpr int SB = 4;                            // k-steps per batch
    static constexpr int ROW = SB * 64 + 16;                // bytes of a staged row; +16: rows 4 banks apart
    GroupLds64 g;
    alignas(16) unsigned char a[4][16 * ROW];               // (16-byte LDS accesses)
    alignas(16) unsigned char x[4][16 * ROW];
};

template <bool A8>
__device__ __forceinline__ void shrink_block(const LayerArgs &a, const ProjArgs &P, int pi, int local, ShrinkLds &lds)
{
    using L = ShrinkLds;
    constexpr int SB = L::SB;
    GroupLds64 &g = lds.g;
    const int jblocks = P.r16 / 16;
    const int shares = shrink_tile_shares(a.M_plan, P.n_adapters);
    const int kc = local % P.kch;
    const int jb = (local / P.kch) % jblocks;
    const int share = (local / (P.kch * jblocks)) % shares;
    const int chunk = local / (P.kch * jblocks * shares);
    const int m_base = chunk * SHRINK_CHUNK_ROWS;

    group_rows_lds64(a.row_adapter + m_base, min(SHRINK_CHUNK_ROWS, a.M - m_base), P.n_adapters, g);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    // k-steps of this block's K chunk (balanced split)
    const int nks = P.K / KSTEP;
    const int q = nks / P.kch, r = nks % P.kch;
    const int blk_beg = kc * q + min(kc, r), blk_cnt = q + (kc < r ? 1 : 0);
    unsigned char *la = lds.a[wave], *lx = lds.x[wave];
    const u32x4 zero = {0u, 0u, 0u, 0u};

    // tiles of the chunk in segment order; tile t belongs to wave (t mod 4 * shares) - 4 * share
    const int n_seg = g.n_seg;
    int t = 0;
    for (int sg = 0; sg < n_seg; ++sg) {
        const int seg_first = (int)g.seg_start[sg], seg_len = (int)g.seg_start[sg + 1] - seg_first;
        const int adapter = g.seg_adapter[sg];
        for (int u = 0; u < seg_len; u += 16, ++t) {
            if (t % (4 * shares) != 4 * share + wave) continue;
            const int first = seg_first + u;
            const int rows_here = min(16, seg_len - u);
            // loads: instruction i covers staged rows 4*i + lane/16, 16 bytes per lane (lane%16 of 16)
            const uint16_t *xsrc[4], *asrc[4];
            bool x_ok[4], a_ok[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int rr = 4 * i + lq;                  // staged row: tile row of x, rank row of A
                x_ok[i] = rr < rows_here;
                const int row = m_base + (x_ok[i] ? (int)g.perm[first + rr] : 0);
                // (int8 rows: the same element offsets, one byte each; kept as a uint16 pointer and
                // turned into a byte address where it is used)
                xsrc[i] = A8 ? reinterpret_cast<const uint16_t *>(reinterpret_cast<const unsigned char *>(P.x) + (size_t)row * P.K + (size_t)blk_beg * KSTEP + l16 * 8)
                             : P.x + (size_t)row * P.K + (size_t)blk_beg * KSTEP + l16 * 8;
                const int j = jb * 16 + rr;
                a_ok[i] = j < P.rank;
                asrc[i] = P.lora_a + ((size_t)adapter * P.rank + (a_ok[i] ? j : 0)) * P.K + (size_t)blk_beg * KSTEP + l16 * 8;
            }
            // four batches (a K chunk of 512 inputs, whole) in flight: the base blocks fill the
            // memory queues at the same time, and a tile should cost one round trip, not four
            constexpr int DEPTH = 2;
            u32x4 xv[DEPTH][4], av[DEPTH][4];
            auto request = [&](int set, int s0) {
                const bool k_ok = (l16 >> 2) < blk_cnt - s0;    // this lane's 8 inputs lie in k-step s0 + l16/4
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if constexpr (A8) {
                        // eight int8 -> eight bf16 (exact: seven bits and a sign)
                        uint2 q = make_uint2(0u, 0u);
                        if (x_ok[i] && k_ok) q = *reinterpret_cast<const uint2 *>(reinterpret_cast<const unsigned char *>(xsrc[i]) + (size_t)s0 * KSTEP);
                        const uint32_t src2[2] = {q.x, q.y};
                        u32x4 o;
#pragma unroll
                        for (int h = 0; h < 4; ++h) {
                            const uint32_t word = src2[h >> 1];
                            const int e0 = (int)(signed char)(word >> (16 * (h & 1)));
                            const int e1 = (int)(signed char)(word >> (16 * (h & 1) + 8));
                            o[h] = (__float_as_uint((float)e0) >> 16) | (__float_as_uint((float)e1) & 0xFFFF0000u);
                        }
                        xv[set][i] = o;
                    } else {
                        xv[set][i] = (x_ok[i] && k_ok) ? *reinterpret_cast<const u32x4 *>(xsrc[i] + (size_t)s0 * KSTEP) : zero;
                    }
                    av[set][i] = (a_ok[i] && k_ok) ? *reinterpret_cast<const u32x4 *>(asrc[i] + (size_t)s0 * KSTEP) : zero;
                }
            };
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            auto consume = [&](int set) {
                // (wave-private buffers: the wave's own LDS accesses are ordered, no barrier)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    *reinterpret_cast<u32x4 *>(lx + (4 * i + lq) * L::ROW + l16 * 16) = xv[set][i];
                    *reinterpret_cast<u32x4 *>(la + (4 * i + lq) * L::ROW + l16 * 16) = av[set][i];
                }
#pragma unroll
                for (int s = 0; s < SB; ++s) {
                    const uint4 xa = *reinterpret_cast<const uint4 *>(lx + l16 * L::ROW + s * 64 + 16 * lq);
                    const uint4 ab = *reinterpret_cast<const uint4 *>(la + l16 * L::ROW + s * 64 + 16 * lq);
                    acc = mfma16(xa, ab, acc);
                }
            };
#pragma unroll
            for (int d = 0; d < DEPTH; ++d)
                if (d * SB < blk_cnt) request(d, d * SB);
            for (int s0 = 0; s0 < blk_cnt; s0 += DEPTH * SB) {
#pragma unroll
                for (int d = 0; d < DEPTH; ++d) {
                    if (s0 + d * SB < blk_cnt) {
                        consume(d);
                        if (s0 + (d + DEPTH) * SB < blk_cnt) request(d, s0 + (d + DEPTH) * SB);
                    }
                }
            }
            // lane (rank column l16, quarter lq) holds tile rows 4*lq + e
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = 4 * lq + e;
                if (i < rows_here) {
                    const int m = m_base + g.perm[first + i];
                    store_shared(P.t_part + ((size_t)kc * a.M + m) * P.r16 + jb * 16 + l16, acc[e]);
                }
            }
        }
    }
    signal_done(a.ctrl + shrink_ctr(pi, 0), P.ctr_copies);
}


// Decode shapes (at most 16 rows): one block per (row, block of 16 ranks, K chunk) and no
// grouping.  The row's adapter index is one scalar load away, so the block's requests go out
// before the base blocks have filled the memory queues; rows that share an adapter read its A
// once each, from the cache.  Row 0 of the MFMA's A operand carries x[m]; the other rows are 0.
//
// A[adapter] is read in runs of 512 contiguous bytes per rank row and turned into MFMA fragments
// through a wave-private LDS buffer.  Reading the fragments directly (16 bytes from each of 16
// rows per lane group) would address rows a power of two apart, which all lie in the same
// memory channel: measured, those requests held up every other wave of their compute unit for
// about 5 us.
struct ShrinkRowLds {
    static constexpr int SB = 8;                            // k-steps per batch
    static constexpr int AROW = SB * 64 + 16;               // bytes of a rank row in a batch; +16: rows 4 banks apart
    unsigned char a[4][16 * AROW];
    unsigned char x[4][SB * 64];
    float red[4][16];
};

__device__ __forceinline__ void shrink_row_block(const LayerArgs &a, const ProjArgs &P, int pi, int local,
                                                 ShrinkRowLds &lds)
{
    using L = ShrinkRowLds;
    constexpr int SB = L::SB;
    const int jblocks = P.r16 / 16;
    const int kc = local % P.kch;
    const int jb = (local / P.kch) % jblocks;
    const int m = local / (P.kch * jblocks);               // < M: the grid has M such rows of blocks
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    const int half = lane >> 5, l32 = lane & 31;            // loads: two rank rows per instruction

    // k-steps of this block, then of this wave (balanced splits)
    const int nks = P.K / KSTEP;
    const int q = nks / P.kch, r = nks % P.kch;
    const int blk_beg = kc * q + min(kc, r), blk_cnt = q + (kc < r ? 1 : 0);
    const int wq_ = blk_cnt / 4, wr = blk_cnt % 4;
    const int my_beg = blk_beg + wave * wq_ + min(wave, wr);
    const int my_cnt = wq_ + (wave < wr ? 1 : 0);

    const u32x4 zero = {0u, 0u, 0u, 0u};
    const int adapter = a.row_adapter[m];
    const bool valid = adapter >= 0 && adapter < P.n_adapters;      // uniform
    const uint16_t *xrow = P.x + (size_t)m * P.K + (size_t)my_beg * KSTEP + l32 * 8;
    const uint16_t *arow = P.lora_a + (size_t)(valid ? adapter : 0) * P.rank * P.K + (size_t)my_beg * KSTEP + l32 * 8;
    unsigned char *la = lds.a[wave], *lx = lds.x[wave];

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < my_cnt && valid; s0 += SB) {
        const int cnt = min(SB, my_cnt - s0);               // k-steps of this batch
        const bool k_ok = (l32 >> 2) < cnt;                 // this lane's 8 inputs lie in k-step l32/4
        const u32x4 xv = (half == 0 && k_ok) ? *reinterpret_cast<const u32x4 *>(xrow + (size_t)s0 * KSTEP) : zero;
        u32x4 av[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int j = jb * 16 + 2 * i + half;
            av[i] = (k_ok && j < P.rank) ? *reinterpret_cast<const u32x4 *>(arow + (size_t)j * P.K + (size_t)s0 * KSTEP)
                                         : zero;
        }
        if (half == 0) *reinterpret_cast<u32x4 *>(lx + l32 * 16) = xv;
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4 *>(la + (2 * i + half) * L::AROW + l32 * 16) = av[i];
        // (wave-private buffer: the wave's own LDS accesses are ordered, no barrier)
#pragma unroll
        for (int s = 0; s < SB; ++s) {
            const uint4 ab = *reinterpret_cast<const uint4 *>(la + l16 * L::AROW + s * 64 + 16 * lq);
            uint4 xa = *reinterpret_cast<const uint4 *>(lx + s * 64 + 16 * lq);
            if (l16 != 0) xa = make_uint4(0, 0, 0, 0);
            acc = mfma16(xa, ab, acc);
        }
    }
    if (valid) {
        // row 0 of the result: element 0 of lanes 0..15
        if (lq == 0) lds.red[wave][l16] = acc[0];
        __syncthreads();
        if (tid < 16) {
            const float v = ((lds.red[0][tid] + lds.red[1][tid]) + lds.red[2][tid]) + lds.red[3][tid];
            store_shared(P.t_part + ((size_t)kc * a.M + m) * P.r16 + jb * 16 + tid, v);
        }
    }
    // (a base-only row has nothing to write, but the finishing blocks count its blocks all the same)
    signal_done(a.ctrl + shrink_ctr(pi, 0), P.ctr_copies);
}

// ------------------------------------------------------------------------------------------
// kernels
// ------------------------------------------------------------------------------------------
// MB blocks of 16 rows per chunk, XR rows staged in LDS (the smallest multiple of 8 that holds
// the rows of a chunk decides which instance runs): 4 waves per block, rounds of R k-steps
// (two rounds = 2*R KiB of codes in flight per wave).
template <int MB> struct Shape;
template <> struct Shape<1> { static constexpr int WAVES = 4, R = 8; };
template <> struct Shape<2> { static constexpr int WAVES = 4, R = 4; };

template <int MB, int XR>
using BaseLdsOf = BaseLds<MB, XR, Shape<MB>::WAVES, Shape<MB>::R>;
template <int MB, int XR>
constexpr int pre_lds_bytes()
{
    constexpr int shrink = MB == 1 ? (int)sizeof(ShrinkRowLds) : (int)sizeof(ShrinkLds);   // (MB == 1: M <= 16)
    return BaseLdsOf<MB, XR>::BYTES > shrink ? BaseLdsOf<MB, XR>::BYTES : shrink;
}

// Fetch every field of a projection's argument block at once.  Kernel arguments sit behind a
// scalar cache that is cold at every launch (about 0.4 us per dependent access); left alone,
// the compiler loads each field where it is first used, one round trip after another.  Pinning
// all fields to registers at one point makes it issue the loads together.
__device__ __forceinline__ ProjArgs fetch_proj(const LayerArgs &a, int pi)
{
    ProjArgs P = a.p[pi];
    asm volatile("" :: "s"(P.codes), "s"(P.scales), "s"(P.x), "s"(P.y), "s"(P.lora_a), "s"(P.lora_b),
                 "s"(P.t_part), "s"(P.partial));
    asm volatile("" :: "s"(P.K), "s"(P.N), "s"(P.spg), "s"(P.n_adapters), "s"(P.rank), "s"(P.r16),
                 "s"(P.kch), "s"(P.alpha), "s"(P.ksplit));
    asm volatile("" :: "s"(P.unit_q), "s"(P.unit_r), "s"(P.spg_shift), "s"(P.ctr_copies), "s"(P.tiles_inv));
    return P;
}

// The three block-table rows of the block's group and the scalar fields at the end of the launch
// arguments, all requested together at the kernel's start: one scalar round trip (the cache
// behind the kernel arguments is cold at every launch) instead of one for the scalars, a
// dependent one for the table of the block's kind and then the projection's record.  Left alone,
// the compiler loads each value where it is first used; and a pointer to the table of the
// block's kind would turn the search below into 16 dependent loads.
typedef int i32x16 __attribute__((ext_vector_type(16)));
static_assert(GROUP_PROJ == 16, "the block tables of a group are read as vectors of 16");
struct LaunchTables {
    i32x16 shrink, pre, main;
    int shrink_blocks, pre_base_blocks, group_blocks;
};
__device__ __forceinline__ LaunchTables pin_launch_args(const LayerArgs &a, int z)
{
    LaunchTables t;
    t.shrink = *reinterpret_cast<const i32x16 *>(a.shrink_begin[z]);
    t.pre = *reinterpret_cast<const i32x16 *>(a.pre_begin[z]);
    t.main = *reinterpret_cast<const i32x16 *>(a.main_begin[z]);
    t.shrink_blocks = a.shrink_blocks[z];
    t.pre_base_blocks = a.pre_base_blocks[z];
    t.group_blocks = a.group_blocks[z];
    asm volatile("" :: "s"(t.shrink), "s"(t.pre), "s"(t.main), "s"(a.row_adapter), "s"(a.M), "s"(a.y_fp32),
                       "s"(a.m_pad), "s"(t.shrink_blocks), "s"(t.pre_base_blocks), "s"(t.group_blocks),
                       "s"(a.ctrl), "s"(a.status), "s"(a.code_mask), "s"(a.code_bias), "s"(a.spin_limit));
    return t;
}

// Entries past the last projection hold INT_MAX, so all 16 comparisons can be made without a
// loop.  first = begin[pi], picked from the same registers (begins are non-decreasing).
__device__ __forceinline__ int find_proj(const i32x16 &begin, int b, int &first)
{
    int pi = 0;
    first = begin[0];
#pragma unroll
    for (int i = 1; i < GROUP_PROJ; ++i) {
        pi += (b >= begin[i]) ? 1 : 0;
        first = (b >= begin[i]) ? begin[i] : first;
    }
    return pi;
}

// blocks per compute unit the registers are budgeted for (LDS allows as many for these shapes)
// Block index -> (block of the group, row chunk).  The row chunks of one block of columns stream
// the same weights.  Workgroups go to the chip's 8 XCDs in turn (index mod 8), and every XCD has
// an L2 of its own, so the grid is laid out in runs of 8 blocks x all chunks with the chunk
// varying in steps of 8: index = (b / 8) * 8 * chunks + chunk * 8 + b % 8.  All chunks of a block
// then run on one XCD at about the same time, and its weights come from HBM once and from that
// L2 for the other chunks.  (Chunk-major order, a whole pass over the weights between two chunks,
// read 5.9 x the algorithmic bytes from HBM at 512 rows.)  A producer still has a smaller index
// than its consumer: shrink blocks work at chunk 0 only, and a split-K block and the block that
// finishes its tile have the same chunk.
__device__ __forceinline__ void split_block_index(const LayerArgs &a, int rows, int &b, int &chunk)
{
    const unsigned id = blockIdx.x;
    const unsigned chunks = (unsigned)(a.m_pad / rows);
    if (chunks == 1) {
        b = (int)id;
        chunk = 0;
    } else {
        const unsigned run = id / (8u * chunks), r = id - run * 8u * chunks;
        chunk = (int)(r >> 3);
        b = (int)(run * 8u + (r & 7u));
    }
}

template <int MB, int XR> constexpr int occupancy_of() { return MB == 1 && XR == 8 ? 3 : 2; }

template <int MB, int XR>
__global__ __launch_bounds__(64 * Shape<MB>::WAVES, (occupancy_of<MB, XR>())) void layer_kernel(const LayerArgs a)
{
    __shared__ __align__(16) unsigned char smem[pre_lds_bytes<MB, XR>()];
    const int z = (int)blockIdx.z;
    const LaunchTables tables = pin_launch_args(a, z);
    int b, chunk;
    split_block_index(a, 16 * MB, b, chunk);
    if (b >= tables.group_blocks) return;                  // (the slices are as long as the longest group)
    int first;
    if (b < tables.shrink_blocks) {
        if (chunk != 0) return;
        const int pi = z * GROUP_PROJ + find_proj(tables.shrink, b, first);
        // (the instances with one block of 16 rows are the ones launched for M <= 16)
        if constexpr (MB == 1) shrink_row_block(a, fetch_proj(a, pi), pi, b - first, *reinterpret_cast<ShrinkRowLds *>(smem));
        else                   shrink_block<false>(a, fetch_proj(a, pi), pi, b - first, *reinterpret_cast<ShrinkLds *>(smem));
        return;
    }
    const BaseLdsOf<MB, XR> lds{smem};
    const int m0 = chunk * 16 * MB;
    // (one call site for both kinds of base block: the kernel's code is large, and what runs
    // once per launch is paid for by instruction fetch)
    const bool pre = b < tables.shrink_blocks + tables.pre_base_blocks;
    const int bb = b - tables.shrink_blocks - (pre ? 0 : tables.pre_base_blocks);
    const int pi = z * GROUP_PROJ + find_proj(pre ? tables.pre : tables.main, bb, first);
    const ProjArgs P = fetch_proj(a, pi);
    const int local = bb - first;
    const int tiles = tiles_n(P.N);
    // local / tiles (tiles_inv = ceil(2^32 / tiles) does not fit 32 bits for a single tile)
    const int unit = !pre ? 0 : tiles == 1 ? local : (int)__umulhi((unsigned)local, P.tiles_inv);
    // (the kernel for 9 to 16 rows also runs the 16-row chunks of short launches of up to 32 rows,
    // among them a fused gate/up projection with its LoRA pair of twice the rank: a second copy of
    // the block with the prefetch for ranks up to 32; a call of rank 16 runs the code it always ran)
    if constexpr (MB == 1 && XR == 16) {
        if (P.rank > fast_rank<MB>()) {
            base_unit<MB, XR, Shape<MB>::WAVES, Shape<MB>::R, 32>(a, P, pi, local - unit * tiles, pre ? 1 + unit : 0, m0, lds);
            return;
        }
    }
    base_unit<MB, XR, Shape<MB>::WAVES, Shape<MB>::R, fast_rank<MB>()>(a, P, pi, local - unit * tiles, pre ? 1 + unit : 0, m0, lds);
}

// ------------------------------------------------------------------------------------------
// Wide shapes (33 rows or more per call): the product is a dense contraction and the matrix
// units are what bounds it.  A block covers 64 rows x 256 columns: its four waves share the rows
// of x (staged in LDS, one super-step of 128 inputs at a time, double-buffered) and each wave
// owns one 64-column tile, whose packed codes it streams into registers two super-steps ahead
// and unpacks once for all 64 rows (4 A fragments x 4 B fragments = 16 MFMAs per k-step, plus
// 4 for the offset term).  No K split inside the block; long K is cut into units as for the
// decode shapes, and a launch with few blocks is cut further by the host.
//
// Scales without a second set of accumulators: the accumulator is kept in units of the current
// group's scale, acc <- acc * (s_prev / s_cur) + (offset term), and the MFMAs of the group add
// their raw code products to it; the last scale is applied at the end.  A zero scale (padding
// columns; legal in a hand-made blob) keeps the previous unit and its codes are replaced by
// code 0, so it contributes exactly nothing.
//
// LoRA term on the matrix units too: t[m] (fp32, from the shrink blocks) is split into two bf16
// halves (hi + lo keeps 16 bits of mantissa), and for every adapter that occurs in the chunk of
// 64 rows its rows of B for the tile are fetched once (four adapters per round trip) and one
// MFMA pair per 16 columns and 32 ranks adds B[a] . t for every block of 16 rows that holds such
// a row, the rows of other adapters masked to zero.
// ------------------------------------------------------------------------------------------
constexpr int WIDE_TILES = 4;

// MB blocks of 16 rows per chunk: 4 (64 rows) from 33 rows on, 2 (32 rows) for 17 to 32 rows.
// A stage of x holds XSTEPS k-steps of every row of the chunk: one super-step (4 k-steps) at 64
// rows, two at 32 rows.
template <int MB>
struct WideLds {
    static constexpr int ROWS = 16 * MB;
    static constexpr int XSTEPS = MB == 2 ? 8 : 4;
    static constexpr int XROW = XSTEPS * 64 + 16;          // bytes of a row of x per stage; +16: rows 4 banks apart
    static constexpr int X_STAGE = ROWS * XROW;
    static constexpr int T_STRIDE = MLORA_MAX_RANK + 4;    // floats per row of t
    static constexpr int T_BYTES = ROWS * T_STRIDE * 4;
    static constexpr int BUF_BYTES = 2 * X_STAGE > T_BYTES ? 2 * X_STAGE : T_BYTES;
    alignas(16) unsigned char buf[BUF_BYTES];              // x stages; after the K loop: t
    alignas(16) float stage[WIDE_TILES][16 * (TILE_N + 4)]; // per wave: 16 rows of outputs on their way out
};

// eight fp32 -> the bf16 A-operand fragments of their high and low halves
__device__ __forceinline__ void split_bf16(const float (&v)[8], uint4 &hi, uint4 &lo)
{
    uint32_t h[8], l[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        h[i] = __float_as_uint(v[i]) & 0xFFFF0000u;
        l[i] = __float_as_uint(v[i] - __uint_as_float(h[i])) & 0xFFFF0000u;
    }
    hi = make_uint4((h[0] >> 16) | h[1], (h[2] >> 16) | h[3], (h[4] >> 16) | h[5], (h[6] >> 16) | h[7]);
    lo = make_uint4((l[0] >> 16) | l[1], (l[2] >> 16) | l[3], (l[4] >> 16) | l[5], (l[6] >> 16) | l[7]);
}

// ------------------------------------------------------------------------------------------
// The K loop of the wide blocks.  Per wave: the packed codes of the next 8 k-steps and their
// scales are in registers (8 KiB in flight), each register set requested again as soon as its
// k-step is consumed; the rows of x come through LDS in stages (8 k-steps of 32 rows, or 4
// k-steps of 64 rows: 16 KiB, double-buffered, one barrier per stage) shared by the block's four
// waves.  The codes enter the matrix units exactly; the scale multiplies the fp32 sum of a
// group with plain fp32 FMAs (the cheapest vector instructions on this chip: integer and mixed
// 16/32-bit operations issue at half their rate), so the loop is as short as the arithmetic
// allows: per k-step 28 integer operations to unpack, 16 * MB FMAs per scale group, 4 * MB + MB
// MFMAs.
// ------------------------------------------------------------------------------------------
template <int SPG, int MB>
__device__ __forceinline__ void stream_loop(f32x4 (&acc)[MB][4], const u32x4 *wp, const uint2 *sp,
                                            const unsigned char *const (&xrow)[4], int piece16, const int (&xdst)[4],
                                            unsigned char *lds_x, const unsigned char *xfrag, int n_ksteps,
                                            uint32_t mask, uint32_t bias)
{
    using L = WideLds<MB>;
    constexpr int S = L::XSTEPS;                           // k-steps per stage of x
    constexpr int W = 8;                                   // k-steps of codes in registers
    constexpr int HALVES = W / S;                          // stages per pass over the register sets
    static_assert(S % SPG == 0 && W % S == 0, "a stage holds whole scale groups; the sets hold whole stages");
    const u32x4 neg24 = {0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u};
    const int last = n_ksteps - 1;
    u32x4 w[W];
    uint2 sc[W / SPG];
    u32x4 xr[4];
    // (requests past the unit's end re-read its last k-step: all loads stay unconditional)
    const int x_last = n_ksteps * 64 - 16;                 // last 16-byte piece of a row inside the unit
#pragma unroll
    for (int i = 0; i < 4; ++i) xr[i] = *reinterpret_cast<const u32x4 *>(xrow[i] + min(piece16, x_last));
#pragma unroll
    for (int k = 0; k < W; ++k) {
        const int kc = min(k, last);
        w[k] = __builtin_nontemporal_load(wp + kc * 64);
        if (k % SPG == 0) sc[k / SPG] = sp[(kc / SPG) * 16];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4 *>(lds_x + xdst[i]) = xr[i];
    const int n_stages = (n_ksteps + S - 1) / S;

    // one stage: register sets [h * S, h * S + S), x buffer st & 1
    auto stage = [&](auto half, int st, auto full) {
        constexpr int H = decltype(half)::value;
        __syncthreads();                                   // this stage's rows of x are in place; the other buffer is free
        const int buf = (st & 1) * L::X_STAGE;
        const int x_off = min(min(st + 1, n_stages - 1) * S * 64 + piece16, x_last);
#pragma unroll
        for (int i = 0; i < 4; ++i) xr[i] = *reinterpret_cast<const u32x4 *>(xrow[i] + x_off);
        // the math of NK k-steps of this stage (NK = S, or 4 in the last stage of a unit that ends
        // on an odd super-step): one straight piece of code, no branches inside
        auto stage_math = [&](auto nk) {
            constexpr int NK = decltype(nk)::value;
            // A scale group is worked through in runs of SG = min(SPG, 2) k-steps: the run's
            // fragments of x stay in registers for the offset term and for all four column
            // blocks, and the products of one column block (MB accumulators of 16 x 16) are folded
            // into acc as soon as the run is done, so few registers live at a time.  A group of 4
            // k-steps is two runs that use the same scale.
            constexpr int SG = SPG < 2 ? SPG : 2;
#pragma unroll
            for (int r = 0; r < NK / SG; ++r) {
                u32x4 xk[SG][MB];
                // offset term of the run: -24 * sum of x over its inputs cancels the offset of the stored codes
                f32x4 corr[MB];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) corr[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < SG; ++t)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        xk[t][mb] = *reinterpret_cast<const u32x4 *>(xfrag + buf + mb * 16 * L::XROW + (r * SG + t) * 64);
                        corr[mb] = mfma16(__builtin_bit_cast(uint4, xk[t][mb]), __builtin_bit_cast(uint4, neg24), corr[mb]);
                    }
                constexpr int G0 = (H * S) / SPG;          // first scale group of this stage's register sets
                const int g = (r * SG) / SPG;              // scale group of the run within the stage
                const uint2 sv = sc[G0 + g];
                if ((r * SG + SG) % SPG == 0) {            // last run of its group: request the set's next group
                    const int gc = min(st * S + g * SPG + W, last) / SPG;
                    sc[G0 + g] = sp[gc * 16];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f32x4 d[MB];
#pragma unroll
                    for (int t = 0; t < SG; ++t) {
                        const uint4 wb = expand_codes(w[H * S + r * SG + t][j], mask, bias);
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb)
                            d[mb] = mfma16(__builtin_bit_cast(uint4, xk[t][mb]), wb, t == 0 ? corr[mb] : d[mb]);
                    }
                    float sj = j == 0 ? half_bits_lo(sv.x) : j == 1 ? half_bits_hi(sv.x)
                             : j == 2 ? half_bits_lo(sv.y) : half_bits_hi(sv.y);
                    asm volatile("" : "+v"(sj));           // a float in a register: plain fp32 FMAs below
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[mb][j][e] = fmaf(d[mb][e], sj, acc[mb][j][e]);
                }
                // the run's register sets are used up: request their next k-steps (after the last
                // use, so that no copy of the old contents has to be kept)
#pragma unroll
                for (int t = 0; t < SG; ++t) {
                    const int k = r * SG + t;              // k-step within the stage
                    const int kc = min(st * S + k + W, last);
                    w[H * S + k] = __builtin_nontemporal_load(wp + kc * 64);
                }
            }
        };
        // (a unit is a whole number of 4-k-step super-steps: a stage of 8 k-steps is full, or the
        // unit's last one with 4)
        if constexpr (decltype(full)::value) stage_math(std::integral_constant<int, S>{});
        else                                 stage_math(std::integral_constant<int, 4>{});
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4 *>(lds_x + (L::X_STAGE - buf) + xdst[i]) = xr[i];
    };
    // The loop holds full stages only; a last stage of 4 k-steps (S = 8) follows it.  One variant of
    // the stage inside the loop: the two would meet at the loop's end with their values in
    // different registers, and the moves that reconcile them were 5 % of the loop's instructions.
    constexpr std::true_type full_stage{};
    if constexpr (HALVES == 2) {
#pragma nounroll
        for (int st = 0; st < n_stages; st += 2) {
            stage(std::integral_constant<int, 0>{}, st, full_stage);
            if (st + 1 < n_stages) stage(std::integral_constant<int, 1>{}, st + 1, full_stage);
        }
    } else {
        const int n_full = n_ksteps / S;
#pragma nounroll
        for (int st = 0; st < n_full; ++st) stage(std::integral_constant<int, 0>{}, st, full_stage);
        if constexpr (S > 4) {
            if (n_full < n_stages) stage(std::integral_constant<int, 0>{}, n_full, std::false_type{});
        }
    }
}

// ------------------------------------------------------------------------------------------
// The same K loop for int8 activations (one scale per tensor): the matrix units multiply int8 by
// int8 into int32, so a scale group's sum is exact without any offset term.
//  * Codes: the blob stores offset-binary nibbles u = code + 8 at bits 3, 7, ... of a dword (see
//    common.hpp).  Flipping the top bit of every nibble turns them into two's complement, and a
//    nibble in the upper half of a byte is the int8 number 16 * code:  t = w ^ 0x44444444,
//    rotl(t, 1) & 0xF0F0F0F0 holds the codes of inputs 0, 4, 1, 5 of the lane's eight,
//    rotl(t, 5) & 0xF0F0F0F0 those of inputs 7, 2, 6, 3: five integer operations for 8 weights.
//    The factor 16 is taken out after the loop.
//  * x: the bytes of a row are put into that same order (0, 4, 1, 5, 7, 2, 6, 3 within every
//    eight) when a stage is written to LDS, so a lane's fragment is one 8-byte read.
//  * int32 -> fp32 without a conversion: the accumulator of a run starts at 0x4B400000, the bit
//    pattern of 1.5 * 2^23, so the int32 result, read as a float, is 12582912 + sum exactly
//    (|sum| <= 2 * 32 * 128 * 127 < 2^22); one fp32 subtraction and one FMA with the group's scale
//    follow, both at the full fp32 rate.
// A stage holds the same k-steps as in the bf16 loop; its rows are half as long.
// ------------------------------------------------------------------------------------------
template <int MB>
struct WideLdsA8 {
    static constexpr int XSTEPS = WideLds<MB>::XSTEPS;
    static constexpr int XROW = XSTEPS * 32 + 16;          // bytes of a row of x per stage (int8)
};

template <int SPG, int MB>
__device__ __forceinline__ void stream_loop_a8(f32x4 (&acc)[MB][4], const u32x4 *wp, const uint2 *sp,
                                               const unsigned char *const (&xrow)[2], int piece16, const int (&xdst)[2],
                                               unsigned char *lds_x, const unsigned char *xfrag, int n_ksteps)
{
    using L = WideLds<MB>;
    using L8 = WideLdsA8<MB>;
    constexpr int S = L::XSTEPS;
    constexpr int W = MB == 4 ? 4 : 8;                     // k-steps of codes in registers
    constexpr int HALVES = W / S;
    const int last = n_ksteps - 1;
    u32x4 w[W];
    uint2 sc[W / SPG];
    u32x4 xr[2];
    const int x_last = n_ksteps * 32 - 16;                 // last 16-byte piece of a row inside the unit
    // bytes (0,1,2,3 | 4,5,6,7) of every eight -> (0,4,1,5 | 7,2,6,3)
    auto shuffled = [](u32x4 v) {
        u32x4 o;
        o[0] = __builtin_amdgcn_perm(v[1], v[0], 0x05010400u);
        o[1] = __builtin_amdgcn_perm(v[1], v[0], 0x03060207u);
        o[2] = __builtin_amdgcn_perm(v[3], v[2], 0x05010400u);
        o[3] = __builtin_amdgcn_perm(v[3], v[2], 0x03060207u);
        return o;
    };
#pragma unroll
    for (int i = 0; i < 2; ++i) xr[i] = *reinterpret_cast<const u32x4 *>(xrow[i] + min(piece16, x_last));
#pragma unroll
    for (int k = 0; k < W; ++k) {
        const int kc = min(k, last);
        w[k] = __builtin_nontemporal_load(wp + kc * 64);
        if (k % SPG == 0) sc[k / SPG] = sp[(kc / SPG) * 16];
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) *reinterpret_cast<u32x4 *>(lds_x + xdst[i]) = shuffled(xr[i]);
    const int n_stages = (n_ksteps + S - 1) / S;
    const i32x4 magic = {0x4B400000, 0x4B400000, 0x4B400000, 0x4B400000};

    auto stage = [&](auto half, int st, auto full) {
        constexpr int H = decltype(half)::value;
        __syncthreads();
        const int buf = (st & 1) * L::X_STAGE;
        const int x_off = min(min(st + 1, n_stages - 1) * S * 32 + piece16, x_last);
#pragma unroll
        for (int i = 0; i < 2; ++i) xr[i] = *reinterpret_cast<const u32x4 *>(xrow[i] + x_off);
        auto stage_math = [&](auto nk) {
            constexpr int NK = decltype(nk)::value;
            constexpr int SG = SPG < 2 ? SPG : 2;
#pragma unroll
            for (int r = 0; r < NK / SG; ++r) {
                long xk[SG][MB];
#pragma unroll
                for (int t = 0; t < SG; ++t)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        xk[t][mb] = *reinterpret_cast<const long *>(xfrag + buf + mb * 16 * L8::XROW + (r * SG + t) * 32);
                u32x4 wv[SG];
#pragma unroll
                for (int t = 0; t < SG; ++t) {
                    const int k = r * SG + t;
                    wv[t] = w[H * S + k] ^ 0x44444444u;
                    const int kc = min(st * S + k + W, last);
                    w[H * S + k] = __builtin_nontemporal_load(wp + kc * 64);
                }
                constexpr int G0 = (H * S) / SPG;
                const int g = (r * SG) / SPG;
                const uint2 sv = sc[G0 + g];
                if ((r * SG + SG) % SPG == 0) {
                    const int gc = min(st * S + g * SPG + W, last) / SPG;
                    sc[G0 + g] = sp[gc * 16];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    i32x4 d[MB];
#pragma unroll
                    for (int t = 0; t < SG; ++t) {
                        const uint32_t v = wv[t][j];
                        const uint32_t hi = __builtin_amdgcn_alignbit(v, v, 31) & 0xF0F0F0F0u;
                        const uint32_t lo = __builtin_amdgcn_alignbit(v, v, 27) & 0xF0F0F0F0u;
                        const long wb = (long)(((unsigned long long)lo << 32) | hi);
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb) d[mb] = mfma16_i8(xk[t][mb], wb, t == 0 ? magic : d[mb]);
                    }
                    float sj = j == 0 ? half_bits_lo(sv.x) : j == 1 ? half_bits_hi(sv.x)
                             : j == 2 ? half_bits_lo(sv.y) : half_bits_hi(sv.y);
                    asm volatile("" : "+v"(sj));
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            acc[mb][j][e] = fmaf(__int_as_float(d[mb][e]) - 12582912.0f, sj, acc[mb][j][e]);
                }
            }
        };
        // (a unit is a whole number of 4-k-step super-steps: a stage of 8 k-steps is full, or the
        // unit's last one with 4)
        if constexpr (decltype(full)::value) stage_math(std::integral_constant<int, S>{});
        else                                 stage_math(std::integral_constant<int, 4>{});
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<u32x4 *>(lds_x + (L::X_STAGE - buf) + xdst[i]) = shuffled(xr[i]);
    };
    // The loop holds full stages only; a last stage of 4 k-steps (S = 8) follows it.  One variant of
    // the stage inside the loop: the two would meet at the loop's end with their values in
    // different registers, and the moves that reconcile them were 5 % of the loop's instructions.
    constexpr std::true_type full_stage{};
    if constexpr (HALVES == 2) {
#pragma nounroll
        for (int st = 0; st < n_stages; st += 2) {
            stage(std::integral_constant<int, 0>{}, st, full_stage);
            if (st + 1 < n_stages) stage(std::integral_constant<int, 1>{}, st + 1, full_stage);
        }
    } else {
        const int n_full = n_ksteps / S;
#pragma nounroll
        for (int st = 0; st < n_full; ++st) stage(std::integral_constant<int, 0>{}, st, full_stage);
        if constexpr (S > 4) {
            if (n_full < n_stages) stage(std::integral_constant<int, 0>{}, n_full, std::false_type{});
        }
    }
}

// group = index of the block's four tiles among the projection's; ku as in base_unit.  SPG =
// k-steps per scale group, the same for every projection of the launch; MB = blocks of 16 rows
// per chunk (2: calls of 17 to 32 rows, 4: 33 rows and more).
template <int SPG, int MB, bool A8>
__device__ __forceinline__ void wide_unit(const LayerArgs &a, const ProjArgs &P, int pi, int group, int ku,
                                          int m0, WideLds<MB> &lds)
{
    using L = WideLds<MB>;
    constexpr int ROWS = L::ROWS;
    const int K = P.K, N = P.N, M = a.M;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const int tiles = tiles_n(N);
    const int tile_raw = group * WIDE_TILES + wave;
    const bool tile_ok = tile_raw < tiles;                 // (uniform per wave; a spare wave computes and drops tile 0)
    const int tile = tile_ok ? tile_raw : 0;

    const int uq = P.unit_q, ur = P.unit_r;
    const int unit_beg = ku * uq + min(ku, ur), unit_cnt = uq + (ku < ur ? 1 : 0);
    const int ksteps = K / KSTEP;
    constexpr int gs = 4 / SPG;
    const u32x4 *wp = reinterpret_cast<const u32x4 *>(P.codes + (size_t)tile * ksteps * 64) + (size_t)unit_beg * 256;
    const uint2 *sp = P.scales + ((size_t)tile * (ksteps / SPG) + (size_t)unit_beg * gs) * 16;

    // Every K unit of a tile takes a share of the LoRA term (the adapters of the chunk are dealt
    // out to the units in turn): the rows of B of many adapters are more than the finishing
    // blocks alone can fetch in good time.  So every unit waits for the shrink blocks, and
    // P.n_finish_blocks counts (tile, chunk, unit) triples here.
    const bool lora = a.row_adapter != nullptr && P.n_adapters > 0;
    const int rows_here = min(ROWS, M - m0);
    const int chunk = m0 / ROWS, chunks = a.m_pad / ROWS;
    const int fin = tile * chunks + chunk;
    const int user = fin * P.ksplit + ku;
    const int copies = P.ctr_copies;
    unsigned *const sctr = a.ctrl + shrink_ctr(pi, user & (copies - 1));
    unsigned *const pctr = a.ctrl + P.part_ctr + fin * CTR_STRIDE;
    const bool need_s = lora, need_p = ku == 0 && P.ksplit > 1;

    const uint32_t mask = a.code_mask;
    uint32_t bias = a.code_bias;
    asm volatile("" : "+v"(bias));

    f32x4 acc[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[mb][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // rows of x: thread t moves, per stage, four 16-byte pieces: piece t % PPR of rows t / PPR + RPI * i
    // (PPR pieces per row and stage, RPI rows per instruction of the block); int8 rows are half as
    // long: two pieces per thread
    if constexpr (!A8) {
        constexpr int PPR = L::XSTEPS * 4, RPI = 256 / PPR;
        const unsigned char *xrow[4];
        int xdst[4];
        const int piece16 = (tid % PPR) * 16;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = tid / PPR + RPI * i;
            xrow[i] = reinterpret_cast<const unsigned char *>(P.x + (size_t)(m0 + min(row, rows_here - 1)) * K +
                                                              (size_t)unit_beg * SUPER_K);
            xdst[i] = row * L::XROW + piece16;
        }
        const unsigned char *xfrag = lds.buf + l16 * L::XROW + lq * 16;
        stream_loop<SPG, MB>(acc, wp + lane, sp + l16, xrow, piece16, xdst, lds.buf, xfrag, unit_cnt * 4, mask, bias);
    } else {
        using L8 = WideLdsA8<MB>;
        constexpr int PPR = L::XSTEPS * 2, RPI = 256 / PPR;
        const unsigned char *xrow[2];
        int xdst[2];
        const int piece16 = (tid % PPR) * 16;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = tid / PPR + RPI * i;
            xrow[i] = reinterpret_cast<const unsigned char *>(P.x) + (size_t)(m0 + min(row, rows_here - 1)) * K +
                      (size_t)unit_beg * SUPER_K;
            xdst[i] = row * L8::XROW + piece16;
        }
        const unsigned char *xfrag = lds.buf + l16 * L8::XROW + lq * 8;
        stream_loop_a8<SPG, MB>(acc, wp + lane, sp + l16, xrow, piece16, xdst, lds.buf, xfrag, unit_cnt * 4);
        // the codes went in as 16 * code, x as integers: one factor for both
        const float f = P.x_scale * 0.0625f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[mb][j] *= f;
    }

    // One pass per (32 ranks, adapter that occurs in the chunk): its rows of B for the
    // tile's 64 columns are fetched once and used by every block of 16 rows that holds
    // such a row.  Four passes are fetched per round trip: four adapters at ranks up to
    // 32, else two adapters x two runs of 32 ranks, so that a round takes whole 128-byte
    // pieces of the rows of B (the halves of a piece fetched in rounds far apart would
    // cost the memory two accesses).
    const int r32 = (P.r16 + 31) / 32 * 32;            // ranks as the MFMAs see them (zero-filled)
    const int n_lane = tile * TILE_N + l16;
    // lane l looks after row l of the chunk (a spare wave and a call without LoRA: no row)
    int ad_row = -1;
    if (lora && tile_ok && lane < rows_here) {
        const int v = a.row_adapter[m0 + lane];
        ad_row = (v >= 0 && v < P.n_adapters) ? v : -1;
    }
    const unsigned long long all = __ballot(ad_row >= 0);
    auto b_request = [&](u32x4 (&bf)[4], int cur, int kk) {
        const bool k_ok = 32 * kk + 8 * lq < P.rank;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = min(n_lane + 16 * j, N - 1);
            bf[j] = *reinterpret_cast<const u32x4 *>(P.lora_b + ((size_t)cur * N + n) * P.rank +
                                                     (k_ok ? 32 * kk + 8 * lq : 0));
        }
    };
    // The rounds form a two-deep pipeline: the rows of B of the next round are on their
    // way while the current round is computed.
    struct Round {
        int curs[4];
        unsigned long long sames[4];
        int kk0, nk;
        bool any;
    };
    const int nkk = r32 / 32;
    int st_kk0 = 0, st_ordinal = 0;                    // where the enumeration stands
    unsigned long long st_remaining = all;
    // skip the adapters that other K units of this tile look after
    auto skip_others = [&]() {
        while (st_remaining && st_ordinal % P.ksplit != ku) {
            const int other = __builtin_amdgcn_readlane(ad_row, (int)__builtin_ctzll(st_remaining));
            st_remaining &= ~__ballot(ad_row == other);
            ++st_ordinal;
        }
    };
    auto next_round = [&](Round &r) {
        skip_others();
        while (!st_remaining && st_kk0 + 2 < nkk) {    // next pair of runs of 32 ranks
            st_kk0 += 2;
            st_remaining = all;
            st_ordinal = 0;
            skip_others();
        }
        r.any = st_remaining != 0;
        r.kk0 = st_kk0;
        r.nk = min(2, nkk - st_kk0);                   // runs of 32 ranks per adapter and round
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            if (r.nk == 2 && (b & 1)) {                // second run of ranks of the same adapter
                r.curs[b] = r.curs[b - 1];
                r.sames[b] = r.sames[b - 1];
                continue;
            }
            skip_others();
            if (st_remaining) {
                r.curs[b] = __builtin_amdgcn_readlane(ad_row, (int)__builtin_ctzll(st_remaining));
                r.sames[b] = __ballot(ad_row == r.curs[b]);
                st_remaining &= ~r.sames[b];
                ++st_ordinal;
            } else {
                r.curs[b] = b ? r.curs[0] : 0;         // (a useless request that stays in bounds)
                r.sames[b] = 0;
            }
        }
    };
    auto request = [&](u32x4 (&bf)[4][4], const Round &r) {
#pragma unroll
        for (int b = 0; b < 4; ++b) b_request(bf[b], r.curs[b], r.kk0 + (r.nk == 2 ? (b & 1) : 0));
    };
    // The first round's rows of B do not depend on t: they are requested before the wait for
    // the shrink blocks and arrive while t is gathered.
    Round ra_, rb_;
    u32x4 bfa[4][4], bfb[4][4];
    ra_.any = false;
    if (lora && tile_ok) {
        next_round(ra_);
        if (ra_.any) request(bfa, ra_);
    }

    // element (mb, j, e) of this lane: row 16*mb + 4*lq + e of the chunk, column 16*j + l16 of the tile
    // (a wave whose wait runs out sets the status word and stores NaN in place of its outputs)
    bool poisoned = false;
    if (tile_ok && need_s && !wait_count(sctr, (unsigned)P.n_shrink_blocks, a.spin_limit)) {
        poisoned = true;
        if (lane == 0) atomicOr(a.status, 1u);
    }
    if (lora) {                                            // (uniform over the block)
        // a spare wave has not looked at the shrink counter: it must, before it reads t
        if (!tile_ok && !wait_count(sctr, (unsigned)P.n_shrink_blocks, a.spin_limit) && lane == 0) atomicOr(a.status, 1u);
        __syncthreads();                                   // every wave is done with the x buffers
        float *tl = reinterpret_cast<float *>(lds.buf);
        // t = alpha * sum over the K chunks of the shrink partials, in fixed order.  A thread takes
        // four neighbouring ranks (16 bytes) at a time; requests go out in batches of 4 such
        // quads x 4 chunks so that the round trips overlap.
        const int qpr = r32 / 4;                           // quads per row of t
        const float t_factor = A8 ? P.alpha * P.x_scale : P.alpha;   // (the shrink blocks saw x as integers)
        for (int i0 = 0; i0 < ROWS * qpr; i0 += 4 * 256) {
            f32x4_t v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            for (int kc0 = 0; kc0 < P.kch; kc0 += 4) {
                f32x4_t pv[16];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = i0 + q * 256 + tid;
                    const int ml = idx / qpr, jj = (idx % qpr) * 4;
                    const bool live = ml < rows_here && jj < P.r16;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int kc = min(kc0 + c, P.kch - 1);
                        const float *src = live ? P.t_part + ((size_t)kc * M + (m0 + ml)) * P.r16 + jj : P.t_part;
                        pv[q * 4 + c] = load_shared16(src);
                    }
                }
                shared16_wait(pv);
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (kc0 + c < P.kch) v[q] += pv[q * 4 + c];
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int idx = i0 + q * 256 + tid;
                const int ml = idx / qpr, jj = (idx % qpr) * 4;
                const bool live = ml < rows_here && jj < P.r16;
                if (ml < ROWS)
                    *reinterpret_cast<f32x4_t *>(tl + ml * L::T_STRIDE + jj) = live ? v[q] * t_factor : f32x4_t{0.f, 0.f, 0.f, 0.f};
            }
        }
        __syncthreads();
        if (tile_ok) {
            auto compute = [&](const u32x4 (&bf)[4][4], const Round &r) {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    if (!r.sames[b]) continue;
                    const int kk = r.kk0 + (r.nk == 2 ? (b & 1) : 0);
                    const bool k_ok = 32 * kk + 8 * lq < P.rank;
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        if (!((r.sames[b] >> (16 * mb)) & 0xFFFFull)) continue;
                        // (a lane whose ranks lie past the adapter's takes zeros of t: its part of
                        // B, a re-read of the first ranks, then needs no masking of its own)
                        const bool mine = k_ok && ((r.sames[b] >> (16 * mb + l16)) & 1ull);
                        float tv[8];
                        // (16-byte aligned: rows of t are 528 bytes apart, a lane's run starts at a multiple of 32)
                        const f32x4_t *trow = reinterpret_cast<const f32x4_t *>(tl + (16 * mb + l16) * L::T_STRIDE + 32 * kk + 8 * lq);
                        const f32x4_t t0 = trow[0], t1 = trow[1];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            tv[i] = mine ? t0[i] : 0.f;
                            tv[4 + i] = mine ? t1[i] : 0.f;
                        }
                        uint4 thi, tlo;
                        split_bf16(tv, thi, tlo);
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const uint4 b4 = __builtin_bit_cast(uint4, bf[b][j]);
                            acc[mb][j] = mfma16(thi, b4, acc[mb][j]);
                            acc[mb][j] = mfma16(tlo, b4, acc[mb][j]);
                        }
                    }
                }
            };
            while (ra_.any) {
                next_round(rb_);
                if (rb_.any) request(bfb, rb_);
                compute(bfa, ra_);
                if (!rb_.any) break;
                next_round(ra_);
                if (ra_.any) request(bfa, ra_);
                compute(bfb, rb_);
            }
        }
    }
    if (ku > 0) {
        // A partial tile (the chunk's rows x 64 columns) lies in the workspace in the order of the
        // MFMA results, block (mb, j) of lane l at ((mb * 4 + j) * 64 + l) * 4: producer and consumer
        // use the same mapping, and a lane moves 16 bytes per instruction.
        if (tile_ok) {
            float *dst = P.partial + (((size_t)(ku - 1) * tiles + tile) * a.m_pad + m0) * TILE_N + lane * 4;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int j = 0; j < 4; ++j) store_shared16(dst + (mb * 4 + j) * 256, acc[mb][j]);
            compiler_fence();
            __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wave's stores have completed
            if (lane == 0) atomicAdd(pctr, 1u);
        }
    } else if (tile_ok && need_p) {
        if (!wait_count(pctr, (unsigned)(P.ksplit - 1), a.spin_limit)) {
            poisoned = true;
            if (lane == 0) atomicOr(a.status, 1u);
        }
        // The other units' partial tiles, added in the order of the units.  Two sets of registers:
        // a unit's tile is added while the next one is on its way (a projection with a long K has
        // a dozen of them, and one round trip after another was most of its finishing block's time).
        // These are loads the compiler sees (it places the waits): values it does not know to be
        // in flight must not stay in registers across other code, which it may spill or reuse.
        constexpr int NP = 4 * MB;
        const int np = P.ksplit - 1;
        auto request = [&](f32x4_t (&pv)[NP], int u) {
            // (the tile of unit u for this wave's chunk: NP KiB, the same place for all lanes)
            const float *base = P.partial + (((size_t)u * tiles + tile) * a.m_pad + m0) * TILE_N;
            const __amdgpu_buffer_rsrc_t rsrc = shared_buffer(base, NP * 1024);
#pragma unroll
            for (int i = 0; i < NP; ++i) pv[i] = load_shared16(rsrc, lane * 16 + i * 1024);
        };
        auto fold = [&](const f32x4_t (&pv)[NP]) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[mb][j] += pv[mb * 4 + j];
        };
        f32x4_t pa[NP], pb[NP];
        if (np > 0) request(pa, 0);
        for (int u = 0; u < np; u += 2) {
            if (u + 1 < np) request(pb, u + 1);
            fold(pa);
            if (u + 1 < np) {
                if (u + 2 < np) request(pa, u + 2);
                fold(pb);
            }
        }
    }
    if (poisoned) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[mb][j] = f32x4{1.f, 1.f, 1.f, 1.f} * __uint_as_float(0x7FC00000u);
    }
    if (tile_ok && ku == 0 && a.fused) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float vv[4] = {acc[mb][0][e], acc[mb][1][e], acc[mb][2][e], acc[mb][3][e]};
                store_fused(a, P, pi, m0 + 16 * mb + 4 * lq + e, tile, l16, vv);
            }
    } else if (tile_ok && ku == 0) {
        const bool full = tile * TILE_N + TILE_N <= N;
        if (full) {
            // rows of 64 outputs through a wave-private LDS buffer, so that a lane stores 16
            // neighbouring columns at once instead of 64 single values
            float *st = lds.stage[wave];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int j = 0; j < 4; ++j) st[(4 * lq + e) * (TILE_N + 4) + 16 * j + l16] = acc[mb][j][e];
                const int row = lane >> 2, c0 = (lane & 3) * 16;
                const int m = m0 + 16 * mb + row;
                const f32x4 *src = reinterpret_cast<const f32x4 *>(st + row * (TILE_N + 4) + c0);
                f32x4 o[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) o[q] = src[q];
                if (m < M) {
                    const size_t at = (size_t)m * N + tile * TILE_N + c0;
                    if (a.y_fp32) {
                        f32x4 *dst = reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(P.y) + at);
#pragma unroll
                        for (int q = 0; q < 4; ++q) dst[q] = o[q];
                    } else {
                        u32x4 pk[2];
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const uint32_t lo2 = float_to_bf16_bits(o[q][0]) | ((uint32_t)float_to_bf16_bits(o[q][1]) << 16);
                            const uint32_t hi2 = float_to_bf16_bits(o[q][2]) | ((uint32_t)float_to_bf16_bits(o[q][3]) << 16);
                            pk[q >> 1][(q & 1) * 2] = lo2;
                            pk[q >> 1][(q & 1) * 2 + 1] = hi2;
                        }
                        u32x4 *dst = reinterpret_cast<u32x4 *>(reinterpret_cast<uint16_t *>(P.y) + at);
                        dst[0] = pk[0];
                        dst[1] = pk[1];
                    }
                }
            }
        } else {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int m = m0 + 16 * mb + 4 * lq + e;
                    if (m >= M) continue;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int n = tile * TILE_N + 16 * j + l16;
                        if (n >= N) continue;
                        if (a.y_fp32) reinterpret_cast<float *>(P.y)[(size_t)m * N + n] = acc[mb][j][e];
                        else reinterpret_cast<uint16_t *>(P.y)[(size_t)m * N + n] = float_to_bf16_bits(acc[mb][j][e]);
                    }
                }
        }
    }

    // counters back to zero for the next call (every wave owns the counters of its tile)
    if (tile_ok && lane == 0) {
        if (need_p) __hip_atomic_store(pctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (need_s) {
            const int users = (P.n_finish_blocks >> (31 - __clz(copies))) + ((user & (copies - 1)) < (P.n_finish_blocks & (copies - 1)) ? 1 : 0);
            if (atomicAdd(sctr + 1, 1u) + 1u == (unsigned)users) {
                __hip_atomic_store(sctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(sctr + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

template <int MB>
constexpr int wide_lds_bytes()
{
    return sizeof(WideLds<MB>) > sizeof(ShrinkLds) ? (int)sizeof(WideLds<MB>) : (int)sizeof(ShrinkLds);
}

template <int SPG, int MB, bool A8>
__global__ __launch_bounds__(256, 2) void wide_kernel(const LayerArgs a)
{
    __shared__ __align__(16) unsigned char smem[wide_lds_bytes<MB>()];
    const int z = (int)blockIdx.z;
    const LaunchTables tables = pin_launch_args(a, z);
    int b, chunk;
    split_block_index(a, 16 * MB, b, chunk);
    if (b >= tables.group_blocks) return;
    int first;
    if (b < tables.shrink_blocks) {
        if (chunk != 0) return;
        const int pi = z * GROUP_PROJ + find_proj(tables.shrink, b, first);
        shrink_block<A8>(a, fetch_proj(a, pi), pi, b - first, *reinterpret_cast<ShrinkLds *>(smem));
        return;
    }
    WideLds<MB> &lds = *reinterpret_cast<WideLds<MB> *>(smem);
    const int m0 = chunk * 16 * MB;
    if (b < tables.shrink_blocks + tables.pre_base_blocks) {
        const int pb = b - tables.shrink_blocks;
        const int pi = z * GROUP_PROJ + find_proj(tables.pre, pb, first);
        const ProjArgs P = fetch_proj(a, pi);
        const int local = pb - first;
        const int groups = (tiles_n(P.N) + WIDE_TILES - 1) / WIDE_TILES;
        wide_unit<SPG, MB, A8>(a, P, pi, local % groups, 1 + local / groups, m0, lds);
    } else {
        const int mb_ = b - tables.shrink_blocks - tables.pre_base_blocks;
        const int pi = z * GROUP_PROJ + find_proj(tables.main, mb_, first);
        const ProjArgs P = fetch_proj(a, pi);
        wide_unit<SPG, MB, A8>(a, P, pi, mb_ - first, 0, m0, lds);
    }
}

template <int MB, int XR>
static hipError_t launch_instance(const LayerArgs &a, const dim3 &grid, hipStream_t s)
{
    layer_kernel<MB, XR><<<grid, dim3(64 * Shape<MB>::WAVES), 0, s>>>(a);
    return hipGetLastError();
}

// grid: x = the longest group's blocks x row chunks (see split_block_index), z = groups of up to 16 projections
hipError_t launch_layer(const LayerArgs &a, int grid_x, int groups, hipStream_t s)
{
    const int n_chunks = a.m_pad / rows_per_chunk(a.M_plan);
    // (several chunks: runs of 8 blocks, see split_block_index; blocks past a group's last one exit at once)
    const long long gx = n_chunks == 1 ? grid_x : (long long)((grid_x + 7) / 8 * 8) * n_chunks;
    if (gx > 0x7FFFFFFFll) return hipErrorInvalidValue;
    const dim3 grid((unsigned)gx, 1u, (unsigned)groups);
    if (a.wide) {
        // (the host puts only projections with the same group size into one such launch)
        const int spg = a.p[0].spg;
        auto go = [&](auto kernel) { kernel<<<grid, dim3(256), 0, s>>>(a); };
        if (a.a8) {
            if (a.M_plan <= 32) {
                if (spg == 1)      go(wide_kernel<1, 2, true>);
                else if (spg == 2) go(wide_kernel<2, 2, true>);
                else               go(wide_kernel<4, 2, true>);
            } else {
                if (spg == 1)      go(wide_kernel<1, 4, true>);
                else if (spg == 2) go(wide_kernel<2, 4, true>);
                else               go(wide_kernel<4, 4, true>);
            }
        } else if (a.M_plan <= 32) {
            if (spg == 1)      go(wide_kernel<1, 2, false>);
            else if (spg == 2) go(wide_kernel<2, 2, false>);
            else               go(wide_kernel<4, 2, false>);
        } else {
            if (spg == 1)      go(wide_kernel<1, 4, false>);
            else if (spg == 2) go(wide_kernel<2, 4, false>);
            else               go(wide_kernel<4, 4, false>);
        }
        return hipGetLastError();
    }
    // (M_plan, not M: a short launch of 17 to 32 rows is laid out as chunks of 16 rows, and the
    // kernel has to be the one the host laid the grid, the shrink blocks and the counters out for)
    const int rows = rows_per_chunk(a.M_plan);
    if (a.m_pad % rows != 0 || n_chunks * rows < a.M) return hipErrorInvalidValue;
    if (rows == 16) return a.M <= 8 ? launch_instance<1, 8>(a, grid, s) : launch_instance<1, 16>(a, grid, s);
    if (a.M <= 24) return launch_instance<2, 24>(a, grid, s);
    return launch_instance<2, 32>(a, grid, s);
}

__global__ void zero_kernel(uint4 *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = make_uint4(0, 0, 0, 0);
}

hipError_t launch_zero(void *p, size_t bytes, hipStream_t s)
{
    const size_t n = bytes / 16;
    if (n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    zero_kernel<<<dim3(blocks), dim3(256), 0, s>>>(reinterpret_cast<uint4 *>(p), n);
    return hipGetLastError();
}

}  // namespace mlora
