// C ABI of the mlora_w4 library: host-side validation, launch planning, no device allocation.
#include <string.h>

#include "common.hpp"

using namespace mlora;

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

mlora_status check_weight_shape(int K, int N, int group)
{
    if (group != 32 && group != 64 && group != 128) return MLORA_ESHAPE;
    if (K <= 0 || N <= 0 || K % SUPER_K != 0) return MLORA_ESHAPE;
    if ((long long)N > (1ll << 24) || (long long)K > (1ll << 24)) return MLORA_ESHAPE;
    return MLORA_OK;
}

mlora_status check_proj(const mlora_w4_proj &p)
{
    mlora_status st = check_weight_shape(p.K, p.N, p.group);
    if (st != MLORA_OK) return st;
    if (!p.w_blob) return MLORA_EINVAL;
    if (!aligned16(p.w_blob)) return MLORA_EALIGN;
    if (p.n_adapters < 0 || p.n_adapters > MLORA_MAX_ADAPTERS) return MLORA_ESHAPE;
    if (p.n_adapters > 0) {
        if (p.rank <= 0 || p.rank > MLORA_MAX_RANK || p.rank % 8 != 0) return MLORA_ESHAPE;
        if (!p.lora_a || !p.lora_b) return MLORA_EINVAL;
        if (!aligned16(p.lora_a) || !aligned16(p.lora_b)) return MLORA_EALIGN;
    }
    return MLORA_OK;
}

int r16_of(const mlora_w4_proj &p) { return p.n_adapters > 0 ? (p.rank + 15) / 16 * 16 : 0; }
// K chunks of the shrink step (at most MAX_KCHUNKS).  Decode shapes: 1024 inputs per chunk, split
// over the four waves of a block (8 k-steps each, requested at once).  More than 16 rows: a wave
// works through a chunk on its own for every row tile it is dealt; measured best with 512 inputs
// per chunk up to 32 rows (the finishing blocks need t early there) and 1024 in the wide kernel
// (fewer partial sums for every finishing block to gather).
int kch_of(const mlora_w4_proj &p, int M)
{
    const int c = p.K / ((M > 16 && M < WIDE_MIN_ROWS) ? 512 : 1024);
    return c < 1 ? 1 : (c > MAX_KCHUNKS ? MAX_KCHUNKS : c);
}
size_t t_part_bytes(const mlora_w4_proj &p, int M)
{
    return round_up((size_t)kch_of(p, M) * (size_t)M * (size_t)r16_of(p) * sizeof(float), 256);
}

int m_pad_of(int M) { return (M + rows_per_chunk(M) - 1) / rows_per_chunk(M) * rows_per_chunk(M); }

// K units per column tile.  Decode kernels: units of at most 2048 inputs (16 super-steps: what a
// block stages of x).  Wide kernel (33 rows and more): any unit length works.  A launch whose
// base blocks with such units (`launch_blocks`) would leave most compute units idle gets shorter
// units, the same length for all its projections: 8 super-steps up to 240 blocks, 4 below 80.
// Measured on single projections and on whole layers: up to 64 rows about 200 to 250 base
// blocks (one per compute unit with the shrink blocks) beat both fewer and more; a layer of 128
// rows (232 blocks) gains a quarter from 464 shorter ones, two per compute unit; from 256 rows on
// (464 blocks and more) the long units win, and not splitting long projections at all is far
// worse at any size (their blocks finish last).
int ksplit_of(const mlora_w4_proj &p, int M, int launch_blocks)
{
    const int nss = p.K / SUPER_K;
    int ks = (nss + UNIT_SUPER_STEPS - 1) / UNIT_SUPER_STEPS;
    if (M >= WIDE_MIN_ROWS && launch_blocks > 0 && launch_blocks <= 240) {
        const int unit = launch_blocks < 80 ? 4 : 8;
        const int cut = (nss + unit / 2) / unit;
        if (cut > ks) ks = cut;
    }
    return ks;
}
// base blocks of a launch over `count` projections with the default K units
int launch_blocks_of(const mlora_w4_proj *projs, int count, int M)
{
    int n = 0;
    const int chunks = m_pad_of(M) / rows_per_chunk(M);
    for (int i = 0; i < count; ++i) {
        const int nss = projs[i].K / SUPER_K;
        n += (tiles_n(projs[i].N) + tiles_per_block(M) - 1) / tiles_per_block(M) * chunks *
             ((nss + UNIT_SUPER_STEPS - 1) / UNIT_SUPER_STEPS);
    }
    return n;
}
size_t partial_bytes(const mlora_w4_proj &p, int M, int launch_blocks)
{
    return (size_t)(ksplit_of(p, M, launch_blocks) - 1) * (size_t)tiles_n(p.N) * (size_t)m_pad_of(M) * TILE_N * sizeof(float);
}

}  // namespace

extern "C" {

const char *mlora_strerror(mlora_status status)
{
    switch (status) {
    case MLORA_OK: return "ok";
    case MLORA_EINVAL: return "invalid argument (null pointer, bad enum or count)";
    case MLORA_ESHAPE: return "unsupported shape (K % 128, group in {32,64,128}, rank % 8, limits)";
    case MLORA_EALIGN: return "pointer not 16-byte aligned";
    case MLORA_EWORKSPACE: return "workspace missing or too small";
    case MLORA_EUNSUPPORTED: return "not implemented in this build";
    case MLORA_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

size_t mlora_w4_blob_bytes(int32_t K, int32_t N, int32_t group)
{
    if (check_weight_shape(K, N, group) != MLORA_OK) return 0;
    return blob_code_bytes(K, N) + blob_scale_bytes(K, N, group) + BLOB_SLACK_BYTES;
}

mlora_status mlora_w4_prepack(int32_t K, int32_t N, int32_t group, const uint8_t *wq,
                              const uint16_t *scales_f16, void *w_blob, void *stream)
{
    mlora_status st = check_weight_shape(K, N, group);
    if (st != MLORA_OK) return st;
    if (!wq || !scales_f16 || !w_blob) return MLORA_EINVAL;
    if (!aligned16(wq) || !aligned16(scales_f16) || !aligned16(w_blob)) return MLORA_EALIGN;
    return launch_prepack(K, N, group, wq, scales_f16, w_blob, (hipStream_t)stream) == hipSuccess
               ? MLORA_OK : MLORA_EHIP;
}

mlora_status mlora_w4_unpack(const mlora_w4_proj *p, int8_t *codes, float *w_f32, void *stream)
{
    if (!p) return MLORA_EINVAL;
    mlora_status st = check_weight_shape(p->K, p->N, p->group);
    if (st != MLORA_OK) return st;
    if (!p->w_blob || (!codes && !w_f32)) return MLORA_EINVAL;
    if (!aligned16(p->w_blob)) return MLORA_EALIGN;
    return launch_unpack(p->K, p->N, p->group, p->w_blob, codes, w_f32, (hipStream_t)stream) == hipSuccess
               ? MLORA_OK : MLORA_EHIP;
}

mlora_status mlora_group_rows(const int32_t *row_adapter, int32_t M, int32_t n_adapters,
                              int32_t *perm, int32_t *seg_adapter, int32_t *seg_start,
                              int32_t *n_seg, void *stream)
{
    if (!perm || !seg_adapter || !seg_start || !n_seg) return MLORA_EINVAL;
    if (M < 0 || M > MLORA_MAX_ROWS || n_adapters < 1 || n_adapters > MLORA_MAX_ADAPTERS)
        return MLORA_ESHAPE;
    if (M > 0 && !row_adapter) return MLORA_EINVAL;
    return launch_group_rows(row_adapter, M, n_adapters, perm, seg_adapter, seg_start, n_seg,
                             (hipStream_t)stream) == hipSuccess ? MLORA_OK : MLORA_EHIP;
}

// Projections of one launch: up to 16, and for the wide kernel (33 rows and more, compiled per
// group size) only as long as the group size stays the same.
static int launch_run(const mlora_w4_proj *projs, int n_left, int M)
{
    int count = 1;
    while (count < n_left && count < MAX_PROJ_PER_LAUNCH &&
           (M < WIDE_MIN_ROWS || projs[count].group == projs[0].group))
        ++count;
    return count;
}

// Workspace layout: [status word, 256 B][counters of launch 0][counters of launch 1]...[data].
// Counters exist only if something is shared between blocks (LoRA or split-K).
static size_t ctrl_bytes_of_launch(const mlora_w4_proj *projs, int count, int M, bool lora)
{
    size_t n = 0;                              // counter lines of the split-K tiles
    bool any = false;
    for (int i = 0; i < count; ++i) {
        if (ksplit_of(projs[i], M, launch_blocks_of(projs, count, M)) > 1) {
            n += (size_t)tiles_n(projs[i].N) * (size_t)(m_pad_of(M) / rows_per_chunk(M));
            any = true;
        }
        any = any || (lora && projs[i].n_adapters > 0);
    }
    return any ? (CTRL_PART + n * CTR_STRIDE) * sizeof(unsigned) : 0;
}

static size_t ctrl_bytes_total(const mlora_w4_proj *projs, int n_proj, int M, bool lora)
{
    size_t total = 0;
    for (int first = 0, count = 0; first < n_proj; first += count) {
        count = launch_run(projs + first, n_proj - first, M);
        total += ctrl_bytes_of_launch(projs + first, count, M, lora);
    }
    return total ? total + WS_HEADER_BYTES : 0;
}

size_t mlora_w4_workspace_bytes(const mlora_w4_proj *projs, int32_t n_proj, int32_t M)
{
    if (!projs || n_proj <= 0 || M <= 0) return 0;
    size_t total = ctrl_bytes_total(projs, n_proj, M, true);
    for (int first = 0, count = 0; first < n_proj; first += count) {
        count = launch_run(projs + first, n_proj - first, M);
        const int lb = launch_blocks_of(projs + first, count, M);
        for (int i = first; i < first + count; ++i) total += t_part_bytes(projs[i], M) + partial_bytes(projs[i], M, lb);
    }
    return total;
}

mlora_status mlora_w4_workspace_init(void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace) return workspace_bytes == 0 ? MLORA_OK : MLORA_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MLORA_EALIGN;
    return launch_zero(workspace, workspace_bytes / 16 * 16, (hipStream_t)stream) == hipSuccess
               ? MLORA_OK : MLORA_EHIP;
}

mlora_status mlora_w4_layer_step(const mlora_w4_proj *projs, int32_t n_proj,
                                 const void *const *xs, void *const *ys,
                                 const int32_t *row_adapter, int32_t M, int32_t y_dtype,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!projs || !xs || !ys || n_proj <= 0) return MLORA_EINVAL;
    if (y_dtype != MLORA_Y_BF16 && y_dtype != MLORA_Y_FP32) return MLORA_EINVAL;
    if (M < 0 || M > MLORA_MAX_ROWS) return MLORA_ESHAPE;
    bool any_lora = false;
    for (int i = 0; i < n_proj; ++i) {
        mlora_status st = check_proj(projs[i]);
        if (st != MLORA_OK) return st;
        if (!xs[i] || !ys[i]) return MLORA_EINVAL;
        if (!aligned16(xs[i]) || !aligned16(ys[i])) return MLORA_EALIGN;
        for (int j = 0; j < i; ++j)
            if (ys[j] == ys[i]) return MLORA_EINVAL;
        any_lora = any_lora || projs[i].n_adapters > 0;
    }
    if (M == 0) return MLORA_OK;
    any_lora = any_lora && row_adapter != nullptr;
    if (row_adapter && (reinterpret_cast<uintptr_t>(row_adapter) & 3u)) return MLORA_EALIGN;
    const size_t need = mlora_w4_workspace_bytes(projs, n_proj, M);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return MLORA_EWORKSPACE;
        if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MLORA_EALIGN;
    }

    hipStream_t s = (hipStream_t)stream;
    char *ctrl = reinterpret_cast<char *>(workspace) + WS_HEADER_BYTES;
    char *ws = reinterpret_cast<char *>(workspace) + ctrl_bytes_total(projs, n_proj, M, true);
    const int chunks = m_pad_of(M) / rows_per_chunk(M);
    for (int first = 0, count = 0; first < n_proj; first += count) {
        count = launch_run(projs + first, n_proj - first, M);
        LayerArgs a;
        memset(&a, 0, sizeof a);
        a.row_adapter = any_lora ? row_adapter : nullptr;
        a.n_proj = count;
        a.M = M;
        a.y_fp32 = (y_dtype == MLORA_Y_FP32);
        for (int i = 0; i < MAX_PROJ_PER_LAUNCH; ++i)
            a.main_begin[i] = a.pre_begin[i] = a.shrink_begin[i] = 0x7FFFFFFF;
        a.m_pad = m_pad_of(M);
        a.code_mask = 0x00780078u;
        a.code_bias = 0x41804180u;
        if (need > 0) {
            a.status = reinterpret_cast<unsigned *>(workspace);
            a.ctrl = reinterpret_cast<unsigned *>(ctrl);
            ctrl += ctrl_bytes_of_launch(projs + first, count, M, true);
        }
        const int lb = launch_blocks_of(projs + first, count, M);
        int main_blocks = 0, pre_blocks = 0, shrink_blocks = 0, part_ctr = CTRL_PART;
        for (int i = 0; i < count; ++i) {
            const mlora_w4_proj &p = projs[first + i];
            ProjArgs &d = a.p[i];
            d.codes = reinterpret_cast<const uint4 *>(p.w_blob);
            d.scales = reinterpret_cast<const uint2 *>(reinterpret_cast<const char *>(p.w_blob) +
                                                       blob_code_bytes(p.K, p.N));
            d.x = reinterpret_cast<const uint16_t *>(xs[first + i]);
            d.y = ys[first + i];
            d.K = p.K;
            d.N = p.N;
            d.spg = p.group / KSTEP;
            d.alpha = p.alpha;
            d.ksplit = ksplit_of(p, M, lb);
            // blocks (wide kernel: waves) that wait for this projection's shrink blocks: the
            // finishing ones, or every K unit where the LoRA term is spread over them
            d.n_finish_blocks = tiles_n(p.N) * chunks * (M >= WIDE_MIN_ROWS ? d.ksplit : 1);
            d.unit_q = (p.K / SUPER_K) / d.ksplit;
            d.unit_r = (p.K / SUPER_K) % d.ksplit;
            d.spg_shift = d.spg == 4 ? 2 : d.spg == 2 ? 1 : 0;
            d.ctr_copies = 1;
            while (d.ctr_copies * 2 <= CTR_REPL && d.ctr_copies * 2 <= d.n_finish_blocks) d.ctr_copies *= 2;
            d.tiles_inv = (unsigned)((0x100000000ull + (unsigned)tiles_n(p.N) - 1) / (unsigned)tiles_n(p.N));
            // (the division by multiplication is exact while index * tiles < 2^32: a projection
            // with more than 2^15 column tiles and K units to match is refused rather than mis-indexed)
            if ((unsigned long long)tiles_n(p.N) * (unsigned long long)tiles_n(p.N) * (unsigned long long)d.ksplit >=
                0x100000000ull)
                return MLORA_ESHAPE;
            // base blocks: one per column tile, or per four of them in the wide kernel
            const int col_blocks = (tiles_n(p.N) + tiles_per_block(M) - 1) / tiles_per_block(M);
            a.main_begin[i] = main_blocks;
            main_blocks += col_blocks;
            a.pre_begin[i] = pre_blocks;
            pre_blocks += col_blocks * (d.ksplit - 1);
            d.partial = reinterpret_cast<float *>(ws);
            ws += partial_bytes(p, M, lb);
            d.part_ctr = part_ctr;
            if (d.ksplit > 1) part_ctr += tiles_n(p.N) * chunks * CTR_STRIDE;
            a.shrink_begin[i] = shrink_blocks;
            if (any_lora && p.n_adapters > 0) {
                d.lora_a = reinterpret_cast<const uint16_t *>(p.lora_a);
                d.lora_b = reinterpret_cast<const uint16_t *>(p.lora_b);
                d.n_adapters = p.n_adapters;
                d.rank = p.rank;
                d.r16 = r16_of(p);
                d.kch = kch_of(p, M);
                d.t_part = reinterpret_cast<float *>(ws);
                ws += t_part_bytes(p, M);
                // at most 16 rows: a shrink block per row; above: per 16-row tile of an adapter segment
                d.n_shrink_blocks = (M <= 16 ? M : (M + SHRINK_CHUNK_ROWS - 1) / SHRINK_CHUNK_ROWS *
                                                          shrink_tile_shares(M, p.n_adapters)) *
                                    (d.r16 / 16) * d.kch;
                shrink_blocks += d.n_shrink_blocks;
            } else {
                d.n_adapters = 0;
                d.rank = 0;
                d.r16 = 16;
                d.kch = 1;
            }
        }
        a.shrink_blocks = shrink_blocks;
        a.pre_base_blocks = pre_blocks;
        if (launch_layer(a, shrink_blocks + pre_blocks + main_blocks, s) != hipSuccess) return MLORA_EHIP;
    }
    return MLORA_OK;
}

mlora_status mlora_w4_linear(const mlora_w4_proj *p, const void *x, const int32_t *row_adapter,
                             int32_t M, void *y, int32_t y_dtype, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    if (!p) return MLORA_EINVAL;
    const void *xs[1] = {x};
    void *ys[1] = {y};
    return mlora_w4_layer_step(p, 1, xs, ys, row_adapter, M, y_dtype, workspace, workspace_bytes,
                               stream);
}

}  // extern "C"
