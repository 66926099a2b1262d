// C ABI of the mlora_w4 library: host-side validation, launch planning, no device allocation.
#include <string.h>

#include <cmath>
#include <algorithm>
#include <memory>
#include <mutex>
#include <vector>

#include "common.hpp"

using namespace mlora;

// ---------------------------------------------------------------------------------------------
// The same call on a scratch buffer that lives in the library's own device image, for callers
// that cannot allocate.  Every device the library runs on holds its own copy of the array at
// its own address; in host code the array's name is only a handle, so the device address is
// looked up once per device (with that device current) and used from then on.
// ---------------------------------------------------------------------------------------------
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)MLORA_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static char *g_scratch_ptr[MAX_DEVICES];

// device address of the current device's copy of `scratch` (null on error)
static char *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = reinterpret_cast<char *>(ptr);
    }
    return g_scratch_ptr[dev];
}


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
// per chunk for tile blocks of 17 to 32 rows (the finishing blocks need t early there) and 1024 in
// the wide kernel at any row count (fewer shrink blocks and fewer partial sums for every unit to
// gather: the 16-layer decode launch at 32 rows 198.0 -> 192.3 us; 2048 everywhere: 196 us), and
// 2048 where K is above 4096 (a projection of 14336 inputs at 64 rows: 14 -> 7 chunks, 64.1 -> 55.0 us).
int kch_of(const mlora_w4_proj &p, int M, bool wide)
{
    const int c = p.K / ((M > 16 && M <= 32 && !wide) ? 512 : (wide && p.K > 4096) ? 2048 : 1024);
    return c < 1 ? 1 : (c > MAX_KCHUNKS ? MAX_KCHUNKS : c);
}

// Calls with int8 activations run wide blocks whatever their row count, and those work on chunks
// of at least 32 rows with grouped shrink blocks: such a call is laid out as for 17 rows or more.
int plan_rows(int M, bool a8) { return a8 && M < WIDE32_MIN_ROWS ? WIDE32_MIN_ROWS : M; }
int m_pad_of(int M) { return (M + rows_per_chunk(M) - 1) / rows_per_chunk(M) * rows_per_chunk(M); }

// K units per column tile.  Tile blocks: units of at most 2048 inputs (16 super-steps: what a
// block stages of x).  Wide blocks: any unit length works.  A wide launch whose base blocks with
// such units (`launch_blocks`) would leave most compute units idle gets shorter units, the same
// length for all its projections: 8 super-steps up to 240 blocks, 4 below 80.
// Measured on single projections and on whole layers: up to 64 rows about 200 to 250 base
// blocks (one per compute unit with the shrink blocks) beat both fewer and more; a layer of 128
// rows (232 blocks) gains a quarter from 464 shorter ones, two per compute unit; from 256 rows on
// (464 blocks and more) the long units win, and not splitting long projections at all is far
// worse at any size (their blocks finish last).
int ksplit_of(const mlora_w4_proj &p, bool wide, int launch_blocks)
{
    const int nss = p.K / SUPER_K;
    int ks = (nss + UNIT_SUPER_STEPS - 1) / UNIT_SUPER_STEPS;
    if (wide && launch_blocks > 0 && launch_blocks <= 240) {
        const int unit = launch_blocks < 80 ? 4 : 8;
        const int cut = (nss + unit / 2) / unit;
        if (cut > ks) ks = cut;
    }
    return ks;
}
// base blocks of a launch over `count` projections with the default K units
int launch_blocks_of(const mlora_w4_proj *projs, int count, int M, bool wide)
{
    int n = 0;
    const int chunks = m_pad_of(M) / rows_per_chunk(M);
    for (int i = 0; i < count; ++i) {
        const int nss = projs[i].K / SUPER_K;
        n += (tiles_n(projs[i].N) + tiles_per_block(wide) - 1) / tiles_per_block(wide) * chunks *
             ((nss + UNIT_SUPER_STEPS - 1) / UNIT_SUPER_STEPS);
    }
    return n;
}
// Which family of base blocks a launch over these projections runs (see common.hpp).
bool launch_is_wide(const mlora_w4_proj *projs, int count, int M, bool a8)
{
    if (a8 || M >= WIDE_ALWAYS_ROWS) return true;
    if (M < WIDE32_MIN_ROWS) return false;
    return launch_blocks_of(projs, count, M, true) >= WIDE32_MIN_BLOCKS;
}
size_t partial_bytes(const mlora_w4_proj &p, int M, bool wide, int launch_blocks)
{
    return (size_t)(ksplit_of(p, wide, launch_blocks) - 1) * (size_t)tiles_n(p.N) * (size_t)m_pad_of(M) * TILE_N * sizeof(float);
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

// Projections of one launch: up to MAX_PROJ_PER_LAUNCH, and where wide blocks are possible (17
// rows and more; those kernels are compiled per group size) only as long as the group size
// stays the same.
static int launch_run(const mlora_w4_proj *projs, int n_left, int M)
{
    int count = 1;
    while (count < n_left && count < MAX_PROJ_PER_LAUNCH &&
           (M < WIDE32_MIN_ROWS || projs[count].group == projs[0].group))
        ++count;
    return count;
}

// What one launch over projs[0 .. count) needs of the workspace, and (with `a`) its argument
// block.  Counters: 16 lines per projection (copies of its shrink counter), then one line per
// (column tile, row chunk) of every projection whose K is cut into several units.  Data: per
// projection the split-K partial tiles, then the shrink step's partial sums.  Both passes of a
// call (sizes first, arguments second) go through this one function.
struct LaunchNeed {
    size_t ctrl_bytes, data_bytes;
    int grid_x, groups, rpc;
};

static mlora_status plan_launch(const mlora_w4_proj *projs, const void *const *xs, void *const *ys,
                                int count, int M, bool a8, bool lora_on, LaunchNeed &need, LayerArgs *a,
                                char *ctrl, char *data, const float *x_scales = nullptr)
{
    const bool wide = launch_is_wide(projs, count, M, a8);
    const int lb = launch_blocks_of(projs, count, M, wide);
    // A short launch of tile blocks at 17 to 32 rows (a few projections: the calls of a decoder
    // layer taken one after another) is a chain of latencies, not a stream: it runs as two chunks
    // of 16 rows on the kernel for up to 16 rows, with a shrink block per row, which reads the
    // weights twice but gets done sooner (measured at 32 rows: o 15.2 us against 9.1 at 16 rows).
    const bool chunk16 = !wide && M > 16 && M <= 32 && lb < CHUNK16_MAX_BLOCKS;
    const int Mc = chunk16 ? 16 : M;           // decides chunk size, kind of shrink blocks, K chunks
    const int rpc = rows_per_chunk(Mc);
    const int m_pad = (M + rpc - 1) / rpc * rpc;
    const int chunks = m_pad / rpc;
    const int groups = (count + GROUP_PROJ - 1) / GROUP_PROJ;
    bool shared = false;                       // anything handed from block to block?
    size_t part_lines = 0, data_bytes = 0;
    int part_ctr = count * CTR_REPL * CTR_STRIDE;
    int grid_x = 0;
    if (a) {
        for (int z = 0; z < MAX_GROUPS; ++z)
            for (int i = 0; i < GROUP_PROJ; ++i)
                a->main_begin[z][i] = a->pre_begin[z][i] = a->shrink_begin[z][i] = 0x7FFFFFFF;
    }
    for (int z = 0; z < groups; ++z) {
        int main_blocks = 0, pre_blocks = 0, shrink_blocks = 0;
        for (int i = z * GROUP_PROJ; i < count && i < (z + 1) * GROUP_PROJ; ++i) {
            const mlora_w4_proj &p = projs[i];
            const int tiles = tiles_n(p.N);
            const int ksplit = ksplit_of(p, wide, lb);
            // The kernels divide a block index by the tile count with a multiplication that is
            // exact while index * tiles < 2^32: a projection with more than 2^15 column tiles and
            // K units to match is refused rather than mis-indexed.
            if ((unsigned long long)tiles * (unsigned long long)tiles * (unsigned long long)ksplit >= 0x100000000ull)
                return MLORA_ESHAPE;
            const bool lora = lora_on && p.n_adapters > 0;
            // base blocks: one per column tile, or per four of them in the wide kernel
            const int col_blocks = (tiles + tiles_per_block(wide) - 1) / tiles_per_block(wide);
            const size_t part_bytes = partial_bytes(p, M, wide, lb);
            // (two chunks of 16 rows have twice the rows of the shapes the per-row shrink blocks were
            // laid out for: at most 4 K chunks then, which also keeps the sum over them on its short path)
            const int kch = chunk16 && kch_of(p, Mc, wide) > 4 ? 4 : kch_of(p, Mc, wide);
            const size_t t_bytes = lora ? round_up((size_t)kch * (size_t)M * (size_t)r16_of(p) * sizeof(float), 256) : 0;
            const int n_shrink = !lora ? 0
                : (Mc <= 16 && !wide ? M : (M + SHRINK_CHUNK_ROWS - 1) / SHRINK_CHUNK_ROWS * shrink_tile_shares(M, p.n_adapters)) *
                      (r16_of(p) / 16) * kch;
            if (a) {
                ProjArgs &d = a->p[i];
                const int j = i - z * GROUP_PROJ;
                d.codes = reinterpret_cast<const uint4 *>(p.w_blob);
                d.scales = reinterpret_cast<const uint2 *>(reinterpret_cast<const char *>(p.w_blob) +
                                                           blob_code_bytes(p.K, p.N));
                d.x = reinterpret_cast<const uint16_t *>(xs[i]);
                d.y = ys[i];
                d.K = p.K;
                d.N = p.N;
                d.spg = p.group / KSTEP;
                d.alpha = p.alpha;
                d.x_scale = x_scales ? x_scales[i] : 1.0f;
                d.ksplit = ksplit;
                // blocks (wide kernel: waves) that wait for this projection's shrink blocks: the
                // finishing ones, or every K unit where the LoRA term is spread over them
                d.n_finish_blocks = tiles * chunks * (wide ? ksplit : 1);
                d.unit_q = (p.K / SUPER_K) / ksplit;
                d.unit_r = (p.K / SUPER_K) % ksplit;
                d.spg_shift = d.spg == 4 ? 2 : d.spg == 2 ? 1 : 0;
                d.ctr_copies = 1;
                while (d.ctr_copies * 2 <= CTR_REPL && d.ctr_copies * 2 <= d.n_finish_blocks) d.ctr_copies *= 2;
                d.tiles_inv = (unsigned)((0x100000000ull + (unsigned)tiles - 1) / (unsigned)tiles);
                a->main_begin[z][j] = main_blocks;
                a->pre_begin[z][j] = pre_blocks;
                a->shrink_begin[z][j] = shrink_blocks;
                d.partial = reinterpret_cast<float *>(data + data_bytes);
                d.part_ctr = part_ctr;
                if (lora) {
                    d.lora_a = reinterpret_cast<const uint16_t *>(p.lora_a);
                    d.lora_b = reinterpret_cast<const uint16_t *>(p.lora_b);
                    d.n_adapters = p.n_adapters;
                    d.rank = p.rank;
                    d.r16 = r16_of(p);
                    d.kch = kch;
                    d.t_part = reinterpret_cast<float *>(data + data_bytes + part_bytes);
                    d.n_shrink_blocks = n_shrink;
                } else {
                    d.n_adapters = 0;
                    d.rank = 0;
                    d.r16 = 16;
                    d.kch = 1;
                }
            }
            main_blocks += col_blocks;
            pre_blocks += col_blocks * (ksplit - 1);
            shrink_blocks += n_shrink;
            data_bytes += part_bytes + t_bytes;
            if (ksplit > 1) {
                part_ctr += tiles * chunks * CTR_STRIDE;
                part_lines += (size_t)tiles * (size_t)chunks;
            }
            shared = shared || ksplit > 1 || lora;
        }
        const int total = shrink_blocks + pre_blocks + main_blocks;
        if (a) {
            a->shrink_blocks[z] = shrink_blocks;
            a->pre_base_blocks[z] = pre_blocks;
            a->group_blocks[z] = total;
        }
        if (total > grid_x) grid_x = total;
    }
    need.ctrl_bytes = shared ? ((size_t)count * CTR_REPL + part_lines) * CTR_STRIDE * sizeof(unsigned) : 0;
    need.data_bytes = data_bytes;
    need.grid_x = grid_x;
    need.groups = groups;
    need.rpc = rpc;
    if (a) {
        a->ctrl = reinterpret_cast<unsigned *>(ctrl);
        a->wide = wide;
        a->m_pad = m_pad;
        if (chunk16) a->M_plan = 16;
    }
    return MLORA_OK;
}

// Sizes of a whole call (all its launches).
static mlora_status plan_call(const mlora_w4_proj *projs, int n_proj, int M, bool lora_on,
                              size_t &ctrl_total, size_t &data_total, bool a8 = false)
{
    ctrl_total = data_total = 0;
    for (int first = 0, count = 0; first < n_proj; first += count) {
        count = launch_run(projs + first, n_proj - first, M);
        LaunchNeed need;
        const mlora_status st = plan_launch(projs + first, nullptr, nullptr, count, M, a8, lora_on, need, nullptr, nullptr, nullptr);
        if (st != MLORA_OK) return st;
        ctrl_total += need.ctrl_bytes;
        data_total += need.data_bytes;
    }
    return MLORA_OK;
}

// Workspace layout: [status word, 256 B][counters of launch 0, 1, ...] ... [data of launch 0, 1, ...]
// with the data at the END of the workspace as handed in.  Counters must read zero when a call
// starts and return to zero by themselves; data is never cleared.  Were the data to follow the
// counters directly, a later call with more counter lines (another shape, more rows) would find
// its extra lines inside the earlier call's data.  With the counters growing from the front, the
// data placed against the end, and a size of 256 + 2 * max(counters, data), the counters of any
// call and the data of any other call that fits the same workspace cannot overlap.
static size_t workspace_need(size_t ctrl_total, size_t data_total)
{
    if (ctrl_total == 0) return 0;
    const size_t c = round_up(ctrl_total, 256), d = round_up(data_total, 256);
    return WS_HEADER_BYTES + 2 * (c > d ? c : d);
}

size_t mlora_w4_workspace_bytes(const mlora_w4_proj *projs, int32_t n_proj, int32_t M)
{
    if (!projs || n_proj <= 0 || M <= 0 || M > MLORA_MAX_ROWS) return 0;
    for (int i = 0; i < n_proj; ++i)
        if (check_weight_shape(projs[i].K, projs[i].N, projs[i].group) != MLORA_OK) return 0;
    size_t ctrl_total, data_total;
    if (plan_call(projs, n_proj, M, true, ctrl_total, data_total) != MLORA_OK) return 0;
    return workspace_need(ctrl_total, data_total);
}

mlora_status mlora_w4_layer_step_plan(const mlora_w4_proj *projs, int32_t n_proj, int32_t M, int32_t *info)
{
    if (!projs || !info || n_proj <= 0) return MLORA_EINVAL;
    if (M <= 0 || M > MLORA_MAX_ROWS) return MLORA_ESHAPE;
    for (int i = 0; i < n_proj; ++i)
        if (check_weight_shape(projs[i].K, projs[i].N, projs[i].group) != MLORA_OK) return MLORA_ESHAPE;
    int launches = 0;
    for (int first = 0, count = 0; first < n_proj; first += count, ++launches) {
        count = launch_run(projs + first, n_proj - first, M);
        LaunchNeed need;
        const mlora_status st = plan_launch(projs + first, nullptr, nullptr, count, M, false, true, need, nullptr, nullptr, nullptr);
        if (st != MLORA_OK) return st;
        if (first == 0) {
            info[1] = launch_is_wide(projs, count, M, false) ? 1 : 0;
            info[2] = need.rpc;
            info[3] = need.grid_x;
            info[4] = need.groups;
        }
    }
    info[0] = launches;
    return MLORA_OK;
}

mlora_status mlora_w4_workspace_init(void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace) return workspace_bytes == 0 ? MLORA_OK : MLORA_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MLORA_EALIGN;
    return launch_zero(workspace, workspace_bytes / 16 * 16, (hipStream_t)stream) == hipSuccess
               ? MLORA_OK : MLORA_EHIP;
}

mlora_status mlora_w4_workspace_status(const void *workspace, int32_t *status_word, void *stream)
{
    if (!workspace || !status_word) return MLORA_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    unsigned word = 0;
    if (hipMemcpyAsync(&word, workspace, sizeof word, hipMemcpyDeviceToHost, s) != hipSuccess) return MLORA_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return MLORA_EHIP;
    *status_word = (int32_t)word;
    return MLORA_OK;
}

static int g_spin_limit = SPIN_LIMIT_DEFAULT;

int32_t mlora_w4_debug_spin_limit(int32_t limit)
{
    const int old = g_spin_limit;
    g_spin_limit = limit < 0 ? SPIN_LIMIT_DEFAULT : limit;
    return old;
}

// Host-side checks of a call: everything that can be refused is refused here, before the first launch.
static mlora_status check_call(const mlora_w4_proj *projs, int32_t n_proj, const void *const *xs,
                               void *const *ys, const int32_t *row_adapter, int32_t M, int32_t y_dtype)
{
    if (!projs || !xs || !ys || n_proj <= 0) return MLORA_EINVAL;
    if (y_dtype != MLORA_Y_BF16 && y_dtype != MLORA_Y_FP32) return MLORA_EINVAL;
    if (M < 0 || M > MLORA_MAX_ROWS) return MLORA_ESHAPE;
    for (int i = 0; i < n_proj; ++i) {
        mlora_status st = check_proj(projs[i]);
        if (st != MLORA_OK) return st;
        if (!xs[i] || !ys[i]) return MLORA_EINVAL;
        if (!aligned16(xs[i]) || !aligned16(ys[i])) return MLORA_EALIGN;
    }
    // outputs may not be shared (sorted copy: a call may bring thousands of projections)
    std::vector<const void *> outs(ys, ys + n_proj);
    std::sort(outs.begin(), outs.end());
    if (std::adjacent_find(outs.begin(), outs.end()) != outs.end()) return MLORA_EINVAL;
    if (row_adapter && (reinterpret_cast<uintptr_t>(row_adapter) & 3u)) return MLORA_EALIGN;
    return MLORA_OK;
}

// Enqueue the launches of a checked call on a workspace whose counters read zero.
static mlora_status enqueue_call(const mlora_w4_proj *projs, int32_t n_proj, const void *const *xs,
                                 void *const *ys, const int32_t *row_adapter, int32_t M, int32_t y_dtype,
                                 bool lora_on, char *workspace, size_t workspace_bytes, size_t data_total,
                                 hipStream_t s, const float *x_scales = nullptr,
                                 const mlora_w4_epilogue *epis = nullptr)
{
    const bool a8 = x_scales != nullptr;
    const int Mp = plan_rows(M, a8);
    char *ctrl = workspace ? workspace + WS_HEADER_BYTES : nullptr;
    char *data = workspace ? workspace + workspace_bytes / 256 * 256 - round_up(data_total, 256) : nullptr;
    // (one argument block on the heap: it is about 19 KiB and is copied by the launch)
    std::unique_ptr<LayerArgs> a(new LayerArgs);
    for (int first = 0, count = 0; first < n_proj; first += count) {
        count = launch_run(projs + first, n_proj - first, Mp);
        memset(a.get(), 0, sizeof(LayerArgs));
        a->row_adapter = lora_on ? row_adapter : nullptr;
        a->n_proj = count;
        a->M = M;
        a->M_plan = Mp;
        a->a8 = a8;
        a->fused = epis != nullptr;
        if (epis) {
            for (int i = 0; i < count && i < GROUP_PROJ; ++i) {
                const mlora_w4_epilogue &e = epis[first + i];
                a->epi[i].row_scale = e.row_scale;
                a->epi[i].rope_cos = e.rope_cos;
                a->epi[i].rope_sin = e.rope_sin;
                a->epi[i].residual = reinterpret_cast<const uint16_t *>(e.residual);
                a->epi[i].pair_op = e.pair_op;
                a->epi[i].sq_in = e.sq_in;
                a->epi[i].sq_parts = e.sq_parts;
                a->epi[i].sq_eps = e.sq_eps;
                a->epi[i].sq_out = e.sq_out;
            }
        }
        a->y_fp32 = (y_dtype == MLORA_Y_FP32);
        a->m_pad = m_pad_of(Mp);
        a->spin_limit = g_spin_limit;
        a->code_mask = 0x00780078u;
        a->code_bias = 0x41804180u;
        a->status = reinterpret_cast<unsigned *>(workspace);
        LaunchNeed need;
        const mlora_status st = plan_launch(projs + first, xs + first, ys + first, count, Mp, a8, lora_on, need,
                                            a.get(), ctrl, data, x_scales ? x_scales + first : nullptr);
        if (st != MLORA_OK) return st;         // (cannot happen: the sizing pass has seen the same shapes)
        if (launch_layer(*a, need.grid_x, need.groups, s) != hipSuccess) return MLORA_EHIP;
        ctrl += need.ctrl_bytes;
        data += need.data_bytes;
    }
    return MLORA_OK;
}

mlora_status mlora_w4_layer_step(const mlora_w4_proj *projs, int32_t n_proj,
                                 const void *const *xs, void *const *ys,
                                 const int32_t *row_adapter, int32_t M, int32_t y_dtype,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    mlora_status st = check_call(projs, n_proj, xs, ys, row_adapter, M, y_dtype);
    if (st != MLORA_OK) return st;
    if (M == 0) return MLORA_OK;
    size_t ctrl_total, data_total;
    st = plan_call(projs, n_proj, M, true, ctrl_total, data_total);
    if (st != MLORA_OK) return st;
    const size_t need = workspace_need(ctrl_total, data_total);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return MLORA_EWORKSPACE;
        if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MLORA_EALIGN;
    }
    bool any_lora = false;
    for (int i = 0; i < n_proj; ++i) any_lora = any_lora || projs[i].n_adapters > 0;
    return enqueue_call(projs, n_proj, xs, ys, row_adapter, M, y_dtype, any_lora && row_adapter != nullptr,
                        need > 0 ? reinterpret_cast<char *>(workspace) : nullptr, workspace_bytes, data_total,
                        (hipStream_t)stream);
}

mlora_status mlora_w4_layer_step_static(const mlora_w4_proj *projs, int32_t n_proj,
                                        const void *const *xs, void *const *ys,
                                        const int32_t *row_adapter, int32_t M, int32_t y_dtype,
                                        void *stream)
{
    mlora_status st = check_call(projs, n_proj, xs, ys, row_adapter, M, y_dtype);
    if (st != MLORA_OK) return st;
    if (M == 0) return MLORA_OK;
    size_t ctrl_total, data_total;
    st = plan_call(projs, n_proj, M, true, ctrl_total, data_total);
    if (st != MLORA_OK) return st;
    // counters at the front, data against the end: the two must not meet
    const size_t head = WS_HEADER_BYTES + round_up(ctrl_total, 256);
    if (head + round_up(data_total, 256) > STATIC_SCRATCH_BYTES) return MLORA_EWORKSPACE;
    char *ws = nullptr;
    if (ctrl_total > 0) {
        ws = static_scratch();
        if (!ws) return MLORA_EHIP;
        // The array keeps what the last call left: status word and counters start from zero again
        // (a fill kernel, not a memset node: the call may be under stream capture).
        if (launch_zero(ws, head, (hipStream_t)stream) != hipSuccess) return MLORA_EHIP;
    }
    bool any_lora = false;
    for (int i = 0; i < n_proj; ++i) any_lora = any_lora || projs[i].n_adapters > 0;
    return enqueue_call(projs, n_proj, xs, ys, row_adapter, M, y_dtype, any_lora && row_adapter != nullptr,
                        ws, STATIC_SCRATCH_BYTES, data_total, (hipStream_t)stream);
}

mlora_status mlora_w4_layer_step_fused(const mlora_w4_proj *projs, const mlora_w4_epilogue *epis, int32_t n_proj,
                                       const void *const *xs, void *const *ys,
                                       const int32_t *row_adapter, int32_t M, int32_t y_dtype,
                                       void *workspace, size_t workspace_bytes, void *stream)
{
    mlora_status st = check_call(projs, n_proj, xs, ys, row_adapter, M, y_dtype);
    if (st != MLORA_OK) return st;
    if (!epis) return MLORA_EINVAL;
    if (n_proj > GROUP_PROJ) return MLORA_ESHAPE;
    for (int i = 0; i < n_proj; ++i) {
        const mlora_w4_epilogue &e = epis[i];
        if (e.pair_op != MLORA_PAIR_NONE && e.pair_op != MLORA_PAIR_ROPE && e.pair_op != MLORA_PAIR_SWIGLU) return MLORA_EINVAL;
        if (e.pair_op != MLORA_PAIR_NONE && projs[i].N % TILE_N != 0) return MLORA_ESHAPE;
        if (e.pair_op == MLORA_PAIR_ROPE && (!e.rope_cos || !e.rope_sin)) return MLORA_EINVAL;
        if (e.sq_in && (e.row_scale || e.sq_parts < 1 || !(e.sq_eps >= 0.0f))) return MLORA_EINVAL;
        if ((e.sq_in && (reinterpret_cast<uintptr_t>(e.sq_in) & 3u)) ||
            (e.sq_out && (reinterpret_cast<uintptr_t>(e.sq_out) & 3u))) return MLORA_EALIGN;
        if ((e.row_scale && (reinterpret_cast<uintptr_t>(e.row_scale) & 3u)) ||
            (e.rope_cos && (reinterpret_cast<uintptr_t>(e.rope_cos) & 3u)) ||
            (e.rope_sin && (reinterpret_cast<uintptr_t>(e.rope_sin) & 3u)) ||
            (e.residual && (reinterpret_cast<uintptr_t>(e.residual) & 1u))) return MLORA_EALIGN;
    }
    if (M == 0) return MLORA_OK;
    size_t ctrl_total, data_total;
    st = plan_call(projs, n_proj, M, true, ctrl_total, data_total);
    if (st != MLORA_OK) return st;
    const size_t need = workspace_need(ctrl_total, data_total);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return MLORA_EWORKSPACE;
        if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MLORA_EALIGN;
    }
    bool any_lora = false;
    for (int i = 0; i < n_proj; ++i) any_lora = any_lora || projs[i].n_adapters > 0;
    return enqueue_call(projs, n_proj, xs, ys, row_adapter, M, y_dtype, any_lora && row_adapter != nullptr,
                        need > 0 ? reinterpret_cast<char *>(workspace) : nullptr, workspace_bytes, data_total,
                        (hipStream_t)stream, nullptr, epis);
}

mlora_status mlora_rms_scale(const void *x, int32_t M, int32_t K, float eps, float *scale, void *stream)
{
    if (M < 0 || M > MLORA_MAX_ROWS || K <= 0 || K % 8 != 0 || K > (1 << 24)) return MLORA_ESHAPE;
    if (M == 0) return MLORA_OK;
    if (!x || !scale || !(eps >= 0.0f)) return MLORA_EINVAL;
    if (!aligned16(x) || (reinterpret_cast<uintptr_t>(scale) & 3u)) return MLORA_EALIGN;
    return launch_rms_scale(reinterpret_cast<const uint16_t *>(x), M, K, eps, scale, (hipStream_t)stream) == hipSuccess
               ? MLORA_OK : MLORA_EHIP;
}

mlora_status mlora_lora_int16_expand(const int16_t *a_q, const int16_t *b_q, int32_t n_adapters, int32_t rank,
                                     int32_t K, int32_t N, float alpha, float s_a, float s_b,
                                     void *lora_a, void *lora_b, float *alpha_out, void *stream)
{
    if (n_adapters < 1 || n_adapters > MLORA_MAX_ADAPTERS || rank <= 0 || rank % 8 != 0 || 4 * rank > MLORA_MAX_RANK)
        return MLORA_ESHAPE;
    if (K <= 0 || K % KSTEP != 0 || K > (1 << 24) || N <= 0 || N > (1 << 24)) return MLORA_ESHAPE;
    const unsigned long long na = (unsigned long long)n_adapters * rank * K, nb = (unsigned long long)n_adapters * N * rank;
    if ((na + 255) / 256 > 0x7FFFFFFFull || (nb + 255) / 256 > 0x7FFFFFFFull) return MLORA_ESHAPE;
    if (!a_q || !b_q || !lora_a || !lora_b || !alpha_out) return MLORA_EINVAL;
    if (!std::isfinite(alpha) || !std::isfinite(s_a) || !std::isfinite(s_b) || !(s_a > 0.0f) || !(s_b > 0.0f)) return MLORA_EINVAL;
    if (!aligned16(a_q) || !aligned16(b_q) || !aligned16(lora_a) || !aligned16(lora_b)) return MLORA_EALIGN;
    *alpha_out = alpha * s_a * s_b;
    return launch_lora_int16_expand(a_q, b_q, n_adapters, rank, K, N, reinterpret_cast<uint16_t *>(lora_a),
                                    reinterpret_cast<uint16_t *>(lora_b), (hipStream_t)stream) == hipSuccess
               ? MLORA_OK : MLORA_EHIP;
}

size_t mlora_w4a8_workspace_bytes(const mlora_w4_proj *projs, int32_t n_proj, int32_t M)
{
    if (!projs || n_proj <= 0 || M <= 0 || M > MLORA_MAX_ROWS) return 0;
    for (int i = 0; i < n_proj; ++i)
        if (check_weight_shape(projs[i].K, projs[i].N, projs[i].group) != MLORA_OK) return 0;
    size_t ctrl_total, data_total;
    if (plan_call(projs, n_proj, plan_rows(M, true), true, ctrl_total, data_total, true) != MLORA_OK) return 0;
    return workspace_need(ctrl_total, data_total);
}

mlora_status mlora_w4a8_layer_step(const mlora_w4_proj *projs, int32_t n_proj,
                                   const void *const *xs, const float *x_scales, void *const *ys,
                                   const int32_t *row_adapter, int32_t M, int32_t y_dtype,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    mlora_status st = check_call(projs, n_proj, xs, ys, row_adapter, M, y_dtype);
    if (st != MLORA_OK) return st;
    if (!x_scales) return MLORA_EINVAL;
    for (int i = 0; i < n_proj; ++i)
        if (!(x_scales[i] > 0.0f) || !(x_scales[i] < 3.0e38f)) return MLORA_EINVAL;     // also refuses NaN
    if (M == 0) return MLORA_OK;
    size_t ctrl_total, data_total;
    st = plan_call(projs, n_proj, plan_rows(M, true), true, ctrl_total, data_total, true);
    if (st != MLORA_OK) return st;
    const size_t need = workspace_need(ctrl_total, data_total);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return MLORA_EWORKSPACE;
        if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MLORA_EALIGN;
    }
    bool any_lora = false;
    for (int i = 0; i < n_proj; ++i) any_lora = any_lora || projs[i].n_adapters > 0;
    return enqueue_call(projs, n_proj, xs, ys, row_adapter, M, y_dtype, any_lora && row_adapter != nullptr,
                        need > 0 ? reinterpret_cast<char *>(workspace) : nullptr, workspace_bytes, data_total,
                        (hipStream_t)stream, x_scales);
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
