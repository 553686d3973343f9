// Host side of the C ABI declared in include/rsparse.h: argument checks, offline packing
// (column-major W, U_r^T appended as extra rows, S_r V_r^T), uploads, launch-shape choice,
// read-back decoding.  No arithmetic of the hot path runs here.
#include "../../include/rsparse.h"
#include "kernels.h"
#include "svd_host.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <new>
#include <thread>
#include <vector>

using namespace rsparse;

namespace {

thread_local char g_err[512] = "";

rsparse_status fail(rsparse_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

#define RS_HIP(call)                                                                             \
    do {                                                                                         \
        hipError_t e_ = (call);                                                                  \
        if (e_ != hipSuccess)                                                                    \
            return fail(e_ == hipErrorOutOfMemory ? RSPARSE_ENOMEM : RSPARSE_EHIP, "%s: %s", #call, \
                        hipGetErrorString(e_));                                                  \
    } while (0)

// Exact widening of the 16-bit storage formats on the host (used by the SVD intake and the
// threshold calibration only).
float half_bits_to_float(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const uint32_t em = h & 0x7fffu;
    uint32_t out;
    if (em >= 0x7c00u) out = sign | 0x7f800000u | ((em & 0x3ffu) << 13);           // inf / nan
    else if (em >= 0x0400u) out = sign | ((em + (112u << 10)) << 13);              // normal
    else if (em == 0) out = sign;
    else {                                                                          // subnormal
        float f = (float)em * (1.0f / 16777216.0f);                                 // em * 2^-24
        uint32_t u;
        memcpy(&u, &f, 4);
        out = sign | u;
    }
    float f;
    memcpy(&f, &out, 4);
    return f;
}
float bf16_bits_to_float(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}
float widen16(uint16_t h, int dtype) { return dtype == RSPARSE_F16 ? half_bits_to_float(h) : bf16_bits_to_float(h); }

uint16_t double_to_bf16(double d)
{
    // One rounding, double -> bf16.  Going through fp32 rounds twice; the only way that can differ is when
    // the first rounding lands exactly on a bf16 tie (low half 0x8000) that d itself was not on: move the
    // fp32 value one step towards d, so that the second rounding goes to d's side of the tie.
    float f = (float)d;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    if ((u & 0xffffu) == 0x8000u && (u & 0x7f800000u) != 0x7f800000u && (double)f != d)
        u += std::fabs(d) > std::fabs((double)f) ? 1u : 0xffffffffu;
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
uint16_t double_to_f16(double d)
{
    _Float16 h = (_Float16)d;
    uint16_t u;
    memcpy(&u, &h, 2);
    return u;
}

template <typename F>
void parallel_for(size_t n, F &&f)
{
    unsigned nt = std::thread::hardware_concurrency();
    if (nt == 0) nt = 1;
    if (nt > 16) nt = 16;
    if (n < 2 * nt) nt = 1;
    std::vector<std::thread> th;
    for (unsigned t = 0; t < nt; ++t)
        th.emplace_back([&, t]() {
            const size_t lo = n * t / nt, hi = n * (t + 1) / nt;
            for (size_t i = lo; i < hi; ++i) f(i);
        });
    for (auto &x : th) x.join();
}

// dst[cols][rows] = transpose of src[rows][cols], 16-bit elements, 64x64 blocks.
void transpose16(const uint16_t *src, size_t rows, size_t cols, uint16_t *dst)
{
    constexpr size_t B = 64;
    const size_t rb = (rows + B - 1) / B;
    parallel_for(rb, [&](size_t bi) {
        const size_t r0 = bi * B, r1 = std::min(rows, r0 + B);
        for (size_t c0 = 0; c0 < cols; c0 += B) {
            const size_t c1 = std::min(cols, c0 + B);
            for (size_t r = r0; r < r1; ++r)
                for (size_t c = c0; c < c1; ++c) dst[c * rows + r] = src[r * cols + c];
        }
    });
}

}  // namespace

struct rsparse_layer {
    rsparse_config cfg{};
    rsparse_tuning tuning{};
    int device = 0;
    int cus = 256;
    uint16_t *M = nullptr, *SVt = nullptr, *U = nullptr, *Wrow = nullptr;
    uint16_t *Ms = nullptr;                // strip-major W + U_r^T: [strips][d_in + rank][strip_w]
    int strip_w = 0, strips = 0;
    long long strip_stride = 0;
    unsigned long long *t_tag = nullptr;   // [t_slots][rank] {generation, t} of the strip kernel
    int t_slots = 0;
    int32_t *act_seg = nullptr;            // [nz_max][d_in / 8] kept channels per channel range (strip kernel)
    bool last_strip = false;               // the last call went through the strip kernel ...
    int last_ranges = 0;                   // ... with this many channel ranges (splits x waves)
    float *t = nullptr, *yacc = nullptr;
    uint16_t *SVc = nullptr;               // [d_in][rank] channel-major copy of S_r V_r^T (cfg.lowrank_channel_major)
    float *t_sum = nullptr;                // [rank] fp32 sums of the stage 1 that reads it (zero between calls)
    float *t_acc = nullptr;                // [rank][32] accumulated t of the matrix-core path (zero between calls)
    uint16_t *t16 = nullptr;               // [2][32][rank] its two 16-bit halves
    uint32_t *act_bits = nullptr, *chan_bits = nullptr;
    bool last_mfma = false;
    int32_t *act_list = nullptr, *act_count = nullptr;
    int *sync = nullptr;
    uint32_t *t_pub = nullptr;
    ScratchView last_scratch{};            // the per-call scratch the last call used: the handle's own, or the static one
    uint16_t *hy = nullptr;                // [max_batch][d_out] 16-bit output scratch (gate / up results of rsparse_mlp_gate_up's fallback)
    float *bias = nullptr;                 // [d_out] fp32 static bias (rsparse_set_bias), or null
    KeepRule *rules = nullptr;             // [max_batch] per-token rules of the fixed-count activation (cfg.topk > 0)
    uint16_t *xg = nullptr;                // [max_batch][d_in] gated input x = round16(silu(g) * u), written out per call
    size_t n_t = 0, n_y = 0, sync_n = 0;
    bool last_fused = false;
    // 4-bit weights (rsparse_prepare_q4): codes, group scales, group zero points; M and Wrow stay null
    uint8_t *Mq = nullptr, *qz = nullptr;
    uint8_t *Qrow = nullptr, *Zrow = nullptr;   // row-major codes and zero points (dense_rowmajor = 1): the row-dot dense baseline
    uint16_t *Srow = nullptr;
    uint16_t *qs = nullptr, *Ut = nullptr;
    int qshift = 0, qtiles = 0;
    bool q4() const { return Mq != nullptr; }
    int tiles = 0, nz_max = 1;
    std::vector<uint16_t> U16, SV16;       // host copies of the stored factors
    hipStream_t last_stream = nullptr;
    int last_batch = 0;
    int last_bt = 0;                       // tokens per batch tile of the last call's kept lists (0 = batch_tile_of(last_batch))

    ScratchView own_scratch() const
    {
        ScratchView sp{};
        sp.t = t; sp.yacc = yacc; sp.act_list = act_list; sp.act_bits = act_bits; sp.act_count = act_count;
        sp.act_seg = act_seg; sp.sync = sync; sp.t_pub = t_pub; sp.t_tag = t_tag; sp.t_slots = t_slots; sp.rules = rules;
        sp.n_t = n_t; sp.n_y = n_y; sp.sync_n = sync_n;
        return sp;
    }

    // The view of one call: `batch` decides the mask mode when the configuration leaves it to the library; the dense
    // baseline gets no bias and no fixed-count rules.
    LayerView view(const ScratchView *ov = nullptr, int batch = 1, bool dense = false) const
    {
        const ScratchView sp = ov ? *ov : own_scratch();
        LayerView v{};
        v.M = M; v.SVt = SVt; v.U = U; v.Wrow = Wrow; v.t = sp.t; v.yacc = sp.yacc; v.t_acc = ov ? nullptr : t_acc; v.SVc = SVc; v.t_sum = ov ? nullptr : t_sum; v.t16 = ov ? nullptr : t16;
        v.act_list = sp.act_list; v.act_bits = sp.act_bits; v.act_count = sp.act_count; v.sync = sp.sync; v.t_pub = sp.t_pub;
        v.d_in = cfg.d_in; v.d_out = cfg.d_out; v.rank = cfg.rank;
        v.dtype = cfg.dtype; v.out_dtype = cfg.out_dtype; v.cmp_mode = cfg.cmp_mode;
        v.batch_mask_mode = cfg.batch_mask_mode == 2 ? (batch >= 4 ? 1 : 0) : cfg.batch_mask_mode;
        v.tau = cfg.tau;
        // |x| > tau is |x| >= the next fp32 above tau; nothing is above +inf (a NaN bound keeps nothing)
        v.tau_ge = cfg.tau;
        if (cfg.cmp_mode == 1)
            v.tau_ge = cfg.tau == INFINITY ? NAN : std::nextafterf(cfg.tau, INFINITY);
        v.keep_signed = cfg.cmp_mode == 2 ? 1 : 0;
        v.rules = (cfg.topk > 0 && !dense) ? sp.rules : nullptr;
        v.bias = dense ? nullptr : bias;
        v.Mq = Mq; v.qs = qs; v.qz = qz; v.Ut = Ut; v.qshift = qshift; v.qtiles = qtiles;
        v.Ms = Ms; v.strip_w = strip_w; v.strip_stride = strip_stride; v.t_tag = sp.t_tag; v.t_slots = sp.t_slots; v.act_seg = sp.act_seg;
        return v;
    }
};

namespace {

int batch_tile_of(int batch) { return batch <= 1 ? 1 : batch <= 2 ? 2 : batch <= 4 ? 4 : 8; }

rsparse_status check_config(const rsparse_config *c)
{
    if (!c) return fail(RSPARSE_EINVAL, "config is NULL");
    if (c->d_in < 8 || c->d_out < 8 || (c->d_in % 8) || (c->d_out % 8))
        return fail(RSPARSE_EINVAL, "d_in and d_out must be positive multiples of 8 (got %d, %d)", c->d_in, c->d_out);
    // the gather kernels keep 5 bytes of LDS per 8 input channels for the scan of the token
    if (c->d_in > 65536 || c->d_out > (1 << 20)) return fail(RSPARSE_EINVAL, "dimension too large (d_in <= 65536, d_out <= 2^20)");
    if (c->rank < 0 || c->rank > std::min(c->d_in, c->d_out) || (c->rank % 8))
        return fail(RSPARSE_EINVAL, "rank %d must be a multiple of 8 in [0, min(d_in, d_out)]", c->rank);
    if (c->max_batch < 1 || c->max_batch > RSPARSE_MAX_BATCH)
        return fail(RSPARSE_EINVAL, "max_batch %d outside [1, %d]", c->max_batch, RSPARSE_MAX_BATCH);
    if (std::isnan(c->tau)) return fail(RSPARSE_EINVAL, "tau is NaN");
    if (c->dtype != RSPARSE_F16 && c->dtype != RSPARSE_BF16) return fail(RSPARSE_EINVAL, "dtype must be F16 or BF16");
    if (c->out_dtype != c->dtype && c->out_dtype != RSPARSE_F32)
        return fail(RSPARSE_EINVAL, "out_dtype must equal dtype or be F32");
    if (c->cmp_mode < 0 || c->cmp_mode > 2) return fail(RSPARSE_EINVAL, "cmp_mode must be 0, 1 or 2");
    if (c->batch_mask_mode < 0 || c->batch_mask_mode > 2) return fail(RSPARSE_EINVAL, "batch_mask_mode must be 0, 1 or 2");
    if (c->topk < 0 || c->topk > c->d_in) return fail(RSPARSE_EINVAL, "topk %d outside [0, d_in]", c->topk);
    if (c->topk > 0 && c->cmp_mode != 0) return fail(RSPARSE_EINVAL, "the fixed-count activation (topk > 0) needs cmp_mode 0");
    if (c->dense_rowmajor != 0 && c->dense_rowmajor != 1) return fail(RSPARSE_EINVAL, "dense_rowmajor must be 0 or 1");
    if (c->lowrank_channel_major != 0 && c->lowrank_channel_major != 1) return fail(RSPARSE_EINVAL, "lowrank_channel_major must be 0 or 1");
    if (c->strip_cols != 0 && !strip_width_ok(c->strip_cols)) return fail(RSPARSE_EINVAL, "strip_cols must be 0, 32, 64, 128, 256 or 512");
    return RSPARSE_OK;
}

// Launch shape: column tiles x channel splits ~ a few workgroups per compute unit, each with
// enough rows to amortise its scan, and the staged share small enough for 64 KiB of LDS.
// Stage-1 workgroups get about as many bytes of S_r V_r^T as a gather workgroup gets of W.
Launch resolve_launch(const rsparse_layer *L, int batch, bool dense, int group, int waves_of_group = 0,
                      bool fused = false, size_t launch_weights = 0)
{
    Launch c{};
    const rsparse_tuning &t = L->tuning;
    const int bt = batch_tile_of(batch);
    // 8 waves per workgroup and ~1.5 workgroups per compute unit measured best on MI355X: enough
    // loads in flight, while each output column only receives `splits` atomic adds (same-address
    // device-scope atomics serialise at ~0.1 us each, which sets the kernel's tail).
    c.waves = (t.waves == 1 || t.waves == 2 || t.waves == 4 || t.waves == 8) ? t.waves : (bt >= 8 ? 4 : 8);
    if (waves_of_group > 0) c.waves = waves_of_group;   // one block size per launch: the first layer's
    if (bt >= 8 && c.waves > 4) c.waves = 4;      // the 8-token kernels are built for at most 256 lanes
    c.nontemporal = t.nontemporal == 2 ? 0 : 1;      // non-temporal weight loads measured 5-10 % faster: the default
    c.wait_polls = t.debug_wait_polls;
    c.skip_stage1 = t.debug_skip_stage1 ? 1 : 0;
    c.tile_map = t.tile_map == 0 ? 1 : t.tile_map;
    const int rows = dense ? L->cfg.d_in : std::max(8, L->cfg.d_in / 2);     // expected rows to stream
    int splits = t.splits;
    if (splits <= 0) {
        // one resident round of workgroups for the whole launch (a group of layers shares it):
        // ~1.5 per compute unit, for the 8-wave kernels and for the 4-wave 8-token kernels alike
        // (those hold two workgroups per compute unit at their register count)
        const int target_wgs = std::max(L->tiles, (3 * L->cus) / 2 / std::max(1, group));
        splits = (target_wgs + L->tiles - 1) / L->tiles;
        const int max_by_rows = std::max(1, rows / (c.waves * 4));          // >= 4 rows per wave
        splits = std::max(1, std::min(splits, max_by_rows));
        // every output receives `splits` same-address atomic adds, which serialise at the end of the
        // kernel: beyond 32 they cost more than the extra workgroups bring, as long as one workgroup
        // per compute unit remains (measured on 11008 -> 4096: 32 splits beat 48)
        if (fused) splits = std::min(splits, std::max(32, (L->cus + L->tiles - 1) / L->tiles));
    }
    splits = std::min(splits, 4096);
    while (gather_lds_bytes(L->cfg.d_in, splits, c.waves, bt, fused ? L->cfg.rank : 0) > 60 * 1024 && splits < 65536) splits *= 2;
    c.splits = splits;
    int lr = t.lowrank_rows;
    if (lr <= 0) {
        const double wg_bytes = (double)rows / splits * kTile * 2.0;          // W bytes of one gather workgroup
        lr = (int)(wg_bytes / (2.0 * L->cfg.d_in) + 0.5);
    }
    c.lowrank_rows = std::max(1, std::min(lr, 4 * c.waves));                  // at most 4 rows per wave
    // one launch: the gather workgroups end with rows that need t, so stage 1 is cut as fine as the
    // launch allows: its workgroups get the resident slots (two per compute unit, shared by the
    // layers of a group) that the gather workgroups leave free, with one row per wave on at least
    // half of the waves.  A launch that needs a second round of workgroups loses more than finer
    // stage-1 workgroups gain (measured on 4096 -> 11008 and 28672 -> 8192).
    if (fused && t.lowrank_rows <= 0) {
        const int free_slots = 2 * L->cus / std::max(1, group) - L->tiles * splits;
        const int need = free_slots > 0 ? (L->cfg.rank + free_slots - 1) / free_slots : 4 * c.waves;
        c.lowrank_rows = std::max(std::max(1, c.waves / 2), std::min(4 * c.waves, need));
    }
    // one token over a channel-major copy of S_r V_r^T: stage 1 reads the dropped channels' rows only, each of its
    // workgroups on a fixed channel range.  64 workgroups, 128 from 16 MB of expected rows (measured on 4096 x 4096
    // up to 28672 -> 8192: fewer publish t too late for the gather workgroups' rows of U_r^T, more only add atomics) ...
    // By default only where it was measured to pay: in launches that read 2^26 weights or more (t is published one
    // dependent phase later than by the row dots, which a shorter launch does not hide), and at four tokens under the
    // union mask (hardly any channel is dropped then, so stage 1 reads almost nothing).  lowrank_wgs > 0 forces it.
    const size_t lw = launch_weights ? launch_weights : (size_t)L->cfg.d_in * L->cfg.d_out;
    const bool union_now = L->cfg.batch_mask_mode == 1 || (L->cfg.batch_mask_mode == 2 && batch >= 4);
    const bool pays = lw >= ((size_t)1 << 26) || (bt == 4 && union_now);
    if (fused && !dense && bt <= 4 && L->SVc && L->cfg.rank > 0 && (t.lowrank_wgs > 0 || (t.lowrank_wgs == 0 && pays))) {
        const double s1_bytes = 2.0 * L->cfg.rank * (L->cfg.d_in - rows);
        // ... as many as the resident slots (two per compute unit, shared by the layers of a group) that this layer's
        // gather workgroups leave free, between 16 and that number (measured: gate/up grouped 32 each, q/k/v grouped
        // 42 + 64 + 64, o 64, down 128 -- a launch that needs a second round of workgroups loses more)
        const int base = s1_bytes >= 16.0 * 1024 * 1024 ? 128 : 64;
        const int free_slots = 2 * L->cus / std::max(1, group) - L->tiles * splits;
        c.lowrank_wgs = t.lowrank_wgs > 0 ? t.lowrank_wgs : std::max(16, std::min(base, free_slots));
        // skinny layers (d_out of the order of the rank: the k / v projections of grouped-query attention), where stage 1
        // is half or more of what the gather workgroups read: 128 whatever the slots (measured in the q/k/v group of
        // 8192 -> 8192 / 1024 / 1024, r = 1024: 30.2 us against 32.0 us)
        const double gather_bytes = 2.0 * ((double)rows + L->cfg.rank) * L->cfg.d_out;
        if (t.lowrank_wgs == 0 && 2.0 * s1_bytes >= gather_bytes) c.lowrank_wgs = 128;
    }
    return c;
}

// Launch shape of the strip kernel: one workgroup per strip when the launch then still has a workgroup for at
// least half of the compute units; layers with fewer strips split the channels over several workgroups per strip.
Launch resolve_strip(const rsparse_layer *L, int batch, bool dense, int group, bool fused)
{
    Launch c{};
    const rsparse_tuning &t = L->tuning;
    const int bt = batch_tile_of(batch);
    c.waves = strip_waves(batch);
    c.nontemporal = 1;
    c.tile_map = 1;
    c.wait_polls = t.debug_wait_polls;
    c.skip_stage1 = t.debug_skip_stage1 ? 1 : 0;
    const int rank = dense ? 0 : L->cfg.rank;
    int splits = t.splits;
    if (splits <= 0) {
        // measured: small layers (under 2^26 weights) run best at about one workgroup per two compute units, large
        // ones at one per compute unit, the linears of a grouped call sharing that number
        const bool large = (size_t)L->cfg.d_in * L->cfg.d_out >= ((size_t)1 << 26);
        const int target = std::max(1, (large ? L->cus : L->cus / 2) / std::max(1, group));
        splits = std::max(1, (target + L->strips / 2) / L->strips);
    }
    splits = std::max(1, std::min(splits, 4096));
    while (strip_list_cap(L->cfg.d_in, rank, splits, c.waves, bt, L->strip_w) <= 0 && splits < 4096) ++splits;
    c.splits = splits;
    // stage 1: a row of S_r V_r^T is shared by enough waves that a wave's part is one batch of loads (8 KiB), as long
    // as that leaves at most about one stage-1 workgroup per compute unit
    const int chunk = std::min(L->cfg.d_in, (24576 / bt) & ~7);
    int ws = 1;
    while (ws < c.waves && chunk * 2 / ws > 8192) ws *= 2;
    int rpw = c.waves / ws;
    while (rpw < c.waves && (L->cfg.rank + rpw - 1) / rpw > L->cus / std::max(1, group)) rpw *= 2;
    if (t.lowrank_rows > 0) {
        rpw = 1;
        while (rpw * 2 <= std::min(t.lowrank_rows, c.waves)) rpw *= 2;
    }
    c.lowrank_rows = rpw;
    (void)fused;
    return c;
}

rsparse_status check_call(rsparse_layer *L, const void *X, int32_t batch, void *Y)
{
    if (!L) return fail(RSPARSE_EINVAL, "layer is NULL");
    if (!X || !Y) return fail(RSPARSE_EINVAL, "X and Y must be non-NULL device pointers");
    if (batch < 1 || batch > L->cfg.max_batch)
        return fail(RSPARSE_EBATCH, "batch %d outside [1, max_batch=%d]", batch, L->cfg.max_batch);
    if (((uintptr_t)X & 15u) || ((uintptr_t)Y & 15u)) return fail(RSPARSE_EALIGN, "X and Y must be 16-byte aligned");
    return RSPARSE_OK;
}

void free_layer(rsparse_layer *L)
{
    if (!L) return;
    (void)hipFree(L->M); (void)hipFree(L->SVt); (void)hipFree(L->U); (void)hipFree(L->Wrow); (void)hipFree(L->t);
    (void)hipFree(L->yacc); (void)hipFree(L->act_bits); (void)hipFree(L->chan_bits);
    (void)hipFree(L->act_list); (void)hipFree(L->act_count); (void)hipFree(L->sync); (void)hipFree(L->t_pub); (void)hipFree(L->xg); (void)hipFree(L->hy);
    (void)hipFree(L->Ms); (void)hipFree(L->t_tag); (void)hipFree(L->act_seg); (void)hipFree(L->bias); (void)hipFree(L->rules); (void)hipFree(L->t_acc); (void)hipFree(L->SVc); (void)hipFree(L->t_sum); (void)hipFree(L->t16);
    (void)hipFree(L->Mq); (void)hipFree(L->qs); (void)hipFree(L->qz); (void)hipFree(L->Ut);
    (void)hipFree(L->Qrow); (void)hipFree(L->Srow); (void)hipFree(L->Zrow);
    delete L;
}

// 4-bit weights as the caller hands them over (rsparse_prepare_q4); all host pointers.
struct Q4Host {
    const uint8_t *Q;        // [d_out][d_in] codes
    const uint16_t *S16;     // [d_out][d_in / group]
    const uint8_t *Z;        // [d_out][d_in / group]
    int group;
};

rsparse_status build_layer(const rsparse_config *cfg, const uint16_t *W, const uint16_t *U16, const uint16_t *SV16,
                           rsparse_layer **out, const Q4Host *q4 = nullptr)
{
    rsparse_layer *L = new (std::nothrow) rsparse_layer();
    if (!L) return fail(RSPARSE_ENOMEM, "host allocation failed");
    L->cfg = *cfg;
    const size_t d_in = cfg->d_in, d_out = cfg->d_out, r = cfg->rank;
    L->tiles = (int)((d_out + kTile - 1) / kTile);
    // (the 4-bit kernels hold at most 4 tokens per batch tile)
    L->nz_max = std::max(1, q4 ? (cfg->max_batch + 3) / 4 : (cfg->max_batch + kMaxBT - 1) / kMaxBT);

    rsparse_status st = RSPARSE_OK;
    auto body = [&]() -> rsparse_status {
        RS_HIP(hipGetDevice(&L->device));
        hipDeviceProp_t prop;
        RS_HIP(hipGetDeviceProperties(&prop, L->device));
        L->cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

        // pack W column-major: row c of M = W[:, c]; rows d_in.. = U_r^T (row d_in + j = U_r[:, j]), which the
        // one-launch kernel streams as r more channels
        std::vector<uint16_t> host;
        try {
            if (!q4) host.resize((d_in + r) * d_out);
            if (r) { L->U16.assign(U16, U16 + d_out * r); L->SV16.assign(SV16, SV16 + r * d_in); }
        } catch (const std::bad_alloc &) { return fail(RSPARSE_ENOMEM, "host allocation failed"); }
        if (!q4) {
            transpose16(W, d_out, d_in, host.data());
            if (r) transpose16(U16, d_out, r, host.data() + d_in * d_out);
            if (cfg->strip_cols == 0) {
                RS_HIP(hipMalloc((void **)&L->M, host.size() * 2));
                RS_HIP(hipMemcpy(L->M, host.data(), host.size() * 2, hipMemcpyHostToDevice));
            } else {
            // strip layout: the same rows cut into strips of strip_cols columns, strip after strip (columns past
            // d_out are zero); the strip kernel gives each strip to one workgroup (or to a few that split the channels)
            const int sw = cfg->strip_cols;
            L->strip_w = sw;
            L->strips = (int)((d_out + sw - 1) / sw);
            const size_t rows = d_in + r, W = sw;
            L->strip_stride = (long long)(rows * W);
            std::vector<uint16_t> ms;
            try { ms.assign((size_t)L->strips * rows * W, 0); } catch (const std::bad_alloc &) { return fail(RSPARSE_ENOMEM, "host allocation failed"); }
            parallel_for(rows, [&](size_t c) {
                const uint16_t *src = host.data() + c * d_out;
                for (size_t o = 0; o < d_out; ++o) ms[((o / W) * rows + c) * W + (o % W)] = src[o];
            });
            RS_HIP(hipMalloc((void **)&L->Ms, ms.size() * 2));
            RS_HIP(hipMemcpy(L->Ms, ms.data(), ms.size() * 2, hipMemcpyHostToDevice));
            }
        } else {
            // codes channel-major in the lane order of the 4-bit kernel (layout: kernels.h), scales and zero
            // points group-major in plain column order; rows padded to whole 1024-column tiles with zeros
            L->qtiles = (int)((d_out + kQ4Tile - 1) / kQ4Tile);
            L->qshift = 0;
            while ((1 << L->qshift) < q4->group) ++L->qshift;
            const size_t G = d_in >> L->qshift, ldq = (size_t)L->qtiles * (kQ4Tile / 2), lds = (size_t)L->qtiles * kQ4Tile;
            std::vector<uint8_t> mq, zq;
            std::vector<uint16_t> sq;
            try {
                mq.assign(d_in * ldq, 0); zq.assign(G * lds, 0); sq.assign(G * lds, 0);
            } catch (const std::bad_alloc &) { return fail(RSPARSE_ENOMEM, "host allocation failed"); }
            parallel_for(d_in, [&](size_t c) {
                for (size_t o = 0; o < d_out; ++o) {
                    const size_t T = o / kQ4Tile, within = o % kQ4Tile;
                    const size_t h = within / 512, l = (within % 512) / 8, e = within % 8;
                    const size_t byte = c * ldq + T * (kQ4Tile / 2) + l * 8 + h * 4 + (e & 3);
                    const uint8_t code = q4->Q[o * d_in + c] & 15u;
                    mq[byte] |= (uint8_t)(e < 4 ? code : code << 4);
                }
            });
            for (size_t o = 0; o < d_out; ++o)
                for (size_t g = 0; g < G; ++g) {
                    sq[g * lds + o] = q4->S16[o * G + g];
                    zq[g * lds + o] = q4->Z[o * G + g];
                }
            RS_HIP(hipMalloc((void **)&L->Mq, mq.size()));
            RS_HIP(hipMemcpy(L->Mq, mq.data(), mq.size(), hipMemcpyHostToDevice));
            RS_HIP(hipMalloc((void **)&L->qs, sq.size() * 2));
            RS_HIP(hipMemcpy(L->qs, sq.data(), sq.size() * 2, hipMemcpyHostToDevice));
            RS_HIP(hipMalloc((void **)&L->qz, zq.size()));
            RS_HIP(hipMemcpy(L->qz, zq.data(), zq.size(), hipMemcpyHostToDevice));
            if (cfg->dense_rowmajor && q4->group >= 32 && (d_in % 32) == 0) {
                // row-major copy for the row-dot dense baseline: two codes per byte, channel 2j in the low nibble
                std::vector<uint8_t> qr;
                try { qr.assign(d_out * (d_in / 2), 0); } catch (const std::bad_alloc &) { return fail(RSPARSE_ENOMEM, "host allocation failed"); }
                parallel_for(d_out, [&](size_t o) {
                    for (size_t j = 0; j < d_in / 2; ++j)
                        qr[o * (d_in / 2) + j] = (uint8_t)((q4->Q[o * d_in + 2 * j] & 15u) | ((q4->Q[o * d_in + 2 * j + 1] & 15u) << 4));
                });
                RS_HIP(hipMalloc((void **)&L->Qrow, qr.size()));
                RS_HIP(hipMemcpy(L->Qrow, qr.data(), qr.size(), hipMemcpyHostToDevice));
                RS_HIP(hipMalloc((void **)&L->Srow, d_out * G * 2));
                RS_HIP(hipMemcpy(L->Srow, q4->S16, d_out * G * 2, hipMemcpyHostToDevice));
                RS_HIP(hipMalloc((void **)&L->Zrow, d_out * G));
                RS_HIP(hipMemcpy(L->Zrow, q4->Z, d_out * G, hipMemcpyHostToDevice));
            }
            if (r) {
                // U_r^T with rows padded to whole tiles, for the one-launch kernel
                std::vector<uint16_t> ut;
                try { ut.assign(r * lds, 0); } catch (const std::bad_alloc &) { return fail(RSPARSE_ENOMEM, "host allocation failed"); }
                for (size_t o = 0; o < d_out; ++o)
                    for (size_t j = 0; j < r; ++j) ut[j * lds + o] = U16[o * r + j];
                RS_HIP(hipMalloc((void **)&L->Ut, ut.size() * 2));
                RS_HIP(hipMemcpy(L->Ut, ut.data(), ut.size() * 2, hipMemcpyHostToDevice));
            }
        }
        if (r) {
            RS_HIP(hipMalloc((void **)&L->SVt, r * d_in * 2));
            RS_HIP(hipMemcpy(L->SVt, SV16, r * d_in * 2, hipMemcpyHostToDevice));
            RS_HIP(hipMalloc((void **)&L->U, d_out * r * 2));
            RS_HIP(hipMemcpy(L->U, U16, d_out * r * 2, hipMemcpyHostToDevice));
        }
        if (cfg->lowrank_channel_major && !q4 && r) {
            std::vector<uint16_t> svc(d_in * r);
            transpose16(SV16, r, d_in, svc.data());
            RS_HIP(hipMalloc((void **)&L->SVc, d_in * r * 2));
            RS_HIP(hipMemcpy(L->SVc, svc.data(), d_in * r * 2, hipMemcpyHostToDevice));
            const size_t n_sum = r * (size_t)L->nz_max * kMaxBT;
            RS_HIP(hipMalloc((void **)&L->t_sum, n_sum * 4));
            RS_HIP(hipMemset(L->t_sum, 0, n_sum * 4));
        }
        if (cfg->dense_rowmajor && !q4) {
            RS_HIP(hipMalloc((void **)&L->Wrow, d_in * d_out * 2));
            RS_HIP(hipMemcpy(L->Wrow, W, d_in * d_out * 2, hipMemcpyHostToDevice));
        }
        if (cfg->dense_rowmajor && !q4 && r) {
            RS_HIP(hipMalloc((void **)&L->t_acc, (size_t)32 * r * 4));
            RS_HIP(hipMemset(L->t_acc, 0, (size_t)32 * r * 4));
            RS_HIP(hipMalloc((void **)&L->t16, (size_t)2 * 32 * r * 2));
            RS_HIP(hipMemset(L->t16, 0, (size_t)2 * 32 * r * 2));
        }
        RS_HIP(hipMalloc((void **)&L->xg, (size_t)cfg->max_batch * d_in * 2));
        RS_HIP(hipMalloc((void **)&L->hy, (size_t)cfg->max_batch * d_out * 2));
        const size_t bpad = (size_t)L->nz_max * kMaxBT;
        const size_t n_t = std::max<size_t>(1, r * bpad);
        // the matrix-core kernels keep these accumulators as [d_out][16 or 32 tokens]
        const size_t n_y = (size_t)(cfg->dense_rowmajor ? std::max(cfg->max_batch, cfg->max_batch > 16 ? 32 : 16)
                                                          : cfg->max_batch) * d_out;
        L->n_y = n_y;
        const size_t n_list = (size_t)L->nz_max * d_in;
        RS_HIP(hipMalloc((void **)&L->t, n_t * 4));
        RS_HIP(hipMalloc((void **)&L->yacc, n_y * 4));
        RS_HIP(hipMalloc((void **)&L->act_list, n_list * 4));
        RS_HIP(hipMalloc((void **)&L->act_bits, n_list * 4));
        RS_HIP(hipMalloc((void **)&L->act_count, (size_t)L->nz_max * 4));
        RS_HIP(hipMalloc((void **)&L->chan_bits, d_in * 4));
        RS_HIP(hipMalloc((void **)&L->rules, (size_t)cfg->max_batch * sizeof(KeepRule)));
        RS_HIP(hipMemset(L->rules, 0, (size_t)cfg->max_batch * sizeof(KeepRule)));
        L->sync_n = sync_words(std::max(L->tiles, L->strips));
        RS_HIP(hipMalloc((void **)&L->sync, L->sync_n * 4));
        RS_HIP(hipMemset(L->sync, 0, L->sync_n * 4));
        {
            const int one = 1;                        // generation 1: no entry of t_tag (all zero) carries it
            RS_HIP(hipMemcpy(L->sync + kSyncGen, &one, 4, hipMemcpyHostToDevice));
        }
        L->t_slots = (int)bpad;
        RS_HIP(hipMalloc((void **)&L->t_tag, n_t * 8));
        RS_HIP(hipMemset(L->t_tag, 0, n_t * 8));
        RS_HIP(hipMalloc((void **)&L->act_seg, (size_t)L->nz_max * (d_in / 8) * 4));
        RS_HIP(hipMemset(L->act_seg, 0, (size_t)L->nz_max * (d_in / 8) * 4));
        L->n_t = n_t;
        RS_HIP(hipMalloc((void **)&L->t_pub, n_t * 4));
        RS_HIP(hipMemset(L->t_pub, 0xff, n_t * 4));          // every entry "not ready"
        RS_HIP(hipMemset(L->chan_bits, 0, d_in * 4));
        RS_HIP(hipMemset(L->t, 0, n_t * 4));
        RS_HIP(hipMemset(L->yacc, 0, n_y * 4));
        RS_HIP(hipMemset(L->act_list, 0, n_list * 4));
        RS_HIP(hipMemset(L->act_bits, 0, n_list * 4));
        RS_HIP(hipMemset(L->act_count, 0, (size_t)L->nz_max * 4));
        RS_HIP(hipDeviceSynchronize());
        return RSPARSE_OK;
    };
    st = body();
    if (st != RSPARSE_OK) { free_layer(L); return st; }
    *out = L;
    return RSPARSE_OK;
}

}  // namespace

extern "C" {

const char *rsparse_last_error(void) { return g_err; }

rsparse_status rsparse_prepare_factors(const rsparse_config *cfg, const void *W_host, const void *U16_host,
                                       const void *SV16_host, rsparse_layer **out)
{
    if (!out) return fail(RSPARSE_EINVAL, "out is NULL");
    *out = nullptr;
    rsparse_status st = check_config(cfg);
    if (st != RSPARSE_OK) return st;
    if (!W_host) return fail(RSPARSE_EINVAL, "W_host is NULL");
    if (cfg->rank > 0 && (!U16_host || !SV16_host)) return fail(RSPARSE_EINVAL, "factors are NULL but rank > 0");
    return build_layer(cfg, (const uint16_t *)W_host, (const uint16_t *)U16_host, (const uint16_t *)SV16_host, out);
}

rsparse_status rsparse_compute_factors(const rsparse_config *cfg, const void *W_host, void *U16_host,
                                       void *SV16_host, double *sigma_host)
{
    rsparse_status st = check_config(cfg);
    if (st != RSPARSE_OK) return st;
    if (!W_host) return fail(RSPARSE_EINVAL, "W_host is NULL");
    const size_t d_in = cfg->d_in, d_out = cfg->d_out, r = cfg->rank;
    if (r == 0) return RSPARSE_OK;
    if (!U16_host || !SV16_host) return fail(RSPARSE_EINVAL, "factor buffers are NULL but rank > 0");
    std::vector<double> W, U, S, V;
    try {
        W.resize(d_in * d_out);
        U.resize(d_out * r); S.resize(r); V.resize(d_in * r);
    } catch (const std::bad_alloc &) { return fail(RSPARSE_ENOMEM, "host allocation failed"); }
    const uint16_t *w16 = (const uint16_t *)W_host;
    const int dt = cfg->dtype;
    parallel_for(d_out, [&](size_t o) {
        for (size_t c = 0; c < d_in; ++c) W[o * d_in + c] = (double)widen16(w16[o * d_in + c], dt);
    });
    char msg[256] = "";
    if (svd_top_r(W.data(), (int)d_out, (int)d_in, (int)r, U.data(), S.data(), V.data(), msg, sizeof msg) != 0)
        return fail(RSPARSE_ESVD, "host SVD failed: %s", msg);
    // U_r [d_out][r];  S_r V_r^T [r][d_in]; each rounded once to the storage type
    uint16_t *U16 = (uint16_t *)U16_host, *SV16 = (uint16_t *)SV16_host;
    for (size_t o = 0; o < d_out; ++o)
        for (size_t i = 0; i < r; ++i)
            U16[o * r + i] = dt == RSPARSE_F16 ? double_to_f16(U[o * r + i]) : double_to_bf16(U[o * r + i]);
    for (size_t i = 0; i < r; ++i)
        for (size_t c = 0; c < d_in; ++c) {
            const double v = S[i] * V[c * r + i];
            SV16[i * d_in + c] = dt == RSPARSE_F16 ? double_to_f16(v) : double_to_bf16(v);
        }
    if (sigma_host) memcpy(sigma_host, S.data(), r * sizeof(double));
    return RSPARSE_OK;
}

rsparse_status rsparse_prepare(const rsparse_config *cfg, const void *W_host, rsparse_layer **out)
{
    if (!out) return fail(RSPARSE_EINVAL, "out is NULL");
    *out = nullptr;
    rsparse_status st = check_config(cfg);
    if (st != RSPARSE_OK) return st;
    if (!W_host) return fail(RSPARSE_EINVAL, "W_host is NULL");
    std::vector<uint16_t> U16, SV16;
    try {
        U16.resize((size_t)cfg->d_out * cfg->rank);
        SV16.resize((size_t)cfg->rank * cfg->d_in);
    } catch (const std::bad_alloc &) { return fail(RSPARSE_ENOMEM, "host allocation failed"); }
    st = rsparse_compute_factors(cfg, W_host, U16.data(), SV16.data(), nullptr);
    if (st != RSPARSE_OK) return st;
    return build_layer(cfg, (const uint16_t *)W_host, U16.data(), SV16.data(), out);
}

rsparse_status rsparse_prepare_q4(const rsparse_config *cfg, const uint8_t *Q_host, const void *S16_host,
                                  const uint8_t *Z_host, int32_t group_size, const void *U16_host,
                                  const void *SV16_host, rsparse_layer **out)
{
    if (!out) return fail(RSPARSE_EINVAL, "out is NULL");
    *out = nullptr;
    rsparse_status st = check_config(cfg);
    if (st != RSPARSE_OK) return st;
    if (!Q_host || !S16_host || !Z_host) return fail(RSPARSE_EINVAL, "Q_host, S16_host and Z_host must be non-NULL");
    if (cfg->rank > 0 && (!U16_host || !SV16_host)) return fail(RSPARSE_EINVAL, "factors are NULL but rank > 0");
    if (group_size < 32 || group_size > 1024 || (group_size & (group_size - 1)) || cfg->d_in % group_size)
        return fail(RSPARSE_EINVAL, "group_size must be a power of two in [32, 1024] that divides d_in (got %d)", group_size);
    if (cfg->strip_cols) return fail(RSPARSE_EINVAL, "strip_cols is not available with 4-bit weights");
    if (cfg->topk) return fail(RSPARSE_EINVAL, "the fixed-count activation (topk > 0) is not available with 4-bit weights");
    const size_t n = (size_t)cfg->d_in * cfg->d_out, ng = n / group_size;
    for (size_t i = 0; i < n; ++i)
        if (Q_host[i] > 15) return fail(RSPARSE_EINVAL, "code %u at %zu is not a 4-bit value", (unsigned)Q_host[i], i);
    for (size_t i = 0; i < ng; ++i)
        if (Z_host[i] > 15) return fail(RSPARSE_EINVAL, "zero point %u at %zu is not a 4-bit value", (unsigned)Z_host[i], i);
    const Q4Host q4{Q_host, (const uint16_t *)S16_host, Z_host, group_size};
    return build_layer(cfg, nullptr, (const uint16_t *)U16_host, (const uint16_t *)SV16_host, out, &q4);
}

namespace {

// Launch shape of the 4-bit kernel: the weight stream is a quarter of the 16-bit one, so fewer, 4-wave
// workgroups with longer contiguous runs (a wave folds scale and zero point once per quantisation group it meets).
Launch resolve_launch_q4(const rsparse_layer *L, int batch, bool dense, bool fused)
{
    Launch c{};
    const rsparse_tuning &t = L->tuning;
    const int bt = std::min(4, batch_tile_of(batch));
    c.waves = (t.waves == 1 || t.waves == 2 || t.waves == 4 || t.waves == 8) ? t.waves : 4;
    if (bt >= 4 && c.waves > 4) c.waves = 4;         // the 4-token kernel is built for at most 256 lanes
    c.nontemporal = t.nontemporal == 2 ? 0 : 1;
    c.tile_map = 1;
    const int rows = dense ? L->cfg.d_in : std::max(8, L->cfg.d_in / 2);
    int splits = t.splits;
    if (splits <= 0) {
        const int target_wgs = std::max(L->qtiles, 2 * L->cus);
        splits = (target_wgs + L->qtiles - 1) / L->qtiles;
        splits = std::max(1, std::min(splits, std::max(1, rows / (c.waves * 8))));      // >= 8 rows per wave
    }
    splits = std::min(splits, 4096);
    while (gather_lds_bytes(L->cfg.d_in, splits, c.waves, bt, fused ? L->cfg.rank : 0) > 60 * 1024 && splits < 65536) splits *= 2;
    c.splits = splits;
    c.wait_polls = t.debug_wait_polls;
    c.skip_stage1 = t.debug_skip_stage1 ? 1 : 0;
    int lr = t.lowrank_rows;
    if (lr <= 0) {
        const double wg_bytes = (double)rows / splits * (kQ4Tile / 2);
        lr = (int)(wg_bytes / (2.0 * L->cfg.d_in) + 0.5);
        lr = std::max(lr, c.waves);                                                      // a row for every wave
    }
    c.lowrank_rows = std::max(1, std::min(lr, 4 * c.waves));
    // one launch: stage 1 is cut as fine as the resident slots that the gather workgroups leave free allow
    // (the rule of the 16-bit kernel), so that t is there when the rows of U_r^T come up
    if (fused && t.lowrank_rows <= 0) {
        const int free_slots = 2 * L->cus - L->qtiles * splits;
        const int need = free_slots > 0 ? (L->cfg.rank + free_slots - 1) / free_slots : 4 * c.waves;
        c.lowrank_rows = std::max(std::max(1, c.waves / 2), std::min(4 * c.waves, need));
    }
    return c;
}

// One layer with 4-bit weights: first launch (codes dequantised in registers), then the common finish.
rsparse_status linear_q4(rsparse_layer *L, const void *X_dev, int32_t batch, void *Y_dev, bool dense, hipStream_t s)
{
    const LayerView v = L->view(nullptr, batch, dense);
    const int stages = L->tuning.stages;
    // two launches by default: the one-launch form (launches = 1) measured no faster on these weights --
    // its tail waits for up to `splits` same-address atomics that the two-launch form never waits for
    // (its arrival counters cover up to kSyncMaxZ batch tiles of 4 tokens)
    const bool fused = !dense && L->tuning.launches == 1 && stages == 0 && (batch + 3) / 4 <= kSyncMaxZ;
    const Launch lc = resolve_launch_q4(L, batch, dense, fused);
    if (fused) {
        RS_HIP(launch_q4(v, lc, X_dev, batch, true, false, Y_dev, s));
    } else {
        if (stages != 2) RS_HIP(launch_q4(v, lc, X_dev, batch, true, dense, nullptr, s));
        if (stages != 1) RS_HIP(launch_finish(&v, 1, batch, &Y_dev, !dense, s));
    }
    if (!dense) {
        L->last_stream = s; L->last_batch = batch; L->last_mfma = false; L->last_fused = fused;
        L->last_scratch = L->own_scratch();
        L->last_bt = std::min(4, batch_tile_of(batch));
        L->last_strip = false;
    }
    return RSPARSE_OK;
}

rsparse_status check_group(rsparse_layer *const *layers, int32_t n, const void *X, int32_t batch, void *const *Y)
{
    if (!layers || !Y) return fail(RSPARSE_EINVAL, "layers and Y_devs must be non-NULL");
    if (n < 1 || n > RSPARSE_MAX_GROUP) return fail(RSPARSE_EINVAL, "n_layers %d outside [1, %d]", n, RSPARSE_MAX_GROUP);
    for (int i = 0; i < n; ++i) {
        rsparse_status st = check_call(layers[i], X, batch, Y[i]);
        if (st != RSPARSE_OK) return st;
        if (layers[i]->cfg.d_in != layers[0]->cfg.d_in || layers[i]->cfg.dtype != layers[0]->cfg.dtype)
            return fail(RSPARSE_EINVAL, "grouped layers must share d_in and dtype");
        for (int k = 0; k < i; ++k)
            if (layers[k] == layers[i]) return fail(RSPARSE_EINVAL, "a layer appears twice in the group");
    }
    return RSPARSE_OK;
}

}  // namespace

namespace {
rsparse_status linear_group_impl(rsparse_layer *const *layers, int32_t n_layers, const void *X_dev, const void *G_dev,
                                 int32_t batch, void *const *Y_devs, void *stream, const ScratchView *ov = nullptr);
}

rsparse_status rsparse_linear_group(rsparse_layer *const *layers, int32_t n_layers, const void *X_dev, int32_t batch,
                                    void *const *Y_devs, void *stream)
{
    return linear_group_impl(layers, n_layers, X_dev, nullptr, batch, Y_devs, stream);
}

rsparse_status rsparse_gated_input(const void *G_dev, const void *Up_dev, void *out_dev, size_t n, int32_t dtype,
                                   void *stream)
{
    if (!G_dev || !Up_dev || !out_dev) return fail(RSPARSE_EINVAL, "NULL device pointer");
    if (dtype != RSPARSE_F16 && dtype != RSPARSE_BF16) return fail(RSPARSE_EINVAL, "dtype must be F16 or BF16");
    if (n == 0 || (n % 8) != 0) return fail(RSPARSE_EINVAL, "n must be a positive multiple of 8");
    if (((uintptr_t)G_dev | (uintptr_t)Up_dev | (uintptr_t)out_dev) & 15u)
        return fail(RSPARSE_EALIGN, "buffers must be 16-byte aligned");
    RS_HIP(launch_gated_input(G_dev, Up_dev, out_dev, n, dtype, (hipStream_t)stream));
    return RSPARSE_OK;
}

rsparse_status rsparse_linear_gated(rsparse_layer *L, const void *G_dev, const void *Up_dev, int32_t batch, void *Y_dev,
                                    void *stream)
{
    if (!G_dev) return fail(RSPARSE_EINVAL, "G_dev is NULL");
    if ((uintptr_t)G_dev & 15u) return fail(RSPARSE_EALIGN, "G_dev must be 16-byte aligned");
    return linear_group_impl(&L, 1, Up_dev, G_dev, batch, &Y_dev, stream);
}

namespace {
// ov: per-call scratch to use instead of the handles' own (rsparse_linear_static; one layer, vector path only)
rsparse_status linear_group_impl(rsparse_layer *const *layers, int32_t n_layers, const void *X_dev, const void *G_dev,
                                 int32_t batch, void *const *Y_devs, void *stream, const ScratchView *ov)
{
    rsparse_status st = check_group(layers, n_layers, X_dev, batch, Y_devs);
    if (st != RSPARSE_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    bool any_q4 = false;
    for (int i = 0; i < n_layers; ++i) any_q4 = any_q4 || layers[i]->q4();
    if (any_q4) {
        // layers with 4-bit weights run one at a time, each in its own pair of launches
        if (G_dev) {
            RS_HIP(launch_gated_input(G_dev, X_dev, layers[0]->xg, (size_t)batch * layers[0]->cfg.d_in, layers[0]->cfg.dtype, s));
            X_dev = layers[0]->xg;
        }
        for (int i = 0; i < n_layers; ++i) {
            rsparse_status qs = layers[i]->q4() ? linear_q4(layers[i], X_dev, batch, Y_devs[i], false, s)
                                                : linear_group_impl(&layers[i], 1, X_dev, nullptr, batch, &Y_devs[i], stream);
            if (qs != RSPARSE_OK) return qs;
        }
        return RSPARSE_OK;
    }
    LayerView v[RSPARSE_MAX_GROUP];
    Launch lc[RSPARSE_MAX_GROUP];
    const int stages = layers[0]->tuning.stages;
    // one launch unless asked otherwise (timing a stage alone needs the two-launch form)
    const bool fused = layers[0]->tuning.launches != 2 && stages == 0;
    size_t launch_weights = 0;
    for (int i = 0; i < n_layers; ++i) launch_weights += (size_t)layers[i]->cfg.d_in * layers[i]->cfg.d_out;
    for (int i = 0; i < n_layers; ++i) {
        v[i] = layers[i]->view(ov, batch);
        lc[i] = resolve_launch(layers[i], batch, false, n_layers, i ? lc[0].waves : 0, fused, launch_weights);
        layers[i]->last_scratch = ov ? *ov : layers[i]->own_scratch();
    }
    bool mfma = !ov && batch >= (layers[0]->tuning.mfma_min_batch > 0 ? layers[0]->tuning.mfma_min_batch : kMfmaDefaultMinBatch);
    for (int i = 0; i < n_layers; ++i) mfma = mfma && mfma_path_supported(v[i], batch) && layers[i]->cfg.topk == 0;
    // a gated input is written out once first (one small launch), then the layer runs on it
    if (G_dev) {
        RS_HIP(launch_gated_input(G_dev, X_dev, layers[0]->xg, (size_t)batch * layers[0]->cfg.d_in, layers[0]->cfg.dtype, s));
        X_dev = layers[0]->xg;
    }
    // fixed-count activation: each token's rule (its k-th magnitude and tie cut) first, one small launch per layer
    for (int i = 0; i < n_layers; ++i)
        if (layers[i]->cfg.topk > 0 && v[i].rules)
            RS_HIP(launch_topk_rules(X_dev, layers[i]->cfg.dtype, batch, layers[i]->cfg.d_in, layers[i]->cfg.topk,
                                     const_cast<KeepRule *>(v[i].rules), s));
    // layers packed in strips go through the strip kernel; a group must share one layout (and one strip width),
    // otherwise its layers run one at a time
    if (!mfma && n_layers > 1) {
        bool same = true;
        for (int i = 1; i < n_layers; ++i) same = same && layers[i]->strip_w == layers[0]->strip_w;
        if (!same) {
            for (int i = 0; i < n_layers; ++i) {
                rsparse_status one = linear_group_impl(&layers[i], 1, X_dev, nullptr, batch, &Y_devs[i], stream);
                if (one != RSPARSE_OK) return one;
            }
            return RSPARSE_OK;
        }
    }
    const bool strip = !mfma && layers[0]->Ms != nullptr;
    if (strip) {
        Launch sc[RSPARSE_MAX_GROUP];
        for (int i = 0; i < n_layers; ++i) sc[i] = resolve_strip(layers[i], batch, false, n_layers, fused);
        if (fused) {
            RS_HIP(launch_strip(v, sc, n_layers, X_dev, batch, Y_devs, true, false, layers[0]->cus, s));
        } else {
            if (stages != 2) RS_HIP(launch_sparse_and_t(v, lc, n_layers, X_dev, batch, true, false, s));
            if (stages != 1) RS_HIP(launch_strip(v, sc, n_layers, X_dev, batch, Y_devs, false, false, layers[0]->cus, s));
        }
        for (int i = 0; i < n_layers; ++i) {
            layers[i]->last_stream = s;
            layers[i]->last_batch = batch;
            layers[i]->last_mfma = false;
            layers[i]->last_fused = true;           // rsparse_synchronize looks at the device-side error word
            layers[i]->last_bt = 0;
            layers[i]->last_strip = true;
            layers[i]->last_ranges = sc[i].splits * sc[i].waves;
        }
        return RSPARSE_OK;
    }
    if (mfma) {
        // matrix-core path, one layer at a time (each is already a full-chip launch)
        for (int i = 0; i < n_layers; ++i)
            RS_HIP(launch_mfma_linear(v[i], X_dev, batch, Y_devs[i], layers[i]->chan_bits, layers[i]->cus, stages, false, layers[0]->tuning.mfma_rows, s));
    } else if (fused) {
        RS_HIP(launch_fused(v, lc, n_layers, X_dev, batch, Y_devs, s));
    } else {
        if (stages != 2) RS_HIP(launch_sparse_and_t(v, lc, n_layers, X_dev, batch, true, true, s));
        if (stages != 1) RS_HIP(launch_finish(v, n_layers, batch, Y_devs, true, s));
    }
    for (int i = 0; i < n_layers; ++i) {
        layers[i]->last_stream = s;
        layers[i]->last_batch = batch;
        layers[i]->last_mfma = mfma;
        layers[i]->last_fused = !mfma && fused;
        layers[i]->last_bt = 0;
        layers[i]->last_strip = false;
    }
    return RSPARSE_OK;
}
}  // namespace

rsparse_status rsparse_mlp_gate_up(rsparse_layer *gate, rsparse_layer *up, const void *X_dev, int32_t batch,
                                   void *H_dev, void *stream)
{
    rsparse_layer *pair[2] = {gate, up};
    void *outs[2] = {H_dev, H_dev};
    rsparse_status st = check_group(pair, 2, X_dev, batch, outs);
    if (st != RSPARSE_OK) return st;
    if (gate->cfg.d_out != up->cfg.d_out) return fail(RSPARSE_EINVAL, "gate and up must have the same d_out");
    if (gate->cfg.out_dtype != gate->cfg.dtype || up->cfg.out_dtype != up->cfg.dtype)
        return fail(RSPARSE_EINVAL, "rsparse_mlp_gate_up needs out_dtype == dtype on both layers");
    hipStream_t s = (hipStream_t)stream;
    const int stages = gate->tuning.stages;
    const bool fused = gate->tuning.launches != 2 && stages == 0;
    LayerView v[2];
    Launch lc[2];
    for (int i = 0; i < 2; ++i) {
        v[i] = pair[i]->view(nullptr, batch);
        lc[i] = resolve_launch(pair[i], batch, false, 2, i ? lc[0].waves : 0, fused,
                               (size_t)pair[0]->cfg.d_in * pair[0]->cfg.d_out + (size_t)pair[1]->cfg.d_in * pair[1]->cfg.d_out);
    }
    bool mfma = batch >= (gate->tuning.mfma_min_batch > 0 ? gate->tuning.mfma_min_batch : kMfmaDefaultMinBatch);
    for (int i = 0; i < 2; ++i) mfma = mfma && mfma_path_supported(v[i], batch) && pair[i]->cfg.topk == 0;
    const int bt = batch_tile_of(batch);
    const bool one_tile = (batch + bt - 1) / bt == 1;
    if (fused && !mfma && one_tile && lc[0].tile_map != 2 && lc[1].tile_map != 2 && gate->M && up->M) {
        // both projections and the activation in one launch: the last workgroup of a column tile
        // rounds g and u, applies silu(g) * u and stores H
        for (int i = 0; i < 2; ++i)
            if (pair[i]->cfg.topk > 0)
                RS_HIP(launch_topk_rules(X_dev, pair[i]->cfg.dtype, batch, pair[i]->cfg.d_in, pair[i]->cfg.topk,
                                         const_cast<KeepRule *>(v[i].rules), s));
        RS_HIP(launch_fused(v, lc, 2, X_dev, batch, outs, s, true));
        for (int i = 0; i < 2; ++i) {
            pair[i]->last_stream = s; pair[i]->last_batch = batch; pair[i]->last_mfma = false; pair[i]->last_fused = true; pair[i]->last_bt = 0; pair[i]->last_strip = false;
            pair[i]->last_scratch = pair[i]->own_scratch();
        }
        return RSPARSE_OK;
    }
    // otherwise: the two layers into scratch, then the elementwise recipe
    void *tmp[2] = {gate->hy, up->hy};
    st = rsparse_linear_group(pair, 2, X_dev, batch, tmp, stream);
    if (st != RSPARSE_OK) return st;
    RS_HIP(launch_gated_input(gate->hy, up->hy, H_dev, (size_t)batch * gate->cfg.d_out, gate->cfg.dtype, s));
    return RSPARSE_OK;
}

rsparse_status rsparse_linear(rsparse_layer *L, const void *X_dev, int32_t batch, void *Y_dev, void *stream)
{
    return rsparse_linear_group(&L, 1, X_dev, batch, &Y_dev, stream);
}

rsparse_status rsparse_linear_static(rsparse_layer *L, const void *X_dev, int32_t batch, void *Y_dev, void *stream)
{
    rsparse_status st = check_call(L, X_dev, batch, Y_dev);
    if (st != RSPARSE_OK) return st;
    if (L->q4()) return fail(RSPARSE_EINVAL, "rsparse_linear_static runs 16-bit weights only");
    if (batch > kStaticMaxBatch)
        return fail(RSPARSE_EBATCH, "rsparse_linear_static: batch %d exceeds the static scratch's %d tokens", batch, kStaticMaxBatch);
    if (L->cfg.d_in > kStaticMaxDim || L->cfg.d_out > kStaticMaxDim || L->cfg.rank > kStaticMaxRank)
        return fail(RSPARSE_EINVAL, "rsparse_linear_static: layer %d -> %d, rank %d exceeds the static scratch (d_in, d_out <= %d, rank <= %d)",
                    L->cfg.d_in, L->cfg.d_out, L->cfg.rank, kStaticMaxDim, kStaticMaxRank);
    int dev = -1;
    RS_HIP(hipGetDevice(&dev));
    if (dev != L->device) return fail(RSPARSE_EINVAL, "the layer lives on device %d, the current device is %d", L->device, dev);
    ScratchView sp{};
    RS_HIP(static_scratch_for_call(dev, L->cfg.d_out, L->cfg.rank, batch, (hipStream_t)stream, &sp));
    return linear_group_impl(&L, 1, X_dev, nullptr, batch, &Y_dev, stream, &sp);
}

rsparse_status rsparse_dense_ref_group(rsparse_layer *const *layers, int32_t n_layers, const void *X_dev,
                                       int32_t batch, void *const *Y_devs, void *stream)
{
    rsparse_status st = check_group(layers, n_layers, X_dev, batch, Y_devs);
    if (st != RSPARSE_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    bool any_q4 = false;
    for (int i = 0; i < n_layers; ++i) any_q4 = any_q4 || layers[i]->q4();
    if (any_q4) {
        for (int i = 0; i < n_layers; ++i) {
            rsparse_layer *Lq = layers[i];
            // row-dot over row-major codes when the copy is kept (dense_rowmajor = 1) and asked for or left to the library
            if (Lq->q4() && Lq->Qrow && Lq->tuning.dense_kernel != 1 && q4_rowdot_supported(Lq->cfg.d_in, batch)) {
                RS_HIP(launch_q4_dense_rowdot(Lq->Qrow, Lq->Srow, Lq->Zrow, Lq->qshift, Lq->cfg.dtype, Lq->cfg.out_dtype, Lq->cfg.d_in,
                                              Lq->cfg.d_out, X_dev, batch, Y_devs[i], s));
                continue;
            }
            if (Lq->q4() && Lq->tuning.dense_kernel == 2)
                return fail(RSPARSE_EINVAL, "row-dot dense kernel on 4-bit weights needs dense_rowmajor=1, groups >= 32 and batch_tile*d_in*2.125 <= 64 KiB");
            rsparse_status qs = layers[i]->q4() ? linear_q4(layers[i], X_dev, batch, Y_devs[i], true, s)
                                                : rsparse_dense_ref_group(&layers[i], 1, X_dev, batch, &Y_devs[i], stream);
            if (qs != RSPARSE_OK) return qs;
        }
        return RSPARSE_OK;
    }
    LayerView v[RSPARSE_MAX_GROUP];
    Launch lc[RSPARSE_MAX_GROUP];
    bool can_rowdot = true;
    for (int i = 0; i < n_layers; ++i) {
        v[i] = layers[i]->view(nullptr, batch, true);
        lc[i] = resolve_launch(layers[i], batch, true, n_layers, i ? lc[0].waves : 0);
        can_rowdot = can_rowdot && layers[i]->Wrow != nullptr && rowdot_supported(layers[i]->cfg.d_in, batch);
    }
    // the dense baseline moves to the matrix cores from 2 tokens on small layers and from 4 on large ones
    // (measured: 4096 x 11008 and 8192 x 8192 are still faster on the vector path at 2-3 tokens)
    const bool large = (size_t)layers[0]->cfg.d_in * layers[0]->cfg.d_out >= ((size_t)1 << 25);
    bool mfma = batch >= (layers[0]->tuning.mfma_min_batch > 0 ? layers[0]->tuning.mfma_min_batch
                                                                 : (large ? 4 : kMfmaDefaultMinBatchDense));
    for (int i = 0; i < n_layers; ++i) mfma = mfma && mfma_path_supported(v[i], batch);
    if (mfma) {
        for (int i = 0; i < n_layers; ++i)
            RS_HIP(launch_mfma_linear(v[i], X_dev, batch, Y_devs[i], layers[i]->chan_bits, layers[i]->cus, 0, true, layers[0]->tuning.mfma_rows, s));
        return RSPARSE_OK;
    }
    int kernel = layers[0]->tuning.dense_kernel;
    if (kernel == 2 && !can_rowdot)
        return fail(RSPARSE_EINVAL, "row-dot dense kernel needs dense_rowmajor=1 and batch_tile*d_in*2 <= 64 KiB");
    // row dots win for short rows; for long rows (and for more than one token) the axpy form streams better
    if (kernel == 0) kernel = (can_rowdot && layers[0]->cfg.d_in <= 8192 && batch == 1) ? 2 : 1;
    bool strip = true, colmajor = true;
    for (int i = 0; i < n_layers; ++i) {
        strip = strip && layers[i]->Ms != nullptr && layers[i]->strip_w == layers[0]->strip_w;
        colmajor = colmajor && layers[i]->M != nullptr;
    }
    if (kernel != 2 && !strip && !colmajor) {
        // mixed layouts: one layer at a time
        for (int i = 0; i < n_layers; ++i) {
            rsparse_status one = rsparse_dense_ref_group(&layers[i], 1, X_dev, batch, &Y_devs[i], stream);
            if (one != RSPARSE_OK) return one;
        }
        return RSPARSE_OK;
    }
    if (kernel == 2) {
        RS_HIP(launch_dense_rowdot(v, lc, n_layers, X_dev, batch, Y_devs, s));
    } else if (strip) {
        // the strip kernel with every channel kept and no low-rank part
        Launch sc[RSPARSE_MAX_GROUP];
        for (int i = 0; i < n_layers; ++i) sc[i] = resolve_strip(layers[i], batch, true, n_layers, false);
        RS_HIP(launch_strip(v, sc, n_layers, X_dev, batch, Y_devs, false, true, layers[0]->cus, s));
    } else {
        RS_HIP(launch_dense_axpy(v, lc, n_layers, X_dev, batch, Y_devs, s));
    }
    return RSPARSE_OK;
}

rsparse_status rsparse_linear_group_planned(rsparse_layer *const *layers, int32_t n_layers, const void *X_dev,
                                            int32_t batch, void *const *Y_devs, void *stream, double keep_fraction,
                                            int32_t *used_rsparse_out)
{
    rsparse_status st = check_group(layers, n_layers, X_dev, batch, Y_devs);
    if (st != RSPARSE_OK) return st;
    int32_t use[RSPARSE_MAX_GROUP];
    bool all = true, none = true;
    for (int i = 0; i < n_layers; ++i) {
        const rsparse_config &c = layers[i]->cfg;
        st = rsparse_plan_layer(c.d_in, c.d_out, c.rank, keep_fraction, n_layers, batch, nullptr, nullptr, &use[i]);
        if (st != RSPARSE_OK) return st;
        all = all && use[i];
        none = none && !use[i];
    }
    if (used_rsparse_out) *used_rsparse_out = all ? 1 : 0;
    if (all) return rsparse_linear_group(layers, n_layers, X_dev, batch, Y_devs, stream);
    if (none) return rsparse_dense_ref_group(layers, n_layers, X_dev, batch, Y_devs, stream);
    for (int i = 0; i < n_layers; ++i) {
        st = use[i] ? rsparse_linear_group(&layers[i], 1, X_dev, batch, &Y_devs[i], stream)
                    : rsparse_dense_ref_group(&layers[i], 1, X_dev, batch, &Y_devs[i], stream);
        if (st != RSPARSE_OK) return st;
    }
    return RSPARSE_OK;
}

rsparse_status rsparse_dense_ref(rsparse_layer *L, const void *X_dev, int32_t batch, void *Y_dev, void *stream)
{
    return rsparse_dense_ref_group(&L, 1, X_dev, batch, &Y_dev, stream);
}

rsparse_status rsparse_synchronize(rsparse_layer *L)
{
    if (!L) return fail(RSPARSE_EINVAL, "layer is NULL");
    if (L->last_batch == 0) return RSPARSE_OK;
    RS_HIP(hipStreamSynchronize(L->last_stream));
    if (L->last_fused) {
        const ScratchView &sp = L->last_scratch;
        int flag = 0;
        RS_HIP(hipMemcpy(&flag, sp.sync + kSyncError, 4, hipMemcpyDeviceToHost));
        if (flag != 0) {
            // leave the counters usable for the next call
            int gen = 0;                              // the generation of the strip kernel's hand-off survives the reset
            RS_HIP(hipMemcpy(&gen, sp.sync + kSyncGen, 4, hipMemcpyDeviceToHost));
            RS_HIP(hipMemset(sp.sync, 0, sp.sync_n * 4));
            RS_HIP(hipMemcpy(sp.sync + kSyncGen, &gen, 4, hipMemcpyHostToDevice));
            RS_HIP(hipMemset(sp.t_pub, 0xff, sp.n_t * 4));
            RS_HIP(hipMemset(sp.yacc, 0, sp.n_y * 4));
            return fail(RSPARSE_EHIP, "a cross-workgroup wait of the one-launch kernel ran out; the last result is invalid");
        }
    }
    return RSPARSE_OK;
}

rsparse_status rsparse_last_active(rsparse_layer *L, int32_t token, int32_t *idx_host, int32_t *count)
{
    if (!L || !idx_host || !count) return fail(RSPARSE_EINVAL, "NULL argument");
    if (L->last_batch == 0) return fail(RSPARSE_EINVAL, "no rsparse_linear call has been made on this layer");
    if (token < -1 || token >= L->last_batch) return fail(RSPARSE_EINVAL, "token %d outside [-1, %d)", token, L->last_batch);
    rsparse_status sst = rsparse_synchronize(L);
    if (sst != RSPARSE_OK) return sst;
    if (L->last_mfma) {
        // the matrix-core path keeps per-channel token bits instead of compacted lists
        std::vector<uint32_t> cb(L->cfg.d_in);
        RS_HIP(hipMemcpy(cb.data(), L->chan_bits, cb.size() * 4, hipMemcpyDeviceToHost));
        int32_t n = 0;
        for (size_t c = 0; c < cb.size(); ++c)
            if (token < 0 ? cb[c] != 0u : ((cb[c] >> token) & 1u) != 0u) idx_host[n++] = (int32_t)c;
        *count = n;
        return RSPARSE_OK;
    }
    const int bt = L->last_bt > 0 ? L->last_bt : batch_tile_of(L->last_batch);
    const int nz = (L->last_batch + bt - 1) / bt;
    const size_t d_in = L->cfg.d_in;
    std::vector<int32_t> cnt(nz), list;
    std::vector<uint32_t> bits;
    const ScratchView &sp = L->last_scratch;
    RS_HIP(hipMemcpy(cnt.data(), sp.act_count, nz * 4, hipMemcpyDeviceToHost));
    std::vector<int32_t> seg, seg_list;
    std::vector<uint32_t> seg_bits;
    auto fetch = [&](int z) -> rsparse_status {
        if (L->last_strip) {
            // the strip kernel leaves one ascending list per channel range, at the range's first channel; the
            // ranges in order are the ascending list of the batch tile
            const size_t nq = d_in / 8;
            const size_t R = std::min<size_t>((size_t)L->last_ranges, nq);
            seg.resize(R); seg_list.resize(d_in); seg_bits.resize(d_in);
            RS_HIP(hipMemcpy(seg.data(), sp.act_seg + z * nq, R * 4, hipMemcpyDeviceToHost));
            RS_HIP(hipMemcpy(seg_list.data(), sp.act_list + z * d_in, d_in * 4, hipMemcpyDeviceToHost));
            RS_HIP(hipMemcpy(seg_bits.data(), sp.act_bits + z * d_in, d_in * 4, hipMemcpyDeviceToHost));
            list.clear(); bits.clear();
            const size_t parts = (size_t)L->last_ranges, base = nq / parts, rem = nq - base * parts;
            for (size_t rho = 0; rho < R; ++rho) {
                const size_t lo = (rho * base + std::min(rho, rem)) * 8, len = (base + (rho < rem ? 1 : 0)) * 8;
                if (seg[rho] < 0 || (size_t)seg[rho] > len) return fail(RSPARSE_EHIP, "corrupt list count %d", seg[rho]);
                list.insert(list.end(), seg_list.begin() + lo, seg_list.begin() + lo + seg[rho]);
                bits.insert(bits.end(), seg_bits.begin() + lo, seg_bits.begin() + lo + seg[rho]);
            }
            return RSPARSE_OK;
        }
        if (cnt[z] < 0 || (size_t)cnt[z] > d_in) return fail(RSPARSE_EHIP, "corrupt list count %d", cnt[z]);
        list.resize(cnt[z]); bits.resize(cnt[z]);
        if (cnt[z]) {
            RS_HIP(hipMemcpy(list.data(), sp.act_list + z * d_in, (size_t)cnt[z] * 4, hipMemcpyDeviceToHost));
            RS_HIP(hipMemcpy(bits.data(), sp.act_bits + z * d_in, (size_t)cnt[z] * 4, hipMemcpyDeviceToHost));
        }
        return RSPARSE_OK;
    };
    if (token >= 0) {
        const int z = token / bt, b = token % bt;
        rsparse_status st = fetch(z);
        if (st != RSPARSE_OK) return st;
        int32_t n = 0;
        for (size_t j = 0; j < list.size(); ++j)
            if ((bits[j] >> b) & 1u) idx_host[n++] = list[j];
        *count = n;
        return RSPARSE_OK;
    }
    // union over the batch: merge the batch tiles' ascending lists
    std::vector<uint8_t> seen(d_in, 0);
    for (int z = 0; z < nz; ++z) {
        rsparse_status st = fetch(z);
        if (st != RSPARSE_OK) return st;
        for (int32_t c : list)
            if (c >= 0 && (size_t)c < d_in) seen[c] = 1;
    }
    int32_t n = 0;
    for (size_t c = 0; c < d_in; ++c)
        if (seen[c]) idx_host[n++] = (int32_t)c;
    *count = n;
    return RSPARSE_OK;
}

rsparse_status rsparse_get_factors(const rsparse_layer *L, void *U16_host, void *SV16_host)
{
    if (!L) return fail(RSPARSE_EINVAL, "layer is NULL");
    if (U16_host && !L->U16.empty()) memcpy(U16_host, L->U16.data(), L->U16.size() * 2);
    if (SV16_host && !L->SV16.empty()) memcpy(SV16_host, L->SV16.data(), L->SV16.size() * 2);
    return RSPARSE_OK;
}

rsparse_status rsparse_set_tau(rsparse_layer *L, float tau)
{
    if (!L) return fail(RSPARSE_EINVAL, "layer is NULL");
    if (std::isnan(tau)) return fail(RSPARSE_EINVAL, "tau is NaN");
    L->cfg.tau = tau;
    return RSPARSE_OK;
}

rsparse_status rsparse_set_bias(rsparse_layer *L, const float *bias_host)
{
    if (!L) return fail(RSPARSE_EINVAL, "layer is NULL");
    RS_HIP(hipSetDevice(L->device));
    RS_HIP(hipDeviceSynchronize());                 // no call may still be reading the old bias
    if (!bias_host) {
        (void)hipFree(L->bias);
        L->bias = nullptr;
        return RSPARSE_OK;
    }
    if (!L->bias) RS_HIP(hipMalloc((void **)&L->bias, (size_t)L->cfg.d_out * 4));
    RS_HIP(hipMemcpy(L->bias, bias_host, (size_t)L->cfg.d_out * 4, hipMemcpyHostToDevice));
    return RSPARSE_OK;
}

rsparse_status rsparse_multiphase_bias(const void *W_host, int32_t dtype, int32_t d_in, int32_t d_out, const void *H_host,
                                       int32_t n_tokens, const float *T, int32_t l, float *bias_out)
{
    if (!W_host || !H_host || !T || !bias_out) return fail(RSPARSE_EINVAL, "NULL argument");
    if (d_in < 1 || d_out < 1 || n_tokens < 1 || l < 1) return fail(RSPARSE_EINVAL, "sizes must be positive");
    if (dtype != RSPARSE_F16 && dtype != RSPARSE_BF16) return fail(RSPARSE_EINVAL, "dtype must be F16 or BF16");
    for (int i = 0; i < l; ++i) {
        if (!std::isfinite(T[i])) return fail(RSPARSE_EINVAL, "T[%d] is not finite", i);
        if (i > 0 && !(T[i - 1] > T[i])) return fail(RSPARSE_EINVAL, "T must be strictly decreasing");
    }
    const uint16_t *W = (const uint16_t *)W_host, *H = (const uint16_t *)H_host;
    // m[k] = mean over the tokens of the value the multi-phase activation puts in place of h_k when h_k < T[0]
    std::vector<double> m((size_t)d_in, 0.0);
    for (int n = 0; n < n_tokens; ++n)
        for (int k = 0; k < d_in; ++k) {
            const double h = (double)widen16(H[(size_t)n * d_in + k], dtype);
            if (!(h < (double)T[0]) || l < 2) continue;          // sparse component, NaN, or nothing below T[0] is kept
            int i = l - 2;                                       // below T[l-1]: the last interval
            for (int j = 0; j + 1 < l; ++j)
                if (h >= (double)T[j + 1]) { i = j; break; }
            m[(size_t)k] += 0.5 * ((double)T[i] + (double)T[i + 1]);
        }
    for (int k = 0; k < d_in; ++k) m[(size_t)k] /= (double)n_tokens;
    parallel_for((size_t)d_out, [&](size_t o) {
        double acc = 0.0;
        for (int k = 0; k < d_in; ++k) acc += (double)widen16(W[o * (size_t)d_in + k], dtype) * m[(size_t)k];
        bias_out[o] = (float)acc;
    });
    return RSPARSE_OK;
}

rsparse_status rsparse_set_tuning(rsparse_layer *L, const rsparse_tuning *t)
{
    if (!L || !t) return fail(RSPARSE_EINVAL, "NULL argument");
    if (t->nontemporal < 0 || t->nontemporal > 2) return fail(RSPARSE_EINVAL, "nontemporal must be 0, 1 or 2");
    if (t->splits < 0 || t->waves < 0 || t->lowrank_rows < 0 || t->lowrank_wgs < -1 || t->lowrank_wgs > 65536 || t->dense_kernel < 0 || t->dense_kernel > 2)
        return fail(RSPARSE_EINVAL, "negative or unknown tuning value");
    if (t->mfma_rows != 0 && t->mfma_rows != 64 && t->mfma_rows != 128 && t->mfma_rows != 256)
        return fail(RSPARSE_EINVAL, "mfma_rows must be 0, 64, 128 or 256");
    if (t->mfma_min_batch < 0 || t->mfma_min_batch > 33) return fail(RSPARSE_EINVAL, "mfma_min_batch must be in [0, 33]");
    if (t->tile_map < 0 || t->tile_map > 2) return fail(RSPARSE_EINVAL, "tile_map must be 0, 1 or 2");
    if (t->stages < 0 || t->stages > 2) return fail(RSPARSE_EINVAL, "stages must be 0, 1 or 2");
    if (t->launches < 0 || t->launches > 2) return fail(RSPARSE_EINVAL, "launches must be 0, 1 or 2");
    if (t->debug_wait_polls < 0 || t->debug_skip_stage1 < 0 || t->debug_skip_stage1 > 1)
        return fail(RSPARSE_EINVAL, "debug_wait_polls must be >= 0 and debug_skip_stage1 0 or 1");
    if (t->debug_skip_stage1 && (t->debug_wait_polls < 1 || t->debug_wait_polls > 64))
        return fail(RSPARSE_EINVAL, "debug_skip_stage1 needs debug_wait_polls in [1, 64] (a short, bounded wait)");
    if (t->waves != 0 && t->waves != 1 && t->waves != 2 && t->waves != 4 && t->waves != 8)
        return fail(RSPARSE_EINVAL, "waves must be 0, 1, 2, 4 or 8");
    L->tuning = *t;
    return RSPARSE_OK;
}

rsparse_status rsparse_get_config(const rsparse_layer *L, rsparse_config *out)
{
    if (!L || !out) return fail(RSPARSE_EINVAL, "NULL argument");
    *out = L->cfg;
    return RSPARSE_OK;
}

rsparse_status rsparse_calibrate_tau(const void *X_host, int32_t dtype, size_t n, double s, float *tau_out)
{
    if (!X_host || !tau_out) return fail(RSPARSE_EINVAL, "NULL argument");
    if (dtype != RSPARSE_F16 && dtype != RSPARSE_BF16) return fail(RSPARSE_EINVAL, "dtype must be F16 or BF16");
    if (n == 0) return fail(RSPARSE_EINVAL, "no calibration activations");
    if (!(s >= 0.0) || s > 1.0) return fail(RSPARSE_EINVAL, "s must be in [0, 1]");
    std::vector<float> a;
    try { a.resize(n); } catch (const std::bad_alloc &) { return fail(RSPARSE_ENOMEM, "host allocation failed"); }
    const uint16_t *x = (const uint16_t *)X_host;
    for (size_t i = 0; i < n; ++i) a[i] = std::fabs(widen16(x[i], dtype));   // exact: 16-bit values fit fp32
    size_t idx = (size_t)std::floor(s * (double)n);
    if (idx > n - 1) idx = n - 1;
    std::nth_element(a.begin(), a.begin() + idx, a.end());
    *tau_out = a[idx];
    return RSPARSE_OK;
}

rsparse_status rsparse_io_model(const rsparse_config *cfg, int32_t q4_group, int32_t batch, int32_t k_union,
                                size_t *required_out, size_t *dense_out, size_t *required_inactive_only_out)
{
    rsparse_status st = check_config(cfg);
    if (st != RSPARSE_OK) return st;
    if (batch < 1 || batch > RSPARSE_MAX_BATCH) return fail(RSPARSE_EBATCH, "batch %d outside [1, %d]", batch, RSPARSE_MAX_BATCH);
    if (k_union < 0 || k_union > cfg->d_in) return fail(RSPARSE_EINVAL, "k_union %d outside [0, d_in]", k_union);
    if (q4_group != 0 && (q4_group < 32 || q4_group > 1024 || (q4_group & (q4_group - 1)) || cfg->d_in % q4_group))
        return fail(RSPARSE_EINVAL, "q4_group must be 0 or a power of two in [32, 1024] that divides d_in");
    const size_t e = 2, d_in = cfg->d_in, d_out = cfg->d_out, r = cfg->rank, B = batch, k = k_union;
    const size_t eo = cfg->out_dtype == RSPARSE_F32 ? 4 : 2;
    const size_t io = e * B * d_in + eo * B * d_out;
    size_t w_kept, w_all;
    if (q4_group) {
        // half a byte per weight; scale (2 bytes) and zero point (half a byte) per output and group -- of every
        // group that holds a kept channel (at most min(groups, k))
        const size_t groups = d_in / (size_t)q4_group;
        w_kept = k * d_out / 2 + std::min(groups, k) * d_out * 5 / 2;
        w_all = d_in * d_out / 2 + groups * d_out * 5 / 2;
    } else {
        w_kept = e * k * d_out;
        w_all = e * d_in * d_out;
    }
    if (required_out) *required_out = w_kept + e * (r * d_out + r * d_in) + io;
    if (dense_out) *dense_out = w_all + io;
    if (required_inactive_only_out) *required_inactive_only_out = w_kept + e * (r * d_out + r * (d_in - k)) + io;
    return RSPARSE_OK;
}

size_t rsparse_required_bytes(const rsparse_layer *L, int32_t batch, int32_t k_union)
{
    size_t v = 0;
    if (!L || rsparse_io_model(&L->cfg, L->q4() ? 1 << L->qshift : 0, batch, k_union, &v, nullptr, nullptr) != RSPARSE_OK) return 0;
    return v;
}

size_t rsparse_dense_bytes(const rsparse_layer *L, int32_t batch)
{
    size_t v = 0;
    if (!L || rsparse_io_model(&L->cfg, L->q4() ? 1 << L->qshift : 0, batch, 0, nullptr, &v, nullptr) != RSPARSE_OK) return 0;
    return v;
}

rsparse_status rsparse_recipe(int32_t d_in, int32_t d_out, double budget_c, double rho, double *keep_fraction_out,
                              int32_t *rank_out, double *io_out)
{
    if (!keep_fraction_out || !rank_out) return fail(RSPARSE_EINVAL, "NULL argument");
    if (d_in < 1 || d_out < 1) return fail(RSPARSE_EINVAL, "dimensions must be positive");
    if (!(budget_c >= 0.0) || budget_c > 1.0 || !(rho >= 0.0) || rho > 1.0)
        return fail(RSPARSE_EINVAL, "budget and rho must be in [0, 1]");
    const double mn = (double)d_in * (double)d_out, m_plus_n = (double)d_in + (double)d_out;
    const double s = rho * budget_c;
    long long r = (long long)std::floor((1.0 - rho) * budget_c * mn / m_plus_n + 1e-9);
    r -= r % 8;
    const long long rmax = std::min(d_in, d_out) - std::min(d_in, d_out) % 8;
    r = std::max(0LL, std::min(r, rmax));
    *keep_fraction_out = s;
    *rank_out = (int32_t)r;
    if (io_out) *io_out = (double)r * m_plus_n / mn + s;
    return RSPARSE_OK;
}

rsparse_status rsparse_plan_layer(int32_t d_in, int32_t d_out, int32_t rank, double keep_fraction, int32_t group,
                                  int32_t batch, double *us_rsparse_out, double *us_dense_out, int32_t *use_rsparse_out)
{
    if (d_in < 1 || d_out < 1 || rank < 0 || rank > std::min(d_in, d_out)) return fail(RSPARSE_EINVAL, "bad layer shape");
    if (!(keep_fraction >= 0.0) || keep_fraction > 1.0) return fail(RSPARSE_EINVAL, "keep_fraction must be in [0, 1]");
    if (group < 1 || group > RSPARSE_MAX_GROUP) return fail(RSPARSE_EINVAL, "group %d outside [1, %d]", group, RSPARSE_MAX_GROUP);
    if (batch < 1 || batch > RSPARSE_MAX_BATCH) return fail(RSPARSE_EINVAL, "batch %d outside [1, %d]", batch, RSPARSE_MAX_BATCH);
    // measured on MI355X with this library's kernels (16-bit weights): time = fixed cost of the launch(es) + bytes / rate
    const double m = d_out, n = d_in, r = rank, e = 2.0, B = batch;
    const double io = e * B * (n + m);
    // the columns that are loaded are the union of the tokens' kept channels (independent tokens)
    const double u = 1.0 - std::pow(1.0 - keep_fraction, B);
    double us_rs, us_dense;
    if (batch == 1) {
        constexpr double kBytesPerUs = 6.5e6, kFixedRsparseUs = 8.5, kFixedDenseUs = 3.6;
        us_rs = kFixedRsparseUs / group + (e * (keep_fraction * n * m + r * (n + m)) + io) / kBytesPerUs;
        us_dense = kFixedDenseUs / group + (e * n * m + io) / kBytesPerUs;
    } else {
        if (batch <= 4) {
            // vector path, one launch shared by the group; the fixed part grows with the batch tile (token loads,
            // coefficient fetch, accumulators per token)
            us_rs = (8.5 + 3.0 * std::log2(B)) / group + (e * (u * n * m + r * (n + m)) + io) / 6.7e6;
        } else {
            // matrix-core path: W is streamed whole whatever the masks are, three launches, no sharing in a group
            us_rs = 15.0 + (e * (n * m + r * (n + m)) + io) / 4.65e6;
        }
        // dense product on the matrix cores
        us_dense = (batch > 16 ? 9.2 : 7.3) + (e * n * m + io) / (batch > 16 ? 4.86e6 : 5.26e6);
    }
    if (us_rsparse_out) *us_rsparse_out = us_rs;
    if (us_dense_out) *us_dense_out = us_dense;
    if (use_rsparse_out) *use_rsparse_out = us_rs < us_dense ? 1 : 0;
    return RSPARSE_OK;
}

rsparse_status rsparse_debug_stamps(void *buf_dev, int32_t capacity_waves)
{
    if (capacity_waves < 0 || (buf_dev == nullptr) != (capacity_waves == 0)) return fail(RSPARSE_EINVAL, "buffer and capacity must both be set or both be zero");
    hipError_t e = set_stamp_buffer(buf_dev, capacity_waves);
    if (e == hipErrorNotSupported) return fail(RSPARSE_EINVAL, "this library was built without RSPARSE_STAMPS");
    RS_HIP(e);
    return RSPARSE_OK;
}

void rsparse_destroy(rsparse_layer *L) { free_layer(L); }

}  // extern "C"
