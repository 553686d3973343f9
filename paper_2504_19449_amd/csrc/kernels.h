// Internal launch interface between the C-ABI host code (api.cpp) and the gfx950 kernels
// (kernels.hip).  Not installed; the public boundary is include/rsparse.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rsparse {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kTile = 512;       // output columns per wave: 64 lanes x one 16-byte load (8 x 16-bit)
constexpr int kMaxBT = 8;        // tokens held in registers per workgroup (batch tile)
// Smallest batch that takes the matrix-core path by default (measured cross-over on MI355X: the
// vector path wins up to 4 tokens for R-Sparse; the dense baseline is faster on MFMA from 2 tokens).
constexpr int kMfmaDefaultMinBatch = 5;
constexpr int kMfmaDefaultMinBatchDense = 2;

// Which channels of a token are kept (R-Sparse, Sec. 3.4: the sparsification function, and its fixed-count variant),
// in one form:  v >= ge  ||  (v == eq && channel <= cut),  with v = |x| (v = x for the signed threshold).
//   |x| >= t:   ge = t, eq = NaN (never equal).        |x| > t:  ge = the next fp32 above t.
//   fixed count k:  eq = the k-th largest magnitude of the token, ge = the next fp32 above it, cut = the last channel
//   among those equal to it that still belongs to the k (lower channels first).
struct KeepRule {
    float ge, eq;
    int cut, pad;
};

// Device-side view of one prepared layer plus its per-call scratch.
struct LayerView {
    const uint16_t *M;      // [d_in + rank][d_out]: W column-major (row c = W[:, c]), then U_r^T (row d_in + j = U_r[:, j])
    const uint16_t *SVt;    // [rank][d_in]  = S_r V_r^T
    const uint16_t *U;      // [d_out][rank] = U_r, row-major
    const uint16_t *SVc;    // [d_in][rank] channel-major copy of S_r V_r^T (row c = its column c), or nullptr
    float *t_sum;           // [nz][BT][rank] fp32 sums of the stage 1 that reads SVc; zero between calls (or nullptr)
    const uint16_t *Wrow;   // [d_out][d_in] row-major copy of W, or nullptr
    float *t;               // [nz][BT][rank] stage-1 result, fp32
    float *t_acc;           // [rank][16 or 32 tokens] matrix-core path: t summed over the K slices; zero between calls (or nullptr)
    uint16_t *t16;          // [2][32][rank] matrix-core path: t split into two 16-bit halves, [token][rank] each (or nullptr)
    float *yacc;            // [max_batch][d_out] fp32 accumulators; zero between calls
    int32_t *act_list;      // [nz][d_in] ascending kept channels of batch tile z (union over its tokens)
    uint32_t *act_bits;     // [nz][d_in] per list entry: bit b = token b of the tile keeps it
    int32_t *act_count;     // [nz]
    int *sync;              // arrival counters of the one-launch path (layout: kSync* below); zero between calls
    uint32_t *t_pub;        // [nz][BT][rank] one-launch path: t as fp32 bits; all-ones (not ready) between calls
    unsigned long long *t_tag;  // [t_slots][rank] strip kernel: {generation of the launch that wrote it, t as fp32 bits}
    int t_slots;            // token slots of t_tag (max_batch rounded up to whole batch tiles)
    // strip-major W for the strip kernel: strip s holds columns [s * strip_w, (s + 1) * strip_w) of all d_in + rank
    // rows (row c = W[:, c], row d_in + j = U_r[:, j]) contiguously, [strips][d_in + rank][strip_w]; columns past
    // d_out are zero
    const uint16_t *Ms;
    int strip_w;
    long long strip_stride; // 16-bit elements from one strip to the next: (d_in + rank + padding rows) * strip_w
    int32_t *act_seg;       // [nz][d_in / 8] strip kernel: kept channels found in each channel range of batch tile z
    // 4-bit weights (Mq != nullptr; then M and Wrow are null).  A column tile is kQ4Tile = 1024 outputs: lane l
    // of a wave owns the 8 bytes T * 512 + l * 8 .. of a row, two words h = 0, 1; byte k of word h holds the
    // code of column T * 1024 + h * 512 + l * 8 + k in its low nibble and of column ... + 4 + k in its high one.
    const uint8_t *Mq;      // [d_in][qtiles * 512] bytes, row c = the codes of W[:, c]
    const uint16_t *qs;     // [d_in >> qshift][qtiles * 1024] group scales, 16-bit of dtype, plain column order
    const uint8_t *qz;      // [d_in >> qshift][qtiles * 1024] group zero points, one per byte
    const uint16_t *Ut;     // [rank][qtiles * 1024] = U_r^T, zero-padded rows (the one-launch 4-bit kernel streams it)
    int qshift, qtiles;     // log2(group size); column tiles of 1024
    int d_in, d_out, rank;
    int dtype, out_dtype, cmp_mode, batch_mask_mode;
    float tau;
    float tau_ge;           // the threshold as a KeepRule::ge (host-computed from tau and cmp_mode)
    int keep_signed;        // cmp_mode 2: the rule applies to x itself, not to |x|
    const KeepRule *rules;  // fixed-count activation: [batch] per-token rules written by launch_topk_rules; else nullptr
    const float *bias;      // [d_out] fp32 added to every token's output before the rounding, or nullptr
};

// Dense 4-bit baseline over row-major codes (kernels_q4row.hip): Qrow [d_out][d_in/2] (channel 2j in the low nibble of byte
// j), Srow / Zrow [d_out][d_in >> qshift].  Needs batch_tile * d_in * (2 + 1/8) bytes of LDS <= 64 KiB and groups >= 32.
bool q4_rowdot_supported(int d_in, int batch);
hipError_t launch_q4_dense_rowdot(const uint8_t *Qrow, const uint16_t *Srow, const uint8_t *Zrow, int qshift, int dtype, int out_dtype,
                                  int d_in, int d_out, const void *X, int batch, void *Y, hipStream_t stream);

// Fixed-count activation: per token of X [batch][d_in] the KeepRule that keeps exactly min(k, non-NaN channels)
// channels of largest magnitude (ties: lower channel first).  One workgroup per token.
hipError_t launch_topk_rules(const void *X, int dtype, int batch, int d_in, int k, KeepRule *rules, hipStream_t stream);

// Per-call scratch of a layer: what the kernels write besides Y.  Normally owned by the handle (allocated when the
// layer is prepared); rsparse_linear_static points it into a file-scope device array instead.
struct ScratchView {
    float *t, *yacc;
    int32_t *act_list;
    uint32_t *act_bits;
    int32_t *act_count, *act_seg;
    int *sync;
    uint32_t *t_pub;
    unsigned long long *t_tag;
    KeepRule *rules;
    int t_slots;
    size_t n_t, n_y, sync_n;       // 32-bit words of t / t_pub (and 64-bit words of t_tag), of yacc, of sync
};

// Limits of the static scratch (static_scratch.hip): one batch tile of up to 8 tokens, dimensions up to 32768,
// rank up to 2048 -- 1.6 MB carved out of a 2 MiB array.
constexpr int kStaticMaxBatch = 8, kStaticMaxDim = 32768, kStaticMaxRank = 2048;
// The scratch of one call in the calling device's static array (its address is looked up once per device), cleared
// for this call by one fill launch on `stream`: accumulators and counters zero, hand-off entries "not written".
// Allocates nothing.
hipError_t static_scratch_for_call(int device, int d_out, int rank, int batch, hipStream_t stream, ScratchView *out);

struct Launch {
    int splits;        // channel splits per column tile
    int waves;         // waves per workgroup (first launch / dense axpy)
    int lowrank_rows;  // rows of S_r V_r^T per stage-1 workgroup
    int lowrank_wgs;   // > 0: stage 1 of the one-launch kernel at one token reads the channel-major copy of S_r V_r^T
                       // (dropped channels' rows only) with this many workgroups, each on a fixed channel range
    int nontemporal;
    int tile_map;      // 1: tile-fastest workgroup order, 2: XCD-aware (a tile's splits share id mod 8)
    int wait_polls;    // one-launch kernel: bound on re-reads of an unpublished t entry; 0 = default
    int skip_stage1;   // one-launch kernel, test hook: stage 1 publishes nothing, so every wait runs out
};

// Arrival counters of the one-launch path, as offsets into LayerView::sync (32-bit words).
constexpr int kSyncTilesDone = 0;   // column tiles (over all batch tiles) whose outputs have been stored
constexpr int kSyncError = 1;       // set when a bounded wait ran out (results of that call are invalid)
constexpr int kSyncStage1 = 3;      // [kSyncMaxZ] one-launch kernel, per batch tile: stage-1 workgroups (channel-major form) that have added their partial t
constexpr int kSyncGen = 2;         // strip kernel: generation number of the next launch (bumped once per launch)
constexpr int kSyncStarted = 8;     // strip kernel: [kSyncStartedN] how many waves of the launch have read the generation
constexpr int kSyncStartedN = 256;
constexpr int kSyncMaxZ = 4;        // batch tiles per launch
constexpr int kSyncTile = kSyncStarted + kSyncStartedN;   // [nz][tiles] channel splits of the tile that have added their sums
inline size_t sync_words(int tiles) { return (size_t)kSyncTile + (size_t)kSyncMaxZ * tiles; }

// All launchers take a group of n <= kMaxGroupLayers layers that read the same input X (same d_in and
// dtype); cfg[0].waves and cfg[0].nontemporal apply to the whole launch.
constexpr int kMaxGroupLayers = 4;

// First launch: stage 1 of the low-rank part (with_t) and threshold + compaction + gather-GEMV over
// the kept columns into yacc (with_gather), as independent workgroups of one grid.
hipError_t launch_sparse_and_t(const LayerView *L, const Launch *cfg, int n, const void *X, int batch, bool with_t,
                               bool with_gather, hipStream_t stream);
// The whole layer in ONE launch: the stage-1 workgroups publish t, every gather workgroup also streams
// its share of the rows of U_r^T (as channels d_in.. with coefficients t), and the last workgroup to
// arrive at a column tile rounds and stores that tile of Y.  cfg[i].splits must satisfy
// gather_lds_bytes(d_in, splits, waves, bt, rank) <= 64 KiB.
// gate_up: L[0], L[1] are the gate and up projections of an MLP (same d_out, out_dtype == dtype); the kernel
// stores H = round(silu(round(g)) * round(u)) to Y[0] instead of the two outputs (Y[1] is not written).
hipError_t launch_fused(const LayerView *L, const Launch *cfg, int n, const void *X, int batch, void *const *Y,
                        hipStream_t stream, bool gate_up = false);
// First launch of a layer with 4-bit weights (batch tiles of at most 4 tokens): as launch_sparse_and_t, with the codes
// dequantised in registers -- per quantisation group the kernel accumulates sum_c x_c q_c and sum_c x_c and
// applies scale and zero point once, when the group ends.  dense: every channel is kept (the dense baseline
// on the same weights).  Y_fused == nullptr: launch_finish completes the layer.  Y_fused != nullptr: the whole
// layer in this one launch, as launch_fused (not with dense).
constexpr int kQ4Tile = 1024;
hipError_t launch_q4(const LayerView &L, const Launch &cfg, const void *X, int batch, bool with_t, bool dense,
                     void *Y_fused, hipStream_t stream);
// Second launch: Y = round(yacc + U_r t) (use_rank) or round(yacc); re-zeroes yacc.
hipError_t launch_finish(const LayerView *L, int n, int batch, void *const *Y, bool use_rank, hipStream_t stream);
// Dense baselines.
hipError_t launch_dense_axpy(const LayerView *L, const Launch *cfg, int n, const void *X, int batch, void *const *Y,
                             hipStream_t stream);
hipError_t launch_dense_rowdot(const LayerView *L, const Launch *cfg, int n, const void *X, int batch, void *const *Y,
                               hipStream_t stream);
// Matrix-core path for 2 <= batch <= 32 (needs the row-major copy of W): both launches of one layer.
// chan_bits [d_in] receives, per channel, the bit mask of the tokens that keep it.  stages as in
// rsparse_tuning.  Zeroes L.t with a fill kernel first (its stage-1 partial sums meet in atomics).
// dense = the dense baseline Y = X W^T through the same kernels (no masks, no low-rank part).
bool mfma_path_supported(const LayerView &L, int batch);
hipError_t launch_mfma_linear(const LayerView &L, const void *X, int batch, void *Y, uint32_t *chan_bits, int cus,
                              int stages, bool dense, int rows_per_wg_hint, hipStream_t stream);
// The whole layer over strip-major weights (LayerView::Ms), up to 8 tokens per batch tile: one workgroup per strip
// of strip_w output columns streams all kept rows of the strip and stores its slice of Y (cfg[i].splits == 1), or
// `splits` workgroups per strip meet in yacc.  fused: stage 1 runs in the same launch and hands t over through
// LayerView::t_tag; otherwise t must have been stored to LayerView::t by an earlier launch
// (launch_sparse_and_t with with_gather = false).  dense: the dense product Y = X W^T through the same kernel
// (every channel kept, no low-rank part).  Layers of a group share d_in, dtype and strip_w.
hipError_t launch_strip(const LayerView *L, const Launch *cfg, int n, const void *X, int batch, void *const *Y,
                        bool fused, bool dense, int cus, hipStream_t stream);
// Stamps builds only (see device_stage1.h): where the strip kernel's waves write their phase time stamps;
// hipErrorNotSupported in product builds.
hipError_t set_stamp_buffer(void *buf_dev, int capacity_waves);
int strip_waves(int batch);                       // waves per workgroup the strip kernel runs with
// list entries per wave that fit in LDS for this launch shape; 0 = the shape does not fit (more splits needed)
int strip_list_cap(int d_in, int rank, int splits, int waves, int bt, int strip_w);
bool strip_width_ok(int w);
// out[0:n) = round16(silu(G) * Up), n a multiple of 8, all 16-byte aligned.
hipError_t launch_gated_input(const void *G, const void *Up, void *out, size_t n, int dtype, hipStream_t stream);
// Zero `n` 32-bit words (a fill kernel, safe to record into a HIP graph).
hipError_t launch_zero(void *p, size_t n_words, hipStream_t stream);

size_t gather_lds_bytes(int d_in, int splits, int waves, int bt, int fused_rank = 0);
size_t lowrank_lds_bytes(int d_in, int bt);
bool rowdot_supported(int d_in, int batch);

}  // namespace rsparse
