/*
 * rsparse.h -- C ABI of the MI355X (gfx950) R-Sparse linear layer.
 *
 * The library implements one operation, the rank-aware sparse linear layer of
 * R-Sparse (Sec. 3.4, "R-Sparse Inference") for small-batch decode:
 *
 *     Y = sigma_t(X) W^T  +  (X - sigma_t(X)) (U_r S_r V_r^T)^T
 *
 * where sigma_t keeps the input channels with |x| >= t (Sec. 3.4, "Sparsifying Input
 * Activation"), the first term only touches the columns of W whose channel was
 * kept (W is held column-major, as Sec. 3.4 asks, so each kept channel is one
 * contiguous run), and the second term sends the remaining channels through the
 * rank-r factors of W's top singular components.
 *
 * Conventions
 *   - W is [d_out][d_in] row-major on the host (nn.Linear orientation, Y = X W^T,
 *     Sec. 3.1); "columns" of W are input channels.
 *   - X is [batch][d_in], Y is [batch][d_out], row-major, on the DEVICE.
 *   - 16-bit values are raw IEEE fp16 or bfloat16 bit patterns (uint16_t).
 *   - Every function returns an rsparse_status; nothing throws or aborts across
 *     the ABI.  rsparse_last_error() gives a thread-local message for the last failure.
 *   - "host" / "device" is stated for every pointer.  The caller owns everything it
 *     passes in; the handle owns its packed weights and scratch (all allocated at
 *     prepare time -- the hot calls never allocate and never synchronise, and they
 *     leave the scratch ready for the next call, so they can be captured into a HIP graph).
 *   - A handle must not be used by two calls at once (its scratch is shared); calls
 *     on one stream are ordered by the stream.
 */
#ifndef RSPARSE_H
#define RSPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rsparse_layer rsparse_layer; /* opaque; owns device memory */

typedef enum {
    RSPARSE_F16 = 0,
    RSPARSE_BF16 = 1,
    RSPARSE_F32 = 2 /* legal for out_dtype only: unrounded accumulators, for tight parity checks */
} rsparse_dtype;

typedef enum {
    RSPARSE_OK = 0,
    RSPARSE_EINVAL = 1,  /* bad argument (null, range, NaN tau, unsupported shape) */
    RSPARSE_ENOMEM = 2,  /* host or device allocation failed */
    RSPARSE_EHIP = 3,    /* a HIP call failed; message holds the HIP error string */
    RSPARSE_EBATCH = 4,  /* batch outside [1, max_batch] */
    RSPARSE_EALIGN = 5,  /* X or Y not 16-byte aligned */
    RSPARSE_ESVD = 6     /* the host SVD did not converge */
} rsparse_status;

#define RSPARSE_MAX_BATCH 32

typedef struct {
    int32_t d_in;            /* input channels; multiple of 8, at most 65536 */
    int32_t d_out;           /* output features; multiple of 8 */
    int32_t rank;            /* r in [0, min(d_in, d_out)], multiple of 8; 0 = sparse part only */
    int32_t max_batch;       /* 1..RSPARSE_MAX_BATCH; scratch is sized for it */
    float   tau;             /* threshold t(s) (Sec. 3.4); fp32 so that the compare is exact.
                                -INFINITY keeps every channel, +INFINITY none; NaN is rejected */
    int32_t dtype;           /* of W, X and the factors: RSPARSE_F16 or RSPARSE_BF16 */
    int32_t out_dtype;       /* of Y: equal to dtype, or RSPARSE_F32 */
    int32_t cmp_mode;        /* 0: keep |x| >= tau (the paper's definition)   1: keep |x| > tau
                                2: keep x >= tau, signed -- the sparse components of the multi-phase activation of
                                Sec. 3.2 are the values at or above T_0 (see rsparse_set_bias) */
    int32_t batch_mask_mode; /* 0: every token uses its own mask (sigma_t is elementwise)
                                1: every token uses the union of the batch's masks
                                2: own masks up to 3 tokens, the union from 4 tokens on (there the union is ~90 % of the
                                channels anyway, its columns are loaded either way, and using them for every token is
                                strictly more accurate at the same bytes) */
    int32_t dense_rowmajor;  /* 1: also keep W row-major on the device (doubles the weight footprint).  Needed by
                                the row-dot kernel of rsparse_dense_ref and by the matrix-core path that
                                rsparse_linear takes from 5 tokens on (see mfma_min_batch); without it those
                                batches run in tiles of up to 8 tokens on the vector ALU */
    int32_t strip_cols;      /* layout of W on the device for the vector path (up to 8 tokens per batch tile).  0: column-major
                                (Sec. 3.4), run by the column-tile kernel: tiles of 512 outputs x channel splits whose partial
                                sums meet in fp32 atomics.  32, 64, 128, 256 or 512: the columns are cut into strips of that
                                many outputs, stored strip after strip, and run by the strip kernel: one workgroup (or a few,
                                tuning `splits`) per strip, every wave on a fixed range of input channels; with one workgroup
                                per strip no sums cross workgroups and Y is bit-reproducible from run to run.  Same results
                                within the stated tolerance; see rsparse_tuning.splits.  Not with 4-bit weights. */
    int32_t topk;            /* 0: channels are kept by the threshold tau.  k > 0: fixed-count activation -- every token keeps
                                exactly its min(k, non-NaN channels) channels of largest magnitude (among equal magnitudes
                                the lower channel first; NaN never), so the sparsity is exact per token instead of holding
                                in expectation; tau is ignored, cmp_mode must be 0.  One small extra launch per call finds
                                each token's k-th magnitude.  Vector path only (batches above 8 run in tiles of 8); not with
                                4-bit weights.  k <= d_in. */
    int32_t lowrank_channel_major; /* 1: also keep S_r V_r^T channel-major on the device ([d_in][rank]: rank * d_in more
                                elements).  Up to four tokens the one-launch column-tile kernel then forms t from the rows of
                                the DROPPED channels only (the low-rank part acts on x - sigma_t(x), whose kept channels are
                                zero): rank * (d_in - k) elements read instead of rank * d_in (k: channels that every token of
                                the batch tile keeps), summed with fp32 atomics.  Same results within the stated tolerance.
                                Measured to pay in launches (one layer, or the layers of a grouped call) of about 2^26 weights
                                or more (28672 -> 8192: 7 %; q/k/v grouped at 8192: 17 %) and at four tokens with the union mask
                                (few channels are dropped then: 1-7 %), and to cost time in smaller launches at one or two tokens
                                (t is published later): the library uses the copy in exactly those two cases unless
                                rsparse_tuning.lowrank_wgs says otherwise.  Ignored by the strip kernel, batches above four, the two-launch
                                form, rsparse_linear_static and 4-bit weights (those read the row-major copy). */
} rsparse_config;

/* Launch-shape overrides for measurements; 0 = library default. */
typedef struct {
    int32_t splits;          /* channel splits per column tile of the gather / dense-axpy kernels */
    int32_t waves;           /* waves (of 64 lanes) per workgroup in those kernels: 1, 2, 4 or 8 */
    int32_t lowrank_rows;    /* rows of S_r V_r^T per stage-1 workgroup */
    int32_t dense_kernel;    /* rsparse_dense_ref: 0 auto, 1 axpy over column-major W, 2 row-dot */
    int32_t nontemporal;     /* weight loads of the vector-path kernels: 0 default (non-temporal), 1 non-temporal,
                                2 ordinary (temporal) loads */
    int32_t stages;          /* rsparse_linear, two-launch form: 0 the whole layer, 1 first launch only, 2 second
                                only -- for timing one kernel in isolation; results are only valid with 0 */
    int32_t tile_map;        /* workgroup -> (column tile, split) mapping: 0 default, 1 tile-fastest (plain),
                                2 XCD-aware (all splits of a tile on ids congruent mod 8) */
    int32_t mfma_min_batch;  /* smallest batch that takes the matrix-core path (needs dense_rowmajor = 1):
                                0 = default (5 for rsparse_linear; 2 for rsparse_dense_ref, 4 on layers of 2^25 weights or more), 33 = never (all batches
                                then run in tiles of up to 8 tokens on the vector ALU) */
    int32_t mfma_rows;       /* output rows per workgroup of the matrix-core kernels: 0 default, or 64, 128, 256 */
    int32_t launches;        /* rsparse_linear up to 8 tokens (and beyond without the row-major copy): 0 default
                                (one launch; two on 4-bit weights), 1 one launch, 2 two launches (stage 2 and the
                                rounding in a second kernel).  stages != 0 implies two launches */
    int32_t lowrank_wgs;     /* stage-1 workgroups of the channel-major form (cfg.lowrank_channel_major): 0 default (64, or 128
                                from 16 MB of rows to read, within the resident slots the layer's other workgroups leave free;
                                128 on skinny layers; the copy is used only where it was measured to pay), > 0: that many,
                                always, -1: always the row-major copy */
    int32_t debug_wait_polls;   /* one-launch kernel: bound on the re-reads of a low-rank intermediate that stage 1 has
                                   not published yet; 0 = default (2^20, or 0.5 s) */
    int32_t debug_skip_stage1;  /* test hook for the error path, needs debug_wait_polls in [1, 64]: stage 1 publishes
                                   nothing, every bounded wait runs out, the kernel still finishes, the result is
                                   invalid and rsparse_synchronize reports RSPARSE_EHIP */
} rsparse_tuning;

/*
 * Offline preparation (Sec. 3.4: the low-rank factors come from one SVD of W, done ahead of time).
 * W_host: host, [d_out][d_in] 16-bit of cfg->dtype.  The library computes the top-`rank`
 * singular triplets on the host in fp64, forms U_r and S_r V_r^T, rounds each entry once (fp64 to cfg->dtype, nearest even),
 * packs W column-major and uploads everything.  *out receives a new handle.
 */
rsparse_status rsparse_prepare(const rsparse_config *cfg, const void *W_host, rsparse_layer **out);

/*
 * The host SVD step of rsparse_prepare on its own (no device needed): top-`rank` singular
 * triplets of W_host, written as the stored factors U16_host [d_out][rank] and SV16_host
 * [rank][d_in] (host, 16-bit of cfg->dtype) and, if sigma_host != NULL, the singular values
 * [rank] in fp64.  Lets callers cache factors and feed rsparse_prepare_factors.
 */
rsparse_status rsparse_compute_factors(const rsparse_config *cfg, const void *W_host, void *U16_host,
                                       void *SV16_host, double *sigma_host);

/*
 * Same as rsparse_prepare, with the factors supplied by the caller (closed form or an external SVD):
 * U16_host [d_out][rank] and SV16_host [rank][d_in] (= S_r V_r^T), host, 16-bit of cfg->dtype.
 * Both may be NULL when rank == 0.  The product U_r (S_r V_r^T) equals the paper's A_r B_r.
 */
rsparse_status rsparse_prepare_factors(const rsparse_config *cfg, const void *W_host,
                                       const void *U16_host, const void *SV16_host,
                                       rsparse_layer **out);

/*
 * The same layer on 4-bit weights (Sec. 4.4 combines R-Sparse with 4-bit GPTQ weights in groups of 128 and
 * names a kernel that fuses sparsity and dequantisation as the open efficiency gain).  The weights arrive in
 * GPTQ's storage format, all host: Q_host [d_out][d_in] codes 0..15, one per byte; S16_host
 * [d_out][d_in / group_size] scales, 16-bit of cfg->dtype; Z_host [d_out][d_in / group_size] zero points
 * 0..15, one per byte.  The weight they stand for is W~[o][c] = s[o][g] * (q[o][c] - z[o][g]),
 * g = c / group_size, and the layer computes Sec. 3.4's formula with W~ in place of W; the factors
 * U16_host / SV16_host stay 16-bit and are the caller's (of the unquantised W, or of W~).  group_size: a power
 * of two in [32, 1024] that divides d_in.  The library packs the codes channel-major (one kept channel = one
 * contiguous run of d_out / 2 bytes) and dequantises in registers: per quantisation group it accumulates
 * sum x_c q_c and sum x_c and applies scale and zero point once.  Limits of this path: no matrix-core path
 * (batches above 4 tokens run as tiles of 4, the codes streamed once per tile); rsparse_linear and friends run it as
 * two launches per layer by default (tuning launches = 1 selects a one-launch form, measured no faster); grouped
 * calls and rsparse_mlp_gate_up take such layers one at a time.  rsparse_dense_ref gives the dense product with W~:
 * with dense_rowmajor = 1 (a second, row-major copy of the codes, scales and zero points: + d_in * d_out / 2 bytes)
 * as a row-dot GEMV over row-major codes, the form a dense 4-bit decoder would use (tuning dense_kernel = 1 forces the
 * other form); without it through the channel-major kernel with every channel kept.
 * Non-finite inputs: NaN behaves as on 16-bit weights (never kept, reaches every output through the low-rank part; with
 * rank 0 it is simply dropped).  A KEPT channel whose value is +-Inf makes the outputs of that token NaN here, where
 * W~ x by the definition above would give +-Inf or NaN output by output: the group sums sum x_c q_c - z sum x_c meet
 * Inf - Inf.  -0 is 0.
 */
rsparse_status rsparse_prepare_q4(const rsparse_config *cfg, const uint8_t *Q_host, const void *S16_host,
                                  const uint8_t *Z_host, int32_t group_size, const void *U16_host,
                                  const void *SV16_host, rsparse_layer **out);

/*
 * The hot path (Sec. 3.4): threshold X, build the kept-channel lists, gather-multiply the
 * kept columns of W, run the other channels through the rank-r factors, sum, round once.
 * X_dev: device, [batch][d_in] 16-bit, 16-byte aligned.  Y_dev: device, [batch][d_out] of
 * out_dtype, 16-byte aligned.  stream: a hipStream_t (NULL = default stream).  Asynchronous:
 * returns after enqueueing; no allocation, no synchronisation.
 */
rsparse_status rsparse_linear(rsparse_layer *layer, const void *X_dev, int32_t batch,
                              void *Y_dev, void *stream);

/*
 * rsparse_linear for callers that cannot allocate device memory while they run -- code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc: same arguments, same result, but the call's scratch
 * (partial sums, arrival counters, the hand-off of the low-rank intermediate, the kept-channel lists) lies in a
 * file-scope device array of 2 MiB inside the library instead of in buffers the handle allocated, and the call
 * itself allocates and frees nothing (no hipMalloc / hipFree, no allocating library routine; the array's device
 * address is looked up once per device, on the first call there).  Each GPU the library runs on holds its copy of
 * the array until the process ends.  Limits: 16-bit weights, batch <= 8, d_in and d_out <= 32768, rank <= 2048;
 * anything larger is rejected with RSPARSE_EBATCH / RSPARSE_EINVAL before anything is launched.  Runs the vector
 * path (never the matrix cores) preceded by one small fill launch that clears the part of the array the call uses,
 * all on `stream` and capturable.  Every call on a GPU shares that GPU's array: calls that overlap on one GPU
 * (different streams, different handles) race -- order them.  rsparse_last_active and rsparse_synchronize work
 * afterwards as long as no other rsparse_linear_static call has run on that GPU in between.
 */
rsparse_status rsparse_linear_static(rsparse_layer *layer, const void *X_dev, int32_t batch,
                                     void *Y_dev, void *stream);

/*
 * The same layer applied to the gated MLP input (Sec. 3.1: H = X W_up^T (.) sigma(X W_gate^T) feeds the
 * down projection; Sec. 3.4 sparsifies that input like any other): x = round(silu(g) * u), rounded
 * once to the layer's 16-bit type and written to the handle's scratch by one small launch ahead of
 * the layer's own.  G_dev, Up_dev: device, [batch][d_in] 16-bit of cfg.dtype, 16-byte aligned (the
 * outputs of the gate and up projections).  silu is evaluated by a fixed fp32 recipe (range
 * reduction x = -g = n ln2 + r, degree-7 polynomial for exp(r), one division) so that the 16-bit x,
 * and with it the kept-channel sets, are reproducible bit for bit; it is within 3 ulp (fp32; measured 2.4) of
 * g / (1 + exp(-g)).  Everything else as rsparse_linear (rsparse_last_active reports the kept
 * channels of x).
 */
rsparse_status rsparse_linear_gated(rsparse_layer *layer, const void *G_dev, const void *Up_dev,
                                    int32_t batch, void *Y_dev, void *stream);

/*
 * The first half of the MLP (Sec. 3.1: H = X W_up^T (.) silu(X W_gate^T)) with R-Sparse on both
 * projections (Sec. 3.4): H_dev [batch][d_out] receives round(silu(g) * u), where g and u are the two
 * layers' outputs, each rounded once to the 16-bit type first -- i.e. what rsparse_linear on `gate` and on
 * `up` followed by rsparse_gated_input would store, without storing g and u.  gate, up: distinct
 * handles with equal d_in, d_out and dtype, out_dtype == dtype; X_dev, H_dev as in rsparse_linear.
 * Up to 8 tokens on the vector path this is ONE launch (the last workgroup of each column tile applies
 * the activation); other cases run the two layers into the handles' scratch and then one elementwise
 * launch.  rsparse_last_active works on either handle afterwards.
 */
rsparse_status rsparse_mlp_gate_up(rsparse_layer *gate, rsparse_layer *up, const void *X_dev,
                                   int32_t batch, void *H_dev, void *stream);

/*
 * The gated input on its own: out[i] = round(silu(G[i]) * Up[i]) for n values (n a multiple of 8), all
 * three device buffers of 16-bit `dtype`, 16-byte aligned; the recipe of rsparse_linear_gated (Sec. 3.1).  Asynchronous on `stream`.
 */
rsparse_status rsparse_gated_input(const void *G_dev, const void *Up_dev, void *out_dev, size_t n,
                                   int32_t dtype, void *stream);

/* The full layer Y = X W^T (Sec. 3.1) with the hand-written dense GEMV; same argument rules. */
rsparse_status rsparse_dense_ref(rsparse_layer *layer, const void *X_dev, int32_t batch,
                                 void *Y_dev, void *stream);

/*
 * Several layers applied to the SAME input in one pair of launches -- q/k/v, or gate/up of the MLP
 * (Sec. 3.1: H = X W_up^T (.) sigma(X W_gate^T); Sec. 3.4 applies R-Sparse to every linear layer).
 * layers: host array of n_layers (1..RSPARSE_MAX_GROUP) distinct handles with equal d_in and dtype;
 * each keeps its own tau, rank and d_out.  Y_devs: host array of n_layers device pointers.  Results
 * equal n_layers separate rsparse_linear / rsparse_dense_ref calls.  Launch-shape overrides
 * (waves, nontemporal, stages, dense_kernel) are taken from layers[0].
 */
#define RSPARSE_MAX_GROUP 4
rsparse_status rsparse_linear_group(rsparse_layer *const *layers, int32_t n_layers, const void *X_dev,
                                    int32_t batch, void *const *Y_devs, void *stream);
rsparse_status rsparse_dense_ref_group(rsparse_layer *const *layers, int32_t n_layers, const void *X_dev,
                                       int32_t batch, void *const *Y_devs, void *stream);

/*
 * rsparse_linear_group with the per-layer decision of rsparse_plan_layer applied: if the byte model plus the fixed
 * launch costs say that R-Sparse does not pay for these layers at this batch (small attention projections at any
 * batch; every layer from about 8 tokens on), the call runs rsparse_dense_ref_group instead -- the exact dense product,
 * which Sec. 3.5's per-layer recipe allows as the limit of zero sparsity.  keep_fraction: the share of channels one
 * token keeps at the layers' threshold (1 - the sparsity the threshold was calibrated for).  The decision is taken for
 * every layer with the group's size as `group`; if the layers disagree, each runs on its own as decided.  *used_rsparse_out (may be NULL): 1 if the R-Sparse path ran
 * for all layers, 0 if the dense one did for at least one.  After a dense run rsparse_last_active reports the previous
 * R-Sparse call.  Same arguments, asynchrony and errors as rsparse_linear_group.
 */
rsparse_status rsparse_linear_group_planned(rsparse_layer *const *layers, int32_t n_layers, const void *X_dev,
                                            int32_t batch, void *const *Y_devs, void *stream, double keep_fraction,
                                            int32_t *used_rsparse_out);

/*
 * Kept-channel index set of the last rsparse_linear call on this handle (synchronises that
 * call's stream).  token in [0, batch): that token's ascending list; token == -1: the ascending
 * union over the batch.  idx_host: host, room for d_in int32; *count receives the length.
 */
rsparse_status rsparse_last_active(rsparse_layer *layer, int32_t token, int32_t *idx_host,
                                   int32_t *count);

/*
 * Wait for the last rsparse_linear call on this handle (synchronises that call's stream) and report
 * device-side trouble: RSPARSE_EHIP if a bounded cross-workgroup wait of the one-launch kernel ran
 * out (the result of that call is then invalid; the handle stays usable).  For callers that want a
 * checked result; the hot path itself never synchronises and keeps returning RSPARSE_OK: after a wait has run out,
 * nothing computed on this handle may be trusted until rsparse_synchronize (or rsparse_last_active) has been called
 * on it -- that call reports the error once and puts the handle's counters, accumulators and hand-off entries back to
 * their idle state; calls enqueued before it may have read leftovers of the failed one.
 */
rsparse_status rsparse_synchronize(rsparse_layer *layer);

/* Stored 16-bit factors, host buffers U16 [d_out][rank] and SV16 [rank][d_in] (either may be NULL). */
rsparse_status rsparse_get_factors(const rsparse_layer *layer, void *U16_host, void *SV16_host);

/*
 * Static output bias (R-Sparse, Sec. 3.2: the part of the input below the sparse components can be approximated by a
 * few biases, which can be made static and pre-computed).  bias_host: [d_out] fp32 on the host, copied to the device
 * (owned by the handle), or NULL to remove it.  From then on rsparse_linear and its variants compute
 * Y = round(Y_s + Y_r + bias); rsparse_dense_ref does not add it.  Works with any rank (rank = 0 with cmp_mode = 2 is the
 * pure multi-phase form of Sec. 3.2).  Synchronises the device.  Errors: RSPARSE_EINVAL (NULL layer), RSPARSE_EHIP.
 */
rsparse_status rsparse_set_bias(rsparse_layer *layer, const float *bias_host);

/*
 * The static bias of the multi-phase activation of Sec. 3.2, host code (prepare time).  T[0] > T[1] > ... > T[l-1] are the
 * thresholds; a value h >= T[0] is a sparse component (kept as it is), a value in [T[i+1], T[i]) becomes the midpoint
 * (T[i] + T[i+1]) / 2 (values below T[l-1] count into the last interval; l = 1: everything below T[0] becomes 0).  For one
 * token the residual output is  sum_i midpoint_i * sum_{k in U_i} W[:, k]  with U_i the channels in interval i; the
 * static bias is its mean over the n_tokens calibration tokens H_host [n_tokens][d_in] (16-bit of `dtype`, host):
 *   bias[o] = sum_k W[o][k] * mean_tokens( midpoint of h_k's interval, or 0 if h_k >= T[0] ),  accumulated in fp64.
 * W_host [d_out][d_in] row-major 16-bit of `dtype`.  bias_out: [d_out] fp32, host, caller-owned.
 * Errors: RSPARSE_EINVAL (NULL pointers, sizes < 1, T not strictly decreasing or not finite).
 */
rsparse_status rsparse_multiphase_bias(const void *W_host, int32_t dtype, int32_t d_in, int32_t d_out, const void *H_host,
                                       int32_t n_tokens, const float *T, int32_t l, float *bias_out);

/* Threshold and launch-shape changes apply to calls made afterwards; a call already captured into a HIP
 * graph replays with the threshold, tuning and pointers it was captured with. */
rsparse_status rsparse_set_tau(rsparse_layer *layer, float tau);
rsparse_status rsparse_set_tuning(rsparse_layer *layer, const rsparse_tuning *tuning);
rsparse_status rsparse_get_config(const rsparse_layer *layer, rsparse_config *cfg_out);

/*
 * Threshold estimation (Sec. 3.4: P(|X| < t(s)) = s).  X_host: host, n 16-bit activations of
 * `dtype` pooled over the calibration tokens; s in [0,1].  *tau_out = the order statistic
 * a_(floor(s n)) of the ascending magnitudes (0-based, clamped, no interpolation).  Host code.
 */
rsparse_status rsparse_calibrate_tau(const void *X_host, int32_t dtype, size_t n, double s,
                                     float *tau_out);

/*
 * Bytes the method must move for one call (Sec. 3.4's I/O model, in bytes): the k_union kept
 * columns of W, both factors, X and Y.  rsparse_dense_bytes: all of W, X and Y.
 */
size_t rsparse_required_bytes(const rsparse_layer *layer, int32_t batch, int32_t k_union);
size_t rsparse_dense_bytes(const rsparse_layer *layer, int32_t batch);

/*
 * The same byte model from the layer's shape alone (host code, no handle, no device): Sec. 3.4 gives the
 * memory I/O of the layer relative to the full one as r (m + n) / (m n) + s, s the share of weight columns
 * loaded; in bytes, with e = 2 per 16-bit value, k_union kept channels, B = batch:
 *   *required_out = e (k d_out + r d_out + r d_in + B d_in) + e_out B d_out
 *   *dense_out    = e (d_in d_out + B d_in) + e_out B d_out
 *   *required_inactive_only_out = the same as required with r (d_in - k) for r d_in: what a layout of
 *                   S_r V_r^T that reads only the dropped channels' entries would move
 * (e_out = 4 for fp32 output).  q4_group = 0: 16-bit weights; otherwise the group size of 4-bit weights
 * (rsparse_prepare_q4): half a byte per weight plus 2.5 bytes per output and group that holds a kept channel.
 * Only d_in, d_out, rank, dtype and out_dtype of cfg matter (the rest must still be valid).  Any output
 * pointer may be NULL.
 */
rsparse_status rsparse_io_model(const rsparse_config *cfg, int32_t q4_group, int32_t batch, int32_t k_union,
                                size_t *required_out, size_t *dense_out, size_t *required_inactive_only_out);

/*
 * Sparsification recipe of one layer (Sec. 3.5): a budget C (memory I/O relative to the full layer)
 * is split by rho in [0,1] into a sparse part s = rho * C -- the fraction of weight columns that may
 * be loaded -- and a rank r = (1 - rho) * C * d_in*d_out / (d_in + d_out).  Host code.
 * *keep_fraction_out = s (so the threshold belongs at channel sparsity 1 - s, see rsparse_calibrate_tau);
 * *rank_out = r rounded down to a multiple of 8 (this library's rank granularity), clamped to
 * [0, min(d_in, d_out)].  *io_out (may be NULL) = the relative I/O of the rounded recipe,
 * r (d_in + d_out) / (d_in d_out) + s, the paper's cost model (Sec. 3.4).
 */
rsparse_status rsparse_recipe(int32_t d_in, int32_t d_out, double budget_c, double rho,
                              double *keep_fraction_out, int32_t *rank_out, double *io_out);

/*
 * Whether R-Sparse is expected to pay for one layer on this card: Sec. 3.4's I/O model in bytes (kept columns of W +
 * both factors, against all of W) plus the per-launch costs that do not scale with bytes.  Sec. 3.5 lets the recipe
 * differ per layer; this is the complementary per-layer decision to run a layer dense, e.g. the small attention
 * projections, or every layer once the batch is so large that the union of the tokens' kept channels is nearly all of
 * them.  keep_fraction: share of channels ONE token keeps (s of rsparse_recipe); for `batch` tokens the loaded columns
 * are their union, modelled as 1 - (1 - s)^batch.  group: layers that share one launch (rsparse_linear_group), whose
 * fixed cost they split.  Constants (MI355X, measured with this library, 16-bit weights): one token -- 6.5 TB/s
 * marginal rate, 8.5 us fixed per R-Sparse launch, 3.6 us per dense launch; 2-4 tokens (vector path) -- 6.7 TB/s,
 * 8.5 + 3 log2(batch) us; 5-32 tokens (matrix cores, all of W read) -- 4.65 TB/s, 15 us; dense from 2 tokens --
 * 5.26 TB/s, 7.3 us (4.86 TB/s, 9.2 us above 16 tokens).  The estimates land within about 20 % of the measured times
 * on the benchmark shapes.  Host code.  Any output pointer may be NULL.  Errors: RSPARSE_EINVAL.
 */
rsparse_status rsparse_plan_layer(int32_t d_in, int32_t d_out, int32_t rank, double keep_fraction, int32_t group,
                                  int32_t batch, double *us_rsparse_out, double *us_dense_out, int32_t *use_rsparse_out);

/*
 * Search for the per-layer shares rho_i of the sparse part (Sec. 3.5, the search algorithm for the
 * sparsification recipe): a population of `population` recipes, `generations` rounds of mutation
 * m = rho^{x1} + p_m (rho^{x2} - rho^{x3}) and coordinate-wise crossover (mutant where alpha > p_c), the
 * lowest-loss `population` of parents and offspring survive; layers are optimised `group_size` at a
 * time with the others held at the best recipe so far.  The paper runs population 32, 5 generations,
 * p_m = p_c = 0.5, groups of 28 with the model's perplexity as loss; the loss here is the caller's:
 * loss(rho, n_layers, user), called from this thread only.  Recipes stay in [lo, hi]; rho_start (may
 * be NULL = random) seeds the best-so-far.  rho_out [n_layers], *loss_out receive the best recipe;
 * history_out (may be NULL) has room for 1 + ceil(n_layers / group_size) * generations best-loss values.
 * Deterministic for a given seed.  Host code, no device needed; feed the result to rsparse_recipe.
 */
typedef double (*rsparse_loss_fn)(const double *rho, int32_t n_layers, void *user);
rsparse_status rsparse_search_recipe(rsparse_loss_fn loss, void *user, int32_t n_layers, int32_t population,
                                     int32_t generations, double p_m, double p_c, int32_t group_size,
                                     uint64_t seed, double lo, double hi, const double *rho_start,
                                     double *rho_out, double *loss_out, double *history_out);

/*
 * Measurement aid, only in libraries built with RSPARSE_STAMPS=1 (python -m paper_2504_19449_amd.build --stamps; any other
 * build returns RSPARSE_EINVAL): from now on every wave of the strip kernel's launches writes one record of 16
 * 64-bit words into buf_dev (device, room for capacity_waves records; record i belongs to wave i of the launch,
 * workgroups in grid order) -- word 0: kind (0 strip wave, 1 stage-1 wave, 2 strip wave that finished a split
 * strip) | workgroup << 8 | wave << 40; words 1..14: the 100 MHz wall clock at the wave's phase boundaries (0 = phase
 * not reached); word 15: rows streamed.  NULL / 0 switches it off.  Launches overwrite each other's records.
 */
rsparse_status rsparse_debug_stamps(void *buf_dev, int32_t capacity_waves);

void rsparse_destroy(rsparse_layer *layer);

const char *rsparse_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RSPARSE_H */
