// gfx950 matrix-core path of the R-Sparse linear layer for batch > 8 (R-Sparse, Sec. 3.4).
//
// At 16-32 tokens the union of kept channels is ~all of them (measured 99.5 % at 16 tokens with
// 50 % per-token sparsity), and 2*B flops per weight byte is more than the vector ALU sustains
// at HBM speed, so all three products become skinny GEMMs on MFMA, still one pass over the
// weights:
//
//   Y_s = (X (.) m)  W^T            rows of W   [d_out][d_in] row-major  (dense, per-token masks in X)
//   t   = (X (.) !m) (S_r V_r^T)^T  rows of SVt [r][d_in]
//   Y   = round(Y_s + t U_r^T)      rows of U   [d_out][r]
//
// All three weight matrices are stored "output row major, contraction index contiguous", which is
// exactly the operand layout of v_mfma_f32_16x16x32_{bf16,f16}: lane l supplies 8 consecutive k
// (one 16-byte load) of row l%16 at k-group l/16.  A = 16 weight rows x 32 k, B = 32 k x 16
// tokens (from LDS), D[row][token] fp32: lane l, register j holds row 4*(l/16)+j, token l%16.
//
// Launch 1 (k_mfma_sparse_and_t): grid = (row groups of W + row groups of SVt) x K slices; a row group is a balanced
// share of the matrix's 16-row blocks, the number of groups such that the grid is two rounds of one workgroup per
// compute unit.  A workgroup stages the masked tokens of ITS K slice once (kept part for W rows, dropped part for SVt
// rows; the slice is sized to fill the 64 KiB of LDS a workgroup may use) and then streams all its 16-row blocks
// against it with no further barrier: eight 16-byte weight loads per lane and batch, two batches in flight, a block's
// D tile in registers until its slice is done, then added to yacc / t_acc (both [row][16 or 32 tokens]) with fp32
// atomics (one add per K slice and output; stored directly when there is one slice).
// Between the launches (k_mfma_split_t): t_acc -> two 16-bit halves hi + lo (so the contraction keeps ~16 mantissa
// bits of the fp32 t), [token][rank]; t_acc re-zeroed.
// Launch 2 (k_mfma_finish): D = U_r t from the staged halves, Y = round(yacc + D + bias), yacc re-zeroed.
#include "kernels.h"
#include "device_common.h"

#include <algorithm>

namespace rsparse {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMfmaK = 32;        // contraction depth of one MFMA
constexpr int kMfmaUnroll = 8;    // weight loads in flight per lane
constexpr int kRowsPerBlock = 16;

template <int DT>
__device__ __forceinline__ f32x4 mfma16(const u32x4 a, const u32x4 b, const f32x4 c)
{
    if (DT == BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

template <int DT>
__device__ __forceinline__ uint16_t narrow(float f) { return DT == F16 ? to_f16(f) : to_bf16(f); }
template <int DT>
__device__ __forceinline__ float widen(uint16_t h)
{
    return DT == F16 ? (float)__builtin_bit_cast(_Float16, h) : as_f((uint32_t)h << 16);
}

struct MfmaArgs {
    LayerView L;
    const uint16_t *X;
    int batch, tok_pad;          // tokens, padded to 16 or 32
    int ks;                      // K slice staged in LDS, multiple of 32 * kMfmaUnroll
    int k_slices;
    int w_chunks, t_chunks;      // row groups of W and of SVt (balanced shares of their 16-row blocks);
                                 // grid.x = (w_chunks + t_chunks) * k_slices
    uint32_t *chan_bits;         // [d_in] bit b = token b keeps the channel (read-back)
    int dense;                   // 1: dense baseline -- every channel kept, no masks, no stage 1
};

constexpr int kStageBatch = 8;      // 16-byte token loads in flight per thread while staging

// One batch of weight loads of a 16-row block: kMfmaUnroll steps of 32 k, starting at step s0.
__device__ __forceinline__ void load_a_batch(const uint16_t *__restrict__ rowptr, bool row_ok, int klen, int s0, int kg,
                                             u32x4 (&v)[kMfmaUnroll])
{
#pragma unroll
    for (int u = 0; u < kMfmaUnroll; ++u) {
        const int k = (s0 + u) * kMfmaK + kg;
        v[u] = (row_ok && k < klen) ? *reinterpret_cast<const u32x4 *>(rowptr + k) : u32x4{0, 0, 0, 0};
    }
}

template <int DT>
__device__ __forceinline__ void mfma_a_batch(const u32x4 (&v)[kMfmaUnroll], int s0, const unsigned char *b_lo,
                                             const unsigned char *b_hi, bool two, f32x4 &acc0, f32x4 &acc1)
{
#pragma unroll
    for (int u = 0; u < kMfmaUnroll; ++u) {
        const size_t off = (size_t)(s0 + u) * kMfmaK * 2;
        acc0 = mfma16<DT>(v[u], *reinterpret_cast<const u32x4 *>(b_lo + off), acc0);
        if (two) acc1 = mfma16<DT>(v[u], *reinterpret_cast<const u32x4 *>(b_hi + off), acc1);
    }
}

template <int DT>
__global__ __launch_bounds__(256) void k_mfma_sparse_and_t(const MfmaArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const LayerView &L = a.L;
    const int d_in = L.d_in;
    const int ksl = blockIdx.x % a.k_slices;
    int rc = blockIdx.x / a.k_slices;
    const bool is_t = rc >= a.w_chunks;
    if (is_t) rc -= a.w_chunks;
    const int nq = a.ks / 8;                            // 16-byte pieces per token in the slice
    const int pitch = a.ks * 2 + 16;                    // odd multiple of 16 bytes: conflict-free B reads
    unsigned char *s_act = smem;                        // [tok_pad][pitch]
    const bool union_all = L.batch_mask_mode == 1 && !a.dense;
    const bool publish = !is_t && rc == 0 && !a.dense;  // these workgroups cover every channel once
    const int k0 = ksl * a.ks;
    const int klen = min(a.ks, d_in - k0);              // > 0 by construction of k_slices
    const uint32_t all_tokens = a.batch >= 32 ? 0xffffffffu : ((1u << a.batch) - 1u);
    // the layer's threshold as a rule (the fixed-count activation never takes this path: its rules are per token)
    const KeepRule thr = {L.tau_ge, __builtin_nanf(""), -1, 0};

    // ---- per-channel keep bits of every token: needed for the union mask and for read-back
    uint32_t *s_bits = reinterpret_cast<uint32_t *>(smem + (size_t)a.tok_pad * pitch);   // [ks]
    if (union_all || publish) {
        for (int i = tid; i < a.ks; i += 256) s_bits[i] = 0u;
        __syncthreads();
        for (int q = tid; q < a.tok_pad * nq; q += 256) {
            const int tok = q / nq, kq = q % nq;
            if (tok < a.batch && kq * 8 < klen) {
                float f[8];
                unpack8<DT>(*reinterpret_cast<const u32x4 *>(a.X + (size_t)tok * d_in + k0 + kq * 8), f);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (keep(f[e], k0 + kq * 8 + e, thr, L.keep_signed != 0)) atomicOr(&s_bits[kq * 8 + e], 1u << tok);
            }
        }
        __syncthreads();
        if (publish)
            for (int i = tid; i < klen; i += 256) a.chan_bits[k0 + i] = union_all && s_bits[i] ? all_tokens : s_bits[i];
    }

    // ---- stage the kept part (W rows) or the dropped part (SVt rows) of every token, once.
    //      All of a round's loads are issued before the first is used (one L2 round trip per round).
    const int total = a.tok_pad * nq;
    for (int q0 = tid; q0 < total; q0 += 256 * kStageBatch) {
        u32x4 raw[kStageBatch];
#pragma unroll
        for (int u = 0; u < kStageBatch; ++u) {
            const int q = q0 + u * 256;
            const int tok = q / nq, kq = q % nq;
            raw[u] = (q < total && tok < a.batch && kq * 8 < klen)
                         ? *reinterpret_cast<const u32x4 *>(a.X + (size_t)tok * d_in + k0 + kq * 8)
                         : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < kStageBatch; ++u) {
            const int q = q0 + u * 256;
            if (q < total) {
                const int tok = q / nq, kq = q % nq;
                u32x4 o = raw[u];
                if (!a.dense) {
                    float f[8];
                    unpack8<DT>(o, f);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const bool kept = union_all ? s_bits[kq * 8 + e] != 0u : keep(f[e], k0 + kq * 8 + e, thr, L.keep_signed != 0);
                        if (kept == is_t) o[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;   // not this part's
                    }
                }
                *reinterpret_cast<u32x4 *>(s_act + (size_t)tok * pitch + kq * 16) = o;
            }
        }
    }
    __syncthreads();

    // ---- stream my 16-row blocks against the staged slice: no barrier from here on
    const uint16_t *Mat = is_t ? L.SVt : L.Wrow;
    const int nrows = is_t ? L.rank : L.d_out;
    float *out = is_t ? L.t_acc : L.yacc;               // both [row][tok_pad]
    const int kg = (lane >> 4) * 8;
    const unsigned char *b_lo = s_act + (size_t)(lane & 15) * pitch + kg * 2;
    const unsigned char *b_hi = b_lo + (size_t)16 * pitch;
    const bool two = a.tok_pad > 16;
    const bool direct = a.k_slices == 1;
    const int tok = lane & 15;
    const int bpb = a.ks / (kMfmaK * kMfmaUnroll);      // batches per block
    // my balanced share of the matrix's 16-row blocks: the first (blocks % groups) groups hold one block more
    const int nblk = (nrows + kRowsPerBlock - 1) / kRowsPerBlock, ngrp = is_t ? a.t_chunks : a.w_chunks;
    const int bbase = nblk / ngrp, brem = nblk % ngrp;
    const int blk_lo = rc * bbase + min(rc, brem);
    const int blocks = bbase + (rc < brem ? 1 : 0);     // >= 1: the host keeps groups <= blocks
    const int row_base = blk_lo * kRowsPerBlock;
    const int my_blocks = blocks > w ? (blocks - w + 3) / 4 : 0;                                     // blocks w, w+4, ...
    const int n_batches = my_blocks * bpb;

    auto row_of = [&](int batch_i, const uint16_t *&rowptr, bool &row_ok) {
        const int row = row_base + (w + 4 * (batch_i / bpb)) * kRowsPerBlock + (lane & 15);
        row_ok = row < nrows;
        rowptr = Mat + (size_t)(row_ok ? row : 0) * d_in + k0;
    };
    auto flush = [&](int batch_i, f32x4 &acc0, f32x4 &acc1) {
        const int row0 = row_base + (w + 4 * (batch_i / bpb)) * kRowsPerBlock;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int orow = row0 + 4 * (lane >> 4) + j;
            if (orow < nrows) {
                // the accumulators of Y and of t are [row][tok_pad], so that the 16 lanes of one D register hit one
                // 64-byte run instead of 16 lines (t used to be [token][rank]: 64 separate lines per atomic
                // instruction, and the few workgroups that own the rows of S_r V_r^T finished last)
                float *p0 = out + (size_t)orow * a.tok_pad + tok;
                float *p1 = p0 + 16;
                if (direct) {
                    if (tok < a.batch) *p0 = acc0[j];
                    if (tok + 16 < a.batch) *p1 = acc1[j];
                } else {
                    if (tok < a.batch) __hip_atomic_fetch_add(p0, acc0[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (tok + 16 < a.batch) __hip_atomic_fetch_add(p1, acc1[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        acc0 = f32x4{0.f, 0.f, 0.f, 0.f};
        acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
    };

    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    u32x4 va[kMfmaUnroll], vb[kMfmaUnroll];
    const uint16_t *rowptr;
    bool row_ok;
    if (n_batches > 0) {
        row_of(0, rowptr, row_ok);
        load_a_batch(rowptr, row_ok, klen, 0, kg, va);
    }
    for (int i = 0; i < n_batches; i += 2) {
        if (i + 1 < n_batches) {
            row_of(i + 1, rowptr, row_ok);
            load_a_batch(rowptr, row_ok, klen, ((i + 1) % bpb) * kMfmaUnroll, kg, vb);
        }
        mfma_a_batch<DT>(va, (i % bpb) * kMfmaUnroll, b_lo, b_hi, two, acc0, acc1);
        if (i % bpb == bpb - 1) flush(i, acc0, acc1);
        if (i + 1 >= n_batches) break;
        if (i + 2 < n_batches) {
            row_of(i + 2, rowptr, row_ok);
            load_a_batch(rowptr, row_ok, klen, ((i + 2) % bpb) * kMfmaUnroll, kg, va);
        }
        mfma_a_batch<DT>(vb, ((i + 1) % bpb) * kMfmaUnroll, b_lo, b_hi, two, acc0, acc1);
        if ((i + 1) % bpb == bpb - 1) flush(i + 1, acc0, acc1);
    }
}

// The lo half of t is stored scaled by a power of two (exact): in fp16 the remainder t - hi would otherwise fall into
// the subnormals for |t| below ~0.1 and lose the bits it is there to keep.
template <int DT> struct LoScale { static constexpr float value = DT == F16 ? 2048.0f : 1.0f; };

// Between the two launches: t_acc [rank][tok_pad] fp32 (complete now: the launch that summed it has ended) ->
// t_hi, t_lo [tok_pad][rank] in the storage type, t = hi + lo / scale, so that the contraction with U_r keeps ~16
// mantissa bits of t; puts t_acc back to zero for the next call.  One thread per (rank index, four tokens).
template <int DT>
__global__ __launch_bounds__(256) void k_mfma_split_t(float *t_acc, int rank, int tok_pad, uint16_t *t_hi, uint16_t *t_lo)
{
    const int q = tok_pad / 4;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= rank * q) return;
    const int k = i / q, tok0 = (i % q) * 4;
    float4 *src = reinterpret_cast<float4 *>(t_acc + (size_t)k * tok_pad + tok0);
    const float4 v4 = *src;
    *src = float4{0.f, 0.f, 0.f, 0.f};
    const float v[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint16_t hi = narrow<DT>(v[e]);
        const uint16_t lo = narrow<DT>((v[e] - widen<DT>(hi)) * LoScale<DT>::value);
        t_hi[(size_t)(tok0 + e) * rank + k] = hi;
        t_lo[(size_t)(tok0 + e) * rank + k] = lo;
    }
}

struct MfmaFinishArgs {
    LayerView L;
    void *Y;
    int batch, tok_pad;
    int use_rank;
    const uint16_t *t_hi, *t_lo; // [tok_pad][rank] each: t = hi + lo / kLoScale in the storage type (k_mfma_split_t)
};

// Second launch: Y = round(yacc + U_r t + bias).  One wave = one 16-row block of U_r, a workgroup = 64 output rows.
// t arrives already split into its two 16-bit halves (k_mfma_split_t) and is staged through LDS in chunks of 256 rank
// indices (the MFMA B operand of all four waves); nothing a chunk needs depends on what the kernel computes, so the
// U_r loads run three chunks ahead and the t loads one chunk ahead, the latter issued BEFORE the former so that they
// do not queue behind them (loads return in order).
// Tried and dropped: both operands straight from memory, no LDS -- the 128 KiB of t do not stay in the first-level
// cache and every workgroup's re-reads went to L2: 20 us instead of 14 us at 8192 x 1024, 60 instead of 23 us at
// 28672 x 1024 (32 tokens).
template <int DT>
__global__ __launch_bounds__(256) void k_mfma_finish(const MfmaFinishArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const LayerView &L = a.L;
    const int d_out = L.d_out, r = a.use_rank;
    constexpr int RC = kMfmaK * kMfmaUnroll;                         // rank indices per chunk: one batch of U loads per lane
    const int pitch = RC * 2 + 16;
    unsigned char *s_hi = smem, *s_lo = smem + (size_t)a.tok_pad * pitch;
    const int row0 = (blockIdx.x * 4 + w) * kRowsPerBlock;
    const int row = row0 + (lane & 15);
    const bool row_ok = row < d_out;
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    f32x4 lo0 = {0.f, 0.f, 0.f, 0.f}, lo1 = {0.f, 0.f, 0.f, 0.f};    // the lo halves' products, scaled by kLoScale
    constexpr float kLoScale = LoScale<DT>::value;
    const int kg = (lane >> 4) * 8;
    const size_t lane_off = (size_t)(lane & 15) * pitch + kg * 2;
    const bool two = a.tok_pad > 16;
    const uint16_t *urow = L.U + (size_t)(row_ok ? row : 0) * r;
    const int rc8 = RC / 8, total8 = a.tok_pad * rc8;                // 16-byte pieces of one staged chunk (per half)
    constexpr int kTV = 4;                                           // pieces per thread and half: 32 tokens x 256 / 8 / 256 threads
    u32x4 th[kTV], tl[kTV];
    auto request_t = [&](int c0) {
        const int clen = min(RC, r - c0);
#pragma unroll
        for (int u = 0; u < kTV; ++u) {
            const int i = tid + u * 256;
            const int tok = i / rc8, k = (i % rc8) * 8;
            const bool ok = i < total8 && k < clen;                  // rows of tokens past the batch hold zeros
            th[u] = ok ? *reinterpret_cast<const u32x4 *>(a.t_hi + (size_t)tok * r + c0 + k) : u32x4{0, 0, 0, 0};
            tl[u] = ok ? *reinterpret_cast<const u32x4 *>(a.t_lo + (size_t)tok * r + c0 + k) : u32x4{0, 0, 0, 0};
        }
    };
    auto stage_t = [&]() {
#pragma unroll
        for (int u = 0; u < kTV; ++u) {
            const int i = tid + u * 256;
            if (i < total8) {
                const int tok = i / rc8, k = (i % rc8) * 8;
                *reinterpret_cast<u32x4 *>(s_hi + (size_t)tok * pitch + k * 2) = th[u];
                *reinterpret_cast<u32x4 *>(s_lo + (size_t)tok * pitch + k * 2) = tl[u];
            }
        }
    };
    auto both_halves = [&](const u32x4 (&v)[kMfmaUnroll]) {
        mfma_a_batch<DT>(v, 0, s_hi + lane_off, s_hi + lane_off + (size_t)16 * pitch, two, acc0, acc1);
        mfma_a_batch<DT>(v, 0, s_lo + lane_off, s_lo + lane_off + (size_t)16 * pitch, two, lo0, lo1);
    };
    // the epilogue's inputs do not depend on the products either: requested first
    const int orow = row0 + 4 * (lane >> 4);
    float ya[2][4];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int tok = (lane & 15) + 16 * half;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            ya[half][j] = (orow + j < d_out && tok < a.batch) ? L.yacc[(size_t)(orow + j) * a.tok_pad + tok] : 0.f;
    }
    const int nch = (r + RC - 1) / RC;
    u32x4 ua[4][kMfmaUnroll];                                        // ring of U batches, chunk c in slot c % 4
#pragma unroll
    for (int c = 0; c < 3; ++c)
        if (c < nch) load_a_batch(urow + c * RC, row_ok, min(RC, r - c * RC), 0, kg, ua[c]);
    if (nch > 0) request_t(0);
    for (int c0 = 0; c0 < nch; c0 += 4) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = c0 + i;
            if (c < nch) {                                           // wave-uniform
                if (c > 0) __syncthreads();                          // every wave has read the chunk before
                stage_t();
                __syncthreads();
                if (c + 1 < nch) request_t((c + 1) * RC);
                if (c + 3 < nch) load_a_batch(urow + (c + 3) * RC, row_ok, min(RC, r - (c + 3) * RC), 0, kg, ua[(i + 3) & 3]);
                both_halves(ua[i]);
            }
        }
    }
    // lane l holds rows row0 + 4*(l/16) + 0..3 of token l%16 (and l%16 + 16): 4 consecutive outputs
    if (orow < d_out) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int tok = (lane & 15) + 16 * half;
            if (tok < a.batch) {
                const f32x4 acc = half ? acc1 : acc0, lo = half ? lo1 : lo0;
                float *yp = L.yacc + (size_t)orow * a.tok_pad + tok;          // [row][tok_pad], see launch 1
                float o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    o[j] = ya[half][j] + acc[j] + lo[j] * (1.0f / kLoScale) + (orow + j < d_out ? bias_at(L, orow + j) : 0.f);
                const size_t oi = (size_t)tok * d_out + orow;
                if (L.out_dtype == F32) {
                    *reinterpret_cast<float4 *>((float *)a.Y + oi) = float4{o[0], o[1], o[2], o[3]};
                } else {
                    uint2 pk;
                    pk.x = (uint32_t)narrow<DT>(o[0]) | ((uint32_t)narrow<DT>(o[1]) << 16);
                    pk.y = (uint32_t)narrow<DT>(o[2]) | ((uint32_t)narrow<DT>(o[3]) << 16);
                    *reinterpret_cast<uint2 *>((uint16_t *)a.Y + oi) = pk;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (orow + j < d_out) yp[(size_t)j * a.tok_pad] = 0.f;
            }
        }
    }
}

}  // namespace

namespace {
// K slice: a few load batches (256 k each) of every token in LDS next to the keep-bit words, so that 3-4 workgroups
// fit a compute unit; slices are evened out over d_in (measured: 768 k for 17-32 tokens, 1024 k for up to 16; larger
// slices cost occupancy).  Returns the number of slices, ks = their length.
int mfma_k_slices(int d_in, int tok_pad, int &ks)
{
    constexpr int kStep = kMfmaK * kMfmaUnroll;
    const int ks_max = tok_pad > 16 ? 3 * kStep : 4 * kStep;
    int n = (d_in + ks_max - 1) / ks_max;
    ks = (((d_in + n - 1) / n + kStep - 1) / kStep) * kStep;
    return (d_in + ks - 1) / ks;
}
}  // namespace

bool mfma_path_supported(const LayerView &L, int batch)
{
    return batch >= 1 && batch <= 32 && L.Wrow != nullptr && (L.d_in % 8) == 0 && (L.d_out % 8) == 0;
}

hipError_t launch_mfma_linear(const LayerView &L, const void *X, int batch, void *Y, uint32_t *chan_bits, int cus,
                              int stages, bool dense, int rows_per_wg_hint, hipStream_t stream)
{
    const int tok_pad = batch > 16 ? 32 : 16;
    const int rank = dense ? 0 : L.rank;
    if (stages != 2) {
        MfmaArgs a{};
        a.L = L; a.X = (const uint16_t *)X; a.batch = batch; a.tok_pad = tok_pad; a.chan_bits = chan_bits;
        a.dense = dense ? 1 : 0;
        a.k_slices = mfma_k_slices(L.d_in, tok_pad, a.ks);
        // row groups: the 16-row blocks of W and of S_r V_r^T dealt out evenly to as many workgroups as two rounds of
        // one per compute unit (measured: with whole 64-row units the busiest compute unit carried 3 workgroups of 192
        // rows against an average of 2.1 -- 48.7 us against 32.6 us for the dense layer on 8192 x 8192 at 32 tokens,
        // for 12 % more rows)
        const int blk_w = (L.d_out + kRowsPerBlock - 1) / kRowsPerBlock, blk_t = (rank + kRowsPerBlock - 1) / kRowsPerBlock;
        int groups = std::max(1, (2 * cus) / a.k_slices);
        groups = std::max(1, std::min(groups, (blk_w + blk_t) / 4));        // at least one block per wave
        if (rows_per_wg_hint == 64 || rows_per_wg_hint == 128 || rows_per_wg_hint == 256)
            groups = std::max(1, (blk_w + blk_t) * kRowsPerBlock / rows_per_wg_hint);
        // the split of the groups between W and S_r V_r^T that keeps the largest share of blocks smallest
        int g_t = 0;
        if (rank > 0) {
            int best = 1 << 30;
            for (int t = 1; t < std::max(2, groups) && t <= blk_t; ++t) {
                const int w = std::max(1, std::min(blk_w, groups - t));
                const int worst = std::max((blk_t + t - 1) / t, (blk_w + w - 1) / w);
                if (worst < best) { best = worst; g_t = t; }
            }
        }
        const int g_w = std::max(1, std::min(blk_w, groups - g_t));
        a.w_chunks = g_w;
        a.t_chunks = g_t;
        const size_t lds = (size_t)tok_pad * (a.ks * 2 + 16) + (size_t)a.ks * 4;
        if (lds > 64 * 1024) return hipErrorInvalidValue;
        // stage 1 goes to t_acc (summed over the K slices with atomics, or stored when there is one slice), which the
        // split launch of the second stage leaves at zero; a first launch timed alone (stages = 1) clears it itself
        if (rank > 0 && (!L.t_acc || !L.t16)) return hipErrorInvalidValue;
        if (rank > 0 && stages != 0) {
            hipError_t e = launch_zero(L.t_acc, (size_t)tok_pad * L.rank, stream);
            if (e != hipSuccess) return e;
        }
        dim3 grid((a.w_chunks + a.t_chunks) * a.k_slices), block(256);
        if (L.dtype == F16) hipLaunchKernelGGL(k_mfma_sparse_and_t<F16>, grid, block, lds, stream, a);
        else hipLaunchKernelGGL(k_mfma_sparse_and_t<BF16>, grid, block, lds, stream, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (stages != 1) {
        MfmaFinishArgs f{};
        f.L = L; f.Y = Y; f.batch = batch; f.tok_pad = tok_pad; f.use_rank = rank;
        if (rank > 0) {
            if (!L.t_acc || !L.t16) return hipErrorInvalidValue;
            f.t_hi = L.t16;
            f.t_lo = L.t16 + (size_t)32 * L.rank;
            const int items = rank * (tok_pad / 4);
            dim3 sgrid((items + 255) / 256), sblock(256);
            if (L.dtype == F16) hipLaunchKernelGGL(k_mfma_split_t<F16>, sgrid, sblock, 0, stream, L.t_acc, rank, tok_pad, L.t16, L.t16 + (size_t)32 * L.rank);
            else hipLaunchKernelGGL(k_mfma_split_t<BF16>, sgrid, sblock, 0, stream, L.t_acc, rank, tok_pad, L.t16, L.t16 + (size_t)32 * L.rank);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        const size_t lds = 2 * (size_t)tok_pad * (kMfmaK * kMfmaUnroll * 2 + 16);
        dim3 grid((L.d_out + 63) / 64), block(256);
        if (L.dtype == F16) hipLaunchKernelGGL(k_mfma_finish<F16>, grid, block, lds, stream, f);
        else hipLaunchKernelGGL(k_mfma_finish<BF16>, grid, block, lds, stream, f);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rsparse
