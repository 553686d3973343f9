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
// Launch 1 (k_mfma_sparse_and_t): grid = (row chunks of W + row chunks of SVt) x K splits.  A
// workgroup walks its K range in LDS-sized chunks: it stages the masked tokens of the chunk (kept
// part for W rows, dropped part for SVt rows), each wave runs its 16-row blocks over it, and the D
// tiles stay in registers until the end; they are stored directly (one K split) or added to yacc / t
// with fp32 atomics (k_splits adds per output; t is then zeroed by a fill kernel first).
// Launch 2 (k_mfma_finish): t is split into hi + lo 16-bit halves (so the contraction keeps ~16
// mantissa bits of the fp32 t), D = U_r t, Y = round(yacc + D), yacc re-zeroed.
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
    int kc;                      // K chunk staged in LDS at a time, multiple of 32
    int k_splits;                // workgroups along K; each loops over chunks_per_split chunks
    int chunks_per_split;
    int rows_per_wg;             // multiple of 16, at most 64 * kMaxBlocksPerWave
    int w_chunks, t_chunks;      // row chunks of W and of SVt; grid.x = (w_chunks + t_chunks) * k_splits
    uint32_t *chan_bits;         // [d_in] bit b = token b keeps the channel (read-back)
    int dense;                   // 1: dense baseline -- every channel kept, no masks, no stage 1
};

constexpr int kMaxBlocksPerWave = 4;
constexpr int kStageBatch = 8;      // 16-byte token loads in flight per thread while staging

// One 16-row block over the staged K chunk: acc0 = tokens 0-15, acc1 = tokens 16-31.
template <int DT>
__device__ __forceinline__ void block_over_chunk(const uint16_t *__restrict__ rowptr, bool row_ok, int klen, int kc,
                                                 const unsigned char *s_act, int pitch, int tok_pad, int lane,
                                                 f32x4 &acc0, f32x4 &acc1)
{
    const int kg = (lane >> 4) * 8;                     // this lane's k offset inside a 32-deep step
    const unsigned char *b_lo = s_act + (size_t)(lane & 15) * pitch + kg * 2;
    const unsigned char *b_hi = b_lo + (size_t)16 * pitch;
    for (int ks = 0; ks < kc; ks += kMfmaK * kMfmaUnroll) {
        u32x4 v[kMfmaUnroll];
#pragma unroll
        for (int u = 0; u < kMfmaUnroll; ++u) {
            const int k = ks + u * kMfmaK + kg;
            v[u] = (row_ok && k < klen) ? *reinterpret_cast<const u32x4 *>(rowptr + k) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < kMfmaUnroll; ++u) {
            const int k = ks + u * kMfmaK;
            if (k < kc) {
                const u32x4 b0 = *reinterpret_cast<const u32x4 *>(b_lo + (size_t)k * 2);
                acc0 = mfma16<DT>(v[u], b0, acc0);
                if (tok_pad > 16) {
                    const u32x4 b1 = *reinterpret_cast<const u32x4 *>(b_hi + (size_t)k * 2);
                    acc1 = mfma16<DT>(v[u], b1, acc1);
                }
            }
        }
    }
}

// A workgroup owns rows_per_wg output rows (of W, or of S_r V_r^T) and one K split; it walks its K
// range in LDS-sized chunks, re-staging the masked tokens for each, and keeps the D tiles in
// registers throughout.  Results are stored directly when there is a single K split, else added
// with fp32 atomics (k_splits adds per output).
template <int DT>
__global__ __launch_bounds__(256) void k_mfma_sparse_and_t(const MfmaArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const LayerView &L = a.L;
    const int d_in = L.d_in;
    const int ksp = blockIdx.x % a.k_splits;
    int rc = blockIdx.x / a.k_splits;
    const bool is_t = rc >= a.w_chunks;
    if (is_t) rc -= a.w_chunks;
    const int nq = a.kc / 8;                            // 16-byte pieces per token in a chunk
    const int pitch = a.kc * 2 + 16;                    // odd multiple of 16 bytes: conflict-free B reads
    unsigned char *s_act = smem;                        // [tok_pad][pitch]
    uint32_t *s_bits = reinterpret_cast<uint32_t *>(smem + (size_t)a.tok_pad * pitch);   // [kc] per-channel token bits
    const bool union_all = L.batch_mask_mode == 1 && !a.dense;
    const bool publish = !is_t && rc == 0 && !a.dense;  // these workgroups cover every channel once

    const uint16_t *Mat = is_t ? L.SVt : L.Wrow;
    const int nrows = is_t ? L.rank : L.d_out;
    float *out = is_t ? L.t : L.yacc;                   // [token][nrows]
    const int blocks = a.rows_per_wg / kRowsPerBlock;

    f32x4 acc0[kMaxBlocksPerWave], acc1[kMaxBlocksPerWave];
#pragma unroll
    for (int bi = 0; bi < kMaxBlocksPerWave; ++bi) {
        acc0[bi] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc1[bi] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const int chunk_lo = ksp * a.chunks_per_split;
    for (int ci = 0; ci < a.chunks_per_split; ++ci) {
        const int k0 = (chunk_lo + ci) * a.kc;
        if (k0 >= d_in) break;
        const int klen = min(a.kc, d_in - k0);
        if (ci > 0) __syncthreads();
        // pass A: per-channel keep bits of every token (needed for the union mask and for read-back)
        if (union_all || publish) {
            for (int i = tid; i < a.kc; i += 256) s_bits[i] = 0u;
            __syncthreads();
            for (int q = tid; q < a.tok_pad * nq; q += 256) {
                const int tok = q / nq, kq = q % nq;
                if (tok < a.batch && kq * 8 < klen) {
                    float f[8];
                    unpack8<DT>(*reinterpret_cast<const u32x4 *>(a.X + (size_t)tok * d_in + k0 + kq * 8), f);
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (keep(f[e], L.tau, L.cmp_mode)) atomicOr(&s_bits[kq * 8 + e], 1u << tok);
                }
            }
            __syncthreads();
            if (union_all) {
                const uint32_t all = a.batch >= 32 ? 0xffffffffu : ((1u << a.batch) - 1u);
                for (int i = tid; i < a.kc; i += 256) s_bits[i] = s_bits[i] ? all : 0u;
                __syncthreads();
            }
            if (publish)
                for (int i = tid; i < klen; i += 256) a.chan_bits[k0 + i] = s_bits[i];
        }
        // pass B: stage the kept part (W rows) or the dropped part (SVt rows) of every token.
        // All of a batch's loads are issued before the first is used (one L2 round trip per batch).
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
                            const bool kept = union_all ? ((s_bits[kq * 8 + e] >> (tok & 31)) & 1u) != 0u
                                                        : keep(f[e], L.tau, L.cmp_mode);
                            if (kept == is_t) o[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;   // not this part's
                        }
                    }
                    *reinterpret_cast<u32x4 *>(s_act + (size_t)tok * pitch + kq * 16) = o;
                }
            }
        }
        __syncthreads();

#pragma unroll
        for (int bi = 0; bi < kMaxBlocksPerWave; ++bi) {
            const int blk = w + 4 * bi;
            const int row0 = rc * a.rows_per_wg + blk * kRowsPerBlock;
            if (blk < blocks && row0 < nrows) {
                const int row = row0 + (lane & 15);
                const bool row_ok = row < nrows;
                const uint16_t *rowptr = Mat + (size_t)(row_ok ? row : 0) * d_in + k0;
                block_over_chunk<DT>(rowptr, row_ok, klen, a.kc, s_act, pitch, a.tok_pad, lane, acc0[bi], acc1[bi]);
            }
        }
    }

    const int tok = lane & 15;
    const bool direct = a.k_splits == 1;
#pragma unroll
    for (int bi = 0; bi < kMaxBlocksPerWave; ++bi) {
        const int blk = w + 4 * bi;
        const int row0 = rc * a.rows_per_wg + blk * kRowsPerBlock;
        if (blk < blocks && row0 < nrows) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int orow = row0 + 4 * (lane >> 4) + j;
                if (orow < nrows) {
                    float *p0 = out + (size_t)tok * nrows + orow;
                    float *p1 = out + (size_t)(tok + 16) * nrows + orow;
                    if (direct) {
                        if (tok < a.batch) *p0 = acc0[bi][j];
                        if (tok + 16 < a.batch) *p1 = acc1[bi][j];
                    } else {
                        if (tok < a.batch) __hip_atomic_fetch_add(p0, acc0[bi][j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (tok + 16 < a.batch) __hip_atomic_fetch_add(p1, acc1[bi][j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
        }
    }
}

struct MfmaFinishArgs {
    LayerView L;
    void *Y;
    int batch, tok_pad;
    int rc;                      // chunk of the rank staged at a time, multiple of 32
    int use_rank;
};

// One wave = one 16-row block of U_r; a workgroup = 64 output rows.
template <int DT>
__global__ __launch_bounds__(256) void k_mfma_finish(const MfmaFinishArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const LayerView &L = a.L;
    const int d_out = L.d_out, r = a.use_rank;
    const int pitch = a.rc * 2 + 16;
    unsigned char *s_hi = smem, *s_lo = smem + (size_t)a.tok_pad * pitch;
    const int row0 = (blockIdx.x * 4 + w) * kRowsPerBlock;
    const int row = row0 + (lane & 15);
    const bool row_ok = row < d_out;
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};

    for (int c0 = 0; c0 < r; c0 += a.rc) {
        const int clen = min(a.rc, r - c0);
        if (c0 > 0) __syncthreads();
        // t = hi + lo in the storage type: the MFMA contraction then carries ~16 mantissa bits of t.
        // Four values per thread and step, a batch of loads issued before the first conversion.
        const int rc4 = a.rc / 4, total4 = a.tok_pad * rc4;
        for (int i0 = tid; i0 < total4; i0 += 256 * kStageBatch) {
            float4 tv[kStageBatch];
#pragma unroll
            for (int u = 0; u < kStageBatch; ++u) {
                const int i = i0 + u * 256;
                const int tok = i / rc4, k = (i % rc4) * 4;
                tv[u] = (i < total4 && tok < a.batch && k < clen)
                            ? *reinterpret_cast<const float4 *>(L.t + (size_t)tok * r + c0 + k)
                            : float4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < kStageBatch; ++u) {
                const int i = i0 + u * 256;
                if (i < total4) {
                    const int tok = i / rc4, k = (i % rc4) * 4;
                    const float v[4] = {tv[u].x, tv[u].y, tv[u].z, tv[u].w};
                    uint16_t hi[4], lo[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        hi[e] = narrow<DT>(v[e]);
                        lo[e] = narrow<DT>(v[e] - widen<DT>(hi[e]));
                    }
                    uint2 ph, pl;
                    ph.x = (uint32_t)hi[0] | ((uint32_t)hi[1] << 16); ph.y = (uint32_t)hi[2] | ((uint32_t)hi[3] << 16);
                    pl.x = (uint32_t)lo[0] | ((uint32_t)lo[1] << 16); pl.y = (uint32_t)lo[2] | ((uint32_t)lo[3] << 16);
                    *reinterpret_cast<uint2 *>(s_hi + (size_t)tok * pitch + k * 2) = ph;
                    *reinterpret_cast<uint2 *>(s_lo + (size_t)tok * pitch + k * 2) = pl;
                }
            }
        }
        __syncthreads();
        const uint16_t *rowptr = L.U + (size_t)(row_ok ? row : 0) * r + c0;
        block_over_chunk<DT>(rowptr, row_ok, clen, a.rc, s_hi, pitch, a.tok_pad, lane, acc0, acc1);
        block_over_chunk<DT>(rowptr, row_ok, clen, a.rc, s_lo, pitch, a.tok_pad, lane, acc0, acc1);
    }
    // lane l holds rows row0 + 4*(l/16) + 0..3 of token l%16 (and l%16 + 16): 4 consecutive outputs
    const int orow = row0 + 4 * (lane >> 4);
    if (orow < d_out) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int tok = (lane & 15) + 16 * half;
            if (tok < a.batch) {
                const f32x4 acc = half ? acc1 : acc0;
                float4 *yp = reinterpret_cast<float4 *>(L.yacc + (size_t)tok * d_out + orow);
                const float4 ya = *yp;
                const float o0 = ya.x + acc[0], o1 = ya.y + acc[1], o2 = ya.z + acc[2], o3 = ya.w + acc[3];
                const size_t oi = (size_t)tok * d_out + orow;
                if (L.out_dtype == F32) {
                    *reinterpret_cast<float4 *>((float *)a.Y + oi) = float4{o0, o1, o2, o3};
                } else {
                    uint2 pk;
                    pk.x = (uint32_t)narrow<DT>(o0) | ((uint32_t)narrow<DT>(o1) << 16);
                    pk.y = (uint32_t)narrow<DT>(o2) | ((uint32_t)narrow<DT>(o3) << 16);
                    *reinterpret_cast<uint2 *>((uint16_t *)a.Y + oi) = pk;
                }
                *yp = float4{0.f, 0.f, 0.f, 0.f};
            }
        }
    }
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
        a.kc = tok_pad > 16 ? 512 : 1024;
        if (a.kc > ((L.d_in + 31) / 32) * 32) a.kc = ((L.d_in + 31) / 32) * 32;
        const int n_kchunks = (L.d_in + a.kc - 1) / a.kc;
        // 64 output rows per workgroup (one 16-row block per wave), 128 for very wide layers; K is split
        // only as far as needed for ~3 workgroups per compute unit (k_splits atomic adds per output)
        const int rows_per_wg = (rows_per_wg_hint == 64 || rows_per_wg_hint == 128 || rows_per_wg_hint == 256)
                                    ? rows_per_wg_hint : (L.d_out / 128 >= 3 * cus ? 128 : 64);
        a.rows_per_wg = rows_per_wg;
        a.w_chunks = (L.d_out + rows_per_wg - 1) / rows_per_wg;
        a.t_chunks = rank > 0 ? (rank + rows_per_wg - 1) / rows_per_wg : 0;
        int k_splits = (3 * cus + a.w_chunks - 1) / a.w_chunks;
        k_splits = std::max(1, std::min(k_splits, n_kchunks));
        a.chunks_per_split = (n_kchunks + k_splits - 1) / k_splits;
        a.k_splits = (n_kchunks + a.chunks_per_split - 1) / a.chunks_per_split;
        const size_t lds = (size_t)tok_pad * (a.kc * 2 + 16) + (size_t)a.kc * 4;
        if (rank > 0 && a.k_splits > 1) {             // stage-1 partial sums meet in atomics: start from zero
            hipError_t e = launch_zero(L.t, (size_t)batch * L.rank, stream);
            if (e != hipSuccess) return e;
        }
        dim3 grid((a.w_chunks + a.t_chunks) * a.k_splits), block(256);
        if (L.dtype == F16) hipLaunchKernelGGL(k_mfma_sparse_and_t<F16>, grid, block, lds, stream, a);
        else hipLaunchKernelGGL(k_mfma_sparse_and_t<BF16>, grid, block, lds, stream, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (stages != 1) {
        MfmaFinishArgs f{};
        f.L = L; f.Y = Y; f.batch = batch; f.tok_pad = tok_pad; f.use_rank = rank;
        f.rc = tok_pad > 16 ? 256 : 512;
        const size_t lds = 2 * (size_t)tok_pad * (f.rc * 2 + 16);
        dim3 grid((L.d_out + 63) / 64), block(256);
        if (L.dtype == F16) hipLaunchKernelGGL(k_mfma_finish<F16>, grid, block, lds, stream, f);
        else hipLaunchKernelGGL(k_mfma_finish<BF16>, grid, block, lds, stream, f);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rsparse
