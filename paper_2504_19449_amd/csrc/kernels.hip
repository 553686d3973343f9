// gfx950 (MI355X, CDNA4) kernels of the R-Sparse linear layer (R-Sparse, Sec. 3.4).
//
// Everything here is bound by HBM bandwidth at decode batch sizes (2*B flops per 2-byte
// weight), so the kernels are organised around the weight stream: 16-byte loads, one
// 1 KiB row segment per 64-lane wave, many rows in flight, fp32 accumulation on the
// vector ALU.  Three storage layouts make all three products the same primitive
// "out[0:N] += coef_j * row_j[0:N]" or a plain row dot:
//
//   M    [d_in + r][d_out]   rows 0..d_in-1: W column-major (row c = all outputs of input
//                            channel c; Sec. 3.4 asks for this layout so a kept channel is one
//                            contiguous run); rows d_in..: U_r^T.  One row index space for both.
//   SVt  [r][d_in]           S_r V_r^T, one singular component per row.
//
//   stage 1 (k_lowrank_t)  t_i = SVt[i,:] . (x - sigma_t(x))           one workgroup per few rows
//   stage 2 (k_gather)     y   = sum_{c kept} x_c M[c,:] + sum_i t_i M[d_in+i,:]
//
// k_gather thresholds and compacts x itself (every workgroup scans the whole token -- 2*d_in
// bytes from L2 -- and keeps only its balanced share of the ascending kept list), so there
// is no separate compaction launch and no cross-workgroup dependency before the stream starts.
// Column tiles x channel splits fill the chip; partial sums meet in fp32 atomics, and the
// last workgroup to arrive at a column tile rounds it once and stores Y.
#include "kernels.h"

namespace rsparse {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

constexpr int F16 = 0, BF16 = 1, F32 = 2;
constexpr int kUnroll = 8;       // rows in flight per wave in the streaming loop

__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u(float f) { return __builtin_bit_cast(uint32_t, f); }

// Exact widening of eight packed 16-bit values (element 0 in the low half of word 0).
template <int DT>
__device__ __forceinline__ void unpack8(const u32x4 v, float (&f)[8])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (DT == F16) {
            const uint32_t word = v[i];      // bit_cast needs a scalar copy, not a vector-element lvalue
            h2 p = __builtin_bit_cast(h2, word);
            f[2 * i] = (float)p[0];          // v_cvt_f32_f16 keeps fp16 subnormals
            f[2 * i + 1] = (float)p[1];
        } else {
            f[2 * i] = as_f(v[i] << 16);
            f[2 * i + 1] = as_f(v[i] & 0xffff0000u);
        }
    }
}

// One round-to-nearest-even from the fp32 accumulator to the output type.
__device__ __forceinline__ uint16_t to_bf16(float f)
{
    uint32_t u = as_u(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint16_t to_f16(float f)
{
    _Float16 h = (_Float16)f;
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ void store_out(void *Y, size_t i, float v, int out_dtype)
{
    if (out_dtype == F32) ((float *)Y)[i] = v;
    else if (out_dtype == F16) ((uint16_t *)Y)[i] = to_f16(v);
    else ((uint16_t *)Y)[i] = to_bf16(v);
}

// Keep-predicate of the sparsification function: |x| >= t (mode 0) or |x| > t (mode 1).
// NaN compares false and is never kept.
__device__ __forceinline__ bool keep(float x, float tau, int mode)
{
    float a = __builtin_fabsf(x);
    return mode == 0 ? (a >= tau) : (a > tau);
}

template <bool NT>
__device__ __forceinline__ u32x4 ldg16(const uint16_t *p)
{
    const u32x4 *q = reinterpret_cast<const u32x4 *>(p);
    return NT ? __builtin_nontemporal_load(q) : *q;
}

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float uniform(float v) { return as_f(__builtin_amdgcn_readfirstlane(as_u(v))); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// Exclusive prefix sum of `v` over the workgroup (<= 8 waves); `total` receives the sum.
// s_wave: 8 ints of LDS.  Contains one __syncthreads.
__device__ __forceinline__ int block_exclusive_scan(int v, int *s_wave, int &total)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    int inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int n = __shfl_up(inc, d, 64);
        if (lane >= d) inc += n;
    }
    if (lane == 63) s_wave[w] = inc;
    __syncthreads();
    int base = 0, tot = 0;
    for (int i = 0; i < nw; ++i) {
        int s = s_wave[i];
        if (i < w) base += s;
        tot += s;
    }
    total = tot;
    return base + inc - v;
}

// Load channels [c, c+8) of the nb tokens of one batch tile; per-token keep masks (bit e =
// channel c+e kept).  With union_all (batch_mask_mode 1) every token's mask becomes the union
// over the WHOLE batch.  Returns the union over the tile's tokens.
template <int DT, int BT>
__device__ __forceinline__ uint32_t load_tokens8(const uint16_t *X, int batch, int b0, int nb, int d_in,
                                                 int c, float tau, int mode, bool union_all,
                                                 u32x4 (&raw)[BT], float (&xv)[BT][8], uint32_t (&m)[BT])
{
    uint32_t u = 0;
#pragma unroll
    for (int b = 0; b < BT; ++b) {
        m[b] = 0;
        if (b < nb) {
            raw[b] = *reinterpret_cast<const u32x4 *>(X + (size_t)(b0 + b) * d_in + c);
            unpack8<DT>(raw[b], xv[b]);
#pragma unroll
            for (int e = 0; e < 8; ++e) m[b] |= (uint32_t)keep(xv[b][e], tau, mode) << e;
        } else {
            raw[b] = u32x4{0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 8; ++e) xv[b][e] = 0.f;
        }
        u |= m[b];
    }
    if (union_all) {
        for (int bb = 0; bb < batch; ++bb) {
            if (bb >= b0 && bb < b0 + nb) continue;
            u32x4 r2 = *reinterpret_cast<const u32x4 *>(X + (size_t)bb * d_in + c);
            float f[8];
            unpack8<DT>(r2, f);
#pragma unroll
            for (int e = 0; e < 8; ++e) u |= (uint32_t)keep(f[e], tau, mode) << e;
        }
#pragma unroll
        for (int b = 0; b < BT; ++b) m[b] = (b < nb) ? u : 0u;
    }
    return u;
}

// ---------------------------------------------------------------------------------------------
// Streaming primitive: acc[b][0:8] += sum_j coef[j][b] * M[idx[j], col:col+8] over the n staged rows.
// Wave w of nw takes kUnroll consecutive rows at a time; all of a group's loads are issued
// before the first FMA.  idx / coef live in LDS and are wave-uniform (scalar registers).
// ---------------------------------------------------------------------------------------------
template <int DT, int BT, bool NT>
__device__ __forceinline__ void stream_rows(const uint16_t *__restrict__ M, size_t ld, int col, bool colok,
                                            const int *s_idx, const float *s_coef, int n, int w, int nw,
                                            float (&acc)[BT][8])
{
    for (int j0 = w * kUnroll; j0 < n; j0 += nw * kUnroll) {
        u32x4 v[kUnroll];
        if (j0 + kUnroll <= n) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int idx = uniform(s_idx[j0 + u]);
                v[u] = colok ? ldg16<NT>(M + (size_t)idx * ld + col) : u32x4{0, 0, 0, 0};
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                float f[8];
                unpack8<DT>(v[u], f);
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    const float cf = uniform(s_coef[(j0 + u) * BT + b]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[b][e] = __builtin_fmaf(cf, f[e], acc[b][e]);
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                v[u] = u32x4{0, 0, 0, 0};
                if (j0 + u < n) {
                    const int idx = uniform(s_idx[j0 + u]);
                    if (colok) v[u] = ldg16<NT>(M + (size_t)idx * ld + col);
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                if (j0 + u < n) {
                    float f[8];
                    unpack8<DT>(v[u], f);
#pragma unroll
                    for (int b = 0; b < BT; ++b) {
                        const float cf = uniform(s_coef[(j0 + u) * BT + b]);
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[b][e] = __builtin_fmaf(cf, f[e], acc[b][e]);
                    }
                }
            }
        }
    }
}

// Cross-wave reduction of a column tile through LDS, fp32 atomics into yacc, and -- for the last
// workgroup to arrive at this (batch tile, column tile) -- one rounding and the store of Y.
// yacc and the arrival counter are left zero for the next call.
template <int BT>
__device__ __forceinline__ void reduce_and_finish(float (&acc)[BT][8], float *s_red, int *s_flag,
                                                  float *yacc, uint32_t *done_ctr, void *Y, int out_dtype,
                                                  int b0, int nb, int d_out, int tile, int splits)
{
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63, w = tid >> 6, nw = nthr >> 6;
    const int colbase = tile * kTile;
    for (int b = 0; b < nb; ++b) {
        float *yrow = yacc + (size_t)(b0 + b) * d_out;
        if (nw > 1) {
            float4 *dst = reinterpret_cast<float4 *>(s_red + w * kTile + lane * 8);
            dst[0] = float4{acc[b][0], acc[b][1], acc[b][2], acc[b][3]};
            dst[1] = float4{acc[b][4], acc[b][5], acc[b][6], acc[b][7]};
            __syncthreads();
            for (int col = tid; col < kTile; col += nthr) {
                float s = 0.f;
                for (int i = 0; i < nw; ++i) s += s_red[i * kTile + col];
                if (colbase + col < d_out)
                    __hip_atomic_fetch_add(yrow + colbase + col, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __syncthreads();
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int col = lane * 8 + e;
                if (colbase + col < d_out)
                    __hip_atomic_fetch_add(yrow + colbase + col, acc[b][e], __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    // Arrival: make this workgroup's atomics visible, then count in.
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        uint32_t old = __hip_atomic_fetch_add(done_ctr, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = (old == (uint32_t)(splits - 1));
    }
    __syncthreads();
    if (*s_flag) {
        __threadfence();
        for (int b = 0; b < nb; ++b) {
            float *yrow = yacc + (size_t)(b0 + b) * d_out;
            for (int col = tid; col < kTile; col += nthr) {
                const int gc = colbase + col;
                if (gc < d_out) {
                    float v = __hip_atomic_load(yrow + gc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    store_out(Y, (size_t)(b0 + b) * d_out + gc, v, out_dtype);
                    __hip_atomic_store(yrow + gc, 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        if (tid == 0) __hip_atomic_store(done_ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

struct GatherArgs {
    LayerView L;
    const uint16_t *X;
    void *Y;
    int batch, splits, tiles, cap;
};

// LDS carve-up shared by k_gather and k_dense_axpy.
struct GatherLds {
    int *idx;
    float *coef;
    float *red;
    int *misc;
};
__device__ __forceinline__ GatherLds carve(unsigned char *smem, int cap, int bt, int nw)
{
    GatherLds s;
    s.red = reinterpret_cast<float *>(smem);                       // 16-byte aligned
    s.coef = s.red + (nw > 1 ? nw * kTile : 0);
    s.idx = reinterpret_cast<int *>(s.coef + (size_t)cap * bt);
    s.misc = s.idx + cap;
    return s;
}

// ---------------------------------------------------------------------------------------------
// Steps 1-2 and 4-5 of the layer in one launch: sparsification mask and ascending kept-channel
// list (Sec. 3.4, sigma_t), the sparse part over the kept columns of W, the second low-rank
// product U_r t, their sum and the single rounding.
// grid.x = tiles * splits, grid.z = batch tiles of BT tokens, block = 64 * waves.
// ---------------------------------------------------------------------------------------------
template <int DT, int BT, bool NT>
__global__ __launch_bounds__(512) void k_gather(const GatherArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63, w = tid >> 6, nw = nthr >> 6;
    const int z = blockIdx.z;
    const int tile = blockIdx.x % a.tiles, split = blockIdx.x / a.tiles;
    const LayerView &L = a.L;
    const int d_in = L.d_in, d_out = L.d_out, r = L.rank;
    const int b0 = z * BT;
    const int nb = min(BT, a.batch - b0);
    const bool union_all = L.batch_mask_mode == 1;
    const GatherLds s = carve(smem, a.cap, BT, nw);

    // ---- mask + count over my contiguous chunk of channels
    const int CH = 8 * ((d_in + 8 * nthr - 1) / (8 * nthr));
    const int c_begin = tid * CH, c_end = min(d_in, c_begin + CH);
    int cnt = 0;
    for (int c = c_begin; c < c_end; c += 8) {
        u32x4 raw[BT]; float xv[BT][8]; uint32_t m[BT];
        uint32_t u = load_tokens8<DT, BT>(a.X, a.batch, b0, nb, d_in, c, L.tau, L.cmp_mode, union_all, raw, xv, m);
        cnt += __popc(u);
    }
    int k;
    int pos = block_exclusive_scan(cnt, s.misc, k);

    // ---- my balanced share of the kept list and of the U_r^T rows
    const int lo = (int)(((long long)split * k) / a.splits);
    const int hi = (int)(((long long)(split + 1) * k) / a.splits);
    const int ulo = (int)(((long long)split * r) / a.splits);
    const int uhi = (int)(((long long)(split + 1) * r) / a.splits);
    const int nW = hi - lo, nU = uhi - ulo, n = nW + nU;

    if (cnt > 0 && pos < hi && pos + cnt > lo) {
        for (int c = c_begin; c < c_end; c += 8) {
            u32x4 raw[BT]; float xv[BT][8]; uint32_t m[BT];
            uint32_t u = load_tokens8<DT, BT>(a.X, a.batch, b0, nb, d_in, c, L.tau, L.cmp_mode, union_all, raw, xv, m);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if ((u >> e) & 1u) {
                    const int p = pos++;
                    if (p >= lo && p < hi) {
                        const int j = p - lo;
                        s.idx[j] = c + e;
                        uint32_t bits = 0;
#pragma unroll
                        for (int b = 0; b < BT; ++b) {
                            const bool kb = (m[b] >> e) & 1u;
                            s.coef[j * BT + b] = kb ? xv[b][e] : 0.f;
                            bits |= (uint32_t)kb << b;
                        }
                        if (tile == 0) {          // the tile-0 workgroups publish the list for read-back
                            L.act_list[(size_t)z * d_in + p] = c + e;
                            L.act_bits[(size_t)z * d_in + p] = bits;
                        }
                    }
                }
            }
        }
    }
    for (int j = tid; j < nU; j += nthr) {
        s.idx[nW + j] = d_in + ulo + j;
#pragma unroll
        for (int b = 0; b < BT; ++b)
            s.coef[(nW + j) * BT + b] = L.t[((size_t)z * r + ulo + j) * BT + b];
    }
    if (tile == 0 && split == 0 && tid == 0) L.act_count[z] = k;
    __syncthreads();

    // ---- stream my rows
    const int col = tile * kTile + lane * 8;
    const bool colok = col < d_out;
    float acc[BT][8];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[b][e] = 0.f;
    stream_rows<DT, BT, NT>(L.M, (size_t)d_out, col, colok, s.idx, s.coef, n, w, nw, acc);

    reduce_and_finish<BT>(acc, s.red, s.misc + 15, L.yacc, L.tile_done + (size_t)z * a.tiles + tile, a.Y,
                          L.out_dtype, b0, nb, d_out, tile, a.splits);
}

// ---------------------------------------------------------------------------------------------
// Dense baseline, axpy form over the same column-major W: every channel, no mask, no low rank.
// ---------------------------------------------------------------------------------------------
template <int DT, int BT, bool NT>
__global__ __launch_bounds__(512) void k_dense_axpy(const GatherArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63, w = tid >> 6, nw = nthr >> 6;
    const int z = blockIdx.z;
    const int tile = blockIdx.x % a.tiles, split = blockIdx.x / a.tiles;
    const LayerView &L = a.L;
    const int d_in = L.d_in, d_out = L.d_out;
    const int b0 = z * BT;
    const int nb = min(BT, a.batch - b0);
    const GatherLds s = carve(smem, a.cap, BT, nw);

    const int lo = (int)(((long long)split * d_in) / a.splits);
    const int hi = (int)(((long long)(split + 1) * d_in) / a.splits);
    const int n = hi - lo;
    for (int j = tid; j < n; j += nthr) {
        s.idx[j] = lo + j;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            float xf = 0.f;
            if (b < nb) {
                const uint16_t h = a.X[(size_t)(b0 + b) * d_in + lo + j];
                xf = (DT == F16) ? (float)__builtin_bit_cast(_Float16, h) : as_f((uint32_t)h << 16);
            }
            s.coef[j * BT + b] = xf;
        }
    }
    __syncthreads();

    const int col = tile * kTile + lane * 8;
    const bool colok = col < d_out;
    float acc[BT][8];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[b][e] = 0.f;
    stream_rows<DT, BT, NT>(L.M, (size_t)d_out, col, colok, s.idx, s.coef, n, w, nw, acc);

    reduce_and_finish<BT>(acc, s.red, s.misc + 15, L.yacc, L.tile_done + (size_t)z * a.tiles + tile, a.Y,
                          L.out_dtype, b0, nb, d_out, tile, a.splits);
}

// ---------------------------------------------------------------------------------------------
// Stage 1 of the low-rank part (Sec. 3.4): t_i = sum_c (S_r V_r^T)[i, c] * (x - sigma_t(x))_c.
// Each workgroup stages the masked token(s) in LDS (kept channels zeroed) and dots RU rows of
// S_r V_r^T against it; a row is complete inside one workgroup, so t needs no cross-workgroup sum.
// grid.x = ceil(r / RU), grid.z = batch tiles, block = 256.
// ---------------------------------------------------------------------------------------------
struct LowrankArgs {
    LayerView L;
    const uint16_t *X;
    int batch, chunk;
};

template <int DT, int BT, int RU>
__global__ __launch_bounds__(256) void k_lowrank_t(const LowrankArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int z = blockIdx.z;
    const LayerView &L = a.L;
    const int d_in = L.d_in, r = L.rank;
    const int b0 = z * BT;
    const int nb = min(BT, a.batch - b0);
    const bool union_all = L.batch_mask_mode == 1;
    const int i0 = blockIdx.x * RU;
    uint16_t *s_xm = reinterpret_cast<uint16_t *>(smem);                        // [BT][chunk]
    float *s_part = reinterpret_cast<float *>(smem + (size_t)BT * a.chunk * 2); // [4][RU*BT]

    float part[RU][BT];
#pragma unroll
    for (int ru = 0; ru < RU; ++ru)
#pragma unroll
        for (int b = 0; b < BT; ++b) part[ru][b] = 0.f;

    for (int c0 = 0; c0 < d_in; c0 += a.chunk) {
        const int len = min(a.chunk, d_in - c0);
        if (c0 > 0) __syncthreads();
        for (int q = tid; q < len / 8; q += 256) {
            u32x4 raw[BT]; float xv[BT][8]; uint32_t m[BT];
            load_tokens8<DT, BT>(a.X, a.batch, b0, nb, d_in, c0 + q * 8, L.tau, L.cmp_mode, union_all, raw, xv, m);
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                u32x4 o = raw[b];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if ((m[b] >> e) & 1u) o[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;   // kept -> 0
                *reinterpret_cast<u32x4 *>(s_xm + (size_t)b * a.chunk + q * 8) = o;
            }
        }
        __syncthreads();
        for (int q = tid; q < len / 8; q += 256) {
            float xf[BT][8];
#pragma unroll
            for (int b = 0; b < BT; ++b)
                unpack8<DT>(*reinterpret_cast<const u32x4 *>(s_xm + (size_t)b * a.chunk + q * 8), xf[b]);
            u32x4 v[RU];
#pragma unroll
            for (int ru = 0; ru < RU; ++ru)
                v[ru] = (i0 + ru < r) ? ldg16<false>(L.SVt + (size_t)(i0 + ru) * d_in + c0 + q * 8)
                                      : u32x4{0, 0, 0, 0};
#pragma unroll
            for (int ru = 0; ru < RU; ++ru) {
                float f[8];
                unpack8<DT>(v[ru], f);
#pragma unroll
                for (int b = 0; b < BT; ++b)
#pragma unroll
                    for (int e = 0; e < 8; ++e) part[ru][b] = __builtin_fmaf(f[e], xf[b][e], part[ru][b]);
            }
        }
    }
#pragma unroll
    for (int ru = 0; ru < RU; ++ru)
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            float v = wave_sum(part[ru][b]);
            if (lane == 0) s_part[w * (RU * BT) + ru * BT + b] = v;
        }
    __syncthreads();
    if (tid < RU * BT) {
        const int ru = tid / BT, b = tid % BT;
        if (i0 + ru < r) {
            float v = s_part[tid] + s_part[RU * BT + tid] + s_part[2 * RU * BT + tid] + s_part[3 * RU * BT + tid];
            L.t[((size_t)z * r + i0 + ru) * BT + b] = v;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Dense baseline, row-dot form over row-major W [d_out][d_in]: one wave per output row, x staged
// in LDS, no cross-workgroup reduction at all.  grid.x workgroups of 4 waves; grid.z batch tiles.
// ---------------------------------------------------------------------------------------------
struct RowdotArgs {
    LayerView L;
    const uint16_t *X;
    void *Y;
    int batch;
};

template <int DT, int BT, bool NT>
__global__ __launch_bounds__(256) void k_dense_rowdot(const RowdotArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int z = blockIdx.z;
    const LayerView &L = a.L;
    const int d_in = L.d_in, d_out = L.d_out;
    const int b0 = z * BT;
    const int nb = min(BT, a.batch - b0);
    uint16_t *s_x = reinterpret_cast<uint16_t *>(smem);   // [BT][d_in]
    const int nq = d_in / 8;
    for (int q = tid; q < nq; q += 256)
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            u32x4 v = u32x4{0, 0, 0, 0};
            if (b < nb) v = *reinterpret_cast<const u32x4 *>(a.X + (size_t)(b0 + b) * d_in + q * 8);
            *reinterpret_cast<u32x4 *>(s_x + (size_t)b * d_in + q * 8) = v;
        }
    __syncthreads();
    for (int o = blockIdx.x * 4 + w; o < d_out; o += gridDim.x * 4) {
        const uint16_t *row = L.Wrow + (size_t)o * d_in;
        float acc[BT];
#pragma unroll
        for (int b = 0; b < BT; ++b) acc[b] = 0.f;
#pragma unroll 8
        for (int q = lane; q < nq; q += 64) {
            float f[8];
            unpack8<DT>(ldg16<NT>(row + q * 8), f);
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                float xf[8];
                unpack8<DT>(*reinterpret_cast<const u32x4 *>(s_x + (size_t)b * d_in + q * 8), xf);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[b] = __builtin_fmaf(f[e], xf[e], acc[b]);
            }
        }
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            float v = wave_sum(acc[b]);
            if (lane == 0 && b < nb) store_out(a.Y, (size_t)(b0 + b) * d_out + o, v, L.out_dtype);
        }
    }
}

__global__ void k_zero(uint32_t *p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0u;
}

int batch_tile(int batch)
{
    if (batch <= 1) return 1;
    if (batch <= 2) return 2;
    if (batch <= 4) return 4;
    return 8;
}

int gather_cap(int d_in, int rank, int splits)
{
    return (d_in + splits - 1) / splits + (rank + splits - 1) / splits + 2;
}

}  // namespace

size_t gather_lds_bytes(int d_in, int rank, int splits, int waves, int bt)
{
    const size_t cap = gather_cap(d_in, rank, splits);
    return (waves > 1 ? (size_t)waves * kTile * 4 : 0) + cap * bt * 4 + cap * 4 + 16 * 4;
}

static int lowrank_chunk(int d_in, int bt)
{
    int chunk = (24576 / bt) & ~7;
    return d_in < chunk ? d_in : chunk;
}

size_t lowrank_lds_bytes(int d_in, int bt)
{
    return (size_t)bt * lowrank_chunk(d_in, bt) * 2 + 4 * 4 * kMaxBT * 4;
}

bool rowdot_supported(int d_in, int batch)
{
    return (size_t)batch_tile(batch) * d_in * 2 <= 65536;
}

#define RS_DISPATCH_BT(BTV, ...)                      \
    switch (BTV) {                                    \
    case 1: { constexpr int BT = 1; __VA_ARGS__; } break; \
    case 2: { constexpr int BT = 2; __VA_ARGS__; } break; \
    case 4: { constexpr int BT = 4; __VA_ARGS__; } break; \
    default: { constexpr int BT = 8; __VA_ARGS__; } break; \
    }

hipError_t launch_lowrank_t(const LayerView &L, const Launch &cfg, const void *X, int batch, hipStream_t stream)
{
    if (L.rank == 0) return hipSuccess;
    const int bt = batch_tile(batch);
    const int nz = (batch + bt - 1) / bt;
    LowrankArgs a{L, (const uint16_t *)X, batch, lowrank_chunk(L.d_in, bt)};
    const size_t lds = lowrank_lds_bytes(L.d_in, bt);
    const int ru = cfg.lowrank_rows;
    dim3 grid((L.rank + ru - 1) / ru, 1, nz), block(256);
#define RS_LR(DT)                                                                                       \
    RS_DISPATCH_BT(bt, {                                                                                \
        if (ru == 1) hipLaunchKernelGGL((k_lowrank_t<DT, BT, 1>), grid, block, lds, stream, a);         \
        else if (ru == 2) hipLaunchKernelGGL((k_lowrank_t<DT, BT, 2>), grid, block, lds, stream, a);    \
        else hipLaunchKernelGGL((k_lowrank_t<DT, BT, 4>), grid, block, lds, stream, a);                 \
    })
    if (L.dtype == F16) { RS_LR(F16) } else { RS_LR(BF16) }
#undef RS_LR
    return hipGetLastError();
}

hipError_t launch_gather(const LayerView &L, const Launch &cfg, const void *X, int batch, void *Y,
                         hipStream_t stream)
{
    const int bt = batch_tile(batch);
    const int nz = (batch + bt - 1) / bt;
    const int tiles = (L.d_out + kTile - 1) / kTile;
    GatherArgs a{L, (const uint16_t *)X, Y, batch, cfg.splits, tiles, gather_cap(L.d_in, L.rank, cfg.splits)};
    const size_t lds = gather_lds_bytes(L.d_in, L.rank, cfg.splits, cfg.waves, bt);
    dim3 grid(tiles * cfg.splits, 1, nz), block(kWave * cfg.waves);
#define RS_G(DT)                                                                                         \
    RS_DISPATCH_BT(bt, {                                                                                 \
        if (cfg.nontemporal) hipLaunchKernelGGL((k_gather<DT, BT, true>), grid, block, lds, stream, a);  \
        else hipLaunchKernelGGL((k_gather<DT, BT, false>), grid, block, lds, stream, a);                 \
    })
    if (L.dtype == F16) { RS_G(F16) } else { RS_G(BF16) }
#undef RS_G
    return hipGetLastError();
}

hipError_t launch_dense_axpy(const LayerView &L, const Launch &cfg, const void *X, int batch, void *Y,
                             hipStream_t stream)
{
    const int bt = batch_tile(batch);
    const int nz = (batch + bt - 1) / bt;
    const int tiles = (L.d_out + kTile - 1) / kTile;
    GatherArgs a{L, (const uint16_t *)X, Y, batch, cfg.splits, tiles, gather_cap(L.d_in, L.rank, cfg.splits)};
    const size_t lds = gather_lds_bytes(L.d_in, L.rank, cfg.splits, cfg.waves, bt);
    dim3 grid(tiles * cfg.splits, 1, nz), block(kWave * cfg.waves);
#define RS_D(DT)                                                                                             \
    RS_DISPATCH_BT(bt, {                                                                                     \
        if (cfg.nontemporal) hipLaunchKernelGGL((k_dense_axpy<DT, BT, true>), grid, block, lds, stream, a);  \
        else hipLaunchKernelGGL((k_dense_axpy<DT, BT, false>), grid, block, lds, stream, a);                 \
    })
    if (L.dtype == F16) { RS_D(F16) } else { RS_D(BF16) }
#undef RS_D
    return hipGetLastError();
}

hipError_t launch_dense_rowdot(const LayerView &L, const Launch &cfg, const void *X, int batch, void *Y,
                               hipStream_t stream)
{
    const int bt = batch_tile(batch);
    const int nz = (batch + bt - 1) / bt;
    RowdotArgs a{L, (const uint16_t *)X, Y, batch};
    const size_t lds = (size_t)bt * L.d_in * 2;
    int wgs = (L.d_out + 3) / 4;
    if (wgs > 2048) wgs = 2048;
    dim3 grid(wgs, 1, nz), block(256);
#define RS_R(DT)                                                                                              \
    RS_DISPATCH_BT(bt, {                                                                                      \
        if (cfg.nontemporal) hipLaunchKernelGGL((k_dense_rowdot<DT, BT, true>), grid, block, lds, stream, a); \
        else hipLaunchKernelGGL((k_dense_rowdot<DT, BT, false>), grid, block, lds, stream, a);                \
    })
    if (L.dtype == F16) { RS_R(F16) } else { RS_R(BF16) }
#undef RS_R
    return hipGetLastError();
}

hipError_t launch_zero(void *p, size_t n_words, hipStream_t stream)
{
    if (n_words == 0) return hipSuccess;
    size_t blocks = (n_words + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(k_zero, dim3((unsigned)blocks), dim3(256), 0, stream, (uint32_t *)p, n_words);
    return hipGetLastError();
}

}  // namespace rsparse
