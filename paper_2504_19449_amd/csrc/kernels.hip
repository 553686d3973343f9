// gfx950 (MI355X, CDNA4) kernels of the R-Sparse linear layer (R-Sparse, Sec. 3.4).
//
// Everything here is bound by HBM bandwidth at decode batch sizes (2*B flops per 2-byte
// weight), so the kernels are organised around the weight stream: 16-byte loads, one
// 1 KiB row segment per 64-lane wave, many rows in flight, fp32 accumulation on the
// vector ALU.  Storage:
//
//   M    [d_in + r][d_out]  W column-major (row c = all outputs of input channel c; Sec. 3.4 asks
//                        for this layout so that a kept channel is one contiguous run), followed by
//                        U_r^T (row d_in + j = U_r[:, j]) for the one-launch kernel
//   SVt  [r][d_in]       S_r V_r^T, one singular component per row
//   SVc  [d_in][r]       optional channel-major copy of S_r V_r^T (row c = its column c): at one token the stage 1 of
//                        the one-launch kernel then reads the rows of the dropped channels only (lowrank_gather)
//   U    [d_out][r]      U_r row-major
//
// One call is either two launches, ordered by the stream (no intra-kernel cross-workgroup waits):
//
//   k_sparse_and_t   workgroups [0, lr_wgs):  t_i = SVt[i,:] . (x - sigma_t(x))      (row dots)
//                    the others:              yacc += sum_{c kept} x_c M[c,:]         (gather-axpy)
//                    Each gather workgroup thresholds and compacts x itself (it scans the whole
//                    token -- 2*d_in bytes from L2 -- and keeps its balanced share of the ascending
//                    kept list), so there is no compaction launch.  Column tiles x channel splits
//                    fill the chip; partial sums meet in fp32 atomics.
//   k_finish         Y = round(yacc + U t)   (row dots over U, no reduction), yacc re-zeroed.
//
// or ONE launch (k_rsparse_fused), which removes the second kernel's launch and start-up latency:
// M carries r more rows, U_r^T, so that stage 2 of the low-rank part is r more "channels" whose
// coefficients are t.  Every gather workgroup appends its share of those rows to its list; only the
// FMAs of those rows need t, which the stage-1 workgroups (at the front of the grid, so dispatched
// first) publish into t_pub.  An entry of t_pub holds an all-ones bit pattern until it is written, so
// a consumer needs no separate flag: it requests its entries one batch ahead and re-reads (bounded)
// while it still sees that pattern.  All cross-workgroup data (t_pub, yacc, arrival counters) moves
// through agent-scope relaxed atomics, which are performed at the device's coherence point, so no
// cache write-back or invalidate is needed; a workgroup waits for its own atomics to be acknowledged
// (s_waitcnt) before it bumps a counter.  The last workgroup to arrive at a column tile swaps the
// tile's sums out of yacc (which re-zeroes them), rounds once and stores Y; the last tile of the
// layer puts t_pub and the counters back.  For the gate / up pair of an MLP (Sec. 3.1) the two layers
// share one set of counters and the finisher stores H = round(silu(g) * u) instead of g and u.
#include "kernels.h"
#include "device_common.h"
#include "device_stage1.h"

#include <algorithm>

namespace rsparse {
namespace {

// ---------------------------------------------------------------------------------------------
// Streaming primitive: acc[b][0:8] += sum_j coef[j][b] * M[idx[j], col:col+8] over the n staged rows.
// Wave w of nw takes kUnroll consecutive rows per batch; a batch's loads are all issued before its
// first FMA, and the next batch is issued before the current one is consumed (two batches of
// 16-byte loads in flight per lane).  idx / coef live in LDS and are wave-uniform (scalar registers).
// ---------------------------------------------------------------------------------------------
template <bool NT>
__device__ __forceinline__ void load_batch(const uint16_t *__restrict__ M, size_t ld, int col, bool colok,
                                           const int *s_idx, int n, int j0, u32x4 (&v)[kUnroll])
{
    if (j0 + kUnroll <= n) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int idx = uniform(s_idx[j0 + u]);
            v[u] = colok ? ldg16<NT>(M + (size_t)idx * ld + col) : u32x4{0, 0, 0, 0};
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
    }
}

template <int DT, int BT>
__device__ __forceinline__ void fma_batch(const u32x4 (&v)[kUnroll], const float *s_coef, int n, int j0,
                                          float (&acc)[BT][8])
{
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

// Consume the already-issued batch `va` (rows j0..) and stream the rest of the wave's rows.
// before_fma(j0) runs ahead of the FMAs of the batch that starts at row j0 (its loads, and those of
// the following batch, are already in flight).
template <int DT, int BT, bool NT, typename Hook>
__device__ __forceinline__ void stream_rest(const uint16_t *__restrict__ M, size_t ld, int col, bool colok,
                                            const int *s_idx, const float *s_coef, int n, int j0, int step,
                                            u32x4 (&va)[kUnroll], float (&acc)[BT][8], Hook &&before_fma)
{
    u32x4 vb[kUnroll];
    while (j0 < n) {
        load_batch<NT>(M, ld, col, colok, s_idx, n, j0 + step, vb);
        before_fma(j0);
        fma_batch<DT, BT>(va, s_coef, n, j0, acc);
        j0 += step;
        if (j0 >= n) break;
        load_batch<NT>(M, ld, col, colok, s_idx, n, j0 + step, va);
        before_fma(j0);
        fma_batch<DT, BT>(vb, s_coef, n, j0, acc);
        j0 += step;
    }
}

// Cross-wave reduction of a column tile through LDS, then fp32 atomics into yacc.  No fences: in the
// two-launch form the kernel boundary before k_finish orders the atomics, in the one-launch form the
// caller waits for their acknowledgement (an agent-scope fence per workgroup costs an L2 write-back +
// invalidate on this chip and dominated the run time).
template <int BT>
__device__ __forceinline__ void reduce_to_yacc(float (&acc)[BT][8], float *s_red, float *yacc, int b0, int nb,
                                               int d_out, int tile)
{
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63, w = tid >> 6, nw = nthr >> 6;
    const int colbase = tile * kTile;
    // b must stay a compile-time index: a run-time subscript would push acc[][] into scratch memory
#pragma unroll
    for (int b = 0; b < BT; ++b) {
        if (b >= nb) break;
        float *yrow = yacc + (size_t)(b0 + b) * d_out;
        if (nw > 1) {
            if (b > 0) __syncthreads();
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
}

struct GatherArgs {
    LayerView L;
    const uint16_t *X;
    int batch, splits, tiles, cap;
    int lr_wgs, lr_rows, lr_chunk;     // stage-1 workgroups at the front of the grid, rows each, LDS chunk
    int lr_gather, lr_cap;             // one-launch kernel, one token: stage 1 over the channel-major copy of S_r V_r^T
                                       // (lowrank_gather); lr_cap = list slots of a stage-1 workgroup
    int tile_map;
    void *Y;                           // one-launch path only: the output, [batch][d_out]
    int nz;                            // one-launch path only: batch tiles in the grid
    int wait_polls;                    // one-launch path only: bound on re-reads of a t entry that is not ready
    int skip_stage1;                   // test hook: the stage-1 workgroups publish nothing (exercises the bound)
    int dense;                         // 4-bit kernel only: keep every channel (the dense baseline)
    int gen_readers;                   // (strip kernel only; here for the shared stage-1 code)
};

// All of this wave's earlier atomics and stores have been acknowledged by the memory system.
__device__ __forceinline__ void wait_own_writes()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
}

// Workgroup index -> (column tile, channel split).  Plain: tile-fastest.  XCD-aware: workgroups are
// handed to the 8 XCDs round-robin by index, and fp32 atomics from different XCDs to one line move
// it between their L2s; giving every split of a tile an index congruent to (tile mod 8) keeps a
// tile's accumulators in one L2.  Indices past the last real pair are idle.
__device__ __forceinline__ bool map_tile(int tile_map, int tiles, int splits, int g, int &tile, int &split)
{
    if (tile_map != 2) {
        tile = g % tiles;
        split = g / tiles;
        return true;
    }
    const int x = g & 7, slot = g >> 3;              // slot enumerates (tile / 8, split)
    const int tgroup = slot / splits;
    split = slot % splits;
    tile = tgroup * 8 + x;
    return tile < tiles;
}
__device__ __forceinline__ bool map_tile(const GatherArgs &a, int g, int &tile, int &split)
{
    return map_tile(a.tile_map, a.tiles, a.splits, g, tile, split);
}

// ---------------------------------------------------------------------------------------------
// Stage 1 of the low-rank part over the channel-major copy SVc [d_in][rank] (row c = (S_r V_r^T)[:, c]), one
// token (or a batch tile of up to 4, every token with its own coefficients): t = sum over the DROPPED channels c of x_c SVc[c, :] (Sec. 3.4: the low-rank part acts on x - sigma_t(x),
// whose kept channels are zero), so only the rows of dropped channels are read -- rank * (d_in - k) elements
// instead of rank * d_in.  Stage-1 workgroup wg of lr_wgs owns a fixed range of channels: it thresholds that range
// only, compacts the dropped channels with wave scans, streams their rows (a wave covers 512 columns of a row per
// load, the waves of a 512-column part share the list in batches of kUnroll rows), sums its waves in LDS and adds
// the range's partial t to t_sum with fp32 atomics.  The last workgroup to arrive swaps the sums out (which
// re-zeroes them) and publishes t.  No workgroup waits for another here.
// ---------------------------------------------------------------------------------------------
template <int DT, int BT, bool NT, bool EXT>
__device__ __forceinline__ void lowrank_gather(const GatherArgs &a, unsigned char *smem, int wg, int z)
{
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63, w = uniform(tid >> 6), nw = nthr >> 6;
    const LayerView &L = a.L;
    const int d_in = L.d_in, r = L.rank, cap = a.lr_cap;
    const int b0 = z * BT;
    const int nb = min(BT, a.batch - b0);
    const bool union_all = L.batch_mask_mode == 1;
    TileRules<BT> rules;
    load_rules<BT, EXT>(L, b0, nb, rules);
    float *s_red = reinterpret_cast<float *>(smem);                 // [nw][kTile]
    float *s_coef = s_red + (size_t)nw * kTile;                     // [cap][BT]
    int *s_idx = reinterpret_cast<int *>(s_coef + (size_t)cap * BT);// [cap]
    int *s_wtot = s_idx + cap;                                      // [nw], then the arrival flag
    int q_lo, q_hi;
    balanced_share(d_in / 8, a.lr_wgs, wg, q_lo, q_hi);             // my chunks of 8 channels
    // every list slot starts as a valid row with zero coefficients
    for (int i = tid; i < cap; i += nthr) s_idx[i] = 0;
    for (int i = tid; i < cap * BT; i += nthr) s_coef[i] = 0.f;
    int n = 0;
    for (int qb = q_lo; qb < q_hi; qb += nthr) {
        const int q = qb + tid;
        u32x4 raw[BT];
        uint32_t dm[BT];                                            // per token: the channels of the chunk it drops
        uint32_t drop = 0u;                                         // dropped by at least one token of the tile
#pragma unroll
        for (int b = 0; b < BT; ++b) { raw[b] = u32x4{0, 0, 0, 0}; dm[b] = 0u; }
        if (q < q_hi) {
            load_raw8<BT>(a.X, b0, nb, d_in, q * 8, raw);
            uint32_t m[BT];
            masks_of8<DT, BT>(L, a.X, a.batch, b0, nb, d_in, q * 8, rules, union_all, raw, m);
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                dm[b] = b < nb ? (~m[b] & 0xffu) : 0u;
                drop |= dm[b];
            }
        }
        const int c = __popc(drop);
        const int inc = wave_inclusive_scan(c);
        if (lane == 63) s_wtot[w] = inc;
        __syncthreads();
        int woff = 0, tot = 0;
        for (int i = 0; i < nw; ++i) {
            const int v = s_wtot[i];
            woff += i < w ? v : 0;
            tot += v;
        }
        if (drop != 0u) {
            float f[BT][8];
#pragma unroll
            for (int b = 0; b < BT; ++b) unpack8<DT>(raw[b], f[b]);
            int p = n + woff + inc - c;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (((drop >> e) & 1u) && p < cap) {
                    s_idx[p] = q * 8 + e;
#pragma unroll
                    for (int b = 0; b < BT; ++b) s_coef[p * BT + b] = ((dm[b] >> e) & 1u) ? f[b][e] : 0.f;
                    ++p;
                }
        }
        n += tot;
        __syncthreads();
    }
    n = min(uniform(n), cap);

    // ---- stream the dropped channels' rows: wave w -> 512-column part w % parts, row group w / parts
    const int parts = (r + kTile - 1) / kTile;                      // host: parts <= nw
    const int ng = nw / parts;
    const int part = w % parts, g = w / parts;
    const int col = part * kTile + lane * 8;
    const bool colok = col < r;
    float acc[BT][8];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[b][e] = 0.f;
    if (g < ng) {
        u32x4 va[kUnroll];
        const int j_first = g * kUnroll, step = ng * kUnroll;
        load_batch<NT>(L.SVc, (size_t)r, col, colok, s_idx, n, j_first, va);
        stream_rest<DT, BT, NT>(L.SVc, (size_t)r, col, colok, s_idx, s_coef, n, j_first, step, va, acc, [](int) {});
    }
    // b must stay a compile-time index (a run-time subscript would push acc[][] into scratch memory)
    float *const t_sum = L.t_sum + (size_t)z * BT * r;
#pragma unroll
    for (int b = 0; b < BT; ++b) {
        if (b >= nb) break;
        if (b > 0) __syncthreads();
        float4 *dst = reinterpret_cast<float4 *>(s_red + w * kTile + lane * 8);
        dst[0] = float4{acc[b][0], acc[b][1], acc[b][2], acc[b][3]};
        dst[1] = float4{acc[b][4], acc[b][5], acc[b][6], acc[b][7]};
        __syncthreads();
        for (int i = tid; i < parts * kTile; i += nthr) {
            const int pt = i / kTile, cl = i % kTile;
            float sum = 0.f;
            for (int gg = 0; gg < ng; ++gg) sum += s_red[(gg * parts + pt) * kTile + cl];
            if (i < r) __hip_atomic_fetch_add(t_sum + (size_t)b * r + i, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    // ---- arrive; the last stage-1 workgroup of the batch tile publishes its t
    wait_own_writes();
    __syncthreads();
    if (tid == 0) {
        int *ctr = L.sync + kSyncStage1 + z;
        const int arrived = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_wtot[nw] = arrived == a.lr_wgs - 1;
        if (arrived == a.lr_wgs - 1) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!s_wtot[nw]) return;
    uint32_t *const t_pub = L.t_pub + (size_t)z * BT * r;
    for (int i = tid; i < nb * r; i += nthr) {
        uint32_t bits = as_u(__hip_atomic_exchange(t_sum + i, 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        if (bits == kNotReady) bits = 0x7fc00000u;
        if (!a.skip_stage1) __hip_atomic_store(t_pub + i, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Several layers that read the same input share one launch: job i owns workgroups
// [wg_end[i-1], wg_end[i]) of the grid.
constexpr int kMaxGroup = 4;
struct GroupArgs {
    GatherArgs job[kMaxGroup];
    int wg_end[kMaxGroup];
    int n;
    int gate_up;       // one-launch kernel: jobs 0 and 1 are the gate and up projections of an MLP (same d_out);
                       // the column tiles are finished jointly and H = round(silu(g) * u) is stored to job[0].Y
};
__device__ __forceinline__ int find_job(const int (&wg_end)[kMaxGroup], int n, int wg, int &local)
{
    int li = 0, begin = 0;
#pragma unroll
    for (int i = 0; i < kMaxGroup - 1; ++i)
        if (i + 1 < n && wg >= wg_end[i]) { li = i + 1; begin = wg_end[i]; }
    local = wg - begin;
    return li;
}

// LDS carve-up of the gather part.
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
// 4-bit weights (Sec. 4.4: R-Sparse on GPTQ weights, groups of 128 input channels): W~[o][c] =
// s[o][g] (q[o][c] - z[o][g]).  A wave streams a CONTIGUOUS run of its workgroup's kept-channel list, so
// the channels of one quantisation group arrive together: it accumulates grp = sum_c x_c q_c and
// sumx = sum_c x_c while the group lasts and folds acc += s (grp - z sumx) once when it ends -- the
// codes go from nibble to float and into one FMA per token, nothing else per weight.  Scale and zero
// point of a group are requested when the group opens and used when it closes.
// A lane owns 16 output columns of a 1024-column tile: 8 bytes per row, words h = 0, 1 (layout: kernels.h).
// ---------------------------------------------------------------------------------------------
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// A batch of kUnroll rows as one register vector (word 2u + h = word h of row u): the rolled loop below
// picks a row by a run-time index, which the compiler serves with relative register addressing on a
// vector type (an array would go to scratch memory).
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
static_assert(kUnroll == 8, "u32x16 holds 8 rows of two words");

template <bool NT>
__device__ __forceinline__ u32x2 ldg8(const uint8_t *p)
{
    const u32x2 *q = reinterpret_cast<const u32x2 *>(p);
    return NT ? __builtin_nontemporal_load(q) : *q;
}

// kUnroll rows starting at list position j0 of a non-empty run that ends at j_hi.  Positions past the end
// re-read the run's last row (a cache hit) and are given a zero coefficient by the consumer, so that a batch
// is always eight unconditional loads: the compiler can then count outstanding loads exactly and lets the
// next batch stay in flight while this one is consumed.  Rows and the scale / zero-point rows are padded
// to whole tiles, so lanes past d_out read zeros instead of being masked off.
template <bool NT>
__device__ __forceinline__ void load_batch_q4(const uint8_t *__restrict__ Mq, size_t ld, int off, const int *s_idx,
                                              int j_hi, int j0, u32x16 &v)
{
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int idx = uniform(s_idx[min(j0 + u, j_hi - 1)]);
        const u32x2 w = ldg8<NT>(Mq + (size_t)idx * ld + off);
        v[2 * u] = w[0];
        v[2 * u + 1] = w[1];
    }
}

// The eight codes of one word as floats: element e < 4 is the low nibble of byte e, element 4 + e its high nibble.
__device__ __forceinline__ void codes8(uint32_t w, float (&f)[8])
{
    uint32_t lo = w & 0x0f0f0f0fu, hi = (w >> 4) & 0x0f0f0f0fu;
    // keep the two masked words as they are: each byte then converts with one byte-select instruction,
    // where the compiler would otherwise extract every nibble with a bit-field op first
    __asm__ volatile("" : "+v"(lo), "+v"(hi));
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        f[k] = (float)((lo >> (8 * k)) & 0xffu);
        f[4 + k] = (float)((hi >> (8 * k)) & 0xffu);
    }
}

template <int BT>
struct Q4State {
    float acc[2][BT][8];    // finished groups, scaled
    float grp[2][BT][8];    // sum_c x_c q_c of the open group
    float sumx[BT];         // sum_c x_c of the open group
    u32x4 sv[2];            // scales of the open group, 8 columns per word h
    u32x2 zv[2];            // its zero points, one byte per column
    int g;                  // the open group, -1 = none
};

template <int BT>
__device__ __forceinline__ void q4_open(Q4State<BT> &st, const LayerView &L, int g, int colq)
{
    st.g = g;
    const size_t at = (size_t)g * ((size_t)L.qtiles * kQ4Tile) + colq;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        st.sv[h] = *reinterpret_cast<const u32x4 *>(L.qs + at + h * 512);
        st.zv[h] = *reinterpret_cast<const u32x2 *>(L.qz + at + h * 512);
    }
}

template <int DT, int BT>
__device__ __forceinline__ void q4_close(Q4State<BT> &st)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        float sf[8];
        unpack8<DT>(st.sv[h], sf);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t zw = st.zv[h][e >> 2];
            const float zf = (float)((zw >> (8 * (e & 3))) & 0xffu);
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                const float d = __builtin_fmaf(-zf, st.sumx[b], st.grp[h][b][e]);
                st.acc[h][b][e] = __builtin_fmaf(sf[e], d, st.acc[h][b][e]);
                st.grp[h][b][e] = 0.f;
            }
        }
    }
#pragma unroll
    for (int b = 0; b < BT; ++b) st.sumx[b] = 0.f;
}

// One row: its 16 codes times the token coefficients, into the open group's sums.
template <int BT>
__device__ __forceinline__ void q4_row(Q4State<BT> &st, const u32x2 w, const float *s_coef, int j, int j_hi)
{
    float cf[BT];
#pragma unroll
    for (int b = 0; b < BT; ++b) {
        cf[b] = uniform(s_coef[min(j, j_hi - 1) * BT + b]);
        cf[b] = j < j_hi ? cf[b] : 0.f;
        st.sumx[b] += cf[b];
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        float f[8];
        codes8(w[h], f);
#pragma unroll
        for (int b = 0; b < BT; ++b)
#pragma unroll
            for (int e = 0; e < 8; ++e) st.grp[h][b][e] = __builtin_fmaf(cf[b], f[e], st.grp[h][b][e]);
    }
}

// A batch of up to kUnroll rows.  The list is ascending, so when its first and last row lie in the open
// group all of them do: that common case is straight-line code.  A batch that crosses a group boundary
// takes the rolled loop, which holds the only copy of the fold (close) and of the scale request (open).
template <int DT, int BT>
__device__ __forceinline__ void q4_consume(Q4State<BT> &st, const LayerView &L, const u32x16 &v,
                                           const int *s_idx, const float *s_coef, int j_hi, int j0, int colq)
{
    const int j_last = min(j0 + kUnroll, j_hi) - 1;
    const int g_first = uniform(s_idx[j0]) >> L.qshift, g_last = uniform(s_idx[j_last]) >> L.qshift;
    if (g_first == st.g && g_last == st.g) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) q4_row<BT>(st, u32x2{v[2 * u], v[2 * u + 1]}, s_coef, j0 + u, j_hi);
    } else {
#pragma unroll 1
        for (int u = 0; u < kUnroll; ++u) {
            if (j0 + u >= j_hi) break;
            const int g = uniform(s_idx[j0 + u]) >> L.qshift;
            if (g != st.g) {
                if (st.g >= 0) q4_close<DT, BT>(st);
                q4_open<BT>(st, L, g, colq);
            }
            q4_row<BT>(st, u32x2{v[2 * u], v[2 * u + 1]}, s_coef, j0 + u, j_hi);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// First launch of the layer.  Workgroups [0, lr_wgs) compute stage 1 of the low-rank part; the
// others do steps 1-2 of the sparse part: sparsification mask and ascending kept-channel list
// (Sec. 3.4, sigma_t) -- every workgroup scans the whole token and keeps its balanced share --
// then the gather-GEMV over the kept columns of W, accumulated into yacc with fp32 atomics.
// The two groups are independent, so they share one launch.
// grid.x = lr_wgs + tiles * splits, grid.z = batch tiles of BT tokens, block = 64 * waves.
// ---------------------------------------------------------------------------------------------
template <int DT, int BT, bool NT, bool FUSED, bool Q4 = false, bool EXT = true>
__device__ __forceinline__ void sparse_body(const GroupArgs &ga, unsigned char *smem)
{
    const int z = blockIdx.z;
    int wg;
    const GatherArgs &a = ga.job[find_job(ga.wg_end, ga.n, blockIdx.x, wg)];
    const LayerView &L = a.L;
    // everything the path to the first weight load needs, fetched in one go
    const int lr_wgs = pin(a.lr_wgs), tile_map = pin(a.tile_map), n_tiles = pin(a.tiles), n_splits = pin(a.splits);
    const uint16_t *const X = pin(a.X);
    const int d_in = pin(L.d_in), d_out = pin(L.d_out), batch = pin(a.batch), cap = pin(a.cap);
    const bool union_all = pin(L.batch_mask_mode) == 1;
    if (__builtin_expect(wg < lr_wgs, 0)) {
        // every gather workgroup ends with rows that need t: the stage-1 waves issue ahead of the gather waves they
        // share a compute unit with (measured: q/k/v grouped at 8192 wide 37.0 -> 35.6 us, the other launches unchanged)
        if constexpr (FUSED) __builtin_amdgcn_s_setprio(3);
        if constexpr (FUSED && BT <= 4 && !Q4) {
            if (a.lr_gather) {
                lowrank_gather<DT, BT, NT, EXT>(a, smem, wg, z);
                return;
            }
        }
        lowrank_rows<DT, BT, FUSED ? kPubNotReady : kPubPlain, GatherArgs, EXT>(a, smem, wg, z);
        return;
    }
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63, w = tid >> 6, nw = nthr >> 6;
    int tile, split;
    if (!map_tile(tile_map, n_tiles, n_splits, wg - lr_wgs, tile, split)) return;
    const int b0 = z * BT;
    const int nb = min(BT, batch - b0);
    TileRules<BT> rules;
    load_rules<BT, EXT>(L, b0, nb, rules);
    const GatherLds s = carve(smem, cap, BT, nw);
    const int col = tile * kTile + lane * 8;
    const bool colok = col < d_out;

    // ---- pass 1, coalesced over the token(s): keep-bits of every 8 channels (union over the batch
    //      tile, or over the whole batch with the union mask).  A wave covers 64 consecutive 8-channel
    //      chunks at a time and scans their kept counts in registers straight away; per chunk it leaves
    //      the keep-bits and the count of kept channels before it inside those 64 chunks, per 64 chunks
    //      their total.  No barrier up to here: every thread only touches its own slots.
    const int nq = d_in / 8;
    uint8_t *s_u = reinterpret_cast<uint8_t *>(s.misc + 16);
    int *s_P = reinterpret_cast<int *>(s_u + ((nq + 3) & ~3));
    const int E = (nq + 63) >> 6;                      // blocks of 64 chunks
    int *s_tot = s_P + nq, *s_base = s_tot + E;
    constexpr int PB = TokenBatch<BT>::kGroups;
    // every list slot starts as a valid channel, so that no later arithmetic slip can turn LDS leftovers into addresses
    for (int i = tid; i < cap; i += nthr) s.idx[i] = 0;
    for (int qb = w * 64; qb < nq; qb += nthr * PB) {
        u32x4 raw[PB][BT];
#pragma unroll
        for (int p = 0; p < PB; ++p)
            if (qb + p * nthr + lane < nq) load_raw8<BT>(X, b0, nb, d_in, (qb + p * nthr + lane) * 8, raw[p]);
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            const int qrow = qb + p * nthr;            // first chunk of this wave's block: the same for all its lanes
            if (qrow < nq) {
                const int q = qrow + lane;
                uint32_t kept = 0u;
                if (q < nq) {
                    uint32_t m[BT];
                    kept = masks_of8<DT, BT>(L, X, batch, b0, nb, d_in, q * 8, rules, union_all, raw[p], m);
                    if (Q4 && a.dense) kept = 0xffu;
                }
                const int c = __popc(kept);
                const int inc = wave_inclusive_scan(c);
                if (q < nq) {
                    s_u[q] = (uint8_t)kept;
                    s_P[q] = inc - c;
                }
                if (lane == 63) s_tot[qrow >> 6] = inc;
            }
        }
    }
    __syncthreads();

    // ---- pass 2: every wave turns the block totals into block bases for itself (identical values from
    //      every wave, read back only by the wave that wrote them), which also gives the list length k
    int k = 0;
    for (int eb = 0; eb < E; eb += 64) {
        const int e = eb + lane;
        const int v = e < E ? s_tot[e] : 0;
        const int inc = wave_inclusive_scan(v);
        if (e < E) s_base[e] = k + inc - v;
        k += __shfl(inc, 63, 64);
    }
    k = min(max(uniform(k), 0), d_in);

    // ---- my balanced share [lo, hi) of the ascending kept list: each thread writes out the entries of its
    //      own chunks that fall into it
    int lo, hi;
    balanced_share(k, n_splits, split, lo, hi);
    const int n = hi - lo;
    for (int qrow = w * 64; qrow < nq; qrow += nthr) {
        const int q = qrow + lane;
        if (q < nq) {
            const uint32_t u = s_u[q];
            const int P = s_base[qrow >> 6] + s_P[q];
            if (u != 0u && P < hi && P + __popc(u) > lo) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int p = P + __popc(u & ((1u << e) - 1u));
                    if (((u >> e) & 1u) && p >= lo && p < hi) s.idx[p - lo] = q * 8 + e;
                }
            }
        }
    }
    // ---- one launch: my share of the rows of U_r^T follows the kept channels as rows d_in + j of M
    int n_all = n;
    if (FUSED) {
        int r_lo, r_hi;
        balanced_share(L.rank, n_splits, split, r_lo, r_hi);
        for (int i = tid; i < r_hi - r_lo; i += nthr) s.idx[n + i] = d_in + r_lo + i;
        n_all = n + (r_hi - r_lo);
    }
    if (tile == 0 && split == 0 && tid == 0) L.act_count[z] = k;
    __syncthreads();

    // ---- issue the first batch of weight loads (they need only the indices) ...
    float acc[BT][8];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[b][e] = 0.f;
    u32x4 va[kUnroll];
    const int j_first = w * kUnroll, step = nw * kUnroll;
    // 4-bit weights: this wave's contiguous run [jq_lo, jq_hi) of the list, 8 bytes per lane and row
    // (wave index and row count go through readfirstlane: the compiler cannot know they are wave-uniform, and
    //  would otherwise run the row loop and the group tests under execution masks)
    const int wq = uniform(w), nq_rows = uniform(n);
    int jq_lo, jq_hi;
    balanced_share(nq_rows, nw, wq, jq_lo, jq_hi);
    const int colq = tile * kQ4Tile + lane * 8;
    const size_t ldq = (size_t)L.qtiles * (kQ4Tile / 2);
    const int offq = tile * (kQ4Tile / 2) + lane * 8;
    u32x16 qa, qb;
    Q4State<Q4 ? BT : 1> st;
    if constexpr (Q4) {
        st.g = -1;
        if (jq_lo < jq_hi) {
            // two batches of rows and the first group's scale and zero point are requested before the
            // coefficients are fetched: a wave with up to 16 rows has everything in flight at once
            load_batch_q4<NT>(L.Mq, ldq, offq, s.idx, jq_hi, jq_lo, qa);
            load_batch_q4<NT>(L.Mq, ldq, offq, s.idx, jq_hi, jq_lo + kUnroll, qb);
            q4_open<BT>(st, L, uniform(s.idx[jq_lo]) >> L.qshift, colq);
        }
    } else {
        load_batch<NT>(L.M, (size_t)d_out, col, colok, s.idx, n_all, j_first, va);
    }

    // ---- ... and fetch the coefficients x[b, c] * m[b, c] of my rows while those loads fly
    for (int j = tid; j < n; j += nthr) {
        const int c = s.idx[j];
        uint32_t bits = 0;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            float xf = 0.f;
            bool kb = false;
            if (b < nb) {
                const uint16_t h = X[(size_t)(b0 + b) * d_in + c];
                xf = (DT == F16) ? (float)__builtin_bit_cast(_Float16, h) : as_f((uint32_t)h << 16);
                kb = (union_all || (Q4 && a.dense)) ? true
                     : rules.exact ? keep(xf, c, rules.r[b], rules.sgn) : keep_threshold(xf, rules.r[b]);
            }
            s.coef[j * BT + b] = kb ? xf : 0.f;
            bits |= (uint32_t)kb << b;
        }
        if (tile == 0) {          // the tile-0 workgroups publish the list for read-back
            L.act_list[(size_t)z * d_in + lo + j] = c;
            L.act_bits[(size_t)z * d_in + lo + j] = bits;
        }
    }
    __syncthreads();

    // ---- one launch.  The coefficients of the U_r^T rows are t.  Lane l of a wave looks after row
    //      l / BT, token l % BT of a batch; the entries of a batch are requested while the batch
    //      before it is consumed, and written to this wave's own coefficient slots when it is due.
    const uint32_t *t_pub = L.t_pub + (size_t)z * BT * L.rank;
    uint32_t tq = 0u;
    int tq_at = 0;
    bool tq_valid = false;
    auto request_t = [&](int jb) {
        const int j = jb + lane / BT, b = lane % BT;
        tq = 0u;
        tq_valid = jb < n_all && jb + kUnroll > n && lane < kUnroll * BT && j >= n && j < n_all && b < nb;
        if (tq_valid) {
            tq_at = b * L.rank + (s.idx[j] - d_in);
            tq = __hip_atomic_load(t_pub + tq_at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };
    auto settle_t = [&]() {
        if (!__any(tq_valid && tq == kNotReady)) return;
        const long long t0 = wall_clock64();             // rare: stage 1 has not finished yet
        bool ok = false;
        for (int polls = 0; polls < a.wait_polls && !ok; ++polls) {
            __builtin_amdgcn_s_sleep(8);
            if (tq_valid && tq == kNotReady) tq = __hip_atomic_load(t_pub + tq_at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ok = !__any(tq_valid && tq == kNotReady);
            if (!ok && wall_clock64() - t0 > kWaitLimitTicks) break;
        }
        if (!ok && lane == 0) __hip_atomic_store(L.sync + kSyncError, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    auto need_t = [&](int j0) {
        if (j0 + kUnroll > n) {                      // this batch holds rows of U_r^T
            settle_t();
            const int j = j0 + lane / BT;
            if (lane < kUnroll * BT && j >= n && j < n_all) s.coef[j * BT + lane % BT] = tq_valid ? as_f(tq) : 0.f;
            __builtin_amdgcn_wave_barrier();          // read back by this wave only
        }
        request_t(j0 + step);
    };

    if constexpr (Q4) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int b = 0; b < BT; ++b)
#pragma unroll
                for (int e = 0; e < 8; ++e) { st.acc[h][b][e] = 0.f; st.grp[h][b][e] = 0.f; }
#pragma unroll
        for (int b = 0; b < BT; ++b) st.sumx[b] = 0.f;
        for (int j0 = jq_lo; j0 < jq_hi; j0 += 2 * kUnroll) {
            q4_consume<DT, BT>(st, L, qa, s.idx, s.coef, jq_hi, j0, colq);
            if (j0 + kUnroll >= jq_hi) break;
            load_batch_q4<NT>(L.Mq, ldq, offq, s.idx, jq_hi, j0 + 2 * kUnroll, qa);
            q4_consume<DT, BT>(st, L, qb, s.idx, s.coef, jq_hi, j0 + kUnroll, colq);
            if (j0 + 2 * kUnroll >= jq_hi) break;
            load_batch_q4<NT>(L.Mq, ldq, offq, s.idx, jq_hi, j0 + 3 * kUnroll, qb);
        }
        if (st.g >= 0) q4_close<DT, BT>(st);
        if constexpr (FUSED) {
            // one launch: my share of the rows of U_r^T (16-bit, row j = U_r[:, j], padded to whole tiles)
            // with coefficients t, through the 16-bit path's stream, once per 512-column half of the tile.
            // The list holds them as rows d_in + j, so the base is moved back by d_in rows.
            const size_t ldu = (size_t)L.qtiles * kQ4Tile;
            const uint16_t *Uv = reinterpret_cast<const uint16_t *>(reinterpret_cast<uintptr_t>(L.Ut) -
                                                                    (uintptr_t)d_in * ldu * sizeof(uint16_t));
            const int ju = n + j_first;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                u32x4 ua[kUnroll];
                load_batch<NT>(Uv, ldu, colq + h * 512, true, s.idx, n_all, ju, ua);
                request_t(ju);
                stream_rest<DT, BT, NT>(Uv, ldu, colq + h * 512, true, s.idx, s.coef, n_all, ju, step, ua, st.acc[h], need_t);
            }
        }
        // the two 512-column halves of the tile go through the 16-bit path's reduction one after the other
        reduce_to_yacc<BT>(st.acc[0], s.red, L.yacc, b0, nb, d_out, tile * 2);
        __syncthreads();
        reduce_to_yacc<BT>(st.acc[1], s.red, L.yacc, b0, nb, d_out, tile * 2 + 1);
        if constexpr (!FUSED) return;
    } else if (!FUSED) {
        stream_rest<DT, BT, NT>(L.M, (size_t)d_out, col, colok, s.idx, s.coef, n, j_first, step, va, acc, [](int) {});
        reduce_to_yacc<BT>(acc, s.red, L.yacc, b0, nb, d_out, tile);
        return;
    } else {
        request_t(j_first);
        stream_rest<DT, BT, NT>(L.M, (size_t)d_out, col, colok, s.idx, s.coef, n_all, j_first, step, va, acc, need_t);
        reduce_to_yacc<BT>(acc, s.red, L.yacc, b0, nb, d_out, tile);
    }

    // ---- arrive at the tile; the last of its `splits` workgroups owns the finish.  For a gate/up pair
    //      the two layers share the gate layer's counters and the tile is finished once, by the last
    //      of both layers' workgroups (Sec. 3.1: H = X W_up^T (.) silu(X W_gate^T)).
    wait_own_writes();
    __syncthreads();
    const bool pair = ga.gate_up != 0;
    int *const sync = pair ? ga.job[0].L.sync : L.sync;    // owner of the counters: the gate layer
    float *const yacc_g = pair ? ga.job[0].L.yacc : L.yacc;
    const int arrivals = pair ? ga.job[0].splits + ga.job[1].splits : a.splits;
    int *tile_ctr = sync + kSyncTile + z * a.tiles + tile;
    if (tid == 0) {
        const int arrived = __hip_atomic_fetch_add(tile_ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int last_of_layer = 0;
        if (arrived == arrivals - 1) {
            // every workgroup of this tile has consumed t; when that holds for all tiles, t_pub can go back
            __hip_atomic_store(tile_ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int done = __hip_atomic_fetch_add(sync + kSyncTilesDone, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (done == a.tiles * a.nz - 1) {
                __hip_atomic_store(sync + kSyncTilesDone, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                last_of_layer = 1;
            }
        }
        s.misc[12] = arrived;
        s.misc[13] = last_of_layer;
    }
    __syncthreads();
    if (s.misc[12] != arrivals - 1) return;

    // ---- Y = round(Y_s + Y_r): swap the sums out (this re-zeroes yacc for the next call), round once
    constexpr int TW = Q4 ? kQ4Tile : kTile;
    for (int c = tid; c < TW; c += nthr) {
        const int o = tile * TW + c;
        if (o < d_out) {
            float v[BT], vu[BT];
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                const size_t at = (size_t)(b0 + b) * d_out + o;
                v[b] = b < nb ? __hip_atomic_exchange(yacc_g + at, 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
                vu[b] = (pair && b < nb)
                            ? __hip_atomic_exchange(ga.job[1].L.yacc + at, 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                            : 0.f;
            }
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                if (b >= nb) continue;
                const size_t at = (size_t)(b0 + b) * d_out + o;
                if (!pair) {
                    store_out(a.Y, at, EXT ? v[b] + bias_at(L, o) : v[b], L.out_dtype);
                } else {
                    // g and u are rounded to the storage type first, as the two projections would store them
                    const float gb = EXT ? v[b] + bias_at(ga.job[0].L, o) : v[b], ub = EXT ? vu[b] + bias_at(ga.job[1].L, o) : vu[b];
                    const uint16_t g16 = DT == F16 ? to_f16(gb) : to_bf16(gb);
                    const uint16_t u16 = DT == F16 ? to_f16(ub) : to_bf16(ub);
                    ((uint16_t *)ga.job[0].Y)[at] = gated1<DT>(g16, u16);
                }
            }
        }
    }
    if (s.misc[13]) {
        auto reset_t = [&](uint32_t *t_pub, int rank) {
            const int words = a.nz * BT * rank;
            for (int i = tid; i < words; i += nthr)
                __hip_atomic_store(t_pub + i, kNotReady, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        };
        if (pair) {
            reset_t(ga.job[0].L.t_pub, ga.job[0].L.rank);
            reset_t(ga.job[1].L.t_pub, ga.job[1].L.rank);
        } else {
            reset_t(L.t_pub, L.rank);
        }
    }
}

// 4-bit weights, up to 4 tokens: the same scan, list and stage-1 workgroups, the weight stream as above.
// (four tokens need two sets of 16 x 4 accumulators: at most 4 waves per workgroup, one per SIMD, so that a
//  wave may use the whole register file)
template <int DT, int BT, bool NT>
__global__ __launch_bounds__(BT >= 4 ? 256 : 512) void k_q4_sparse_and_t(const GroupArgs ga)
{
    extern __shared__ __align__(16) unsigned char smem[];
    sparse_body<DT, BT, NT, false, true>(ga, smem);
}

// The whole layer on 4-bit weights in one launch (as k_rsparse_fused: stage-1 workgroups publish t, the gather
// workgroups add their share of U_r^T t, the last workgroup of a column tile rounds and stores).
template <int DT, int BT, bool NT>
__global__ __launch_bounds__(BT >= 4 ? 256 : 512) void k_q4_fused(const GroupArgs ga)
{
    extern __shared__ __align__(16) unsigned char smem[];
    sparse_body<DT, BT, NT, true, true>(ga, smem);
}

// Eight tokens of accumulators need the full register file: 4 waves per workgroup, one per SIMD.
template <int DT, int BT, bool NT>
__global__ __launch_bounds__(BT >= 8 ? 256 : 512) void k_sparse_and_t(const GroupArgs ga)
{
    extern __shared__ __align__(16) unsigned char smem[];
    sparse_body<DT, BT, NT, false>(ga, smem);
}

// The whole layer in one launch (see the file header).  Same grid as k_sparse_and_t.
// EXT = false: no layer of the launch has a fixed-count rule, a signed threshold or a bias (the host checks), and the
// code for those is left out -- this kernel's once-per-launch code runs from a cold instruction cache, and the
// general keep-predicate in its token scan measured +0.3 us per launch.
template <int DT, int BT, bool NT, bool EXT>
__global__ __launch_bounds__(BT >= 8 ? 256 : 512, BT >= 8 ? 3 : 4) void k_rsparse_fused(const GroupArgs ga)
{
    extern __shared__ __align__(16) unsigned char smem[];
    sparse_body<DT, BT, NT, true, false, EXT>(ga, smem);
}

// ---------------------------------------------------------------------------------------------
// Dense baseline, axpy form over the same column-major W: every channel, no mask, no low rank.
// Followed by k_finish with rank 0.
// ---------------------------------------------------------------------------------------------
template <int DT, int BT, bool NT>
__global__ __launch_bounds__(BT >= 8 ? 256 : 512) void k_dense_axpy(const GroupArgs ga)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63, w = tid >> 6, nw = nthr >> 6;
    const int z = blockIdx.z;
    int wg;
    const GatherArgs &a = ga.job[find_job(ga.wg_end, ga.n, blockIdx.x, wg)];
    int tile, split;
    if (!map_tile(a, wg, tile, split)) return;
    const LayerView &L = a.L;
    const int d_in = L.d_in, d_out = L.d_out;
    const int b0 = z * BT;
    const int nb = min(BT, a.batch - b0);
    const GatherLds s = carve(smem, a.cap, BT, nw);

    int lo, hi;
    balanced_share(d_in, a.splits, split, lo, hi);
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
    u32x4 va[kUnroll];
    load_batch<NT>(L.M, (size_t)d_out, col, colok, s.idx, n, w * kUnroll, va);
    stream_rest<DT, BT, NT>(L.M, (size_t)d_out, col, colok, s.idx, s.coef, n, w * kUnroll, nw * kUnroll, va, acc,
                            [](int) {});
    reduce_to_yacc<BT>(acc, s.red, L.yacc, b0, nb, d_out, tile);
}

// ---------------------------------------------------------------------------------------------
// Second launch: steps 3b-4 of the layer.  Y[b, o] = round(yacc[b, o] + U_r[o, :] . t[b, :]), a row
// dot over U_r [d_out][rank] row-major (no cross-workgroup reduction), then yacc is re-zeroed for
// the next call.  LPR = lanes that cover one row of U_r (power of two, 16 bytes per lane and pass);
// a wave handles 64/LPR rows per pass.  rank == 0 just rounds yacc.
// grid.x workgroups of 4 waves over row groups, grid.z batch tiles.
// ---------------------------------------------------------------------------------------------
struct FinishArgs {
    LayerView L;
    void *Y;
    int batch, lpr, passes, use_rank;
};

constexpr int kFinishGroups = 4;     // row groups per wave, all loads issued up front
struct FinishGroupArgs {
    FinishArgs job[kMaxGroup];
    int wg_end[kMaxGroup];
    int n;
};

// PASSES = 16-byte pieces per lane and row (rank <= 512 * PASSES); 0 = any rank, loads not batched.
template <int DT, int BT, int PASSES>
__global__ __launch_bounds__(256) void k_finish(const FinishGroupArgs ga)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int z = blockIdx.z;
    int wg;
    const FinishArgs &a = ga.job[find_job(ga.wg_end, ga.n, blockIdx.x, wg)];
    const LayerView &L = a.L;
    const int d_out = L.d_out, r = a.use_rank;
    const int b0 = z * BT;
    const int nb = min(BT, a.batch - b0);
    float *s_t = reinterpret_cast<float *>(smem);             // [BT][r]
    const int lpr = a.lpr, rpi = 64 / lpr;                    // lanes per row, rows per wave and group
    const int sub = lane % lpr, rsel = lane / lpr;
    const int o_wave = (wg * 4 + w) * (rpi * kFinishGroups);
    constexpr int NP = PASSES > 0 ? PASSES : 1;

    // U_r rows and the accumulators first: their latency covers the staging of t
    u32x4 v[kFinishGroups][NP];
    float ya[kFinishGroups][BT];
#pragma unroll
    for (int g = 0; g < kFinishGroups; ++g) {
        const int o = o_wave + g * rpi + rsel;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int i = (p * lpr + sub) * 8;
            v[g][p] = (PASSES > 0 && o < d_out && i < r) ? ldg16<true>(L.U + (size_t)o * r + i) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int b = 0; b < BT; ++b)
            ya[g][b] = (sub == 0 && o < d_out && b < nb) ? L.yacc[(size_t)(b0 + b) * d_out + o] : 0.f;
    }
    {   // stage t [BT][r] in LDS: four values per thread and step, eight steps of loads in flight
        constexpr int SB = 8;
        const int total4 = BT * r / 4;                     // r is a multiple of 8
        const float4 *src = reinterpret_cast<const float4 *>(L.t + ((size_t)z * BT) * r);
        for (int i0 = tid; i0 < total4; i0 += 256 * SB) {
            float4 tv[SB];
#pragma unroll
            for (int u = 0; u < SB; ++u) {
                const int i = i0 + u * 256;
                tv[u] = (i < total4 && (i * 4) / r < nb) ? src[i] : float4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < SB; ++u) {
                const int i = i0 + u * 256;
                if (i < total4) reinterpret_cast<float4 *>(s_t)[i] = tv[u];
            }
        }
    }
    __syncthreads();

    float acc[kFinishGroups][BT];
#pragma unroll
    for (int g = 0; g < kFinishGroups; ++g) {
        const int o = o_wave + g * rpi + rsel;
#pragma unroll
        for (int b = 0; b < BT; ++b) acc[g][b] = 0.f;
        if (PASSES > 0) {
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const int i = (p * lpr + sub) * 8;
                if (o < d_out && i < r) {
                    float f[8];
                    unpack8<DT>(v[g][p], f);
#pragma unroll
                    for (int b = 0; b < BT; ++b) {
                        const float4 t0 = *reinterpret_cast<const float4 *>(s_t + b * r + i);
                        const float4 t1 = *reinterpret_cast<const float4 *>(s_t + b * r + i + 4);
                        float s = acc[g][b];
                        s = __builtin_fmaf(f[0], t0.x, s); s = __builtin_fmaf(f[1], t0.y, s);
                        s = __builtin_fmaf(f[2], t0.z, s); s = __builtin_fmaf(f[3], t0.w, s);
                        s = __builtin_fmaf(f[4], t1.x, s); s = __builtin_fmaf(f[5], t1.y, s);
                        s = __builtin_fmaf(f[6], t1.z, s); s = __builtin_fmaf(f[7], t1.w, s);
                        acc[g][b] = s;
                    }
                }
            }
        } else if (o < d_out) {
            for (int p = 0; p < a.passes; ++p) {
                const int i = (p * lpr + sub) * 8;
                if (i < r) {
                    float f[8];
                    unpack8<DT>(ldg16<true>(L.U + (size_t)o * r + i), f);
#pragma unroll
                    for (int b = 0; b < BT; ++b)
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[g][b] = __builtin_fmaf(f[e], s_t[b * r + i + e], acc[g][b]);
                }
            }
        }
    }
    // Segmented butterfly over the lpr lanes of a row.  The distance is a compile-time constant and
    // all groups x tokens move together, so the cross-lane operations of one step overlap instead of
    // each waiting for the previous one.
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        if (d < lpr) {
#pragma unroll
            for (int g = 0; g < kFinishGroups; ++g)
#pragma unroll
                for (int b = 0; b < BT; ++b) acc[g][b] += __shfl_xor(acc[g][b], d, 64);
        }
    }
#pragma unroll
    for (int g = 0; g < kFinishGroups; ++g) {
        const int o = o_wave + g * rpi + rsel;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            if (sub == 0 && o < d_out && b < nb) {
                store_out(a.Y, (size_t)(b0 + b) * d_out + o, ya[g][b] + acc[g][b] + bias_at(L, o), L.out_dtype);
                L.yacc[(size_t)(b0 + b) * d_out + o] = 0.f;
            }
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

struct RowdotGroupArgs {
    RowdotArgs job[kMaxGroup];
    int wg_end[kMaxGroup];
    int n;
};

template <int DT, int BT, bool NT>
__global__ __launch_bounds__(256) void k_dense_rowdot(const RowdotGroupArgs ga)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int z = blockIdx.z;
    int wg, wg_count;
    {
        const int li = find_job(ga.wg_end, ga.n, blockIdx.x, wg);
        wg_count = ga.wg_end[li] - (li ? ga.wg_end[li - 1] : 0);
    }
    const RowdotArgs &a = ga.job[find_job(ga.wg_end, ga.n, blockIdx.x, wg)];
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
    for (int o = wg * 4 + w; o < d_out; o += wg_count * 4) {
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

int gather_cap(int d_in, int splits, int fused_rank = 0)
{
    return (d_in + splits - 1) / splits + 2 + (fused_rank > 0 ? (fused_rank + splits - 1) / splits + 1 : 0);
}

int lowrank_chunk(int d_in, int bt)
{
    int chunk = (24576 / bt) & ~7;
    return d_in < chunk ? d_in : chunk;
}

}  // namespace

size_t gather_lds_bytes(int d_in, int splits, int waves, int bt, int fused_rank)
{
    const size_t cap = gather_cap(d_in, splits, fused_rank);
    return (waves > 1 ? (size_t)waves * kTile * 4 : 0) + cap * bt * 4 + cap * 4 + 16 * 4 + (size_t)d_in / 8 + 16 +
           (size_t)d_in / 2 + 4 + 2 * ((size_t)d_in / 512 + 2) * 4;   // ... + keep-bits of every 8 channels + their list positions
}

size_t lowrank_lds_bytes(int d_in, int bt)
{
    return (size_t)bt * lowrank_chunk(d_in, bt) * 2 + 16;
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

static bool same_shape_class(const LayerView *L, int n)
{
    for (int i = 1; i < n; ++i)
        if (L[i].d_in != L[0].d_in || L[i].dtype != L[0].dtype) return false;
    return n >= 1 && n <= kMaxGroup;
}

hipError_t launch_sparse_and_t(const LayerView *L, const Launch *cfg, int n, const void *X, int batch, bool with_t,
                               bool with_gather, hipStream_t stream)
{
    if (!same_shape_class(L, n)) return hipErrorInvalidValue;
    const int bt = batch_tile(batch);
    const int nz = (batch + bt - 1) / bt;
    GroupArgs ga{};
    ga.n = n;
    size_t lds = 0;
    int total = 0;
    for (int i = 0; i < n; ++i) {
        GatherArgs &a = ga.job[i];
        const int tiles = (L[i].d_out + kTile - 1) / kTile;
        a.L = L[i]; a.X = (const uint16_t *)X; a.batch = batch; a.splits = cfg[i].splits; a.tiles = tiles;
        a.cap = gather_cap(L[i].d_in, cfg[i].splits);
        a.lr_rows = cfg[i].lowrank_rows;
        a.lr_wgs = (with_t && L[i].rank > 0) ? (L[i].rank + cfg[i].lowrank_rows - 1) / cfg[i].lowrank_rows : 0;
        a.lr_chunk = lowrank_chunk(L[i].d_in, bt);
        a.tile_map = cfg[i].tile_map;
        const int gather_wgs = !with_gather ? 0
                               : cfg[i].tile_map == 2 ? ((tiles + 7) / 8) * 8 * cfg[i].splits : tiles * cfg[i].splits;
        total += a.lr_wgs + gather_wgs;
        ga.wg_end[i] = total;
        lds = std::max(lds, gather_lds_bytes(L[i].d_in, cfg[i].splits, cfg[0].waves, bt));
        if (a.lr_wgs > 0) lds = std::max(lds, lowrank_lds_bytes(L[i].d_in, bt));
    }
    for (int i = n; i < kMaxGroup; ++i) ga.wg_end[i] = total;
    if (total == 0) return hipSuccess;
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    dim3 grid(total, 1, nz), block(kWave * cfg[0].waves);
    const bool nt = cfg[0].nontemporal != 0;
#define RS_G(DT)                                                                                       \
    RS_DISPATCH_BT(bt, {                                                                               \
        if (nt) hipLaunchKernelGGL((k_sparse_and_t<DT, BT, true>), grid, block, lds, stream, ga);      \
        else hipLaunchKernelGGL((k_sparse_and_t<DT, BT, false>), grid, block, lds, stream, ga);        \
    })
    if (L[0].dtype == F16) { RS_G(F16) } else { RS_G(BF16) }
#undef RS_G
    return hipGetLastError();
}

hipError_t launch_q4(const LayerView &L, const Launch &cfg, const void *X, int batch, bool with_t, bool dense,
                     void *Y_fused, hipStream_t stream)
{
    const bool fused = Y_fused != nullptr;
    if (fused && (dense || !with_t || !L.sync || !L.t_pub || (L.rank > 0 && !L.Ut))) return hipErrorInvalidValue;
    if (!L.Mq || !L.qs || !L.qz || batch < 1 || batch > 32 || L.qshift < 3 || (L.d_in >> L.qshift) < 1 ||
        ((L.d_in >> L.qshift) << L.qshift) != L.d_in || L.qtiles != (L.d_out + kQ4Tile - 1) / kQ4Tile ||
        cfg.splits < 1 || cfg.lowrank_rows < 1 || cfg.lowrank_rows > kRowsPerWave * cfg.waves)
        return hipErrorInvalidValue;
    // batches above 4 tokens run as batch tiles of 4 in the grid's z dimension (the codes are streamed once per tile)
    const int bt = std::min(4, batch_tile(batch));
    const int nz = (batch + bt - 1) / bt;
    if (bt >= 4 && cfg.waves > 4) return hipErrorInvalidValue;
    if (fused && nz > kSyncMaxZ) return hipErrorInvalidValue;
    GroupArgs ga{};
    ga.n = 1;
    GatherArgs &a = ga.job[0];
    a.L = L; a.X = (const uint16_t *)X; a.batch = batch; a.splits = cfg.splits; a.tiles = L.qtiles;
    a.cap = gather_cap(L.d_in, cfg.splits, fused ? L.rank : 0);
    a.lr_rows = cfg.lowrank_rows;
    a.lr_wgs = (with_t && !dense && L.rank > 0) ? (L.rank + cfg.lowrank_rows - 1) / cfg.lowrank_rows : 0;
    a.lr_chunk = lowrank_chunk(L.d_in, bt);
    a.tile_map = 1;
    a.dense = dense ? 1 : 0;
    a.Y = Y_fused;
    a.nz = nz;
    a.wait_polls = cfg.wait_polls > 0 ? cfg.wait_polls : kWaitLimitPolls;
    a.skip_stage1 = cfg.skip_stage1;
    const int total = a.lr_wgs + L.qtiles * cfg.splits;
    for (int i = 0; i < kMaxGroup; ++i) ga.wg_end[i] = total;
    size_t lds = gather_lds_bytes(L.d_in, cfg.splits, cfg.waves, bt, fused ? L.rank : 0);
    if (a.lr_wgs > 0) lds = std::max(lds, lowrank_lds_bytes(L.d_in, bt));
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    dim3 grid(total, 1, nz), block(kWave * cfg.waves);
    const bool nt = cfg.nontemporal != 0;
#define RS_Q1(DT, BTV)                                                                                  \
    do {                                                                                                \
        if (fused) {                                                                                    \
            if (nt) hipLaunchKernelGGL((k_q4_fused<DT, BTV, true>), grid, block, lds, stream, ga);      \
            else hipLaunchKernelGGL((k_q4_fused<DT, BTV, false>), grid, block, lds, stream, ga);        \
        } else {                                                                                        \
            if (nt) hipLaunchKernelGGL((k_q4_sparse_and_t<DT, BTV, true>), grid, block, lds, stream, ga);  \
            else hipLaunchKernelGGL((k_q4_sparse_and_t<DT, BTV, false>), grid, block, lds, stream, ga);    \
        }                                                                                               \
    } while (0)
#define RS_Q(DT)                     \
    switch (bt) {                    \
    case 1: RS_Q1(DT, 1); break;     \
    case 2: RS_Q1(DT, 2); break;     \
    default: RS_Q1(DT, 4); break;    \
    }
    if (L.dtype == F16) { RS_Q(F16) } else { RS_Q(BF16) }
#undef RS_Q1
#undef RS_Q
    return hipGetLastError();
}

hipError_t launch_fused(const LayerView *L, const Launch *cfg, int n, const void *X, int batch, void *const *Y,
                        hipStream_t stream, bool gate_up)
{
    if (!same_shape_class(L, n)) return hipErrorInvalidValue;
    if (gate_up && (n != 2 || L[0].d_out != L[1].d_out || L[0].out_dtype != L[0].dtype || cfg[0].tile_map == 2 ||
                    cfg[1].tile_map == 2))
        return hipErrorInvalidValue;
    const int bt = batch_tile(batch);
    const int nz = (batch + bt - 1) / bt;
    if (nz > kSyncMaxZ) return hipErrorInvalidValue;
    GroupArgs ga{};
    ga.n = n;
    size_t lds = 0;
    int total = 0;
    for (int i = 0; i < n; ++i) {
        if (!L[i].sync || !Y[i]) return hipErrorInvalidValue;
        GatherArgs &a = ga.job[i];
        const int tiles = (L[i].d_out + kTile - 1) / kTile;
        a.L = L[i]; a.X = (const uint16_t *)X; a.batch = batch; a.splits = cfg[i].splits; a.tiles = tiles;
        a.cap = gather_cap(L[i].d_in, cfg[i].splits, L[i].rank);
        a.lr_rows = cfg[i].lowrank_rows;
        a.lr_wgs = L[i].rank > 0 ? (L[i].rank + cfg[i].lowrank_rows - 1) / cfg[i].lowrank_rows : 0;
        a.lr_chunk = lowrank_chunk(L[i].d_in, bt);
        size_t lr_lds = a.lr_wgs > 0 ? lowrank_lds_bytes(L[i].d_in, bt) : 0;
        // one token and a channel-major copy of S_r V_r^T: stage 1 reads only the dropped channels' rows
        if (bt <= 4 && cfg[i].lowrank_wgs > 0 && L[i].rank > 0 && L[i].SVc && L[i].t_sum &&
            (L[i].rank + kTile - 1) / kTile <= cfg[0].waves) {
            const int nq = L[i].d_in / 8;
            const int entry = 4 + 4 * bt;                            // bytes of a list entry: index + a coefficient per token
            a.lr_gather = 1;
            a.lr_wgs = std::min(cfg[i].lowrank_wgs, nq);
            // a workgroup's list of dropped channels (all of its range at worst) has to fit LDS next to the reduction
            // buffer: at least as many workgroups as keep it under 32 KiB
            a.lr_wgs = std::max(a.lr_wgs, (nq * 8 * entry + 32 * 1024 - 1) / (32 * 1024));
            a.lr_cap = ((nq + a.lr_wgs - 1) / a.lr_wgs) * 8;
            lr_lds = (size_t)cfg[0].waves * kTile * 4 + (size_t)a.lr_cap * entry + (size_t)(cfg[0].waves + 1) * 4;
        }
        a.tile_map = cfg[i].tile_map;
        a.Y = Y[i];
        a.nz = nz;
        a.wait_polls = cfg[i].wait_polls > 0 ? cfg[i].wait_polls : kWaitLimitPolls;
        a.skip_stage1 = cfg[i].skip_stage1;
        const int gather_wgs = cfg[i].tile_map == 2 ? ((tiles + 7) / 8) * 8 * cfg[i].splits : tiles * cfg[i].splits;
        total += a.lr_wgs + gather_wgs;
        ga.wg_end[i] = total;
        const size_t need = gather_lds_bytes(L[i].d_in, cfg[i].splits, cfg[0].waves, bt, L[i].rank);
        if (need > 64 * 1024) return hipErrorInvalidValue;
        lds = std::max(lds, need);
        if (lr_lds > 64 * 1024) return hipErrorInvalidValue;
        lds = std::max(lds, lr_lds);
    }
    for (int i = n; i < kMaxGroup; ++i) ga.wg_end[i] = total;
    ga.gate_up = gate_up ? 1 : 0;
    dim3 grid(total, 1, nz), block(kWave * cfg[0].waves);
    const bool nt = cfg[0].nontemporal != 0;
    bool ext = false;
    for (int i = 0; i < n; ++i) ext = ext || L[i].rules || L[i].bias || L[i].keep_signed;
#define RS_U(DT)                                                                                        \
    RS_DISPATCH_BT(bt, {                                                                                \
        if (nt && !ext) hipLaunchKernelGGL((k_rsparse_fused<DT, BT, true, false>), grid, block, lds, stream, ga);      \
        else if (nt) hipLaunchKernelGGL((k_rsparse_fused<DT, BT, true, true>), grid, block, lds, stream, ga);          \
        else if (!ext) hipLaunchKernelGGL((k_rsparse_fused<DT, BT, false, false>), grid, block, lds, stream, ga);      \
        else hipLaunchKernelGGL((k_rsparse_fused<DT, BT, false, true>), grid, block, lds, stream, ga);                 \
    })
    if (L[0].dtype == F16) { RS_U(F16) } else { RS_U(BF16) }
#undef RS_U
    return hipGetLastError();
}

hipError_t launch_finish(const LayerView *L, int n, int batch, void *const *Y, bool use_rank, hipStream_t stream)
{
    if (!same_shape_class(L, n)) return hipErrorInvalidValue;
    const int bt = batch_tile(batch);
    const int nz = (batch + bt - 1) / bt;
    FinishGroupArgs ga{};
    ga.n = n;
    size_t lds = 16;
    int total = 0, max_passes = 0;
    for (int i = 0; i < n; ++i) {
        FinishArgs &a = ga.job[i];
        a.L = L[i]; a.Y = Y[i]; a.batch = batch;
        a.use_rank = use_rank ? L[i].rank : 0;
        const int chunks = (a.use_rank + 7) / 8;          // 16-byte pieces per row of U_r
        int lpr = 1;
        while (lpr < chunks && lpr < 64) lpr <<= 1;
        a.lpr = lpr;
        a.passes = chunks == 0 ? 0 : (chunks + lpr - 1) / lpr;
        max_passes = std::max(max_passes, a.passes);
        const int rows_per_wg = 4 * (64 / lpr) * kFinishGroups;
        total += (L[i].d_out + rows_per_wg - 1) / rows_per_wg;
        ga.wg_end[i] = total;
        lds = std::max(lds, (size_t)bt * a.use_rank * 4 + 16);
    }
    for (int i = n; i < kMaxGroup; ++i) ga.wg_end[i] = total;
    dim3 grid(total, 1, nz), block(256);
#define RS_F(DT)                                                                                           \
    RS_DISPATCH_BT(bt, {                                                                                   \
        if (max_passes <= 1) hipLaunchKernelGGL((k_finish<DT, BT, 1>), grid, block, lds, stream, ga);      \
        else if (max_passes == 2) hipLaunchKernelGGL((k_finish<DT, BT, 2>), grid, block, lds, stream, ga); \
        else hipLaunchKernelGGL((k_finish<DT, BT, 0>), grid, block, lds, stream, ga);                      \
    })
    if (L[0].dtype == F16) { RS_F(F16) } else { RS_F(BF16) }
#undef RS_F
    return hipGetLastError();
}

hipError_t launch_dense_axpy(const LayerView *L, const Launch *cfg, int n, const void *X, int batch, void *const *Y,
                             hipStream_t stream)
{
    if (!same_shape_class(L, n)) return hipErrorInvalidValue;
    const int bt = batch_tile(batch);
    const int nz = (batch + bt - 1) / bt;
    GroupArgs ga{};
    ga.n = n;
    size_t lds = 0;
    int total = 0;
    for (int i = 0; i < n; ++i) {
        GatherArgs &a = ga.job[i];
        const int tiles = (L[i].d_out + kTile - 1) / kTile;
        a.L = L[i]; a.X = (const uint16_t *)X; a.batch = batch; a.splits = cfg[i].splits; a.tiles = tiles;
        a.cap = gather_cap(L[i].d_in, cfg[i].splits);
        a.tile_map = cfg[i].tile_map;
        total += cfg[i].tile_map == 2 ? ((tiles + 7) / 8) * 8 * cfg[i].splits : tiles * cfg[i].splits;
        ga.wg_end[i] = total;
        lds = std::max(lds, gather_lds_bytes(L[i].d_in, cfg[i].splits, cfg[0].waves, bt));
    }
    for (int i = n; i < kMaxGroup; ++i) ga.wg_end[i] = total;
    dim3 grid(total, 1, nz), block(kWave * cfg[0].waves);
    const bool nt = cfg[0].nontemporal != 0;
#define RS_D(DT)                                                                                     \
    RS_DISPATCH_BT(bt, {                                                                             \
        if (nt) hipLaunchKernelGGL((k_dense_axpy<DT, BT, true>), grid, block, lds, stream, ga);      \
        else hipLaunchKernelGGL((k_dense_axpy<DT, BT, false>), grid, block, lds, stream, ga);        \
    })
    if (L[0].dtype == F16) { RS_D(F16) } else { RS_D(BF16) }
#undef RS_D
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_finish(L, n, batch, Y, false, stream);
}

hipError_t launch_dense_rowdot(const LayerView *L, const Launch *cfg, int n, const void *X, int batch, void *const *Y,
                               hipStream_t stream)
{
    if (!same_shape_class(L, n)) return hipErrorInvalidValue;
    const int bt = batch_tile(batch);
    const int nz = (batch + bt - 1) / bt;
    RowdotGroupArgs ga{};
    ga.n = n;
    int total = 0;
    for (int i = 0; i < n; ++i) {
        ga.job[i] = RowdotArgs{L[i], (const uint16_t *)X, Y[i], batch};
        int wgs = (L[i].d_out + 3) / 4;
        if (wgs > 2048) wgs = 2048;
        total += wgs;
        ga.wg_end[i] = total;
    }
    for (int i = n; i < kMaxGroup; ++i) ga.wg_end[i] = total;
    const size_t lds = (size_t)bt * L[0].d_in * 2;
    dim3 grid(total, 1, nz), block(256);
    const bool nt = cfg[0].nontemporal != 0;
#define RS_R(DT)                                                                                      \
    RS_DISPATCH_BT(bt, {                                                                              \
        if (nt) hipLaunchKernelGGL((k_dense_rowdot<DT, BT, true>), grid, block, lds, stream, ga);     \
        else hipLaunchKernelGGL((k_dense_rowdot<DT, BT, false>), grid, block, lds, stream, ga);       \
    })
    if (L[0].dtype == F16) { RS_R(F16) } else { RS_R(BF16) }
#undef RS_R
    return hipGetLastError();
}

// x = round16(silu(g) * u) written out (Sec. 3.1).  Forming it inside the gather kernel's own token loads was
// measured and lost: every workgroup scans the whole token, so the activation was evaluated ~400 times over
// (24.0 us against 22.1 us for this kernel followed by the plain layer, 11008 -> 4096).
template <int DT>
__global__ void k_gated_input(const uint16_t *G, const uint16_t *Up, uint16_t *out, size_t n8)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n8; i += stride) *reinterpret_cast<u32x4 *>(out + i * 8) = load_x8<DT>(Up, G, i * 8);
}

hipError_t launch_gated_input(const void *G, const void *Up, void *out, size_t n, int dtype, hipStream_t stream)
{
    if (n == 0 || (n % 8) != 0) return hipErrorInvalidValue;
    const size_t n8 = n / 8;
    size_t blocks = (n8 + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    if (dtype == F16)
        hipLaunchKernelGGL(k_gated_input<F16>, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint16_t *)G,
                           (const uint16_t *)Up, (uint16_t *)out, n8);
    else
        hipLaunchKernelGGL(k_gated_input<BF16>, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint16_t *)G,
                           (const uint16_t *)Up, (uint16_t *)out, n8);
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
