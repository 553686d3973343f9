// gfx950 (MI355X, CDNA4): the R-Sparse linear layer (Sec. 3.4) over STRIP-MAJOR weights, up to 8 tokens.
//
// Sec. 3.4 stores W column-major so that a kept input channel is one contiguous run.  Here that run is cut into
// strips of strip_w = 32 .. 512 output columns and the strips are stored one after the other,
//
//   Ms [strips][d_in + r][strip_w]     row c < d_in: W[strip columns, c];  row d_in + j: U_r[strip columns, j]
//
// so that ONE workgroup can own a strip of outputs for ALL input channels: it streams the strip's kept rows
// (each still one contiguous run of 2 * strip_w bytes; the strip is one contiguous region of memory that the
// workgroup walks front to back), adds the rows of U_r^T weighted by t (stage 2 of the low-rank part is the same
// gather with r more "channels"), and stores its slice of Y itself: no partial sums cross workgroups, no atomics,
// no arrival counters, no finishing pass.  Layers with few strips can still split the channels over `splits`
// workgroups per strip; those meet in fp32 atomics and the last one to arrive rounds and stores.
//
// Inside a workgroup every wave is on its own until the final sum: wave w of split s owns a FIXED range of
// input channels (an equal share of d_in, not of the kept list), reads only that part of the token, thresholds it
// (Sec. 3.4, sigma_t), compacts the kept channels with a register scan into a list in its own piece of LDS, and
// starts streaming -- no workgroup barrier and no whole-token scan ahead of the first weight load.  Ranges are
// long (hundreds of channels), so the binomial spread of kept counts between waves stays at a few per cent.
// A wave-wide 16-byte load covers 64 / LPR rows of the strip at once (LPR = strip_w / 8 lanes per row); row index
// and coefficient are per lane, read from the wave's list.
//
// Stage 1 of the low-rank part, t = S_r V_r^T (x - sigma_t(x)), runs in workgroups at the front of the same grid
// (dispatched first).  They publish each t_j as one 64-bit word {generation, fp32 bits}.  The generation number
// of a launch is a word in device memory that every wave reads at its start; a wave reports its read with a
// store-and-forget atomic, and the first stage-1 workgroup, once all waves of the launch have reported, bumps the
// number for the next launch.  A consumer accepts an entry only when it carries the launch's generation, so
// entries left by earlier launches never match, nothing has to be reset at the end of a launch, and no workgroup
// waits for anything at its end.
#include "kernels.h"
#include "device_common.h"
#include "device_stage1.h"

#include <algorithm>

namespace rsparse {
#if RSPARSE_STAMPS
__device__ unsigned long long *g_stamp_buf = nullptr;
__device__ int g_stamp_cap = 0;
hipError_t set_stamp_buffer(void *buf, int capacity_waves)
{
    hipError_t e = hipMemcpyToSymbol(HIP_SYMBOL(g_stamp_buf), &buf, sizeof buf);
    if (e != hipSuccess) return e;
    return hipMemcpyToSymbol(HIP_SYMBOL(g_stamp_cap), &capacity_waves, sizeof capacity_waves);
}
#else
hipError_t set_stamp_buffer(void *, int) { return hipErrorNotSupported; }
#endif
namespace {

struct StripArgs {
    LayerView L;
    const uint16_t *X;
    void *Y;
    int batch;
    int tiles, splits;                 // strips of the layer; workgroups (channel splits) per strip
    int cap;                           // list entries per wave (LDS)
    int lr_wgs, lr_rows, lr_chunk;     // stage-1 workgroups at the front of the job's range, rows each, LDS chunk
    int lr_last;                       // stage-1 workgroups at the END of the job's range instead (see launch_strip)
    int wait_polls, skip_stage1;
    int dense;                         // every channel kept and no low-rank part: the dense product Y = X W^T
    int gen_readers;                   // waves of the layer's part of the launch (all batch tiles): each reads the generation
};

struct StripGroupArgs {
    StripArgs job[kMaxGroupLayers];
    int wg_end[kMaxGroupLayers];
    int n;
};

__device__ __forceinline__ int job_of(const int (&wg_end)[kMaxGroupLayers], int n, int wg, int &local)
{
    int li = 0, begin = 0;
#pragma unroll
    for (int i = 0; i < kMaxGroupLayers - 1; ++i)
        if (i + 1 < n && wg >= wg_end[i]) { li = i + 1; begin = wg_end[i]; }
    local = wg - begin;
    return li;
}

// ---------------------------------------------------------------------------------------------
// Stage 1 of the low-rank part inside the strip kernel's launch: t_i = sum_c (S_r V_r^T)[i, c] (x - sigma_t(x))_c.
// The rows of S_r V_r^T do not depend on the token, so a wave requests its part of its row FIRST and stages the
// masked token afterwards: the requests are on their way before the strip workgroups (which need the token to
// know their rows) start to load, and t is ready long before they need it.  A row is shared by `ws` waves of the
// workgroup (so that a wave's part of a row is one batch of loads for the usual row lengths); the parts meet in
// LDS.  a.lr_rows = rows per workgroup = waves / ws.
// ---------------------------------------------------------------------------------------------
constexpr int kS1Batches = 2;      // batches of row loads a stage-1 wave keeps in flight

template <int DT, int BT, typename Args>
__device__ __forceinline__ void stage1_tagged(const Args &a, unsigned char *smem, int wg, int z)
{
    constexpr int LU = 8;
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63, w = uniform(tid >> 6), nw = nthr >> 6;
    const LayerView &L = a.L;
    const int d_in = L.d_in, r = L.rank;
    const int b0 = z * BT;
    const int nb = min(BT, a.batch - b0);
    const bool union_all = L.batch_mask_mode == 1;
    TileRules<BT> rules;
    load_rules<BT>(L, b0, nb, rules);
    const int rpw = a.lr_rows, ws = nw / rpw;              // rows per workgroup, waves per row
    const int row = wg * rpw + w / ws, seg = w % ws;
    const bool have = row < r;
    uint16_t *s_xm = reinterpret_cast<uint16_t *>(smem);                                   // [BT][chunk]
    float *s_part = reinterpret_cast<float *>(smem + (((size_t)BT * a.lr_chunk * 2 + 15) & ~(size_t)15));   // [nw][BT]
    const uint32_t gen = __hip_atomic_load(L.sync + kSyncGen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    RS_STAMP_DECL;
    RS_STAMP(1);

    float part[BT];
#pragma unroll
    for (int b = 0; b < BT; ++b) part[b] = 0.f;

    for (int c0 = 0; c0 < d_in; c0 += a.lr_chunk) {
        const int len = min(a.lr_chunk, d_in - c0);
        const int nq = len / 8;
        int s_lo, s_hi;                                     // my part of the chunk, in 16-byte pieces
        balanced_share(nq, ws, seg, s_lo, s_hi);
        const uint16_t *rowp = L.SVt + (size_t)(have ? row : 0) * d_in + c0;
        // up to kS1Batches batches of LU loads in flight per lane.  The loads are unconditional (positions past the
        // wave's part re-read its last piece and are dropped when consumed) so that the compiler counts the
        // outstanding ones exactly and a wave really keeps the later batches in flight while it consumes the first;
        // with one batch at a time a wave of the 28672-channel down projection needed four dependent round trips
        // through a memory system that the strip waves keep saturated, and the strips waited 9 us for t
        u32x4 v[kS1Batches][LU];
        const int q_last = max(nq - 1, 0);
        auto request = [&](u32x4 (&dst)[LU], int q0) {
#pragma unroll
            for (int u = 0; u < LU; ++u) dst[u] = ldg16<true>(rowp + min(q0 + u * 64, q_last) * 8);
        };
        constexpr int kStep = 64 * LU;
        int q0 = s_lo + lane;
#pragma unroll
        for (int i = 0; i < kS1Batches; ++i)
            if (s_lo + i * kStep < s_hi) request(v[i], q0 + i * kStep);     // before the token: these loads need only the row
        if (c0 > 0) __syncthreads();
        constexpr int PB = TokenBatch<BT>::kGroups;
        for (int p0 = tid; p0 < nq; p0 += nthr * PB) {
            u32x4 raw[PB][BT];
#pragma unroll
            for (int p = 0; p < PB; ++p)
                if (p0 + p * nthr < nq) load_raw8<BT>(a.X, b0, nb, d_in, c0 + (p0 + p * nthr) * 8, raw[p]);
#pragma unroll
            for (int p = 0; p < PB; ++p) {
                const int q = p0 + p * nthr;
                if (q < nq) {
                    uint32_t m[BT];
                    masks_of8<DT, BT>(L, a.X, a.batch, b0, nb, d_in, c0 + q * 8, rules, union_all, raw[p], m);
#pragma unroll
                    for (int b = 0; b < BT; ++b) {
                        u32x4 o = raw[p][b];
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if ((m[b] >> e) & 1u) o[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;   // kept -> 0
                        *reinterpret_cast<u32x4 *>(s_xm + (size_t)b * a.lr_chunk + q * 8) = o;
                    }
                }
            }
        }
        __syncthreads();
        if (c0 == 0) {
            RS_STAMP(2);
            generation_was_read(L.sync, gen, (int)blockIdx.x * nw + w);
        }
        bool more = s_lo < s_hi;                            // wave-uniform
        while (more) {
#pragma unroll
            for (int i = 0; i < kS1Batches; ++i) {
                if (more) {
#pragma unroll
                    for (int u = 0; u < LU; ++u) {
                        const int q = q0 + u * 64;
                        if (have && q < s_hi) {
                            float f[8];
                            unpack8<DT>(v[i][u], f);
#pragma unroll
                            for (int b = 0; b < BT; ++b) {
                                float xf[8];
                                unpack8<DT>(*reinterpret_cast<const u32x4 *>(s_xm + (size_t)b * a.lr_chunk + q * 8), xf);
#pragma unroll
                                for (int e = 0; e < 8; ++e) part[b] = __builtin_fmaf(f[e], xf[e], part[b]);
                            }
                        }
                    }
                    const int qn = q0 + kS1Batches * kStep;
                    if (qn - lane < s_hi) request(v[i], qn);
                    q0 += kStep;
                    more = q0 - lane < s_hi;
                }
            }
        }
    }
    RS_STAMP(3);
    // the ws parts of a row meet in LDS; the first wave of the row publishes
#pragma unroll
    for (int b = 0; b < BT; ++b) {
        const float v = wave_sum(part[b]);
        if (lane == 0) s_part[w * BT + b] = v;
    }
    __syncthreads();
    if (seg == 0 && have && lane < BT && !a.skip_stage1) {
        float v = 0.f;
        for (int i = 0; i < ws; ++i) v += s_part[(w + i) * BT + lane];
        __hip_atomic_store(L.t_tag + ((size_t)z * BT + lane) * r + row, ((unsigned long long)gen << 32) | as_u(v),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // the token slots this call does not use get the generation too (value 0), so that no slot ever carries a tag
    // older than the previous call's -- a slot left alone for 2^32 calls could otherwise match again
    if (z == (int)gridDim.z - 1 && seg == 0 && have && !a.skip_stage1) {
        for (int sl = (int)gridDim.z * BT + lane; sl < L.t_slots; sl += 64)
            __hip_atomic_store(L.t_tag + (size_t)sl * r + row, (unsigned long long)gen << 32, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }
    RS_STAMP(4);
    // the layer's first stage-1 workgroup doubles as the launch's poller (see device_stage1.h)
    if (wg == 0 && z == 0 && w == 0) close_generation(L.sync, a.gen_readers);
    RS_STAMP(5);
    RS_STAMP_FLUSH(1, wg, w);
}

// The wave's list lives in LDS in blocks of kUnroll wave-wide loads (BLK = kUnroll * RPI entries, RPI = rows per
// load): inside a block the entry of load u, row group g sits at g * kUnroll + u, so that a lane finds the rows of
// its eight loads in one 16-byte LDS read and their coefficients in two per token.  An entry is a 16-bit row code
// -- a kept channel relative to the start of the wave's range, or 0x8000 | j for row j of the wave's share of
// U_r^T -- and one fp32 coefficient per token: the token's value on a kept channel (0 where that token does not
// keep it), t_j on a row of U_r^T.
template <int RPI>
__device__ __forceinline__ int list_slot(int p)
{
    constexpr int BLK = kUnroll * RPI;
    return (p & ~(BLK - 1)) + (p & (RPI - 1)) * kUnroll + ((p & (BLK - 1)) / RPI);
}

__host__ __device__ inline int strip_wave_bytes(int cap, int bt) { return (cap * (2 + 4 * bt) + 15) & ~15; }

template <int DT, int BT, int LPR, bool FUSED>
__device__ __forceinline__ void strip_body(const StripGroupArgs &ga, unsigned char *smem)
{
    constexpr int W = LPR * 8, RPI = 64 / LPR, BLK = kUnroll * RPI;
    static_assert(kUnroll == 8, "a lane reads the row codes of a block as one 16-byte vector");
    const int z = blockIdx.z;
    int wg;
    const StripArgs &a = ga.job[job_of(ga.wg_end, ga.n, blockIdx.x, wg)];
    const LayerView &L = a.L;
    const int lr_wgs = FUSED ? pin(a.lr_wgs) : 0;
    const int n_strip_wgs = pin(a.tiles) * pin(a.splits);
    if (FUSED && lr_wgs > 0) {
        const bool lr_last = pin(a.lr_last) != 0;
        if (lr_last ? wg >= n_strip_wgs : wg < lr_wgs) {
            stage1_tagged<DT, BT>(a, smem, lr_last ? wg - n_strip_wgs : wg, z);
            return;
        }
        if (!lr_last) wg -= lr_wgs;
    }
    RS_STAMP_DECL;
    RS_STAMP(1);
    const int tid = threadIdx.x, lane = tid & 63, w = uniform(tid >> 6), nw = (int)blockDim.x >> 6;
    const int tiles = pin(a.tiles), n_splits = pin(a.splits);
    const uint16_t *const X = pin(a.X);
    const int d_in = pin(L.d_in), d_out = pin(L.d_out), batch = pin(a.batch), cap = pin(a.cap);
    const bool dense = pin(a.dense) != 0;
    const int rank = dense ? 0 : pin(L.rank);
    const bool union_all = pin(L.batch_mask_mode) == 1;
    RS_STAMP(11);                                   // kernel arguments are here
    const int g = wg;
    const int tile = g % tiles, split = g / tiles;
    const int b0 = z * BT;
    const int nb = min(BT, batch - b0);
    const int grp = lane / LPR, part = lane % LPR;

    // my fixed share of the input channels (in units of 8) and of the rows of U_r^T
    const int R = n_splits * nw, rho = split * nw + w;
    int q_lo, q_hi, r_lo, r_hi;
    balanced_share(d_in >> 3, R, rho, q_lo, q_hi);
    balanced_share(rank, R, rho, r_lo, r_hi);
    const int nu = r_hi - r_lo;
    // the generation of this launch, requested before anything else
    uint32_t gen = 0;
    const bool tagged = FUSED && rank > 0;
    if (tagged) gen = __hip_atomic_load(L.sync + kSyncGen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    bool reported = !tagged;

    unsigned char *const wbase = smem + (size_t)w * strip_wave_bytes(cap, BT);
    float *const s_cf = reinterpret_cast<float *>(wbase);                         // [cap][BT], blocked (see list_slot)
    uint16_t *const s_idx = reinterpret_cast<uint16_t *>(wbase + (size_t)cap * BT * 4);
    float *const s_red = reinterpret_cast<float *>(smem + (size_t)nw * strip_wave_bytes(cap, BT));
    int *const s_misc = reinterpret_cast<int *>(s_red + nw * BT * W);

    // the strip: rows of strip_w values, row c at c * W; this lane reads 8 consecutive columns of a row
    const uint16_t *const Mt = L.Ms + (size_t)tile * (size_t)L.strip_stride + part * 8;
    const int row_kept = q_lo * 8, row_u = d_in + r_lo - 0x8000;       // row = code + (code < 0x8000 ? row_kept : row_u)
    const bool publish = !dense && tile == 0;        // strip 0's workgroups leave the kept lists for read-back

    float acc[BT][8];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[b][e] = 0.f;

    TileRules<BT> rules;
    load_rules<BT>(L, b0, nb, rules);
    constexpr int SC = BT >= 8 ? 1 : (BT == 1 ? 6 : 8 / BT);           // 64-channel pieces of the token held in registers per round
    const int c_lo = q_lo * 8, c_hi = q_hi * 8;
    int c = c_lo, pub = 0;
    bool last;
    uint32_t xr[SC][BT];
    auto request_x = [&]() {
#pragma unroll
        for (int j = 0; j < SC; ++j) {
            const int cc = c + j * 64 + lane;
#pragma unroll
            for (int b = 0; b < BT; ++b) xr[j][b] = (cc < c_hi && b < nb) ? X[(size_t)(b0 + b) * d_in + cc] : 0u;
        }
    };
    request_x();
    do {
        // ---- sigma_t on my part of the token, one lane per channel: the kept channels of 64 are a ballot, their
        //      places in the list a count of the lower lanes' bits.  As many pieces of 64 as the list has room for.
#if RSPARSE_STAMPS
        if (c == c_lo) {
            __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
            RS_STAMP(12);                           // my part of the token has arrived
        }
#endif
        int n = 0, taken = 0;
        bool open = true;
#pragma unroll
        for (int j = 0; j < SC; ++j) {
            const int cj = c + j * 64;
            const bool take = open && cj < c_hi && n + 64 + nu + BLK <= cap;        // wave-uniform
            if (take) {
                const int cc = cj + lane;
                const bool valid = cc < c_hi;
                float xf[BT];
                bool kb[BT];
                bool any = false;
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    xf[b] = widen16<DT>((uint16_t)xr[j][b]);
                    kb[b] = valid && b < nb && (dense || keep(xf[b], cc, rules.r[b], rules.sgn));
                    any = any || kb[b];
                }
                if (union_all && !dense) {
                    // every token uses the union over the WHOLE batch (also the tokens of other batch tiles)
                    for (int bb = 0; bb < batch; ++bb) {
                        if (bb >= b0 && bb < b0 + nb) continue;
                        const float xo = valid ? widen16<DT>(X[(size_t)bb * d_in + cc]) : 0.f;
                        any = any || (valid && keep(xo, cc, rule_of(L, bb), rules.sgn));
                    }
#pragma unroll
                    for (int b = 0; b < BT; ++b) kb[b] = any && b < nb;
                }
                const unsigned long long mask = __ballot(any);
                const int pp = n + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                if (any) {
                    const int at = list_slot<RPI>(pp);
                    s_idx[at] = (uint16_t)(cc - c_lo);
                    uint32_t bits = 0;
#pragma unroll
                    for (int b = 0; b < BT; ++b) {
                        s_cf[(at & ~(kUnroll - 1)) * BT + b * kUnroll + (at & (kUnroll - 1))] = kb[b] ? xf[b] : 0.f;
                        bits |= (uint32_t)kb[b] << b;
                    }
                    if (publish) {
                        const size_t o = (size_t)z * d_in + (size_t)c_lo + pub + pp;
                        L.act_list[o] = cc;
                        L.act_bits[o] = bits;
                    }
                }
                n += __popcll(mask);
                ++taken;
            } else {
                open = false;
            }
        }
        const int c_seg = c;                     // first channel of this segment
        c += taken * 64;
        last = c >= c_hi;
        if (!last) request_x();                  // the next round's part of the token travels while this segment streams
        // the last segment ends with my rows of U_r^T (coefficients filled in when t arrives); the rest of the last
        // block repeats the segment's first row with coefficient zero (a cache hit that adds nothing)
        const int nus = last ? nu : 0;
        const int ne = n + nus;
        const int nblk = (ne + BLK - 1) / BLK;
        for (int p = n + lane; p < nblk * BLK; p += 64) {
            const int at = list_slot<RPI>(p);
            s_idx[at] = (uint16_t)(p < ne ? (0x8000 | (p - n)) : (n > 0 ? c_seg - c_lo : 0));
#pragma unroll
            for (int b = 0; b < BT; ++b) s_cf[(at & ~(kUnroll - 1)) * BT + b * kUnroll + (at & (kUnroll - 1))] = 0.f;
        }
        __builtin_amdgcn_wave_barrier();         // the list is read back by this wave only
        if (pub == 0) RS_STAMP(2);               // (first segment) my part of the token is here and compacted
        pub += n;
        // the token has arrived, and with it the generation requested before it: say so (once)
        if (!reported) {
            generation_was_read(L.sync, gen, (int)blockIdx.x * nw + w);
            reported = true;
        }

        // ---- stream the segment, block by block: a block's eight loads are requested while the block before it is
        //      consumed (two blocks in flight)
        if (nblk > 0) {
            typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
            auto issue = [&](int k, u32x4(&v)[kUnroll]) {
                const int kc = min(k, nblk - 1);                     // past the end: the last block again (cache hits)
                const u16x8 codes = *reinterpret_cast<const u16x8 *>(s_idx + kc * BLK + grp * kUnroll);
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int code = codes[u];
                    const int row = code + ((code & 0x8000) ? row_u : row_kept);
                    v[u] = ldg16<true>(Mt + (size_t)row * W);
                }
            };
            auto fma = [&](int k, const u32x4(&v)[kUnroll]) {
                if (k >= nblk) return;                                // wave-uniform
                float cf[BT][kUnroll];
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    const float4 *src = reinterpret_cast<const float4 *>(s_cf + (k * BLK + grp * kUnroll) * BT + b * kUnroll);
                    const float4 c0 = src[0], c1 = src[1];
                    cf[b][0] = c0.x; cf[b][1] = c0.y; cf[b][2] = c0.z; cf[b][3] = c0.w;
                    cf[b][4] = c1.x; cf[b][5] = c1.y; cf[b][6] = c1.z; cf[b][7] = c1.w;
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    float f[8];
                    unpack8<DT>(v[u], f);
#pragma unroll
                    for (int b = 0; b < BT; ++b)
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[b][e] = __builtin_fmaf(cf[b][u], f[e], acc[b][e]);
                }
            };
            // t of my rows of U_r^T: requested three blocks ahead of the first block that needs it, written into the
            // coefficient slots of those rows when that block is due
            const int k_use = n / BLK;
            const int k_req = max(0, k_use - 3);
            unsigned long long tq[2] = {0ull, 0ull};
            const unsigned long long *t_tag = L.t_tag;
            auto slot_addr = [&](int v) -> size_t {          // value v of the wave: row v / BT of its share, token v % BT
                return (size_t)(b0 + v % BT) * L.rank + r_lo + v / BT;
            };
            auto put_t = [&](int v, float val) {
                const int at = list_slot<RPI>(n + v / BT);
                s_cf[(at & ~(kUnroll - 1)) * BT + (v % BT) * kUnroll + (at & (kUnroll - 1))] = val;
            };
            auto hook = [&](int k) {
                if (nus == 0) return;
                if (FUSED) {
                    if (k == k_req) {
#pragma unroll
                        for (int i = 0; i < 2; ++i) {
                            const int v = lane + 64 * i;
                            if (v < nus * BT)
                                tq[i] = __hip_atomic_load(t_tag + slot_addr(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
                    if (k == k_use) {
                        RS_STAMP(4);
                        // anything not there yet is re-read, with a bound (stage 1 runs in workgroups dispatched before
                        // this one and waits for nothing, so it ends; the bound turns the impossible into an error flag)
                        bool bad = false;
                        for (int v0 = 0; v0 < nus * BT; v0 += 64) {
                            const int v = v0 + lane;
                            const bool mine = v < nus * BT;
                            unsigned long long val = v0 == 0 ? tq[0] : (v0 == 64 ? tq[1] : 0ull);
                            auto ready = [&]() { return !mine || (uint32_t)(val >> 32) == gen; };
                            if (v0 >= 128 && mine)
                                val = __hip_atomic_load(t_tag + slot_addr(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            if (__any(!ready())) {
                                const long long t0 = wall_clock64();
                                bool ok = false;
                                for (int polls = 0; polls < a.wait_polls && !ok; ++polls) {
                                    __builtin_amdgcn_s_sleep(8);
                                    if (!ready())
                                        val = __hip_atomic_load(t_tag + slot_addr(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                    ok = !__any(!ready());
                                    if (!ok && wall_clock64() - t0 > kWaitLimitTicks) break;
                                }
                                bad = bad || !ok;
                            }
                            if (mine) put_t(v, ready() ? as_f((uint32_t)val) : 0.f);
                        }
                        if (bad && lane == 0)
                            __hip_atomic_fetch_or(L.sync + kSyncError, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        __builtin_amdgcn_wave_barrier();
                        RS_STAMP(5);
                    }
                } else if (k == k_use) {
                    // two launches: t was stored by the launch before this one
                    for (int v = lane; v < nus * BT; v += 64)
                        put_t(v, L.t[((size_t)z * BT + v % BT) * L.rank + r_lo + v / BT]);
                    __builtin_amdgcn_wave_barrier();
                }
            };

            u32x4 va[kUnroll], vb[kUnroll];
            issue(0, va);
            for (int k = 0; k < nblk; k += 2) {
                issue(k + 1, vb);
                if (k == 0 && pub == n) RS_STAMP(13);      // (first segment) two blocks of loads are on their way
                hook(k);
                fma(k, va);
                if (k == 0 && pub == n) RS_STAMP(3);       // (first segment) the first block of rows has been consumed
                if (k + 1 >= nblk) break;
                issue(k + 2, va);
                hook(k + 1);
                fma(k + 1, vb);
            }
        }
        __builtin_amdgcn_wave_barrier();
    } while (!last);

    RS_STAMP(6);
    RS_STAMP_SET(15, pub + nu);
    if (publish && lane == 0 && rho < (d_in >> 3)) L.act_seg[(size_t)z * (d_in >> 3) + rho] = pub;   // (ranges past d_in / 8 are empty)

    // ---- the wave's rows -> one sum per column: over the row groups inside the wave, then over the waves
#pragma unroll
    for (int d = LPR; d < 64; d <<= 1)
#pragma unroll
        for (int b = 0; b < BT; ++b)
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[b][k] += __shfl_xor(acc[b][k], d, 64);
    if (lane < LPR) {
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            float4 *dst = reinterpret_cast<float4 *>(s_red + (w * BT + b) * W + lane * 8);
            dst[0] = float4{acc[b][0], acc[b][1], acc[b][2], acc[b][3]};
            dst[1] = float4{acc[b][4], acc[b][5], acc[b][6], acc[b][7]};
        }
    }
    __syncthreads();
    RS_STAMP(7);
    const bool split_k = n_splits > 1;
    for (int t = tid; t < BT * W; t += (int)blockDim.x) {
        const int b = t / W, col = t % W, o = tile * W + col;
        float s = 0.f;
        for (int i = 0; i < nw; ++i) s += s_red[(i * BT + b) * W + col];
        if (b < nb && o < d_out) {
            const size_t at = (size_t)(b0 + b) * d_out + o;
            // one workgroup per strip: this IS Y_s + Y_r (Sec. 3.4); round once and store
            if (!split_k) store_out(a.Y, at, s + bias_at(L, o), L.out_dtype);
            else __hip_atomic_fetch_add(L.yacc + at, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    RS_STAMP(8);
    if (!split_k) {
        RS_STAMP_FLUSH(0, wg, w);
        return;
    }

    // ---- channel splits: arrive at the strip; the last of its `splits` workgroups swaps the sums out of yacc
    //      (which re-zeroes them for the next call), rounds once and stores
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);               // my own adds have been performed
    __syncthreads();
    int *tile_ctr = L.sync + kSyncTile + z * tiles + tile;
    if (tid == 0) {
        const int arrived = __hip_atomic_fetch_add(tile_ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (arrived == n_splits - 1) __hip_atomic_store(tile_ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_misc[0] = arrived;
    }
    __syncthreads();
    RS_STAMP(9);
    if (s_misc[0] != n_splits - 1) {
        RS_STAMP_FLUSH(0, wg, w);
        return;
    }
    for (int t = tid; t < BT * W; t += (int)blockDim.x) {
        const int b = t / W, col = t % W, o = tile * W + col;
        if (b < nb && o < d_out) {
            const size_t at = (size_t)(b0 + b) * d_out + o;
            const float v = __hip_atomic_exchange(L.yacc + at, 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            store_out(a.Y, at, v + bias_at(L, o), L.out_dtype);
        }
    }
    RS_STAMP(10);
    RS_STAMP_FLUSH(2, wg, w);
}

// Eight tokens of accumulators plus two batches of loads need the whole register file: 4 waves per workgroup.
// One token: at most 128 registers, so that two 8-wave workgroups fit a compute unit.
template <int DT, int BT, int LPR, bool FUSED>
__global__ __launch_bounds__(BT >= 8 ? 256 : 512, BT == 1 ? 4 : 1) void k_rsparse_strip(const StripGroupArgs ga)
{
    extern __shared__ __align__(16) unsigned char smem[];
    strip_body<DT, BT, LPR, FUSED>(ga, smem);
}

int strip_batch_tile(int batch) { return batch <= 1 ? 1 : batch <= 2 ? 2 : batch <= 4 ? 4 : 8; }

}  // namespace

int strip_waves(int batch) { return strip_batch_tile(batch) >= 8 ? 4 : 8; }

// List entries per wave (a multiple of the block size) that fit the 64 KiB of LDS of a workgroup; 0 = this launch
// shape does not fit.  Room for one 512-channel chunk, the wave's rows of U_r^T and the padding of the last block
// is the minimum.
int strip_list_cap(int d_in, int rank, int splits, int waves, int bt, int strip_w)
{
    const int R = splits * waves, blk = kUnroll * (64 / (strip_w / 8));
    const int nu_cap = rank > 0 ? (rank + R - 1) / R : 0;
    const long long fixed = (long long)waves * bt * strip_w * 4 + 64;            // cross-wave sums + flags
    const long long per_wave = (60 * 1024 - fixed) / waves - 16;
    long long entries = per_wave / (2 + 4 * bt);
    // no point in more than the wave's whole range plus its rows of U_r^T plus the padding of the last block
    const long long range = (((long long)(d_in / 8 + R - 1) / R) * 8 + 63) / 64 * 64;      // in whole pieces of 64
    const long long all = (range + nu_cap + blk + blk - 1) / blk * blk;
    entries -= entries % blk;
    entries = std::min(entries, all);
    if (entries < 64 + nu_cap + blk) return 0;             // one piece of 64 channels must fit
    return (int)entries;
}

size_t strip_lds_bytes(int waves, int bt, int strip_w, int cap)
{
    return (size_t)waves * strip_wave_bytes(cap, bt) + (size_t)waves * bt * strip_w * 4 + 64;
}

bool strip_width_ok(int w) { return w == 32 || w == 64 || w == 128 || w == 256 || w == 512; }

#define RS_STRIP_BT(BTV, ...)                             \
    switch (BTV) {                                        \
    case 1: { constexpr int BT = 1; __VA_ARGS__; } break; \
    case 2: { constexpr int BT = 2; __VA_ARGS__; } break; \
    case 4: { constexpr int BT = 4; __VA_ARGS__; } break; \
    default: { constexpr int BT = 8; __VA_ARGS__; } break; \
    }
#define RS_STRIP_W(WV, ...)                                  \
    switch (WV) {                                            \
    case 32: { constexpr int LPR = 4; __VA_ARGS__; } break;   \
    case 64: { constexpr int LPR = 8; __VA_ARGS__; } break;   \
    case 128: { constexpr int LPR = 16; __VA_ARGS__; } break; \
    case 256: { constexpr int LPR = 32; __VA_ARGS__; } break; \
    default: { constexpr int LPR = 64; __VA_ARGS__; } break;  \
    }

hipError_t launch_strip(const LayerView *L, const Launch *cfg, int n, const void *X, int batch, void *const *Y,
                        bool fused, bool dense, int cus, hipStream_t stream)
{
    if (n < 1 || n > kMaxGroupLayers || batch < 1) return hipErrorInvalidValue;
    const int bt = strip_batch_tile(batch);
    const int nz = (batch + bt - 1) / bt;
    const int waves = strip_waves(batch);
    StripGroupArgs ga{};
    ga.n = n;
    size_t lds = 0;
    int total = 0;
    for (int i = 0; i < n; ++i) {
        if (L[i].d_in != L[0].d_in || L[i].dtype != L[0].dtype || L[i].strip_w != L[0].strip_w) return hipErrorInvalidValue;
        if (!L[i].Ms || !strip_width_ok(L[i].strip_w) || !Y[i] || cfg[i].splits < 1) return hipErrorInvalidValue;
        const int rank = dense ? 0 : L[i].rank;
        if (fused && rank > 0 && (!L[i].t_tag || !L[i].sync || L[i].t_slots < nz * bt)) return hipErrorInvalidValue;
        if (cfg[i].splits > 1 && (!L[i].yacc || !L[i].sync || nz > kSyncMaxZ)) return hipErrorInvalidValue;
        StripArgs &a = ga.job[i];
        a.L = L[i]; a.X = (const uint16_t *)X; a.Y = Y[i]; a.batch = batch;
        a.tiles = (L[i].d_out + L[i].strip_w - 1) / L[i].strip_w;
        a.splits = cfg[i].splits;
        a.cap = strip_list_cap(L[i].d_in, rank, a.splits, waves, bt, L[i].strip_w);
        if (a.cap <= 0) return hipErrorInvalidValue;
        a.dense = dense ? 1 : 0;
        // stage 1: lowrank_rows rows per workgroup, waves / lowrank_rows waves per row
        a.lr_rows = cfg[i].lowrank_rows;
        a.lr_wgs = (fused && rank > 0) ? (rank + cfg[i].lowrank_rows - 1) / cfg[i].lowrank_rows : 0;
        if (a.lr_wgs > 0 && (cfg[i].lowrank_rows < 1 || cfg[i].lowrank_rows > waves || waves % cfg[i].lowrank_rows)) return hipErrorInvalidValue;
        a.lr_chunk = std::min(L[i].d_in, (24576 / bt) & ~7);
        a.wait_polls = cfg[i].wait_polls > 0 ? cfg[i].wait_polls : kWaitLimitPolls;
        a.skip_stage1 = cfg[i].skip_stage1;
        a.gen_readers = nz * (a.lr_wgs + a.tiles * a.splits) * waves;
        total += a.lr_wgs + a.tiles * a.splits;
        ga.wg_end[i] = total;
        lds = std::max(lds, strip_lds_bytes(waves, bt, L[i].strip_w, a.cap));
        if (a.lr_wgs > 0) lds = std::max(lds, (size_t)bt * a.lr_chunk * 2 + 32 + (size_t)waves * bt * 4);
    }
    for (int i = n; i < kMaxGroupLayers; ++i) ga.wg_end[i] = total;
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    // Where the stage-1 workgroups sit.  When every workgroup of the launch is resident at once (two 8-wave
    // workgroups of the one-token kernel per compute unit, one otherwise), they go to the END of each layer's range:
    // the strip workgroups' small reads of the token then reach memory ahead of stage 1's rows, and those rows
    // stream while the strip workgroups are still compacting -- a time in which the memory system is otherwise
    // idle.  A launch that needs more than one round of workgroups keeps them at the front, so that they are
    // dispatched before any workgroup that will wait for t.
    const int resident = cus * (bt == 1 ? 2 : 1);
    const int lr_last = (long long)total * nz <= resident ? 1 : 0;
    for (int i = 0; i < n; ++i) ga.job[i].lr_last = lr_last;
    dim3 grid(total, 1, nz), block(kWave * waves);
#define RS_S(DT)                                                                                             \
    RS_STRIP_BT(bt, RS_STRIP_W(L[0].strip_w, {                                                                \
        if (fused) hipLaunchKernelGGL((k_rsparse_strip<DT, BT, LPR, true>), grid, block, lds, stream, ga);   \
        else hipLaunchKernelGGL((k_rsparse_strip<DT, BT, LPR, false>), grid, block, lds, stream, ga);        \
    }))
    if (L[0].dtype == F16) { RS_S(F16) } else { RS_S(BF16) }
#undef RS_S
    return hipGetLastError();
}

}  // namespace rsparse
