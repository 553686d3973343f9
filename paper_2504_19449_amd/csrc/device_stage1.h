// Device code shared by the vector-path kernel files: the register scan used for compaction, token loads and
// keep-masks, the hand-off constants of the one-launch kernels, and stage 1 of the low-rank part.
#pragma once
#include "device_common.h"
#include "kernels.h"

namespace rsparse {

// Phase time stamps, only in builds with -DRSPARSE_STAMPS=1 (python -m paper_2504_19449_amd.build --stamps): every wave of
// the strip kernel's launches writes one record of kStampWords 64-bit words -- {kind | workgroup << 8 | wave << 40,
// stamps of the 100 MHz wall clock at its phase boundaries (words 1..14), rows streamed (word 15)} -- into a caller's buffer
// (rsparse_debug_stamps).  Product builds compile none of it.
constexpr int kStampWords = 16;
#if RSPARSE_STAMPS
extern __device__ unsigned long long *g_stamp_buf;
extern __device__ int g_stamp_cap;
#define RS_STAMP_DECL unsigned long long rs_tt[kStampWords] = {}
#define RS_STAMP(i) rs_tt[i] = (unsigned long long)wall_clock64()
#define RS_STAMP_SET(i, v) rs_tt[i] = (unsigned long long)(v)
#define RS_STAMP_FLUSH(kind, wg, w)                                                                      \
    do {                                                                                                 \
        const int rs_id = (int)((blockIdx.z * gridDim.x + blockIdx.x) * (blockDim.x >> 6)) + (w);        \
        if (g_stamp_buf && (threadIdx.x & 63) == 0 && rs_id < g_stamp_cap) {                             \
            rs_tt[0] = (unsigned long long)(kind) | ((unsigned long long)(wg) << 8) | ((unsigned long long)(w) << 40); \
            for (int rs_i = 0; rs_i < kStampWords; ++rs_i) g_stamp_buf[(size_t)rs_id * kStampWords + rs_i] = rs_tt[rs_i]; \
        }                                                                                                \
    } while (0)
#else
#define RS_STAMP_DECL
#define RS_STAMP(i)
#define RS_STAMP_SET(i, v)
#define RS_STAMP_FLUSH(kind, wg, w)
#endif

namespace {

// Inclusive prefix sum of `v` over the 64 lanes of a wave (all lanes must be active), with data-parallel
// primitives: three shifted adds inside groups of four lanes, two masked row shifts that complete each row
// of 16, then the row totals are broadcast down (lane 15 into rows 1 and 3, lane 31 into rows 2 and 3).
// Lanes without a source, and lanes masked off, add zero.  Seven register-to-register steps; the same scan
// through LDS-routed shuffles measured 0.3-0.4 us per call on the path to the first weight load.
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    constexpr int kRowShr = 0x110, kRowBcast15 = 0x142, kRowBcast31 = 0x143;
    int x = v;
    x += __builtin_amdgcn_update_dpp(0, v, kRowShr + 1, 0xf, 0xf, false);
    x += __builtin_amdgcn_update_dpp(0, v, kRowShr + 2, 0xf, 0xf, false);
    x += __builtin_amdgcn_update_dpp(0, v, kRowShr + 3, 0xf, 0xf, false);
    x += __builtin_amdgcn_update_dpp(0, x, kRowShr + 4, 0xf, 0xe, false);
    x += __builtin_amdgcn_update_dpp(0, x, kRowShr + 8, 0xf, 0xc, false);
    x += __builtin_amdgcn_update_dpp(0, x, kRowBcast15, 0xa, 0xf, false);
    x += __builtin_amdgcn_update_dpp(0, x, kRowBcast31, 0xc, 0xf, false);
    return x;
}

// Channels [c, c+8) of the nb tokens of one batch tile, in two steps so that callers can put the
// loads of several channel groups in flight before the first compare.
template <int BT>
__device__ __forceinline__ void load_raw8(const uint16_t *X, int b0, int nb, int d_in, int c, u32x4 (&raw)[BT])
{
#pragma unroll
    for (int b = 0; b < BT; ++b)
        raw[b] = b < nb ? *reinterpret_cast<const u32x4 *>(X + (size_t)(b0 + b) * d_in + c) : u32x4{0, 0, 0, 0};
}

// The rules of the tokens of one batch tile (wave-uniform).
template <int BT>
struct TileRules {
    KeepRule r[BT];
    bool sgn;
    bool exact;          // false: plain thresholds on the magnitude (keep_threshold applies); true: the general form
    bool per_token;      // the rules differ from token to token (fixed-count activation)
};
// EXT = false: the launch is known (on the host) to use nothing but a plain threshold on the magnitude; the
// general forms then drop out at compile time.
template <int BT, bool EXT = true>
__device__ __forceinline__ void load_rules(const LayerView &L, int b0, int nb, TileRules<BT> &t)
{
    if (EXT) {
        t.sgn = L.keep_signed != 0;
        t.per_token = L.rules != nullptr;
        t.exact = t.per_token || t.sgn;
#pragma unroll
        for (int b = 0; b < BT; ++b) t.r[b] = rule_of(L, b0 + (b < nb ? b : 0));
    } else {
        t.sgn = t.per_token = t.exact = false;
#pragma unroll
        for (int b = 0; b < BT; ++b) t.r[b] = KeepRule{L.tau_ge, __builtin_nanf(""), -1, 0};
    }
}

// Per-token keep masks (bit e = channel c+e kept) of loaded channels.  With union_all
// (batch_mask_mode 1) every token's mask becomes the union over the WHOLE batch.  Returns the union
// over the tile's tokens.
template <int DT, int BT>
__device__ __forceinline__ uint32_t masks_of8(const LayerView &L, const uint16_t *X, int batch, int b0, int nb, int d_in, int c,
                                              const TileRules<BT> &rules, bool union_all, const u32x4 (&raw)[BT],
                                              uint32_t (&m)[BT])
{
    uint32_t u = 0;
    // the threshold form is the common one and sits on every workgroup's path to its first weight load (this code runs
    // once per launch, from a cold instruction cache): it keeps its own short loop; the fixed-count form is out of line
    if (__builtin_expect(!rules.exact, 1)) {
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            m[b] = 0;
            if (b < nb) {
                float xv[8];
                unpack8<DT>(raw[b], xv);
#pragma unroll
                for (int e = 0; e < 8; ++e) m[b] |= (uint32_t)keep_threshold(xv[e], rules.r[b]) << e;
            }
            u |= m[b];
        }
    } else {
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            m[b] = 0;
            if (b < nb) {
                float xv[8];
                unpack8<DT>(raw[b], xv);
#pragma unroll
                for (int e = 0; e < 8; ++e) m[b] |= (uint32_t)keep(xv[e], c + e, rules.r[b], rules.sgn) << e;
            }
            u |= m[b];
        }
    }
    if (union_all) {
        for (int bb = 0; bb < batch; ++bb) {
            if (bb >= b0 && bb < b0 + nb) continue;
            const KeepRule rr = rules.per_token ? rule_of(L, bb) : rules.r[0];
            u32x4 r2 = *reinterpret_cast<const u32x4 *>(X + (size_t)bb * d_in + c);
            float f[8];
            unpack8<DT>(r2, f);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                u |= (uint32_t)(rules.exact ? keep(f[e], c + e, rr, rules.sgn) : keep_threshold(f[e], rr)) << e;
        }
#pragma unroll
        for (int b = 0; b < BT; ++b) m[b] = (b < nb) ? u : 0u;
    }
    return u;
}

// Channel groups (of 8 channels) a thread keeps in flight while it reads the token(s).  The code that turns a
// group into keep-bits is unrolled once per group and runs once per launch, straight from a cold
// instruction cache: 3 groups (24 channels per thread and trip, 12288 channels per trip of 512 lanes) measured
// faster than 8 (14.8 vs 15.0 us per linear on the benchmark), 2 and 4 in between.
template <int BT>
struct TokenBatch { static constexpr int kGroups = BT >= 8 ? 1 : (BT == 4 ? 2 : 3); };

// t_pub entries hold this pattern until the stage-1 workgroups have written them.  No computed
// value has it: NaNs made by the ALU are canonical, and NaNs widened from 16-bit inputs have zero
// low bits; the producer maps it to the canonical NaN anyway.
constexpr uint32_t kNotReady = 0xffffffffu;
// How lowrank_rows hands t over: plain stores for a following launch, or -- for the one-launch column-tile kernel,
// which reads t while the launch runs -- entries that hold kNotReady until written (reset at the end of the launch).
constexpr int kPubPlain = 0, kPubNotReady = 1;
// Bound on re-reads of an entry that is not ready.  The producers are workgroups with lower
// indices (dispatched before the caller), so the wait ends; the bound only turns an impossible
// schedule into an error flag instead of a hang.
constexpr long long kWaitLimitTicks = 50000000;      // 0.5 s of the 100 MHz wall clock
constexpr int kWaitLimitPolls = 1 << 20;

// Keep a wave-uniform kernel argument in scalar registers from here on.  Left alone, the compiler re-reads
// kernel arguments at their uses -- a scalar-cache round trip and a wait each time, e.g. in front of every
// single load of the token (six dependent waits before the first token load became three; the scalar cache
// hits are cheap, so this measured neutral on the benchmark).
__device__ __forceinline__ int pin(int v) { __asm__ volatile("" : "+s"(v)); return v; }
__device__ __forceinline__ float pin(float v) { __asm__ volatile("" : "+s"(v)); return v; }
template <typename T>
__device__ __forceinline__ const T *pin(const T *p)
{
    uintptr_t u = reinterpret_cast<uintptr_t>(p);
    __asm__ volatile("" : "+s"(u));
    // back through a global-memory pointer type, so that loads stay global loads (not generic ones)
    typedef const T __attribute__((address_space(1))) *global_ptr;
    return (const T *)reinterpret_cast<global_ptr>(u);
}

// Balanced share [lo, hi) of n items for part p of `parts`: the first n % parts shares hold one item more.
// 32-bit arithmetic on wave-uniform values -- a 64-bit division is some 200 emulated instructions here,
// and it sat on every workgroup's path to its first weight load.
__device__ __forceinline__ void balanced_share(int n, int parts, int p, int &lo, int &hi)
{
    const unsigned un = (unsigned)uniform(n), up = (unsigned)uniform(parts), pp = (unsigned)uniform(p);
    const unsigned base = un / up, rem = un - base * up;
    lo = (int)(pp * base + min(pp, rem));
    hi = lo + (int)base + (pp < rem ? 1 : 0);
}

// Tagged hand-off of t (strip kernel).  Entries are {generation, fp32 bits}; a launch's generation G is the value of
// sync[kSyncGen] while the launch runs.  Every wave that reads G reports so with one store-and-forget atomic, after
// its read has returned; the poller waits until all `readers` waves of the launch have reported (they all start:
// they wait for nothing but stage 1, which waits for nothing), clears the counts and bumps the generation.  The next
// launch therefore sees G + 1 in every wave, and entries tagged G or older never match it.  No wave can read the
// generation after the bump, since the bump waits for its report.
__device__ __forceinline__ void generation_was_read(int *sync, uint32_t gen, int wave_id)
{
    // the read has returned once its value can be consumed: the empty asm consumes it, and nothing after it is
    // issued before
    __asm__ volatile("s_waitcnt vmcnt(0)" : "+v"(gen) : : "memory");
    if ((threadIdx.x & 63) == 0)
        __hip_atomic_fetch_add(sync + kSyncStarted + (wave_id & (kSyncStartedN - 1)), 1, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void close_generation(int *sync, int readers)
{
    const int lane = threadIdx.x & 63;
    const long long t0 = wall_clock64();
    bool ok = false;
    while (!ok) {
        int v = 0;
#pragma unroll
        for (int k = 0; k < kSyncStartedN / 64; ++k)
            v += __hip_atomic_load(sync + kSyncStarted + k * 64 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
        ok = v == readers;
        if (!ok) {
            if (wall_clock64() - t0 > kWaitLimitTicks) break;
            __builtin_amdgcn_s_sleep(16);
        }
    }
#pragma unroll
    for (int k = 0; k < kSyncStartedN / 64; ++k)
        __hip_atomic_store(sync + kSyncStarted + k * 64 + lane, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (lane == 0) {
        if (!ok) __hip_atomic_fetch_or(sync + kSyncError, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(sync + kSyncGen, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---------------------------------------------------------------------------------------------
// Stage 1 of the low-rank part (Sec. 3.4): t_i = sum_c (S_r V_r^T)[i, c] * (x - sigma_t(x))_c.
// A workgroup stages the masked token(s) in LDS (kept channels zeroed); each of its waves then dots
// whole rows of S_r V_r^T against them, eight 16-byte loads in flight per lane.  A row is complete
// inside one wave, so t needs no cross-workgroup sum, no atomics and no zeroing.
// t is stored [batch tile][token][rank].  At most kRowsPerWave rows per wave (host-enforced).
// ---------------------------------------------------------------------------------------------
constexpr int kRowsPerWave = 4;

template <int DT, int BT, int PUB, typename Args, bool EXT = true>
__device__ __forceinline__ void lowrank_rows(const Args &a, unsigned char *smem, int wg, int z)
{
    // loads per batch and lane, batches in flight: two batches of six for one token; more tokens keep more of the
    // register file for the token values, and a second batch then spills
    constexpr int LU = BT == 1 ? 6 : 8, kRowBatches = BT == 1 ? 2 : 1;
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63, w = tid >> 6, nw = nthr >> 6;
    const LayerView &L = a.L;
    const int d_in = L.d_in, r = L.rank;
    const int b0 = z * BT;
    const int nb = min(BT, a.batch - b0);
    const bool union_all = L.batch_mask_mode == 1;
    TileRules<BT> rules;
    load_rules<BT, EXT>(L, b0, nb, rules);
    uint16_t *s_xm = reinterpret_cast<uint16_t *>(smem);                           // [BT][chunk]
    const int row_lo = wg * a.lr_rows, row_hi = min(r, row_lo + a.lr_rows);

    float part[kRowsPerWave][BT];
#pragma unroll
    for (int sl = 0; sl < kRowsPerWave; ++sl)
#pragma unroll
        for (int b = 0; b < BT; ++b) part[sl][b] = 0.f;

    for (int c0 = 0; c0 < d_in; c0 += a.lr_chunk) {
        const int len = min(a.lr_chunk, d_in - c0);
        const int nq = len / 8;
        if (c0 > 0) __syncthreads();
        constexpr int PB = TokenBatch<BT>::kGroups;
        for (int q0 = tid; q0 < nq; q0 += nthr * PB) {
            u32x4 raw[PB][BT];
#pragma unroll
            for (int p = 0; p < PB; ++p)
                if (q0 + p * nthr < nq) load_raw8<BT>(a.X, b0, nb, d_in, c0 + (q0 + p * nthr) * 8, raw[p]);
#pragma unroll
            for (int p = 0; p < PB; ++p) {
                const int q = q0 + p * nthr;
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
#pragma unroll
        for (int sl = 0; sl < kRowsPerWave; ++sl) {
            const int i = row_lo + w + sl * nw;
            if (i < row_hi) {
                const uint16_t *row = L.SVt + (size_t)i * d_in + c0;
                if constexpr (kRowBatches == 1) {
                    for (int q0 = lane; q0 < nq; q0 += 64 * LU) {
                        u32x4 v[LU];
#pragma unroll
                        for (int u = 0; u < LU; ++u) {
                            const int q = q0 + u * 64;
                            v[u] = (q < nq) ? ldg16<true>(row + q * 8) : u32x4{0, 0, 0, 0};       // streamed once
                        }
#pragma unroll
                        for (int u = 0; u < LU; ++u) {
                            const int q = q0 + u * 64;
                            if (q < nq) {
                                float f[8];
                                unpack8<DT>(v[u], f);
#pragma unroll
                                for (int b = 0; b < BT; ++b) {
                                    float xf[8];
                                    unpack8<DT>(*reinterpret_cast<const u32x4 *>(s_xm + (size_t)b * a.lr_chunk + q * 8), xf);
#pragma unroll
                                    for (int e = 0; e < 8; ++e) part[sl][b] = __builtin_fmaf(f[e], xf[e], part[sl][b]);
                                }
                            }
                        }
                    }
                } else {
                // kRowBatches batches of LU loads in flight per lane; unconditional loads (positions past the row's
                // end re-read its last piece and are dropped) so that the compiler counts the outstanding ones
                // exactly -- with one batch at a time a wave needed one dependent round trip per 8 KiB of its row
                // (seven for a 28672-channel down projection) through a saturated memory system
                u32x4 v[kRowBatches][LU];
                const int q_last = nq - 1;
                constexpr int kStep = 64 * LU;
                auto request = [&](u32x4 (&dst)[LU], int q0) {
#pragma unroll
                    for (int u = 0; u < LU; ++u) dst[u] = ldg16<true>(row + min(q0 + u * 64, q_last) * 8);      // streamed once
                };
                int q0 = lane;
#pragma unroll
                for (int j = 0; j < kRowBatches; ++j)
                    if (j * kStep < nq) request(v[j], q0 + j * kStep);
                bool more = nq > 0;                      // wave-uniform
                while (more) {
#pragma unroll
                    for (int j = 0; j < kRowBatches; ++j) {
                        if (more) {
#pragma unroll
                            for (int u = 0; u < LU; ++u) {
                                const int q = q0 + u * 64;
                                if (q < nq) {
                                    float f[8];
                                    unpack8<DT>(v[j][u], f);
#pragma unroll
                                    for (int b = 0; b < BT; ++b) {
                                        float xf[8];
                                        unpack8<DT>(*reinterpret_cast<const u32x4 *>(s_xm + (size_t)b * a.lr_chunk + q * 8), xf);
#pragma unroll
                                        for (int e = 0; e < 8; ++e) part[sl][b] = __builtin_fmaf(f[e], xf[e], part[sl][b]);
                                    }
                                }
                            }
                            const int qn = q0 + kRowBatches * kStep;
                            if (qn - lane < nq) request(v[j], qn);
                            q0 += kStep;
                            more = q0 - lane < nq;
                        }
                    }
                }
                }
            }
        }
    }
#pragma unroll
    for (int sl = 0; sl < kRowsPerWave; ++sl) {
        const int i = row_lo + w + sl * nw;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            const float v = wave_sum(part[sl][b]);
            if (lane == 0 && i < row_hi) {
                const size_t at = ((size_t)z * BT + b) * r + i;
                if (PUB == kPubNotReady) {
                    if (a.skip_stage1) continue;
                    uint32_t bits = as_u(v);
                    if (bits == kNotReady) bits = 0x7fc00000u;
                    __hip_atomic_store(L.t_pub + at, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    L.t[at] = v;
                }
            }
        }
    }
}

}  // namespace
}  // namespace rsparse
