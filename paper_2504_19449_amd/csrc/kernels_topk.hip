// Fixed-count activation for the R-Sparse linear layer: instead of the threshold t(s) of Sec. 3.4, which gives the
// sparsity s in expectation over tokens, keep exactly k channels of largest magnitude of every token.  This kernel
// turns a token into the KeepRule (kernels.h) that the layer's kernels then apply channel by channel:
//   eq  = the k-th largest magnitude,  ge = the next fp32 above it,
//   cut = the channel of the last of the values equal to eq that is still among the k (lower channels first).
// Magnitudes of fp16 / bf16 values order like their low 15 bits, so the k-th largest is found exactly by a two-level
// radix select on those bits (256 bins on bits 14..7, then 128 bins on bits 6..0 inside the bin that holds it); a third
// pass counts the equal values in channel order.  NaN is never kept.  One workgroup of 1024 lanes per token; the token
// (at most 128 KiB) is read three times from L2.
#include "kernels.h"
#include "device_common.h"
#include "device_stage1.h"

namespace rsparse {
namespace {

constexpr int kTopkThreads = 1024;

// Position (from the top) at which the running count of `hist[nbins-1], hist[nbins-2], ...` first reaches `want`
// (want >= 1, total >= want): returns the bin; `above` = how many lie in higher bins.  Wave 0 only, all 64 lanes.
template <int NBINS>
__device__ __forceinline__ int bin_from_top(const int *hist, int want, int &above)
{
    constexpr int PER = NBINS / 64;
    const int lane = threadIdx.x & 63;
    int v = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) v += hist[NBINS - 1 - (lane * PER + i)];
    const int inc = wave_inclusive_scan(v);
    const bool mine = inc - v < want && want <= inc;
    int bin = 0, ab = 0;
    if (mine) {
        int run = inc - v;
        for (int i = 0; i < PER; ++i) {
            const int b = NBINS - 1 - (lane * PER + i);
            if (run + hist[b] >= want) { bin = b; ab = run; break; }
            run += hist[b];
        }
    }
    const unsigned long long who = __ballot(mine);
    const int src = (int)__builtin_ctzll(who);
    above = __shfl(ab, src, 64);
    return __shfl(bin, src, 64);
}

template <int DT>
__global__ __launch_bounds__(kTopkThreads) void k_topk_rules(const uint16_t *X, int d_in, int k, KeepRule *rules)
{
    __shared__ int s_h1[256], s_h2[128], s_w[kTopkThreads / 64], s_pick[4];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint16_t *x = X + (size_t)blockIdx.x * d_in;
    constexpr uint32_t kNanAbove = DT == F16 ? 0x7c00u : 0x7f80u;      // magnitude patterns above this are NaN
    if (tid < 256) s_h1[tid] = 0;
    if (tid < 128) s_h2[tid] = 0;
    __syncthreads();
    for (int c = tid; c < d_in; c += kTopkThreads) {
        const uint32_t m = x[c] & 0x7fffu;
        if (m <= kNanAbove) atomicAdd(&s_h1[m >> 7], 1);
    }
    __syncthreads();
    if (w == 0) {
        int tot = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) tot += s_h1[lane * 4 + i];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) tot += __shfl_xor(tot, d, 64);
        int above = 0, bin = -1;
        if (k >= 1 && tot > k) bin = bin_from_top<256>(s_h1, k, above);     // else: everything (or nothing) is kept
        if (lane == 0) { s_pick[0] = bin; s_pick[1] = above; s_pick[2] = tot; }
    }
    __syncthreads();
    const int bin1 = s_pick[0], above1 = s_pick[1], total = s_pick[2];
    if (bin1 < 0) {
        if (tid == 0) {
            KeepRule r;
            r.eq = __builtin_nanf("");
            r.cut = -1;
            r.pad = 0;
            r.ge = k >= 1 ? 0.f : __builtin_nanf("");       // k >= non-NaN channels: all of them (|x| >= 0); k = 0: none
            (void)total;
            rules[blockIdx.x] = r;
        }
        return;
    }
    for (int c = tid; c < d_in; c += kTopkThreads) {
        const uint32_t m = x[c] & 0x7fffu;
        if (m <= kNanAbove && (int)(m >> 7) == bin1) atomicAdd(&s_h2[m & 127u], 1);
    }
    __syncthreads();
    if (w == 0) {
        int above2 = 0;
        const int bin2 = bin_from_top<128>(s_h2, k - above1, above2);
        if (lane == 0) { s_pick[0] = (bin1 << 7) | bin2; s_pick[1] = k - above1 - above2; }   // the pattern; how many of it to keep
    }
    __syncthreads();
    const uint32_t pat = (uint32_t)s_pick[0];
    const int need = s_pick[1];                              // >= 1 and <= the number of channels whose magnitude is pat
    // the need-th channel, in ascending order, whose magnitude pattern is pat: contiguous runs of channels per thread
    const int per = (d_in + kTopkThreads - 1) / kTopkThreads;
    const int c_lo = min(d_in, tid * per), c_hi = min(d_in, c_lo + per);
    int mine = 0;
    for (int c = c_lo; c < c_hi; ++c) mine += (x[c] & 0x7fffu) == pat;
    const int inc = wave_inclusive_scan(mine);
    if (lane == 63) s_w[w] = inc;
    __syncthreads();
    int before = inc - mine;
    for (int i = 0; i < w; ++i) before += s_w[i];
    if (before < need && need <= before + mine) {
        int run = before, cut = c_lo;
        for (int c = c_lo; c < c_hi; ++c) {
            if ((x[c] & 0x7fffu) == pat && ++run == need) { cut = c; break; }
        }
        KeepRule r;
        r.eq = widen16<DT>((uint16_t)pat);
        // the next fp32 above eq (eq >= 0); above +inf there is nothing
        r.ge = pat == kNanAbove ? __builtin_nanf("") : as_f(as_u(r.eq) + 1u);
        r.cut = cut;
        r.pad = 0;
        rules[blockIdx.x] = r;
    }
}

}  // namespace

hipError_t launch_topk_rules(const void *X, int dtype, int batch, int d_in, int k, KeepRule *rules, hipStream_t stream)
{
    if (!X || !rules || batch < 1 || d_in < 1 || k < 0) return hipErrorInvalidValue;
    if (dtype == F16) hipLaunchKernelGGL(k_topk_rules<F16>, dim3(batch), dim3(kTopkThreads), 0, stream, (const uint16_t *)X, d_in, k, rules);
    else hipLaunchKernelGGL(k_topk_rules<BF16>, dim3(batch), dim3(kTopkThreads), 0, stream, (const uint16_t *)X, d_in, k, rules);
    return hipGetLastError();
}

}  // namespace rsparse
