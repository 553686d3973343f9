// The scratch of rsparse_linear_static: callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc) get the per-call scratch of the layer -- partial sums,
// arrival counters, the hand-off entries of t, the kept-channel lists -- out of one file-scope device array instead
// of buffers that a handle allocated.  Every call on a GPU shares that GPU's array (calls that overlap on one GPU
// race); it keeps the last call's contents, so each call starts with one fill launch that puts back what must start
// at zero.
#include "kernels.h"

#include <mutex>

namespace rsparse {
namespace {

constexpr size_t kAlign = 256;
constexpr size_t up(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }
// carve-up for the largest call (kStaticMax*): offsets in bytes
constexpr size_t kOffYacc = 0;
constexpr size_t kOffT = kOffYacc + up((size_t)kStaticMaxBatch * kStaticMaxDim * 4);
constexpr size_t kOffTpub = kOffT + up((size_t)kStaticMaxBatch * kStaticMaxRank * 4);
constexpr size_t kOffTtag = kOffTpub + up((size_t)kStaticMaxBatch * kStaticMaxRank * 4);
constexpr size_t kOffList = kOffTtag + up((size_t)kStaticMaxBatch * kStaticMaxRank * 8);
constexpr size_t kOffBits = kOffList + up((size_t)kStaticMaxDim * 4);
constexpr size_t kOffSeg = kOffBits + up((size_t)kStaticMaxDim * 4);
constexpr size_t kOffCount = kOffSeg + up((size_t)kStaticMaxDim / 8 * 4);
constexpr size_t kOffRules = kOffCount + up(16);
constexpr size_t kOffSync = kOffRules + up((size_t)kStaticMaxBatch * sizeof(KeepRule));
constexpr size_t kSyncWords = kSyncTile + (size_t)kSyncMaxZ * (kStaticMaxDim / 32);     // strips of 32 columns at most
constexpr size_t kStaticBytes = 2u << 20;
static_assert(kOffSync + up(kSyncWords * 4) <= kStaticBytes, "the carve-up must fit the array");

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// One address per device: each GPU holds its own copy of the array.
constexpr int kMaxDevices = 64;
unsigned char *g_ptr[kMaxDevices] = {};
std::mutex g_mu;

// What must start at zero (or at "not written") for one call: the accumulators of its outputs, every counter
// (the generation of the strip kernel's hand-off is kept, but never 0: fresh entries carry tag 0), the hand-off
// entries of both kernels, the list count.
__global__ void k_static_clear(float *yacc, size_t n_y, int *sync, size_t n_sync, uint32_t *t_pub, unsigned long long *t_tag,
                               size_t n_t, int32_t *act_count)
{
    const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = i0; i < n_y; i += stride) yacc[i] = 0.f;
    for (size_t i = i0; i < n_sync; i += stride) {
        if (i == (size_t)kSyncGen) {
            if (sync[i] == 0) sync[i] = 1;
        } else {
            sync[i] = 0;
        }
    }
    for (size_t i = i0; i < n_t; i += stride) {
        t_pub[i] = 0xffffffffu;
        t_tag[i] = 0ull;
    }
    if (i0 == 0) act_count[0] = 0;
}

}  // namespace

hipError_t static_scratch_for_call(int device, int d_out, int rank, int batch, hipStream_t stream, ScratchView *out)
{
    if (device < 0 || device >= kMaxDevices || !out || batch < 1 || batch > kStaticMaxBatch || d_out < 1 ||
        d_out > kStaticMaxDim || rank < 0 || rank > kStaticMaxRank)
        return hipErrorInvalidValue;
    unsigned char *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        if (!g_ptr[device]) {
            // set-up, once per device, with that device current: the array's name is a host-side stand-in, its
            // device address comes from the runtime
            void *p = nullptr;
            hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            g_ptr[device] = static_cast<unsigned char *>(p);
        }
        ptr = g_ptr[device];
    }
    ScratchView sp{};
    sp.yacc = reinterpret_cast<float *>(ptr + kOffYacc);
    sp.t = reinterpret_cast<float *>(ptr + kOffT);
    sp.t_pub = reinterpret_cast<uint32_t *>(ptr + kOffTpub);
    sp.t_tag = reinterpret_cast<unsigned long long *>(ptr + kOffTtag);
    sp.act_list = reinterpret_cast<int32_t *>(ptr + kOffList);
    sp.act_bits = reinterpret_cast<uint32_t *>(ptr + kOffBits);
    sp.act_seg = reinterpret_cast<int32_t *>(ptr + kOffSeg);
    sp.act_count = reinterpret_cast<int32_t *>(ptr + kOffCount);
    sp.rules = reinterpret_cast<KeepRule *>(ptr + kOffRules);
    sp.sync = reinterpret_cast<int *>(ptr + kOffSync);
    sp.t_slots = kStaticMaxBatch;
    sp.n_t = (size_t)kStaticMaxBatch * (size_t)(rank > 0 ? rank : 1);
    sp.n_y = (size_t)batch * d_out;
    sp.sync_n = kSyncWords;
    const size_t most = sp.n_y > sp.sync_n ? sp.n_y : sp.sync_n;
    unsigned blocks = (unsigned)((most + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(k_static_clear, dim3(blocks), dim3(256), 0, stream, sp.yacc, sp.n_y, sp.sync, sp.sync_n, sp.t_pub,
                       sp.t_tag, sp.n_t, sp.act_count);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    *out = sp;
    return hipSuccess;
}

}  // namespace rsparse
