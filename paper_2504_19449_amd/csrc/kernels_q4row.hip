// Dense baseline for 4-bit weights (R-Sparse, Sec. 4.4 runs the method on GPTQ weights): Y = X W~^T with
// W~[o][c] = s[o][g] (q[o][c] - z[o][g]), g = c / group, as a row-dot GEMV over ROW-major codes -- the form a dense
// 4-bit decoder kernel would use, and the baseline the channel-major R-Sparse kernel has to beat (the channel-major
// kernel with every channel kept is the other dense form the library has).  One wave per output row: a lane takes 16
// bytes = 32 consecutive codes, which lie inside one quantisation group (groups are powers of two >= 32), accumulates
// sum q x over them and folds  s (sum q x - z sum x)  with the group's scale and zero point; sum x per 32 channels is
// formed once per workgroup while the token is staged in LDS.
#include "kernels.h"
#include "device_common.h"

namespace rsparse {
namespace {

struct Q4RowArgs {
    const uint8_t *Q;        // [d_out][d_in / 2]: byte j of a row = code of channel 2j (low nibble), 2j + 1 (high nibble)
    const uint16_t *S;       // [d_out][d_in >> qshift] group scales, 16-bit of dtype
    const uint8_t *Z;        // [d_out][d_in >> qshift] group zero points
    const uint16_t *X;
    void *Y;
    int d_in, d_out, batch, qshift, out_dtype;
};

template <int DT, int BT>
__global__ __launch_bounds__(256) void k_q4_dense_rowdot(const Q4RowArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int d_in = a.d_in, d_out = a.d_out;
    const int b0 = blockIdx.z * BT;
    const int nb = min(BT, a.batch - b0);
    const int n32 = d_in / 32;                                      // 32-channel pieces of a row
    uint16_t *s_x = reinterpret_cast<uint16_t *>(smem);             // [BT][d_in]
    float *s_sum = reinterpret_cast<float *>(smem + (size_t)BT * d_in * 2);   // [BT][n32] sum of x over each piece
    for (int p = tid; p < n32; p += 256)
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            float sum = 0.f;
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                u32x4 v = u32x4{0, 0, 0, 0};
                if (b < nb) v = *reinterpret_cast<const u32x4 *>(a.X + (size_t)(b0 + b) * d_in + p * 32 + h * 8);
                *reinterpret_cast<u32x4 *>(s_x + (size_t)b * d_in + p * 32 + h * 8) = v;
                float f[8];
                unpack8<DT>(v, f);
#pragma unroll
                for (int e = 0; e < 8; ++e) sum += f[e];
            }
            s_sum[b * n32 + p] = sum;
        }
    __syncthreads();
    const int G = d_in >> a.qshift;
    for (int o = blockIdx.x * 4 + w; o < d_out; o += gridDim.x * 4) {
        const uint8_t *row = a.Q + (size_t)o * (d_in / 2);
        float acc[BT];
#pragma unroll
        for (int b = 0; b < BT; ++b) acc[b] = 0.f;
#pragma unroll 4
        for (int p = lane; p < n32; p += 64) {
            const u32x4 qv = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row + p * 16));
            const int g = (p * 32) >> a.qshift;
            const float sc = widen16<DT>(a.S[(size_t)o * G + g]);
            const float zp = (float)a.Z[(size_t)o * G + g];
            float dq[BT];
#pragma unroll
            for (int b = 0; b < BT; ++b) dq[b] = 0.f;
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                // word h holds channels 8h .. 8h + 7 of the piece, nibble k = channel 8h + k
                const uint32_t lo = qv[h] & 0x0f0f0f0fu, hi = (qv[h] >> 4) & 0x0f0f0f0fu;
                float c[8];
                c[0] = (float)(lo & 0xffu);          c[1] = (float)(hi & 0xffu);
                c[2] = (float)((lo >> 8) & 0xffu);   c[3] = (float)((hi >> 8) & 0xffu);
                c[4] = (float)((lo >> 16) & 0xffu);  c[5] = (float)((hi >> 16) & 0xffu);
                c[6] = (float)(lo >> 24);            c[7] = (float)(hi >> 24);
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    float xf[8];
                    unpack8<DT>(*reinterpret_cast<const u32x4 *>(s_x + (size_t)b * d_in + p * 32 + h * 8), xf);
#pragma unroll
                    for (int e = 0; e < 8; ++e) dq[b] = __builtin_fmaf(c[e], xf[e], dq[b]);
                }
            }
#pragma unroll
            for (int b = 0; b < BT; ++b) acc[b] = __builtin_fmaf(sc, dq[b] - zp * s_sum[b * n32 + p], acc[b]);
        }
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            const float v = wave_sum(acc[b]);
            if (lane == 0 && b < nb) store_out(a.Y, (size_t)(b0 + b) * d_out + o, v, a.out_dtype);
        }
    }
}

}  // namespace

bool q4_rowdot_supported(int d_in, int batch)
{
    const int bt = batch <= 1 ? 1 : batch <= 2 ? 2 : 4;
    return (d_in % 32) == 0 && (size_t)bt * d_in * 2 + (size_t)bt * (d_in / 32) * 4 <= 64 * 1024;
}

hipError_t launch_q4_dense_rowdot(const uint8_t *Qrow, const uint16_t *Srow, const uint8_t *Zrow, int qshift, int dtype, int out_dtype,
                                  int d_in, int d_out, const void *X, int batch, void *Y, hipStream_t stream)
{
    if (!Qrow || !Srow || !Zrow || !X || !Y || batch < 1 || !q4_rowdot_supported(d_in, batch) || (1 << qshift) < 32)
        return hipErrorInvalidValue;
    const int bt = batch <= 1 ? 1 : batch <= 2 ? 2 : 4;
    const int nz = (batch + bt - 1) / bt;
    Q4RowArgs a{Qrow, Srow, Zrow, (const uint16_t *)X, Y, d_in, d_out, batch, qshift, out_dtype};
    const size_t lds = (size_t)bt * d_in * 2 + (size_t)bt * (d_in / 32) * 4;
    int wgs = (d_out + 3) / 4;
    if (wgs > 2048) wgs = 2048;
    dim3 grid(wgs, 1, nz), block(256);
#define RS_Q(DT)                                                                                         \
    switch (bt) {                                                                                        \
        case 1: hipLaunchKernelGGL((k_q4_dense_rowdot<DT, 1>), grid, block, lds, stream, a); break;      \
        case 2: hipLaunchKernelGGL((k_q4_dense_rowdot<DT, 2>), grid, block, lds, stream, a); break;      \
        default: hipLaunchKernelGGL((k_q4_dense_rowdot<DT, 4>), grid, block, lds, stream, a); break;     \
    }
    if (dtype == F16) { RS_Q(F16) } else { RS_Q(BF16) }
#undef RS_Q
    return hipGetLastError();
}

}  // namespace rsparse
