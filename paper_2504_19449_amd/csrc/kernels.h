// Internal launch interface between the C-ABI host code (api.cpp) and the gfx950 kernels
// (kernels.hip).  Not installed; the public boundary is include/rsparse.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rsparse {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kTile = 512;       // output columns per wave: 64 lanes x one 16-byte load (8 x 16-bit)
constexpr int kScanThreads = 256;
constexpr int kMaxBT = 8;        // tokens held in registers per workgroup (batch tile)

// Device-side view of one prepared layer plus its per-call scratch.
struct LayerView {
    const uint16_t *M;      // [d_in + rank][d_out]: rows 0..d_in-1 = W column-major (row c = W[:, c]),
                            // rows d_in.. = U_r^T (row d_in + i = U_r[:, i])
    const uint16_t *SVt;    // [rank][d_in]  = S_r V_r^T
    const uint16_t *Wrow;   // [d_out][d_in] row-major copy, or nullptr
    float *t;               // [nz][rank][BT] stage-1 result, fp32
    float *yacc;            // [max_batch][d_out] fp32 accumulators; zero between calls
    uint32_t *tile_done;    // [nz][tiles] arrival counters; zero between calls
    int32_t *act_list;      // [nz][d_in] ascending kept channels of batch tile z (union over its tokens)
    uint32_t *act_bits;     // [nz][d_in] per list entry: bit b = token b of the tile keeps it
    int32_t *act_count;     // [nz]
    int d_in, d_out, rank;
    int dtype, out_dtype, cmp_mode, batch_mask_mode;
    float tau;
};

struct Launch {
    int splits;        // channel splits per column tile
    int waves;         // waves per workgroup (gather / dense axpy)
    int lowrank_rows;  // rows per workgroup (stage 1): 1, 2 or 4
    int nontemporal;
};

// Stage 1 of the low-rank part: t = (S_r V_r^T)(x - sigma_t(x)) for every token.
hipError_t launch_lowrank_t(const LayerView &L, const Launch &cfg, const void *X, int batch,
                            hipStream_t stream);
// Threshold + compaction + gather-GEMV over kept columns + U_r t + sum + store.
hipError_t launch_gather(const LayerView &L, const Launch &cfg, const void *X, int batch, void *Y,
                         hipStream_t stream);
// Dense baselines.
hipError_t launch_dense_axpy(const LayerView &L, const Launch &cfg, const void *X, int batch, void *Y,
                             hipStream_t stream);
hipError_t launch_dense_rowdot(const LayerView &L, const Launch &cfg, const void *X, int batch, void *Y,
                               hipStream_t stream);
// Zero `n` 32-bit words (a fill kernel, safe to record into a HIP graph).
hipError_t launch_zero(void *p, size_t n_words, hipStream_t stream);

size_t gather_lds_bytes(int d_in, int rank, int splits, int waves, int bt);
size_t lowrank_lds_bytes(int d_in, int bt);
bool rowdot_supported(int d_in, int batch);

}  // namespace rsparse
