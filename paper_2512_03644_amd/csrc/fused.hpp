// Launch wrapper of the fused optimizer-step + snapshot kernels (fused.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"
#include "layout.hpp"

namespace ffsnap {

// Scalars shared by every element, derived on the host in double and rounded once to fp32.
struct AdamConsts {
    float decay, b1, omb1, b2, omb2, step_size, bc2s, eps;
};

struct FusedConsts {
    AdamConsts adam;
    float inv_scale = 1.0f;            // fp16 variant: reciprocal of the loss scale
    uint64_t* n_nonfinite = nullptr;   // fp16 variant: device counter of inf/NaN gradients, or null
    uint32_t xcd_group = 0;            // XCD-aware order of the work tiles (see xcd_order.h)
    // Chained step: master, m and v are read from this snapshot buffer (at the segments' stream
    // offsets) instead of their tensors, and those tensors are not written.  Null: in-place step.
    const uint8_t* prev = nullptr;
};

// Device table of the fused kernels (kFusedTabWords entries): byte tables of multiplication by
// x^8192 (1 KiB rows) and by x^4096 (512 B rows), then the lane constants x^(128 * (63 - lane))
// and x^(64 * (63 - lane)).
constexpr int kFusedTabWords = 2048 + 128;
void build_fused_tabs(uint32_t* tab);

// Gradient pointers of up to kGradsPerLaunch consecutive parameter groups, handed to the kernel by
// value in its arguments (3 KiB).
constexpr uint32_t kGradsPerLaunch = 384;
struct GradPtrs {
    uint64_t p[kGradsPerLaunch];
};

// Enqueues prepare (crcs = affine, zero tail, counter = 0) and the tile kernels.
// tiles/tabs: device tables (tabs = tables for 1024-byte rows, then for 512-byte rows); tiles holds
// the parameter tiles first, sorted by parameter group, then the RAW tiles (a kernel of their own).
// grads: HOST array of n_params device pointers, read during the call only.  group_tile_begin:
// HOST array, entry k = index of the first parameter tile of group k * kGradsPerLaunch, one more
// entry = n_param_tiles.  f16: gradients and working weights are fp16 (else bf16).  bare: the
// step's traffic alone -- every parameter tile's loads and stores with no arithmetic and no CRC
// (16-bit weights := gradient bits, master, m, v unchanged); crcs, the RAW segments and the zero
// tail are not touched.
hipError_t launch_fused(bool f16, const WorkTile* tiles, uint32_t n_param_tiles,
                        uint32_t n_raw_tiles, const void* const* grads, uint32_t n_params,
                        const uint32_t* group_tile_begin, const uint32_t* tabs, void* chunks,
                        uint32_t* crcs, uint64_t n_chunks, uint64_t payload, uint64_t buffer_bytes,
                        uint32_t affine, const FusedConsts& consts, bool bare, hipStream_t stream);

}  // namespace ffsnap
