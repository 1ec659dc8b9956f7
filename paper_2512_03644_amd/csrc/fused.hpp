// Launch wrapper of the fused optimizer-step + snapshot kernels (fused.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "layout.hpp"

namespace ffsnap {

// Scalars shared by every element, derived on the host in double and rounded once to fp32.
struct AdamConsts {
    float decay, b1, omb1, b2, omb2, step_size, bc2s, eps;
};

struct FusedConsts {
    AdamConsts adam;
    uint32_t x32, x16;  // x^32, x^16 mod P
    uint32_t z16[6];    // x^(128 * 2^l): lane merge for 16-byte-per-lane rows
    uint32_t z8[6];     // x^(64 * 2^l):  lane merge for 8-byte-per-lane rows
};

void fill_fused_crc_consts(FusedConsts& c);

// tab[4][256]: byte tables of multiplication by x^(8*row_bytes).
void build_tab(uint32_t* tab, uint64_t row_bytes);

// Enqueues prepare (crcs = 0, zero tail), the tile kernel and finish (crcs ^= affine).
// tiles/grads/tabs: device tables (tabs = tables for 1024-byte rows, then for 512-byte rows).
hipError_t launch_fused(const WorkTile* tiles, uint32_t n_tiles, const uint64_t* grads,
                        const uint32_t* tabs, void* chunks, uint32_t* crcs, uint64_t n_chunks,
                        uint64_t payload, uint64_t buffer_bytes, uint32_t affine,
                        const FusedConsts& consts, hipStream_t stream);

}  // namespace ffsnap
