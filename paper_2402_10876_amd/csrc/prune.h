// Internal: device-side one-shot pruner (prune.hip).
#pragma once
#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace twg {

// Bytes of device scratch prune_device needs for a K x N weight and tile width G.
size_t prune_workspace_bytes(int K, int N, int G);

// Enqueues the pruning kernels on `stream`: the n_cols_pruned lowest-scoring columns go, the
// kept columns are cut into tiles of G, every tile keeps its rows_per_tile best rows;
// tvw: 2 of every 4 consecutive kept rows per column.  mask / tile_mask: K x N bytes
// (tile_mask may be null).  Arguments are validated by the caller.
hipError_t prune_device(const uint16_t* B, int K, int N, int ldb, int G, bool tvw, int n_cols_pruned,
                        int rows_per_tile, uint8_t* mask, uint8_t* tile_mask, void* workspace,
                        hipStream_t stream);

// The entry point that allocates nothing keeps its scratch in a device array of this size
// inside the library (one per GPU, for the life of the process).
constexpr size_t PRUNE_STATIC_SCRATCH_BYTES = 8u << 20;

// Device address of the current device's copy of that array (looked up once per device).
hipError_t prune_static_scratch(void** out);

}  // namespace twg
