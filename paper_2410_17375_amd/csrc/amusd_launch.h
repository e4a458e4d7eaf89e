// Host-callable launchers of the kernels in amusd_kernels.hip.
#pragma once
#include "amusd_dev.h"

namespace amusd {

enum RelayoutKind {
    kNatural = 0,   // tile t, row r  <- source row 16t + r
    kRopePairs = 1, // per head: tile th, row r <- feature 8th + (r%8) + (r/8)*hd/2   (rotary partners share a tile)
    kGate = 2,      // tile t, rows 0-7  <- source row 8t + r
    kUp = 3         // tile t, rows 8-15 <- source row 8t + r - 8
};

// One-time per process: raises the dynamic-LDS limit of the stage kernels.
hipError_t configure_kernels();

// Re-lays a row-major [rows, K] matrix into matrix-core operand order at
// dst[(tile_offset + t) * (K/KB) + kb][lane].  n_tiles counts destination tiles.
hipError_t launch_relayout(int dtype, uint4* dst, const void* src, int K, int n_tiles, int tile_offset, int kind,
                           int hd, hipStream_t stream);

// Optional bracketing of one stage's launches with events (one pair per launch).
struct StageTimer {
    int stage = -1;
    hipEvent_t* begin = nullptr;   // [n_layers]
    hipEvent_t* end = nullptr;
    int used = 0;                  // pairs recorded by the last launch_pass
};

// Plain copy of n 16-byte words (profiler calibration).
hipError_t launch_copy(uint4* dst, const uint4* src, size_t n, hipStream_t stream);

// Writes n zeroed 16-byte words (a kernel: usable where a memset node is not).
hipError_t launch_fill_zero(uint4* dst, size_t n, hipStream_t stream);

// Enqueues n_kernels bare streaming kernels (256 workgroups, words_per_kernel 16-byte words each, regions of buf in
// rotation), each depending on the one before.  io: 512 floats, fold: 256 words (device scratch of the caller).
hipError_t launch_stream_chain(const uint4* buf, size_t buf_words, size_t words_per_kernel, int n_kernels, float* io,
                               unsigned* fold, hipStream_t stream);

// Enqueues one whole pass (all stages) on the stream.
hipError_t launch_pass(const DevModel& M, const DevLayer* layers_host, const PassArgs& P, int nwg, hipStream_t stream,
                       StageTimer* timer);

}  // namespace amusd
