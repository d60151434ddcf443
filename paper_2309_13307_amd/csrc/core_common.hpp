// Constants shared by the kernels of the CORE hot path (gfx950).
#pragma once

namespace core {

constexpr int kThreads = 256;     // threads per block in every kernel
constexpr int kTile = 256;        // coordinates of G staged in LDS per step (64 Philox blocks)
constexpr int kPbarTile = 1024;   // pbar values staged in LDS per step

}  // namespace core
