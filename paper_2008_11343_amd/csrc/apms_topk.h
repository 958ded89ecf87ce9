// Host-callable launchers of the top-k compressor kernels (Section 5.1, second bullet): keep the K
// elements of largest magnitude of every chunk, ties towards the lower index, under the same
// error-compensated worker / server / gather structure as the 1-bit path.
//
// Selection is exact and deterministic: a 3-level radix select on the 31 magnitude bits finds the K-th
// largest key T of a chunk; if more elements equal T than may be kept, a second 3-level radix select on the
// element index finds the last tie to keep.  Kept elements are then emitted in index order.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "apms_launch.h"

namespace apms {

constexpr int kTopkBins = 2048;        // histogram bins per (slice, chunk) pair: 11 bits per radix level
constexpr int kTopkStateWords = 8;     // per-pair selection state, see topk.hip
constexpr int kTopkTile = 4096;        // elements per tile of the count / emit / server / gather kernels

// Device scratch of the selection, owned by the context: hist [pairs][kTopkBins] u32,
// state [pairs][kTopkStateWords] u32, tile_counts [pairs][ceil(L / kTopkTile)] u32.
struct TopkScratch {
    uint32_t* hist;
    uint32_t* state;
    uint32_t* tile_counts;
};

// Worker: u = beta*m + (1-beta)*g + delta for all (worker, chunk) pairs, written into werr, then the K
// largest-magnitude elements of every chunk go to idx/val [n][C][K] (chunk-local indices, ascending) and
// their positions in werr are zeroed, which leaves werr = u - C[u].
hipError_t launch_topk_compress(const Geometry& geo, int64_t K, const float* m, const float* g, float* werr,
                                uint32_t* idx, float* val, float beta, float one_minus_beta,
                                const TopkScratch& scratch, hipStream_t stream);

// Server: ubar = (sum over workers of the decoded lists, worker order) * inv_n + serr, written into serr,
// then top-K per chunk to sidx/sval [C][K], kept positions of serr zeroed.
hipError_t launch_topk_server_reduce(const Geometry& geo, int64_t K, const uint32_t* idx, const float* val,
                                     float* serr, uint32_t* sidx, float* sval, float inv_n,
                                     const TopkScratch& scratch, hipStream_t stream);

// Gather + model update: every slice of m becomes the decoded server list (zero elsewhere);
// x <- x - lr * m / (sqrt(v) + eps).
hipError_t launch_topk_apply(const Geometry& geo, int64_t K, const uint32_t* sidx, const float* sval,
                             const float* v, float* x, float* m, float lr, float eps, hipStream_t stream);

}  // namespace apms
