// Host-callable launchers of the top-k compressor kernels (Section 5.1, second bullet): keep the K
// elements of largest magnitude of every chunk, ties towards the lower index, under the same
// error-compensated worker / server / gather structure as the 1-bit path.
//
// Selection is exact and deterministic: a 3-level radix select on the 31 magnitude bits finds the K-th
// largest key T of a chunk; if more elements equal T than may be kept, the lower indices are (found from a
// short list of the elements next to T, or by a second radix select on the element index).  Kept elements
// are then emitted in index order.
//
// Passes over the dense buffer: the one that forms u (worker) or ubar (server).  It works on a guess of the
// threshold (the previous call's, less a margin of 0.2 to 6 % that follows how far the threshold moves):
// every element at or above that floor is counted in the level-0 histogram and copied to the tile's slots
// (1.1 to 1.5 % of a tile when K is 1 % of a chunk); the rest is neither counted nor copied.  Where the guess proves too high (always in a context's
// first call) one more pass builds the whole histogram and another re-fills the slots from the bin then
// known.  Key levels 1 and 2, the tie rule, the per-tile counts and the emission work on the slots alone.
// A chunk with a tile that has more such elements than slots (constant or heavily tied data, or a K far
// beyond what the slots were sized for) takes full passes over the buffer instead: slower, same result.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "apms_launch.h"

namespace apms {

constexpr int kTopkBins = 2048;        // histogram bins per (slice, chunk) pair: 11 bits per radix level
constexpr int kTopkStateWords = 16;    // per-pair selection state, see topk.hip
constexpr int kTopkTile = 4096;        // elements per tile of the split / emit / server / gather kernels
constexpr int kTopkMinSlots = 64;      // slots per tile: a power of two in this range, see topk_slots_for
constexpr int kTopkMaxSlots = 512;
constexpr int kTopkNearCap = 1024;     // entries of a pair's near list, see topk_near_kernel

// Slots per tile for keeping K of L elements per chunk: room for three times the tile's expected share of
// the kept elements (those above the threshold's level-0 bin plus the bin's own, typically under twice the
// share) and a margin for small shares.
inline int32_t topk_slots_for(int64_t K, int64_t L) {
    const int64_t want = 3 * ((K * kTopkTile + L - 1) / L) + 64;
    int32_t slots = kTopkMinSlots;
    while (slots < want && slots < kTopkMaxSlots) slots *= 2;
    return slots;
}

// Device scratch of the selection, owned by the context; pairs = n * C, tiles = ceil(L / kTopkTile):
//   hist        [pairs][kTopkBins] u32
//   state       [pairs][kTopkStateWords] u32
//   tile_counts [pairs][tiles] u32       kept elements per tile, then their exclusive scan; the server and
//                                        gather kernels first use it for the tile offsets of their input lists
//   tile_split  [pairs][tiles] u32       elements of the tile at or above the level-0 bin of the threshold
//   slots       [pairs][tiles][slots_per_tile] uint2   those elements: (tile-local index, value bits)
//   guess       [pairs + C] u32          the floor of the first pass (the previous call's threshold key less a
//                                        margin): the worker call's n * C entries, then the server call's C;
//                                        0xFFFFFFFF in a new context and whenever the slots are re-allocated
//   last_T      [pairs + C] u32          that threshold key itself (the margin follows how far it moves), same layout
//   near        [pairs][kTopkNearCap] uint2   the slot entries that share the top 22 key bits of the pair's threshold:
//                                        (chunk-local index, key), in no particular order
//   gather_offsets [C][tiles] u32        tile offsets of the server's list while its gather is pending on m
//   keep        [pairs + C] uint2        {T, idxT} of the last call per pair, for an error buffer left in deferred
//                                        form (APMS_DEFER_ERRORS): worker pairs, then the server's chunks
struct TopkScratch {
    uint32_t* hist;
    uint32_t* state;
    uint32_t* guess;
    uint32_t* last_T;
    uint2* keep;
    uint2* near;
    uint32_t* gather_offsets;
    uint32_t* tile_counts;
    uint32_t* tile_split;
    uint2* slots;
    int32_t slots_per_tile;
};

// The server's list of the previous step while its gather is pending on m: [C][K] (index, value) pairs, with
// their tile offsets in TopkScratch.gather_offsets (left by launch_topk_apply with write_m = false).
struct TopkGather {
    const uint32_t* idx;
    const float* val;
    int64_t K;
};

// Worker: u = beta*m + (1-beta)*g + delta for all (worker, chunk) pairs, written into werr, then the K
// largest-magnitude elements of every chunk go to idx/val [n][C][K] (chunk-local indices, ascending) and
// their positions in werr are zeroed, which leaves werr = u - C[u].
// werr_pending: werr holds the previous call's compensated vector with the kept positions still in (deferred
// form; scratch.keep says which they are).  defer: leave it in that form again instead of zeroing them.
// gather: null = m is read; else the momentum is that list decoded (zero elsewhere) and is written to m
// unless m is null.
hipError_t launch_topk_compress(const Geometry& geo, int64_t K, float* m, const float* g, float* werr, uint32_t* idx,
                                float* val, float beta, float one_minus_beta, bool werr_pending, bool defer,
                                const TopkGather* gather, const TopkScratch& scratch, hipStream_t stream);

// Server: ubar = (sum over workers of the decoded lists, worker order) * inv_n + serr, written into serr,
// then top-K per chunk to sidx/sval [C][K], kept positions of serr zeroed.
hipError_t launch_topk_server_reduce(const Geometry& geo, int64_t K, const uint32_t* idx, const float* val,
                                     float* serr, uint32_t* sidx, float* sval, float inv_n, bool serr_pending,
                                     bool defer, const TopkScratch& scratch, hipStream_t stream);

// Zero the kept positions of an error buffer in deferred form (worker errors [n][d], or the server's [d]).
hipError_t launch_topk_finalize(const Geometry& geo, bool server, float* err, const TopkScratch& scratch,
                                hipStream_t stream);

// Gather + model update: every slice of m becomes the decoded server list (zero elsewhere);
// x <- x - lr * m / (sqrt(v) + eps).  write_m false: the model step alone, m is not touched and the list's tile
// offsets are left in scratch.gather_offsets for the worker call that carries the gather out; model_step false
// (with write_m): the gather alone.
hipError_t launch_topk_apply(const Geometry& geo, int64_t K, const uint32_t* sidx, const float* sval,
                             const float* v, float* x, float* m, float lr, float eps, bool write_m, bool model_step,
                             const TopkScratch& scratch, hipStream_t stream);

}  // namespace apms
