// Host-callable launchers of the libapms kernels.  Each queues work on `stream`
// and returns hipGetLastError() of its launches; none synchronises.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace apms {

// Workgroup shape: kThreads threads, each owning ROWS 128-bit rows (4 floats) of a tile, so a tile is
// kThreads * 4 * ROWS consecutive elements of one chunk.  Rows per kernel were chosen by measurement
// on MI355X (short-lived workgroups with few bytes in flight each stream best).
constexpr int kThreads = 256;
constexpr int kCompressRows = 4;
constexpr int kServerRows = 4;
constexpr int kApplyRows = 1;
constexpr int kFinalizeRows = 1;

constexpr int tile_elems(int rows) { return kThreads * 4 * rows; }
constexpr int kCompressTile = tile_elems(kCompressRows);
constexpr int kServerTile = tile_elems(kServerRows);
constexpr int kApplyTile = tile_elems(kApplyRows);
constexpr int kFinalizeTile = tile_elems(kFinalizeRows);

// The one-pass worker kernel: one workgroup of kOnePassThreads threads holds a whole chunk of up to
// kOnePassMaxTiles compress tiles (65536 elements) on chip.
constexpr int kOnePassThreads = 1024;
constexpr int kOnePassMaxTiles = 16;
constexpr int64_t kOnePassMaxChunk = static_cast<int64_t>(kOnePassMaxTiles) * kCompressTile;
constexpr int32_t kOnePassLdsBytes = (kOnePassMaxTiles / (kOnePassThreads / kThreads) / 2) * kCompressRows * kOnePassThreads * 16;

// Most workers the server kernel takes: their scales of one chunk are staged in LDS (16 KB).
constexpr int kServerMaxWorkers = 4096;

// Element type of the gradient input (values match APMS_GRAD_* of the C ABI, 0 = binary32).
constexpr int kGradF32 = 0;
constexpr int kGradF16 = 1;
constexpr int kGradBF16 = 2;

// Source of the momentum term in the worker kernel.
constexpr int kMomRead = 0;    // read m
constexpr int kMomGather = 1;  // decode the pending server message, write it to m (if non-null), use it
constexpr int kMomNone = 2;    // no momentum term: u = g + delta (APGSqueeze variant, Section 5.3)

// Problem geometry shared by the chunked kernels.
struct Geometry {
    int64_t d;   // vector length
    int64_t L;   // chunk length (multiple of 32)
    int32_t n;   // workers
    int32_t C;   // chunks = d / L
};

// Dynamic LDS a launch asks for WITHOUT using it: LDS is the one resource that caps how many workgroups
// a CU holds at once without costing anything else, and on MI355X these streaming kernels reach their
// best HBM efficiency with few workgroups in flight per CU.
constexpr int32_t kMaxLdsPad = 128 * 1024;     // leaves room for the kernels' own LDS (up to 17 KB) in the CU's 160 KB

// Raise each kernel's dynamic-LDS limit so that pads above 64 KB can be launched (once per process).
hipError_t enable_large_lds_pads();

inline int64_t tiles_per_chunk(const Geometry& g, int tile) { return g.C ? (g.L + tile - 1) / tile : 0; }

// Worker step over all (worker, chunk) pairs: writes u into werr, sign words into packed, one binary64
// partial sum of u^2 per workgroup into partials [n*C][blocks_per_chunk]; a workgroup streams
// tiles_per_block consecutive tiles of kCompressTile elements.  prev_scales (nullable, [n*C]) marks werr
// as holding last step's u (deferred form).  `momentum` is kMomRead, kMomGather (gather_words [d/32] and
// gather_scales [C] describe the pending gather; m may be null: nothing is written) or kMomNone.  g holds grad_format elements (kGradF32 / kGradF16 / kGradBF16).
hipError_t launch_compress(const Geometry& geo, int32_t tiles_per_block, int32_t blocks_per_chunk, int momentum,
                           float* m, const void* g, int grad_format, float* werr, uint32_t* packed,
                           double* partials, const float* prev_scales, const uint32_t* gather_words,
                           const float* gather_scales, float beta, float one_minus_beta, int32_t lds_pad,
                           hipStream_t stream);

// The same worker step for chunks of at most kOnePassMaxChunk elements, with the finished error delta' = u - C[u]
// in werr and the scales in scales_out (and pending_out, nullable) when the kernel ends: no partials, no
// second pass.  The scales have the bits launch_compress (one tile per workgroup) + launch_scales give.
hipError_t launch_compress_onepass(const Geometry& geo, int momentum, float* m, const void* g, int grad_format,
                                   float* werr, uint32_t* packed, float* scales_out, float* pending_out,
                                   const float* prev_scales, const uint32_t* gather_words,
                                   const float* gather_scales, float beta, float one_minus_beta, hipStream_t stream);

// Reduce partials [pairs][blocks_per_chunk] in fixed order, scale = fl32(sqrt(S / L));
// writes scales_out[pair] and pending_out[pair] (either may be null).
hipError_t launch_scales(int64_t pairs, int32_t blocks_per_chunk, int64_t L, const double* partials,
                         float* scales_out, float* pending_out, hipStream_t stream);

// err[p][j] <- err[p][j] - (err >= 0 ? +s_p : -s_p) for pairs p = slice*C + chunk,
// slices = n (worker errors) or 1 (server error).
hipError_t launch_finalize(const Geometry& geo, int32_t slices, float* err, const float* scales,
                           int32_t lds_pad, hipStream_t stream);

// Server step over all chunks (tiles of kServerTile elements).
hipError_t launch_server_reduce(const Geometry& geo, int32_t tiles_per_block, int32_t blocks_per_chunk,
                                const uint32_t* packed, const float* scales, float* serr, uint32_t* spacked,
                                double* partials, const float* prev_scales, float inv_n, int32_t lds_pad,
                                hipStream_t stream);

// Gather (write_m: decoded server message to all n slices of m) and/or model update (model_step).
// With write_m false the server scales are also saved to scales_copy [C] for a later gather.
hipError_t launch_apply(const Geometry& geo, const uint32_t* spacked, const float* sscales, const float* v,
                        float* x, float* m, float* scales_copy, bool write_m, bool model_step, float lr,
                        float eps, int32_t lds_pad, hipStream_t stream);

// APGSqueeze variant: m_i <- beta*m_i + (1-beta)*ghat for all n slices, model step with the new momentum.
hipError_t launch_apply_gradient(const Geometry& geo, const uint32_t* spacked, const float* sscales,
                                 const float* v, float* x, float* m, float lr, float beta, float one_minus_beta,
                                 float eps, int32_t lds_pad, hipStream_t stream);

// Adam warm-up step on the averaged gradient (g in grad_format).
hipError_t launch_warmup(int64_t d, int32_t n, float* x, float* m, float* v, const void* g, int grad_format, float lr,
                         float beta1, float one_minus_beta1, float beta2, float one_minus_beta2, float bc1,
                         float bc2, float eps, float inv_n, int32_t lds_pad, hipStream_t stream);

// m[i] <- m[0] for i >= 1; werr, serr <- 0.
hipError_t launch_freeze(int64_t d, int32_t n, float* m, float* werr, float* serr, hipStream_t stream);

}  // namespace apms
