// HIP kernels of libapms for gfx950: the compression stage of APMSqueeze
// (Algorithm 1 lines 3-12; supplement "Proof to the Updating Form") and the
// Adam warm-up step (Section 3.2).  All kernels are HBM-bandwidth bound:
// 128-bit coalesced streaming accesses, sign packing by an OR across 8-lane
// groups, binary64 norm partials reduced in a fixed order (no atomics).
//
// Built with -ffp-contract=off: every binary32 operation below rounds once, in
// the order written.  The only fused operation is the explicit binary64
// fma(u, u, acc), which equals mul-then-add because the product of two
// binary32 values is exact in binary64.

#include "apms_device.h"
#include "apms_launch.h"

namespace apms {

namespace {

// ------------------------------------------------------------------------
// Worker step (Algorithm 1 lines 6-7): u = beta*m + (1-beta)*g + delta, sign
// words, partial sums of u^2; u is parked in the error buffer.
// ------------------------------------------------------------------------

// If the error buffer holds last step's compensated vector u' (deferred form),
// the error is delta = u' - C[u'] = u' - (u' >= 0 ? +s' : -s').  With s' = 0 this
// is the identity, which is how a buffer that already holds delta is read.
__device__ __forceinline__ float read_error(float stored, float prev_scale) {
    return stored - signed_scale(stored >= 0.0f, prev_scale);
}

__device__ __forceinline__ f32x4 compensated(f32x4 vm, f32x4 vg, f32x4 ve, float beta, float omb,
                                             float prev_scale) {
    f32x4 u;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const float bm = beta * vm[c];
        const float bg = omb * vg[c];
        const float mi = bm + bg;                       // local momentum m_t^(i)
        u[c] = mi + read_error(ve[c], prev_scale);      // + delta^(i)
    }
    return u;
}

__device__ __forceinline__ void accumulate_squares(double (&acc)[4], f32x4 u) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const double w = static_cast<double>(u[c]);
        acc[c] = fma(w, w, acc[c]);
    }
}

// Where the momentum term of u comes from:
//   kMomRead    m is read.
//   kMomGather  a deferred gather is pending on m (Algorithm 1 line 10 not yet carried out): the momentum
//               of every worker is the decoded server message (gather_words, gather_scale); write it to m
//               (unless m is null: implicit-momentum mode) and use it directly instead of reading m back.
//   kMomNone    APGSqueeze variant (Section 5.3): the gradient itself is compensated, u = g + delta.
//
// kKeep: u is handed back in `keep` (zero where the tile has no row) instead of being stored into the error
// buffer: the one-pass kernel holds the whole chunk on chip and writes the finished error itself.
template <bool kFull, int MOM, int G, bool kKeep = false>
__device__ __forceinline__ void compress_tile(float* __restrict__ m, const void* __restrict__ g,
                                              float* __restrict__ e, uint32_t* __restrict__ packed,
                                              const uint32_t* __restrict__ gather_words, float gather_scale,
                                              int64_t vec_base, int64_t chunk_base, int64_t tile_off, int64_t L,
                                              int lane_off, int lane, int wave, float beta, float omb,
                                              float prev_scale, double (&acc)[4],
                                              f32x4 (*keep)[kCompressRows] = nullptr) {
    constexpr int ROWS = kCompressRows;
    const int64_t off0 = tile_off + lane_off;             // inside the chunk
    bool ok[ROWS];
    f32x4 vm[ROWS], vg[ROWS], ve[ROWS];
    uint32_t gw[ROWS];
    const int shift = 4 * (lane & 7);
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        ok[r] = kFull || (off0 + 32 * r < L);
        if (ok[r]) {
            const int64_t p = chunk_base + off0 + 32 * r;
            if (MOM == kMomGather)
                gw[r] = gather_words[(vec_base + off0 + 32 * r) >> 5];
            else if (MOM == kMomRead)
                vm[r] = load_stream(m + p);
            vg[r] = load_grad4<G>(g, p);
            ve[r] = load_stream(e + p);
        }
    }
    uint32_t words[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        uint32_t nib = 0u;
        if (ok[r]) {
            if (MOM == kMomGather) {
                const uint32_t gn = gw[r] >> shift;
#pragma unroll
                for (int c = 0; c < 4; ++c) vm[r][c] = signed_scale((gn >> c) & 1u, gather_scale);
                if (m) store_stream(m + chunk_base + off0 + 32 * r, vm[r]);
            }
            f32x4 u;
            if (MOM == kMomNone) {
#pragma unroll
                for (int c = 0; c < 4; ++c) u[c] = vg[r][c] + read_error(ve[r][c], prev_scale);
            } else {
                u = compensated(vm[r], vg[r], ve[r], beta, omb, prev_scale);
            }
            if constexpr (kKeep)
                (*keep)[r] = u;
            else
                store_stream(e + chunk_base + off0 + 32 * r, u);
            accumulate_squares(acc, u);
            nib = sign_nibble(u) << shift;
        } else if constexpr (kKeep) {
            (*keep)[r] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        }
        words[r] = or_across_group8(nib);                 // all 64 lanes take part
    }
    if ((lane & 7) == 0) {
        // first of the ROWS consecutive words this 8-lane group owns
        const int64_t w0 = (chunk_base + off0) >> 5;
        store_group_words<ROWS, kFull>(packed, w0, words, ok);
    }
}

template <int MOM, int G>
__global__ __launch_bounds__(kThreads) void compress_kernel(
    float* __restrict__ m, const void* __restrict__ g, float* __restrict__ e, uint32_t* __restrict__ packed,
    double* __restrict__ partials, const float* __restrict__ prev_scales,
    const uint32_t* __restrict__ gather_words, const float* __restrict__ gather_scales, int64_t d, int64_t L,
    int32_t C, int32_t tiles_per_chunk, int32_t tiles_per_block, int32_t blocks_per_chunk, float beta,
    float omb) {
    __shared__ double lds[kWaves];
    const int64_t blk = blockIdx.x;
    const int64_t pair = blk / blocks_per_chunk;          // worker * C + chunk
    const int32_t b = static_cast<int32_t>(blk - pair * blocks_per_chunk);
    const int64_t worker = pair / C;
    const int64_t chunk = pair - worker * C;
    const int64_t vec_base = chunk * L;                   // inside one [d] vector
    const int64_t chunk_base = worker * d + vec_base;     // inside [n][d]
    const float prev_scale = prev_scales ? prev_scales[pair] : 0.0f;
    const float gather_scale = (MOM == kMomGather) ? gather_scales[chunk] : 0.0f;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int lane_off = packing_lane_offset<kCompressRows>(wave, lane);
    const int32_t t0 = b * tiles_per_block;
    const int32_t t1 = min(t0 + tiles_per_block, tiles_per_chunk);
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int32_t t = t0; t < t1; ++t) {
        const int64_t tile_off = static_cast<int64_t>(t) * kCompressTile;
        if (tile_off + kCompressTile <= L)
            compress_tile<true, MOM, G>(m, g, e, packed, gather_words, gather_scale, vec_base, chunk_base,
                                         tile_off, L, lane_off, lane, wave, beta, omb, prev_scale, acc);
        else
            compress_tile<false, MOM, G>(m, g, e, packed, gather_words, gather_scale, vec_base, chunk_base,
                                          tile_off, L, lane_off, lane, wave, beta, omb, prev_scale, acc);
    }
    const double mine = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    const double total = block_sum_f64(mine, lds);
    if (threadIdx.x == 0) partials[blk] = total;
}

// ------------------------------------------------------------------------
// Scale of every chunk (Section 5.1): ||u||_2 / sqrt(L).
// ------------------------------------------------------------------------

__global__ __launch_bounds__(kThreads) void scales_kernel(const double* __restrict__ partials,
                                                          int32_t blocks_per_chunk, int64_t L,
                                                          float* __restrict__ scales_out,
                                                          float* __restrict__ pending_out) {
    __shared__ double lds[kWaves];
    const int64_t pair = blockIdx.x;
    const double* p = partials + pair * blocks_per_chunk;
    double mine = 0.0;
    for (int32_t j = threadIdx.x; j < blocks_per_chunk; j += kThreads) mine += p[j];
    const double S = block_sum_f64(mine, lds);
    if (threadIdx.x == 0) {
        const double mean_sq = S / static_cast<double>(L);
        const float s = static_cast<float>(sqrt(mean_sq));
        if (scales_out) scales_out[pair] = s;
        if (pending_out) pending_out[pair] = s;
    }
}

// ------------------------------------------------------------------------
// Worker step in ONE pass, for chunks that fit on chip (Algorithm 1 lines 6-7 with the error final when the
// kernel ends): one workgroup of kOnePassThreads threads per (worker, chunk) forms u for the whole chunk, keeps
// it (half in registers, half in LDS), reduces the squared norm, and writes delta' = u - C[u] without u
// ever going to memory: 16.125 B per worker element where the two-pass eager route moves 24.125.
//
// The workgroup works as kOnePassGroups groups of kThreads threads; a group takes tiles exactly as a workgroup
// of compress_kernel does (same lane layout, same per-thread sums, same wave tree, wave sums added in wave
// order), and the tile sums are then combined as scales_kernel combines them, so the scale has the bits of the
// two-pass route.
// ------------------------------------------------------------------------
constexpr int kOnePassGroups = kOnePassThreads / kThreads;
constexpr int kOnePassTilesPerGroup = kOnePassMaxTiles / kOnePassGroups;
constexpr int kOnePassInRegs = kOnePassTilesPerGroup / 2;       // tiles per group whose u stays in registers
static_assert(kOnePassMaxTiles <= kWaveSize, "the tile sums are combined by one wave");

__device__ __forceinline__ double wave_sum_f64(double v) {     // the tree of block_sum_f64
#pragma unroll
    for (int off = kWaveSize / 2; off > 0; off >>= 1) v += __shfl_down(v, off);
    return v;
}

template <int MOM, int G>
__global__ __launch_bounds__(kOnePassThreads) void compress_onepass_kernel(
    float* __restrict__ m, const void* __restrict__ g, float* __restrict__ e, uint32_t* __restrict__ packed,
    float* __restrict__ scales_out, float* __restrict__ pending_out, const float* __restrict__ prev_scales,
    const uint32_t* __restrict__ gather_words, const float* __restrict__ gather_scales, int64_t d, int64_t L,
    int32_t C, int32_t tiles_per_chunk, float beta, float omb) {
    constexpr int ROWS = kCompressRows;
    extern __shared__ __align__(16) unsigned char onepass_lds[];
    // u of the tiles that do not stay in registers: [tile slot][row][thread]
    f32x4* stash = reinterpret_cast<f32x4*>(onepass_lds);
    __shared__ double wave_sums[kOnePassMaxTiles][kWaves];
    __shared__ double tile_sums[kOnePassMaxTiles];
    __shared__ float chunk_scale;
    const int64_t pair = blockIdx.x;                      // worker * C + chunk
    const int64_t worker = pair / C;
    const int64_t chunk = pair - worker * C;
    const int64_t vec_base = chunk * L;
    const int64_t chunk_base = worker * d + vec_base;
    const float prev_scale = prev_scales ? prev_scales[pair] : 0.0f;
    const float gather_scale = (MOM == kMomGather) ? gather_scales[chunk] : 0.0f;
    const int group = threadIdx.x / kThreads;
    const int t = threadIdx.x - group * kThreads;          // thread inside the group
    const int lane = t & (kWaveSize - 1);
    const int wave = t >> 6;
    const int lane_off = packing_lane_offset<ROWS>(wave, lane);
    f32x4 in_regs[kOnePassInRegs][ROWS];
#pragma unroll
    for (int q = 0; q < kOnePassTilesPerGroup; ++q) {
        const int32_t tile = q * kOnePassGroups + group;
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        f32x4 keep[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) keep[r] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (tile < tiles_per_chunk) {                      // uniform inside a group: the shuffles in there are whole waves'
            const int64_t tile_off = static_cast<int64_t>(tile) * kCompressTile;
            if (tile_off + kCompressTile <= L)
                compress_tile<true, MOM, G, true>(m, g, e, packed, gather_words, gather_scale, vec_base, chunk_base,
                                                  tile_off, L, lane_off, lane, wave, beta, omb, prev_scale, acc, &keep);
            else
                compress_tile<false, MOM, G, true>(m, g, e, packed, gather_words, gather_scale, vec_base, chunk_base,
                                                   tile_off, L, lane_off, lane, wave, beta, omb, prev_scale, acc, &keep);
        }
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            if (q < kOnePassInRegs)
                in_regs[q < kOnePassInRegs ? q : 0][r] = keep[r];
            else
                stash[((q - kOnePassInRegs) * ROWS + r) * kOnePassThreads + threadIdx.x] = keep[r];
        }
        const double mine = (acc[0] + acc[1]) + (acc[2] + acc[3]);
        const double wsum = wave_sum_f64(mine);
        if (lane == 0) wave_sums[tile][wave] = wsum;
    }
    __syncthreads();
    if (threadIdx.x < kOnePassMaxTiles) {                  // as thread 0 of a compress_kernel workgroup does
        double total = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) total += wave_sums[threadIdx.x][w];
        tile_sums[threadIdx.x] = static_cast<int32_t>(threadIdx.x) < tiles_per_chunk ? total : 0.0;
    }
    __syncthreads();
    if (threadIdx.x < kWaveSize) {                         // as scales_kernel does with one partial per thread
        const double mine = threadIdx.x < kOnePassMaxTiles ? tile_sums[threadIdx.x] : 0.0;
        const double S = wave_sum_f64(mine);
        if (threadIdx.x == 0) {
            const double mean_sq = S / static_cast<double>(L);
            const float s = static_cast<float>(sqrt(mean_sq));
            chunk_scale = s;
            scales_out[pair] = s;
            if (pending_out) pending_out[pair] = s;
        }
    }
    __syncthreads();
    const float s = chunk_scale;
#pragma unroll
    for (int q = 0; q < kOnePassTilesPerGroup; ++q) {
        const int32_t tile = q * kOnePassGroups + group;
        if (tile >= tiles_per_chunk) continue;
        const int64_t off0 = static_cast<int64_t>(tile) * kCompressTile + lane_off;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            if (off0 + 32 * r >= L) continue;
            const f32x4 u = q < kOnePassInRegs ? in_regs[q < kOnePassInRegs ? q : 0][r]
                                               : stash[((q - kOnePassInRegs) * ROWS + r) * kOnePassThreads + threadIdx.x];
            f32x4 out;
#pragma unroll
            for (int c = 0; c < 4; ++c) out[c] = read_error(u[c], s);
            store_stream(e + chunk_base + off0 + 32 * r, out);
        }
    }
}

// ------------------------------------------------------------------------
// Eager error: delta' = u - C[u] in place (Section 3.1).
// ------------------------------------------------------------------------

__global__ __launch_bounds__(kThreads) void finalize_kernel(float* __restrict__ err,
                                                            const float* __restrict__ scales, int64_t d,
                                                            int64_t L, int32_t C, int32_t tiles_per_chunk) {
    constexpr int ROWS = kFinalizeRows;
    const int64_t blk = blockIdx.x;
    const int64_t pair = blk / tiles_per_chunk;           // slice * C + chunk
    const int64_t tile = blk - pair * tiles_per_chunk;
    const int64_t slice = pair / C;
    const int64_t chunk = pair - slice * C;
    const int64_t chunk_base = slice * d + chunk * L;
    const float s = scales[pair];
    const int64_t off0 = tile * kFinalizeTile + threadIdx.x * 4;      // plain layout
    f32x4 ve[ROWS];
    bool ok[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        ok[r] = off0 + r * (kThreads * 4) < L;
        if (ok[r]) ve[r] = load_stream(err + chunk_base + off0 + r * (kThreads * 4));
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        if (!ok[r]) continue;
        f32x4 out;
#pragma unroll
        for (int c = 0; c < 4; ++c) out[c] = read_error(ve[r][c], s);
        store_stream(err + chunk_base + off0 + r * (kThreads * 4), out);
    }
}

// ------------------------------------------------------------------------
// Server step (Algorithm 1 line 9): average the n decoded messages in worker
// order, add the server error, re-compress.
// ------------------------------------------------------------------------

// worker_scales[i] is worker i's scale of this chunk (staged in LDS by the kernel).
// kWide: the tile is full and its sign words are 16-byte aligned in EVERY worker's stream (chunk base and
// vector length both multiples of 128 elements), so a group's ROWS = 4 consecutive words are taken as one
// 128-bit load.
template <bool kFull, bool kWide>
__device__ __forceinline__ void server_tile(const uint32_t* __restrict__ packed,
                                            const float* __restrict__ worker_scales, float* __restrict__ serr,
                                            uint32_t* __restrict__ spacked, int64_t d, int64_t L, int32_t C,
                                            int32_t n, int64_t chunk, int64_t tile_off, int lane_off, int lane,
                                            int wave, float inv_n, float prev_scale, double (&acc)[4]) {
    constexpr int ROWS = kServerRows;
    const int64_t chunk_base = chunk * L;                 // inside one [d] vector
    const int64_t off0 = tile_off + lane_off;
    const int shift = 4 * (lane & 7);
    // element c of a row sits at bit shift + c of the row's sign word: this many places below bit 31
    uint32_t to_msb[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) to_msb[c] = 31u - static_cast<uint32_t>(shift + c);
    // first of this group's ROWS consecutive words, inside one worker's [d/32] words
    const int64_t w0 = (chunk_base + off0) >> 5;
    const int64_t words_per_worker = d >> 5;
    bool ok[ROWS];
    f32x4 ve[ROWS];
    f32x4 sum[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        ok[r] = kFull || (off0 + 32 * r < L);
        if (ok[r]) ve[r] = load_stream(serr + chunk_base + off0 + 32 * r);
        sum[r] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
    static_assert(!kWide || (kFull && ROWS == 4), "the wide load covers four full rows");
    uint32_t magnitude_bits = 0x7fffffffu;
    asm("" : "+v"(magnitude_bits));                         // pinned in a vector register for the inserts below
    // the ROWS sign words worker i holds for this lane's rows
    auto load_words = [&](int32_t i, uint32_t (&w)[ROWS]) {
        const uint32_t* wp = packed + i * words_per_worker + w0;
        if constexpr (kWide) {
            const u32x4 wq = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wp));
#pragma unroll
            for (int r = 0; r < ROWS; ++r) w[r] = wq[r & 3];
        } else {
#pragma unroll
            for (int r = 0; r < ROWS; ++r) w[r] = ok[r] ? wp[r] : 0u;
        }
    };
    // One worker's contribution to the running sums, in place.  Three VALU operations per decoded element:
    // shift the element's sign bit to the top, insert it into the scale as ITS sign (bit set = positive gives
    // -s), subtract: sum - (-s) = sum + s exactly.
    auto add_worker = [&](int32_t i, const uint32_t (&w)[ROWS]) {
        const float s = worker_scales[i];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                sum[r][c] = sum[r][c] - scale_signed_by_msb_bfi(magnitude_bits, s, w[r] << to_msb[c]);
        }
    };
    // worker order 0 .. n-1; the sign words of a group of workers are requested together
    constexpr int kGroup = 8;
    int32_t i = 0;
#pragma unroll 1
    for (; i + kGroup <= n; i += kGroup) {
        uint32_t w[kGroup][ROWS];
#pragma unroll
        for (int q = 0; q < kGroup; ++q) load_words(i + q, w[q]);
#pragma unroll
        for (int q = 0; q < kGroup; ++q) add_worker(i + q, w[q]);
    }
#pragma unroll 1
    for (; i < n; ++i) {
        uint32_t w[ROWS];
        load_words(i, w);
        add_worker(i, w);
    }
    uint32_t words[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        uint32_t nib = 0u;
        if (ok[r]) {
            f32x4 ubar;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float avg = sum[r][c] * inv_n;
                ubar[c] = avg + read_error(ve[r][c], prev_scale);
            }
            store_stream(serr + chunk_base + off0 + 32 * r, ubar);
            accumulate_squares(acc, ubar);
            nib = sign_nibble(ubar) << shift;
        }
        words[r] = or_across_group8(nib);
    }
    if ((lane & 7) == 0) store_group_words<ROWS, kFull>(spacked, w0, words, ok);
}

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 8))) void server_kernel(
    const uint32_t* __restrict__ packed, const float* __restrict__ scales, float* __restrict__ serr,
    uint32_t* __restrict__ spacked, double* __restrict__ partials, const float* __restrict__ prev_scales,
    int64_t d, int64_t L, int32_t C, int32_t n, int32_t tiles_per_chunk, int32_t tiles_per_block,
    int32_t blocks_per_chunk, float inv_n) {
    __shared__ double lds[kWaves];
    __shared__ float lds_scales[kServerMaxWorkers];
    const int64_t blk = blockIdx.x;
    const int64_t chunk = blk / blocks_per_chunk;
    const int32_t b = static_cast<int32_t>(blk - chunk * blocks_per_chunk);
    const float prev_scale = prev_scales ? prev_scales[chunk] : 0.0f;
    // the n scales of this chunk, one per worker (the launcher checked n <= kServerMaxWorkers)
    for (int32_t i = threadIdx.x; i < n; i += kThreads) lds_scales[i] = scales[static_cast<int64_t>(i) * C + chunk];
    __syncthreads();
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int lane_off = packing_lane_offset<kServerRows>(wave, lane);
    const int32_t t0 = b * tiles_per_block;
    const int32_t t1 = min(t0 + tiles_per_block, tiles_per_chunk);
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int32_t t = t0; t < t1; ++t) {
        const int64_t tile_off = static_cast<int64_t>(t) * kServerTile;
        if (tile_off + kServerTile <= L) {
            // tile offsets are multiples of 128 anyway; worker i's words start at i * d / 32
            if ((((chunk * L) | d) & 127) == 0)
                server_tile<true, kServerRows == 4>(packed, lds_scales, serr, spacked, d, L, C, n, chunk, tile_off,
                                                    lane_off, lane, wave, inv_n, prev_scale, acc);
            else
                server_tile<true, false>(packed, lds_scales, serr, spacked, d, L, C, n, chunk, tile_off, lane_off, lane,
                                         wave, inv_n, prev_scale, acc);
        } else {
            server_tile<false, false>(packed, lds_scales, serr, spacked, d, L, C, n, chunk, tile_off, lane_off, lane, wave,
                                      inv_n, prev_scale, acc);
        }
    }
    const double mine = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    const double total = block_sum_f64(mine, lds);
    if (threadIdx.x == 0) partials[blk] = total;
}

// ------------------------------------------------------------------------
// Gather + model update (Algorithm 1 lines 10-11).
// ------------------------------------------------------------------------

// One workgroup = one tile of ONE worker's momentum slice, slice-major, so the n slices are written as
// one long contiguous fill of m[n][d]; the workgroups of slice 0 also take the model step for their tile.
//   <kWriteM = true,  kModelStep = true >  eager apms_apply (grid: n slices)
//   <kWriteM = false, kModelStep = true >  apms_apply with the gather deferred (grid: 1 slice); also saves
//                                          the server scales for the kernel that will carry out the gather
//   <kWriteM = true,  kModelStep = false>  the gather alone (apms_finalize on m)
template <bool kWriteM, bool kModelStep>
__global__ __launch_bounds__(kThreads) void apply_kernel(const uint32_t* __restrict__ spacked,
                                                         const float* __restrict__ sscales,
                                                         const float* __restrict__ v, float* __restrict__ x,
                                                         float* __restrict__ m, float* __restrict__ scales_copy,
                                                         int64_t d, int64_t L, int64_t tiles_per_slice,
                                                         int32_t tiles_per_chunk, float lr, float eps) {
    constexpr int ROWS = kApplyRows;
    constexpr int kRowStride = kThreads * 4;              // plain layout
    const int64_t blk = blockIdx.x;
    const int64_t slice = blk / tiles_per_slice;
    const int64_t ct = blk - slice * tiles_per_slice;     // chunk * tiles_per_chunk + tile
    const int64_t chunk = ct / tiles_per_chunk;
    const int64_t tile = ct - chunk * tiles_per_chunk;
    const int64_t chunk_base = chunk * L;
    const float s = sscales[chunk];
    if (!kWriteM && tile == 0 && threadIdx.x == 0) scales_copy[chunk] = s;
    const int64_t off0 = tile * kApplyTile + threadIdx.x * 4;
    const int shift = 4 * (threadIdx.x & 7);
    const bool model_step = kModelStep && (slice == 0);
    float* __restrict__ mslice = m + slice * d;
    bool ok[ROWS];
    f32x4 vv[ROWS], vx[ROWS];
    uint32_t w[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        ok[r] = off0 + r * kRowStride < L;
        if (ok[r]) {
            const int64_t p = chunk_base + off0 + r * kRowStride;
            w[r] = spacked[p >> 5];
            if (model_step) {
                vv[r] = load_stream(v + p);
                vx[r] = load_stream(x + p);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        if (!ok[r]) continue;
        const int64_t p = chunk_base + off0 + r * kRowStride;
        const uint32_t nib = w[r] >> shift;
        f32x4 mom;
#pragma unroll
        for (int c = 0; c < 4; ++c) mom[c] = signed_scale((nib >> c) & 1u, s);   // decoded server message
        if (kWriteM) store_stream(mslice + p, mom);
        if (model_step) {
            f32x4 xn;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float root = sqrtf(vv[r][c]);
                const float denom = root + eps;
                const float ratio = mom[c] / denom;
                const float step = lr * ratio;
                xn[c] = vx[r][c] - step;
            }
            store_stream(x + p, xn);
        }
    }
}

// APGSqueeze variant (Section 5.3): the decoded server message is the averaged gradient ghat; every
// worker's momentum slice takes m <- beta*m + (1-beta)*ghat, and slice 0's workgroups take the model step
// with the new momentum.  Same slice-major tiling as apply_kernel.
__global__ __launch_bounds__(kThreads) void apply_gradient_kernel(const uint32_t* __restrict__ spacked,
                                                                  const float* __restrict__ sscales,
                                                                  const float* __restrict__ v,
                                                                  float* __restrict__ x, float* __restrict__ m,
                                                                  int64_t d, int64_t L, int64_t tiles_per_slice,
                                                                  int32_t tiles_per_chunk, float lr, float beta,
                                                                  float omb, float eps) {
    constexpr int ROWS = kApplyRows;
    constexpr int kRowStride = kThreads * 4;              // plain layout
    const int64_t blk = blockIdx.x;
    const int64_t slice = blk / tiles_per_slice;
    const int64_t ct = blk - slice * tiles_per_slice;
    const int64_t chunk = ct / tiles_per_chunk;
    const int64_t tile = ct - chunk * tiles_per_chunk;
    const int64_t chunk_base = chunk * L;
    const float s = sscales[chunk];
    const int64_t off0 = tile * kApplyTile + threadIdx.x * 4;
    const int shift = 4 * (threadIdx.x & 7);
    const bool model_step = (slice == 0);
    float* __restrict__ mslice = m + slice * d;
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        if (off0 + r * kRowStride >= L) continue;
        const int64_t p = chunk_base + off0 + r * kRowStride;
        const uint32_t nib = spacked[p >> 5] >> shift;
        const f32x4 mo = load_stream(mslice + p);
        f32x4 vv, vx;
        if (model_step) {
            vv = load_stream(v + p);
            vx = load_stream(x + p);
        }
        f32x4 mn;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float ghat = signed_scale((nib >> c) & 1u, s);
            const float keep = beta * mo[c];
            const float inc = omb * ghat;
            mn[c] = keep + inc;
        }
        store_stream(mslice + p, mn);
        if (model_step) {
            f32x4 xn;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float root = sqrtf(vv[c]);
                const float denom = root + eps;
                const float ratio = mn[c] / denom;
                const float step = lr * ratio;
                xn[c] = vx[c] - step;
            }
            store_stream(x + p, xn);
        }
    }
}

// ------------------------------------------------------------------------
// Warm-up: original Adam on the averaged gradient (Section 3.2).
// ------------------------------------------------------------------------

template <int G>
__global__ __launch_bounds__(kThreads) void warmup_kernel(float* __restrict__ x, float* __restrict__ m,
                                                          float* __restrict__ v, const void* __restrict__ g,
                                                          int64_t d, int32_t n, float lr, float beta1,
                                                          float omb1, float beta2, float omb2, float bc1,
                                                          float bc2, float eps, float inv_n) {
    // one 128-bit quad per thread, one short-lived workgroup per 1024 elements
    const int64_t q = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (q >= (d >> 2)) return;
    const int64_t p = q << 2;
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 8
    for (int32_t i = 0; i < n; ++i) {
        const f32x4 gi = load_grad4<G>(g, static_cast<int64_t>(i) * d + p);
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = acc[c] + gi[c];      // worker order 0..n-1
    }
    const f32x4 mo = load_stream(m + p), vo = load_stream(v + p), xo = load_stream(x + p);
    f32x4 mn, vn, xn;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const float gbar = acc[c] * inv_n;
        const float m_keep = beta1 * mo[c];
        const float m_inc = omb1 * gbar;
        mn[c] = m_keep + m_inc;
        const float gsq = gbar * gbar;
        const float v_keep = beta2 * vo[c];
        const float v_inc = omb2 * gsq;
        vn[c] = v_keep + v_inc;
        const float mhat = mn[c] / bc1;
        const float vhat = vn[c] / bc2;
        const float root = sqrtf(vhat);
        const float denom = root + eps;
        const float ratio = mhat / denom;
        const float step = lr * ratio;
        xn[c] = xo[c] - step;
    }
    store_stream(m + p, mn);
    store_stream(v + p, vn);
    store_stream(x + p, xn);
}

__global__ __launch_bounds__(kThreads) void freeze_kernel(float* __restrict__ m, float* __restrict__ werr,
                                                          float* __restrict__ serr, int64_t d, int32_t n) {
    const int64_t quads = d >> 2;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t q = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; q < quads; q += stride) {
        const int64_t p = q << 2;
        const f32x4 m0 = load_stream(m + p);
        store_stream(serr + p, zero);
        store_stream(werr + p, zero);
        for (int32_t i = 1; i < n; ++i) {
            store_stream(m + static_cast<int64_t>(i) * d + p, m0);
            store_stream(werr + static_cast<int64_t>(i) * d + p, zero);
        }
    }
}

inline uint32_t stride_grid(int64_t d) {
    const int64_t quads = d >> 2;
    int64_t blocks = (quads + kThreads - 1) / kThreads;
    const int64_t cap = 256 * 16;                         // 16 workgroups per CU, grid-stride beyond that
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return static_cast<uint32_t>(blocks);
}

}  // namespace

namespace {

template <int MOM, int G>
void launch_compress_as(int64_t grid, int32_t lds_pad, hipStream_t stream, float* m, const void* g, float* werr,
                        uint32_t* packed, double* partials, const float* prev_scales, const uint32_t* gather_words,
                        const float* gather_scales, const Geometry& geo, int32_t tpc, int32_t tiles_per_block,
                        int32_t blocks_per_chunk, float beta, float omb) {
    hipLaunchKernelGGL((compress_kernel<MOM, G>), dim3(static_cast<uint32_t>(grid)), dim3(kThreads), lds_pad,
                       stream, m, g, werr, packed, partials, prev_scales, gather_words, gather_scales, geo.d, geo.L,
                       geo.C, tpc, tiles_per_block, blocks_per_chunk, beta, omb);
}

template <int G>
hipError_t set_compress_lds_limit() {
    const void* kernels[] = {reinterpret_cast<const void*>(compress_kernel<kMomRead, G>),
                             reinterpret_cast<const void*>(compress_kernel<kMomGather, G>),
                             reinterpret_cast<const void*>(compress_kernel<kMomNone, G>)};
    for (const void* k : kernels) {
        hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsPad);
        if (e != hipSuccess) return e;
    }
    const void* onepass[] = {reinterpret_cast<const void*>(compress_onepass_kernel<kMomRead, G>),
                             reinterpret_cast<const void*>(compress_onepass_kernel<kMomGather, G>),
                             reinterpret_cast<const void*>(compress_onepass_kernel<kMomNone, G>)};
    for (const void* k : onepass) {
        hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kOnePassLdsBytes);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <int MOM, int G>
void launch_onepass_as(int64_t pairs, hipStream_t stream, float* m, const void* g, float* werr, uint32_t* packed,
                       float* scales_out, float* pending_out, const float* prev_scales, const uint32_t* gather_words,
                       const float* gather_scales, const Geometry& geo, int32_t tpc, float beta, float omb) {
    hipLaunchKernelGGL((compress_onepass_kernel<MOM, G>), dim3(static_cast<uint32_t>(pairs)), dim3(kOnePassThreads),
                       kOnePassLdsBytes, stream, m, g, werr, packed, scales_out, pending_out, prev_scales, gather_words,
                       gather_scales, geo.d, geo.L, geo.C, tpc, beta, omb);
}

template <int G>
hipError_t launch_onepass_mom(int momentum, int64_t pairs, hipStream_t stream, float* m, const void* g, float* werr,
                              uint32_t* packed, float* scales_out, float* pending_out, const float* prev_scales,
                              const uint32_t* gather_words, const float* gather_scales, const Geometry& geo,
                              int32_t tpc, float beta, float omb) {
    switch (momentum) {
        case kMomRead:
            launch_onepass_as<kMomRead, G>(pairs, stream, m, g, werr, packed, scales_out, pending_out, prev_scales,
                                           gather_words, gather_scales, geo, tpc, beta, omb);
            break;
        case kMomGather:
            launch_onepass_as<kMomGather, G>(pairs, stream, m, g, werr, packed, scales_out, pending_out, prev_scales,
                                             gather_words, gather_scales, geo, tpc, beta, omb);
            break;
        case kMomNone:
            launch_onepass_as<kMomNone, G>(pairs, stream, m, g, werr, packed, scales_out, pending_out, prev_scales,
                                           gather_words, gather_scales, geo, tpc, beta, omb);
            break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int G>
hipError_t launch_compress_mom(int momentum, int64_t grid, int32_t lds_pad, hipStream_t stream, float* m,
                               const void* g, float* werr, uint32_t* packed, double* partials,
                               const float* prev_scales, const uint32_t* gather_words, const float* gather_scales,
                               const Geometry& geo, int32_t tpc, int32_t tiles_per_block, int32_t blocks_per_chunk,
                               float beta, float omb) {
    switch (momentum) {
        case kMomRead:
            launch_compress_as<kMomRead, G>(grid, lds_pad, stream, m, g, werr, packed, partials, prev_scales,
                                            gather_words, gather_scales, geo, tpc, tiles_per_block,
                                            blocks_per_chunk, beta, omb);
            break;
        case kMomGather:
            launch_compress_as<kMomGather, G>(grid, lds_pad, stream, m, g, werr, packed, partials, prev_scales,
                                              gather_words, gather_scales, geo, tpc, tiles_per_block,
                                              blocks_per_chunk, beta, omb);
            break;
        case kMomNone:
            launch_compress_as<kMomNone, G>(grid, lds_pad, stream, m, g, werr, packed, partials, prev_scales,
                                            gather_words, gather_scales, geo, tpc, tiles_per_block,
                                            blocks_per_chunk, beta, omb);
            break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t enable_large_lds_pads() {
    hipError_t e = set_compress_lds_limit<kGradF32>();
    if (e == hipSuccess) e = set_compress_lds_limit<kGradF16>();
    if (e == hipSuccess) e = set_compress_lds_limit<kGradBF16>();
    if (e != hipSuccess) return e;
    const void* kernels[] = {reinterpret_cast<const void*>(server_kernel),
                             reinterpret_cast<const void*>(apply_kernel<true, true>),
                             reinterpret_cast<const void*>(apply_kernel<false, true>),
                             reinterpret_cast<const void*>(apply_kernel<true, false>),
                             reinterpret_cast<const void*>(apply_gradient_kernel),
                             reinterpret_cast<const void*>(finalize_kernel),
                             reinterpret_cast<const void*>(warmup_kernel<kGradF32>),
                             reinterpret_cast<const void*>(warmup_kernel<kGradF16>),
                             reinterpret_cast<const void*>(warmup_kernel<kGradBF16>)};
    for (const void* k : kernels) {
        e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsPad);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_compress(const Geometry& geo, int32_t tiles_per_block, int32_t blocks_per_chunk, int momentum,
                           float* m, const void* g, int grad_format, float* werr, uint32_t* packed,
                           double* partials, const float* prev_scales, const uint32_t* gather_words,
                           const float* gather_scales, float beta, float one_minus_beta, int32_t lds_pad,
                           hipStream_t stream) {
    const int64_t grid = static_cast<int64_t>(geo.n) * geo.C * blocks_per_chunk;
    if (grid <= 0) return hipSuccess;
    const int32_t tpc = static_cast<int32_t>(tiles_per_chunk(geo, kCompressTile));
    switch (grad_format) {
        case kGradF32:
            return launch_compress_mom<kGradF32>(momentum, grid, lds_pad, stream, m, g, werr, packed, partials,
                                                 prev_scales, gather_words, gather_scales, geo, tpc, tiles_per_block,
                                                 blocks_per_chunk, beta, one_minus_beta);
        case kGradF16:
            return launch_compress_mom<kGradF16>(momentum, grid, lds_pad, stream, m, g, werr, packed, partials,
                                                 prev_scales, gather_words, gather_scales, geo, tpc, tiles_per_block,
                                                 blocks_per_chunk, beta, one_minus_beta);
        case kGradBF16:
            return launch_compress_mom<kGradBF16>(momentum, grid, lds_pad, stream, m, g, werr, packed, partials,
                                                  prev_scales, gather_words, gather_scales, geo, tpc, tiles_per_block,
                                                  blocks_per_chunk, beta, one_minus_beta);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_compress_onepass(const Geometry& geo, int momentum, float* m, const void* g, int grad_format,
                                   float* werr, uint32_t* packed, float* scales_out, float* pending_out,
                                   const float* prev_scales, const uint32_t* gather_words,
                                   const float* gather_scales, float beta, float one_minus_beta, hipStream_t stream) {
    const int64_t pairs = static_cast<int64_t>(geo.n) * geo.C;
    if (pairs <= 0) return hipSuccess;
    if (geo.L > kOnePassMaxChunk) return hipErrorInvalidValue;
    const int32_t tpc = static_cast<int32_t>(tiles_per_chunk(geo, kCompressTile));
    switch (grad_format) {
        case kGradF32:
            return launch_onepass_mom<kGradF32>(momentum, pairs, stream, m, g, werr, packed, scales_out, pending_out,
                                                prev_scales, gather_words, gather_scales, geo, tpc, beta, one_minus_beta);
        case kGradF16:
            return launch_onepass_mom<kGradF16>(momentum, pairs, stream, m, g, werr, packed, scales_out, pending_out,
                                                prev_scales, gather_words, gather_scales, geo, tpc, beta, one_minus_beta);
        case kGradBF16:
            return launch_onepass_mom<kGradBF16>(momentum, pairs, stream, m, g, werr, packed, scales_out, pending_out,
                                                 prev_scales, gather_words, gather_scales, geo, tpc, beta, one_minus_beta);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_scales(int64_t pairs, int32_t blocks_per_chunk, int64_t L, const double* partials,
                         float* scales_out, float* pending_out, hipStream_t stream) {
    if (pairs <= 0) return hipSuccess;
    hipLaunchKernelGGL(scales_kernel, dim3(static_cast<uint32_t>(pairs)), dim3(kThreads), 0, stream, partials,
                       blocks_per_chunk, L, scales_out, pending_out);
    return hipGetLastError();
}

hipError_t launch_finalize(const Geometry& geo, int32_t slices, float* err, const float* scales,
                           int32_t lds_pad, hipStream_t stream) {
    const int64_t tpc = tiles_per_chunk(geo, kFinalizeTile);
    const int64_t grid = static_cast<int64_t>(slices) * geo.C * tpc;
    if (grid <= 0) return hipSuccess;
    hipLaunchKernelGGL(finalize_kernel, dim3(static_cast<uint32_t>(grid)), dim3(kThreads), lds_pad, stream, err,
                       scales, geo.d, geo.L, geo.C, static_cast<int32_t>(tpc));
    return hipGetLastError();
}

hipError_t launch_server_reduce(const Geometry& geo, int32_t tiles_per_block, int32_t blocks_per_chunk,
                                const uint32_t* packed, const float* scales, float* serr, uint32_t* spacked,
                                double* partials, const float* prev_scales, float inv_n, int32_t lds_pad,
                                hipStream_t stream) {
    const int64_t grid = static_cast<int64_t>(geo.C) * blocks_per_chunk;
    if (grid <= 0) return hipSuccess;
    hipLaunchKernelGGL(server_kernel, dim3(static_cast<uint32_t>(grid)), dim3(kThreads), lds_pad, stream, packed,
                       scales, serr, spacked, partials, prev_scales, geo.d, geo.L, geo.C, geo.n,
                       static_cast<int32_t>(tiles_per_chunk(geo, kServerTile)), tiles_per_block,
                       blocks_per_chunk, inv_n);
    return hipGetLastError();
}

hipError_t launch_apply(const Geometry& geo, const uint32_t* spacked, const float* sscales, const float* v,
                        float* x, float* m, float* scales_copy, bool write_m, bool model_step, float lr,
                        float eps, int32_t lds_pad, hipStream_t stream) {
    const int64_t tpc = tiles_per_chunk(geo, kApplyTile);
    const int64_t tiles_per_slice = static_cast<int64_t>(geo.C) * tpc;
    const int64_t grid = tiles_per_slice * (write_m ? geo.n : 1);
    if (grid <= 0 || !(write_m || model_step)) return hipSuccess;
    const dim3 g(static_cast<uint32_t>(grid)), b(kThreads);
    if (write_m && model_step)
        hipLaunchKernelGGL((apply_kernel<true, true>), g, b, lds_pad, stream, spacked, sscales, v, x, m, scales_copy,
                           geo.d, geo.L, tiles_per_slice, static_cast<int32_t>(tpc), lr, eps);
    else if (model_step)
        hipLaunchKernelGGL((apply_kernel<false, true>), g, b, lds_pad, stream, spacked, sscales, v, x, m, scales_copy,
                           geo.d, geo.L, tiles_per_slice, static_cast<int32_t>(tpc), lr, eps);
    else
        hipLaunchKernelGGL((apply_kernel<true, false>), g, b, lds_pad, stream, spacked, sscales, v, x, m, scales_copy,
                           geo.d, geo.L, tiles_per_slice, static_cast<int32_t>(tpc), lr, eps);
    return hipGetLastError();
}

hipError_t launch_apply_gradient(const Geometry& geo, const uint32_t* spacked, const float* sscales,
                                 const float* v, float* x, float* m, float lr, float beta, float one_minus_beta,
                                 float eps, int32_t lds_pad, hipStream_t stream) {
    const int64_t tpc = tiles_per_chunk(geo, kApplyTile);
    const int64_t tiles_per_slice = static_cast<int64_t>(geo.C) * tpc;
    const int64_t grid = tiles_per_slice * geo.n;
    if (grid <= 0) return hipSuccess;
    hipLaunchKernelGGL(apply_gradient_kernel, dim3(static_cast<uint32_t>(grid)), dim3(kThreads), lds_pad, stream,
                       spacked, sscales, v, x, m, geo.d, geo.L, tiles_per_slice, static_cast<int32_t>(tpc), lr, beta,
                       one_minus_beta, eps);
    return hipGetLastError();
}

hipError_t launch_warmup(int64_t d, int32_t n, float* x, float* m, float* v, const void* g, int grad_format, float lr,
                         float beta1, float one_minus_beta1, float beta2, float one_minus_beta2, float bc1,
                         float bc2, float eps, float inv_n, int32_t lds_pad, hipStream_t stream) {
    if (d <= 0) return hipSuccess;
    const dim3 grid(static_cast<uint32_t>(((d >> 2) + kThreads - 1) / kThreads)), block(kThreads);
    switch (grad_format) {
        case kGradF32:
            hipLaunchKernelGGL(warmup_kernel<kGradF32>, grid, block, lds_pad, stream, x, m, v, g, d, n, lr, beta1,
                               one_minus_beta1, beta2, one_minus_beta2, bc1, bc2, eps, inv_n);
            break;
        case kGradF16:
            hipLaunchKernelGGL(warmup_kernel<kGradF16>, grid, block, lds_pad, stream, x, m, v, g, d, n, lr, beta1,
                               one_minus_beta1, beta2, one_minus_beta2, bc1, bc2, eps, inv_n);
            break;
        case kGradBF16:
            hipLaunchKernelGGL(warmup_kernel<kGradBF16>, grid, block, lds_pad, stream, x, m, v, g, d, n, lr, beta1,
                               one_minus_beta1, beta2, one_minus_beta2, bc1, bc2, eps, inv_n);
            break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_freeze(int64_t d, int32_t n, float* m, float* werr, float* serr, hipStream_t stream) {
    if (d <= 0) return hipSuccess;
    hipLaunchKernelGGL(freeze_kernel, dim3(stride_grid(d)), dim3(kThreads), 0, stream, m, werr, serr, d, n);
    return hipGetLastError();
}

}  // namespace apms
