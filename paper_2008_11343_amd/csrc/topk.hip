// Top-k compressor kernels (Section 5.1, second bullet) for gfx950: keep the K elements of largest
// magnitude of every chunk, ties towards the lower index, and emit them as (index, value) pairs in index
// order; everything else stays in the error buffer (error feedback, Section 3.1).
//
// Exact selection without sorting: the magnitude key of a value is its binary32 pattern without the sign
// bit, which orders like |u|.  A 3-level radix select (11 + 11 + 9 bits) over per-chunk histograms finds
// the K-th largest key T and how many elements equal to T may still be kept; only if that is fewer than
// there are, the index rule picks the last such element to keep: from the short list of elements that share
// T's leading 22 bits (topk_resolve_kernel), or, where that list or a tile's slots overflow, by a second
// 3-level radix select (11 + 11 + 10 bits) over the chunk-local index.  Histograms use integer atomics
// (order-independent), the emission order comes from per-tile counts and a scan, so the result does not
// depend on scheduling.
//
// Only the level-0 histogram needs every element, and only if nothing is known: the first pass histograms
// the elements whose key is at or above a guessed floor (the previous call's threshold key less a margin) and
// leaves the rest uncounted, so that the few populated exponent bins of ordinary data do not serialise on LDS
// atomics; if it counted fewer than K elements the threshold lies below the floor, and one more pass over the
// buffer builds the whole level-0 histogram for that chunk.  What the later steps need are the elements at or
// above the level-0 bin of T (kept whatever T turns out to be if above, candidates if inside).  They are
// copied to per-tile slots - by the first pass itself, on its floor (about 1.5 % of a tile when K is 1 % of a
// chunk), else by one more pass once the bin is known - and key levels 1 and 2, the tie rule, the per-tile
// kept counts and the emission work on the slots alone.  A chunk with a tile that has more such elements
// than slots is flagged and takes full passes over the buffer instead.
//
// Built with -ffp-contract=off: the elementwise arithmetic is that of the 1-bit path.

#include "apms_device.h"
#include "apms_topk.h"

namespace apms {

namespace {

// Per-pair selection state (uint32 words).
enum : int {
    kStPrefix = 0,        // key bits fixed so far (bits below the current level are zero)
    kStRemaining = 1,     // how many elements are still to be taken from inside the current prefix
    kStCountEq = 2,       // number of elements with key == T
    kStTieNeeded = 3,     // 1 if only some of the elements equal to T may be kept
    kStIdxPrefix = 4,     // index bits fixed so far (tie selection)
    kStIdxRemaining = 5,  // how many ties are still to be taken from inside the current index prefix
    kStKeyT = 6,          // T: the K-th largest key
    kStIdxT = 7,          // ties are kept up to and including this chunk-local index
    kStOverflow = 8,      // 1 if a tile of this pair had more entries than slots: full passes instead
    kStResplit = 9,       // 1 if the pair's slots have to be filled again, from the threshold bin now known
    kStRehist = 10,       // 1 if the level-0 histogram of the first pass did not reach down to the threshold bin
    kStNearCount = 11,    // slot entries that share the threshold's top 22 key bits (appended to the near list)
    kStNearOverflow = 12, // 1 if there were more of them than the near list holds: tie levels and counts from the slots
    kStTieDone = 13,      // 1 if kStIdxT and the per-tile counts were settled from the near list
};

// The floor of the next call's first pass (guess[pair]) lies a margin below the threshold key found.  Only a
// threshold that FALLS below the floor costs extra passes, so the margin follows how far it fell since the
// call before (last_T[pair] remembers it): eight times that, at least half the previous margin (it shrinks
// over a few calls while the threshold rises or stands still), between 2^15 (0.2 to 0.4 % in magnitude) and
// half a level-0 bin (2^19: 3 to 6 %); half a bin when there is no history or this call's floor proved too
// high.  The tighter the floor, the fewer elements the first pass copies to the slots and the later passes
// read: with K at 1 % of a chunk of normal data 1.5 % of the elements pass a floor half a bin down, 1.1 % one
// at 2^16, and the worker call is 4 % faster.  With no earlier call to go by the tables hold 0xFFFFFFFF, a
// floor that no key reaches.
constexpr uint32_t kGuessMarginMax = 1u << 19;
constexpr uint32_t kGuessMarginMin = 1u << 15;
constexpr uint32_t kGuessMarginPerFall = 8u;

constexpr uint32_t kTopMask = 0x7FF00000u;      // the level-0 digit of a key

struct Level {
    int shift;
    int bits;
    uint32_t match_mask;  // bits above this level: they must equal the prefix for an element to count
};

__host__ __device__ constexpr Level key_level(int l) {
    return l == 0 ? Level{20, 11, 0u} : l == 1 ? Level{9, 11, 0x7FF00000u} : Level{0, 9, 0x7FFFFE00u};
}
__host__ __device__ constexpr Level idx_level(int l) {
    return l == 0 ? Level{21, 11, 0u} : l == 1 ? Level{10, 11, 0xFFE00000u} : Level{0, 10, 0xFFFFFC00u};
}

__device__ __forceinline__ uint32_t key_of(float u) { return __builtin_bit_cast(uint32_t, u) & 0x7FFFFFFFu; }

__device__ __forceinline__ bool kept(uint32_t key, uint32_t j, uint32_t T, uint32_t idxT) {
    return key > T || (key == T && j <= idxT);
}

// What an error buffer left in deferred form holds is the compensated vector v of the previous call; its
// error is v where the element was not kept and zero where it was.  `keep` = {T, idxT} of that call for the
// pair ({0xFFFFFFFF, 0}: nothing was kept, which is also how a buffer in final form is read).
__device__ __forceinline__ float deferred_error(float stored, uint32_t j, uint2 keep) {
    return kept(key_of(stored), j, keep.x, keep.y) ? 0.0f : stored;
}

// One atomic per distinct bin per wave.  Must be called by all 64 lanes (inactive ones pass active = false).
__device__ __forceinline__ void hist_add_aggregated(uint32_t* __restrict__ hist, bool active, uint32_t bin) {
    const int lane = threadIdx.x & (kWaveSize - 1);
    uint64_t todo = __ballot(active);
    while (todo) {
        const int leader = __ffsll(static_cast<unsigned long long>(todo)) - 1;
        const uint32_t lbin = static_cast<uint32_t>(__shfl(static_cast<int>(bin), leader));
        const uint64_t same = __ballot(active && bin == lbin) & todo;
        if (lane == leader) atomicAdd(&hist[lbin], static_cast<uint32_t>(__popcll(static_cast<unsigned long long>(same))));
        todo &= ~same;
    }
}

// Exclusive scan of one uint32 per thread over the workgroup (thread order); `total` gets the sum.
__device__ __forceinline__ uint32_t block_exclusive_scan_u32(uint32_t v, uint32_t* lds /* kWaves */, uint32_t& total) {
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int off = 1; off < kWaveSize; off <<= 1) {
        const uint32_t up = static_cast<uint32_t>(__shfl_up(static_cast<int>(inc), off));
        if (lane >= off) inc += up;
    }
    if (lane == kWaveSize - 1) lds[wave] = inc;
    __syncthreads();
    uint32_t before = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t t = lds[w];
        if (w < wave) before += t;
        sum += t;
    }
    __syncthreads();
    total = sum;
    return before + inc - v;
}

// The same for one uint64 per thread (used to scan four 16-bit counters at once).
__device__ __forceinline__ uint64_t block_exclusive_scan_u64(uint64_t v, uint64_t* lds /* kWaves */, uint64_t& total) {
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    uint64_t inc = v;
#pragma unroll
    for (int off = 1; off < kWaveSize; off <<= 1) {
        const uint64_t up = static_cast<uint64_t>(__shfl_up(static_cast<unsigned long long>(inc), off));
        if (lane >= off) inc += up;
    }
    if (lane == kWaveSize - 1) lds[wave] = inc;
    __syncthreads();
    uint64_t before = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint64_t t = lds[w];
        if (w < wave) before += t;
        sum += t;
    }
    __syncthreads();
    total = sum;
    return before + inc - v;
}

// Decomposition of blockIdx into (pair, tile) for kernels that take one kTopkTile tile per workgroup.
struct TileRef {
    int64_t pair;        // slice * C + chunk
    int64_t chunk;
    int64_t tile;
    int64_t base;        // element offset of the chunk inside the [slices][d] buffer
};
__device__ __forceinline__ TileRef tile_ref(int64_t d, int64_t L, int32_t C, int32_t tiles_per_chunk,
                                            int64_t blk = blockIdx.x) {
    TileRef r;
    r.pair = blk / tiles_per_chunk;
    r.tile = blk - r.pair * tiles_per_chunk;
    const int64_t slice = r.pair / C;
    r.chunk = r.pair - slice * C;
    r.base = slice * d + r.chunk * L;
    return r;
}

constexpr int kTileRows = kTopkTile / (kThreads * 4);   // 128-bit rows per thread per tile, plain layout
constexpr int kServerStage = 1024;                       // entries of the server kernel's LDS stage (8 KB)
constexpr int kRowStride = kThreads * 4;

// Flush a workgroup's LDS histogram into the pair's global histogram (non-zero bins only).
__device__ __forceinline__ void flush_histogram(const uint32_t* lds_hist, uint32_t* __restrict__ hist,
                                                int bins = kTopkBins) {
    for (int b = threadIdx.x; b < bins; b += kThreads) {
        const uint32_t c = lds_hist[b];
        if (c) atomicAdd(&hist[b], c);
    }
}

// The first pass counts only the elements at or above its floor, and ordinary data reaches a few dozen bins
// above the threshold's (8 bins per binade): a workgroup keeps a window of kHistWindow bins starting at the
// floor's bin in LDS and sends the rare element beyond it to the pair's histogram directly.  (The floor's own
// bin is counted in part: enough, because the selection only ever looks for elements above the floor.)
constexpr int kHistWindow = 256;
static_assert(kHistWindow == kThreads, "one window bin per thread");
__device__ __forceinline__ void count_in_window(uint32_t* lds_window, uint32_t* __restrict__ hist, uint32_t guessed,
                                                uint32_t bin) {
    const uint32_t rel = bin - guessed;                        // callers pass bins at or above the floor's only
    if (rel < static_cast<uint32_t>(kHistWindow)) atomicAdd(&lds_window[rel], 1u); else atomicAdd(&hist[bin], 1u);
}
__device__ __forceinline__ void flush_window(const uint32_t* lds_window, uint32_t* __restrict__ hist, uint32_t guessed) {
    const uint32_t c = lds_window[threadIdx.x];
    if (c) atomicAdd(&hist[guessed + threadIdx.x], c);         // counted, so the bin exists
}

// Copies the marked elements of a tile (bit 4*r + c of take_mask: element c of row r of this thread; packed:
// the four per-row counts as 16-bit fields) to the tile's slots as (tile-local index, value bits), in index
// order, as far as there are slots; returns how many elements were marked in the whole tile.  Index order
// inside a tile is row by row (plain layout), thread by thread inside a row: one workgroup scan of the packed
// counts gives every thread its rank in each row.  Contains workgroup barriers.
__device__ __forceinline__ uint32_t write_tile_slots(const f32x4 (&v)[kTileRows], uint32_t take_mask, uint64_t packed,
                                                     uint64_t* lds /* kWaves */, uint2* __restrict__ my_slots,
                                                     int32_t slots_per_tile) {
    static_assert(kTileRows == 4 && kThreads * 4 < 65536, "four 16-bit row counters");
    uint64_t totals;
    const uint64_t before = block_exclusive_scan_u64(packed, lds, totals);
    uint32_t row_base = 0;
#pragma unroll
    for (int r = 0; r < kTileRows; ++r) {
        uint32_t rank = row_base + static_cast<uint32_t>((before >> (16 * r)) & 0xFFFFu);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (take_mask & (1u << (4 * r + c))) {
                const uint32_t local = static_cast<uint32_t>(threadIdx.x * 4 + r * kRowStride + c);
                // by value: a bit cast applied to the vector element expression itself reads element 0
                const float value = v[r][c];
                if (rank < static_cast<uint32_t>(slots_per_tile))
                    my_slots[rank] = make_uint2(local, __builtin_bit_cast(uint32_t, value));
                ++rank;
            }
        }
        row_base += static_cast<uint32_t>((totals >> (16 * r)) & 0xFFFFu);
    }
    return row_base;
}

// The same for a tile whose values also lie in LDS (tile_values[tile-local index]), and with the histogram
// window: every marked element is counted in the window and copied to the tile's slots.  A thread walks the
// set bits of its mask (a tile has a few dozen marked elements among 4096, so most threads have none)
// instead of testing all sixteen of its elements.  Contains workgroup barriers and ends with one: the
// window is complete.  Returns how many elements were marked in the whole tile.
__device__ __forceinline__ uint32_t count_and_slot_marked(const float* tile_values /* LDS */, uint32_t take_mask,
                                                          uint64_t* lds_scan /* kWaves */, uint32_t* lds_window,
                                                          uint32_t* __restrict__ pair_hist, uint32_t guessed,
                                                          uint2* __restrict__ my_slots, int32_t slots_per_tile) {
    static_assert(kTileRows == 4 && kThreads * 4 < 65536, "four 16-bit row counters");
    uint64_t packed = 0;
#pragma unroll
    for (int r = 0; r < kTileRows; ++r)
        packed |= static_cast<uint64_t>(__popc((take_mask >> (4 * r)) & 0xFu)) << (16 * r);
    uint64_t totals;
    const uint64_t before = block_exclusive_scan_u64(packed, lds_scan, totals);
    // field r: the rank of this thread's first marked element of row r = marked elements of the rows before
    // (the fields stay below 2^16, so the shifted sums do not carry into each other) + those of row r in the
    // threads before
    const uint64_t rank0 = (totals << 16) + (totals << 32) + (totals << 48) + before;
    uint32_t todo = take_mask;
    while (todo) {
        const int b = __ffs(static_cast<int>(todo)) - 1;
        todo &= todo - 1u;
        const int r = b >> 2;
        const uint32_t local = static_cast<uint32_t>(threadIdx.x * 4 + r * kRowStride + (b & 3));
        const float value = tile_values[local];
        const uint32_t bits = __builtin_bit_cast(uint32_t, value);
        count_in_window(lds_window, pair_hist, guessed, (bits & 0x7FFFFFFFu) >> 20);
        const uint32_t rank = static_cast<uint32_t>((rank0 >> (16 * r)) & 0xFFFFu) +
                              static_cast<uint32_t>(__popc(take_mask & ((1u << b) - 1u) & (0xFu << (4 * r))));
        if (rank < static_cast<uint32_t>(slots_per_tile)) my_slots[rank] = make_uint2(local, bits);
    }
    __syncthreads();
    return static_cast<uint32_t>((totals & 0xFFFFu) + ((totals >> 16) & 0xFFFFu) + ((totals >> 32) & 0xFFFFu) + (totals >> 48));
}

// ------------------------------------------------------------------------
// Worker: u into the error buffer + level-0 key histogram (Algorithm 1 lines 6-7).
// ------------------------------------------------------------------------
// The threshold hardly moves from one step to the next, so the pass works on a guess: a floor a margin
// below the previous call's threshold key (guess[pair]; 0xFFFFFFFF before the first call).  Elements at or above
// the floor are histogrammed and copied to the slots, the others are left alone.  The guess is good if at
// least K elements passed it: the K-th largest key is then among them, histogram and slots hold a superset
// of what the selection looks at, and the extra entries fail every later test.  If fewer passed, the pair is
// marked kStRehist and takes a full histogram pass; there, and where a tile overflowed its slots, the pair
// is marked kStResplit and topk_split_kernel fills its slots again.
// One tile per workgroup: taking several tiles in a loop (one histogram flush for all of them, or with the
// next tile's loads requested ahead) was measured 3 to 10 % slower, like the 1-bit worker kernel this pass
// streams best as many short-lived workgroups.
//
// kGather: a gather is pending on m (Algorithm 1 line 10 not yet carried out): the momentum of every worker
// is the server's list of the previous step (gather_idx, gather_val: [C][gather_K], with the table of tile
// offsets apms_topk_apply left), zero elsewhere.  The tile's stretch of the list is decoded into the LDS
// tile, used directly as the momentum term and written to m (unless m is null: implicit-momentum mode).
template <bool kGather>
__global__ __launch_bounds__(kThreads) void topk_worker_u_kernel(float* __restrict__ m, const float* __restrict__ g,
                                                                 float* __restrict__ e, uint32_t* __restrict__ hist,
                                                                 uint32_t* __restrict__ state,
                                                                 const uint32_t* __restrict__ guess,
                                                                 uint32_t* __restrict__ tile_split,
                                                                 uint2* __restrict__ slots, int32_t slots_per_tile,
                                                                 const uint2* __restrict__ prev_keep,
                                                                 const uint32_t* __restrict__ gather_idx,
                                                                 const float* __restrict__ gather_val,
                                                                 const uint32_t* __restrict__ gather_offsets,
                                                                 int32_t gather_K, int64_t d, int64_t L, int32_t C,
                                                                 int32_t tiles_per_chunk, float beta, float omb) {
    __shared__ uint32_t lds_window[kHistWindow];
    __shared__ uint64_t lds_scan[kWaves];
    __shared__ __align__(16) float tile_u[kTopkTile];          // the tile's u, for the marked elements' second look
    lds_window[threadIdx.x] = 0u;
    const TileRef tr = tile_ref(d, L, C, tiles_per_chunk);
    uint32_t* pair_hist = hist + tr.pair * kTopkBins;
    const int64_t off0 = tr.tile * kTopkTile + threadIdx.x * 4;
    const uint2 keep = prev_keep ? prev_keep[tr.pair] : make_uint2(0xFFFFFFFFu, 0u);   // error buffer in deferred form?
    const uint32_t floor_key = guess[tr.pair];                // 0xFFFFFFFF: no earlier call, nothing passes
    const uint32_t guessed = floor_key >> 20;                 // first bin of the histogram window
    f32x4 vg[kTileRows], ve[kTileRows], vm[kTileRows];
#pragma unroll
    for (int r = 0; r < kTileRows; ++r) {                      // requested first: they arrive during the decode
        const int64_t off = off0 + r * kRowStride;
        vg[r] = ve[r] = vm[r] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (off >= L) continue;
        const int64_t p = tr.base + off;
        vg[r] = load_stream(g + p);
        ve[r] = load_stream(e + p);
        if (!kGather) vm[r] = load_stream(m + p);
    }
    if (kGather) {
        const int64_t chunk = tr.chunk;
        const uint32_t* off = gather_offsets + chunk * tiles_per_chunk + tr.tile;
        const int last = min((tr.tile + 1 < tiles_per_chunk) ? static_cast<int>(off[1]) : gather_K, gather_K);   // min, first >= 0:
        const int first = max(static_cast<int>(off[0]), 0);                                                     // no-ops for sorted lists
#pragma unroll
        for (int r = 0; r < kTileRows; ++r)
            *reinterpret_cast<f32x4*>(&tile_u[threadIdx.x * 4 + r * kRowStride]) = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        __syncthreads();
        const int64_t list = chunk * gather_K;
        const uint32_t tile_lo = static_cast<uint32_t>(tr.tile * kTopkTile);
        for (int t = first + threadIdx.x; t < last; t += kThreads) {
            const uint32_t j = gather_idx[list + t] - tile_lo;
            if (j < static_cast<uint32_t>(kTopkTile)) tile_u[j] = gather_val[list + t];      // always true for sorted lists
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kTileRows; ++r) {
            const int64_t off = off0 + r * kRowStride;
            if (off >= L) continue;
            vm[r] = *reinterpret_cast<const f32x4*>(&tile_u[threadIdx.x * 4 + r * kRowStride]);
            if (m) store_stream(m + tr.base + off, vm[r]);
        }
    }
    uint32_t take_mask = 0;
#pragma unroll
    for (int r = 0; r < kTileRows; ++r) {
        const int64_t off = off0 + r * kRowStride;
        if (off >= L) continue;
        f32x4 u;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float bm = beta * vm[r][c];
            const float bg = omb * vg[r][c];
            const float mi = bm + bg;
            const float stored = ve[r][c];
            u[c] = mi + deferred_error(stored, static_cast<uint32_t>(off + c), keep);
            const float value = u[c];
            take_mask |= key_of(value) >= floor_key ? 1u << (4 * r + c) : 0u;   // at or above the floor: counted and slotted
        }
        *reinterpret_cast<f32x4*>(&tile_u[threadIdx.x * 4 + r * kRowStride]) = u;   // this thread's own four positions
        store_stream(e + tr.base + off, u);
    }
    const int64_t tile_id = tr.pair * tiles_per_chunk + tr.tile;
    const uint32_t marked = count_and_slot_marked(tile_u, take_mask, lds_scan, lds_window, pair_hist, guessed,
                                                  slots + tile_id * slots_per_tile, slots_per_tile);   // its barriers also cover lds_window
    if (threadIdx.x == 0) {
        tile_split[tile_id] = marked;
        if (marked > static_cast<uint32_t>(slots_per_tile)) state[tr.pair * kTopkStateWords + kStResplit] = 1u;
    }
    flush_window(lds_window, pair_hist, guessed);
}

// ------------------------------------------------------------------------
// Server: decode + average the n sparse messages of a tile in LDS, add the server error, write ubar into
// the error buffer + level-0 key histogram (Algorithm 1 line 9).
// ------------------------------------------------------------------------
// offsets[list][tile] = how many entries of the sorted index list `list` lie below the tile's first element:
// where the tile's stretch of the list starts (it ends where the next tile's starts, or at K).  One thread per
// list entry (four per thread): the entry that is the first of its list at or beyond a tile's start writes that tile's offset
// (and those of the empty tiles before it), the last entry those of the tiles after it.  Tiles are
// 1 << tile_shift elements.  Indices at or beyond the chunk's end count as lying in its last tile, so every
// store stays inside the table whatever the lists hold.
constexpr int kOffsetsPerThread = 4;
__global__ __launch_bounds__(kThreads) void topk_tile_offsets_kernel(const uint32_t* __restrict__ idx,
                                                                     uint32_t* __restrict__ offsets,
                                                                     int32_t tiles_per_chunk, int tile_shift,
                                                                     int32_t K, int32_t blocks_per_list) {
    const int64_t list = blockIdx.x / blocks_per_list;
    const int32_t e0 = static_cast<int32_t>(blockIdx.x - list * blocks_per_list) * (kThreads * kOffsetsPerThread) +
                       static_cast<int32_t>(threadIdx.x);
    const uint32_t* mine = idx + list * K;
    uint32_t* row = offsets + list * tiles_per_chunk;
    const uint32_t last_tile = static_cast<uint32_t>(tiles_per_chunk - 1);
    uint32_t at[kOffsetsPerThread], before[kOffsetsPerThread];
#pragma unroll
    for (int k = 0; k < kOffsetsPerThread; ++k) {              // all loads first
        const int32_t e = e0 + k * kThreads;
        at[k] = e < K ? mine[e] : 0u;
        before[k] = (e > 0 && e < K) ? mine[e - 1] : 0u;
    }
#pragma unroll
    for (int k = 0; k < kOffsetsPerThread; ++k) {
        const int32_t e = e0 + k * kThreads;
        if (e >= K) continue;
        const int32_t to = static_cast<int32_t>(min(at[k] >> tile_shift, last_tile));
        const int32_t from = e == 0 ? 0 : static_cast<int32_t>(min(before[k] >> tile_shift, last_tile)) + 1;
        for (int32_t tile = from; tile <= to; ++tile) row[tile] = static_cast<uint32_t>(e);
        if (e == K - 1)
            for (int32_t tile = to + 1; tile <= static_cast<int32_t>(last_tile); ++tile) row[tile] = static_cast<uint32_t>(K);
    }
}

// Like the worker's first pass, it counts and slots only the elements at or above a guessed floor
// (guess[chunk], the server's own table).
//
// The decoded messages have to be added position by position in worker order, and walking the workers one
// after the other straight from memory is a chain of dependent loads (where a worker's stretch for this tile
// starts, then its entries) per worker.  So, `workers_per_batch` workers at a time (the host sizes the batch
// so that its entries usually fit the stage): (A) one thread per worker fetches its stretch's bounds, a
// workgroup scan lays the stretches out back to back; (B) all threads copy the entries of all those workers
// into an LDS stage at once; (C) each wave, which owns a quarter of the tile's positions, walks the stage
// worker by worker and adds the entries that fall into its quarter.  A wave's LDS operations complete in
// program order, and positions are unique inside one worker's list, so the running sums see the workers in
// order without any barrier in (C).  The kernel waits on memory in (A) and again in (B), so what it reaches
// depends on how many workgroups a CU holds: its LDS is kept to 26 KB (six per CU).
constexpr int kServerBatchMax = 64;                          // workers per batch at most
__global__ __launch_bounds__(kThreads) void topk_server_u_kernel(const uint32_t* __restrict__ idx,
                                                                 const float* __restrict__ val,
                                                                 float* __restrict__ serr, uint32_t* __restrict__ hist,
                                                                 uint32_t* __restrict__ state,
                                                                 const uint32_t* __restrict__ guess,
                                                                 const uint32_t* __restrict__ offsets,
                                                                 uint32_t* __restrict__ tile_split,
                                                                 uint2* __restrict__ slots, int32_t slots_per_tile,
                                                                 const uint2* __restrict__ prev_keep,
                                                                 int64_t d, int64_t L, int32_t C, int32_t n,
                                                                 int32_t K, int32_t tiles_per_chunk,
                                                                 int32_t workers_per_batch, float inv_n) {
    __shared__ uint32_t lds_window[kHistWindow];
    __shared__ uint64_t lds_scan[kWaves];
    __shared__ __align__(16) float acc[kTopkTile];
    __shared__ uint2 stage[kServerStage];                      // (tile-local position, value bits), worker-major
    __shared__ uint32_t stage_first[kServerBatchMax];          // per worker of the batch: first list entry of the tile
    __shared__ uint32_t stage_start[kServerBatchMax + 1];      // ... and where its entries start in the stage
    __shared__ uint32_t stage_scan[kWaves];
    lds_window[threadIdx.x] = 0u;
    for (int j = threadIdx.x; j < kTopkTile; j += kThreads) acc[j] = 0.0f;
    const TileRef tr = tile_ref(d, L, C, tiles_per_chunk);    // slices = 1: pair = chunk
    uint32_t* pair_hist = hist + tr.pair * kTopkBins;
    const int64_t tile_lo = tr.tile * kTopkTile;
    const uint32_t floor_key = guess[tr.pair];                // 0xFFFFFFFF: no earlier call, nothing passes
    const uint32_t guessed = floor_key >> 20;                 // first bin of the histogram window
    const uint2 keep = prev_keep ? prev_keep[tr.pair] : make_uint2(0xFFFFFFFFu, 0u);
    // the tile of the server error, requested now: it arrives while the messages are being decoded
    f32x4 ve[kTileRows];
#pragma unroll
    for (int r = 0; r < kTileRows; ++r) {
        const int64_t off = tile_lo + threadIdx.x * 4 + r * kRowStride;
        ve[r] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (off < L) ve[r] = load_stream(serr + tr.base + off);
    }
    __syncthreads();
    {
        const uint32_t lane = threadIdx.x & (kWaveSize - 1);
        const uint32_t wave = threadIdx.x >> 6;
        constexpr uint32_t kQuarterShift = 10;                 // kTopkTile / kWaves = 1024 positions per wave
        static_assert((kTopkTile / kWaves) == (1 << kQuarterShift), "a wave's share of the tile");
        const auto add_entry = [&](uint2 entry) {
            const uint32_t j = entry.x;
            if (j < static_cast<uint32_t>(kTopkTile) && (j >> kQuarterShift) == wave)
                acc[j] = acc[j] + __builtin_bit_cast(float, entry.y);
        };
        for (int32_t i0 = 0; i0 < n; i0 += workers_per_batch) {
            const int32_t batch = min(n - i0, workers_per_batch);
            // (A)
            uint32_t first = 0, count = 0;
            if (static_cast<int32_t>(threadIdx.x) < batch) {
                const int64_t which = static_cast<int64_t>(i0 + threadIdx.x) * C + tr.pair;
                const uint32_t* off = offsets + which * tiles_per_chunk + tr.tile;
                first = off[0];
                const uint32_t last = (tr.tile + 1 < tiles_per_chunk) ? off[1] : static_cast<uint32_t>(K);
                count = (first < last && last <= static_cast<uint32_t>(K)) ? last - first : 0u;   // always, for sorted lists
            }
            uint32_t total;
            const uint32_t start = block_exclusive_scan_u32(count, stage_scan, total);
            if (threadIdx.x < kServerBatchMax) {
                stage_first[threadIdx.x] = first;
                stage_start[threadIdx.x] = start;              // = total for the threads beyond the batch
            }
            if (threadIdx.x == 0) stage_start[kServerBatchMax] = total;
            __syncthreads();
            if (total <= static_cast<uint32_t>(kServerStage)) {
                // (B) entry e of the stage belongs to the worker w with stage_start[w] <= e < stage_start[w + 1]
                for (uint32_t e = threadIdx.x; e < total; e += kThreads) {
                    int lo = 0, hi = batch;                    // last w with stage_start[w] <= e
                    while (hi - lo > 1) {
                        const int mid = (lo + hi) >> 1;
                        if (stage_start[mid] <= e) lo = mid; else hi = mid;
                    }
                    const int64_t src = (static_cast<int64_t>(i0 + lo) * C + tr.pair) * K + stage_first[lo] + (e - stage_start[lo]);
                    const float value = val[src];
                    stage[e] = make_uint2(idx[src] - static_cast<uint32_t>(tile_lo), __builtin_bit_cast(uint32_t, value));
                }
                __syncthreads();
                // (C) four workers' first 64 entries are read from the stage together, then added in worker order
                constexpr int kAhead = 4;
                for (int32_t w = 0; w < batch; w += kAhead) {
                    uint32_t bound[kAhead + 1];
                    uint2 entry[kAhead];
#pragma unroll
                    for (int u = 0; u <= kAhead; ++u) bound[u] = stage_start[min(w + u, static_cast<int32_t>(kServerBatchMax))];
#pragma unroll
                    for (int u = 0; u < kAhead; ++u) {
                        const uint32_t e = bound[u] + lane;
                        entry[u] = make_uint2(0xFFFFFFFFu, 0u);
                        if (e < bound[u + 1]) entry[u] = stage[e];
                    }
#pragma unroll
                    for (int u = 0; u < kAhead; ++u) {
                        add_entry(entry[u]);
                        for (uint32_t e = bound[u] + lane + kWaveSize; e < bound[u + 1]; e += kWaveSize) add_entry(stage[e]);
                    }
                }
            } else {
                // more entries than the stage holds (a K far above what the batch was sized for): worker by worker
                for (int32_t w = 0; w < batch; ++w) {
                    const int64_t list = (static_cast<int64_t>(i0 + w) * C + tr.pair) * K;
                    const uint32_t lo = stage_first[w], hi = lo + (stage_start[w + 1] - stage_start[w]);
                    for (uint32_t t = lo + lane; t < hi; t += kWaveSize) {
                        const float value = val[list + t];
                        add_entry(make_uint2(idx[list + t] - static_cast<uint32_t>(tile_lo), __builtin_bit_cast(uint32_t, value)));
                    }
                }
            }
            __syncthreads();                                   // before the next batch reuses the stage tables
        }
    }
    // ubar = mean + server error, into the error buffer and back into the LDS tile; marked if at or above the floor
    uint32_t take_mask = 0;
#pragma unroll
    for (int r = 0; r < kTileRows; ++r) {
        const int local = threadIdx.x * 4 + r * kRowStride;
        const int64_t off = tile_lo + local;
        if (off >= L) continue;
        const f32x4 sums = *reinterpret_cast<const f32x4*>(&acc[local]);
        f32x4 ubar;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float mean = sums[c] * inv_n;
            const float stored = ve[r][c];
            ubar[c] = mean + deferred_error(stored, static_cast<uint32_t>(off + c), keep);
            const float value = ubar[c];
            take_mask |= key_of(value) >= floor_key ? 1u << (4 * r + c) : 0u;
        }
        *reinterpret_cast<f32x4*>(&acc[local]) = ubar;
        store_stream(serr + tr.base + off, ubar);
    }
    const int64_t tile_id = tr.pair * tiles_per_chunk + tr.tile;
    const uint32_t marked = count_and_slot_marked(acc, take_mask, lds_scan, lds_window, pair_hist, guessed,
                                                  slots + tile_id * slots_per_tile, slots_per_tile);
    if (threadIdx.x == 0) {
        tile_split[tile_id] = marked;
        if (marked > static_cast<uint32_t>(slots_per_tile)) state[tr.pair * kTopkStateWords + kStResplit] = 1u;
    }
    flush_window(lds_window, pair_hist, guessed);
}

// ------------------------------------------------------------------------
// Radix select: pick the bin that holds the wanted element, refine the histogram inside it.
// ------------------------------------------------------------------------

// One workgroup per pair.  Scans the level's histogram (from the top bin down for keys, from bin 0 up for
// indices) to the bin where the running count reaches `remaining`, records it in the state and clears the
// histogram for the next level.
// only_rehist: the second level-0 pick of a call, for the pairs whose first histogram fell short (kStRehist:
// the floor they were counted and slotted on was too high, so their slots are filled again).
// At key level 2 with a guess table: leaves the floor of the next call's first pass (see kGuessMarginMax).
template <bool kIdx>
__global__ __launch_bounds__(kThreads) void topk_pick_kernel(uint32_t* __restrict__ hist, uint32_t* __restrict__ state,
                                                             int level, uint32_t K, uint32_t* __restrict__ guess,
                                                             uint32_t* __restrict__ last_T, bool only_rehist) {
    __shared__ uint32_t lds[kWaves];
    const int64_t pair = blockIdx.x;
    uint32_t* h = hist + pair * kTopkBins;
    uint32_t* st = state + pair * kTopkStateWords;
    if (only_rehist && st[kStRehist] == 0u) return;            // whole workgroup
    if (kIdx && st[kStTieDone] != 0u) return;                  // topk_resolve_kernel has settled kStIdxT
    const bool tie_needed = kIdx ? (st[kStTieNeeded] != 0u) : true;
    if (kIdx && !tie_needed) {                                 // every element equal to T is kept
        if (level == 2 && threadIdx.x == 0) st[kStIdxT] = 0xFFFFFFFFu;
        return;                                                // the histogram was never filled: still zero
    }
    const Level lv = kIdx ? idx_level(level) : key_level(level);
    const int nb = 1 << lv.bits;
    const uint32_t remaining = kIdx ? st[kStIdxRemaining] : (level == 0 ? K : st[kStRemaining]);
    const uint32_t prefix = level == 0 ? 0u : (kIdx ? st[kStIdxPrefix] : st[kStPrefix]);
    constexpr int kPer = kTopkBins / kThreads;                 // scan positions per thread
    uint32_t cnt[kPer];
    uint32_t mine = 0;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
        const int pos = threadIdx.x * kPer + q;                // position in scan order
        const int bin = kIdx ? pos : nb - 1 - pos;
        cnt[q] = (pos < nb) ? h[bin] : 0u;
        mine += cnt[q];
    }
    uint32_t total;
    const uint32_t before_me = block_exclusive_scan_u32(mine, lds, total);   // contains __syncthreads
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
        const int pos = threadIdx.x * kPer + q;
        if (pos < nb) h[kIdx ? pos : nb - 1 - pos] = 0u;
    }
    if (!kIdx && level == 0 && !only_rehist && total < remaining) {
        // the elements the first pass counted (those at or above its floor) do not reach down to the K-th largest
        // key: the whole level-0 histogram is needed (topk_key_hist_walk_kernel, then this kernel again)
        if (threadIdx.x == 0) st[kStRehist] = 1u;
        return;
    }
    if (before_me < remaining && remaining <= before_me + mine) {           // exactly one thread
        uint32_t before = before_me;
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            if (before < remaining && remaining <= before + cnt[q]) {
                const int pos = threadIdx.x * kPer + q;
                const uint32_t bin = static_cast<uint32_t>(kIdx ? pos : nb - 1 - pos);
                const uint32_t new_prefix = prefix | (bin << lv.shift);
                const uint32_t left = remaining - before;      // still to take from inside this bin
                if (kIdx) {
                    st[kStIdxPrefix] = new_prefix;
                    st[kStIdxRemaining] = left;
                    if (level == 2) st[kStIdxT] = new_prefix;
                } else {
                    st[kStPrefix] = new_prefix;
                    st[kStRemaining] = left;
                    if (level == 0 && only_rehist) st[kStResplit] = 1u;
                    if (level == 2) {
                        if (guess) {
                            const uint32_t before = last_T[pair], floor_before = guess[pair];   // 0xFFFFFFFF: no call before
                            uint32_t margin = kGuessMarginMax;
                            if (before != 0xFFFFFFFFu && floor_before <= before && st[kStRehist] == 0u) {
                                const uint32_t fell = before > new_prefix ? before - new_prefix : 0u;
                                const uint32_t wanted = fell < kGuessMarginMax / kGuessMarginPerFall ? kGuessMarginPerFall * fell
                                                                                                     : kGuessMarginMax;
                                margin = min(kGuessMarginMax, max(kGuessMarginMin, max(wanted, (before - floor_before) / 2u)));
                            }
                            guess[pair] = new_prefix > margin ? new_prefix - margin : 0u;
                            last_T[pair] = new_prefix;
                        }
                        st[kStKeyT] = new_prefix;
                        st[kStCountEq] = cnt[q];
                        st[kStTieNeeded] = (left < cnt[q]) ? 1u : 0u;
                        st[kStIdxPrefix] = 0u;
                        st[kStIdxRemaining] = left;
                    }
                }
            }
            before += cnt[q];
        }
    }
}

// Histogram of the next radix digit of the elements of one tile that lie inside the current prefix.
template <bool kIdx>
__device__ __forceinline__ void hist_tile(const float* __restrict__ buf, uint32_t* __restrict__ h, int64_t base,
                                          int64_t tile_lo, int64_t L, Level lv, uint32_t prefix, uint32_t T) {
    const uint32_t digit_mask = (1u << lv.bits) - 1u;
#pragma unroll
    for (int r = 0; r < kTileRows; ++r) {
        const int64_t off = tile_lo + threadIdx.x * 4 + r * kRowStride;
        const bool valid = off < L;                            // no branch: every lane takes part in the ballots
        f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
        if (valid) v = load_stream(buf + base + off);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t key = key_of(v[c]);
            const uint32_t j = static_cast<uint32_t>(off + c);
            bool active;
            uint32_t bin;
            if (kIdx) {
                active = valid && key == T && (j & lv.match_mask) == prefix;
                bin = (j >> lv.shift) & digit_mask;
            } else {
                active = valid && (key & lv.match_mask) == prefix;
                bin = (key >> lv.shift) & digit_mask;
            }
            hist_add_aggregated(h, active, bin);
        }
    }
}

// The kernels for the rare cases (ties to break, pairs that overflowed their slots) run on a small grid in
// which every workgroup visits the flagged pairs and strides over their tiles.  The flags are read kThreads
// pairs at a time, one per thread, so a launch with nothing to do costs one state read per thread.  A pair
// is flagged if both state words named are non-zero (name one word twice to test it alone).
// `body(pair)` may contain workgroup barriers: all threads see the same flags.
template <class Body>
__device__ __forceinline__ void for_flagged_pairs(const uint32_t* __restrict__ state, int64_t pairs, int flag_word,
                                                  int second_flag_word, Body body) {
    __shared__ uint32_t flags[kThreads];
    for (int64_t p0 = 0; p0 < pairs; p0 += kThreads) {
        const int64_t p = p0 + threadIdx.x;
        const uint32_t mine = (p < pairs && state[p * kTopkStateWords + flag_word] != 0u &&
                               state[p * kTopkStateWords + second_flag_word] != 0u) ? 1u : 0u;
        if (!__syncthreads_or(mine != 0u)) continue;           // same answer in every thread
        flags[threadIdx.x] = mine;
        __syncthreads();
        for (int q = 0; q < kThreads; ++q)
            if (flags[q] != 0u) body(p0 + q);
        __syncthreads();                                       // before the next round overwrites the flags
    }
}

// The whole level-0 histogram of the pairs marked kStRehist (their first pass counted only the bins at or
// above a guess that proved too high, or had no guess to go by), from the buffer: per-element LDS atomics,
// one flush per workgroup and pair.  topk_pick_kernel has cleared those pairs' histograms.
__global__ __launch_bounds__(kThreads) void topk_rehist_kernel(const float* __restrict__ buf, uint32_t* __restrict__ hist,
                                                               const uint32_t* __restrict__ state, int64_t d, int64_t L,
                                                               int32_t C, int64_t pairs, int32_t tiles_per_chunk) {
    __shared__ uint32_t lds_hist[kTopkBins];
    for_flagged_pairs(state, pairs, kStRehist, kStRehist, [&](int64_t pair) {
        for (int b = threadIdx.x; b < kTopkBins; b += kThreads) lds_hist[b] = 0u;
        __syncthreads();
        const int64_t slice = pair / C;
        const int64_t base = slice * d + (pair - slice * C) * L;
        for (int64_t tile = blockIdx.x; tile < tiles_per_chunk; tile += gridDim.x) {
#pragma unroll
            for (int r = 0; r < kTileRows; ++r) {
                const int64_t off = tile * kTopkTile + threadIdx.x * 4 + r * kRowStride;
                if (off >= L) continue;
                const f32x4 v = load_stream(buf + base + off);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float value = v[c];
                    atomicAdd(&lds_hist[key_of(value) >> 20], 1u);
                }
            }
        }
        __syncthreads();
        flush_histogram(lds_hist, hist + pair * kTopkBins);
        __syncthreads();                                       // before the next pair clears the LDS histogram
    });
}

// After the level-0 pick, for the pairs marked kStResplit (every pair of a call that had no guess to go by):
// fill the slots of every tile from the buffer, by the level-0 digit b0 of T.  Elements above b0 (kept
// whatever T turns out to be) and inside b0 (candidates) are copied, everything below b0 is dropped for
// certain.  With K at 1 % of a chunk that is under 2 % of the elements.  A tile with more such elements than
// slots stores the first `slots_per_tile` of them and flags its pair kStOverflow, which then takes full
// passes over the buffer.
__global__ __launch_bounds__(kThreads) void topk_split_kernel(const float* __restrict__ buf, uint32_t* __restrict__ state,
                                                              uint32_t* __restrict__ tile_split,
                                                              uint2* __restrict__ slots, int32_t slots_per_tile,
                                                              int64_t d, int64_t L, int32_t C, int64_t pairs,
                                                              int32_t tiles_per_chunk) {
    __shared__ uint64_t lds[kWaves];
    for_flagged_pairs(state, pairs, kStResplit, kStResplit, [&](int64_t pair) {
        uint32_t* st = state + pair * kTopkStateWords;
        const uint32_t b0 = st[kStPrefix] & kTopMask;
        const int64_t slice = pair / C;
        const int64_t base = slice * d + (pair - slice * C) * L;
        for (int64_t tile = blockIdx.x; tile < tiles_per_chunk; tile += gridDim.x) {
            f32x4 v[kTileRows];
            uint32_t take_mask = 0;                            // bit 4*r + c: element c of row r goes to a slot
            uint64_t packed = 0;
#pragma unroll
            for (int r = 0; r < kTileRows; ++r) {
                const int64_t off = tile * kTopkTile + threadIdx.x * 4 + r * kRowStride;
                v[r] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                if (off < L) {
                    v[r] = load_stream(buf + base + off);
                    uint32_t count = 0;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        if ((key_of(v[r][c]) & kTopMask) >= b0) {
                            take_mask |= 1u << (4 * r + c);
                            ++count;
                        }
                    }
                    packed |= static_cast<uint64_t>(count) << (16 * r);
                }
            }
            const int64_t tile_id = pair * tiles_per_chunk + tile;
            const uint32_t marked = write_tile_slots(v, take_mask, packed, lds, slots + tile_id * slots_per_tile,
                                                     slots_per_tile);     // barriers: uniform trip counts
            if (threadIdx.x == 0) {
                tile_split[tile_id] = marked;
                if (marked > static_cast<uint32_t>(slots_per_tile)) st[kStOverflow] = 1u;
            }
        }
    });
}

// The kernels that read the slots take a block of consecutive tiles of one pair per workgroup.  Walking the
// tiles one after the other is a chain of dependent loads per tile (how many slots it filled, then the
// slots), and a tile fills about a hundred slots: too little per step to hide that latency.  So the
// workgroup first reads all its tiles' counts into LDS with one load per thread, and then every wave takes
// kSlotUnroll tiles at a time and requests the first 2 * 64 slots of all of them before it looks at any.
constexpr int kSlotUnroll = 4;
constexpr int kSlotDepth = 2;                                 // 64-entry rounds requested up front per tile

// counts[q] = filled slots of tile t0 + q of the pair (0 beyond the pair's last tile), for q < block_tiles
// <= kThreads.  Ends with a workgroup barrier.
__device__ __forceinline__ void load_slot_counts(const uint32_t* __restrict__ tile_split, int32_t slots_per_tile,
                                                 int64_t pair, int32_t t0, int32_t tiles_per_chunk, int block_tiles,
                                                 uint32_t* counts /* LDS */) {
    if (static_cast<int>(threadIdx.x) < block_tiles) {
        const int32_t tile = t0 + static_cast<int32_t>(threadIdx.x);
        counts[threadIdx.x] = tile < tiles_per_chunk
                                  ? min(tile_split[pair * tiles_per_chunk + tile], static_cast<uint32_t>(slots_per_tile))
                                  : 0u;
    }
    __syncthreads();
}

// For the tiles q = first, first + 1, ... < first + kSlotUnroll of the block (q indexes `counts`): calls
// visit(q, e, entry, valid) for every 64-entry round of every tile, in slot order per tile, by all 64 lanes
// (valid = false for lanes beyond the tile's count), so visit may vote across the wave.
template <class Visit>
__device__ __forceinline__ void for_slots_of_tiles(const uint2* __restrict__ slots, int32_t slots_per_tile,
                                                   int64_t tile_id0 /* of q = 0 */, const uint32_t* counts, int first,
                                                   Visit visit) {
    const uint32_t lane = threadIdx.x & (kWaveSize - 1);
    uint32_t cnt[kSlotUnroll];
    uint2 entry[kSlotUnroll][kSlotDepth];
#pragma unroll
    for (int u = 0; u < kSlotUnroll; ++u) {
        cnt[u] = counts[first + u];
        const uint2* mine = slots + (tile_id0 + first + u) * slots_per_tile;
#pragma unroll
        for (int h = 0; h < kSlotDepth; ++h) {
            const uint32_t e = lane + h * kWaveSize;
            entry[u][h] = make_uint2(0u, 0u);
            if (e < cnt[u]) entry[u][h] = mine[e];
        }
    }
#pragma unroll
    for (int u = 0; u < kSlotUnroll; ++u) {
#pragma unroll
        for (int h = 0; h < kSlotDepth; ++h) {
            const uint32_t e = lane + h * kWaveSize;
            if (static_cast<uint32_t>(h * kWaveSize) < cnt[u]) visit(first + u, e, entry[u][h], e < cnt[u]);   // wave-uniform test
        }
        const uint2* mine = slots + (tile_id0 + first + u) * slots_per_tile;
        for (uint32_t e0 = kSlotDepth * kWaveSize; e0 < cnt[u]; e0 += kWaveSize) {   // a tile with more entries: rare
            const uint32_t e = e0 + lane;
            uint2 late = make_uint2(0u, 0u);
            if (e < cnt[u]) late = mine[e];
            visit(first + u, e, late, e < cnt[u]);
        }
    }
}

// Key levels 1 and 2 (kIdx = false) and the index levels of the tie selection (kIdx = true: only pairs with
// a tie to break) from the slots.  One workgroup takes kCandTilesPerBlock consecutive tiles of one pair,
// kCandSubBlock at a time, accumulates the level's digit histogram in LDS and flushes it once (one
// device-wide atomic per populated bin: level 1 populates nearly all of them, hence the large blocks).
constexpr int kCandSubBlock = 256;
constexpr int kCandTilesPerBlock = 256;                      // key levels
constexpr int kTieTilesPerBlock = 256;                       // tie levels: few pairs, few matches: more workgroups each
static_assert(kCandSubBlock <= kThreads && kCandSubBlock % (kWaves * kSlotUnroll) == 0 &&
              kCandTilesPerBlock % kCandSubBlock == 0 && kTieTilesPerBlock % kCandSubBlock == 0, "tile blocks");
template <bool kIdx>
__global__ __launch_bounds__(kThreads) void topk_cand_hist_kernel(const uint2* __restrict__ slots, int32_t slots_per_tile,
                                                                  const uint32_t* __restrict__ tile_split,
                                                                  uint32_t* __restrict__ hist,
                                                                  const uint32_t* __restrict__ state,
                                                                  int32_t tiles_per_chunk, int32_t blocks_per_pair,
                                                                  int level) {
    __shared__ uint32_t lds_hist[kTopkBins];
    __shared__ uint32_t lds_count[kCandSubBlock];
    const int64_t pair = blockIdx.x / blocks_per_pair;
    const int32_t b = static_cast<int32_t>(blockIdx.x - pair * blocks_per_pair);
    const uint32_t* st = state + pair * kTopkStateWords;
    if (st[kStOverflow] != 0u) return;                         // whole workgroup: the full passes take this pair
    if (kIdx && (st[kStTieNeeded] == 0u || st[kStTieDone] != 0u)) return;
    for (int q = threadIdx.x; q < kTopkBins; q += kThreads) lds_hist[q] = 0u;
    const Level lv = kIdx ? idx_level(level) : key_level(level);
    const uint32_t digit_mask = (1u << lv.bits) - 1u;
    const uint32_t prefix = kIdx ? (level == 0 ? 0u : st[kStIdxPrefix]) : st[kStPrefix];
    const uint32_t T = st[kStKeyT];                            // final only when kIdx
    const int wave = threadIdx.x >> 6;
    constexpr int kBlockTiles = kIdx ? kTieTilesPerBlock : kCandTilesPerBlock;
    const int32_t block_end = min((b + 1) * kBlockTiles, tiles_per_chunk);
    for (int32_t t0 = b * kBlockTiles; t0 < block_end; t0 += kCandSubBlock) {
        load_slot_counts(tile_split, slots_per_tile, pair, t0, tiles_per_chunk, kCandSubBlock, lds_count);   // barrier
        const int sub_tiles = min(kCandSubBlock, tiles_per_chunk - t0);
        for (int first = wave * kSlotUnroll; first < sub_tiles; first += kWaves * kSlotUnroll) {
            for_slots_of_tiles(slots, slots_per_tile, pair * tiles_per_chunk + t0, lds_count, first,
                               [&](int q, uint32_t, uint2 entry, bool valid) {
                                   const uint32_t key = entry.y & 0x7FFFFFFFu;
                                   if (kIdx) {
                                       const uint32_t j = static_cast<uint32_t>(t0 + q) * kTopkTile + entry.x;
                                       if (valid && key == T && (j & lv.match_mask) == prefix)
                                           atomicAdd(&lds_hist[(j >> lv.shift) & digit_mask], 1u);
                                   } else {
                                       if (valid && (key & lv.match_mask) == prefix)
                                           atomicAdd(&lds_hist[(key >> lv.shift) & digit_mask], 1u);
                                   }
                               });
        }
        __syncthreads();                                       // before the next round overwrites the counts
    }
    flush_histogram(lds_hist, hist + pair * kTopkBins);
}

// Key level 2 from the slots, and with it everything the rest of the selection needs from them.  The level-1
// pick has fixed the top 22 bits of the threshold T; of a chunk's slot entries a few dozen share them (the
// "near" entries), the others lie above (kept whatever the last 9 bits of T turn out to be) or below.  This
// pass builds the level-2 histogram of the near entries, appends them to the pair's near list (in any order:
// a counter in the state, entries beyond the list's capacity are only counted) and leaves the number of
// entries above in tile_counts.  Ties at T and the kept elements among the near entries are then settled
// from the list by topk_resolve_kernel, without further passes over the slots.
__global__ __launch_bounds__(kThreads) void topk_near_kernel(const uint2* __restrict__ slots, int32_t slots_per_tile,
                                                             const uint32_t* __restrict__ tile_split,
                                                             uint32_t* __restrict__ hist, uint32_t* __restrict__ state,
                                                             uint32_t* __restrict__ tile_counts,
                                                             uint2* __restrict__ near, int32_t tiles_per_chunk,
                                                             int32_t blocks_per_pair) {
    constexpr Level lv = key_level(2);
    constexpr int kBins = 1 << lv.bits;
    __shared__ uint32_t lds_hist[kBins];
    __shared__ uint32_t lds_count[kCandSubBlock];
    const int64_t pair = blockIdx.x / blocks_per_pair;
    const int32_t b = static_cast<int32_t>(blockIdx.x - pair * blocks_per_pair);
    uint32_t* st = state + pair * kTopkStateWords;
    if (st[kStOverflow] != 0u) return;                         // whole workgroup: the full passes take this pair
    for (int q = threadIdx.x; q < kBins; q += kThreads) lds_hist[q] = 0u;
    const uint32_t prefix = st[kStPrefix];
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    uint2* my_near = near + pair * kTopkNearCap;
    const int32_t block_end = min((b + 1) * kCandTilesPerBlock, tiles_per_chunk);
    for (int32_t t0 = b * kCandTilesPerBlock; t0 < block_end; t0 += kCandSubBlock) {
        load_slot_counts(tile_split, slots_per_tile, pair, t0, tiles_per_chunk, kCandSubBlock, lds_count);   // barrier
        const int sub_tiles = min(kCandSubBlock, tiles_per_chunk - t0);
        for (int first = wave * kSlotUnroll; first < sub_tiles; first += kWaves * kSlotUnroll) {
            uint32_t above[kSlotUnroll] = {};
            for_slots_of_tiles(slots, slots_per_tile, pair * tiles_per_chunk + t0, lds_count, first,
                               [&](int q, uint32_t, uint2 entry, bool valid) {
                                   const uint32_t key = entry.y & 0x7FFFFFFFu;
                                   const uint32_t top = key & lv.match_mask;
                                   above[q - first] += static_cast<uint32_t>(__popcll(static_cast<unsigned long long>(__ballot(valid && top > prefix))));
                                   if (valid && top == prefix) {
                                       atomicAdd(&lds_hist[key & (kBins - 1)], 1u);
                                       const uint32_t at = atomicAdd(&st[kStNearCount], 1u);
                                       if (at < static_cast<uint32_t>(kTopkNearCap))
                                           my_near[at] = make_uint2(static_cast<uint32_t>(t0 + q) * kTopkTile + entry.x, key);
                                   }
                               });
#pragma unroll
            for (int u = 0; u < kSlotUnroll; ++u)
                if (lane == 0 && first + u < sub_tiles) tile_counts[pair * tiles_per_chunk + t0 + first + u] = above[u];
        }
        __syncthreads();                                       // before the next round overwrites the counts
    }
    flush_histogram(lds_hist, hist + pair * kTopkBins, kBins);
}

// After the level-2 pick, one workgroup per pair: with T known, settles from the near list (i) the tie rule -
// if only `left` of the elements equal to T may be kept, kStIdxT becomes the left-th smallest index among
// them - and (ii) the per-tile kept counts, by adding the near entries that are kept to the counts of
// entries above that topk_near_kernel left.  A pair whose near list overflowed is flagged instead and takes
// the tie levels and the counts from the slots (topk_cand_hist_kernel<true>, topk_slot_count_kernel).
__global__ __launch_bounds__(kThreads) void topk_resolve_kernel(uint32_t* __restrict__ state,
                                                                const uint2* __restrict__ near,
                                                                uint32_t* __restrict__ tile_counts,
                                                                int32_t tiles_per_chunk) {
    __shared__ uint2 lds_near[kTopkNearCap];
    __shared__ uint32_t lds_idxT;
    const int64_t pair = blockIdx.x;
    uint32_t* st = state + pair * kTopkStateWords;
    if (st[kStOverflow] != 0u) return;                         // whole workgroup: the full passes take this pair
    const uint32_t count = st[kStNearCount];
    if (count > static_cast<uint32_t>(kTopkNearCap)) {
        if (threadIdx.x == 0) st[kStNearOverflow] = 1u;
        return;
    }
    const uint32_t T = st[kStKeyT], left = st[kStIdxRemaining];
    const bool tie_needed = st[kStTieNeeded] != 0u;
    for (uint32_t i = threadIdx.x; i < count; i += kThreads) lds_near[i] = near[pair * kTopkNearCap + i];
    if (threadIdx.x == 0) lds_idxT = 0xFFFFFFFFu;              // every element equal to T is kept
    __syncthreads();
    if (tie_needed) {
        for (uint32_t i = threadIdx.x; i < count; i += kThreads) {
            const uint2 mine = lds_near[i];
            if (mine.y != T) continue;
            uint32_t before = 0;                               // elements equal to T at lower indices
            for (uint32_t k = 0; k < count; ++k) {
                const uint2 other = lds_near[k];
                before += (other.y == T && other.x < mine.x) ? 1u : 0u;
            }
            if (before + 1u == left) lds_idxT = mine.x;        // indices are distinct: exactly one thread
        }
        __syncthreads();
    }
    const uint32_t idxT = lds_idxT;
    if (threadIdx.x == 0) {
        st[kStIdxT] = idxT;
        st[kStTieDone] = 1u;
    }
    for (uint32_t i = threadIdx.x; i < count; i += kThreads) {
        const uint2 mine = lds_near[i];
        if (kept(mine.y, mine.x, T, idxT)) atomicAdd(&tile_counts[pair * tiles_per_chunk + mine.x / kTopkTile], 1u);
    }
}

// Key levels 1 and 2 for pairs that overflowed their slots: full passes over the buffer.
__global__ __launch_bounds__(kThreads) void topk_key_hist_walk_kernel(const float* __restrict__ buf,
                                                                      uint32_t* __restrict__ hist,
                                                                      const uint32_t* __restrict__ state, int64_t d,
                                                                      int64_t L, int32_t C, int64_t pairs,
                                                                      int32_t tiles_per_chunk, int level) {
    for_flagged_pairs(state, pairs, kStOverflow, kStOverflow, [&](int64_t pair) {
        const uint32_t* st = state + pair * kTopkStateWords;
        const int64_t slice = pair / C;
        const int64_t base = slice * d + (pair - slice * C) * L;
        for (int64_t tile = blockIdx.x; tile < tiles_per_chunk; tile += gridDim.x)
            hist_tile<false>(buf, hist + pair * kTopkBins, base, tile * kTopkTile, L, key_level(level), st[kStPrefix], 0u);
    });
}

// Index (tie) levels for pairs that overflowed their slots, from the buffer.  Tiles outside the index range
// of the current prefix are skipped.
__global__ __launch_bounds__(kThreads) void topk_tie_hist_kernel(const float* __restrict__ buf, uint32_t* __restrict__ hist,
                                                                 const uint32_t* __restrict__ state, int64_t d, int64_t L,
                                                                 int32_t C, int64_t pairs, int32_t tiles_per_chunk,
                                                                 int level) {
    const Level lv = idx_level(level);
    for_flagged_pairs(state, pairs, kStTieNeeded, kStOverflow, [&](int64_t pair) {
        const uint32_t* st = state + pair * kTopkStateWords;
        const uint32_t prefix = level == 0 ? 0u : st[kStIdxPrefix];
        const uint32_t T = st[kStKeyT];
        const int64_t slice = pair / C;
        const int64_t base = slice * d + (pair - slice * C) * L;
        // tiles that intersect the index range [prefix, prefix + span) of the current prefix
        int64_t first = 0, last = tiles_per_chunk;
        if (level > 0) {
            const int64_t span = int64_t{1} << idx_level(level - 1).shift;
            first = static_cast<int64_t>(prefix) / kTopkTile;
            last = min(static_cast<int64_t>(tiles_per_chunk), (static_cast<int64_t>(prefix) + span + kTopkTile - 1) / kTopkTile);
        }
        for (int64_t tile = first + blockIdx.x; tile < last; tile += gridDim.x)
            hist_tile<true>(buf, hist + pair * kTopkBins, base, tile * kTopkTile, L, lv, prefix, T);
    });
}

// ------------------------------------------------------------------------
// Emission in index order: per-tile counts, scan, write.
// ------------------------------------------------------------------------
// Kept elements per tile, from the tile's slots (entries above the level-0 bin of T pass the test by
// themselves), for the pairs whose near list overflowed.  One workgroup per block of kEmitTilesPerBlock
// consecutive tiles of one pair.
constexpr int kEmitTilesPerBlock = 64;
static_assert(kEmitTilesPerBlock <= kThreads && kEmitTilesPerBlock % (kWaves * kSlotUnroll) == 0, "tile blocks");
__global__ __launch_bounds__(kThreads) void topk_slot_count_kernel(const uint2* __restrict__ slots, int32_t slots_per_tile,
                                                                   const uint32_t* __restrict__ tile_split,
                                                                   const uint32_t* __restrict__ state,
                                                                   uint32_t* __restrict__ tile_counts,
                                                                   int32_t tiles_per_chunk, int32_t blocks_per_pair) {
    __shared__ uint32_t lds_count[kEmitTilesPerBlock];
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t pair = blockIdx.x / blocks_per_pair;
    const int32_t t0 = static_cast<int32_t>(blockIdx.x - pair * blocks_per_pair) * kEmitTilesPerBlock;
    const uint32_t* st = state + pair * kTopkStateWords;
    if (st[kStOverflow] != 0u) return;                         // whole workgroup: topk_count_walk_kernel takes this pair
    if (st[kStNearOverflow] == 0u) return;                     // topk_resolve_kernel has settled the counts
    const uint32_t T = st[kStKeyT], idxT = st[kStIdxT];
    load_slot_counts(tile_split, slots_per_tile, pair, t0, tiles_per_chunk, kEmitTilesPerBlock, lds_count);
    const int block_tiles = min(kEmitTilesPerBlock, tiles_per_chunk - t0);
    for (int first = wave * kSlotUnroll; first < block_tiles; first += kWaves * kSlotUnroll) {
        uint32_t kept_in[kSlotUnroll] = {};
        for_slots_of_tiles(slots, slots_per_tile, pair * tiles_per_chunk + t0, lds_count, first,
                           [&](int q, uint32_t, uint2 entry, bool valid) {
                               const uint32_t j = static_cast<uint32_t>(t0 + q) * kTopkTile + entry.x;
                               const bool keep = valid && kept(entry.y & 0x7FFFFFFFu, j, T, idxT);
                               kept_in[q - first] += static_cast<uint32_t>(__popcll(static_cast<unsigned long long>(__ballot(keep))));
                           });
#pragma unroll
        for (int u = 0; u < kSlotUnroll; ++u)
            if (lane == 0 && first + u < block_tiles) tile_counts[pair * tiles_per_chunk + t0 + first + u] = kept_in[u];
    }
}

// The same from the buffer, for pairs that overflowed their slots.
__global__ __launch_bounds__(kThreads) void topk_count_walk_kernel(const float* __restrict__ buf,
                                                                   const uint32_t* __restrict__ state,
                                                                   uint32_t* __restrict__ tile_counts, int64_t d,
                                                                   int64_t L, int32_t C, int64_t pairs,
                                                                   int32_t tiles_per_chunk) {
    __shared__ uint32_t lds[kWaves];
    for_flagged_pairs(state, pairs, kStOverflow, kStOverflow, [&](int64_t pair) {
        const uint32_t* st = state + pair * kTopkStateWords;
        const uint32_t T = st[kStKeyT], idxT = st[kStIdxT];
        const int64_t slice = pair / C;
        const int64_t base = slice * d + (pair - slice * C) * L;
        for (int64_t tile = blockIdx.x; tile < tiles_per_chunk; tile += gridDim.x) {
            uint32_t mine = 0;
#pragma unroll
            for (int r = 0; r < kTileRows; ++r) {
                const int64_t off = tile * kTopkTile + threadIdx.x * 4 + r * kRowStride;
                if (off >= L) continue;
                const f32x4 v = load_stream(buf + base + off);
#pragma unroll
                for (int c = 0; c < 4; ++c) mine += kept(key_of(v[c]), static_cast<uint32_t>(off + c), T, idxT) ? 1u : 0u;
            }
            uint32_t total;
            (void)block_exclusive_scan_u32(mine, lds, total);     // contains __syncthreads: uniform trip counts
            if (threadIdx.x == 0) tile_counts[pair * tiles_per_chunk + tile] = total;
        }
    });
}

// One workgroup per pair: tile_counts -> exclusive offsets, in place.
__global__ __launch_bounds__(kThreads) void topk_scan_kernel(uint32_t* __restrict__ tile_counts, int32_t tiles_per_chunk) {
    __shared__ uint32_t lds[kWaves];
    uint32_t* tc = tile_counts + static_cast<int64_t>(blockIdx.x) * tiles_per_chunk;
    uint32_t carry = 0;
    for (int32_t t0 = 0; t0 < tiles_per_chunk; t0 += kThreads) {
        const int32_t t = t0 + threadIdx.x;
        const uint32_t c = t < tiles_per_chunk ? tc[t] : 0u;
        uint32_t total;
        const uint32_t before = block_exclusive_scan_u32(c, lds, total);
        if (t < tiles_per_chunk) tc[t] = carry + before;
        carry += total;
    }
}

// Writes the kept elements of a tile to the pair's (idx, val) list at the tile's offset, in index order,
// and (zero_kept) zeroes them in the buffer: what stays there is u - C[u].  From the slots (already in index
// order): a ballot over 64 entries at a time ranks the kept ones.  Workgroups as in topk_slot_count_kernel.
__global__ __launch_bounds__(kThreads) void topk_slot_emit_kernel(float* __restrict__ buf, const uint2* __restrict__ slots,
                                                                  int32_t slots_per_tile,
                                                                  const uint32_t* __restrict__ tile_split,
                                                                  const uint32_t* __restrict__ state,
                                                                  const uint32_t* __restrict__ tile_offsets,
                                                                  uint32_t* __restrict__ idx, float* __restrict__ val,
                                                                  int64_t d, int64_t L, int32_t C,
                                                                  int32_t tiles_per_chunk, int32_t blocks_per_pair,
                                                                  int64_t K, bool zero_kept) {
    __shared__ uint32_t lds_count[kEmitTilesPerBlock];
    __shared__ uint32_t lds_offset[kEmitTilesPerBlock];
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t pair = blockIdx.x / blocks_per_pair;
    const int32_t t0 = static_cast<int32_t>(blockIdx.x - pair * blocks_per_pair) * kEmitTilesPerBlock;
    const uint32_t* st = state + pair * kTopkStateWords;
    if (st[kStOverflow] != 0u) return;                         // whole workgroup: topk_emit_walk_kernel takes this pair
    const uint32_t T = st[kStKeyT], idxT = st[kStIdxT];
    const int64_t slice = pair / C;
    float* chunk_buf = buf + slice * d + (pair - slice * C) * L;
    uint32_t* out_idx = idx + pair * K;
    float* out_val = val + pair * K;
    if (threadIdx.x < kEmitTilesPerBlock) {                    // list position of each tile's first kept element
        const int32_t tile = t0 + static_cast<int32_t>(threadIdx.x);
        lds_offset[threadIdx.x] = tile < tiles_per_chunk ? tile_offsets[pair * tiles_per_chunk + tile] : 0u;
    }
    load_slot_counts(tile_split, slots_per_tile, pair, t0, tiles_per_chunk, kEmitTilesPerBlock, lds_count);
    const int block_tiles = min(kEmitTilesPerBlock, tiles_per_chunk - t0);
    for (int first = wave * kSlotUnroll; first < block_tiles; first += kWaves * kSlotUnroll) {
        uint32_t done[kSlotUnroll];
#pragma unroll
        for (int u = 0; u < kSlotUnroll; ++u) done[u] = lds_offset[first + u];
        for_slots_of_tiles(slots, slots_per_tile, pair * tiles_per_chunk + t0, lds_count, first,
                           [&](int q, uint32_t, uint2 entry, bool valid) {
                               const uint32_t j = static_cast<uint32_t>(t0 + q) * kTopkTile + entry.x;   // chunk-local index
                               const bool keep = valid && j < L && kept(entry.y & 0x7FFFFFFFu, j, T, idxT);
                               const uint64_t votes = __ballot(keep);
                               uint32_t& next = done[q - first];
                               if (keep) {
                                   const uint32_t rank = next + static_cast<uint32_t>(__popcll(static_cast<unsigned long long>(votes & ((uint64_t{1} << lane) - 1))));
                                   if (rank < K) {             // holds by construction; guards the list bounds
                                       out_idx[rank] = j;
                                       const uint32_t bits = entry.y;
                                       out_val[rank] = __builtin_bit_cast(float, bits);
                                   }
                                   if (zero_kept) chunk_buf[j] = 0.0f;
                               }
                               next += static_cast<uint32_t>(__popcll(static_cast<unsigned long long>(votes)));
                           });
    }
}

// The same from the buffer, for pairs that overflowed their slots.  Index order inside a tile is row by row
// (plain layout), thread by thread inside a row, ranked as in topk_split_kernel.
__global__ __launch_bounds__(kThreads) void topk_emit_walk_kernel(float* __restrict__ buf, const uint32_t* __restrict__ state,
                                                                  const uint32_t* __restrict__ tile_offsets,
                                                                  uint32_t* __restrict__ idx, float* __restrict__ val,
                                                                  int64_t d, int64_t L, int32_t C, int64_t pairs,
                                                                  int32_t tiles_per_chunk, int64_t K, bool zero_kept) {
    static_assert(kTileRows == 4 && kThreads * 4 < 65536, "four 16-bit row counters");
    __shared__ uint64_t lds[kWaves];
    for_flagged_pairs(state, pairs, kStOverflow, kStOverflow, [&](int64_t pair) {
        const uint32_t* st = state + pair * kTopkStateWords;
        const uint32_t T = st[kStKeyT], idxT = st[kStIdxT];
        const int64_t slice = pair / C;
        const int64_t base = slice * d + (pair - slice * C) * L;
        uint32_t* out_idx = idx + pair * K;
        float* out_val = val + pair * K;
        for (int64_t tile = blockIdx.x; tile < tiles_per_chunk; tile += gridDim.x) {
            const uint32_t tile_base = tile_offsets[pair * tiles_per_chunk + tile];
            f32x4 v[kTileRows];
            uint32_t keep_mask = 0;                            // bit 4*r + c: element c of row r is kept
            uint64_t packed = 0;
#pragma unroll
            for (int r = 0; r < kTileRows; ++r) {
                const int64_t off = tile * kTopkTile + threadIdx.x * 4 + r * kRowStride;
                v[r] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                if (off < L) {
                    v[r] = load_stream(buf + base + off);
                    uint32_t count = 0;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        if (kept(key_of(v[r][c]), static_cast<uint32_t>(off + c), T, idxT)) {
                            keep_mask |= 1u << (4 * r + c);
                            ++count;
                        }
                    }
                    packed |= static_cast<uint64_t>(count) << (16 * r);
                }
            }
            uint64_t totals;
            const uint64_t before = block_exclusive_scan_u64(packed, lds, totals);   // barriers: uniform trip counts
            uint32_t row_base = tile_base;
#pragma unroll
            for (int r = 0; r < kTileRows; ++r) {
                const int64_t off = tile * kTopkTile + threadIdx.x * 4 + r * kRowStride;
                uint32_t rank = row_base + static_cast<uint32_t>((before >> (16 * r)) & 0xFFFFu);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (keep_mask & (1u << (4 * r + c))) {
                        if (rank < K) {                        // holds by construction; guards the list bounds
                            out_idx[rank] = static_cast<uint32_t>(off + c);
                            out_val[rank] = v[r][c];
                        }
                        if (zero_kept) buf[base + off + c] = 0.0f;
                        ++rank;
                    }
                }
                row_base += static_cast<uint32_t>((totals >> (16 * r)) & 0xFFFFu);
            }
        }
    });
}

// ------------------------------------------------------------------------
// Gather + model update (Algorithm 1 lines 10-11) from the server's list.
// ------------------------------------------------------------------------
// One workgroup = one tile of ROWS * 1024 elements of ONE worker's momentum slice, slice-major like the
// 1-bit gather: the n slices are one long contiguous fill.  The tile's stretch of the list is staged
// through LDS (zero, scatter, read back as quads).
template <int ROWS, bool kWriteM, bool kModelStep>
__global__ __launch_bounds__(kThreads) void topk_apply_kernel(const uint32_t* __restrict__ sidx,
                                                              const float* __restrict__ sval,
                                                              const float* __restrict__ v, float* __restrict__ x,
                                                              float* __restrict__ m,
                                                              const uint32_t* __restrict__ offsets, int64_t d,
                                                              int64_t L, int32_t C, int32_t tiles_per_chunk,
                                                              int32_t K, float lr, float eps) {
    constexpr int kTile = ROWS * kRowStride;
    __shared__ float dense[kTile];
    const TileRef tr = tile_ref(d, L, C, tiles_per_chunk);    // pair = slice * C + chunk; slice 0 only if !kWriteM
    const int64_t slice = tr.pair / C;
    const int64_t chunk = tr.pair - slice * C;
    const int64_t tile_lo = tr.tile * kTile;
    for (int j = threadIdx.x; j < kTile; j += kThreads) dense[j] = 0.0f;
    const int64_t list = chunk * K;
    const uint32_t* off = offsets + chunk * tiles_per_chunk + tr.tile;
    const int last = min((tr.tile + 1 < tiles_per_chunk) ? static_cast<int>(off[1]) : K, K);   // min, first >= 0: no-ops
    const int first = max(static_cast<int>(off[0]), 0);                                       // for sorted lists
    __syncthreads();
    for (int t = first + threadIdx.x; t < last; t += kThreads) {
        const uint32_t j = sidx[list + t] - static_cast<uint32_t>(tile_lo);
        if (j < static_cast<uint32_t>(kTile)) dense[j] = sval[list + t];                 // always true for sorted lists
    }
    __syncthreads();
    const bool model_step = kModelStep && (slice == 0);
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int local = threadIdx.x * 4 + r * kRowStride;
        const int64_t off = tile_lo + local;
        if (off >= L) continue;
        const f32x4 mom = {dense[local], dense[local + 1], dense[local + 2], dense[local + 3]};
        if (kWriteM) store_stream(m + tr.base + off, mom);
        if (model_step) {
            const int64_t p = chunk * L + off;
            const f32x4 vv = load_stream(v + p), vx = load_stream(x + p);
            f32x4 xn;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float root = sqrtf(vv[c]);
                const float denom = root + eps;
                const float ratio = mom[c] / denom;
                const float step = lr * ratio;
                xn[c] = vx[c] - step;
            }
            store_stream(x + p, xn);
        }
    }
}

// End of a call that leaves its error buffer in deferred form: remember {T, idxT} of every pair.
__global__ __launch_bounds__(kThreads) void topk_save_keep_kernel(const uint32_t* __restrict__ state,
                                                                  uint2* __restrict__ keep, int64_t pairs) {
    const int64_t p = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (p < pairs) keep[p] = make_uint2(state[p * kTopkStateWords + kStKeyT], state[p * kTopkStateWords + kStIdxT]);
}

// apms_finalize on an error buffer in deferred form: zero the kept positions, which leaves v - C[v].
__global__ __launch_bounds__(kThreads) void topk_finalize_kernel(float* __restrict__ buf, const uint2* __restrict__ keep,
                                                                 int64_t d, int64_t L, int32_t C, int32_t tiles_per_chunk) {
    const TileRef tr = tile_ref(d, L, C, tiles_per_chunk);
    const uint2 k = keep[tr.pair];
#pragma unroll
    for (int r = 0; r < kTileRows; ++r) {
        const int64_t off = tr.tile * kTopkTile + threadIdx.x * 4 + r * kRowStride;
        if (off >= L) continue;
        const f32x4 v = load_stream(buf + tr.base + off);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float value = v[c];
            if (kept(key_of(value), static_cast<uint32_t>(off + c), k.x, k.y)) buf[tr.base + off + c] = 0.0f;
        }
    }
}

// Start of a call: clear the histograms and the per-pair flags.  resplit = 1 marks every pair for
// topk_split_kernel (calls whose first pass does not fill the slots).
__global__ __launch_bounds__(kThreads) void topk_begin_kernel(uint32_t* __restrict__ hist, int64_t count,
                                                              uint32_t* __restrict__ state, int64_t pairs,
                                                              uint32_t resplit) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < count; i += stride) hist[i] = 0u;
    for (int64_t p = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; p < pairs; p += stride) {
        state[p * kTopkStateWords + kStOverflow] = 0u;
        state[p * kTopkStateWords + kStResplit] = resplit;
        state[p * kTopkStateWords + kStRehist] = 0u;
        state[p * kTopkStateWords + kStNearCount] = 0u;
        state[p * kTopkStateWords + kStNearOverflow] = 0u;
        state[p * kTopkStateWords + kStTieDone] = 0u;
    }
}

#define APMS_RETURN_IF_ERROR()                 \
    do {                                       \
        const hipError_t e_ = hipGetLastError(); \
        if (e_ != hipSuccess) return e_;       \
    } while (0)

// The selection + emission over `slices` x C pairs of `buf` ([slices][d]) whose level-0 histogram is filled.
// `guess`, `last_T`: the per-pair tables of the first pass's floor and of the threshold found (see kGuessMarginMax).
// `save_keep`: null = eager (the kept positions of buf are zeroed); else the call leaves buf in deferred form
// and {T, idxT} of every pair go there.
hipError_t select_and_emit(const Geometry& geo, int32_t slices, int64_t K, float* buf, uint32_t* idx, float* val,
                           uint32_t* guess, uint32_t* last_T, uint2* save_keep, const TopkScratch& s,
                           hipStream_t stream) {
    const int64_t pairs = static_cast<int64_t>(slices) * geo.C;
    const int32_t tpc = static_cast<int32_t>(tiles_per_chunk(geo, kTopkTile));
    const dim3 per_pair(static_cast<uint32_t>(pairs)), block(kThreads);
    const uint32_t K32 = static_cast<uint32_t>(K);
    const dim3 tie_grid(static_cast<uint32_t>(tpc < 4096 ? tpc : 4096));   // the pair-walking kernels
    const int32_t cand_blocks = (tpc + kCandTilesPerBlock - 1) / kCandTilesPerBlock;
    const dim3 cand_grid(static_cast<uint32_t>(pairs * cand_blocks));
    const int32_t tie_cand_blocks = (tpc + kTieTilesPerBlock - 1) / kTieTilesPerBlock;
    const dim3 tie_cand_grid(static_cast<uint32_t>(pairs * tie_cand_blocks));
    const int32_t emit_blocks = (tpc + kEmitTilesPerBlock - 1) / kEmitTilesPerBlock;
    const dim3 emit_grid(static_cast<uint32_t>(pairs * emit_blocks));
    for (int level = 0; level < 3; ++level) {
        if (level == 1) {
            hipLaunchKernelGGL(topk_split_kernel, tie_grid, block, 0, stream, buf, s.state, s.tile_split, s.slots,
                               s.slots_per_tile, geo.d, geo.L, geo.C, pairs, tpc);
            APMS_RETURN_IF_ERROR();
        }
        if (level > 0) {
            if (level == 1)
                hipLaunchKernelGGL(topk_cand_hist_kernel<false>, cand_grid, block, 0, stream, s.slots, s.slots_per_tile,
                                   s.tile_split, s.hist, s.state, tpc, cand_blocks, level);
            else
                hipLaunchKernelGGL(topk_near_kernel, cand_grid, block, 0, stream, s.slots, s.slots_per_tile, s.tile_split,
                                   s.hist, s.state, s.tile_counts, s.near, tpc, cand_blocks);
            APMS_RETURN_IF_ERROR();
            hipLaunchKernelGGL(topk_key_hist_walk_kernel, tie_grid, block, 0, stream, buf, s.hist, s.state, geo.d,
                               geo.L, geo.C, pairs, tpc, level);
            APMS_RETURN_IF_ERROR();
        }
        hipLaunchKernelGGL(topk_pick_kernel<false>, per_pair, block, 0, stream, s.hist, s.state, level, K32,
                           level == 2 ? guess : static_cast<uint32_t*>(nullptr), last_T, false);
        APMS_RETURN_IF_ERROR();
        if (level == 0) {
            // pairs whose first pass did not count down to the threshold bin: full histogram, pick again
            hipLaunchKernelGGL(topk_rehist_kernel, tie_grid, block, 0, stream, buf, s.hist, s.state, geo.d, geo.L, geo.C,
                               pairs, tpc);
            APMS_RETURN_IF_ERROR();
            hipLaunchKernelGGL(topk_pick_kernel<false>, per_pair, block, 0, stream, s.hist, s.state, level, K32,
                               static_cast<uint32_t*>(nullptr), last_T, true);
            APMS_RETURN_IF_ERROR();
        }
    }
    hipLaunchKernelGGL(topk_resolve_kernel, per_pair, block, 0, stream, s.state, s.near, s.tile_counts, tpc);
    APMS_RETURN_IF_ERROR();
    for (int level = 0; level < 3; ++level) {                  // tie selection from the slots or the buffer: rare
        hipLaunchKernelGGL(topk_cand_hist_kernel<true>, tie_cand_grid, block, 0, stream, s.slots, s.slots_per_tile,
                           s.tile_split, s.hist, s.state, tpc, tie_cand_blocks, level);
        APMS_RETURN_IF_ERROR();
        hipLaunchKernelGGL(topk_tie_hist_kernel, tie_grid, block, 0, stream, buf, s.hist, s.state, geo.d, geo.L,
                           geo.C, pairs, tpc, level);
        APMS_RETURN_IF_ERROR();
        hipLaunchKernelGGL(topk_pick_kernel<true>, per_pair, block, 0, stream, s.hist, s.state, level, K32,
                           static_cast<uint32_t*>(nullptr), static_cast<uint32_t*>(nullptr), false);
        APMS_RETURN_IF_ERROR();
    }
    hipLaunchKernelGGL(topk_slot_count_kernel, emit_grid, block, 0, stream, s.slots, s.slots_per_tile, s.tile_split,
                       s.state, s.tile_counts, tpc, emit_blocks);
    APMS_RETURN_IF_ERROR();
    hipLaunchKernelGGL(topk_count_walk_kernel, tie_grid, block, 0, stream, buf, s.state, s.tile_counts, geo.d, geo.L,
                       geo.C, pairs, tpc);
    APMS_RETURN_IF_ERROR();
    hipLaunchKernelGGL(topk_scan_kernel, per_pair, block, 0, stream, s.tile_counts, tpc);
    APMS_RETURN_IF_ERROR();
    hipLaunchKernelGGL(topk_slot_emit_kernel, emit_grid, block, 0, stream, buf, s.slots, s.slots_per_tile,
                       s.tile_split, s.state, s.tile_counts, idx, val, geo.d, geo.L, geo.C, tpc, emit_blocks, K,
                       save_keep == nullptr);
    APMS_RETURN_IF_ERROR();
    hipLaunchKernelGGL(topk_emit_walk_kernel, tie_grid, block, 0, stream, buf, s.state, s.tile_counts, idx, val, geo.d,
                       geo.L, geo.C, pairs, tpc, K, save_keep == nullptr);
    APMS_RETURN_IF_ERROR();
    if (save_keep) {
        hipLaunchKernelGGL(topk_save_keep_kernel, dim3(static_cast<uint32_t>((pairs + kThreads - 1) / kThreads)), block, 0,
                           stream, s.state, save_keep, pairs);
        APMS_RETURN_IF_ERROR();
    }
    return hipSuccess;
}

// Fills table[lists][tiles_per_chunk] with the tile offsets of `lists` sorted index lists of K entries;
// tile_elems is a power of two.
hipError_t tile_offsets(int64_t lists, int32_t tpc, int32_t tile_elems, int64_t K, const uint32_t* idx,
                        uint32_t* table, hipStream_t stream) {
    const int64_t per_block = kThreads * kOffsetsPerThread;
    const int64_t blocks_per_list = (K + per_block - 1) / per_block;
    const int64_t blocks = lists * blocks_per_list;
    if (blocks <= 0) return hipSuccess;
    int tile_shift = 0;
    while ((1 << tile_shift) < tile_elems) ++tile_shift;
    hipLaunchKernelGGL(topk_tile_offsets_kernel, dim3(static_cast<uint32_t>(blocks)), dim3(kThreads), 0, stream, idx,
                       table, tpc, tile_shift, static_cast<int32_t>(K), static_cast<int32_t>(blocks_per_list));
    return hipGetLastError();
}

hipError_t begin_call(int64_t pairs, bool resplit, const TopkScratch& s, hipStream_t stream) {
    const int64_t count = pairs * kTopkBins;
    const int64_t blocks = (count + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(topk_begin_kernel, dim3(static_cast<uint32_t>(blocks < 4096 ? blocks : 4096)), dim3(kThreads), 0,
                       stream, s.hist, count, s.state, pairs, resplit ? 1u : 0u);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_topk_compress(const Geometry& geo, int64_t K, float* m, const float* g, float* werr, uint32_t* idx,
                                float* val, float beta, float one_minus_beta, bool werr_pending, bool defer,
                                const TopkGather* gather, const TopkScratch& scratch, hipStream_t stream) {
    const int64_t pairs = static_cast<int64_t>(geo.n) * geo.C;
    if (pairs <= 0) return hipSuccess;
    const int32_t tpc = static_cast<int32_t>(tiles_per_chunk(geo, kTopkTile));
    hipError_t e = begin_call(pairs, /*resplit=*/false, scratch, stream);
    if (e != hipSuccess) return e;
    // unused dynamic LDS that caps the pass at 3 workgroups per CU: measured 3 % faster than uncapped, 2
    // workgroups per CU are slower again
    constexpr uint32_t kWorkerPassPad = 34 * 1024;           // beside the kernel's own 17 KB
    const dim3 grid(static_cast<uint32_t>(pairs * tpc)), block(kThreads);
    const uint2* prev_keep = werr_pending ? scratch.keep : static_cast<const uint2*>(nullptr);
    if (gather)
        hipLaunchKernelGGL(topk_worker_u_kernel<true>, grid, block, kWorkerPassPad, stream, m, g, werr, scratch.hist,
                           scratch.state, scratch.guess, scratch.tile_split, scratch.slots, scratch.slots_per_tile,
                           prev_keep, gather->idx, gather->val, scratch.gather_offsets, static_cast<int32_t>(gather->K),
                           geo.d, geo.L, geo.C, tpc, beta, one_minus_beta);
    else
        hipLaunchKernelGGL(topk_worker_u_kernel<false>, grid, block, kWorkerPassPad, stream, m, g, werr, scratch.hist,
                           scratch.state, scratch.guess, scratch.tile_split, scratch.slots, scratch.slots_per_tile,
                           prev_keep, static_cast<const uint32_t*>(nullptr), static_cast<const float*>(nullptr),
                           static_cast<const uint32_t*>(nullptr), 0, geo.d, geo.L, geo.C, tpc, beta, one_minus_beta);
    APMS_RETURN_IF_ERROR();
    return select_and_emit(geo, geo.n, K, werr, idx, val, scratch.guess, scratch.last_T, defer ? scratch.keep : nullptr, scratch,
                           stream);
}

hipError_t launch_topk_server_reduce(const Geometry& geo, int64_t K, const uint32_t* idx, const float* val,
                                     float* serr, uint32_t* sidx, float* sval, float inv_n, bool serr_pending,
                                     bool defer, const TopkScratch& scratch, hipStream_t stream) {
    if (geo.C <= 0) return hipSuccess;
    const int32_t tpc = static_cast<int32_t>(tiles_per_chunk(geo, kTopkTile));
    hipError_t e = begin_call(geo.C, /*resplit=*/false, scratch, stream);
    if (e != hipSuccess) return e;
    e = tile_offsets(static_cast<int64_t>(geo.n) * geo.C, tpc, kTopkTile, K, idx, scratch.tile_counts, stream);
    if (e != hipSuccess) return e;
    uint32_t* server_guess = scratch.guess + static_cast<int64_t>(geo.n) * geo.C;   // after the workers' entries
    uint2* server_keep = scratch.keep + static_cast<int64_t>(geo.n) * geo.C;
    // workers per batch of the decode: as many as fill three quarters of the LDS stage with the share of a
    // list that falls into one tile, so that an uneven tile still fits
    const int64_t per_tile = (K * kTopkTile + geo.L - 1) / geo.L;
    const int64_t fit = (kServerStage * 3 / 4) / (per_tile > 0 ? per_tile : 1);
    const int32_t workers_per_batch = static_cast<int32_t>(fit < 1 ? 1 : (fit > kServerBatchMax ? kServerBatchMax : fit));
    hipLaunchKernelGGL(topk_server_u_kernel, dim3(static_cast<uint32_t>(static_cast<int64_t>(geo.C) * tpc)),
                       dim3(kThreads), 0, stream, idx, val, serr, scratch.hist, scratch.state, server_guess,
                       scratch.tile_counts, scratch.tile_split, scratch.slots, scratch.slots_per_tile,
                       serr_pending ? server_keep : static_cast<const uint2*>(nullptr), geo.d, geo.L, geo.C, geo.n,
                       static_cast<int32_t>(K), tpc, workers_per_batch, inv_n);
    APMS_RETURN_IF_ERROR();
    return select_and_emit(geo, 1, K, serr, sidx, sval, server_guess, scratch.last_T + static_cast<int64_t>(geo.n) * geo.C,
                           defer ? server_keep : nullptr, scratch, stream);
}

hipError_t launch_topk_finalize(const Geometry& geo, bool server, float* err, const TopkScratch& scratch,
                                hipStream_t stream) {
    const int64_t pairs = server ? geo.C : static_cast<int64_t>(geo.n) * geo.C;
    if (pairs <= 0) return hipSuccess;
    const int32_t tpc = static_cast<int32_t>(tiles_per_chunk(geo, kTopkTile));
    const uint2* keep = scratch.keep + (server ? static_cast<int64_t>(geo.n) * geo.C : 0);
    hipLaunchKernelGGL(topk_finalize_kernel, dim3(static_cast<uint32_t>(pairs * tpc)), dim3(kThreads), 0, stream, err, keep,
                       geo.d, geo.L, geo.C, tpc);
    return hipGetLastError();
}

hipError_t launch_topk_apply(const Geometry& geo, int64_t K, const uint32_t* sidx, const float* sval,
                             const float* v, float* x, float* m, float lr, float eps, bool write_m, bool model_step,
                             const TopkScratch& scratch, hipStream_t stream) {
    const int64_t pairs = static_cast<int64_t>(geo.n) * geo.C;
    if (pairs <= 0) return hipSuccess;
    const dim3 block(kThreads);
    const int32_t K32 = static_cast<int32_t>(K);
    if (!write_m) {
        // the model step alone (the gather stays pending): 4096-element tiles over the one [d] vector, with the
        // offsets table the worker's first pass will decode the list by (scratch.gather_offsets)
        const int32_t tpc = static_cast<int32_t>(tiles_per_chunk(geo, kTopkTile));
        const hipError_t e = tile_offsets(geo.C, tpc, kTopkTile, K, sidx, scratch.gather_offsets, stream);
        if (e != hipSuccess) return e;
        if (model_step)
            hipLaunchKernelGGL((topk_apply_kernel<kTileRows, false, true>), dim3(static_cast<uint32_t>(geo.C) * tpc), block, 0,
                               stream, sidx, sval, v, x, m, scratch.gather_offsets, geo.d, geo.L, geo.C, tpc, K32, lr, eps);
        return hipGetLastError();
    }
    // 2048-element tiles (measured best: 4.1 ms against 4.4 ms for 4096 and 5.3 ms for 1024 on the
    // BERT-Large-sized buffer), provided the offsets table for them fits the tile_counts array
    // ([n * C][L / 4096]: n >= 2)
    const int rows = geo.n >= 2 ? 2 : kTileRows;
    const int32_t tile = rows * kRowStride;
    const int32_t tpc = static_cast<int32_t>(tiles_per_chunk(geo, tile));
    const hipError_t e = tile_offsets(geo.C, tpc, tile, K, sidx, scratch.tile_counts, stream);
    if (e != hipSuccess) return e;
    const dim3 grid(static_cast<uint32_t>(pairs * tpc));
#define APMS_LAUNCH_TOPK_APPLY(ROWS, STEP)                                                                          \
    hipLaunchKernelGGL((topk_apply_kernel<ROWS, true, STEP>), grid, block, 0, stream, sidx, sval, v, x, m,           \
                       scratch.tile_counts, geo.d, geo.L, geo.C, tpc, K32, lr, eps)
    if (rows == 2) {
        if (model_step) APMS_LAUNCH_TOPK_APPLY(2, true); else APMS_LAUNCH_TOPK_APPLY(2, false);
    } else {
        if (model_step) APMS_LAUNCH_TOPK_APPLY(kTileRows, true); else APMS_LAUNCH_TOPK_APPLY(kTileRows, false);
    }
#undef APMS_LAUNCH_TOPK_APPLY
    return hipGetLastError();
}

}  // namespace apms
