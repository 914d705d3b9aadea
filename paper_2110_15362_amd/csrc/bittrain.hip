// libbittrain: BitTrain's sparse bitmap activation codec as HIP kernels for
// CDNA4 (gfx950, wave64).  See include/bittrain.h for the contract.
//
// Section 3.2 of the paper defines the format (a bit per element plus the
// non-zero elements in index order); Algorithm 1 builds it with a sequential
// push loop and Algorithm 2 undoes it with a running counter j.  Both loops
// carry one dependency: the position of an element's value is the number of
// non-zero elements before it.  On a GPU that is an exclusive prefix sum over
// the non-zero predicate, and the kernels below compute it in ONE pass over the
// data so that the tensor is read from HBM exactly once:
//
//   lane    16-byte loads; per-lane non-zero mask by integer compare
//   wave    packed DPP prefix sum of the per-lane popcounts (no LDS, no barrier)
//   block   four wave totals through LDS
//   grid    per-tile counts published in the workspace; one extra wave turns them
//           into per-tile prefixes; a tile polls only its own prefix
//
// There is no matrix contraction anywhere, so no MFMA: the path is bound by HBM
// bandwidth and everything here is about moving each byte once, coalesced, and
// about keeping enough bytes in flight while a tile waits for its prefix.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "bittrain.h"

namespace {

constexpr int kWaveSize = 64;
constexpr int kWaves = 4;                 // waves per block
constexpr int kBlock = kWaveSize * kWaves;
#ifndef BT_ROWS
#define BT_ROWS 8
#endif
constexpr int kRows = BT_ROWS;            // 16-byte loads per lane per tile
constexpr int kPhaseRows = 4;             // rows that go through a wave's LDS strip at a time
#ifndef BT_LOAD_AHEAD
#define BT_LOAD_AHEAD BT_ROWS
#endif
constexpr int kLoadAhead = BT_LOAD_AHEAD; // rows a wave has in flight while it reads its tile
constexpr int kVecBytes = 16;
#ifndef BT_RELU_ROWS
#define BT_RELU_ROWS 1
#endif
constexpr int kReluRows = BT_RELU_ROWS;   // 16-byte vectors per lane in the ReLU-backward stream

// ---- workspace layout -----------------------------------------------------------------
// Header (uint32 words), then one 768-byte record per 32 tiles.
constexpr int kHdrSeq = 0;       // calls completed on this workspace; its low bit picks the copy in use
constexpr int kHdrPrevTiles = 1; // tiles of the previous call (what it left behind in the other copy)
constexpr int kHdrError = BT_WS_ERROR_WORD;           // set if a wait was given up
constexpr int kHdrSpinLimit = BT_WS_WAIT_LIMIT_WORD;  // polls before a wait is given up; 0: kSpinLimit
constexpr size_t kHeaderBytes = 256;
// Record of 32 tiles, two copies c = 0, 1 of everything, in separate 128-byte lines:
//   [128*c, 128*c + 128)          uint32 count + 1 of each tile, written by the tile
//   [256 + 256*c, 256*c + 512)    uint64 prefix + 1 of each tile, written by the scanner
// 0 means "not published yet".  A call uses copy (seq & 1) and zeroes what the
// previous call left in the other copy, so the copy the next call uses is clean
// when it starts and no clearing launch is ever needed.
constexpr size_t kRecordBytes = 768;
constexpr int kTilesPerRecord = 32;
constexpr uint32_t kSpinLimit = 1u << 20; // polls before a wait is given up
#ifndef BT_SCANNER_SLEEP
#define BT_SCANNER_SLEEP 1
#endif
#ifndef BT_TILE_SLEEP
#define BT_TILE_SLEEP 16
#endif
constexpr int kScannerSleep = BT_SCANNER_SLEEP;   // pause between two polls, in units of 64 clocks
constexpr int kTileSleep = BT_TILE_SLEEP;

template <int S> struct Geo {
    static constexpr int E = kVecBytes / S;          // elements per lane per load
    static constexpr int G = 32 / E;                 // lanes that share a bitmap word
    static constexpr int WPR = kWaveSize / G;        // bitmap words per row
    static constexpr int ROW = kWaveSize * E;        // elements per wave-wide load
    static constexpr int WAVE = kRows * ROW;         // elements per wave per tile
    static constexpr int TILE = kWaves * WAVE;       // elements per tile
    static constexpr int LDS_WAVE = kPhaseRows * ROW * S + 2 * kVecBytes;  // staging bytes per wave: the rows of a phase, the
                                                                          // shift to a 16-byte boundary, and a vector nobody reads
    static constexpr int DUMP = (LDS_WAVE - kVecBytes) / S;             // element index of that vector in a wave's strip
    static constexpr int RPM = 32 / E;               // rows whose E-bit lane masks share one register
    static constexpr int MW = (kRows + RPM - 1) / RPM;   // registers that hold a lane's masks
    static_assert(kRows % kPhaseRows == 0 && kPhaseRows % 2 == 0, "rows are scanned two to a register");
};

// ---- wave-level primitives (all 64 lanes must be active) ---------------------

#define BT_DPP(old, src, ctrl, rmask, bound) \
    ((uint32_t)__builtin_amdgcn_update_dpp((int)(old), (int)(src), (ctrl), (rmask), 0xf, (bound)))

// Inclusive prefix sum over the 64 lanes.  Four shift-and-add steps inside each
// row of 16 lanes (lanes shifted in from outside the row read 0), then the last
// lane of row 0 / row 2 is added to row 1 / row 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t x) {
    x += BT_DPP(0, x, 0x111, 0xf, true);   // row_shr:1
    x += BT_DPP(0, x, 0x112, 0xf, true);   // row_shr:2
    x += BT_DPP(0, x, 0x114, 0xf, true);   // row_shr:4
    x += BT_DPP(0, x, 0x118, 0xf, true);   // row_shr:8
    x += BT_DPP(0, x, 0x142, 0xa, false);  // row_bcast:15 into rows 1 and 3
    x += BT_DPP(0, x, 0x143, 0xc, false);  // row_bcast:31 into rows 2 and 3
    return x;
}

// OR over each aligned group of G lanes (G = 4, 8 or 16); every lane gets the result.
template <int G> __device__ __forceinline__ uint32_t group_or(uint32_t x) {
    x |= BT_DPP(0, x, 0xB1, 0xf, true);       // quad_perm [1,0,3,2]: lane ^ 1
    x |= BT_DPP(0, x, 0x4E, 0xf, true);       // quad_perm [2,3,0,1]: lane ^ 2
    if (G >= 8) x |= BT_DPP(0, x, 0x141, 0xf, true);   // row_half_mirror: lane i <-> 7 - i
    if (G == 16) x |= BT_DPP(0, x, 0x140, 0xf, true);  // row_mirror: lane i <-> 15 - i
    return x;
}

// Order LDS traffic between the lanes of one wave (no block barrier involved).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- per-lane helpers -----------------------------------------------------------

// Bulk data is touched exactly once per call, so most of it is moved with the
// "non-temporal" hint: it then does not displace what the caches hold.  Measured per
// kernel on MI355X (fp32, 25.7 M elements, cold / warm microseconds):
//   compress    plain 38.1/31.3   nt loads 34.2/32.8   nt stores 35.0/30.0   both 33.3/31.3
//   decompress  plain 35.6/27.6   nt loads 36.3/32.8   nt stores 34.4/27.3   both 35.0/34.2
//   relu bwd    plain 37.2        nt loads 36.6        nt stores 35.4        both 34.7
// so compress and the ReLU stream use both hints (their input is dead after the call:
// "delete T" in Algorithm 1), decompress only the store hint.
typedef uint32_t bt_u4 __attribute__((ext_vector_type(4)));
template <bool NT> __device__ __forceinline__ uint4 stream_load(const uint4 *p) {
    if (NT) {
        const bt_u4 v = __builtin_nontemporal_load(reinterpret_cast<const bt_u4 *>(p));
        return make_uint4(v.x, v.y, v.z, v.w);
    }
    return *p;
}
template <bool NT> __device__ __forceinline__ void stream_store(uint4 *p, const uint4 v) {
    if (NT) {
        bt_u4 t;
        t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
        __builtin_nontemporal_store(t, reinterpret_cast<bt_u4 *>(p));
    } else {
        *p = v;
    }
}
constexpr bool kCompressNtLoad = true, kCompressNtStore = true;
constexpr bool kDecompressNtLoad = false, kDecompressNtStore = true;
constexpr bool kReluNtLoad = true, kReluNtStore = true;

// Bit j set <=> element j of the 16-byte vector has a non-zero bit pattern.
// min(bits, 1) instead of a compare: a compare result lives in a scalar register
// pair, and 8 rows x 4..8 compares in flight exhaust the scalar registers.
template <int S> __device__ __forceinline__ uint32_t nonzero_mask(const uint4 v) {
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    uint32_t m = 0;
    if (S == 8) {
        m = min(d[0] | d[1], 1u) | (min(d[2] | d[3], 1u) << 1);
    } else if (S == 4) {
#pragma unroll
        for (int i = 0; i < 4; ++i) m |= min(d[i], 1u) << i;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            m |= min(d[i] & 0xffffu, 1u) << (2 * i);
            m |= min(d[i] >> 16, 1u) << (2 * i + 1);
        }
    }
    return m;
}

// Which elements of the 16-byte vector are stored.  KEEP = kKeepNonZero: Algorithm 1's
// test (non-zero bit pattern).  Otherwise activation pruning (Section 4.3) followed by
// that test, in one pass: an element survives pruning where its value exceeds
// `threshold`, compared in single precision after widening (exact for half and
// bfloat16; a double is compared with the threshold widened to double, also exact; a
// NaN exceeds nothing), and is then stored if its bit pattern is non-zero (a +0.0 that
// survives a negative threshold is still a zero for Algorithm 1).
enum { kKeepNonZero = 0, kKeepAboveF32 = 1, kKeepAboveF16 = 2, kKeepAboveBF16 = 3, kKeepAboveF64 = 4 };
template <int S, int KEEP> __device__ __forceinline__ uint32_t keep_mask(const uint4 v, const float threshold) {
    if (KEEP == kKeepNonZero) return nonzero_mask<S>(v);
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    uint32_t m = 0;
    if (KEEP == kKeepAboveF64) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            m |= (__longlong_as_double((long long)(((uint64_t)d[2 * i + 1] << 32) | d[2 * i])) > (double)threshold ? 1u : 0u) << i;
    } else if (KEEP == kKeepAboveF32) {
#pragma unroll
        for (int i = 0; i < 4; ++i) m |= (__uint_as_float(d[i]) > threshold ? 1u : 0u) << i;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float lo, hi;
            if (KEEP == kKeepAboveBF16) {
                lo = __uint_as_float(d[i] << 16);
                hi = __uint_as_float(d[i] & 0xffff0000u);
            } else {
                lo = (float)__builtin_bit_cast(_Float16, (uint16_t)(d[i] & 0xffffu));
                hi = (float)__builtin_bit_cast(_Float16, (uint16_t)(d[i] >> 16));
            }
            m |= (lo > threshold ? 1u : 0u) << (2 * i);
            m |= (hi > threshold ? 1u : 0u) << (2 * i + 1);
        }
    }
    return m & nonzero_mask<S>(v);
}

// 16 bytes at element index e0 of a buffer of n > 0 elements; elements at or beyond n
// read as 0.  Branch-free: every address is clamped into the buffer, then selected.
template <int S> __device__ __forceinline__ uint4 load_vec_guarded(const void *base, uint64_t e0, uint64_t n) {
    uint32_t d[4] = {0, 0, 0, 0};
    if (S == 8) {
        const uint64_t *p = static_cast<const uint64_t *>(base);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint64_t e = e0 + j;
            const uint64_t v = p[e < n ? e : n - 1];
            d[2 * j] = e < n ? (uint32_t)v : 0u;
            d[2 * j + 1] = e < n ? (uint32_t)(v >> 32) : 0u;
        }
    } else if (S == 4) {
        const uint32_t *p = static_cast<const uint32_t *>(base);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint64_t e = e0 + j;
            const uint32_t v = p[e < n ? e : n - 1];
            d[j] = e < n ? v : 0u;
        }
    } else {
        const uint16_t *p = static_cast<const uint16_t *>(base);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint64_t e = e0 + j;
            const uint32_t v = p[e < n ? e : n - 1];
            d[j >> 1] |= (e < n ? v : 0u) << (16 * (j & 1));
        }
    }
    return make_uint4(d[0], d[1], d[2], d[3]);
}

template <int S> __device__ __forceinline__ void store_vec_guarded(void *base, uint64_t e0, uint64_t n, const uint4 v) {
    constexpr int E = Geo<S>::E;
    if (e0 + E <= n) {
        *reinterpret_cast<uint4 *>(static_cast<char *>(base) + e0 * S) = v;
        return;
    }
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    if (S == 8) {
        uint64_t *p = static_cast<uint64_t *>(base);
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (e0 + j < n) p[e0 + j] = ((uint64_t)d[2 * j + 1] << 32) | d[2 * j];
    } else if (S == 4) {
        uint32_t *p = static_cast<uint32_t *>(base);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (e0 + j < n) p[e0 + j] = d[j];
    } else {
        uint16_t *p = static_cast<uint16_t *>(base);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (e0 + j < n) p[e0 + j] = (uint16_t)(d[j >> 1] >> (16 * (j & 1)));
    }
}

// The E bitmap bits of the 16-byte vector that starts at element e0 (e0 % E == 0).
// Words at or beyond n_words read as 0, bits at or beyond n are cleared.
template <int S>
__device__ __forceinline__ uint32_t bitmap_bits(const uint32_t *bitmap, uint64_t e0, uint64_t n, uint64_t n_words) {
    constexpr int E = Geo<S>::E;
    const uint64_t w = e0 >> 5;
    uint32_t word = (w < n_words) ? bitmap[w] : 0u;
    uint32_t m = (word >> (uint32_t)(e0 & 31)) & ((1u << E) - 1u);
    if (e0 + E > n) m &= (e0 < n) ? ((1u << (uint32_t)(n - e0)) - 1u) : 0u;
    return m;
}

// ---- grid prefix ---------------------------------------------------------------------------
//
// The position of a tile's first value is the number of non-zero elements in all
// tiles before it (Algorithm 1 appends in index order; Algorithm 2's counter j).
// Tiles do not talk to each other.  Each tile publishes its count in the workspace;
// ONE extra workgroup (workgroup 0, a single wave: the "scanner") reads the counts
// in index order, up to 448 at a time, keeps the running sum, and writes every tile's
// prefix back; a tile then polls its own prefix, one 8-byte load.  Per tile that
// is one store and one polled load on lines shared with few other tiles.  (Having
// every tile read its predecessors' counts itself -- a look-back window or a tree --
// makes a few hot lines that thousands of tiles read at once, and those reads
// queue up at one memory channel.)
//
// Nothing a tile waits for depends on another tile having been started: the
// scanner is workgroup 0, started first, and only waits for counts, which tiles
// publish before they wait for anything.  Waits are bounded anyway (kSpinLimit).
//
// Entries are value + 1 (0 = not published), written and read with relaxed
// device-scope atomics: the entry is the only thing that is communicated.

// ---- timeline (only in a build with -DBT_TIMELINE) ---------------------------------------------
// Every tile of a single-tensor bt_compress / bt_decompress launch leaves five times of the
// 100 MHz device clock and its number of polls in the caller's buffer (8 words per tile: started,
// counted, prefix seen, stores issued, stores acknowledged, polls), and the scanner two words per
// pass that consumed something (time, first slot << 32 | end slot), after the tiles' words.
#ifdef BT_TIMELINE
__device__ uint64_t *g_timeline = nullptr;
__device__ uint32_t g_timeline_tiles = 0, g_timeline_passes = 0;
#define BT_TL(slot, k)                                                                            \
    do {                                                                                          \
        if (threadIdx.x == 0 && g_timeline != nullptr && (slot) < g_timeline_tiles)               \
            g_timeline[8 * (size_t)(slot) + (k)] = wall_clock64();                                \
    } while (0)
#define BT_TL_VALUE(slot, k, v)                                                                   \
    do {                                                                                          \
        if (threadIdx.x == 0 && g_timeline != nullptr && (slot) < g_timeline_tiles)               \
            g_timeline[8 * (size_t)(slot) + (k)] = (v);                                           \
    } while (0)
#else
#define BT_TL(slot, k) do {} while (0)
#define BT_TL_VALUE(slot, k, v) do {} while (0)
#endif

__device__ __forceinline__ uint64_t ws_load64(const void *p) {
    return __hip_atomic_load(static_cast<const uint64_t *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ws_store64(void *p, uint64_t v) {
    __hip_atomic_store(static_cast<uint64_t *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ws_store32(void *p, uint32_t v) {
    __hip_atomic_store(static_cast<uint32_t *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// count + 1 of `tile` in copy c
__device__ __forceinline__ char *ws_count(char *ws, uint32_t tile, uint32_t copy) {
    return ws + kHeaderBytes + (size_t)(tile >> 5) * kRecordBytes + 128u * copy + 4u * (tile & 31u);
}
// prefix + 1 of `tile` in copy c
__device__ __forceinline__ char *ws_prefix(char *ws, uint32_t tile, uint32_t copy) {
    return ws + kHeaderBytes + (size_t)(tile >> 5) * kRecordBytes + 256u + 256u * copy + 8u * (tile & 31u);
}

// Polls after which a wait is given up: what the caller asked for in the header, else the
// built-in limit.  Read once, before the wait (a load inside the polling loop would
// lengthen every poll by a round trip).
__device__ __forceinline__ uint32_t wait_limit(const uint32_t *hdr) {
    const uint32_t asked = hdr[kHdrSpinLimit];          // never written by a kernel
    return asked != 0 ? asked : kSpinLimit;
}

template <int SLEEP> __device__ __forceinline__ bool spin_expired(uint32_t *hdr, uint32_t &spins, const uint32_t limit) {
    // bounded wait: give up after the limit of polls, or soon after anyone has given up
    ++spins;
    if (spins > limit ||
        ((spins & 255u) == 0 && __hip_atomic_load(&hdr[kHdrError], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
        __hip_atomic_store(&hdr[kHdrError], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    __builtin_amdgcn_s_sleep(SLEEP);   // units of 64 clocks
    return false;
}

// The scanner: one wave.  Each pass looks at kScanRows x 64 counts starting at the
// frontier rounded down to a multiple of 64; lane l of row j looks at tile
// w0 + 64*j + l, so every load and store of a row is one contiguous run.  The pass
// takes the leading run of published counts, turns it into prefixes (a wave prefix
// sum per row, carried from row to row), writes them, and moves the frontier.
// When a tensor's counts are all in it writes the tensor's total (nnz); at the end it
// advances the header for the next call.
// Rows per pass, measured on MI355X (25.7 M fp32 elements, cold, compress / decompress
// microseconds at 50 % zeros): 2 rows 39.0 / 36.8, 4 rows 34.9 / 33.5, 6 rows 33.6 / 33.6,
// 7 rows 33.4 / 33.9, 8 rows 33.6 / 34.0, 16 rows 35.2 / 34.2, 32 rows 37.4 / 36.6 (at 90 % zeros
// 6 rows cost compress 0.9): a pass costs a load round trip whatever its width, but a
// wider pass waits for the slowest of more loads.
#ifndef BT_SCAN_ROWS
#define BT_SCAN_ROWS 7
#endif
constexpr int kScanRows = BT_SCAN_ROWS;
// What the scanner has to know about the tensors of one call.  A call on one tensor
// has one segment, slots == tiles.  A batched call lays its tensors end to end in
// the slot (= workspace entry) numbering, each starting at a multiple of 64 slots, so
// that a scanner row never spans two tensors; the slots between a tensor's last tile
// and the next tensor's first slot belong to no tile, and their workgroups publish a
// count of zero.  Prefixes restart at 0 with every tensor, and each tensor's total
// goes to its nnz.
struct Segments {
    uint32_t count;           // tensors
    const uint32_t *start;    // count + 1 entries: first slot of tensor i; start[count] = slots of the call
    uint64_t *const *nnz;     // where tensor i's number of stored values goes; the array or an entry may be null
};

__device__ __forceinline__ void scan_counts(char *ws, const Segments seg) {
    const uint32_t lane = threadIdx.x & (kWaveSize - 1);
    uint32_t *hdr = reinterpret_cast<uint32_t *>(ws);
    const uint32_t seq = hdr[kHdrSeq];
    const uint32_t cur = seq & 1u;
    const uint32_t n_slots = seg.start[seg.count];
    uint32_t frontier = 0;     // slots [0, frontier) are done
    uint32_t item = 0;         // tensor that slot `frontier` belongs to
    uint64_t running = 0;      // stored values of tensor `item` in its tiles before `frontier`
    uint32_t spins = 0;
    const uint32_t limit = wait_limit(hdr);
#ifdef BT_TIMELINE
    uint64_t *const timeline = g_timeline;      // read once: a load in the loop would join the scanner's waits
    uint32_t timeline_pass = 0;
#endif
    while (frontier < n_slots) {
        const uint32_t w0 = frontier & ~63u;
        uint32_t c[kScanRows];
#pragma unroll
        for (int j = 0; j < kScanRows; ++j) {
            const uint32_t t = w0 + 64u * j + lane;
            c[j] = 0;
            if (t < n_slots)
                c[j] = __hip_atomic_load(reinterpret_cast<const uint32_t *>(ws_count(ws, t, cur)), __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
        }
        // Look at every row before writing anything: on this hardware one counter tracks
        // loads and stores alike, so a load waited for after a store also waits for that
        // store to reach memory.
        uint64_t usable_lanes[kScanRows];
#pragma unroll
        for (int j = 0; j < kScanRows; ++j) {
            const uint32_t t = w0 + 64u * j + lane;
            usable_lanes[j] = __ballot(t < frontier || (t < n_slots && c[j] != 0));   // done before, or published
        }
        // rows are consumed in order while every slot of the row is usable
        bool open = true;
        uint32_t new_frontier = frontier;
#pragma unroll
        for (int j = 0; j < kScanRows; ++j) {
            const uint32_t row0 = w0 + 64u * j;
            const uint32_t t = row0 + lane;
            if (open && row0 < n_slots) {
                const uint64_t bad = ~usable_lanes[j];                             // lanes that stop the run
                const uint32_t run = bad == 0 ? 64u : (uint32_t)__ffsll((unsigned long long)bad) - 1u;
                const uint32_t row_end = row0 + run;                               // slots [row0, row_end) usable
                if (row_end > new_frontier) {
                    while (item + 1 < seg.count && row0 >= seg.start[item + 1]) ++item;
                    if (row0 == seg.start[item] && new_frontier <= row0) running = 0;   // a new tensor begins
                    const bool fresh = t >= frontier && t < row_end;
                    const uint32_t mine = fresh ? c[j] - 1u : 0u;
                    const uint32_t incl = wave_inclusive_sum(mine);
                    if (fresh) ws_store64(ws_prefix(ws, t, cur), running + (incl - mine) + 1);
                    running += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                    new_frontier = row_end;
                    if (row_end == seg.start[item + 1] && lane == 0 && seg.nnz != nullptr && seg.nnz[item] != nullptr)
                        *seg.nnz[item] = running;                                  // length(B.values) of this tensor
                }
                open = run == 64u;
            }
        }
        if (new_frontier == frontier) {
            if (spin_expired<kScannerSleep>(hdr, spins, limit)) return;
            continue;
        }
#ifdef BT_TIMELINE
        if (timeline != nullptr && lane == 0 && timeline_pass < g_timeline_passes) {
            timeline[8 * (size_t)g_timeline_tiles + 2 * timeline_pass] = wall_clock64();
            timeline[8 * (size_t)g_timeline_tiles + 2 * timeline_pass + 1] = ((uint64_t)frontier << 32) | new_frontier;
            ++timeline_pass;
        }
#endif
        frontier = new_frontier;
    }
    if (lane == 0) {
        // every tile has published its count by now, hence has read the header: advance it
        __hip_atomic_store(&hdr[kHdrPrevTiles], n_slots, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&hdr[kHdrSeq], seq + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// A workspace on which a wait was given up is in no defined state: later calls on it do
// nothing (and stay away from its stale entries) until bt_workspace_init has been run.
// Uniform over the workgroup, tested before anything else.
__device__ __forceinline__ bool workspace_failed(const char *ws) {
    return reinterpret_cast<const uint32_t *>(ws)[kHdrError] != 0;
}

struct PrefixShared {
    uint32_t wave_total[kWaves];
    uint64_t tile_prefix;
};

// What a workgroup reads from the header before it publishes anything.  The scanner
// rewrites the header once every slot of the call has published, so a workgroup must
// not read it after its own publication.
struct Epoch {
    uint32_t cur;          // copy of the entries this call uses
    uint32_t prev_slots;   // entries the previous call used in the other copy
};

__device__ __forceinline__ Epoch read_epoch(const char *ws) {
    const uint32_t *hdr = reinterpret_cast<const uint32_t *>(ws);
    return Epoch{hdr[kHdrSeq] & 1u, hdr[kHdrPrevTiles]};
}

// Zero what the previous call left in the other copy of the workspace entries: slots
// [0, prev_slots), shared out over the threads of all slots of this call.
__device__ __forceinline__ void zero_previous(char *ws, const Epoch ep, const uint32_t slot, const uint32_t n_slots) {
    const uint32_t other = ep.cur ^ 1u;
    for (uint32_t i = slot + (uint32_t)threadIdx.x * n_slots; i < ep.prev_slots; i += kBlock * n_slots) {
        ws_store32(ws_count(ws, i, other), 0);
        ws_store64(ws_prefix(ws, i, other), 0);
    }
}

// A slot of a batched call that belongs to no tile: it publishes an empty count, so
// that the scanner knows its workgroup has read the header, and does its share of
// the clean-up.
__device__ __forceinline__ void idle_slot(char *ws, const uint32_t slot, const uint32_t n_slots) {
    const Epoch ep = read_epoch(ws);
    __syncthreads();       // every thread has read the header
    if (threadIdx.x == 0) ws_store32(ws_count(ws, slot, ep.cur), 1);
    zero_previous(ws, ep, slot, n_slots);
}

// Run by every thread of a tile's block: publishes the tile's count in its slot, waits
// for the scanner's answer, and returns the number of stored values of this tensor
// before this wave's part of the tile (wave-uniform).  Contains two block barriers.
// If `index_entry` is not null the tile's own prefix is also written there (the tile index
// that bt_compress_indexed leaves for bt_decompress_indexed).
__device__ __forceinline__ uint64_t tile_prefix(char *ws, PrefixShared &sh, const uint32_t slot,
                                                const uint32_t n_slots, const uint32_t wave_total,
                                                uint64_t *index_entry = nullptr) {
    const int tid = threadIdx.x;
    const uint32_t lane = tid & (kWaveSize - 1), wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6);
    uint32_t *hdr = reinterpret_cast<uint32_t *>(ws);
    // written at the end of the previous call; constant until every slot of this call has published
    const Epoch ep = read_epoch(ws);
    const uint32_t cur = ep.cur;
    const uint32_t limit = wait_limit(hdr);

    if (lane == 0) sh.wave_total[wave] = wave_total;
    __syncthreads();
    BT_TL(slot, 1);
    if (tid == 0) {
        const uint32_t tile_total = sh.wave_total[0] + sh.wave_total[1] + sh.wave_total[2] + sh.wave_total[3];
        ws_store32(ws_count(ws, slot, cur), tile_total + 1);
    }
    zero_previous(ws, ep, slot, n_slots);
    // what the waves before this one hold: read before the wait, so that after it only the prefix is missing
    uint32_t before = 0;
    for (uint32_t w = 0; w < wave; ++w) before += sh.wave_total[w];
    before = (uint32_t)__builtin_amdgcn_readfirstlane((int)before);
    if (tid == 0) {
        uint64_t v;
        uint32_t spins = 0;
        for (;;) {
            v = ws_load64(ws_prefix(ws, slot, cur));
            if (v != 0) break;
            if (spin_expired<kTileSleep>(hdr, spins, limit)) { v = 1; break; }
        }
        sh.tile_prefix = v - 1;
        BT_TL(slot, 2);
        BT_TL_VALUE(slot, 5, spins);
        if (index_entry != nullptr) *index_entry = v - 1;
    }
    __syncthreads();
    uint64_t prefix = sh.tile_prefix + before;
    // the same value in every lane: tell the compiler, so that addresses built on it stay scalar
    prefix = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(prefix >> 32)) << 32) |
             (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)prefix);
    return prefix;
}

// A lane's E-bit non-zero masks of all rows, packed RPM rows to a register.
#define BT_MASK(S_, mp, k) (((mp)[(k) / Geo<S_>::RPM] >> (Geo<S_>::E * ((k) % Geo<S_>::RPM))) & ((1u << Geo<S_>::E) - 1u))

// Per-row popcounts -> exclusive rank of each lane inside its row (two rows per
// register, 16-bit fields: a row holds at most 512 non-zeros) and the row totals
// (same packing, wave-uniform).
template <int S>
__device__ __forceinline__ void rank_rows(const uint32_t (&mp)[Geo<S>::MW], uint32_t (&rank2)[kRows / 2],
                                          uint32_t (&total2)[kRows / 2]) {
#pragma unroll
    for (int k = 0; k < kRows; k += 2) {
        const uint32_t packed = (uint32_t)__popc(BT_MASK(S, mp, k)) | ((uint32_t)__popc(BT_MASK(S, mp, k + 1)) << 16);
        const uint32_t incl = wave_inclusive_sum(packed);
        rank2[k / 2] = incl - packed;
        total2[k / 2] = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    }
}
#define BT_FIELD(arr2, k) (((arr2)[(k) / 2] >> (16 * ((k) & 1))) & 0xffffu)

// Write `cnt` elements from a wave's LDS strip to global memory with aligned 16-byte
// stores.  LDS element `pad + i` corresponds to global element g0 + i, where pad makes
// LDS byte 0 line up with a 16-byte boundary of the global buffer.  The first and
// last vector go element by element, so nothing outside [g0, g0 + cnt) is touched.
// All LDS reads of the inner vectors are issued before the first store and the two edge
// vectors are left to 2 E lanes at the end: this runs after the tile has received its
// prefix, where every instruction delays the tile's exit (a loop over the vectors with
// the edge cases inside cost compress 2 % on fp32 and 6-7 % on 16-bit tensors).
template <int S>
__device__ __forceinline__ void strip_store(const unsigned char *strip, char *g0_ptr, const uint32_t pad,
                                            const uint32_t cnt, const int lane) {
    constexpr int E = Geo<S>::E;
    static_assert(kPhaseRows * Geo<S>::ROW / E + 1 <= 2 + 4 * kWaveSize, "a phase must fit four inner vectors per lane");
    if (cnt == 0) return;
    char *gvec = g0_ptr - (size_t)pad * S;      // 16-byte aligned; may start before g0
    const uint32_t hi_valid = pad + cnt;
    const uint32_t n_vec = (hi_valid + E - 1) / E;
    // the inner vectors (all but the first and the last: at most 255, wholly inside the range), four to a lane
    uint4 t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t v = 1u + (uint32_t)lane + (uint32_t)kWaveSize * i;
        if (v + 1 < n_vec) t[i] = *reinterpret_cast<const uint4 *>(strip + (size_t)v * kVecBytes);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t v = 1u + (uint32_t)lane + (uint32_t)kWaveSize * i;
        if (v + 1 < n_vec) stream_store<kCompressNtStore>(reinterpret_cast<uint4 *>(gvec + (size_t)v * kVecBytes), t[i]);
    }
    // the first and the last vector, an element a lane: lane j < E element j of the first, lane E + j element j
    // of the last, each only if it lies inside [pad, pad + cnt)
    if (lane < 2 * E) {
        const uint32_t e = lane < E ? (uint32_t)lane : (n_vec - 1) * E + (uint32_t)(lane - E);
        if (e >= pad && e < hi_valid && (lane < E || n_vec > 1)) {
            if (S == 8) reinterpret_cast<uint64_t *>(gvec)[e] = reinterpret_cast<const uint64_t *>(strip)[e];
            else if (S == 4) reinterpret_cast<uint32_t *>(gvec)[e] = reinterpret_cast<const uint32_t *>(strip)[e];
            else reinterpret_cast<uint16_t *>(gvec)[e] = reinterpret_cast<const uint16_t *>(strip)[e];
        }
    }
}

// The reverse direction in two steps, so that the loads of several phases can be in
// flight together: strip_fetch issues the loads of values[g0, g0 + cnt) into
// registers, strip_commit later writes them into the wave's LDS strip (same layout
// as strip_store).  A phase holds at most kPhaseRows * ROW elements, i.e. 257 aligned
// vectors: the inner ones (at most 255, all fully inside the range) go four to a
// lane; of the first and the last vector, lane j < E takes element j of the first
// and lane E + j element j of the last, each only if it lies inside the range.
template <int S> struct Fetched {
    uint4 inner[4];
    typename std::conditional<S == 8, uint64_t, uint32_t>::type edge;
};

template <int S>
__device__ __forceinline__ void strip_fetch(const char *g0_ptr, const uint32_t pad, const uint32_t cnt, const int lane,
                                            Fetched<S> &f) {
    constexpr int E = Geo<S>::E;
    static_assert(kPhaseRows * Geo<S>::ROW / E + 1 <= 2 + 4 * kWaveSize, "a phase must fit four inner vectors per lane");
    const char *gvec = g0_ptr - (size_t)pad * S;
    const uint32_t hi_valid = pad + cnt;
    const uint32_t n_vec = cnt ? (hi_valid + E - 1) / E : 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t v = 1u + (uint32_t)lane + (uint32_t)kWaveSize * i;
        f.inner[i] = make_uint4(0, 0, 0, 0);
        if (v + 1 < n_vec) f.inner[i] = stream_load<kDecompressNtLoad>(reinterpret_cast<const uint4 *>(gvec + (size_t)v * kVecBytes));
    }
    f.edge = 0;
    if (lane < 2 * E && n_vec != 0) {
        const uint32_t e = lane < E ? (uint32_t)lane : (n_vec - 1) * E + (uint32_t)(lane - E);
        const bool wanted = e >= pad && e < hi_valid && (lane < E || n_vec > 1);
        if (wanted) {
            if (S == 8) f.edge = reinterpret_cast<const uint64_t *>(gvec)[e];
            else if (S == 4) f.edge = reinterpret_cast<const uint32_t *>(gvec)[e];
            else f.edge = reinterpret_cast<const uint16_t *>(gvec)[e];
        }
    }
}

template <int S>
__device__ __forceinline__ void strip_commit(unsigned char *strip, const uint32_t pad, const uint32_t cnt, const int lane,
                                             const Fetched<S> &f) {
    constexpr int E = Geo<S>::E;
    const uint32_t hi_valid = pad + cnt;
    const uint32_t n_vec = cnt ? (hi_valid + E - 1) / E : 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t v = 1u + (uint32_t)lane + (uint32_t)kWaveSize * i;
        if (v + 1 < n_vec) *reinterpret_cast<uint4 *>(strip + (size_t)v * kVecBytes) = f.inner[i];
    }
    if (lane < 2 * E && n_vec != 0) {
        const uint32_t e = lane < E ? (uint32_t)lane : (n_vec - 1) * E + (uint32_t)(lane - E);
        const bool wanted = e >= pad && e < hi_valid && (lane < E || n_vec > 1);
        if (wanted) {
            if (S == 8) reinterpret_cast<uint64_t *>(strip)[e] = f.edge;
            else if (S == 4) reinterpret_cast<uint32_t *>(strip)[e] = (uint32_t)f.edge;
            else reinterpret_cast<uint16_t *>(strip)[e] = (uint16_t)f.edge;
        }
    }
}

// ---- Algorithm 1: dense -> bitmap -------------------------------------------------------

// One tile of one tensor: `tile` counts the tensor's own tiles (it addresses the data),
// `slot` is the tile's entry in the workspace (equal to `tile` unless the call is batched).
template <int S, int KEEP, bool DENSE = false>
__device__ __forceinline__ void compress_tile(const void *in, const uint64_t n,
                                              uint32_t *__restrict__ bitmap, void *__restrict__ values,
                                              const uint64_t values_cap, char *ws, const uint32_t tile,
                                              const uint32_t slot, const uint32_t n_slots, const float threshold,
                                              unsigned char *s_stage, PrefixShared &s_prefix,
                                              uint64_t *__restrict__ index = nullptr, void *dense = nullptr) {
    using G = Geo<S>;
    constexpr int E = G::E;
    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it in a scalar register

    const uint64_t n_words = (n + 31) >> 5;
    const uint64_t wave_e0 = (uint64_t)tile * G::TILE + (uint64_t)wave * G::WAVE;
    const bool full = (uint64_t)(tile + 1) * G::TILE <= n;

    // (1) load: lane l of row k owns elements wave_e0 + k*ROW + l*E ... + E-1, and
    // (2) Algorithm 1's test "T[i] == 0", on the bit pattern.
    //     kLoadAhead rows per wave are in flight at a time; a row's mask is taken as
    //     soon as the row arrives.  (Measured on MI355X: asking for all rows at once,
    //     kLoadAhead == kRows, is fastest; 1, 2 and 4 rows ahead were 15 %, 9 % and 2 %
    //     slower on a 25.7 M element fp32 tensor.)
    uint4 x[kRows];
    uint32_t mp[G::MW], rank2[kRows / 2], total2[kRows / 2];
#pragma unroll
    for (int i = 0; i < G::MW; ++i) mp[i] = 0;
    if (full) {
        const uint4 *p = reinterpret_cast<const uint4 *>(static_cast<const char *>(in) + wave_e0 * S) + lane;
#pragma unroll
        for (int k = 0; k < kLoadAhead && k < kRows; ++k) x[k] = stream_load<kCompressNtLoad>(p + k * kWaveSize);
#pragma unroll
        for (int k = 0; k < kRows; ++k) {
            uint32_t mk = keep_mask<S, KEEP>(x[k], threshold);
            asm volatile("" : "+v"(mk));             // row k has arrived: its mask exists from here on
            mp[k / G::RPM] |= mk << (E * (k % G::RPM));
            if (k + kLoadAhead < kRows) {
                __builtin_amdgcn_sched_barrier(0);   // do not ask for the next row any earlier
                x[k + kLoadAhead] = stream_load<kCompressNtLoad>(p + (k + kLoadAhead) * kWaveSize);
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < kRows; ++k) {
            const uint64_t e0 = wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E;
            x[k] = load_vec_guarded<S>(in, e0, n);
            // elements at or beyond n read as 0, which a negative threshold would keep: mask them
            const uint32_t in_range = e0 >= n ? 0u : (n - e0 >= (uint64_t)E ? (1u << E) - 1u : (1u << (uint32_t)(n - e0)) - 1u);
            mp[k / G::RPM] |= (keep_mask<S, KEEP>(x[k], threshold) & in_range) << (E * (k % G::RPM));
        }
    }
    // Keep the masks as values of their own: otherwise the compiler keeps one compare
    // result (a scalar register pair) per element alive until the values are written.
#pragma unroll
    for (int i = 0; i < G::MW; ++i) asm volatile("" : "+v"(mp[i]));
    rank_rows<S>(mp, rank2, total2);
    uint32_t wave_total = 0;
#pragma unroll
    for (int k = 0; k < kRows; ++k) wave_total += BT_FIELD(total2, k);

    // (3) "push bit to B.bitmap": G lanes OR their E-bit masks into one 32-bit word;
    //     lane (g*G + i) keeps the word of row r0 + i, group g: one store per G rows.
    //     The store itself waits until after (4): a store in flight would delay the
    //     polling loads there, which share its completion counter.
    constexpr int kWordRegs = (kRows + G::G - 1) / G::G;
    uint32_t word[kWordRegs];
    {
        const int i = lane % G::G;
#pragma unroll
        for (int r0 = 0; r0 < kRows; r0 += G::G) {
            word[r0 / G::G] = 0;
#pragma unroll
            for (int k = r0; k < r0 + G::G && k < kRows; ++k) {
                const uint32_t w = group_or<G::G>(BT_MASK(S, mp, k) << (uint32_t)(E * i));
                if (i == k - r0) word[r0 / G::G] = w;
                // finish this row's word now: left alone, the compiler sinks the selects below
                // the wait in (4) and keeps one partial result per row alive across it
                asm volatile("" : "+v"(word[r0 / G::G]));
            }
        }
    }

    // (4) block total -> count for the scanner -> this wave's position in B.values
    uint64_t g0 = tile_prefix(ws, s_prefix, slot, n_slots, wave_total,     // index in B.values of this wave's next value
                              index != nullptr ? index + tile : nullptr);
    {
        const int g = lane / G::G, i = lane % G::G;
#pragma unroll
        for (int r0 = 0; r0 < kRows; r0 += G::G) {
            const uint64_t widx = (wave_e0 >> 5) + (uint64_t)(r0 + i) * G::WPR + (uint64_t)g;
            if (r0 + i < kRows && widx < n_words) bitmap[widx] = word[r0 / G::G];
        }
    }

    // (5) "push T[i] to B.values": kPhaseRows rows at a time, compact this wave's
    //     non-zeros into its LDS strip, then write the strip out with aligned stores.
    unsigned char *strip = s_stage + wave * G::LDS_WAVE;
#pragma unroll
    for (int r0 = 0; r0 < kRows; r0 += kPhaseRows) {
        char *gdst = static_cast<char *>(values) + g0 * S;
        const uint32_t pad = (uint32_t)(reinterpret_cast<uintptr_t>(gdst) & (kVecBytes - 1)) / S;   // elements
        if (r0 != 0) wave_lds_sync();   // the previous phase's reads are done before the strip is reused
        uint32_t row_start = pad;
#pragma unroll
        for (int k = r0; k < r0 + kPhaseRows; ++k) {
            // byte offset of this lane's next kept element from the spare vector (negative: the strip lies before it)
            int rb = ((int)(row_start + BT_FIELD(rank2, k)) - G::DUMP) * S;
            unsigned char *const dump = strip + G::DUMP * S;
            const uint32_t mk = BT_MASK(S, mp, k);
            const uint32_t d[4] = {x[k].x, x[k].y, x[k].z, x[k].w};
            // every element is written, a dropped one to a place nobody reads: a select on the address instead of
            // a branch around the write keeps the execution mask alone (half the instructions; measured 1 % on
            // compress, 4-8 % on the restoration of 16-bit tensors, where the same is done with the reads)
            if (S == 8) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int keep = (int)((mk >> j) & 1u);
                    *reinterpret_cast<uint64_t *>(dump + __mul24(keep, rb)) = ((uint64_t)d[2 * j + 1] << 32) | d[2 * j];
                    rb += keep * S;
                }
            } else if (S == 4) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int keep = (int)((mk >> j) & 1u);
                    *reinterpret_cast<uint32_t *>(dump + __mul24(keep, rb)) = d[j];
                    rb += keep * S;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int keep = (int)((mk >> j) & 1u);
                    *reinterpret_cast<uint16_t *>(dump + __mul24(keep, rb)) = (uint16_t)(d[j >> 1] >> (16 * (j & 1)));
                    rb += keep * S;
                }
            }
            row_start += BT_FIELD(total2, k);
        }
        wave_lds_sync();
        const uint32_t phase_total = row_start - pad;
        // capacity clamp: never write at or beyond values_cap
        uint32_t cnt = phase_total;
        if (g0 >= values_cap) cnt = 0;
        else if (values_cap - g0 < cnt) cnt = (uint32_t)(values_cap - g0);
        strip_store<S>(strip, gdst, pad, cnt, lane);
        g0 += phase_total;
    }

    // (6) the dense tensor after pruning, if asked for (bt_activation_compress): what survives keeps its
    //     bits, the rest is +0.  Last, so that no store precedes the polling loads of (4); `dense` may be
    //     `in` itself (every lane rewrites exactly the vectors it has read).
    if (DENSE) {
#pragma unroll
        for (int k = 0; k < kRows; ++k) {
            const uint32_t mk = BT_MASK(S, mp, k);
            uint32_t d[4] = {x[k].x, x[k].y, x[k].z, x[k].w};
            // masks by arithmetic (0 - bit is all ones or zero), not by compares: see nonzero_mask
            if (S == 8) {
#pragma unroll
                for (int j = 0; j < 4; ++j) d[j] &= 0u - ((mk >> (j >> 1)) & 1u);
            } else if (S == 4) {
#pragma unroll
                for (int j = 0; j < 4; ++j) d[j] &= 0u - ((mk >> j) & 1u);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    d[j] &= (((mk >> (2 * j)) & 1u) * 0x0000ffffu) | (((mk >> (2 * j + 1)) & 1u) * 0xffff0000u);
            }
            const uint64_t e0 = wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E;
            const uint4 o = make_uint4(d[0], d[1], d[2], d[3]);
            if (full) stream_store<kCompressNtStore>(reinterpret_cast<uint4 *>(static_cast<char *>(dense) + e0 * S), o);
            else store_vec_guarded<S>(dense, e0, n, o);
        }
    }
}

// bt_compress / bt_compress_pruned: one tensor.  Workgroup 0 is the scanner, workgroup
// t + 1 is tile t.
template <int S, int KEEP, bool DENSE>
__global__ __launch_bounds__(kBlock, 8) void compress_kernel(const void *in, const uint64_t n,
                                                          uint32_t *__restrict__ bitmap, void *__restrict__ values,
                                                          const uint64_t values_cap, uint64_t *__restrict__ nnz_out,
                                                          char *ws, const uint32_t n_tiles, const float threshold,
                                                          uint64_t *__restrict__ index, void *dense) {
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[kWaves * Geo<S>::LDS_WAVE];
    __shared__ PrefixShared s_prefix;
    if (workspace_failed(ws)) return;
    if (blockIdx.x == 0) {
        if (threadIdx.x < kWaveSize) {
            const uint32_t start[2] = {0, n_tiles};
            uint64_t *const nnz[1] = {nnz_out};
            scan_counts(ws, Segments{1, start, nnz});
        }
        return;
    }
    const uint32_t tile = blockIdx.x - 1;
    BT_TL(tile, 0);
    compress_tile<S, KEEP, DENSE>(in, n, bitmap, values, values_cap, ws, tile, tile, n_tiles, threshold, s_stage,
                                  s_prefix, index, dense);
#ifdef BT_TIMELINE
    BT_TL(tile, 3);
    if (threadIdx.x == 0) __builtin_amdgcn_s_waitcnt(0);     // this wave's stores have been acknowledged
    BT_TL(tile, 4);
#endif
}

// Several tensors in one launch (bt_compress_batch): the kernel arguments carry the
// per-tensor pointers; a workgroup finds its tensor by binary search over the slot
// starts.  Slots that belong to no tile only do their share of the workspace clean-up.
constexpr int kMaxBatch = BT_MAX_BATCH;
struct BatchLayout {
    uint32_t count;
    uint32_t start[kMaxBatch + 1];
    uint32_t tiles[kMaxBatch];
};
struct CompressBatch {
    BatchLayout lay;
    const void *in[kMaxBatch];
    uint32_t *bitmap[kMaxBatch];
    void *values[kMaxBatch];
    uint64_t cap[kMaxBatch];
    uint64_t *nnz[kMaxBatch];
    uint64_t n[kMaxBatch];
};

__device__ __forceinline__ uint32_t batch_item_of(const BatchLayout &lay, const uint32_t slot) {
    uint32_t lo = 0, hi = lay.count;          // start[lo] <= slot < start[hi]
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (slot >= lay.start[mid]) lo = mid; else hi = mid;
    }
    return lo;
}

template <int S>
__global__ __launch_bounds__(kBlock, 8) void compress_batch_kernel(const CompressBatch b, char *ws) {
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[kWaves * Geo<S>::LDS_WAVE];
    __shared__ PrefixShared s_prefix;
    if (workspace_failed(ws)) return;
    const uint32_t n_slots = b.lay.start[b.lay.count];
    if (blockIdx.x == 0) {
        if (threadIdx.x < kWaveSize) scan_counts(ws, Segments{b.lay.count, b.lay.start, b.nnz});
        return;
    }
    const uint32_t slot = blockIdx.x - 1;
    const uint32_t i = batch_item_of(b.lay, slot);
    const uint32_t tile = slot - b.lay.start[i];
    if (tile >= b.lay.tiles[i]) {
        idle_slot(ws, slot, n_slots);
        return;
    }
    compress_tile<S, kKeepNonZero>(b.in[i], b.n[i], b.bitmap[i], b.values[i], b.cap[i], ws, tile, slot, n_slots, 0.0f,
                                   s_stage, s_prefix);
}

// ---- Algorithm 2: bitmap -> dense ---------------------------------------------------------

// INDEXED: Algorithm 2's j at the start of the tile is read from a tile index (written by
// bt_compress_indexed) instead of being found by the grid scan: no workspace, no waiting;
// values at or beyond values_cap are never read.
template <int S, bool INDEXED = false>
__device__ __forceinline__ void decompress_tile(const uint32_t *__restrict__ bitmap, const void *__restrict__ values,
                                                const uint64_t n, void *__restrict__ out, char *ws,
                                                const uint32_t tile, const uint32_t slot, const uint32_t n_slots,
                                                unsigned char *s_stage, PrefixShared &s_prefix,
                                                const uint64_t *__restrict__ index = nullptr,
                                                const uint64_t values_cap = ~(uint64_t)0) {
    using G = Geo<S>;
    constexpr int E = G::E;
    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it in a scalar register
    uint64_t tile_j = 0;
    if (INDEXED) tile_j = index[tile];                           // asked for first, needed last

    const uint64_t n_words = (n + 31) >> 5;
    const uint64_t wave_e0 = (uint64_t)tile * G::TILE + (uint64_t)wave * G::WAVE;

    // (1) this lane's bits of "B.bitmap[i] is set", and Algorithm 2's counter j as ranks
    uint32_t mp[G::MW], rank2[kRows / 2], total2[kRows / 2];
#pragma unroll
    for (int i = 0; i < G::MW; ++i) mp[i] = 0;
    const bool full = (uint64_t)(tile + 1) * G::TILE <= n;
    if (full) {
        // every word of the tile exists and every bit of it counts: G lanes read the same word and take E bits each
        const uint32_t *p = bitmap + (wave_e0 >> 5) + (uint32_t)(lane / G::G);
        const uint32_t shift = (uint32_t)(lane % G::G) * E;
#pragma unroll
        for (int k = 0; k < kRows; ++k)
            mp[k / G::RPM] |= ((p[k * G::WPR] >> shift) & ((1u << E) - 1u)) << (E * (k % G::RPM));
    } else {
#pragma unroll
        for (int k = 0; k < kRows; ++k)
            mp[k / G::RPM] |= bitmap_bits<S>(bitmap, wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E, n, n_words)
                              << (E * (k % G::RPM));
    }
    rank_rows<S>(mp, rank2, total2);
    uint32_t wave_total = 0;
#pragma unroll
    for (int k = 0; k < kRows; ++k) wave_total += BT_FIELD(total2, k);

    // (2) block total -> count for the scanner -> this wave's value of j
    uint64_t g0;                                                          // Algorithm 2's j for this wave
    if (INDEXED) {
        if (lane == 0) s_prefix.wave_total[wave] = wave_total;
        __syncthreads();
        g0 = tile_j;
        for (int w = 0; w < wave; ++w) g0 += s_prefix.wave_total[w];
        g0 = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(g0 >> 32)) << 32) |
             (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)g0);
    } else {
        g0 = tile_prefix(ws, s_prefix, slot, n_slots, wave_total);
    }

    // (3) Ask for the values of every phase (kPhaseRows rows each) first, so that all of
    //     them are in flight together; then, phase by phase, put them into the LDS strip
    //     and "push B.values[j] / push 0.0 to T": expand from LDS by rank and store 16
    //     bytes per lane.  No load is issued after the first store: loads and stores
    //     share one completion counter, and a load waited for after a store would also
    //     wait for that store to reach memory.
    constexpr int kPhases = kRows / kPhaseRows;
    unsigned char *strip = s_stage + wave * G::LDS_WAVE;
    Fetched<S> fetched[kPhases];
    uint32_t pads[kPhases], cnts[kPhases];
#pragma unroll
    for (int ph = 0; ph < kPhases; ++ph) {
        cnts[ph] = 0;
#pragma unroll
        for (int k = ph * kPhaseRows; k < (ph + 1) * kPhaseRows; ++k) cnts[ph] += BT_FIELD(total2, k);
        const char *gsrc = static_cast<const char *>(values) + g0 * S;
        pads[ph] = (uint32_t)(reinterpret_cast<uintptr_t>(gsrc) & (kVecBytes - 1)) / S;
        const uint32_t phase_total = cnts[ph];
        if (INDEXED) {   // an index that does not belong to this bitmap must not lead outside d_values
            if (g0 >= values_cap) cnts[ph] = 0;
            else if (values_cap - g0 < cnts[ph]) cnts[ph] = (uint32_t)(values_cap - g0);
        }
        strip_fetch<S>(gsrc, pads[ph], cnts[ph], lane, fetched[ph]);
        g0 += phase_total;
    }
#pragma unroll
    for (int ph = 0; ph < kPhases; ++ph) {
        if (ph != 0) wave_lds_sync();   // the previous phase's reads are done before the strip is reused
        strip_commit<S>(strip, pads[ph], cnts[ph], lane, fetched[ph]);
        wave_lds_sync();
        uint32_t row_start = pads[ph];
#pragma unroll
        for (int k = ph * kPhaseRows; k < (ph + 1) * kPhaseRows; ++k) {
            uint32_t r = row_start + BT_FIELD(rank2, k);
            const uint32_t mk = BT_MASK(S, mp, k);
            uint32_t d[4] = {0, 0, 0, 0};
            // every lane reads at its running rank whether the bit is set or not (the index stays inside the strip)
            // and a select drops what a cleared bit read
            if (S == 8) {
                const uint64_t *l = reinterpret_cast<const uint64_t *>(strip);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const uint32_t keep = (mk >> j) & 1u;
                    const uint64_t v = l[r];
                    d[2 * j] = keep ? (uint32_t)v : 0u;
                    d[2 * j + 1] = keep ? (uint32_t)(v >> 32) : 0u;
                    r += keep;
                }
            } else if (S == 4) {
                const uint32_t *l = reinterpret_cast<const uint32_t *>(strip);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t keep = (mk >> j) & 1u;
                    const uint32_t v = l[r];
                    d[j] = keep ? v : 0u;
                    r += keep;
                }
            } else {
                const uint16_t *l = reinterpret_cast<const uint16_t *>(strip);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t keep = (mk >> j) & 1u;
                    const uint32_t v = l[r];
                    d[j >> 1] |= (keep ? v : 0u) << (16 * (j & 1));
                    r += keep;
                }
            }
            const uint64_t e0 = wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E;
            const uint4 o = make_uint4(d[0], d[1], d[2], d[3]);
            if (full) stream_store<kDecompressNtStore>(reinterpret_cast<uint4 *>(static_cast<char *>(out) + e0 * S), o);
            else store_vec_guarded<S>(out, e0, n, o);
            row_start += BT_FIELD(total2, k);
        }
    }
}

template <int S>
__global__ __launch_bounds__(kBlock, 8) void decompress_kernel(const uint32_t *__restrict__ bitmap,
                                                            const void *__restrict__ values, const uint64_t n,
                                                            void *__restrict__ out, char *ws, const uint32_t n_tiles) {
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[kWaves * Geo<S>::LDS_WAVE];
    __shared__ PrefixShared s_prefix;
    if (workspace_failed(ws)) return;
    if (blockIdx.x == 0) {
        if (threadIdx.x < kWaveSize) {
            const uint32_t start[2] = {0, n_tiles};
            scan_counts(ws, Segments{1, start, nullptr});
        }
        return;
    }
    const uint32_t tile = blockIdx.x - 1;
    BT_TL(tile, 0);
    decompress_tile<S>(bitmap, values, n, out, ws, tile, tile, n_tiles, s_stage, s_prefix);
#ifdef BT_TIMELINE
    BT_TL(tile, 3);
    if (threadIdx.x == 0) __builtin_amdgcn_s_waitcnt(0);     // this wave's stores have been acknowledged
    BT_TL(tile, 4);
#endif
}

struct DecompressBatch {
    BatchLayout lay;
    const uint32_t *bitmap[kMaxBatch];
    const void *values[kMaxBatch];
    void *out[kMaxBatch];
    uint64_t n[kMaxBatch];
};

template <int S>
__global__ __launch_bounds__(kBlock, 8) void decompress_batch_kernel(const DecompressBatch b, char *ws) {
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[kWaves * Geo<S>::LDS_WAVE];
    __shared__ PrefixShared s_prefix;
    if (workspace_failed(ws)) return;
    const uint32_t n_slots = b.lay.start[b.lay.count];
    if (blockIdx.x == 0) {
        if (threadIdx.x < kWaveSize) scan_counts(ws, Segments{b.lay.count, b.lay.start, nullptr});
        return;
    }
    const uint32_t slot = blockIdx.x - 1;
    const uint32_t i = batch_item_of(b.lay, slot);
    const uint32_t tile = slot - b.lay.start[i];
    if (tile >= b.lay.tiles[i]) {
        idle_slot(ws, slot, n_slots);
        return;
    }
    decompress_tile<S>(b.bitmap[i], b.values[i], b.n[i], b.out[i], ws, tile, slot, n_slots, s_stage, s_prefix);
}

// bt_decompress_indexed: one workgroup per tile and nothing else.
template <int S>
__global__ __launch_bounds__(kBlock, 8) void decompress_indexed_kernel(const uint32_t *__restrict__ bitmap,
                                                                    const void *__restrict__ values,
                                                                    const uint64_t values_cap,
                                                                    const uint64_t *__restrict__ index, const uint64_t n,
                                                                    void *__restrict__ out) {
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[kWaves * Geo<S>::LDS_WAVE];
    __shared__ PrefixShared s_prefix;
    decompress_tile<S, true>(bitmap, values, n, out, nullptr, blockIdx.x, 0, 0, s_stage, s_prefix, index, values_cap);
}

// ---- ReLU backward from the bitmap -----------------------------------------------------------

// grad_in[i] = bit(i) ? grad_out[i] : +0.  Pure streaming: no scan, no LDS.  Each
// lane selects per element with the E bits that cover its 16-byte vector.
template <int S>
__global__ __launch_bounds__(kBlock) void relu_backward_kernel(const uint32_t *__restrict__ bitmap,
                                                               const void *grad_out, const uint64_t n,
                                                               void *grad_in) {
    using G = Geo<S>;
    constexpr int E = G::E;
    constexpr int kR = kReluRows;                       // 16-byte vectors per lane
    constexpr int kTile = kBlock * kR * E;              // elements per block
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t n_words = (n + 31) >> 5;
    const uint64_t wave_e0 = (uint64_t)blockIdx.x * kTile + (uint64_t)wave * (kR * G::ROW);
    const bool full = ((uint64_t)blockIdx.x + 1) * kTile <= n;

    uint4 g[kR];
    uint32_t m[kR];
#pragma unroll
    for (int k = 0; k < kR; ++k) {
        const uint64_t e0 = wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E;
        if (full) {
            g[k] = stream_load<kReluNtLoad>(reinterpret_cast<const uint4 *>(static_cast<const char *>(grad_out) + e0 * S));
            m[k] = (bitmap[e0 >> 5] >> (uint32_t)(e0 & 31)) & ((1u << E) - 1u);
        } else {
            g[k] = load_vec_guarded<S>(grad_out, e0, n);
            m[k] = bitmap_bits<S>(bitmap, e0, n, n_words);
        }
    }
#pragma unroll
    for (int k = 0; k < kR; ++k) {
        const uint64_t e0 = wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E;
        uint32_t d[4] = {g[k].x, g[k].y, g[k].z, g[k].w};
        if (S == 8) {
#pragma unroll
            for (int j = 0; j < 4; ++j) d[j] = (m[k] & (1u << (j >> 1))) ? d[j] : 0u;
        } else if (S == 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) d[j] = (m[k] & (1u << j)) ? d[j] : 0u;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t keep = ((m[k] & (1u << (2 * j))) ? 0x0000ffffu : 0u) |
                                      ((m[k] & (1u << (2 * j + 1))) ? 0xffff0000u : 0u);
                d[j] &= keep;
            }
        }
        const uint4 o = make_uint4(d[0], d[1], d[2], d[3]);
        if (full) stream_store<kReluNtStore>(reinterpret_cast<uint4 *>(static_cast<char *>(grad_in) + e0 * S), o);
        else store_vec_guarded<S>(grad_in, e0, n, o);
    }
}

// ---- measurement aid: a stream with the codec's traffic and no dependency -----------------

// Workgroup t reads R rows of 256 16-byte vectors from `in` and writes W such rows to `out`,
// both contiguous per workgroup and per wave, with the same cache hints as the codec.
// Nothing waits for anything: this is what the memory system gives the codec's access
// pattern at best, the figure the codec kernels are compared with.
constexpr int kProbeThreads = 256;     // a row is 256 lanes x 16 bytes = 4 KiB, whatever the codec's workgroup size
template <int R, int W>
__global__ __launch_bounds__(kProbeThreads) void stream_probe_kernel(const uint4 *__restrict__ in, uint4 *__restrict__ out,
                                                              const uint32_t tiles) {
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t t = blockIdx.x;
    if (t >= tiles) return;
    uint4 acc = make_uint4(1, 2, 3, (uint32_t)t);
    if (R > 0) {
        uint4 v[R > 0 ? R : 1];
        const uint64_t base = (t * (kProbeThreads / kWaveSize) + wave) * (uint64_t)(kWaveSize * R) + lane;
#pragma unroll
        for (int k = 0; k < R; ++k) v[k] = stream_load<true>(in + base + kWaveSize * k);
#pragma unroll
        for (int k = 0; k < R; ++k) {
            acc.x ^= v[k].x; acc.y ^= v[k].y; acc.z ^= v[k].z; acc.w ^= v[k].w;
        }
    }
    if (W > 0) {
        const uint64_t base = (t * (kProbeThreads / kWaveSize) + wave) * (uint64_t)(kWaveSize * W) + lane;
#pragma unroll
        for (int k = 0; k < W; ++k) {
            uint4 o = acc;
            o.x += k;
            stream_store<true>(out + base + kWaveSize * k, o);
        }
    } else if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) {
        out[t] = acc;          // keeps the loads alive; practically never taken
    }
}

// ---- small fills ---------------------------------------------------------------------------

__global__ void fill_u64_kernel(uint64_t *p, uint64_t count, uint64_t value) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = value;
}

// ---- host side ---------------------------------------------------------------------------------

int elem_size(bt_dtype dt) {
    switch (dt) {
        case BT_F32: return 4;
        case BT_F16: return 2;
        case BT_BF16: return 2;
        case BT_F64: return 8;
    }
    return 0;
}

uint64_t tile_elems(int s) { return (uint64_t)kBlock * kRows * (kVecBytes / s); }

uint64_t tiles_for(uint64_t n, int s) {
    const uint64_t t = tile_elems(s);
    return (n + t - 1) / t;
}

uint64_t relu_blocks_for(uint64_t n, int s) {
    const uint64_t t = (uint64_t)kBlock * kReluRows * (kVecBytes / s);
    return (n + t - 1) / t;
}

bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

bt_status launched() { return hipGetLastError() == hipSuccess ? BT_OK : BT_ERR_HIP; }

bt_status check_common(uint64_t n, bt_dtype dt, const void *d_ws, size_t ws_bytes) {
    if (elem_size(dt) == 0) return BT_ERR_DTYPE;
    if (n > BT_MAX_ELEMENTS) return BT_ERR_SIZE;
    if (n == 0) return BT_OK;
    if (d_ws == nullptr) return BT_ERR_NULL;
    if (misaligned(d_ws, 128)) return BT_ERR_ALIGN;
    if (ws_bytes < bt_workspace_bytes(n, dt)) return BT_ERR_WORKSPACE;
    return BT_OK;
}

// Slots a tensor of n elements takes in a batched launch: its tiles rounded up to whole
// scanner rows; an empty tensor still takes one row, so that the scanner writes its nnz.
uint64_t batch_slots_for(uint64_t n, int s) {
    const uint64_t tiles = tiles_for(n, s);
    return ((tiles == 0 ? 1 : tiles) + kWaveSize - 1) / kWaveSize * kWaveSize;
}

size_t workspace_bytes_for_slots(uint64_t slots) {
    uint64_t records = (slots + kTilesPerRecord - 1) / kTilesPerRecord;
    if (records == 0) records = 1;
    return kHeaderBytes + (size_t)records * kRecordBytes;
}

// Tensors [first, first + lay.count) of a batch, laid end to end.  `n_of(i)` is tensor i's element count.
template <class NOf>
void lay_out(BatchLayout &lay, size_t first, size_t count, int s, NOf n_of) {
    lay.count = (uint32_t)count;
    uint64_t at = 0;
    for (size_t i = 0; i < count; ++i) {
        const uint64_t n = n_of(first + i);
        lay.start[i] = (uint32_t)at;
        lay.tiles[i] = (uint32_t)tiles_for(n, s);
        at += batch_slots_for(n, s);
    }
    for (size_t i = count; i <= (size_t)kMaxBatch; ++i) lay.start[i] = (uint32_t)at;
    for (size_t i = count; i < (size_t)kMaxBatch; ++i) lay.tiles[i] = 0;
}

// Largest workspace any launch of the batch needs (a batch of more than kMaxBatch
// tensors is cut into consecutive launches of kMaxBatch, which reuse the workspace).
template <class NOf>
size_t batch_workspace_bytes(size_t count, int s, NOf n_of) {
    size_t need = workspace_bytes_for_slots(0);
    for (size_t first = 0; first < count; first += kMaxBatch) {
        const size_t c = count - first < (size_t)kMaxBatch ? count - first : (size_t)kMaxBatch;
        uint64_t slots = 0;
        for (size_t i = 0; i < c; ++i) slots += batch_slots_for(n_of(first + i), s);
        const size_t b = workspace_bytes_for_slots(slots);
        if (b > need) need = b;
    }
    return need;
}

bt_status check_batch_common(const void *items, size_t count, bt_dtype dt, const void *d_ws) {
    if (elem_size(dt) == 0) return BT_ERR_DTYPE;
    if (count == 0) return BT_OK;
    if (items == nullptr || d_ws == nullptr) return BT_ERR_NULL;
    if (misaligned(d_ws, 128)) return BT_ERR_ALIGN;
    return BT_OK;
}

}  // namespace

extern "C" {

size_t bt_dtype_size(bt_dtype dtype) { return (size_t)elem_size(dtype); }

size_t bt_bitmap_bytes(uint64_t n) { return (size_t)(4 * ((n + 31) / 32)); }

size_t bt_compressed_size(uint64_t n, uint64_t nnz, bt_dtype dtype) {
    const int s = elem_size(dtype);
    if (s == 0 || nnz > n) return 0;
    return (size_t)(4 * ((n + 31) / 32) + nnz * (uint64_t)s);
}

size_t bt_dense_size(uint64_t n, bt_dtype dtype) { return (size_t)(n * (uint64_t)elem_size(dtype)); }

size_t bt_coo_size(uint64_t nnz, uint32_t ndim, uint32_t index_bytes, bt_dtype dtype) {
    const int s = elem_size(dtype);
    if (s == 0 || ndim == 0 || (index_bytes != 4 && index_bytes != 8)) return 0;
    return (size_t)(((uint64_t)s + (uint64_t)index_bytes * ndim) * nnz);
}

size_t bt_workspace_bytes(uint64_t n, bt_dtype dtype) {
    const int s = elem_size(dtype);
    if (s == 0) return 0;
    return workspace_bytes_for_slots(tiles_for(n, s));
}

const char *bt_status_str(bt_status status) {
    switch (status) {
        case BT_OK: return "ok";
        case BT_ERR_NULL: return "null pointer";
        case BT_ERR_DTYPE: return "unknown dtype";
        case BT_ERR_ALIGN: return "misaligned pointer";
        case BT_ERR_WORKSPACE: return "workspace too small";
        case BT_ERR_HIP: return "HIP launch failed";
        case BT_ERR_SIZE: return "element count too large";
        case BT_ERR_UNSUPPORTED: return "not available in this build of the library";
    }
    return "unknown status";
}

bt_status bt_workspace_init(void *d_workspace, size_t workspace_bytes, bt_stream stream) {
    if (d_workspace == nullptr) return BT_ERR_NULL;
    if (misaligned(d_workspace, 128)) return BT_ERR_ALIGN;
    const uint64_t count = workspace_bytes / 8;
    if (count == 0) return BT_OK;
    const unsigned blocks = (unsigned)((count + 255) / 256);
    fill_u64_kernel<<<dim3(blocks), dim3(256), 0, (hipStream_t)stream>>>((uint64_t *)d_workspace, count, 0);
    return launched();
}

static bt_status compress_common(const void *d_in, uint64_t n, bt_dtype dtype, bool prune, float threshold,
                                 uint32_t *d_bitmap, void *d_values, uint64_t values_cap, uint64_t *d_nnz,
                                 uint64_t *d_index, void *d_dense, void *d_workspace, size_t workspace_bytes,
                                 bt_stream stream) {
    const bt_status st = check_common(n, dtype, d_workspace, workspace_bytes);
    if (st != BT_OK) return st;
    if (d_nnz == nullptr) return BT_ERR_NULL;
    if (misaligned(d_nnz, 8)) return BT_ERR_ALIGN;
    const int s = elem_size(dtype);
    hipStream_t hs = (hipStream_t)stream;
    if (n == 0) {
        fill_u64_kernel<<<dim3(1), dim3(64), 0, hs>>>(d_nnz, 1, 0);
        return launched();
    }
    if (d_in == nullptr || d_bitmap == nullptr) return BT_ERR_NULL;
    if (d_values == nullptr && values_cap != 0) return BT_ERR_NULL;
    if (misaligned(d_in, 16) || misaligned(d_bitmap, 4) || misaligned(d_values, (size_t)s)) return BT_ERR_ALIGN;

    const uint32_t n_tiles = (uint32_t)tiles_for(n, s);
    char *ws = static_cast<char *>(d_workspace);
    const dim3 grid(n_tiles + 1), block(kBlock);
#define BT_LAUNCH_COMPRESS(S_, KEEP_, DENSE_) \
    compress_kernel<S_, KEEP_, DENSE_><<<grid, block, 0, hs>>>(d_in, n, d_bitmap, d_values, values_cap, d_nnz, ws, n_tiles, threshold, d_index, d_dense)
    if (!prune) {
        if (s == 8) BT_LAUNCH_COMPRESS(8, kKeepNonZero, false);
        else if (s == 4) BT_LAUNCH_COMPRESS(4, kKeepNonZero, false);
        else BT_LAUNCH_COMPRESS(2, kKeepNonZero, false);
    } else if (d_dense == nullptr) {
        if (dtype == BT_F64) BT_LAUNCH_COMPRESS(8, kKeepAboveF64, false);
        else if (dtype == BT_F32) BT_LAUNCH_COMPRESS(4, kKeepAboveF32, false);
        else if (dtype == BT_F16) BT_LAUNCH_COMPRESS(2, kKeepAboveF16, false);
        else BT_LAUNCH_COMPRESS(2, kKeepAboveBF16, false);
    } else {
        if (dtype == BT_F64) BT_LAUNCH_COMPRESS(8, kKeepAboveF64, true);
        else if (dtype == BT_F32) BT_LAUNCH_COMPRESS(4, kKeepAboveF32, true);
        else if (dtype == BT_F16) BT_LAUNCH_COMPRESS(2, kKeepAboveF16, true);
        else BT_LAUNCH_COMPRESS(2, kKeepAboveBF16, true);
    }
#undef BT_LAUNCH_COMPRESS
    return launched();
}

bt_status bt_compress(const void *d_in, uint64_t n, bt_dtype dtype, uint32_t *d_bitmap, void *d_values,
                      uint64_t values_cap, uint64_t *d_nnz, void *d_workspace, size_t workspace_bytes,
                      bt_stream stream) {
    return compress_common(d_in, n, dtype, false, 0.0f, d_bitmap, d_values, values_cap, d_nnz, nullptr, nullptr,
                           d_workspace, workspace_bytes, stream);
}

bt_status bt_compress_pruned(const void *d_in, uint64_t n, bt_dtype dtype, float threshold, uint32_t *d_bitmap,
                             void *d_values, uint64_t values_cap, uint64_t *d_nnz, void *d_workspace,
                             size_t workspace_bytes, bt_stream stream) {
    return compress_common(d_in, n, dtype, true, threshold, d_bitmap, d_values, values_cap, d_nnz, nullptr, nullptr,
                           d_workspace, workspace_bytes, stream);
}

bt_status bt_activation_compress(const void *d_in, uint64_t n, bt_dtype dtype, float threshold, void *d_dense_out,
                                 uint32_t *d_bitmap, void *d_values, uint64_t values_cap, uint64_t *d_nnz,
                                 void *d_workspace, size_t workspace_bytes, bt_stream stream) {
    if (elem_size(dtype) != 0 && n != 0 && n <= BT_MAX_ELEMENTS) {
        if (d_dense_out == nullptr) return BT_ERR_NULL;
        if (misaligned(d_dense_out, 16)) return BT_ERR_ALIGN;
    }
    return compress_common(d_in, n, dtype, true, threshold, d_bitmap, d_values, values_cap, d_nnz, nullptr, d_dense_out,
                           d_workspace, workspace_bytes, stream);
}

size_t bt_tile_elems(bt_dtype dtype) {
    const int s = elem_size(dtype);
    return s == 0 ? 0 : (size_t)tile_elems(s);
}

size_t bt_index_bytes(uint64_t n, bt_dtype dtype) {
    const int s = elem_size(dtype);
    return s == 0 ? 0 : (size_t)(8 * tiles_for(n, s));
}

bt_status bt_compress_indexed(const void *d_in, uint64_t n, bt_dtype dtype, uint32_t *d_bitmap, void *d_values,
                              uint64_t values_cap, uint64_t *d_nnz, uint64_t *d_index, void *d_workspace,
                              size_t workspace_bytes, bt_stream stream) {
    if (elem_size(dtype) != 0 && n != 0 && n <= BT_MAX_ELEMENTS) {
        if (d_index == nullptr) return BT_ERR_NULL;
        if (misaligned(d_index, 8)) return BT_ERR_ALIGN;
    }
    return compress_common(d_in, n, dtype, false, 0.0f, d_bitmap, d_values, values_cap, d_nnz, d_index, nullptr,
                           d_workspace, workspace_bytes, stream);
}

bt_status bt_decompress_indexed(const uint32_t *d_bitmap, const void *d_values, uint64_t values_cap,
                                const uint64_t *d_index, uint64_t n, bt_dtype dtype, void *d_out, bt_stream stream) {
    const int s = elem_size(dtype);
    if (s == 0) return BT_ERR_DTYPE;
    if (n > BT_MAX_ELEMENTS) return BT_ERR_SIZE;
    if (n == 0) return BT_OK;
    if (d_bitmap == nullptr || d_out == nullptr || d_index == nullptr) return BT_ERR_NULL;
    if (d_values == nullptr && values_cap != 0) return BT_ERR_NULL;
    if (misaligned(d_out, 16) || misaligned(d_bitmap, 4) || misaligned(d_values, (size_t)s) || misaligned(d_index, 8))
        return BT_ERR_ALIGN;
    hipStream_t hs = (hipStream_t)stream;
    const dim3 grid((uint32_t)tiles_for(n, s)), block(kBlock);
    if (s == 8) decompress_indexed_kernel<8><<<grid, block, 0, hs>>>(d_bitmap, d_values, values_cap, d_index, n, d_out);
    else if (s == 4) decompress_indexed_kernel<4><<<grid, block, 0, hs>>>(d_bitmap, d_values, values_cap, d_index, n, d_out);
    else decompress_indexed_kernel<2><<<grid, block, 0, hs>>>(d_bitmap, d_values, values_cap, d_index, n, d_out);
    return launched();
}

bt_status bt_decompress(const uint32_t *d_bitmap, const void *d_values, uint64_t n, bt_dtype dtype, void *d_out,
                        void *d_workspace, size_t workspace_bytes, bt_stream stream) {
    const bt_status st = check_common(n, dtype, d_workspace, workspace_bytes);
    if (st != BT_OK) return st;
    if (n == 0) return BT_OK;
    const int s = elem_size(dtype);
    if (d_bitmap == nullptr || d_out == nullptr) return BT_ERR_NULL;   // d_values may be NULL when nnz == 0
    if (misaligned(d_out, 16) || misaligned(d_bitmap, 4) || misaligned(d_values, (size_t)s)) return BT_ERR_ALIGN;

    hipStream_t hs = (hipStream_t)stream;
    const uint32_t n_tiles = (uint32_t)tiles_for(n, s);
    char *ws = static_cast<char *>(d_workspace);
    if (s == 8)
        decompress_kernel<8><<<dim3(n_tiles + 1), dim3(kBlock), 0, hs>>>(d_bitmap, d_values, n, d_out, ws, n_tiles);
    else if (s == 4)
        decompress_kernel<4><<<dim3(n_tiles + 1), dim3(kBlock), 0, hs>>>(d_bitmap, d_values, n, d_out, ws, n_tiles);
    else
        decompress_kernel<2><<<dim3(n_tiles + 1), dim3(kBlock), 0, hs>>>(d_bitmap, d_values, n, d_out, ws, n_tiles);
    return launched();
}

bt_status bt_relu_backward_from_bitmap(const uint32_t *d_bitmap, const void *d_grad_out, uint64_t n, bt_dtype dtype,
                                       void *d_grad_in, bt_stream stream) {
    const int s = elem_size(dtype);
    if (s == 0) return BT_ERR_DTYPE;
    if (n > BT_MAX_ELEMENTS) return BT_ERR_SIZE;
    if (n == 0) return BT_OK;
    if (d_bitmap == nullptr || d_grad_out == nullptr || d_grad_in == nullptr) return BT_ERR_NULL;
    if (misaligned(d_grad_out, 16) || misaligned(d_grad_in, 16) || misaligned(d_bitmap, 4)) return BT_ERR_ALIGN;
    hipStream_t hs = (hipStream_t)stream;
    const uint32_t blocks = (uint32_t)relu_blocks_for(n, s);
    if (s == 8)
        relu_backward_kernel<8><<<dim3(blocks), dim3(kBlock), 0, hs>>>(d_bitmap, d_grad_out, n, d_grad_in);
    else if (s == 4)
        relu_backward_kernel<4><<<dim3(blocks), dim3(kBlock), 0, hs>>>(d_bitmap, d_grad_out, n, d_grad_in);
    else
        relu_backward_kernel<2><<<dim3(blocks), dim3(kBlock), 0, hs>>>(d_bitmap, d_grad_out, n, d_grad_in);
    return launched();
}

bt_status bt_mask_apply(const uint32_t *d_bitmap, const void *d_in, uint64_t n, bt_dtype dtype, void *d_out,
                        bt_stream stream) {
    return bt_relu_backward_from_bitmap(d_bitmap, d_in, n, dtype, d_out, stream);
}

bt_status bt_stream_probe(const void *d_in, void *d_out, uint64_t tiles, int read_rows, int write_rows,
                          bt_stream stream) {
    if (d_in == nullptr || d_out == nullptr) return BT_ERR_NULL;
    if (misaligned(d_in, 16) || misaligned(d_out, 16)) return BT_ERR_ALIGN;
    if (tiles == 0) return BT_OK;
    if (tiles > 0x7fffffffu) return BT_ERR_SIZE;
    hipStream_t hs = (hipStream_t)stream;
    const dim3 grid((uint32_t)tiles), block(kProbeThreads);
    const uint4 *in = static_cast<const uint4 *>(d_in);
    uint4 *out = static_cast<uint4 *>(d_out);
    const uint32_t t = (uint32_t)tiles;
    if (read_rows == 8 && write_rows == 4) stream_probe_kernel<8, 4><<<grid, block, 0, hs>>>(in, out, t);
    else if (read_rows == 4 && write_rows == 8) stream_probe_kernel<4, 8><<<grid, block, 0, hs>>>(in, out, t);
    else if (read_rows == 8 && write_rows == 8) stream_probe_kernel<8, 8><<<grid, block, 0, hs>>>(in, out, t);
    else if (read_rows == 8 && write_rows == 0) stream_probe_kernel<8, 0><<<grid, block, 0, hs>>>(in, out, t);
    else if (read_rows == 0 && write_rows == 8) stream_probe_kernel<0, 8><<<grid, block, 0, hs>>>(in, out, t);
    else return BT_ERR_SIZE;
    return launched();
}

bt_status bt_timeline_set(uint64_t *d_buf, uint64_t buf_words, uint32_t tiles, uint32_t max_passes) {
#ifdef BT_TIMELINE
    if (d_buf == nullptr) tiles = max_passes = 0;
    else if (misaligned(d_buf, 8)) return BT_ERR_ALIGN;
    if (8 * (uint64_t)tiles + 2 * (uint64_t)max_passes > buf_words) return BT_ERR_SIZE;
    // blocking copies: this call is the one place where the library waits for the device
    if (hipMemcpyToSymbol(HIP_SYMBOL(g_timeline_tiles), &tiles, sizeof(tiles)) != hipSuccess ||
        hipMemcpyToSymbol(HIP_SYMBOL(g_timeline_passes), &max_passes, sizeof(max_passes)) != hipSuccess ||
        hipMemcpyToSymbol(HIP_SYMBOL(g_timeline), &d_buf, sizeof(d_buf)) != hipSuccess)
        return BT_ERR_HIP;
    return BT_OK;
#else
    (void)d_buf; (void)buf_words; (void)tiles; (void)max_passes;
    return BT_ERR_UNSUPPORTED;
#endif
}

size_t bt_batch_workspace_bytes(const uint64_t *n, size_t count, bt_dtype dtype) {
    const int s = elem_size(dtype);
    if (s == 0 || (n == nullptr && count != 0)) return 0;
    return batch_workspace_bytes(count, s, [n](size_t i) { return n[i] > BT_MAX_ELEMENTS ? BT_MAX_ELEMENTS : n[i]; });
}

bt_status bt_compress_batch(const bt_compress_item *items, size_t count, bt_dtype dtype, void *d_workspace,
                            size_t workspace_bytes, bt_stream stream) {
    const bt_status st = check_batch_common(items, count, dtype, d_workspace);
    if (st != BT_OK || count == 0) return st;
    const int s = elem_size(dtype);
    for (size_t i = 0; i < count; ++i) {
        const bt_compress_item &it = items[i];
        if (it.n > BT_MAX_ELEMENTS) return BT_ERR_SIZE;
        if (it.d_nnz == nullptr) return BT_ERR_NULL;
        if (misaligned(it.d_nnz, 8)) return BT_ERR_ALIGN;
        if (it.n == 0) continue;
        if (it.d_in == nullptr || it.d_bitmap == nullptr) return BT_ERR_NULL;
        if (it.d_values == nullptr && it.values_cap != 0) return BT_ERR_NULL;
        if (misaligned(it.d_in, 16) || misaligned(it.d_bitmap, 4) || misaligned(it.d_values, (size_t)s))
            return BT_ERR_ALIGN;
    }
    const auto n_of = [items](size_t i) { return items[i].n; };
    if (workspace_bytes < batch_workspace_bytes(count, s, n_of)) return BT_ERR_WORKSPACE;

    hipStream_t hs = (hipStream_t)stream;
    char *ws = static_cast<char *>(d_workspace);
    for (size_t first = 0; first < count; first += kMaxBatch) {
        const size_t c = count - first < (size_t)kMaxBatch ? count - first : (size_t)kMaxBatch;
        CompressBatch b;
        lay_out(b.lay, first, c, s, n_of);
        for (size_t i = 0; i < (size_t)kMaxBatch; ++i) {
            const bt_compress_item it = i < c ? items[first + i] : bt_compress_item{nullptr, 0, nullptr, nullptr, 0, nullptr};
            b.in[i] = it.d_in;
            b.n[i] = it.n;
            b.bitmap[i] = it.d_bitmap;
            b.values[i] = it.d_values;
            b.cap[i] = it.values_cap;
            b.nnz[i] = it.d_nnz;
        }
        const dim3 grid(b.lay.start[c] + 1), block(kBlock);
        if (s == 8) compress_batch_kernel<8><<<grid, block, 0, hs>>>(b, ws);
        else if (s == 4) compress_batch_kernel<4><<<grid, block, 0, hs>>>(b, ws);
        else compress_batch_kernel<2><<<grid, block, 0, hs>>>(b, ws);
        const bt_status ls = launched();
        if (ls != BT_OK) return ls;
    }
    return BT_OK;
}

bt_status bt_decompress_batch(const bt_decompress_item *items, size_t count, bt_dtype dtype, void *d_workspace,
                              size_t workspace_bytes, bt_stream stream) {
    const bt_status st = check_batch_common(items, count, dtype, d_workspace);
    if (st != BT_OK || count == 0) return st;
    const int s = elem_size(dtype);
    for (size_t i = 0; i < count; ++i) {
        const bt_decompress_item &it = items[i];
        if (it.n > BT_MAX_ELEMENTS) return BT_ERR_SIZE;
        if (it.n == 0) continue;
        if (it.d_bitmap == nullptr || it.d_out == nullptr) return BT_ERR_NULL;   // d_values may be NULL when nnz == 0
        if (misaligned(it.d_out, 16) || misaligned(it.d_bitmap, 4) || misaligned(it.d_values, (size_t)s))
            return BT_ERR_ALIGN;
    }
    const auto n_of = [items](size_t i) { return items[i].n; };
    if (workspace_bytes < batch_workspace_bytes(count, s, n_of)) return BT_ERR_WORKSPACE;

    hipStream_t hs = (hipStream_t)stream;
    char *ws = static_cast<char *>(d_workspace);
    for (size_t first = 0; first < count; first += kMaxBatch) {
        const size_t c = count - first < (size_t)kMaxBatch ? count - first : (size_t)kMaxBatch;
        DecompressBatch b;
        lay_out(b.lay, first, c, s, n_of);
        for (size_t i = 0; i < (size_t)kMaxBatch; ++i) {
            const bt_decompress_item it = i < c ? items[first + i] : bt_decompress_item{nullptr, nullptr, 0, nullptr};
            b.bitmap[i] = it.d_bitmap;
            b.values[i] = it.d_values;
            b.n[i] = it.n;
            b.out[i] = it.d_out;
        }
        const dim3 grid(b.lay.start[c] + 1), block(kBlock);
        if (s == 8) decompress_batch_kernel<8><<<grid, block, 0, hs>>>(b, ws);
        else if (s == 4) decompress_batch_kernel<4><<<grid, block, 0, hs>>>(b, ws);
        else decompress_batch_kernel<2><<<grid, block, 0, hs>>>(b, ws);
        const bt_status ls = launched();
        if (ls != BT_OK) return ls;
    }
    return BT_OK;
}

}  // extern "C"
