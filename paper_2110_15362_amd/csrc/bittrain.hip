// libbittrain: BitTrain's sparse bitmap activation codec as HIP kernels for
// CDNA4 (gfx950, wave64).  See include/bittrain.h for the contract.
//
// Section 3.2 of the paper defines the format (a bit per element plus the
// non-zero elements in index order); Algorithm 1 builds it with a sequential
// append loop and Algorithm 2 undoes it with a running counter j.  Both loops
// carry one dependency: the position of an element's value is the number of
// non-zero elements before it.  On a GPU that is an exclusive prefix sum over
// the non-zero predicate, and the kernels below compute it in ONE pass over the
// data so that the tensor is read from HBM exactly once:
//
//   lane    16-byte loads; per-lane non-zero mask by integer compare
//   wave    packed DPP prefix sum of the per-lane popcounts (no LDS, no barrier)
//   block   four wave totals through LDS
//   grid    per-tile counts published in the workspace; one extra wave turns them
//           into per-tile prefixes; a wave polls only the prefix of its own tile
//
// A codec launch has one workgroup per 32 KiB tile (plus one, whose first wave is the
// scanner).  No workgroup depends on another for progress: a workgroup whose prefix has
// not come after a bounded number of polls counts the elements before its tile itself,
// from the input (compression) or from the bitmap (restoration), so the order in which
// the hardware starts the workgroups does not matter.  A workgroup ends with its stores
// on their way; it never waits for them to land.
//
// There is no matrix contraction anywhere, so no MFMA: the path is bound by HBM
// bandwidth and everything here is about moving each byte once, coalesced, and
// about keeping the memory system busy while prefixes are on their way.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <atomic>
#include <cmath>
#include <type_traits>

#include "bittrain.h"

namespace {

constexpr int kWaveSize = 64;
constexpr int kWaves = 4;                 // waves per block
constexpr int kBlock = kWaveSize * kWaves;
constexpr int kRows = 8;                  // 16-byte loads per lane per tile
constexpr int kPhaseRows = 4;             // rows that are compacted / expanded through LDS at a time
constexpr int kVecBytes = 16;
#ifndef BT_RELU_ROWS
#define BT_RELU_ROWS 1
#endif
constexpr int kReluRows = BT_RELU_ROWS;   // 16-byte vectors per lane in the ReLU-backward stream

// Workgroups per compute unit (= waves per SIMD) the codec kernels are built for: eight, i.e. at
// most 64 vector registers per lane.
#ifndef BT_COMPRESS_OCC
#define BT_COMPRESS_OCC 8
#endif
#ifndef BT_DECOMPRESS_OCC
#define BT_DECOMPRESS_OCC 8
#endif
constexpr int kCompressOcc = BT_COMPRESS_OCC;
constexpr int kDecompressOcc = BT_DECOMPRESS_OCC;

// ---- workspace layout -----------------------------------------------------------------
// Header (uint32 words), then one 6 KiB block per 256 slots.
constexpr int kHdrSeq = 0;       // calls completed on this workspace; its low bit picks the copy in use
constexpr int kHdrPrevTiles = 1; // slots of the previous call (what it left behind in the other copy)
constexpr int kHdrError = BT_WS_ERROR_WORD;           // set if a wait was given up
constexpr int kHdrSpinLimit = BT_WS_WAIT_LIMIT_WORD;  // scanner passes before its wait is given up; 0: kSpinLimit
constexpr int kHdrWide = BT_WS_WIDE_WORD;             // non-zero: the one-tensor scanner writes 8-byte entries only
constexpr int kHdrPatience = BT_WS_PATIENCE_WORD;     // polls before a workgroup counts what precedes its tile itself; 0: kPatience
constexpr size_t kHeaderBytes = 256;
constexpr size_t kHdrSpare = 128;      // bytes [128, 256) of the header take stores that mean nothing (see the scanner)
// Block of 256 slots, two copies c = 0, 1 of everything:
//   [1024*c, 1024*c + 1024)            uint32 count + 1 of each slot, written by the slot's workgroup
//   [2048 + 2048*c, 2048*c + 4096)     uint64 prefix + 1 of each slot, written by the scanner
// 0 means "not published yet".  A call uses copy (seq & 1) and zeroes what the
// previous call left in the other copy, so the copy the next call uses is clean
// when it starts and no clearing launch is ever needed.  The layout depends only on the
// slot number, never on the size of the workspace or of the call.
constexpr int kSlotsPerBlock = 256;
constexpr size_t kBlockBytes = 6144;
constexpr uint32_t kSpinLimit = 1u << 20; // scanner passes before its wait is given up
constexpr uint32_t kPatience = 1u << 12;  // polls before a workgroup counts what precedes its tile itself instead of waiting on
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
    static constexpr int TILE_WORDS = TILE / 32;     // bitmap words per tile
    static constexpr int LANE_WORDS = TILE_WORDS / kWaveSize;   // of which a lane counts this many when a wave counts a tile
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

// A workgroup barrier that orders LDS traffic only.  (__syncthreads() also waits for every global load
// and store of the wave, which would make a wave that has the next tile's loads in flight wait for them.)
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
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
// Algorithm 1 ends by giving the dense tensor up), decompress only the store hint.
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
// that test, in one pass: an element survives pruning where its value exceeds the
// threshold, compared in single precision after widening (exact for half and
// bfloat16; a double is compared in double precision with `threshold_f64`; a NaN
// exceeds nothing), and is then stored if its bit pattern is non-zero (a +0.0 that
// survives a negative threshold is still a zero for Algorithm 1).
enum { kKeepNonZero = 0, kKeepAboveF32 = 1, kKeepAboveF16 = 2, kKeepAboveBF16 = 3, kKeepAboveF64 = 4 };
template <int S, int KEEP>
__device__ __forceinline__ uint32_t keep_mask(const uint4 v, const float threshold, const double threshold_f64) {
    if (KEEP == kKeepNonZero) return nonzero_mask<S>(v);
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    uint32_t m = 0;
    if (KEEP == kKeepAboveF64) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            m |= (__longlong_as_double((long long)(((uint64_t)d[2 * i + 1] << 32) | d[2 * i])) > threshold_f64 ? 1u : 0u) << i;
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

// ---- the tensors of a call ------------------------------------------------------------------
//
// A call works on one tensor or (the batched calls) on a list.  The tensors are laid end to
// end in a numbering of SLOTS (= workspace entries): a call on one tensor has slot == tile;
// a batched call starts every tensor at a multiple of 128 slots, so that a scanner row never
// spans two tensors, and the slots between a tensor's last tile and the next tensor's first
// slot belong to no tile ("idle": they publish a count of zero).  Prefixes restart at 0 with
// every tensor and each tensor's total goes to its nnz.  The kernels see the call through a
// small interface (count, start, tiles, at, and the per-tensor pointers) that the
// single-tensor and the batched argument structs both provide; the per-tensor pointers of a
// batched call travel as kernel arguments and are read with scalar loads.

struct Slot {
    uint32_t item;   // tensor of the call
    uint32_t tile;   // tile inside that tensor
    bool idle;       // the slot belongs to no tile
};

constexpr int kMaxBatchDecompress = BT_MAX_BATCH;   // tensors per launch: what keeps the kernel arguments under 4 KiB
constexpr int kMaxBatchCompress = 52;

template <int MAXB> struct BatchLayout {
    uint32_t count;
    uint32_t start[MAXB + 1];
    uint32_t tiles[MAXB];
    __device__ __forceinline__ Slot at(const uint32_t slot) const {
        uint32_t lo = 0, hi = count;          // start[lo] <= slot < start[hi]
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (slot >= start[mid]) lo = mid; else hi = mid;
        }
        const uint32_t tile = slot - start[lo];
        return Slot{lo, tile, tile >= tiles[lo]};
    }
};

struct CompressOne {
    static constexpr bool kMany = false;      // several tensors in one launch
    const void *in_;
    uint64_t n_;
    uint32_t *bitmap_;
    void *values_;
    uint64_t cap_;
    uint64_t *nnz_;
    uint64_t *index_;
    void *dense_;
    uint32_t tiles_;
    __device__ __forceinline__ uint32_t count() const { return 1; }
    __device__ __forceinline__ uint32_t start(uint32_t i) const { return i == 0 ? 0u : tiles_; }
    __device__ __forceinline__ uint32_t slots() const { return tiles_; }
    __device__ __forceinline__ uint32_t tiles(uint32_t) const { return tiles_; }
    __device__ __forceinline__ Slot at(uint32_t slot) const { return Slot{0, slot, false}; }
    __device__ __forceinline__ const void *in(uint32_t) const { return in_; }
    __device__ __forceinline__ uint64_t n(uint32_t) const { return n_; }
    __device__ __forceinline__ uint32_t *bitmap(uint32_t) const { return bitmap_; }
    __device__ __forceinline__ void *values(uint32_t) const { return values_; }
    __device__ __forceinline__ uint64_t cap(uint32_t) const { return cap_; }
    __device__ __forceinline__ uint64_t *nnz(uint32_t) const { return nnz_; }
    __device__ __forceinline__ uint64_t *index(uint32_t) const { return index_; }
    __device__ __forceinline__ void *dense(uint32_t) const { return dense_; }
};

struct CompressMany {
    static constexpr bool kMany = true;      // several tensors in one launch
    BatchLayout<kMaxBatchCompress> lay;
    const void *in_[kMaxBatchCompress];
    uint64_t n_[kMaxBatchCompress];
    uint32_t *bitmap_[kMaxBatchCompress];
    void *values_[kMaxBatchCompress];
    uint64_t cap_[kMaxBatchCompress];
    uint64_t *nnz_[kMaxBatchCompress];
    uint64_t *index_[kMaxBatchCompress];
    void *dense_[kMaxBatchCompress];
    __device__ __forceinline__ uint32_t count() const { return lay.count; }
    __device__ __forceinline__ uint32_t start(uint32_t i) const { return lay.start[i]; }
    __device__ __forceinline__ uint32_t slots() const { return lay.start[lay.count]; }
    __device__ __forceinline__ uint32_t tiles(uint32_t i) const { return lay.tiles[i]; }
    __device__ __forceinline__ Slot at(uint32_t slot) const { return lay.at(slot); }
    __device__ __forceinline__ const void *in(uint32_t i) const { return in_[i]; }
    __device__ __forceinline__ uint64_t n(uint32_t i) const { return n_[i]; }
    __device__ __forceinline__ uint32_t *bitmap(uint32_t i) const { return bitmap_[i]; }
    __device__ __forceinline__ void *values(uint32_t i) const { return values_[i]; }
    __device__ __forceinline__ uint64_t cap(uint32_t i) const { return cap_[i]; }
    __device__ __forceinline__ uint64_t *nnz(uint32_t i) const { return nnz_[i]; }
    __device__ __forceinline__ uint64_t *index(uint32_t i) const { return index_[i]; }
    __device__ __forceinline__ void *dense(uint32_t i) const { return dense_[i]; }
};
static_assert(sizeof(CompressMany) <= 3840, "kernel arguments of a batched compression");

struct DecompressOne {
    static constexpr bool kMany = false;      // several tensors in one launch
    const uint32_t *bitmap_;
    const void *values_;
    uint64_t cap_;
    const uint64_t *index_;
    uint64_t n_;
    void *out_;
    uint32_t tiles_;
    __device__ __forceinline__ uint32_t count() const { return 1; }
    __device__ __forceinline__ uint32_t start(uint32_t i) const { return i == 0 ? 0u : tiles_; }
    __device__ __forceinline__ uint32_t slots() const { return tiles_; }
    __device__ __forceinline__ uint32_t tiles(uint32_t) const { return tiles_; }
    __device__ __forceinline__ Slot at(uint32_t slot) const { return Slot{0, slot, false}; }
    __device__ __forceinline__ const uint32_t *bitmap(uint32_t) const { return bitmap_; }
    __device__ __forceinline__ const void *values(uint32_t) const { return values_; }
    __device__ __forceinline__ uint64_t cap(uint32_t) const { return cap_; }
    __device__ __forceinline__ const uint64_t *tile_index(uint32_t) const { return index_; }
    __device__ __forceinline__ uint64_t n(uint32_t) const { return n_; }
    __device__ __forceinline__ void *out(uint32_t) const { return out_; }
    __device__ __forceinline__ uint64_t *nnz(uint32_t) const { return nullptr; }
    __device__ __forceinline__ uint64_t *index(uint32_t) const { return nullptr; }
};

struct DecompressMany {
    static constexpr bool kMany = true;      // several tensors in one launch
    BatchLayout<kMaxBatchDecompress> lay;
    const uint32_t *bitmap_[kMaxBatchDecompress];
    const void *values_[kMaxBatchDecompress];
    uint64_t cap_[kMaxBatchDecompress];
    const uint64_t *index_[kMaxBatchDecompress];
    uint64_t n_[kMaxBatchDecompress];
    void *out_[kMaxBatchDecompress];
    __device__ __forceinline__ uint32_t count() const { return lay.count; }
    __device__ __forceinline__ uint32_t start(uint32_t i) const { return lay.start[i]; }
    __device__ __forceinline__ uint32_t slots() const { return lay.start[lay.count]; }
    __device__ __forceinline__ uint32_t tiles(uint32_t i) const { return lay.tiles[i]; }
    __device__ __forceinline__ Slot at(uint32_t slot) const { return lay.at(slot); }
    __device__ __forceinline__ const uint32_t *bitmap(uint32_t i) const { return bitmap_[i]; }
    __device__ __forceinline__ const void *values(uint32_t i) const { return values_[i]; }
    __device__ __forceinline__ uint64_t cap(uint32_t i) const { return cap_[i]; }
    __device__ __forceinline__ const uint64_t *tile_index(uint32_t i) const { return index_[i]; }
    __device__ __forceinline__ uint64_t n(uint32_t i) const { return n_[i]; }
    __device__ __forceinline__ void *out(uint32_t i) const { return out_[i]; }
    __device__ __forceinline__ uint64_t *nnz(uint32_t) const { return nullptr; }
    __device__ __forceinline__ uint64_t *index(uint32_t) const { return nullptr; }
};
static_assert(sizeof(DecompressMany) <= 3840, "kernel arguments of a batched restoration");

// ---- grid prefix ---------------------------------------------------------------------------
//
// The position of a tile's first value is the number of non-zero elements in all
// tiles before it (Algorithm 1 appends in index order; Algorithm 2's counter j).
// Tiles do not talk to each other.  Each tile's workgroup publishes its count in the
// workspace; ONE extra workgroup (workgroup 0, a single wave: the "scanner") reads the
// counts in index order, keeps the running sum, and writes every tile's prefix back; the
// tile then polls its own prefix, one 8-byte load.  Per tile that is one store and a few
// polled loads on lines shared with few other tiles.  (Having every tile read its
// predecessors' counts itself -- a look-back window or a tree -- makes a few hot lines that
// thousands of tiles read at once, and those reads queue up at one memory channel.)
//
// Forward progress does not rest on the order in which workgroups are started.  A workgroup
// publishes its count before it waits for anything, the scanner waits only for counts, and
// a workgroup whose prefix has not come after kPatience polls stops waiting and counts what
// lies before its tile itself, from the call's inputs alone (prefix_from_bitmap,
// prefix_from_input): slow, but then every workgroup that has been started ends, whatever
// the others do, and every workgroup is started in the end.  The scanner's own wait is
// bounded (kSpinLimit): if it runs out the call ends with the error word set.
//
// Entries are value + 1 (0 = not published), written and read with relaxed
// device-scope atomics: the entry is the only thing that is communicated.

// ---- timeline (only in a build with -DBT_TIMELINE) ---------------------------------------------
// Every slot of a bt_compress / bt_decompress launch leaves times of the 100 MHz device
// clock in the caller's buffer (8 words per slot: loads asked for, counted, prefix seen, stores
// issued, -, polls), and the scanner two words per pass that consumed something (time, first
// slot << 32 | end slot), after the slots' words.
#ifdef BT_TIMELINE
__device__ uint64_t *g_timeline = nullptr;
__device__ uint32_t g_timeline_tiles = 0, g_timeline_passes = 0;
// read the recording state once per kernel: a stamp must not cost a memory round trip of its own
#define BT_TL_INIT uint64_t *const tl_buf = g_timeline; const uint32_t tl_tiles = g_timeline_tiles; (void)tl_buf; (void)tl_tiles
#define BT_TL(slot, k)                                                                            \
    do {                                                                                          \
        if (threadIdx.x == 0 && tl_buf != nullptr && (slot) < tl_tiles)                           \
            tl_buf[8 * (size_t)(slot) + (k)] = wall_clock64();                                    \
    } while (0)
#define BT_TL_VALUE(slot, k, v)                                                                   \
    do {                                                                                          \
        if (threadIdx.x == 0 && tl_buf != nullptr && (slot) < tl_tiles)                           \
            tl_buf[8 * (size_t)(slot) + (k)] = (v);                                               \
    } while (0)
#else
#define BT_TL_INIT do {} while (0)
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
    return ws + kHeaderBytes + (size_t)(tile >> 8) * kBlockBytes + 1024u * copy + 4u * (tile & 255u);
}
// prefix + 1 of `tile` in copy c
__device__ __forceinline__ char *ws_prefix(char *ws, uint32_t tile, uint32_t copy) {
    return ws + kHeaderBytes + (size_t)(tile >> 8) * kBlockBytes + 2048u + 2048u * copy + 8u * (tile & 255u);
}

// The same value in every lane: tell the compiler, so that what is built on it stays in scalar registers.
__device__ __forceinline__ uint32_t uniform32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ uint64_t uniform64(uint64_t v) {
    return ((uint64_t)uniform32((uint32_t)(v >> 32)) << 32) | uniform32((uint32_t)v);
}

// Polls after which a wait is given up: what the caller asked for in the header, else the
// built-in limit.  Read once, before the wait (a load inside the polling loop would
// lengthen every poll by a round trip).
__device__ __forceinline__ uint32_t wait_limit(const uint32_t *hdr) {
    const uint32_t asked = hdr[kHdrSpinLimit];          // never written by a kernel
    return asked != 0 ? asked : kSpinLimit;
}

// Polls after which a tile's workgroup counts for itself instead of waiting on.  Looked at every 256th poll
// only: read from the header then, it costs neither a register nor a round trip per poll.
__device__ __forceinline__ uint32_t patience_of(const uint32_t *hdr) {
    const uint32_t asked = hdr[kHdrPatience];          // never written by a kernel
    return asked != 0 ? asked : kPatience;
}

// The scanner: one wave.  Workgroups come and go (one per tile) and a count is published as soon as its tile
// has arrived; the scanner takes a few rows of 128 counts starting at the frontier's row in every pass, consumes
// the leading run of published ones (to the slot, not to the row) and asks again.  Every tile of a launch waits
// for the pass that reaches it, so the launch pays for each instruction of this one wave:
//   - what is the same in all lanes (frontier, running sum) is kept in scalar registers;
//   - a lane takes two neighbouring slots (slots 2 i and 2 i + 1 of the row, one 8-byte load), sums its two counts
//     before the DPP prefix sum over the lanes, and stores its two prefixes with one 16-byte store;
//   - a row's prefixes are stored as soon as they are known, and rows behind the first unpublished slot are not
//     looked at.
// The frontier's row is summed again from its first slot in every pass (the slots done before still hold their
// counts, and they are given the prefixes they have already), so the running sum kept between passes is the one
// at that row's start.  Batched tensors are laid out in whole rows of 128 slots: the running sum restarts where
// a tensor begins and goes to that tensor's nnz where it ends.  All rows are asked for before anything is
// written: on this hardware one counter tracks a wave's loads and stores in order of issue, so a load waited for
// after a store would also wait for that store.  At the end the scanner advances the header for the next call.
// Measured alternatives, all slower or no faster: one slot per lane (rows of 64; 1 to 1.5 % slower), four or
// eight slots per lane (loads and stores spread over more lines), four waves with a window of 28 rows and an
// exchange through LDS, four waves taking rows round robin with the running sum handed on through LDS, a second
// wave that does the stores, whole rows only, a wider window when the last one was used up, more rows per pass
// (restoration is best with two, compression with three).
constexpr uint32_t kBatchRow = 128;     // slots: a batched tensor's share of a launch is a whole number of these

typedef uint32_t bt_u32x4 __attribute__((ext_vector_type(4)));
// Two prefix entries in one store that is written through to where every compute unit sees it.  Only for
// entries below 2^32: their upper halves stay the zero they were, so a reader that polls one entry with an
// 8-byte load sees it change in one piece whatever order the four words land in.
__device__ __forceinline__ void ws_store_two_small(void *p, uint32_t first, uint32_t second) {
    const bt_u32x4 v = {first, 0u, second, 0u};
    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}

template <int kRowScan, class Job> __device__ __forceinline__ void scan_counts(char *ws, const Job &job) {
    const uint32_t lane = threadIdx.x & (kWaveSize - 1);
    uint32_t *hdr = reinterpret_cast<uint32_t *>(ws);
    const uint32_t seq = uniform32(hdr[kHdrSeq]);
    const uint32_t cur = seq & 1u;
    const uint32_t n_items = job.count();
    const uint32_t n_slots = job.slots();
    uint32_t frontier = 0;     // slots [0, frontier) are done
    uint32_t item = 0;         // tensor that the frontier's row belongs to
    uint64_t base = 0;         // stored values of that tensor in the tiles before the frontier's row of 128 slots
    uint32_t spins = 0;
    const uint32_t limit = uniform32(wait_limit(hdr));
    const bool wide = uniform32(hdr[kHdrWide]) != 0;      // never written by a kernel
#ifdef BT_TIMELINE
    uint64_t *const timeline = g_timeline;      // read once: a load in the loop would join the scanner's waits
    uint32_t timeline_pass = 0;
#endif
    while (frontier < n_slots) {
        frontier = uniform32(frontier);
        item = uniform32(item);
        base = uniform64(base);
        const uint32_t row = frontier >> 7;
        uint32_t ca[kRowScan], cb[kRowScan];          // count + 1 of the lane's two slots; 0: not published yet, or past the end
#pragma unroll
        for (int j = 0; j < kRowScan; ++j) {
            const uint32_t t = 128u * (row + j) + 2u * lane;
            uint64_t two = 0;
            if (t < n_slots)
                two = __hip_atomic_load(reinterpret_cast<const uint64_t *>(ws_count(ws, t, cur)), __ATOMIC_RELAXED,
                                        __HIP_MEMORY_SCOPE_AGENT);
            ca[j] = (uint32_t)two;
            cb[j] = t + 1 < n_slots ? (uint32_t)(two >> 32) : 0u;
        }
        const bool small = !wide && (base >> 32) == 0 && (uint32_t)base < 0xF0000000u;   // all of this pass's entries below 2^32
        bool open = true;
        uint32_t new_frontier = frontier;
#pragma unroll
        for (int j = 0; j < kRowScan; ++j) {
            if (open) {
                const uint32_t slot0 = 128u * (row + j);
                const uint64_t bad_a = __ballot(ca[j] == 0), bad_b = __ballot(cb[j] == 0);
                const uint32_t run_a = bad_a == 0 ? 64u : (uint32_t)__builtin_ctzll(bad_a);
                const uint32_t run_b = bad_b == 0 ? 64u : (uint32_t)__builtin_ctzll(bad_b);
                const uint32_t run = uniform32(min(2u * run_a, 2u * run_b + 1u));   // usable slots of the row, in slot order
                const uint32_t row_end = slot0 + run;
                if constexpr (Job::kMany) {
                    // batched tensors begin at multiples of 128 slots: the sum restarts there
                    while (item + 1 < n_items && slot0 >= job.start(item + 1)) ++item;
                    if (slot0 == job.start(item)) base = 0;
                    item = uniform32(item);
                }
                if (row_end > new_frontier) {
                    const bool use_a = 2u * lane < run, use_b = 2u * lane + 1u < run;
                    const uint32_t va = use_a ? ca[j] - 1u : 0u, vb = use_b ? cb[j] - 1u : 0u;
                    const uint32_t incl = wave_inclusive_sum(va + vb);
                    const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                    char *const entry = ws_prefix(ws, slot0 + 2u * lane, cur);
                    if (small) {
                        const uint32_t pa = (uint32_t)base + 1u + (incl - va - vb);
                        if (use_b) ws_store_two_small(entry, pa, pa + va);
                        else if (use_a) ws_store32(entry, pa);
                    } else {
                        const uint64_t pa = (base + 1) + (incl - va - vb);
                        if (use_a) ws_store64(entry, pa);
                        if (use_b) ws_store64(entry + 8, pa + va);
                    }
                    new_frontier = row_end;
                    if (row_end == (Job::kMany ? job.start(item + 1) : n_slots)) {      // this tensor's number of values
                        uint64_t *const nnz = job.nnz(item);
                        if (lane == 0 && nnz != nullptr) *nnz = base + total;
                    }
                    if (run == 128u) base = uniform64(base + total);
                }
                open = run == 128u;
            }
        }
        // the scanner's wait for the call's counts is bounded in passes, fruitful or not
        if (++spins > limit) {
            if (lane == 0) __hip_atomic_store(&hdr[kHdrError], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        if (new_frontier == frontier) {
            __builtin_amdgcn_s_sleep(kScannerSleep);
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
        // every slot's workgroup has published its count by now, hence has read the header: advance it
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

// What a workgroup reads from the header before it publishes anything.  The scanner
// rewrites the header once every slot of the call has published, so no wave may read it
// after any wave of its workgroup has published a count.
struct Epoch {
    uint32_t cur;          // copy of the entries this call uses
    uint32_t prev_slots;   // entries the previous call used in the other copy
};

__device__ __forceinline__ Epoch read_epoch(const char *ws) {
    const uint32_t *hdr = reinterpret_cast<const uint32_t *>(ws);
    return Epoch{hdr[kHdrSeq] & 1u, hdr[kHdrPrevTiles]};
}

// Zero what the previous call left in the other copy of the workspace entries: slots
// [0, prev_slots), shared out over the threads of this call's `workers` workgroups.
__device__ __forceinline__ void zero_previous(char *ws, const Epoch ep, const uint32_t worker, const uint32_t workers,
                                              const uint32_t block = kBlock) {
    const uint32_t other = ep.cur ^ 1u;
    for (uint64_t i = (uint64_t)worker * block + threadIdx.x; i < ep.prev_slots; i += (uint64_t)workers * block) {
        ws_store32(ws_count(ws, (uint32_t)i, other), 0);
        ws_store64(ws_prefix(ws, (uint32_t)i, other), 0);
    }
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

// ---- Algorithm 1: dense -> bitmap -------------------------------------------------------

// Write `cnt` elements from a wave's LDS strip to global memory with aligned 16-byte
// stores.  LDS element `pad + i` corresponds to global element g0 + i, where pad makes
// LDS byte 0 line up with a 16-byte boundary of the global buffer.  The first and
// last vector go element by element, so nothing outside [g0, g0 + cnt) is touched.
// All LDS reads of the inner vectors are issued before the first store and the two edge
// vectors are left to 2 E lanes at the end: this runs after the tile has received its
// prefix, where every instruction delays the tile's exit.
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

// What a compressing workgroup does when the scanner's answer for its tile does not come: its first
// wave counts the kept elements of the tensor before the tile itself, with the same test.  Slow (the
// whole input up to the tile), but it needs nothing from any other workgroup.
template <int S, int KEEP>
__device__ __forceinline__ uint64_t prefix_from_input(const void *__restrict__ in, const uint32_t tile, const float threshold_f,
                                                   const double threshold, const int lane) {
    const uint64_t vectors = (uint64_t)tile * (Geo<S>::TILE / Geo<S>::E);      // all of them whole and inside the tensor
    const uint4 *const end = static_cast<const uint4 *>(in) + vectors;
    uint64_t mine = 0;
    for (const uint4 *q = static_cast<const uint4 *>(in) + lane; q < end; q += kWaveSize)
        mine += (uint32_t)__popc(keep_mask<S, KEEP>(*q, threshold_f, threshold));
#pragma unroll
    for (int d = 1; d < kWaveSize; d <<= 1) mine += __shfl_xor((unsigned long long)mine, d, kWaveSize);
    return uniform64(mine);
}

// bt_compress and its relatives (pruning, dense output, tile index, batches): workgroup 0 is the scanner
// (one wave of it), workgroup 1 + t compresses slot t.
// 1. load: lane l of row k owns elements wave_e0 + k * ROW + l * E ... + E - 1 of its wave's quarter of the
//    tile; all eight rows are asked for at once.
// 2. the test of Algorithm 1 (on the bit pattern), or the pruning test; masks packed RPM rows to a register;
//    ranks by one DPP wave prefix sum per two rows.
// 3. bitmap words: G lanes OR their E-bit masks into one 32-bit word.
// 4. the waves' totals meet in LDS, the tile's count is published, the first wave polls the tile's prefix.
// 5. values: kPhaseRows rows at a time, the wave compacts its kept elements into its LDS strip at their ranks,
//    shifted so that LDS byte 0 maps to a 16-byte boundary of the value array, and writes the strip out with
//    aligned stores; then the dense pruned tensor, if asked for.
// The workgroup ends with its stores on their way: nothing waits for them to land.  (A persistent version
// of this kernel -- as many workgroups as are resident, each taking tiles w, w + G, ..., the next tile's loads
// asked for before the current tile's prefix wait, compacted values parked in rings in LDS -- was built and
// measured: 1 % faster on a 25.7 M element fp32 tensor, 5 to 15 % slower on 16-bit and on larger tensors.)
template <int S, int KEEP, bool DENSE, class Job>
__global__ __launch_bounds__(kBlock, kCompressOcc) void compress_kernel(const Job job, char *ws, const double threshold, const float threshold_f) {
    using G = Geo<S>;
    constexpr int E = G::E;
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[kWaves * G::LDS_WAVE];
    __shared__ uint64_t s_tile_prefix;
    __shared__ uint32_t s_wave_total[kWaves];
    if (workspace_failed(ws)) return;
    if (blockIdx.x == 0) {
        if (threadIdx.x < kWaveSize) scan_counts<3>(ws, job);
        return;
    }
    BT_TL_INIT;
    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it in a scalar register
    const uint32_t slot = blockIdx.x - 1, n_slots = gridDim.x - 1;
    uint32_t *hdr = reinterpret_cast<uint32_t *>(ws);
    const Slot sl = job.at(slot);
    if (sl.idle) {
        // a slot of a batched call that belongs to no tile: it publishes an empty count (so that the scanner gets
        // past it) and does its share of the clean-up
        const Epoch ep = read_epoch(ws);
        const uint32_t cur = uniform32(ep.cur);
        const uint32_t prev_slots = uniform32(ep.prev_slots);
        lds_barrier();                  // every wave has read the header before the first wave publishes anything
        if (tid == 0) ws_store32(ws_count(ws, slot, cur), 1);
        zero_previous(ws, Epoch{cur, prev_slots}, slot, n_slots);
        return;
    }
    const uint32_t tile = sl.tile;
    const uint64_t n = job.n(sl.item);
    const void *const in = job.in(sl.item);
    const uint64_t n_words = (n + 31) >> 5;
    const uint64_t wave_e0 = (uint64_t)tile * G::TILE + (uint64_t)wave * G::WAVE;
    const bool full = (uint64_t)(tile + 1) * G::TILE <= n;

    // (1), (2)
    uint4 x[kRows];
    uint32_t mp[G::MW], rank2[kRows / 2], total2[kRows / 2];
#pragma unroll
    for (int i = 0; i < G::MW; ++i) mp[i] = 0;
    BT_TL(slot, 0);
    if (__builtin_expect(full, 1)) {
        const uint4 *p = reinterpret_cast<const uint4 *>(static_cast<const char *>(in) + wave_e0 * S) + lane;
#pragma unroll
        for (int k = 0; k < kRows; ++k) x[k] = stream_load<kCompressNtLoad>(p + k * kWaveSize);
    }
    if (full) {
#pragma unroll
        for (int k = 0; k < kRows; ++k) {
            uint32_t mk = keep_mask<S, KEEP>(x[k], threshold_f, threshold);
            asm volatile("" : "+v"(mk));             // row k has arrived: its mask exists from here on
            mp[k / G::RPM] |= mk << (E * (k % G::RPM));
        }
    } else {
        // A tensor's ragged last tile, element by element and one row after the other: each row's addresses are
        // made to depend on the row before having arrived (`after`, which is 0), because with the loads of all
        // rows in flight together the addresses alone would need more registers than there are.
        uint32_t after = 0;
#pragma unroll
        for (int k = 0; k < kRows; ++k) {
            const uint64_t e0 = wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E + after;
            x[k] = load_vec_guarded<S>(in, e0, n);
            asm volatile("" : "+v"(after), "+v"(x[k].x), "+v"(x[k].y), "+v"(x[k].z), "+v"(x[k].w));
            // elements at or beyond n read as 0, which a negative threshold would keep: mask them
            const uint32_t in_range = e0 >= n ? 0u : (n - e0 >= (uint64_t)E ? (1u << E) - 1u : (1u << (uint32_t)(n - e0)) - 1u);
            mp[k / G::RPM] |= (keep_mask<S, KEEP>(x[k], threshold_f, threshold) & in_range) << (E * (k % G::RPM));
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

    // (3) lane (g * G + i) keeps the word of row r0 + i, group g: one store per G rows.
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

    const auto store_words = [&]() {
        uint32_t *const bitmap = job.bitmap(sl.item);
        const int g = lane / G::G, i = lane % G::G;
#pragma unroll
        for (int r0 = 0; r0 < kRows; r0 += G::G) {
            const uint64_t widx = (wave_e0 >> 5) + (uint64_t)(r0 + i) * G::WPR + (uint64_t)g;
            if (r0 + i < kRows && widx < n_words) bitmap[widx] = word[r0 / G::G];
        }
    };
    // Before the wait of (4) or after it?  After is better (a store in flight delays the polling loads, which share
    // its completion counter: 3 % on fp32), but the words cost registers across the wait, and kernels for 16-bit
    // elements have none to spare: there a spilled value would come back from memory right behind the value stores
    // and wait for them (7 %).
    constexpr bool kWordsEarly = S == 2;
    if (kWordsEarly) store_words();

    // (4)
    // written at the end of the previous call; constant until every slot of this call has published
    const Epoch ep = read_epoch(ws);
    const uint32_t cur = uniform32(ep.cur);      // (the wave has the header's words from here on)
    const uint32_t prev_slots = uniform32(ep.prev_slots);
    if (lane == 0) s_wave_total[wave] = wave_total;
    lds_barrier();                      // also: every wave has read the header before the first wave publishes anything
    uint32_t before_wave = 0, tile_total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t c = s_wave_total[w];
        if (w < wave) before_wave += c;
        tile_total += c;
    }
    before_wave = uniform32(before_wave);       // the same in every lane: tell the compiler, so that addresses built on it stay scalar
    if (tid == 0) ws_store32(ws_count(ws, slot, cur), tile_total + 1);
    BT_TL(slot, 1);
    zero_previous(ws, Epoch{cur, prev_slots}, slot, n_slots);
    uint32_t polls = 0;
    if (wave == 0) {
        uint64_t v;
        for (;;) {
            v = uniform64(ws_load64(ws_prefix(ws, slot, cur)));
            ++polls;
            if (v != 0) { v -= 1; break; }
            if (__builtin_expect((polls & 255u) == 0 && polls > patience_of(hdr), 0)) {
                // Count for ourselves.  The loop needs registers and the tile's elements fill them: park the elements
                // in LDS meanwhile (the strips are not in use before the barrier below).
                static_assert(kRows * kWaveSize * kVecBytes <= kWaves * G::LDS_WAVE, "room to park a wave's elements");
                uint4 *const park = reinterpret_cast<uint4 *>(s_stage) + lane;
#pragma unroll
                for (int k = 0; k < kRows; ++k) park[k * kWaveSize] = x[k];
                v = prefix_from_input<S, KEEP>(in, tile, threshold_f, threshold, lane);
#pragma unroll
                for (int k = 0; k < kRows; ++k) x[k] = park[k * kWaveSize];
                break;
            }
            __builtin_amdgcn_s_sleep(kTileSleep);
        }
        if (lane == 0) {
            s_tile_prefix = v;
            uint64_t *const index = job.index(sl.item);
            if (index != nullptr) index[tile] = v;     // Algorithm 2's j at the start of this tile, for bt_decompress_indexed
        }
    }
    lds_barrier();
    uint64_t g0 = uniform64(s_tile_prefix) + before_wave;          // index in the value array of this wave's next value
    BT_TL(slot, 2);
    BT_TL_VALUE(slot, 5, polls);
    if (!kWordsEarly) store_words();

    // (5)
    unsigned char *strip = s_stage + wave * G::LDS_WAVE;
    const uint64_t values_cap = job.cap(sl.item);
#pragma unroll
    for (int r0 = 0; r0 < kRows; r0 += kPhaseRows) {
        char *gdst = static_cast<char *>(job.values(sl.item)) + g0 * S;
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
            // a branch around the write keeps the execution mask alone
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

    // the dense tensor after pruning, if asked for (bt_activation_compress): what survives keeps its bits, the
    // rest is +0.  Last, so that no store precedes the polling loads of (4); the dense output may be the input
    // itself (every lane rewrites exactly the vectors it has read).
    if (DENSE) {
        void *const dense = job.dense(sl.item);
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
    BT_TL(slot, 3);
}

// ---- Algorithm 2: bitmap -> dense ---------------------------------------------------------

// The reverse of ring_flush in two steps, so that the loads of several phases can be in
// flight together: strip_fetch issues the loads of values[g0, g0 + cnt) into
// registers, strip_commit later writes them into the wave's LDS strip, LDS element
// pad + i being global element g0 + i (pad lines LDS byte 0 up with a 16-byte boundary
// of the global buffer).  A phase holds at most kPhaseRows * ROW elements, i.e. 257 aligned
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

// Restoration of one wave's quarter of a tile goes in three steps, so that a wave can have the
// steps of consecutive tiles overlap:
//   ahead_load      asks for the bitmap words the wave needs (always the same number of loads,
//                   from somewhere harmless if there is no such tile);
//   restore_fetch   turns them into the lane's masks and ranks (Algorithm 2's counter j inside the
//                   tile) and, given j at the start of the tile, asks for the wave's values;
//   restore_store   puts the values into the LDS strip, expands them by rank (a value where
//                   the bit is set, +0 where it is clear) and stores the dense quarter tile.
// The waves of a workgroup do not talk to each other: each counts what the waves before it hold
// from the bitmap itself.
template <int S> struct Ahead {
    uint32_t rows[kRows];                      // the bitmap word that holds this lane's bits of row k
    uint32_t mine[Geo<S>::LANE_WORDS];         // this lane's share of the tile's words (lane l: words l * LANE_WORDS ...)
};

// `bitmap` == nullptr: there is no tile; everything is read from `harmless` (4-byte aligned, readable).
template <int S>
__device__ __forceinline__ void rows_load(const uint32_t *bitmap, const uint64_t n, const uint32_t tile, const int lane,
                                          const int wave, const uint32_t *harmless, uint32_t (&rows)[kRows]) {
    using G = Geo<S>;
    const bool real = bitmap != nullptr;
    const uint32_t *const base = real ? bitmap : harmless;
    const uint64_t last = real ? ((n + 31) >> 5) - 1 : 0;         // a real tile has n >= 1
    const uint64_t row_w0 = (real ? (uint64_t)tile * G::TILE_WORDS : 0) + (uint64_t)wave * (G::TILE_WORDS / kWaves) + (uint32_t)(lane / G::G);
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
        const uint64_t wi = row_w0 + (uint64_t)k * G::WPR;
        rows[k] = base[wi < last ? wi : last];
    }
}

template <int S>
__device__ __forceinline__ void words_load(const uint32_t *bitmap, const uint64_t n, const uint32_t tile, const int lane,
                                           const uint32_t *harmless, uint32_t (&words)[Geo<S>::LANE_WORDS]) {
    using G = Geo<S>;
    const bool real = bitmap != nullptr;
    const uint32_t *const base = real ? bitmap : harmless;
    const uint64_t last = real ? ((n + 31) >> 5) - 1 : 0;
    const uint64_t w0 = real ? (uint64_t)tile * G::TILE_WORDS + (uint64_t)lane * G::LANE_WORDS : 0;
#pragma unroll
    for (int j = 0; j < G::LANE_WORDS; ++j) words[j] = base[w0 + j < last ? w0 + j : last];
}

template <int S>
__device__ __forceinline__ void ahead_load(const uint32_t *bitmap, const uint64_t n, const uint32_t tile, const int lane,
                                           const int wave, const uint32_t *harmless, Ahead<S> &a) {
    rows_load<S>(bitmap, n, tile, lane, wave, harmless, a.rows);
    words_load<S>(bitmap, n, tile, lane, harmless, a.mine);
}

// The set bits of a whole tile from the words words_load has brought, as a running sum over the lanes: lane l
// holds LANE_WORDS consecutive words, so the 16 lanes [16 v, 16 v + 16) hold the words of the tile's v-th wave,
// lane 63 ends up with the tile's total and lane 16 v - 1 with the set bits of the waves before v.  Words at or
// beyond the bitmap's end count as 0 and so do bits at or beyond n (Algorithm 2 visits n bits).
template <int S>
__device__ __forceinline__ uint32_t tile_inclusive(const uint32_t (&words)[Geo<S>::LANE_WORDS], const uint64_t n, const uint32_t tile,
                                                   const int lane) {
    using G = Geo<S>;
    const uint64_t n_words = (n + 31) >> 5;
    const uint64_t w0 = (uint64_t)tile * G::TILE_WORDS + (uint64_t)lane * G::LANE_WORDS;
    const bool full = (uint64_t)(tile + 1) * G::TILE <= n;
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < G::LANE_WORDS; ++j) {
        uint32_t word = words[j];
        if (!full) {
            const uint64_t wi = w0 + j;
            if (wi >= n_words) word = 0;
            if (wi + 1 == n_words && (n & 31) != 0) word &= (1u << (uint32_t)(n & 31)) - 1u;
        }
        mine += (uint32_t)__popc(word);
    }
    return wave_inclusive_sum(mine);
}

// Returns the tile's total, and in `before` the set bits of the waves before `wave`.
template <int S>
__device__ __forceinline__ uint32_t count_words(const uint32_t (&words)[Geo<S>::LANE_WORDS], const uint64_t n, const uint32_t tile,
                                                const int lane, const int wave, uint32_t &before) {
    const uint32_t incl = tile_inclusive<S>(words, n, tile, lane);
    before = wave == 0 ? 0u : (uint32_t)__builtin_amdgcn_readlane((int)incl, (int)uniform32(16u * (uint32_t)wave - 1u));
    return (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
}

// The same straight from memory (one wave counts one tile).
template <int S>
__device__ __forceinline__ uint32_t count_tile(const uint32_t *__restrict__ bitmap, const uint64_t n, const uint32_t tile,
                                               const int lane, const int wave, uint32_t &before) {
    using G = Geo<S>;
    const uint64_t last = ((n + 31) >> 5) - 1;
    uint32_t words[G::LANE_WORDS];
#pragma unroll
    for (int j = 0; j < G::LANE_WORDS; ++j) {
        const uint64_t wi = (uint64_t)tile * G::TILE_WORDS + (uint64_t)lane * G::LANE_WORDS + j;
        words[j] = bitmap[wi < last ? wi : last];
    }
    return count_words<S>(words, n, tile, lane, wave, before);
}

template <int S> struct Restoring {            // a quarter tile between restore_fetch and restore_store
    uint32_t mp[Geo<S>::MW], rank2[kRows / 2], total2[kRows / 2];
    Fetched<S> fetched[kRows / kPhaseRows];
    uint32_t pads[kRows / kPhaseRows], cnts[kRows / kPhaseRows];
};

// (1) this lane's bits of the bitmap (G lanes read the same word and take E bits each), and Algorithm 2's
//     counter j as ranks.  Returns the set bits of this wave's quarter of the tile.
template <int S>
__device__ __forceinline__ uint32_t restore_ranks(const uint32_t (&rows)[kRows], const uint64_t n, const uint32_t tile, const int lane,
                                                  const int wave, Restoring<S> &r) {
    using G = Geo<S>;
    constexpr int E = G::E;
    const uint64_t n_words = (n + 31) >> 5;
    const uint64_t wave_e0 = (uint64_t)tile * G::TILE + (uint64_t)wave * G::WAVE;
    const bool full = (uint64_t)(tile + 1) * G::TILE <= n;
#pragma unroll
    for (int i = 0; i < G::MW; ++i) r.mp[i] = 0;
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
        const uint64_t e0 = wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E;
        uint32_t m = (rows[k] >> (uint32_t)(e0 & 31)) & ((1u << E) - 1u);
        if (!full) {                       // words beyond the bitmap read as 0, bits at or beyond n are cleared
            if ((e0 >> 5) >= n_words) m = 0;
            if (e0 + E > n) m &= (e0 < n) ? ((1u << (uint32_t)(n - e0)) - 1u) : 0u;
        }
        r.mp[k / G::RPM] |= m << (E * (k % G::RPM));
    }
    rank_rows<S>(r.mp, r.rank2, r.total2);
    uint32_t wave_total = 0;
#pragma unroll
    for (int k = 0; k < kRows; ++k) wave_total += BT_FIELD(r.total2, k);
    return wave_total;
}

// (2) ask for the values of every phase (kPhaseRows rows each), so that all of them are in flight together
template <int S>
__device__ __forceinline__ void restore_fetch(const void *__restrict__ values, const uint64_t values_cap, const uint64_t tile_j,
                                              const uint32_t before_wave, const int lane, Restoring<S> &r) {
    uint64_t g0 = tile_j + before_wave;                                   // Algorithm 2's j for this wave
#pragma unroll
    for (int ph = 0; ph < kRows / kPhaseRows; ++ph) {
        r.cnts[ph] = 0;
#pragma unroll
        for (int k = ph * kPhaseRows; k < (ph + 1) * kPhaseRows; ++k) r.cnts[ph] += BT_FIELD(r.total2, k);
        const char *gsrc = static_cast<const char *>(values) + g0 * S;
        r.pads[ph] = (uint32_t)(reinterpret_cast<uintptr_t>(gsrc) & (kVecBytes - 1)) / S;
        const uint32_t phase_total = r.cnts[ph];
        // nothing at or beyond the capacity is read (an index that does not belong to the bitmap, a wait that ran out)
        if (g0 >= values_cap) r.cnts[ph] = 0;
        else if (values_cap - g0 < r.cnts[ph]) r.cnts[ph] = (uint32_t)(values_cap - g0);
        strip_fetch<S>(gsrc, r.pads[ph], r.cnts[ph], lane, r.fetched[ph]);
        g0 += phase_total;
    }
}

template <int S>
__device__ __forceinline__ void restore_store(const Restoring<S> &r, const uint64_t n, void *__restrict__ out, const uint32_t tile,
                                              unsigned char *strip, const int lane, const int wave) {
    using G = Geo<S>;
    constexpr int E = G::E;
    const uint64_t wave_e0 = (uint64_t)tile * G::TILE + (uint64_t)wave * G::WAVE;
    const bool full = (uint64_t)(tile + 1) * G::TILE <= n;
#pragma unroll
    for (int ph = 0; ph < kRows / kPhaseRows; ++ph) {
        if (ph != 0) wave_lds_sync();   // the previous phase's reads are done before the strip is reused
        strip_commit<S>(strip, r.pads[ph], r.cnts[ph], lane, r.fetched[ph]);
        wave_lds_sync();
        uint32_t row_start = r.pads[ph];
#pragma unroll
        for (int k = ph * kPhaseRows; k < (ph + 1) * kPhaseRows; ++k) {
            uint32_t at = row_start + BT_FIELD(r.rank2, k);
            const uint32_t mk = BT_MASK(S, r.mp, k);
            uint32_t d[4] = {0, 0, 0, 0};
            // every lane reads at its running rank whether the bit is set or not (the index stays inside the strip)
            // and a select drops what a cleared bit read
            if (S == 8) {
                const uint64_t *l = reinterpret_cast<const uint64_t *>(strip);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const uint32_t keep = (mk >> j) & 1u;
                    const uint64_t v = l[at];
                    d[2 * j] = keep ? (uint32_t)v : 0u;
                    d[2 * j + 1] = keep ? (uint32_t)(v >> 32) : 0u;
                    at += keep;
                }
            } else if (S == 4) {
                const uint32_t *l = reinterpret_cast<const uint32_t *>(strip);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t keep = (mk >> j) & 1u;
                    const uint32_t v = l[at];
                    d[j] = keep ? v : 0u;
                    at += keep;
                }
            } else {
                const uint16_t *l = reinterpret_cast<const uint16_t *>(strip);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t keep = (mk >> j) & 1u;
                    const uint32_t v = l[at];
                    d[j >> 1] |= (keep ? v : 0u) << (16 * (j & 1));
                    at += keep;
                }
            }
            const uint64_t e0 = wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E;
            const uint4 o = make_uint4(d[0], d[1], d[2], d[3]);
            if (full) stream_store<kDecompressNtStore>(reinterpret_cast<uint4 *>(static_cast<char *>(out) + e0 * S), o);
            else store_vec_guarded<S>(out, e0, n, o);
            row_start += BT_FIELD(r.total2, k);
        }
    }
    wave_lds_sync();                    // this tile's reads are done before the next tile's values are committed
    // a ragged tile's stores are element by element, as many as it takes: let them finish here, so that what is
    // outstanding after a tile does not depend on the tile (see the kernel)
    if (!full) __builtin_amdgcn_s_waitcnt(0x0f70);                        // vmcnt(0)
}

// What a restoring wave does when the scanner's answer for its tile does not come: it counts the set
// bits of the tensor's bitmap before the tile itself.  Slow (the whole bitmap up to the tile), but it
// needs nothing from any other workgroup.  Every bit before a tile is a bit of the tensor, so no mask.
template <int S>
__device__ __noinline__ uint64_t prefix_from_bitmap(const uint32_t *__restrict__ bitmap, const uint32_t tile, const int lane) {
    const uint64_t words = (uint64_t)tile * Geo<S>::TILE_WORDS;
    uint64_t mine = 0;
    for (uint64_t w = (uint32_t)lane; w < words; w += kWaveSize) mine += (uint32_t)__popc(bitmap[w]);
#pragma unroll
    for (int d = 1; d < kWaveSize; d <<= 1) mine += __shfl_xor((unsigned long long)mine, d, kWaveSize);
    return uniform64(mine);
}

// bt_decompress and bt_decompress_batch: workgroup 0 is the scanner (one wave of it), workgroup 1 + t
// restores slot t.  A tile's count depends on the bitmap alone: every wave turns its bitmap words into
// masks and ranks, whose totals are the wave's share of the count; the workgroup adds the shares up
// and publishes the count; then the first wave waits for the tile's prefix, every wave fetches its
// values, expands and stores them, and the workgroup ends.
//
// Why a workgroup per tile and no loop over tiles as in compression.  A wave that has issued its stores
// is gone (nothing waits for them to land) and the next workgroup takes its place, whereas a wave that
// went on to a next tile would, on this hardware, wait for its own stores whenever it waits for that
// tile's loads (one counter tracks both, in order).  Two thirds of a restoration's traffic are stores;
// kernels that loop measured 10 to 25 % slower, with or without the next tile's loads in flight.
//
// Forward progress does not rest on the order in which workgroups are started.  A workgroup publishes
// its count before it waits for anything, and one whose prefix has not come after kPatience polls
// stops waiting and counts the bitmap itself (prefix_from_bitmap): so every workgroup that has been
// started ends, whatever the others do, and every workgroup is started in the end.
template <int S, class Job>
__global__ __launch_bounds__(kBlock, kDecompressOcc) void decompress_kernel(const Job job, char *ws) {
    using G = Geo<S>;
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[kWaves * G::LDS_WAVE];
    __shared__ uint64_t s_tile_j;
    __shared__ uint32_t s_wave_total[kWaves];
    if (workspace_failed(ws)) return;
    if (blockIdx.x == 0) {
        if (threadIdx.x < kWaveSize) scan_counts<2>(ws, job);
        return;
    }
    BT_TL_INIT;
    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t slot = blockIdx.x - 1, n_slots = gridDim.x - 1;
    uint32_t *hdr = reinterpret_cast<uint32_t *>(ws);
    const Slot sl = job.at(slot);
    // the bitmap words first: everything else waits for them
    const uint32_t *const bitmap = sl.idle ? nullptr : job.bitmap(sl.item);
    const uint64_t n = sl.idle ? 0 : job.n(sl.item);
    uint32_t rows[kRows];
    rows_load<S>(bitmap, n, sl.tile, lane, wave, reinterpret_cast<const uint32_t *>(ws + kHdrSpare), rows);
    BT_TL(slot, 0);
    const Epoch ep = read_epoch(ws);
    const uint32_t cur = uniform32(ep.cur);      // (the wave has the header's words from here on)
    const uint32_t prev_slots = uniform32(ep.prev_slots);
    // masks and ranks; what they add up to is this wave's share of the tile's count
    Restoring<S> r;
    const uint32_t wave_total = sl.idle ? 0u : restore_ranks<S>(rows, n, sl.tile, lane, wave, r);
    if (lane == 0) s_wave_total[wave] = wave_total;
    lds_barrier();                      // also: every wave has read the header before the first wave publishes anything
    uint32_t before_wave = 0, tile_total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t c = s_wave_total[w];
        if (w < wave) before_wave += c;
        tile_total += c;
    }
    before_wave = uniform32(before_wave);       // the same in every lane: tell the compiler, so that addresses built on it stay scalar
    if (tid == 0) ws_store32(ws_count(ws, slot, cur), tile_total + 1);
    BT_TL(slot, 1);
    zero_previous(ws, Epoch{cur, prev_slots}, slot, n_slots);
    if (sl.idle) return;
    // Algorithm 2's counter j at the start of the tile: the first wave asks (one poller a tile keeps the
    // traffic on the workspace's few lines low) and passes the answer on through LDS
    uint32_t polls = 0;
    if (wave == 0) {
        uint64_t v;
        for (;;) {
            v = uniform64(ws_load64(ws_prefix(ws, slot, cur)));
            ++polls;
            if (v != 0) { v -= 1; break; }
            if ((polls & 255u) == 0 && polls > patience_of(hdr)) { v = prefix_from_bitmap<S>(bitmap, sl.tile, lane); break; }
            __builtin_amdgcn_s_sleep(kTileSleep);
        }
        if (lane == 0) s_tile_j = v;
    }
    lds_barrier();
    const uint64_t tile_j = uniform64(s_tile_j);
    BT_TL(slot, 2);
    restore_fetch<S>(job.values(sl.item), job.cap(sl.item), tile_j, before_wave, lane, r);
    restore_store<S>(r, n, job.out(sl.item), sl.tile, s_stage + wave * G::LDS_WAVE, lane, wave);
    BT_TL(slot, 3);
    BT_TL_VALUE(slot, 5, polls);
}

// bt_decompress_indexed and its batched form: one workgroup per slot and nothing else.  Algorithm 2's
// j at the start of the tile comes from the tile index.
template <int S, class Job>
__global__ __launch_bounds__(kBlock, 8) void decompress_indexed_kernel(const Job job) {
    using G = Geo<S>;
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[kWaves * G::LDS_WAVE];
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Slot sl = job.at(blockIdx.x);
    if (sl.idle) return;
    const uint64_t tile_j = job.tile_index(sl.item)[sl.tile];             // asked for first, needed last
    const uint32_t *const bitmap = job.bitmap(sl.item);
    const uint64_t n = job.n(sl.item);
    Ahead<S> ahead;
    ahead_load<S>(bitmap, n, sl.tile, lane, wave, bitmap, ahead);
    uint32_t before_wave;
    count_words<S>(ahead.mine, n, sl.tile, lane, wave, before_wave);
    Restoring<S> r;
    restore_ranks<S>(ahead.rows, n, sl.tile, lane, wave, r);
    restore_fetch<S>(job.values(sl.item), job.cap(sl.item), tile_j, before_wave, lane, r);
    restore_store<S>(r, n, job.out(sl.item), sl.tile, s_stage + wave * G::LDS_WAVE, lane, wave);
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

// ---- small fills ---------------------------------------------------------------------------

__global__ void fill_u64_kernel(uint64_t *p, uint64_t count, uint64_t value) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = value;
}

// bt_workspace_status: d_status[0] = 1 if a wait was given up on the workspace (else 0), d_status[1] = calls completed.
__global__ void copy_status_kernel(const uint32_t *ws, uint32_t *d_status) {
    if (threadIdx.x == 0) {
        d_status[0] = ws[kHdrError] != 0 ? 1u : 0u;
        d_status[1] = ws[kHdrSeq];
    }
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

constexpr int kMaxDevices = 64;          // devices the static workspace keeps an address for

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
    return ((tiles == 0 ? 1 : tiles) + kBatchRow - 1) / kBatchRow * kBatchRow;
}

size_t workspace_bytes_for_slots(uint64_t slots) {
    uint64_t blocks = (slots + kSlotsPerBlock - 1) / kSlotsPerBlock;
    if (blocks == 0) blocks = 1;
    return kHeaderBytes + (size_t)blocks * kBlockBytes;
}

// Tensors [first, first + count) of a batch, laid end to end.  `n_of(i)` is tensor i's element count.
template <int MAXB, class NOf>
void lay_out(BatchLayout<MAXB> &lay, size_t first, size_t count, int s, NOf n_of) {
    lay.count = (uint32_t)count;
    uint64_t at = 0;
    for (size_t i = 0; i < count; ++i) {
        const uint64_t n = n_of(first + i);
        lay.start[i] = (uint32_t)at;
        lay.tiles[i] = (uint32_t)tiles_for(n, s);
        at += batch_slots_for(n, s);
    }
    for (size_t i = count; i <= (size_t)MAXB; ++i) lay.start[i] = (uint32_t)at;
    for (size_t i = count; i < (size_t)MAXB; ++i) lay.tiles[i] = 0;
}

// Largest workspace any launch of the batch needs when it is cut into consecutive launches of `per_launch`
// tensors, which reuse the workspace.
template <class NOf>
size_t batch_workspace_bytes(size_t count, size_t per_launch, int s, NOf n_of) {
    size_t need = workspace_bytes_for_slots(0);
    for (size_t first = 0; first < count; first += per_launch) {
        const size_t c = count - first < per_launch ? count - first : per_launch;
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

// Launch the compression kernel for a dtype / pruning / dense-output combination on `job`.
template <class Job>
bt_status launch_compress(const Job &job, uint64_t slots, bt_dtype dtype, bool prune, bool dense, double threshold,
                          char *ws, hipStream_t hs) {
    const dim3 block(kBlock);
    // Elements narrower than a double are compared in single precision.  For a single x, x > threshold exactly when
    // x > the largest single at or below the threshold, so that is what the kernel gets (a NaN stays one: nothing
    // exceeds it).
    float threshold_f = (float)threshold;
    if ((double)threshold_f > threshold) threshold_f = std::nextafterf(threshold_f, -INFINITY);
#define BT_LAUNCH_COMPRESS(S_, KEEP_, DENSE_)                                                   \
    do {                                                                                        \
        auto kernel = compress_kernel<S_, KEEP_, DENSE_, Job>;                                  \
        kernel<<<dim3((unsigned)(slots + 1)), block, 0, hs>>>(job, ws, threshold, threshold_f);  \
    } while (0)
    const int s = elem_size(dtype);
    if (!prune) {
        if (s == 8) BT_LAUNCH_COMPRESS(8, kKeepNonZero, false);
        else if (s == 4) BT_LAUNCH_COMPRESS(4, kKeepNonZero, false);
        else BT_LAUNCH_COMPRESS(2, kKeepNonZero, false);
    } else if (!dense) {
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

template <class Job>
bt_status launch_decompress(const Job &job, uint64_t slots, int s, char *ws, hipStream_t hs) {
    const dim3 block(kBlock);
#define BT_LAUNCH_DECOMPRESS(S_)                                                                \
    do {                                                                                        \
        auto kernel = decompress_kernel<S_, Job>;                                               \
        kernel<<<dim3((unsigned)(slots + 1)), block, 0, hs>>>(job, ws);                         \
    } while (0)
    if (s == 8) BT_LAUNCH_DECOMPRESS(8);
    else if (s == 4) BT_LAUNCH_DECOMPRESS(4);
    else BT_LAUNCH_DECOMPRESS(2);
#undef BT_LAUNCH_DECOMPRESS
    return launched();
}

template <class Job>
bt_status launch_decompress_indexed(const Job &job, uint64_t slots, int s, hipStream_t hs) {
    const dim3 grid((unsigned)slots), block(kBlock);
    if (s == 8) decompress_indexed_kernel<8, Job><<<grid, block, 0, hs>>>(job);
    else if (s == 4) decompress_indexed_kernel<4, Job><<<grid, block, 0, hs>>>(job);
    else decompress_indexed_kernel<2, Job><<<grid, block, 0, hs>>>(job);
    return launched();
}

// ---- a workspace that belongs to the library -------------------------------------------------
//
// For callers that cannot allocate (see bt_compress_static in the header): a workspace for tensors of
// up to BT_STATIC_MAX_TILES tiles, one copy on every device the library is used on, held until the
// process ends.  In host code the array's name only stands for the symbol: what kernels and fills get is
// the address that the runtime reports for it on the current device, looked up once per device.
constexpr size_t kStaticBytes = kHeaderBytes + (size_t)(BT_STATIC_MAX_TILES / kSlotsPerBlock) * kBlockBytes;
static_assert(BT_STATIC_MAX_TILES % kSlotsPerBlock == 0, "whole blocks");
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

bt_status static_workspace(char **ws) {
    static std::atomic<char *> known[kMaxDevices];
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) {
        (void)hipGetLastError();
        return BT_ERR_HIP;
    }
    char *ptr = known[device].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        if (hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return BT_ERR_HIP;
        }
        known[device].store(ptr, std::memory_order_release);      // (two threads may both look it up: same answer)
    }
    *ws = ptr;
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

static bt_status compress_common(const void *d_in, uint64_t n, bt_dtype dtype, bool prune, double threshold,
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
    const CompressOne job{d_in, n, d_bitmap, d_values, values_cap, d_nnz, d_index, d_dense, n_tiles};
    return launch_compress(job, n_tiles, dtype, prune, d_dense != nullptr, threshold, static_cast<char *>(d_workspace), hs);
}

bt_status bt_compress(const void *d_in, uint64_t n, bt_dtype dtype, uint32_t *d_bitmap, void *d_values,
                      uint64_t values_cap, uint64_t *d_nnz, void *d_workspace, size_t workspace_bytes,
                      bt_stream stream) {
    return compress_common(d_in, n, dtype, false, 0.0, d_bitmap, d_values, values_cap, d_nnz, nullptr, nullptr,
                           d_workspace, workspace_bytes, stream);
}

bt_status bt_compress_static(const void *d_in, uint64_t n, bt_dtype dtype, uint32_t *d_bitmap, void *d_values,
                             uint64_t values_cap, uint64_t *d_nnz, bt_stream stream) {
    const int s = elem_size(dtype);
    if (s == 0) return BT_ERR_DTYPE;
    if (n > BT_MAX_ELEMENTS || tiles_for(n, s) > BT_STATIC_MAX_TILES) return BT_ERR_SIZE;
    char *ws = nullptr;
    const bt_status st = static_workspace(&ws);
    if (st != BT_OK) return st;
    // The array keeps what the last call left, possibly a call that gave up a wait: start from a clean workspace
    // every time (a fill kernel rather than a memset, which callers that record the stream could not replay).
    const uint64_t words = kStaticBytes / 8;
    fill_u64_kernel<<<dim3((unsigned)((words + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
        reinterpret_cast<uint64_t *>(ws), words, 0);
    const bt_status fs = launched();
    if (fs != BT_OK) return fs;
    return compress_common(d_in, n, dtype, false, 0.0, d_bitmap, d_values, values_cap, d_nnz, nullptr, nullptr, ws,
                           kStaticBytes, stream);
}

bt_status bt_compress_pruned(const void *d_in, uint64_t n, bt_dtype dtype, double threshold, uint32_t *d_bitmap,
                             void *d_values, uint64_t values_cap, uint64_t *d_nnz, void *d_workspace,
                             size_t workspace_bytes, bt_stream stream) {
    return compress_common(d_in, n, dtype, true, threshold, d_bitmap, d_values, values_cap, d_nnz, nullptr, nullptr,
                           d_workspace, workspace_bytes, stream);
}

bt_status bt_activation_compress(const void *d_in, uint64_t n, bt_dtype dtype, double threshold, void *d_dense_out,
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
    return compress_common(d_in, n, dtype, false, 0.0, d_bitmap, d_values, values_cap, d_nnz, d_index, nullptr,
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
    const uint32_t n_tiles = (uint32_t)tiles_for(n, s);
    const DecompressOne job{d_bitmap, d_values, values_cap, d_index, n, d_out, n_tiles};
    return launch_decompress_indexed(job, n_tiles, s, (hipStream_t)stream);
}

bt_status bt_decompress(const uint32_t *d_bitmap, const void *d_values, uint64_t n, bt_dtype dtype, void *d_out,
                        void *d_workspace, size_t workspace_bytes, bt_stream stream) {
    const bt_status st = check_common(n, dtype, d_workspace, workspace_bytes);
    if (st != BT_OK) return st;
    if (n == 0) return BT_OK;
    const int s = elem_size(dtype);
    if (d_bitmap == nullptr || d_out == nullptr) return BT_ERR_NULL;   // d_values may be NULL when nnz == 0
    if (misaligned(d_out, 16) || misaligned(d_bitmap, 4) || misaligned(d_values, (size_t)s)) return BT_ERR_ALIGN;
    const uint32_t n_tiles = (uint32_t)tiles_for(n, s);
    const DecompressOne job{d_bitmap, d_values, ~(uint64_t)0, nullptr, n, d_out, n_tiles};
    return launch_decompress(job, n_tiles, s, static_cast<char *>(d_workspace), (hipStream_t)stream);
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

size_t bt_batch_workspace_bytes(const uint64_t *n, size_t count, bt_dtype dtype) {
    const int s = elem_size(dtype);
    if (s == 0 || (n == nullptr && count != 0)) return 0;
    const auto n_of = [n](size_t i) { return n[i] > BT_MAX_ELEMENTS ? BT_MAX_ELEMENTS : n[i]; };
    const size_t a = batch_workspace_bytes(count, (size_t)kMaxBatchCompress, s, n_of);
    const size_t b = batch_workspace_bytes(count, (size_t)kMaxBatchDecompress, s, n_of);
    return a > b ? a : b;
}

static bt_status compress_batch_common(const bt_compress_item *items, size_t count, bt_dtype dtype, bool prune,
                                       double threshold, void *d_workspace, size_t workspace_bytes, bt_stream stream) {
    const bt_status st = check_batch_common(items, count, dtype, d_workspace);
    if (st != BT_OK || count == 0) return st;
    const int s = elem_size(dtype);
    size_t with_dense = 0, not_empty = 0;
    for (size_t i = 0; i < count; ++i) {
        const bt_compress_item &it = items[i];
        if (it.n > BT_MAX_ELEMENTS) return BT_ERR_SIZE;
        if (it.d_nnz == nullptr) return BT_ERR_NULL;
        if (misaligned(it.d_nnz, 8)) return BT_ERR_ALIGN;
        if (it.n == 0) continue;
        ++not_empty;
        if (it.d_in == nullptr || it.d_bitmap == nullptr) return BT_ERR_NULL;
        if (it.d_values == nullptr && it.values_cap != 0) return BT_ERR_NULL;
        if (misaligned(it.d_in, 16) || misaligned(it.d_bitmap, 4) || misaligned(it.d_values, (size_t)s) ||
            misaligned(it.d_index, 8) || misaligned(it.d_dense_out, 16))
            return BT_ERR_ALIGN;
        if (it.d_dense_out != nullptr) ++with_dense;
    }
    // the dense output is a property of the launch: for every tensor that has elements, or for none
    if (with_dense != 0 && (!prune || with_dense != not_empty)) return BT_ERR_NULL;
    const auto n_of = [items](size_t i) { return items[i].n; };
    if (workspace_bytes < batch_workspace_bytes(count, (size_t)kMaxBatchCompress, s, n_of)) return BT_ERR_WORKSPACE;

    hipStream_t hs = (hipStream_t)stream;
    char *ws = static_cast<char *>(d_workspace);
    for (size_t first = 0; first < count; first += kMaxBatchCompress) {
        const size_t c = count - first < (size_t)kMaxBatchCompress ? count - first : (size_t)kMaxBatchCompress;
        CompressMany b;
        lay_out(b.lay, first, c, s, n_of);
        for (size_t i = 0; i < (size_t)kMaxBatchCompress; ++i) {
            const bt_compress_item it =
                i < c ? items[first + i] : bt_compress_item{nullptr, 0, nullptr, nullptr, 0, nullptr, nullptr, nullptr};
            b.in_[i] = it.d_in;
            b.n_[i] = it.n;
            b.bitmap_[i] = it.d_bitmap;
            b.values_[i] = it.d_values;
            b.cap_[i] = it.values_cap;
            b.nnz_[i] = it.d_nnz;
            b.index_[i] = it.n != 0 ? it.d_index : nullptr;
            b.dense_[i] = it.n != 0 ? it.d_dense_out : nullptr;
        }
        const bt_status ls = launch_compress(b, b.lay.start[c], dtype, prune, with_dense != 0, threshold, ws, hs);
        if (ls != BT_OK) return ls;
    }
    return BT_OK;
}

bt_status bt_compress_batch(const bt_compress_item *items, size_t count, bt_dtype dtype, void *d_workspace,
                            size_t workspace_bytes, bt_stream stream) {
    return compress_batch_common(items, count, dtype, false, 0.0, d_workspace, workspace_bytes, stream);
}

bt_status bt_compress_batch_pruned(const bt_compress_item *items, size_t count, bt_dtype dtype, double threshold,
                                   void *d_workspace, size_t workspace_bytes, bt_stream stream) {
    return compress_batch_common(items, count, dtype, true, threshold, d_workspace, workspace_bytes, stream);
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
    if (workspace_bytes < batch_workspace_bytes(count, (size_t)kMaxBatchDecompress, s, n_of)) return BT_ERR_WORKSPACE;

    hipStream_t hs = (hipStream_t)stream;
    char *ws = static_cast<char *>(d_workspace);
    for (size_t first = 0; first < count; first += kMaxBatchDecompress) {
        const size_t c = count - first < (size_t)kMaxBatchDecompress ? count - first : (size_t)kMaxBatchDecompress;
        DecompressMany b;
        lay_out(b.lay, first, c, s, n_of);
        for (size_t i = 0; i < (size_t)kMaxBatchDecompress; ++i) {
            const bt_decompress_item it = i < c ? items[first + i] : bt_decompress_item{nullptr, nullptr, 0, nullptr, 0, nullptr};
            b.bitmap_[i] = it.d_bitmap;
            b.values_[i] = it.d_values;
            b.cap_[i] = ~(uint64_t)0;
            b.index_[i] = nullptr;
            b.n_[i] = it.n;
            b.out_[i] = it.d_out;
        }
        const bt_status ls = launch_decompress(b, b.lay.start[c], s, ws, hs);
        if (ls != BT_OK) return ls;
    }
    return BT_OK;
}

bt_status bt_decompress_batch_indexed(const bt_decompress_item *items, size_t count, bt_dtype dtype, bt_stream stream) {
    const int s = elem_size(dtype);
    if (s == 0) return BT_ERR_DTYPE;
    if (count == 0) return BT_OK;
    if (items == nullptr) return BT_ERR_NULL;
    for (size_t i = 0; i < count; ++i) {
        const bt_decompress_item &it = items[i];
        if (it.n > BT_MAX_ELEMENTS) return BT_ERR_SIZE;
        if (it.n == 0) continue;
        if (it.d_bitmap == nullptr || it.d_out == nullptr || it.d_index == nullptr) return BT_ERR_NULL;
        if (it.d_values == nullptr && it.values_cap != 0) return BT_ERR_NULL;
        if (misaligned(it.d_out, 16) || misaligned(it.d_bitmap, 4) || misaligned(it.d_values, (size_t)s) || misaligned(it.d_index, 8))
            return BT_ERR_ALIGN;
    }
    const auto n_of = [items](size_t i) { return items[i].n; };
    hipStream_t hs = (hipStream_t)stream;
    for (size_t first = 0; first < count; first += kMaxBatchDecompress) {
        const size_t c = count - first < (size_t)kMaxBatchDecompress ? count - first : (size_t)kMaxBatchDecompress;
        DecompressMany b;
        lay_out(b.lay, first, c, s, n_of);
        for (size_t i = 0; i < (size_t)kMaxBatchDecompress; ++i) {
            const bt_decompress_item it = i < c ? items[first + i] : bt_decompress_item{nullptr, nullptr, 0, nullptr, 0, nullptr};
            b.bitmap_[i] = it.d_bitmap;
            b.values_[i] = it.d_values;
            b.cap_[i] = it.values_cap;
            b.index_[i] = it.d_index;
            b.n_[i] = it.n;
            b.out_[i] = it.d_out;
        }
        const bt_status ls = launch_decompress_indexed(b, b.lay.start[c], s, hs);
        if (ls != BT_OK) return ls;
    }
    return BT_OK;
}

// What the kernels leave in a workspace's header when they had to give up, as words a caller can copy back and look
// at without knowing the layout.
bt_status bt_workspace_status(const void *d_workspace, uint32_t *d_status, bt_stream stream) {
    if (d_workspace == nullptr || d_status == nullptr) return BT_ERR_NULL;
    if (misaligned(d_workspace, 128) || misaligned(d_status, 4)) return BT_ERR_ALIGN;
    copy_status_kernel<<<dim3(1), dim3(64), 0, (hipStream_t)stream>>>(static_cast<const uint32_t *>(d_workspace), d_status);
    return launched();
}

}  // extern "C"
