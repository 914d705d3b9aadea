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
//   grid    decoupled look-back over per-tile descriptors {epoch, status, count}
//
// There is no matrix contraction anywhere, so no MFMA: the path is bound by HBM
// bandwidth and everything here is about moving each byte once, coalesced.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bittrain.h"

namespace {

constexpr int kWaveSize = 64;
constexpr int kWaves = 4;                 // waves per block
constexpr int kBlock = kWaveSize * kWaves;
constexpr int kRows = 4;                  // 16-byte loads per lane per tile
constexpr int kVecBytes = 16;

// Workspace header (uint32 words); descriptors start at byte kHeaderBytes.
constexpr int kHdrTicket = 0;   // next tile to hand out
constexpr int kHdrDone = 1;     // tiles whose look-back has finished
constexpr int kHdrEpoch = 2;    // tag of the current call, 24 bits
constexpr int kHdrError = 3;    // set if a look-back gave up waiting
constexpr size_t kHeaderBytes = 256;

// Descriptor word: [63:40] epoch, [39:38] status, [37:0] count.
constexpr int kEpochShift = 40;
constexpr int kStatusShift = 38;
constexpr uint64_t kCountMask = ((uint64_t)1 << kStatusShift) - 1;
constexpr uint32_t kEpochMask = (1u << 24) - 1;
constexpr uint64_t kStAggregate = 1;      // count = non-zeros of this tile alone
constexpr uint64_t kStPrefix = 2;         // count = non-zeros of tiles [0, this]
constexpr uint32_t kSpinLimit = 1u << 20; // polls before a look-back gives up

template <int S> struct Geo {
    static constexpr int E = kVecBytes / S;          // elements per lane per load
    static constexpr int G = 32 / E;                 // lanes that share a bitmap word
    static constexpr int WPR = kWaveSize / G;        // bitmap words per row
    static constexpr int ROW = kWaveSize * E;        // elements per wave-wide load
    static constexpr int WAVE = kRows * ROW;         // elements per wave per tile
    static constexpr int TILE = kWaves * WAVE;       // elements per tile
    static constexpr int LDS_WAVE = WAVE * S + kVecBytes;  // staging bytes per wave
    static_assert(kRows <= G, "one bitmap store per wave needs rows <= lanes per word");
    static_assert(kRows % 2 == 0, "row counts are scanned two to a register");
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

__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_sum(x), 63);
}

// OR over each aligned group of G lanes (G = 4 or 8); every lane gets the result.
template <int G> __device__ __forceinline__ uint32_t group_or(uint32_t x) {
    x |= BT_DPP(0, x, 0xB1, 0xf, true);       // quad_perm [1,0,3,2]: lane ^ 1
    x |= BT_DPP(0, x, 0x4E, 0xf, true);       // quad_perm [2,3,0,1]: lane ^ 2
    if (G == 8) x |= BT_DPP(0, x, 0x141, 0xf, true);  // row_half_mirror: lane i <-> 7 - i
    return x;
}

// Order LDS traffic between the lanes of one wave (no block barrier involved).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- per-lane helpers -----------------------------------------------------------

// Bit j set <=> element j of the 16-byte vector has a non-zero bit pattern.
template <int S> __device__ __forceinline__ uint32_t nonzero_mask(const uint4 v) {
    if (S == 4) {
        return (v.x != 0 ? 1u : 0u) | (v.y != 0 ? 2u : 0u) | (v.z != 0 ? 4u : 0u) | (v.w != 0 ? 8u : 0u);
    } else {
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
        uint32_t m = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            m |= ((d[i] & 0xffffu) != 0 ? 1u : 0u) << (2 * i);
            m |= ((d[i] >> 16) != 0 ? 1u : 0u) << (2 * i + 1);
        }
        return m;
    }
}

// 16 bytes at element index e0 of a buffer of n elements; elements at or beyond n read as 0.
template <int S> __device__ __forceinline__ uint4 load_vec_guarded(const void *base, uint64_t e0, uint64_t n) {
    constexpr int E = Geo<S>::E;
    if (e0 + E <= n) return *reinterpret_cast<const uint4 *>(static_cast<const char *>(base) + e0 * S);
    uint32_t d[4] = {0, 0, 0, 0};
    if (S == 4) {
        const uint32_t *p = static_cast<const uint32_t *>(base);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (e0 + j < n) d[j] = p[e0 + j];
    } else {
        const uint16_t *p = static_cast<const uint16_t *>(base);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (e0 + j < n) d[j >> 1] |= (uint32_t)p[e0 + j] << (16 * (j & 1));
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
    if (S == 4) {
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

// ---- tile bookkeeping ----------------------------------------------------------------

__device__ __forceinline__ uint64_t desc_load(const uint64_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void desc_store(uint64_t *p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Tiles are handed out by an atomic ticket, so a tile only ever waits for tiles
// that are already running: the look-back below cannot deadlock whatever order
// the hardware starts workgroups in.  Called by thread 0 of the block.
__device__ __forceinline__ void take_ticket(uint32_t *hdr, uint32_t *tile, uint32_t *epoch) {
    *tile = __hip_atomic_fetch_add(&hdr[kHdrTicket], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *epoch = __hip_atomic_load(&hdr[kHdrEpoch], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kEpochMask;
}

// Decoupled look-back, run by one whole wave.  Publishes this tile's count, then
// walks back over the predecessors' descriptors 64 at a time, adding aggregates
// until it meets a tile that already knows its inclusive prefix.  Returns the
// number of non-zero elements in all tiles before `tile`.  A descriptor carries
// count and status in one 64-bit word, so relaxed device-scope atomics are enough:
// no other memory is communicated between tiles.  Descriptors of earlier calls
// carry another epoch and read as "not there yet", so nothing is cleared per call.
__device__ __forceinline__ uint64_t look_back(uint64_t *desc, uint32_t *hdr, uint32_t tile, uint32_t epoch,
                                              uint32_t aggregate, int lane) {
    const uint64_t tag = (uint64_t)epoch << kEpochShift;
    if (tile == 0) {
        if (lane == 0) desc_store(&desc[0], tag | (kStPrefix << kStatusShift) | aggregate);
        return 0;
    }
    if (lane == 0) desc_store(&desc[tile], tag | (kStAggregate << kStatusShift) | aggregate);

    uint64_t exclusive = 0;
    int64_t pos = (int64_t)tile - 1;   // lane 0 looks at the nearest predecessor
    uint32_t spins = 0;
    bool gave_up = false;
    for (;;) {
        const int64_t idx = pos - lane;
        uint64_t d = 0;
        uint32_t st = 0;
        uint64_t need = 0;
        uint64_t have_prefix = 0;
        for (;;) {
            if (idx >= 0) {
                d = desc_load(&desc[idx]);
                st = ((uint32_t)(d >> kEpochShift) == epoch) ? (uint32_t)(d >> kStatusShift) & 3u : 0u;
            } else {
                d = 0;                      // before tile 0: an inclusive prefix of 0
                st = (uint32_t)kStPrefix;
            }
            have_prefix = __ballot(st == (uint32_t)kStPrefix);
            const uint64_t missing = __ballot(st == 0u);
            // lanes 0 .. first prefix lane (all 64 if there is none) must be published
            const uint64_t first = have_prefix & (~have_prefix + 1);
            need = have_prefix ? (first | (first - 1)) : ~(uint64_t)0;
            if ((missing & need) == 0) break;
            // bounded wait: give up after kSpinLimit polls, or soon after any tile has given up
            ++spins;
            if (spins > kSpinLimit ||
                ((spins & 255u) == 0 &&
                 __hip_atomic_load(&hdr[kHdrError], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                gave_up = true;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        if (gave_up) break;
        const bool mine = (need >> lane) & 1;
        const uint32_t agg = (mine && st == (uint32_t)kStAggregate) ? (uint32_t)(d & kCountMask) : 0u;
        exclusive += wave_sum(agg);
        if (have_prefix) {
            const int fl = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)have_prefix) - 1);
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)d, fl);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(d >> 32), fl);
            exclusive += (((uint64_t)hi << 32) | lo) & kCountMask;
            break;
        }
        pos -= kWaveSize;
    }
    if (gave_up) {
        if (lane == 0) __hip_atomic_store(&hdr[kHdrError], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return exclusive;
    }
    if (lane == 0) desc_store(&desc[tile], tag | (kStPrefix << kStatusShift) | (exclusive + aggregate));
    return exclusive;
}

// Called once per tile (one lane) after its look-back.  The tile that finishes
// last puts the header back into the state the next call expects: ticket and
// done counter at 0, epoch advanced.  When the 24-bit epoch wraps, every
// descriptor is cleared so a tag can never be mistaken for one of 2^24 calls ago.
__device__ __forceinline__ void tile_done(uint32_t *hdr, uint64_t *desc, uint32_t n_tiles, uint32_t desc_capacity,
                                          uint32_t epoch) {
    const uint32_t before = __hip_atomic_fetch_add(&hdr[kHdrDone], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (before + 1 != n_tiles) return;
    const uint32_t next = (epoch + 1) & kEpochMask;
    if (next == 0)
        for (uint32_t i = 0; i < desc_capacity; ++i) desc_store(&desc[i], 0);
    __hip_atomic_store(&hdr[kHdrTicket], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&hdr[kHdrDone], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&hdr[kHdrEpoch], next, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Per-row popcounts -> exclusive rank of each lane inside its row, and row totals.
// Two rows share a register (16-bit fields; a row holds at most 512 non-zeros).
__device__ __forceinline__ void rank_rows(const uint32_t (&m)[kRows], uint32_t (&lane_rank)[kRows],
                                          uint32_t (&row_total)[kRows]) {
#pragma unroll
    for (int k = 0; k < kRows; k += 2) {
        const uint32_t packed = (uint32_t)__popc(m[k]) | ((uint32_t)__popc(m[k + 1]) << 16);
        const uint32_t incl = wave_inclusive_sum(packed);
        const uint32_t excl = incl - packed;
        const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        lane_rank[k] = excl & 0xffffu;
        lane_rank[k + 1] = excl >> 16;
        row_total[k] = tot & 0xffffu;
        row_total[k + 1] = tot >> 16;
    }
}

// ---- Algorithm 1: dense -> bitmap -------------------------------------------------------

template <int S>
__global__ __launch_bounds__(kBlock) void compress_kernel(const void *__restrict__ in, const uint64_t n,
                                                          uint32_t *__restrict__ bitmap, void *__restrict__ values,
                                                          const uint64_t values_cap, uint64_t *__restrict__ nnz_out,
                                                          uint32_t *hdr, uint64_t *desc, const uint32_t n_tiles,
                                                          const uint32_t desc_capacity) {
    using G = Geo<S>;
    constexpr int E = G::E;
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[kWaves * G::LDS_WAVE];
    __shared__ uint32_t s_wave_total[kWaves];
    __shared__ uint32_t s_tile, s_epoch;
    __shared__ uint64_t s_tile_base;

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = tid >> 6;

    if (tid == 0) {
        uint32_t t, e;
        take_ticket(hdr, &t, &e);
        s_tile = t;
        s_epoch = e;
    }
    __syncthreads();
    const uint32_t tile = s_tile;
    const uint32_t epoch = s_epoch;
    if (tile >= n_tiles) return;   // cannot happen with grid == n_tiles; keeps every access in bounds

    const uint64_t n_words = (n + 31) >> 5;
    const uint64_t wave_e0 = (uint64_t)tile * G::TILE + (uint64_t)wave * G::WAVE;
    const bool full = (uint64_t)(tile + 1) * G::TILE <= n;

    // (1) load: lane l of row k owns elements wave_e0 + k*ROW + l*E ... + E-1
    uint4 x[kRows];
    if (full) {
        const uint4 *p = reinterpret_cast<const uint4 *>(static_cast<const char *>(in) + wave_e0 * S) + lane;
#pragma unroll
        for (int k = 0; k < kRows; ++k) x[k] = p[k * kWaveSize];
    } else {
#pragma unroll
        for (int k = 0; k < kRows; ++k) x[k] = load_vec_guarded<S>(in, wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E, n);
    }

    // (2) Algorithm 1's test "T[i] == 0", on the bit pattern, and the ranks
    uint32_t m[kRows], lane_rank[kRows], row_total[kRows];
#pragma unroll
    for (int k = 0; k < kRows; ++k) m[k] = nonzero_mask<S>(x[k]);
    rank_rows(m, lane_rank, row_total);
    uint32_t wave_total = 0;
    uint32_t row_base[kRows];
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
        row_base[k] = wave_total;
        wave_total += row_total[k];
    }

    // (3) "push bit to B.bitmap": G lanes OR their E-bit masks into one 32-bit word,
    //     then lane (g*G + i) stores the word of row i, group g: one store per wave.
    {
        const int g = lane / G::G, i = lane % G::G;
        uint32_t word = 0;
#pragma unroll
        for (int k = 0; k < kRows; ++k) {
            const uint32_t w = group_or<G::G>(m[k] << (uint32_t)(E * i));
            if (i == k) word = w;
        }
        const uint64_t widx = (wave_e0 >> 5) + (uint64_t)i * G::WPR + (uint64_t)g;
        if (i < kRows && widx < n_words) bitmap[widx] = word;
    }

    // (4) block total, grid prefix
    if (lane == 0) s_wave_total[wave] = wave_total;
    __syncthreads();
    if (wave == 0) {
        const uint32_t tile_total = s_wave_total[0] + s_wave_total[1] + s_wave_total[2] + s_wave_total[3];
        const uint64_t base = look_back(desc, hdr, tile, epoch, tile_total, lane);
        if (lane == 0) {
            s_tile_base = base;
            if (tile == n_tiles - 1) *nnz_out = base + tile_total;   // length(B.values)
            tile_done(hdr, desc, n_tiles, desc_capacity, epoch);
        }
    }
    __syncthreads();
    uint64_t wave_base = s_tile_base;
    for (int w = 0; w < wave; ++w) wave_base += s_wave_total[w];

    // (5) "push T[i] to B.values": compact this wave's non-zeros into its LDS strip,
    //     shifted so that LDS byte 0 maps to a 16-byte aligned address of `values`,
    //     then write the strip out with aligned 16-byte stores.
    unsigned char *strip = s_stage + wave * G::LDS_WAVE;
    char *gdst = static_cast<char *>(values) + wave_base * S;                 // first value of this wave
    const uint32_t pad = (uint32_t)(reinterpret_cast<uintptr_t>(gdst) & (kVecBytes - 1)) / S;   // elements
    if (S == 4) {
        uint32_t *l = reinterpret_cast<uint32_t *>(strip);
#pragma unroll
        for (int k = 0; k < kRows; ++k) {
            uint32_t r = pad + row_base[k] + lane_rank[k];
            const uint32_t d[4] = {x[k].x, x[k].y, x[k].z, x[k].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (m[k] & (1u << j)) l[r] = d[j];
                r += (m[k] >> j) & 1u;
            }
        }
    } else {
        uint16_t *l = reinterpret_cast<uint16_t *>(strip);
#pragma unroll
        for (int k = 0; k < kRows; ++k) {
            uint32_t r = pad + row_base[k] + lane_rank[k];
            const uint32_t d[4] = {x[k].x, x[k].y, x[k].z, x[k].w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (m[k] & (1u << j)) l[r] = (uint16_t)(d[j >> 1] >> (16 * (j & 1)));
                r += (m[k] >> j) & 1u;
            }
        }
    }
    wave_lds_sync();

    // capacity clamp: never write at or beyond values_cap
    uint32_t cnt = wave_total;
    if (wave_base >= values_cap) cnt = 0;
    else if (values_cap - wave_base < cnt) cnt = (uint32_t)(values_cap - wave_base);
    if (cnt == 0) return;
    char *gvec = gdst - (size_t)pad * S;                    // 16-byte aligned; may start before the first value
    const uint32_t lo_valid = pad, hi_valid = pad + cnt;    // LDS element range to write out
    const uint32_t n_vec = (hi_valid + E - 1) / E;
    for (uint32_t v = lane; v < n_vec; v += kWaveSize) {
        const uint32_t lo = v * E, hi = lo + E;
        if (lo >= lo_valid && hi <= hi_valid) {
            *reinterpret_cast<uint4 *>(gvec + (size_t)lo * S) = *reinterpret_cast<const uint4 *>(strip + (size_t)lo * S);
        } else {
#pragma unroll
            for (int j = 0; j < E; ++j) {
                const uint32_t e = lo + j;
                if (e >= lo_valid && e < hi_valid) {
                    if (S == 4) reinterpret_cast<uint32_t *>(gvec)[e] = reinterpret_cast<const uint32_t *>(strip)[e];
                    else reinterpret_cast<uint16_t *>(gvec)[e] = reinterpret_cast<const uint16_t *>(strip)[e];
                }
            }
        }
    }
}

// ---- Algorithm 2: bitmap -> dense ---------------------------------------------------------

template <int S>
__global__ __launch_bounds__(kBlock) void decompress_kernel(const uint32_t *__restrict__ bitmap,
                                                            const void *__restrict__ values, const uint64_t n,
                                                            void *__restrict__ out, uint32_t *hdr, uint64_t *desc,
                                                            const uint32_t n_tiles, const uint32_t desc_capacity) {
    using G = Geo<S>;
    constexpr int E = G::E;
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[kWaves * G::LDS_WAVE];
    __shared__ uint32_t s_wave_total[kWaves];
    __shared__ uint32_t s_tile, s_epoch;
    __shared__ uint64_t s_tile_base;

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = tid >> 6;

    if (tid == 0) {
        uint32_t t, e;
        take_ticket(hdr, &t, &e);
        s_tile = t;
        s_epoch = e;
    }
    __syncthreads();
    const uint32_t tile = s_tile;
    const uint32_t epoch = s_epoch;
    if (tile >= n_tiles) return;

    const uint64_t n_words = (n + 31) >> 5;
    const uint64_t wave_e0 = (uint64_t)tile * G::TILE + (uint64_t)wave * G::WAVE;

    // (1) this lane's bits of "B.bitmap[i] is set", and Algorithm 2's counter j as ranks
    uint32_t m[kRows], lane_rank[kRows], row_total[kRows];
#pragma unroll
    for (int k = 0; k < kRows; ++k)
        m[k] = bitmap_bits<S>(bitmap, wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E, n, n_words);
    rank_rows(m, lane_rank, row_total);
    uint32_t wave_total = 0;
    uint32_t row_base[kRows];
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
        row_base[k] = wave_total;
        wave_total += row_total[k];
    }

    // (2) block total, grid prefix
    if (lane == 0) s_wave_total[wave] = wave_total;
    __syncthreads();
    if (wave == 0) {
        const uint32_t tile_total = s_wave_total[0] + s_wave_total[1] + s_wave_total[2] + s_wave_total[3];
        const uint64_t base = look_back(desc, hdr, tile, epoch, tile_total, lane);
        if (lane == 0) {
            s_tile_base = base;
            tile_done(hdr, desc, n_tiles, desc_capacity, epoch);
        }
    }
    __syncthreads();
    uint64_t wave_base = s_tile_base;
    for (int w = 0; w < wave; ++w) wave_base += s_wave_total[w];

    // (3) bring this wave's values[wave_base .. +wave_total) into its LDS strip with
    //     aligned 16-byte loads (first and last vector element by element: nothing
    //     outside the wave's own range is ever read)
    unsigned char *strip = s_stage + wave * G::LDS_WAVE;
    const char *gsrc = static_cast<const char *>(values) + wave_base * S;
    const uint32_t pad = (uint32_t)(reinterpret_cast<uintptr_t>(gsrc) & (kVecBytes - 1)) / S;
    const char *gvec = gsrc - (size_t)pad * S;
    const uint32_t lo_valid = pad, hi_valid = pad + wave_total;
    const uint32_t n_vec = wave_total ? (hi_valid + E - 1) / E : 0;
    for (uint32_t v = lane; v < n_vec; v += kWaveSize) {
        const uint32_t lo = v * E, hi = lo + E;
        if (lo >= lo_valid && hi <= hi_valid) {
            *reinterpret_cast<uint4 *>(strip + (size_t)lo * S) = *reinterpret_cast<const uint4 *>(gvec + (size_t)lo * S);
        } else {
#pragma unroll
            for (int j = 0; j < E; ++j) {
                const uint32_t e = lo + j;
                if (e >= lo_valid && e < hi_valid) {
                    if (S == 4) reinterpret_cast<uint32_t *>(strip)[e] = reinterpret_cast<const uint32_t *>(gvec)[e];
                    else reinterpret_cast<uint16_t *>(strip)[e] = reinterpret_cast<const uint16_t *>(gvec)[e];
                }
            }
        }
    }
    wave_lds_sync();

    // (4) "push B.values[j] / push 0.0 to T": expand from LDS by rank, store 16 bytes per lane
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
        uint32_t r = pad + row_base[k] + lane_rank[k];
        uint32_t d[4] = {0, 0, 0, 0};
        if (S == 4) {
            const uint32_t *l = reinterpret_cast<const uint32_t *>(strip);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (m[k] & (1u << j)) d[j] = l[r];
                r += (m[k] >> j) & 1u;
            }
        } else {
            const uint16_t *l = reinterpret_cast<const uint16_t *>(strip);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (m[k] & (1u << j)) d[j >> 1] |= (uint32_t)l[r] << (16 * (j & 1));
                r += (m[k] >> j) & 1u;
            }
        }
        store_vec_guarded<S>(out, wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E, n, make_uint4(d[0], d[1], d[2], d[3]));
    }
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
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const uint64_t n_words = (n + 31) >> 5;
    const uint64_t wave_e0 = (uint64_t)blockIdx.x * G::TILE + (uint64_t)wave * G::WAVE;
    const bool full = ((uint64_t)blockIdx.x + 1) * G::TILE <= n;

    uint4 g[kRows];
    uint32_t m[kRows];
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
        const uint64_t e0 = wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E;
        if (full) {
            g[k] = *reinterpret_cast<const uint4 *>(static_cast<const char *>(grad_out) + e0 * S);
            m[k] = (bitmap[e0 >> 5] >> (uint32_t)(e0 & 31)) & ((1u << E) - 1u);
        } else {
            g[k] = load_vec_guarded<S>(grad_out, e0, n);
            m[k] = bitmap_bits<S>(bitmap, e0, n, n_words);
        }
    }
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
        const uint64_t e0 = wave_e0 + (uint64_t)k * G::ROW + (uint64_t)lane * E;
        uint32_t d[4] = {g[k].x, g[k].y, g[k].z, g[k].w};
        if (S == 4) {
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
        if (full) *reinterpret_cast<uint4 *>(static_cast<char *>(grad_in) + e0 * S) = o;
        else store_vec_guarded<S>(grad_in, e0, n, o);
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
    }
    return 0;
}

uint64_t tile_elems(int s) { return s == 4 ? (uint64_t)Geo<4>::TILE : (uint64_t)Geo<2>::TILE; }

uint64_t tiles_for(uint64_t n, int s) {
    const uint64_t t = tile_elems(s);
    return (n + t - 1) / t;
}

bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

bt_status launched() { return hipGetLastError() == hipSuccess ? BT_OK : BT_ERR_HIP; }

bt_status check_common(uint64_t n, bt_dtype dt, const void *d_ws, size_t ws_bytes) {
    if (elem_size(dt) == 0) return BT_ERR_DTYPE;
    if (n > BT_MAX_ELEMENTS) return BT_ERR_SIZE;
    if (n == 0) return BT_OK;
    if (d_ws == nullptr) return BT_ERR_NULL;
    if (misaligned(d_ws, 8)) return BT_ERR_ALIGN;
    if (ws_bytes < bt_workspace_bytes(n, dt)) return BT_ERR_WORKSPACE;
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

size_t bt_workspace_bytes(uint64_t n, bt_dtype dtype) {
    const int s = elem_size(dtype);
    if (s == 0) return 0;
    uint64_t tiles = tiles_for(n, s);
    if (tiles == 0) tiles = 1;
    return kHeaderBytes + (size_t)tiles * sizeof(uint64_t);
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
    }
    return "unknown status";
}

bt_status bt_workspace_init(void *d_workspace, size_t workspace_bytes, bt_stream stream) {
    if (d_workspace == nullptr) return BT_ERR_NULL;
    if (misaligned(d_workspace, 8)) return BT_ERR_ALIGN;
    const uint64_t count = workspace_bytes / 8;
    if (count == 0) return BT_OK;
    const unsigned blocks = (unsigned)((count + 255) / 256);
    fill_u64_kernel<<<dim3(blocks), dim3(256), 0, (hipStream_t)stream>>>((uint64_t *)d_workspace, count, 0);
    return launched();
}

bt_status bt_compress(const void *d_in, uint64_t n, bt_dtype dtype, uint32_t *d_bitmap, void *d_values,
                      uint64_t values_cap, uint64_t *d_nnz, void *d_workspace, size_t workspace_bytes,
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
    uint32_t *hdr = static_cast<uint32_t *>(d_workspace);
    uint64_t *desc = reinterpret_cast<uint64_t *>(static_cast<char *>(d_workspace) + kHeaderBytes);
    const uint32_t desc_cap = (uint32_t)((workspace_bytes - kHeaderBytes) / 8);
    if (s == 4)
        compress_kernel<4><<<dim3(n_tiles), dim3(kBlock), 0, hs>>>(d_in, n, d_bitmap, d_values, values_cap, d_nnz, hdr,
                                                                   desc, n_tiles, desc_cap);
    else
        compress_kernel<2><<<dim3(n_tiles), dim3(kBlock), 0, hs>>>(d_in, n, d_bitmap, d_values, values_cap, d_nnz, hdr,
                                                                   desc, n_tiles, desc_cap);
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
    uint32_t *hdr = static_cast<uint32_t *>(d_workspace);
    uint64_t *desc = reinterpret_cast<uint64_t *>(static_cast<char *>(d_workspace) + kHeaderBytes);
    const uint32_t desc_cap = (uint32_t)((workspace_bytes - kHeaderBytes) / 8);
    if (s == 4)
        decompress_kernel<4><<<dim3(n_tiles), dim3(kBlock), 0, hs>>>(d_bitmap, d_values, n, d_out, hdr, desc, n_tiles,
                                                                     desc_cap);
    else
        decompress_kernel<2><<<dim3(n_tiles), dim3(kBlock), 0, hs>>>(d_bitmap, d_values, n, d_out, hdr, desc, n_tiles,
                                                                     desc_cap);
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
    const uint32_t n_tiles = (uint32_t)tiles_for(n, s);
    if (s == 4)
        relu_backward_kernel<4><<<dim3(n_tiles), dim3(kBlock), 0, hs>>>(d_bitmap, d_grad_out, n, d_grad_in);
    else
        relu_backward_kernel<2><<<dim3(n_tiles), dim3(kBlock), 0, hs>>>(d_bitmap, d_grad_out, n, d_grad_in);
    return launched();
}

}  // extern "C"
