// libbittrain_bench.so: the codec compiled with per-tile time stamps, plus a dependency-free
// stream with the codec's traffic shape.  Measurement aids for bench.py; see bench_aids.h.
#define BT_TIMELINE 1
#include "bittrain.hip"
#include "bench_aids.h"

namespace {

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

}  // namespace

extern "C" {

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
    if (d_buf == nullptr) tiles = max_passes = 0;
    else if (misaligned(d_buf, 8)) return BT_ERR_ALIGN;
    if (8 * (uint64_t)tiles + 2 * (uint64_t)max_passes > buf_words) return BT_ERR_SIZE;
    // blocking copies: this call is the one place where the library waits for the device
    if (hipMemcpyToSymbol(HIP_SYMBOL(g_timeline_tiles), &tiles, sizeof(tiles)) != hipSuccess ||
        hipMemcpyToSymbol(HIP_SYMBOL(g_timeline_passes), &max_passes, sizeof(max_passes)) != hipSuccess ||
        hipMemcpyToSymbol(HIP_SYMBOL(g_timeline), &d_buf, sizeof(d_buf)) != hipSuccess)
        return BT_ERR_HIP;
    return BT_OK;
}

}  // extern "C"
