// Streaming-read probe for gfx950: what a kernel that does nothing but read reaches on this machine,
// the figure the attention kernels' achieved bandwidth is set against next to the published 8 TB/s.
// Built into libspin_probe.so, a measurement aid loaded by bench.py --calib-stream only; it is not
// part of the verification library and exports nothing of the method.
//
// One wavefront per workgroup walks a list of 4 KiB blocks (the size of one page-head of the K/V
// cache at head dim 128 and 16 tokens per page) given by a table of block numbers -- in order, or
// shuffled like a fragmented paged cache -- with non-temporal 16-byte loads, 16 per lane in flight
// (four blocks), which is how the single-wavefront attention kernel loads.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace {

template <bool NT>
__global__ __launch_bounds__(64) void read_blocks_kernel(const u32x4* buf, const uint32_t* table, int blocks_per_wave,
                                                         uint32_t* sink) {
    const uint32_t* t = table + (size_t)blockIdx.x * blocks_per_wave;
    u32x4 acc = {0, 0, 0, 0};
    for (int b = 0; b + 4 <= blocks_per_wave; b += 4) {
        u32x4 v[16];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const u32x4* q = buf + (size_t)t[b + k] * 256 + threadIdx.x;
#pragma unroll
            for (int j = 0; j < 4; ++j) v[k * 4 + j] = NT ? __builtin_nontemporal_load(q + j * 64) : q[j * 64];
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) acc ^= v[k];
    }
    // (never true for the buffers the benchmark fills; keeps the loads alive)
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[0] = 1;
}

}  // namespace

// Read n_waves * blocks_per_wave blocks of 4 KiB from buf_dev, wavefront w taking entries
// [w * blocks_per_wave, (w+1) * blocks_per_wave) of table_dev (block numbers, device uint32).
// blocks_per_wave must be a multiple of 4.  Asynchronous on the stream; returns a hipError_t value.
extern "C" int spin_probe_read_blocks(const void* buf_dev, const uint32_t* table_dev, int32_t n_waves,
                                      int32_t blocks_per_wave, int32_t nontemporal, uint32_t* sink_dev, void* hip_stream) {
    if (!buf_dev || !table_dev || !sink_dev || n_waves < 1 || blocks_per_wave < 4 || blocks_per_wave % 4) return (int)hipErrorInvalidValue;
    hipStream_t s = (hipStream_t)hip_stream;
    if (nontemporal)
        hipLaunchKernelGGL(read_blocks_kernel<true>, dim3((unsigned)n_waves), dim3(64), 0, s, (const u32x4*)buf_dev, table_dev, blocks_per_wave, sink_dev);
    else
        hipLaunchKernelGGL(read_blocks_kernel<false>, dim3((unsigned)n_waves), dim3(64), 0, s, (const u32x4*)buf_dev, table_dev, blocks_per_wave, sink_dev);
    return (int)hipGetLastError();
}
