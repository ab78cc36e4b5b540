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

// What sparse writes cost a saturated read stream: the same readers, and beside them writer wavefronts that
// each put `n_chunks` chunks of 4 KiB into `out`, one every `pause` naps of about two microseconds, as whole
// 1 KiB store instructions.  MODE 0: plain stores to fresh lines, 1: non-temporal, 2: write-through (sc1),
// 3: plain stores that all go to the writer's first chunk (which stays in the cache).
template <int MODE>
__global__ __launch_bounds__(64) void read_beside_writers_kernel(const u32x4* buf, const uint32_t* table, int n_readers,
                                                                 int blocks_per_wave, u32x4* out, uint64_t out_chunks,
                                                                 int n_chunks, int pause, uint32_t* sink) {
    if ((int)blockIdx.x >= n_readers) {
        const uint64_t w = blockIdx.x - n_readers;
        const u32x4 val = {1u, 2u, 3u, (uint32_t)w};
        for (int i = 0; i < n_chunks; ++i) {
            const uint64_t chunk = w * n_chunks + (MODE == 3 ? 0 : i);
            if (chunk >= out_chunks) return;                   // (the host has checked this as well)
            u32x4* o = out + chunk * 256 + threadIdx.x;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                u32x4* p = o + j * 64;
                if (MODE == 0 || MODE == 3) *p = val;
                if (MODE == 1) __builtin_nontemporal_store(val, p);
                if (MODE == 2) asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(val) : "memory");
            }
            for (int s = 0; s < pause; ++s) __builtin_amdgcn_s_sleep(64);
        }
        return;
    }
    const uint32_t* t = table + (size_t)blockIdx.x * blocks_per_wave;
    u32x4 acc = {0, 0, 0, 0};
    for (int b = 0; b + 4 <= blocks_per_wave; b += 4) {
        u32x4 v[16];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const u32x4* q = buf + (size_t)t[b + k] * 256 + threadIdx.x;
#pragma unroll
            for (int j = 0; j < 4; ++j) v[k * 4 + j] = __builtin_nontemporal_load(q + j * 64);
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) acc ^= v[k];
    }
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

// The readers of spin_probe_read_blocks (non-temporal loads) with n_writers writer wavefronts beside them:
// writer w puts chunks [w * n_chunks, (w+1) * n_chunks) of 4 KiB into out_dev (out_bytes of device memory;
// refused unless n_writers * n_chunks * 4096 <= out_bytes), one every `pause` naps.  mode: 0 plain stores,
// 1 non-temporal, 2 write-through, 3 plain stores to one chunk per writer.  Returns a hipError_t value.
extern "C" int spin_probe_read_beside_writers(const void* buf_dev, const uint32_t* table_dev, int32_t n_readers,
                                              int32_t blocks_per_wave, void* out_dev, uint64_t out_bytes, int32_t n_writers,
                                              int32_t n_chunks, int32_t pause, int32_t mode, uint32_t* sink_dev, void* hip_stream) {
    if (!buf_dev || !table_dev || !sink_dev || !out_dev || n_readers < 1 || blocks_per_wave < 4 || blocks_per_wave % 4 ||
        n_writers < 0 || n_chunks < 0 || pause < 0 || mode < 0 || mode > 3 ||
        (uint64_t)n_writers * (uint64_t)n_chunks * 4096 > out_bytes)
        return (int)hipErrorInvalidValue;
    hipStream_t s = (hipStream_t)hip_stream;
    const dim3 grid((unsigned)(n_readers + n_writers)), block(64);
    const uint64_t out_chunks = out_bytes / 4096;
#define SPIN_PROBE_LAUNCH(M)                                                                                            \
    hipLaunchKernelGGL(read_beside_writers_kernel<M>, grid, block, 0, s, (const u32x4*)buf_dev, table_dev, n_readers,    \
                       blocks_per_wave, (u32x4*)out_dev, out_chunks, n_chunks, pause, sink_dev)
    if (mode == 0) SPIN_PROBE_LAUNCH(0);
    else if (mode == 1) SPIN_PROBE_LAUNCH(1);
    else if (mode == 2) SPIN_PROBE_LAUNCH(2);
    else SPIN_PROBE_LAUNCH(3);
#undef SPIN_PROBE_LAUNCH
    return (int)hipGetLastError();
}
