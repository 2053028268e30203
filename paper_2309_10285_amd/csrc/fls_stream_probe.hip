// Measurement code, not part of the library's C ABI: a plain streaming read of a buffer, the
// empirical ceiling that bench.py states beside the SpMM kernel's achieved bandwidth (the kernel is
// bound by the HBM stream of its compressed words, the paper's Sec. 3.2 / Sec. 6.2.1 argument).
//
// The read is shaped like the SpMM kernel's: persistent workgroups of eight waves, every wave walks
// a contiguous run of the buffer with 16 B non-temporal buffer loads, two chunks of `U` of them in flight per
// lane; no LDS, no MFMA, nothing stored (the words are folded into one register that is written
// only if it has a value it cannot have).  Built into libfls_probe.so.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kBufferFlags = 0x00020000;
constexpr int kAuxNonTemporal = 2;
constexpr int kWaves = 8;

template <int U>
__global__ __launch_bounds__(kWaves * 64) void stream_read_kernel(const unsigned char* buf, uint64_t bytes, uint32_t* sink) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint64_t g = (uint64_t)blockIdx.x * kWaves + (threadIdx.x >> 6), G = (uint64_t)gridDim.x * kWaves;
  // the run of this wave, in chunks of U KB (the tail of the buffer that fills no chunk is left out)
  const uint64_t chunks = bytes / (U * 1024u);
  const uint64_t c0 = g * chunks / G, c1 = (g + 1) * chunks / G;
  u32x4 fold = {0u, 0u, 0u, 0u};
  // two chunks in flight, straight-line in the loads (a chunk past the run gets an empty descriptor and
  // moves no data), so that the waits are exact counts and the stream never drains inside the loop
  auto load = [&](u32x4(&v)[U], uint64_t c) {
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(buf + c * (U * 1024u)), 0, c < c1 ? U * 1024 : 0, kBufferFlags);
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (u * 64 + lane) * 16, 0, kAuxNonTemporal);
  };
  u32x4 a[U], b[U];
  load(a, c0);
  for (uint64_t c = c0; c < c1; c += 2) {
    load(b, c + 1);
#pragma unroll
    for (int u = 0; u < U; ++u) fold |= a[u];
    load(a, c + 2);
#pragma unroll
    for (int u = 0; u < U; ++u) fold |= b[u];
  }
  // NonZeros words never have all bits set in all four lanes' words at once
  if ((fold[0] & fold[1] & fold[2] & fold[3]) == 0xffffffffu && bytes == 1) sink[0] = fold[0];
}

}  // namespace

extern "C" {

// Enqueues one streaming read of buf[0, bytes) on `stream` with `grid` workgroups and `unroll`
// (4, 8 or 16; twice that many loads of 16 B are in flight per lane).  Returns 0, or -1 for bad arguments / a failed launch.
int fls_probe_stream_read(const void* buf_dev, uint64_t bytes, int grid, int unroll, void* sink_dev, void* stream) {
  if (!buf_dev || !sink_dev || grid < 1 || grid > 4096 || ((uintptr_t)buf_dev & 15u)) return -1;
  hipStream_t s = (hipStream_t)stream;
  const unsigned char* b = (const unsigned char*)buf_dev;
  uint32_t* k = (uint32_t*)sink_dev;
  switch (unroll) {
    case 4: hipLaunchKernelGGL(stream_read_kernel<4>, dim3(grid), dim3(kWaves * 64), 0, s, b, bytes, k); break;
    case 8: hipLaunchKernelGGL(stream_read_kernel<8>, dim3(grid), dim3(kWaves * 64), 0, s, b, bytes, k); break;
    case 16: hipLaunchKernelGGL(stream_read_kernel<16>, dim3(grid), dim3(kWaves * 64), 0, s, b, bytes, k); break;
    default: return -1;
  }
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // extern "C"
