// fls_compress: dense masked W -> Tiled-CSL blob on the GPU (the paper's offline weight
// reformatting step, Sec. 5; format Sec. 4.3.1-4.3.2; tile walk of Alg. 3).
//
// Three kernels, all integer work on fp16 bit patterns (no value passes through a float op):
//   count : one wave per tile counts the non-zero bit patterns and leaves the count in the
//           tile's TileOffsets entry
//   scan  : one workgroup turns the counts into padded run lengths and their exclusive prefix
//           sums, fills the guard entries, and writes the header (nnz, longest run included)
//   emit  : one wave per tile walks the tile in location order; per step every lane holds the 8
//           halves of one (row, K-chunk) cell, a wave prefix sum of the per-lane counts gives each
//           lane its slot in the run (ordered compaction)
#include "fls_device.h"
#include "fls_launch.h"

namespace fls {

constexpr uint32_t kMagic = 0x31534C46u;  // "FLS1"
constexpr uint32_t kPad = 4;

struct CompressParams {
  const uint16_t* W;
  unsigned char* out;
  uint32_t M, K, KT, T, n_off, policy;
};

__device__ __forceinline__ uint32_t* offs_of(const CompressParams& p) { return (uint32_t*)(p.out + 64); }
__device__ __forceinline__ uint32_t* words_of(const CompressParams& p) { return (uint32_t*)(p.out + 64 + 4 * (size_t)p.n_off); }

__device__ __forceinline__ uint32_t nonzero_mask(const u32x4& v) {
  uint32_t m = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    m |= ((v[i] & 0xffffu) != 0u ? 1u : 0u) << (2 * i);
    m |= ((v[i] >> 16) != 0u ? 1u : 0u) << (2 * i + 1);
  }
  return m;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t up = __shfl_up(v, d, 64);
    if (lane >= d) v += up;
  }
  return v;
}

__global__ __launch_bounds__(256) void compress_count_kernel(CompressParams p) {
  const int lane = threadIdx.x & 63;
  const uint32_t t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= p.T) return;
  const uint32_t band = t / p.KT, kt = t - band * p.KT;
  // lane covers rows (lane >> 2) + 16*i, K chunk (lane & 3): 16 rows x 64 B per step
  const uint16_t* src = p.W + ((size_t)band * kTileM + (lane >> 2)) * p.K + kt * kTileK + (lane & 3) * 8;
  uint32_t cnt = 0;
#pragma unroll
  for (int i = 0; i < kTileM / 16; ++i) {
    const u32x4 v = *(const u32x4*)(src + (size_t)i * 16 * p.K);
    cnt += __popc(nonzero_mask(v));
  }
  cnt = wave_sum(cnt);
  if (lane == 0) offs_of(p)[t] = cnt;
}

__device__ __forceinline__ uint32_t padded(uint32_t cnt) { return (cnt + kPad - 1) / kPad * kPad; }

// single workgroup of 1024 threads
__global__ __launch_bounds__(1024) void compress_scan_kernel(CompressParams p) {
  __shared__ unsigned long long part[1024];
  __shared__ unsigned long long nnz_total;
  __shared__ uint32_t longest;
  uint32_t* offs = offs_of(p);
  const uint32_t tid = threadIdx.x;
  const uint32_t per = (p.T + 1023) / 1024;
  const uint32_t a = tid * per < p.T ? tid * per : p.T, b = (tid + 1) * per < p.T ? (tid + 1) * per : p.T;
  if (tid == 0) {
    nnz_total = 0;
    longest = 0;
  }
  __syncthreads();
  unsigned long long s = 0, nnz = 0;
  uint32_t mx = 0;
  for (uint32_t i = a; i < b; ++i) {
    const uint32_t cnt = offs[i], w = padded(cnt);
    nnz += cnt;
    s += w;
    mx = w > mx ? w : mx;
  }
  part[tid] = s;
  atomicAdd(&nnz_total, nnz);  // 1024 LDS atomics in all
  atomicMax(&longest, mx);
  __syncthreads();
  // Hillis-Steele inclusive scan over the 1024 partial sums
  for (uint32_t d = 1; d < 1024; d <<= 1) {
    unsigned long long v = tid >= d ? part[tid - d] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  unsigned long long run = tid ? part[tid - 1] : 0;
  const unsigned long long total = part[1023];
  for (uint32_t i = a; i < b; ++i) {
    const uint32_t w = padded(offs[i]);
    offs[i] = (uint32_t)run;
    run += w;
  }
  for (uint32_t i = p.T + tid; i < p.n_off; i += 1024) offs[i] = (uint32_t)total;
  if (tid == 0) {
    uint32_t* h = (uint32_t*)p.out;
    h[0] = kMagic;
    h[1] = 1u;
    h[2] = kTileM;
    h[3] = kTileK;
    h[4] = kPad;
    h[5] = p.policy;
    h[6] = longest;
    h[7] = 0u;
    unsigned long long* q = (unsigned long long*)(p.out + 32);
    q[0] = p.M;
    q[1] = p.K;
    q[2] = nnz_total;
    q[3] = total;
  }
}

__global__ __launch_bounds__(256) void compress_emit_kernel(CompressParams p) {
  const int lane = threadIdx.x & 63;
  const uint32_t t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= p.T) return;
  const uint32_t band = t / p.KT, kt = t - band * p.KT;
  const uint32_t* offs = offs_of(p);
  uint32_t* dst = words_of(p) + offs[t];
  const uint32_t run_words = offs[t + 1] - offs[t];
  uint32_t pos = 0;
  // location order: K chunk, then row, then position in the chunk
  for (uint32_t c = 0; c < kTileK / 8; ++c) {
    for (uint32_t half = 0; half < kTileM / 64; ++half) {
      const uint32_t row = half * 64 + lane;
      const u32x4 v = *(const u32x4*)(p.W + ((size_t)band * kTileM + row) * p.K + kt * kTileK + c * 8);
      const uint32_t mask = nonzero_mask(v);
      const uint32_t cnt = __popc(mask);
      const uint32_t incl = wave_inclusive_scan(cnt, lane);
      uint32_t slot = pos + incl - cnt;
      const uint32_t loc0 = c * (kTileM * 8) + row * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (mask >> e & 1u) {
          const uint32_t bits = (e & 1) ? (v[e >> 1] >> 16) : (v[e >> 1] & 0xffffu);
          dst[slot++] = (bits << 16) | (loc0 + e);
        }
      }
      pos += __shfl(incl, 63, 64);
    }
  }
  // padding words: value +0, location one past the tile
  if (pos + lane < run_words) dst[pos + lane] = (uint32_t)kTileElems;
}

__global__ void fill_zero_kernel(u32x4* p, size_t n16) {
  const u32x4 z = {0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) p[i] = z;
}

hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t stream) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (u32x4*)ptr, n16);
  return hipGetLastError();
}

// ---------------------------------------------------------------- format version 2
//
// Three bytes per entry (the index bytes that the footnote under the paper's Eq. 2 leaves out of
// its model are what version 1 pays in full): a tile's entries, in ascending location, go in
// groups of four that take three words - two of values, one with the first entry's location in
// 12 bits and the other three as 6-bit distances from the entry before.  An entry is a stored
// element, a bridge (value 0) every 63 locations where the next stored element lies more than 63
// behind the entry before it, or padding (value 0, distance 1) up to a multiple of four.  Same
// three kernels: count (entries per tile, bridges included; stored elements summed into the
// header), scan, emit.

constexpr uint32_t kMagic2 = 0x32534C46u;  // "FLS2"
constexpr uint32_t kGroup = 4;              // entries per group of three words

// inclusive running maximum over the 64 lanes
__device__ __forceinline__ uint32_t wave_inclusive_max(uint32_t v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t up = __shfl_up(v, d, 64);
    if (lane >= d) v = up > v ? up : v;
  }
  return v;
}

// One wave walks tile (band, kt) in location order, as compress_emit_kernel does: per step a lane
// holds the 8 halves of one (row, K-chunk) cell, i.e. 8 consecutive locations.  Returns the number
// of entries before padding; *stored = stored elements seen by this lane.  With EMIT the entries
// (and the padding) are put together in `stage`, the tile's words in LDS, zeroed by the caller:
// entry e is entry e & 3 of group e >> 2, whose three words different lanes fill, so values and
// location fields are OR-ed in.
constexpr uint32_t kReach2 = 63;  // largest distance a 6-bit field holds: a bridge entry every 63 empty locations
template <bool EMIT>
__device__ __forceinline__ uint32_t walk_tile_v2(const CompressParams& p, uint32_t band, uint32_t kt, int lane,
                                                 uint32_t* stage, uint32_t* stored) {
  auto put = [&](uint32_t e, uint32_t bits, uint32_t loc, uint32_t dist) {
    const uint32_t g = e >> 2, k = e & 3u;
    atomicOr(&stage[g * 3u + (k >> 1)], (k & 1u) ? bits << 16 : bits);
    atomicOr(&stage[g * 3u + 2u], k == 0 ? loc : dist << (6u + 6u * k));  // the group's first location in full, then distances
  };
  uint32_t pos = 0;      // entries so far
  uint32_t counter = 0;  // the location of the last entry of the steps done so far (0 before the first)
  uint32_t nz = 0;
  for (uint32_t c = 0; c < kTileK / 8; ++c) {
    for (uint32_t half = 0; half < kTileM / 64; ++half) {
      const uint32_t row = half * 64 + lane;
      const u32x4 v = *(const u32x4*)(p.W + ((size_t)band * kTileM + row) * p.K + kt * kTileK + c * 8);
      const uint32_t mask = nonzero_mask(v);
      const uint32_t cnt = __popc(mask);
      const uint32_t loc0 = c * (kTileM * 8) + row * 8;
      // the entry this lane's first element follows: the last stored location in the lanes
      // before it (0 stands for "none", which is also what the first element of a tile follows)
      const uint32_t last = cnt ? loc0 + (31u - (uint32_t)__clz((int)mask)) : 0u;
      const uint32_t run_max = wave_inclusive_max(last, lane);
      uint32_t prev = __shfl_up(run_max, 1, 64);
      if (lane == 0) prev = 0;
      prev = prev > counter ? prev : counter;
      const uint32_t first = loc0 + (uint32_t)__builtin_ctz(mask | 0x100u);
      const uint32_t gap = first - prev;
      const uint32_t bridges = (cnt && gap > 0u) ? (gap - 1u) / kReach2 : 0u;
      const uint32_t entries = cnt + bridges;
      const uint32_t incl = wave_inclusive_scan(entries, lane);
      if (EMIT) {
        uint32_t slot = pos + incl - entries, cur = prev;
        for (uint32_t b = 0; b < bridges; ++b) {
          cur += kReach2;
          put(slot++, 0u, cur, kReach2);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (mask >> e & 1u) {
            const uint32_t bits = (e & 1) ? (v[e >> 1] >> 16) : (v[e >> 1] & 0xffffu);
            put(slot++, bits, loc0 + e, loc0 + e - cur);
            cur = loc0 + e;
          }
        }
      }
      pos += __shfl(incl, 63, 64);
      const uint32_t step_max = __shfl(run_max, 63, 64);
      counter = step_max > counter ? step_max : counter;
      nz += cnt;
    }
  }
  if (EMIT) {
    // padding never starts a group, so only its distance (1) goes in
    const uint32_t padded_entries = (pos + kGroup - 1) / kGroup * kGroup;
    if (pos + lane < padded_entries) put(pos + lane, 0u, 0u, 1u);
  }
  *stored = nz;
  return pos;
}

__global__ __launch_bounds__(256) void compress2_count_kernel(CompressParams p) {
  const int lane = threadIdx.x & 63;
  const uint32_t t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= p.T) return;
  uint32_t nz;
  const uint32_t entries = walk_tile_v2<false>(p, t / p.KT, t % p.KT, lane, nullptr, &nz);
  nz = wave_sum(nz);
  if (lane == 0) {
    offs_of(p)[t] = entries;
    atomicAdd((unsigned long long*)(p.out + 48), (unsigned long long)nz);  // the header's nnz (cleared before the launch)
  }
}

__device__ __forceinline__ uint32_t words_v2(uint32_t entries) { return (entries + kGroup - 1) / kGroup * 3u; }

// single workgroup of 1024 threads: entries per tile -> word offsets, guard entries, header
__global__ __launch_bounds__(1024) void compress2_scan_kernel(CompressParams p) {
  __shared__ unsigned long long part[1024];
  __shared__ uint32_t longest;
  uint32_t* offs = offs_of(p);
  const uint32_t tid = threadIdx.x;
  const uint32_t per = (p.T + 1023) / 1024;
  const uint32_t a = tid * per < p.T ? tid * per : p.T, b = (tid + 1) * per < p.T ? (tid + 1) * per : p.T;
  if (tid == 0) longest = 0;
  __syncthreads();
  unsigned long long s = 0;
  uint32_t mx = 0;
  for (uint32_t i = a; i < b; ++i) {
    const uint32_t w = words_v2(offs[i]);
    s += w;
    mx = w > mx ? w : mx;
  }
  part[tid] = s;
  atomicMax(&longest, mx);
  __syncthreads();
  for (uint32_t d = 1; d < 1024; d <<= 1) {
    unsigned long long v = tid >= d ? part[tid - d] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  unsigned long long run = tid ? part[tid - 1] : 0;
  const unsigned long long total = part[1023];
  for (uint32_t i = a; i < b; ++i) {
    const uint32_t w = words_v2(offs[i]);
    offs[i] = (uint32_t)run;
    run += w;
  }
  for (uint32_t i = p.T + tid; i < p.n_off; i += 1024) offs[i] = (uint32_t)total;
  if (tid == 0) {
    uint32_t* h = (uint32_t*)p.out;
    h[0] = kMagic2;
    h[1] = 2u;
    h[2] = kTileM;
    h[3] = kTileK;
    h[4] = kGroup;
    h[5] = 0u;
    h[6] = longest;
    h[7] = 0u;
    unsigned long long* q = (unsigned long long*)(p.out + 32);
    q[0] = p.M;
    q[1] = p.K;  // q[2], the stored elements, was summed by the count kernel
    q[3] = total;
  }
}

// A wave per tile: the tile's words are put together in LDS (at most 1024 groups of 12 B) and copied out.
__global__ __launch_bounds__(256) void compress2_emit_kernel(CompressParams p) {
  __shared__ uint32_t stages[4][kTileM * kTileK / kGroup * 3];
  const int lane = threadIdx.x & 63;
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t t = blockIdx.x * 4 + wave;
  if (t >= p.T) return;
  uint32_t* stage = stages[wave];
  const uint32_t begin = offs_of(p)[t], nwords = offs_of(p)[t + 1] - begin;
  for (uint32_t i = lane; i < nwords; i += 64) stage[i] = 0u;
  __builtin_amdgcn_wave_barrier();  // (LDS executes a wave's operations in order; this keeps the compiler from moving them)
  uint32_t nz;
  walk_tile_v2<true>(p, t / p.KT, t % p.KT, lane, stage, &nz);
  __builtin_amdgcn_wave_barrier();
  uint32_t* dst = words_of(p) + begin;
  for (uint32_t i = lane; i < nwords; i += 64) dst[i] = stage[i];
}

static CompressParams make_params(const CompressLaunch& a) {
  CompressParams p;
  p.W = a.W;
  p.out = a.out;
  p.M = a.M;
  p.K = a.K;
  p.KT = a.K / kTileK;
  p.T = (a.M / kTileM) * p.KT;
  p.n_off = (p.T + 4 + 15) / 16 * 16;
  p.policy = a.policy;
  return p;
}

hipError_t launch_compress_index(const CompressLaunch& a, hipStream_t stream) {
  const CompressParams p = make_params(a);
  hipError_t e = launch_fill_zero(a.out, 64, stream);
  if (e != hipSuccess) return e;
  if (a.version == 2) hipLaunchKernelGGL(compress2_count_kernel, dim3((p.T + 3) / 4), dim3(256), 0, stream, p);
  else hipLaunchKernelGGL(compress_count_kernel, dim3((p.T + 3) / 4), dim3(256), 0, stream, p);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (a.version == 2) hipLaunchKernelGGL(compress2_scan_kernel, dim3(1), dim3(1024), 0, stream, p);
  else hipLaunchKernelGGL(compress_scan_kernel, dim3(1), dim3(1024), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_compress_emit(const CompressLaunch& a, hipStream_t stream) {
  const CompressParams p = make_params(a);
  if (a.version == 2) hipLaunchKernelGGL(compress2_emit_kernel, dim3((p.T + 3) / 4), dim3(256), 0, stream, p);
  else hipLaunchKernelGGL(compress_emit_kernel, dim3((p.T + 3) / 4), dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace fls
