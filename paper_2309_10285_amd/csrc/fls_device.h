// Device-side building blocks shared by the sparse and the dense kernel: MFMA operand types,
// the split-K hand-over of partial bands.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fls {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTileM = 128;               // rows of a tile (one row band)
constexpr int kTileK = 32;                // K extent of a tile = K of one 16x16x32 MFMA
constexpr int kTileElems = kTileM * kTileK;
constexpr int kTileBytes = kTileElems * 2;  // dense fp16 tile in LDS
constexpr int kRowBlocks = kTileM / 16;     // 16-row MFMA blocks per tile

constexpr int kHeaderWords = 16;            // the blob's 64-byte header, in 32-bit words; TileOffsets follow it
constexpr int kHeaderMaxTileWords = 6;      // header word that holds the length of the longest tile
constexpr int kHeaderTotalWords = 14;       // header word that holds the number of words in NonZeros (low half of a u64)

constexpr int kAccPerBlock = kTileM * 16;   // fp32 values of one 128 x 16 column block
constexpr int kMaxGrid = 512;               // workgroups a launch may use (sizes the workspace)
constexpr int kBufferFlags = 0x00020000;    // raw buffer, 32-bit data format (gfx9 descriptor word 3)
constexpr int kAuxNonTemporal = 2;          // nt: streamed once, do not keep in the caches
constexpr int kAuxCoherent = 16;            // sc1: device scope - through to memory / past the per-XCD L2

// LDS byte address a word of a tile goes to: base + 2 * location (the word's low half), in one
// instruction (v_mad_u32_u16: D = S0.u16 * S1.u16 + S2.u32).
__device__ __forceinline__ uint32_t scatter_addr(uint32_t word, uint32_t base) {
  uint32_t addr;
  asm("v_mad_u32_u16 %0, %1, 2, %2" : "=v"(addr) : "v"(word), "v"(base));
  return addr;
}

// What both kernels need to hand results over.
//
// Split-K: the band-major tile sequence [0, T) is cut evenly over the workgroups, then over the
// waves of a workgroup.  Partial results of one band meet in two steps:
//   1. inside a workgroup, in LDS (wg_reduce): waves add their accumulators to one of two band
//      slots and count their tiles; the wave that completes the workgroup's share takes the sum;
//   2. between workgroups, in HBM: that wave stores the sum to its workgroup's slot and later
//      raises the workgroup's flag; the workgroup that owns the band adds up the slots in
//      workgroup order and writes fp16 C (see "between workgroups" below).
// No floating-point atomics touch HBM.
struct OutParams {
  _Float16* C;      // column-major M x N
  float* parts;     // [workgroup][NB * 2048] fp32 partial sums in accumulator order
  uint32_t* flags;  // [workgroup] 1 while a published partial sum waits for its band's owner; [kMaxGrid] error word
  uint32_t M, N;    // N = columns of the whole problem
  uint32_t n0;      // first column of this launch's column group
  uint32_t KT;      // K tiles per band
  uint32_t T;       // tiles in total
};

// First tile of workgroup q's share when T tiles are cut over P workgroups.
__device__ __forceinline__ uint32_t share_begin(uint32_t q, uint32_t T, uint32_t P) {
  return (uint32_t)((uint64_t)q * T / P);
}

// MFMA 16x16 accumulator layout: lane l holds column (l & 15), rows 4*(l >> 4) .. +3 of its block.
// Converts a wave's 128 x (NB*16) accumulators to fp16 and stores them to column-major C.
template <int NB>
__device__ __forceinline__ void store_band(const OutParams& o, const float4v (&acc)[kRowBlocks][NB], uint32_t band,
                                           int lane) {
  const uint32_t col = lane & 15, rsub = (lane >> 4) * 4;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const uint32_t n = o.n0 + nb * 16 + col;
    if (n < o.N) {
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb) {
        half4 h;
#pragma unroll
        for (int r = 0; r < 4; ++r) h[r] = (_Float16)acc[rb][nb][r];
        *(half4*)(o.C + (size_t)n * o.M + band * kTileM + rb * 16 + rsub) = h;
      }
    }
  }
}

// LDS area of the in-workgroup step: band slots and their control words.  A slot keeps a band's
// running sum as [column block][row block][lane] float4.  Consecutive bands of a workgroup's
// share alternate between two slots, so that waves already in the next band need not wait for
// the previous one to be collected.
template <int NB>
struct WgReduceLds {
  static constexpr uint32_t kSlots = 2;
  static constexpr int kParts = 4;  // a slot is added to in four parts, each under its own lock
  float4v slot[kSlots][NB * kRowBlocks * 64];
  uint32_t cnt[kSlots];           // tiles added to the slot so far
  uint32_t gen[kSlots];           // how many bands the slot has served
  uint32_t lock[kSlots][kParts];  // 1 while a wave is adding to that part of the slot
};

template <int NB>
__device__ __forceinline__ void wg_reduce_init(WgReduceLds<NB>* red, int tid, int nthreads) {
  for (int i = tid; i < (int)WgReduceLds<NB>::kSlots * NB * kRowBlocks * 64; i += nthreads) (&red->slot[0][0])[i] = float4v{0.f, 0.f, 0.f, 0.f};
  if (tid < (int)WgReduceLds<NB>::kSlots) {
    red->cnt[tid] = 0;
    red->gen[tid] = 0;
#pragma unroll
    for (int part = 0; part < WgReduceLds<NB>::kParts; ++part) red->lock[tid][part] = 0;
  }
}

// Adds a wave's accumulators for the seq-th band of its workgroup (seq counts from the
// workgroup's first band) to the band's slot.  Returns true for exactly one wave per band: the
// one whose tiles complete `expected`; the slot then holds the workgroup's sum (wg_reduce_take
// collects it).  Waves add with plain 16 B read-add-write under spin locks, one per quarter of
// the slot, all taking the quarters in the same order: waves that arrive together follow each
// other through the slot like an assembly line instead of waiting for the whole of it.  (LDS
// floating-point atomics would need no lock but run about fifty times slower per instruction
// on this chip than a plain LDS access.)
template <int NB>
__device__ __forceinline__ bool wg_reduce_add(WgReduceLds<NB>* red, const float4v (&acc)[kRowBlocks][NB], uint32_t seq,
                                              uint32_t tiles, uint32_t expected, int lane) {
  const uint32_t s = seq % WgReduceLds<NB>::kSlots, turn = seq / WgReduceLds<NB>::kSlots;
  // the slot may still serve an earlier band (only when a share spans more bands than there are slots)
  while (__hip_atomic_load(&red->gen[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != turn)
    __builtin_amdgcn_s_sleep(2);
  constexpr int kParts = WgReduceLds<NB>::kParts, kPerPart = NB * kRowBlocks / kParts;
  float4v* d = &red->slot[s][lane];
#pragma unroll
  for (int part = 0; part < kParts; ++part) {
    for (;;) {
      uint32_t got = 1;
      if (lane == 0) got = __hip_atomic_exchange(&red->lock[s][part], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      if (__builtin_amdgcn_readfirstlane(got) == 0) break;
      __builtin_amdgcn_s_sleep(1);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
#pragma unroll
    for (int e = part * kPerPart; e < (part + 1) * kPerPart; ++e) d[e * 64] += acc[e % kRowBlocks][e / kRowBlocks];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    if (lane == 0) __hip_atomic_store(&red->lock[s][part], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  // counted in after the last part: the wave that completes the count finds every part added
  uint32_t old = 0;
  if (lane == 0) old = __hip_atomic_fetch_add(&red->cnt[s], tiles, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  old = __builtin_amdgcn_readfirstlane(old);
  return old + tiles == expected;
}

// Run by the wave wg_reduce_add picked: moves the slot's sum into acc and frees the slot for band seq + 2.
template <int NB>
__device__ __forceinline__ void wg_reduce_take(WgReduceLds<NB>* red, float4v (&acc)[kRowBlocks][NB], uint32_t seq,
                                               int lane) {
  const uint32_t s = seq % WgReduceLds<NB>::kSlots, turn = seq / WgReduceLds<NB>::kSlots;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  float4v* d = &red->slot[s][lane];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb) {
      acc[rb][nb] = d[(nb * kRowBlocks + rb) * 64];
      d[(nb * kRowBlocks + rb) * 64] = float4v{0.f, 0.f, 0.f, 0.f};
    }
  if (lane == 0) red->cnt[s] = 0;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  if (lane == 0) __hip_atomic_store(&red->gen[s], turn + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// A wave that saw a whole band by itself has nothing to reduce, but the band still takes its turn
// on the slot so that the turn count of later bands stays right.
template <int NB>
__device__ __forceinline__ void wg_reduce_skip(WgReduceLds<NB>* red, uint32_t seq, int lane) {
  const uint32_t s = seq % WgReduceLds<NB>::kSlots, turn = seq / WgReduceLds<NB>::kSlots;
  while (__hip_atomic_load(&red->gen[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != turn)
    __builtin_amdgcn_s_sleep(2);
  if (lane == 0) __hip_atomic_store(&red->gen[s], turn + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// ---- between workgroups
//
// A band that is cut between workgroups is finished by its owner: the workgroup whose share holds
// the band's first tile.  The owner's piece of the band is the last thing in its share, so its
// sum is still in registers when its run ends.  Every other workgroup that holds tiles of the
// band stores its sum to its slot when its piece ends (write-through stores, nothing waits for
// them) and publishes the slot when its own run ends, by raising its flag behind a device-scope
// release.  The owner then polls those flags, acquires, adds the slots in workgroup order and
// writes fp16 C.
//
// Partial sums cross between the L2 caches of different XCDs, which are not coherent with each
// other inside a kernel: the contributor releases at device scope before it raises its flag, the
// owner acquires at device scope after it has seen the flags (2 - 3 us of the kernel's tail on
// shapes that split bands; the stores and loads of the slots also carry sc1, so little is left for
// the release to write back).  A workgroup publishes at most one
// partial sum per launch (only the first band of a share can begin outside it) and exactly one
// owner waits for it; the owner lowers the flag it has seen, so all flags are down again when the
// launch ends: nothing is cleared between calls, and a launch recorded in a graph can be replayed.
//
// A workgroup publishes before it polls, and only polls workgroups of higher index, so the wait
// ends as soon as those workgroups have run; the spin is bounded all the same.
constexpr uint32_t kSpinLimit = 1u << 20;

template <int NB>
__device__ __forceinline__ void store_partial(const OutParams& o, const float4v (&acc)[kRowBlocks][NB], uint32_t wg,
                                              int lane) {
  const __amdgpu_buffer_rsrc_t mine = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(o.parts + (size_t)wg * (NB * kAccPerBlock)), 0, NB * kAccPerBlock * 4, kBufferFlags);
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb)
      __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[rb][nb]), mine,
                                             ((nb * kRowBlocks + rb) * 64 + lane) * 16, 0, kAuxCoherent);
}

// A device-scope release in two halves, so that the time the write-back takes can pass behind
// other work: release_begin right after the stores (the L2 of this XCD starts writing back what
// it holds), release_end before the flag is raised (waits for that and for every earlier store).
// Together they are the instruction sequence of a release fence at device scope.  Waiting for the
// stores alone is not enough: a store counts as done when the XCD's L2 has it, and the flag could
// reach memory before the data does (seen as a wrong band about once in a thousand calls).
__device__ __forceinline__ void release_begin() { asm volatile("buffer_wbl2 sc1" ::: "memory"); }
__device__ __forceinline__ void release_end() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// By the wave that called store_partial, once its run is over; `begun` tells whether it has called
// release_begin behind the stores already.
__device__ __forceinline__ void publish_partial(const OutParams& o, uint32_t wg, int lane, bool begun) {
  if (!begun) release_begin();
  release_end();
  if (lane == 0) __hip_atomic_store(o.flags + wg, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// acc holds the owner's own sum for `band`; adds the other workgroups' and writes C.
template <int NB>
__device__ __forceinline__ void owner_finish(const OutParams& o, float4v (&acc)[kRowBlocks][NB], uint32_t band,
                                             uint32_t wg, uint32_t P, int lane) {
  const uint32_t band_hi = (band + 1) * o.KT;
  // The flags of all contributors are polled at once, one per lane: a look at a flag is a trip to
  // memory (it lives behind another XCD's L2), and one after the other those trips would add up at the
  // very end of the kernel.
  for (uint32_t base = wg + 1; base < P && share_begin(base, o.T, P) < band_hi; base += 64) {
    const uint32_t q = base + (uint32_t)lane;
    // workgroup q holds tiles of the band (an empty share contributes nothing)
    const bool mine = q < P && share_begin(q, o.T, P) < band_hi && share_begin(q + 1, o.T, P) != share_begin(q, o.T, P);
    uint32_t spins = 0;
    bool seen = !mine;
    for (;;) {
      if (!seen) seen = __hip_atomic_load(o.flags + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
      if (__builtin_amdgcn_ballot_w64(!seen) == 0) break;
      __builtin_amdgcn_s_sleep(8);
      if (++spins == kSpinLimit) {  // never seen; gives up rather than hang, and says so
        if (lane == 0) __hip_atomic_store(o.flags + kMaxGrid, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
    }
    // workgroup q raises its flag once per launch and nobody else looks at it: down again for the next launch
    if (mine && seen) __hip_atomic_store(o.flags + q, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // What pairs with the contributors' release: the loads below are issued after the flags have been
  // seen, and each carries sc1 like the look at a flag does - a load at device scope, which nothing
  // that this CU's L1 or this XCD's L2 still holds of the slots may serve.  (An acquire fence here
  // would invalidate both caches wholesale on top of that: a microsecond at the very end of the kernel.)
  // As many loads as the registers allow are issued before the first is used: each is a trip
  // to memory, and this runs when the kernel is about to end, with nothing left to hide it behind.
  constexpr int kBatch = NB == 1 ? 4 : 2;  // slots in flight
  constexpr int kBlocks = NB > 2 ? 2 : NB;  // column blocks of a slot in flight
  uint32_t q = wg + 1;
  while (q < P && share_begin(q, o.T, P) < band_hi) {
    __amdgpu_buffer_rsrc_t src[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      // next workgroup with tiles of the band; past the last one the descriptor is empty and reads 0
      bool found = false;
      while (!found && q < P && share_begin(q, o.T, P) < band_hi) {
        found = share_begin(q + 1, o.T, P) != share_begin(q, o.T, P);
        if (!found) ++q;
      }
      src[j] = __builtin_amdgcn_make_buffer_rsrc((void*)(o.parts + (size_t)(found ? q : 0u) * (NB * kAccPerBlock)), 0,
                                                 found ? NB * kAccPerBlock * 4 : 0, kBufferFlags);
      if (found) ++q;
    }
#pragma unroll
    for (int nb0 = 0; nb0 < NB; nb0 += kBlocks) {
      u32x4 v[kBatch][kBlocks][kRowBlocks];
#pragma unroll
      for (int j = 0; j < kBatch; ++j)
#pragma unroll
        for (int nb = 0; nb < kBlocks; ++nb)
#pragma unroll
          for (int rb = 0; rb < kRowBlocks; ++rb)
            v[j][nb][rb] = __builtin_amdgcn_raw_buffer_load_b128(src[j], (((nb0 + nb) * kRowBlocks + rb) * 64 + lane) * 16, 0,
                                                                 kAuxCoherent);
#pragma unroll
      for (int j = 0; j < kBatch; ++j)
#pragma unroll
        for (int nb = 0; nb < kBlocks; ++nb)
#pragma unroll
          for (int rb = 0; rb < kRowBlocks; ++rb) acc[rb][nb0 + nb] += __builtin_bit_cast(float4v, v[j][nb][rb]);
    }
  }
  store_band<NB>(o, acc, band, lane);
}

// What a wave carries from the tile loop to the end of its run.
struct HandoverState {
  bool publish = false;  // it stored its workgroup's partial sum and still has to publish it
  bool released = false; // release_begin has been called behind those stores
  bool own = false;      // it holds the owner's sum of band own_band in its accumulators
  uint32_t own_band = 0;
};

// Hand-over of a wave's piece (tiles of one band), inside the tile loop: LDS work and, at most,
// stores that nothing waits for.  `tiles` = tiles in the piece, [share0, share1) = the
// workgroup's share.  Leaves acc cleared for the next band unless the wave became an owner.
template <int NB>
__device__ __forceinline__ void hand_over_piece(const OutParams& o, WgReduceLds<NB>* red, float4v (&acc)[kRowBlocks][NB],
                                                HandoverState& st, uint32_t band, uint32_t tiles, uint32_t share0,
                                                uint32_t share1, uint32_t wg, int lane, bool local_only,
                                                bool early_release) {
  const uint32_t seq = band - share0 / o.KT;
  if (tiles == o.KT) {
    store_band<NB>(o, acc, band, lane);  // this wave alone saw the whole band
    wg_reduce_skip<NB>(red, seq, lane);
  } else {
    const uint32_t band_lo = band * o.KT, band_hi = band_lo + o.KT;
    const uint32_t lo = share0 > band_lo ? share0 : band_lo;
    const uint32_t hi = share1 < band_hi ? share1 : band_hi;
    if (wg_reduce_add<NB>(red, acc, seq, tiles, hi - lo, lane)) {
      wg_reduce_take<NB>(red, acc, seq, lane);  // acc = the workgroup's sum over [lo, hi)
      if ((lo == band_lo && hi == band_hi) || local_only) {
        store_band<NB>(o, acc, band, lane);
      } else if (lo == band_lo) {
        st.own = true;  // the share ends inside this band: nothing follows, keep the sum
        st.own_band = band;
      } else {
        store_partial<NB>(o, acc, wg, lane);
        // the sparse kernel's load ring is empty at the end of a piece, so nothing of it has to be
        // waited for to start the write-back here; the dense kernel keeps its ring going and
        // releases in one go at the end
        if (early_release) {
          release_begin();
          st.released = true;
        }
        st.publish = true;
      }
    }
  }
  if (!st.own) {
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};
  }
}

// After the tile loop.
template <int NB>
__device__ __forceinline__ void hand_over_finish(const OutParams& o, float4v (&acc)[kRowBlocks][NB],
                                                 const HandoverState& st, uint32_t wg, uint32_t P, int lane) {
  if (st.publish) {
    publish_partial(o, wg, lane, st.released);
  }
  if (st.own) {
    owner_finish<NB>(o, acc, st.own_band, wg, P, lane);
  }
}

// B operand fragments (X) of one K tile.  An MFMA wants lane l to hold column (l & 15) and the 8
// consecutive k of chunk (l >> 4), but loading X that way makes the four neighbouring lanes of
// every quad read four different cache lines (X is column-major).  So the load assigns lane j
// column (j >> 2) and chunk (j & 3) - a quad reads 64 contiguous bytes - and the fragment is put
// into MFMA order through a 1 KB LDS block per 16 columns: written as loaded, read back
// transposed.  The slot permutation keeps both the 16 B writes and the 16 B reads free of bank
// conflicts (any 16 neighbouring lanes touch 16 different 16 B slots modulo 256 B).
//
// The loads go through a buffer descriptor that ends after column N - 1, so the columns that pad
// N up to a multiple of 16 read as zero without a branch or a select after the load (either
// would make the compiler wait for the load on the spot).
struct XFrags {
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t lane_off;  // byte offset of the column and k chunk this lane loads
  uint32_t col_step;  // bytes between column blocks
  uint32_t wslot;     // byte offset in a column block's LDS stage where this lane's load goes
  uint32_t rslot;     // ... and where this lane's MFMA fragment comes from

  // 16 B slot of (column c, chunk g) of a 16-column block
  static __device__ __forceinline__ uint32_t slot(uint32_t c, uint32_t g) {
    return 16u * (c >> 2) + 4u * (c & 3u) + (g ^ (c >> 2));
  }
  __device__ __forceinline__ void init(const _Float16* X, uint32_t K, uint32_t N, uint32_t n0, int lane) {
    rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)X, 0, (int)(N * K * 2u), kBufferFlags);
    const uint32_t c = (uint32_t)lane >> 2, g = (uint32_t)lane & 3u;
    lane_off = ((n0 + c) * K + g * 8u) * 2u;
    col_step = 16u * K * 2u;
    wslot = slot(c, g) * 16u;
    rslot = slot((uint32_t)lane & 15u, (uint32_t)lane >> 4) * 16u;
  }
  template <int NB>
  __device__ __forceinline__ void load(u32x4 (&x)[NB], uint32_t kt) const {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
      x[nb] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane_off + nb * col_step, kt * (kTileK * 2u), 0);
  }
  // loaded registers -> the wave's LDS stage (NB KB)
  template <int NB>
  __device__ __forceinline__ void stage(unsigned char* xs, const u32x4 (&x)[NB]) const {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) *(u32x4*)(xs + nb * 1024 + wslot) = x[nb];
  }
  // MFMA B fragment of column block nb
  __device__ __forceinline__ half8 frag(const unsigned char* xs, int nb) const {
    return *(const half8*)(xs + nb * 1024 + rslot);
  }
};

}  // namespace fls
