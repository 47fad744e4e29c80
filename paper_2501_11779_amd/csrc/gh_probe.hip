// Streaming-read probe (measurement aid): contract in include/gh_probe.h.
#include "gh_probe.h"

#include <hip/hip_runtime.h>

#include "gh_tier2.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kTileVec = 1024;            // 16-byte vectors per 16 KiB tile (16 per lane)
constexpr int kRawBufferFlags = 0x00020000;

struct ProbeTile { u32x4 r[16]; };

__device__ __forceinline__ void probe_load(ProbeTile& t, const u32x4* p) {
#pragma unroll
  for (int u = 0; u < 16; ++u) t.r[u] = __builtin_nontemporal_load(p + u * 64);   // 1 KiB per instruction
}
__device__ __forceinline__ void probe_eat(const ProbeTile& t, u32x4 (&acc)[4]) {
#pragma unroll
  for (int u = 0; u < 16; ++u) acc[u & 3] ^= t.r[u];
}

// A loop the compiler cannot see through (idle is always 0): it keeps the loads of one tile and the
// use of the other in the order written.  Without it the compiler sinks the loads below the uses
// and every iteration starts with nothing in flight.
__device__ __forceinline__ void probe_fence(int idle) {
  for (int i = 0; i < idle; ++i) __builtin_amdgcn_s_sleep(1);
}

// POLICY: -1 no stores, else gh_probe_store.
template <int POLICY>
__global__ __launch_bounds__(256, 2) void probe_stream_kernel(const u32x4* src,
                                                              uint32_t tiles_per_wave, int store_every,
                                                              u32x4* rec, uint32_t* sink, int idle) {
  const int lane = threadIdx.x & 63;
  const size_t gw = (size_t)blockIdx.x * 4 + (size_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const u32x4* p = src + gw * tiles_per_wave * kTileVec + lane;
  u32x4 acc[4] = {u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}};
  u32x4* mine = rec + gw * 256 + lane;                    // 4 KiB per wave
  ProbeTile ta, tb;
  auto record = [&]() {
    if constexpr (POLICY == GH_PROBE_STORE_PLAIN) {
#pragma unroll
      for (int i = 0; i < 4; ++i) mine[i * 64] = acc[i];
    } else if constexpr (POLICY == GH_PROBE_STORE_NT) {
#pragma unroll
      for (int i = 0; i < 4; ++i) __builtin_nontemporal_store(acc[i], mine + i * 64);
    } else if constexpr (POLICY == GH_PROBE_STORE_WRITE_THROUGH) {
      const __amdgpu_buffer_rsrc_t dst = __builtin_amdgcn_make_buffer_rsrc(rec + gw * 256, 0, 4096, kRawBufferFlags);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        __builtin_amdgcn_raw_buffer_store_b128(acc[i], dst, (i * 64 + lane) * 16, 0, 0x11 /* sc0 sc1 */);
    }
  };
  // tiles_per_wave is even (checked on the host); past the end the last tile is loaded again.
  // The loads of a tile are issued before the tile that arrived earlier is used: one to three
  // tiles in flight, never none.
  const uint32_t last = tiles_per_wave - 1;
  // (0 = no stores: one group holding every tile; tiles go in pairs, so an odd store_every acts as
  // the next even number)
  const uint32_t group = POLICY >= 0 && store_every > 0 ? (uint32_t)store_every : tiles_per_wave;
  probe_load(ta, p);
  for (uint32_t t = 0; t < tiles_per_wave;) {
    const uint32_t end = t + group < tiles_per_wave ? t + group : tiles_per_wave;
    for (; t < end; t += 2) {
      probe_load(tb, p + (size_t)(t + 1) * kTileVec);
      probe_eat(ta, acc);
      probe_fence(idle);
      probe_load(ta, p + (size_t)(t + 2 < last ? t + 2 : last) * kTileVec);
      probe_eat(tb, acc);
      probe_fence(idle);
    }
    if constexpr (POLICY >= 0) record();
  }
  const u32x4 x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  if ((x[0] ^ x[1] ^ x[2] ^ x[3]) == 0x9e3779b9u && lane == 63) *sink = x[0];
}

// A workgroup uses few registers, so several fit a compute unit and the dispatcher may stack them
// while other units stay empty.  When there are no more workgroups than compute units, each asks
// for more than half a unit's LDS (which it never touches) and so gets a unit of its own: one wave
// per SIMD, the way the attention kernel's register budget spreads its workgroups.
constexpr int kComputeUnits = 256;
constexpr size_t kSpreadLdsBytes = 96 * 1024;

template <int POLICY>
int32_t launch_probe(dim3 grid, hipStream_t s, const u32x4* in, uint32_t tiles, int store_every,
                     u32x4* out, uint32_t* sink) {
  const size_t lds = grid.x <= (unsigned)kComputeUnits ? kSpreadLdsBytes : 0;
  if (lds && hipFuncSetAttribute(reinterpret_cast<const void*>(&probe_stream_kernel<POLICY>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
    return GH_ERR_HIP;
  hipLaunchKernelGGL(probe_stream_kernel<POLICY>, grid, dim3(256), lds, s, in, tiles, store_every, out,
                     sink, 0);
  return hipGetLastError() == hipSuccess ? GH_OK : GH_ERR_HIP;
}

}  // namespace

extern "C" int32_t gh_probe_stream_read(const void* src, size_t bytes, int32_t n_waves,
                                        int32_t store_every, int32_t store_policy, void* rec,
                                        uint32_t* sink, void* hip_stream) {
  if (!src || !sink || (store_every > 0 && !rec)) return GH_ERR_NULL;
  if (n_waves < 4 || n_waves > 65536 || n_waves % 4 != 0 || store_every < 0 || bytes == 0)
    return GH_ERR_SHAPE;
  const size_t per_pair = (size_t)n_waves * 2 * kTileVec * 16;          // two tiles per wave
  if (bytes % per_pair != 0 || bytes / per_pair > 0x3fffffffu) return GH_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(rec) & 15u))
    return GH_ERR_UNSUPPORTED;
  if (store_every > 0 && (store_policy < 0 || store_policy > 2)) return GH_ERR_UNSUPPORTED;
  const uint32_t tiles = (uint32_t)(bytes / per_pair) * 2;
  const dim3 grid(n_waves / 4);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const u32x4* in = static_cast<const u32x4*>(src);
  u32x4* out = static_cast<u32x4*>(rec);
  if (store_every == 0) return launch_probe<-1>(grid, s, in, tiles, 0, out, sink);
  if (store_policy == GH_PROBE_STORE_PLAIN) return launch_probe<0>(grid, s, in, tiles, store_every, out, sink);
  if (store_policy == GH_PROBE_STORE_NT) return launch_probe<1>(grid, s, in, tiles, store_every, out, sink);
  return launch_probe<2>(grid, s, in, tiles, store_every, out, sink);
}
