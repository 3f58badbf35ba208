// probe.hip — the memory traffic of a handoff without its arithmetic: a measurement aid.
//
// Card creation reads 8 KiB of fp16 rows per tile and writes about 2 KiB of card; injection does
// the reverse.  These kernels move the same amounts in the same launch shape — one wave per unit of
// READS + WRITES kilobytes, four independent waves per workgroup, 128-bit accesses, the same cache
// policies — and do nothing else, so their time is what this memory system gives that traffic mix.
// Every stored word depends on every loaded one (an exclusive-or), so nothing is optimised away.
#include "qkv_common.h"

namespace qkv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Unit u reads chunks [u * READS * 64, (u + 1) * READS * 64) of src and writes chunks
// [u * WRITES * 64, (u + 1) * WRITES * 64) of dst; lane l takes chunk k * 64 + l of each.
template <int READS, int WRITES, bool NT_LOAD, bool NT_STORE>
__global__ __launch_bounds__(kBlockThreads) void stream_probe_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                                    uint64_t units) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint64_t gw = (uint64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const uint64_t n_waves = (uint64_t)gridDim.x * kWavesPerBlock;
  for (uint64_t u = gw; u < units; u += n_waves) {
    const u32x4* s = src + u * (READS * kWaveSize) + lane;
    u32x4 v[READS];
#pragma unroll
    for (int k = 0; k < READS; ++k) v[k] = NT_LOAD ? __builtin_nontemporal_load(s + k * kWaveSize) : s[k * kWaveSize];
    u32x4 x = v[0];
#pragma unroll
    for (int k = 1; k < READS; ++k) x ^= v[k];
    u32x4* d = dst + u * (WRITES * kWaveSize) + lane;
#pragma unroll
    for (int k = 0; k < WRITES; ++k) {
      const u32x4 w = x + (u32x4)((uint32_t)k);
      if (NT_STORE) __builtin_nontemporal_store(w, d + k * kWaveSize); else d[k * kWaveSize] = w;
    }
  }
}

template <int READS, int WRITES>
void launch_mix(const void* src, void* dst, uint64_t units, int nontemporal, hipStream_t stream) {
  const dim3 grid(grid_blocks(units)), block(kBlockThreads);
  const u32x4* s = static_cast<const u32x4*>(src);
  u32x4* d = static_cast<u32x4*>(dst);
  switch (nontemporal & 3) {
    case 0: hipLaunchKernelGGL((stream_probe_kernel<READS, WRITES, false, false>), grid, block, 0, stream, s, d, units); break;
    case 1: hipLaunchKernelGGL((stream_probe_kernel<READS, WRITES, true, false>), grid, block, 0, stream, s, d, units); break;
    case 2: hipLaunchKernelGGL((stream_probe_kernel<READS, WRITES, false, true>), grid, block, 0, stream, s, d, units); break;
    default: hipLaunchKernelGGL((stream_probe_kernel<READS, WRITES, true, true>), grid, block, 0, stream, s, d, units); break;
  }
}

}  // namespace

// reads_kib : writes_kib is 8 : 2 (card creation), 2 : 8 (injection) or 8 : 8 (a copy); the caller has
// checked that `units` units fit both buffers.
hipError_t launch_stream_probe(const void* src, void* dst, uint64_t units, int reads_kib, int writes_kib, int nontemporal,
                               hipStream_t stream) {
  if (units == 0) return hipSuccess;
  if (reads_kib == 8 && writes_kib == 2) launch_mix<8, 2>(src, dst, units, nontemporal, stream);
  else if (reads_kib == 2 && writes_kib == 8) launch_mix<2, 8>(src, dst, units, nontemporal, stream);
  else launch_mix<8, 8>(src, dst, units, nontemporal, stream);
  return hipGetLastError();
}

}  // namespace qkv
