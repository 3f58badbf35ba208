// stream_probe.hip — a measurement aid for bench.py, NOT part of the CacheCard library: the memory
// traffic of a handoff without its arithmetic.
//
// Card creation reads 8 KiB of fp16 rows per tile and writes about 2 KiB of card; injection does
// the reverse.  These kernels move the same amounts in the same launch shape — one wave per unit of
// READS + WRITES kilobytes, four independent waves per workgroup, 128-bit accesses, the same cache
// policies — and do nothing else, so their time is what this memory system gives that traffic mix.
// Every stored word depends on every loaded one (an exclusive-or), so nothing is optimised away.
//
// Built by build() into bench_probe/libqkvprobe.so; one extern "C" entry point:
//
//   int qkv_stream_probe(const void* src_dev, uint64_t src_bytes, void* dst_dev, uint64_t dst_bytes,
//                        int32_t reads_kib, int32_t writes_kib, int32_t nontemporal,
//                        uint64_t* units_out, void* stream);
//
// Unit u reads reads_kib KiB at src + u * reads_kib KiB and writes writes_kib KiB at
// dst + u * writes_kib KiB; every written word is the exclusive-or of the unit's 16-byte chunks that
// the writing lane read (chunk k * 64 + lane, k = 0 .. reads_kib - 1, as four 32-bit words), plus the
// index of the write (0 .. writes_kib - 1) in each word.
//   reads_kib : writes_kib   8 : 2 (card creation at about 3 bits), 2 : 8 (injection), 8 : 8 (copy).
//   nontemporal: bit 0 loads, bit 1 stores bypass the caches' keep policy.
//   units_out:  host, may be NULL: the whole units that fit both buffers = units processed.
// src_dev, dst_dev: device, 16-byte aligned, not overlapping.  Asynchronous on `stream`.
// Returns 0, or -1 (null pointer), -2 (another mix or flag), -6 (alignment), -10 (overlap), -8 (HIP error).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kWaveSize = 64;
constexpr int kBlockThreads = 256;                    // four independent waves, as in the card kernels
constexpr int kWavesPerBlock = kBlockThreads / kWaveSize;

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
  uint64_t blocks = (units + kWavesPerBlock - 1) / kWavesPerBlock;      // one wave per unit
  if (blocks > 0x7FFFFFFFull) blocks = 0x7FFFFFFFull;
  const dim3 grid((uint32_t)blocks), block(kBlockThreads);
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

extern "C" int qkv_stream_probe(const void* src_dev, uint64_t src_bytes, void* dst_dev, uint64_t dst_bytes, int32_t reads_kib,
                                int32_t writes_kib, int32_t nontemporal, uint64_t* units_out, void* stream) {
  if (!src_dev || !dst_dev) return -1;
  const bool known = (reads_kib == 8 && writes_kib == 2) || (reads_kib == 2 && writes_kib == 8) ||
                     (reads_kib == 8 && writes_kib == 8);
  if (!known || nontemporal < 0 || nontemporal > 3) return -2;
  if (reinterpret_cast<uintptr_t>(src_dev) % 16 != 0 || reinterpret_cast<uintptr_t>(dst_dev) % 16 != 0) return -6;
  {
    const uintptr_t s0 = reinterpret_cast<uintptr_t>(src_dev), d0 = reinterpret_cast<uintptr_t>(dst_dev);
    if (s0 < d0 + dst_bytes && d0 < s0 + src_bytes) return -10;
  }
  const uint64_t units_r = src_bytes / ((uint64_t)reads_kib * 1024u), units_w = dst_bytes / ((uint64_t)writes_kib * 1024u);
  const uint64_t units = units_r < units_w ? units_r : units_w;      // whole units that fit both buffers
  if (units_out) *units_out = units;
  if (units == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (reads_kib == 8 && writes_kib == 2) launch_mix<8, 2>(src_dev, dst_dev, units, nontemporal, s);
  else if (reads_kib == 2 && writes_kib == 8) launch_mix<2, 8>(src_dev, dst_dev, units, nontemporal, s);
  else launch_mix<8, 8>(src_dev, dst_dev, units, nontemporal, s);
  return hipGetLastError() == hipSuccess ? 0 : -8;
}
