// Measurement aids, not part of the method and not part of libbc.so: plain streaming reads of a
// buffer by a given number of workgroups.  They put a number on what a read-only kernel of the
// decode step's size and grid costs on this chip (launch gap, first-byte latency, streaming rate),
// the floor the decode kernel's duration is compared with.  Built into libbc_diag.so.
#include "../bc_common.h"
#include "../../../include/bc_diag.h"

namespace bc {

// Mode 0.  Every workgroup of 512 threads reads its contiguous share with 16-byte non-temporal
// loads into registers, eight in flight per thread (8 KB per wave), and leaves one word so that
// the loads cannot be dropped.
__global__ __launch_bounds__(512) void stream_read_kernel(const char* src, int64_t units,
                                                          uint32_t* sink) {
  const int64_t per_wg = (units + gridDim.x - 1) / gridDim.x;
  const int64_t u0 = (int64_t)blockIdx.x * per_wg;
  const int64_t u1 = u0 + per_wg < units ? u0 + per_wg : units;
  const u32x4_t* p = reinterpret_cast<const u32x4_t*>(src);
  uint32_t acc = 0;
  for (int64_t u = u0 + threadIdx.x; u < u1; u += 8 * 512) {
    u32x4_t r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int64_t i = u + (int64_t)j * 512;
      r[j] = i < u1 ? __builtin_nontemporal_load(p + i) : u32x4_t{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= r[j].x ^ r[j].y ^ r[j].z ^ r[j].w;
  }
  if (acc == 0x9e3779b9u && sink) sink[blockIdx.x] = acc;     // practically never taken
  if (threadIdx.x == 0 && sink) sink[blockIdx.x] = 1u;
}

// Mode 1.  The same share read by LDS-DMA, the way the decode kernel moves its tiles: every wave
// issues its 1 KB instructions back to back, all of its share in flight at once (up to
// kDmaMaxPerWave instructions, 48 KB, per pass), into a 4 KB LDS region of its own that is simply
// overwritten - nothing consumes the data, the kernel only waits for it.  No register ever holds
// a byte, so the number in flight is not bounded by the register file.
constexpr int kDmaWaves = 8;
constexpr int kDmaMaxPerWave = 48;      // below the 63 loads the wave's counter can track
__global__ __launch_bounds__(kDmaWaves * 64) void stream_read_dma_kernel(const char* src, int64_t kb_units,
                                                                          uint32_t* sink) {
  __shared__ __attribute__((aligned(1024))) char lds[kDmaWaves * 4096];
  // kb_units: 1 KB pieces of the buffer; a workgroup owns a contiguous run, its waves take the
  // pieces in turn
  const int64_t per_wg = (kb_units + gridDim.x - 1) / gridDim.x;
  const int64_t u0 = (int64_t)blockIdx.x * per_wg;
  const int64_t u1 = u0 + per_wg < kb_units ? u0 + per_wg : kb_units;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  char* mine = lds + wave * 4096;
  for (int64_t u = u0 + wave; u < u1; u += (int64_t)kDmaWaves * kDmaMaxPerWave) {
#pragma unroll 8
    for (int j = 0; j < kDmaMaxPerWave; ++j) {
      const int64_t i = u + (int64_t)j * kDmaWaves;
      if (i < u1) lds_dma16<true>(src + i * 1024 + lane * 16, mine + (j & 3) * 1024);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  if (threadIdx.x == 0 && sink) sink[blockIdx.x] = 1u;
}

}  // namespace bc

using namespace bc;

extern "C" int32_t bc_diag_stream_read(const void* src, size_t bytes, int32_t workgroups, int32_t mode,
                                       uint32_t* sink, void* stream) {
  if (workgroups < 1 || workgroups > 65536) return BC_ERR_ARG;
  if (mode != 0 && mode != 1) return BC_ERR_ARG;
  if (bytes > 0 && (!src || !aligned16(src))) return BC_ERR_ARG;
  if (bytes & (mode == 1 ? 1023u : 15u)) return BC_ERR_ARG;
  if (mode == 0)
    stream_read_kernel<<<workgroups, 512, 0, as_stream(stream)>>>(static_cast<const char*>(src),
                                                                 (int64_t)(bytes / 16), sink);
  else
    stream_read_dma_kernel<<<workgroups, kDmaWaves * 64, 0, as_stream(stream)>>>(
        static_cast<const char*>(src), (int64_t)(bytes / 1024), sink);
  return launch_status();
}
