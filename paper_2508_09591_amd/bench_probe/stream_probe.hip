// libhmprobe.so -- a measurement aid for bench.py, not part of the library: flat streams with a
// chosen mix of read and write streams and NO indirection, so that the rates of hm_dispatch_pack
// (1 read + c writes per token) and hm_combine (c reads + 1 write) can be put next to what the
// memory system gives a plain kernel moving the same bytes with the same mix.  The launch shape
// is the caller's: workgroup size and a cap on resident waves per CU (set, as in the row kernels,
// with an unused dynamic LDS allocation), so a benchmark can sweep them and quote the best --
// a ceiling that does not inherit the row kernels' own choices.  One wave moves 1 KiB of every
// stream with 16-byte vectors; several read streams are read with non-temporal loads, a single
// one with plain loads, all stores are non-temporal.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kMaxStreams = 16;

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void stream_probe_kernel(const u32x4 *__restrict__ src, int nr, u32x4 *__restrict__ dst,
                                                             int nw, int64_t n) {
  const int64_t v = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
  if (v >= n) return;
  u32x4 acc = {0u, 0u, 0u, 0u};
  if (nr == 1) {
    acc = src[v];
  } else {
    for (int i = 0; i < nr; ++i) acc ^= __builtin_nontemporal_load(src + (int64_t)i * n + v);
  }
  for (int j = 0; j < nw; ++j) __builtin_nontemporal_store(acc, dst + (int64_t)j * n + v);
}

template <int BLOCK>
int launch(const u32x4 *src, int nr, u32x4 *dst, int nw, int64_t n, unsigned lds, hipStream_t stream) {
  const int64_t blocks = (n + BLOCK - 1) / BLOCK;
  if (blocks > 2147483647LL) return -2;
  hipLaunchKernelGGL(stream_probe_kernel<BLOCK>, dim3((unsigned)blocks), dim3(BLOCK), lds, stream, src, nr, dst, nw, n);
  return hipGetLastError() == hipSuccess ? 0 : -8;
}

}  // namespace

// src holds read_streams inputs back to back, dst write_streams outputs, each of vectors_per_stream
// 16-byte vectors (device pointers, 16-byte aligned); every output vector is the XOR of the input
// vectors at its index.  block_threads is 64, 128 or 256; waves_per_cu in [1,32] caps the resident
// waves per CU (32 or more = no cap).  Returns 0, or -1 (null), -2 (bad shape), -8 (HIP error).
extern "C" int bench_stream_probe(const void *src, int32_t read_streams, void *dst, int32_t write_streams,
                                  int64_t vectors_per_stream, int32_t block_threads, int32_t waves_per_cu,
                                  void *hip_stream) {
  if (!src || !dst) return -1;
  if (read_streams < 1 || read_streams > kMaxStreams || write_streams < 1 || write_streams > kMaxStreams) return -2;
  if (vectors_per_stream < 0 || (((uintptr_t)src | (uintptr_t)dst) & 15u) != 0) return -2;
  if (block_threads != 64 && block_threads != 128 && block_threads != 256) return -2;
  if (waves_per_cu < 1) return -2;
  if (vectors_per_stream == 0) return 0;
  unsigned lds = 0;
  const int blocks_per_cu = waves_per_cu / (block_threads / 64);
  if (waves_per_cu < 32 && blocks_per_cu >= 1) {
    int dev = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&per_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess)
      return -8;
    if (per_cu >= 65536) {
      const int bytes = (per_cu / blocks_per_cu) & ~511;
      lds = bytes > 65536 ? 65536u : (unsigned)bytes;
    }
  }
  hipStream_t stream = (hipStream_t)hip_stream;
  const u32x4 *s = (const u32x4 *)src;
  u32x4 *d = (u32x4 *)dst;
  if (block_threads == 64) return launch<64>(s, read_streams, d, write_streams, vectors_per_stream, lds, stream);
  if (block_threads == 128) return launch<128>(s, read_streams, d, write_streams, vectors_per_stream, lds, stream);
  return launch<256>(s, read_streams, d, write_streams, vectors_per_stream, lds, stream);
}
