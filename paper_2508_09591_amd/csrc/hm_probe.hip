// hm_stream_probe: a measurement aid.  A flat stream with a chosen mix of read and write streams
// and no indirection, shaped like the row kernels (one wave per 1 KiB of every stream, 16-byte
// vectors, non-temporal stores), so that a benchmark can put the rate of hm_dispatch_pack
// (1 read + c writes per token) and hm_combine (c reads + 1 write) next to what the memory system
// gives for the same mix.  Not part of the paper's method.
#include "hm_device.h"

namespace hm {

constexpr int kProbeThreads = 128;
constexpr int kProbeMaxStreams = 16;

__global__ __launch_bounds__(kProbeThreads) void stream_probe_kernel(const u32x4 *__restrict__ src, int nr, u32x4 *__restrict__ dst,
                                                                     int nw, int64_t n) {
  const int64_t v = ((int64_t)blockIdx.x * (kProbeThreads / kWave) + (threadIdx.x >> 6)) * kWave + lane_id();
  if (v >= n) return;
  u32x4 acc = {0u, 0u, 0u, 0u};
  if (nr == 1) {
    acc = src[v];   // a single read stream is read the way dispatch reads its token rows
  } else {
    for (int i = 0; i < nr; ++i) {   // several: non-temporal, the way combine reads packed rows
      const u32x4 r = load_stream(src + (int64_t)i * n + v);
      acc ^= r;
    }
  }
  for (int j = 0; j < nw; ++j) store_stream(dst + (int64_t)j * n + v, acc);
}

}  // namespace hm

extern "C" hm_status hm_stream_probe(const void *src, int32_t read_streams, void *dst, int32_t write_streams,
                                     int64_t vectors_per_stream, void *hip_stream) {
  using namespace hm;
  if (!src || !dst) return HM_ERR_NULL;
  if (read_streams < 1 || read_streams > kProbeMaxStreams || write_streams < 1 || write_streams > kProbeMaxStreams)
    return HM_ERR_SHAPE;
  if (vectors_per_stream < 0 || (((uintptr_t)src | (uintptr_t)dst) & 15u) != 0) return HM_ERR_SHAPE;
  if (vectors_per_stream == 0) return HM_OK;
  const int64_t waves = (vectors_per_stream + kWave - 1) / kWave;
  const int64_t blocks = (waves + (kProbeThreads / kWave) - 1) / (kProbeThreads / kWave);
  if (blocks > 2147483647LL) return HM_ERR_SHAPE;
  hipLaunchKernelGGL(stream_probe_kernel, dim3((unsigned)blocks), dim3(kProbeThreads), 0, (hipStream_t)hip_stream,
                     (const u32x4 *)src, read_streams, (u32x4 *)dst, write_streams, vectors_per_stream);
  return hm_launch_status();
}
