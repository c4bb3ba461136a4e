// The calibration kernels declared in include/sailor_microbench.h.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#include "../../include/sailor_microbench.h"

namespace {

// Eight independent chains of dependent FMAs per lane: enough to cover the ALU latency with
// the waves a compute unit holds, so the loop runs at the issue rate of v_fma_f32.
__global__ __launch_bounds__(256) void k_fma_chain(float *out, int iters, float a, float b) {
  float x[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) x[j] = (float)(threadIdx.x + j) * 1.0e-3f;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = fmaf(x[j], a, b);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) s += x[j];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;  // keeps the chains alive
}

// A workgroup fills one contiguous 16 KiB tile: every lane stores 16 bytes four times,
// consecutive lanes consecutive addresses.
constexpr int kWriteUnroll = 4;
__global__ __launch_bounds__(256) void k_stream_write(float4 *dst, size_t n4, float v) {
  const float4 val = make_float4(v, v, v, v);
  const size_t base = (size_t)blockIdx.x * (256 * kWriteUnroll) + threadIdx.x;
#pragma unroll
  for (int j = 0; j < kWriteUnroll; ++j) {
    const size_t i = base + (size_t)j * 256;
    if (i < n4) dst[i] = val;
  }
}

// The store pattern of the per-candidate evaluation and nothing else: four arrays (4 + 4 + 8 + 4
// bytes per element), a workgroup covers 16 Ki consecutive elements, a lane stores one element of
// each array per step, consecutive lanes consecutive elements.
constexpr uint32_t kRecordChunk = 16384;
__global__ __launch_bounds__(512) void k_record_write(float *t, float *c, uint64_t *m, uint32_t *k, uint64_t n) {
  const uint64_t lo = (uint64_t)blockIdx.x * kRecordChunk;
  for (uint32_t i = threadIdx.x; i < kRecordChunk; i += blockDim.x) {
    const uint64_t idx = lo + i;
    if (idx >= n) break;
    t[idx] = (float)i;
    c[idx] = (float)i * 2.f;
    m[idx] = idx;
    k[idx] = i & 63u;
  }
}

struct Events {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool make() { return hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess; }
  ~Events() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  }
};

}  // namespace

extern "C" {

int sailor_microbench_fma(int32_t workgroups, int32_t iters, int32_t reps, double *tflops,
                          double *best_ms, void *hip_stream) {
  if (workgroups < 1 || iters < 1 || reps < 1 || !tflops) return -1;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float *out = nullptr;
  if (hipMalloc(reinterpret_cast<void **>(&out), (size_t)workgroups * 256 * sizeof(float)) != hipSuccess)
    return -2;
  Events ev;
  int rc = ev.make() ? 0 : -3;
  double best = 1e300;
  for (int r = 0; r <= reps && rc == 0; ++r) {  // (the first repetition warms up)
    if (hipEventRecord(ev.e0, st) != hipSuccess) { rc = -3; break; }
    k_fma_chain<<<(unsigned)workgroups, 256, 0, st>>>(out, iters, 0.999f, 1.0e-3f);
    float ms = 0.f;
    if (hipEventRecord(ev.e1, st) != hipSuccess || hipEventSynchronize(ev.e1) != hipSuccess ||
        hipEventElapsedTime(&ms, ev.e0, ev.e1) != hipSuccess || hipGetLastError() != hipSuccess) {
      rc = -3;
      break;
    }
    if (r > 0 && ms < best) best = ms;
  }
  (void)hipFree(out);
  if (rc != 0) return rc;
  const double flops = 2.0 * 8.0 * (double)iters * 256.0 * (double)workgroups;
  *tflops = flops / (best * 1e-3) / 1e12;
  if (best_ms) *best_ms = best;
  return 0;
}

int sailor_microbench_write(uint64_t bytes, int32_t reps, double *gbytes_per_s, double *best_ms,
                            void *hip_stream) {
  if (bytes == 0 || bytes % 4096 != 0 || bytes > (1ull << 36) || reps < 1 || !gbytes_per_s) return -1;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float4 *buf = nullptr;
  if (hipMalloc(reinterpret_cast<void **>(&buf), bytes) != hipSuccess) return -2;
  Events ev;
  int rc = ev.make() ? 0 : -3;
  double best = 1e300;
  const size_t n4 = bytes / sizeof(float4);
  for (int r = 0; r <= reps && rc == 0; ++r) {
    if (hipEventRecord(ev.e0, st) != hipSuccess) { rc = -3; break; }
    const size_t tiles = (n4 + 256 * kWriteUnroll - 1) / (256 * kWriteUnroll);
    k_stream_write<<<(unsigned)tiles, 256, 0, st>>>(buf, n4, (float)r);
    float ms = 0.f;
    if (hipEventRecord(ev.e1, st) != hipSuccess || hipEventSynchronize(ev.e1) != hipSuccess ||
        hipEventElapsedTime(&ms, ev.e0, ev.e1) != hipSuccess || hipGetLastError() != hipSuccess) {
      rc = -3;
      break;
    }
    if (r > 0 && ms < best) best = ms;
  }
  (void)hipFree(buf);
  if (rc != 0) return rc;
  *gbytes_per_s = (double)bytes / (best * 1e-3) / 1e9;
  if (best_ms) *best_ms = best;
  return 0;
}

int sailor_microbench_write_records(uint64_t elements, int32_t reps, double *gbytes_per_s, double *best_ms,
                                    void *hip_stream) {
  if (elements == 0 || elements > (1ull << 32) || reps < 1 || !gbytes_per_s) return -1;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  unsigned char *buf = nullptr;  // one allocation: [n] u64, then three [n] 4-byte arrays
  if (hipMalloc(reinterpret_cast<void **>(&buf), elements * 20) != hipSuccess) return -2;
  uint64_t *m = reinterpret_cast<uint64_t *>(buf);
  float *t = reinterpret_cast<float *>(buf + elements * 8);
  float *c = t + elements;
  uint32_t *k = reinterpret_cast<uint32_t *>(c + elements);
  Events ev;
  int rc = ev.make() ? 0 : -3;
  double best = 1e300;
  for (int r = 0; r <= reps && rc == 0; ++r) {
    if (hipEventRecord(ev.e0, st) != hipSuccess) { rc = -3; break; }
    k_record_write<<<(unsigned)((elements + kRecordChunk - 1) / kRecordChunk), 512, 0, st>>>(t, c, m, k, elements);
    float ms = 0.f;
    if (hipEventRecord(ev.e1, st) != hipSuccess || hipEventSynchronize(ev.e1) != hipSuccess ||
        hipEventElapsedTime(&ms, ev.e0, ev.e1) != hipSuccess || hipGetLastError() != hipSuccess) {
      rc = -3;
      break;
    }
    if (r > 0 && ms < best) best = ms;
  }
  (void)hipFree(buf);
  if (rc != 0) return rc;
  *gbytes_per_s = 20.0 * (double)elements / (best * 1e-3) / 1e9;
  if (best_ms) *best_ms = best;
  return 0;
}

}  // extern "C"
