// Reference rates for reports, measured on the chip the library runs on: what the MFMA pipe
// sustains with nothing else going on, and what a plain streaming read of HBM sustains.  The
// contraction kernels are held against the vendor peaks; these two figures say how much of the
// distance to the peak is the chip's own (clocks under load, DRAM efficiency).
#include "pipe_internal.h"

#include <cstdint>
#include <vector>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// Every wave issues back-to-back independent v_mfma_i32_16x16x64_i8 on registers (no memory
// traffic in the loop).  Operands come from memory once: the chip lowers its clock with the
// toggle rate of the operands, so constant operands overstate what a real layer can reach.
__global__ __launch_bounds__(256, 2) void mfma_probe_kernel(int iters, const v4i* __restrict__ ops, int* sink) {
  v4i a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = ops[i * 256 + threadIdx.x];
    b[i] = ops[(4 + i) * 256 + threadIdx.x];
  }
  v4i c[4][4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int t = 0; t < 4; ++t) c[r][t] = v4i{0, 0, 0, 0};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int t = 0; t < 4; ++t) c[r][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[r], b[t], c[r][t], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int t = 0; t < 4; ++t) s += c[r][t][0] + c[r][t][1] + c[r][t][2] + c[r][t][3];
  if (s == 0x7fffffff) sink[0] = s;   // keeps the loop alive; practically never true
}

// The same loop on v_mfma_i32_32x32x32_i8 (twice the multiply-adds per operand byte): eight
// independent instructions per round, the same 16 x 16384 multiply-adds per round and wave.
typedef int v16i __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256, 2) void mfma_probe32_kernel(int iters, const v4i* __restrict__ ops, int* sink) {
  v4i a[4], b[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = ops[i * 256 + threadIdx.x];
#pragma unroll
  for (int i = 0; i < 2; ++i) b[i] = ops[(4 + i) * 256 + threadIdx.x];
  v16i c[4][2];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) c[r][t][i] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int t = 0; t < 2; ++t) c[r][t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[r], b[t], c[r][t], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) s += c[r][t][i];
  if (s == 0x7fffffff) sink[0] = s;   // keeps the loop alive; practically never true
}

// Streaming read: every 512-thread workgroup reads a contiguous 128 KiB, wave w the 1-KiB tiles
// w, w+8, ..., four loads in flight per lane -- the access pattern of the weight-streaming kernel.
__global__ __launch_bounds__(512) void hbm_probe_kernel(const uint4* __restrict__ x, unsigned* sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint4* base = x + (size_t)blockIdx.x * 8192;
  unsigned acc = 0;
  for (int t = wave; t + 24 < 128; t += 32) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = base[(size_t)(t + u * 8) * 64 + lane];
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x12345678u) sink[0] = acc;
}

}  // namespace

extern "C" int pipe_mfma_probe(int iters, int operands, double* tops_out, void* stream) {
  const bool wide = operands >= 10;   // 10..12: the same operand kinds on the 32x32x32 instruction
  if (wide) operands -= 10;
  if (iters <= 0 || !tops_out || operands < 0 || operands > 2) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  int* sink = (int*)pipe_ws_get(WS_MISC, 256 + 8 * 256 * 16);
  if (!sink) return pipe_ws_error();
  v4i* ops_dev = reinterpret_cast<v4i*>(reinterpret_cast<uint8_t*>(sink) + 256);
  // operands: 0 = constant bytes; 1 = ternary offset codes {0,1,2} against random int8
  // activations (what the ternary layers feed the pipe); 2 = random int8 against random int8
  std::vector<uint8_t> host(8 * 256 * 16);
  uint64_t z = 0x9E3779B97F4A7C15ull;
  auto next = [&]() { z ^= z << 13; z ^= z >> 7; z ^= z << 17; return (uint32_t)(z >> 24); };
  for (size_t i = 0; i < host.size(); ++i) {
    const bool is_a = i < host.size() / 2;
    const uint32_t r = next();
    host[i] = operands == 0 ? (uint8_t)1 : (operands == 1 && is_a ? (uint8_t)(r % 3) : (uint8_t)r);
  }
  PIPE_HIP(hipMemcpyAsync(ops_dev, host.data(), host.size(), hipMemcpyHostToDevice, st));
  PIPE_HIP(hipStreamSynchronize(st));
  hipEvent_t e0, e1;
  PIPE_HIP(hipEventCreate(&e0));
  PIPE_HIP(hipEventCreate(&e1));
  const int blocks = 256 * 2 * 4;   // 2 workgroups per CU resident, 4 rounds
  if (wide) PIPE_KLAUNCH(mfma_probe32_kernel, dim3(blocks), dim3(256), 0, st, 16, ops_dev, sink);   // warm-up
  else PIPE_KLAUNCH(mfma_probe_kernel, dim3(blocks), dim3(256), 0, st, 16, ops_dev, sink);
  PIPE_HIP(hipEventRecord(e0, st));
  if (wide) PIPE_KLAUNCH(mfma_probe32_kernel, dim3(blocks), dim3(256), 0, st, iters, ops_dev, sink);
  else PIPE_KLAUNCH(mfma_probe_kernel, dim3(blocks), dim3(256), 0, st, iters, ops_dev, sink);
  PIPE_HIP(hipEventRecord(e1, st));
  PIPE_HIP(hipEventSynchronize(e1));
  float ms = 0.f;
  PIPE_HIP(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  const double ops = (double)blocks * 4.0 * iters * 16.0 * (2.0 * 16 * 16 * 64);
  *tops_out = ops / (ms * 1e-3) / 1e12;
  return PIPE_OK;
}

extern "C" int pipe_hbm_probe(int64_t bytes, double* gbps_out, void* stream) {
  if (!gbps_out || bytes < (int64_t)(1 << 20)) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const int64_t blocks = bytes / (128 << 10);
  uint8_t* buf = nullptr;
  PIPE_HIP(hipMalloc(&buf, (size_t)blocks * (128 << 10) + 256));
  unsigned* sink = reinterpret_cast<unsigned*>(buf + (size_t)blocks * (128 << 10));
  hipError_t he = hipMemsetAsync(buf, 1, (size_t)blocks * (128 << 10) + 256, st);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (he == hipSuccess) he = hipEventCreate(&e0);
  if (he == hipSuccess) he = hipEventCreate(&e1);
  float ms = 0.f;
  if (he == hipSuccess) {
    PIPE_KLAUNCH(hbm_probe_kernel, dim3((unsigned)blocks), dim3(512), 0, st, reinterpret_cast<const uint4*>(buf), sink);
    he = hipEventRecord(e0, st);
    PIPE_KLAUNCH(hbm_probe_kernel, dim3((unsigned)blocks), dim3(512), 0, st, reinterpret_cast<const uint4*>(buf), sink);
    if (he == hipSuccess) he = hipEventRecord(e1, st);
    if (he == hipSuccess) he = hipEventSynchronize(e1);
    if (he == hipSuccess) he = hipEventElapsedTime(&ms, e0, e1);
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(buf);
  if (he != hipSuccess) { pipe_note_hip_error(he, "pipe_hbm_probe"); return PIPE_EDEVICE; }
  *gbps_out = (double)blocks * (128 << 10) / (ms * 1e-3) / 1e9;
  return PIPE_OK;
}
