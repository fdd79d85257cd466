// Machine probes behind the roofline fractions the benchmark reports: what a plain streaming
// read and a dense matrix-core loop reach on the GPU at hand.  Measurement support only - no part
// of the CaliDrop path uses this file.  C ABI, device pointers, caller times the launches with
// events on `stream`.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

// Every workgroup reads its own contiguous slice, 16 bytes per lane, 8 loads in flight per lane.
// kNonTemporal: the loads carry the non-temporal hint (data that is not read again soon).
template <bool kNonTemporal>
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ p, uint64_t vec_per_block, uint32_t* out) {
  const u32x4* q = p + static_cast<uint64_t>(blockIdx.x) * vec_per_block;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (uint64_t i = threadIdx.x; i < vec_per_block; i += 256 * 8) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      v[u] = u32x4{0u, 0u, 0u, 0u};
      if (i + u * 256 < vec_per_block) v[u] = kNonTemporal ? __builtin_nontemporal_load(q + i + u * 256) : q[i + u * 256];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) out[blockIdx.x] = 1u;   // keeps the loads alive
}

// The same bytes requested the way a matrix-operand fragment load requests rows of 256 bytes: per
// wave instruction 16 rows x 64 bytes (lane (i, c) = 16 bytes at row i, piece c), four instructions
// per 16 rows.  Every wave owns a contiguous slice (a multiple of 8 KiB).
__global__ __launch_bounds__(256) void stream_read_pieces_kernel(const char* __restrict__ p, uint64_t bytes_per_wave, uint32_t* out) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int i = lane & 15, c = lane >> 4;
  const char* q = p + (static_cast<uint64_t>(blockIdx.x) * 4 + wv) * bytes_per_wave;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (uint64_t off = 0; off < bytes_per_wave; off += 8192) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(q + off + (u >> 2) * 4096 + i * 256 + (u & 3) * 64 + c * 16));
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) out[blockIdx.x] = 1u;
}

// A streaming read (non-temporal, 16 KiB per workgroup and stage) with full-line stores mixed in: after
// every stage 64 threads store one float each to each of `rows` output streams (256 bytes per stream
// and stage).  rows = 0: the read alone.
__global__ __launch_bounds__(256) void stream_read_store_kernel(const u32x4* __restrict__ src, float* __restrict__ dst, int stages, int rows,
                                                                int64_t row_stride, uint32_t* out) {
  const int64_t wg = blockIdx.x;
  const u32x4* q = src + wg * stages * 1024;
  float* w = dst + wg * stages * 64;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (int s = 0; s < stages; ++s) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(q + s * 1024 + u * 256 + threadIdx.x);
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= v[u];
    if (threadIdx.x < 64) {
      const float val = __uint_as_float(acc[0] & 0x3fffffffu);
      for (int r = 0; r < rows; ++r) w[r * row_stride + s * 64 + threadIdx.x] = val;
    }
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) out[blockIdx.x] = 1u;
}

// Each wave runs `iters` rounds of 8 independent accumulate chains of the bf16 16x16x32 matrix
// instruction: 8 * 16384 flop per round and wave, nothing else in the loop.
__global__ __launch_bounds__(256) void mfma_loop_kernel(float* out, int iters) {
  const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});   // 1.0
  const bf16x8 b = __builtin_bit_cast(bf16x8, u32x4{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u});   // 2^-7
  f32x4 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
  }
  f32x4 s = acc[0];
#pragma unroll
  for (int j = 1; j < 8; ++j) s += acc[j];
  out[static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x] = s[0] + s[1] + s[2] + s[3];
}

// Matrix instructions and ordinary vector instructions side by side.  A round is 8 x (two bf16
// 16x16x32 matrix instructions, each followed by NV / 2 independent vector instructions): fused
// multiply-adds, or exp2 when kExp.  kMatrix = false leaves the matrix instructions out, NV = 0 the
// vector ones: three launches (matrix only, vector only, both) show how much of the vector work
// issues in the shadow of the matrix pipe.  The register budget is held to 128 so that 4 waves fit
// a SIMD (launch 4 workgroups per compute unit).
template <bool kMatrix, int NV, bool kExp>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void mfma_valu_kernel(float* out, int iters) {
  const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});   // 1.0
  const bf16x8 b = __builtin_bit_cast(bf16x8, u32x4{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u});   // 2^-7
  f32x4 acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  float v[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) v[j] = 0.001f * static_cast<float>(threadIdx.x + j);
  const float c1 = 0.999f, c2 = 1e-6f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      if constexpr (kMatrix) acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[u], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = 0; q < NV / 2; ++q) {
        const int x = (u * (NV / 2) + q) % 16;
        v[x] = kExp ? __builtin_amdgcn_exp2f(v[x]) : fmaf(v[x], c1, c2);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 16; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3] + v[j];
  out[static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x] = s;
}

}  // namespace

extern "C" {

// Reads `bytes` (a multiple of 16 * blocks) starting at `buf` with `blocks` workgroups.  `out`
// needs `blocks` uint32.  Returns 0, or -1 on bad arguments / launch failure.
int calidrop_probe_stream_read(const void* buf, uint64_t bytes, int32_t blocks, void* out, void* stream) {
  if (!buf || !out || blocks < 1 || bytes == 0 || bytes % (16ull * blocks) != 0) return -1;
  hipLaunchKernelGGL(stream_read_kernel<false>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(buf), bytes / 16 / blocks, static_cast<uint32_t*>(out));
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// The same read with non-temporal loads.
int calidrop_probe_stream_read_nt(const void* buf, uint64_t bytes, int32_t blocks, void* out, void* stream) {
  if (!buf || !out || blocks < 1 || bytes == 0 || bytes % (16ull * blocks) != 0) return -1;
  hipLaunchKernelGGL(stream_read_kernel<true>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(buf), bytes / 16 / blocks, static_cast<uint32_t*>(out));
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Reads `bytes` (a multiple of 32768 * blocks) in 64-byte pieces, 16 rows of 256 bytes per wave instruction.
int calidrop_probe_stream_read_pieces(const void* buf, uint64_t bytes, int32_t blocks, void* out, void* stream) {
  if (!buf || !out || blocks < 1 || bytes == 0 || bytes % (32768ull * blocks) != 0) return -1;
  hipLaunchKernelGGL(stream_read_pieces_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const char*>(buf), bytes / blocks / 4, static_cast<uint32_t*>(out));
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// `blocks` workgroups read `stages` x 16 KiB each from `src` (blocks * stages * 16 KiB bytes) and store
// `rows` x 256 bytes per stage into `dst` (rows * blocks * stages * 256 bytes).  `out`: blocks uint32.
int calidrop_probe_stream_read_store(const void* src, void* dst, int32_t blocks, int32_t stages, int32_t rows, void* out,
                                     void* stream) {
  if (!src || !out || blocks < 1 || stages < 1 || rows < 0 || (rows > 0 && !dst)) return -1;
  hipLaunchKernelGGL(stream_read_store_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(src), static_cast<float*>(dst), stages, rows,
                     static_cast<int64_t>(blocks) * stages * 64, static_cast<uint32_t*>(out));
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Launches `blocks` workgroups of 4 waves, each wave doing iters * 8 matrix instructions
// (16384 flop each).  `out` needs blocks * 256 floats.
int calidrop_probe_mfma_loop(void* out, int32_t blocks, int32_t iters, void* stream) {
  if (!out || blocks < 1 || iters < 1) return -1;
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<float*>(out), iters);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// `blocks` workgroups of 4 waves (1024 = 4 waves on every SIMD of the chip); every wave runs iters
// rounds of 16 matrix instructions (`matrix` != 0) with `valu_per_pair` / 2 vector instructions
// behind each: fused multiply-adds, or exp2 when `use_exp` != 0.  valu_per_pair: 0 or 8.  `out`:
// blocks * 256 floats.
int calidrop_probe_mfma_valu(void* out, int32_t blocks, int32_t iters, int32_t matrix, int32_t valu_per_pair,
                             int32_t use_exp, void* stream) {
  if (!out || blocks < 1 || iters < 1 || (valu_per_pair != 0 && valu_per_pair != 8) || (!matrix && !valu_per_pair)) return -1;
  const dim3 g(blocks), t(256);
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* o = static_cast<float*>(out);
  if (matrix && !valu_per_pair) hipLaunchKernelGGL((mfma_valu_kernel<true, 0, false>), g, t, 0, st, o, iters);
  else if (matrix && !use_exp) hipLaunchKernelGGL((mfma_valu_kernel<true, 8, false>), g, t, 0, st, o, iters);
  else if (matrix) hipLaunchKernelGGL((mfma_valu_kernel<true, 8, true>), g, t, 0, st, o, iters);
  else if (!use_exp) hipLaunchKernelGGL((mfma_valu_kernel<false, 8, false>), g, t, 0, st, o, iters);
  else hipLaunchKernelGGL((mfma_valu_kernel<false, 8, true>), g, t, 0, st, o, iters);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // extern "C"
