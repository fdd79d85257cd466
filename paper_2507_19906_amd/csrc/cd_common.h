// Device-side building blocks shared by the CaliDrop kernels (gfx950 / CDNA4, wave64).
//
// Matrix-core convention used everywhere: one "mma step" multiplies a 16 x KD tile A by a
// KD x 16 tile B into a 16x16 fp32 tile, where every lane contributes one 16-byte fragment of
// A and one of B.  Lane l = 16*c + i holds, for A, row i and the c-th 16-byte piece of the
// step's K range; for B, column i and the same piece.  The result tile is spread as
// acc[r] = C[4*c + r][i].  For bf16 a step is one v_mfma_f32_16x16x32_bf16 (KD = 32); for
// fp32 it is four v_mfma_f32_16x16x4_f32 (KD = 16, the x-th instruction takes element x of
// each fragment).  Because A and B fragments use the same K placement, any contraction over
// the step's K range comes out right.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cd {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

struct bf16_t { uint16_t bits; };   // storage type tag for bf16 tensors

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kWave = 64;

template <typename T> struct Elem;
template <> struct Elem<bf16_t> {
  static constexpr int kPer16B = 8;    // elements in one 16-byte fragment
  static constexpr int kStepK = 32;    // contraction depth of one mma step
};
template <> struct Elem<float> {
  static constexpr int kPer16B = 4;
  static constexpr int kStepK = 16;
};

// Index of the calling wave inside its workgroup, as a value the compiler knows to be the same in
// every lane: what is derived from it (tile ranges, "is this stage fully visible" flags, LDS buffer
// addresses) then lives in scalar registers and branches on it are scalar branches, instead of
// per-lane arithmetic and exec-masked execution of both sides.
__device__ __forceinline__ int wave_index() {
  return __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
}

__device__ __forceinline__ u32x4 ld16(const void* p) { return *reinterpret_cast<const u32x4*>(p); }
// The same for data that is read once and not again soon (the K/V streams): a non-temporal load,
// which leaves the caches to data that is reused (measured on the decode stream of a 256 MiB
// cache: 5.85 -> 6.50 TB/s).
__device__ __forceinline__ u32x4 ld16_stream(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
__device__ __forceinline__ void st16(void* p, u32x4 v) { *reinterpret_cast<u32x4*>(p) = v; }
__device__ __forceinline__ u32x4 zero16() { return u32x4{0u, 0u, 0u, 0u}; }

// LDS-direct loads: each lane reads `bytes` from its own global address and the load unit stores
// the wave's 64 pieces contiguously (lane order) at the wave-uniform LDS address `lds`.  Tracked
// by vmcnt like any global load.
__device__ __forceinline__ void load_to_lds16(const void* g, void* lds) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)lds, 16, 0, 0);
}
// the same with the non-temporal hint (rows that are read once and not again soon)
__device__ __forceinline__ void load_to_lds16_stream(const void* g, void* lds) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)lds, 16, 0, 2);
}
__device__ __forceinline__ void load_to_lds4(const void* g, void* lds) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)lds, 4, 0, 0);
}

// Reinterpret a 32-bit lane value (always pass vector elements through this by-value helper:
// bit-casting a vector element expression directly reads element 0 with this compiler).
__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }

template <typename T>
__device__ __forceinline__ void mma_step(f32x4& acc, const u32x4& a, const u32x4& b);

template <>
__device__ __forceinline__ void mma_step<bf16_t>(f32x4& acc, const u32x4& a, const u32x4& b) {
  acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mma_step<float>(f32x4& acc, const u32x4& a, const u32x4& b) {
#pragma unroll
  for (int x = 0; x < 4; ++x)
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(as_f32(a[x]), as_f32(b[x]), acc, 0, 0, 0);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// bf16 <-> fp32 (round to nearest even; inputs are finite)
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __builtin_bit_cast(float, static_cast<uint32_t>(b) << 16);
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
}

template <typename T> __device__ __forceinline__ float load_elem(const T* p, int64_t i);
template <> __device__ __forceinline__ float load_elem<bf16_t>(const bf16_t* p, int64_t i) {
  return bf16_to_f32(p[i].bits);
}
template <> __device__ __forceinline__ float load_elem<float>(const float* p, int64_t i) { return p[i]; }

// An element as its storage bits (zero-extended), and those bits as a float: a load split from its
// conversion, for places where the value must not be touched until later.
template <typename T> __device__ __forceinline__ uint32_t load_bits(const T* p, int64_t i);
template <> __device__ __forceinline__ uint32_t load_bits<bf16_t>(const bf16_t* p, int64_t i) { return p[i].bits; }
template <> __device__ __forceinline__ uint32_t load_bits<float>(const float* p, int64_t i) {
  return __builtin_bit_cast(uint32_t, p[i]);
}
template <typename T> __device__ __forceinline__ float bits_to_f32(uint32_t u);
template <> __device__ __forceinline__ float bits_to_f32<bf16_t>(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
template <> __device__ __forceinline__ float bits_to_f32<float>(uint32_t u) { return __builtin_bit_cast(float, u); }

template <typename T> __device__ __forceinline__ void store_elem(T* p, int64_t i, float v);
template <> __device__ __forceinline__ void store_elem<bf16_t>(bf16_t* p, int64_t i, float v) {
  p[i].bits = f32_to_bf16(v);
}
template <> __device__ __forceinline__ void store_elem<float>(float* p, int64_t i, float v) { p[i] = v; }

// Data-parallel-primitive lane exchange inside a row of 16 lanes.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive adds only (no LDS
// round trips): shifts by 1, 2, 4, 8 inside each row of 16 lanes (a lane whose source falls outside
// its row adds 0), then the last lane of row 0 / 2 is added to rows 1 / 3 and the last lane of
// row 1 - by then the total of rows 0 and 1 - to rows 2 and 3.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_u32_or_zero(uint32_t x) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
  x += dpp_u32_or_zero<0x111, 0xF>(x);   // row_shr:1
  x += dpp_u32_or_zero<0x112, 0xF>(x);   // row_shr:2
  x += dpp_u32_or_zero<0x114, 0xF>(x);   // row_shr:4
  x += dpp_u32_or_zero<0x118, 0xF>(x);   // row_shr:8
  x += dpp_u32_or_zero<0x142, 0xA>(x);   // row_bcast:15 into rows 1 and 3
  x += dpp_u32_or_zero<0x143, 0xC>(x);   // row_bcast:31 into rows 2 and 3
  return x;
}
// the value lane 63 holds, in every lane
__device__ __forceinline__ uint32_t last_lane(uint32_t x) {
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(x), 63));
}

// Sum over the 16 lanes that share l/16; every lane ends with the same bits (fixed tree).
__device__ __forceinline__ float row16_sum(float x) {
  x += dpp_f32<0xB1>(x);    // quad_perm [1,0,3,2]
  x += dpp_f32<0x4E>(x);    // quad_perm [2,3,0,1]
  x += dpp_f32<0x141>(x);   // row_half_mirror
  x += dpp_f32<0x140>(x);   // row_mirror
  return x;
}
// Lane l's value together with that of lane l ^ 16 (pair16) or l ^ 32 (pair32), the lower lane's
// first, through the gfx950 lane-swap instructions: two registers that start as copies of x trade
// rows (odd rows of one with even rows of the other) or halves (upper half of one with the lower
// half of the other), after which one holds the even-row / lower-half values in every lane and the
// other the odd-row / upper-half values.  Plain vector-ALU instructions: no LDS round trip, unlike
// a general lane permutation.
typedef unsigned lane_pair_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void pair16(float x, float& lo, float& hi) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const lane_pair_t r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned r0 = r.x, r1 = r.y;
  lo = __builtin_bit_cast(float, r0);
  hi = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ void pair32(float x, float& lo, float& hi) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const lane_pair_t r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const unsigned r0 = r.x, r1 = r.y;
  lo = __builtin_bit_cast(float, r0);
  hi = __builtin_bit_cast(float, r1);
}
// Reductions over the four lanes {i, i+16, i+32, i+48} (same column, different c): every lane ends
// with the same bits, (x_0 + x_16) + (x_32 + x_48).
__device__ __forceinline__ float col4_max(float x) {
  float lo, hi;
  pair16(x, lo, hi);
  pair32(fmaxf(lo, hi), lo, hi);
  return fmaxf(lo, hi);
}
__device__ __forceinline__ float col4_sum(float x) {
  float lo, hi;
  pair16(x, lo, hi);
  pair32(lo + hi, lo, hi);
  return lo + hi;
}
// Sum over all 64 lanes, every lane ends with the same bits (fixed tree: inside rows of 16, then across).
__device__ __forceinline__ float wave_sum(float x) { return col4_sum(row16_sum(x)); }

// Workgroups are dealt to the 8 XCDs (each with its own L2) round-robin in launch order.  For a
// grid of (blocks, heads) whose heads divide by 8, this re-reads the launch index so that every
// XCD works through whole heads, the blocks of a head one after the other: the workgroups that
// stream the same operand at the same time then share one L2 instead of every L2 fetching the
// stream for itself.  vx in [0, gridDim.x), vh in [0, gridDim.y * gridDim.z); a bijection.
__device__ __forceinline__ void xcd_head_major(int& vx, int& vh) {
  vx = static_cast<int>(blockIdx.x);
  vh = static_cast<int>(blockIdx.y + gridDim.y * blockIdx.z);
  const int gx = static_cast<int>(gridDim.x), H = static_cast<int>(gridDim.y * gridDim.z);
  if (H % 8 == 0) {
    const int L = vx + gx * vh;
    const int slot = L / 8;
    vx = slot % gx;
    vh = (L % 8) * (H / 8) + slot / gx;
  }
}

// The same for a grid (chunks, rows) whose rows are (sequence, KV head, ...) units of possibly very
// different lengths: XCD x takes the rows x, x + 8, x + 16, ... (every sequence's work is spread over
// the XCDs the same way) and works through them chunk by chunk, so that all workgroups which share a
// row's stationary operand sit behind one L2.  Returns false (vx, vy = the launch indices) when the
// row count does not divide by 8.
__device__ __forceinline__ bool xcd_rows_interleaved(int& vx, int& vy) {
  vx = static_cast<int>(blockIdx.x);
  vy = static_cast<int>(blockIdx.y);
  const int gx = static_cast<int>(gridDim.x), H = static_cast<int>(gridDim.y);
  if (H % 8 != 0) return false;
  const int L = vx + gx * vy;
  const int slot = L / 8;
  vx = slot % gx;
  vy = (slot / gx) * 8 + (L % 8);
  return true;
}

// Merge two (max, sum-of-exp2) pairs in the log2 domain; (-inf, 0) is the identity.
__device__ __forceinline__ void merge_ml(float& m, float& l, float m2, float l2) {
  float mn = fmaxf(m, m2);
  if (mn == -INFINITY) { m = mn; l = 0.f; return; }
  l = l * fast_exp2(m - mn) + l2 * fast_exp2(m2 - mn);
  m = mn;
}

}  // namespace cd
