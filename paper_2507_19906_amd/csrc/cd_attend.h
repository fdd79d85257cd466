// Streaming GQA attention of one query per head over a range of K/V rows, with the running
// softmax kept as (max, sum, unnormalised output) so that partial results over disjoint row
// sets merge by the attention-decomposition identity (Eq. 1-2).  Used twice:
//   * calibration precompute (Alg. 1 steps 5-8): q = calibration query, rows = the prefix of
//     the prompt with the retained positions masked out (i.e. KV_evict);
//   * decode (Alg. 2 step 1): q = current query, rows = the compressed cache.
// A workgroup owns one (sequence, KV head, split of the rows); its 4 waves take 32-row tiles
// round-robin.  Per tile: S^T = K Q^T on the matrix cores (rows are the A rows, the G heads
// are B columns 0..G-1, the other columns are zero padding), softmax weights stay in the
// lanes that produced them and feed O^T += V^T P^T directly as the B operand.
#pragma once
#include "cd_common.h"
#include "cd_score.h"

namespace cd {

constexpr int kTileRows = 32;
constexpr int kAttWaves = 4;

struct AttendArgs {
  const void* q;              // [batch][Hq][D] or, when q_is_window, [batch][Hq][w][D] (last row used)
  const void* k; const void* v;
  const int32_t* row_off;     // [batch+1] token offsets of the K/V buffers
  const int32_t* row_len;     // decode: live rows per sequence; NULL in calibration mode
  const uint32_t* bitmap;     // calibration mode: [batch*Hkv][W32] not-evicted bits; else NULL
  int64_t total_tokens;       // calibration mode: contract check of row_off
  int batch, Hq, Hkv, G, w, B, max_len, W32, rows_per_split, NS;
  int q_is_window;            // 1: q points at q_win and the last window row is the query
  float sl2;                  // scale * log2(e)
  const float* cal_logit;     // calibration mode: [batch*Hq][zstride] precomputed log2-unit logits, or NULL
  int zstride;
  const uint8_t* only_flagged; // optional [batch][Hq]: skip KV groups in which no head carries flag 2
  float* part_o;              // [batch][Hq][NS][D]
  float2* part_ml;            // [batch][Hq][NS]  (max in log2 units, sum)
};

// Number of rows the streaming pass covers for sequence b, the stride between heads and the
// token offset, for both modes.  rows = 0 means nothing to do.
__device__ __forceinline__ void attend_geometry(const AttendArgs& a, int b, int& rows, int& head_stride, int& off0) {
  if (a.bitmap) {                                   // calibration: prefix rows of the prompt
    int n = seq_len_checked(a.row_off, b, a.max_len, a.total_tokens, off0);
    head_stride = n;
    rows = (n > a.B) ? n - a.w : 0;
  } else {                                          // decode: live rows of the cache
    if (a.row_off) { off0 = a.row_off[b]; head_stride = a.row_off[b + 1] - off0; }
    else { head_stride = a.max_len; off0 = b * a.max_len; }      // uniform capacity
    int len = a.row_len[b];
    rows = (len < 0 || len > head_stride || len > a.max_len) ? 0 : len;
  }
}

// Per-wave state and tile loop of the streaming attention.  Lane l = 16 c + i.
template <typename T, int D>
struct AttendWave {
  static constexpr int EPL = Elem<T>::kPer16B;
  static constexpr int KD = Elem<T>::kStepK;
  static constexpr int NK = D / KD;
  static constexpr bool kBf16 = sizeof(T) == 2;
  static constexpr int NACC = kBf16 ? 8 : D / 16;   // output accumulators per lane (x4 floats)

  u32x4 qf[NK];          // B operand: column i = head i of the group (zero beyond G)
  f32x4 acc_o[NACC];     // O^T tile: acc_o[x][r] <-> d slot 4c+r, head i
  float m, l;            // running max (log2 units, shared by the 4 lanes of a head) and this lane's sum share

  __device__ __forceinline__ void init(const T* q_row, bool valid, int c) {
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) qf[kk] = valid ? ld16(q_row + kk * KD + c * EPL) : zero16();
#pragma unroll
    for (int x = 0; x < NACC; ++x) acc_o[x] = f32x4{0.f, 0.f, 0.f, 0.f};
    m = -INFINITY;
    l = 0.f;
  }

  // The K rows of the wave's first tile, requested before the number of live rows is known (it may
  // still be on its way from memory): `clamp` is a row count that is certainly addressable.
  u32x4 kpre[2][NK];
  __device__ __forceinline__ void request_first_k(const T* kbase, int row0, int clamp, int i, int c) {
    load_k(kbase, row0, clamp, i, c, kpre);
  }

  __device__ __forceinline__ void load_k(const T* kbase, int row0, int rows, int i, int c, u32x4 (&kf)[2][NK]) const {
#pragma unroll
    for (int g2 = 0; g2 < 2; ++g2) {
      const int krow = min(row0 + 16 * g2 + i, rows - 1);
      const T* kp = kbase + static_cast<int64_t>(krow) * D + c * EPL;
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) kf[g2][kk] = ld16_stream(kp + kk * KD);
    }
  }

  // The same K rows requested as whole rows: instruction kk of a 16-row group reads the group's bytes
  // 1024 kk .. 1024 kk + 1023 (16 bytes per lane in lane order) - what a link that moves small reads
  // badly wants (rows in page-locked host memory: 55 GB/s against 41 GB/s for the 64-byte pieces of
  // the operand layout).  regroup_k() turns the result into the operand layout.
  __device__ __forceinline__ void load_k_rows(const T* kbase, int row0, int rows, int lane, u32x4 (&kf)[2][NK]) const {
    constexpr int kRowBytes = D * static_cast<int>(sizeof(T));
#pragma unroll
    for (int g2 = 0; g2 < 2; ++g2)
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) {
        const int o = kk * 1024 + lane * 16;
        const int krow = min(row0 + 16 * g2 + o / kRowBytes, rows - 1);
        kf[g2][kk] = ld16_stream(reinterpret_cast<const char*>(kbase + static_cast<int64_t>(krow) * D) + o % kRowBytes);
      }
  }
  // Through a wave-private LDS area of 16 rows: written in the order loaded, read back as lane (i, c),
  // step kk = bytes 64 kk + 16 c of row i.  One wave only, so the in-order LDS queue is all the
  // synchronisation needed; the fences keep the compiler from moving the accesses across each other.
  __device__ __forceinline__ void regroup_k(char* stage, u32x4 (&kf)[2][NK], int lane, int i, int c) const {
    constexpr int kRowBytes = D * static_cast<int>(sizeof(T));
#pragma unroll
    for (int g2 = 0; g2 < 2; ++g2) {
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) *reinterpret_cast<u32x4*>(stage + kk * 1024 + lane * 16) = kf[g2][kk];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) kf[g2][kk] = *reinterpret_cast<const u32x4*>(stage + i * kRowBytes + kk * 64 + c * 16);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  }

  // bf16 V rows of a tile: lane (i, c) loads, for e = 4 g2 + r, the 16-byte piece i of row
  // row0 + 16 g2 + 4 c + r (each instruction reads four whole rows, fully coalesced)
  __device__ __forceinline__ void load_v(const T* vbase, int row0, int rows, int i, int c, u32x4 (&vf)[8]) const {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int vrow = min(row0 + 16 * (e >> 2) + 4 * c + (e & 3), rows - 1);
      vf[e] = (i < D / 8) ? ld16_stream(vbase + static_cast<int64_t>(vrow) * D + i * 8) : zero16();
    }
  }

  // Online-softmax update for one tile of logits: acc_s[g2][r] <-> row row0 + 16 g2 + 4 c + r,
  // head i.  Rescales the running sum and output, returns the tile's weights in p.
  template <bool kLogits>
  __device__ __forceinline__ void softmax_tile(const f32x4 (&acc_s)[2], int row0, int row_end, uint32_t skip,
                                               float sl2, int c, float (&p)[2][4]) {
    float x[2][4];
    float tm = -INFINITY;
#pragma unroll
    for (int g2 = 0; g2 < 2; ++g2)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int rr = 16 * g2 + 4 * c + r;
        const bool live = (row0 + rr < row_end) && !((skip >> rr) & 1u);
        x[g2][r] = live ? (kLogits ? acc_s[g2][r] : acc_s[g2][r] * sl2) : -INFINITY;
        tm = fmaxf(tm, x[g2][r]);
      }
    tm = col4_max(tm);
    const float mn = fmaxf(m, tm);
    const float ms = (mn == -INFINITY) ? 0.f : mn;
    const float alpha = fast_exp2(m - ms);
    m = mn;
    float ps = 0.f;
#pragma unroll
    for (int g2 = 0; g2 < 2; ++g2)
#pragma unroll
      for (int r = 0; r < 4; ++r) { p[g2][r] = fast_exp2(x[g2][r] - ms); ps += p[g2][r]; }
    l = l * alpha + ps;
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int xx = 0; xx < NACC; ++xx) acc_o[xx] *= alpha;
    }
  }

  // O^T += V^T P^T for a tile whose bf16 V rows sit in vf (as loaded by load_v)
  __device__ __forceinline__ void pv_bf16(const u32x4 (&vf)[8], const float (&p)[2][4]) {
    u32x4 pf;
    pf[0] = pack_bf16x2(p[0][0], p[0][1]);
    pf[1] = pack_bf16x2(p[0][2], p[0][3]);
    pf[2] = pack_bf16x2(p[1][0], p[1][1]);
    pf[3] = pack_bf16x2(p[1][2], p[1][3]);
#pragma unroll
    for (int xx = 0; xx < 8; ++xx) {
      // A fragment of instruction xx: element xx of each of the 8 loaded pieces (8 rows)
      u32x4 af;
#pragma unroll
      for (int ww = 0; ww < 4; ++ww) {
        const uint32_t lo = vf[2 * ww][xx >> 1], hi = vf[2 * ww + 1][xx >> 1];
        af[ww] = (xx & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u)) : ((lo & 0xFFFFu) | (hi << 16));
      }
      mma_step<bf16_t>(acc_o[xx], af, pf);
    }
  }

  // Process the 32-row tiles row_first, row_first + row_step, ... below row_end.  `rows` is
  // the number of valid rows of the head (loads are clamped to it); `bm` (optional) marks rows
  // to skip, one bit per row, word index = row / 32.
  // Logits of rows row0 + 16 g2 + 4 c + r (r = 0..3) of head i, precomputed by the scoring pass.
  __device__ __forceinline__ static void load_z(const float* zhead, int row0, int c, bool valid, f32x4 (&z)[2]) {
#pragma unroll
    for (int g2 = 0; g2 < 2; ++g2)
      z[g2] = valid ? __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(zhead + row0 + 16 * g2 + 4 * c))
                    : f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // kLogits: the logits come from `zhead` (this lane's head, log2 units) instead of K Q^T.
  struct NoWork { __device__ __forceinline__ void operator()() const {} };
  // `while_waiting` runs once, after the loads of the wave's first tile have been issued and before
  // anything waits for them: arithmetic placed there is hidden behind the memory latency.
  // `k_requested`: the K rows of the wave's first tile are already on their way into kpre
  // (request_first_k).
  // `kRowsK`: K is fetched as whole rows and regrouped through `k_stage` (16 rows of wave-private LDS).
  template <bool kPrefetch = true, bool kLogits = false, typename F = NoWork, bool kRowsK = false>
  __device__ __forceinline__ void run(const T* kbase, const T* vbase, const uint32_t* bm, int rows, int row_first,
                                      int row_end, int row_step, float sl2, int i, int c,
                                      const float* zhead = nullptr, bool zvalid = false, bool k_requested = false,
                                      F while_waiting = F(), char* k_stage = nullptr) {
    u32x4 kf[2][NK];
    f32x4 zf[2];
    auto fetch_k = [&](int row0) {
      if constexpr (kRowsK) load_k_rows(kbase, row0, rows, 16 * c + i, kf);
      else load_k(kbase, row0, rows, i, c, kf);
    };
    if (row_first >= row_end) { while_waiting(); return; }
    if constexpr (kLogits) {
      load_z(zhead, row_first, c, zvalid, zf);
    } else {
      if (k_requested) {
#pragma unroll
        for (int g2 = 0; g2 < 2; ++g2)
#pragma unroll
          for (int kk = 0; kk < NK; ++kk) kf[g2][kk] = kpre[g2][kk];
      } else {
        fetch_k(row_first);
      }
    }
    for (int row0 = row_first; row0 < row_end; row0 += row_step) {
      // V of this tile first, then K of the next tile: both in flight during the QK product
      u32x4 vf[8];
      if constexpr (kBf16) load_v(vbase, row0, rows, i, c, vf);
      if (row0 == row_first) while_waiting();
      f32x4 acc_s[2];
      const int next0 = row0 + row_step;
      if constexpr (kLogits) {
        acc_s[0] = zf[0];
        acc_s[1] = zf[1];
        if (next0 < row_end) load_z(zhead, next0, c, zvalid, zf);
      } else {
        if constexpr (kRowsK) regroup_k(k_stage, kf, 16 * c + i, i, c);
#pragma unroll
        for (int g2 = 0; g2 < 2; ++g2) {
          acc_s[g2] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kk = 0; kk < NK; ++kk) mma_step<T>(acc_s[g2], kf[g2][kk], qf[kk]);
        }
        if constexpr (kPrefetch) {
          if (next0 < row_end) fetch_k(next0);
        }
      }
      const uint32_t skip = bm ? bm[row0 >> 5] : 0u;
      float p[2][4];
      softmax_tile<kLogits>(acc_s, row0, row_end, skip, sl2, c, p);
      // ---- O^T += V^T P^T -----------------------------------------------------------------
      if constexpr (kBf16) {
        pv_bf16(vf, p);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int vrow = min(row0 + 16 * (e >> 2) + 4 * c + (e & 3), rows - 1);
          const float pe = p[e >> 2][e & 3];
#pragma unroll
          for (int dh = 0; dh < D / 64; ++dh) {
            u32x4 v4 = ld16_stream(vbase + static_cast<int64_t>(vrow) * D + (i + 16 * dh) * 4);
#pragma unroll
            for (int xx = 0; xx < 4; ++xx)
              acc_o[dh * 4 + xx] =
                  __builtin_amdgcn_mfma_f32_16x16x4f32(as_f32(v4[xx]), pe, acc_o[dh * 4 + xx], 0, 0, 0);
          }
        }
      }
      if constexpr (!kPrefetch && !kLogits) {
        if (next0 < row_end) fetch_k(next0);
      }
    }
  }

  // Publish this wave's (max, sum) and unnormalised outputs for heads < G: s_o [G][D], s_ml [G].
  __device__ __forceinline__ void publish(float* s_o, float2* s_ml, int G, int i, int c) {
    const float lsum = col4_sum(l);
    if (i < G) {
      if (c == 0) s_ml[i] = make_float2(m, lsum);
      if constexpr (kBf16) {
        // d = 8 * slot + xx: the 8 accumulators of one (c, r) are 8 consecutive outputs
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int d0 = 8 * (4 * c + r);
          if (d0 < D) {
            f32x4* dst = reinterpret_cast<f32x4*>(s_o + i * D + d0);
            dst[0] = f32x4{acc_o[0][r], acc_o[1][r], acc_o[2][r], acc_o[3][r]};
            dst[1] = f32x4{acc_o[4][r], acc_o[5][r], acc_o[6][r], acc_o[7][r]};
          }
        }
      } else {
#pragma unroll
        for (int xx = 0; xx < NACC; ++xx)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int d = 4 * ((4 * c + r) + 16 * (xx >> 2)) + (xx & 3);     // output row of the tile = d slot
            if (d < D) s_o[i * D + d] = acc_o[xx][r];
          }
      }
    }
  }
};

// kLogits: calibration mode with the logits precomputed by the scoring pass (K is not read).
// kRowsK: K rows are requested whole and regrouped in LDS (rows that live in host memory).
template <typename T, int D, bool kLogits, bool kRowsK = false>
__global__ __launch_bounds__(256) void attend_partial_kernel(AttendArgs a) {
  // grid: x = split of the rows (rotated per head so that the splits every sequence has do not
  // all land on the same XCDs of the round-robin deal), y = KV head, z = sequence
  const int g = blockIdx.y, b = blockIdx.z;
  const int split = (blockIdx.x + g + a.Hkv * b) % gridDim.x;
  int rows, head_stride, off0;
  attend_geometry(a, b, rows, head_stride, off0);
  const int row_begin = split * a.rows_per_split;
  if (row_begin >= rows) return;
  if (a.only_flagged) {
    bool any = false;
    for (int hh = 0; hh < a.G; ++hh) any |= a.only_flagged[b * a.Hq + g * a.G + hh] == 2;
    if (!any) return;
  }
  const int row_end = min(rows, row_begin + a.rows_per_split);
  const int lane = threadIdx.x & 63, wv = wave_index();
  const int i = lane & 15, c = lane >> 4;
  const int64_t head_tok = static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * head_stride;
  const T* kbase = static_cast<const T*>(a.k) + head_tok * D;
  const T* vbase = static_cast<const T*>(a.v) + head_tok * D;
  const uint32_t* bm = a.bitmap ? a.bitmap + static_cast<int64_t>(b * a.Hkv + g) * a.W32 : nullptr;

  __shared__ __attribute__((aligned(16))) float s_o[kAttWaves][16 * D];
  __shared__ float2 s_ml[kAttWaves][16];
  AttendWave<T, D> w;
  {
    const int h = g * a.G + i;
    const T* qp = static_cast<const T*>(a.q);
    if (a.q_is_window) qp += (static_cast<int64_t>(b * a.Hq + h) * a.w + (a.w - 1)) * D;
    else qp += static_cast<int64_t>(b * a.Hq + h) * D;
    w.init(qp, i < a.G, c);
  }
  if constexpr (kLogits) {
    // padding rows of the last tile hold whatever the workspace held: they are masked before use
    const float* zhead = a.cal_logit + static_cast<int64_t>(b * a.Hq + g * a.G + i) * a.zstride;
    w.template run<true, true>(kbase, vbase, bm, rows, row_begin + wv * kTileRows, row_end, kAttWaves * kTileRows,
                               a.sl2, i, c, zhead, i < a.G);
  } else if constexpr (kRowsK) {
    // 16 rows of K fit the area the wave publishes its outputs to afterwards
    static_assert(16 * D * sizeof(T) <= sizeof(s_o[0]), "K staging area");
    w.template run<true, false, typename AttendWave<T, D>::NoWork, true>(
        kbase, vbase, bm, rows, row_begin + wv * kTileRows, row_end, kAttWaves * kTileRows, a.sl2, i, c, nullptr, false,
        false, typename AttendWave<T, D>::NoWork(), reinterpret_cast<char*>(s_o[wv]));
  } else {
    w.run(kbase, vbase, bm, rows, row_begin + wv * kTileRows, row_end, kAttWaves * kTileRows, a.sl2, i, c);
  }

  // ---- merge the 4 waves through LDS and write this split's partial ------------------------
  w.publish(s_o[wv], s_ml[wv], a.G, i, c);
  __syncthreads();
  for (int t = threadIdx.x; t < a.G * D; t += 256) {
    const int hh = t / D, d = t - hh * D;
    float mm = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < kAttWaves; ++ww) mm = fmaxf(mm, s_ml[ww][hh].x);
    const float ms = (mm == -INFINITY) ? 0.f : mm;
    float o = 0.f, ll = 0.f;
#pragma unroll
    for (int ww = 0; ww < kAttWaves; ++ww) {
      const float sc = fast_exp2(s_ml[ww][hh].x - ms);
      o += s_o[ww][hh * D + d] * sc;
      ll += s_ml[ww][hh].y * sc;
    }
    const int64_t slot = (static_cast<int64_t>(b * a.Hq + g * a.G + hh)) * a.NS + split;
    a.part_o[slot * D + d] = o;
    if (d == 0) a.part_ml[slot] = make_float2(mm, ll);
  }
}

struct FinalArgs {
  const float* part_o; const float2* part_ml;
  const int32_t* row_off; const int32_t* row_len;
  int64_t total_tokens;
  int batch, Hq, Hkv, G, w, B, max_len, rows_per_split, NS, calib_mode, q_is_window;
  float theta1, theta2;
  const void* q;                 // query tensor (see AttendArgs)
  // calibration mode outputs / decode mode inputs
  float* c_q; float* c_out; float* c_lse;
  // decode outputs (recalibration mode, calib_mode = 2: out, a_lse and flags are inputs too)
  void* out; float* a_lse; uint8_t* flags;
};

__device__ __forceinline__ float block_sum(float x, float* red, int nthreads) {
  // sum over the workgroup (nthreads = 64 or 128), fixed order; result in every thread
  x = wave_sum(x);
  const int wv = wave_index();
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wv] = x;
  __syncthreads();
  float t = red[0];
  for (int ww = 1; ww < nthreads / 64; ++ww) t += red[ww];
  return t;
}

// One workgroup of D threads per (sequence, query head): merge the split partials (Eq. 1-2
// applied NS-1 times), then either store the calibration state (Alg. 1 steps 6-8) or apply
// the cosine gate and the calibration merge (Alg. 2 steps 2-15).
template <typename T, int D>
__global__ __launch_bounds__(D) void attend_finalize_kernel(FinalArgs a) {
  const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
  const int g = h / a.G;
  __shared__ float red[4];
  if (a.calib_mode == 2 && a.flags[b * a.Hq + h] != 2) return;      // only heads flagged for recomputation
  int rows;
  if (!a.row_len) {                   // rows of a prompt (minus the window); else live rows of a packed buffer
    int off0;
    int n = seq_len_checked(a.row_off, b, a.max_len, a.total_tokens, off0);
    rows = (n > a.B) ? n - a.w : 0;
  } else {
    int cap = a.row_off ? a.row_off[b + 1] - a.row_off[b] : a.max_len;
    int len = a.row_len[b];
    rows = (len < 0 || len > cap || len > a.max_len) ? 0 : len;
  }
  (void)g;
  const int ns = (rows + a.rows_per_split - 1) / a.rows_per_split;
  const int64_t slot0 = static_cast<int64_t>(b * a.Hq + h) * a.NS;
  const int64_t hd = static_cast<int64_t>(b * a.Hq + h);
  // operands of the tail are fetched now, together with the partials (one round trip, not five)
  const T* qp = static_cast<const T*>(a.q);
  const float qd = a.q_is_window ? load_elem<T>(qp, (hd * a.w + (a.w - 1)) * D + d) : load_elem<T>(qp, hd * D + d);
  float cq = 0.f, co = 0.f, c_lse_in = -INFINITY;
  if (a.calib_mode == 0) { cq = a.c_q[hd * D + d]; co = a.c_out[hd * D + d]; c_lse_in = a.c_lse[hd]; }
  float mm = -INFINITY;
#pragma unroll 8
  for (int s = 0; s < ns; ++s) mm = fmaxf(mm, a.part_ml[slot0 + s].x);
  const float ms = (mm == -INFINITY) ? 0.f : mm;
  float o = 0.f, ll = 0.f;
#pragma unroll 8
  for (int s = 0; s < ns; ++s) {
    const float2 ml = a.part_ml[slot0 + s];
    const float sc = fast_exp2(ml.x - ms);
    o += a.part_o[(slot0 + s) * D + d] * sc;
    ll += ml.y * sc;
  }
  const bool any = ll > 0.f;
  const float o_n = any ? o / ll : 0.f;
  const float lse = any ? (mm + fast_log2(ll)) * kLn2 : -INFINITY;     // natural-log units
  if (a.calib_mode) {
    a.c_q[hd * D + d] = qd;
    a.c_out[hd * D + d] = o_n;
    if (a.calib_mode == 2) {
      // Alg. 2 steps 7-8: the state now belongs to the current query; calibrate this step's output
      const float a_lse = a.a_lse[hd];
      const float aj = any ? 1.f / (1.f + __expf(a_lse - lse)) : 0.f;
      const float o_a = load_elem<T>(static_cast<const T*>(a.out), hd * D + d);
      store_elem<T>(static_cast<T*>(a.out), hd * D + d, (1.f - aj) * o_a + aj * o_n);
      __syncthreads();                 // every thread has read the flag before it changes
      if (d == 0) a.flags[hd] = 3;
    }
    if (d == 0) a.c_lse[hd] = lse;
    return;
  }
  // decode: rho = cos(q_t, c_q) in fp32
  const float dot = block_sum(qd * cq, red, D);
  const float nq2 = block_sum(qd * qd, red, D);
  const float nc2 = block_sum(cq * cq, red, D);
  float rho = 0.f;
  if (nq2 > 0.f && nc2 > 0.f) rho = dot / (sqrtf(nq2) * sqrtf(nc2));
  const float c_lse = c_lse_in;
  uint8_t flag = 0;
  float res = o_n;
  if (rho < a.theta1) {
    flag = 2;
  } else if (rho > a.theta2 && c_lse > -INFINITY) {
    flag = 1;
    // alpha_j = sigmoid(c_lse - a_lse); a_lse = -inf (empty cache) gives alpha_j = 1
    const float aj = 1.f / (1.f + __expf(lse - c_lse));
    res = (1.f - aj) * o_n + aj * co;
  }
  store_elem<T>(static_cast<T*>(a.out), hd * D + d, res);
  if (d == 0) {
    if (a.a_lse) a.a_lse[hd] = lse;
    if (a.flags) a.flags[hd] = flag;
  }
}

struct BitmapArgs {
  const int32_t* seq_off; const int32_t* indices; const int32_t* cal_indices; uint32_t* bitmap;
  int64_t total_tokens;
  int batch, Hkv, B, calib, max_seq_len, W32;
  const uint8_t* only_flagged;   // [batch][Hq] or NULL: KV groups without a head flagged 2 are left alone
  int Hq, G;
};

// Rebuild the skip bitmap of the calibration pass for every (sequence, KV head): either "not
// evicted" from the retained index list, or "not in the calibration set" from that set's list.
__global__ __launch_bounds__(256) void bitmap_from_indices_kernel(BitmapArgs a) {
  const int bg = blockIdx.x;
  const int b = bg / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  uint32_t* bm = a.bitmap + static_cast<int64_t>(bg) * a.W32;
  const int words = (n + 31) / 32;
  const bool from_cal = a.cal_indices != nullptr && a.calib > 0;
  for (int wd = threadIdx.x; wd < words; wd += 256) bm[wd] = from_cal ? 0xFFFFFFFFu : 0u;
  __threadfence();
  __syncthreads();
  if (from_cal) {
    const int32_t* cal = a.cal_indices + static_cast<int64_t>(bg) * a.calib;
    for (int r = threadIdx.x; r < a.calib; r += 256) {
      const int pos = cal[r];
      if (pos >= 0 && pos < n) atomicAnd(&bm[pos >> 5], ~(1u << (pos & 31)));
    }
  } else {
    const int32_t* idx = a.indices + static_cast<int64_t>(bg) * a.B;
    for (int r = threadIdx.x; r < a.B; r += 256) {
      const int pos = idx[r];
      if (pos >= 0 && pos < n) atomicOr(&bm[pos >> 5], 1u << (pos & 31));
    }
  }
}

// The same bitmap built in LDS (W32 words of dynamic shared memory) and written out once, whole words,
// coalesced: the bits are set with LDS atomics instead of one trip to L2 per retained position.
__global__ __launch_bounds__(256) void bitmap_from_indices_lds_kernel(BitmapArgs a) {
  extern __shared__ uint32_t s_bits[];
  const int bg = blockIdx.x;
  const int b = bg / a.Hkv;
  if (a.only_flagged) {
    const int g = bg - b * a.Hkv;
    bool any = false;
    for (int hh = 0; hh < a.G; ++hh) any |= a.only_flagged[b * a.Hq + g * a.G + hh] == 2;
    if (!any) return;                              // the recomputation skips this KV group as well
  }
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  uint32_t* bm = a.bitmap + static_cast<int64_t>(bg) * a.W32;
  const int words = min((n + 31) / 32, a.W32);
  const bool from_cal = a.cal_indices != nullptr && a.calib > 0;
  for (int wd = threadIdx.x; wd < words; wd += 256) s_bits[wd] = from_cal ? 0xFFFFFFFFu : 0u;
  __syncthreads();
  if (from_cal) {
    const int32_t* cal = a.cal_indices + static_cast<int64_t>(bg) * a.calib;
    for (int r = threadIdx.x; r < a.calib; r += 256) {
      const int pos = cal[r];
      if (pos >= 0 && pos < n) atomicAnd(&s_bits[pos >> 5], ~(1u << (pos & 31)));
    }
  } else {
    const int32_t* idx = a.indices + static_cast<int64_t>(bg) * a.B;
    for (int r = threadIdx.x; r < a.B; r += 256) {
      const int pos = idx[r];
      if (pos >= 0 && pos < n) atomicOr(&s_bits[pos >> 5], 1u << (pos & 31));
    }
  }
  __syncthreads();
  for (int wd = threadIdx.x; wd < words; wd += 256) bm[wd] = s_bits[wd];
}

struct DecodeFusedArgs {
  const void* q; const void* k; const void* v;
  const int32_t* row_off; const int32_t* row_len;
  int batch, Hq, Hkv, G, max_len;
  int xcd_blocks;   // 1: workgroups are re-dealt so that each XCD takes a contiguous block of sequences (batch % 8 == 0)
  float sl2, theta1, theta2;
  const float* c_q; const float* c_out; const float* c_lse;
  void* out; float* a_lse; uint8_t* flags;
};

// cos(q, c) of two vectors spread over the wave (lane holds elements lane + 64 u); 0 when either is 0.
template <int N>
__device__ __forceinline__ float cosine_of(const float (&q)[N], const float (&cvec)[N]) {
  float dot = 0.f, nq2 = 0.f, nc2 = 0.f;
#pragma unroll
  for (int u = 0; u < N; ++u) {
    dot += q[u] * cvec[u];
    nq2 += q[u] * q[u];
    nc2 += cvec[u] * cvec[u];
  }
  dot = wave_sum(dot); nq2 = wave_sum(nq2); nc2 = wave_sum(nc2);
  return (nq2 > 0.f && nc2 > 0.f) ? dot / (sqrtf(nq2) * sqrtf(nc2)) : 0.f;
}

// Whole decode step of one (sequence, KV head) in a single workgroup of NW waves: streaming
// attention over the live cache rows (Alg. 2 step 1), merge of the waves' partials by
// Eq. 1-2, cosine gate (step 2) and calibration merge (steps 9-11).  No workspace.
#ifndef CD_DECODE_WAVES_PER_SIMD
#define CD_DECODE_WAVES_PER_SIMD 1
#endif
template <typename T, int D, int NW>
__global__ __launch_bounds__(NW * 64, CD_DECODE_WAVES_PER_SIMD) void decode_fused_kernel(DecodeFusedArgs a) {
  // Workgroups are dealt to the 8 XCDs round-robin in launch order.  With xcd_blocks the launch index
  // is re-read so that XCD x takes the sequences [x * batch/8, (x+1) * batch/8) with all their heads:
  // the outputs, log-sum-exps and flags of neighbouring heads and sequences, which share cache lines,
  // are then written through one L2 instead of eight (measured on long caches: 2-3 % per call).
  int g = blockIdx.x, b = blockIdx.y;
  if (a.xcd_blocks) {
    const int L = static_cast<int>(blockIdx.x + gridDim.x * blockIdx.y);
    const int slot = L >> 3;
    g = slot % static_cast<int>(gridDim.x);
    b = (L & 7) * static_cast<int>(gridDim.y >> 3) + slot / static_cast<int>(gridDim.x);
  }
  const int lane = threadIdx.x & 63, wv = wave_index();
  const int i = lane & 15, c = lane >> 4;
  // row_off == NULL: every sequence has capacity max_len and starts at b * max_len, so the K/V
  // addresses need no load
  const bool uniform = a.row_off == nullptr;
  const int off0 = uniform ? b * a.max_len : a.row_off[b];
  const int cap = uniform ? a.max_len : a.row_off[b + 1] - off0;
  const int len = a.row_len[b];
  const int rows = (len < 0 || len > cap || len > a.max_len) ? 0 : len;
  const int64_t head_tok = static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * cap;
  const T* kbase = static_cast<const T*>(a.k) + head_tok * D;
  const T* vbase = static_cast<const T*>(a.v) + head_tok * D;
  const T* qbase = static_cast<const T*>(a.q) + static_cast<int64_t>(b * a.Hq + g * a.G) * D;

  AttendWave<T, D> w;
  w.init(qbase + static_cast<int64_t>(i) * D, i < a.G, c);

  // The wave's first K rows are requested at once, clamped to the capacity (addressable whatever the
  // number of live rows turns out to be; rows beyond it are masked later): with a uniform layout
  // not a single load has to return before this request can go out.
  if (cap > 0) w.request_first_k(kbase, wv * kTileRows, cap, i, c);

  // Operands of the gate/merge tail (wave wv finishes head wv; groups larger than the wave count loop
  // and reload), requested right behind those K rows - nothing may delay that request - and only
  // looked at (not even converted) once the first tile's loads are all on their way: a conversion at
  // the point of the load would make the wave wait for the data there, a full memory round trip
  // before its stream has started.
  uint32_t qraw[D / 64];      // storage bits of the query elements
  float qd[D / 64], cq[D / 64], co[D / 64];
  float c_lse0 = -INFINITY;
  const bool has_tail = wv < a.G;
  if (has_tail) {
    const int64_t hd = static_cast<int64_t>(b * a.Hq + g * a.G + wv);
#pragma unroll
    for (int u = 0; u < D / 64; ++u) {
      qraw[u] = load_bits<T>(qbase, static_cast<int64_t>(wv) * D + lane + 64 * u);
      cq[u] = a.c_q[hd * D + lane + 64 * u];
      co[u] = a.c_out[hd * D + lane + 64 * u];
    }
    c_lse0 = a.c_lse[hd];
  }
  // (issuing the loads of both tiles of a wave before any arithmetic was measured slower than this
  // one-tile-ahead pipeline: 5 % more time per call at 512 rows)
  // The gate of Alg. 2 step 2 depends on the query and C_q only: wave wv works out the cosine of its
  // head while its first K/V tile is on the way (those operands were requested before the tile).
  // The wave-wide sums are chains of cross-lane exchanges, about a microsecond of pure latency
  // when they sit between the merge barrier and the output store instead.
  float rho0 = 0.f;
  auto gate_cosine = [&]() {
    if (has_tail) {
#pragma unroll
      for (int u = 0; u < D / 64; ++u) {
        // (the empty statement pins the conversion here: the compiler would otherwise move it, and the
        // wait for the data that comes with it, up to the load)
        asm volatile("" : "+v"(qraw[u]) : : "memory");
        qd[u] = bits_to_f32<T>(qraw[u]);
      }
      rho0 = cosine_of(qd, cq);
    }
  };
  w.template run<true, false>(kbase, vbase, nullptr, rows, wv * kTileRows, rows, NW * kTileRows, a.sl2, i, c, nullptr,
                              false, true, gate_cosine);

  extern __shared__ __attribute__((aligned(16))) float s_dyn[];                 // [NW][G][D] outputs, then [NW][G] (max, sum)
  float* s_o = s_dyn;
  float2* s_ml = reinterpret_cast<float2*>(s_dyn + NW * a.G * D);
  w.publish(s_o + wv * a.G * D, s_ml + wv * a.G, a.G, i, c);
  __syncthreads();

  for (int hh = wv; hh < a.G; hh += NW) {           // one wave finishes one head
    const int64_t hd = static_cast<int64_t>(b * a.Hq + g * a.G + hh);
    float c_lse = c_lse0;
    if (hh != wv) {
#pragma unroll
      for (int u = 0; u < D / 64; ++u) {
        qd[u] = load_elem<T>(qbase, static_cast<int64_t>(hh) * D + lane + 64 * u);
        cq[u] = a.c_q[hd * D + lane + 64 * u];
        co[u] = a.c_out[hd * D + lane + 64 * u];
      }
      c_lse = a.c_lse[hd];
    }
    float mm = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) mm = fmaxf(mm, s_ml[ww * a.G + hh].x);
    const float ms = (mm == -INFINITY) ? 0.f : mm;
    float ll = 0.f;
    float o[D / 64];
#pragma unroll
    for (int u = 0; u < D / 64; ++u) o[u] = 0.f;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) {
      const float2 ml = s_ml[ww * a.G + hh];
      const float sc = fast_exp2(ml.x - ms);
      ll += ml.y * sc;
#pragma unroll
      for (int u = 0; u < D / 64; ++u) o[u] += s_o[(ww * a.G + hh) * D + lane + 64 * u] * sc;
    }
    const bool any = ll > 0.f;
    const float lse = any ? (mm + fast_log2(ll)) * kLn2 : -INFINITY;
    const float rho = (hh == wv) ? rho0 : cosine_of(qd, cq);      // groups larger than the wave count recompute
    uint8_t flag = 0;
    float aj = 0.f;
    if (rho < a.theta1) flag = 2;
    else if (rho > a.theta2 && c_lse > -INFINITY) { flag = 1; aj = 1.f / (1.f + __expf(lse - c_lse)); }
#pragma unroll
    for (int u = 0; u < D / 64; ++u) {
      float res = any ? o[u] / ll : 0.f;
      if (flag == 1) res = (1.f - aj) * res + aj * co[u];
      store_elem<T>(static_cast<T*>(a.out), hd * D + lane + 64 * u, res);
    }
    if (lane == 0) {
      if (a.a_lse) a.a_lse[hd] = lse;
      if (a.flags) a.flags[hd] = flag;
    }
  }
}

}  // namespace cd
