// Observation-window scoring of the eviction strategy f (Alg. 1 step 3, SnapKV-style,
// Sec. 4.1.3): S = Q_win K^T on the matrix cores in two passes over K.
//   pass 1 (score_rowstats): per window-query row, max and sum of exp2 of its logits over the
//           keys of one chunk; the chunks are merged into a row log-sum-exp (rowstats_merge).
//   pass 2 (score_votes):    S recomputed, p = exp2(s - lse_row), column sums over the G*w
//           rows of the KV head -> vote[j] for prefix columns j < P.
//   pool_scores: 1-D average pooling of the votes.
// Tile orientation: S^T = K Q^T, i.e. keys are the A rows and query rows the B columns, so a
// lane owns one query row per 16-row tile (cheap running row statistics) and 4 keys.
// A workgroup owns a block of up to 128 query rows (8 tiles) and a chunk of kChunkKeys keys.
#pragma once
#include "cd_common.h"

namespace cd {

constexpr int kRowBlock = 128;     // query rows per workgroup (8 MFMA tiles of 16)
constexpr int kRowTiles = 8;
constexpr int kMinChunkKeys = 256; // keys per workgroup in the scoring passes: a multiple of this

struct ScoreArgs {
  const void* q_win;
  const void* k;
  const int32_t* seq_off;
  int64_t total_tokens;
  int batch, Hq, Hkv, G, w, B, R, NRB, NCH, max_seq_len, pool_k;
  int chunk_keys;       // keys per workgroup (multiple of 64); each wave takes chunk_keys/4 contiguous keys
  float sl2;            // scale * log2(e)
  float2* rowpart;      // [batch*Hkv*NRB*128][NCH] (max, sum) per chunk
  float* row_lse;       // [batch*Hkv*NRB*128] log2-domain row log-sum-exp
  float* vote;          // [NRB][total_tokens*Hkv]
  float* score;         // [total_tokens*Hkv]
};

// Length of sequence b as the kernels use it: 0 when the offsets break the host-side contract
// (so nothing out of bounds is ever touched).
__device__ __forceinline__ int seq_len_checked(const int32_t* seq_off, int b, int max_seq_len,
                                               int64_t total_tokens, int& off0) {
  off0 = seq_off[b];
  int off1 = seq_off[b + 1];
  int n = off1 - off0;
  if (off0 < 0 || n < 0 || n > max_seq_len || static_cast<int64_t>(off1) > total_tokens) return 0;
  return n;
}

template <typename T, int D>
struct ScoreTile {
  static constexpr int EPL = Elem<T>::kPer16B;
  static constexpr int KD = Elem<T>::kStepK;
  static constexpr int NK = D / KD;

  u32x4 qf[kRowTiles][NK];
  int lim[kRowTiles];      // last visible key position of this lane's row in tile rt (-1: none)

  // Fragments of the row block's queries: lane (i, c) holds row 16*rt + i.
  __device__ __forceinline__ void load_q(const ScoreArgs& a, int b, int g, int rb, int P, int i, int c) {
    const T* q = static_cast<const T*>(a.q_win);
#pragma unroll
    for (int rt = 0; rt < kRowTiles; ++rt) {
      int rho = rb * kRowBlock + rt * 16 + i;
      bool valid = rho < a.R;
      int hh = valid ? rho / a.w : 0;
      int wi = valid ? rho - hh * a.w : 0;
      const T* qp = q + (static_cast<int64_t>(b * a.Hq + g * a.G + hh) * a.w + wi) * D + c * EPL;
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) qf[rt][kk] = valid ? ld16(qp + kk * KD) : zero16();
      lim[rt] = valid ? P + wi : -1;
    }
  }

  // Key fragments of the 16-key tile starting at key0 (rows clamped to the sequence).
  __device__ __forceinline__ void load_k(const T* kbase, int key0, int n, int i, int c, u32x4 (&kf)[NK]) const {
    int krow = min(key0 + i, n - 1);
    const T* kp = kbase + static_cast<int64_t>(krow) * D + c * EPL;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) kf[kk] = ld16(kp + kk * KD);
  }

  // acc[rt][r] = raw dot product of key (key0 + 4c + r) with query row (16 rt + i).
  __device__ __forceinline__ void logits(const u32x4 (&kf)[NK], f32x4 (&acc)[kRowTiles]) const {
#pragma unroll
    for (int rt = 0; rt < kRowTiles; ++rt) {
      acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) mma_step<T>(acc[rt], kf[kk], qf[rt][kk]);
    }
  }
};

template <typename T, int D>
__global__ __launch_bounds__(256) void score_rowstats_kernel(ScoreArgs a) {
  const int chunk = blockIdx.x;
  const int y = blockIdx.y;
  const int rb = y % a.NRB;
  const int bg = y / a.NRB;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  if (n <= a.B) return;
  const int key_base = chunk * a.chunk_keys;
  if (key_base >= n) return;
  const int P = n - a.w;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int i = lane & 15, c = lane >> 4;
  const T* kbase = static_cast<const T*>(a.k) + (static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n) * D;

  ScoreTile<T, D> st;
  st.load_q(a, b, g, rb, P, i, c);
  float m[kRowTiles], l[kRowTiles];
#pragma unroll
  for (int rt = 0; rt < kRowTiles; ++rt) { m[rt] = -INFINITY; l[rt] = 0.f; }

  const int wave_keys = a.chunk_keys >> 2;
  const int wave_first = key_base + wv * wave_keys;
  const int wave_end = min(n, wave_first + wave_keys);
  if (wave_first < wave_end) {
    u32x4 kf[ScoreTile<T, D>::NK];
    st.load_k(kbase, wave_first, n, i, c, kf);
    for (int key0 = wave_first; key0 < wave_end; key0 += 16) {
      f32x4 acc[kRowTiles];
      st.logits(kf, acc);
      if (key0 + 16 < wave_end) st.load_k(kbase, key0 + 16, n, i, c, kf);   // next tile in flight
      const int kfirst = key0 + 4 * c;
      float x[kRowTiles][4];
      float tm[kRowTiles];
      bool grow = false;
#pragma unroll
      for (int rt = 0; rt < kRowTiles; ++rt) {
#pragma unroll
        for (int r = 0; r < 4; ++r) x[rt][r] = (kfirst + r <= st.lim[rt]) ? acc[rt][r] * a.sl2 : -INFINITY;
        tm[rt] = fmaxf(fmaxf(x[rt][0], x[rt][1]), fmaxf(x[rt][2], x[rt][3]));
        grow |= tm[rt] > m[rt];
      }
      if (__any(grow)) {                 // some row's running maximum rises: rescale its sum
#pragma unroll
        for (int rt = 0; rt < kRowTiles; ++rt) {
          const float mn = fmaxf(m[rt], tm[rt]);
          const float ms = (mn == -INFINITY) ? 0.f : mn;
          l[rt] *= fast_exp2(m[rt] - ms);
          m[rt] = mn;
        }
      }
#pragma unroll
      for (int rt = 0; rt < kRowTiles; ++rt) {
        const float ms = (m[rt] == -INFINITY) ? 0.f : m[rt];
        l[rt] += (fast_exp2(x[rt][0] - ms) + fast_exp2(x[rt][1] - ms)) + (fast_exp2(x[rt][2] - ms) + fast_exp2(x[rt][3] - ms));
      }
    }
  }
  // merge the four lanes that hold the same row (different keys), then the four waves
  __shared__ float2 sm[4][kRowBlock];
#pragma unroll
  for (int rt = 0; rt < kRowTiles; ++rt) {
    merge_ml(m[rt], l[rt], __shfl_xor(m[rt], 16), __shfl_xor(l[rt], 16));
    merge_ml(m[rt], l[rt], __shfl_xor(m[rt], 32), __shfl_xor(l[rt], 32));
    if (c == 0) sm[wv][rt * 16 + i] = make_float2(m[rt], l[rt]);
  }
  __syncthreads();
  if (threadIdx.x < kRowBlock) {
    float mm = sm[0][threadIdx.x].x, ll = sm[0][threadIdx.x].y;
#pragma unroll
    for (int ww = 1; ww < 4; ++ww) merge_ml(mm, ll, sm[ww][threadIdx.x].x, sm[ww][threadIdx.x].y);
    a.rowpart[(static_cast<int64_t>(y) * kRowBlock + threadIdx.x) * a.NCH + chunk] = make_float2(mm, ll);
  }
}

// One wave per query row: merge its chunk partials into the log2-domain row log-sum-exp.
__global__ __launch_bounds__(256) void rowstats_merge_kernel(ScoreArgs a) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int64_t gr = static_cast<int64_t>(blockIdx.x) * 4 + wv;
  const int64_t rows_total = static_cast<int64_t>(a.batch) * a.Hkv * a.NRB * kRowBlock;
  if (gr >= rows_total) return;
  const int y = static_cast<int>(gr / kRowBlock);
  const int b = y / (a.NRB * a.Hkv);
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  if (n <= a.B) return;
  const int nch = (n + a.chunk_keys - 1) / a.chunk_keys;
  float m = -INFINITY, l = 0.f;
  for (int ch = lane; ch < nch; ch += 64) {
    float2 v = a.rowpart[gr * a.NCH + ch];
    merge_ml(m, l, v.x, v.y);
  }
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) merge_ml(m, l, __shfl_xor(m, s), __shfl_xor(l, s));
  if (lane == 0) a.row_lse[gr] = (l > 0.f) ? m + fast_log2(l) : INFINITY;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void score_votes_kernel(ScoreArgs a) {
  const int chunk = blockIdx.x;
  const int y = blockIdx.y;
  const int rb = y % a.NRB;
  const int bg = y / a.NRB;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  if (n <= a.B) return;
  const int P = n - a.w;
  const int key_base = chunk * a.chunk_keys;
  if (key_base >= P) return;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int i = lane & 15, c = lane >> 4;
  const int64_t head_tok = static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n;
  const T* kbase = static_cast<const T*>(a.k) + head_tok * D;
  float* vote = a.vote + static_cast<int64_t>(rb) * a.total_tokens * a.Hkv + head_tok;

  ScoreTile<T, D> st;
  st.load_q(a, b, g, rb, P, i, c);
  float lse[kRowTiles];
#pragma unroll
  for (int rt = 0; rt < kRowTiles; ++rt) lse[rt] = a.row_lse[static_cast<int64_t>(y) * kRowBlock + rt * 16 + i];

  const int wave_keys = a.chunk_keys >> 2;
  const int wave_first = key_base + wv * wave_keys;
  const int wave_end = min(P, wave_first + wave_keys);
  if (wave_first >= wave_end) return;
  u32x4 kf[ScoreTile<T, D>::NK];
  st.load_k(kbase, wave_first, n, i, c, kf);
  for (int key0 = wave_first; key0 < wave_end; key0 += 16) {
    f32x4 acc[kRowTiles];
    st.logits(kf, acc);
    if (key0 + 16 < wave_end) st.load_k(kbase, key0 + 16, n, i, c, kf);     // next tile in flight
    float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int rt = 0; rt < kRowTiles; ++rt) {
#pragma unroll
      for (int r = 0; r < 4; ++r) v[r] += fast_exp2(acc[rt][r] * a.sl2 - lse[rt]);   // padded rows: lse = +inf -> 0
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r] = row16_sum(v[r]);
    if (i == 0) {
      const int kfirst = key0 + 4 * c;
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (kfirst + r < P) vote[kfirst + r] = v[r];
    }
  }
}

// score[j] = (1/k) * sum_{d=-k/2..k/2} vote[j+d], zero outside [0, P); votes of the row
// blocks are added first, always in the same order.
__global__ __launch_bounds__(256) void pool_scores_kernel(ScoreArgs a) {
  const int bg = blockIdx.y;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  if (n <= a.B) return;
  const int P = n - a.w;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= P) return;
  const int64_t head_tok = static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n;
  const int64_t plane = a.total_tokens * a.Hkv;
  const int half = a.pool_k / 2;
  float sum = 0.f;
  for (int d = -half; d <= half; ++d) {
    int jj = j + d;
    float val = 0.f;
    if (jj >= 0 && jj < P) {
      for (int rb = 0; rb < a.NRB; ++rb) val += a.vote[rb * plane + head_tok + jj];
    }
    sum += val;
  }
  a.score[head_tok + j] = sum / static_cast<float>(a.pool_k);
}

}  // namespace cd
