// H2O as the eviction strategy f of Alg. 1 step 3 (Sec. 4.1.3: importance = accumulated
// attention score): every prompt query attends causally to the prompt, and a position's score
// is the probability mass it received, summed over all queries and over the G query heads of
// its KV head.  Unlike the observation-window scoring this is a dense n x n contraction per head
// (matrix-core bound), done in two passes that mirror each other:
//   pass 1 (h2o_rowlse): query rows stay in registers, keys stream through LDS; a lane owns a
//           query row, so the running (max, sum exp2) of its softmax stay in the lane -> row
//           log-sum-exp for every prompt position.
//   pass 2 (h2o_votes):  keys stay in registers, query rows stream through LDS; a lane owns a
//           key, so the column sum of p = exp2(s - lse_row) over all rows that see the key stays
//           in the lane -> vote[j], written once, no atomics, fixed summation order.
// Both passes skip the tiles above the diagonal and mask only the tiles on it.
#pragma once
#include "cd_common.h"
#include "cd_score.h"

namespace cd {

#ifndef CD_H2O_ROW_TILES
#define CD_H2O_ROW_TILES 2     // 16-row tiles of stationary rows per wave (build-time tuning knob)
#endif

struct H2oArgs {
  const void* q_full;        // packed like K with Hq heads: sequence b at token seq_off[b], inside [Hq][n_b][D]
  const void* k;
  const int32_t* seq_off;
  int64_t total_tokens;
  int batch, Hq, Hkv, G, B, max_seq_len;
  int lse_stride;            // floats per (sequence, query head) in row_lse; a multiple of the row block
  float sl2;                 // scale * log2(e)
  float* row_lse;            // [batch*Hq][lse_stride], log2 units; rows >= n_b hold +inf
  float* vote;               // [G][plane]: one plane per query head of the group, each packed like K with one float per row
  int64_t plane;             // floats per plane: total_tokens*Hkv rounded up to a multiple of 64
  void* q_last;              // [batch][Hq][D]: the last prompt query of every head (Q_{-1})
};

// RT = 16-row tiles of stationary rows per wave (a workgroup holds 4 * 16 * RT of them).
template <typename T, int D, int RT>
__global__ __launch_bounds__(256) void h2o_rowlse_kernel(H2oArgs a) {
  using KS = KeyStream<T, D>;
  constexpr int KT = KS::KT, NK = KS::NK, SK = KS::kStageKeys, EPL = KS::EPL, KD = KS::KD;
  constexpr int WR = 16 * RT, BR = 4 * WR;
  int vx, vh;                                    // row block and (sequence, query head) of this workgroup
  xcd_head_major(vx, vh);
  const int hq = vh % a.Hq, b = vh / a.Hq, g = hq / a.G;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  const T* qbase = static_cast<const T*>(a.q_full) + (static_cast<int64_t>(off0) * a.Hq + static_cast<int64_t>(hq) * n) * D;
  // Q_{-1} of this head, the calibration query of Alg. 1 step 5 (also for prompts within the budget)
  if (vx == 0 && n > 0 && threadIdx.x < D)
    store_elem<T>(static_cast<T*>(a.q_last), static_cast<int64_t>(b * a.Hq + hq) * D + threadIdx.x,
                  load_elem<T>(qbase, static_cast<int64_t>(n - 1) * D + threadIdx.x));
  if (n <= a.B) return;
  const int nrb = (n + BR - 1) / BR;
  const int rbp = nrb - 1 - vx;                  // late rows (most keys) are launched first
  if (rbp < 0) return;
  const int i0 = rbp * BR;
  const int lane = threadIdx.x & 63, wv = wave_index();
  const int i = lane & 15, c = lane >> 4;
  const T* kbase = static_cast<const T*>(a.k) + (static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n) * D;
  const int wrow0 = i0 + wv * WR;                // first row of this wave

  __shared__ __attribute__((aligned(16))) char s_k[2][KS::kStageBytes];
  u32x4 qf[RT][NK];
  int lim[RT];                                   // last key the row sees (= its position), -1 for padding rows
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int row = wrow0 + rt * 16 + i;
    const bool valid = row < n;
    const T* qp = qbase + static_cast<int64_t>(valid ? row : 0) * D + c * EPL;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) qf[rt][kk] = valid ? ld16(qp + kk * KD) : zero16();
    lim[rt] = valid ? row : -1;
  }
  float m[RT], l[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) { m[rt] = -INFINITY; l[rt] = 0.f; }

  const int key_end = min(n, i0 + BR);           // no row of the block sees a key beyond its last row
  const int nstages = (key_end + SK - 1) / SK;
  KeyStreamDirect<T, D> ks;
  ks.init();
  ks.issue(kbase, 0, n, s_k[0]);

  // S^T tile kt of a stage: keys 16 kt .. 16 kt + 15 against this wave's rows
  auto mma_tile = [&](const char* lds, int kt, f32x4 (&acc)[RT]) {
    u32x4 kf[NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) kf[kk] = KS::frag(lds, kt, kk, i, c);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) mma_step<T>(acc[rt], kf[kk], qf[rt][kk]);
    }
  };
  // acc[rt][r] <-> key kfirst + r, row (rt, i)
  auto softmax_tile = [&](const f32x4 (&acc)[RT], int kfirst, bool full, bool first) {
    if (full) {
      // The sum is taken against a reference m that need not be the row maximum: m + log2(sum of
      // exp2(s - m)) is the same number for any m that keeps the terms in range.  The reference is
      // the logit of key 0 (every row sees it); only when a sum outgrows 2^64 is the tile redone
      // against its true maximum.  This saves the running-maximum arithmetic on every tile.
      if (first) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) m[rt] = __shfl(acc[rt][0] * a.sl2, i);     // lane (i, c = 0), r = 0: key 0
      }
      float l_old[RT];
      bool big = false;
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        l_old[rt] = l[rt];
        const float nm = -m[rt];
        l[rt] += (fast_exp2(fmaf(acc[rt][0], a.sl2, nm)) + fast_exp2(fmaf(acc[rt][1], a.sl2, nm))) +
                 (fast_exp2(fmaf(acc[rt][2], a.sl2, nm)) + fast_exp2(fmaf(acc[rt][3], a.sl2, nm)));
        big |= !(l[rt] <= 0x1p+64f);
      }
      if (__any(big)) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          const float tm = fmaxf(fmaxf(acc[rt][0], acc[rt][1]), fmaxf(acc[rt][2], acc[rt][3])) * a.sl2;
          const float mn = fmaxf(m[rt], tm);
          const float nm = -mn;
          l[rt] = l_old[rt] * fast_exp2(m[rt] - mn) +
                  ((fast_exp2(fmaf(acc[rt][0], a.sl2, nm)) + fast_exp2(fmaf(acc[rt][1], a.sl2, nm))) +
                   (fast_exp2(fmaf(acc[rt][2], a.sl2, nm)) + fast_exp2(fmaf(acc[rt][3], a.sl2, nm))));
          m[rt] = mn;
        }
      }
    } else {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        float x[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = (kfirst + r <= lim[rt]) ? acc[rt][r] * a.sl2 : -INFINITY;
        const float tm = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
        const float mn = fmaxf(m[rt], tm);
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        l[rt] = l[rt] * fast_exp2(m[rt] - ms) +
                ((fast_exp2(x[0] - ms) + fast_exp2(x[1] - ms)) + (fast_exp2(x[2] - ms) + fast_exp2(x[3] - ms)));
        m[rt] = mn;
      }
    }
  };
  // One stage.  The matrix products of tile kt+1 are issued before the softmax arithmetic of
  // tile kt, so that the matrix cores and the vector ALU of this wave work at the same time.
  auto compute = [&](const char* lds, int key0) {
    if (key0 > wrow0 + WR - 1 || wrow0 >= n) return;        // nothing of this stage is visible to the wave
    const bool full = key0 + SK - 1 <= wrow0 && wrow0 + WR <= n;   // every key visible to every (real) row
    f32x4 acc[2][RT];
    mma_tile(lds, 0, acc[0]);
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      if (kt + 1 < KT) mma_tile(lds, kt + 1, acc[(kt + 1) & 1]);
      softmax_tile(acc[kt & 1], key0 + 16 * kt + 4 * c, full, key0 == 0 && kt == 0);
    }
  };

  // stage s is computed from buffer s & 1 while the loads of stage s + 1 fill the other one; the
  // barrier both publishes stage s and says that everyone is done reading the buffer about to be
  // refilled
  for (int s = 0; s < nstages; ++s) {
    ks.wait_all();
    __syncthreads();
    if (s + 1 < nstages) ks.issue(kbase, (s + 1) * SK, n, s_k[(s + 1) & 1]);
    compute(s_k[s & 1], s * SK);
  }

  // merge the four lanes that hold the same row (different keys); padding rows get +inf so that
  // pass 2 turns them into probability 0
  float* out = a.row_lse + static_cast<int64_t>(b * a.Hq + hq) * a.lse_stride;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    merge_ml(m[rt], l[rt], __shfl_xor(m[rt], 16), __shfl_xor(l[rt], 16));
    merge_ml(m[rt], l[rt], __shfl_xor(m[rt], 32), __shfl_xor(l[rt], 32));
    const int row = wrow0 + rt * 16 + i;
    if (c == 0 && row < a.lse_stride) out[row] = (row < n && l[rt] > 0.f) ? m[rt] + fast_log2(l[rt]) : INFINITY;
  }
}

template <typename T, int D, int RT>
__global__ __launch_bounds__(256) void h2o_votes_kernel(H2oArgs a) {
  using KS = KeyStream<T, D>;
  constexpr int KT = KS::KT, NK = KS::NK, SK = KS::kStageKeys, EPL = KS::EPL, KD = KS::KD;
  constexpr int WR = 16 * RT, BR = 4 * WR;
  // grid: x = pair of key blocks (block x and its mirror nblk-1-x: early keys are seen by many
  // rows, late keys by few, so every workgroup gets the same amount of work), y = (sequence, KV
  // head), z = query head of the group; each query head writes its own plane of votes, which
  // the selection adds up in a fixed order.
  int vx, vh;                                    // block pair and ((sequence, KV head), head in group) of this workgroup
  xcd_head_major(vx, vh);
  const int bg = vh / static_cast<int>(gridDim.z), hh = vh % static_cast<int>(gridDim.z);   // a group's heads side by side
  const int g = bg % a.Hkv, b = bg / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  if (n <= a.B) return;
  const int nblk = (n + BR - 1) / BR;
  const int lane = threadIdx.x & 63, wv = wave_index();
  const int i = lane & 15, c = lane >> 4;
  const int64_t head_tok = static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n;
  const T* kbase = static_cast<const T*>(a.k) + head_tok * D;
  const int hq = g * a.G + hh;
  const T* qbase = static_cast<const T*>(a.q_full) + (static_cast<int64_t>(off0) * a.Hq + static_cast<int64_t>(hq) * n) * D;
  const float* lse_row = a.row_lse + static_cast<int64_t>(b * a.Hq + hq) * a.lse_stride;
  float* vote = a.vote + static_cast<int64_t>(hh) * a.plane + head_tok;

  __shared__ __attribute__((aligned(16))) char s_q[2][KS::kStageBytes];
  __shared__ __attribute__((aligned(16))) float s_z[2][64];      // row log-sum-exp of the staged rows
  KeyStreamDirect<T, D> ks;
  ks.init();

  for (int job = 0; job < 2; ++job) {
    const int blk = job == 0 ? vx : nblk - 1 - vx;
    // uniform over the workgroup: the first half of the blocks as job 0, their mirrors as job 1
    if (job == 0 ? 2 * blk >= nblk : (blk < 0 || blk <= vx)) continue;
    const int j0 = blk * BR;
    const int wkey0 = j0 + wv * WR;                // first key of this wave
    u32x4 kf[RT][NK];
    int kpos[RT];                                  // position of the lane's key; beyond every row for padding keys
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int key = wkey0 + rt * 16 + i;
      const bool valid = key < n;
      const T* kp = kbase + static_cast<int64_t>(valid ? key : 0) * D + c * EPL;
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) kf[rt][kk] = valid ? ld16(kp + kk * KD) : zero16();
      kpos[rt] = valid ? key : 0x7fffffff;
    }
    float v[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) v[rt] = 0.f;

    // streamed rows: j0 .. n-1 of this query head, SK per stage, with their log-sum-exp
    const int nstages = (n - j0 + SK - 1) / SK;
    auto issue = [&](int s) {                      // rows and their log-sum-exp, straight into LDS
      const int q0 = j0 + s * SK;
      ks.issue(qbase, q0, n, s_q[s & 1]);
      if (threadIdx.x < SK) load_to_lds4(lse_row + q0 + threadIdx.x, &s_z[s & 1][0]);
    };
    __syncthreads();                               // the previous job is done with the buffers
    issue(0);

    // S^T tile kt of a stage: rows 16 kt .. 16 kt + 15 of the stage against this wave's keys
    auto mma_tile = [&](const char* lds, int kt, f32x4 (&acc)[RT]) {
      u32x4 qf[NK];
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) qf[kk] = KS::frag(lds, kt, kk, i, c);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) mma_step<T>(acc[rt], qf[kk], kf[rt][kk]);
      }
    };
    // the matrix products of tile kt+1 are issued before the exponentials of tile kt
    auto compute = [&](int buf, int s) {
      const int q0 = j0 + s * SK;
      if (q0 + SK - 1 < wkey0 || wkey0 >= n) return;          // no row of the stage sees a key of this wave
      const bool full = q0 >= wkey0 + WR - 1;                  // every row sees every key of the wave
      const char* lds = s_q[buf];
      f32x4 acc[2][RT];
      mma_tile(lds, 0, acc[0]);
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        if (kt + 1 < KT) mma_tile(lds, kt + 1, acc[(kt + 1) & 1]);
        const f32x4 z = *reinterpret_cast<const f32x4*>(&s_z[buf][16 * kt + 4 * c]);   // rows q0+16kt+4c+r; +inf beyond n
        const int qfirst = q0 + 16 * kt + 4 * c;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          const f32x4& t = acc[kt & 1][rt];                    // t[r] <-> row qfirst + r, key (rt, i)
          if (full) {
            v[rt] += (fast_exp2(fmaf(t[0], a.sl2, -z[0])) + fast_exp2(fmaf(t[1], a.sl2, -z[1]))) +
                     (fast_exp2(fmaf(t[2], a.sl2, -z[2])) + fast_exp2(fmaf(t[3], a.sl2, -z[3])));
          } else {
            float p[4];
#pragma unroll
            for (int r = 0; r < 4; ++r)
              p[r] = (qfirst + r >= kpos[rt]) ? fast_exp2(fmaf(t[r], a.sl2, -z[r])) : 0.f;
            v[rt] += (p[0] + p[1]) + (p[2] + p[3]);
          }
        }
      }
    };

    for (int s = 0; s < nstages; ++s) {
      ks.wait_all();
      __syncthreads();
      if (s + 1 < nstages) issue(s + 1);
      compute(s & 1, s);
    }

#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const float tot = col4_sum(v[rt]);           // the four row groups c, fixed tree
      const int key = wkey0 + rt * 16 + i;
      if (c == 0 && key < n) vote[key] = tot;
    }
  }
}

}  // namespace cd
