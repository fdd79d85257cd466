// Observation-window scoring of the eviction strategy f (Alg. 1 step 3, SnapKV-style,
// Sec. 4.1.3): S = Q_win K^T on the matrix cores in two passes over K.
//   pass 1 (score_rowstats): per window-query row, max and sum of exp2 of its logits over the
//           keys of one chunk; the chunks are merged into a row log-sum-exp (rowstats_merge).
//   pass 2 (score_votes):    S recomputed, p = exp2(s - lse_row), column sums over the G*w
//           rows of the KV head -> vote[j] for prefix columns j < P.
//   pool_scores: 1-D average pooling of the votes.
// A workgroup owns a block of query rows (128, or 256 when the KV head has more than 128 - so that
// such heads stream their keys once per pass, not once per 128 rows) and a chunk of keys; its waves
// own 32 or 64 rows each and share the key tiles through LDS.  Pass 1 forms S^T = K Q^T (a lane owns
// one query row per tile: running row statistics stay in registers); pass 2 forms S = Q K^T (a
// lane owns one key: the column sum over rows is an in-lane sum plus a 4-lane tree).
#pragma once
#include "cd_common.h"

namespace cd {

constexpr int kRowBlock = 128;     // query rows per workgroup, doubled for KV heads with more than 128 window rows
#define CD_VOTES_WAVES 4          // waves per SIMD the bf16 vote kernel is compiled for
constexpr int kMaxCalHeads = 8;    // largest GQA group whose calibration logits the vote pass exports
constexpr int kMinChunkKeys = 256; // keys per workgroup in the scoring passes: a multiple of this

struct ScoreArgs {
  const void* q_win;
  const void* k;
  const int32_t* seq_off;
  int64_t total_tokens;
  int batch, Hq, Hkv, G, w, B, R, NRB, NCH, max_seq_len, pool_k;
  int RB;               // window-query rows per row block: 128, or 256 when a KV head has more than 128 (R = G*w)
  int row_stride;       // rows per KV head in rowpart / row_lse: NRB * RB
  int chunk_keys;       // keys per workgroup (multiple of 64); each wave takes chunk_keys/4 contiguous keys
  float sl2;            // scale * log2(e)
  int keep_k;           // pass 1 leaves K in the last-level cache for pass 2 (K of the whole call fits it)
  float2* rowpart;      // [batch*Hkv][row_stride][NCH] (max, sum) per chunk
  float* row_lse;       // [batch*Hkv][row_stride] log2-domain row log-sum-exp (+inf for padding rows)
  float* vote;          // [NRB][plane]: one plane of votes per row block, each packed like K with one float per row
  int64_t plane;        // floats per plane: total_tokens*Hkv rounded up to a multiple of 64 (planes stay 256-byte aligned)
  float* score;         // [total_tokens*Hkv]
  float* cal_logit;     // [batch*Hq][zstride] log2-unit logits of the last window query, or NULL
  int zstride;
  uint32_t* zero_words; // pool_scores_kernel only: [batch*Hkv][zero_per_head] words to clear, or NULL
  int zero_per_head;
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

// Layout of a stage of keys in LDS, shared by the waves of a workgroup (which own different query
// rows and all read every key tile from LDS instead of each loading it from memory).  LDS rows
// are 16-byte chunks stored at chunk' = chunk ^ swz(key), chosen so that 16 consecutive lanes
// always touch 16 different 16-byte bank groups of a 256-byte window, both for row-wise writes
// (lanes = consecutive chunks) and for the column-wise fragment reads (lanes = consecutive keys).
template <typename T, int D, int NT = 256>
struct KeyStream {
  static constexpr int EPL = Elem<T>::kPer16B;
  static constexpr int KD = Elem<T>::kStepK;
  static constexpr int NK = D / KD;
  static constexpr int kStageKeys = sizeof(T) == 2 ? 64 : 32;
  static constexpr int KT = kStageKeys / 16;                       // key tiles per stage
  static constexpr int CH = D * static_cast<int>(sizeof(T)) / 16;  // 16-byte chunks per key row
  static constexpr int NLD = kStageKeys * CH / NT;                 // loads per thread per stage
  static constexpr int kStageBytes = kStageKeys * CH * 16;
  static_assert(CH == 8 || CH == 16 || CH == 32, "row size not covered by the LDS swizzle");
  __device__ __forceinline__ static int swz(int key) { return CH == 8 ? ((key >> 1) & 7) : (key & 15); }

  // fragment of key tile kt for mma step kk: lane (i, c) gets key 16 kt + i, chunk 4 kk + c
  __device__ __forceinline__ static u32x4 frag(const char* lds, int kt, int kk, int i, int c) {
    const int key = 16 * kt + i;
    return ld16(lds + key * (CH * 16) + (((4 * kk + c) ^ swz(key)) * 16));
  }
};

// The same stage layout filled by LDS-direct loads: every lane fetches the 16-byte chunk that
// belongs in "its" LDS slot (slot = threadIdx.x + NT u, in the swizzled order above) and the
// load unit writes it there, so the stage needs no staging registers and no LDS store
// instructions.  A wave instruction fills 1 KiB of contiguous LDS; the caller waits for its
// own loads (vmcnt) before the workgroup barrier that publishes the stage.
template <typename T, int D, int NT = 256>
struct KeyStreamDirect {
  using KS = KeyStream<T, D, NT>;
  static constexpr int CH = KS::CH, NLD = KS::NLD, kStageKeys = KS::kStageKeys;
  int goff[NLD];         // byte offset, inside an in-range stage, of the chunk for slot threadIdx.x + NT u
  int lkey[NLD], lch[NLD];   // the slot's stage-local key and its global chunk index (for the clamped tail)

  __device__ __forceinline__ void init() {
#pragma unroll
    for (int u = 0; u < NLD; ++u) {
      const int slot = threadIdx.x + u * NT;
      const int key = slot / CH, chp = slot % CH;
      lkey[u] = key;
      lch[u] = chp ^ KS::swz(key);
      goff[u] = key * (CH * 16) + lch[u] * 16;
    }
  }
  // kStream: the rows are read once and not again soon - non-temporal loads
  template <bool kStream = false>
  __device__ __forceinline__ void issue(const T* kbase, int key0, int n, char* lds) const {
    const char* base = reinterpret_cast<const char*>(kbase);
    char* dst = lds + (threadIdx.x >> 6) * 1024;           // wave-uniform
    if (key0 + kStageKeys <= n) {
      const char* sbase = base + static_cast<int64_t>(key0) * (CH * 16);
#pragma unroll
      for (int u = 0; u < NLD; ++u) {
        if constexpr (kStream) load_to_lds16_stream(sbase + goff[u], dst + u * (NT * 16));
        else load_to_lds16(sbase + goff[u], dst + u * (NT * 16));
      }
    } else {
#pragma unroll
      for (int u = 0; u < NLD; ++u) {
        const int key = min(key0 + lkey[u], n - 1);          // the tail repeats the last row
        load_to_lds16(base + static_cast<int64_t>(key) * (CH * 16) + lch[u] * 16, dst + u * (NT * 16));
      }
    }
  }
  // all LDS-direct loads this wave has issued have landed
  __device__ __forceinline__ static void wait_all() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
};

// Query fragments of the 32 rows a wave owns: lane (i, c) holds row 16 rt + i of the wave.
template <typename T, int D>
struct WaveQueries {
  static constexpr int EPL = Elem<T>::kPer16B;
  static constexpr int KD = Elem<T>::kStepK;
  static constexpr int NK = D / KD;
  u32x4 qf[2][NK];
  int lim[2];        // last visible key position of row (rt, i), -1 for padding rows
  bool any_rows;     // wave-uniform: this wave owns at least one real row

  // row0: first row (inside the KV head) of the 32 rows of this wave
  __device__ __forceinline__ void load(const ScoreArgs& a, int b, int g, int row0, int P, int i, int c) {
    const T* q = static_cast<const T*>(a.q_win);
    any_rows = row0 < a.R;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const int rho = row0 + rt * 16 + i;
      const bool valid = rho < a.R;
      const int hh = valid ? rho / a.w : 0;
      const int wi = valid ? rho - hh * a.w : 0;
      const T* qp = q + (static_cast<int64_t>(b * a.Hq + g * a.G + hh) * a.w + wi) * D + c * EPL;
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) qf[rt][kk] = valid ? ld16(qp + kk * KD) : zero16();
      lim[rt] = valid ? P + wi : -1;
    }
  }
};

// Pass 1 with the key stream loaded straight into LDS (no staging registers, one barrier per stage)
// and the matrix products of the next key tile issued ahead of the exponentials of the current one.
// A workgroup of 4 waves keeps 64 RT window-query rows stationary (RT = 2: 128 rows; RT = 4: 256 rows,
// so that a KV head with up to 256 window rows - G*w - streams its keys once), 16 RT rows per wave.
template <typename T, int D, int RT>
__global__ __launch_bounds__(256) void score_rowstats_direct_kernel(ScoreArgs a) {
  using KS = KeyStream<T, D>;
  constexpr int KT = KS::KT, NK = KS::NK, SK = KS::kStageKeys, EPL = KS::EPL, KD = KS::KD;
  constexpr int WR = 16 * RT, RB = 4 * WR;
  // every chunk of a (sequence, KV head, row block) behind the same L2, so that its query rows are fetched
  // from memory once and not once per XCD; when the rows do not divide over the XCDs, the chunk index is
  // rotated instead so that the chunks every sequence has do not all land on the same XCDs
  int chunk, y;
  if (!xcd_rows_interleaved(chunk, y)) chunk = (chunk + y) % static_cast<int>(gridDim.x);
  const int rb = y % a.NRB;
  const int bg = y / a.NRB;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  if (n <= a.B) return;
  const int key_base = chunk * a.chunk_keys;
  if (key_base >= n) return;
  const int key_end = min(n, key_base + a.chunk_keys);
  const int nstages = (key_end - key_base + SK - 1) / SK;
  const int P = n - a.w;
  const int lane = threadIdx.x & 63, wv = wave_index();
  const int i = lane & 15, c = lane >> 4;
  const T* kbase = static_cast<const T*>(a.k) + (static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n) * D;

  __shared__ __attribute__((aligned(16))) char s_k[2][KS::kStageBytes];
  KeyStreamDirect<T, D> ks;
  ks.init();
  if (a.keep_k) ks.template issue<false>(kbase, key_base, n, s_k[0]);
  else ks.template issue<true>(kbase, key_base, n, s_k[0]);

  // stationary rows: row (rt, i) of this wave is row rb*RB + wv*WR + 16 rt + i of the KV head
  const T* q = static_cast<const T*>(a.q_win);
  u32x4 qf[RT][NK];
  int lim[RT];                                   // last key the row sees, -1 for padding rows
  const bool any_rows = rb * RB + wv * WR < a.R;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int rho = rb * RB + wv * WR + rt * 16 + i;
    const bool valid = rho < a.R;
    const int hh = valid ? rho / a.w : 0;
    const int wi = valid ? rho - hh * a.w : 0;
    const T* qp = q + (static_cast<int64_t>(b * a.Hq + g * a.G + hh) * a.w + wi) * D + c * EPL;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) qf[rt][kk] = valid ? ld16(qp + kk * KD) : zero16();
    lim[rt] = valid ? P + wi : -1;
  }
  float m[RT], l[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) { m[rt] = -INFINITY; l[rt] = 0.f; }

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
      // every key of the tile is a prefix key, visible to all rows.  The sum is taken against a reference
      // that need not be the maximum (m + log2 sum exp2(s - m) is the same number for any m that keeps
      // the terms in range): the logit of the chunk's first key.  Only when a sum outgrows 2^64 is the
      // tile redone against its true maximum.
      if (first) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) m[rt] = __shfl(acc[rt][0] * a.sl2, i);     // lane (i, c = 0), r = 0: first key
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
      // tile reaches into the window: causal mask per row, and the end of the sequence
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
  auto compute = [&](const char* lds, int key0) {
    if (!any_rows) return;
    const bool full = key0 + SK <= P;
    f32x4 acc[2][RT];
    mma_tile(lds, 0, acc[0]);
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      if (kt + 1 < KT) mma_tile(lds, kt + 1, acc[(kt + 1) & 1]);
      softmax_tile(acc[kt & 1], key0 + 16 * kt + 4 * c, full, key0 == key_base && kt == 0);
    }
  };

  // stage s is computed from buffer s & 1 while the loads of stage s + 1 fill the other one; the
  // barrier both publishes stage s and says that everyone is done reading the buffer about to be refilled
  for (int s = 0; s < nstages; ++s) {
    ks.wait_all();
    __syncthreads();
    if (s + 1 < nstages) {
      if (a.keep_k) ks.template issue<false>(kbase, key_base + (s + 1) * SK, n, s_k[(s + 1) & 1]);
      else ks.template issue<true>(kbase, key_base + (s + 1) * SK, n, s_k[(s + 1) & 1]);
    }
    compute(s_k[s & 1], key_base + s * SK);
  }

  // merge the four lanes that hold the same row (different keys) and write the chunk partial
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    merge_ml(m[rt], l[rt], __shfl_xor(m[rt], 16), __shfl_xor(l[rt], 16));
    merge_ml(m[rt], l[rt], __shfl_xor(m[rt], 32), __shfl_xor(l[rt], 32));
    if (c == 0)
      a.rowpart[(static_cast<int64_t>(bg) * a.row_stride + rb * RB + wv * WR + rt * 16 + i) * a.NCH + chunk] = make_float2(m[rt], l[rt]);
  }
}

// A group of GS lanes (16, or a whole wave of 64 when a row has more than 64 partials) per query row:
// lane j of the group merges the chunk partials j, j + GS, ... in that order, then the GS lane results
// are merged by a fixed tree, into the log2-domain row log-sum-exp.  (A prompt of 131072 tokens has
// hundreds of partials per row: one thread per row spent as long on them as a scoring pass.)
template <int GS>
__global__ __launch_bounds__(256) void rowstats_merge_kernel(ScoreArgs a) {
  const int64_t gr = static_cast<int64_t>(blockIdx.x) * (256 / GS) + threadIdx.x / GS;
  const int lane = threadIdx.x % GS;
  const int64_t rows_total = static_cast<int64_t>(a.batch) * a.Hkv * a.row_stride;
  if (gr >= rows_total) return;
  const int b = static_cast<int>(gr / a.row_stride) / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  if (n <= a.B) return;
  const int rho = static_cast<int>(gr % a.row_stride);    // row inside the KV head
  const int nch = (n + a.chunk_keys - 1) / a.chunk_keys;
  const float2* part = a.rowpart + gr * a.NCH;
  float m = -INFINITY, l = 0.f;
  if (rho < a.R) {                                        // padding rows have no partials worth reading
    for (int ch = lane; ch < nch; ch += GS) {
      const float2 v = part[ch];
      merge_ml(m, l, v.x, v.y);
    }
  }
#pragma unroll
  for (int sft = 1; sft < GS; sft <<= 1) merge_ml(m, l, __shfl_xor(m, sft), __shfl_xor(l, sft));
  if (lane == 0) a.row_lse[gr] = (l > 0.f && rho < a.R) ? m + fast_log2(l) : INFINITY;          // padding rows: +inf
}

// The row log-sum-exp taken from the caller instead of pass 1: win_lse [batch][Hq][w] holds, in
// natural-log units, log sum_j exp(scale q_i.K_j) of window query i over the keys it may attend to
// (positions 0..P+i) - the by-product a prefill attention kernel has for these rows anyway.  One
// thread per row slot; padding rows get +inf like above.
__global__ __launch_bounds__(256) void rowlse_import_kernel(ScoreArgs a, const float* win_lse) {
  const int64_t gr = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int64_t rows_total = static_cast<int64_t>(a.batch) * a.Hkv * a.row_stride;
  if (gr >= rows_total) return;
  const int bg = static_cast<int>(gr / a.row_stride);
  const int g = bg % a.Hkv, b = bg / a.Hkv;
  const int rho = static_cast<int>(gr % a.row_stride);    // row inside the KV head
  float val = INFINITY;
  if (rho < a.R) {
    const int hh = rho / a.w, wi = rho - hh * a.w;
    val = win_lse[(static_cast<int64_t>(b) * a.Hq + g * a.G + hh) * a.w + wi] * kLog2e;
  }
  a.row_lse[gr] = val;
}

// NW waves of 32 rows each: a row block of RB = 32 NW rows (4 waves: 128 rows, 8 waves: 256 rows).
template <typename T, int D, int NW>
__global__ __launch_bounds__(NW * 64, sizeof(T) == 2 ? CD_VOTES_WAVES : 2) void score_votes_kernel(ScoreArgs a) {
  using KS = KeyStream<T, D, NW * 64>;
  constexpr int KT = KS::KT, NK = KS::NK, SK = KS::kStageKeys, RB = 32 * NW;
  // grid: x = key chunk, y = (sequence, KV head, row block).  Workgroups are dealt to the 8 XCDs
  // round-robin in launch order: the launch index is re-read so that every chunk of a y sits behind the
  // same L2 (the stationary query rows are then fetched from memory once, not once per XCD); when y
  // does not divide over the XCDs the chunk index is rotated by y instead, so that with sequences of
  // different lengths the chunks every sequence has do not all land on the same XCDs.
  int chunk, y;
  if (!xcd_rows_interleaved(chunk, y)) chunk = (chunk + y) % static_cast<int>(gridDim.x);
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
  const int key_end = min(P, key_base + a.chunk_keys);
  const int nstages = (key_end - key_base + SK - 1) / SK;
  const int lane = threadIdx.x & 63, wv = wave_index();
  const int i = lane & 15, c = lane >> 4;
  const int64_t head_tok = static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n;
  const T* kbase = static_cast<const T*>(a.k) + head_tok * D;
  float* vote = a.vote + static_cast<int64_t>(rb) * a.plane + head_tok;

  __shared__ __attribute__((aligned(16))) char s_k[2][KS::kStageBytes];
  __shared__ float s_v[2][NW][2][SK];              // partial votes of a stage per wave and pair of row groups
  __shared__ float s_z[2][kMaxCalHeads][SK];       // exported calibration logits of a stage, per head
  WaveQueries<T, D> wq;
  wq.load(a, b, g, rb * RB + wv * 32, P, i, c);
  // S tiles are rows x keys here: lane (i, c) holds key i and rows 16 rt + 4 c + r of the wave
  float lse[2][4];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int r = 0; r < 4; ++r)
      lse[rt][r] = a.row_lse[static_cast<int64_t>(bg) * a.row_stride + rb * RB + wv * 32 + rt * 16 + 4 * c + r];   // padding rows: +inf

  // Rows that are the last window query of a head (the default calibration query, Alg. 1
  // step 5) also export their logits, so that the calibration pass need not read K again.
  // (the export needs w % 4 == 0, so that such a row is always slot r = 3 of its lane)
  int cal_head[2];                      // head in group whose last window row is this lane's (rt, r = 3), or -1
  bool cal_lane = false;
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const int rho = rb * RB + wv * 32 + rt * 16 + 4 * c + 3;
    const bool is_cal = a.cal_logit != nullptr && rho < a.R && (rho % a.w) == a.w - 1;
    cal_head[rt] = is_cal ? rho / a.w : -1;
    cal_lane |= is_cal;
  }
  const bool cal_wave = __any(cal_lane);
  float* zrow = a.cal_logit ? a.cal_logit + static_cast<int64_t>(b * a.Hq + g * a.G) * a.zstride : nullptr;

  // the key stream goes straight into LDS (no staging registers: one more wave per SIMD fits)
  KeyStreamDirect<T, D, NW * 64> ks;
  ks.init();
  ks.template issue<true>(kbase, key_base, n, s_k[0]);

  auto compute = [&](const char* lds, float (*sv)[2][SK], float (*sz)[SK]) {
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      u32x4 kf[NK];
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) kf[kk] = KS::frag(lds, kt, kk, i, c);
      float v = 0.f;
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) mma_step<T>(acc, wq.qf[rt][kk], kf[kk]);
#pragma unroll
        for (int r = 0; r < 4; ++r) v += fast_exp2(fmaf(acc[r], a.sl2, -lse[rt][r]));
        if (cal_wave && cal_head[rt] >= 0) sz[cal_head[rt]][16 * kt + i] = acc[3] * a.sl2;
      }
      // only neighbouring row groups are added here (one lane swap); the rest of the sum is left to the
      // flush: the full four-way reduction costs as many vector instructions per key tile as a third
      // of the exponentials, and keeping all four shares would cost a workgroup per compute unit in LDS
      {
        float lo, hi;
        pair16(v, lo, hi);
        if ((c & 1) == 0) sv[wv][c >> 1][16 * kt + i] = lo + hi;
      }
    }
  };
  // after the stage barrier: add the partial votes in a fixed order (waves ascending, inside a wave
  // (c0 + c1) + (c2 + c3), the inner sums already taken) and store; the second wave stores the exported logits, one coalesced row
  // per head
  auto flush = [&](const float (*sv)[2][SK], const float (*sz)[SK], int key0) {
    if (threadIdx.x < SK) {
      const int key = key0 + threadIdx.x;
      if (key < P) {
        float tot = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww)
          tot += sv[ww][0][threadIdx.x] + sv[ww][1][threadIdx.x];
        __builtin_nontemporal_store(tot, vote + key);    // written once, read by a later kernel: kept out of the caches the K stream uses
      }
    } else if (zrow != nullptr && threadIdx.x >= 64 && threadIdx.x < 64 + SK) {
      const int t = threadIdx.x - 64;
      const int key = key0 + t;
      if (key < P)
        for (int hh = 0; hh < a.G; ++hh)
          if ((hh * a.w + a.w - 1) / RB == rb)             // heads whose last window row is in this row block
            __builtin_nontemporal_store(sz[hh][t], zrow + static_cast<int64_t>(hh) * a.zstride + key);
    }
  };

  // stage s is computed from buffer s & 1 while the loads of stage s + 1 fill the other one; the barrier
  // publishes stage s, says that everyone is done reading the buffer about to be refilled, and hands
  // the partial votes of stage s - 1 to the flush
  for (int s = 0; s < nstages; ++s) {
    ks.wait_all();
    __syncthreads();
    if (s + 1 < nstages) ks.template issue<true>(kbase, key_base + (s + 1) * SK, n, s_k[(s + 1) & 1]);
    if (s > 0) flush(s_v[(s - 1) & 1], s_z[(s - 1) & 1], key_base + (s - 1) * SK);
    compute(s_k[s & 1], s_v[s & 1], s_z[s & 1]);
  }
  __syncthreads();
  flush(s_v[(nstages - 1) & 1], s_z[(nstages - 1) & 1], key_base + (nstages - 1) * SK);
}

// score[j] = (1/k) * sum_{d=-k/2..k/2} vote[j+d], zero outside [0, P); votes of the row
// blocks are added first, always in the same order.
__global__ __launch_bounds__(256) void pool_scores_kernel(ScoreArgs a) {
  const int bg = blockIdx.y;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  if (blockIdx.x == 0 && a.zero_words)          // clears the selection histograms of this head
    for (int t = threadIdx.x; t < a.zero_per_head; t += 256) a.zero_words[static_cast<int64_t>(bg) * a.zero_per_head + t] = 0u;
  if (n <= a.B) return;
  const int P = n - a.w;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= P) return;
  const int64_t head_tok = static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n;
  const int64_t plane = a.plane;
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
