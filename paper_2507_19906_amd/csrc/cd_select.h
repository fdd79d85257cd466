// Pooling, per-KV-head top-k of the pooled scores (the selection inside Alg. 1 step 3), the
// optional "calibration size" cut of the evicted tokens (Sec. 5.3) and the gather of
// KV_compress, one workgroup per (sequence, KV head).
//
// Selection is exact: a most-significant-digit-first radix select on the fp32 bit patterns
// (scores are >= 0, so unsigned order equals numeric order) finds the value of a given rank
// and how many entries equal to it fall inside the rank; an ordered compaction then keeps
// everything above it plus the first equal entries in position order - the "ties to the lower
// index" rule - and emits positions in ascending order.  Integer work only: bit-exact and
// deterministic.  Two ranks are used: k_sel = B - w (the retained prefix tokens) and, when a
// calibration size m is set, k_sel + m (retained + the m most important evicted tokens, which
// form the calibration set; everything below is dropped for good).
//
// Two variants: select_gather_lds_kernel (prefix up to 32768 positions: one workgroup per head
// pools the votes itself and keeps the keys in registers) and the wide_* kernels (longer
// prefixes: many workgroups per head, keys read from the pooled-score buffer that
// pool_scores_kernel wrote, histograms and counts combined in global memory).
#pragma once
#include "cd_common.h"
#include "cd_score.h"

namespace cd {

constexpr int kSelThreads = 1024;
constexpr int kSelPerThread = 32;              // LDS variant: positions per thread (= one bitmap word)
constexpr int kSelMaxLdsKeys = kSelThreads * kSelPerThread;   // longest prefix the LDS variant takes
constexpr int kSelMaxPool = 15;                // widest pooling kernel the LDS variant takes

struct SelectArgs {
  const int32_t* seq_off;
  const int32_t* cache_off;
  int64_t total_tokens;
  int batch, Hkv, w, B, max_seq_len, W32, NRB, pool_k, row_bytes;
  int calib;               // calibration size m (0 = every evicted token)
  int write_scores;        // LDS variant: also store the pooled scores (inspection only)
  const float* vote;       // [NRB][plane]   (LDS-key variant pools these itself)
  int64_t plane;           // floats per vote plane, a multiple of 64
  float* score;            // [total_tokens*Hkv] pooled scores: written (LDS variant) or read
  int32_t* indices;        // [batch][Hkv][B]
  int32_t* cal_indices;    // [batch][Hkv][calib] positions of the calibration set, or NULL
  int32_t* cache_lens;     // [batch]
  uint32_t* bitmap;        // [batch*Hkv][W32]: bit set = position is NOT in the calibration set
  const void* k; const void* v; void* k_c; void* v_c;
};

struct RadixShared {
  uint32_t hist[256];
  uint32_t prefix, remaining;
};

// Radix select of the `rank`-th largest key (rank >= 1, at most the number of keys).
// `for_each_key(visit)` must call visit(u) once for every key this thread owns.  On return
// thr = that key's bit pattern and need_eq = how many keys equal to thr lie within the rank.
// Must be called by every thread of the workgroup.
template <int NT, typename ForEach>
__device__ __forceinline__ void radix_select(RadixShared& sh, uint32_t rank, ForEach&& for_each_key, uint32_t& thr,
                                             uint32_t& need_eq) {
  const int tid = threadIdx.x, lane = tid & 63, wv = wave_index();
  uint32_t prefix = 0;            // bits decided so far (the high bits of the answer)
  uint32_t remaining = rank;      // rank of the answer among the keys matching `prefix`
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t himask = (pass == 0) ? 0u : (0xFFFFFFFFu << (shift + 8));
    for (int t = tid; t < 256; t += NT) sh.hist[t] = 0;
    __syncthreads();
    {
      // run-length compressed updates: scores share their leading digits, so consecutive keys
      // of a thread mostly fall in the same bin and only bin changes touch the histogram
      uint32_t run_bin = 0, run_len = 0;
      for_each_key([&](uint32_t u) {
        if ((u & himask) == prefix) {
          const uint32_t bin = (u >> shift) & 0xFF;
          if (bin != run_bin && run_len) { atomicAdd(&sh.hist[run_bin], run_len); run_len = 0; }
          run_bin = bin;
          ++run_len;
        }
      });
      if (run_len) atomicAdd(&sh.hist[run_bin], run_len);
    }
    __syncthreads();
    if (wv == 0) {
      // lane t owns bins 4t..4t+3; find the bin where the count from the top reaches `remaining`
      const uint32_t h0 = sh.hist[4 * lane], h1 = sh.hist[4 * lane + 1], h2 = sh.hist[4 * lane + 2],
                     h3 = sh.hist[4 * lane + 3];
      const uint32_t mine = h0 + h1 + h2 + h3;
      const uint32_t upto = wave_inclusive_scan(mine);
      const uint32_t above = last_lane(upto) - upto;    // keys in bins owned by higher lanes
      const uint32_t acc = above + mine;
      if (above < remaining && remaining <= acc) {      // exactly one lane
        uint32_t cum = above;
        int bin;
        if (cum + h3 >= remaining) bin = 3;
        else { cum += h3; if (cum + h2 >= remaining) bin = 2;
          else { cum += h2; if (cum + h1 >= remaining) bin = 1; else { cum += h1; bin = 0; } } }
        sh.prefix = prefix | (static_cast<uint32_t>(4 * lane + bin) << shift);
        sh.remaining = remaining - cum;
      }
    }
    __syncthreads();
    // (no barrier after these reads: sh.prefix is next written two barriers further on, and the
    // histogram, which the next pass clears right away, was last read before the barrier above)
    prefix = sh.prefix;
    remaining = sh.remaining;
  }
  __syncthreads();                  // the caller may reuse `sh` at once
  thr = prefix;
  need_eq = remaining;
}

// K_c[g][r] = K[g][idx[r]], V likewise, for r < len; 16 bytes per thread per copy, 8 independent
// copies in flight per thread.  `idx` may live in LDS or in global memory.
template <int NT>
__device__ __forceinline__ void gather_rows(const SelectArgs& a, const int32_t* idx, int len, int b, int g,
                                            int64_t head_tok) {
  const int tid = threadIdx.x;
  const int c0 = a.cache_off[b];
  const int cap = a.cache_off[b + 1] - c0;
  if (cap < len) return;                 // capacity contract broken: write nothing
  const int vec_per_row = a.row_bytes / 16;
  const char* ksrc = static_cast<const char*>(a.k) + head_tok * a.row_bytes;
  const char* vsrc = static_cast<const char*>(a.v) + head_tok * a.row_bytes;
  const int64_t dst_head = (static_cast<int64_t>(c0) * a.Hkv + static_cast<int64_t>(g) * cap) * a.row_bytes;
  char* kdst = static_cast<char*>(a.k_c) + dst_head;
  char* vdst = static_cast<char*>(a.v_c) + dst_head;
  constexpr int kBatch = 8;
  const int total = len * vec_per_row;
  for (int t0 = tid; t0 < total; t0 += kBatch * NT) {
    u32x4 kk[kBatch], vv[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int t = t0 + u * NT;
      if (t < total) {
        const int64_t so = static_cast<int64_t>(idx[t / vec_per_row]) * a.row_bytes + (t % vec_per_row) * 16;
        kk[u] = ld16(ksrc + so);
        vv[u] = ld16(vsrc + so);
      }
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int t = t0 + u * NT;
      const int64_t dof = static_cast<int64_t>(t / vec_per_row) * a.row_bytes + (t % vec_per_row) * 16;
      if (t < total) { st16(kdst + dof, kk[u]); st16(vdst + dof, vv[u]); }
    }
  }
}

// Membership of one candidate, given how many greater / equal keys precede it in position order.
struct Cut {
  uint32_t thr, need_eq;
  bool all;              // no cut: every candidate is inside
  __device__ __forceinline__ bool inside(uint32_t u, uint32_t eq_before) const {
    return all || u > thr || (u == thr && eq_before < need_eq);
  }
  // number of inside candidates among the first `pos` positions, from the running counts
  __device__ __forceinline__ uint32_t rank(uint32_t pos, uint32_t gt_before, uint32_t eq_before) const {
    return all ? pos : gt_before + min(eq_before, need_eq);
  }
};

// ---- long prefixes: selection spread over many workgroups ------------------------------------
// One workgroup per head cannot sweep hundreds of thousands of scores quickly, so the prefix is
// cut into segments of kWideSeg positions, one workgroup each, and the radix select becomes a
// chain of launches that meet in global memory: four histogram passes (each adds its segment's
// digit counts to the head's 256-bin histogram of that pass), a count pass (greater / equal
// counts per segment once the thresholds are known) and an emit pass (ordered compaction:
// counts of the earlier segments + a scan inside the segment).  Nothing waits inside a kernel;
// every workgroup re-derives the decided digits from the finished histograms of earlier passes.
constexpr int kWideThreads = 256;
constexpr int kWidePer = 32;                          // positions per thread (= one bitmap word)
constexpr int kWideSeg = kWideThreads * kWidePer;     // positions per workgroup

struct WideArgs {
  SelectArgs s;
  uint32_t* hist;        // [batch*Hkv][2 cuts][4 passes][256], zero before the first pass
  uint32_t* seg_cnt;     // [batch*Hkv][NSEG][4]: greater1, equal1, greater2, equal2 per segment
  int NSEG, pass;
};

// The bin of a finished 256-bin histogram in which the count from the top reaches `remaining`;
// updates prefix / remaining like one radix pass.  Lane l holds bins 4l..4l+3 in `hb`.  Called
// by all 64 lanes of a wave.
__device__ __forceinline__ void wide_pick(const u32x4 hb, int shift, uint32_t& prefix, uint32_t& remaining) {
  const int lane = threadIdx.x & 63;
  const uint32_t h0 = hb[0], h1 = hb[1], h2 = hb[2], h3 = hb[3];
  const uint32_t mine = h0 + h1 + h2 + h3;
  const uint32_t upto = wave_inclusive_scan(mine);
  const uint32_t above = last_lane(upto) - upto;      // keys in bins owned by higher lanes
  const uint32_t acc = above + mine;
  const bool hit = above < remaining && remaining <= acc;
  uint32_t cum = above;
  int bin = 0;
  if (cum + h3 >= remaining) bin = 3;
  else { cum += h3; if (cum + h2 >= remaining) bin = 2;
    else { cum += h2; if (cum + h1 >= remaining) bin = 1; else { cum += h1; bin = 0; } } }
  const uint64_t who = __ballot(hit);
  if (who == 0) return;                              // inconsistent histogram: leave the digit 0
  const int src = __ffsll(static_cast<long long>(who)) - 1;
  const uint32_t digit = __shfl(static_cast<uint32_t>(4 * lane + bin), src);
  const uint32_t rem = __shfl(remaining - cum, src);
  prefix |= digit << shift;
  remaining = rem;
}

struct WideHead {
  int n, P, k_sel, b, g, bg;
  int64_t head_tok;
  bool all2;             // no second cut (no calibration size, or it covers every evicted token)
};

__device__ __forceinline__ WideHead wide_head(const SelectArgs& a, int bg) {
  WideHead h;
  h.bg = bg; h.g = bg % a.Hkv; h.b = bg / a.Hkv;
  int off0;
  h.n = seq_len_checked(a.seq_off, h.b, a.max_seq_len, a.total_tokens, off0);
  h.P = h.n - a.w; h.k_sel = a.B - a.w;
  h.head_tok = static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(h.g) * h.n;
  h.all2 = a.calib <= 0 || h.k_sel + a.calib >= h.P;
  return h;
}

// Digits decided by passes 0..upto-1, for both cuts.  The histograms of all those passes are
// fetched together (one round trip); only the scans depend on each other.
__device__ __forceinline__ void wide_derive(const WideArgs& a, const WideHead& h, int upto, uint32_t (&prefix)[2],
                                            uint32_t (&remaining)[2]) {
  const int lane = threadIdx.x & 63;
  const int ncut = h.all2 ? 1 : 2;
  u32x4 hb[2][4];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int ps = 0; ps < 4; ++ps)
      if (c < ncut && ps < upto)
        hb[c][ps] = ld16(a.hist + ((static_cast<int64_t>(h.bg) * 2 + c) * 4 + ps) * 256 + 4 * lane);
  prefix[0] = prefix[1] = 0;
  remaining[0] = h.k_sel;
  remaining[1] = h.k_sel + a.s.calib;
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int ps = 0; ps < 4; ++ps)
      if (c < ncut && ps < upto) wide_pick(hb[c][ps], 24 - 8 * ps, prefix[c], remaining[c]);
}

__global__ __launch_bounds__(kWideThreads) void wide_hist_kernel(WideArgs a) {
  const WideHead h = wide_head(a.s, blockIdx.y);
  const int lo = blockIdx.x * kWideSeg;
  if (h.n <= a.s.B || lo >= h.P) return;
  const int tid = threadIdx.x;
  const uint32_t* gkey = reinterpret_cast<const uint32_t*>(a.s.score) + h.head_tok;
  uint32_t u[kWidePer];                 // issued first: in flight while the digits are derived
#pragma unroll
  for (int q = 0; q < kWidePer; ++q) { const int j = lo + tid + q * kWideThreads; u[q] = j < h.P ? gkey[j] : 0u; }
  uint32_t prefix[2], remaining[2];
  wide_derive(a, h, a.pass, prefix, remaining);
  __shared__ uint32_t s_hist[2][256];
  s_hist[0][tid] = 0; s_hist[1][tid] = 0;
  __syncthreads();
  const int shift = 24 - 8 * a.pass;
  const uint32_t himask = a.pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
  for (int c = 0; c < (h.all2 ? 1 : 2); ++c) {
    uint32_t run_bin = 0, run_len = 0;               // run-length compressed updates
#pragma unroll
    for (int q = 0; q < kWidePer; ++q) {
      if (lo + tid + q * kWideThreads < h.P && (u[q] & himask) == prefix[c]) {
        const uint32_t bin = (u[q] >> shift) & 0xFF;
        if (bin != run_bin && run_len) { atomicAdd(&s_hist[c][run_bin], run_len); run_len = 0; }
        run_bin = bin;
        ++run_len;
      }
    }
    if (run_len) atomicAdd(&s_hist[c][run_bin], run_len);
  }
  __syncthreads();
  for (int c = 0; c < (h.all2 ? 1 : 2); ++c) {
    const uint32_t v = s_hist[c][tid];
    if (v) atomicAdd(a.hist + ((static_cast<int64_t>(h.bg) * 2 + c) * 4 + a.pass) * 256 + tid, v);
  }
}

__device__ __forceinline__ void wide_cuts(const WideArgs& a, const WideHead& h, Cut& c1, Cut& c2) {
  uint32_t prefix[2], remaining[2];
  wide_derive(a, h, 4, prefix, remaining);
  c1.all = false; c1.thr = prefix[0]; c1.need_eq = remaining[0];
  c2.all = h.all2; c2.thr = h.all2 ? 0u : prefix[1]; c2.need_eq = h.all2 ? 0u : remaining[1];
}

// Sum over the workgroup of four counters; result in every thread.  `red` holds 4 x 4 words.
__device__ __forceinline__ void wide_block_sum4(uint32_t (&v)[4], uint32_t (*red)[4]) {
  const int lane = threadIdx.x & 63, wv = wave_index();
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) v[q] += __shfl_xor(v[q], sft);
  __syncthreads();
  if (lane == 0)
#pragma unroll
    for (int q = 0; q < 4; ++q) red[wv][q] = v[q];
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 4; ++q) v[q] = red[0][q] + red[1][q] + red[2][q] + red[3][q];
}

__global__ __launch_bounds__(kWideThreads) void wide_count_kernel(WideArgs a) {
  const WideHead h = wide_head(a.s, blockIdx.y);
  const int lo = blockIdx.x * kWideSeg;
  if (h.n <= a.s.B || lo >= h.P) return;
  const int tid = threadIdx.x;
  const uint32_t* gkey = reinterpret_cast<const uint32_t*>(a.s.score) + h.head_tok;
  uint32_t u[kWidePer];
#pragma unroll
  for (int q = 0; q < kWidePer; ++q) { const int j = lo + tid + q * kWideThreads; u[q] = j < h.P ? gkey[j] : 0u; }
  Cut c1, c2;
  wide_cuts(a, h, c1, c2);
  uint32_t cnt[4] = {0, 0, 0, 0};
#pragma unroll
  for (int q = 0; q < kWidePer; ++q)
    if (lo + tid + q * kWideThreads < h.P) {
      cnt[0] += u[q] > c1.thr; cnt[1] += u[q] == c1.thr;
      cnt[2] += u[q] > c2.thr; cnt[3] += u[q] == c2.thr;
    }
  __shared__ uint32_t red[4][4];
  wide_block_sum4(cnt, red);
  if (tid < 4) a.seg_cnt[(static_cast<int64_t>(h.bg) * a.NSEG + blockIdx.x) * 4 + tid] = cnt[tid];
}

__global__ __launch_bounds__(kWideThreads) void wide_emit_kernel(WideArgs a) {
  const SelectArgs& s = a.s;
  const WideHead h = wide_head(s, blockIdx.y);
  const int seg = blockIdx.x;
  const int lo = seg * kWideSeg;
  const int tid = threadIdx.x, lane = tid & 63, wv = wave_index();
  int32_t* idx = s.indices + static_cast<int64_t>(h.bg) * s.B;
  int32_t* cal = (s.cal_indices && s.calib > 0) ? s.cal_indices + static_cast<int64_t>(h.bg) * s.calib : nullptr;
  if (seg == 0 && h.g == 0 && tid == 0) s.cache_lens[h.b] = min(h.n, s.B);
  if (h.n <= s.B) {                     // nothing to evict: keep every position
    if (seg == 0) {
      for (int r = tid; r < s.B; r += kWideThreads) idx[r] = (r < h.n) ? r : -1;
      if (cal) for (int r = tid; r < s.calib; r += kWideThreads) cal[r] = -1;
    }
    return;
  }
  if (seg == 0) {
    for (int r = tid; r < s.w; r += kWideThreads) idx[h.k_sel + r] = h.P + r;    // the window is always kept
    if (cal) {                                                                   // pad a short calibration set
      const int n_cal = min(s.calib, h.P - h.k_sel);
      for (int r = n_cal + tid; r < s.calib; r += kWideThreads) cal[r] = -1;
    }
  }
  if (lo >= h.P) return;
  // keys of the segment: coalesced loads, then blocked ownership (thread t: positions lo+32t..)
  // through LDS, padded by one word per 32 so that the stride-32 reads do not collide
  __shared__ uint32_t s_key[kWideSeg + kWideSeg / 32];
  __shared__ uint32_t red[4][4];
  __shared__ uint32_t wave_tot[2][kWideThreads / 64];
  auto pad = [](int j) { return j + (j >> 5); };
  const uint32_t* gkey = reinterpret_cast<const uint32_t*>(s.score) + h.head_tok;
  Cut c1, c2;
  uint32_t pre[4] = {0, 0, 0, 0};
  {
    uint32_t u[kWidePer];
#pragma unroll
    for (int q = 0; q < kWidePer; ++q) { const int j = lo + tid + q * kWideThreads; u[q] = j < h.P ? gkey[j] : 0u; }
    // counts of all earlier segments and the thresholds, while the keys are in flight
    for (int sg = tid; sg < seg; sg += kWideThreads) {
      const u32x4 cp = ld16(a.seg_cnt + (static_cast<int64_t>(h.bg) * a.NSEG + sg) * 4);
#pragma unroll
      for (int q = 0; q < 4; ++q) pre[q] += cp[q];
    }
    wide_cuts(a, h, c1, c2);
#pragma unroll
    for (int q = 0; q < kWidePer; ++q) s_key[pad(tid + q * kWideThreads)] = u[q];
  }
  wide_block_sum4(pre, red);            // its barriers also publish s_key
  uint32_t key[kWidePer];
  const int j0 = lo + tid * kWidePer;
#pragma unroll
  for (int u = 0; u < kWidePer; ++u) key[u] = s_key[pad(tid * kWidePer + u)];
  uint32_t cnt1 = 0, cnt2 = 0;          // (greater | equal << 16) of this thread's positions, per cut
#pragma unroll
  for (int u = 0; u < kWidePer; ++u)
    if (j0 + u < h.P) {
      cnt1 += (key[u] > c1.thr ? 1u : 0u) + (key[u] == c1.thr ? 0x10000u : 0u);
      cnt2 += (key[u] > c2.thr ? 1u : 0u) + (key[u] == c2.thr ? 0x10000u : 0u);
    }
  const uint32_t inc1 = wave_inclusive_scan(cnt1), inc2 = wave_inclusive_scan(cnt2);
  if (lane == 63) { wave_tot[0][wv] = inc1; wave_tot[1][wv] = inc2; }
  __syncthreads();
  uint32_t bef1 = inc1 - cnt1, bef2 = inc2 - cnt2;
  for (int ww = 0; ww < wv; ++ww) { bef1 += wave_tot[0][ww]; bef2 += wave_tot[1][ww]; }
  uint32_t gt1 = pre[0] + (bef1 & 0xFFFFu), eq1 = pre[1] + (bef1 >> 16);
  uint32_t gt2 = pre[2] + (bef2 & 0xFFFFu), eq2 = pre[3] + (bef2 >> 16);
  uint32_t word = 0;
#pragma unroll
  for (int u = 0; u < kWidePer; ++u) {
    const int j = j0 + u;
    const bool in = j < h.P;
    const bool keep = in && c1.inside(key[u], eq1);
    const bool calib = in && !keep && c2.inside(key[u], eq2);
    if (keep) idx[c1.rank(j, gt1, eq1)] = j;
    if (calib && cal) cal[c2.rank(j, gt2, eq2) - c1.rank(j, gt1, eq1)] = j;
    if (in) {
      gt1 += key[u] > c1.thr; eq1 += key[u] == c1.thr;
      gt2 += key[u] > c2.thr; eq2 += key[u] == c2.thr;
    }
    word |= (calib ? 0u : 1u) << u;       // bit = skip in the calibration pass
  }
  if (j0 < h.P) s.bitmap[static_cast<int64_t>(h.bg) * s.W32 + (j0 >> 5)] = word;
}

// K_c[g][r] = K[g][idx[g][r]], V likewise (long-prefix path and caller-supplied lists); 16 bytes
// per thread.
__global__ __launch_bounds__(256) void gather_kv_kernel(SelectArgs a) {
  const int bg = blockIdx.y;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  const int len = min(n, a.B);
  const int c0 = a.cache_off[b];
  const int cap = a.cache_off[b + 1] - c0;
  if (cap < len) return;                 // capacity contract broken: write nothing
  const int vec_per_row = a.row_bytes / 16;
  const int t = blockIdx.x * 256 + threadIdx.x;
  const int r = t / vec_per_row, vcol = t - r * vec_per_row;
  if (r >= len) return;
  // clamped: the list may be the caller's (a strategy applied outside the library)
  const int src = min(max(a.indices[static_cast<int64_t>(bg) * a.B + r], 0), n - 1);
  const int64_t so = ((static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n + src) * a.row_bytes) + vcol * 16;
  const int64_t dof = ((static_cast<int64_t>(c0) * a.Hkv + static_cast<int64_t>(g) * cap + r) * a.row_bytes) + vcol * 16;
  st16(static_cast<char*>(a.k_c) + dof, ld16(static_cast<const char*>(a.k) + so));
  st16(static_cast<char*>(a.v_c) + dof, ld16(static_cast<const char*>(a.v) + so));
}

// LDS variant for prefixes of up to PER * NT positions (NT = 1024 threads in use: smaller
// workgroups were measured slower, their staging and gather phases have too few threads).
// Thread t owns positions PER*t..PER*t+PER-1: their pooled scores live in its registers for the
// radix passes and the compaction.  PER = 32: their bits are exactly bitmap word t (prefixes up
// to 32768); PER = 16 / 8: half a word / a byte, so that prefixes up to 16384 / 8192 still keep
// every thread busy.  The votes are staged once in LDS
// (padded by one word per 32 so that the stride-32 accesses do not collide), and the same
// LDS later holds the retained indices for the gather.
template <int NT, int PER>
__global__ __launch_bounds__(NT) void select_gather_lds_kernel(SelectArgs a) {
  extern __shared__ uint32_t s_sel[];
  float* s_vote = reinterpret_cast<float*>(s_sel);
  int32_t* s_idx = reinterpret_cast<int32_t*>(s_sel);      // reused after pooling
  const int bg = blockIdx.x;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wv = wave_index();
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  int32_t* idx = a.indices + static_cast<int64_t>(bg) * a.B;
  int32_t* cal = (a.cal_indices && a.calib > 0) ? a.cal_indices + static_cast<int64_t>(bg) * a.calib : nullptr;
  const int len = min(n, a.B);
  if (g == 0 && tid == 0) a.cache_lens[b] = len;
  const int64_t head_tok = static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n;

  __shared__ RadixShared sh;
  __shared__ uint32_t wave_tot[2][NT / 64];
  static_assert(PER == 32 || PER == 16 || PER == 8, "a thread owns a whole bitmap word, a half or a byte of one");
  auto pad = [](int j) { return j + (j >> 5); };

  if (n <= a.B) {                       // nothing to evict: keep every position
    for (int r = tid; r < a.B; r += NT) {
      idx[r] = (r < n) ? r : -1;
      if (r < n) s_idx[r] = r;
    }
    if (cal) for (int r = tid; r < a.calib; r += NT) cal[r] = -1;
  } else {
    const int P = n - a.w;
    const int k_sel = a.B - a.w;
    // ---- stage the votes (row-block partials added first, fixed order) ---------------------
    {
      // 16 bytes per lane from the 16-byte boundary at or below the head's first vote (every vote
      // plane starts 256-byte aligned - the plane stride is a multiple of 64 floats - and a head
      // starts anywhere inside): vector v covers positions
      // 4v - shift .. 4v - shift + 3.  All loads of a thread are in flight together.
      const int64_t plane = a.plane;
      const int shift = static_cast<int>(head_tok & 3);
      const float* vsrc = a.vote + (head_tok - shift);
      f32x4 tmp[PER / 4];
#pragma unroll
      for (int u = 0; u < PER / 4; ++u) {
        const int v4 = tid + u * NT;
        f32x4 val = f32x4{0.f, 0.f, 0.f, 0.f};
        if (4 * v4 - shift < P) {
          val = *reinterpret_cast<const f32x4*>(vsrc + 4 * v4);
          for (int rb = 1; rb < a.NRB; ++rb) val += *reinterpret_cast<const f32x4*>(vsrc + rb * plane + 4 * v4);
        }
        tmp[u] = val;
      }
#pragma unroll
      for (int u = 0; u < PER / 4; ++u) {
        const int jb = 4 * (tid + u * NT) - shift;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const int j = jb + x;
          if (j >= 0 && j < P) s_vote[pad(j)] = tmp[u][x];
        }
      }
      // the vectors end `shift` positions short of PER * NT: the last few of a full-length prefix
      const int jt = PER * NT - shift + tid;
      if (tid < shift && jt < P) {
        float val = a.vote[head_tok + jt];
        for (int rb = 1; rb < a.NRB; ++rb) val += a.vote[rb * plane + head_tok + jt];
        s_vote[pad(jt)] = val;
      }
    }
    __syncthreads();
    // ---- pooling: score[j] = (1/k) sum_{d=-k/2..k/2} vote[j+d], zeros outside [0, P), summed
    //      left to right at every position ------------------------------------------------------
    uint32_t key[PER];
    const int j0 = tid * PER;
    {
      // the thread's window of votes: w[x] = vote[j0 - half + x], zeros outside [0, P)
      const int half = a.pool_k / 2;
      const float kf = static_cast<float>(a.pool_k);
      float w[PER + kSelMaxPool - 1];
#pragma unroll
      for (int x = 0; x < PER + kSelMaxPool - 1; ++x) {
        const int jj = j0 - half + x;
        w[x] = (x < PER + a.pool_k - 1 && jj >= 0 && jj < P) ? s_vote[pad(jj)] : 0.f;
      }
      float sum[PER];
#pragma unroll
      for (int u = 0; u < PER; ++u) sum[u] = 0.f;
#pragma unroll
      for (int dd = 0; dd < kSelMaxPool; ++dd) {      // taps left to right
        if (dd < a.pool_k) {
#pragma unroll
          for (int u = 0; u < PER; ++u) sum[u] += w[u + dd];
        }
      }
#pragma unroll
      for (int u = 0; u < PER; ++u) key[u] = __builtin_bit_cast(uint32_t, sum[u] / kf);
      if (a.write_scores) {
        // pooled scores go out through LDS so that the global stores are coalesced
        __syncthreads();
#pragma unroll
        for (int u = 0; u < PER; ++u)
          if (j0 + u < P) s_sel[pad(j0 + u)] = key[u];
        __syncthreads();
        float* dst = a.score + head_tok;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
          const int j = tid + u * NT;
          if (j < P) dst[j] = __builtin_bit_cast(float, s_sel[pad(j)]);
        }
      }
    }
    auto each_key = [&](auto&& visit) {
#pragma unroll
      for (int u = 0; u < PER; ++u)
        if (j0 + u < P) visit(key[u]);
    };
    Cut c1, c2;                          // c1: retained prefix tokens; c2: retained + calibration set
    c1.all = false;
    radix_select<NT>(sh, k_sel, each_key, c1.thr, c1.need_eq);
    c2.all = a.calib <= 0 || k_sel + a.calib >= P;
    c2.thr = 0; c2.need_eq = 0;
    if (!c2.all) radix_select<NT>(sh, k_sel + a.calib, each_key, c2.thr, c2.need_eq);

    // ---- ordered compaction: exclusive scans of the per-thread (greater, equal) counts of
    //      both cuts, greater in the low half-word and equal in the high half-word -------------
    // per-thread bit masks over its PER positions: key above the threshold / equal to it
    constexpr uint32_t kAll = PER == 32 ? 0xFFFFFFFFu : (1u << (PER & 31)) - 1u;
    const uint32_t valid = j0 >= P ? 0u : (P - j0 >= PER ? kAll : (1u << ((P - j0) & 31)) - 1u);
    uint32_t gtm1 = 0, eqm1 = 0, gtm2 = 0, eqm2 = 0;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      gtm1 |= (key[u] > c1.thr ? 1u : 0u) << u;
      eqm1 |= (key[u] == c1.thr ? 1u : 0u) << u;
      gtm2 |= (key[u] > c2.thr ? 1u : 0u) << u;
      eqm2 |= (key[u] == c2.thr ? 1u : 0u) << u;
    }
    gtm1 &= valid; eqm1 &= valid; gtm2 &= valid; eqm2 &= valid;
    const uint32_t cnt1 = __popc(gtm1) + (static_cast<uint32_t>(__popc(eqm1)) << 16);
    const uint32_t cnt2 = __popc(gtm2) + (static_cast<uint32_t>(__popc(eqm2)) << 16);
    const uint32_t inc1 = wave_inclusive_scan(cnt1), inc2 = wave_inclusive_scan(cnt2);
    if (lane == 63) { wave_tot[0][wv] = inc1; wave_tot[1][wv] = inc2; }
    __syncthreads();                      // also: every thread is done reading the staged votes
    uint32_t bef1 = inc1 - cnt1, bef2 = inc2 - cnt2;
    for (int ww = 0; ww < wv; ++ww) { bef1 += wave_tot[0][ww]; bef2 += wave_tot[1][ww]; }
    const uint32_t gt1 = bef1 & 0xFFFFu, eq1 = bef1 >> 16, gt2 = bef2 & 0xFFFFu, eq2 = bef2 >> 16;
    // positions of this thread inside a cut: everything above the threshold, and of the keys equal
    // to it the first (need_eq - equal ones at earlier positions), i.e. ties go to the lower index
    auto inside_mask = [&](const Cut& c, uint32_t gtm, uint32_t eqm, uint32_t eq_before) -> uint32_t {
      if (c.all) return valid;
      const uint32_t allow = c.need_eq > eq_before ? c.need_eq - eq_before : 0u;
      if (allow < static_cast<uint32_t>(__popc(eqm))) {
        uint32_t kept = 0;
        for (uint32_t t = 0; t < allow; ++t) { const uint32_t low = eqm & (0u - eqm); kept |= low; eqm ^= low; }
        eqm = kept;
      }
      return gtm | eqm;
    };
    const uint32_t keepm = inside_mask(c1, gtm1, eqm1, eq1);
    const uint32_t calm = inside_mask(c2, gtm2, eqm2, eq2) & ~keepm;
    // the cut's members are emitted in position order: a thread's first one lands at the number of
    // members at earlier positions
    const uint32_t base1 = c1.rank(j0, gt1, eq1);
    {
      uint32_t pos = base1;
      for (uint32_t m = keepm; m; m &= m - 1u, ++pos) {
        const int j = j0 + (__ffs(m) - 1);
        idx[pos] = j;
        s_idx[pos] = j;
      }
    }
    if (cal) {
      uint32_t pos = c2.rank(j0, gt2, eq2) - base1;
      for (uint32_t m = calm; m; m &= m - 1u, ++pos) cal[pos] = j0 + (__ffs(m) - 1);
    }
    const uint32_t word = ~calm;            // bit = skip in the calibration pass
    if constexpr (PER == 32) {
      if (j0 < P) a.bitmap[static_cast<int64_t>(bg) * a.W32 + tid] = word;
    } else {
      // 32 / PER neighbouring lanes hold the pieces of one word (positions beyond the prefix were
      // marked "skip" above, so the pieces of idle threads are all ones)
      constexpr int LPW = 32 / PER;
      constexpr uint32_t kMask = (1u << PER) - 1u;
      uint32_t w32 = word & kMask;
#pragma unroll
      for (int q = 1; q < LPW; ++q) w32 |= (__shfl_down(word, q) & kMask) << (q * PER);
      if ((tid & (LPW - 1)) == 0 && j0 < P) a.bitmap[static_cast<int64_t>(bg) * a.W32 + (j0 >> 5)] = w32;
    }
    for (int r = tid; r < a.w; r += NT) { idx[k_sel + r] = P + r; s_idx[k_sel + r] = P + r; }
    if (cal) {                                                              // pad a short calibration set
      const int n_cal = min(a.calib, P - k_sel);
      for (int r = n_cal + tid; r < a.calib; r += NT) cal[r] = -1;
    }
  }
  __syncthreads();
  gather_rows<NT>(a, s_idx, len, b, g, head_tok);
}

}  // namespace cd
