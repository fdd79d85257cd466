// Per-KV-head top-k of the pooled scores (the selection inside Alg. 1 step 3) and the gather
// of KV_compress.  Selection is exact: a most-significant-digit-first radix select on the
// fp32 bit patterns (scores are >= 0, so unsigned order equals numeric order) finds the
// k_sel-th largest value; an ordered compaction then keeps everything above it plus the
// first equal entries in position order, which is the "ties to the lower index" rule, and
// emits positions in ascending order.  One workgroup owns one (sequence, KV head).
#pragma once
#include "cd_common.h"
#include "cd_score.h"

namespace cd {

constexpr int kSelThreads = 1024;

struct SelectArgs {
  const int32_t* seq_off;
  int64_t total_tokens;
  int batch, Hkv, w, B, max_seq_len, W32;
  const float* score;      // [total_tokens*Hkv]
  int32_t* indices;        // [batch][Hkv][B]
  int32_t* cache_lens;     // [batch]
  uint32_t* bitmap;        // [batch*Hkv][W32]: bit set = position is NOT evicted
};

__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(SelectArgs a) {
  const int bg = blockIdx.x;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  int32_t* idx = a.indices + static_cast<int64_t>(bg) * a.B;
  if (g == 0 && tid == 0) a.cache_lens[b] = min(n, a.B);
  if (n <= a.B) {                       // nothing to evict: keep every position
    for (int r = tid; r < a.B; r += kSelThreads) idx[r] = (r < n) ? r : -1;
    return;
  }
  const int P = n - a.w;
  const int k_sel = a.B - a.w;
  const uint32_t* key = reinterpret_cast<const uint32_t*>(a.score) +
                        static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n;

  __shared__ uint32_t hist[256];
  __shared__ uint32_t s_prefix, s_remaining;
  __shared__ uint32_t wave_cnt[kSelThreads / 64];

  // ---- radix select: 4 digits of 8 bits, most significant first -------------------------
  uint32_t prefix = 0;            // bits decided so far (the high bits of the threshold)
  uint32_t remaining = k_sel;     // rank of the threshold among the keys matching `prefix`
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t himask = (pass == 0) ? 0u : (0xFFFFFFFFu << (shift + 8));
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int j = tid; j < P; j += kSelThreads) {
      uint32_t u = key[j];
      if ((u & himask) == prefix) atomicAdd(&hist[(u >> shift) & 0xFF], 1u);
    }
    __syncthreads();
    if (wv == 0) {
      // lane t owns bins 4t..4t+3; find the bin where the count from the top reaches `remaining`
      uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
      uint32_t mine = h0 + h1 + h2 + h3;
      uint32_t above = 0;             // keys in bins owned by higher lanes
      uint32_t acc = mine;
#pragma unroll
      for (int s = 1; s < 64; s <<= 1) {        // suffix-inclusive scan over lanes
        uint32_t o = __shfl_down(acc, s);
        if (lane + s < 64) acc += o;
      }
      above = acc - mine;
      if (above < remaining && remaining <= acc) {      // exactly one lane
        uint32_t cum = above;
        int bin;
        if (cum + h3 >= remaining) bin = 3;
        else { cum += h3; if (cum + h2 >= remaining) bin = 2;
          else { cum += h2; if (cum + h1 >= remaining) bin = 1; else { cum += h1; bin = 0; } } }
        s_prefix = prefix | (static_cast<uint32_t>(4 * lane + bin) << shift);
        s_remaining = remaining - cum;
      }
    }
    __syncthreads();
    prefix = s_prefix;
    remaining = s_remaining;
    __syncthreads();
  }
  const uint32_t thr = prefix;          // bit pattern of the k_sel-th largest score
  const uint32_t need_eq = remaining;   // how many entries equal to thr are kept (>= 1)

  // ---- ordered compaction + retained bitmap ---------------------------------------------
  uint32_t* bm = a.bitmap + static_cast<int64_t>(bg) * a.W32;
  uint32_t run_gt = 0, run_eq = 0;      // counts over all earlier positions
  const int n_round = (n + kSelThreads - 1) / kSelThreads * kSelThreads;
  for (int base = 0; base < n_round; base += kSelThreads) {
    const int j = base + tid;
    uint32_t u = (j < P) ? key[j] : 0u;
    const bool gt = (j < P) && (u > thr);
    const bool eq = (j < P) && (u == thr);
    const uint64_t mgt = __ballot(gt), meq = __ballot(eq);
    const uint64_t below = (1ull << lane) - 1ull;
    if (lane == 0) wave_cnt[wv] = __popcll(mgt) | (__popcll(meq) << 16);
    __syncthreads();
    uint32_t pre_gt = run_gt + __popcll(mgt & below);
    uint32_t pre_eq = run_eq + __popcll(meq & below);
    uint32_t tot_gt = 0, tot_eq = 0;
#pragma unroll
    for (int ww = 0; ww < kSelThreads / 64; ++ww) {
      uint32_t cnt = wave_cnt[ww];
      if (ww < wv) { pre_gt += cnt & 0xFFFFu; pre_eq += cnt >> 16; }
      tot_gt += cnt & 0xFFFFu;
      tot_eq += cnt >> 16;
    }
    const bool keep = gt || (eq && pre_eq < need_eq);
    if (keep) idx[pre_gt + min(pre_eq, need_eq)] = j;
    // bit = not evicted: selected prefix positions and everything from the window on
    const uint64_t mk = __ballot(keep || j >= P);
    if (lane == 0 && base + wv * 64 < n) {
      bm[(base + wv * 64) >> 5] = static_cast<uint32_t>(mk);
      bm[((base + wv * 64) >> 5) + 1] = static_cast<uint32_t>(mk >> 32);
    }
    run_gt += tot_gt;
    run_eq += tot_eq;
    __syncthreads();
  }
  for (int r = tid; r < a.w; r += kSelThreads) idx[k_sel + r] = P + r;   // the window is always kept
}

struct GatherArgs {
  const void* k; const void* v; void* k_c; void* v_c;
  const int32_t* seq_off; const int32_t* cache_off; const int32_t* indices;
  int64_t total_tokens;
  int batch, Hkv, B, max_seq_len, row_bytes;     // row_bytes = D * sizeof(T)
};

// K_c[g][r] = K[g][idx[g][r]], V likewise; 16 bytes per thread.
__global__ __launch_bounds__(256) void gather_kv_kernel(GatherArgs a) {
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
  const int src = a.indices[static_cast<int64_t>(bg) * a.B + r];
  const int64_t src_off = ((static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n + src) * a.row_bytes) + vcol * 16;
  const int64_t dst_off = ((static_cast<int64_t>(c0) * a.Hkv + static_cast<int64_t>(g) * cap + r) * a.row_bytes) + vcol * 16;
  st16(static_cast<char*>(a.k_c) + dst_off, ld16(static_cast<const char*>(a.k) + src_off));
  st16(static_cast<char*>(a.v_c) + dst_off, ld16(static_cast<const char*>(a.v) + src_off));
}

}  // namespace cd
