// Pooling, per-KV-head top-k of the pooled scores (the selection inside Alg. 1 step 3) and
// the gather of KV_compress, one workgroup per (sequence, KV head).
//
// Selection is exact: a most-significant-digit-first radix select on the fp32 bit patterns
// (scores are >= 0, so unsigned order equals numeric order) finds the k_sel-th largest value
// and how many entries equal to it are kept; an ordered compaction then keeps everything
// above it plus the first equal entries in position order - the "ties to the lower index"
// rule - and emits positions in ascending order.  Integer work only: bit-exact and
// deterministic.
//
// Two variants: select_gather_lds_kernel (prefix up to 32768 positions: pools the votes itself,
// keys in registers) and select_gather_kernel (longer prefixes: keys read from the pooled-score
// buffer that pool_scores_kernel wrote).
#pragma once
#include "cd_common.h"
#include "cd_score.h"

namespace cd {

constexpr int kSelThreads = 1024;
constexpr int kSelPerThread = 32;              // LDS variant: positions per thread (= one bitmap word)
constexpr int kSelMaxLdsKeys = kSelThreads * kSelPerThread;   // longest prefix the LDS variant takes
constexpr int kSelMaxPool = 15;                // widest pooling kernel the LDS variant takes
constexpr int kSelLdsBytes = (kSelMaxLdsKeys + kSelMaxLdsKeys / 32) * 4;   // votes, 1 pad word per 32

struct SelectArgs {
  const int32_t* seq_off;
  const int32_t* cache_off;
  int64_t total_tokens;
  int batch, Hkv, w, B, max_seq_len, W32, NRB, pool_k, row_bytes;
  int write_scores;        // LDS variant: also store the pooled scores (inspection only)
  const float* vote;       // [NRB][total_tokens*Hkv]   (LDS-key variant pools these itself)
  float* score;            // [total_tokens*Hkv] pooled scores: written (LDS variant) or read
  int32_t* indices;        // [batch][Hkv][B]
  int32_t* cache_lens;     // [batch]
  uint32_t* bitmap;        // [batch*Hkv][W32]: bit set = position is NOT evicted
  const void* k; const void* v; void* k_c; void* v_c;
};

// Variant for prefixes too long for LDS: the pooled scores are read from the buffer that
// pool_scores_kernel wrote, position j of a sweep handled by thread j mod 1024.
__global__ __launch_bounds__(kSelThreads) void select_gather_kernel(SelectArgs a) {
  const int bg = blockIdx.x;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  int32_t* idx = a.indices + static_cast<int64_t>(bg) * a.B;
  const int len = min(n, a.B);
  if (g == 0 && tid == 0) a.cache_lens[b] = len;
  const int64_t head_tok = static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n;

  __shared__ uint32_t hist[256];
  __shared__ uint32_t s_prefix, s_remaining;
  __shared__ uint32_t wave_gt[kSelThreads / 64], wave_eq[kSelThreads / 64];

  if (n <= a.B) {                       // nothing to evict: keep every position
    for (int r = tid; r < a.B; r += kSelThreads) idx[r] = (r < n) ? r : -1;
  } else {
    const int P = n - a.w;
    const int k_sel = a.B - a.w;
    const uint32_t* gkey = reinterpret_cast<const uint32_t*>(a.score) + head_tok;
    auto key_at = [&](int j) -> uint32_t { return gkey[j]; };

    // ---- radix select: 4 digits of 8 bits, most significant first -----------------------
    uint32_t prefix = 0;            // bits decided so far (the high bits of the threshold)
    uint32_t remaining = k_sel;     // rank of the threshold among the keys matching `prefix`
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      const uint32_t himask = (pass == 0) ? 0u : (0xFFFFFFFFu << (shift + 8));
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      {
        // run-length compressed updates (scores share their leading digits); 8 independent
        // loads per thread are in flight at a time
        uint32_t run_bin = 0, run_len = 0;
        for (int j0 = tid; j0 < P; j0 += 8 * kSelThreads) {
          uint32_t u[8];
#pragma unroll
          for (int q = 0; q < 8; ++q) u[q] = (j0 + q * kSelThreads < P) ? key_at(j0 + q * kSelThreads) : 0u;
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            if (j0 + q * kSelThreads < P && (u[q] & himask) == prefix) {
              const uint32_t bin = (u[q] >> shift) & 0xFF;
              if (bin != run_bin && run_len) { atomicAdd(&hist[run_bin], run_len); run_len = 0; }
              run_bin = bin;
              ++run_len;
            }
          }
        }
        if (run_len) atomicAdd(&hist[run_bin], run_len);
      }
      __syncthreads();
      if (wv == 0) {
        // lane t owns bins 4t..4t+3; find the bin where the count from the top reaches `remaining`
        const uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
        const uint32_t mine = h0 + h1 + h2 + h3;
        uint32_t acc = mine;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {        // suffix-inclusive scan over lanes
          const uint32_t o = __shfl_down(acc, s);
          if (lane + s < 64) acc += o;
        }
        const uint32_t above = acc - mine;        // keys in bins owned by higher lanes
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

    // ---- ordered compaction + retained bitmap: wave w owns the contiguous positions
    //      [w*seg, (w+1)*seg); one counting sweep, one barrier, one emitting sweep --------------
    uint32_t* bm = a.bitmap + static_cast<int64_t>(bg) * a.W32;
    constexpr int NWV = kSelThreads / 64;
    const int seg = ((n + NWV - 1) / NWV + 63) / 64 * 64;
    const int seg_lo = wv * seg, seg_hi = min(n, seg_lo + seg);
    const int key_hi = min(P, seg_hi);    // candidates of this wave: prefix positions of its segment
    uint32_t cnt_gt = 0, cnt_eq = 0;
    for (int base = seg_lo; base < seg_hi; base += 4 * 64) {
      uint32_t u[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) { const int j = base + q * 64 + lane; u[q] = (j < key_hi) ? key_at(j) : 0u; }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int j = base + q * 64 + lane;
        cnt_gt += __popcll(__ballot(j < key_hi && u[q] > thr));
        cnt_eq += __popcll(__ballot(j < key_hi && u[q] == thr));
      }
    }
    if (lane == 0) { wave_gt[wv] = cnt_gt; wave_eq[wv] = cnt_eq; }
    __syncthreads();
    uint32_t pre_gt = 0, pre_eq = 0;      // counts over all earlier positions (wave-uniform)
    for (int ww = 0; ww < wv; ++ww) { pre_gt += wave_gt[ww]; pre_eq += wave_eq[ww]; }
    const uint64_t below = (1ull << lane) - 1ull;
    for (int base = seg_lo; base < seg_hi; base += 4 * 64) {
      uint32_t u[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) { const int j = base + q * 64 + lane; u[q] = (j < key_hi) ? key_at(j) : 0u; }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int j = base + q * 64 + lane;
        if (base + q * 64 < seg_hi) {
          const bool gt = j < key_hi && u[q] > thr;
          const bool eq = j < key_hi && u[q] == thr;
          const uint64_t mgt = __ballot(gt), meq = __ballot(eq);
          const uint32_t my_eq = pre_eq + __popcll(meq & below);
          const bool keep = gt || (eq && my_eq < need_eq);
          if (keep) idx[pre_gt + __popcll(mgt & below) + min(my_eq, need_eq)] = j;
          // bit = not evicted: selected prefix positions and everything from the window on
          const uint64_t mk = __ballot(keep || j >= P);
          if (lane == 0) {
            bm[(base + q * 64) >> 5] = static_cast<uint32_t>(mk);
            bm[((base + q * 64) >> 5) + 1] = static_cast<uint32_t>(mk >> 32);
          }
          pre_gt += __popcll(mgt);
          pre_eq += __popcll(meq);
        }
      }
    }
    for (int r = tid; r < a.w; r += kSelThreads) idx[k_sel + r] = P + r;   // the window is always kept
  }

  // ---- gather: K_c[g][r] = K[g][idx[g][r]], V likewise; 16 bytes per thread per step -------
  __threadfence_block();
  __syncthreads();                       // idx[] written above is read back by other threads
  const int c0 = a.cache_off[b];
  const int cap = a.cache_off[b + 1] - c0;
  if (cap < len) return;                 // capacity contract broken: write nothing
  const int vec_per_row = a.row_bytes / 16;
  const char* ksrc = static_cast<const char*>(a.k) + head_tok * a.row_bytes;
  const char* vsrc = static_cast<const char*>(a.v) + head_tok * a.row_bytes;
  const int64_t dst_head = (static_cast<int64_t>(c0) * a.Hkv + static_cast<int64_t>(g) * cap) * a.row_bytes;
  char* kdst = static_cast<char*>(a.k_c) + dst_head;
  char* vdst = static_cast<char*>(a.v_c) + dst_head;
  constexpr int kBatch = 8;              // independent row copies in flight per thread
  const int total = len * vec_per_row;
  for (int t0 = tid; t0 < total; t0 += kBatch * kSelThreads) {
    int src[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int t = t0 + u * kSelThreads;
      src[u] = (t < total) ? idx[t / vec_per_row] : 0;
    }
    u32x4 kk[kBatch], vv[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int t = t0 + u * kSelThreads;
      const int vcol = t % vec_per_row;
      const int64_t so = static_cast<int64_t>(src[u]) * a.row_bytes + vcol * 16;
      if (t < total) { kk[u] = ld16(ksrc + so); vv[u] = ld16(vsrc + so); }
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int t = t0 + u * kSelThreads;
      const int64_t dof = static_cast<int64_t>(t / vec_per_row) * a.row_bytes + (t % vec_per_row) * 16;
      if (t < total) { st16(kdst + dof, kk[u]); st16(vdst + dof, vv[u]); }
    }
  }
}

// LDS variant for prefixes of up to 32 * NT positions (NT = 256, 512 or 1024 threads; the
// smaller workgroups let two or four heads share a compute unit).  Thread t owns positions
// 32t..32t+31: their pooled scores live in its registers for the radix passes and the
// compaction, and their retained bits are exactly bitmap word t.  The votes are staged once in
// LDS (padded by one word per 32 so that the stride-32 accesses do not collide), and the same
// LDS later holds the retained indices for the gather.
template <int NT>
__global__ __launch_bounds__(NT) void select_gather_lds_kernel(SelectArgs a) {
  extern __shared__ uint32_t s_sel[];
  float* s_vote = reinterpret_cast<float*>(s_sel);
  int32_t* s_idx = reinterpret_cast<int32_t*>(s_sel);      // reused after pooling
  const int bg = blockIdx.x;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  int32_t* idx = a.indices + static_cast<int64_t>(bg) * a.B;
  const int len = min(n, a.B);
  if (g == 0 && tid == 0) a.cache_lens[b] = len;
  const int64_t head_tok = static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n;

  __shared__ uint32_t hist[256];
  __shared__ uint32_t s_prefix, s_remaining;
  __shared__ uint32_t wave_tot[NT / 64];
  constexpr int PER = kSelPerThread;
  auto pad = [](int j) { return j + (j >> 5); };

  if (n <= a.B) {                       // nothing to evict: keep every position
    for (int r = tid; r < a.B; r += NT) {
      idx[r] = (r < n) ? r : -1;
      if (r < n) s_idx[r] = r;
    }
  } else {
    const int P = n - a.w;
    const int k_sel = a.B - a.w;
    // ---- stage the votes (row-block partials added first, fixed order) ---------------------
    {
      const int64_t plane = a.total_tokens * a.Hkv;
      const float* vsrc = a.vote + head_tok;
      float tmp[PER];
#pragma unroll
      for (int u = 0; u < PER; ++u) {               // all loads of a thread in flight together
        const int j = tid + u * NT;
        float val = 0.f;
        if (j < P) {
          val = vsrc[j];
          for (int rb = 1; rb < a.NRB; ++rb) val += vsrc[rb * plane + j];
        }
        tmp[u] = val;
      }
#pragma unroll
      for (int u = 0; u < PER; ++u) {
        const int j = tid + u * NT;
        if (j < P) s_vote[pad(j)] = tmp[u];
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
    // ---- radix select: 4 digits of 8 bits, most significant first ---------------------------
    uint32_t prefix = 0;            // bits decided so far (the high bits of the threshold)
    uint32_t remaining = k_sel;     // rank of the threshold among the keys matching `prefix`
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      const uint32_t himask = (pass == 0) ? 0u : (0xFFFFFFFFu << (shift + 8));
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      {
        // run-length compressed updates: neighbouring pooled scores share their leading digits
        uint32_t run_bin = 0, run_len = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
          if (j0 + u < P && (key[u] & himask) == prefix) {
            const uint32_t bin = (key[u] >> shift) & 0xFF;
            if (bin != run_bin && run_len) { atomicAdd(&hist[run_bin], run_len); run_len = 0; }
            run_bin = bin;
            ++run_len;
          }
        }
        if (run_len) atomicAdd(&hist[run_bin], run_len);
      }
      __syncthreads();
      if (wv == 0) {
        // lane t owns bins 4t..4t+3; find the bin where the count from the top reaches `remaining`
        const uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
        const uint32_t mine = h0 + h1 + h2 + h3;
        uint32_t acc = mine;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {        // suffix-inclusive scan over lanes
          const uint32_t o = __shfl_down(acc, s);
          if (lane + s < 64) acc += o;
        }
        const uint32_t above = acc - mine;        // keys in bins owned by higher lanes
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

    // ---- ordered compaction: exclusive scan of per-thread (greater, equal) counts -----------
    uint32_t cnt = 0;                     // greater in the low half, equal in the high half
#pragma unroll
    for (int u = 0; u < PER; ++u)
      if (j0 + u < P) cnt += (key[u] > thr ? 1u : 0u) + (key[u] == thr ? 0x10000u : 0u);
    uint32_t incl = cnt;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const uint32_t o = __shfl_up(incl, s);
      if (lane >= s) incl += o;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();                      // also: every thread is done reading the staged votes
    uint32_t before = incl - cnt;
    for (int ww = 0; ww < wv; ++ww) before += wave_tot[ww];
    uint32_t pre_gt = before & 0xFFFFu, pre_eq = before >> 16;
    uint32_t word = 0;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int j = j0 + u;
      const bool in = j < P;
      const bool gt = in && key[u] > thr;
      const bool eq = in && key[u] == thr;
      const bool keep = gt || (eq && pre_eq < need_eq);
      if (keep) {
        const uint32_t pos = pre_gt + min(pre_eq, need_eq);
        idx[pos] = j;
        s_idx[pos] = j;
      }
      pre_gt += gt ? 1u : 0u;
      pre_eq += eq ? 1u : 0u;
      word |= ((keep || !in) ? 1u : 0u) << u;       // bit = not evicted (window and beyond count as kept)
    }
    if (j0 < P) a.bitmap[static_cast<int64_t>(bg) * a.W32 + tid] = word;
    for (int r = tid; r < a.w; r += NT) { idx[k_sel + r] = P + r; s_idx[k_sel + r] = P + r; }
  }

  // ---- gather: K_c[g][r] = K[g][idx[g][r]], V likewise; 16 bytes per thread per copy ---------
  __syncthreads();
  const int c0 = a.cache_off[b];
  const int cap = a.cache_off[b + 1] - c0;
  if (cap < len) return;                 // capacity contract broken: write nothing
  const int vec_per_row = a.row_bytes / 16;
  const char* ksrc = static_cast<const char*>(a.k) + head_tok * a.row_bytes;
  const char* vsrc = static_cast<const char*>(a.v) + head_tok * a.row_bytes;
  const int64_t dst_head = (static_cast<int64_t>(c0) * a.Hkv + static_cast<int64_t>(g) * cap) * a.row_bytes;
  char* kdst = static_cast<char*>(a.k_c) + dst_head;
  char* vdst = static_cast<char*>(a.v_c) + dst_head;
  constexpr int kBatch = 8;              // independent row copies in flight per thread
  const int total = len * vec_per_row;
  for (int t0 = tid; t0 < total; t0 += kBatch * NT) {
    u32x4 kk[kBatch], vv[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int t = t0 + u * NT;
      if (t < total) {
        const int64_t so = static_cast<int64_t>(s_idx[t / vec_per_row]) * a.row_bytes + (t % vec_per_row) * 16;
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

}  // namespace cd
