// Eviction strategies whose retained set is plain index arithmetic or comes from the caller
// (Alg. 1 step 3 with f other than the SnapKV-style scoring; Sec. 4.1.3 lists StreamingLLM:
// attention sinks plus the most recent tokens).  These kernels only prepare the index list and
// the skip bitmap; the gather of KV_compress and the calibration pass over KV_evict are the
// same kernels the scored path uses.
#pragma once
#include "cd_common.h"
#include "cd_score.h"

namespace cd {

struct StreamingArgs {
  const int32_t* seq_off;
  int64_t total_tokens;
  int batch, Hkv, B, n_sink, max_seq_len;
  int32_t* indices;        // [batch][Hkv][B]
};

// retained = the first n_sink positions and the last B - n_sink ones (all of them when n <= B,
// -1 padded), ascending, the same list for every KV head of a sequence.
__global__ __launch_bounds__(256) void streaming_indices_kernel(StreamingArgs a) {
  const int bg = blockIdx.y;
  const int b = bg / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= a.B) return;
  int pos;
  if (n <= a.B) pos = r < n ? r : -1;
  else pos = r < a.n_sink ? r : n - a.B + r;
  a.indices[static_cast<int64_t>(bg) * a.B + r] = pos;
}

struct GivenArgs {
  const int32_t* seq_off;
  int64_t total_tokens;
  int batch, Hkv, B, max_seq_len, W32;
  int32_t* indices;        // [batch][Hkv][B] in; rewritten for sequences with n <= B
  int32_t* cache_lens;     // [batch] out
  uint32_t* bitmap;        // [batch*Hkv][W32] out: bit set = position is retained
};

// From a caller-supplied retained list: cache_lens, the "retained" bitmap the calibration pass
// skips by, and - for sequences that fit the budget, where nothing is evicted - the identity
// list.  Entries outside [0, n) mark nothing.
__global__ __launch_bounds__(256) void given_prepare_kernel(GivenArgs a) {
  const int bg = blockIdx.x;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  int32_t* idx = a.indices + static_cast<int64_t>(bg) * a.B;
  if (g == 0 && threadIdx.x == 0) a.cache_lens[b] = min(n, a.B);
  if (n <= a.B) {
    for (int r = threadIdx.x; r < a.B; r += 256) idx[r] = r < n ? r : -1;
    return;                                 // nothing evicted: the calibration pass covers no row
  }
  uint32_t* bm = a.bitmap + static_cast<int64_t>(bg) * a.W32;
  const int words = (n + 31) / 32;
  for (int wd = threadIdx.x; wd < words; wd += 256) bm[wd] = 0u;
  __threadfence();
  __syncthreads();
  for (int r = threadIdx.x; r < a.B; r += 256) {
    const int pos = idx[r];
    if (pos >= 0 && pos < n) atomicOr(&bm[pos >> 5], 1u << (pos & 31));
  }
}

// ---- packing KV_evict for offloading (Alg. 1 step 4: the evicted cache is moved, not deleted) ----
struct PackArgs {
  const int32_t* seq_off;      // prompt token offsets
  const int32_t* evict_off;    // [batch+1] token offsets of the packed buffers (capacity per sequence)
  int64_t total_tokens;
  int batch, Hkv, B, calib, max_seq_len, W32, row_bytes;
  const uint32_t* bitmap;      // [batch*Hkv][W32]: bit clear = position belongs to the packed set
  int32_t* evict_lens;         // [batch] out: rows per KV head in the packed buffers
  int32_t* evict_indices;      // out, packed like K with one int per row: prompt position of each packed row
  const void* k; const void* v; void* k_e; void* v_e;
};

// Rows per KV head the packed set of a sequence of length n has: everything evicted, or the
// calibration set when a calibration size is given.
__device__ __forceinline__ int packed_rows(int n, int B, int calib) {
  if (n <= B) return 0;
  return calib > 0 ? min(calib, n - B) : n - B;
}

// Ascending list of the positions whose bitmap bit is clear, one workgroup per (sequence, KV head).
// Thread t owns a contiguous run of bitmap words, so a block-wide scan of the per-thread counts
// gives every thread the slot of its first position.
__global__ __launch_bounds__(256) void evict_list_kernel(PackArgs a) {
  const int bg = blockIdx.x;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wv = wave_index();
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  const int e0 = a.evict_off[b];
  const int cap = a.evict_off[b + 1] - e0;
  int want = packed_rows(n, a.B, a.calib);
  if (want > cap) want = 0;                       // capacity contract broken: pack nothing
  if (g == 0 && tid == 0) a.evict_lens[b] = want;
  if (want == 0) return;
  const uint32_t* bm = a.bitmap + static_cast<int64_t>(bg) * a.W32;
  const int words = (n + 31) / 32;
  const int wpt = (words + 255) / 256;
  const int w_lo = min(words, tid * wpt), w_hi = min(words, w_lo + wpt);
  auto clear_bits = [&](int wd) -> uint32_t {
    uint32_t z = ~bm[wd];
    if (wd == words - 1 && (n & 31)) z &= (1u << (n & 31)) - 1u;
    return z;
  };
  int cnt = 0;
  for (int wd = w_lo; wd < w_hi; ++wd) cnt += __popc(clear_bits(wd));
  // exclusive scan over the 256 threads
  const int incl = static_cast<int>(wave_inclusive_scan(static_cast<uint32_t>(cnt)));
  __shared__ int s_wave[4];
  if (lane == 63) s_wave[wv] = incl;
  __syncthreads();
  int base = incl - cnt;
  for (int ww = 0; ww < wv; ++ww) base += s_wave[ww];
  const int total = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
  int32_t* list = a.evict_indices + static_cast<int64_t>(e0) * a.Hkv + static_cast<int64_t>(g) * cap;
  for (int wd = w_lo; wd < w_hi; ++wd) {
    uint32_t z = clear_bits(wd);
    while (z) {
      const int bit = __ffs(z) - 1;
      z &= z - 1;
      if (base < want) list[base] = wd * 32 + bit;
      ++base;
    }
  }
  // a list that marks fewer positions than it should (not one the library wrote): pad
  for (int r = total + tid; r < want; r += 256) list[r] = -1;
}

// k_e[g][r] = K[g][list[r]], V likewise; 16 bytes per thread.  Rows padded with -1 are zero-filled.
__global__ __launch_bounds__(256) void pack_gather_kernel(PackArgs a) {
  const int bg = blockIdx.y;
  const int g = bg % a.Hkv;
  const int b = bg / a.Hkv;
  int off0;
  const int n = seq_len_checked(a.seq_off, b, a.max_seq_len, a.total_tokens, off0);
  const int e0 = a.evict_off[b];
  const int cap = a.evict_off[b + 1] - e0;
  int want = packed_rows(n, a.B, a.calib);
  if (want > cap) want = 0;
  const int vec_per_row = a.row_bytes / 16;
  const int t = blockIdx.x * 256 + threadIdx.x;
  const int r = t / vec_per_row, vcol = t - r * vec_per_row;
  if (r >= want) return;
  const int64_t head_row = static_cast<int64_t>(e0) * a.Hkv + static_cast<int64_t>(g) * cap;
  const int src = a.evict_indices[head_row + r];
  const int64_t dof = (head_row + r) * a.row_bytes + vcol * 16;
  u32x4 kk = zero16(), vv = zero16();
  if (src >= 0 && src < n) {
    const int64_t so = ((static_cast<int64_t>(off0) * a.Hkv + static_cast<int64_t>(g) * n + src) * a.row_bytes) + vcol * 16;
    kk = ld16(static_cast<const char*>(a.k) + so);
    vv = ld16(static_cast<const char*>(a.v) + so);
  }
  st16(static_cast<char*>(a.k_e) + dof, kk);
  st16(static_cast<char*>(a.v_e) + dof, vv);
}

// ---- decode-time growth of the compressed cache ----------------------------------------------
struct AppendArgs {
  const void* k_new; const void* v_new;     // [batch][Hkv][D]: the K/V rows of the token just generated
  void* k_c; void* v_c;
  const int32_t* cache_off;
  int32_t* cache_lens;
  int batch, Hkv, row_bytes;
};

// One workgroup per sequence: the new row of every KV head goes to position cache_lens[b], then
// cache_lens[b] grows by one.  A sequence whose capacity is used up is left as it is.
__global__ __launch_bounds__(256) void append_rows_kernel(AppendArgs a) {
  const int b = blockIdx.x;
  const int c0 = a.cache_off[b];
  const int cap = a.cache_off[b + 1] - c0;
  const int pos = a.cache_lens[b];
  __syncthreads();                              // everyone has read the length before it changes
  if (pos < 0 || pos >= cap) return;
  const int vec_per_row = a.row_bytes / 16;
  for (int t = threadIdx.x; t < a.Hkv * vec_per_row; t += 256) {
    const int g = t / vec_per_row, vcol = t - g * vec_per_row;
    const int64_t so = (static_cast<int64_t>(b) * a.Hkv + g) * a.row_bytes + vcol * 16;
    const int64_t dof = ((static_cast<int64_t>(c0) * a.Hkv + static_cast<int64_t>(g) * cap + pos) * a.row_bytes) + vcol * 16;
    st16(static_cast<char*>(a.k_c) + dof, ld16(static_cast<const char*>(a.k_new) + so));
    st16(static_cast<char*>(a.v_c) + dof, ld16(static_cast<const char*>(a.v_new) + so));
  }
  if (threadIdx.x == 0) a.cache_lens[b] = pos + 1;
}

}  // namespace cd
