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

}  // namespace cd
