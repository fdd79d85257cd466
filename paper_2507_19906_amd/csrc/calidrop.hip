// C ABI of the CaliDrop hot path: argument validation, workspace carving and kernel launches.
// Everything here runs on the host; validation never touches HIP, so it can be exercised on a
// machine without a GPU.
#include "../../include/calidrop.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "cd_attend.h"
#include "cd_common.h"
#include "cd_given.h"
#include "cd_h2o.h"
#include "cd_score.h"
#include "cd_select.h"

// Fixed device memory for calidrop_decode_static, the decode entry point for callers that cannot
// bring a workspace: every GPU the library runs on holds its own copy of this array until the
// process ends.  Host code never uses the array's name as an address: the per-device address comes
// from hipGetSymbolAddress (static_scratch_ptr below).
constexpr size_t kStaticScratchBytes = static_cast<size_t>(CALIDROP_STATIC_SCRATCH_BYTES);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
// floats per vote plane: a multiple of 64, so that every plane starts 256-byte aligned
inline int64_t vote_plane(int64_t total_tokens, int n_kv_heads) { return (total_tokens * n_kv_heads + 63) / 64 * 64; }

constexpr uint32_t kParamsSizeV1 = 48;      // layout up to theta2, without calib_size and flags
constexpr uint32_t kParamsSizeV2 = 52;      // layout up to calib_size, without flags

// Copies the caller's struct (either known layout) into `q` with every field defined.
int load_params(const calidrop_params* in, calidrop_params* q) {
  if (!in) return fail(CALIDROP_EINVAL, "params is NULL");
  if (in->struct_size != sizeof(calidrop_params) && in->struct_size != kParamsSizeV1 &&
      in->struct_size != kParamsSizeV2)
    return fail(CALIDROP_EINVAL, "params.struct_size is %u, this library expects %zu (or %u, %u)", in->struct_size,
                sizeof(calidrop_params), kParamsSizeV2, kParamsSizeV1);
  std::memset(q, 0, sizeof(*q));
  std::memcpy(q, in, in->struct_size);
  q->struct_size = sizeof(calidrop_params);
  return CALIDROP_OK;
}

int check_params(const calidrop_params* p) {
  if (p->dtype != CALIDROP_BF16 && p->dtype != CALIDROP_FP32)
    return fail(CALIDROP_EUNSUPPORTED, "dtype %d is not CALIDROP_BF16 or CALIDROP_FP32", p->dtype);
  if (p->batch < 1) return fail(CALIDROP_EINVAL, "batch must be >= 1 (got %d)", p->batch);
  if (p->n_q_heads < 1 || p->n_kv_heads < 1)
    return fail(CALIDROP_EINVAL, "head counts must be >= 1 (got %d query, %d KV)", p->n_q_heads, p->n_kv_heads);
  if (p->n_q_heads % p->n_kv_heads != 0)
    return fail(CALIDROP_ESHAPE, "n_q_heads %d is not a multiple of n_kv_heads %d", p->n_q_heads, p->n_kv_heads);
  if (p->n_q_heads / p->n_kv_heads > 16)
    return fail(CALIDROP_EUNSUPPORTED, "GQA group size %d exceeds 16", p->n_q_heads / p->n_kv_heads);
  if (p->head_dim != 64 && p->head_dim != 128)
    return fail(CALIDROP_EUNSUPPORTED, "head_dim %d is not 64 or 128", p->head_dim);
  if (p->window < 1) return fail(CALIDROP_EINVAL, "window must be >= 1 (got %d)", p->window);
  if (p->budget <= p->window)
    return fail(CALIDROP_EINVAL, "budget %d must exceed window %d (the window counts toward the budget)", p->budget,
                p->window);
  if (p->budget > (1 << 24))
    return fail(CALIDROP_EUNSUPPORTED, "budget %d exceeds %d", p->budget, 1 << 24);
  if (p->pool_kernel < 1 || p->pool_kernel % 2 == 0)
    return fail(CALIDROP_EINVAL, "pool_kernel must be odd and >= 1 (got %d)", p->pool_kernel);
  if (!(p->scale >= 0.f) || std::isinf(p->scale))
    return fail(CALIDROP_EINVAL, "scale must be finite and >= 0 (0 selects 1/sqrt(head_dim))");
  if (std::isnan(p->theta1) || std::isnan(p->theta2) || p->theta1 > p->theta2)
    return fail(CALIDROP_EINVAL, "thresholds must satisfy theta1 <= theta2 and not be NaN");
  if (p->calib_size < 0) return fail(CALIDROP_EINVAL, "calib_size must be >= 0 (got %d)", p->calib_size);
  if (p->flags & ~(CALIDROP_OPT_WRITE_SCORES | CALIDROP_OPT_WIDE_SELECTION))
    return fail(CALIDROP_EINVAL, "flags 0x%x holds bits that are no CALIDROP_OPT_* option", p->flags);
  {  // launch grids put (sequence, KV head, row block) on one grid axis of at most 65535
    const int64_t nrb = (static_cast<int64_t>(p->n_q_heads / p->n_kv_heads) * p->window + cd::kRowBlock - 1) / cd::kRowBlock;
    if (static_cast<int64_t>(p->batch) * p->n_kv_heads * nrb > 65535 || p->n_q_heads > 65535)
      return fail(CALIDROP_EUNSUPPORTED, "batch * n_kv_heads * ceil(G*window/128) exceeds 65535");
  }
  return CALIDROP_OK;
}

float logit_scale(const calidrop_params* p) {
  return p->scale > 0.f ? p->scale : 1.0f / std::sqrt(static_cast<float>(p->head_dim));
}

// Decode runs as one workgroup per (sequence, KV head) - one launch, no workspace - unless there
// are too few pairs to fill the chip AND the cache is long enough for a row split to pay for the
// second launch.
constexpr int kFusedMinPairs = 192;
constexpr int kFusedMaxRowsFewPairs = 2048;

// How the rows of a streaming-attention pass are split over workgroups.
struct SplitPlan { int rows_per_split, NS; };
SplitPlan plan_splits(int heads_kv_total, int max_rows) {
  const int kTargetGroups = 4096;                      // ~16 workgroups per compute unit
  const int kMaxSplits = 32;                           // the merge of the partials is sequential
  const int kMinRows = cd::kTileRows * cd::kAttWaves;  // one tile per wave
  if (max_rows < 1) max_rows = 1;
  int want = ceil_div(kTargetGroups, heads_kv_total);
  if (want < 1) want = 1;
  if (want > kMaxSplits) want = kMaxSplits;
  int rps = ceil_div(ceil_div(max_rows, want), kMinRows) * kMinRows;
  if (rps < kMinRows) rps = kMinRows;
  return SplitPlan{rps, ceil_div(max_rows, rps)};
}

struct CompressLayout {
  size_t rowpart, row_lse, vote, score, bitmap, cal_logit, part_o, part_ml, sel_hist, sel_cnt, total;
  int RB, NRB, NCH, W32, chunk_keys, zstride, NSEG;
  SplitPlan sp;
};

CompressLayout compress_layout(const calidrop_params* p, int64_t total_tokens, int32_t max_seq_len) {
  CompressLayout L{};
  const int G = p->n_q_heads / p->n_kv_heads;
  L.RB = G * p->window > cd::kRowBlock ? 2 * cd::kRowBlock : cd::kRowBlock;     // 256-row blocks: such heads stream K once
  L.NRB = ceil_div(G * p->window, L.RB);
  {  // keys per scoring workgroup, 256..2048: as large as keeps >= ~4096 workgroups in the launch (four rounds
     // of the chip: with sequences of different lengths the last round is otherwise too ragged), but never
     // below 512 for the sake of that while >= ~2048 workgroups remain
    const int64_t groups256 = (total_tokens + cd::kMinChunkKeys - 1) / cd::kMinChunkKeys * p->n_kv_heads * L.NRB;
    int mult = static_cast<int>(groups256 / 4096);
    if (mult < 2) mult = static_cast<int>(std::min<int64_t>(groups256 / 2048, 2));
    if (mult < 1) mult = 1;
    if (mult > 8) mult = 8;
    L.chunk_keys = mult * cd::kMinChunkKeys;
  }
  L.NCH = ceil_div(max_seq_len, L.chunk_keys);
  L.W32 = ceil_div(max_seq_len, 64) * 2;
  L.sp = plan_splits(p->batch * p->n_kv_heads, max_seq_len);
  const size_t rows = static_cast<size_t>(p->batch) * p->n_kv_heads * L.NRB * L.RB;
  const size_t toks = static_cast<size_t>(total_tokens) * p->n_kv_heads;
  size_t off = 0;
  L.rowpart = off; off += round256(rows * L.NCH * sizeof(float2));
  L.row_lse = off; off += round256(rows * sizeof(float));
  L.vote = off;    off += round256(static_cast<size_t>(vote_plane(total_tokens, p->n_kv_heads)) * L.NRB * sizeof(float));
  L.score = off;   off += round256(toks * sizeof(float));
  L.bitmap = off;  off += round256(static_cast<size_t>(p->batch) * p->n_kv_heads * L.W32 * sizeof(uint32_t));
  L.zstride = ceil_div(max_seq_len, 32) * 32;
  L.cal_logit = off; off += round256(static_cast<size_t>(p->batch) * p->n_q_heads * L.zstride * sizeof(float));
  const size_t slots = static_cast<size_t>(p->batch) * p->n_q_heads * L.sp.NS;
  L.part_o = off;  off += round256(slots * p->head_dim * sizeof(float));
  L.part_ml = off; off += round256(slots * sizeof(float2));
  // multi-workgroup selection (prefixes beyond the single-workgroup variant): histograms and counts
  L.NSEG = ceil_div(std::max(max_seq_len - p->window, 1), cd::kWideSeg);
  L.sel_hist = off; off += round256(static_cast<size_t>(p->batch) * p->n_kv_heads * 2 * 4 * 256 * sizeof(uint32_t));
  L.sel_cnt = off;  off += round256(static_cast<size_t>(p->batch) * p->n_kv_heads * L.NSEG * 4 * sizeof(uint32_t));
  L.total = off;
  return L;
}

struct DecodeLayout { size_t part_o, part_ml, total; SplitPlan sp; };

DecodeLayout decode_layout(const calidrop_params* p, int32_t max_cache_len) {
  DecodeLayout L{};
  L.sp = plan_splits(p->batch * p->n_kv_heads, max_cache_len);
  const size_t slots = static_cast<size_t>(p->batch) * p->n_q_heads * L.sp.NS;
  size_t off = 0;
  L.part_o = off;  off += round256(slots * p->head_dim * sizeof(float));
  L.part_ml = off; off += round256(slots * sizeof(float2));
  L.total = off;
  return L;
}

int check_sizes(const calidrop_params* p, int64_t total_tokens, int32_t max_seq_len) {
  if (total_tokens < 1 || max_seq_len < 1 || max_seq_len > total_tokens)
    return fail(CALIDROP_ESHAPE, "need 1 <= max_seq_len <= total_tokens (got %d, %lld)", max_seq_len,
                static_cast<long long>(total_tokens));
  if (total_tokens > (static_cast<int64_t>(1) << 31) - 1)
    return fail(CALIDROP_EUNSUPPORTED, "total_tokens exceeds int32 offsets");
  if (static_cast<int64_t>(p->batch) * max_seq_len < total_tokens)
    return fail(CALIDROP_ESHAPE, "batch * max_seq_len < total_tokens");
  return CALIDROP_OK;
}

int launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(CALIDROP_EHIP, "%s: %s", what, hipGetErrorString(e));
  return CALIDROP_OK;
}

// The skip bitmap of a sequence fits LDS up to 48 KiB (393216 positions): built there, stored once.
void launch_bitmap(const cd::BitmapArgs& ba, int pairs, hipStream_t st) {
  const size_t lds = static_cast<size_t>(ba.W32) * sizeof(uint32_t);
  if (lds <= 48 * 1024) hipLaunchKernelGGL(cd::bitmap_from_indices_lds_kernel, dim3(pairs), dim3(256), lds, st, ba);
  else hipLaunchKernelGGL(cd::bitmap_from_indices_kernel, dim3(pairs), dim3(256), 0, st, ba);
}

// The single-workgroup selection kernels stage up to kSelMaxLdsKeys votes (padded) in dynamic LDS, more
// than the 48 KiB a kernel may use without asking.  The limit is raised to the largest size any call
// can need, once per (kernel variant, device) at that variant's first use on the device - a host-side
// setting that enqueues nothing - and never again, so that calls on the enqueue path (also under
// stream capture) only launch.
constexpr size_t kSelMaxLdsBytes = (static_cast<size_t>(cd::kSelMaxLdsKeys) + cd::kSelMaxLdsKeys / 32 + 1) * sizeof(float);
constexpr int kMaxDevices = 64;
constexpr int kLdsSlots = 16;                             // kernels that ask for more than 48 KiB of dynamic LDS
enum { kLdsSelect8 = 0, kLdsSelect16, kLdsSelect32, kLdsVotes };   // first slot of each family (votes: + variant)
std::atomic<uint8_t> g_lds_ready[kLdsSlots][kMaxDevices]; // zero-initialised: nothing raised yet

// `bytes` is the largest size any call can ask of this kernel, so one setting per (slot, device) is enough.
int ensure_kernel_lds(int slot, const void* fn, size_t bytes, const char* what) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return fail(CALIDROP_EHIP, "hipGetDevice failed or device index %d is beyond %d", dev, kMaxDevices - 1);
  if (g_lds_ready[slot][dev].load(std::memory_order_acquire)) return CALIDROP_OK;
  hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
  if (e != hipSuccess) return fail(CALIDROP_EHIP, "hipFuncSetAttribute(%s): %s", what, hipGetErrorString(e));
  g_lds_ready[slot][dev].store(1, std::memory_order_release);
  return CALIDROP_OK;
}

// Device address of `scratch` on the current device, looked up once per device.
std::atomic<void*> g_scratch_ptr[kMaxDevices];            // zero-initialised: not looked up yet

int static_scratch_ptr(char** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return fail(CALIDROP_EHIP, "hipGetDevice failed or device index %d is beyond %d", dev, kMaxDevices - 1);
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(CALIDROP_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = static_cast<char*>(ptr);
  return CALIDROP_OK;
}

// Pooling + selection + gather for scores already in sa.vote.  Heads whose pooled scores fit in
// LDS are pooled inside the single-workgroup selection kernel; longer ones go through the
// pooled-score buffer and the multi-workgroup chain.  `window` = trailing positions always kept.
int run_selection(const calidrop_params* p, int window, int pool_k, int max_seq_len, cd::SelectArgs& se,
                  cd::ScoreArgs& sa, uint32_t* sel_hist, uint32_t* sel_cnt, int NSEG, hipStream_t st) {
  int rc;
  const int bg = p->batch * p->n_kv_heads;
  const int max_prefix = max_seq_len - window;
  se.write_scores = (p->flags & CALIDROP_OPT_WRITE_SCORES) ? 1 : 0;
  if (max_prefix <= cd::kSelMaxLdsKeys && p->budget <= cd::kSelMaxLdsKeys && pool_k <= cd::kSelMaxPool &&
      !(p->flags & CALIDROP_OPT_WIDE_SELECTION)) {
    // dynamic LDS: staged votes (padded), later reused for the retained indices
    size_t lds = static_cast<size_t>(p->budget) * sizeof(int32_t);
    if (max_seq_len > p->budget) {
      const size_t votes = (static_cast<size_t>(max_prefix) + max_prefix / 32 + 1) * sizeof(float);
      if (votes > lds) lds = votes;
    }
    // positions per thread: the smallest of 8 / 16 / 32 that covers the longest prefix
    const int per = max_prefix <= cd::kSelThreads * 8 ? 8 : max_prefix <= cd::kSelThreads * 16 ? 16 : 32;
    const void* fn = per == 8    ? reinterpret_cast<const void*>(&cd::select_gather_lds_kernel<cd::kSelThreads, 8>)
                     : per == 16 ? reinterpret_cast<const void*>(&cd::select_gather_lds_kernel<cd::kSelThreads, 16>)
                                 : reinterpret_cast<const void*>(&cd::select_gather_lds_kernel<cd::kSelThreads, 32>);
    if ((rc = ensure_kernel_lds(per == 8 ? kLdsSelect8 : per == 16 ? kLdsSelect16 : kLdsSelect32, fn, kSelMaxLdsBytes, "select_gather"))) return rc;
    const dim3 grid(bg), block(cd::kSelThreads);
    if (per == 8) hipLaunchKernelGGL((cd::select_gather_lds_kernel<cd::kSelThreads, 8>), grid, block, lds, st, se);
    else if (per == 16) hipLaunchKernelGGL((cd::select_gather_lds_kernel<cd::kSelThreads, 16>), grid, block, lds, st, se);
    else hipLaunchKernelGGL((cd::select_gather_lds_kernel<cd::kSelThreads, 32>), grid, block, lds, st, se);
  } else {
    cd::WideArgs wa{};
    wa.s = se; wa.NSEG = NSEG;
    wa.hist = sel_hist;
    wa.seg_cnt = sel_cnt;
    sa.zero_words = wa.hist; sa.zero_per_head = 2 * 4 * 256;
    hipLaunchKernelGGL(cd::pool_scores_kernel, dim3(ceil_div(max_seq_len, 256), bg), dim3(256), 0, st, sa);
    if ((rc = launch_status("pool_scores"))) return rc;
    const dim3 grid_w(NSEG, bg);
    if (max_seq_len > p->budget) {
      for (wa.pass = 0; wa.pass < 4; ++wa.pass) {
        hipLaunchKernelGGL(cd::wide_hist_kernel, grid_w, dim3(cd::kWideThreads), 0, st, wa);
        if ((rc = launch_status("wide_hist"))) return rc;
      }
      hipLaunchKernelGGL(cd::wide_count_kernel, grid_w, dim3(cd::kWideThreads), 0, st, wa);
      if ((rc = launch_status("wide_count"))) return rc;
    }
    hipLaunchKernelGGL(cd::wide_emit_kernel, grid_w, dim3(cd::kWideThreads), 0, st, wa);
    if ((rc = launch_status("wide_emit"))) return rc;
    const int vecs = p->budget * (se.row_bytes / 16);
    hipLaunchKernelGGL(cd::gather_kv_kernel, dim3(ceil_div(vecs, 256), bg), dim3(256), 0, st, se);
  }
  return launch_status("select_gather");
}

template <typename T, int D>
int compress_impl(const calidrop_params* p, const void* q_win, const void* k, const void* v,
                  const int32_t* seq_offsets, int64_t total_tokens, int32_t max_seq_len, const float* win_lse,
                  const void* q_cal, void* k_c, void* v_c, const int32_t* cache_offsets, int32_t* cache_lens,
                  int32_t* indices, int32_t* cal_indices, float* c_q, float* c_out, float* c_lse, char* ws,
                  const CompressLayout& L, hipStream_t st) {
  const int G = p->n_q_heads / p->n_kv_heads;
  const float sl2 = logit_scale(p) * cd::kLog2e;
  int rc;

  cd::ScoreArgs sa{};
  sa.q_win = q_win; sa.k = k; sa.seq_off = seq_offsets; sa.total_tokens = total_tokens;
  sa.batch = p->batch; sa.Hq = p->n_q_heads; sa.Hkv = p->n_kv_heads; sa.G = G; sa.w = p->window;
  sa.B = p->budget; sa.R = G * p->window; sa.RB = L.RB; sa.row_stride = L.NRB * L.RB; sa.NRB = L.NRB; sa.NCH = L.NCH; sa.max_seq_len = max_seq_len;
  sa.pool_k = p->pool_kernel; sa.sl2 = sl2; sa.chunk_keys = L.chunk_keys;
  // K of the whole call well inside the 256 MB last-level cache: pass 1 reads it with cached loads so
  // that pass 2 finds it there; larger calls stream it both times
  sa.keep_k = static_cast<int64_t>(total_tokens) * p->n_kv_heads * D * static_cast<int64_t>(sizeof(T)) <= (160ll << 20);
  sa.rowpart = reinterpret_cast<float2*>(ws + L.rowpart);
  sa.row_lse = reinterpret_cast<float*>(ws + L.row_lse);
  sa.vote = reinterpret_cast<float*>(ws + L.vote);
  sa.plane = vote_plane(total_tokens, p->n_kv_heads);
  sa.score = reinterpret_cast<float*>(ws + L.score);
  // default calibration query = last window query: the vote pass exports its logits
  sa.cal_logit = (q_cal || G > cd::kMaxCalHeads || p->window % 4 != 0)
                     ? nullptr : reinterpret_cast<float*>(ws + L.cal_logit);
  sa.zstride = L.zstride;

  const int bg = p->batch * p->n_kv_heads;
  if (max_seq_len > p->budget) {       // otherwise no sequence can need eviction
    dim3 grid_s(L.NCH, bg * L.NRB);
    const int64_t rows = static_cast<int64_t>(bg) * L.NRB * L.RB;
    if (win_lse) {      // pass 1 is the caller's: only a unit conversion into the row table
      hipLaunchKernelGGL(cd::rowlse_import_kernel, dim3(static_cast<unsigned>((rows + 255) / 256)), dim3(256), 0, st, sa,
                         win_lse);
      if ((rc = launch_status("rowlse_import"))) return rc;
    } else {
      if (L.RB == 256) hipLaunchKernelGGL((cd::score_rowstats_direct_kernel<T, D, 4>), grid_s, dim3(256), 0, st, sa);
      else hipLaunchKernelGGL((cd::score_rowstats_direct_kernel<T, D, 2>), grid_s, dim3(256), 0, st, sa);
      if ((rc = launch_status("score_rowstats"))) return rc;
      if (L.NCH > 64) hipLaunchKernelGGL(cd::rowstats_merge_kernel<64>, dim3(static_cast<unsigned>((rows + 3) / 4)), dim3(256), 0, st, sa);
      else hipLaunchKernelGGL(cd::rowstats_merge_kernel<16>, dim3(static_cast<unsigned>((rows + 15) / 16)), dim3(256), 0, st, sa);
      if ((rc = launch_status("rowstats_merge"))) return rc;
    }
    if (L.RB == 256) hipLaunchKernelGGL((cd::score_votes_kernel<T, D, 8>), grid_s, dim3(512), 0, st, sa);
    else hipLaunchKernelGGL((cd::score_votes_kernel<T, D, 4>), grid_s, dim3(256), 0, st, sa);
    if ((rc = launch_status("score_votes"))) return rc;
  }

  // Pooling + selection + gather.  Heads whose pooled scores fit in LDS are pooled inside the
  // selection kernel; longer ones go through the pooled-score buffer in the workspace.
  cd::SelectArgs se{};
  se.seq_off = seq_offsets; se.cache_off = cache_offsets; se.total_tokens = total_tokens; se.batch = p->batch;
  se.Hkv = p->n_kv_heads; se.w = p->window; se.B = p->budget; se.max_seq_len = max_seq_len; se.W32 = L.W32;
  se.NRB = L.NRB; se.pool_k = p->pool_kernel; se.row_bytes = D * static_cast<int>(sizeof(T));
  se.vote = sa.vote; se.plane = sa.plane; se.score = sa.score; se.indices = indices; se.cache_lens = cache_lens;
  se.calib = p->calib_size; se.cal_indices = cal_indices;
  se.bitmap = reinterpret_cast<uint32_t*>(ws + L.bitmap);
  se.k = k; se.v = v; se.k_c = k_c; se.v_c = v_c;
  if ((rc = run_selection(p, p->window, p->pool_kernel, max_seq_len, se, sa, reinterpret_cast<uint32_t*>(ws + L.sel_hist),
                          reinterpret_cast<uint32_t*>(ws + L.sel_cnt), L.NSEG, st)))
    return rc;

  cd::AttendArgs aa{};
  aa.q = q_cal ? q_cal : q_win; aa.q_is_window = q_cal ? 0 : 1;
  aa.k = k; aa.v = v; aa.row_off = seq_offsets; aa.row_len = nullptr; aa.bitmap = se.bitmap;
  aa.total_tokens = total_tokens; aa.batch = p->batch; aa.Hq = p->n_q_heads; aa.Hkv = p->n_kv_heads; aa.G = G;
  aa.w = p->window; aa.B = p->budget; aa.max_len = max_seq_len; aa.W32 = L.W32;
  aa.rows_per_split = L.sp.rows_per_split; aa.NS = L.sp.NS; aa.sl2 = sl2;
  aa.cal_logit = sa.cal_logit; aa.zstride = L.zstride;
  aa.part_o = reinterpret_cast<float*>(ws + L.part_o);
  aa.part_ml = reinterpret_cast<float2*>(ws + L.part_ml);
  if (max_seq_len > p->budget) {
    const dim3 grid_a(L.sp.NS, p->n_kv_heads, p->batch);
    if (aa.cal_logit) hipLaunchKernelGGL((cd::attend_partial_kernel<T, D, true>), grid_a, dim3(256), 0, st, aa);
    else hipLaunchKernelGGL((cd::attend_partial_kernel<T, D, false>), grid_a, dim3(256), 0, st, aa);
    if ((rc = launch_status("attend_partial(calibration)"))) return rc;
  }
  cd::FinalArgs fa{};
  fa.part_o = aa.part_o; fa.part_ml = aa.part_ml; fa.row_off = seq_offsets; fa.row_len = nullptr;
  fa.total_tokens = total_tokens; fa.batch = p->batch; fa.Hq = p->n_q_heads; fa.Hkv = p->n_kv_heads; fa.G = G;
  fa.w = p->window; fa.B = p->budget; fa.max_len = max_seq_len; fa.rows_per_split = L.sp.rows_per_split;
  fa.NS = L.sp.NS; fa.calib_mode = 1; fa.q_is_window = aa.q_is_window; fa.q = aa.q;
  fa.c_q = c_q; fa.c_out = c_out; fa.c_lse = c_lse;
  hipLaunchKernelGGL((cd::attend_finalize_kernel<T, D>), dim3(p->n_q_heads, p->batch), dim3(D), 0, st, fa);
  return launch_status("attend_finalize(calibration)");
}

template <typename T, int D>
int decode_impl(const calidrop_params* p, const void* q_t, const void* k_c, const void* v_c,
                const int32_t* cache_offsets, const int32_t* cache_lens, int32_t max_cache_len, const float* c_q,
                const float* c_out, const float* c_lse, void* out, float* a_lse, uint8_t* flags, char* ws,
                const DecodeLayout& L, hipStream_t st) {
  const int G = p->n_q_heads / p->n_kv_heads;
  int rc;
  // Enough (sequence, KV head) pairs to fill the chip: one workgroup does a pair's whole step.
  if (p->batch * p->n_kv_heads >= kFusedMinPairs || max_cache_len <= kFusedMaxRowsFewPairs) {
    cd::DecodeFusedArgs fa{};
    fa.q = q_t; fa.k = k_c; fa.v = v_c; fa.row_off = cache_offsets; fa.row_len = cache_lens;
    fa.batch = p->batch; fa.Hq = p->n_q_heads; fa.Hkv = p->n_kv_heads; fa.G = G; fa.max_len = max_cache_len;
    fa.sl2 = logit_scale(p) * cd::kLog2e; fa.theta1 = p->theta1; fa.theta2 = p->theta2;
    fa.c_q = c_q; fa.c_out = c_out; fa.c_lse = c_lse; fa.out = out; fa.a_lse = a_lse; fa.flags = flags;
    const int tiles = ceil_div(max_cache_len, cd::kTileRows);
    const size_t lds_per_wave = static_cast<size_t>(G) * (D + 2) * sizeof(float);
    // 4 waves per workgroup when the pairs fill the chip (measured against 8 waves, same call: 12.8 vs
    // 13.0 us at 512 rows; 40.5 vs 42.0 us at 2048 rows, where three such workgroups share a compute
    // unit and one's merge overlaps the others' streaming) and for caches of at most 4 tiles; 8 waves
    // when few pairs have to cover the latency with more rows in flight each.
    const bool many_pairs = p->batch * p->n_kv_heads >= kFusedMinPairs;
    int nw = (tiles <= 4 || many_pairs) ? 4 : 8;
    while (nw > 4 && nw * lds_per_wave > 48 * 1024) nw /= 2;     // what a launch may use without raising the limit
    fa.xcd_blocks = (tiles >= 32 && p->batch % 8 == 0) ? 1 : 0;
    const dim3 grid(p->n_kv_heads, p->batch);
    const size_t lds = nw * lds_per_wave;
    if (nw == 8) hipLaunchKernelGGL((cd::decode_fused_kernel<T, D, 8>), grid, dim3(512), lds, st, fa);
    else hipLaunchKernelGGL((cd::decode_fused_kernel<T, D, 4>), grid, dim3(256), lds, st, fa);
    return launch_status("decode_fused");
  }
  cd::AttendArgs aa{};
  aa.q = q_t; aa.q_is_window = 0; aa.k = k_c; aa.v = v_c; aa.row_off = cache_offsets; aa.row_len = cache_lens;
  aa.bitmap = nullptr; aa.total_tokens = 0; aa.batch = p->batch; aa.Hq = p->n_q_heads; aa.Hkv = p->n_kv_heads;
  aa.G = G; aa.w = p->window; aa.B = p->budget; aa.max_len = max_cache_len; aa.W32 = 0;
  aa.rows_per_split = L.sp.rows_per_split; aa.NS = L.sp.NS; aa.sl2 = logit_scale(p) * cd::kLog2e;
  aa.cal_logit = nullptr; aa.zstride = 0;
  aa.part_o = reinterpret_cast<float*>(ws + L.part_o);
  aa.part_ml = reinterpret_cast<float2*>(ws + L.part_ml);
  hipLaunchKernelGGL((cd::attend_partial_kernel<T, D, false>), dim3(L.sp.NS, p->n_kv_heads, p->batch), dim3(256), 0,
                     st, aa);
  if ((rc = launch_status("attend_partial(decode)"))) return rc;
  cd::FinalArgs fa{};
  fa.part_o = aa.part_o; fa.part_ml = aa.part_ml; fa.row_off = cache_offsets; fa.row_len = cache_lens;
  fa.total_tokens = 0; fa.batch = p->batch; fa.Hq = p->n_q_heads; fa.Hkv = p->n_kv_heads; fa.G = G;
  fa.w = p->window; fa.B = p->budget; fa.max_len = max_cache_len; fa.rows_per_split = L.sp.rows_per_split;
  fa.NS = L.sp.NS; fa.calib_mode = 0; fa.q_is_window = 0; fa.q = q_t; fa.theta1 = p->theta1; fa.theta2 = p->theta2;
  fa.c_q = const_cast<float*>(c_q); fa.c_out = const_cast<float*>(c_out); fa.c_lse = const_cast<float*>(c_lse);
  fa.out = out; fa.a_lse = a_lse; fa.flags = flags;
  hipLaunchKernelGGL((cd::attend_finalize_kernel<T, D>), dim3(p->n_q_heads, p->batch), dim3(D), 0, st, fa);
  return launch_status("attend_finalize(decode)");
}

struct RecalLayout { size_t bitmap, part_o, part_ml, total; int W32; SplitPlan sp; };

RecalLayout recal_layout(const calidrop_params* p, int32_t max_seq_len) {
  RecalLayout L{};
  L.W32 = ceil_div(max_seq_len, 64) * 2;
  L.sp = plan_splits(p->batch * p->n_kv_heads, max_seq_len);
  const size_t slots = static_cast<size_t>(p->batch) * p->n_q_heads * L.sp.NS;
  size_t off = 0;
  L.bitmap = off;  off += round256(static_cast<size_t>(p->batch) * p->n_kv_heads * L.W32 * sizeof(uint32_t));
  L.part_o = off;  off += round256(slots * p->head_dim * sizeof(float));
  L.part_ml = off; off += round256(slots * sizeof(float2));
  L.total = off;
  return L;
}

template <typename T, int D>
int recal_impl(const calidrop_params* p, const void* q_t, const void* k, const void* v, const int32_t* seq_offsets,
               int64_t total_tokens, int32_t max_seq_len, const int32_t* indices, const int32_t* cal_indices,
               uint8_t* flags, const float* a_lse, void* out, float* c_q, float* c_out, float* c_lse, char* ws,
               const RecalLayout& L, hipStream_t st) {
  const int G = p->n_q_heads / p->n_kv_heads;
  int rc;
  cd::BitmapArgs ba{};
  ba.seq_off = seq_offsets; ba.indices = indices; ba.cal_indices = cal_indices;
  ba.bitmap = reinterpret_cast<uint32_t*>(ws + L.bitmap); ba.calib = p->calib_size;
  ba.total_tokens = total_tokens; ba.batch = p->batch; ba.Hkv = p->n_kv_heads; ba.B = p->budget;
  ba.max_seq_len = max_seq_len; ba.W32 = L.W32;
  ba.only_flagged = flags; ba.Hq = p->n_q_heads; ba.G = G;
  launch_bitmap(ba, p->batch * p->n_kv_heads, st);
  if ((rc = launch_status("bitmap_from_indices"))) return rc;

  cd::AttendArgs aa{};
  aa.q = q_t; aa.q_is_window = 0; aa.k = k; aa.v = v; aa.row_off = seq_offsets; aa.row_len = nullptr;
  aa.bitmap = ba.bitmap; aa.total_tokens = total_tokens; aa.batch = p->batch; aa.Hq = p->n_q_heads;
  // w = 0: the pass covers every position; the bitmap masks the retained ones, window included
  aa.Hkv = p->n_kv_heads; aa.G = G; aa.w = 0; aa.B = p->budget; aa.max_len = max_seq_len; aa.W32 = L.W32;
  aa.rows_per_split = L.sp.rows_per_split; aa.NS = L.sp.NS; aa.sl2 = logit_scale(p) * cd::kLog2e;
  aa.cal_logit = nullptr; aa.zstride = 0; aa.only_flagged = flags;
  aa.part_o = reinterpret_cast<float*>(ws + L.part_o);
  aa.part_ml = reinterpret_cast<float2*>(ws + L.part_ml);
  hipLaunchKernelGGL((cd::attend_partial_kernel<T, D, false>), dim3(L.sp.NS, p->n_kv_heads, p->batch), dim3(256), 0,
                     st, aa);
  if ((rc = launch_status("attend_partial(recalibrate)"))) return rc;

  cd::FinalArgs fa{};
  fa.part_o = aa.part_o; fa.part_ml = aa.part_ml; fa.row_off = seq_offsets; fa.row_len = nullptr;
  fa.total_tokens = total_tokens; fa.batch = p->batch; fa.Hq = p->n_q_heads; fa.Hkv = p->n_kv_heads; fa.G = G;
  fa.w = 0; fa.B = p->budget; fa.max_len = max_seq_len; fa.rows_per_split = L.sp.rows_per_split;
  fa.NS = L.sp.NS; fa.calib_mode = 2; fa.q_is_window = 0; fa.q = q_t;
  fa.c_q = c_q; fa.c_out = c_out; fa.c_lse = c_lse; fa.out = out; fa.a_lse = const_cast<float*>(a_lse); fa.flags = flags;
  hipLaunchKernelGGL((cd::attend_finalize_kernel<T, D>), dim3(p->n_q_heads, p->batch), dim3(D), 0, st, fa);
  return launch_status("attend_finalize(recalibrate)");
}

// Alg. 1 steps 4-8 for a retained set that is already known (caller's strategy, or the
// StreamingLLM list): bitmap + cache_lens, gather, calibration pass over everything else.
template <typename T, int D>
int compress_given_impl(const calidrop_params* p, const void* q_cal, const void* k, const void* v,
                        const int32_t* seq_offsets, int64_t total_tokens, int32_t max_seq_len, int32_t* indices,
                        void* k_c, void* v_c, const int32_t* cache_offsets, int32_t* cache_lens, float* c_q,
                        float* c_out, float* c_lse, char* ws, const RecalLayout& L, hipStream_t st) {
  const int G = p->n_q_heads / p->n_kv_heads;
  const int bg = p->batch * p->n_kv_heads;
  int rc;
  cd::GivenArgs ga{};
  ga.seq_off = seq_offsets; ga.total_tokens = total_tokens; ga.batch = p->batch; ga.Hkv = p->n_kv_heads;
  ga.B = p->budget; ga.max_seq_len = max_seq_len; ga.W32 = L.W32; ga.indices = indices; ga.cache_lens = cache_lens;
  ga.bitmap = reinterpret_cast<uint32_t*>(ws + L.bitmap);
  hipLaunchKernelGGL(cd::given_prepare_kernel, dim3(bg), dim3(256), 0, st, ga);
  if ((rc = launch_status("given_prepare"))) return rc;

  cd::SelectArgs se{};
  se.seq_off = seq_offsets; se.cache_off = cache_offsets; se.total_tokens = total_tokens; se.batch = p->batch;
  se.Hkv = p->n_kv_heads; se.w = 0; se.B = p->budget; se.max_seq_len = max_seq_len; se.W32 = L.W32;
  se.row_bytes = D * static_cast<int>(sizeof(T)); se.indices = indices; se.cache_lens = cache_lens;
  se.k = k; se.v = v; se.k_c = k_c; se.v_c = v_c;
  const int vecs = p->budget * (se.row_bytes / 16);
  hipLaunchKernelGGL(cd::gather_kv_kernel, dim3(ceil_div(vecs, 256), bg), dim3(256), 0, st, se);
  if ((rc = launch_status("gather_kv"))) return rc;

  cd::AttendArgs aa{};
  aa.q = q_cal; aa.q_is_window = 0; aa.k = k; aa.v = v; aa.row_off = seq_offsets; aa.row_len = nullptr;
  aa.bitmap = ga.bitmap; aa.total_tokens = total_tokens; aa.batch = p->batch; aa.Hq = p->n_q_heads;
  aa.Hkv = p->n_kv_heads; aa.G = G; aa.w = 0; aa.B = p->budget; aa.max_len = max_seq_len; aa.W32 = L.W32;
  aa.rows_per_split = L.sp.rows_per_split; aa.NS = L.sp.NS; aa.sl2 = logit_scale(p) * cd::kLog2e;
  aa.part_o = reinterpret_cast<float*>(ws + L.part_o);
  aa.part_ml = reinterpret_cast<float2*>(ws + L.part_ml);
  if (max_seq_len > p->budget) {
    hipLaunchKernelGGL((cd::attend_partial_kernel<T, D, false>), dim3(L.sp.NS, p->n_kv_heads, p->batch), dim3(256), 0,
                       st, aa);
    if ((rc = launch_status("attend_partial(given)"))) return rc;
  }
  cd::FinalArgs fa{};
  fa.part_o = aa.part_o; fa.part_ml = aa.part_ml; fa.row_off = seq_offsets; fa.row_len = nullptr;
  fa.total_tokens = total_tokens; fa.batch = p->batch; fa.Hq = p->n_q_heads; fa.Hkv = p->n_kv_heads; fa.G = G;
  fa.w = 0; fa.B = p->budget; fa.max_len = max_seq_len; fa.rows_per_split = L.sp.rows_per_split;
  fa.NS = L.sp.NS; fa.calib_mode = 1; fa.q_is_window = 0; fa.q = q_cal;
  fa.c_q = c_q; fa.c_out = c_out; fa.c_lse = c_lse;
  hipLaunchKernelGGL((cd::attend_finalize_kernel<T, D>), dim3(p->n_q_heads, p->batch), dim3(D), 0, st, fa);
  return launch_status("attend_finalize(given)");
}

int packed_rows_host(const calidrop_params* p, int n) {
  if (n <= p->budget) return 0;
  return p->calib_size > 0 ? std::min(p->calib_size, n - p->budget) : n - p->budget;
}

struct PackLayout { size_t bitmap, total; int W32; };
PackLayout pack_layout(const calidrop_params* p, int32_t max_seq_len) {
  PackLayout L{};
  L.W32 = ceil_div(max_seq_len, 64) * 2;
  L.bitmap = 0;
  L.total = round256(static_cast<size_t>(p->batch) * p->n_kv_heads * L.W32 * sizeof(uint32_t));
  return L;
}

// KV_evict (or the calibration set) of every head as contiguous rows, ready to be moved elsewhere.
int pack_impl(const calidrop_params* p, const void* k, const void* v, const int32_t* seq_offsets, int64_t total_tokens,
              int32_t max_seq_len, const int32_t* indices, const int32_t* cal_indices, void* k_e, void* v_e,
              const int32_t* evict_offsets, int32_t* evict_lens, int32_t* evict_indices, char* ws,
              const PackLayout& L, hipStream_t st) {
  int rc;
  const int bg = p->batch * p->n_kv_heads;
  cd::BitmapArgs ba{};
  ba.seq_off = seq_offsets; ba.indices = indices; ba.cal_indices = cal_indices;
  ba.bitmap = reinterpret_cast<uint32_t*>(ws + L.bitmap); ba.calib = p->calib_size;
  ba.total_tokens = total_tokens; ba.batch = p->batch; ba.Hkv = p->n_kv_heads; ba.B = p->budget;
  ba.max_seq_len = max_seq_len; ba.W32 = L.W32;
  ba.only_flagged = nullptr; ba.Hq = p->n_q_heads; ba.G = p->n_q_heads / p->n_kv_heads;
  launch_bitmap(ba, bg, st);
  if ((rc = launch_status("bitmap_from_indices"))) return rc;
  cd::PackArgs pa{};
  pa.seq_off = seq_offsets; pa.evict_off = evict_offsets; pa.total_tokens = total_tokens; pa.batch = p->batch;
  pa.Hkv = p->n_kv_heads; pa.B = p->budget; pa.calib = p->calib_size; pa.max_seq_len = max_seq_len; pa.W32 = L.W32;
  pa.row_bytes = p->head_dim * (p->dtype == CALIDROP_BF16 ? 2 : 4);
  pa.bitmap = ba.bitmap; pa.evict_lens = evict_lens; pa.evict_indices = evict_indices;
  pa.k = k; pa.v = v; pa.k_e = k_e; pa.v_e = v_e;
  hipLaunchKernelGGL(cd::evict_list_kernel, dim3(bg), dim3(256), 0, st, pa);
  if ((rc = launch_status("evict_list"))) return rc;
  const int max_rows = packed_rows_host(p, max_seq_len);
  if (max_rows > 0) {
    const int64_t vecs = static_cast<int64_t>(max_rows) * (pa.row_bytes / 16);
    hipLaunchKernelGGL(cd::pack_gather_kernel, dim3(static_cast<unsigned>((vecs + 255) / 256), bg), dim3(256), 0, st, pa);
    if ((rc = launch_status("pack_gather"))) return rc;
  }
  return CALIDROP_OK;
}

// Recomputation branch over the packed rows: the same streaming pass and tail as calidrop_recalibrate,
// with the geometry of a packed buffer (offsets + live rows) instead of a prompt and its skip bitmap.
bool is_host_memory(const void* ptr) {
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, ptr) != hipSuccess) {
    (void)hipGetLastError();                     // a pointer the runtime does not know: treat as device memory
    return false;
  }
  return attr.type == hipMemoryTypeHost;
}

template <typename T, int D>
int recal_packed_impl(const calidrop_params* p, const void* q_t, const void* k_e, const void* v_e,
                      const int32_t* evict_offsets, const int32_t* evict_lens, int32_t max_evict_len, uint8_t* flags,
                      const float* a_lse, void* out, float* c_q, float* c_out, float* c_lse, char* ws,
                      const DecodeLayout& L, hipStream_t st) {
  const int G = p->n_q_heads / p->n_kv_heads;
  int rc;
  cd::AttendArgs aa{};
  aa.q = q_t; aa.q_is_window = 0; aa.k = k_e; aa.v = v_e; aa.row_off = evict_offsets; aa.row_len = evict_lens;
  aa.bitmap = nullptr; aa.total_tokens = 0; aa.batch = p->batch; aa.Hq = p->n_q_heads; aa.Hkv = p->n_kv_heads;
  aa.G = G; aa.w = 0; aa.B = p->budget; aa.max_len = max_evict_len; aa.W32 = 0;
  aa.rows_per_split = L.sp.rows_per_split; aa.NS = L.sp.NS; aa.sl2 = logit_scale(p) * cd::kLog2e;
  aa.only_flagged = flags;
  aa.part_o = reinterpret_cast<float*>(ws + L.part_o);
  aa.part_ml = reinterpret_cast<float2*>(ws + L.part_ml);
  // rows in host memory (the offloaded form) are requested as whole rows: the host link moves the
  // 64-byte pieces of the operand layout a quarter slower
  const dim3 grid(L.sp.NS, p->n_kv_heads, p->batch);
  if (is_host_memory(k_e)) hipLaunchKernelGGL((cd::attend_partial_kernel<T, D, false, true>), grid, dim3(256), 0, st, aa);
  else hipLaunchKernelGGL((cd::attend_partial_kernel<T, D, false>), grid, dim3(256), 0, st, aa);
  if ((rc = launch_status("attend_partial(recalibrate, packed)"))) return rc;
  cd::FinalArgs fa{};
  fa.part_o = aa.part_o; fa.part_ml = aa.part_ml; fa.row_off = evict_offsets; fa.row_len = evict_lens;
  fa.total_tokens = 0; fa.batch = p->batch; fa.Hq = p->n_q_heads; fa.Hkv = p->n_kv_heads; fa.G = G;
  fa.w = 0; fa.B = p->budget; fa.max_len = max_evict_len; fa.rows_per_split = L.sp.rows_per_split;
  fa.NS = L.sp.NS; fa.calib_mode = 2; fa.q_is_window = 0; fa.q = q_t;
  fa.c_q = c_q; fa.c_out = c_out; fa.c_lse = c_lse; fa.out = out; fa.a_lse = const_cast<float*>(a_lse); fa.flags = flags;
  hipLaunchKernelGGL((cd::attend_finalize_kernel<T, D>), dim3(p->n_q_heads, p->batch), dim3(D), 0, st, fa);
  return launch_status("attend_finalize(recalibrate, packed)");
}

constexpr int kH2oRowTiles = CD_H2O_ROW_TILES;        // 16-row tiles per wave in the H2O scoring passes
constexpr int kH2oBlock = 4 * 16 * kH2oRowTiles;      // stationary rows (or keys) per workgroup

struct H2oLayout {
  size_t row_lse, vote, score, bitmap, q_last, part_o, part_ml, sel_hist, sel_cnt, total;
  int lse_stride, W32, NSEG;
  SplitPlan sp;
};

H2oLayout h2o_layout(const calidrop_params* p, int64_t total_tokens, int32_t max_seq_len, int n_local) {
  H2oLayout L{};
  L.lse_stride = ceil_div(max_seq_len, 256) * 256;
  L.W32 = ceil_div(max_seq_len, 64) * 2;
  L.sp = plan_splits(p->batch * p->n_kv_heads, max_seq_len);
  L.NSEG = ceil_div(std::max(max_seq_len - n_local, 1), cd::kWideSeg);
  const size_t toks = static_cast<size_t>(total_tokens) * p->n_kv_heads;
  const size_t slots = static_cast<size_t>(p->batch) * p->n_q_heads * L.sp.NS;
  size_t off = 0;
  L.row_lse = off; off += round256(static_cast<size_t>(p->batch) * p->n_q_heads * L.lse_stride * sizeof(float));
  L.vote = off;    // one plane per head of a group
  off += round256(static_cast<size_t>(vote_plane(total_tokens, p->n_kv_heads)) * (p->n_q_heads / p->n_kv_heads) * sizeof(float));
  L.score = off;   off += round256(toks * sizeof(float));
  L.bitmap = off;  off += round256(static_cast<size_t>(p->batch) * p->n_kv_heads * L.W32 * sizeof(uint32_t));
  L.q_last = off;  off += round256(static_cast<size_t>(p->batch) * p->n_q_heads * p->head_dim * sizeof(float));
  L.part_o = off;  off += round256(slots * p->head_dim * sizeof(float));
  L.part_ml = off; off += round256(slots * sizeof(float2));
  L.sel_hist = off; off += round256(static_cast<size_t>(p->batch) * p->n_kv_heads * 2 * 4 * 256 * sizeof(uint32_t));
  L.sel_cnt = off;  off += round256(static_cast<size_t>(p->batch) * p->n_kv_heads * L.NSEG * 4 * sizeof(uint32_t));
  L.total = off;
  return L;
}

// Alg. 1 steps 3-8 with H2O as f: accumulated attention of every prompt query (two dense passes),
// top-(B - n_local) among the positions outside the local window, gather, calibration state.
template <typename T, int D>
int h2o_impl(const calidrop_params* p, int n_local, const void* q_full, const void* k, const void* v,
             const int32_t* seq_offsets, int64_t total_tokens, int32_t max_seq_len, void* k_c, void* v_c,
             const int32_t* cache_offsets, int32_t* cache_lens, int32_t* indices, int32_t* cal_indices, float* c_q,
             float* c_out, float* c_lse, char* ws, const H2oLayout& L, hipStream_t st) {
  const int G = p->n_q_heads / p->n_kv_heads;
  const int bg = p->batch * p->n_kv_heads;
  const float sl2 = logit_scale(p) * cd::kLog2e;
  int rc;
  cd::H2oArgs ha{};
  ha.q_full = q_full; ha.k = k; ha.seq_off = seq_offsets; ha.total_tokens = total_tokens; ha.batch = p->batch;
  ha.Hq = p->n_q_heads; ha.Hkv = p->n_kv_heads; ha.G = G; ha.B = p->budget; ha.max_seq_len = max_seq_len;
  ha.lse_stride = L.lse_stride; ha.sl2 = sl2;
  ha.row_lse = reinterpret_cast<float*>(ws + L.row_lse);
  ha.vote = reinterpret_cast<float*>(ws + L.vote);
  ha.plane = vote_plane(total_tokens, p->n_kv_heads);
  ha.q_last = ws + L.q_last;
  const int nblk = ceil_div(max_seq_len, kH2oBlock);
  // always launched: it also extracts Q_{-1}, which prompts within the budget need as C_q
  hipLaunchKernelGGL((cd::h2o_rowlse_kernel<T, D, kH2oRowTiles>), dim3(nblk, p->batch * p->n_q_heads), dim3(256), 0, st, ha);
  if ((rc = launch_status("h2o_rowlse"))) return rc;
  if (max_seq_len > p->budget) {
    hipLaunchKernelGGL((cd::h2o_votes_kernel<T, D, kH2oRowTiles>), dim3((nblk + 1) / 2, bg, G), dim3(256), 0, st, ha);
    if ((rc = launch_status("h2o_votes"))) return rc;
  }
  // selection: the votes are the scores (no pooling); the local window plays the part of the
  // observation window (always kept, not a candidate)
  cd::ScoreArgs sa{};
  sa.seq_off = seq_offsets; sa.total_tokens = total_tokens; sa.batch = p->batch; sa.Hq = p->n_q_heads;
  sa.Hkv = p->n_kv_heads; sa.G = G; sa.w = n_local; sa.B = p->budget; sa.NRB = G; sa.max_seq_len = max_seq_len;
  sa.pool_k = 1; sa.vote = ha.vote; sa.plane = ha.plane; sa.score = reinterpret_cast<float*>(ws + L.score);
  cd::SelectArgs se{};
  se.seq_off = seq_offsets; se.cache_off = cache_offsets; se.total_tokens = total_tokens; se.batch = p->batch;
  se.Hkv = p->n_kv_heads; se.w = n_local; se.B = p->budget; se.max_seq_len = max_seq_len; se.W32 = L.W32;
  se.NRB = G; se.pool_k = 1; se.row_bytes = D * static_cast<int>(sizeof(T));
  se.vote = sa.vote; se.plane = sa.plane; se.score = sa.score; se.indices = indices; se.cache_lens = cache_lens;
  se.calib = p->calib_size; se.cal_indices = cal_indices;
  se.bitmap = reinterpret_cast<uint32_t*>(ws + L.bitmap);
  se.k = k; se.v = v; se.k_c = k_c; se.v_c = v_c;
  if ((rc = run_selection(p, n_local, 1, max_seq_len, se, sa, reinterpret_cast<uint32_t*>(ws + L.sel_hist),
                          reinterpret_cast<uint32_t*>(ws + L.sel_cnt), L.NSEG, st)))
    return rc;

  cd::AttendArgs aa{};
  aa.q = ha.q_last; aa.q_is_window = 0; aa.k = k; aa.v = v; aa.row_off = seq_offsets; aa.row_len = nullptr;
  aa.bitmap = se.bitmap; aa.total_tokens = total_tokens; aa.batch = p->batch; aa.Hq = p->n_q_heads;
  aa.Hkv = p->n_kv_heads; aa.G = G; aa.w = n_local; aa.B = p->budget; aa.max_len = max_seq_len; aa.W32 = L.W32;
  aa.rows_per_split = L.sp.rows_per_split; aa.NS = L.sp.NS; aa.sl2 = sl2;
  aa.part_o = reinterpret_cast<float*>(ws + L.part_o);
  aa.part_ml = reinterpret_cast<float2*>(ws + L.part_ml);
  if (max_seq_len > p->budget) {
    hipLaunchKernelGGL((cd::attend_partial_kernel<T, D, false>), dim3(L.sp.NS, p->n_kv_heads, p->batch), dim3(256), 0,
                       st, aa);
    if ((rc = launch_status("attend_partial(h2o)"))) return rc;
  }
  cd::FinalArgs fa{};
  fa.part_o = aa.part_o; fa.part_ml = aa.part_ml; fa.row_off = seq_offsets; fa.row_len = nullptr;
  fa.total_tokens = total_tokens; fa.batch = p->batch; fa.Hq = p->n_q_heads; fa.Hkv = p->n_kv_heads; fa.G = G;
  fa.w = n_local; fa.B = p->budget; fa.max_len = max_seq_len; fa.rows_per_split = L.sp.rows_per_split;
  fa.NS = L.sp.NS; fa.calib_mode = 1; fa.q_is_window = 0; fa.q = ha.q_last;
  fa.c_q = c_q; fa.c_out = c_out; fa.c_lse = c_lse;
  hipLaunchKernelGGL((cd::attend_finalize_kernel<T, D>), dim3(p->n_q_heads, p->batch), dim3(D), 0, st, fa);
  return launch_status("attend_finalize(h2o)");
}

}  // namespace

extern "C" {

const char* calidrop_last_error(void) { return g_err; }
int calidrop_version(void) { return 200; }

size_t calidrop_compress_workspace_bytes(const calidrop_params* p_in, int64_t total_tokens, int32_t max_seq_len) {
  calidrop_params pp; const calidrop_params* p = &pp;
  if (load_params(p_in, &pp) != CALIDROP_OK) return 0;
  if (check_params(p) != CALIDROP_OK || check_sizes(p, total_tokens, max_seq_len) != CALIDROP_OK) return 0;
  return compress_layout(p, total_tokens, max_seq_len).total;
}

size_t calidrop_decode_workspace_bytes(const calidrop_params* p_in, int32_t max_cache_len) {
  calidrop_params pp; const calidrop_params* p = &pp;
  if (load_params(p_in, &pp) != CALIDROP_OK) return 0;
  if (check_params(p) != CALIDROP_OK) return 0;
  if (max_cache_len < 1) { fail(CALIDROP_ESHAPE, "max_cache_len must be >= 1"); return 0; }
  return decode_layout(p, max_cache_len).total;
}

int calidrop_compress_workspace_region(const calidrop_params* p_in, int64_t total_tokens, int32_t max_seq_len,
                                       int32_t region, size_t* offset, size_t* bytes) {
  int rc;
  calidrop_params pp; const calidrop_params* p = &pp;
  if ((rc = load_params(p_in, &pp))) return rc;
  if ((rc = check_params(p))) return rc;
  if ((rc = check_sizes(p, total_tokens, max_seq_len))) return rc;
  if (!offset || !bytes) return fail(CALIDROP_EINVAL, "offset/bytes is NULL");
  const CompressLayout L = compress_layout(p, total_tokens, max_seq_len);
  if (region == CALIDROP_REGION_ROW_LSE) {
    *offset = L.row_lse;
    *bytes = static_cast<size_t>(p->batch) * p->n_kv_heads * L.NRB * L.RB * sizeof(float);
  } else if (region == CALIDROP_REGION_SCORE) {
    *offset = L.score;
    *bytes = static_cast<size_t>(total_tokens) * p->n_kv_heads * sizeof(float);
  } else {
    return fail(CALIDROP_EINVAL, "unknown workspace region %d", region);
  }
  return CALIDROP_OK;
}

int calidrop_compress(const calidrop_params* p_in, const void* q_win, const void* k, const void* v,
                      const int32_t* seq_offsets, int64_t total_tokens, int32_t max_seq_len, const void* q_cal,
                      void* k_c, void* v_c, const int32_t* cache_offsets, int32_t* cache_lens, int32_t* indices,
                      int32_t* cal_indices, float* c_q, float* c_out, float* c_lse, void* workspace,
                      size_t workspace_bytes, void* stream) {
  return calidrop_compress_with_lse(p_in, q_win, k, v, seq_offsets, total_tokens, max_seq_len, nullptr, q_cal, k_c, v_c,
                                    cache_offsets, cache_lens, indices, cal_indices, c_q, c_out, c_lse, workspace,
                                    workspace_bytes, stream);
}

int calidrop_compress_with_lse(const calidrop_params* p_in, const void* q_win, const void* k, const void* v,
                               const int32_t* seq_offsets, int64_t total_tokens, int32_t max_seq_len,
                               const float* win_lse, const void* q_cal, void* k_c, void* v_c,
                               const int32_t* cache_offsets, int32_t* cache_lens, int32_t* indices,
                               int32_t* cal_indices, float* c_q, float* c_out, float* c_lse, void* workspace,
                               size_t workspace_bytes, void* stream) {
  int rc;
  calidrop_params pp; const calidrop_params* p = &pp;
  if ((rc = load_params(p_in, &pp))) return rc;
  if ((rc = check_params(p))) return rc;
  if ((rc = check_sizes(p, total_tokens, max_seq_len))) return rc;
  const struct { const void* ptr; const char* name; } req[] = {
      {q_win, "q_win"}, {k, "k"}, {v, "v"}, {seq_offsets, "seq_offsets"}, {k_c, "k_c"}, {v_c, "v_c"},
      {cache_offsets, "cache_offsets"}, {cache_lens, "cache_lens"}, {indices, "indices"}, {c_q, "c_q"},
      {c_out, "c_out"}, {c_lse, "c_lse"}};
  for (const auto& r : req)
    if (!r.ptr) return fail(CALIDROP_EINVAL, "%s is NULL", r.name);
  for (const auto& r : req)
    if (!aligned16(r.ptr)) return fail(CALIDROP_EALIGN, "%s is not 16-byte aligned", r.name);
  if (q_cal && !aligned16(q_cal)) return fail(CALIDROP_EALIGN, "q_cal is not 16-byte aligned");
  if (win_lse && !aligned16(win_lse)) return fail(CALIDROP_EALIGN, "win_lse is not 16-byte aligned");
  if (p->calib_size > 0) {
    if (!cal_indices) return fail(CALIDROP_EINVAL, "cal_indices is NULL although calib_size is %d", p->calib_size);
    if (!aligned16(cal_indices)) return fail(CALIDROP_EALIGN, "cal_indices is not 16-byte aligned");
  } else {
    cal_indices = nullptr;
  }
  const CompressLayout L = compress_layout(p, total_tokens, max_seq_len);
  if (!workspace || workspace_bytes < L.total)
    return fail(CALIDROP_EWORKSPACE, "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : 0,
                L.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(CALIDROP_EALIGN, "workspace is not 256-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
#define CD_DISPATCH(T, D)                                                                                       \
  return compress_impl<T, D>(p, q_win, k, v, seq_offsets, total_tokens, max_seq_len, win_lse, q_cal, k_c, v_c,  \
                             cache_offsets, cache_lens, indices, cal_indices, c_q, c_out, c_lse, ws, L, st)
  if (p->dtype == CALIDROP_BF16) {
    if (p->head_dim == 128) CD_DISPATCH(cd::bf16_t, 128);
    CD_DISPATCH(cd::bf16_t, 64);
  }
  if (p->head_dim == 128) CD_DISPATCH(float, 128);
  CD_DISPATCH(float, 64);
#undef CD_DISPATCH
}

namespace {
// calidrop_decode and calidrop_decode_static: the same validation and launches; they differ in where
// the scratch for the split partials comes from (the caller's workspace, or the fixed per-GPU array).
int decode_entry(const calidrop_params* p_in, const void* q_t, const void* k_c, const void* v_c,
                 const int32_t* cache_offsets, const int32_t* cache_lens, int32_t max_cache_len, const float* c_q,
                 const float* c_out, const float* c_lse, void* out, float* a_lse, uint8_t* flags, void* workspace,
                 size_t workspace_bytes, bool fixed_scratch, void* stream) {
  int rc;
  calidrop_params pp; const calidrop_params* p = &pp;
  if ((rc = load_params(p_in, &pp))) return rc;
  if ((rc = check_params(p))) return rc;
  if (max_cache_len < 1) return fail(CALIDROP_ESHAPE, "max_cache_len must be >= 1 (got %d)", max_cache_len);
  const struct { const void* ptr; const char* name; } req[] = {
      {q_t, "q_t"}, {k_c, "k_c"}, {v_c, "v_c"}, {cache_lens, "cache_lens"},
      {c_q, "c_q"}, {c_out, "c_out"}, {c_lse, "c_lse"}, {out, "out"}};
  for (const auto& r : req)
    if (!r.ptr) return fail(CALIDROP_EINVAL, "%s is NULL", r.name);
  for (const auto& r : req)
    if (!aligned16(r.ptr)) return fail(CALIDROP_EALIGN, "%s is not 16-byte aligned", r.name);
  if (cache_offsets) {
    if (!aligned16(cache_offsets)) return fail(CALIDROP_EALIGN, "cache_offsets is not 16-byte aligned");
  } else if (static_cast<int64_t>(p->batch) * max_cache_len > (static_cast<int64_t>(1) << 31) - 1) {
    return fail(CALIDROP_EUNSUPPORTED, "batch * max_cache_len exceeds int32 offsets (uniform layout)");
  }
  const DecodeLayout L = decode_layout(p, max_cache_len);
  char* ws = static_cast<char*>(workspace);
  if (fixed_scratch) {
    if (L.total > kStaticScratchBytes)
      return fail(CALIDROP_EWORKSPACE, "this call needs %zu bytes of scratch and the fixed array holds %zu: use "
                  "calidrop_decode with a workspace", L.total, kStaticScratchBytes);
    if ((rc = static_scratch_ptr(&ws))) return rc;       // the first HIP call, after all validation
  } else {
    if (!workspace || workspace_bytes < L.total)
      return fail(CALIDROP_EWORKSPACE, "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : 0,
                  L.total);
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(CALIDROP_EALIGN, "workspace is not 256-byte aligned");
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
#define CD_DISPATCH(T, D)                                                                                      \
  return decode_impl<T, D>(p, q_t, k_c, v_c, cache_offsets, cache_lens, max_cache_len, c_q, c_out, c_lse, out, \
                           a_lse, flags, ws, L, st)
  if (p->dtype == CALIDROP_BF16) {
    if (p->head_dim == 128) CD_DISPATCH(cd::bf16_t, 128);
    CD_DISPATCH(cd::bf16_t, 64);
  }
  if (p->head_dim == 128) CD_DISPATCH(float, 128);
  CD_DISPATCH(float, 64);
#undef CD_DISPATCH
}
}  // namespace

int calidrop_decode(const calidrop_params* p_in, const void* q_t, const void* k_c, const void* v_c,
                    const int32_t* cache_offsets, const int32_t* cache_lens, int32_t max_cache_len,
                    const float* c_q, const float* c_out, const float* c_lse, void* out, float* a_lse,
                    uint8_t* flags, void* workspace, size_t workspace_bytes, void* stream) {
  return decode_entry(p_in, q_t, k_c, v_c, cache_offsets, cache_lens, max_cache_len, c_q, c_out, c_lse, out, a_lse,
                      flags, workspace, workspace_bytes, false, stream);
}

int calidrop_decode_static(const calidrop_params* p_in, const void* q_t, const void* k_c, const void* v_c,
                           const int32_t* cache_offsets, const int32_t* cache_lens, int32_t max_cache_len,
                           const float* c_q, const float* c_out, const float* c_lse, void* out, float* a_lse,
                           uint8_t* flags, void* stream) {
  return decode_entry(p_in, q_t, k_c, v_c, cache_offsets, cache_lens, max_cache_len, c_q, c_out, c_lse, out, a_lse,
                      flags, nullptr, 0, true, stream);
}

size_t calidrop_recalibrate_workspace_bytes(const calidrop_params* p_in, int32_t max_seq_len) {
  calidrop_params pp; const calidrop_params* p = &pp;
  if (load_params(p_in, &pp) != CALIDROP_OK) return 0;
  if (check_params(p) != CALIDROP_OK) return 0;
  if (max_seq_len < 1) { fail(CALIDROP_ESHAPE, "max_seq_len must be >= 1"); return 0; }
  return recal_layout(p, max_seq_len).total;
}

int calidrop_recalibrate(const calidrop_params* p_in, const void* q_t, const void* k, const void* v,
                         const int32_t* seq_offsets, int64_t total_tokens, int32_t max_seq_len,
                         const int32_t* indices, const int32_t* cal_indices, uint8_t* flags, const float* a_lse,
                         void* out, float* c_q, float* c_out, float* c_lse, void* workspace, size_t workspace_bytes,
                         void* stream) {
  int rc;
  calidrop_params pp; const calidrop_params* p = &pp;
  if ((rc = load_params(p_in, &pp))) return rc;
  if ((rc = check_params(p))) return rc;
  if ((rc = check_sizes(p, total_tokens, max_seq_len))) return rc;
  const struct { const void* ptr; const char* name; } req[] = {
      {q_t, "q_t"}, {k, "k"}, {v, "v"}, {seq_offsets, "seq_offsets"}, {indices, "indices"}, {flags, "flags"},
      {a_lse, "a_lse"}, {out, "out"}, {c_q, "c_q"}, {c_out, "c_out"}, {c_lse, "c_lse"}};
  for (const auto& r : req)
    if (!r.ptr) return fail(CALIDROP_EINVAL, "%s is NULL", r.name);
  for (const auto& r : req)
    if (r.ptr != flags && !aligned16(r.ptr)) return fail(CALIDROP_EALIGN, "%s is not 16-byte aligned", r.name);
  if (p->calib_size > 0) {
    if (!cal_indices) return fail(CALIDROP_EINVAL, "cal_indices is NULL although calib_size is %d", p->calib_size);
    if (!aligned16(cal_indices)) return fail(CALIDROP_EALIGN, "cal_indices is not 16-byte aligned");
  } else {
    cal_indices = nullptr;
  }
  const RecalLayout L = recal_layout(p, max_seq_len);
  if (!workspace || workspace_bytes < L.total)
    return fail(CALIDROP_EWORKSPACE, "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : 0,
                L.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(CALIDROP_EALIGN, "workspace is not 256-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
#define CD_DISPATCH(T, D)                                                                                        \
  return recal_impl<T, D>(p, q_t, k, v, seq_offsets, total_tokens, max_seq_len, indices, cal_indices, flags, a_lse, \
                          out, c_q, c_out, c_lse, ws, L, st)
  if (p->dtype == CALIDROP_BF16) {
    if (p->head_dim == 128) CD_DISPATCH(cd::bf16_t, 128);
    CD_DISPATCH(cd::bf16_t, 64);
  }
  if (p->head_dim == 128) CD_DISPATCH(float, 128);
  CD_DISPATCH(float, 64);
#undef CD_DISPATCH
}

size_t calidrop_compress_given_workspace_bytes(const calidrop_params* p_in, int32_t max_seq_len) {
  return calidrop_recalibrate_workspace_bytes(p_in, max_seq_len);   // same regions: bitmap + split partials
}

int calidrop_streaming_indices(const calidrop_params* p_in, int32_t n_sink, const int32_t* seq_offsets,
                               int64_t total_tokens, int32_t max_seq_len, int32_t* indices, void* stream) {
  int rc;
  calidrop_params pp; const calidrop_params* p = &pp;
  if ((rc = load_params(p_in, &pp))) return rc;
  if ((rc = check_params(p))) return rc;
  if ((rc = check_sizes(p, total_tokens, max_seq_len))) return rc;
  if (n_sink < 0 || n_sink > p->budget)
    return fail(CALIDROP_EINVAL, "n_sink must lie in [0, budget] (got %d, budget %d)", n_sink, p->budget);
  if (!seq_offsets) return fail(CALIDROP_EINVAL, "seq_offsets is NULL");
  if (!indices) return fail(CALIDROP_EINVAL, "indices is NULL");
  if (!aligned16(seq_offsets) || !aligned16(indices))
    return fail(CALIDROP_EALIGN, "seq_offsets / indices is not 16-byte aligned");
  cd::StreamingArgs sa{};
  sa.seq_off = seq_offsets; sa.total_tokens = total_tokens; sa.batch = p->batch; sa.Hkv = p->n_kv_heads;
  sa.B = p->budget; sa.n_sink = n_sink; sa.max_seq_len = max_seq_len; sa.indices = indices;
  hipLaunchKernelGGL(cd::streaming_indices_kernel, dim3(ceil_div(p->budget, 256), p->batch * p->n_kv_heads), dim3(256),
                     0, static_cast<hipStream_t>(stream), sa);
  return launch_status("streaming_indices");
}

int calidrop_compress_given(const calidrop_params* p_in, const void* q_cal, const void* k, const void* v,
                            const int32_t* seq_offsets, int64_t total_tokens, int32_t max_seq_len, int32_t* indices,
                            void* k_c, void* v_c, const int32_t* cache_offsets, int32_t* cache_lens, float* c_q,
                            float* c_out, float* c_lse, void* workspace, size_t workspace_bytes, void* stream) {
  int rc;
  calidrop_params pp; const calidrop_params* p = &pp;
  if ((rc = load_params(p_in, &pp))) return rc;
  if ((rc = check_params(p))) return rc;
  if ((rc = check_sizes(p, total_tokens, max_seq_len))) return rc;
  const struct { const void* ptr; const char* name; } req[] = {
      {q_cal, "q_cal"}, {k, "k"}, {v, "v"}, {seq_offsets, "seq_offsets"}, {indices, "indices"}, {k_c, "k_c"},
      {v_c, "v_c"}, {cache_offsets, "cache_offsets"}, {cache_lens, "cache_lens"}, {c_q, "c_q"}, {c_out, "c_out"},
      {c_lse, "c_lse"}};
  for (const auto& r : req)
    if (!r.ptr) return fail(CALIDROP_EINVAL, "%s is NULL", r.name);
  for (const auto& r : req)
    if (!aligned16(r.ptr)) return fail(CALIDROP_EALIGN, "%s is not 16-byte aligned", r.name);
  if (p->calib_size != 0)
    return fail(CALIDROP_EUNSUPPORTED, "calib_size needs the scored strategy (got %d with a given retained set)",
                p->calib_size);
  const RecalLayout L = recal_layout(p, max_seq_len);
  if (!workspace || workspace_bytes < L.total)
    return fail(CALIDROP_EWORKSPACE, "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : 0,
                L.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(CALIDROP_EALIGN, "workspace is not 256-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
#define CD_DISPATCH(T, D)                                                                                         \
  return compress_given_impl<T, D>(p, q_cal, k, v, seq_offsets, total_tokens, max_seq_len, indices, k_c, v_c,     \
                                   cache_offsets, cache_lens, c_q, c_out, c_lse, ws, L, st)
  if (p->dtype == CALIDROP_BF16) {
    if (p->head_dim == 128) CD_DISPATCH(cd::bf16_t, 128);
    CD_DISPATCH(cd::bf16_t, 64);
  }
  if (p->head_dim == 128) CD_DISPATCH(float, 128);
  CD_DISPATCH(float, 64);
#undef CD_DISPATCH
}

size_t calidrop_pack_evicted_workspace_bytes(const calidrop_params* p_in, int32_t max_seq_len) {
  calidrop_params pp; const calidrop_params* p = &pp;
  if (load_params(p_in, &pp) != CALIDROP_OK) return 0;
  if (check_params(p) != CALIDROP_OK) return 0;
  if (max_seq_len < 1) { fail(CALIDROP_ESHAPE, "max_seq_len must be >= 1"); return 0; }
  return pack_layout(p, max_seq_len).total;
}

int32_t calidrop_packed_rows(const calidrop_params* p_in, int32_t seq_len) {
  calidrop_params pp;
  if (load_params(p_in, &pp) != CALIDROP_OK) return -1;
  if (check_params(&pp) != CALIDROP_OK) return -1;
  if (seq_len < 0) { fail(CALIDROP_ESHAPE, "seq_len must be >= 0"); return -1; }
  return packed_rows_host(&pp, seq_len);
}

int calidrop_pack_evicted(const calidrop_params* p_in, const void* k, const void* v, const int32_t* seq_offsets,
                          int64_t total_tokens, int32_t max_seq_len, const int32_t* indices,
                          const int32_t* cal_indices, void* k_e, void* v_e, const int32_t* evict_offsets,
                          int32_t* evict_lens, int32_t* evict_indices, void* workspace, size_t workspace_bytes,
                          void* stream) {
  int rc;
  calidrop_params pp; const calidrop_params* p = &pp;
  if ((rc = load_params(p_in, &pp))) return rc;
  if ((rc = check_params(p))) return rc;
  if ((rc = check_sizes(p, total_tokens, max_seq_len))) return rc;
  const struct { const void* ptr; const char* name; } req[] = {
      {k, "k"}, {v, "v"}, {seq_offsets, "seq_offsets"}, {indices, "indices"}, {k_e, "k_e"}, {v_e, "v_e"},
      {evict_offsets, "evict_offsets"}, {evict_lens, "evict_lens"}, {evict_indices, "evict_indices"}};
  for (const auto& r : req)
    if (!r.ptr) return fail(CALIDROP_EINVAL, "%s is NULL", r.name);
  for (const auto& r : req)
    if (!aligned16(r.ptr)) return fail(CALIDROP_EALIGN, "%s is not 16-byte aligned", r.name);
  if (p->calib_size > 0) {
    if (!cal_indices) return fail(CALIDROP_EINVAL, "cal_indices is NULL although calib_size is %d", p->calib_size);
    if (!aligned16(cal_indices)) return fail(CALIDROP_EALIGN, "cal_indices is not 16-byte aligned");
  } else {
    cal_indices = nullptr;
  }
  const PackLayout L = pack_layout(p, max_seq_len);
  if (!workspace || workspace_bytes < L.total)
    return fail(CALIDROP_EWORKSPACE, "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : 0,
                L.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(CALIDROP_EALIGN, "workspace is not 256-byte aligned");
  return pack_impl(p, k, v, seq_offsets, total_tokens, max_seq_len, indices, cal_indices, k_e, v_e, evict_offsets,
                   evict_lens, evict_indices, static_cast<char*>(workspace), L, static_cast<hipStream_t>(stream));
}

size_t calidrop_recalibrate_packed_workspace_bytes(const calidrop_params* p_in, int32_t max_evict_len) {
  return calidrop_decode_workspace_bytes(p_in, max_evict_len);      // the same split partials
}

int calidrop_recalibrate_packed(const calidrop_params* p_in, const void* q_t, const void* k_e, const void* v_e,
                                const int32_t* evict_offsets, const int32_t* evict_lens, int32_t max_evict_len,
                                uint8_t* flags, const float* a_lse, void* out, float* c_q, float* c_out, float* c_lse,
                                void* workspace, size_t workspace_bytes, void* stream) {
  int rc;
  calidrop_params pp; const calidrop_params* p = &pp;
  if ((rc = load_params(p_in, &pp))) return rc;
  if ((rc = check_params(p))) return rc;
  if (max_evict_len < 1) return fail(CALIDROP_ESHAPE, "max_evict_len must be >= 1 (got %d)", max_evict_len);
  const struct { const void* ptr; const char* name; } req[] = {
      {q_t, "q_t"}, {k_e, "k_e"}, {v_e, "v_e"}, {evict_offsets, "evict_offsets"}, {evict_lens, "evict_lens"},
      {flags, "flags"}, {a_lse, "a_lse"}, {out, "out"}, {c_q, "c_q"}, {c_out, "c_out"}, {c_lse, "c_lse"}};
  for (const auto& r : req)
    if (!r.ptr) return fail(CALIDROP_EINVAL, "%s is NULL", r.name);
  for (const auto& r : req)
    if (r.ptr != flags && !aligned16(r.ptr)) return fail(CALIDROP_EALIGN, "%s is not 16-byte aligned", r.name);
  const DecodeLayout L = decode_layout(p, max_evict_len);
  if (!workspace || workspace_bytes < L.total)
    return fail(CALIDROP_EWORKSPACE, "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : 0,
                L.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(CALIDROP_EALIGN, "workspace is not 256-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
#define CD_DISPATCH(T, D)                                                                                        \
  return recal_packed_impl<T, D>(p, q_t, k_e, v_e, evict_offsets, evict_lens, max_evict_len, flags, a_lse, out,   \
                                 c_q, c_out, c_lse, ws, L, st)
  if (p->dtype == CALIDROP_BF16) {
    if (p->head_dim == 128) CD_DISPATCH(cd::bf16_t, 128);
    CD_DISPATCH(cd::bf16_t, 64);
  }
  if (p->head_dim == 128) CD_DISPATCH(float, 128);
  CD_DISPATCH(float, 64);
#undef CD_DISPATCH
}

namespace {
int h2o_local(const calidrop_params* p, int32_t n_local) {
  if (n_local == 0) n_local = p->budget / 2;              // the even split of Sec. 4.1.3
  if (n_local < 1 || n_local >= p->budget) {
    fail(CALIDROP_EINVAL, "n_local must satisfy 1 <= n_local < budget (got %d, budget %d)", n_local, p->budget);
    return -1;
  }
  return n_local;
}
}  // namespace

size_t calidrop_compress_h2o_workspace_bytes(const calidrop_params* p_in, int32_t n_local, int64_t total_tokens,
                                             int32_t max_seq_len) {
  calidrop_params pp; const calidrop_params* p = &pp;
  if (load_params(p_in, &pp) != CALIDROP_OK) return 0;
  if (check_params(p) != CALIDROP_OK || check_sizes(p, total_tokens, max_seq_len) != CALIDROP_OK) return 0;
  if ((n_local = h2o_local(p, n_local)) < 0) return 0;
  return h2o_layout(p, total_tokens, max_seq_len, n_local).total;
}

int calidrop_compress_h2o_workspace_region(const calidrop_params* p_in, int32_t n_local, int64_t total_tokens,
                                           int32_t max_seq_len, int32_t region, size_t* offset, size_t* bytes) {
  int rc;
  calidrop_params pp; const calidrop_params* p = &pp;
  if ((rc = load_params(p_in, &pp))) return rc;
  if ((rc = check_params(p))) return rc;
  if ((rc = check_sizes(p, total_tokens, max_seq_len))) return rc;
  if ((n_local = h2o_local(p, n_local)) < 0) return CALIDROP_EINVAL;
  if (!offset || !bytes) return fail(CALIDROP_EINVAL, "offset/bytes is NULL");
  const H2oLayout L = h2o_layout(p, total_tokens, max_seq_len, n_local);
  if (region == CALIDROP_REGION_ROW_LSE) {
    *offset = L.row_lse;
    *bytes = static_cast<size_t>(p->batch) * p->n_q_heads * L.lse_stride * sizeof(float);
  } else if (region == CALIDROP_REGION_SCORE) {
    *offset = L.score;
    *bytes = static_cast<size_t>(total_tokens) * p->n_kv_heads * sizeof(float);
  } else if (region == CALIDROP_REGION_VOTE_PLANES) {
    *offset = L.vote;
    *bytes = static_cast<size_t>(vote_plane(total_tokens, p->n_kv_heads)) * (p->n_q_heads / p->n_kv_heads) * sizeof(float);
  } else {
    return fail(CALIDROP_EINVAL, "unknown workspace region %d", region);
  }
  return CALIDROP_OK;
}

int calidrop_compress_h2o(const calidrop_params* p_in, int32_t n_local, const void* q_full, const void* k,
                          const void* v, const int32_t* seq_offsets, int64_t total_tokens, int32_t max_seq_len,
                          void* k_c, void* v_c, const int32_t* cache_offsets, int32_t* cache_lens, int32_t* indices,
                          int32_t* cal_indices, float* c_q, float* c_out, float* c_lse, void* workspace,
                          size_t workspace_bytes, void* stream) {
  int rc;
  calidrop_params pp; const calidrop_params* p = &pp;
  if ((rc = load_params(p_in, &pp))) return rc;
  if ((rc = check_params(p))) return rc;
  if ((rc = check_sizes(p, total_tokens, max_seq_len))) return rc;
  if ((n_local = h2o_local(p, n_local)) < 0) return CALIDROP_EINVAL;
  if (static_cast<int64_t>(p->batch) * p->n_q_heads > 65535)
    return fail(CALIDROP_EUNSUPPORTED, "batch * n_q_heads exceeds 65535");
  const struct { const void* ptr; const char* name; } req[] = {
      {q_full, "q_full"}, {k, "k"}, {v, "v"}, {seq_offsets, "seq_offsets"}, {k_c, "k_c"}, {v_c, "v_c"},
      {cache_offsets, "cache_offsets"}, {cache_lens, "cache_lens"}, {indices, "indices"}, {c_q, "c_q"},
      {c_out, "c_out"}, {c_lse, "c_lse"}};
  for (const auto& r : req)
    if (!r.ptr) return fail(CALIDROP_EINVAL, "%s is NULL", r.name);
  for (const auto& r : req)
    if (!aligned16(r.ptr)) return fail(CALIDROP_EALIGN, "%s is not 16-byte aligned", r.name);
  if (p->calib_size > 0) {
    if (!cal_indices) return fail(CALIDROP_EINVAL, "cal_indices is NULL although calib_size is %d", p->calib_size);
    if (!aligned16(cal_indices)) return fail(CALIDROP_EALIGN, "cal_indices is not 16-byte aligned");
  } else {
    cal_indices = nullptr;
  }
  const H2oLayout L = h2o_layout(p, total_tokens, max_seq_len, n_local);
  if (!workspace || workspace_bytes < L.total)
    return fail(CALIDROP_EWORKSPACE, "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : 0,
                L.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(CALIDROP_EALIGN, "workspace is not 256-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
#define CD_DISPATCH(T, D)                                                                                      \
  return h2o_impl<T, D>(p, n_local, q_full, k, v, seq_offsets, total_tokens, max_seq_len, k_c, v_c,             \
                        cache_offsets, cache_lens, indices, cal_indices, c_q, c_out, c_lse, ws, L, st)
  if (p->dtype == CALIDROP_BF16) {
    if (p->head_dim == 128) CD_DISPATCH(cd::bf16_t, 128);
    CD_DISPATCH(cd::bf16_t, 64);
  }
  if (p->head_dim == 128) CD_DISPATCH(float, 128);
  CD_DISPATCH(float, 64);
#undef CD_DISPATCH
}

int calidrop_append(const calidrop_params* p_in, const void* k_new, const void* v_new, void* k_c, void* v_c,
                    const int32_t* cache_offsets, int32_t* cache_lens, void* stream) {
  int rc;
  calidrop_params pp; const calidrop_params* p = &pp;
  if ((rc = load_params(p_in, &pp))) return rc;
  if ((rc = check_params(p))) return rc;
  const struct { const void* ptr; const char* name; } req[] = {
      {k_new, "k_new"}, {v_new, "v_new"}, {k_c, "k_c"}, {v_c, "v_c"}, {cache_offsets, "cache_offsets"},
      {cache_lens, "cache_lens"}};
  for (const auto& r : req)
    if (!r.ptr) return fail(CALIDROP_EINVAL, "%s is NULL", r.name);
  for (const auto& r : req)
    if (!aligned16(r.ptr)) return fail(CALIDROP_EALIGN, "%s is not 16-byte aligned", r.name);
  cd::AppendArgs aa{};
  aa.k_new = k_new; aa.v_new = v_new; aa.k_c = k_c; aa.v_c = v_c; aa.cache_off = cache_offsets; aa.cache_lens = cache_lens;
  aa.batch = p->batch; aa.Hkv = p->n_kv_heads; aa.row_bytes = p->head_dim * (p->dtype == CALIDROP_BF16 ? 2 : 4);
  hipLaunchKernelGGL(cd::append_rows_kernel, dim3(p->batch), dim3(256), 0, static_cast<hipStream_t>(stream), aa);
  return launch_status("append_rows");
}

}  // extern "C"
