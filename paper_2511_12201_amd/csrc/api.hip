// C-ABI entry points: argument validation, workspace carving, dispatch.
// Everything here runs on the host; no entry point allocates device memory.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "common.h"
#include "kernels.h"
#include "sched.h"

namespace omni {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
void clear_error() { g_err[0] = 0; }

int validate_layer(const omni_layer_desc* d) {
  if (!d) OMNI_FAIL(OMNI_ERR_INVALID, "descriptor is null");
  if (d->batch < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_tokens < 1)
    OMNI_FAIL(OMNI_ERR_INVALID, "batch, head counts and n_tokens must be positive");
  if (d->n_q_heads % d->n_kv_heads) OMNI_FAIL(OMNI_ERR_INVALID, "n_q_heads must be a multiple of n_kv_heads");
  if (d->head_dim != 64 && d->head_dim != 128) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
  if (d->dtype != OMNI_F32 && d->dtype != OMNI_BF16) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "dtype must be OMNI_F32 or OMNI_BF16");
  if (!(d->vis_begin >= 0 && d->vis_begin < d->vis_end && d->vis_end <= d->n_tokens))
    OMNI_FAIL(OMNI_ERR_INVALID, "need 0 <= vis_begin < vis_end <= n_tokens");
  if (d->sink_index < 0 || d->sink_index >= d->n_tokens) OMNI_FAIL(OMNI_ERR_INVALID, "sink_index out of range");
  if (d->causal != 0 && d->causal != 1) OMNI_FAIL(OMNI_ERR_INVALID, "causal must be 0 or 1");
  if (!(d->softmax_scale > 0.f) || !std::isfinite(d->softmax_scale))
    OMNI_FAIL(OMNI_ERR_INVALID, "softmax_scale must be positive and finite");
  if ((long long)d->batch * d->n_q_heads * (long long)d->n_tokens >= (1ll << 31))
    OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "batch * n_q_heads * n_tokens must be below 2^31");
  const long long nat_q[3] = {(long long)d->n_q_heads * d->n_tokens * d->head_dim, (long long)d->n_tokens * d->head_dim,
                              d->head_dim};
  const long long nat_k[3] = {(long long)d->n_kv_heads * d->n_tokens * d->head_dim,
                              (long long)d->n_tokens * d->head_dim, d->head_dim};
  for (int k = 0; k < 3; ++k) {
    if (d->q_stride[k] % 8 || d->kv_stride[k] % 8) OMNI_FAIL(OMNI_ERR_INVALID, "strides must be multiples of 8 elements");
  }
  if (d->q_stride[2] < nat_q[2] || d->kv_stride[2] < nat_k[2]) OMNI_FAIL(OMNI_ERR_INVALID, "token stride below head_dim");
  if (d->q_stride[1] < nat_q[2] || d->kv_stride[1] < nat_k[2] || d->q_stride[0] < nat_q[2] || d->kv_stride[0] < nat_k[2])
    OMNI_FAIL(OMNI_ERR_INVALID, "head / batch stride below head_dim");
  (void)nat_q;
  (void)nat_k;
  return OMNI_OK;
}

int validate_decode(const omni_decode_desc* d) {
  if (!d) OMNI_FAIL(OMNI_ERR_INVALID, "descriptor is null");
  if (d->batch < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->cache_capacity < 1)
    OMNI_FAIL(OMNI_ERR_INVALID, "batch, head counts and cache_capacity must be positive");
  if (d->n_q_heads % d->n_kv_heads) OMNI_FAIL(OMNI_ERR_INVALID, "n_q_heads must be a multiple of n_kv_heads");
  if (d->head_dim != 64 && d->head_dim != 128) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
  if (d->dtype != OMNI_F32 && d->dtype != OMNI_BF16) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "dtype must be OMNI_F32 or OMNI_BF16");
  if (!(d->vis_begin >= 0 && d->vis_begin <= d->vis_end && d->vis_end <= d->cache_capacity))
    OMNI_FAIL(OMNI_ERR_INVALID, "need 0 <= vis_begin <= vis_end <= cache_capacity");
  if (!(d->softmax_scale > 0.f) || !std::isfinite(d->softmax_scale))
    OMNI_FAIL(OMNI_ERR_INVALID, "softmax_scale must be positive and finite");
  for (int k = 0; k < 3; ++k)
    if (d->kv_stride[k] % 8 || d->kv_stride[k] < d->head_dim)
      OMNI_FAIL(OMNI_ERR_INVALID, "cache strides must be multiples of 8 elements and at least head_dim");
  if (d->static_lists != 0 && d->static_lists != 1) OMNI_FAIL(OMNI_ERR_INVALID, "static_lists must be 0 or 1");
  return OMNI_OK;
}

int check_ws(const void* ws, size_t have, size_t need) {
  if (!ws) OMNI_FAIL(OMNI_ERR_INVALID, "workspace pointer is null");
  if (reinterpret_cast<uintptr_t>(ws) % 256) OMNI_FAIL(OMNI_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (have < need) OMNI_FAIL(OMNI_ERR_WORKSPACE, "workspace too small: have %zu bytes, need %zu", have, need);
  return OMNI_OK;
}

Layer make_layer(const omni_layer_desc* d) {
  Layer L;
  L.B = d->batch;
  L.Hq = d->n_q_heads;
  L.Hkv = d->n_kv_heads;
  L.G = L.Hq / L.Hkv;
  L.D = d->head_dim;
  L.N = d->n_tokens;
  L.ld = d->n_tokens;
  L.v0 = d->vis_begin;
  L.v1 = d->vis_end;
  L.sink = d->sink_index;
  L.causal = d->causal;
  L.bph = 0;
  L.scale = d->softmax_scale;
  for (int k = 0; k < 3; ++k) {
    L.qs[k] = d->q_stride[k];
    L.ks[k] = d->kv_stride[k];
  }
  return L;
}

// ---- kernel timing with HIP events (off by default)
constexpr int kProfSlots = 64;
struct ProfEntry {
  hipEvent_t start[kProfSlots], stop[kProfSlots];
  int created, used;
};
static ProfEntry g_prof[kProfCount];
static unsigned g_prof_mask = 0;     // bit k: kernel id k is timed

void prof_begin(int id, hipStream_t st) {
  if (!(g_prof_mask >> id & 1u)) return;
  ProfEntry& e = g_prof[id];
  if (e.used >= kProfSlots) return;
  if (e.used >= e.created) {
    if (hipEventCreate(&e.start[e.created]) != hipSuccess || hipEventCreate(&e.stop[e.created]) != hipSuccess) return;
    e.created++;
  }
  (void)hipEventRecord(e.start[e.used], st);
}
void prof_end(int id, hipStream_t st) {
  if (!(g_prof_mask >> id & 1u)) return;
  ProfEntry& e = g_prof[id];
  if (e.used >= e.created || e.used >= kProfSlots) return;
  (void)hipEventRecord(e.stop[e.used], st);
  e.used++;
}

static bool aligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

static size_t prefill_select_ws(const Layer& L, int dtype, int pb) {
  return align_up(score_queries_ws(L), 256) + align_up(probe_ws(L, dtype, pb), 256) +
         align_up(budget_stats_ws(L), 256) + select_ws(L);
}

static size_t kv_budget_ws(const Layer& L, int dtype, int pb) {
  return align_up(probe_ws(L, dtype, pb), 256) + budget_stats_ws(L);
}

}  // namespace omni

using namespace omni;

#define REQUIRE_PTR(p)                                                     \
  do {                                                                     \
    if (!(p)) OMNI_FAIL(OMNI_ERR_INVALID, "argument %s is null", #p);      \
  } while (0)
#define REQUIRE_PTR_EARLY(p) REQUIRE_PTR(p)
#define REQUIRE_ALIGNED(p)                                                            \
  do {                                                                                \
    if (!aligned16(p)) OMNI_FAIL(OMNI_ERR_INVALID, "argument %s must be 16-byte aligned", #p); \
  } while (0)
#define CHECK(expr)            \
  do {                         \
    int rc__ = (expr);         \
    if (rc__ != OMNI_OK) return rc__; \
  } while (0)

// ---- omni_slim_decode with static_lists: the merged group lists kept in the caller's workspace

namespace omni {
namespace {

// Where omni_slim_decode_prepare keeps the merged lists: behind the partial states of the decode call.
struct StaticLists {
  int* grp_idx;         // [B, Hkv, nv]
  unsigned* grp_mask;   // [B, Hkv, nv]
  int* grp_cnt;         // [B, Hkv]
  void* scratch;        // of the merge
  int nv;
  Layer L;              // the shapes the merge kernels take
};

size_t static_lists_bytes(const omni_decode_desc* d);

StaticLists carve_static_lists(const omni_decode_desc* d, void* ws) {
  StaticLists m;
  m.nv = d->vis_end - d->vis_begin;
  const size_t pairs = (size_t)d->batch * d->n_kv_heads;
  Arena a(static_cast<unsigned char*>(ws) + decode_ws(d));
  m.grp_idx = a.take<int>(pairs * m.nv);
  m.grp_mask = a.take<unsigned>(pairs * m.nv);
  m.grp_cnt = a.take<int>(pairs);
  m.L = Layer{};
  m.L.B = d->batch; m.L.Hq = d->n_q_heads; m.L.Hkv = d->n_kv_heads; m.L.G = m.L.Hq / m.L.Hkv; m.L.D = d->head_dim;
  m.L.N = d->cache_capacity; m.L.v0 = d->vis_begin; m.L.v1 = d->vis_end; m.L.bph = 1;
  m.scratch = a.take<unsigned char>(group_subset_ws(m.L));
  return m;
}

// Bytes behind the partial states: grp_idx, grp_mask [B, Hkv, nv], grp_cnt [B, Hkv], the merge's own scratch.
size_t static_lists_bytes(const omni_decode_desc* d) {
  if (!d->static_lists || d->n_q_heads / d->n_kv_heads > 32) return 0;
  const size_t nv = (size_t)(d->vis_end - d->vis_begin), pairs = (size_t)d->batch * d->n_kv_heads;
  Arena a(nullptr);
  a.take<int>(pairs * nv);
  a.take<unsigned>(pairs * nv);
  a.take<int>(pairs);
  Layer L{};
  L.B = d->batch; L.Hq = d->n_q_heads; L.Hkv = d->n_kv_heads; L.v0 = d->vis_begin; L.v1 = d->vis_end;
  a.take<unsigned char>(group_subset_ws(L));
  return a.used();
}

}  // namespace
}  // namespace omni

// ---- library-owned scratch for the entry point that takes no workspace (omni_slim_decode_grouped_static)

namespace omni {
namespace {

constexpr size_t kStaticScratchBytes = size_t(16) << 20;
constexpr int kMaxDevices = 64;

// One copy per GPU the library runs on, held until the process ends.  In host code the name below is only a
// stand-in for the symbol: the memory is reached through the address hipGetSymbolAddress returns on each device.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static void* g_scratch_ptr[kMaxDevices];          // per device, filled on the first call on that device
static std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch` (nullptr + error message on failure).  No allocation.
void* static_scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    set_error("static scratch: no current device (or device id >= %d)", kMaxDevices);
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      set_error("static scratch: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace
}  // namespace omni

extern "C" {

const char* omni_last_error(void) { return g_err; }

int omni_debug_work_list(const omni_layer_desc* desc, const int32_t* q_cnt, const int32_t* budget, int32_t b_cap,
                         int32_t tile_rows, int32_t queues, int32_t* item_head, int32_t* item_tile, int32_t* item_cost,
                         int32_t capacity, int32_t* n_items, int32_t* queue_end) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(item_head); REQUIRE_PTR(item_tile); REQUIRE_PTR(item_cost); REQUIRE_PTR(n_items);
  if (b_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap must be >= 1");
  if (tile_rows != 128 && tile_rows != 256) OMNI_FAIL(OMNI_ERR_INVALID, "tile_rows must be 128 or 256");
  if (queues != 1 && queues != kSchedQueues) OMNI_FAIL(OMNI_ERR_INVALID, "queues must be 1 or %d", kSchedQueues);
  const int BH = desc->batch * desc->n_q_heads;
  std::vector<int> sched(sched_ints(BH, desc->n_tokens, tile_rows));
  sched_build_host(q_cnt, budget, desc->batch, desc->n_q_heads, desc->n_tokens, b_cap, desc->causal, tile_rows,
                   sched.data(), queues);
  const int items = sched[kSchedTotal];
  *n_items = items;
  if (queue_end)
    for (int q = 0; q < kSchedQueues; ++q) queue_end[q] = sched[kSchedEnd + q];
  if (items > capacity) OMNI_FAIL(OMNI_ERR_WORKSPACE, "work list has %d items, capacity is %d", items, capacity);
  const size_t order_off = sched_order_off(BH, desc->n_tokens, tile_rows);
  for (int it = 0; it < items; ++it) {
    int bh, tq;
    sched_decode(sched.data(), order_off, it, bh, tq);
    item_head[it] = bh;
    item_tile[it] = tq;
    const int nt = sched[kSchedPrefix + bh + 1] - sched[kSchedPrefix + bh];
    int nk = budget ? budget[bh / desc->n_q_heads] : desc->n_tokens;
    nk = nk < 0 ? 0 : (nk > b_cap ? b_cap : nk);
    item_cost[it] = sched_estimate(tq, nt, nk, desc->causal);
  }
  return OMNI_OK;
}

int omni_debug_copy(const void* src, void* dst, size_t bytes, void* stream) {
  clear_error();
  REQUIRE_PTR(src); REQUIRE_PTR(dst);
  if (bytes == 0 || bytes % 16) OMNI_FAIL(OMNI_ERR_INVALID, "bytes must be a positive multiple of 16");
  return run_calibration_copy(src, dst, bytes, static_cast<hipStream_t>(stream));
}

int omni_debug_key_split_len(int tiles) {
  clear_error();
  set_key_split_len(tiles);
  return OMNI_OK;
}

int omni_debug_mfma_rate(int random_operands, int iters, double* tflops, double* shader_mhz) {
  clear_error();
  REQUIRE_PTR(tflops); REQUIRE_PTR(shader_mhz);
  if (iters < 1 || iters > (1 << 22)) OMNI_FAIL(OMNI_ERR_INVALID, "iters must be in [1, 2^22]");
  if (random_operands < 0 || random_operands > 2) OMNI_FAIL(OMNI_ERR_INVALID, "random_operands must be 0, 1 or 2");
  return run_mfma_rate(random_operands, iters, tflops, shader_mhz);
}

int omni_profile_enable(int mask) {
  clear_error();
  g_prof_mask = mask < 0 ? ~0u : (unsigned)mask;
  for (int i = 0; i < kProfCount; ++i) g_prof[i].used = 0;
  return OMNI_OK;
}

int omni_profile_read(int kernel_id, float* total_ms, int* launches) {
  clear_error();
  if (kernel_id < 0 || kernel_id >= kProfCount) OMNI_FAIL(OMNI_ERR_INVALID, "kernel_id out of range");
  REQUIRE_PTR_EARLY(total_ms);
  REQUIRE_PTR_EARLY(launches);
  ProfEntry& e = g_prof[kernel_id];
  float sum = 0.f;
  for (int i = 0; i < e.used; ++i) {
    OMNI_HIP_CHECK(hipEventSynchronize(e.stop[i]));
    float ms = 0.f;
    OMNI_HIP_CHECK(hipEventElapsedTime(&ms, e.start[i], e.stop[i]));
    sum += ms;
  }
  *total_ms = sum;
  *launches = e.used;
  return OMNI_OK;
}
int omni_version(void) { return 100; }

size_t omni_workspace_bytes(int call_id, const void* desc, int32_t param) {
  clear_error();
  if (!desc) return 0;
  if (call_id == OMNI_CALL_SLIM_DECODE || call_id == OMNI_CALL_DENSE_DECODE) {
    const omni_decode_desc* d = static_cast<const omni_decode_desc*>(desc);
    if (validate_decode(d) != OMNI_OK) return 0;
    return decode_ws(d) + (call_id == OMNI_CALL_SLIM_DECODE ? static_lists_bytes(d) : 0);
  }
  const omni_layer_desc* d = static_cast<const omni_layer_desc*>(desc);
  if (validate_layer(d) != OMNI_OK) return 0;
  const Layer L = make_layer(d);
  switch (call_id) {
    case OMNI_CALL_SCORE_QUERIES: return score_queries_ws(L);
    case OMNI_CALL_SELECT_QUERIES: return select_ws(L);
    case OMNI_CALL_SELECT_KV: return select_ws(L);
    case OMNI_CALL_KV_BUDGET:
      if (param < 1) { set_error("probe block must be >= 1"); return 0; }
      return kv_budget_ws(L, d->dtype, param);
    case OMNI_CALL_SPARSE_ATTN_FWD:
      if (param < 1) { set_error("b_cap must be >= 1"); return 0; }
      return attn_fwd_ws(L, d->dtype, param, true);
    case OMNI_CALL_SPARSE_ATTN_BWD:
      if (param < 1) { set_error("b_cap must be >= 1"); return 0; }
      return attn_bwd_ws(L, d->dtype, param);
    case OMNI_CALL_DENSE_ATTN_FWD: return attn_fwd_ws(L, d->dtype, L.N, false);
    case OMNI_CALL_GROUP_SUBSET: return group_subset_ws(L);
    case OMNI_CALL_PREFILL_SELECT:
      if (param < 1) { set_error("probe block must be >= 1"); return 0; }
      return prefill_select_ws(L, d->dtype, param);
    case OMNI_CALL_BLOCK_SCORES:
      if (param < 1) { set_error("block must be >= 1"); return 0; }
      return block_scores_ws(L, param);
    case OMNI_CALL_BLOCK_ATTN_FWD:
      if (param < 64 || param % 64) { set_error("blk_cap * block must be a positive multiple of 64"); return 0; }
      return attn_fwd_blocks_ws(L, param);
    case OMNI_CALL_BLOCK_ATTN_BWD:
      if (param < 64 || param % 64) { set_error("blk_cap * block must be a positive multiple of 64"); return 0; }
      return attn_bwd_blocks_ws(L, param);
    default: set_error("unknown call id %d", call_id); return 0;
  }
}

int omni_score_queries(const omni_layer_desc* desc, const void* Q, const void* K, float* probe_keys, float* scores,
                       void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(Q); REQUIRE_PTR(K); REQUIRE_PTR(probe_keys); REQUIRE_PTR(scores);
  REQUIRE_ALIGNED(Q); REQUIRE_ALIGNED(K);
  const Layer L = make_layer(desc);
  CHECK(check_ws(ws, ws_bytes, score_queries_ws(L)));
  return run_score_queries(L, desc->dtype, Q, K, probe_keys, scores, ws, static_cast<hipStream_t>(stream));
}

int omni_select_queries(const omni_layer_desc* desc, const float* scores, int mode, float param, int32_t* q_idx,
                        int32_t* q_cnt, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(scores); REQUIRE_PTR(q_idx); REQUIRE_PTR(q_cnt);
  if (mode != 0 && mode != 1) OMNI_FAIL(OMNI_ERR_INVALID, "mode must be 0 (threshold) or 1 (top fraction)");
  if (!std::isfinite(param)) OMNI_FAIL(OMNI_ERR_INVALID, "param must be finite");
  if (mode == 1 && !(param > 0.f && param <= 1.f)) OMNI_FAIL(OMNI_ERR_INVALID, "top fraction must be in (0, 1]");
  const Layer L = make_layer(desc);
  CHECK(check_ws(ws, ws_bytes, select_ws(L)));
  return run_select_queries(L, scores, mode, param, q_idx, q_cnt, ws, static_cast<hipStream_t>(stream));
}

int omni_kv_budget(const omni_layer_desc* desc, const void* Q, const void* K, float recall_p, int probe_block,
                   int budget_mode, float* key_scores, double* kurtosis, int32_t* flattest, int32_t* budget,
                   float* recall, int32_t* budget_host, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(Q); REQUIRE_PTR(K); REQUIRE_PTR(key_scores); REQUIRE_PTR(kurtosis); REQUIRE_PTR(flattest);
  REQUIRE_PTR(budget); REQUIRE_PTR(recall);
  REQUIRE_ALIGNED(Q); REQUIRE_ALIGNED(K);
  if (!(recall_p > 0.f && recall_p <= 1.f)) OMNI_FAIL(OMNI_ERR_INVALID, "recall_p must be in (0, 1]");
  if (probe_block < 1) OMNI_FAIL(OMNI_ERR_INVALID, "probe_block must be >= 1");
  if (budget_mode < 0 || budget_mode > 2) OMNI_FAIL(OMNI_ERR_INVALID, "budget_mode must be 0, 1 or 2");
  const Layer L = make_layer(desc);
  CHECK(check_ws(ws, ws_bytes, kv_budget_ws(L, desc->dtype, probe_block)));
  hipStream_t st = static_cast<hipStream_t>(stream);
  CHECK(run_probe(L, desc->dtype, Q, K, probe_block, key_scores, ws, st));
  void* ws2 = static_cast<char*>(ws) + align_up(probe_ws(L, desc->dtype, probe_block), 256);
  CHECK(run_budget_stats(L, key_scores, recall_p, budget_mode, kurtosis, flattest, budget, recall, ws2, st));
  if (budget_host)
    OMNI_HIP_CHECK(hipMemcpyAsync(budget_host, budget, sizeof(int32_t) * L.B * (budget_mode == 2 ? L.Hq : 1),
                                   hipMemcpyDeviceToHost, st));
  return OMNI_OK;
}

int omni_prefill_select(const omni_layer_desc* desc, const void* Q, const void* K, int q_mode, float q_param,
                        float recall_p, int probe_block, int budget_mode, float* probe_keys, float* scores,
                        int32_t* q_idx, int32_t* q_cnt, float* key_scores, double* kurtosis, int32_t* flattest,
                        int32_t* budget, float* recall, int32_t* kv_idx, int32_t b_cap, void* ws, size_t ws_bytes,
                        void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(Q); REQUIRE_PTR(K); REQUIRE_PTR(probe_keys); REQUIRE_PTR(scores); REQUIRE_PTR(q_idx); REQUIRE_PTR(q_cnt);
  REQUIRE_PTR(key_scores); REQUIRE_PTR(kurtosis); REQUIRE_PTR(flattest); REQUIRE_PTR(budget); REQUIRE_PTR(recall);
  REQUIRE_PTR(kv_idx);
  REQUIRE_ALIGNED(Q); REQUIRE_ALIGNED(K);
  if (q_mode != 0 && q_mode != 1) OMNI_FAIL(OMNI_ERR_INVALID, "mode must be 0 (threshold) or 1 (top fraction)");
  if (!std::isfinite(q_param)) OMNI_FAIL(OMNI_ERR_INVALID, "param must be finite");
  if (q_mode == 1 && !(q_param > 0.f && q_param <= 1.f)) OMNI_FAIL(OMNI_ERR_INVALID, "top fraction must be in (0, 1]");
  if (!(recall_p > 0.f && recall_p <= 1.f)) OMNI_FAIL(OMNI_ERR_INVALID, "recall_p must be in (0, 1]");
  if (probe_block < 1) OMNI_FAIL(OMNI_ERR_INVALID, "probe_block must be >= 1");
  if (budget_mode < 0 || budget_mode > 2) OMNI_FAIL(OMNI_ERR_INVALID, "budget_mode must be 0, 1 or 2");
  if (b_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap must be >= 1");
  Layer L = make_layer(desc);
  L.bph = budget_mode == 2;
  CHECK(check_ws(ws, ws_bytes, prefill_select_ws(L, desc->dtype, probe_block)));
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws_score = static_cast<char*>(ws);
  char* ws_probe = ws_score + align_up(score_queries_ws(L), 256);
  char* ws_stats = ws_probe + align_up(probe_ws(L, desc->dtype, probe_block), 256);
  char* ws_sel = ws_stats + align_up(budget_stats_ws(L), 256);
  CHECK(run_probe_keys(L, desc->dtype, K, probe_keys, ws_score, st));
  // one pass over Q: lazy/active scores and pooled queries; then the two probe passes over K
  CHECK(run_probe(L, desc->dtype, Q, K, probe_block, key_scores, ws_probe, st, probe_keys, scores));
  CHECK(run_select_queries(L, scores, q_mode, q_param, q_idx, q_cnt, ws_sel, st));
  // the recall pass already finds each head's cut for its budget: the key lists are compacted from it
  CHECK(run_budget_stats(L, key_scores, recall_p, budget_mode, kurtosis, flattest, budget, recall, ws_stats, st, b_cap));
  return run_select_kv_from_stats(L, key_scores, ws_stats, b_cap, kv_idx, ws_sel, st);
}

size_t omni_sparse_prefill_workspace_bytes(const omni_layer_desc* desc, int32_t probe_block, int32_t b_cap) {
  clear_error();
  if (validate_layer(desc) != OMNI_OK) return 0;
  if (probe_block < 1) { set_error("probe_block must be >= 1"); return 0; }
  if (b_cap < 1) { set_error("b_cap must be >= 1"); return 0; }
  const Layer L = make_layer(desc);
  return align_up(prefill_select_ws(L, desc->dtype, probe_block), 256) + attn_fwd_ws(L, desc->dtype, b_cap, true);
}

int omni_sparse_prefill(const omni_layer_desc* desc, const void* Q, const void* K, const void* V, int q_mode,
                        float q_param, float recall_p, int probe_block, int budget_mode, float* probe_keys,
                        float* scores, int32_t* q_idx, int32_t* q_cnt, float* key_scores, double* kurtosis,
                        int32_t* flattest, int32_t* budget, float* recall, int32_t* kv_idx, int32_t b_cap, void* O,
                        float* lse, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(Q); REQUIRE_PTR(K); REQUIRE_PTR(V); REQUIRE_PTR(probe_keys); REQUIRE_PTR(scores); REQUIRE_PTR(q_idx);
  REQUIRE_PTR(q_cnt); REQUIRE_PTR(key_scores); REQUIRE_PTR(kurtosis); REQUIRE_PTR(flattest); REQUIRE_PTR(budget);
  REQUIRE_PTR(recall); REQUIRE_PTR(kv_idx); REQUIRE_PTR(O); REQUIRE_PTR(lse);
  REQUIRE_ALIGNED(Q); REQUIRE_ALIGNED(K); REQUIRE_ALIGNED(V); REQUIRE_ALIGNED(O);
  if (q_mode != 0 && q_mode != 1) OMNI_FAIL(OMNI_ERR_INVALID, "mode must be 0 (threshold) or 1 (top fraction)");
  if (!std::isfinite(q_param)) OMNI_FAIL(OMNI_ERR_INVALID, "param must be finite");
  if (q_mode == 1 && !(q_param > 0.f && q_param <= 1.f)) OMNI_FAIL(OMNI_ERR_INVALID, "top fraction must be in (0, 1]");
  if (!(recall_p > 0.f && recall_p <= 1.f)) OMNI_FAIL(OMNI_ERR_INVALID, "recall_p must be in (0, 1]");
  if (probe_block < 1) OMNI_FAIL(OMNI_ERR_INVALID, "probe_block must be >= 1");
  if (budget_mode < 0 || budget_mode > 2) OMNI_FAIL(OMNI_ERR_INVALID, "budget_mode must be 0, 1 or 2");
  if (b_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap must be >= 1");
  Layer L = make_layer(desc);
  L.bph = budget_mode == 2;
  const size_t sel_bytes = align_up(prefill_select_ws(L, desc->dtype, probe_block), 256);
  CHECK(check_ws(ws, ws_bytes, sel_bytes + attn_fwd_ws(L, desc->dtype, b_cap, true)));
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws_score = static_cast<char*>(ws);
  char* ws_probe = ws_score + align_up(score_queries_ws(L), 256);
  char* ws_stats = ws_probe + align_up(probe_ws(L, desc->dtype, probe_block), 256);
  char* ws_sel = ws_stats + align_up(budget_stats_ws(L), 256);
  char* ws_fwd = static_cast<char*>(ws) + sel_bytes;
  CHECK(run_probe_keys(L, desc->dtype, K, probe_keys, ws_score, st));
  CHECK(run_probe(L, desc->dtype, Q, K, probe_block, key_scores, ws_probe, st, probe_keys, scores));
  CHECK(run_select_queries(L, scores, q_mode, q_param, q_idx, q_cnt, ws_sel, st));
  CHECK(run_budget_stats(L, key_scores, recall_p, budget_mode, kurtosis, flattest, budget, recall, ws_stats, st, b_cap));
  // the chunk counts of the key lists; the lists themselves come out of the attention's gather
  SelectSource src;
  CHECK(run_select_kv_counts(L, key_scores, ws_stats, b_cap, kv_idx, ws_sel, &src, st));
  return run_attn_fwd(L, desc->dtype, Q, K, V, q_idx, q_cnt, kv_idx, budget, b_cap, O, lse, ws_fwd, true, st, &src);
}

int omni_prefill_select_varlen(const omni_layer_desc* desc, const void* Q, const void* K, const int32_t* seq_tokens,
                               const int32_t* seq_vis_begin, const int32_t* seq_vis_end, int q_mode, float q_param,
                               float recall_p, int probe_block, int budget_mode, float* probe_keys, float* scores,
                               int32_t* q_idx, int32_t* q_cnt, float* key_scores, double* kurtosis, int32_t* flattest,
                               int32_t* budget, float* recall, int32_t* kv_idx, int32_t b_cap, void* ws,
                               size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(Q); REQUIRE_PTR(K); REQUIRE_PTR(seq_tokens); REQUIRE_PTR(seq_vis_begin); REQUIRE_PTR(seq_vis_end);
  REQUIRE_PTR(probe_keys); REQUIRE_PTR(scores); REQUIRE_PTR(q_idx); REQUIRE_PTR(q_cnt);
  REQUIRE_PTR(key_scores); REQUIRE_PTR(kurtosis); REQUIRE_PTR(flattest); REQUIRE_PTR(budget); REQUIRE_PTR(recall);
  REQUIRE_PTR(kv_idx);
  REQUIRE_ALIGNED(Q); REQUIRE_ALIGNED(K);
  if (q_mode != 0 && q_mode != 1) OMNI_FAIL(OMNI_ERR_INVALID, "mode must be 0 (threshold) or 1 (top fraction)");
  if (!std::isfinite(q_param)) OMNI_FAIL(OMNI_ERR_INVALID, "param must be finite");
  if (q_mode == 1 && !(q_param > 0.f && q_param <= 1.f)) OMNI_FAIL(OMNI_ERR_INVALID, "top fraction must be in (0, 1]");
  if (!(recall_p > 0.f && recall_p <= 1.f)) OMNI_FAIL(OMNI_ERR_INVALID, "recall_p must be in (0, 1]");
  if (probe_block < 1) OMNI_FAIL(OMNI_ERR_INVALID, "probe_block must be >= 1");
  if (budget_mode < 0 || budget_mode > 2) OMNI_FAIL(OMNI_ERR_INVALID, "budget_mode must be 0, 1 or 2");
  if (b_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap must be >= 1");
  for (int b = 0; b < desc->batch; ++b) {
    const int n = seq_tokens[b], v0 = seq_vis_begin[b], v1 = seq_vis_end[b];
    if (n < 1 || n > desc->n_tokens) OMNI_FAIL(OMNI_ERR_INVALID, "sequence %d: need 1 <= seq_tokens <= n_tokens", b);
    if (!(v0 >= 0 && v0 < v1 && v1 <= n)) OMNI_FAIL(OMNI_ERR_INVALID, "sequence %d: need 0 <= vis_begin < vis_end <= seq_tokens", b);
    if (desc->sink_index >= n) OMNI_FAIL(OMNI_ERR_INVALID, "sequence %d: sink_index beyond the sequence", b);
  }
  Layer Lmax = make_layer(desc);
  Lmax.B = 1;
  Lmax.bph = budget_mode == 2;
  CHECK(check_ws(ws, ws_bytes, prefill_select_ws(Lmax, desc->dtype, probe_block)));
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t es = desc->dtype == OMNI_BF16 ? 2 : 4;
  const long long Hq = desc->n_q_heads, Hkv = desc->n_kv_heads, Np = desc->n_tokens, D = desc->head_dim;
  for (int b = 0; b < desc->batch; ++b) {
    // the sequence as a layer of its own inside the padded tensors: its length and visual range, the batch's row
    // pitch; every kernel is sized to the sequence, and the result is bit for bit what the sequence gives alone
    Layer L = Lmax;
    L.N = seq_tokens[b];
    L.v0 = seq_vis_begin[b];
    L.v1 = seq_vis_end[b];
    const char* Qb = static_cast<const char*>(Q) + (size_t)b * desc->q_stride[0] * es;
    const char* Kb = static_cast<const char*>(K) + (size_t)b * desc->kv_stride[0] * es;
    float* probe_b = probe_keys + b * Hkv * 2 * D;
    float* scores_b = scores + b * Hq * Np;
    float* a_b = key_scores + b * Hq * Np;
    int32_t* budget_b = budget + (budget_mode == 2 ? b * Hq : b);
    char* ws_score = static_cast<char*>(ws);
    char* ws_probe = ws_score + align_up(score_queries_ws(L), 256);
    char* ws_stats = ws_probe + align_up(probe_ws(L, desc->dtype, probe_block), 256);
    char* ws_sel = ws_stats + align_up(budget_stats_ws(L), 256);
    CHECK(run_probe_keys(L, desc->dtype, Kb, probe_b, ws_score, st));
    CHECK(run_probe(L, desc->dtype, Qb, Kb, probe_block, a_b, ws_probe, st, probe_b, scores_b));
    CHECK(run_select_queries(L, scores_b, q_mode, q_param, q_idx + b * Hq * Np, q_cnt + b * Hq, ws_sel, st));
    CHECK(run_budget_stats(L, a_b, recall_p, budget_mode, kurtosis + b * Hq, flattest + b, budget_b, recall + b * Hq,
                           ws_stats, st, b_cap));
    CHECK(run_select_kv_from_stats(L, a_b, ws_stats, b_cap, kv_idx + b * Hq * b_cap, ws_sel, st));
  }
  return OMNI_OK;
}

int omni_budget_from_scores(const omni_layer_desc* desc, const float* key_scores, float recall_p, int budget_mode,
                            double* kurtosis, int32_t* flattest, int32_t* budget, float* recall, void* ws,
                            size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(key_scores); REQUIRE_PTR(kurtosis); REQUIRE_PTR(flattest); REQUIRE_PTR(budget); REQUIRE_PTR(recall);
  if (!(recall_p > 0.f && recall_p <= 1.f)) OMNI_FAIL(OMNI_ERR_INVALID, "recall_p must be in (0, 1]");
  if (budget_mode < 0 || budget_mode > 2) OMNI_FAIL(OMNI_ERR_INVALID, "budget_mode must be 0, 1 or 2");
  const Layer L = make_layer(desc);
  CHECK(check_ws(ws, ws_bytes, budget_stats_ws(L)));
  return run_budget_stats(L, key_scores, recall_p, budget_mode, kurtosis, flattest, budget, recall, ws,
                          static_cast<hipStream_t>(stream));
}

static int select_kv_impl(const omni_layer_desc* desc, int per_head, const float* key_scores, const int32_t* budget,
                          int32_t b_cap, int32_t* kv_idx, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(key_scores); REQUIRE_PTR(budget); REQUIRE_PTR(kv_idx);
  if (b_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap must be >= 1");
  Layer L = make_layer(desc);
  L.bph = per_head;
  CHECK(check_ws(ws, ws_bytes, select_ws(L)));
  return run_select_kv(L, key_scores, budget, b_cap, kv_idx, ws, static_cast<hipStream_t>(stream));
}

int omni_select_kv(const omni_layer_desc* desc, const float* key_scores, const int32_t* budget, int32_t b_cap,
                   int32_t* kv_idx, void* ws, size_t ws_bytes, void* stream) {
  return select_kv_impl(desc, 0, key_scores, budget, b_cap, kv_idx, ws, ws_bytes, stream);
}

int omni_select_kv_per_head(const omni_layer_desc* desc, const float* key_scores, const int32_t* budget,
                            int32_t b_cap, int32_t* kv_idx, void* ws, size_t ws_bytes, void* stream) {
  return select_kv_impl(desc, 1, key_scores, budget, b_cap, kv_idx, ws, ws_bytes, stream);
}

static int visual_subset_impl(const omni_layer_desc* desc, int per_head, const int32_t* kv_idx, const int32_t* budget,
                              int32_t b_cap, int32_t* vis_idx, int32_t* vis_cnt, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(kv_idx); REQUIRE_PTR(budget); REQUIRE_PTR(vis_idx); REQUIRE_PTR(vis_cnt);
  if (b_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap must be >= 1");
  Layer L = make_layer(desc);
  L.bph = per_head;
  return run_visual_subset(L, kv_idx, budget, b_cap, vis_idx, vis_cnt, static_cast<hipStream_t>(stream));
}

int omni_visual_subset(const omni_layer_desc* desc, const int32_t* kv_idx, const int32_t* budget, int32_t b_cap,
                       int32_t* vis_idx, int32_t* vis_cnt, void* stream) {
  return visual_subset_impl(desc, 0, kv_idx, budget, b_cap, vis_idx, vis_cnt, stream);
}

int omni_visual_subset_per_head(const omni_layer_desc* desc, const int32_t* kv_idx, const int32_t* budget,
                                int32_t b_cap, int32_t* vis_idx, int32_t* vis_cnt, void* stream) {
  return visual_subset_impl(desc, 1, kv_idx, budget, b_cap, vis_idx, vis_cnt, stream);
}

static int group_subset_impl(const omni_layer_desc* desc, int per_head, const int32_t* kv_idx, const int32_t* budget,
                             int32_t b_cap, int32_t* grp_idx, uint32_t* grp_mask, int32_t* grp_cnt, int32_t u_cap,
                             void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(kv_idx); REQUIRE_PTR(budget); REQUIRE_PTR(grp_idx); REQUIRE_PTR(grp_mask); REQUIRE_PTR(grp_cnt);
  if (b_cap < 1 || u_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap and u_cap must be >= 1");
  if (desc->n_q_heads / desc->n_kv_heads > 32) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "more than 32 query heads per KV head");
  Layer L = make_layer(desc);
  L.bph = per_head;
  CHECK(check_ws(ws, ws_bytes, group_subset_ws(L)));
  return run_group_subset(L, kv_idx, budget, b_cap, grp_idx, grp_mask, grp_cnt, u_cap, ws, static_cast<hipStream_t>(stream));
}

int omni_group_subset(const omni_layer_desc* desc, const int32_t* kv_idx, const int32_t* budget, int32_t b_cap,
                      int32_t* grp_idx, uint32_t* grp_mask, int32_t* grp_cnt, int32_t u_cap, void* ws, size_t ws_bytes,
                      void* stream) {
  return group_subset_impl(desc, 0, kv_idx, budget, b_cap, grp_idx, grp_mask, grp_cnt, u_cap, ws, ws_bytes, stream);
}

int omni_group_subset_per_head(const omni_layer_desc* desc, const int32_t* kv_idx, const int32_t* budget,
                               int32_t b_cap, int32_t* grp_idx, uint32_t* grp_mask, int32_t* grp_cnt, int32_t u_cap,
                               void* ws, size_t ws_bytes, void* stream) {
  return group_subset_impl(desc, 1, kv_idx, budget, b_cap, grp_idx, grp_mask, grp_cnt, u_cap, ws, ws_bytes, stream);
}

int omni_block_scores(const omni_layer_desc* desc, const void* Q, const void* K, int32_t block, float* block_scores,
                      void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(Q); REQUIRE_PTR(K); REQUIRE_PTR(block_scores);
  REQUIRE_ALIGNED(Q); REQUIRE_ALIGNED(K);
  if (block < 1) OMNI_FAIL(OMNI_ERR_INVALID, "block must be >= 1");
  const Layer L = make_layer(desc);
  if (cdiv(L.N, block) > block_scores_max_blocks())
    OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "more than %d key blocks", block_scores_max_blocks());
  CHECK(check_ws(ws, ws_bytes, block_scores_ws(L, block)));
  return run_block_scores(L, desc->dtype, Q, K, block, block_scores, ws, static_cast<hipStream_t>(stream));
}

int omni_expand_blocks(const omni_layer_desc* desc, const int32_t* blk_idx, const int32_t* blk_budget, int32_t blk_cap,
                       int32_t block, int32_t* kv_idx, int32_t* budget, int32_t b_cap, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(blk_idx); REQUIRE_PTR(blk_budget); REQUIRE_PTR(kv_idx); REQUIRE_PTR(budget);
  if (blk_cap < 1 || block < 1 || b_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "blk_cap, block and b_cap must be >= 1");
  if ((long long)blk_cap * block > b_cap) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap must be >= blk_cap * block");
  if (!desc->causal && desc->n_tokens % block)     // the pad entries of a partial last block are hidden by the causal mask only
    OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "without the causal mask n_tokens must be a multiple of block");
  return run_expand_blocks(make_layer(desc), blk_idx, blk_budget, blk_cap, block, kv_idx, budget, b_cap,
                           static_cast<hipStream_t>(stream));
}

static int sparse_attn_fwd_impl(const omni_layer_desc* desc, int per_head, const void* Q, const void* K, const void* V,
                                const int32_t* q_idx, const int32_t* q_cnt, const int32_t* kv_idx,
                                const int32_t* budget, int32_t b_cap, void* O, float* lse, void* ws, size_t ws_bytes,
                                void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(Q); REQUIRE_PTR(K); REQUIRE_PTR(V); REQUIRE_PTR(q_idx); REQUIRE_PTR(q_cnt); REQUIRE_PTR(kv_idx);
  REQUIRE_PTR(budget); REQUIRE_PTR(O); REQUIRE_PTR(lse);
  REQUIRE_ALIGNED(Q); REQUIRE_ALIGNED(K); REQUIRE_ALIGNED(V); REQUIRE_ALIGNED(O);
  if (b_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap must be >= 1");
  Layer L = make_layer(desc);
  L.bph = per_head;
  CHECK(check_ws(ws, ws_bytes, attn_fwd_ws(L, desc->dtype, b_cap, true)));
  return run_attn_fwd(L, desc->dtype, Q, K, V, q_idx, q_cnt, kv_idx, budget, b_cap, O, lse, ws, true,
                      static_cast<hipStream_t>(stream));
}

int omni_sparse_attn_fwd(const omni_layer_desc* desc, const void* Q, const void* K, const void* V,
                         const int32_t* q_idx, const int32_t* q_cnt, const int32_t* kv_idx, const int32_t* budget,
                         int32_t b_cap, void* O, float* lse, void* ws, size_t ws_bytes, void* stream) {
  return sparse_attn_fwd_impl(desc, 0, Q, K, V, q_idx, q_cnt, kv_idx, budget, b_cap, O, lse, ws, ws_bytes, stream);
}

int omni_sparse_attn_fwd_per_head(const omni_layer_desc* desc, const void* Q, const void* K, const void* V,
                                  const int32_t* q_idx, const int32_t* q_cnt, const int32_t* kv_idx,
                                  const int32_t* budget, int32_t b_cap, void* O, float* lse, void* ws, size_t ws_bytes,
                                  void* stream) {
  return sparse_attn_fwd_impl(desc, 1, Q, K, V, q_idx, q_cnt, kv_idx, budget, b_cap, O, lse, ws, ws_bytes, stream);
}

int omni_block_attn_fwd(const omni_layer_desc* desc, const void* Q, const void* K, const void* V, const int32_t* q_idx,
                        const int32_t* q_cnt, const int32_t* blk_idx, const int32_t* blk_budget, int32_t blk_cap,
                        int32_t block, void* O, float* lse, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(Q); REQUIRE_PTR(K); REQUIRE_PTR(V); REQUIRE_PTR(q_idx); REQUIRE_PTR(q_cnt); REQUIRE_PTR(blk_idx);
  REQUIRE_PTR(blk_budget); REQUIRE_PTR(O); REQUIRE_PTR(lse);
  REQUIRE_ALIGNED(Q); REQUIRE_ALIGNED(K); REQUIRE_ALIGNED(V); REQUIRE_ALIGNED(O);
  if (desc->dtype != OMNI_BF16) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "omni_block_attn_fwd runs in bf16 only");
  if (blk_cap < 1 || block < 1) OMNI_FAIL(OMNI_ERR_INVALID, "blk_cap and block must be >= 1");
  if (block % 64) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "block must be a multiple of 64 (the kernel's key tile)");
  if ((long long)blk_cap * block > attn_fwd_blocks_max_keys())
    OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "blk_cap * block above %d", attn_fwd_blocks_max_keys());
  if (!desc->causal && desc->n_tokens % block)
    OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "without the causal mask n_tokens must be a multiple of block");
  const Layer L = make_layer(desc);
  CHECK(check_ws(ws, ws_bytes, attn_fwd_blocks_ws(L, blk_cap * block)));
  return run_attn_fwd_blocks(L, Q, K, V, q_idx, q_cnt, blk_idx, blk_budget, blk_cap, block, O, lse, ws,
                             static_cast<hipStream_t>(stream));
}

int omni_block_attn_bwd(const omni_layer_desc* desc, const void* Q, const void* K, const void* V, const void* O,
                        const void* dO, const float* lse, const int32_t* q_idx, const int32_t* q_cnt,
                        const int32_t* blk_idx, const int32_t* blk_budget, int32_t blk_cap, int32_t block, void* dQ,
                        void* dK, void* dV, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(Q); REQUIRE_PTR(K); REQUIRE_PTR(V); REQUIRE_PTR(O); REQUIRE_PTR(dO); REQUIRE_PTR(lse);
  REQUIRE_PTR(q_idx); REQUIRE_PTR(q_cnt); REQUIRE_PTR(blk_idx); REQUIRE_PTR(blk_budget);
  REQUIRE_PTR(dQ); REQUIRE_PTR(dK); REQUIRE_PTR(dV);
  REQUIRE_ALIGNED(Q); REQUIRE_ALIGNED(K); REQUIRE_ALIGNED(V); REQUIRE_ALIGNED(O); REQUIRE_ALIGNED(dO);
  REQUIRE_ALIGNED(dQ); REQUIRE_ALIGNED(dK); REQUIRE_ALIGNED(dV);
  if (desc->dtype != OMNI_BF16) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "omni_block_attn_bwd runs in bf16 only");
  if (blk_cap < 1 || block < 1) OMNI_FAIL(OMNI_ERR_INVALID, "blk_cap and block must be >= 1");
  if (block % 64) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "block must be a multiple of 64 (the kernels' key tile)");
  if ((long long)blk_cap * block > attn_bwd_blocks_max_keys())
    OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "blk_cap * block above %d", attn_bwd_blocks_max_keys());
  if (!desc->causal && desc->n_tokens % block)
    OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "without the causal mask n_tokens must be a multiple of block");
  const Layer L = make_layer(desc);
  CHECK(check_ws(ws, ws_bytes, attn_bwd_blocks_ws(L, blk_cap * block)));
  return run_attn_bwd_blocks(L, Q, K, V, O, dO, lse, q_idx, q_cnt, blk_idx, blk_budget, blk_cap, block, dQ, dK, dV, ws,
                             static_cast<hipStream_t>(stream));
}

int omni_dense_attn_fwd(const omni_layer_desc* desc, const void* Q, const void* K, const void* V, void* O, float* lse,
                        void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(Q); REQUIRE_PTR(K); REQUIRE_PTR(V); REQUIRE_PTR(O); REQUIRE_PTR(lse);
  REQUIRE_ALIGNED(Q); REQUIRE_ALIGNED(K); REQUIRE_ALIGNED(V); REQUIRE_ALIGNED(O);
  const Layer L = make_layer(desc);
  CHECK(check_ws(ws, ws_bytes, attn_fwd_ws(L, desc->dtype, L.N, false)));
  return run_attn_fwd(L, desc->dtype, Q, K, V, nullptr, nullptr, nullptr, nullptr, L.N, O, lse, ws, false,
                      static_cast<hipStream_t>(stream));
}

static int sparse_attn_bwd_impl(const omni_layer_desc* desc, int per_head, const void* Q, const void* K, const void* V,
                                const void* O, const void* dO, const float* lse, const int32_t* q_idx,
                                const int32_t* q_cnt, const int32_t* kv_idx, const int32_t* budget, int32_t b_cap,
                                void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_layer(desc));
  REQUIRE_PTR(Q); REQUIRE_PTR(K); REQUIRE_PTR(V); REQUIRE_PTR(O); REQUIRE_PTR(dO); REQUIRE_PTR(lse);
  REQUIRE_PTR(q_idx); REQUIRE_PTR(q_cnt); REQUIRE_PTR(kv_idx); REQUIRE_PTR(budget);
  REQUIRE_PTR(dQ); REQUIRE_PTR(dK); REQUIRE_PTR(dV);
  REQUIRE_ALIGNED(Q); REQUIRE_ALIGNED(K); REQUIRE_ALIGNED(V); REQUIRE_ALIGNED(O); REQUIRE_ALIGNED(dO);
  REQUIRE_ALIGNED(dQ); REQUIRE_ALIGNED(dK); REQUIRE_ALIGNED(dV);
  if (b_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap must be >= 1");
  Layer L = make_layer(desc);
  L.bph = per_head;
  CHECK(check_ws(ws, ws_bytes, attn_bwd_ws(L, desc->dtype, b_cap)));
  return run_attn_bwd(L, desc->dtype, Q, K, V, O, dO, lse, q_idx, q_cnt, kv_idx, budget, b_cap, dQ, dK, dV, ws,
                      static_cast<hipStream_t>(stream));
}

int omni_sparse_attn_bwd(const omni_layer_desc* desc, const void* Q, const void* K, const void* V, const void* O,
                         const void* dO, const float* lse, const int32_t* q_idx, const int32_t* q_cnt,
                         const int32_t* kv_idx, const int32_t* budget, int32_t b_cap, void* dQ, void* dK, void* dV,
                         void* ws, size_t ws_bytes, void* stream) {
  return sparse_attn_bwd_impl(desc, 0, Q, K, V, O, dO, lse, q_idx, q_cnt, kv_idx, budget, b_cap, dQ, dK, dV, ws,
                              ws_bytes, stream);
}

int omni_sparse_attn_bwd_per_head(const omni_layer_desc* desc, const void* Q, const void* K, const void* V,
                                  const void* O, const void* dO, const float* lse, const int32_t* q_idx,
                                  const int32_t* q_cnt, const int32_t* kv_idx, const int32_t* budget, int32_t b_cap,
                                  void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes, void* stream) {
  return sparse_attn_bwd_impl(desc, 1, Q, K, V, O, dO, lse, q_idx, q_cnt, kv_idx, budget, b_cap, dQ, dK, dV, ws,
                              ws_bytes, stream);
}

int omni_slim_decode(const omni_decode_desc* desc, const void* q, const void* Kcache, const void* Vcache,
                     const int32_t* ctx_len, const float* probe_keys, const int32_t* vis_idx, const int32_t* vis_cnt,
                     int32_t b_cap, void* O, uint8_t* active, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_decode(desc));
  REQUIRE_PTR(q); REQUIRE_PTR(Kcache); REQUIRE_PTR(Vcache); REQUIRE_PTR(ctx_len); REQUIRE_PTR(probe_keys);
  REQUIRE_PTR(vis_idx); REQUIRE_PTR(vis_cnt); REQUIRE_PTR(O); REQUIRE_PTR(active);
  REQUIRE_ALIGNED(q); REQUIRE_ALIGNED(Kcache); REQUIRE_ALIGNED(Vcache);
  if (b_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap must be >= 1");
  if (!std::isfinite(desc->tau)) OMNI_FAIL(OMNI_ERR_INVALID, "tau must be finite");
  const size_t lists_bytes = static_lists_bytes(desc);
  CHECK(check_ws(ws, ws_bytes, decode_ws(desc) + lists_bytes));
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (lists_bytes) {
    // the lists as omni_slim_decode_prepare left them in the workspace, merged per KV group
    StaticLists m = carve_static_lists(desc, ws);
    return run_decode(desc, q, Kcache, Vcache, ctx_len, probe_keys, m.grp_idx, m.grp_cnt, m.grp_mask, m.nv, O, active, ws, st);
  }
  return run_decode(desc, q, Kcache, Vcache, ctx_len, probe_keys, vis_idx, vis_cnt, nullptr, b_cap, O, active, ws, st);
}

int omni_slim_decode_prepare(const omni_decode_desc* desc, const int32_t* vis_idx, const int32_t* vis_cnt, int32_t b_cap,
                             void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_decode(desc));
  REQUIRE_PTR(vis_idx); REQUIRE_PTR(vis_cnt);
  if (b_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "b_cap must be >= 1");
  if (!desc->static_lists) OMNI_FAIL(OMNI_ERR_INVALID, "omni_slim_decode_prepare is for descriptors with static_lists = 1");
  const size_t lists_bytes = static_lists_bytes(desc);
  CHECK(check_ws(ws, ws_bytes, decode_ws(desc) + lists_bytes));
  if (!lists_bytes) return OMNI_OK;      // groups wider than the membership word: the decode call reads the per-head lists
  StaticLists m = carve_static_lists(desc, ws);
  return run_group_subset(m.L, vis_idx, vis_cnt, b_cap, m.grp_idx, m.grp_mask, m.grp_cnt, m.nv, m.scratch,
                          static_cast<hipStream_t>(stream));
}

int omni_slim_decode_grouped(const omni_decode_desc* desc, const void* q, const void* Kcache, const void* Vcache,
                             const int32_t* ctx_len, const float* probe_keys, const int32_t* grp_idx,
                             const uint32_t* grp_mask, const int32_t* grp_cnt, int32_t u_cap, void* O, uint8_t* active,
                             void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_decode(desc));
  REQUIRE_PTR(q); REQUIRE_PTR(Kcache); REQUIRE_PTR(Vcache); REQUIRE_PTR(ctx_len); REQUIRE_PTR(probe_keys);
  REQUIRE_PTR(grp_idx); REQUIRE_PTR(grp_mask); REQUIRE_PTR(grp_cnt); REQUIRE_PTR(O); REQUIRE_PTR(active);
  REQUIRE_ALIGNED(q); REQUIRE_ALIGNED(Kcache); REQUIRE_ALIGNED(Vcache);
  if (u_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "u_cap must be >= 1");
  if (desc->n_q_heads / desc->n_kv_heads > 32) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "more than 32 query heads per KV head");
  if (!std::isfinite(desc->tau)) OMNI_FAIL(OMNI_ERR_INVALID, "tau must be finite");
  CHECK(check_ws(ws, ws_bytes, decode_ws(desc)));
  return run_decode(desc, q, Kcache, Vcache, ctx_len, probe_keys, grp_idx, grp_cnt, grp_mask, u_cap, O, active, ws,
                    static_cast<hipStream_t>(stream));
}

size_t omni_static_scratch_bytes(void) { return kStaticScratchBytes; }

int omni_slim_decode_grouped_static(const omni_decode_desc* desc, const void* q, const void* Kcache,
                                    const void* Vcache, const int32_t* ctx_len, const float* probe_keys,
                                    const int32_t* grp_idx, const uint32_t* grp_mask, const int32_t* grp_cnt,
                                    int32_t u_cap, void* O, uint8_t* active, void* stream) {
  clear_error();
  CHECK(validate_decode(desc));
  REQUIRE_PTR(q); REQUIRE_PTR(Kcache); REQUIRE_PTR(Vcache); REQUIRE_PTR(ctx_len); REQUIRE_PTR(probe_keys);
  REQUIRE_PTR(grp_idx); REQUIRE_PTR(grp_mask); REQUIRE_PTR(grp_cnt); REQUIRE_PTR(O); REQUIRE_PTR(active);
  REQUIRE_ALIGNED(q); REQUIRE_ALIGNED(Kcache); REQUIRE_ALIGNED(Vcache);
  if (u_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "u_cap must be >= 1");
  if (desc->n_q_heads / desc->n_kv_heads > 32) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "more than 32 query heads per KV head");
  if (!std::isfinite(desc->tau)) OMNI_FAIL(OMNI_ERR_INVALID, "tau must be finite");
  const size_t need = decode_ws(desc);
  if (need > kStaticScratchBytes)
    OMNI_FAIL(OMNI_ERR_WORKSPACE, "this shape needs %zu bytes of scratch, the built-in buffer holds %zu: use "
              "omni_slim_decode_grouped with a workspace", need, kStaticScratchBytes);
  void* ws = static_scratch_of_current_device();
  if (!ws) return OMNI_ERR_HIP;
  // the kernels write every partial state they later read, so nothing of the previous call's contents is cleared
  return run_decode(desc, q, Kcache, Vcache, ctx_len, probe_keys, grp_idx, grp_cnt, grp_mask, u_cap, O, active, ws,
                    static_cast<hipStream_t>(stream));
}

int omni_compact_cache(const omni_decode_desc* desc, const void* Kcache, const void* Vcache, const int32_t* grp_idx,
                       const int32_t* grp_cnt, int32_t u_cap, void* Kcomp, void* Vcomp, void* stream) {
  clear_error();
  CHECK(validate_decode(desc));
  REQUIRE_PTR(Kcache); REQUIRE_PTR(Vcache); REQUIRE_PTR(grp_idx); REQUIRE_PTR(grp_cnt); REQUIRE_PTR(Kcomp);
  REQUIRE_PTR(Vcomp);
  REQUIRE_ALIGNED(Kcache); REQUIRE_ALIGNED(Vcache); REQUIRE_ALIGNED(Kcomp); REQUIRE_ALIGNED(Vcomp);
  if (u_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "u_cap must be >= 1");
  return run_compact_cache(desc, Kcache, Vcache, grp_idx, grp_cnt, u_cap, Kcomp, Vcomp,
                           static_cast<hipStream_t>(stream));
}

int omni_slim_decode_compact(const omni_decode_desc* desc, const void* q, const void* Kcache, const void* Vcache,
                             const int32_t* ctx_len, const float* probe_keys, const void* Kcomp, const void* Vcomp,
                             const int32_t* grp_idx, const uint32_t* grp_mask, const int32_t* grp_cnt, int32_t u_cap,
                             void* O, uint8_t* active, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_decode(desc));
  REQUIRE_PTR(q); REQUIRE_PTR(Kcache); REQUIRE_PTR(Vcache); REQUIRE_PTR(ctx_len); REQUIRE_PTR(probe_keys);
  REQUIRE_PTR(Kcomp); REQUIRE_PTR(Vcomp);
  REQUIRE_PTR(grp_idx); REQUIRE_PTR(grp_mask); REQUIRE_PTR(grp_cnt); REQUIRE_PTR(O); REQUIRE_PTR(active);
  REQUIRE_ALIGNED(q); REQUIRE_ALIGNED(Kcache); REQUIRE_ALIGNED(Vcache); REQUIRE_ALIGNED(Kcomp); REQUIRE_ALIGNED(Vcomp);
  if (u_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "u_cap must be >= 1");
  if (desc->n_q_heads / desc->n_kv_heads > 32) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "more than 32 query heads per KV head");
  if (!std::isfinite(desc->tau)) OMNI_FAIL(OMNI_ERR_INVALID, "tau must be finite");
  CHECK(check_ws(ws, ws_bytes, decode_ws(desc)));
  return run_decode(desc, q, Kcache, Vcache, ctx_len, probe_keys, grp_idx, grp_cnt, grp_mask, u_cap, O, active, ws,
                    static_cast<hipStream_t>(stream), Kcomp, Vcomp);
}

static int validate_pool(const omni_page_pool* pool, int32_t u_cap, PagePool* out) {
  if (!pool) OMNI_FAIL(OMNI_ERR_INVALID, "pool is null");
  if (!pool->K || !pool->V || !pool->page_table) OMNI_FAIL(OMNI_ERR_INVALID, "pool: K, V or page_table is null");
  if ((reinterpret_cast<uintptr_t>(pool->K) | reinterpret_cast<uintptr_t>(pool->V)) & 15)
    OMNI_FAIL(OMNI_ERR_INVALID, "pool: K and V must be 16-byte aligned");
  if (pool->n_pages < 1 || pool->page_rows < 1 || pool->pages_cap < 1)
    OMNI_FAIL(OMNI_ERR_INVALID, "pool: n_pages, page_rows and pages_cap must be >= 1");
  if (pool->page_rows & (pool->page_rows - 1)) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "pool: page_rows must be a power of two");
  if ((long long)pool->n_pages * pool->page_rows >= (1ll << 31)) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "pool: 2^31 rows or more");
  if ((long long)pool->pages_cap * pool->page_rows < u_cap)
    OMNI_FAIL(OMNI_ERR_INVALID, "pool: pages_cap * page_rows must be >= u_cap");
  out->page_table = pool->page_table;
  out->page_shift = __builtin_ctz((unsigned)pool->page_rows);
  out->pages_cap = pool->pages_cap;
  out->pool_pages = pool->n_pages;
  return OMNI_OK;
}

int omni_compact_cache_paged(const omni_decode_desc* desc, const void* Kcache, const void* Vcache,
                             const int32_t* grp_idx, const int32_t* grp_cnt, int32_t u_cap, const omni_page_pool* pool,
                             void* stream) {
  clear_error();
  CHECK(validate_decode(desc));
  REQUIRE_PTR(Kcache); REQUIRE_PTR(Vcache); REQUIRE_PTR(grp_idx); REQUIRE_PTR(grp_cnt);
  REQUIRE_ALIGNED(Kcache); REQUIRE_ALIGNED(Vcache);
  if (u_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "u_cap must be >= 1");
  PagePool pp;
  CHECK(validate_pool(pool, u_cap, &pp));
  return run_compact_cache(desc, Kcache, Vcache, grp_idx, grp_cnt, u_cap, pool->K, pool->V,
                           static_cast<hipStream_t>(stream), &pp);
}

int omni_slim_decode_paged(const omni_decode_desc* desc, const void* q, const void* Kcache, const void* Vcache,
                           const int32_t* ctx_len, const float* probe_keys, const omni_page_pool* pool,
                           const int32_t* grp_idx, const uint32_t* grp_mask, const int32_t* grp_cnt, int32_t u_cap,
                           void* O, uint8_t* active, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_decode(desc));
  REQUIRE_PTR(q); REQUIRE_PTR(Kcache); REQUIRE_PTR(Vcache); REQUIRE_PTR(ctx_len); REQUIRE_PTR(probe_keys);
  REQUIRE_PTR(grp_idx); REQUIRE_PTR(grp_mask); REQUIRE_PTR(grp_cnt); REQUIRE_PTR(O); REQUIRE_PTR(active);
  REQUIRE_ALIGNED(q); REQUIRE_ALIGNED(Kcache); REQUIRE_ALIGNED(Vcache);
  if (u_cap < 1) OMNI_FAIL(OMNI_ERR_INVALID, "u_cap must be >= 1");
  if (desc->n_q_heads / desc->n_kv_heads > 32) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "more than 32 query heads per KV head");
  if (!std::isfinite(desc->tau)) OMNI_FAIL(OMNI_ERR_INVALID, "tau must be finite");
  PagePool pp;
  CHECK(validate_pool(pool, u_cap, &pp));
  CHECK(check_ws(ws, ws_bytes, decode_ws(desc)));
  return run_decode(desc, q, Kcache, Vcache, ctx_len, probe_keys, grp_idx, grp_cnt, grp_mask, u_cap, O, active, ws,
                    static_cast<hipStream_t>(stream), pool->K, pool->V, &pp);
}

int omni_dense_decode(const omni_decode_desc* desc, const void* q, const void* Kcache, const void* Vcache,
                      const int32_t* ctx_len, void* O, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  CHECK(validate_decode(desc));
  REQUIRE_PTR(q); REQUIRE_PTR(Kcache); REQUIRE_PTR(Vcache); REQUIRE_PTR(ctx_len); REQUIRE_PTR(O);
  REQUIRE_ALIGNED(q); REQUIRE_ALIGNED(Kcache); REQUIRE_ALIGNED(Vcache);
  CHECK(check_ws(ws, ws_bytes, decode_ws(desc)));
  return run_decode(desc, q, Kcache, Vcache, ctx_len, nullptr, nullptr, nullptr, nullptr, 1, O, nullptr, ws,
                    static_cast<hipStream_t>(stream));
}

}  // extern "C"
