// C ABI of the RoCo library: argument validation, workspace layout and kernel launches.
// Nothing here allocates, frees or synchronises.
#include <math.h>
#include <stdlib.h>

#include <mutex>

#include "../../include/roco.h"
#include "kernels.hpp"
#include "profile.hpp"

// Scratch of roco_decode_step_static: device memory that belongs to the library's code object, so the call needs no
// allocation and no workspace from the caller.  Every GPU the library runs on holds its own copy, at its own
// address, until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; kernels get the
// address that call returns.
static __device__ __align__(256) unsigned char scratch[ROCO_STATIC_SCRATCH_BYTES];

namespace {

using namespace roco;

constexpr size_t kAlign = 256;
constexpr int kStreamingAboveMiB = 192;
constexpr int kMaxPrefillGroup = 64;  // query heads per key/value head in the grouped-query prefill
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_params(const roco_params* p) {
  if (p == nullptr) return ROCO_EINVAL;
  if (p->units < 1 || p->budget < 1 || p->scope < 1 || p->scope > p->budget) return ROCO_EINVAL;
  if (p->recency_window < 0) return ROCO_EINVAL;
  if (p->importance < 0 || p->importance > 4 || p->scope_kind < 0 || p->scope_kind > 2 || p->sinks < 0) return ROCO_EINVAL;
  if ((p->importance == ROCO_IMPORTANCE_LAST || p->importance == ROCO_IMPORTANCE_COUNT) &&
      p->scope_kind == ROCO_SCOPE_STD)
    return ROCO_EINVAL;  // these scores live where the squares would be: no variance to rank by
  if (!(p->scale == p->scale) || !(p->recency_bias == p->recency_bias)) return ROCO_EINVAL;  // NaN
  if (p->dtype != ROCO_F32 && p->dtype != ROCO_BF16) return ROCO_EUNSUPPORTED;
  if (p->head_dim != 64 && p->head_dim != 128) return ROCO_EUNSUPPORTED;
  if (p->budget > (1 << 24)) return ROCO_EUNSUPPORTED;  // Count is kept exactly in fp32
  if (p->units > 65535) return ROCO_EUNSUPPORTED;       // several kernels index units with the grid's y dimension
  return ROCO_OK;
}

Policy policy_of(const roco_params* p) { return Policy{p->importance, p->scope_kind, p->sinks}; }

float scale_log2(const roco_params* p) {
  const float s = p->scale > 0.0f ? p->scale : 1.0f / sqrtf(static_cast<float>(p->head_dim));
  return s * 1.4426950408889634f;
}

// ---- decode workspace: z | part_m | part_l | part_o | keys
struct DecodeLayout { size_t z, part_m, part_l, part_o, keys, total; };
DecodeLayout decode_layout(const roco_params* p) {
  DecodeLayout l;
  const size_t U = p->units, B = p->budget, D = p->head_dim;
  size_t off = 0;
  l.z = off;      off += align_up(U * B * sizeof(float));
  l.part_m = off; off += align_up(U * kMaxSplits * sizeof(float));
  l.part_l = off; off += align_up(U * kMaxSplits * sizeof(float));
  l.part_o = off; off += align_up(U * kMaxSplits * D * sizeof(float));
  l.keys = off;   off += (p->budget > kMaxDecodeBudgetLds) ? align_up(U * 2 * B * sizeof(uint32_t)) : 0;
  l.total = off;
  return l;
}

// ---- prefill workspace: acc | acc2 | var_key | mas_key, each [units][L_max], then lse [units][group][L_max]
struct PrefillLayout { size_t lse, acc, acc2, var_key, mas_key, total; };
PrefillLayout prefill_layout(const roco_params* p, int32_t L_max, int32_t group) {
  PrefillLayout l;
  const size_t plane = align_up(static_cast<size_t>(p->units) * L_max * sizeof(float));
  l.acc = 0; l.acc2 = plane; l.var_key = 2 * plane; l.mas_key = 3 * plane; l.lse = 4 * plane;
  l.total = 4 * plane + align_up(static_cast<size_t>(p->units) * group * L_max * sizeof(float));
  return l;
}

// ---- block-wise workspace: blk_idx | z | part_m | part_l | part_o | keys
struct BlockLayout { size_t blk_idx, z, part_m, part_l, part_o, keys, total; };
BlockLayout block_layout(const roco_params* p) {
  BlockLayout l;
  const size_t U = p->units, B = p->budget, D = p->head_dim;
  size_t off = 0;
  l.blk_idx = off; off += align_up(U * B * sizeof(int32_t));
  l.z = off;       off += align_up(U * kMaxBlock * B * sizeof(float));
  l.part_m = off;  off += align_up(U * kMaxBlockSplits * kMaxBlock * sizeof(float));
  l.part_l = off;  off += align_up(U * kMaxBlockSplits * kMaxBlock * sizeof(float));
  l.part_o = off;  off += align_up(U * kMaxBlockSplits * kMaxBlock * D * sizeof(float));
  l.keys = off;    off += (p->budget > kMaxDecodeBudgetLds) ? align_up(U * 2 * B * sizeof(uint32_t)) : 0;
  l.total = off;
  return l;
}

int check_block(const roco_params* p, int32_t block) {
  const int rc = check_params(p);
  if (rc != ROCO_OK) return rc;
  if (block < 1 || block > p->budget) return ROCO_EINVAL;
  if (block > kMaxBlock || (p->budget & 3) != 0) return ROCO_EUNSUPPORTED;
  return ROCO_OK;
}

int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  return (v && *v) ? atoi(v) : dflt;
}

// Split the budget so that a step with few units still launches a workgroup for every other compute unit.
void choose_splits(const roco_params* p, int unroll, int& splits, int& rows_per_split) {
  const int gran = decode_rows_per_pass(p->dtype, p->head_dim, unroll);
  const int max_splits_by_rows = (p->budget + gran - 1) / gran;
  int want = env_int("ROCO_DECODE_SPLITS", 0);
  if (want <= 0) {
    // Measured (bf16, d = 128, 8 to 63 units, budgets 1024 to 16384): about one workgroup per two compute units is
    // enough for the attention kernel, and every further split costs the finishing kernel a partial to merge.
    const int target_wgs = 128;
    want = (target_wgs + p->units - 1) / p->units;
  }
  if (want > kMaxSplits) want = kMaxSplits;
  if (want > max_splits_by_rows) want = max_splits_by_rows;
  if (want < 1) want = 1;
  int rows = (p->budget + want - 1) / want;
  rows = (rows + gran - 1) / gran * gran;
  splits = (p->budget + rows - 1) / rows;
  rows_per_split = rows;
}

// Whether the K / V rows are read with the non-temporal hint.  Measured (B = 2048, bf16, d = 128): a cache of up to
// about 160 MiB is partly found again in the chip's last-level cache by the next step when loaded normally (31 vs 34
// us at 128 units); from 256 MiB on it only thrashes that cache and displaces the statistics (75 vs 69 us at 320
// units, 106 vs 92 us at 512).
bool streaming_loads(const roco_params* p) {
  const int want = env_int("ROCO_STREAMING_LOADS", -1);
  if (want >= 0) return want != 0;
  const size_t row = static_cast<size_t>(p->head_dim) * (p->dtype == ROCO_BF16 ? 2 : 4);
  return static_cast<size_t>(p->units) * p->budget * row * 2 > (static_cast<size_t>(kStreamingAboveMiB) << 20);
}

// One workgroup per unit once the units cover half of the compute units (measured, bf16, d = 128: 31 vs 34 us per
// step at 128 units x 2048 slots and 19 vs 23 at 128 x 1024, but 30 vs 24 at 64 x 2048 and 54 vs 36 at 64 x 4096,
// where a workgroup per unit leaves most of the chip without work).
bool decode_is_fused(const roco_params* p) {
  const int want = env_int("ROCO_DECODE_FUSED", -1);
  return (want < 0 ? p->units >= 128 : want != 0) && p->budget <= kMaxFusedBudget;
}

}  // namespace

extern "C" {

size_t roco_prefill_workspace_bytes(const roco_params* params, int32_t L_max) {
  if (check_params(params) != ROCO_OK || L_max < 1) return 0;
  return prefill_layout(params, L_max, 1).total;
}

size_t roco_prefill_gqa_workspace_bytes(const roco_params* params, int32_t group, int32_t L_max) {
  if (check_params(params) != ROCO_OK || L_max < 1 || group < 1 || group > kMaxPrefillGroup) return 0;
  if (static_cast<long long>(params->units) * group > 65535) return 0;
  return prefill_layout(params, L_max, group).total;
}

size_t roco_decode_workspace_bytes(const roco_params* params) {
  if (check_params(params) != ROCO_OK) return 0;
  return decode_layout(params).total;
}

int roco_decode_step_launches(const roco_params* params) {
  const int rc = check_params(params);
  if (rc != ROCO_OK) return rc;
  return decode_is_fused(params) ? 1 : 2;
}

}  // extern "C"

namespace {
// roco_prefill_compress (group == 1) and roco_prefill_compress_gqa
int run_prefill(const roco_params* params, int group, const void* Q, const void* K, const void* V,
                const int32_t* len, int32_t L_max, void* K_cache, void* V_cache, float* stats,
                int32_t* pos, int32_t* n_used, int32_t* next_slot, void* O, void* workspace,
                size_t workspace_bytes, void* hip_stream, const float* lse_given = nullptr, bool want_lse = false) {
  const int rc = check_params(params);
  if (rc != ROCO_OK) return rc;
  if (want_lse && (lse_given == nullptr || !aligned16(lse_given) || O != nullptr)) return ROCO_EINVAL;
  if (L_max < 1 || L_max > (1 << 24)) return ROCO_EINVAL;
  if (group < 1) return ROCO_EINVAL;
  if (group > kMaxPrefillGroup || static_cast<long long>(params->units) * group > 65535) return ROCO_EUNSUPPORTED;
  const void* need[] = {Q, K, V, len, K_cache, V_cache, stats, pos, n_used, next_slot, workspace};
  for (const void* ptr : need)
    if (ptr == nullptr || !aligned16(ptr)) return ROCO_EINVAL;
  if (O != nullptr && !aligned16(O)) return ROCO_EINVAL;
  const PrefillLayout lay = prefill_layout(params, L_max, group);
  if (workspace_bytes < lay.total) return ROCO_EWORKSPACE;

  PrefillArgs a;
  a.units = params->units; a.L_max = L_max; a.B = params->budget; a.scope = params->scope;
  a.group = group;
  a.pol = policy_of(params);
  a.pairs = 0;
  a.paired = env_int("ROCO_PREFILL_PAIRED", -1);
  a.skip_rows = want_lse ? 1 : 0;
  a.qsplit = 1;
  a.ksplit = 1;
  a.scale_log2 = scale_log2(params);
  a.recency_window = params->recency_window;
  a.recency_bias_log2 = params->recency_bias * 1.4426950408889634f;
  a.Q = Q; a.K = K; a.V = V; a.len = len;
  a.K_cache = K_cache; a.V_cache = V_cache; a.stats = stats; a.pos = pos; a.n_used = n_used; a.next_slot = next_slot; a.O = O;
  char* ws = static_cast<char*>(workspace);
  a.lse = reinterpret_cast<float*>(ws + lay.lse);
  a.acc = reinterpret_cast<float*>(ws + lay.acc);
  a.acc2 = reinterpret_cast<float*>(ws + lay.acc2);
  a.var_key = reinterpret_cast<uint32_t*>(ws + lay.var_key);
  a.mas_key = reinterpret_cast<uint32_t*>(ws + lay.mas_key);

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  // (the matrix-core kernels address a unit's rows with 32-bit byte offsets: up to 4M tokens of 256 bytes)
  const bool mfma = params->dtype == ROCO_BF16 && params->head_dim == 128 && L_max <= (1 << 22) &&
                    env_int("ROCO_PREFILL_SIMPLE", 0) == 0;
  if (want_lse) {  // the kernels keep base-2 normalisers
    const size_t count = static_cast<size_t>(params->units) * group * L_max;
    if (launch_lse_to_base2(lse_given, a.lse, count, s) != hipSuccess) return ROCO_EHIP;
  }
  hipError_t e = mfma ? launch_prefill_attention_mfma(a, s)
                      : launch_prefill_attention_simple(params->dtype, params->head_dim, a, s);
  if (e != hipSuccess) return ROCO_EHIP;
  if (a.pol.keeps_last_score()) {
    e = launch_prefill_last_row(params->dtype, params->head_dim, a, s);
    if (e != hipSuccess) return ROCO_EHIP;
  }
  e = launch_prefill_select_compact(params->dtype, params->head_dim, a, s);
  return e == hipSuccess ? ROCO_OK : ROCO_EHIP;
}
}  // namespace

namespace {
// Argument checks shared by the two entry points of the token-wise decode step (host only, nothing is launched).
int check_decode_args(const roco_params* params, const void* q, const void* k_new, const void* v_new,
                      const int32_t* qpos, void* K_cache, void* V_cache, float* stats, int32_t* pos, int32_t* n_used,
                      int32_t* next_slot, void* out) {
  const int rc = check_params(params);
  if (rc != ROCO_OK) return rc;
  const void* need[] = {q, k_new, v_new, qpos, K_cache, V_cache, stats, pos, n_used, next_slot, out};
  for (const void* ptr : need)
    if (ptr == nullptr || !aligned16(ptr)) return ROCO_EINVAL;
  return ROCO_OK;
}

// The decode step's kernels on `workspace` (device memory of at least decode_layout(params).total bytes).
int launch_decode_step(const roco_params* params, const void* q, const void* k_new, const void* v_new,
                       const int32_t* qpos, void* K_cache, void* V_cache, float* stats, int32_t* pos,
                       int32_t* n_used, int32_t* next_slot, void* out, int32_t* evicted_slot, int32_t* evicted_pos,
                       void* workspace, void* hip_stream) {
  const DecodeLayout lay = decode_layout(params);
  DecodeArgs a;
  a.units = params->units; a.B = params->budget; a.scope = params->scope;
  a.pol = policy_of(params);
  a.unroll = env_int("ROCO_DECODE_UNROLL", 8);  // rows per lane group per block; 8 measured best on workload 3
  if (a.unroll != 2 && a.unroll != 4) a.unroll = 8;
  a.rotate = env_int("ROCO_DECODE_ROTATE", 1);
  choose_splits(params, a.unroll, a.splits, a.rows_per_split);
  a.fused = decode_is_fused(params) ? 1 : 0;
  a.streaming = streaming_loads(params) ? 1 : 0;
  a.scale_log2 = scale_log2(params);
  a.recency_window = params->recency_window;
  a.recency_bias_log2 = params->recency_bias * 1.4426950408889634f;
  a.q = q; a.k_new = k_new; a.v_new = v_new; a.qpos = qpos;
  a.K = K_cache; a.V = V_cache; a.stats = stats; a.pos = pos; a.n_used = n_used; a.next_slot = next_slot; a.out = out;
  a.evicted_slot = evicted_slot; a.evicted_pos = evicted_pos;
  char* ws = static_cast<char*>(workspace);
  a.z = reinterpret_cast<float*>(ws + lay.z);
  a.part_m = reinterpret_cast<float*>(ws + lay.part_m);
  a.part_l = reinterpret_cast<float*>(ws + lay.part_l);
  a.part_o = reinterpret_cast<float*>(ws + lay.part_o);
  a.keys = reinterpret_cast<uint32_t*>(ws + lay.keys);
  const hipError_t e = launch_decode(params->dtype, params->head_dim, a, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? ROCO_OK : ROCO_EHIP;
}

// Device address of `scratch` on the current device: looked up once per device, with that device current, and kept.
constexpr int kMaxDevices = 64;
bool static_scratch(void** out) {
  static std::mutex mu;
  static void* addr[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
  std::lock_guard<std::mutex> lock(mu);
  if (addr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return false;
    addr[dev] = p;
  }
  *out = addr[dev];
  return true;
}
}  // namespace

extern "C" {

int roco_prefill_compress(const roco_params* params, const void* Q, const void* K, const void* V,
                          const int32_t* len, int32_t L_max, void* K_cache, void* V_cache, float* stats,
                          int32_t* pos, int32_t* n_used, int32_t* next_slot, void* O, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  return run_prefill(params, 1, Q, K, V, len, L_max, K_cache, V_cache, stats, pos, n_used, next_slot, O, workspace,
                     workspace_bytes, hip_stream);
}

int roco_prefill_compress_gqa(const roco_params* params, int32_t group, const void* Q, const void* K, const void* V,
                              const int32_t* len, int32_t L_max, void* K_cache, void* V_cache, float* stats,
                              int32_t* pos, int32_t* n_used, int32_t* next_slot, void* O, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  return run_prefill(params, group, Q, K, V, len, L_max, K_cache, V_cache, stats, pos, n_used, next_slot, O,
                     workspace, workspace_bytes, hip_stream);
}

int roco_prefill_compress_lse(const roco_params* params, int32_t group, const void* Q, const void* K, const void* V,
                              const int32_t* len, int32_t L_max, const float* lse, void* K_cache, void* V_cache,
                              float* stats, int32_t* pos, int32_t* n_used, int32_t* next_slot, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  return run_prefill(params, group, Q, K, V, len, L_max, K_cache, V_cache, stats, pos, n_used, next_slot, nullptr,
                     workspace, workspace_bytes, hip_stream, lse, true);
}

int roco_decode_step(const roco_params* params, const void* q, const void* k_new, const void* v_new,
                     const int32_t* qpos, void* K_cache, void* V_cache, float* stats, int32_t* pos,
                     int32_t* n_used, int32_t* next_slot, void* out, int32_t* evicted_slot,
                     int32_t* evicted_pos, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int rc = check_decode_args(params, q, k_new, v_new, qpos, K_cache, V_cache, stats, pos, n_used, next_slot, out);
  if (rc != ROCO_OK) return rc;
  if (workspace == nullptr || !aligned16(workspace)) return ROCO_EINVAL;
  if (workspace_bytes < decode_layout(params).total) return ROCO_EWORKSPACE;
  return launch_decode_step(params, q, k_new, v_new, qpos, K_cache, V_cache, stats, pos, n_used, next_slot, out,
                            evicted_slot, evicted_pos, workspace, hip_stream);
}

int roco_decode_step_static(const roco_params* params, const void* q, const void* k_new, const void* v_new,
                            const int32_t* qpos, void* K_cache, void* V_cache, float* stats, int32_t* pos,
                            int32_t* n_used, int32_t* next_slot, void* out, int32_t* evicted_slot,
                            int32_t* evicted_pos, void* hip_stream) {
  const int rc = check_decode_args(params, q, k_new, v_new, qpos, K_cache, V_cache, stats, pos, n_used, next_slot, out);
  if (rc != ROCO_OK) return rc;
  if (decode_layout(params).total > static_cast<size_t>(ROCO_STATIC_SCRATCH_BYTES)) return ROCO_ESCRATCH;
  if (roco::g_prof_which >= 0) return ROCO_EUNSUPPORTED;  // the profiling aid creates HIP events
  void* ptr = nullptr;
  if (!static_scratch(&ptr)) return ROCO_EHIP;
  return launch_decode_step(params, q, k_new, v_new, qpos, K_cache, V_cache, stats, pos, n_used, next_slot, out,
                            evicted_slot, evicted_pos, ptr, hip_stream);
}

size_t roco_block_workspace_bytes(const roco_params* params, int32_t block) {
  if (check_block(params, block) != ROCO_OK) return 0;
  return block_layout(params).total;
}

namespace {
// Shared by the block-wise step (one query head per unit) and the grouped-query steps (g heads per unit).
int run_block(const roco_params* params, int tokens, int heads, const void* q, const void* k_new,
              const void* v_new, const int32_t* qpos0, void* K_cache, void* V_cache, float* stats, int32_t* pos,
              int32_t* n_used, int32_t* next_slot, void* out, int32_t* evicted_slot, int32_t* evicted_pos,
              void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (heads < 1) return ROCO_EINVAL;
  const int rc = check_block(params, tokens);
  if (rc != ROCO_OK) return rc;
  if (static_cast<long long>(tokens) * heads > kMaxBlock) return ROCO_EUNSUPPORTED;
  const void* need[] = {q, k_new, v_new, qpos0, K_cache, V_cache, stats, pos, n_used, next_slot, out, workspace};
  for (const void* ptr : need)
    if (ptr == nullptr || !aligned16(ptr)) return ROCO_EINVAL;
  const BlockLayout lay = block_layout(params);
  if (workspace_bytes < lay.total) return ROCO_EWORKSPACE;

  BlockArgs a;
  a.units = params->units; a.B = params->budget; a.scope = params->scope;
  a.pol = policy_of(params);
  a.block = tokens; a.heads = heads; a.queries = tokens * heads;
  a.qrows = a.queries > 32 ? 64 : 32;
  a.row_bytes = params->head_dim * (params->dtype == ROCO_BF16 ? 2 : 4);
  a.streaming = streaming_loads(params) ? 1 : 0;
  {  // split the budget into 64-slot-aligned ranges: two resident workgroups per compute unit measured best
    // (more splits cost more partial results to write and merge than they gain in balance)
    int want = env_int("ROCO_BLOCK_SPLITS", 0);
    if (want <= 0) want = (512 + params->units - 1) / params->units;
    if (want > kMaxBlockSplits) want = kMaxBlockSplits;
    const int max_by_rows = (params->budget + 63) / 64;
    if (want > max_by_rows) want = max_by_rows;
    if (want < 1) want = 1;
    int rows = (params->budget + want - 1) / want;
    rows = (rows + 63) / 64 * 64;
    a.splits = (params->budget + rows - 1) / rows;
    a.rows_per_split = rows;
  }
  a.scale_log2 = scale_log2(params);
  a.recency_window = params->recency_window;
  a.recency_bias_log2 = params->recency_bias * 1.4426950408889634f;
  a.q = q; a.k_new = k_new; a.v_new = v_new; a.qpos0 = qpos0;
  a.K = K_cache; a.V = V_cache; a.stats = stats; a.pos = pos; a.n_used = n_used; a.next_slot = next_slot;
  a.out = out; a.evicted_slot = evicted_slot; a.evicted_pos = evicted_pos;
  char* ws = static_cast<char*>(workspace);
  a.blk_idx = reinterpret_cast<int32_t*>(ws + lay.blk_idx);
  a.z = reinterpret_cast<float*>(ws + lay.z);
  a.part_m = reinterpret_cast<float*>(ws + lay.part_m);
  a.part_l = reinterpret_cast<float*>(ws + lay.part_l);
  a.part_o = reinterpret_cast<float*>(ws + lay.part_o);
  a.keys = reinterpret_cast<uint32_t*>(ws + lay.keys);
  const hipError_t e = launch_block(params->dtype, params->head_dim, a, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? ROCO_OK : ROCO_EHIP;
}
}  // namespace

int roco_encode_block(const roco_params* params, int32_t block, const void* q, const void* k_new, const void* v_new,
                      const int32_t* qpos0, void* K_cache, void* V_cache, float* stats, int32_t* pos, int32_t* n_used,
                      int32_t* next_slot, void* out, int32_t* evicted_slot, int32_t* evicted_pos, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  return run_block(params, block, 1, q, k_new, v_new, qpos0, K_cache, V_cache, stats, pos, n_used,
                   next_slot, out, evicted_slot, evicted_pos, workspace, workspace_bytes, hip_stream);
}

int roco_encode_block_gqa(const roco_params* params, int32_t block, int32_t group, const void* q, const void* k_new,
                          const void* v_new, const int32_t* qpos0, void* K_cache, void* V_cache, float* stats,
                          int32_t* pos, int32_t* n_used, int32_t* next_slot, void* out, int32_t* evicted_slot,
                          int32_t* evicted_pos, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return run_block(params, block, group, q, k_new, v_new, qpos0, K_cache, V_cache, stats, pos, n_used, next_slot, out,
                   evicted_slot, evicted_pos, workspace, workspace_bytes, hip_stream);
}

int roco_decode_step_gqa(const roco_params* params, int32_t group, const void* q, const void* k_new,
                         const void* v_new, const int32_t* qpos, void* K_cache, void* V_cache, float* stats,
                         int32_t* pos, int32_t* n_used, int32_t* next_slot, void* out, int32_t* evicted_slot,
                         int32_t* evicted_pos, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return run_block(params, 1, group, q, k_new, v_new, qpos, K_cache, V_cache, stats, pos, n_used, next_slot, out,
                   evicted_slot, evicted_pos, workspace, workspace_bytes, hip_stream);
}

int roco_select_retained(const roco_params* params, int32_t keep, const float* stats, const int32_t* pos,
                         const int32_t* n_used, int32_t* mask, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  const int rc = check_params(params);
  if (rc != ROCO_OK) return rc;
  if (keep < 0) return ROCO_EINVAL;
  if (policy_of(params).needs_pos() && pos == nullptr) return ROCO_EINVAL;
  const void* need[] = {stats, n_used, mask, workspace};
  for (const void* ptr : need)
    if (ptr == nullptr || !aligned16(ptr)) return ROCO_EINVAL;
  const DecodeLayout lay = decode_layout(params);
  if (workspace_bytes < lay.total) return ROCO_EWORKSPACE;
  DecodeArgs a = {};
  a.units = params->units; a.B = params->budget; a.scope = params->scope;
  a.pol = policy_of(params);
  a.pos = const_cast<int32_t*>(pos);
  a.stats = const_cast<float*>(stats);
  a.n_used = const_cast<int32_t*>(n_used);
  a.keys = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + lay.keys);
  const hipError_t e = launch_select_retained(a, keep, mask, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? ROCO_OK : ROCO_EHIP;
}

int roco_set_overlap(int32_t units, int32_t slots_a, const int32_t* pos_a, const int32_t* mask_a, const int32_t* n_used_a,
                     int32_t slots_b, const int32_t* pos_b, const int32_t* mask_b, const int32_t* n_used_b,
                     int32_t max_pos, int32_t* inter, int32_t* uni, void* hip_stream) {
  if (units < 1 || slots_a < 1 || slots_b < 1 || max_pos < 1) return ROCO_EINVAL;
  if (units > 65535 || max_pos > (1 << 19)) return ROCO_EUNSUPPORTED;  // the bitmap of a unit sits in 64 KiB of LDS
  const void* need[] = {pos_a, n_used_a, pos_b, n_used_b, inter, uni};
  for (const void* ptr : need)
    if (ptr == nullptr || !aligned16(ptr)) return ROCO_EINVAL;
  if ((mask_a != nullptr && !aligned16(mask_a)) || (mask_b != nullptr && !aligned16(mask_b))) return ROCO_EINVAL;
  const hipError_t e = launch_set_overlap(units, slots_a, pos_a, mask_a, n_used_a, slots_b, pos_b, mask_b, n_used_b,
                                          max_pos, inter, uni, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? ROCO_OK : ROCO_EHIP;
}

int roco_select_victims(const roco_params* params, const float* stats, const int32_t* pos, const int32_t* n_used,
                        int32_t* next_slot, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int rc = check_params(params);
  if (rc != ROCO_OK) return rc;
  if (policy_of(params).needs_pos() && pos == nullptr) return ROCO_EINVAL;
  const void* need[] = {stats, n_used, next_slot, workspace};
  for (const void* ptr : need)
    if (ptr == nullptr || !aligned16(ptr)) return ROCO_EINVAL;
  const DecodeLayout lay = decode_layout(params);
  if (workspace_bytes < lay.total) return ROCO_EWORKSPACE;
  DecodeArgs a = {};
  a.units = params->units; a.B = params->budget; a.scope = params->scope;
  a.pol = policy_of(params);
  a.pos = const_cast<int32_t*>(pos);
  a.stats = const_cast<float*>(stats);
  a.n_used = const_cast<int32_t*>(n_used);
  a.next_slot = next_slot;
  a.keys = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + lay.keys);
  const hipError_t e = launch_select_victims(a, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? ROCO_OK : ROCO_EHIP;
}

int roco_probe_cache_read(const roco_params* params, const void* K_cache, const void* V_cache,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int rc = check_params(params);
  if (rc != ROCO_OK) return rc;
  const void* need[] = {K_cache, V_cache, workspace};
  for (const void* ptr : need)
    if (ptr == nullptr || !aligned16(ptr)) return ROCO_EINVAL;
  const DecodeLayout lay = decode_layout(params);
  if (workspace_bytes < lay.total) return ROCO_EWORKSPACE;
  DecodeArgs a = {};
  a.units = params->units; a.B = params->budget;
  a.streaming = streaming_loads(params) ? 1 : 0;
  choose_splits(params, 8, a.splits, a.rows_per_split);
  a.K = const_cast<void*>(K_cache); a.V = const_cast<void*>(V_cache);
  a.part_m = reinterpret_cast<float*>(static_cast<char*>(workspace) + lay.part_m);
  const hipError_t e = launch_cache_read_probe(params->dtype, params->head_dim, a, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? ROCO_OK : ROCO_EHIP;
}

int roco_probe_mfma(int32_t workgroups, int32_t iters, int32_t operands, float* sink, size_t sink_bytes,
                    void* hip_stream) {
  if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || iters > (1 << 20)) return ROCO_EINVAL;
  if (operands < ROCO_PROBE_CONSTANT_OPERANDS || operands > ROCO_PROBE_COLUMN_PASS_MIX) return ROCO_EINVAL;
  if (sink == nullptr || !aligned16(sink)) return ROCO_EINVAL;
  if (sink_bytes < static_cast<size_t>(workgroups) * 256 * sizeof(float)) return ROCO_EWORKSPACE;
  const hipError_t e = launch_mfma_probe(workgroups, iters, operands, sink, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? ROCO_OK : ROCO_EHIP;
}

const char* roco_strerror(int code) {
  switch (code) {
    case ROCO_OK: return "success";
    case ROCO_EINVAL: return "invalid argument (null or misaligned pointer, or a size out of range)";
    case ROCO_EUNSUPPORTED: return "unsupported dtype, head_dim or budget";
    case ROCO_EWORKSPACE: return "workspace too small";
    case ROCO_EHIP: return "HIP kernel launch failed";
    case ROCO_ESCRATCH: return "the call needs more scratch than the library's static buffer holds";
    default: return "unknown error code";
  }
}

int roco_version(void) { return ROCO_VERSION; }

}  // extern "C"
