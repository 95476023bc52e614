// Internal launch interface between the C ABI (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace roco {

// Eviction policy in the paper's two-stage framework (section 4): an eviction scope, then an importance score
// inside it.  All zeros is RoCo (section 4.3).
enum : int { kImpMas = 0, kImpAas = 1, kImpOldest = 2, kImpLast = 3, kImpCount = 4 };
enum : int { kScopeStd = 0, kScopeWindow = 1, kScopeAll = 2 };
struct Policy {
  int importance;  // kImpMas: Acc/Count; kImpAas: Acc; kImpOldest: position, the first `sinks` positions last;
                   // kImpLast: the attention from the latest query, kept in the second statistics plane;
                   // kImpCount: how many queries gave the token more than their row's average attention, ditto
  int scope_kind;  // kScopeStd: lowest variance; kScopeWindow: lowest position (oldest); kScopeAll: everything
  int sinks;
  // the second plane holds the latest query's probability instead of the accumulated squares
  __host__ __device__ bool keeps_last_score() const { return importance == kImpLast; }
  // ... or counts the queries whose probability for the token was above 1 / (tokens the query attended)
  __host__ __device__ bool counts_above_average() const { return importance == kImpCount; }
  // The second statistic after a query that attended `attended` tokens gave the token probability p.
  __host__ __device__ float second_statistic(float old, float p, float attended) const {
    if (importance == kImpLast) return p;
    if (importance == kImpCount) return old + (p * attended > 1.0f ? 1.0f : 0.0f);
    return old + p * p;
  }
  __host__ __device__ bool needs_pos() const { return importance == kImpOldest || scope_kind == kScopeWindow; }
  // number of tokens inside the scope when n are cached
  __host__ __device__ int scope_size(int scope, int n) const { return scope_kind == kScopeAll ? n : scope; }
};

constexpr int kMaxSplits = 64;        // upper bound on split-K partials per unit (sizes the workspace)
constexpr int kDecodeSelectThreads = 256;
constexpr int kMaxFusedBudget = 4096;       // largest budget of the one-kernel decode step (keys and logits in LDS)
constexpr int kMaxDecodeBudgetLds = 16384;  // ranking keys of a unit are kept in LDS up to here (128 KiB), else in the workspace
constexpr size_t kDefaultDynamicLds = 65536;  // LDS a kernel may use without raising its limit first
constexpr size_t kStaticLdsAllowance = 8192;  // upper bound on the statically declared LDS of the kernels that ask

// Dynamic LDS for the ranking keys of one unit (0: they go to the workspace); raises the kernel's limit when the
// request, together with what the kernel declares statically, may be above the default one.  Returns false if the
// runtime refuses.
inline size_t key_lds_bytes(int B) {
  return B <= kMaxDecodeBudgetLds ? static_cast<size_t>(B) * 2 * sizeof(uint32_t) : 0;
}
inline bool allow_key_lds(const void* kernel, size_t bytes) {
  if (bytes + kStaticLdsAllowance <= kDefaultDynamicLds) return true;
  return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes)) == hipSuccess;
}

struct DecodeArgs {
  int units, B, scope, splits, rows_per_split;
  Policy pol;
  int unroll;            // rows in flight per lane group in decode_attend: 2, 4 or 8
  int fused;             // 1: one workgroup does the whole step of a unit (decode_fused), no workspace traffic
  int streaming;         // 1: K / V rows are loaded with the non-temporal hint (cache far larger than the last-level cache)
  int rotate;            // stagger the start offset of every workgroup inside its slot range
  float scale_log2;      // scale * log2(e)
  int recency_window;
  float recency_bias_log2;
  const void *q, *k_new, *v_new;
  const int32_t* qpos;
  void *K, *V;
  float* stats;          // [units][3][B]
  int32_t *pos, *n_used;
  int32_t* next_slot;    // [units] victim chosen for the next step (valid while the unit is full)
  void* out;
  int32_t *evicted_slot, *evicted_pos;
  // workspace
  float* z;              // [units][B]   base-2 logits of this step
  float* part_m;         // [units][splits]
  float* part_l;         // [units][splits]
  float* part_o;         // [units][splits][D]
  uint32_t* keys;        // [units][2][B] ranking keys when B is too large for LDS, else unused
};

struct PrefillArgs {
  int units, L_max, B, scope;
  int group;             // query heads per unit (1 without grouped-query attention): Q and lse are [units][group][L_max]
  Policy pol;
  int pairs;             // matrix-core path: workgroup ids per unit (set by its launcher)
  int paired;            // matrix-core path: 1 = long+short block per workgroup, 0 = one block, -1 = choose
  int skip_rows;         // 1: lse already holds the row normalisers, pass 1 is not run
  int qsplit;            // matrix-core path: 1, or 2 = two workgroups share a block's queries (set by its launcher)
  int ksplit;            // matrix-core path, row pass: 1, or 2 = two workgroups share a block's keys (ditto)
  float scale_log2;
  int recency_window;
  float recency_bias_log2;
  const void *Q, *K, *V;
  const int32_t* len;
  void *K_cache, *V_cache;
  float* stats;          // [units][3][B]
  int32_t *pos, *n_used;
  int32_t* next_slot;    // [units]
  void* O;               // may be null
  // workspace
  float* lse;            // [units][group][L_max]  base-2 log-sum-exp of every query row
  float* acc;            // [units][L_max]
  float* acc2;           // [units][L_max]
  uint32_t* var_key;     // [units][L_max]
  uint32_t* mas_key;     // [units][L_max]
};

constexpr int kMaxBlock = 64;        // query rows (tokens x heads) per block-wise step: two 32-wide matrix tiles
constexpr int kMaxBlockSplits = 8;   // split-K partials per unit of the block-wise step

struct BlockArgs {
  int units, B, scope, block, splits, rows_per_split;
  Policy pol;
  int streaming;  // as DecodeArgs::streaming
  int row_bytes;  // bytes of a K / V / q row
  int single;     // 1: single-token step without block_prepare (set by launch_block)
  int heads;    // query heads that share the unit's keys and values (1 without grouped-query attention)
  int queries;  // query rows per unit = block * heads <= 64; row r belongs to token r / heads, head r % heads
  int qrows;    // rows per unit of the z / part_* planes: 32, or 64 when queries > 32
  float scale_log2;
  int recency_window;
  float recency_bias_log2;
  const void *q, *k_new, *v_new;   // q [units][block][heads][128], k_new / v_new [units][block][128] bf16
  const int32_t* qpos0;            // [units]
  void *K, *V;
  float* stats;
  int32_t *pos, *n_used, *next_slot;
  void* out;                       // [units][block][heads][128] bf16
  int32_t *evicted_slot, *evicted_pos;  // [units][block], may be null
  // workspace
  int32_t* blk_idx;                // [units][B]   block token index held by a slot, -1 for older tokens
  float* z;                        // [units][qrows][B] base-2 logits
  float* part_m;                   // [units][splits][qrows]
  float* part_l;                   // [units][splits][qrows]
  float* part_o;                   // [units][splits][qrows][128]
  uint32_t* keys;                  // [units][2][B] when B is too large for LDS
};
hipError_t launch_block(int dtype, int head_dim, const BlockArgs& a, hipStream_t s);  // B % 4 == 0

// dtype: 0 = f32, 1 = bf16; head_dim: 64 or 128.  Each returns hipGetLastError() of its launches.
hipError_t launch_decode(int dtype, int head_dim, const DecodeArgs& a, hipStream_t s);
int decode_rows_per_pass(int dtype, int head_dim, int unroll);  // granularity of DecodeArgs::rows_per_split
hipError_t launch_cache_read_probe(int dtype, int head_dim, const DecodeArgs& a, hipStream_t s);
hipError_t launch_mfma_probe(int workgroups, int iters, int mode, float* sink, hipStream_t s);  // mode: ROCO_PROBE_*
hipError_t launch_select_victims(const DecodeArgs& a, hipStream_t s);
// uses stats, pos, n_used, keys; writes mask[units][B] (1 = survives a shrink of the unit to `keep` tokens)
hipError_t launch_select_retained(const DecodeArgs& a, int keep, int32_t* mask, hipStream_t s);  // uses stats, n_used, next_slot, keys
// |A and B| and |A or B| per unit of two sets of cached positions in [0, max_pos), max_pos <= 524288
hipError_t launch_set_overlap(int units, int slots_a, const int32_t* pos_a, const int32_t* mask_a, const int32_t* n_a,
                              int slots_b, const int32_t* pos_b, const int32_t* mask_b, const int32_t* n_b, int max_pos,
                              int32_t* inter, int32_t* uni, hipStream_t s);
hipError_t launch_prefill_attention_simple(int dtype, int head_dim, const PrefillArgs& a, hipStream_t s);
hipError_t launch_prefill_attention_mfma(const PrefillArgs& a, hipStream_t s);  // bf16, head_dim 128
// overwrites PrefillArgs::acc2 with the attention row of each unit's last prompt token (kImpLast)
hipError_t launch_lse_to_base2(const float* lse_ln, float* lse_log2, size_t n, hipStream_t s);
hipError_t launch_prefill_last_row(int dtype, int head_dim, const PrefillArgs& a, hipStream_t s);
hipError_t launch_prefill_select_compact(int dtype, int head_dim, const PrefillArgs& a, hipStream_t s);

}  // namespace roco
