/*
 * roco.h -- C ABI of the MI355X (gfx950) RoCo library.
 *
 * RoCo (arxiv 2402.06262) keeps the key/value cache of every attention head
 * inside a fixed buffer of B tokens (section 3, "Key-Value Constrained
 * Inference"; section 4, first paragraph).  Per head it maintains three
 * B-sized arrays -- Acc, the accumulated attention probability a cached token
 * has received; Acc2, the accumulated squared probability; Count, how many
 * queries attended it (section 4.3; section 5.3 "Overhead": L x H x B x 3
 * elements) -- and, when the buffer is full, removes the token with the lowest
 * mean attention score Acc/Count among the tokens whose attention variance
 * Acc2/Count - (Acc/Count)^2 is lowest (section 4.3, RoCo = mean attention
 * score + standard-deviation eviction scope).
 *
 * A *unit* is one (layer, sequence, head).  Units are independent (Fig. 1
 * caption: every head evicts at its own positions); the caller folds
 * layers x batch x heads into `units`.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers into memory owned by the caller
 *     (16-byte aligned, dense row-major in the stated shape).  `params` is a
 *     HOST pointer.  `hip_stream` is a hipStream_t passed as void* (NULL = the
 *     null stream).
 *   - The library allocates nothing, frees nothing and never synchronises:
 *     kernels are enqueued on `hip_stream` and the call returns.
 *   - Argument errors are detected on the host before anything is launched
 *     and are reported by a negative return code; 0 is success.
 *   - Values held in device memory (`len`, `n_used`, `qpos`) are trusted.
 *   - A workspace is scratch for the duration of one call's kernels and carries nothing from call to call.  Calls
 *     that may run at the same time (different streams) need workspaces of their own, and caches of their own:
 *     splitting the units of a batch over two streams, each half with its own workspace, is the intended way to
 *     overlap one half's selection with the other half's streaming.
 */
#ifndef ROCO_H
#define ROCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ROCO_VERSION 1

/* storage type of Q, K, V, q, k_new, v_new, the cache and the attention outputs */
enum { ROCO_F32 = 0, ROCO_BF16 = 1 };

/* return codes */
enum {
  ROCO_OK = 0,
  ROCO_EINVAL = -1,        /* null / misaligned pointer, budget < 1, scope outside [1, budget], ... */
  ROCO_EUNSUPPORTED = -2,  /* dtype or head_dim the kernels are not built for                       */
  ROCO_EWORKSPACE = -3,    /* workspace smaller than the matching *_workspace_bytes() query        */
  ROCO_EHIP = -4,          /* a kernel launch failed (hipGetLastError)                             */
  ROCO_ESCRATCH = -5       /* roco_decode_step_static: the shape needs more than ROCO_STATIC_SCRATCH_BYTES */
};

typedef struct roco_params {
  int32_t units;          /* number of independent (layer, sequence, head) units, 1 .. 65535 per call
                             (more: ROCO_EUNSUPPORTED; split the call)                               */
  int32_t head_dim;       /* d': 64 or 128                                                          */
  int32_t budget;         /* B >= 1: slots per unit (section 3: n <= B at every step)               */
  int32_t scope;          /* s in [1, B]: the eviction scope holds the s occupied slots of lowest
                             attention variance; the paper's r (top-r Std protected) is n - s       */
  int32_t dtype;          /* ROCO_F32 or ROCO_BF16                                                  */
  float   scale;          /* softmax scale; <= 0 selects 1/sqrt(head_dim) (section 2.1, eq. 1)      */
  int32_t recency_window; /* w >= 0; 0 = off.  The scaled logit of (query at position qp, key at
                             position kp) gets + recency_bias when 0 <= qp - kp < w.  Not part of
                             the paper; used by the long-context stress workload only.             */
  float   recency_bias;
  /* Eviction policy in the paper's two-stage framework (section 4: an eviction scope, then an importance score
   * inside it).  All three zero is RoCo (section 4.3); the other values are the framework's other members
   * (sections 4.1, 4.2), served by the same kernels.                                                         */
  int32_t importance;     /* ROCO_IMPORTANCE_*: which token of the scope goes first (lowest value)            */
  int32_t scope_kind;     /* ROCO_SCOPE_*: which `scope` tokens form the eviction scope                       */
  int32_t sinks;          /* >= 0; with ROCO_IMPORTANCE_OLDEST, positions < sinks are evicted only when nothing
                             else is in the scope (attention sinks of the window baseline)                   */
} roco_params;

enum {
  ROCO_IMPORTANCE_MAS = 0,    /* mean attention score Acc/Count (section 4.3)                                 */
  ROCO_IMPORTANCE_AAS = 1,    /* accumulated attention score Acc (section 4.1)                                */
  ROCO_IMPORTANCE_OLDEST = 2, /* recency: the lowest position goes first (section 4.1, window / sink baseline) */
  ROCO_IMPORTANCE_LAST = 3,   /* the attention received from the most recent query (section 4.1, LTAS).  The
                                 Acc2 plane of stats then holds that probability instead of the accumulated
                                 squares, so ROCO_SCOPE_STD cannot be combined with it (ROCO_EINVAL)           */
  ROCO_IMPORTANCE_COUNT = 4   /* the number of queries that gave the token more than the average attention of
                                 their row, p > 1 / (tokens attended) (section 4.1, AQAS); kept in the Acc2 plane
                                 like ROCO_IMPORTANCE_LAST, same restriction                                   */
};
enum {
  ROCO_SCOPE_STD = 0,     /* the `scope` tokens of lowest attention variance (section 4.3)                    */
  ROCO_SCOPE_WINDOW = 1,  /* the `scope` oldest tokens: the most recent n - scope are protected (section 4.2)  */
  ROCO_SCOPE_ALL = 2      /* every cached token; `scope` is ignored                                           */
};

/* Bytes of scratch the two calls need for these params (0 on invalid params). */
size_t roco_prefill_workspace_bytes(const roco_params* params, int32_t L_max);
size_t roco_decode_workspace_bytes(const roco_params* params);

/* Kernels one roco_decode_step call launches for these params (for benchmarks that attribute time and bytes):
 * 1 = one workgroup per unit does the whole step (enough units to fill the chip, budget small enough for its
 * logits and ranking keys to sit in LDS); 2 = slot ranges of a unit on several workgroups, then a merge /
 * statistics / selection kernel.  Negative code on invalid params. */
int roco_decode_step_launches(const roco_params* params);

/*
 * Prefill with eviction in one block (section 5.3 "Overhead": block-wise evict-and-encode with the
 * whole prompt as the block; section 5.1.5: B = prompt length x compression rate).
 *
 * Per unit u with length len[u] (1 <= len[u] <= L_max):
 *   P[i,j]   = softmax_j(scale q_i.k_j + bias(i,j)),  j <= i < len         (section 2.1 eq. 1, causal)
 *   Acc[j]   = sum_{i>=j} P[i,j],  Acc2[j] = sum_{i>=j} P[i,j]^2,  Count[j] = len - j   (section 4.3)
 *   if len > B: E = len - B tokens are evicted in one step: among the s+E-1 tokens of lowest variance,
 *   the E of lowest mean attention score (equal keys: lowest position first).  This equals E successive
 *   single evictions by the rule of section 4.3 with the statistics frozen.
 *   The retained min(len,B) tokens are written to the cache in ascending position.
 *
 * Q, K, V   in  [units, L_max, d]   dtype                rows >= len[u] are ignored
 * len       in  [units]             int32
 * K_cache, V_cache  out [units, B, d]  dtype             slots >= n_used[u] are left untouched
 * stats     out [units, 3, B]       fp32  planes Acc, Acc2, Count; unused slots are zeroed
 * pos       out [units, B]          int32 original position of each slot, -1 for unused slots
 * n_used    out [units]             int32 = min(len, B)
 * next_slot out [units]             int32 slot the first decode step will overwrite if the unit is full (its
 *                                   victim by the rule of section 4.3 on the compacted statistics), else -1
 * O         out [units, L_max, d]   dtype attention output of every prompt row, or NULL to skip it
 */
int roco_prefill_compress(const roco_params* params,
                          const void* Q, const void* K, const void* V,
                          const int32_t* len, int32_t L_max,
                          void* K_cache, void* V_cache, float* stats, int32_t* pos, int32_t* n_used,
                          int32_t* next_slot, void* O,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * roco_prefill_compress for grouped-query attention (section 5.3, "Extension to Grouped-Query Attention"): a
 * unit is one key/value head shared by `group` query heads (1 <= group <= 64, units * group <= 65535; else
 * ROCO_EUNSUPPORTED).  Every query head has its own causal softmax; Acc and Acc2 are taken on the mean of the
 * group's probability matrices, Pbar[i,j] = mean_h P_h[i,j]: Acc[j] = sum_i Pbar[i,j], Acc2[j] = sum_i Pbar[i,j]^2.
 * Eviction, compaction and every output are those of roco_prefill_compress.
 * Q in [units, group, L_max, d]; K, V in [units, L_max, d]; O out [units, group, L_max, d] (the attention output of
 * every query head and prompt row) or NULL; workspace of roco_prefill_gqa_workspace_bytes.
 */
size_t roco_prefill_gqa_workspace_bytes(const roco_params* params, int32_t group, int32_t L_max);
int roco_prefill_compress_gqa(const roco_params* params, int32_t group,
                              const void* Q, const void* K, const void* V,
                              const int32_t* len, int32_t L_max,
                              void* K_cache, void* V_cache, float* stats, int32_t* pos, int32_t* n_used,
                              int32_t* next_slot, void* O,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * roco_prefill_compress_gqa for callers whose attention kernel has already produced the row normalisers of the
 * prompt (a flash-attention forward returns them next to its output): the row pass is skipped and only the column
 * statistics (section 4.3), the eviction and the compaction run.
 * lse in [units, group, L_max] fp32 (device): lse[u,h,i] = ln sum_{j<=i} exp(scale q_i.k_j + bias(i,j)), the natural
 * log-sum-exp of the logits exactly as this library forms them (section 2.1, eq. 1; scale and recency bias from
 * params); rows >= len[u] are ignored.  The probabilities are rebuilt as exp(logit - lse), so normalisers of another
 * scale or mask give statistics of another attention.  group = 1 for ordinary multi-head attention.  No attention
 * output is written.  Workspace of roco_prefill_gqa_workspace_bytes (roco_prefill_workspace_bytes when group = 1).
 */
int roco_prefill_compress_lse(const roco_params* params, int32_t group,
                              const void* Q, const void* K, const void* V, const int32_t* len, int32_t L_max,
                              const float* lse,
                              void* K_cache, void* V_cache, float* stats, int32_t* pos, int32_t* n_used,
                              int32_t* next_slot,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * One auto-regressive decode step on the budgeted cache, in place (Fig. 1: one key/value pair is
 * deleted before the next token's is appended; section 4: evict when the buffer is full).
 *
 * Per unit u:
 *   if n_used == B: scope = the s slots of lowest variance max(0, Acc2/Count - (Acc/Count)^2); victim =
 *   the slot of lowest Acc/Count inside it (equal keys: lowest slot first); slot = victim.  (With another
 *   params->importance / scope_kind the two rankings are the ones described at roco_params.)
 *   else slot = n_used, n_used += 1, nothing evicted.
 *   The victim depends only on the statistics left by the previous call, so the library chooses it at the
 *   end of that call and keeps it in next_slot[u]; this call consumes it and, if the unit is full afterwards,
 *   stores the victim of the following step.  next_slot is part of the cache state: it is written by
 *   roco_prefill_compress and roco_decode_step, and must be refreshed with roco_select_victims if the caller
 *   changes stats / n_used by other means.
 *   K_cache[slot] = k_new, V_cache[slot] = v_new, pos[slot] = qpos, the slot's three statistics = 0.
 *   p = softmax_j(scale q.K_cache[j] + bias(qpos, pos[j])) over the occupied slots; out = sum_j p_j V_cache[j]
 *   Acc += p, Acc2 += p^2, Count += 1 on the occupied slots                  (section 4.3)
 *
 * q, k_new, v_new  in      [units, d]     dtype
 * qpos             in      [units]        int32 position of the new token
 * K_cache, V_cache in/out  [units, B, d]  dtype
 * stats            in/out  [units, 3, B]  fp32
 * pos              in/out  [units, B]     int32
 * n_used           in/out  [units]        int32
 * next_slot        in/out  [units]        int32
 * out              out     [units, d]     dtype
 * evicted_slot, evicted_pos  out [units]  int32; -1 when the unit evicted nothing (either may be NULL)
 */
int roco_decode_step(const roco_params* params,
                     const void* q, const void* k_new, const void* v_new, const int32_t* qpos,
                     void* K_cache, void* V_cache, float* stats, int32_t* pos, int32_t* n_used,
                     int32_t* next_slot, void* out, int32_t* evicted_slot, int32_t* evicted_pos,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * roco_decode_step for callers that cannot allocate device memory or pass a workspace along: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace, same kernels,
 * same results bit for bit.  The scratch the kernels need (base-2 logits, per-range partial results, ranking keys) is
 * a ROCO_STATIC_SCRATCH_BYTES array inside the library's device code: every GPU the library runs on holds its own
 * copy until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no allocating library routine);
 * its first call on a device looks the array's address up once.
 *   - A shape whose roco_decode_workspace_bytes(params) exceeds ROCO_STATIC_SCRATCH_BYTES is refused with
 *     ROCO_ESCRATCH before anything is launched (workload 3's 512 units x 2048 slots need 20.3 MiB and fit).
 *   - All calls on one GPU share that GPU's array, and the array keeps the previous call's contents.  Nothing in it
 *     has to start from zero: every word a kernel reads has been written earlier in the same call.  Calls that may
 *     overlap on one GPU (two streams, two threads) race on it: use roco_decode_step with workspaces of their own.
 *   - Refused with ROCO_EUNSUPPORTED while roco_profile_kernel is switched on (that aid creates HIP events).
 */
#define ROCO_STATIC_SCRATCH_BYTES (32u << 20)
int roco_decode_step_static(const roco_params* params,
                            const void* q, const void* k_new, const void* v_new, const int32_t* qpos,
                            void* K_cache, void* V_cache, float* stats, int32_t* pos, int32_t* n_used,
                            int32_t* next_slot, void* out, int32_t* evicted_slot, int32_t* evicted_pos,
                            void* hip_stream);

/*
 * Block-wise evict-and-encode (section 5.3 "Overhead", appendix B: the block size b is the number of tokens
 * freed and encoded within one eviction step; b = 1 is the token-wise scheme of roco_decode_step).
 *
 * Per unit u with n = n_used[u]:
 *   E = max(0, n + b - B) tokens are evicted in one step from the statistics as they stand: among the s + E - 1
 *   slots of lowest variance, the E of lowest Acc/Count (equal keys: lowest slot first) -- E single evictions
 *   by the rule of section 4.3 with frozen statistics.
 *   The block's tokens 0..b-1 go, in order, to the ascending list of freed and still-empty slots; their pos is
 *   qpos0 + i and their three statistics start at 0.  n_used = min(B, n + b).
 *   Query i attends every retained token and the block's tokens 0..i (causal inside the block):
 *   p_i = softmax(scale q_i.K[j] + bias), out_i = sum_j p_ij V[j]; every attended slot gets p_ij, p_ij^2 and 1
 *   added to Acc, Acc2 and Count.  next_slot is left ready for a following roco_decode_step.
 *
 * block            in  1 <= b <= min(64, B)
 * q, k_new, v_new  in  [units, b, d]   dtype
 * qpos0            in  [units]         int32 position of the block's first token
 * cache state      in/out as in roco_decode_step
 * out              out [units, b, d]   dtype
 * evicted_slot, evicted_pos  out [units, b] int32: the slot token i took over from an evicted token and that
 *                  token's position, or -1 where token i went to an empty slot (either may be NULL)
 * workspace        roco_block_workspace_bytes(params, block) bytes: sized for the largest step (64 query rows per
 *                  unit), so that one workspace serves every block size and group size of a unit count and budget
 * Supported: budget a multiple of 4 (else ROCO_EUNSUPPORTED).  K and V are streamed once per block for every dtype
 * and head_dim: bf16 with head_dim 128 on the matrix cores, the others on the vector ALUs (which bound steps of
 * more than about 8 query rows).
 */
size_t roco_block_workspace_bytes(const roco_params* params, int32_t block);
int roco_encode_block(const roco_params* params, int32_t block,
                      const void* q, const void* k_new, const void* v_new, const int32_t* qpos0,
                      void* K_cache, void* V_cache, float* stats, int32_t* pos, int32_t* n_used,
                      int32_t* next_slot, void* out, int32_t* evicted_slot, int32_t* evicted_pos,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Grouped-query attention (section 5.3, "Extension to Grouped-Query Attention"; appendix A): a unit is one
 * key/value head shared by `group` query heads (multi-query attention is group = all heads).  The statistics of a
 * unit receive the group-wise averaged probability once per encoded token:
 * Acc += mean_h p_h, Acc2 += (mean_h p_h)^2, Count += 1; eviction, slot assignment and everything else are those
 * of roco_encode_block.  K and V are streamed once for the whole group and block.
 *
 * roco_encode_block_gqa: `block` tokens per unit, block * group <= 64 (else ROCO_EUNSUPPORTED; 16 tokens of a group
 * of 4 is appendix A's setting); group = 1 is roco_encode_block.  roco_decode_step_gqa: block = 1, so group <= 64;
 * group = 1 is roco_decode_step.
 *
 * q                in  [units, block, group, d] dtype      ([units, group, d] for the decode step)
 * k_new, v_new     in  [units, block, d]        dtype      ([units, d])
 * qpos0 / qpos     in  [units] int32     position of the (first) new token
 * out              out [units, block, group, d] dtype      ([units, group, d])
 * evicted_slot, evicted_pos  out [units, block] int32 as in roco_encode_block (either may be NULL)
 * workspace        roco_block_workspace_bytes(params, block) bytes
 * Supported shapes and error behaviour as for roco_encode_block; group < 1 is ROCO_EINVAL.
 */
int roco_encode_block_gqa(const roco_params* params, int32_t block, int32_t group,
                          const void* q, const void* k_new, const void* v_new, const int32_t* qpos0,
                          void* K_cache, void* V_cache, float* stats, int32_t* pos, int32_t* n_used,
                          int32_t* next_slot, void* out, int32_t* evicted_slot, int32_t* evicted_pos,
                          void* workspace, size_t workspace_bytes, void* hip_stream);
int roco_decode_step_gqa(const roco_params* params, int32_t group,
                         const void* q, const void* k_new, const void* v_new, const int32_t* qpos,
                         void* K_cache, void* V_cache, float* stats, int32_t* pos, int32_t* n_used,
                         int32_t* next_slot, void* out, int32_t* evicted_slot, int32_t* evicted_pos,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Victim selection alone (section 4.3): for every full unit, next_slot[u] = the slot of lowest Acc/Count among
 * the s slots of lowest variance (or what params' policy ranks by); -1 for units that are not full.  Only needed
 * after the caller has edited stats / n_used itself.  stats in [units,3,B], pos in [units,B] (read only by
 * policies that rank by position: ROCO_IMPORTANCE_OLDEST, ROCO_SCOPE_WINDOW; may be NULL otherwise), n_used in
 * [units], next_slot out [units]; the workspace is the decode workspace.
 */
int roco_select_victims(const roco_params* params, const float* stats, const int32_t* pos, const int32_t* n_used,
                        int32_t* next_slot, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Which cached tokens a smaller budget would keep (the sets compared by the consistency study of section 4.1,
 * Fig. 2: the top-B important tokens under a policy): mask[u][j] = 1 if slot j of unit u survives one eviction
 * step that shrinks the unit to `keep` tokens (n_used - keep evictions by the params' policy with the statistics
 * as they stand: among the scope + E - 1 slots of lowest scope key, the E of lowest importance), else 0; empty
 * slots get 0; units with n_used <= keep keep everything.  Nothing but mask is written.
 * stats in [units,3,B], pos in [units,B] (may be NULL unless the policy ranks by position), n_used in [units],
 * mask out [units,B] int32; the workspace is the decode workspace.
 */
int roco_select_retained(const roco_params* params, int32_t keep, const float* stats, const int32_t* pos,
                         const int32_t* n_used, int32_t* mask, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/*
 * Overlap of two sets of cached tokens per unit: the two counts behind the Jaccard similarity |A and B| / |A or B| of
 * the consistency study (section 4.1, Fig. 2: the tokens a budgeted cache holds against the top-B tokens of the full
 * cache).  Set A of unit u holds the positions pos_a[u][j] of the slots j < n_used_a[u] whose mask_a[u][j] is not 0
 * (mask_a NULL: all of those slots); set B likewise.  Positions outside [0, max_pos) are ignored; positions inside one
 * cache are distinct.
 * pos_a, mask_a in [units, slots_a] int32; n_used_a in [units]; pos_b, mask_b in [units, slots_b]; n_used_b in [units];
 * inter, uni out [units] int32.  max_pos <= 524288 (else ROCO_EUNSUPPORTED).  No workspace.
 */
int roco_set_overlap(int32_t units, int32_t slots_a, const int32_t* pos_a, const int32_t* mask_a, const int32_t* n_used_a,
                     int32_t slots_b, const int32_t* pos_b, const int32_t* mask_b, const int32_t* n_used_b,
                     int32_t max_pos, int32_t* inter, int32_t* uni, void* hip_stream);

/*
 * Profiling aid (not part of the method; for benchmarks).  roco_profile_kernel(k) makes every later call
 * record a pair of HIP events on the caller's stream around kernel k only (k = one of ROCO_PROF_*; -1 turns
 * it off).  roco_profile_read() waits for the recorded events, returns their summed elapsed time in
 * milliseconds and their count since the last read, and recycles them.  This mode creates HIP events (the
 * only resources the library ever creates) and is not thread-safe.  Returns 0 or a negative code.
 */
/* ROCO_PROF_DECODE_ATTEND also stands for the single kernel of a decode step that roco_decode_step_launches
 * reports as 1 launch. */
enum {
  ROCO_PROF_DECODE_SELECT = 0, ROCO_PROF_DECODE_ATTEND = 1, ROCO_PROF_DECODE_FINISH = 2,
  ROCO_PROF_PREFILL_ROWS = 3, ROCO_PROF_PREFILL_COLUMNS = 4, ROCO_PROF_PREFILL_SELECT = 5,
  ROCO_PROF_PREFILL_GATHER = 6, ROCO_PROF_READ_PROBE = 7, ROCO_PROF_BLOCK_PREPARE = 8,
  ROCO_PROF_BLOCK_ATTEND = 9, ROCO_PROF_BLOCK_FINISH = 10, ROCO_PROF_MFMA_PROBE = 11, ROCO_PROF_KERNELS = 12
};
int roco_profile_kernel(int which);
int roco_profile_read(double* total_ms, int64_t* launches);
/* Bracket only every `every`-th launch of the profiled kernel (default 1): a pair of event records costs a few
 * microseconds of stream time, which matters when the kernel itself takes a tenth of a millisecond. */
int roco_profile_sampling(int every);

/*
 * Benchmark aid: reads every row of K_cache and V_cache ([units, B, d]) once with exactly the grid, the loads and
 * the load order of the decode attention kernel and does nothing else, so that a benchmark can measure, on the
 * machine at hand, the bandwidth ceiling of that access pattern.  The workspace is the decode workspace.
 */
int roco_probe_cache_read(const roco_params* params, const void* K_cache, const void* V_cache,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Benchmark aid: `workgroups` workgroups of four waves, each wave issuing iters x 8 dependent-by-four
 * v_mfma_f32_32x32x16_bf16 (the instruction of the prefill statistics passes) on register operands and nothing else,
 * so that a benchmark can measure the matrix throughput the machine at hand sustains (its clock under that load
 * included).  `operands`: ROCO_PROBE_CONSTANT_OPERANDS = one operand pair holding a few small values;
 * ROCO_PROBE_RANDOM_OPERANDS = eight operand pairs of pseudo-random values in (-2, 2), whose bit activity is that of
 * real activations (the matrix units draw more power and the sustained clock is lower).  Flops of one call =
 * workgroups * 4 * iters * 8 * 32768.
 * ROCO_PROBE_ROW_PASS_MIX / ROCO_PROBE_COLUMN_PASS_MIX: the steady state of the row / column pass instead -- per
 * wave `iters` tiles of 32 matrix instructions on pseudo-random values, interleaved as in the passes with the 16
 * fragment reads from an LDS tile (which the workgroup fills itself) and the pass's vector work per score (multiply-
 * add, exponential, add; the column pass one multiply-add more and the row normalisers from LDS), with no global
 * loads, barriers or masks: the ceiling of the passes' instruction mix.  Flops = workgroups * 4 * iters * 32 * 32768.
 * sink out [workgroups * 256] fp32 (device): receives a checksum per lane.
 * 1 <= workgroups <= 1048576, 1 <= iters <= 1048576.
 */
#define ROCO_PROBE_CONSTANT_OPERANDS 0
#define ROCO_PROBE_RANDOM_OPERANDS 1
#define ROCO_PROBE_ROW_PASS_MIX 2
#define ROCO_PROBE_COLUMN_PASS_MIX 3
int roco_probe_mfma(int32_t workgroups, int32_t iters, int32_t operands, float* sink, size_t sink_bytes,
                    void* hip_stream);

/*
 * Environment switches (read on the host at every call; meant for tests and tuning, the defaults are the measured
 * choices).  None of them changes what a call computes, only which kernels and launch shapes do it.
 *   ROCO_DECODE_FUSED=0|1      decode step as the split pair / as one kernel (default: one kernel from 128 units on
 *                              when budget <= 4096); roco_decode_step_launches reports the choice
 *   ROCO_DECODE_SPLITS=n       splits of the budget in the split pair (default: until about 128 workgroups exist)
 *   ROCO_DECODE_UNROLL=2|4|8   cache rows in flight per lane group (default 8)
 *   ROCO_DECODE_ROTATE=0|1     staggered start row per workgroup (default 1)
 *   ROCO_STREAMING_LOADS=0|1   non-temporal loads of the cache rows (default: caches above 192 MiB)
 *   ROCO_PREFILL_SIMPLE=1      vector-ALU prefill passes also for bf16 / head_dim 128
 *   ROCO_PREFILL_PAIRED=0|1    one block of rows per workgroup / a long and a short one (default 1)
 *   ROCO_PREFILL_QSPLIT=1|2    workgroups per block of rows in the two prefill passes (default: 2 with few units)
 *   ROCO_PREFILL_GQA_RING=0    grouped-query column pass with register-staged tiles instead of the LDS ring
 *   ROCO_BLOCK_SPLITS=n        splits of the budget in the block-wise / grouped steps (default: about 512 / units)
 *   ROCO_BLOCK_SINGLE=0        single-token block steps go through the preparing kernel like longer blocks
 */

/* Static description of a return code. */
const char* roco_strerror(int code);

/* ROCO_VERSION the library was built from. */
int roco_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ROCO_H */
