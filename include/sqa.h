/*
 * sqa -- SqueezeAttention hot path for AMD MI355X (gfx950), C ABI.
 *
 * The calls follow the paper's Algorithm 1:
 *   prefill:  sqa_layer_importance   (steps 1-4: cosine similarity of the hidden
 *                                     state before/after self-attention, Sec. 3)
 *             sqa_allocate_budgets   (steps 5-11: cluster layers into 3 groups,
 *                                     move budget from G3 to the others; host)
 *             sqa_prefill_scores     (H2O's accumulated attention over the prompt,
 *                                     Sec. 5.1 "Heavy-Hitter")
 *             sqa_prefill_compress   (steps 12 + 16-17: the sequence-wise policy
 *                                     C_seq applied with the layer's own budget)
 *   decode:   sqa_decode_step        (steps 14-21 with Eq. 2-3: append, evict if
 *                                     over budget, attention, H2O accumulation)
 *   Around them: *_ex forms for batches whose sequences differ (sqa_batch_opts),
 *   sqa_prefill_scores_lse, sqa_residual_add_importance, sqa_decode_plan (what a
 *   decode call would launch), sqa_kept_idx_sorted, and for K/V kept in 16-row
 *   blocks (sqa_layer_cache.block_table) the host free list sqa_block_pool_*.
 *
 * Conventions
 *   - "DEVICE" pointers are HIP device memory owned by the caller and borrowed
 *     until the work enqueued on `stream` has finished; "HOST" pointers are
 *     ordinary host memory read or written before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - The library allocates no device memory and keeps no state between calls
 *     (apart from remembering which kernels it has already allowed to use
 *     more than 64 KiB of on-chip memory on a device); scratch
 *     space comes in through `workspace` (DEVICE, 256-byte aligned), whose
 *     minimum size the matching *_workspace_bytes call returns.  Two exceptions,
 *     both stated where they are declared: sqa_decode_step_static keeps its
 *     scratch in a device array of the library image, and a sqa_block_pool is a
 *     host object that the caller creates and destroys.
 *   - Arguments are validated on the host before any HIP call is made; on an
 *     error nothing is enqueued and no output is touched.  Kernels are
 *     enqueued asynchronously; nothing synchronises the stream except
 *     sqa_read_device_status.
 *   - All tensors are dense, row-major, last index fastest.
 */
#ifndef SQA_H_
#define SQA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SQA_OK = 0,
  SQA_ERR_NULL = 1,      /* a required pointer is NULL                              */
  SQA_ERR_SHAPE = 2,     /* non-positive size, Hq % Hkv != 0, unsupported D or group */
  SQA_ERR_DTYPE = 3,     /* unknown sqa_dtype                                        */
  SQA_ERR_POLICY = 4,    /* unknown sqa_policy or negative n_sink                    */
  SQA_ERR_BUDGET = 5,    /* p outside (0,1], total < n_layers, budget too small      */
  SQA_ERR_CAPACITY = 6,  /* cache capacity / workspace / on-chip memory too small    */
  SQA_ERR_HIP = 7,       /* the HIP runtime reported an error                        */
  SQA_ERR_STATE = 8      /* device-side: a cache was longer than its budget on entry
                            (device-side checks also report SQA_ERR_CAPACITY: no free
                            slot, and SQA_ERR_BUDGET: a per-sequence budget out of range) */
} sqa_status;

typedef enum { SQA_F32 = 0, SQA_BF16 = 1 } sqa_dtype;
typedef enum { SQA_SLIDING = 0, SQA_STREAMING = 1, SQA_H2O = 2 } sqa_policy;
/* Where the policy runs inside a decode step.  Algorithm 1 as printed compresses
 * before the step's attention (steps 16-17, then 19); Sec. 2.2 describes policies
 * that judge tokens by the attention they just received, i.e. after it. */
typedef enum { SQA_EVICT_THEN_ATTEND = 0, SQA_ATTEND_THEN_EVICT = 1 } sqa_order;

enum { SQA_MAX_LAYERS = 128 };
enum { SQA_BLOCK_SLOTS = 16, SQA_MAX_BLOCKS_PER_UNIT = 1024 };   /* blocked K/V allocation (sqa_layer_cache.block_table) */
enum { SQA_ST_LEN = 0, SQA_ST_RING_HEAD = 1, SQA_ST_EVICT_HINT = 2, SQA_ST_WORDS = 4 };

/*
 * One layer's compact KV cache ("K^(i)" of Algorithm 1 after C_seq).  All
 * pointers are DEVICE memory.  A unit is one (sequence b, KV head h); unit
 * index u = b*Hkv + h.  Slot order inside a unit is NOT position order (softmax
 * attention does not depend on it); `pos` says which token sits in each slot.
 *
 * Slot layout of a unit with budget b, hh protected/heavy slots and rec = b-hh
 * recent slots (hh = 0 sliding, n_sink streaming, floor(b/2) H2O):
 *   while len < b : slots [0,len) hold the tokens in ascending position;
 *   once len == b : slots [0,hh) hold the non-recent tokens (sinks / heavy
 *                   hitters, any order), slots [hh,b) are a ring holding the rec
 *                   most recent tokens, the oldest at slot hh + ring_head[u].
 * sqa_prefill_compress writes this layout (ascending position, ring_head 0);
 * sqa_decode_step keeps it.
 */
typedef struct sqa_layer_cache {
  void* K;             /* [B][Hkv][capacity][D], element type = the call's dtype   */
  void* V;             /* [B][Hkv][capacity][D]                                    */
  float* score_acc;    /* [B][Hkv][capacity] accumulated attention (H2O; else may be NULL) */
  int32_t* pos;        /* [B][Hkv][capacity] token position per slot = kept_idx    */
  int32_t* unit_state; /* [B][Hkv][4], 16-byte aligned: one record per unit, read and
                          written as one 16-byte access (a step that updated three
                          separate words per unit paid for three small writes):
                            [SQA_ST_LEN]        number of valid slots ("len")
                            [SQA_ST_RING_HEAD]  offset of the oldest recent token in
                                                the ring ("ring_head")
                            [SQA_ST_EVICT_HINT] H2O: the next eviction, decided at the
                                                end of the previous decode step: -1 =
                                                the token leaving the ring goes, s >= 0
                                                = heavy slot s goes, -2 = not decided
                                                (sqa_prefill_compress writes this; write
                                                it too after editing a unit's scores,
                                                positions or budget) ("evict_hint")
                            [3]                 reserved, written as 0              */
  const int64_t* unit_offset; /* NULL: every unit owns `capacity` slots, unit u the slots
                          [u*capacity, (u+1)*capacity) of K, V, score_acc and pos (the
                          shapes above).  Otherwise DEVICE int64 [B*Hkv + 1], ascending:
                          units are packed, unit u owns slots [unit_offset[u],
                          unit_offset[u+1]) -- as many as ITS budget needs, which is what
                          saves memory when budgets differ per sequence; `capacity` is
                          then the largest of them                                  */
  const int32_t* block_table; /* NULL: K and V rows lie where unit_offset / capacity say (above).  Otherwise
                          DEVICE int32 [B*Hkv][blocks_per_unit]: blocked allocation.  K and V are then
                          POOLS of blocks of SQA_BLOCK_SLOTS rows, [n_blocks][SQA_BLOCK_SLOTS][D], shared by
                          all units of the layer, and the rows of unit u's slots 16i .. 16i+15 are block
                          block_table[u][i] of both pools (only the entries that the unit's own budget
                          needs are read, i < ceil(min(capacity, its budget) / SQA_BLOCK_SLOTS): a sequence
                          with a small budget holds few blocks).  A serving loop hands a leaving sequence's blocks to the next one,
                          whatever their budgets, without moving anything.  score_acc, pos and unit_state
                          stay dense ([B][Hkv][capacity]: 8 bytes per slot); unit_offset must be NULL.
                          An entry outside [0, n_blocks) is reported through the device status
                          (SQA_ERR_SHAPE) and the unit is left untouched                        */
  int32_t capacity;    /* slots per unit; >= min(budget, longest length reached)   */
  int32_t budget;      /* b^(i): most tokens this layer keeps                      */
  int32_t blocks_per_unit; /* row length of block_table; >= ceil(min(capacity, budget) / SQA_BLOCK_SLOTS),
                          at most SQA_MAX_BLOCKS_PER_UNIT (else SQA_ERR_SHAPE)        */
  int32_t n_blocks;    /* blocks in each of the K and V pools                      */
} sqa_layer_cache;

/*
 * Per-sequence variation inside one batch, for the *_ex calls.  The paper states
 * Algorithm 1 for a batch with one prompt length p and one budget list (Sec. 2.1
 * notation, Algorithm 1 "Require"); these fields cover batches whose sequences
 * differ in prompt length, position and -- when each sequence is probed and
 * budgeted on its own -- in budgets.  Every pointer is optional (NULL = the uniform value of the
 * plain call) and DEVICE memory, read when the kernels run.
 */
typedef struct sqa_batch_opts {
  const int32_t* prompt_len;   /* [B] tokens of sequence b's prompt, 0..P; its rows beyond that are padding
                                  (sqa_prefill_scores_ex, sqa_prefill_compress_layers_ex)               */
  const int32_t* budget_seq;   /* [n_layers][B] budget of layer l for sequence b; each must lie between the
                                  policy's minimum and layers[l].budget, which stays the layer's maximum and
                                  sizes capacity and scratch (compress, decode)                          */
  const int32_t* new_pos_seq;  /* [B] position of sequence b's new token; < 0 = the sequence takes no part in
                                  this step: its caches and out rows are left untouched (decode)          */
  int32_t* status;             /* one int32 that compress sets to SQA_ERR_SHAPE / SQA_ERR_BUDGET when a
                                  prompt_len / budget_seq entry is out of range (that unit is left empty);
                                  decode reports through its workspace status word instead               */
  int32_t order;               /* sqa_order (decode)                                                    */
} sqa_batch_opts;

const char* sqa_status_str(sqa_status s);

/* ---- Algorithm 1 steps 1-4; Sec. 3 cosine-similarity equation -------------
 * cos_out[l] = (1/n_tokens) * sum_j  A_j.B_j / (max(|A_j|,1e-8) * max(|B_j|,1e-8))
 * with A_j, B_j the rows of h_in[l], h_out[l] (all tokens of the batch, b*p rows).
 *   h_in, h_out : DEVICE [n_layers][n_tokens][hidden], dtype dt; hidden % 8 == 0
 *   cos_out     : DEVICE float [n_layers]
 *   workspace   : DEVICE, >= sqa_layer_importance_workspace_bytes(...)
 * Products accumulate in fp32, the token mean in fp64, fixed order (results are
 * run-to-run identical). */
size_t sqa_layer_importance_workspace_bytes(int n_layers, int64_t n_tokens, int hidden);
sqa_status sqa_layer_importance(const void* h_in, const void* h_out, sqa_dtype dt,
                                int n_layers, int64_t n_tokens, int hidden,
                                float* cos_out, void* workspace, size_t ws_bytes, void* stream);

/* Per-sequence cosines (Sec. 3 equation with the token mean taken over one
 * sequence's prompt instead of the whole batch), for per-sequence budgets: the token
 * rows of the n_seq sequences lie one after another, sequence s owning rows
 * seq_start[s] .. seq_start[s+1]-1 of every layer.
 *   seq_start : DEVICE int32 [n_seq+1], ascending, seq_start[0] >= 0,
 *               seq_start[n_seq] <= n_tokens; an empty sequence gets cosine 0
 *   cos_out   : DEVICE float [n_layers][n_seq]
 *   workspace : DEVICE, >= n_seq * sqa_layer_importance_workspace_bytes(n_layers, n_tokens, hidden) */
sqa_status sqa_layer_importance_seq(const void* h_in, const void* h_out, sqa_dtype dt,
                                    int n_layers, int64_t n_tokens, int hidden,
                                    const int32_t* seq_start, int n_seq,
                                    float* cos_out, void* workspace, size_t ws_bytes, void* stream);

/* The same probe fused into the producer of the "after" tensor (Sec. 3: the
 * hidden state after the self-attention block is the block's input plus the
 * attention output, the residual connection):
 *   h_out[l][j][k] = h_in[l][j][k] + attn_out[l][j][k]   (fp32 add, rounded to dt)
 * is written and cos_out[l] is taken between h_in and the stored h_out in the
 * same pass, so the probe adds no memory traffic to the residual add.
 *   h_in, attn_out : DEVICE [n_layers][n_tokens][hidden], dtype dt
 *   h_out          : DEVICE, same shape; may be the very buffer h_in or attn_out
 *                    (in-place), otherwise must not overlap them
 * cos_out, workspace as above (same workspace size). */
sqa_status sqa_residual_add_importance(const void* h_in, const void* attn_out, void* h_out, sqa_dtype dt,
                                       int n_layers, int64_t n_tokens, int hidden,
                                       float* cos_out, void* workspace, size_t ws_bytes, void* stream);

/* ---- Algorithm 1 steps 5-11; Sec. 4.2.2; Appendix A.2 ---------------------
 * Host only.  Clusters the n_layers cosines into (up to) 3 groups by the exact
 * optimum of 1-D k-means (contiguous split of the sorted values, cuts only
 * between distinct values, ties -> smallest cuts); G3 = the group with the
 * largest cosines.  G3 layers get floor(total_budget*p/n_layers); the rest of
 * total_budget is split evenly over the other layers, the remainder going +1
 * to those with the lowest layer index, so the budgets sum to total_budget.
 * One distinct cosine value -> uniform budgets.
 *   cos        : HOST float [n_layers]
 *   budget_out : HOST int32 [n_layers]
 *   group_out  : HOST int8 [n_layers] or NULL; 0 = G1 (lowest cos), 1 = G2, 2 = G3
 * SQA_ERR_BUDGET if p is outside (0,1], total_budget < n_layers or a budget
 * would be < 1. */
sqa_status sqa_allocate_budgets(const float* cos, int n_layers, int64_t total_budget, double p,
                                int32_t* budget_out, int8_t* group_out);

/* ---- H2O accumulated attention of the prompt (Sec. 5.1 "Heavy-Hitter") ----
 * scores[b][hkv][j] = sum over the g = Hq/Hkv query heads of the KV head and
 * over prompt queries i >= j of softmax_j'<=i(Q_i.K_j'/sqrt(D))[j].
 *   Q : DEVICE [B][Hq][P][D], K : DEVICE [B][Hkv][P][D], dtype dt
 *   scores_out : DEVICE float [B][Hkv][P]
 *   workspace  : DEVICE, >= sqa_prefill_scores_workspace_bytes(...) */
size_t sqa_prefill_scores_workspace_bytes(int B, int Hq, int Hkv, int P, int D);
sqa_status sqa_prefill_scores(const void* Q, const void* K, sqa_dtype dt,
                              int B, int Hq, int Hkv, int P, int D,
                              float* scores_out, void* workspace, size_t ws_bytes, void* stream);
/* With opts->prompt_len: only queries i < prompt_len[b] are counted; scores of
 * positions >= prompt_len[b] come out 0.  opts may be NULL. */
sqa_status sqa_prefill_scores_ex(const void* Q, const void* K, sqa_dtype dt,
                                 int B, int Hq, int Hkv, int P, int D,
                                 float* scores_out, void* workspace, size_t ws_bytes, void* stream,
                                 const sqa_batch_opts* opts);

/* The same scores when the softmax normalisers of the prompt's attention are already known: a fused
 * attention kernel that runs the prompt returns, per query row, the logarithm of its normaliser, and with it
 * the column sums need one pass over the logits instead of two (half the work of sqa_prefill_scores).
 *   row_lse : DEVICE float [B][Hq][P], row_lse[b][h][i] = ln sum_{j<=i} exp(Q_i.K_j / sqrt(D))
 *             (natural logarithm, logits already scaled by 1/sqrt(D), causal); rows of padding are not read
 * Everything else, the workspace included, as for sqa_prefill_scores_ex.  The values are trusted: a wrong
 * normaliser gives wrong scores, not an error. */
sqa_status sqa_prefill_scores_lse(const void* Q, const void* K, const float* row_lse, sqa_dtype dt,
                                  int B, int Hq, int Hkv, int P, int D,
                                  float* scores_out, void* workspace, size_t ws_bytes, void* stream,
                                  const sqa_batch_opts* opts);

/* ---- Algorithm 1 steps 12 + 16-17: compress the prompt's KV to the budget --
 * Per unit keeps min(P, layer->budget) tokens chosen by the policy
 * (Sec. 2.2 / Sec. 5.1):
 *   SQA_SLIDING   the most recent tokens;
 *   SQA_STREAMING positions < n_sink plus the most recent (budget - n_sink);
 *   SQA_H2O       the (budget - floor(budget/2)) most recent plus, among the
 *                 older ones, the floor(budget/2) with the largest attn_scores,
 *                 equal scores -> lowest position first;
 * and gathers their K, V rows (ascending position) into the layer cache,
 * filling pos, score_acc (H2O) and unit_state (len, ring_head 0, evict_hint -2).
 *   K, V        : DEVICE [B][Hkv][P][D], dtype kv_dt; must not overlap the cache
 *   attn_scores : DEVICE float [B][Hkv][P], values >= 0, required for SQA_H2O
 *   layer       : HOST struct with DEVICE pointers; budget and capacity preset,
 *                 capacity >= min(P, budget)
 * SQA_ERR_BUDGET if budget < 1 (sliding), < n_sink+1 (streaming), < 2 (H2O).
 * SQA_ERR_CAPACITY if capacity < min(P, budget), or for SQA_H2O with budget > 65536 and P > budget (the
 * floor(budget/2) positions chosen by score are listed in LDS; prompts and the other policies' budgets
 * have no such limit). */
sqa_status sqa_prefill_compress(const void* K, const void* V, sqa_dtype kv_dt, const float* attn_scores,
                                int B, int Hkv, int P, int D, sqa_policy policy, int n_sink,
                                const sqa_layer_cache* layer, void* stream);

/* The same for n_layers layers in one launch per 32 layers (Algorithm 1's loop over i at step 12).
 *   K, V, attn_scores : HOST arrays [n_layers] of the DEVICE pointers sqa_prefill_compress takes
 *                       (attn_scores may be NULL unless the policy is SQA_H2O)
 *   layers            : HOST array [n_layers] */
sqa_status sqa_prefill_compress_layers(const void* const* K, const void* const* V, sqa_dtype kv_dt,
                                       const float* const* attn_scores, int B, int Hkv, int P, int D,
                                       sqa_policy policy, int n_sink, const sqa_layer_cache* layers, int n_layers,
                                       void* stream);
/* With opts->prompt_len / opts->budget_seq: unit (b, h) of layer l compresses
 * the first prompt_len[b] tokens to budget_seq[l][b] and needs min(prompt_len[b],
 * budget_seq[l][b]) slots (of layers[l].capacity, or of its own range with
 * unit_offset).  The host cannot see these values: a unit with too few slots is
 * left empty and SQA_ERR_CAPACITY is written to opts->status.  opts may be NULL. */
sqa_status sqa_prefill_compress_layers_ex(const void* const* K, const void* const* V, sqa_dtype kv_dt,
                                          const float* const* attn_scores, int B, int Hkv, int P, int D,
                                          sqa_policy policy, int n_sink, const sqa_layer_cache* layers, int n_layers,
                                          void* stream, const sqa_batch_opts* opts);

/* ---- Algorithm 1 steps 14-21 with Eq. 2-3: one decode step ----------------
 * For each of n_layers layers and each unit, in this order:
 *   1. append the new token's k, v (position new_pos, accumulated score 0);
 *   2. if the unit now holds budget+1 tokens, evict one by the policy (the
 *      token leaving the recent window, or for H2O the worse of that token and
 *      the lowest-scoring heavy hitter; equal scores evict the higher position);
 *   3. out[h] = softmax(q[h].K^T/sqrt(D)) V for the g query heads of the unit;
 *   4. H2O: score_acc[slot] += sum over those heads of the probability.
 * The cache (K, V, score_acc, pos, unit_state) is updated in
 * place; pos is the kept-index result.  Positions are consecutive: the prompt
 * holds 0..P-1 and every step's new_pos is the previous one plus 1.
 *   q            : DEVICE [n_layers][B][Hq][D], dtype dt
 *   k_new, v_new : DEVICE [n_layers][B][Hkv][D]
 *   out          : DEVICE [n_layers][B][Hq][D], dtype dt
 *   layers       : HOST array [n_layers] (read for validation and launch shape)
 *   layers_dev   : DEVICE copy of the same array, or NULL (then the call uploads
 *                  it into the workspace first)
 *   n_layers     : 1 when layers run one after another inside a model; all
 *                  layers at once when their inputs are known up front
 *   workspace    : DEVICE, 256-byte aligned, >= sqa_decode_workspace_bytes(...) for
 *                  the same layers and shapes, zero-filled once before its first
 *                  use (sqa_decode_workspace_init); calls that share a workspace
 *                  must not overlap in time.  Its first int32 is a device-side
 *                  status word (see sqa_read_device_status).
 * Long units are cut into chunks that separate workgroups stream (split-K);
 * the workspace holds their partial results, the step's logits (H2O) and one
 * arrival counter per unit; with 4 or more query heads per KV head (bf16,
 * D = 128) it also holds, for every unit, the step's per-head probabilities
 * that the H2O accumulation sums.  The merge order is fixed: results are
 * identical from run to run.
 * A unit that on entry is longer than its budget, or has no free slot, is left
 * untouched, its out rows are zeroed and the status word is set to
 * SQA_ERR_STATE / SQA_ERR_CAPACITY. */
size_t sqa_decode_workspace_bytes(const sqa_layer_cache* layers /*HOST*/, int n_layers, int B, int Hq, int Hkv,
                                  int D, sqa_policy policy);
sqa_status sqa_decode_workspace_init(void* workspace, size_t ws_bytes, void* stream);
sqa_status sqa_decode_step(const void* q, const void* k_new, const void* v_new, sqa_dtype dt,
                           int B, int Hq, int Hkv, int D, int32_t new_pos,
                           sqa_policy policy, int n_sink,
                           const sqa_layer_cache* layers, const sqa_layer_cache* layers_dev, int n_layers,
                           void* out, void* workspace, size_t ws_bytes, void* stream);

/* The same step with per-sequence positions and budgets and the choice of order
 * (opts may be NULL = sqa_decode_step).  Under SQA_ATTEND_THEN_EVICT steps 2-4
 * above run as 3, 4, 2: the unit attends all len+1 tokens, accumulates, and only
 * then evicts (H2O: by the scores just updated); evict_hint is not used and is
 * left at -2.  With new_pos_seq the scalar new_pos is ignored. */
sqa_status sqa_decode_step_ex(const void* q, const void* k_new, const void* v_new, sqa_dtype dt,
                              int B, int Hq, int Hkv, int D, int32_t new_pos,
                              sqa_policy policy, int n_sink,
                              const sqa_layer_cache* layers, const sqa_layer_cache* layers_dev, int n_layers,
                              void* out, void* workspace, size_t ws_bytes, void* stream,
                              const sqa_batch_opts* opts);

/* ---- the same step for callers that cannot allocate device memory ----------
 * (code running under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc).  Identical to sqa_decode_step_ex -- same kernels, same
 * results bit for bit -- except that the scratch a step needs (layer table,
 * arrival counters, partial results of split units, H2O logits / probabilities)
 * lives in a device array of SQA_STATIC_SCRATCH_BYTES that is part of the
 * library image; each GPU the library runs on holds its copy until the process
 * ends.  The call allocates nothing and frees nothing.
 *   status : DEVICE int32, caller-owned, 4-byte aligned: the device-side status
 *            word (the role a workspace's first word plays in sqa_decode_step);
 *            the caller zeroes and reads it
 *   every other argument as in sqa_decode_step_ex
 * A call whose scratch does not fit (more than 262144 units in the call, or
 * more than about 15 MiB of partial records plus H2O logits / probabilities)
 * returns SQA_ERR_CAPACITY and enqueues nothing: use sqa_decode_step with a
 * workspace for such shapes.
 * The first call on a device looks the array up and clears its counter region
 * (one small kernel and a wait on `stream`): make that call outside any graph
 * capture.  All calls on one GPU share the one array: calls that overlap in
 * time on the same GPU (different streams, different threads) race -- run
 * them one after the other. */
enum { SQA_STATIC_SCRATCH_BYTES = 16 * 1024 * 1024 };
sqa_status sqa_decode_step_static(const void* q, const void* k_new, const void* v_new, sqa_dtype dt,
                                  int B, int Hq, int Hkv, int D, int32_t new_pos,
                                  sqa_policy policy, int n_sink,
                                  const sqa_layer_cache* layers, const sqa_layer_cache* layers_dev, int n_layers,
                                  void* out, int32_t* status, void* stream, const sqa_batch_opts* opts);

/* ---- the launch a decode call would make (host arithmetic only, no GPU call) ----
 * How sqa_decode_step[_ex|_static] would lay the call out on the chip: for sizing, for logs, and so that the
 * launch configuration of a workload can be checked without a GPU.  Of `layers` only budget, capacity and
 * whether block_table is NULL are read.
 *   info      : HOST, filled in
 *   per_layer : HOST [n_layers] or NULL                                                                  */
typedef struct sqa_decode_plan_info {
  int64_t workgroups;       /* grid of the one launch, 256 threads each                                   */
  int64_t workspace_bytes;  /* what the call uses of its workspace (<= sqa_decode_workspace_bytes)        */
  int32_t lds_bytes;        /* dynamic LDS per workgroup                                                  */
  int32_t matrix_cores;     /* 1: the MFMA variant runs (bf16, D = 128, 4 or 8 query heads per KV head)   */
  int32_t wide_tail;        /* 1: so few workgroups that a long unit's score walk keeps all four waves    */
  int32_t table_entries;    /* blocked allocation: block numbers a workgroup stages in LDS (else 0)       */
} sqa_decode_plan_info;
typedef struct sqa_decode_layer_plan {
  int32_t workgroups_per_unit;  /* 1: a workgroup streams the whole unit; k > 1: the unit is cut into k work
                                   items whose partial results the last one to finish merges; 0: see next  */
  int32_t slots_per_workgroup;  /* length of such a work item in slots (a multiple of 64)                   */
  int32_t wave_per_unit;        /* 1: short units, many of them: each of a workgroup's 4 waves owns a unit  */
  int32_t probs_in_lds;         /* MFMA variant under H2O, the step's per-head probabilities of a unit: 1 = all
                                   stay in LDS, 2 = those of its leading tokens do (the rest passes through the
                                   workspace), 0 = none                                                      */
} sqa_decode_layer_plan;
sqa_status sqa_decode_plan(const sqa_layer_cache* layers, int n_layers, int B, int Hq, int Hkv, int D,
                           sqa_dtype dt, sqa_policy policy, sqa_decode_plan_info* info,
                           sqa_decode_layer_plan* per_layer);

/* Zeroes the status word (a small fill kernel enqueued on stream; like
 * sqa_decode_workspace_init it uses no memset, so both may be recorded into a HIP graph). */
sqa_status sqa_clear_device_status(void* workspace, void* stream);
/* Waits for `stream`, then copies the status word to *status_out (HOST). */
sqa_status sqa_read_device_status(const void* workspace, void* stream, int32_t* status_out);

/* ---- kept indices in ascending order (a view for callers and tests) -------
 * out[b][hkv][i] = i-th smallest position held by the unit, -1 for i >= len.
 *   out : DEVICE int32 [B][Hkv][layer->capacity]; with packed units (unit_offset)
 *         laid out like pos: unit u's entries start at out[unit_offset[u]] */
sqa_status sqa_kept_idx_sorted(const sqa_layer_cache* layer, int B, int Hkv, int32_t* out, void* stream);

/* ---- free list for blocked K/V allocation (host only) ----------------------
 * Book-keeping for the block numbers of ONE pool pair (the K and V pools of one layer share numbers, see
 * sqa_layer_cache.block_table): which of 0 .. n_blocks-1 are free.  The paper fixes a layer's budget once the
 * prompt is seen (Algorithm 1 step 11), so a unit takes ceil(min(capacity, budget) / SQA_BLOCK_SLOTS) blocks
 * when its sequence joins and gives them all back when it leaves; nothing is taken in between.  The pool
 * knows nothing of device memory: the caller writes the numbers it takes into its DEVICE block table.
 * HOST memory of the pool object belongs to the library (create / destroy); calls on one pool are serialised
 * by a mutex inside it.
 *   take: all n or nothing (SQA_ERR_CAPACITY, ids_out untouched); the lowest-numbered blocks that were
 *         never used go first, blocks given back are reused last-in first-out
 *   give: every id must be in range, in use and named once (else SQA_ERR_SHAPE and nothing changes)    */
typedef struct sqa_block_pool sqa_block_pool;
sqa_block_pool* sqa_block_pool_create(int32_t n_blocks);          /* NULL if n_blocks < 1 or out of memory */
void sqa_block_pool_destroy(sqa_block_pool* pool);               /* NULL is allowed                       */
int32_t sqa_block_pool_free_count(const sqa_block_pool* pool);   /* -1 for NULL                           */
sqa_status sqa_block_pool_take(sqa_block_pool* pool, int32_t n, int32_t* ids_out /* HOST [n] */);
sqa_status sqa_block_pool_give(sqa_block_pool* pool, const int32_t* ids /* HOST [n] */, int32_t n);

#ifdef __cplusplus
}
#endif
#endif /* SQA_H_ */
