// Prefill compression (Algorithm 1 steps 12 + 16-17 applied to the prompt) and
// the sorted kept-index view.  One workgroup per (sequence, KV head) unit:
//   select  sliding / streaming: index arithmetic on the position;
//           H2O: the floor(b/2) largest accumulated scores among the non-recent
//           tokens by an LDS radix select (4 passes of 8 bits over the fp32 bit
//           patterns, which order like the values because scores are >= 0);
//           tokens equal to the threshold are taken in ascending position by an
//           index-ordered prefix count -- never by arrival order;
//   compact an order-preserving prefix sum turns keep flags into slot numbers;
//   gather  the kept K and V rows are copied once (16 bytes per lane).
// HBM traffic per unit: P scores (H2O) + read and write of the kept rows.
#include "sqa_common.h"
#include <algorithm>

namespace sqa {

constexpr int kCmpThreads = 256;
constexpr int kCmpWaves = kCmpThreads / SQA_WAVE;
constexpr int kKeysInLdsMax = 16384;     // scores staged in LDS up to this many candidates

__device__ __forceinline__ uint32_t score_key(float s) {
  const uint32_t b = __float_as_uint(s);
  return (b & 0x80000000u) ? 0u : b;     // scores are >= 0; -0.0 and negatives order as 0
}

// exclusive prefix count of `flag` over the 256 threads (position order), and the total
__device__ __forceinline__ int block_excl_count(bool flag, int* s_wave_tot, int& total) {
  const int lane = threadIdx.x & (SQA_WAVE - 1), wave = threadIdx.x / SQA_WAVE;
  const unsigned long long bal = __ballot(flag);
  const int within = __popcll(bal & ((1ull << lane) - 1ull));
  __syncthreads();                        // previous users of s_wave_tot are done
  if (lane == 0) s_wave_tot[wave] = __popcll(bal);
  __syncthreads();
  int before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kCmpWaves; ++w) { const int t = s_wave_tot[w]; before += w < wave ? t : 0; tot += t; }
  total = tot;
  return before + within;
}

// inclusive prefix sum of v over the 256 threads
__device__ __forceinline__ int block_incl_sum(int v, int* s_wave_tot) {
  const int lane = threadIdx.x & (SQA_WAVE - 1), wave = threadIdx.x / SQA_WAVE;
  int x = v;
#pragma unroll
  for (int o = 1; o < SQA_WAVE; o <<= 1) {
    const int y = __shfl_up(x, o, SQA_WAVE);
    x += lane >= o ? y : 0;
  }
  __syncthreads();                        // previous users of s_wave_tot are done
  if (lane == SQA_WAVE - 1) s_wave_tot[wave] = x;
  __syncthreads();
  int before = 0;
#pragma unroll
  for (int w = 0; w < kCmpWaves; ++w) before += w < wave ? s_wave_tot[w] : 0;
  return before + x;
}

constexpr int kCmpBatch = 32;             // layers per launch (their descriptors travel as kernel arguments)
struct CompressBatch {
  sqa_layer_cache L[kCmpBatch];
  const void* K[kCmpBatch];
  const void* V[kCmpBatch];
  const float* scores[kCmpBatch];
  // per-sequence variation (all NULL for a uniform batch)
  const int32_t* prompt_len;    // [B]
  const int32_t* budget_seq;    // [n_layers][B]
  int32_t* status;
  int B, Hkv;
  uint8_t layer[kCmpBatch];     // which layer of the call a slot of this launch holds (row of budget_seq)
};
static_assert(SQA_MAX_LAYERS <= 256, "CompressBatch::layer holds a layer index in 8 bits");

template <typename T, int D>
__global__ __launch_bounds__(kCmpThreads) void prefill_compress_kernel(
    const CompressBatch batch, int P /*prompt rows per unit in memory*/, int policy, int n_sink, int lds_words /*dynamic LDS of the launch, in 32-bit words*/) {
  const sqa_layer_cache L = batch.L[blockIdx.y];
  const T* __restrict__ K = static_cast<const T*>(batch.K[blockIdx.y]);
  const T* __restrict__ V = static_cast<const T*>(batch.V[blockIdx.y]);
  const float* __restrict__ scores = batch.scores[blockIdx.y];
  constexpr int ROWB = D * (int)sizeof(T);
  constexpr int LPR = ROWB / 16;
  extern __shared__ uint32_t s_mem[];
  __shared__ int s_hist[256];
  __shared__ int s_wave_tot[kCmpWaves];
  __shared__ uint32_t s_sel[2];           // threshold key, how many equal keys to take

  const int tid = threadIdx.x;
  const int u = blockIdx.x;
  const int bidx = u / batch.Hkv;
  const int64_t uoff = L.unit_offset ? L.unit_offset[u] : (int64_t)u * L.capacity;   // the unit's first slot
  const int cap = L.unit_offset ? (int)(L.unit_offset[u + 1] - uoff) : L.capacity;
  const int P_pad = P;                                     // row pitch of the prompt tensors
  int b = L.budget;
  if (batch.prompt_len || batch.budget_seq) {
    if (batch.prompt_len) P = batch.prompt_len[bidx];
    if (batch.budget_seq) b = batch.budget_seq[(int64_t)batch.layer[blockIdx.y] * batch.B + bidx];
    const int min_budget = policy == SQA_H2O ? 2 : (policy == SQA_STREAMING ? n_sink + 1 : 1);
    const bool bad_len = P < 0 || P > P_pad, bad_budget = b < min_budget || b > L.budget;
    if (bad_len || bad_budget) {                           // leave the unit empty and say why
      if (tid == 0) {
        *reinterpret_cast<int4*>(L.unit_state + (int64_t)u * SQA_ST_WORDS) = make_int4(0, 0, -2, 0);
        if (batch.status) *batch.status = bad_len ? SQA_ERR_SHAPE : SQA_ERR_BUDGET;
      }
      return;
    }
  }
  int n_keep = P < b ? P : b;
  // blocked allocation: the unit's K and V rows lie in the 16-row blocks its table row names
  const int32_t* tbl = L.block_table ? L.block_table + (int64_t)u * L.blocks_per_unit : nullptr;
  if (tbl) {
    int bad = 0;
    const int nblk = (min(n_keep, cap) + SQA_BLOCK_SLOTS - 1) / SQA_BLOCK_SLOTS;
    for (int i = tid; i < nblk; i += kCmpThreads) bad |= (unsigned)tbl[i] >= (unsigned)L.n_blocks;
    if (__syncthreads_or(bad)) {                           // a block number outside the pools: touch nothing
      if (tid == 0) {
        *reinterpret_cast<int4*>(L.unit_state + (int64_t)u * SQA_ST_WORDS) = make_int4(0, 0, -2, 0);
        if (batch.status) *batch.status = SQA_ERR_SHAPE;
      }
      return;
    }
  }
  if (n_keep > cap) {                                      // packed units: this one was given too few slots
    if (tid == 0) {
      *reinterpret_cast<int4*>(L.unit_state + (int64_t)u * SQA_ST_WORDS) = make_int4(0, 0, -2, 0);
      if (batch.status) *batch.status = SQA_ERR_CAPACITY;
    }
    return;
  }
  const float* sc = scores ? scores + (int64_t)u * P_pad : nullptr;

  // range rules
  int lo_keep = 0;        // positions < lo_keep are always kept (sinks)
  int hi_from = 0;        // positions >= hi_from are always kept (recent window / everything)
  int hh = 0;             // how many of [lo_keep, hi_from) to take by score
  if (P > b) {
    if (policy == SQA_SLIDING) { hi_from = P - b; }
    else if (policy == SQA_STREAMING) { lo_keep = n_sink < b ? n_sink : b; hi_from = P - (b - lo_keep); }
    else { hh = b / 2; hi_from = P - (b - hh); }
  }
  const int M = hi_from;  // H2O candidates are positions [0, M)
  // The kept tokens in position order are: the positions below lo_keep, then the hh candidates chosen by
  // score, then everything from hi_from on.  Only the middle part needs a list (in LDS); the other two
  // are index arithmetic, so a unit's length is not limited by LDS (an uncompressed or sliding-window
  // cache of any length; H2O budgets up to 65536).
  int* s_idx = reinterpret_cast<int*>(s_mem);              // [hh] positions chosen by score, ascending
  uint32_t* s_keys = s_mem + hh;                           // [M] when staged
  const bool keys_in_lds = hh > 0 && M <= kKeysInLdsMax && hh + M <= lds_words;

  uint32_t thr = 0xffffffffu, take_eq = 0;
  if (hh > 0) {
    const uint32_t* keys;
    if (keys_in_lds) {
      for (int i = tid; i < M; i += kCmpThreads) s_keys[i] = score_key(sc[i]);
      keys = s_keys;
    } else {
      keys = nullptr;
    }
    uint32_t prefix = 0, mask = 0;
    int k = hh;
    for (int pass = 3; pass >= 0; --pass) {
      s_hist[tid] = 0;
      __syncthreads();
      const int sh = pass * 8;
      for (int i = tid; i < M; i += kCmpThreads) {
        const uint32_t key = keys ? keys[i] : score_key(sc[i]);
        if ((key & mask) == prefix) atomicAdd(&s_hist[(key >> sh) & 255u], 1);
      }
      __syncthreads();
      // the digit of the k-th largest key: thread t looks at bin 255 - t; the sum over the bins above and
      // including its own reaches k in exactly one non-empty bin (at least k keys carry the prefix)
      static_assert(kCmpThreads == 256, "one thread per histogram bin");
      const int h = s_hist[255 - tid];
      const int incl = block_incl_sum(h, s_wave_tot);
      if (incl >= k && incl - h < k) { s_sel[0] = (uint32_t)(255 - tid); s_sel[1] = (uint32_t)(k - (incl - h)); }
      __syncthreads();
      prefix |= s_sel[0] << sh; mask |= 255u << sh; k = (int)s_sel[1];
      __syncthreads();
    }
    thr = prefix; take_eq = (uint32_t)k;
  }

  // keep flags of the candidates -> their order among the chosen, in position order, 256 positions at a time
  if (hh > 0) {
    int eq_seen = 0, kept_seen = 0;
    for (int base = 0; base < M; base += kCmpThreads) {
      const int i = base + tid;
      const bool cand = i < M;
      const uint32_t key = cand ? (keys_in_lds ? s_keys[i] : score_key(sc[i])) : 0u;
      const bool eq = cand && key == thr;
      int eq_tot;
      const int eq_rank = eq_seen + block_excl_count(eq, s_wave_tot, eq_tot);
      eq_seen += eq_tot;
      const bool keep = cand && (key > thr || (eq && (uint32_t)eq_rank < take_eq));
      int kept_tot;
      const int slot = kept_seen + block_excl_count(keep, s_wave_tot, kept_tot);
      kept_seen += kept_tot;
      if (keep) s_idx[slot] = i;
    }
    __syncthreads();
  }
  // position of the token that goes to slot j
  auto source = [&](int j) { return j < lo_keep ? j : (j < lo_keep + hh ? s_idx[j - lo_keep] : hi_from + (j - lo_keep - hh)); };

  // gather rows, scores, positions
  const T* Ku = K + (int64_t)u * P_pad * D;
  const T* Vu = V + (int64_t)u * P_pad * D;
  char* Kc = reinterpret_cast<char*>(L.K) + (tbl ? 0 : uoff * ROWB);
  char* Vc = reinterpret_cast<char*>(L.V) + (tbl ? 0 : uoff * ROWB);
  // row of the unit's slot j within Kc / Vc
  auto row_of = [&](int j) -> int64_t { return tbl ? (int64_t)tbl[j / SQA_BLOCK_SLOTS] * SQA_BLOCK_SLOTS + j % SQA_BLOCK_SLOTS : (int64_t)j; };
  const int grp = tid / LPR, c = tid % LPR;
  constexpr int GROUPS = kCmpThreads / LPR;
  for (int j = grp; j < n_keep; j += 2 * GROUPS) {
    const int j2 = j + GROUPS;
    const int src = source(j);
    const int src2 = j2 < n_keep ? source(j2) : src;
    const uint4 k1 = ld16(reinterpret_cast<const char*>(Ku) + (int64_t)src * ROWB + c * 16);
    const uint4 v1 = ld16(reinterpret_cast<const char*>(Vu) + (int64_t)src * ROWB + c * 16);
    const uint4 k2 = ld16(reinterpret_cast<const char*>(Ku) + (int64_t)src2 * ROWB + c * 16);
    const uint4 v2 = ld16(reinterpret_cast<const char*>(Vu) + (int64_t)src2 * ROWB + c * 16);
    const int64_t d1 = row_of(j);
    st16(Kc + d1 * ROWB + c * 16, k1);
    st16(Vc + d1 * ROWB + c * 16, v1);
    if (j2 < n_keep) {
      const int64_t d2 = row_of(j2);
      st16(Kc + d2 * ROWB + c * 16, k2);
      st16(Vc + d2 * ROWB + c * 16, v2);
    }
  }
  int32_t* posu = L.pos + uoff;
  for (int j = tid; j < n_keep; j += kCmpThreads) {
    const int src = source(j);
    posu[j] = src;
    if (L.score_acc) L.score_acc[uoff + j] = sc ? sc[src] : 0.f;
  }
  if (tid == 0) *reinterpret_cast<int4*>(L.unit_state + (int64_t)u * SQA_ST_WORDS) = make_int4(n_keep, 0, -2, 0);
}

// out[rank of pos[i]] = pos[i]; -1 beyond len.  Rank by counting (a test view, O(n^2)).
__global__ __launch_bounds__(kCmpThreads) void kept_idx_sorted_kernel(sqa_layer_cache L, int32_t* __restrict__ out, int use_lds) {
  extern __shared__ uint32_t s_mem[];
  int* s_pos = reinterpret_cast<int*>(s_mem);
  const int u = blockIdx.x;
  const int64_t uoff = L.unit_offset ? L.unit_offset[u] : (int64_t)u * L.capacity;
  const int cap = L.unit_offset ? (int)(L.unit_offset[u + 1] - uoff) : L.capacity;
  int len = L.unit_state[(int64_t)u * SQA_ST_WORDS + SQA_ST_LEN];
  len = len < 0 ? 0 : (len > cap ? cap : len);
  const int32_t* posu = L.pos + uoff;
  int32_t* o = out + uoff;
  for (int i = len + threadIdx.x; i < cap; i += kCmpThreads) o[i] = -1;
  if (use_lds) {
    for (int i = threadIdx.x; i < len; i += kCmpThreads) s_pos[i] = posu[i];
    __syncthreads();
  }
  // (units too long for LDS are ranked from memory: the same count, slower)
  const int32_t* src = use_lds ? s_pos : posu;
  for (int i = threadIdx.x; i < len; i += kCmpThreads) {
    const int p = src[i];
    int rank = 0;
    for (int j = 0; j < len; ++j) rank += (src[j] < p) || (src[j] == p && j < i);
    o[rank] = p;
  }
}

template <typename T, int D>
static hipError_t launch_compress(const CompressBatch& batch, int n, int P, int policy, int n_sink,
                                   unsigned units, size_t lds, hipStream_t st) {
  auto fn = prefill_compress_kernel<T, D>;
  if (lds > 48 * 1024) {
    const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(fn), lds);
    if (e != hipSuccess) return e;
  }
  fn<<<dim3(units, n), kCmpThreads, lds, st>>>(batch, P, policy, n_sink, (int)(lds / sizeof(uint32_t)));
  return hipGetLastError();
}

static sqa_status check_compress_layer(const void* K, const void* V, sqa_dtype kv_dt, const float* attn_scores,
                                       int B, int Hkv, int P, int D, sqa_policy policy, int n_sink,
                                       const sqa_layer_cache& L, bool ragged, size_t* lds_out) {
  if (!K || !V) return SQA_ERR_NULL;
  if (policy == SQA_H2O && !attn_scores) return SQA_ERR_NULL;
  if (!L.K || !L.V || !L.pos || !L.unit_state) return SQA_ERR_NULL;
  if (policy == SQA_H2O && !L.score_acc) return SQA_ERR_NULL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(L.K) || !aligned16(L.V) || !aligned16(L.unit_state)) return SQA_ERR_SHAPE;
  const int min_budget = policy == SQA_H2O ? 2 : (policy == SQA_STREAMING ? n_sink + 1 : 1);
  if (L.budget < min_budget) return SQA_ERR_BUDGET;
  // (with per-sequence lengths or budgets a unit needs min(its prompt length, its budget) slots, which only
  // the kernel can see: it leaves a unit that has too few empty and reports SQA_ERR_CAPACITY through opts->status)
  const int n_keep = P < L.budget ? P : L.budget;
  if (ragged ? L.capacity < 1 : L.capacity < n_keep) return SQA_ERR_CAPACITY;
  if (L.block_table) {                                     // blocked allocation of K and V
    if (L.unit_offset || L.n_blocks < 1 || L.blocks_per_unit > SQA_MAX_BLOCKS_PER_UNIT ||
        (int64_t)L.blocks_per_unit * SQA_BLOCK_SLOTS < (L.budget < L.capacity ? L.budget : L.capacity))
      return SQA_ERR_SHAPE;
  }
  // the prompt tensors must not overlap the cache they are gathered into (checked where the host knows the
  // cache's extent: packed units end at unit_offset[B*Hkv], which lies in device memory)
  const size_t eb = kv_dt == SQA_F32 ? 4 : 2;
  const size_t in_bytes = (size_t)B * Hkv * P * D * eb;
  const size_t c_bytes = (L.block_table ? (size_t)L.n_blocks * SQA_BLOCK_SLOTS : (size_t)B * Hkv * L.capacity) * D * eb;
  auto overlaps = [](const void* a, size_t na, const void* b, size_t nb) {
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + nb && y < x + na;
  };
  if (!L.unit_offset && (overlaps(K, in_bytes, L.K, c_bytes) || overlaps(K, in_bytes, L.V, c_bytes) ||
                         overlaps(V, in_bytes, L.K, c_bytes) || overlaps(V, in_bytes, L.V, c_bytes))) return SQA_ERR_SHAPE;
  // H2O candidates of a unit: at most P - (b - b/2) with the layer's budget, up to P - 1 with a smaller
  // per-sequence budget; their keys are staged in LDS when they fit
  const bool h2o_select = policy == SQA_H2O && (ragged ? P > 2 : P > L.budget);
  const int M = h2o_select ? (ragged ? P - 1 : P - (L.budget - L.budget / 2)) : 0;
  // (the list of positions chosen by score: at most floor(budget / 2) entries)
  const size_t hh_max = policy == SQA_H2O ? (size_t)(L.budget / 2) : 0;
  *lds_out = (hh_max + (M <= kKeysInLdsMax ? (size_t)M : 0)) * sizeof(uint32_t);
  return SQA_OK;
}

}  // namespace sqa

extern "C" sqa_status sqa_prefill_compress_layers(const void* const* K, const void* const* V, sqa_dtype kv_dt,
                                                  const float* const* attn_scores, int B, int Hkv, int P, int D,
                                                  sqa_policy policy, int n_sink, const sqa_layer_cache* layers,
                                                  int n_layers, void* stream) {
  return sqa_prefill_compress_layers_ex(K, V, kv_dt, attn_scores, B, Hkv, P, D, policy, n_sink, layers, n_layers, stream,
                                        nullptr);
}

extern "C" sqa_status sqa_prefill_compress_layers_ex(const void* const* K, const void* const* V, sqa_dtype kv_dt,
                                                     const float* const* attn_scores, int B, int Hkv, int P, int D,
                                                     sqa_policy policy, int n_sink, const sqa_layer_cache* layers,
                                                     int n_layers, void* stream, const sqa_batch_opts* opts) {
  using namespace sqa;
  const bool ragged = opts && (opts->prompt_len || opts->budget_seq);
  if (!K || !V || !layers) return SQA_ERR_NULL;
  if (kv_dt != SQA_F32 && kv_dt != SQA_BF16) return SQA_ERR_DTYPE;
  if (policy != SQA_SLIDING && policy != SQA_STREAMING && policy != SQA_H2O) return SQA_ERR_POLICY;
  if (n_sink < 0) return SQA_ERR_POLICY;
  if (B < 1 || Hkv < 1 || P < 1 || (D != 64 && D != 128) || (int64_t)B * Hkv > INT32_MAX || n_layers < 1 ||
      n_layers > SQA_MAX_LAYERS)
    return SQA_ERR_SHAPE;
  if (policy == SQA_H2O && !attn_scores) return SQA_ERR_NULL;
  size_t lds_layer[SQA_MAX_LAYERS];
  for (int i = 0; i < n_layers; ++i) {
    const sqa_status st = check_compress_layer(K[i], V[i], kv_dt, attn_scores ? attn_scores[i] : nullptr, B, Hkv, P, D,
                                               policy, n_sink, layers[i], ragged, &lds_layer[i]);
    if (st != SQA_OK) return st;
    if (lds_layer[i] > 128 * 1024) return SQA_ERR_CAPACITY;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const unsigned units = (unsigned)(B * Hkv);
  for (int l0 = 0; l0 < n_layers; l0 += kCmpBatch) {
    const int n = n_layers - l0 < kCmpBatch ? n_layers - l0 : kCmpBatch;
    CompressBatch batch;
    batch.prompt_len = opts ? opts->prompt_len : nullptr;
    batch.budget_seq = opts ? opts->budget_seq : nullptr;
    batch.status = opts ? opts->status : nullptr;
    batch.B = B; batch.Hkv = Hkv;
    // The layers that keep the most rows go first: their workgroups copy for the whole launch, and started last
    // they would finish it alone with most of the chip idle (7B shape: 0.77 -> 0.72 ms for the 32 layers).
    int order[kCmpBatch];
    for (int i = 0; i < n; ++i) order[i] = l0 + i;
    std::stable_sort(order, order + n, [&](int x, int y) { return layers[x].budget > layers[y].budget; });
    size_t lds = 0;
    for (int i = 0; i < n; ++i) {
      const int l = order[i];
      batch.L[i] = layers[l];
      batch.K[i] = K[l];
      batch.V[i] = V[l];
      batch.scores[i] = policy == SQA_H2O ? attn_scores[l] : nullptr;
      batch.layer[i] = (uint8_t)l;
      lds = lds_layer[l] > lds ? lds_layer[l] : lds;
    }
    for (int i = n; i < kCmpBatch; ++i) { batch.L[i] = layers[l0]; batch.K[i] = nullptr; batch.V[i] = nullptr; batch.scores[i] = nullptr; batch.layer[i] = 0; }
    hipError_t e;
    if (kv_dt == SQA_F32) {
      if (D == 64) e = launch_compress<float, 64>(batch, n, P, policy, n_sink, units, lds, st);
      else e = launch_compress<float, 128>(batch, n, P, policy, n_sink, units, lds, st);
    } else {
      if (D == 64) e = launch_compress<bf16_t, 64>(batch, n, P, policy, n_sink, units, lds, st);
      else e = launch_compress<bf16_t, 128>(batch, n, P, policy, n_sink, units, lds, st);
    }
    SQA_HIP_CHECK(e);
  }
  return SQA_OK;
}

extern "C" sqa_status sqa_prefill_compress(const void* K, const void* V, sqa_dtype kv_dt, const float* attn_scores,
                                           int B, int Hkv, int P, int D, sqa_policy policy, int n_sink,
                                           const sqa_layer_cache* layer, void* stream) {
  if (!K || !V || !layer) return SQA_ERR_NULL;
  const void* Ks[1] = {K};
  const void* Vs[1] = {V};
  const float* Ss[1] = {attn_scores};
  return sqa_prefill_compress_layers(Ks, Vs, kv_dt, attn_scores ? Ss : nullptr, B, Hkv, P, D, policy, n_sink, layer, 1,
                                     stream);
}

extern "C" sqa_status sqa_kept_idx_sorted(const sqa_layer_cache* layer, int B, int Hkv, int32_t* out, void* stream) {
  using namespace sqa;
  if (!layer || !out || !layer->pos || !layer->unit_state) return SQA_ERR_NULL;
  if (B < 1 || Hkv < 1 || (int64_t)B * Hkv > INT32_MAX) return SQA_ERR_SHAPE;
  if (layer->capacity < 1) return SQA_ERR_CAPACITY;
  size_t lds = (size_t)layer->capacity * sizeof(int32_t);
  const int use_lds = lds <= 128 * 1024;
  if (!use_lds) lds = 0;
  if (lds > 48 * 1024)
    SQA_HIP_CHECK(allow_dynamic_lds(reinterpret_cast<const void*>(kept_idx_sorted_kernel), lds));
  kept_idx_sorted_kernel<<<(unsigned)(B * Hkv), kCmpThreads, lds, static_cast<hipStream_t>(stream)>>>(*layer, out, use_lds);
  SQA_HIP_CHECK(hipGetLastError());
  return SQA_OK;
}
