// Decode step over per-layer compact KV caches: Algorithm 1 steps 14-21 with the
// append of Eq. 2-3.  One launch covers every (layer, sequence, KV head) unit of
// the call.  A unit's tokens are cut into chunks of `chunk` slots; a workgroup
// of 4 waves owns one chunk:
//   0. read len / ring head / the eviction decision carried over from the
//      previous step (H2O: which heavy slot, if any, the ring leaver replaces);
//   1. stream the chunk's K and V rows once with non-temporal 16-byte loads
//      (1 KiB per wave load), online softmax in fp32;
//   2. combine the 4 waves.  Unit with one chunk: write out[g][D].  Split unit:
//      write the partial (acc, m, l) and the logits to scratch, bump the unit's
//      arrival counter; the workgroup that arrives last merges the partials in
//      chunk order (fixed order: results do not depend on who arrives last);
//   3. H2O: score_acc += softmax probabilities (summed over the g query heads),
//      one read and one write of the score per token, and in the same pass the
//      NEXT step's eviction decision (arg-min over the updated heavy scores
//      against the next ring leaver), stored in evict_hint;
//   4. only now touch the cache: move the surviving ring token into the evicted
//      heavy slot, write the new token's rows, pos, lens, ring_head.
// During 1 the two slots that 4 will rewrite are read through a remap (new
// token from k_new/v_new, moved token from its old ring slot), so the cache is
// read-only until every workgroup of the unit has finished reading.  HBM
// traffic per unit is the kept rows of K and V once plus 8 bytes of score per
// token under H2O (split units add 8 bytes of logit scratch per token and
// head).  The only atomic is the arrival counter; it decides who merges, never
// what is computed: results are bit-identical from run to run.
// Short units (at most kWpuMaxSlots slots, when the call has enough of them)
// are not shared by the 4 waves: each wave of the workgroup owns a unit of its
// own and runs steps 0-4 alone, without a barrier.  A 4-wave pass over 64 rows
// leaves most lanes idle on such a unit and ends in a merge that costs as much
// as the streaming; one wave walks it 16 rows at a time with nothing to merge.
#include "sqa_common.h"

namespace sqa {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / SQA_WAVE;
constexpr int kUnroll = 4;                  // rows per lane group in flight per loop trip

struct DecodeArgs {
  const void* q;
  const void* k_new;
  const void* v_new;
  void* out;
  const sqa_layer_cache* layers;   // DEVICE table
  int32_t* status;
  int32_t* cnt;                    // scratch: arrival counter per unit (zero between launches)
  float* part;                     // scratch: per-chunk partial (acc[D], m, l) of split units
  float* logit;                    // scratch: logits of split units (H2O)
  const int32_t* new_pos_seq;      // DEVICE [B] or NULL: per-sequence position, < 0 = sequence sits this step out
  const int32_t* budget_seq;       // DEVICE [n_layers][B] or NULL: per-sequence budgets
  int B, Hq, Hkv, n_layers;
  int new_pos, policy, n_sink;
  int ae;                          // 1 = attend over all len+1 tokens first, evict afterwards
  float scale_log2;                // log2(e) / sqrt(D)
  uint8_t order[SQA_MAX_LAYERS];       // layers in descending budget (long units start first)
  uint32_t blk_end[SQA_MAX_LAYERS];    // work items up to and including ordered layer i
  int lds_chunk;                       // row length of the LDS logit buffer
  // Per-layer launch plan.  All fields are 32-bit on purpose: with a 16-bit
  // table next to a 32-bit one, hipcc 7.2 folded the two uniform indices into
  // one scalar load whose base address was only 2-byte aligned, and scalar
  // loads drop the low address bits of the base (the wrong entry was read).
  struct Layer {
    uint32_t nsplit;      // chunks per unit, with the tile count and the flag described below the struct
    uint32_t chunk;       // slots per chunk
    uint32_t unit_off;    // first unit number of the layer within the call
    uint32_t part_off;    // first partial record
    uint32_t logit_off;   // first logit (floats)
  } lay[SQA_MAX_LAYERS];
  int lds_chunk_w;                     // row length of a wave's LDS logit buffer in one-wave-per-unit layers
  int wide_tail;                       // the call has few workgroups: a long unit's tail keeps all four waves
  int lds_probs_w;                     // bytes of a wave's own LDS region for those probabilities in one-wave-per-unit layers
  int tbl_off;                         // blocked allocation: where in the dynamic LDS the unit's block numbers are staged (bytes)
};
// Layer::nsplit: bits 0-15 the number of work items per unit, bits 16-29 how many of a unit's leading 32-token
// tiles keep their H2O probabilities in LDS (matrix-core variant), bit 31 one wave per unit
constexpr uint32_t kWpuBit = 0x80000000u;
constexpr int kLdsTilesShift = 16;
constexpr uint32_t kLdsTilesMask = 0x3fffu;

// Data that one workgroup hands to another inside a launch (partial results,
// logits) moves through agent-scope relaxed atomics: such stores are written
// through and such loads read the coherent copy, so the hand-over needs no
// cache write-back or invalidate (each XCD of the chip has an L2 of its own;
// a device-scope fence would flush it, which costs far more than the data).
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(unsigned long long* p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(unsigned short* p, unsigned short v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned short ld_agent(const unsigned short* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// block-wide reductions; every thread gets the result
// solo: only wave 0 of the workgroup is still running (the others have left),
// so the reduction stays inside the wave and no barrier may be used.
__device__ __forceinline__ float block_min(float v, float* s_red, bool solo) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, SQA_WAVE));
  if (solo) return v;
  __syncthreads();
  if ((threadIdx.x & (SQA_WAVE - 1)) == 0) s_red[threadIdx.x / SQA_WAVE] = v;
  __syncthreads();
  v = s_red[0];
#pragma unroll
  for (int w = 1; w < kDecWaves; ++w) v = fminf(v, s_red[w]);
  return v;
}
__device__ __forceinline__ unsigned long long block_max64(unsigned long long v, unsigned long long* s_red, bool solo) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned long long other = __shfl_xor(v, o, SQA_WAVE);
    v = other > v ? other : v;
  }
  if (solo) return v;
  __syncthreads();
  if ((threadIdx.x & (SQA_WAVE - 1)) == 0) s_red[threadIdx.x / SQA_WAVE] = v;
  __syncthreads();
  v = s_red[0];
#pragma unroll
  for (int w = 1; w < kDecWaves; ++w) v = s_red[w] > v ? s_red[w] : v;
  return v;
}

// H2O eviction rule for a full unit: the candidates are the hh heavy slots and
// the token leaving the recent ring; the one with the lowest accumulated score
// goes, equal scores -> the highest position (the ring leaver is newer than
// every heavy hitter).  Returns -1 if the leaver is evicted, else the heavy
// slot that is evicted (the leaver moves there).  `mn` = min over the heavy
// scores, already reduced over the block.  pos_override: slot whose position
// is not yet in memory (or -1).
__device__ __forceinline__ int pick_victim(const float* sc, const int32_t* posu, int hh, float mn, float leaver_score,
                                           int override_slot, int override_pos, unsigned long long* s_red64,
                                           bool solo, int t /*thread index among the nthr threads at work*/) {
  if (leaver_score <= mn) return -1;             // uniform over the block
  unsigned long long best = 0ull;                // (position + 1) << 32 | slot
  const int nthr = solo ? SQA_WAVE : kDecThreads;
  for (int i = t; i < hh; i += nthr)
    if (sc[i] == mn) {
      const int ps = i == override_slot ? override_pos : posu[i];
      const unsigned long long key = ((unsigned long long)(uint32_t)(ps + 1) << 32) | (uint32_t)i;
      best = key > best ? key : best;
    }
  return (int)(uint32_t)block_max64(best, s_red64, solo);
}

// v_exp_f32: 2^x, 1 ulp, denormal results flush to 0 (harmless in a softmax)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int CTRL> __device__ __forceinline__ float dpp_mov(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// sum over the LPR consecutive lanes that share a row; every lane gets the sum
template <int LPR> __device__ __forceinline__ float group_sum(float v) {
  static_assert(sizeof(DecodeArgs) <= 4096, "kernel arguments are limited to 4 KiB");
  static_assert(LPR == 8 || LPR == 16 || LPR == 32, "lanes per row");
  v += dpp_mov<0xB1>(v);            // quad_perm [1,0,3,2]
  v += dpp_mov<0x4E>(v);            // quad_perm [2,3,0,1]
  v += dpp_mov<0x141>(v);           // row_half_mirror
  if (LPR >= 16) v += dpp_mov<0x140>(v);   // row_mirror
  if (LPR >= 32) v += __shfl_xor(v, 16, SQA_WAVE);
  return v;
}

template <typename T> struct RowMath;
template <> struct RowMath<float> {
  static constexpr int EPL = 4;
  static __device__ __forceinline__ float dot(const uint4& q, const uint4& k) {
    float s = __uint_as_float(q.x) * __uint_as_float(k.x);
    s = fmaf(__uint_as_float(q.y), __uint_as_float(k.y), s);
    s = fmaf(__uint_as_float(q.z), __uint_as_float(k.z), s);
    s = fmaf(__uint_as_float(q.w), __uint_as_float(k.w), s);
    return s;
  }
  static __device__ __forceinline__ void axpy(float p, const uint4& v, float* acc) {
    acc[0] = fmaf(p, __uint_as_float(v.x), acc[0]); acc[1] = fmaf(p, __uint_as_float(v.y), acc[1]);
    acc[2] = fmaf(p, __uint_as_float(v.z), acc[2]); acc[3] = fmaf(p, __uint_as_float(v.w), acc[3]);
  }
  static __device__ __forceinline__ void store(void* dst, const float* a) {
    st16(dst, make_uint4(__float_as_uint(a[0]), __float_as_uint(a[1]), __float_as_uint(a[2]), __float_as_uint(a[3])));
  }
};
template <> struct RowMath<bf16_t> {
  static constexpr int EPL = 8;
  static __device__ __forceinline__ float dot(const uint4& q, const uint4& k) {
    float s = dot2_bf16(q.x, k.x, 0.f);
    s = dot2_bf16(q.y, k.y, s); s = dot2_bf16(q.z, k.z, s); s = dot2_bf16(q.w, k.w, s);
    return s;
  }
  static __device__ __forceinline__ void axpy(float p, const uint4& v, float* acc) {
    acc[0] = fmaf(p, bf16_lo(v.x), acc[0]); acc[1] = fmaf(p, bf16_hi(v.x), acc[1]);
    acc[2] = fmaf(p, bf16_lo(v.y), acc[2]); acc[3] = fmaf(p, bf16_hi(v.y), acc[3]);
    acc[4] = fmaf(p, bf16_lo(v.z), acc[4]); acc[5] = fmaf(p, bf16_hi(v.z), acc[5]);
    acc[6] = fmaf(p, bf16_lo(v.w), acc[6]); acc[7] = fmaf(p, bf16_hi(v.w), acc[7]);
  }
  static __device__ __forceinline__ void store(void* dst, const float* a) {
    uint4 o;
    o.x = f32_to_bf16_bits(a[0]) | (f32_to_bf16_bits(a[1]) << 16);
    o.y = f32_to_bf16_bits(a[2]) | (f32_to_bf16_bits(a[3]) << 16);
    o.z = f32_to_bf16_bits(a[4]) | (f32_to_bf16_bits(a[5]) << 16);
    o.w = f32_to_bf16_bits(a[6]) | (f32_to_bf16_bits(a[7]) << 16);
    st16(dst, o);
  }
};


typedef __attribute__((address_space(1))) const void dec_gptr_t;
typedef __attribute__((address_space(3))) void dec_lptr_t;
constexpr int kMfWavesPerSimd = 3;                // waves per SIMD the matrix-core variant is compiled for
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef short v4s_t __attribute__((ext_vector_type(4)));
typedef short v8s_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4s_t* lds_v4s_ptr;
constexpr int kWpuMaxSlots = 256;                 // one wave per unit: for units of at most this many slots
constexpr int kSoloMaxTokens = 512;               // calls with few workgroups: an unsplit unit's tail (scores, decision) is left
                                                  // to wave 0 alone up to this length
constexpr int kLogitPad = 33;                     // a unit's H2O scratch region: G x (slots + kLogitPad) floats: the logit of the
                                                  // new token as one more slot, or whole 32-token tiles of bf16 probabilities
                                                  // plus a reference per tile and head
constexpr int kStageRow = 256 + 16;               // LDS row pitch of a staged bf16 D=128 row (padded: no bank conflicts)
constexpr int kStageBytesPerWave = 32 * kStageRow;   // one 32-token tile

// MF = true (bf16, D = 128, grouped queries): the chunk is streamed in 32-token
// tiles through LDS and q.K^T / P.V run on the matrix cores, see section 1M.
// PG = true: blocked allocation -- the unit's K and V rows lie in 16-row blocks of the layer's pools, named by
// its row of the block table (staged in LDS at the start); everything else is addressed as before.
template <typename T, int D, int G, bool H2O, bool MF, bool PG>
__global__ __launch_bounds__(kDecThreads, MF ? kMfWavesPerSimd : 1) void decode_unit_kernel(const DecodeArgs a) {
  static_assert(!MF || (sizeof(T) == 2 && D == 128 && G <= 16), "matrix-core path: bf16, D = 128");
  constexpr int U = kUnroll;
  constexpr int ROWB = D * (int)sizeof(T);        // bytes per K or V row
  constexpr int LPR = ROWB / 16;                  // lanes per row
  constexpr int RPI = SQA_WAVE / LPR;             // rows per wave load
  constexpr int EPL = RowMath<T>::EPL;            // elements per lane
  constexpr int PREC = D + 2;                     // floats per partial record: acc[D], m, l

  extern __shared__ __align__(256) float s_logit[];   // H2O, unsplit units: [G][lds_chunk]; matrix-core variant: stage buffers (16-byte LDS accesses)
  __shared__ float s_m[kDecWaves][G], s_l[kDecWaves][G];
  // per-wave output accumulators for the merge of a unit's waves; the matrix-core variant puts them where
  // its tiles were staged (a wave's 8.5 KiB stage buffer is free once its last tile is consumed), which leaves
  // the LDS of a CU to three workgroups AND a unit's probabilities (below)
  __shared__ float s_acc_static[MF ? 1 : kDecWaves][MF ? 1 : G][D];
  __shared__ float s_red[kDecWaves];
  __shared__ unsigned long long s_red64[kDecWaves];
  __shared__ int s_ctl[2];
  __shared__ float s_ctlf[kDecWaves][2];

  char* const stage_base = reinterpret_cast<char*>(s_logit + (H2O ? G * a.lds_chunk : 0));     // (matrix-core variant)
  float* const acc_lds = MF ? reinterpret_cast<float*>(stage_base) : &s_acc_static[0][0][0];
  constexpr int kAccWave = MF ? kStageBytesPerWave / 4 : G * D;                               // floats between waves
  static_assert(!MF || G * D * 4 <= kStageBytesPerWave, "a wave's accumulators fit in its stage buffer");
  const int tid = threadIdx.x, lane = tid & (SQA_WAVE - 1);
  // (the wave number is the same in all lanes: say so, or everything derived from it -- the unit a wave
  // owns, its pointers, its length -- lands in vector registers and is loaded with vector loads)
  const int wave = __builtin_amdgcn_readfirstlane(tid / SQA_WAVE);
  const int r = lane / LPR, c = lane % LPR;

  // ---- which work item -----------------------------------------------------
  int lo = 0, hi = a.n_layers - 1;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (blockIdx.x < a.blk_end[mid]) hi = mid; else lo = mid + 1;
  }
  const int layer = a.order[lo];
  const unsigned local = blockIdx.x - (lo ? a.blk_end[lo - 1] : 0u);
  const uint32_t nsplit_w = a.lay[layer].nsplit;
  const int nsplit = (int)(nsplit_w & 0xffffu);
  // one wave per unit: the workgroup's waves own 4 consecutive units and never meet at a barrier
  const bool wpu = (nsplit_w & kWpuBit) != 0;
  const int u = wpu ? (int)local * kDecWaves + wave : (int)(local / (unsigned)nsplit);
  const int chunk = wpu ? 0 : (int)(local % (unsigned)nsplit);
  if (wpu && u >= a.B * a.Hkv) return;
  const int nw = wpu ? 1 : kDecWaves;             // waves that share the unit
  const int wv = wpu ? 0 : wave;                  // this wave's place among them
  const int wq = wpu ? wave : 0;                  // where the unit's final softmax statistics and scalars live in LDS
  const int tix = wpu ? lane : tid;               // this thread's place among the unit's threads
  const int nthr0 = wpu ? SQA_WAVE : kDecThreads;
  const int rows_it = nw * RPI;                   // rows per load of all the unit's waves
  const int lp = wpu ? a.lds_chunk_w : a.lds_chunk;          // LDS logit row length
  float* s_lg = s_logit + (wpu ? wave * G * a.lds_chunk_w : 0);
  const int bidx = u / a.Hkv, kvh = u % a.Hkv;
  const sqa_layer_cache L = a.layers[layer];
  const int64_t uoff = L.unit_offset ? L.unit_offset[u] : (int64_t)u * L.capacity;   // the unit's first slot
  const int cap = L.unit_offset ? (int)(L.unit_offset[u + 1] - uoff) : L.capacity;
  const int budget = a.budget_seq ? a.budget_seq[layer * a.B + bidx] : L.budget;
  const bool sits_out = a.new_pos_seq && a.new_pos_seq[bidx] < 0;
  const int hh = H2O ? budget / 2 : (a.policy == SQA_STREAMING ? min(a.n_sink, budget) : 0);
  const int rec = budget - hh;
  const int csize = (int)a.lay[layer].chunk;
  const int c0 = chunk * csize;

  const int64_t qoff = (((int64_t)layer * a.B + bidx) * a.Hq + (int64_t)kvh * G) * D;
  const int64_t kvoff = (((int64_t)layer * a.B + bidx) * a.Hkv + kvh) * D;
  char* outp = reinterpret_cast<char*>(a.out) + qoff * (int64_t)sizeof(T);
  const char* Kb = reinterpret_cast<const char*>(L.K) + (PG ? 0 : uoff * ROWB);
  const char* Vb = reinterpret_cast<const char*>(L.V) + (PG ? 0 : uoff * ROWB);
  // row of the unit's slot s within Kb / Vb (block numbers staged at the end of the dynamic LDS: the whole
  // row of the table, or a wave's own 16 entries with one wave per unit)
  int* const s_tbl = reinterpret_cast<int*>(reinterpret_cast<char*>(s_logit) + (PG ? a.tbl_off : 0));
  const int tb = wpu ? wave * (kWpuMaxSlots / SQA_BLOCK_SLOTS) : 0;
  auto row_of = [&](int s_) -> int64_t {
    if constexpr (PG) return (int64_t)s_tbl[tb + (s_ >> 4)] * SQA_BLOCK_SLOTS + (s_ & (SQA_BLOCK_SLOTS - 1));
    else return (int64_t)s_;
  };
  // slots this step can touch: with blocks, a unit needs table entries only for its own budget's slots
  // (a sequence with a small budget holds few blocks; the rest of its table row is never read)
  const int span = PG ? min(cap, max(min(budget, L.budget), 0)) : cap;
  bool bad_tbl = false;
  if constexpr (PG) {
    // (every workgroup of the unit stages the whole row: the tail touches any slot; a block number outside
    // the pools is replaced by 0 here, so that the early requests below stay inside them, and reported)
    const int32_t* tbl = L.block_table + (int64_t)u * L.blocks_per_unit;
    const int nblk = (span + SQA_BLOCK_SLOTS - 1) / SQA_BLOCK_SLOTS;
    int bad = 0;
    for (int i = tix; i < nblk; i += nthr0) {
      const int e = tbl[i];
      const bool oob = (unsigned)e >= (unsigned)L.n_blocks;
      bad |= oob;
      s_tbl[tb + i] = oob ? 0 : e;
    }
    bad_tbl = wpu ? __ballot(bad) != 0ull : __syncthreads_or(bad) != 0;
  }
  const char* knew = reinterpret_cast<const char*>(a.k_new) + kvoff * (int64_t)sizeof(T);
  const char* vnew = reinterpret_cast<const char*>(a.v_new) + kvoff * (int64_t)sizeof(T);
  float* sc = H2O ? L.score_acc + uoff : nullptr;
  const int32_t* posu = L.pos + uoff;

  // Everything that does not depend on the unit's length is requested now, so
  // that one memory round trip covers the bookkeeping words, q, the new token's
  // rows, the first rows of the chunk (read as they lie in memory; the two
  // slots the step rewrites are patched below) and the first scores.
  const int4 ust = *reinterpret_cast<const int4*>(L.unit_state + (int64_t)u * SQA_ST_WORDS);   // one 16-byte record
  const int len = ust.x;
  const int head = ust.y;
  const int hint = H2O ? ust.z : -1;
  uint4 qf[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
    qf[g] = ld16(reinterpret_cast<const char*>(a.q) + (qoff + (int64_t)g * D) * (int64_t)sizeof(T) + c * 16);
  const uint4 kn_pre = ld16(knew + c * 16), vn_pre = ld16(vnew + c * 16);
  uint4 kf[U], vf[U];
  int slot[U];
  // (a packed unit may own no slot at all -- it is reported below, once its length is known --: these
  // early requests then read the new token's rows instead, which always exist)
  const bool has_slots = cap > 0;
  if constexpr (!MF) {
    const char* Kpre = has_slots ? Kb : knew;
    const char* Vpre = has_slots ? Vb : vnew;
#pragma unroll
    for (int uu = 0; uu < U; ++uu) {
      slot[uu] = c0 + uu * rows_it + wv * RPI + r;
      const int sl = max(min(slot[uu], span - 1), 0);
      const int64_t rw = (has_slots && span > 0) ? row_of(sl) : 0;
      kf[uu] = ld16_nt(Kpre + rw * ROWB + c * 16);
      vf[uu] = ld16_nt(Vpre + rw * ROWB + c * 16);
    }
  }
  const float sc_pre = (H2O && has_slots) ? sc[min(tix, cap - 1)] : 0.f;

  // ---- 0. where does the new token go, who leaves -------------------------
  if (sits_out) return;                           // the sequence takes no part in this step (every chunk agrees)
  const int min_budget = H2O ? 2 : (a.policy == SQA_STREAMING ? a.n_sink + 1 : 1);
  const bool bad_budget = budget < min_budget || budget > L.budget;
  const bool bad_state = !bad_budget && (len > budget || len > cap || len < 0 || head < 0 || (len == budget && head >= rec));
  const bool bad_cap = !bad_budget && !bad_state && len < budget && len >= cap;
  if (bad_budget || bad_state || bad_cap || bad_tbl) {       // same verdict in every chunk of the unit
    if (chunk == 0) {
      for (int i = tix; i < G * D; i += nthr0) reinterpret_cast<T*>(outp)[i] = T{};
      if (tix == 0)
        *a.status = bad_tbl ? SQA_ERR_SHAPE : (bad_budget ? SQA_ERR_BUDGET : (bad_state ? SQA_ERR_STATE : SQA_ERR_CAPACITY));
    }
    return;
  }
  const bool full = len == budget;
  const bool ae = a.ae != 0;
  // Evict-then-attend: a full unit attends its budget tokens, the new token already
  // sitting (logically) in the slot it will occupy.  Attend-then-evict: the unit
  // attends all len+1 tokens as they lie, the new token as one more slot at
  // index len (which exists only in this step's index space when the unit is
  // full), and the eviction happens after the accumulation (step 3).
  const int n = (full && !ae) ? budget : len + 1; // tokens attended this step
  const int slot_wr = full ? hh + head : len;     // physical slot the new token is written to
  const int slot_new = ae ? len : slot_wr;        // index of the new token while streaming
  // last row that may be read from memory (with blocks: the last one the staged table rows cover; under
  // attend-then-evict a full unit's new token has index budget, which is never read from the cache)
  const int rmax = min(n, span) - 1;
  int moved_to = -1;                              // heavy slot that receives the ring leaver
  if (H2O && full && !ae) {
    if (hint >= -1 && hint < hh) {
      moved_to = hint;
    } else {                                      // no decision carried over: take it now
      float mn = INFINITY;
      for (int i = tix; i < hh; i += nthr0) mn = fminf(mn, sc[i]);
      mn = block_min(mn, s_red, wpu);
      moved_to = pick_victim(sc, posu, hh, mn, sc[slot_wr], -1, 0, s_red64, wpu, tix);
    }
  }
  // the ring leaver's score and position, needed in step 3 if it moves
  const float leaver_score = (H2O && moved_to >= 0) ? sc[slot_wr] : 0.f;
  const int leaver_pos = (H2O && moved_to >= 0) ? posu[slot_wr] : 0;

  // ---- 1. stream the chunk's K and V once, online softmax -------------------
  const int c_end = min(c0 + csize, n);
  const int lpitch = cap + 1;                      // logit row of one head in scratch (the new token may be slot cap)
  // (a unit's scratch region: G x (its slots + kLogitPad) floats, regions in unit order)
  float* glogit = (H2O && (nsplit > 1 || MF)) ? a.logit + a.lay[layer].logit_off + (uoff + (int64_t)kLogitPad * u) * G : nullptr;
  // The matrix-core variant keeps in that region (for every unit, split or not: nothing of it needs LDS), tile
  // by tile of 32 tokens, the bf16 probabilities relative to the tile's reference, [tile][head][32] -- a wave
  // writes a tile's G x 64 bytes in one go, whole cache lines -- and behind them the references, [tile][head]
  // (tiles start at multiples of 32 because chunks do).  They are written and read by the same workgroup unless
  // the unit is split: only then do they need the coherent path.
  // Units short enough keep all of this in LDS instead (behind the stage buffers; a per-layer flag of the
  // launch plan): what a step writes to memory costs several times what it reads, and these 2 bytes per token
  // and head, written and read back by the same workgroup, are not part of what the method has to move.
  const int ntile_max = (lpitch + 31) >> 5;
  const bool handover = nsplit > 1;
  // tiles below lds_tiles keep their probabilities and references in LDS, the others go through the workspace
  const int lds_tiles = (MF && H2O) ? (int)((nsplit_w >> kLdsTilesShift) & kLdsTilesMask) : 0;
  unsigned short* e16 = reinterpret_cast<unsigned short*>(glogit);
  float* tref = (MF && H2O) ? glogit + (int64_t)ntile_max * G * 16 : nullptr;
  char* const probs_lds = stage_base + kDecWaves * kStageBytesPerWave + (wpu ? wave * a.lds_probs_w : 0);
  unsigned short* const e16_l = reinterpret_cast<unsigned short*>(probs_lds);                // [tile][head][32]
  float* const tref_l = reinterpret_cast<float*>(probs_lds + lds_tiles * G * 64);            // [tile][head]

  if constexpr (MF) {
    // ---- 1M. matrix-core streaming ------------------------------------------
    // Lane roles (v_mfma_f32_16x16x32_bf16: A row / B column = lane%16, the 8
    // contraction slots of a lane = 8*(lane/16)+e; C column = lane%16, rows
    // 4*(lane/16)+i):
    //   S^T = K.Q^T : A = 16 tokens of the tile (row = token), B = q of the g
    //                 heads (column = head, zero beyond g); contraction slot
    //                 (j,e) of step i <-> d = 32j + 8i + e for both operands;
    //   O^T = V^T.P^T: per 16-token half of the tile a 16x16x16 step, A = V^T
    //                 (row = d within a block of 16), B = P^T = the probabilities
    //                 exactly where the S^T result left them (column = head);
    //                 contraction slot (j,e) <-> token 4j+e of the half.
    // So softmax statistics and the output accumulator live in the lanes of
    // their head and nothing is moved between lanes except two max/sum steps.
    // K and V tiles pass through a wave-private 8.5 KiB LDS buffer, one after the
    // other.  The V tile (copied from registers) has rows padded by 16 bytes
    // (conflict-free for the transposing reads).  The K tile has 256-byte rows
    // whose 16-byte pieces are XOR-swizzled with the row number: piece p of tile
    // row R lies at piece p ^ (R & 15).  A fragment read takes 16 bytes from each
    // of 16 different rows; with padded rows that ran at 30 cycles per wave
    // instruction on this chip (4-way bank conflicts), swizzled it runs at 8.5.
    // K rows are loaded from global memory straight into that layout (direct
    // global->LDS loads, the swizzle applied to the global address): the 32
    // registers a K tile in flight used to occupy are what kept this variant at 2
    // waves per SIMD; at 3, with a third more bytes in flight per CU, the
    // Llama-2-70B shape went from 1138 to 997 us per step.
    char* stage = stage_base + wave * kStageBytesPerWave;
    const int hd = lane & 15, j4 = lane >> 4;
    bf16x8_t qfr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint4 w = make_uint4(0, 0, 0, 0);
      if (hd < G) w = ld16(reinterpret_cast<const char*>(a.q) + (qoff + (int64_t)hd * D) * 2 + 64 * j4 + 16 * i);
      qfr[i] = __builtin_bit_cast(bf16x8_t, w);
    }
    f32x4_t oacc[8];
#pragma unroll
    for (int db = 0; db < 8; ++db) oacc[db] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;
    // LDS addresses of this lane (tile rows are kStageRow bytes apart, so every
    // other address below is one of these plus a compile-time constant)
    char* st_wr = stage + r * kStageRow + c * 16;                       // V: row-wise writes: + 4i rows
    // K, swizzled: fragment i of row 16tt+hd -> + 4096tt + kr[i]
    int kr[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      kr[x] = hd * 256 + ((4 * j4) ^ (hd & 12)) * 16 + ((x ^ (hd & 3)) * 16);
    }
    auto k_patch = [&](int row, const uint4& val) {   // row of the tile, written by the 16 lanes whose r matches
      if ((row & 3) == r) *reinterpret_cast<uint4*>(stage + row * 256 + ((c ^ (row & 15)) * 16)) = val;
    };
    const char* st_v = stage + (4 * j4 + (hd >> 2)) * kStageRow + (hd & 3) * 8;   // V^T quadruple: + 16 rows, + 32db bytes
    // Registers hold a V tile only between its load and its copy into LDS: the
    // next tile's V is requested as soon as this tile's V has been copied, the
    // next tile's K as soon as the stage is free again (after the P.V reads).
    uint4 vreg[8];
    // A wave instruction of the direct K load fills 1 KB = tile rows 4i .. 4i+3 in
    // lane order, so lane (r, c) fetches the piece that belongs at position c of
    // row 4i + r: piece c ^ ((4i + r) & 15) = (c ^ r) ^ (4 (i & 3)).  Plain loads:
    // here they ran faster than non-temporal ones (997 vs 1021 us), while V is
    // better off non-temporal (plain: 1109 us).
    auto request_k = [&](int base) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const char* g;
        if constexpr (PG) g = Kb + row_of(min(base + 4 * i + r, rmax)) * ROWB + (((c ^ r) ^ (4 * (i & 3))) * 16);
        else g = Kb + ((uint32_t)min(base + 4 * i + r, rmax) * (uint32_t)ROWB + (uint32_t)(((c ^ r) ^ (4 * (i & 3))) * 16));
        __builtin_amdgcn_global_load_lds((dec_gptr_t*)g, (dec_lptr_t*)(stage + 1024 * i), 16, 0, 0);
      }
    };
    auto request_v = [&](int base) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if constexpr (PG) vreg[i] = ld16_nt(Vb + row_of(min(base + 4 * i + r, rmax)) * ROWB + c * 16);
        else vreg[i] = ld16_nt(Vb + ((uint32_t)min(base + 4 * i + r, rmax) * (uint32_t)ROWB + (uint32_t)(c * 16)));
    };
    const int TSTEP = 32 * nw;                      // the unit's waves take its 32-token tiles in turn
    if (c0 + 32 * wv < c_end) { request_k(c0 + 32 * wv); request_v(c0 + 32 * wv); }
    for (int base = c0 + 32 * wv; base < c_end; base += TSTEP) {
      const bool more = base + TSTEP < c_end;
      // The two slots this step rewrites are still old in memory: their rows are
      // patched in the staged tile (wave-uniform tests, true for one tile per unit).
      const bool has_new = slot_new >= base && slot_new < base + 32;
      const bool has_moved = moved_to >= base && moved_to < base + 32;
      uint4 km = make_uint4(0, 0, 0, 0), vm = km;
      if (has_moved) { km = ld16(Kb + row_of(slot_wr) * ROWB + c * 16); vm = ld16(Vb + row_of(slot_wr) * ROWB + c * 16); }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // this tile's K rows have landed in the stage
      if (has_moved) k_patch(moved_to - base, km);
      if (has_new) k_patch(slot_new - base, kn_pre);
      f32x4_t sacc[2];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        sacc[tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint4 w = *reinterpret_cast<const uint4*>(stage + 4096 * tt + kr[i]);
          sacc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, w), qfr[i], sacc[tt], 0, 0, 0);
        }
      }
      float sv[8];
      float mx = -INFINITY;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int tok = base + (e < 4 ? 4 * j4 + e : 16 + 4 * j4 + (e - 4));
        float d = (e < 4 ? sacc[0][e] : sacc[1][e - 4]) * a.scale_log2;
        const bool valid = tok < c_end;
        d = valid ? d : -INFINITY;
        sv[e] = d;
        mx = fmaxf(mx, d);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16, SQA_WAVE));
      mx = fmaxf(mx, __shfl_xor(mx, 32, SQA_WAVE));
      const float m_new = fmaxf(m_run, mx);
      const float ms = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = fast_exp2(m_run - ms);
      m_run = m_new;
      bf16x4_t pfr[2];
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float pe = fast_exp2(sv[e] - ms);
        psum += pe;
        pfr[e >> 2][e & 3] = (__bf16)pe;
      }
      l_run = l_run * alpha + psum;
      if (H2O && hd < G) {
        // What step 3 needs of this tile: the probabilities as the second product uses them (bf16,
        // relative to the tile's reference ms) and that reference, one per head.  2 bytes per token and
        // head instead of a 4-byte logit: for split units these go through memory, where every byte
        // written costs as much as several bytes read.
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {            // (tokens beyond the unit's end get zeros: the region holds whole tiles)
          const unsigned long long four = __builtin_bit_cast(unsigned long long, pfr[tt]);
          if ((base >> 5) < lds_tiles) {
            *reinterpret_cast<unsigned long long*>(e16_l + ((base >> 5) * G + hd) * 32 + 16 * tt + 4 * j4) = four;
          } else {
            unsigned long long* dst = reinterpret_cast<unsigned long long*>(e16 + ((int64_t)(base >> 5) * G + hd) * 32 + 16 * tt + 4 * j4);
            if (handover) st_agent(dst, four); else *dst = four;
          }
        }
        if (j4 == 0) {
          if ((base >> 5) < lds_tiles) {
            tref_l[(base >> 5) * G + hd] = ms;
          } else {
            float* dst = &tref[(base >> 5) * G + hd];
            if (handover) st_agent(dst, ms); else *dst = ms;
          }
        }
      }
      if (__ballot(alpha != 1.f)) {
#pragma unroll
        for (int db = 0; db < 8; ++db) oacc[db] *= alpha;
      }
      // the K fragments are consumed: the same buffer now takes the V tile
#pragma unroll
      for (int i = 0; i < 8; ++i) *reinterpret_cast<uint4*>(st_wr + 4 * i * kStageRow) = vreg[i];
      if (has_moved && ((moved_to - base) & 3) == r)
        *reinterpret_cast<uint4*>(st_wr + ((moved_to - base) >> 2) * 4 * kStageRow) = vm;
      if (has_new && ((slot_new - base) & 3) == r)
        *reinterpret_cast<uint4*>(st_wr + ((slot_new - base) >> 2) * 4 * kStageRow) = vn_pre;
      if (more) request_v(base + TSTEP);
      // V^T fragments with the transposing LDS read (ds_read_b64_tr_b16): in a
      // block of 16 lanes, lane 4e+a supplies the address of 4 consecutive
      // 16-bit values and lane 4a+b receives, as element e, value b of the
      // quadruple supplied by lane 4e+a.  With lane 4e+a pointing at
      // V[token 4j+e][16db + 4a ..], lane m = 4a+b gets V[token 4j+e][16db + m],
      // e = 0..3: the A fragment of a 16x16x16 step over that 16-token half.
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int db = 0; db < 8; ++db) {
          const v4s_t vt = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(st_v + 16 * tt * kStageRow + 32 * db));
          oacc[db] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vt, __builtin_bit_cast(v4s_t, pfr[tt]), oacc[db], 0, 0, 0);
        }
      // the stage is free again (its reads have returned): the next tile's K rows may land in it
      if (more) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        request_k(base + TSTEP);
      }
    }
    l_run += __shfl_xor(l_run, 16, SQA_WAVE);
    l_run += __shfl_xor(l_run, 32, SQA_WAVE);
    if (hd < G) {
      if (j4 == 0) { s_m[wave][hd] = m_run; s_l[wave][hd] = l_run; }
#pragma unroll
      for (int db = 0; db < 8; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc_lds[wave * kAccWave + hd * D + 16 * db + 4 * j4 + i] = oacc[db][i];
    }
  } else {
    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    // patch the rows requested before the layout of this step was known
#pragma unroll
    for (int uu = 0; uu < U; ++uu) {
      if (slot[uu] == slot_new) { kf[uu] = kn_pre; vf[uu] = vn_pre; }
      if (slot[uu] == moved_to) {
        kf[uu] = ld16(Kb + row_of(slot_wr) * ROWB + c * 16);
        vf[uu] = ld16(Vb + row_of(slot_wr) * ROWB + c * 16);
      }
    }

    for (int base = c0; base < c_end; base += rows_it * U) {
      if (base != c0) {
        // A wave that is about to ask for its next rows goes ahead of waves that
        // are doing arithmetic: the sooner its requests are out, the fuller the
        // memory pipeline (267.8 instead of 270.1 us per step at the 7B shape).
        __builtin_amdgcn_s_setprio(3);
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
          slot[uu] = base + uu * rows_it + wv * RPI + r;
          const int sl = min(slot[uu], n - 1);
          // (with blocks: never a table entry beyond the staged ones -- a full unit's new token under
          // attend-then-evict has index budget; its rows come from k_new / v_new just below)
          const int64_t rw = row_of(PG ? min(sl == moved_to ? slot_wr : sl, rmax) : (sl == moved_to ? slot_wr : sl));
          const char* kp = Kb + rw * ROWB;
          const char* vp = Vb + rw * ROWB;
          if (sl == slot_new) { kp = knew; vp = vnew; }
          kf[uu] = ld16_nt(kp + c * 16);
          vf[uu] = ld16_nt(vp + c * 16);
        }
        __builtin_amdgcn_s_setprio(0);
      }
      float s[U][G];
#pragma unroll
      for (int uu = 0; uu < U; ++uu)
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float d = group_sum<LPR>(RowMath<T>::dot(qf[g], kf[uu])) * a.scale_log2;
          const bool valid = slot[uu] < c_end;
          d = valid ? d : -INFINITY;
          s[uu][g] = d;
          if (H2O && c == 0 && valid) {
            if (glogit) st_agent(&glogit[(int64_t)g * lpitch + slot[uu]], d);
            else s_lg[g * lp + slot[uu]] = d;
          }
        }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float mx = m[g];
#pragma unroll
        for (int uu = 0; uu < U; ++uu) mx = fmaxf(mx, s[uu][g]);
        const float ms = mx == -INFINITY ? 0.f : mx;
        const float alpha = fast_exp2(m[g] - ms);
        m[g] = mx;
        float lsum = l[g] * alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] *= alpha;
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
          const float p = fast_exp2(s[uu][g] - ms);
          lsum += p;
          RowMath<T>::axpy(p, vf[uu], acc[g]);
        }
        l[g] = lsum;
      }
    }

    // ---- 2. combine row groups of the wave, then the waves --------------------
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int o = LPR; o < SQA_WAVE; o <<= 1) {
        const float mo = __shfl_xor(m[g], o, SQA_WAVE);
        const float lo2 = __shfl_xor(l[g], o, SQA_WAVE);
        const float mx = fmaxf(m[g], mo);
        const float ms = mx == -INFINITY ? 0.f : mx;
        const float fa = fast_exp2(m[g] - ms), fb = fast_exp2(mo - ms);
        l[g] = l[g] * fa + lo2 * fb;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const float ao = __shfl_xor(acc[g][e], o, SQA_WAVE);
          acc[g][e] = acc[g][e] * fa + ao * fb;
        }
        m[g] = mx;
      }
      if (r == 0) {
        if (c == 0) { s_m[wave][g] = m[g]; s_l[wave][g] = l[g]; }
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc_lds[wave * kAccWave + g * D + c * EPL + e] = acc[g][e];
      }
    }
  }
  if (!wpu) __syncthreads();
  float* part = nsplit > 1 ? a.part + ((int64_t)a.lay[layer].part_off + (int64_t)u * nsplit) * G * PREC : nullptr;
  // one lane group per query head: merge the unit's waves (all 4, or just this one)
  const int w_lo = wpu ? wave : 0, w_hi = wpu ? wave + 1 : kDecWaves;
  for (int g = wv * RPI + r; g < G; g += nw * RPI) {
    float mx = -INFINITY;
    for (int w = w_lo; w < w_hi; ++w) mx = fmaxf(mx, s_m[w][g]);
    const float ms = mx == -INFINITY ? 0.f : mx;  // an empty chunk has nothing
    float lt = 0.f, o[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] = 0.f;
    for (int w = w_lo; w < w_hi; ++w) {
      const float f = fast_exp2(s_m[w][g] - ms);
      lt += s_l[w][g] * f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] += acc_lds[w * kAccWave + g * D + c * EPL + e] * f;
    }
    if (nsplit == 1) {
      const float inv = 1.f / lt;                 // n >= 1: lt > 0
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] *= inv;
      RowMath<T>::store(outp + (int64_t)g * ROWB + c * 16, o);
      if (c == 0) { s_m[wq][g] = mx; s_l[wq][g] = inv; }
    } else {
      float* rec_p = part + ((int64_t)chunk * G + g) * PREC;
#pragma unroll
      for (int e = 0; e < EPL; ++e) st_agent(&rec_p[c * EPL + e], o[e]);
      if (c == 0) { st_agent(&rec_p[D], mx); st_agent(&rec_p[D + 1], lt); }
    }
  }

  if (nsplit > 1) {
    // Publish this chunk, find out whether it is the last one of the unit.  Every
    // thread first waits until its own stores above (partials, logits, probabilities:
    // agent-scope, written through to where every XCD sees them) have been
    // acknowledged -- s_waitcnt vmcnt(0); a workgroup barrier alone orders LDS traffic,
    // not outstanding global stores --, then the barrier collects the threads, and only
    // then does thread 0 bump the counter: whoever sees the count sees the data.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    int32_t* cnt = a.cnt + a.lay[layer].unit_off + u;
    if (tid == 0) s_ctl[0] = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_ctl[0] != nsplit - 1) return;
    for (int g = wave * RPI + r; g < G; g += kDecWaves * RPI) {
      float mx = -INFINITY;
      for (int k = 0; k < nsplit; ++k) mx = fmaxf(mx, ld_agent(&part[((int64_t)k * G + g) * PREC + D]));
      float lt = 0.f, o[EPL];
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] = 0.f;
      for (int k = 0; k < nsplit; ++k) {          // fixed order
        const float* rec_p = part + ((int64_t)k * G + g) * PREC;
        const float f = fast_exp2(ld_agent(&rec_p[D]) - mx);   // some chunk is non-empty: mx is finite
        lt += ld_agent(&rec_p[D + 1]) * f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[e] += ld_agent(&rec_p[c * EPL + e]) * f;
      }
      const float inv = 1.f / lt;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] *= inv;
      RowMath<T>::store(outp + (int64_t)g * ROWB + c * 16, o);
      if (c == 0) { s_m[0][g] = mx; s_l[0][g] = inv; }
    }
    if (tid == 0) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
  }

  // ---- 3. H2O accumulation and the next step's eviction decision ------------
  // What is left is a short tail of dependent loads and stores.  A wave keeps
  // its registers until its last store is acknowledged, so for an unsplit unit
  // waves 1-3 leave here and wave 0 finishes alone: three quarters of the
  // workgroup's registers are free for the next workgroup while the tail runs.
  if (!wpu) __syncthreads();                      // every wave is done reading the cache rows and writing LDS
  // (matrix-core H2O: the whole workgroup walks the unit's probabilities, unless each wave has a unit of its own)
  // (... except in a call with few workgroups, where nothing else would use the registers the other waves
  // free and a long unit's tail -- its scores are walked once more -- is on the critical path)
  const bool solo = nsplit == 1 && (wpu || (!(MF && H2O) && !(a.wide_tail != 0 && n > kSoloMaxTokens)));
  if (solo && !wpu && wave != 0) return;
  const int nthr = solo ? SQA_WAVE : kDecThreads;
  const int tq = solo ? lane : tid;               // this thread's place among the nthr threads still at work
  int next_hint = ae ? -2 : -1;
  const int head_next = full ? (head + 1 == rec ? 0 : head + 1) : head;
  int victim = -1;                                // attend-then-evict: heavy slot evicted in this step (-1: the leaver)
  if (H2O) {
    float fm[G], fi[G];                           // (the matrix-core variant reads them from LDS where it needs them)
#pragma unroll
    for (int g = 0; g < G; ++g) { fm[g] = MF ? 0.f : s_m[wq][g]; fi[g] = MF ? 0.f : s_l[wq][g]; }
    // the heavy region competes with: the NEXT ring leaver for the next step's decision (evict-then-attend),
    // or this step's ring leaver right now (attend-then-evict)
    const bool decide = ae ? full : n == budget;
    const int leaver_slot = ae ? slot_wr : hh + head_next;
    const bool virt = ae && full;                 // the new token has no slot of its own yet
    // Matrix-core variant: one factor per (head, 32-token tile) turns a stored probability into the final
    // one, exp2(reference - m) / l; the table goes where the tiles were staged (if the unit is so long that
    // it does not fit there, the factor is recomputed per token instead).
    float* fac = reinterpret_cast<float*>(stage_base + (wpu ? wave * kStageBytesPerWave : 0));
    const bool use_fac = MF && (size_t)G * ntile_max * sizeof(float) <= (size_t)nw * kStageBytesPerWave;
    if constexpr (MF) {
      if (use_fac) {
        const int ntile = (n + 31) >> 5;
        for (int idx = tq; idx < G * ntile; idx += nthr) {
          const int g = idx % G;                  // idx = tile * G + head
          const float rf = idx < lds_tiles * G ? tref_l[idx] : (handover ? ld_agent(&tref[idx]) : tref[idx]);
          fac[idx] = fast_exp2(rf - s_m[wq][g]) * s_l[wq][g];
        }
        if (!solo) __syncthreads();               // (a wave on its own reads back what it wrote itself: LDS keeps a wave's order)
      }
    }
    float mn = INFINITY;
    constexpr int SB = 4;                         // scores requested together: one round trip per SB tokens
    for (int i0 = tq; i0 < n; i0 += SB * nthr) {
      float cur[SB];
#pragma unroll
      for (int k = 0; k < SB; ++k) {
        const int i = i0 + k * nthr;
        cur[k] = (k == 0 && i0 == tq) ? sc_pre : sc[min(i, rmax)];   // each thread's first score came with the start
      }
#pragma unroll
      for (int k = 0; k < SB; ++k) {
        const int i = i0 + k * nthr;
        if (i < n) {
          float p = 0.f;
#pragma unroll
          for (int g = 0; g < G; ++g) {
            if constexpr (MF) {
              const int at = ((i >> 5) * G + g) * 32 + (i & 31);
              const bool in_lds = (i >> 5) < lds_tiles;
              const unsigned short eb = in_lds ? e16_l[at] : (handover ? ld_agent(&e16[at]) : e16[at]);
              const float e = __uint_as_float((uint32_t)eb << 16);
              p += e * (use_fac ? fac[(i >> 5) * G + g]
                                : fast_exp2((in_lds ? tref_l[(i >> 5) * G + g] : ld_agent(&tref[(i >> 5) * G + g])) - s_m[wq][g]) * s_l[wq][g]);
            } else {
              const float lg = glogit ? ld_agent(&glogit[(int64_t)g * lpitch + i]) : s_lg[g * lp + i];
              p += fast_exp2(lg - fm[g]) * fi[g];
            }
          }
          const float old = i == slot_new ? 0.f : (i == moved_to ? leaver_score : cur[k]);
          const float nv = old + p;
          if (virt && i == slot_new) s_ctlf[wq][1] = nv;   // stored in step 4, once its slot is free
          else sc[i] = nv;
          if (i < hh) mn = fminf(mn, nv);
          if (i == leaver_slot) s_ctlf[wq][0] = nv;
        }
      }
    }
    if (decide) {
      mn = block_min(mn, s_red, solo);            // (the barrier inside also orders the s_ctlf writes)
      // positions as they will be after step 4: the moved token brings its own
      const int v = pick_victim(sc, posu, hh, mn, s_ctlf[wq][0], moved_to, leaver_pos, s_red64, solo, tq);
      if (ae) {
        // Apply it now.  Each score is rewritten by the thread that wrote it
        // above (slot i belongs to thread i mod nthr), so the two writes to one
        // address are ordered by that thread's program order.
        victim = v;
        if (victim >= 0 && tq == victim % nthr) sc[victim] = s_ctlf[wq][0];
        if (tq == slot_wr % nthr) sc[slot_wr] = s_ctlf[wq][1];
      } else {
        next_hint = v;
      }
    }
  }
  const int dst = ae ? victim : moved_to;         // heavy slot that takes over the ring leaver's row

  // ---- 4. the cache update: moved row, new token, bookkeeping ---------------
  if ((wpu || wave == 0) && r == 0) {
    char* Kw = const_cast<char*>(Kb);
    char* Vw = const_cast<char*>(Vb);
    if (dst >= 0) {
      const uint4 kk = ld16(Kw + row_of(slot_wr) * ROWB + c * 16);
      const uint4 vv = ld16(Vw + row_of(slot_wr) * ROWB + c * 16);
      st16(Kw + row_of(dst) * ROWB + c * 16, kk);
      st16(Vw + row_of(dst) * ROWB + c * 16, vv);
    }
    st16(Kw + row_of(slot_wr) * ROWB + c * 16, kn_pre);
    st16(Vw + row_of(slot_wr) * ROWB + c * 16, vn_pre);
    if (c == 0) {
      int32_t* posw = L.pos + uoff;
      if (dst >= 0) posw[dst] = posw[slot_wr];
      posw[slot_wr] = a.new_pos_seq ? a.new_pos_seq[bidx] : a.new_pos;   // (read again: not kept in a register all along)
      *reinterpret_cast<int4*>(L.unit_state + (int64_t)u * SQA_ST_WORDS) =
          make_int4(full ? budget : len + 1, head_next, H2O ? next_hint : -2, 0);
    }
  }
}

typedef void (*decode_fn)(const DecodeArgs);

// Grouped queries of 4 or more heads per KV head in bf16 at D = 128 go to the matrix cores: with 8 heads
// the vector-ALU path is arithmetic bound (4.2 TB/s against 6.5 TB/s on the Llama-2-70B shape), with 4
// heads the matrix-core variant is still slightly ahead (779 against 797 us per step on the Mistral-7B shape).
constexpr int kMfmaMinGroup = 4;      // query heads per KV head from which the matrix-core variant is used
template <typename T, int D, int G> constexpr bool use_mfma() { return sizeof(T) == 2 && D == 128 && G >= kMfmaMinGroup; }
template <typename T, int D, bool H2O, bool PG> decode_fn pick_g(int g) {
  switch (g) {
    case 1: return decode_unit_kernel<T, D, 1, H2O, false, PG>;
    case 2: return decode_unit_kernel<T, D, 2, H2O, false, PG>;
    case 4: return decode_unit_kernel<T, D, 4, H2O, use_mfma<T, D, 4>(), PG>;
    case 8: return decode_unit_kernel<T, D, 8, H2O, use_mfma<T, D, 8>(), PG>;
  }
  return nullptr;
}
template <typename T, bool H2O, bool PG> decode_fn pick_d(int d, int g) {
  if (d == 64) return pick_g<T, 64, H2O, PG>(g);
  if (d == 128) return pick_g<T, 128, H2O, PG>(g);
  return nullptr;
}
template <typename T, bool H2O> decode_fn pick_p(int d, int g, bool paged) {
  return paged ? pick_d<T, H2O, true>(d, g) : pick_d<T, H2O, false>(d, g);
}
static decode_fn pick(sqa_dtype dt, int d, int g, bool h2o, bool paged) {
  if (dt == SQA_F32) return h2o ? pick_p<float, true>(d, g, paged) : pick_p<float, false>(d, g, paged);
  return h2o ? pick_p<bf16_t, true>(d, g, paged) : pick_p<bf16_t, false>(d, g, paged);
}

constexpr size_t kStatusBytes = 256;

// How one call is cut into work items and where its scratch lives.
struct DecodePlan {
  int tbl_entries;                                 // blocked allocation: block numbers a workgroup stages in LDS
  int lds_probs, lds_probs_w;                      // LDS bytes for the probabilities of a workgroup / of one wave's unit
  uint16_t lds_tiles[SQA_MAX_LAYERS];              // matrix-core variant under H2O: leading tiles of a unit whose probabilities stay in LDS
  uint8_t probs_in_lds[SQA_MAX_LAYERS];            // ... 1: all of them (nothing of it in the workspace), 2: the leading part
  int lds_chunk;                                   // longest unsplit unit shared by 4 waves (slots)
  int lds_chunk_w;                                 // longest one-wave unit (slots)
  uint8_t wpu[SQA_MAX_LAYERS];                     // one wave per unit in this layer
  uint16_t nsplit[SQA_MAX_LAYERS];
  uint32_t chunk[SQA_MAX_LAYERS];
  uint32_t unit_off[SQA_MAX_LAYERS], part_off[SQA_MAX_LAYERS], logit_off[SQA_MAX_LAYERS];
  uint64_t blocks;
  size_t cnt_bytes, part_bytes, logit_bytes;       // arrival counters, partial records, H2O logits / probabilities
  size_t off_table, off_cnt, off_part, off_logit, bytes;   // where they lie in a caller's workspace
};

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Units are split only when the call would otherwise leave CUs idle: the target work item is the call's
// tokens divided by the number of CUs (at least 256 slots, and at most what lets a unit's step logits fit
// in LDS -- kMaxUnsplit slots x heads; not for the matrix-core variant, which keeps what H2O needs in the
// workspace), and a unit is cut into equal chunks only if it is more than a quarter longer than that.
// One workgroup per CU already streams at 80 % of what the chip reaches, so what splitting buys is balance,
// and the hand-over between a unit's workgroups costs more than a small imbalance: with 256 equal units (a
// layer of the Llama-2-7B shape at batch 8 launched on its own) whole units take 53 us, halves 60 us,
// quarters 62 us; all layers at batch 2 take 71 us whole and 81 us cut in three.
constexpr int64_t kMinItems = 256;
constexpr int64_t kWideTailMaxBlocks = 512;       // calls with at most this many workgroups: see DecodeArgs::wide_tail
// Matrix-core variant under H2O: LDS a workgroup may use for a unit's per-head probabilities so that three
// workgroups still fit a CU (160 KiB / 3, less the four stage buffers and the small static arrays).
constexpr int kLdsProbsMax = 18 * 1024;
constexpr int kMaxUnsplit = 8192;
// One wave per unit: for units of at most kWpuMaxSlots slots, in calls that have at least kWpuMinUnits
// units (one wave walks a unit 16 rows at a time, so the call needs many units to keep the chip's wave
// slots filled; the matrix-core variant walks it one 32-token tile at a time).
constexpr int64_t kWpuMinUnits = 4096;
// scratch_probs: the H2O step's per-token, per-head values live in the workspace for every unit, split or
// not (the matrix-core variant: they never need LDS, so nothing limits an unsplit unit's length).
static sqa_status plan_decode(const sqa_layer_cache* layers, int n_layers, int B, int Hq, int Hkv, int D, bool h2o,
                              bool allow_wpu, bool scratch_probs, DecodePlan* p) {
  const int64_t units = (int64_t)B * Hkv;
  const int g = Hq / Hkv;
  const bool paged = layers[0].block_table != nullptr;
  int64_t tokens = 0;
  for (int i = 0; i < n_layers; ++i) {
    if (layers[i].capacity < 1) return SQA_ERR_CAPACITY;
    if (layers[i].budget < 1) return SQA_ERR_BUDGET;
    tokens += units * (layers[i].budget < layers[i].capacity ? layers[i].budget : layers[i].capacity);
  }
  int64_t target = tokens / kMinItems;
  target = target < 256 ? 256 : target;
  if (h2o && !scratch_probs && target > kMaxUnsplit / g) target = kMaxUnsplit / g;
  uint64_t blocks = 0, n_units = 0, n_part = 0, n_logit = 0;
  p->tbl_entries = 0;
  if (paged) {
    p->tbl_entries = kDecWaves * (kWpuMaxSlots / SQA_BLOCK_SLOTS);
    for (int i = 0; i < n_layers; ++i) {
      const int used = layers[i].budget < layers[i].capacity ? layers[i].budget : layers[i].capacity;
      const int e = (used + SQA_BLOCK_SLOTS - 1) / SQA_BLOCK_SLOTS;
      p->tbl_entries = e > p->tbl_entries ? e : p->tbl_entries;
    }
  }
  p->lds_probs = p->lds_probs_w = 0;
  p->lds_chunk = scratch_probs ? 0 : 64;           // (no LDS logits at all when they live in the workspace)
  p->lds_chunk_w = scratch_probs ? 0 : 64;
  for (int i = 0; i < n_layers; ++i) {
    // + 1: under attend-then-evict a full unit attends budget + 1 tokens
    const int nmax = (layers[i].budget < layers[i].capacity ? layers[i].budget : layers[i].capacity) + 1;
    int64_t ns = (4 * (int64_t)nmax + 5 * target - 1) / (5 * target);   // ceil(nmax / (1.25 target))
    ns = ns < 1 ? 1 : ns;
    int64_t ch = ((nmax + ns - 1) / ns + 63) / 64 * 64;
    if (h2o && !scratch_probs && ns == 1 && ch * g > kMaxUnsplit) { ns = 2; ch = ((nmax + 1) / 2 + 63) / 64 * 64; }
    ns = (nmax + ch - 1) / ch;
    if (ns > 65535) return SQA_ERR_CAPACITY;
    p->nsplit[i] = (uint16_t)ns;
    p->chunk[i] = (uint32_t)ch;
    p->wpu[i] = allow_wpu && ns == 1 && nmax <= kWpuMaxSlots && units * n_layers >= kWpuMinUnits;
    p->probs_in_lds[i] = 0;
    p->lds_tiles[i] = 0;
    if (h2o && scratch_probs && ns == 1) {
      // per unit: whole 32-token tiles of bf16 values per head, plus one fp32 reference per tile and head;
      // a unit too long for the LDS a workgroup may use keeps its leading tiles there (a written byte costs
      // many read bytes, so every tile that stays on the chip counts); one-wave units: all or nothing
      const int64_t ntile = ((int64_t)layers[i].capacity + 1 + 31) / 32;
      const int64_t per_tile = (int64_t)g * (64 + 4);
      const int64_t avail = kLdsProbsMax - p->tbl_entries * (int)sizeof(int);
      int64_t tiles = p->wpu[i] ? (ntile * per_tile * kDecWaves <= avail ? ntile : 0) : avail / per_tile;
      tiles = tiles > ntile ? ntile : tiles;
      tiles = tiles > (int64_t)kLdsTilesMask ? (int64_t)kLdsTilesMask : tiles;
      if (tiles > 0) {
        const int64_t need = tiles * per_tile;
        p->lds_tiles[i] = (uint16_t)tiles;
        p->probs_in_lds[i] = tiles == ntile ? 1 : 2;
        if (p->wpu[i] && need > p->lds_probs_w) p->lds_probs_w = (int)need;
        if (need * (p->wpu[i] ? kDecWaves : 1) > p->lds_probs) p->lds_probs = (int)(need * (p->wpu[i] ? kDecWaves : 1));
      }
    }
    if (p->wpu[i]) { if (!scratch_probs && ch > p->lds_chunk_w) p->lds_chunk_w = (int)ch; }
    else if (ns == 1 && !scratch_probs && ch > p->lds_chunk) p->lds_chunk = (int)ch;
    p->unit_off[i] = (uint32_t)n_units;
    p->part_off[i] = (uint32_t)n_part;
    p->logit_off[i] = (uint32_t)n_logit;
    n_units += units;
    blocks += p->wpu[i] ? (units + kDecWaves - 1) / kDecWaves : units * ns;
    if (ns > 1) n_part += units * ns;
    if (h2o && (ns > 1 || scratch_probs) && p->probs_in_lds[i] != 1) n_logit += units * g * ((uint64_t)layers[i].capacity + kLogitPad);
    if (n_units > 0x7fffffffull || n_part > 0x7fffffffull || n_logit > 0xffffffffull || blocks > 0x7fffffffull)
      return SQA_ERR_CAPACITY;
  }
  if (kDecWaves * p->lds_probs_w > p->lds_probs) p->lds_probs = kDecWaves * p->lds_probs_w;
  p->blocks = blocks;
  p->cnt_bytes = n_units * sizeof(int32_t);
  p->part_bytes = n_part * g * (D + 2) * sizeof(float);
  p->logit_bytes = n_logit * sizeof(float);
  p->off_table = kStatusBytes;
  p->off_cnt = align256(p->off_table + (size_t)n_layers * sizeof(sqa_layer_cache));
  p->off_part = align256(p->off_cnt + p->cnt_bytes);
  p->off_logit = align256(p->off_part + p->part_bytes);
  p->bytes = align256(p->off_logit + p->logit_bytes);
  return SQA_OK;
}

}  // namespace sqa

extern "C" size_t sqa_decode_workspace_bytes(const sqa_layer_cache* layers, int n_layers, int B, int Hq, int Hkv,
                                             int D, sqa_policy policy) {
  if (!layers || n_layers < 1 || n_layers > SQA_MAX_LAYERS || B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || D < 1)
    return 0;
  sqa::DecodePlan p;
  // (the element type is not known here: size for the variant that needs more, the matrix-core one if the
  // shape allows it)
  const bool h2o = policy == SQA_H2O;
  size_t bytes = 0;
  for (int wpu = 0; wpu < 2; ++wpu) {              // (a call may or may not give short units a wave each)
    if (sqa::plan_decode(layers, n_layers, B, Hq, Hkv, D, h2o, wpu != 0, false, &p) != SQA_OK) return 0;
    bytes = p.bytes > bytes ? p.bytes : bytes;
    if (h2o && D == 128 && Hq / Hkv >= sqa::kMfmaMinGroup) {
      if (sqa::plan_decode(layers, n_layers, B, Hq, Hkv, D, h2o, wpu != 0, true, &p) != SQA_OK) return 0;
      bytes = p.bytes > bytes ? p.bytes : bytes;
    }
  }
  return bytes;
}

namespace sqa {
// Zero fill by a kernel rather than hipMemsetAsync: callers may record these calls into a HIP graph, and
// memset nodes have replayed wrongly on this platform.
__global__ __launch_bounds__(256) void zero_fill_kernel(uint32_t* __restrict__ p, size_t n_words) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_words; i += (size_t)gridDim.x * 256) p[i] = 0u;
}
static sqa_status zero_fill(void* p, size_t bytes, hipStream_t st) {
  const size_t n_words = bytes / 4;
  if (n_words == 0) return SQA_OK;
  size_t blocks = (n_words + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  zero_fill_kernel<<<(unsigned)blocks, 256, 0, st>>>(static_cast<uint32_t*>(p), n_words);
  SQA_HIP_CHECK(hipGetLastError());
  return SQA_OK;
}
}  // namespace sqa

extern "C" sqa_status sqa_decode_workspace_init(void* workspace, size_t ws_bytes, void* stream) {
  if (!workspace) return SQA_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(workspace) & 3u) return SQA_ERR_SHAPE;
  return sqa::zero_fill(workspace, ws_bytes, static_cast<hipStream_t>(stream));   // (sizes are multiples of 256)
}

extern "C" sqa_status sqa_clear_device_status(void* workspace, void* stream) {
  if (!workspace) return SQA_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(workspace) & 3u) return SQA_ERR_SHAPE;
  return sqa::zero_fill(workspace, sizeof(int32_t), static_cast<hipStream_t>(stream));
}

extern "C" sqa_status sqa_read_device_status(const void* workspace, void* stream, int32_t* status_out) {
  if (!workspace || !status_out) return SQA_ERR_NULL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  SQA_HIP_CHECK(hipMemcpyAsync(status_out, workspace, sizeof(int32_t), hipMemcpyDeviceToHost, st));
  SQA_HIP_CHECK(hipStreamSynchronize(st));
  return SQA_OK;
}

extern "C" sqa_status sqa_decode_step(const void* q, const void* k_new, const void* v_new, sqa_dtype dt,
                                      int B, int Hq, int Hkv, int D, int32_t new_pos,
                                      sqa_policy policy, int n_sink,
                                      const sqa_layer_cache* layers, const sqa_layer_cache* layers_dev, int n_layers,
                                      void* out, void* workspace, size_t ws_bytes, void* stream) {
  return sqa_decode_step_ex(q, k_new, v_new, dt, B, Hq, Hkv, D, new_pos, policy, n_sink, layers, layers_dev, n_layers,
                            out, workspace, ws_bytes, stream, nullptr);
}

namespace sqa {

// Where one call's scratch lies: in a caller's workspace, or in the library's static array.
struct DecodeScratch {
  int32_t* status;     // device-side status word
  char* table;         // room for the layer table when the caller gave no device copy
  int32_t* cnt;        // arrival counters (zero on entry; the kernel leaves them zero)
  float* part;         // partial records of split units
  float* logit;        // H2O logits / probabilities
};

// Argument checks shared by the decode entry points; on success the kernel and the launch plan.
// The launch plan of a call and the dynamic LDS its workgroups need (host arithmetic only).
static bool uses_mfma(sqa_dtype dt, int D, int g) { return dt == SQA_BF16 && D == 128 && g >= kMfmaMinGroup; }
static sqa_status plan_call(sqa_dtype dt, int B, int Hq, int Hkv, int D, bool h2o, const sqa_layer_cache* layers,
                            int n_layers, DecodePlan* plan, size_t* lds_out) {
  const int g = Hq / Hkv;
  const bool mfma = uses_mfma(dt, D, g);
  const sqa_status ps = plan_decode(layers, n_layers, B, Hq, Hkv, D, h2o, true, h2o && mfma, plan);
  if (ps != SQA_OK) return ps;
  const size_t lds_shared = (size_t)g * plan->lds_chunk, lds_waves = (size_t)kDecWaves * g * plan->lds_chunk_w;
  const size_t lds = (h2o ? (lds_shared > lds_waves ? lds_shared : lds_waves) * sizeof(float) : 0) +
                     (mfma ? (size_t)kDecWaves * kStageBytesPerWave : 0) + (size_t)plan->lds_probs;
  // (blocked allocation: the staged block numbers come last; decode_launch passes their offset)
  const size_t lds_all = ((lds + 15) & ~(size_t)15) + (size_t)plan->tbl_entries * sizeof(int);
  if (lds_all > 160 * 1024) return SQA_ERR_CAPACITY;
  *lds_out = lds_all;
  return SQA_OK;
}

static sqa_status decode_prepare(const void* q, const void* k_new, const void* v_new, sqa_dtype dt,
                                 int B, int Hq, int Hkv, int D, int32_t new_pos, sqa_policy policy, int n_sink,
                                 const sqa_layer_cache* layers, int n_layers, const void* out,
                                 const sqa_batch_opts* opts, decode_fn* fn_out, DecodePlan* plan, size_t* lds_out) {
  if (!q || !k_new || !v_new || !layers || !out) return SQA_ERR_NULL;
  if (opts && opts->order != SQA_EVICT_THEN_ATTEND && opts->order != SQA_ATTEND_THEN_EVICT) return SQA_ERR_POLICY;
  if (dt != SQA_F32 && dt != SQA_BF16) return SQA_ERR_DTYPE;
  if (policy != SQA_SLIDING && policy != SQA_STREAMING && policy != SQA_H2O) return SQA_ERR_POLICY;
  if (n_sink < 0) return SQA_ERR_POLICY;
  if (B < 1 || Hq < 1 || Hkv < 1 || n_layers < 1 || n_layers > SQA_MAX_LAYERS || Hq % Hkv != 0 ||
      (new_pos < 0 && !(opts && opts->new_pos_seq)))
    return SQA_ERR_SHAPE;
  const int g = Hq / Hkv;
  const bool h2o = policy == SQA_H2O;
  const bool paged = layers[0].block_table != nullptr;        // blocked K/V allocation: all layers of a call or none
  if (!pick(dt, D, g, h2o, paged)) return SQA_ERR_SHAPE;
  if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out)) return SQA_ERR_SHAPE;
  const int min_budget = h2o ? 2 : (policy == SQA_STREAMING ? n_sink + 1 : 1);
  for (int i = 0; i < n_layers; ++i) {
    const sqa_layer_cache& c = layers[i];
    if (!c.K || !c.V || !c.pos || !c.unit_state) return SQA_ERR_NULL;
    if (h2o && !c.score_acc) return SQA_ERR_NULL;
    if (!aligned16(c.K) || !aligned16(c.V) || !aligned16(c.unit_state)) return SQA_ERR_SHAPE;
    if (c.budget < min_budget) return SQA_ERR_BUDGET;
    if (c.capacity < 1) return SQA_ERR_CAPACITY;
    if ((c.block_table != nullptr) != paged) return SQA_ERR_SHAPE;
    if (paged && (c.unit_offset || c.n_blocks < 1 || c.blocks_per_unit > SQA_MAX_BLOCKS_PER_UNIT ||
                  (int64_t)c.blocks_per_unit * SQA_BLOCK_SLOTS < (c.budget < c.capacity ? c.budget : c.capacity)))
      return SQA_ERR_SHAPE;
  }
  const sqa_status ps = plan_call(dt, B, Hq, Hkv, D, h2o, layers, n_layers, plan, lds_out);
  if (ps != SQA_OK) return ps;
  *fn_out = pick(dt, D, g, h2o, paged);
  return SQA_OK;
}

static sqa_status decode_launch(decode_fn fn, const DecodePlan& plan, size_t lds, const DecodeScratch& sc,
                                const void* q, const void* k_new, const void* v_new,
                                int B, int Hq, int Hkv, int D, int32_t new_pos, sqa_policy policy, int n_sink,
                                const sqa_layer_cache* layers, const sqa_layer_cache* layers_dev, int n_layers,
                                void* out, hipStream_t st, const sqa_batch_opts* opts) {
  if (lds > 64 * 1024) SQA_HIP_CHECK(allow_dynamic_lds(reinterpret_cast<const void*>(fn), lds));
  DecodeArgs a;
  a.q = q; a.k_new = k_new; a.v_new = v_new; a.out = out;
  a.status = sc.status;
  a.cnt = sc.cnt;
  a.part = sc.part;
  a.logit = sc.logit;
  a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.n_layers = n_layers;
  a.new_pos = new_pos; a.policy = (int)policy; a.n_sink = n_sink;
  a.new_pos_seq = opts ? opts->new_pos_seq : nullptr;
  a.budget_seq = opts ? opts->budget_seq : nullptr;
  a.ae = (opts && opts->order == SQA_ATTEND_THEN_EVICT) ? 1 : 0;
  a.lds_chunk = plan.lds_chunk;
  a.lds_chunk_w = plan.lds_chunk_w;
  a.scale_log2 = (float)(1.4426950408889634 / sqrt((double)D));
  // long units first: layers in descending budget (stable)
  for (int i = 0; i < n_layers; ++i) a.order[i] = (uint8_t)i;
  for (int i = 1; i < n_layers; ++i) {
    const uint8_t x = a.order[i];
    int j = i - 1;
    while (j >= 0 && layers[a.order[j]].budget < layers[x].budget) { a.order[j + 1] = a.order[j]; --j; }
    a.order[j + 1] = x;
  }
  uint64_t run = 0;
  for (int i = 0; i < n_layers; ++i) {
    const int l = a.order[i];
    run += plan.wpu[l] ? ((uint64_t)B * Hkv + kDecWaves - 1) / kDecWaves : (uint64_t)B * Hkv * plan.nsplit[l];
    a.blk_end[i] = (uint32_t)run;
    a.lay[i].nsplit = plan.nsplit[i] | (plan.wpu[i] ? kWpuBit : 0u) | ((uint32_t)plan.lds_tiles[i] << kLdsTilesShift);
    a.lay[i].chunk = plan.chunk[i];
    a.lay[i].unit_off = plan.unit_off[i];
    a.lay[i].part_off = plan.part_off[i];
    a.lay[i].logit_off = plan.logit_off[i];
  }
  a.wide_tail = plan.blocks <= (uint64_t)kWideTailMaxBlocks ? 1 : 0;
  a.lds_probs_w = plan.lds_probs_w;
  a.tbl_off = (int)(lds - (size_t)plan.tbl_entries * sizeof(int));
  if (layers_dev) {
    a.layers = layers_dev;
  } else {
    SQA_HIP_CHECK(hipMemcpyAsync(sc.table, layers, (size_t)n_layers * sizeof(sqa_layer_cache), hipMemcpyHostToDevice, st));
    a.layers = reinterpret_cast<const sqa_layer_cache*>(sc.table);
  }
  fn<<<(unsigned)plan.blocks, kDecThreads, lds, st>>>(a);
  SQA_HIP_CHECK(hipGetLastError());
  return SQA_OK;
}

}  // namespace sqa

extern "C" sqa_status sqa_decode_plan(const sqa_layer_cache* layers, int n_layers, int B, int Hq, int Hkv, int D,
                                      sqa_dtype dt, sqa_policy policy, sqa_decode_plan_info* info,
                                      sqa_decode_layer_plan* per_layer) {
  using namespace sqa;
  if (!layers || !info) return SQA_ERR_NULL;
  if (dt != SQA_F32 && dt != SQA_BF16) return SQA_ERR_DTYPE;
  if (policy != SQA_SLIDING && policy != SQA_STREAMING && policy != SQA_H2O) return SQA_ERR_POLICY;
  if (B < 1 || Hq < 1 || Hkv < 1 || n_layers < 1 || n_layers > SQA_MAX_LAYERS || Hq % Hkv != 0) return SQA_ERR_SHAPE;
  const bool h2o = policy == SQA_H2O;
  if (!pick(dt, D, Hq / Hkv, h2o, layers[0].block_table != nullptr)) return SQA_ERR_SHAPE;
  DecodePlan plan;
  size_t lds = 0;
  const sqa_status ps = plan_call(dt, B, Hq, Hkv, D, h2o, layers, n_layers, &plan, &lds);
  if (ps != SQA_OK) return ps;
  info->workgroups = (int64_t)plan.blocks;
  info->workspace_bytes = (int64_t)plan.bytes;
  info->lds_bytes = (int32_t)lds;
  info->matrix_cores = uses_mfma(dt, D, Hq / Hkv) ? 1 : 0;
  info->wide_tail = plan.blocks <= (uint64_t)kWideTailMaxBlocks ? 1 : 0;
  info->table_entries = plan.tbl_entries;
  if (per_layer)
    for (int i = 0; i < n_layers; ++i) {
      per_layer[i].workgroups_per_unit = plan.wpu[i] ? 0 : plan.nsplit[i];
      per_layer[i].slots_per_workgroup = (int32_t)plan.chunk[i];
      per_layer[i].wave_per_unit = plan.wpu[i];
      per_layer[i].probs_in_lds = plan.probs_in_lds[i];
    }
  return SQA_OK;
}

extern "C" sqa_status sqa_decode_step_ex(const void* q, const void* k_new, const void* v_new, sqa_dtype dt,
                                         int B, int Hq, int Hkv, int D, int32_t new_pos,
                                         sqa_policy policy, int n_sink,
                                         const sqa_layer_cache* layers, const sqa_layer_cache* layers_dev, int n_layers,
                                         void* out, void* workspace, size_t ws_bytes, void* stream,
                                         const sqa_batch_opts* opts) {
  using namespace sqa;
  if (!workspace) return SQA_ERR_NULL;
  decode_fn fn = nullptr;
  DecodePlan plan;
  size_t lds = 0;
  const sqa_status ps = decode_prepare(q, k_new, v_new, dt, B, Hq, Hkv, D, new_pos, policy, n_sink, layers, n_layers, out,
                                       opts, &fn, &plan, &lds);
  if (ps != SQA_OK) return ps;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SQA_ERR_SHAPE;
  if (ws_bytes < plan.bytes) return SQA_ERR_CAPACITY;
  char* ws = static_cast<char*>(workspace);
  DecodeScratch sc;
  sc.status = reinterpret_cast<int32_t*>(ws);
  sc.table = ws + plan.off_table;
  sc.cnt = reinterpret_cast<int32_t*>(ws + plan.off_cnt);
  sc.part = reinterpret_cast<float*>(ws + plan.off_part);
  sc.logit = reinterpret_cast<float*>(ws + plan.off_logit);
  return decode_launch(fn, plan, lds, sc, q, k_new, v_new, B, Hq, Hkv, D, new_pos, policy, n_sink, layers, layers_dev,
                       n_layers, out, static_cast<hipStream_t>(stream), opts);
}

// ---- the same step for callers that cannot allocate -------------------------------------------------
// The scratch a decode step needs lives in a file-scope device array instead of a caller's workspace.
// Fixed layout (so that a region only ever holds one kind of data, whatever the shapes of successive
// calls): layer table | arrival counters | partial records and H2O logits / probabilities.
// The counters are the only words that must be zero when a kernel starts.  Their region holds nothing
// else, is cleared once per device at set-up, and every launch returns the counters it used to zero
// (the workgroup that merges a split unit resets the unit's counter), so each call finds them zero
// although the array keeps the previous call's contents everywhere else.
namespace sqa {
constexpr size_t kStaticTableBytes = 16 * 1024;                    // >= SQA_MAX_LAYERS * sizeof(sqa_layer_cache)
constexpr size_t kStaticCntBytes = 1024 * 1024;                    // 262144 units per call
constexpr size_t kStaticDataBytes = SQA_STATIC_SCRATCH_BYTES - kStaticTableBytes - kStaticCntBytes;
static_assert(SQA_MAX_LAYERS * sizeof(sqa_layer_cache) <= kStaticTableBytes, "layer table region");
static_assert(SQA_STATIC_SCRATCH_BYTES > kStaticTableBytes + kStaticCntBytes, "scratch size");
}  // namespace sqa

static __device__ __align__(256) unsigned char scratch[SQA_STATIC_SCRATCH_BYTES];

namespace sqa {
constexpr int kMaxDevices = 64;
// Device address of `scratch` on each device (every GPU holds its own copy of the array at its own
// address; in host code the array's name is only a handle for this lookup, never an address).
static sqa_status static_scratch_base(hipStream_t st, char** base_out) {
  static std::mutex mu;
  static char* base[kMaxDevices] = {};
  int dev = -1;
  SQA_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SQA_ERR_CAPACITY;
  std::lock_guard<std::mutex> lock(mu);
  if (!base[dev]) {
    char* p = nullptr;
    SQA_HIP_CHECK(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)));
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return SQA_ERR_HIP;
    // once per device: the counter region starts at zero (fill kernel, then wait, so that the set-up
    // is complete whatever stream later calls use)
    const sqa_status zs = zero_fill(p + kStaticTableBytes, kStaticCntBytes, st);
    if (zs != SQA_OK) return zs;
    SQA_HIP_CHECK(hipStreamSynchronize(st));
    base[dev] = p;
  }
  *base_out = base[dev];
  return SQA_OK;
}
}  // namespace sqa

extern "C" sqa_status sqa_decode_step_static(const void* q, const void* k_new, const void* v_new, sqa_dtype dt,
                                             int B, int Hq, int Hkv, int D, int32_t new_pos,
                                             sqa_policy policy, int n_sink,
                                             const sqa_layer_cache* layers, const sqa_layer_cache* layers_dev,
                                             int n_layers, void* out, int32_t* status, void* stream,
                                             const sqa_batch_opts* opts) {
  using namespace sqa;
  if (!status) return SQA_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(status) & 3u) return SQA_ERR_SHAPE;
  decode_fn fn = nullptr;
  DecodePlan plan;
  size_t lds = 0;
  const sqa_status ps = decode_prepare(q, k_new, v_new, dt, B, Hq, Hkv, D, new_pos, policy, n_sink, layers, n_layers, out,
                                       opts, &fn, &plan, &lds);
  if (ps != SQA_OK) return ps;
  // beyond the array's fixed size: refused, nothing is enqueued (use sqa_decode_step with a workspace)
  const size_t part_bytes = align256(plan.part_bytes);
  if (plan.cnt_bytes > kStaticCntBytes || part_bytes + plan.logit_bytes > kStaticDataBytes) return SQA_ERR_CAPACITY;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* base = nullptr;
  const sqa_status bs = static_scratch_base(st, &base);
  if (bs != SQA_OK) return bs;
  DecodeScratch sc;
  sc.status = status;
  sc.table = base;
  sc.cnt = reinterpret_cast<int32_t*>(base + kStaticTableBytes);
  sc.part = reinterpret_cast<float*>(base + kStaticTableBytes + kStaticCntBytes);
  sc.logit = reinterpret_cast<float*>(base + kStaticTableBytes + kStaticCntBytes + part_bytes);
  return decode_launch(fn, plan, lds, sc, q, k_new, v_new, B, Hq, Hkv, D, new_pos, policy, n_sink, layers, layers_dev,
                       n_layers, out, st, opts);
}
