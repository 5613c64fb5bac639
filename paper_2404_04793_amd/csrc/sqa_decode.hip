// Decode step over per-layer compact KV caches: Algorithm 1 steps 14-21 with the
// append of Eq. 2-3.  One launch covers every (layer, sequence, KV head) unit of
// the call; a workgroup of 4 waves owns one unit and does, in this order,
//   0. read len / ring head, decide where the new token goes and (cache full)
//      which token is evicted -- H2O: arg-min over the heavy-hitter scores held
//      in LDS against the token leaving the recent ring;
//   1. stream the unit's K and V rows once (16 bytes per lane, 1 KiB per wave
//      load), online softmax in fp32; the logits of the step stay in LDS;
//   2. combine the 4 waves, write out[g][D];
//   3. H2O: score_acc += softmax probabilities (summed over the g query heads)
//      from the LDS logits, one read and one write of the score per token;
//   4. only now touch the cache: move the surviving ring token into the evicted
//      heavy slot, write the new token's rows, pos, lens, ring_head.
// During 1 the two slots that 4 will rewrite are read through a remap (new
// token from k_new/v_new, moved token from its old ring slot), so the cache is
// read-only until every wave has finished reading: no fence is needed and no
// row is read twice.  HBM traffic per unit is the kept rows of K and V once,
// plus 8 bytes of score per token under H2O: the algorithmic minimum.
// There are no atomics; results are bit-identical from run to run.
#include "sqa_common.h"

namespace sqa {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / SQA_WAVE;
constexpr int kUnroll = 4;

struct DecodeArgs {
  const void* q;
  const void* k_new;
  const void* v_new;
  void* out;
  const sqa_layer_cache* layers;   // DEVICE table
  int32_t* status;
  int B, Hq, Hkv, n_layers;
  int new_pos, policy, n_sink;
  float scale_log2;                // log2(e) / sqrt(D)
  uint8_t order[SQA_MAX_LAYERS];   // layers in descending budget (long units start first)
};

// v_exp_f32: 2^x, 1 ulp, denormal results flush to 0 (harmless in a softmax)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int CTRL> __device__ __forceinline__ float dpp_mov(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// sum over the LPR consecutive lanes that share a row; every lane gets the sum
template <int LPR> __device__ __forceinline__ float group_sum(float v) {
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

template <typename T, int D, int G, bool H2O>
__global__ __launch_bounds__(kDecThreads) void decode_unit_kernel(const DecodeArgs a) {
  constexpr int ROWB = D * (int)sizeof(T);        // bytes per K or V row
  constexpr int LPR = ROWB / 16;                  // lanes per row
  constexpr int RPI = SQA_WAVE / LPR;             // rows per wave load
  constexpr int EPL = RowMath<T>::EPL;            // elements per lane
  constexpr int ROWS_IT = kDecWaves * RPI;        // rows per workgroup per load

  extern __shared__ float s_dyn[];                // H2O: score[cap], logit[G][cap]
  __shared__ float s_m[kDecWaves][G], s_l[kDecWaves][G];
  __shared__ float s_acc[kDecWaves][G][D];
  __shared__ float s_red[kDecWaves];
  __shared__ unsigned long long s_red64[kDecWaves];
  __shared__ int s_ctl[4];

  const int tid = threadIdx.x, lane = tid & (SQA_WAVE - 1), wave = tid / SQA_WAVE;
  const int r = lane / LPR, c = lane % LPR;
  const int units_per_layer = a.B * a.Hkv;
  const int layer = a.order[blockIdx.x / units_per_layer];
  const int u = blockIdx.x % units_per_layer;
  const int bidx = u / a.Hkv, kvh = u % a.Hkv;
  const sqa_layer_cache L = a.layers[layer];
  const int cap = L.capacity, budget = L.budget;
  const int len = L.lens[u];
  const int head = L.ring_head[u];
  const int hh = H2O ? budget / 2 : (a.policy == SQA_STREAMING ? min(a.n_sink, budget) : 0);
  const int rec = budget - hh;

  const int64_t qoff = (((int64_t)layer * a.B + bidx) * a.Hq + (int64_t)kvh * G) * D;
  const int64_t kvoff = (((int64_t)layer * a.B + bidx) * a.Hkv + kvh) * D;
  char* outp = reinterpret_cast<char*>(a.out) + qoff * (int64_t)sizeof(T);

  // ---- 0. where does the new token go, who leaves -------------------------
  const bool bad_state = len > budget || len > cap || len < 0 || head < 0 || (len == budget && head >= rec);
  const bool bad_cap = !bad_state && len < budget && len >= cap;
  if (bad_state || bad_cap) {
    for (int i = tid; i < G * D; i += kDecThreads) reinterpret_cast<T*>(outp)[i] = T{};
    if (tid == 0) *a.status = bad_state ? SQA_ERR_STATE : SQA_ERR_CAPACITY;
    return;
  }
  const bool full = len == budget;
  const int n = full ? budget : len + 1;          // tokens attended this step
  const int slot_new = full ? hh + head : len;
  float* s_score = s_dyn;
  float* s_logit = s_dyn + cap;
  int moved_to = -1;                              // heavy slot that receives the ring leaver
  if (H2O) {
    float* sc = L.score_acc + (int64_t)u * cap;
    for (int i = tid; i < len; i += kDecThreads) s_score[i] = sc[i];
    __syncthreads();
    if (full && hh > 0) {
      // worst heavy hitter: lowest score, equal scores -> highest position
      float mn = INFINITY;
      for (int i = tid; i < hh; i += kDecThreads) mn = fminf(mn, s_score[i]);
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) mn = fminf(mn, __shfl_xor(mn, o, SQA_WAVE));
      if (lane == 0) s_red[wave] = mn;
      __syncthreads();
      mn = fminf(fminf(s_red[0], s_red[1]), fminf(s_red[2], s_red[3]));
      const int32_t* posu = L.pos + (int64_t)u * cap;
      unsigned long long best = 0ull;             // (position+1) << 32 | slot
      for (int i = tid; i < hh; i += kDecThreads)
        if (s_score[i] == mn) {
          const unsigned long long key = ((unsigned long long)(uint32_t)(posu[i] + 1) << 32) | (uint32_t)i;
          best = key > best ? key : best;
        }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const unsigned long long other = __shfl_xor(best, o, SQA_WAVE);
        best = other > best ? other : best;
      }
      if (lane == 0) s_red64[wave] = best;
      __syncthreads();
      if (tid == 0) {
        unsigned long long bb = s_red64[0];
        for (int w = 1; w < kDecWaves; ++w) bb = s_red64[w] > bb ? s_red64[w] : bb;
        const int worst = (int)(uint32_t)bb;
        const float leaver = s_score[slot_new];
        int mv = -1;
        if (leaver > mn) { mv = worst; s_score[worst] = leaver; }   // leaver survives, worst heavy hitter goes
        s_score[slot_new] = 0.f;
        s_ctl[0] = mv;
      }
      __syncthreads();
      moved_to = s_ctl[0];
    } else {
      if (tid == 0) s_score[slot_new] = 0.f;
      __syncthreads();
    }
  }

  // ---- 1. stream K and V once, online softmax ------------------------------
  uint4 qf[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
    qf[g] = ld16(reinterpret_cast<const char*>(a.q) + (qoff + (int64_t)g * D) * (int64_t)sizeof(T) + c * 16);

  const char* Kb = reinterpret_cast<const char*>(L.K) + (int64_t)u * cap * ROWB;
  const char* Vb = reinterpret_cast<const char*>(L.V) + (int64_t)u * cap * ROWB;
  const char* knew = reinterpret_cast<const char*>(a.k_new) + kvoff * (int64_t)sizeof(T);
  const char* vnew = reinterpret_cast<const char*>(a.v_new) + kvoff * (int64_t)sizeof(T);

  float m[G], l[G], acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  for (int base = 0; base < n; base += ROWS_IT * kUnroll) {
    uint4 kf[kUnroll], vf[kUnroll];
    int slot[kUnroll];
#pragma unroll
    for (int uu = 0; uu < kUnroll; ++uu) {
      slot[uu] = base + uu * ROWS_IT + wave * RPI + r;
      const int sl = min(slot[uu], n - 1);
      const char* kp = Kb + (int64_t)sl * ROWB;
      const char* vp = Vb + (int64_t)sl * ROWB;
      if (sl == moved_to) { kp = Kb + (int64_t)slot_new * ROWB; vp = Vb + (int64_t)slot_new * ROWB; }
      if (sl == slot_new) { kp = knew; vp = vnew; }
      kf[uu] = ld16_nt(kp + c * 16);
      vf[uu] = ld16_nt(vp + c * 16);
    }
    float s[kUnroll][G];
#pragma unroll
    for (int uu = 0; uu < kUnroll; ++uu)
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = group_sum<LPR>(RowMath<T>::dot(qf[g], kf[uu])) * a.scale_log2;
        d = slot[uu] < n ? d : -INFINITY;
        s[uu][g] = d;
        if (H2O && c == 0 && slot[uu] < n) s_logit[g * cap + slot[uu]] = d;
      }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mx = m[g];
#pragma unroll
      for (int uu = 0; uu < kUnroll; ++uu) mx = fmaxf(mx, s[uu][g]);
      const float ms = mx == -INFINITY ? 0.f : mx;
      const float alpha = fast_exp2(m[g] - ms);
      m[g] = mx;
      float lsum = l[g] * alpha;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= alpha;
#pragma unroll
      for (int uu = 0; uu < kUnroll; ++uu) {
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
      const float lo = __shfl_xor(l[g], o, SQA_WAVE);
      const float mx = fmaxf(m[g], mo);
      const float ms = mx == -INFINITY ? 0.f : mx;
      const float fa = fast_exp2(m[g] - ms), fb = fast_exp2(mo - ms);
      l[g] = l[g] * fa + lo * fb;
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
      for (int e = 0; e < EPL; ++e) s_acc[wave][g][c * EPL + e] = acc[g][e];
    }
  }
  __syncthreads();
  // wave 0, row group g (when G <= RPI) or looping: final m, l and the output row
  for (int g = wave * RPI + r; g < G; g += kDecWaves * RPI) {
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) mx = fmaxf(mx, s_m[w][g]);
    float lt = 0.f, o[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {
      const float f = fast_exp2(s_m[w][g] - mx);      // n >= 1, so mx is finite
      lt += s_l[w][g] * f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] += s_acc[w][g][c * EPL + e] * f;
    }
    const float inv = 1.f / lt;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] *= inv;
    RowMath<T>::store(outp + (int64_t)g * ROWB + c * 16, o);
    if (H2O && c == 0) { s_m[0][g] = mx; s_l[0][g] = inv; }   // broadcast for step 3
  }

  // ---- 3. H2O accumulation from the LDS logits -----------------------------
  if (H2O) {
    __syncthreads();
    float fm[G], fi[G];
#pragma unroll
    for (int g = 0; g < G; ++g) { fm[g] = s_m[0][g]; fi[g] = s_l[0][g]; }
    float* sc = L.score_acc + (int64_t)u * cap;
    for (int i = tid; i < n; i += kDecThreads) {
      float p = 0.f;
#pragma unroll
      for (int g = 0; g < G; ++g) p += fast_exp2(s_logit[g * cap + i] - fm[g]) * fi[g];
      sc[i] = s_score[i] + p;
    }
  } else {
    __syncthreads();   // every wave has finished reading the cache
  }

  // ---- 4. the cache update: moved row, new token, bookkeeping ---------------
  if (wave == 0 && r == 0) {
    char* Kw = const_cast<char*>(Kb);
    char* Vw = const_cast<char*>(Vb);
    if (moved_to >= 0) {
      const uint4 kk = ld16(Kw + (int64_t)slot_new * ROWB + c * 16);
      const uint4 vv = ld16(Vw + (int64_t)slot_new * ROWB + c * 16);
      st16(Kw + (int64_t)moved_to * ROWB + c * 16, kk);
      st16(Vw + (int64_t)moved_to * ROWB + c * 16, vv);
    }
    const uint4 kn = ld16(knew + c * 16), vn = ld16(vnew + c * 16);
    st16(Kw + (int64_t)slot_new * ROWB + c * 16, kn);
    st16(Vw + (int64_t)slot_new * ROWB + c * 16, vn);
    if (c == 0) {
      int32_t* posu = L.pos + (int64_t)u * cap;
      if (moved_to >= 0) posu[moved_to] = posu[slot_new];
      posu[slot_new] = a.new_pos;
      L.lens[u] = n;
      if (full) L.ring_head[u] = head + 1 == rec ? 0 : head + 1;
    }
  }
}

typedef void (*decode_fn)(const DecodeArgs);

template <typename T, int D, bool H2O> decode_fn pick_g(int g) {
  switch (g) {
    case 1: return decode_unit_kernel<T, D, 1, H2O>;
    case 2: return decode_unit_kernel<T, D, 2, H2O>;
    case 4: return decode_unit_kernel<T, D, 4, H2O>;
    case 8: return decode_unit_kernel<T, D, 8, H2O>;
  }
  return nullptr;
}
template <typename T, bool H2O> decode_fn pick_d(int d, int g) {
  if (d == 64) return pick_g<T, 64, H2O>(g);
  if (d == 128) return pick_g<T, 128, H2O>(g);
  return nullptr;
}
static decode_fn pick(sqa_dtype dt, int d, int g, bool h2o) {
  if (dt == SQA_F32) return h2o ? pick_d<float, true>(d, g) : pick_d<float, false>(d, g);
  return h2o ? pick_d<bf16_t, true>(d, g) : pick_d<bf16_t, false>(d, g);
}

constexpr size_t kStatusBytes = 256;

}  // namespace sqa

extern "C" size_t sqa_decode_workspace_bytes(int n_layers) {
  if (n_layers < 1 || n_layers > SQA_MAX_LAYERS) return 0;
  return sqa::kStatusBytes + (size_t)n_layers * sizeof(sqa_layer_cache);
}

extern "C" sqa_status sqa_clear_device_status(void* workspace, void* stream) {
  if (!workspace) return SQA_ERR_NULL;
  SQA_HIP_CHECK(hipMemsetAsync(workspace, 0, sqa::kStatusBytes, static_cast<hipStream_t>(stream)));
  return SQA_OK;
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
  using namespace sqa;
  if (!q || !k_new || !v_new || !layers || !out || !workspace) return SQA_ERR_NULL;
  if (dt != SQA_F32 && dt != SQA_BF16) return SQA_ERR_DTYPE;
  if (policy != SQA_SLIDING && policy != SQA_STREAMING && policy != SQA_H2O) return SQA_ERR_POLICY;
  if (n_sink < 0) return SQA_ERR_POLICY;
  if (B < 1 || Hq < 1 || Hkv < 1 || n_layers < 1 || n_layers > SQA_MAX_LAYERS || Hq % Hkv != 0 || new_pos < 0)
    return SQA_ERR_SHAPE;
  const int g = Hq / Hkv;
  decode_fn fn = pick(dt, D, g, policy == SQA_H2O);
  if (!fn) return SQA_ERR_SHAPE;
  if ((int64_t)n_layers * B * Hkv > INT32_MAX) return SQA_ERR_SHAPE;
  if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out) || !aligned16(workspace))
    return SQA_ERR_SHAPE;
  if (ws_bytes < sqa_decode_workspace_bytes(n_layers)) return SQA_ERR_CAPACITY;
  const int min_budget = policy == SQA_H2O ? 2 : (policy == SQA_STREAMING ? n_sink + 1 : 1);
  int max_cap = 0;
  for (int i = 0; i < n_layers; ++i) {
    const sqa_layer_cache& c = layers[i];
    if (!c.K || !c.V || !c.pos || !c.lens || !c.ring_head) return SQA_ERR_NULL;
    if (policy == SQA_H2O && !c.score_acc) return SQA_ERR_NULL;
    if (!aligned16(c.K) || !aligned16(c.V)) return SQA_ERR_SHAPE;
    if (c.budget < min_budget) return SQA_ERR_BUDGET;
    if (c.capacity < 1) return SQA_ERR_CAPACITY;
    max_cap = c.capacity > max_cap ? c.capacity : max_cap;
  }
  const size_t lds = policy == SQA_H2O ? (size_t)(1 + g) * max_cap * sizeof(float) : 0;
  if (lds > 96 * 1024) return SQA_ERR_CAPACITY;

  hipStream_t st = static_cast<hipStream_t>(stream);
  DecodeArgs a;
  a.q = q; a.k_new = k_new; a.v_new = v_new; a.out = out;
  a.status = static_cast<int32_t*>(workspace);
  a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.n_layers = n_layers;
  a.new_pos = new_pos; a.policy = (int)policy; a.n_sink = n_sink;
  a.scale_log2 = (float)(1.4426950408889634 / sqrt((double)D));
  // long units first: layers in descending budget (stable)
  for (int i = 0; i < n_layers; ++i) a.order[i] = (uint8_t)i;
  for (int i = 1; i < n_layers; ++i) {
    const uint8_t x = a.order[i];
    int j = i - 1;
    while (j >= 0 && layers[a.order[j]].budget < layers[x].budget) { a.order[j + 1] = a.order[j]; --j; }
    a.order[j + 1] = x;
  }
  if (layers_dev) {
    a.layers = layers_dev;
  } else {
    char* tbl = static_cast<char*>(workspace) + kStatusBytes;
    SQA_HIP_CHECK(hipMemcpyAsync(tbl, layers, (size_t)n_layers * sizeof(sqa_layer_cache), hipMemcpyHostToDevice, st));
    a.layers = reinterpret_cast<const sqa_layer_cache*>(tbl);
  }
  if (lds > 48 * 1024)
    SQA_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const unsigned blocks = (unsigned)((int64_t)n_layers * B * Hkv);
  fn<<<blocks, kDecThreads, lds, st>>>(a);
  SQA_HIP_CHECK(hipGetLastError());
  return SQA_OK;
}
