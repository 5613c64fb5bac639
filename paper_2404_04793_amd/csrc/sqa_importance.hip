// Layer-importance probe: Algorithm 1 steps 1-4 with the cosine-similarity
// equation of Sec. 3.  A pure streaming reduction (each hidden-state element is
// read once), so the only roofline is HBM bandwidth.
//
// Mapping: grid = (blocks per layer, layers); a workgroup has 4 waves; a wave
// owns whole token rows (row = wave id, stepping by the number of waves of the
// layer) and its 64 lanes read the row in 16-byte pieces, 1 KiB per wave load.
// The three dot products accumulate in fp32 per lane, are summed over the wave,
// and lane 0 adds the row's cosine to a per-wave fp64 sum.  Partial sums go to
// the workspace and a second tiny kernel adds them in a fixed order: no atomics,
// results are bit-identical from run to run.
//
// The same kernel also runs fused into the producer of the "after" tensor: the
// residual connection h_out = h_in + attn_out.  Then it reads h_in and attn_out,
// writes h_out rounded to the storage type, and takes the cosine against those
// stored values in the same pass, so the probe itself moves no extra byte.
#include "sqa_common.h"

namespace sqa {

constexpr int kImpThreads = 256;
constexpr int kImpWaves = kImpThreads / SQA_WAVE;
constexpr int kImpMaxBlocks = 1024;   // partial sums per layer

template <typename T> struct Dots;
template <> struct Dots<float> {
  static __device__ __forceinline__ void acc(const uint4& a, const uint4& b, float& ab, float& aa, float& bb) {
    const float a0 = __uint_as_float(a.x), a1 = __uint_as_float(a.y), a2 = __uint_as_float(a.z), a3 = __uint_as_float(a.w);
    const float b0 = __uint_as_float(b.x), b1 = __uint_as_float(b.y), b2 = __uint_as_float(b.z), b3 = __uint_as_float(b.w);
    ab = fmaf(a0, b0, ab); ab = fmaf(a1, b1, ab); ab = fmaf(a2, b2, ab); ab = fmaf(a3, b3, ab);
    aa = fmaf(a0, a0, aa); aa = fmaf(a1, a1, aa); aa = fmaf(a2, a2, aa); aa = fmaf(a3, a3, aa);
    bb = fmaf(b0, b0, bb); bb = fmaf(b1, b1, bb); bb = fmaf(b2, b2, bb); bb = fmaf(b3, b3, bb);
  }
};
template <> struct Dots<bf16_t> {
  static __device__ __forceinline__ void acc(const uint4& a, const uint4& b, float& ab, float& aa, float& bb) {
    ab = dot2_bf16(a.x, b.x, ab); ab = dot2_bf16(a.y, b.y, ab); ab = dot2_bf16(a.z, b.z, ab); ab = dot2_bf16(a.w, b.w, ab);
    aa = dot2_bf16(a.x, a.x, aa); aa = dot2_bf16(a.y, a.y, aa); aa = dot2_bf16(a.z, a.z, aa); aa = dot2_bf16(a.w, a.w, aa);
    bb = dot2_bf16(b.x, b.x, bb); bb = dot2_bf16(b.y, b.y, bb); bb = dot2_bf16(b.z, b.z, bb); bb = dot2_bf16(b.w, b.w, bb);
  }
};

// a + r element by element: fp32 add, rounded to the storage type
template <typename T> struct Residual;
template <> struct Residual<float> {
  static __device__ __forceinline__ uint4 add(const uint4& a, const uint4& r) {
    return make_uint4(__float_as_uint(__uint_as_float(a.x) + __uint_as_float(r.x)),
                      __float_as_uint(__uint_as_float(a.y) + __uint_as_float(r.y)),
                      __float_as_uint(__uint_as_float(a.z) + __uint_as_float(r.z)),
                      __float_as_uint(__uint_as_float(a.w) + __uint_as_float(r.w)));
  }
};
template <> struct Residual<bf16_t> {
  static __device__ __forceinline__ uint32_t add2(uint32_t a, uint32_t r) {
    return f32_to_bf16_bits(bf16_lo(a) + bf16_lo(r)) | (f32_to_bf16_bits(bf16_hi(a) + bf16_hi(r)) << 16);
  }
  static __device__ __forceinline__ uint4 add(const uint4& a, const uint4& r) {
    return make_uint4(add2(a.x, r.x), add2(a.y, r.y), add2(a.z, r.z), add2(a.w, r.w));
  }
};

// FUSE = false: h_out is read.  FUSE = true: `other` is attn_out and h_out is written.
template <typename T, bool FUSE>
__global__ __launch_bounds__(kImpThreads) void importance_partial_kernel(
    const T* h_in, const T* other, T* h_out_w /*may be h_in or other*/, int64_t n_tokens, int hidden,
    const int32_t* __restrict__ seq_start /*[gridDim.z + 1] or NULL*/,
    double* __restrict__ partial /*[layers][gridDim.z][gridDim.x]*/) {
  constexpr int E = elem<T>::per16;
  const int lane = threadIdx.x & (SQA_WAVE - 1);
  const int wave = threadIdx.x / SQA_WAVE;
  const int layer = blockIdx.y;
  const int64_t row_elems = hidden;
  const char* A = reinterpret_cast<const char*>(h_in + (int64_t)layer * n_tokens * row_elems);
  const char* Bp = reinterpret_cast<const char*>(other + (int64_t)layer * n_tokens * row_elems);
  char* Wp = FUSE ? reinterpret_cast<char*>(h_out_w + (int64_t)layer * n_tokens * row_elems) : nullptr;
  const int chunks = hidden / E;                 // 16-byte pieces per row
  const int64_t row_bytes = row_elems * (int64_t)sizeof(T);
  const int64_t stride = (int64_t)gridDim.x * kImpWaves;

  // rows of this (layer, sequence): all of the layer's unless the tokens are segmented
  int64_t row_lo = 0, row_hi = n_tokens;
  if (seq_start) {
    row_lo = seq_start[blockIdx.z];
    row_hi = seq_start[blockIdx.z + 1];
    row_lo = row_lo < 0 ? 0 : row_lo;
    row_hi = row_hi > n_tokens ? n_tokens : row_hi;
  }
  double wave_cos = 0.0;
  for (int64_t row = row_lo + (int64_t)blockIdx.x * kImpWaves + wave; row < row_hi; row += stride) {
    const char* a = A + row * row_bytes;
    const char* b = Bp + row * row_bytes;
    char* w = FUSE ? Wp + row * row_bytes : nullptr;
    float ab = 0.f, aa = 0.f, bb = 0.f;
    int c = lane;
    for (; c + 3 * SQA_WAVE < chunks; c += 4 * SQA_WAVE) {      // 8 loads in flight per lane
      const uint4 a0 = ld16_nt(a + (int64_t)c * 16);
      uint4 b0 = ld16_nt(b + (int64_t)c * 16);
      const uint4 a1 = ld16_nt(a + (int64_t)(c + SQA_WAVE) * 16);
      uint4 b1 = ld16_nt(b + (int64_t)(c + SQA_WAVE) * 16);
      const uint4 a2 = ld16_nt(a + (int64_t)(c + 2 * SQA_WAVE) * 16);
      uint4 b2 = ld16_nt(b + (int64_t)(c + 2 * SQA_WAVE) * 16);
      const uint4 a3 = ld16_nt(a + (int64_t)(c + 3 * SQA_WAVE) * 16);
      uint4 b3 = ld16_nt(b + (int64_t)(c + 3 * SQA_WAVE) * 16);
      if (FUSE) {
        b0 = Residual<T>::add(a0, b0); b1 = Residual<T>::add(a1, b1);
        b2 = Residual<T>::add(a2, b2); b3 = Residual<T>::add(a3, b3);
        st16(w + (int64_t)c * 16, b0); st16(w + (int64_t)(c + SQA_WAVE) * 16, b1);
        st16(w + (int64_t)(c + 2 * SQA_WAVE) * 16, b2); st16(w + (int64_t)(c + 3 * SQA_WAVE) * 16, b3);
      }
      Dots<T>::acc(a0, b0, ab, aa, bb); Dots<T>::acc(a1, b1, ab, aa, bb);
      Dots<T>::acc(a2, b2, ab, aa, bb); Dots<T>::acc(a3, b3, ab, aa, bb);
    }
    for (; c < chunks; c += SQA_WAVE) {
      const uint4 a0 = ld16_nt(a + (int64_t)c * 16);
      uint4 b0 = ld16_nt(b + (int64_t)c * 16);
      if (FUSE) { b0 = Residual<T>::add(a0, b0); st16(w + (int64_t)c * 16, b0); }
      Dots<T>::acc(a0, b0, ab, aa, bb);
    }
    ab = wave_sum(ab); aa = wave_sum(aa); bb = wave_sum(bb);
    const double na = fmax(sqrt((double)aa), 1e-8), nb = fmax(sqrt((double)bb), 1e-8);
    wave_cos += (double)ab / (na * nb);
  }
  __shared__ double s_part[kImpWaves];
  if (lane == 0) s_part[wave] = wave_cos;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int w = 0; w < kImpWaves; ++w) s += s_part[w];
    partial[((int64_t)layer * gridDim.z + blockIdx.z) * gridDim.x + blockIdx.x] = s;
  }
}

// one wave per (layer, sequence): blockIdx.x = layer * n_seq + sequence
__global__ __launch_bounds__(SQA_WAVE) void importance_final_kernel(
    const double* __restrict__ partial, int n_part, int64_t n_tokens, const int32_t* __restrict__ seq_start, int n_seq,
    float* __restrict__ cos_out) {
  const int item = blockIdx.x;
  const int lane = threadIdx.x;
  double s = 0.0;
  for (int i = lane; i < n_part; i += SQA_WAVE) s += partial[(int64_t)item * n_part + i];
  s = wave_sum(s);
  int64_t rows = n_tokens;
  if (seq_start) {
    const int q = item % n_seq;
    int64_t lo = seq_start[q], hi = seq_start[q + 1];
    lo = lo < 0 ? 0 : lo;
    hi = hi > n_tokens ? n_tokens : hi;
    rows = hi - lo;
  }
  if (lane == 0) cos_out[item] = rows > 0 ? (float)(s / (double)rows) : 0.f;
}

static int imp_blocks(int64_t n_tokens) {
  int64_t b = (n_tokens + kImpWaves - 1) / kImpWaves;
  return (int)(b < kImpMaxBlocks ? b : kImpMaxBlocks);
}

}  // namespace sqa

extern "C" size_t sqa_layer_importance_workspace_bytes(int n_layers, int64_t n_tokens, int hidden) {
  (void)hidden;
  if (n_layers < 1 || n_tokens < 1) return 0;
  return (size_t)n_layers * sqa::imp_blocks(n_tokens) * sizeof(double);
}

namespace sqa {
static sqa_status launch_importance(const void* h_in, const void* other, void* h_out_w, sqa_dtype dt,
                                    int n_layers, int64_t n_tokens, int hidden, const int32_t* seq_start, int n_seq,
                                    float* cos_out, void* workspace, size_t ws_bytes, void* stream) {
  const bool fuse = h_out_w != nullptr;
  if (!h_in || !other || !cos_out || !workspace) return SQA_ERR_NULL;
  if (dt != SQA_F32 && dt != SQA_BF16) return SQA_ERR_DTYPE;
  if (n_layers < 1 || n_layers > 65535 || n_tokens < 1 || hidden < 8 || hidden % 8 != 0) return SQA_ERR_SHAPE;
  if (n_seq < 1 || n_seq > 65535 || (int64_t)n_layers * n_seq > INT32_MAX) return SQA_ERR_SHAPE;
  if (!aligned16(h_in) || !aligned16(other) || !aligned16(h_out_w) || (reinterpret_cast<uintptr_t>(workspace) & 7u))
    return SQA_ERR_SHAPE;
  if (ws_bytes < (size_t)n_seq * sqa_layer_importance_workspace_bytes(n_layers, n_tokens, hidden)) return SQA_ERR_CAPACITY;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int nblk = imp_blocks(n_tokens);
  double* partial = static_cast<double*>(workspace);
  dim3 grid(nblk, n_layers, n_seq);
  if (dt == SQA_F32) {
    const float* a = static_cast<const float*>(h_in);
    const float* b = static_cast<const float*>(other);
    float* w = static_cast<float*>(h_out_w);
    if (fuse) importance_partial_kernel<float, true><<<grid, kImpThreads, 0, st>>>(a, b, w, n_tokens, hidden, seq_start, partial);
    else importance_partial_kernel<float, false><<<grid, kImpThreads, 0, st>>>(a, b, w, n_tokens, hidden, seq_start, partial);
  } else {
    const bf16_t* a = static_cast<const bf16_t*>(h_in);
    const bf16_t* b = static_cast<const bf16_t*>(other);
    bf16_t* w = static_cast<bf16_t*>(h_out_w);
    if (fuse) importance_partial_kernel<bf16_t, true><<<grid, kImpThreads, 0, st>>>(a, b, w, n_tokens, hidden, seq_start, partial);
    else importance_partial_kernel<bf16_t, false><<<grid, kImpThreads, 0, st>>>(a, b, w, n_tokens, hidden, seq_start, partial);
  }
  SQA_HIP_CHECK(hipGetLastError());
  importance_final_kernel<<<n_layers * n_seq, SQA_WAVE, 0, st>>>(partial, nblk, n_tokens, seq_start, n_seq, cos_out);
  SQA_HIP_CHECK(hipGetLastError());
  return SQA_OK;
}
}  // namespace sqa

extern "C" sqa_status sqa_layer_importance(const void* h_in, const void* h_out, sqa_dtype dt,
                                           int n_layers, int64_t n_tokens, int hidden,
                                           float* cos_out, void* workspace, size_t ws_bytes, void* stream) {
  return sqa::launch_importance(h_in, h_out, nullptr, dt, n_layers, n_tokens, hidden, nullptr, 1, cos_out, workspace,
                                ws_bytes, stream);
}

extern "C" sqa_status sqa_layer_importance_seq(const void* h_in, const void* h_out, sqa_dtype dt,
                                               int n_layers, int64_t n_tokens, int hidden,
                                               const int32_t* seq_start, int n_seq,
                                               float* cos_out, void* workspace, size_t ws_bytes, void* stream) {
  if (!seq_start) return SQA_ERR_NULL;
  return sqa::launch_importance(h_in, h_out, nullptr, dt, n_layers, n_tokens, hidden, seq_start, n_seq, cos_out,
                                workspace, ws_bytes, stream);
}

extern "C" sqa_status sqa_residual_add_importance(const void* h_in, const void* attn_out, void* h_out, sqa_dtype dt,
                                                  int n_layers, int64_t n_tokens, int hidden,
                                                  float* cos_out, void* workspace, size_t ws_bytes, void* stream) {
  if (!h_out) return SQA_ERR_NULL;
  return sqa::launch_importance(h_in, attn_out, h_out, dt, n_layers, n_tokens, hidden, nullptr, 1, cos_out, workspace,
                                ws_bytes, stream);
}
