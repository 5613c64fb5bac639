// H2O's accumulated attention over the prompt (Sec. 5.1 "Heavy-Hitter"): column
// sums of the causal softmax(Q K^T / sqrt(D)), added over the g query heads that
// share a KV head.  This is the producer of sqa_prefill_compress's attn_scores.
//
// Two passes over 64x64 logit tiles, fp32 FMA on LDS-staged operands:
//   pass 1  one workgroup per (head, 64 query rows): running max and sum of
//           each softmax row over the key tiles up to the diagonal;
//   pass 2  one workgroup per (KV head, 64 key columns): for the g heads and
//           all query tiles from the diagonal down, p = exp(s - m_i) / l_i is
//           summed down the columns in registers; one fixed-order reduction
//           over the 16 row groups at the end.  No atomics.
// The P x P probabilities never reach HBM: traffic is Q and K re-read per tile
// (L2 resident), so the bound is arithmetic (2 * 2*P^2/2*D flops per head).
#include "sqa_common.h"

namespace sqa {

constexpr int kScThreads = 256;
constexpr int kTile = 64;        // rows and columns of a logit tile
constexpr int kDK = 32;          // slab of the head dimension staged per step
constexpr int kLd = kTile + 4;   // LDS row stride (floats) of the [kDK][kTile] slabs

template <typename T> __device__ __forceinline__ void load8(const T* p, float* o);
template <> __device__ __forceinline__ void load8<float>(const float* p, float* o) {
  const uint4 a = ld16(p), b = ld16(p + 4);
  o[0] = __uint_as_float(a.x); o[1] = __uint_as_float(a.y); o[2] = __uint_as_float(a.z); o[3] = __uint_as_float(a.w);
  o[4] = __uint_as_float(b.x); o[5] = __uint_as_float(b.y); o[6] = __uint_as_float(b.z); o[7] = __uint_as_float(b.w);
}
template <> __device__ __forceinline__ void load8<bf16_t>(const bf16_t* p, float* o) {
  const uint4 a = ld16(p);
  o[0] = bf16_lo(a.x); o[1] = bf16_hi(a.x); o[2] = bf16_lo(a.y); o[3] = bf16_hi(a.y);
  o[4] = bf16_lo(a.z); o[5] = bf16_hi(a.z); o[6] = bf16_lo(a.w); o[7] = bf16_hi(a.w);
}

// s[4][4] (rows ty*4.., cols tx*4..) = Q[row0.., :] . K[col0.., :]^T, both [P][D] row-major
template <typename T, int D>
__device__ __forceinline__ void logit_tile(const T* __restrict__ Q, const T* __restrict__ K, int P, int row0, int col0,
                                           float (*Qs)[kLd], float (*Ks)[kLd], float s[4][4]) {
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) s[i][j] = 0.f;
  const int lr = tid / 4, lk = (tid % 4) * 8;     // this thread stages row lr, 8 elements from lk
  for (int d0 = 0; d0 < D; d0 += kDK) {
    float qv[8], kv[8];
    const int qr = min(row0 + lr, P - 1), kr = min(col0 + lr, P - 1);
    load8<T>(Q + (int64_t)qr * D + d0 + lk, qv);
    load8<T>(K + (int64_t)kr * D + d0 + lk, kv);
    __syncthreads();                               // previous slab fully consumed
#pragma unroll
    for (int e = 0; e < 8; ++e) { Qs[lk + e][lr] = qv[e]; Ks[lk + e][lr] = kv[e]; }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < kDK; ++kk) {
      const float4 a = *reinterpret_cast<const float4*>(&Qs[kk][ty * 4]);
      const float4 b = *reinterpret_cast<const float4*>(&Ks[kk][tx * 4]);
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) s[i][j] = fmaf(av[i], bv[j], s[i][j]);
    }
  }
}

template <int CTRL> __device__ __forceinline__ float dpp16(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp16<0xB1>(v)); v = fmaxf(v, dpp16<0x4E>(v));
  v = fmaxf(v, dpp16<0x141>(v)); v = fmaxf(v, dpp16<0x140>(v));
  return v;
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp16<0xB1>(v); v += dpp16<0x4E>(v); v += dpp16<0x141>(v); v += dpp16<0x140>(v);
  return v;
}

template <typename T, int D>
__global__ __launch_bounds__(kScThreads) void score_rowstats_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, int Hq, int Hkv, int P, float scale_log2,
    float2* __restrict__ stats /*[B*Hq][P] (max, 1/sum) in the exp2 domain*/) {
  __shared__ __attribute__((aligned(16))) float Qs[kDK][kLd];
  __shared__ __attribute__((aligned(16))) float Ks[kDK][kLd];
  const int bh = blockIdx.y, b = bh / Hq, h = bh % Hq, kvh = h / (Hq / Hkv);
  const T* Qh = Q + (int64_t)bh * P * D;
  const T* Kh = K + ((int64_t)b * Hkv + kvh) * P * D;
  const int row0 = blockIdx.x * kTile;
  const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;
  float m[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { m[i] = -INFINITY; l[i] = 0.f; }
  for (int col0 = 0; col0 <= row0; col0 += kTile) {
    float s[4][4];
    logit_tile<T, D>(Qh, Kh, P, row0, col0, Qs, Ks, s);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = row0 + ty * 4 + i;
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = col0 + tx * 4 + j;
        s[i][j] = (col <= row && col < P) ? s[i][j] * scale_log2 : -INFINITY;
        mx = fmaxf(mx, s[i][j]);
      }
      mx = fmaxf(row16_max(mx), m[i]);
      const float ms = mx == -INFINITY ? 0.f : mx;
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) sum += __builtin_amdgcn_exp2f(s[i][j] - ms);
      sum = row16_sum(sum);
      l[i] = l[i] * __builtin_amdgcn_exp2f(m[i] - ms) + sum;
      m[i] = mx;
    }
  }
  if (tx == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = row0 + ty * 4 + i;
      if (row < P) stats[(int64_t)bh * P + row] = make_float2(m[i], 1.f / l[i]);
    }
  }
}

template <typename T, int D>
__global__ __launch_bounds__(kScThreads) void score_colsum_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, int Hq, int Hkv, int P, float scale_log2,
    const float2* __restrict__ stats, float* __restrict__ scores /*[B*Hkv][P]*/) {
  __shared__ __attribute__((aligned(16))) float Qs[kDK][kLd];
  __shared__ __attribute__((aligned(16))) float Ks[kDK][kLd];
  __shared__ float s_col[16][kTile];
  const int bk = blockIdx.y, b = bk / Hkv, kvh = bk % Hkv, g = Hq / Hkv;
  const T* Kh = K + (int64_t)bk * P * D;
  const int col0 = blockIdx.x * kTile;
  const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;
  float colsum[4] = {0.f, 0.f, 0.f, 0.f};
  for (int hg = 0; hg < g; ++hg) {
    const int64_t bh = (int64_t)b * Hq + (int64_t)kvh * g + hg;
    const T* Qh = Q + bh * P * D;
    for (int row0 = col0; row0 < P; row0 += kTile) {
      float s[4][4];
      logit_tile<T, D>(Qh, Kh, P, row0, col0, Qs, Ks, s);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = row0 + ty * 4 + i;
        const float2 st = stats[bh * P + min(row, P - 1)];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int col = col0 + tx * 4 + j;
          const float p = __builtin_amdgcn_exp2f(s[i][j] * scale_log2 - st.x) * st.y;
          colsum[j] += (row < P && col <= row) ? p : 0.f;
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) s_col[ty][tx * 4 + j] = colsum[j];
  __syncthreads();
  if (threadIdx.x < kTile) {
    float t = 0.f;
#pragma unroll
    for (int y = 0; y < 16; ++y) t += s_col[y][threadIdx.x];
    const int col = col0 + threadIdx.x;
    if (col < P) scores[(int64_t)bk * P + col] = t;
  }
}

template <typename T, int D>
static void launch_scores(const void* Q, const void* K, int B, int Hq, int Hkv, int P, float* scores, float2* stats,
                          hipStream_t st) {
  const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)D));
  const int tiles = (P + kTile - 1) / kTile;
  score_rowstats_kernel<T, D><<<dim3(tiles, B * Hq), kScThreads, 0, st>>>(
      static_cast<const T*>(Q), static_cast<const T*>(K), Hq, Hkv, P, scale_log2, stats);
  score_colsum_kernel<T, D><<<dim3(tiles, B * Hkv), kScThreads, 0, st>>>(
      static_cast<const T*>(Q), static_cast<const T*>(K), Hq, Hkv, P, scale_log2, stats, scores);
}

}  // namespace sqa

extern "C" size_t sqa_prefill_scores_workspace_bytes(int B, int Hq, int Hkv, int P, int D) {
  (void)Hkv; (void)D;
  if (B < 1 || Hq < 1 || P < 1) return 0;
  return (size_t)B * Hq * P * sizeof(float2);
}

extern "C" sqa_status sqa_prefill_scores(const void* Q, const void* K, sqa_dtype dt,
                                         int B, int Hq, int Hkv, int P, int D,
                                         float* scores_out, void* workspace, size_t ws_bytes, void* stream) {
  using namespace sqa;
  if (!Q || !K || !scores_out || !workspace) return SQA_ERR_NULL;
  if (dt != SQA_F32 && dt != SQA_BF16) return SQA_ERR_DTYPE;
  if (B < 1 || Hq < 1 || Hkv < 1 || P < 1 || Hq % Hkv != 0 || (D != 64 && D != 128)) return SQA_ERR_SHAPE;
  if ((int64_t)B * Hq > 65535) return SQA_ERR_SHAPE;
  if (!aligned16(Q) || !aligned16(K) || (reinterpret_cast<uintptr_t>(workspace) & 7u)) return SQA_ERR_SHAPE;
  if (ws_bytes < sqa_prefill_scores_workspace_bytes(B, Hq, Hkv, P, D)) return SQA_ERR_CAPACITY;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float2* stats = static_cast<float2*>(workspace);
  if (dt == SQA_F32) {
    if (D == 64) launch_scores<float, 64>(Q, K, B, Hq, Hkv, P, scores_out, stats, st);
    else launch_scores<float, 128>(Q, K, B, Hq, Hkv, P, scores_out, stats, st);
  } else {
    if (D == 64) launch_scores<bf16_t, 64>(Q, K, B, Hq, Hkv, P, scores_out, stats, st);
    else launch_scores<bf16_t, 128>(Q, K, B, Hq, Hkv, P, scores_out, stats, st);
  }
  SQA_HIP_CHECK(hipGetLastError());
  return SQA_OK;
}
