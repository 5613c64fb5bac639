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

constexpr int kScBlocksPerWave = 2;   // 16-row blocks a wave of the matrix-core kernels keeps in registers (4: no faster)
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

// Which (tile, head) a workgroup of a 1-D launch works on.  Consecutive workgroups go to the 8 XCDs of the
// chip in turn, each with an L2 of its own; all tiles of a head re-read that head's K (or Q) rows, so a head
// (with the `per` query heads that share its K rows) is given to one XCD (group mod 8) and an XCD walks its
// groups one after the other, the tile with the most work first: the rows are then fetched into one L2 once
// instead of into all eight.  Measured at the 7B shape: 0.45 -> 0.30 ms and 0.54 -> 0.35 ms per layer.
__device__ __forceinline__ bool xcd_tile_head(int tiles, int heads, int per, bool heavy_is_last, int& tile, int& head) {
  const int n = blockIdx.x, xcd = n & 7, slot = n >> 3;
  const int group = (slot / (tiles * per)) * 8 + xcd, rem = slot % (tiles * per);
  head = group * per + rem / tiles;
  const int t = rem % tiles;
  tile = heavy_is_last ? tiles - 1 - t : t;
  return head < heads;
}

template <typename T, int D>
__global__ __launch_bounds__(kScThreads) void score_rowstats_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, int Hq, int Hkv, int P, float scale_log2,
    int tiles, int heads, float2* __restrict__ stats /*[B*Hq][P] (max, 1/sum) in the exp2 domain*/) {
  __shared__ __attribute__((aligned(16))) float Qs[kDK][kLd];
  __shared__ __attribute__((aligned(16))) float Ks[kDK][kLd];
  int tile_x, bh;
  if (!xcd_tile_head(tiles, heads, Hq / Hkv, true, tile_x, bh)) return;
  const int b = bh / Hq, h = bh % Hq, kvh = h / (Hq / Hkv);
  const T* Qh = Q + (int64_t)bh * P * D;
  const T* Kh = K + ((int64_t)b * Hkv + kvh) * P * D;
  const int row0 = tile_x * kTile;
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
    const float2* __restrict__ stats, const int32_t* __restrict__ prompt_len /*[B] or NULL*/,
    int tiles, int heads, float* __restrict__ scores /*[B*Hkv][P]*/) {
  __shared__ __attribute__((aligned(16))) float Qs[kDK][kLd];
  __shared__ __attribute__((aligned(16))) float Ks[kDK][kLd];
  __shared__ float s_col[16][kTile];
  int tile_x, bk;
  if (!xcd_tile_head(tiles, heads, 1, false, tile_x, bk)) return;
  const int b = bk / Hkv, kvh = bk % Hkv, g = Hq / Hkv;
  const int Pq = prompt_len ? max(0, min(prompt_len[b], P)) : P;   // queries beyond the sequence's own prompt are padding
  const T* Kh = K + (int64_t)bk * P * D;
  const int col0 = tile_x * kTile;
  const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;
  float colsum[4] = {0.f, 0.f, 0.f, 0.f};
  for (int hg = 0; hg < g; ++hg) {
    const int64_t bh = (int64_t)b * Hq + (int64_t)kvh * g + hg;
    const T* Qh = Q + bh * P * D;
    for (int row0 = col0; row0 < Pq; row0 += kTile) {
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
          colsum[j] += (row < Pq && col <= row) ? p : 0.f;
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

// ---------------------------------------------------------------------------
// bf16, D = 128: the same two passes on the matrix cores.
//   v_mfma_f32_16x16x32_bf16: A row / B column = lane%16, contraction slots of
//   a lane = 8*(lane/16)+e; C column = lane%16, rows 4*(lane/16)+i.  For both
//   operands slot (j,e) of step i stands for d = 32j + 8i + e, so a lane's four
//   fragments are 64 contiguous bytes of its row.
//   pass 1  S^T = K.Q^T: a wave keeps NB blocks of 16 query rows as B operands
//           in registers (block b of wave w = rows 16 (w + 4 b) of the
//           workgroup's 64 NB rows, so the diagonal's work is spread evenly);
//           64-key tiles of K go from global memory straight into LDS (direct
//           loads, no register staging; 16-byte pieces XOR-swizzled by the row;
//           two buffers) and are shared by the 4 waves.  Every fragment read
//           from LDS feeds NB products.  A lane sees 4 keys of one query per
//           product and keeps a running (reference, sum) of its own; the 4
//           lanes of a query merge once at the end and store
//           c_i = m_i + log2(l_i), so that pass 2 needs one value per row.
//   pass 2  S = Q.K^T: a wave keeps NB blocks of 16 keys as B operands; 64-row
//           tiles of Q and their c_i are staged in LDS the same way; a lane
//           sees 4 query rows of one key per product and adds exp2(s - c_i)
//           into a per-lane column sum over all row tiles and all g heads.
// Per 16x16 block a lane issues 4 products (64 cycles of the matrix pipeline)
// and at least 4 x (multiply-add, exp2, add); on this chip vector instructions
// hide only partly behind matrix instructions of the same SIMD (measured: 16
// products + 16 such triples take 466 cycles with 4 waves per SIMD, 268 and 297
// on their own), so the two passes are bound by the sum of both, not by the
// products: 31 % of the matrix pipeline's cycles are busy.
typedef __bf16 sc_bf16x8_t __attribute__((ext_vector_type(8)));
typedef float sc_f32x4_t __attribute__((ext_vector_type(4)));
constexpr int kMT = 64;                 // rows of a staged tile
constexpr int kMPitch = 256;            // LDS bytes per staged row; 16-byte piece c of row R lies at piece c ^ (R % 16)
constexpr int kMTileBytes = kMT * kMPitch;
constexpr float kRefFar = 65536.f;       // a row's reference moves when 4 exponentials against it add up to this

typedef __attribute__((address_space(1))) const void sc_gptr_t;
typedef __attribute__((address_space(3))) void sc_lptr_t;
// Copy one [64 x 128] bf16 tile (rows row0.., clamped to P-1) straight into LDS, swizzled: each wave
// instruction fills 1 KB = 4 rows, lane l the 16-byte position l%16 of row l/16 of them, so it fetches the
// piece that belongs there (the permutation stays inside a 256-byte row: the access is still coalesced).
__device__ __forceinline__ void tile_to_lds(const bf16_t* __restrict__ src, int row0, int P, char* lds) {
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int rr = 4 * wave + (lane >> 4);            // row within a group of 16
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = min(row0 + 16 * i + rr, P - 1);
    const bf16_t* g = src + (int64_t)row * 128 + (((lane & 15) ^ rr) * 8);
    __builtin_amdgcn_global_load_lds((sc_gptr_t*)g, (sc_lptr_t*)(lds + (16 * i + 4 * wave) * kMPitch), 16, 0, 0);
  }
}
// the four fragments of row `row` (global memory) for a lane with contraction group j
__device__ __forceinline__ void row_fragments(const bf16_t* __restrict__ src, int row, int j, sc_bf16x8_t (&fr)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) fr[i] = __builtin_bit_cast(sc_bf16x8_t, ld16(src + (int64_t)row * 128 + 32 * j + 8 * i));
}
// the A fragments of rows 16 sub .. 16 sub + 15 of a staged tile
__device__ __forceinline__ void tile_fragments(const char* lds, int sub, sc_bf16x8_t (&fr)[4]) {
  const int lane = threadIdx.x & 63;
  const char* p = lds + (16 * sub + (lane & 15)) * kMPitch;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    fr[i] = __builtin_bit_cast(sc_bf16x8_t, *reinterpret_cast<const uint4*>(p + (((4 * (lane >> 4) + i) ^ (lane & 15)) * 16)));
}
__device__ __forceinline__ sc_f32x4_t block_product(const sc_bf16x8_t (&afr)[4], const sc_bf16x8_t (&bfr)[4]) {
  sc_f32x4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afr[i], bfr[i], c, 0, 0, 0);
  return c;
}

template <int NB>
__global__ __launch_bounds__(kScThreads) void score_rowstats_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, int Hq, int Hkv, int P, float scale_log2,
    int tiles, int heads, float* __restrict__ cstat /*[B*Hq][P]: m_i + log2(l_i) in the exp2 domain*/) {
  extern __shared__ char s_tiles[];                 // 2 x [64][kMPitch]
  constexpr int OWN = kMT * NB;                     // query rows of a workgroup
  int tile_x, bh;
  if (!xcd_tile_head(tiles, heads, Hq / Hkv, true, tile_x, bh)) return;   // (query tile t reads key tiles 0..t: the last is the longest)
  const int b = bh / Hq, h = bh % Hq, kvh = h / (Hq / Hkv);
  const bf16_t* Qh = Q + (int64_t)bh * P * 128;
  const bf16_t* Kh = K + ((int64_t)b * Hkv + kvh) * P * 128;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n16 = lane & 15, j4 = lane >> 4;
  const int r0 = tile_x * OWN + 16 * wave;          // first row of own block 0; block bb starts at r0 + 64 bb
  sc_bf16x8_t qfr[NB][4];
  float m_run[NB], l_run[NB];
#pragma unroll
  for (int bb = 0; bb < NB; ++bb) {
    row_fragments(Qh, min(r0 + 64 * bb + n16, P - 1), j4, qfr[bb]);
    m_run[bb] = -INFINITY; l_run[bb] = 0.f;
  }
  tile_to_lds(Kh, 0, P, s_tiles);
  const int n_tiles = (min((tile_x + 1) * OWN, P) - 1) / kMT + 1;   // key tiles 0 .. the one holding the last row
  for (int kt = 0; kt < n_tiles; ++kt) {
    char* buf = s_tiles + (kt & 1) * kMTileBytes;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of tile kt has landed
    __syncthreads();                                // tile kt visible; everyone is past tile kt-1
    if (kt + 1 < n_tiles) tile_to_lds(Kh, (kt + 1) * kMT, P, s_tiles + ((kt + 1) & 1) * kMTileBytes);
    if ((kt + 1) * kMT - 1 <= r0 && (kt + 1) * kMT <= P) {
      // Every key of the tile is visible to every row of this wave (wave-uniform test, block 0 has the
      // lowest rows; true for all tiles but those on the diagonal): no mask.  The exponentials are taken
      // against the row's current reference without looking for the maximum first; only when a partial
      // sum shows that a logit lies far above the reference (or there is no reference yet: the sum is then
      // infinite) does the wave redo the 16 keys with the reference moved.  After the first tiles that is
      // rare, and the common case costs one comparison per block instead of a maximum per element.
#pragma unroll
      for (int sub = 0; sub < 4; ++sub) {
        sc_bf16x8_t afr[4];
        tile_fragments(buf, sub, afr);
        sc_f32x4_t s4[NB];
        float part[NB];
        bool far = false;
#pragma unroll
        for (int bb = 0; bb < NB; ++bb) {
          s4[bb] = block_product(afr, qfr[bb]);
          const float e0 = __builtin_amdgcn_exp2f(fmaf(s4[bb][0], scale_log2, -m_run[bb]));
          const float e1 = __builtin_amdgcn_exp2f(fmaf(s4[bb][1], scale_log2, -m_run[bb]));
          const float e2 = __builtin_amdgcn_exp2f(fmaf(s4[bb][2], scale_log2, -m_run[bb]));
          const float e3 = __builtin_amdgcn_exp2f(fmaf(s4[bb][3], scale_log2, -m_run[bb]));
          part[bb] = (e0 + e1) + (e2 + e3);
          far |= !(part[bb] < kRefFar);
        }
        if (__builtin_amdgcn_ballot_w64(far)) {
#pragma unroll
          for (int bb = 0; bb < NB; ++bb) {
            const float top = fmaxf(fmaxf(s4[bb][0], s4[bb][1]), fmaxf(s4[bb][2], s4[bb][3])) * scale_log2;
            const float mx = fmaxf(m_run[bb], top);                      // finite: the block has valid keys
            l_run[bb] *= __builtin_amdgcn_exp2f(m_run[bb] - mx);
            m_run[bb] = mx;
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) sum += __builtin_amdgcn_exp2f(fmaf(s4[bb][e], scale_log2, -mx));
            part[bb] = sum;
          }
        }
#pragma unroll
        for (int bb = 0; bb < NB; ++bb) l_run[bb] += part[bb];
      }
      continue;
    }
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      const int c0 = kt * kMT + 16 * sub;
      if (c0 > r0 + 64 * (NB - 1) + 15 || c0 >= P) continue;   // wave-uniform: beyond all rows of this wave
      sc_bf16x8_t afr[4];
      tile_fragments(buf, sub, afr);
#pragma unroll
      for (int bb = 0; bb < NB; ++bb) {
        const int rb = r0 + 64 * bb, my_row = rb + n16;
        if (c0 > rb + 15) continue;                 // wave-uniform: all keys beyond all rows of the block
        const sc_f32x4_t s4 = block_product(afr, qfr[bb]);
        float v[4], mx = m_run[bb];
        if (c0 + 15 <= rb && c0 + 16 <= P) {        // wave-uniform: the whole block is visible, only its neighbours are not
#pragma unroll
          for (int e = 0; e < 4; ++e) { v[e] = s4[e] * scale_log2; mx = fmaxf(mx, v[e]); }
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int key = c0 + 4 * j4 + e;
            v[e] = (key <= my_row && key < P) ? s4[e] * scale_log2 : -INFINITY;
            mx = fmaxf(mx, v[e]);
          }
        }
        const float ms = mx == -INFINITY ? 0.f : mx;
        float sum = l_run[bb] * __builtin_amdgcn_exp2f(m_run[bb] - ms);
#pragma unroll
        for (int e = 0; e < 4; ++e) sum += __builtin_amdgcn_exp2f(v[e] - ms);
        l_run[bb] = sum; m_run[bb] = mx;
      }
    }
  }
  // the 4 lanes of a query row (contraction groups) merge their statistics
#pragma unroll
  for (int bb = 0; bb < NB; ++bb) {
    float m = m_run[bb], l = l_run[bb];
#pragma unroll
    for (int o = 16; o < 64; o <<= 1) {
      const float mo = __shfl_xor(m, o, 64), lo = __shfl_xor(l, o, 64);
      const float mx = fmaxf(m, mo);
      const float ms = mx == -INFINITY ? 0.f : mx;
      l = l * __builtin_amdgcn_exp2f(m - ms) + lo * __builtin_amdgcn_exp2f(mo - ms);
      m = mx;
    }
    const int my_row = r0 + 64 * bb + n16;
    if (j4 == 0 && my_row < P) cstat[(int64_t)bh * P + my_row] = m + __builtin_amdgcn_logf(l);
  }
}

template <int NB>
__global__ __launch_bounds__(kScThreads) void score_colsum_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, int Hq, int Hkv, int P, float scale_log2,
    const float* __restrict__ cstat, const int32_t* __restrict__ prompt_len /*[B] or NULL*/,
    int tiles, int heads, float* __restrict__ scores) {
  extern __shared__ char s_tiles[];                 // 2 x ([64][kMPitch] + 64 floats)
  constexpr int BUF = kMTileBytes + kMT * (int)sizeof(float);
  constexpr int OWN = kMT * NB;                     // keys of a workgroup
  int tile_x, bk;
  if (!xcd_tile_head(tiles, heads, 1, false, tile_x, bk)) return;  // (key tile t is read by query tiles t..last: the first is the longest)
  const int b = bk / Hkv, kvh = bk % Hkv, g = Hq / Hkv;
  const bf16_t* Kh = K + (int64_t)bk * P * 128;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n16 = lane & 15, j4 = lane >> 4;
  const int Pq = prompt_len ? max(0, min(prompt_len[b], P)) : P;   // queries beyond the sequence's own prompt are padding
  const int k0 = tile_x * OWN + 16 * wave;          // first key of own block 0; block bb starts at k0 + 64 bb
  sc_bf16x8_t kfr[NB][4];
  float colsum[NB];
#pragma unroll
  for (int bb = 0; bb < NB; ++bb) {
    row_fragments(Kh, min(k0 + 64 * bb + n16, P - 1), j4, kfr[bb]);
    colsum[bb] = 0.f;
  }
  const int first = tile_x * NB, n_rt = (Pq + kMT - 1) / kMT;      // row tiles first .. n_rt - 1 see these keys
  const int per_head = max(n_rt - first, 0);
  const int total = g * per_head;                   // (head, row tile) pairs, head-major
  int req_h = 0, req_rt = first, req_n = 0;         // the next (head, row tile) to request, requests so far
  auto request = [&]() {
    const int64_t bh = (int64_t)b * Hq + (int64_t)kvh * g + req_h;
    char* dst = s_tiles + (req_n++ & 1) * BUF;
    tile_to_lds(Q + bh * P * 128, req_rt * kMT, P, dst);
    if (wave == 0)                                  // the 64 c_i of the tile's rows, 4 bytes per lane
      __builtin_amdgcn_global_load_lds((sc_gptr_t*)(cstat + bh * P + min(req_rt * kMT + lane, P - 1)),
                                       (sc_lptr_t*)(dst + kMTileBytes), 4, 0, 0);
    if (++req_rt == n_rt) { req_rt = first; ++req_h; }
  };
  if (total > 0) request();
  int rt = first - 1;
  for (int it = 0; it < total; ++it) {
    char* buf = s_tiles + (it & 1) * BUF;
    const float* st_lds = reinterpret_cast<const float*>(buf + kMTileBytes);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of tile `it` has landed
    __syncthreads();                                // tile `it` visible; everyone is past tile it-1
    if (it + 1 < total) request();
    if (++rt == n_rt) rt = first;
    if (rt * kMT >= k0 + 64 * (NB - 1) + 15 && (rt + 1) * kMT <= Pq) {
      // every row of the tile sees every key of this wave and is a real query (wave-uniform; all tiles
      // but those on the diagonal and the last): no mask
#pragma unroll
      for (int sub = 0; sub < 4; ++sub) {
        sc_bf16x8_t afr[4];
        tile_fragments(buf, sub, afr);
        const float4 c4 = *reinterpret_cast<const float4*>(&st_lds[16 * sub + 4 * j4]);   // rows 4 j4 .. 4 j4 + 3
#pragma unroll
        for (int bb = 0; bb < NB; ++bb) {
          const sc_f32x4_t s4 = block_product(afr, kfr[bb]);
          colsum[bb] += __builtin_amdgcn_exp2f(fmaf(s4[0], scale_log2, -c4.x));
          colsum[bb] += __builtin_amdgcn_exp2f(fmaf(s4[1], scale_log2, -c4.y));
          colsum[bb] += __builtin_amdgcn_exp2f(fmaf(s4[2], scale_log2, -c4.z));
          colsum[bb] += __builtin_amdgcn_exp2f(fmaf(s4[3], scale_log2, -c4.w));
        }
      }
      continue;
    }
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      const int i0 = rt * kMT + 16 * sub;
      if (i0 + 15 < k0 || i0 >= Pq) continue;       // wave-uniform: all rows above all of this wave's keys, or padding
      sc_bf16x8_t afr[4];
      tile_fragments(buf, sub, afr);
      const float4 c4 = *reinterpret_cast<const float4*>(&st_lds[16 * sub + 4 * j4]);
      const float crow[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
      for (int bb = 0; bb < NB; ++bb) {
        const int kb = k0 + 64 * bb, my_key = kb + n16;
        if (i0 + 15 < kb) continue;                 // wave-uniform: all rows above all keys of the block
        const sc_f32x4_t s4 = block_product(afr, kfr[bb]);
        if (i0 >= kb + 15 && i0 + 16 <= Pq) {       // wave-uniform: every row of the block sees every key of it
#pragma unroll
          for (int e = 0; e < 4; ++e) colsum[bb] += __builtin_amdgcn_exp2f(fmaf(s4[e], scale_log2, -crow[e]));
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int row = i0 + 4 * j4 + e;
            const float p = __builtin_amdgcn_exp2f(fmaf(s4[e], scale_log2, -crow[e]));
            colsum[bb] += (row >= my_key && row < Pq) ? p : 0.f;
          }
        }
      }
    }
  }
#pragma unroll
  for (int bb = 0; bb < NB; ++bb) {
    float c = colsum[bb];
    c += __shfl_xor(c, 16, 64);
    c += __shfl_xor(c, 32, 64);
    const int my_key = k0 + 64 * bb + n16;
    if (j4 == 0 && my_key < P) scores[(int64_t)bk * P + my_key] = c;
  }
}

template <int NB>
static void launch_scores_mfma(const void* Q, const void* K, int B, int Hq, int Hkv, int P,
                                     const int32_t* prompt_len, float* scores, float* cstat, hipStream_t st,
                                     bool have_stats) {
  const float scale_log2 = (float)(1.4426950408889634 / sqrt(128.0));
  const int tiles = (P + kMT * NB - 1) / (kMT * NB);
  const size_t lds1 = 2 * (size_t)kMTileBytes, lds2 = 2 * ((size_t)kMTileBytes + kMT * sizeof(float));
  auto grid = [&](int heads, int per) { return (unsigned)(((heads / per + 7) / 8) * 8 * per * tiles); };
  if (!have_stats)
    score_rowstats_mfma_kernel<NB><<<grid(B * Hq, Hq / Hkv), kScThreads, lds1, st>>>(
        static_cast<const bf16_t*>(Q), static_cast<const bf16_t*>(K), Hq, Hkv, P, scale_log2, tiles, B * Hq, cstat);
  score_colsum_mfma_kernel<NB><<<grid(B * Hkv, 1), kScThreads, lds2, st>>>(
      static_cast<const bf16_t*>(Q), static_cast<const bf16_t*>(K), Hq, Hkv, P, scale_log2, cstat, prompt_len, tiles,
      B * Hkv, scores);
}

template <typename T, int D>
static void launch_scores(const void* Q, const void* K, int B, int Hq, int Hkv, int P, const int32_t* prompt_len,
                          float* scores, float2* stats, hipStream_t st, bool have_stats) {
  const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)D));
  const int tiles = (P + kTile - 1) / kTile;
  auto grid = [&](int heads, int per) { return (unsigned)(((heads / per + 7) / 8) * 8 * per * tiles); };
  if (!have_stats)
    score_rowstats_kernel<T, D><<<grid(B * Hq, Hq / Hkv), kScThreads, 0, st>>>(
        static_cast<const T*>(Q), static_cast<const T*>(K), Hq, Hkv, P, scale_log2, tiles, B * Hq, stats);
  score_colsum_kernel<T, D><<<grid(B * Hkv, 1), kScThreads, 0, st>>>(
      static_cast<const T*>(Q), static_cast<const T*>(K), Hq, Hkv, P, scale_log2, stats, prompt_len, tiles, B * Hkv,
      scores);
}

// Row statistics supplied by the caller: lse[row] = ln sum_j<=i exp(q_i.k_j / sqrt(D)), as a fused attention
// kernel returns it, rewritten into what the column-sum kernels read (the exp2 domain: c = lse * log2 e;
// the vector-ALU kernels take (reference, 1/sum) = (c, 1)).
__global__ __launch_bounds__(256) void lse_to_rowstats_kernel(const float* __restrict__ lse, int64_t n, int pairs,
                                                              float* __restrict__ out) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const float c = lse[i] * 1.4426950408889634f;
    if (pairs) { out[2 * i] = c; out[2 * i + 1] = 1.f; } else out[i] = c;
  }
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
  return sqa_prefill_scores_ex(Q, K, dt, B, Hq, Hkv, P, D, scores_out, workspace, ws_bytes, stream, nullptr);
}

namespace sqa {
static sqa_status prefill_scores_impl(const void* Q, const void* K, const float* row_lse, sqa_dtype dt,
                                      int B, int Hq, int Hkv, int P, int D,
                                      float* scores_out, void* workspace, size_t ws_bytes, void* stream,
                                      const sqa_batch_opts* opts) {
  const int32_t* plen = opts ? opts->prompt_len : nullptr;
  if (!Q || !K || !scores_out || !workspace) return SQA_ERR_NULL;
  if (dt != SQA_F32 && dt != SQA_BF16) return SQA_ERR_DTYPE;
  if (B < 1 || Hq < 1 || Hkv < 1 || P < 1 || Hq % Hkv != 0 || (D != 64 && D != 128)) return SQA_ERR_SHAPE;
  if (((int64_t)B * Hq + 8) * ((P + 63) / 64) > INT32_MAX) return SQA_ERR_SHAPE;   // workgroups of one launch
  if (!aligned16(Q) || !aligned16(K) || (reinterpret_cast<uintptr_t>(workspace) & 7u)) return SQA_ERR_SHAPE;
  if (row_lse && (reinterpret_cast<uintptr_t>(row_lse) & 3u)) return SQA_ERR_SHAPE;
  if (ws_bytes < sqa_prefill_scores_workspace_bytes(B, Hq, Hkv, P, D)) return SQA_ERR_CAPACITY;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float2* stats = static_cast<float2*>(workspace);
  const bool mfma = dt == SQA_BF16 && D == 128;
  const bool have = row_lse != nullptr;
  if (have) {
    const int64_t n = (int64_t)B * Hq * P;
    const unsigned blocks = (unsigned)(n / 256 + 1 < 4096 ? n / 256 + 1 : 4096);
    lse_to_rowstats_kernel<<<blocks, 256, 0, st>>>(row_lse, n, mfma ? 0 : 1, static_cast<float*>(workspace));
  }
  if (dt == SQA_F32) {
    if (D == 64) launch_scores<float, 64>(Q, K, B, Hq, Hkv, P, plen, scores_out, stats, st, have);
    else launch_scores<float, 128>(Q, K, B, Hq, Hkv, P, plen, scores_out, stats, st, have);
  } else {
    if (D == 64) launch_scores<bf16_t, 64>(Q, K, B, Hq, Hkv, P, plen, scores_out, stats, st, have);
    else launch_scores_mfma<kScBlocksPerWave>(Q, K, B, Hq, Hkv, P, plen, scores_out, reinterpret_cast<float*>(stats), st, have);
  }
  SQA_HIP_CHECK(hipGetLastError());
  return SQA_OK;
}
}  // namespace sqa

extern "C" sqa_status sqa_prefill_scores_ex(const void* Q, const void* K, sqa_dtype dt,
                                            int B, int Hq, int Hkv, int P, int D,
                                            float* scores_out, void* workspace, size_t ws_bytes, void* stream,
                                            const sqa_batch_opts* opts) {
  return sqa::prefill_scores_impl(Q, K, nullptr, dt, B, Hq, Hkv, P, D, scores_out, workspace, ws_bytes, stream, opts);
}

extern "C" sqa_status sqa_prefill_scores_lse(const void* Q, const void* K, const float* row_lse, sqa_dtype dt,
                                             int B, int Hq, int Hkv, int P, int D,
                                             float* scores_out, void* workspace, size_t ws_bytes, void* stream,
                                             const sqa_batch_opts* opts) {
  if (!row_lse) return SQA_ERR_NULL;
  return sqa::prefill_scores_impl(Q, K, row_lse, dt, B, Hq, Hkv, P, D, scores_out, workspace, ws_bytes, stream, opts);
}
