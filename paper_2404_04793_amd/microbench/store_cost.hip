// What a few written bytes cost inside a saturated read stream on MI355X (gfx950).
//
// The decode step of the library reads every kept K/V row once (1.7 GB at the Llama-2-7B shape) and writes about
// 20 MB (accumulated scores, the appended rows, the outputs, unit records).  With its stores removed the kernel runs
// at the chip's streaming-read speed; the stores cost 10 % of the step.  This standalone program measures that cost
// outside the kernel: workgroups stream a region with non-temporal 16-byte loads and then write w bytes each, with
// several kinds of store, cut into several launches, and from a persistent grid that keeps its writes in LDS until
// its item queue is empty.  Build: python -m paper_2404_04793_amd.build --microbench ; run: the executable, no arguments.
// Every access is inside the buffers allocated below; every loop has a bound; nothing is freed (the process ends).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); std::exit(1); } } while (0)
typedef unsigned v4u __attribute__((ext_vector_type(4)));

template <int U>
__device__ __forceinline__ v4u read_region(const v4u* b, size_t n16) {
  v4u acc = {0, 0, 0, 0};
  for (size_t i = threadIdx.x; i < n16; i += 256 * U) {
    v4u v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) { const size_t j = i + (size_t)u * 256; v[u] = __builtin_nontemporal_load(b + (j < n16 ? j : 0)); }
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u];
  }
  return acc;
}

enum Store { PLAIN4 = 0, PLAIN16, NT16, WT16, AGENT4 };   // 4-byte / 16-byte plain, non-temporal, written through (sc1), agent-scope atomic

template <int KIND>
__device__ __forceinline__ void write_region(float* w, int wfloats, v4u acc) {
  if (KIND == PLAIN4 || KIND == AGENT4) {
    for (int i = threadIdx.x; i < wfloats; i += 256) {
      const float val = __uint_as_float(acc.x) + i;
      if (KIND == AGENT4) __hip_atomic_store(w + i, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); else w[i] = val;
    }
  } else {
    v4u* w16 = reinterpret_cast<v4u*>(w);
    for (int i = threadIdx.x; i < wfloats / 4; i += 256) {
      const v4u val = {acc.x + (unsigned)i, acc.y, acc.z, acc.w};
      if (KIND == NT16) __builtin_nontemporal_store(val, w16 + i);
      else if (KIND == WT16) asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(w16 + i), "v"(val) : "memory");
      else w16[i] = val;
    }
  }
}

struct Item { unsigned long long rd_off; unsigned rd_n; unsigned wr_off; unsigned wr_n; };   // read in 16-byte units, written in floats

// one workgroup per item, dispatched by the hardware
template <int KIND>
__global__ __launch_bounds__(256) void per_item(const v4u* __restrict__ p, const Item* items, float* wbuf, uint4* sink, int do_wr) {
  const Item it = items[blockIdx.x];
  const v4u acc = read_region<4>(p + it.rd_off, it.rd_n);
  if (do_wr) write_region<KIND>(wbuf + it.wr_off, (int)it.wr_n, acc);
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[blockIdx.x] = make_uint4(acc.x, acc.y, acc.z, acc.w);
}

// a persistent grid draws items from a queue (the next number is requested while the current item streams);
// HOLD = false: stores after each item; true: kept in LDS and stored when the queue is empty (or LDS is full)
template <bool HOLD, int LOGF>
__global__ __launch_bounds__(256) void persistent(const v4u* __restrict__ p, const Item* items, int nitems, int* queue, float* wbuf, uint4* sink, int do_wr) {
  __shared__ float logd[HOLD ? LOGF : 1];
  __shared__ unsigned rec_off[64], rec_n[64], rec_at[64];
  __shared__ int s_next[2];
  int nrec = 0; unsigned cur = 0;
  if (threadIdx.x == 0) s_next[0] = atomicAdd(queue, 1);
  __syncthreads();
  int ch = s_next[0];
  for (int k = 0; ch < nitems; ++k) {
    if (threadIdx.x == 0) s_next[(k + 1) & 1] = atomicAdd(queue, 1);
    const Item it = items[ch];
    const v4u acc = read_region<4>(p + it.rd_off, it.rd_n);
    if (do_wr) {
      if (!HOLD || nrec == 64 || cur + it.wr_n > (unsigned)LOGF) {
        write_region<PLAIN4>(wbuf + it.wr_off, (int)it.wr_n, acc);
      } else {
        for (unsigned i = threadIdx.x; i < it.wr_n; i += 256) logd[cur + i] = __uint_as_float(acc.x) + i;
        if (threadIdx.x == 0) { rec_off[nrec] = it.wr_off; rec_n[nrec] = it.wr_n; rec_at[nrec] = cur; }
        ++nrec; cur += it.wr_n;
      }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[ch] = make_uint4(acc.x, acc.y, acc.z, acc.w);
    __syncthreads();
    ch = s_next[(k + 1) & 1];
  }
  if (HOLD) {
    __syncthreads();
    for (int k = 0; k < nrec; ++k) {
      float* w = wbuf + rec_off[k];
      const unsigned at = rec_at[k], n = rec_n[k];
      for (unsigned i = threadIdx.x; i < n; i += 256) w[i] = logd[at + i];
    }
  }
}

// the same bytes per workgroup written as PIECES separate runs of `run` bytes each, `stride` bytes apart
// (run * pieces = the bytes per workgroup; stride >= run): does a written byte cost the same whatever it lies next to?
__global__ __launch_bounds__(256) void per_item_pieces(const v4u* __restrict__ p, unsigned rd_n, char* wbuf, int run, int pieces,
                                                       size_t stride, size_t wg_pitch, uint4* sink) {
  const v4u acc = read_region<4>(p + (size_t)blockIdx.x * rd_n, rd_n);
  char* w = wbuf + (size_t)blockIdx.x * wg_pitch;
  const int per_piece = run / 4;                              // floats
  for (int i = threadIdx.x; i < per_piece * pieces; i += 256) {
    const int pc = i / per_piece, k = i % per_piece;
    reinterpret_cast<float*>(w + (size_t)pc * stride)[k] = __uint_as_float(acc.x) + i;
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[blockIdx.x] = make_uint4(acc.x, acc.y, acc.z, acc.w);
}

int main() {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  uint4* sink; CK(hipMalloc(&sink, 1 << 20));
  int* queue; CK(hipMalloc(&queue, 4));
  auto timed = [&](const char* name, size_t bytes, auto launch) {
    for (int i = 0; i < 3; ++i) launch();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int i = 0; i < 20; ++i) launch();
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= 20;
    std::printf("%-86s %8.1f us  %7.1f GB/s read\n", name, ms * 1e3, bytes / ms / 1e6); std::fflush(stdout);
  };
  auto upload = [&](const std::vector<Item>& v) { Item* d; CK(hipMalloc(&d, v.size() * sizeof(Item))); CK(hipMemcpy(d, v.data(), v.size() * sizeof(Item), hipMemcpyHostToDevice)); return d; };
  char nm[160];

  // ---- A. uniform items: 8192 workgroups x 212.5 KB read, w floats written each -----------------------------
  {
    const int n = 8192; const unsigned rd_n = 13600;                      // 16-byte units per item
    const size_t bytes = (size_t)n * rd_n * 16;
    v4u* p; CK(hipMalloc(&p, bytes)); CK(hipMemset(p, 1, bytes));
    float* wb; CK(hipMalloc(&wb, (size_t)n * 576 * 4));
    std::printf("A. %d items of %.1f KB read (%.2f GB); w floats written per item\n", n, rd_n * 16 / 1024.0, bytes / 1e9);
    for (int wf : {0, 144, 572}) {
      std::vector<Item> v; for (int i = 0; i < n; ++i) v.push_back(Item{(unsigned long long)i * rd_n, rd_n, (unsigned)(i * wf), (unsigned)wf});
      Item* d = upload(v);
      const double mb = (double)n * wf * 4 / 1e6;
      std::snprintf(nm, 160, "w=%3d (%5.1f MB)  4-byte stores", wf, mb);           timed(nm, bytes, [&] { per_item<PLAIN4><<<n, 256>>>(p, d, wb, sink, wf > 0); });
      if (wf == 0) continue;
      std::snprintf(nm, 160, "w=%3d            16-byte stores", wf);                timed(nm, bytes, [&] { per_item<PLAIN16><<<n, 256>>>(p, d, wb, sink, 1); });
      std::snprintf(nm, 160, "w=%3d            16-byte non-temporal stores", wf);   timed(nm, bytes, [&] { per_item<NT16><<<n, 256>>>(p, d, wb, sink, 1); });
      std::snprintf(nm, 160, "w=%3d            16-byte stores written through (sc1)", wf); timed(nm, bytes, [&] { per_item<WT16><<<n, 256>>>(p, d, wb, sink, 1); });
      std::snprintf(nm, 160, "w=%3d            4-byte agent-scope atomic stores", wf);     timed(nm, bytes, [&] { per_item<AGENT4><<<n, 256>>>(p, d, wb, sink, 1); });
      if (wf == 572) {
        std::snprintf(nm, 160, "w=%3d            the same as 4 launches of 2048 workgroups (each resident at once)", wf);
        timed(nm, bytes, [&] { for (int q = 0; q < 4; ++q) per_item<PLAIN4><<<2048, 256>>>(p, d + q * 2048, wb, sink, 1); });
        std::snprintf(nm, 160, "w=  0            4 launches of 2048 workgroups, nothing written");
        timed(nm, bytes, [&] { for (int q = 0; q < 4; ++q) per_item<PLAIN4><<<2048, 256>>>(p, d + q * 2048, wb, sink, 0); });
        for (int wr : {0, 1}) {
          std::snprintf(nm, 160, "persistent grid of 1024, stores after each item%s", wr ? "" : " (nothing written)");
          timed(nm, bytes, [&] { CK(hipMemsetAsync(queue, 0, 4)); persistent<false, 1><<<1024, 256>>>(p, d, n, queue, wb, sink, wr); });
          std::snprintf(nm, 160, "persistent grid of 1024, writes held in LDS until the queue is empty%s", wr ? "" : " (nothing written)");
          timed(nm, bytes, [&] { CK(hipMemsetAsync(queue, 0, 4)); persistent<true, 6912><<<1024, 256>>>(p, d, n, queue, wb, sink, wr); });
        }
      }
    }
  }
  // ---- A2. 2304 bytes per workgroup in runs of different length ------------------------------------------------
  {
    const int n = 8192; const unsigned rd_n = 13600;
    const size_t bytes = (size_t)n * rd_n * 16;
    v4u* p; CK(hipMalloc(&p, bytes)); CK(hipMemset(p, 1, bytes));
    const size_t pitch = 144 * 4096;                                    // room for 144 pieces 4 KB apart
    char* wb; CK(hipMalloc(&wb, (size_t)n * pitch));
    std::printf("A2. %d items of %.1f KB read; 2304 bytes written per item as separate runs\n", n, rd_n * 16 / 1024.0);
    struct { int run, pieces; size_t stride; const char* what; } cases[] = {
      {2304, 1, 2304, "1 run of 2304 B"}, {256, 9, 4096, "9 runs of 256 B, 4 KB apart"}, {256, 9, 256, "9 runs of 256 B, adjacent"},
      {128, 18, 4096, "18 runs of 128 B, 4 KB apart"}, {64, 36, 4096, "36 runs of 64 B, 4 KB apart"}, {64, 36, 128, "36 runs of 64 B, one per 128-byte line"},
      {16, 144, 4096, "144 runs of 16 B, 4 KB apart"}, {16, 144, 128, "144 runs of 16 B, one per 128-byte line"}};
    for (auto& cs : cases) {
      std::snprintf(nm, 160, "%s", cs.what);
      timed(nm, bytes, [&] { per_item_pieces<<<n, 256>>>(p, rd_n, wb, cs.run, cs.pieces, cs.stride, pitch, sink); });
    }
  }
  // ---- B. the items of the decode launch at the Llama-2-7B shape --------------------------------------------
  {
    std::vector<Item> v; unsigned long long ro = 0; unsigned wo = 0;
    for (int i = 0; i < 1024; ++i) { Item t{ro, 2271u * 32u, wo, 2271u + 200u}; ro += t.rd_n; wo += t.wr_n; v.push_back(t); }          // a 2271-token unit
    for (int i = 0; i < 1792; ++i) { Item t{ro, 4u * 143u * 32u, wo, 4u * (143u + 200u)}; ro += t.rd_n; wo += t.wr_n; v.push_back(t); } // four 143-token units
    const size_t bytes = ro * 16; const int n = (int)v.size();
    v4u* p; CK(hipMalloc(&p, bytes)); CK(hipMemset(p, 1, bytes));
    float* wb; CK(hipMalloc(&wb, (size_t)wo * 4));
    Item* d = upload(v);
    std::printf("B. %d items: 1024 of %.2f MB, 1792 of %.2f MB (%.2f GB read, %.1f MB written)\n", n, 2271 * 512 / 1e6, 4 * 143 * 512 / 1e6, bytes / 1e9, wo * 4 / 1e6);
    for (int wr : {0, 1}) {
      std::snprintf(nm, 160, "one workgroup per item, hardware dispatch%s", wr ? "" : " (nothing written)");
      timed(nm, bytes, [&] { per_item<PLAIN4><<<n, 256>>>(p, d, wb, sink, wr); });
      std::snprintf(nm, 160, "two launches: the 1024 long items (resident at once), then the 1792 short ones%s", wr ? "" : " (nothing written)");
      timed(nm, bytes, [&] { per_item<PLAIN4><<<1024, 256>>>(p, d, wb, sink, wr); per_item<PLAIN4><<<1792, 256>>>(p, d + 1024, wb, sink, wr); });
      std::snprintf(nm, 160, "persistent grid of 1024, stores after each item%s", wr ? "" : " (nothing written)");
      timed(nm, bytes, [&] { CK(hipMemsetAsync(queue, 0, 4)); persistent<false, 1><<<1024, 256>>>(p, d, n, queue, wb, sink, wr); });
      std::snprintf(nm, 160, "persistent grid of 1024, writes held in LDS until the queue is empty%s", wr ? "" : " (nothing written)");
      timed(nm, bytes, [&] { CK(hipMemsetAsync(queue, 0, 4)); persistent<true, 6912><<<1024, 256>>>(p, d, n, queue, wb, sink, wr); });
    }
  }
  return 0;
}
