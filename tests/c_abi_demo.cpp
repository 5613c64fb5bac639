// The library used from plain C++ through include/sqa.h alone -- no Python, no torch: the HIP runtime supplies the
// device memory, everything else is the C ABI.  Runs Algorithm 1 end to end on a small synthetic job (probe ->
// budgets -> prompt scores -> compression -> decode steps) and checks what can be checked without a second
// implementation of the method: status codes, budget sum, unit lengths, kept positions (sorted, unique, the newest
// token present, sinks of nothing), and -- for a cache whose budget exceeds everything it will ever hold -- the
// attention output against the textbook softmax(q K^T / sqrt(D)) V computed here in double.
// Built by `python -m paper_2404_04793_amd.build --demo`; tests/test_gpu_c_abi_demo.py runs it on the GPU.
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "sqa.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)
#define SQA_CALL(x) do { sqa_status s_ = (x); if (s_ != SQA_OK) { std::printf("%s at line %d\n", sqa_status_str(s_), __LINE__); return 1; } } while (0)
#define CHECK(c) do { if (!(c)) { std::printf("check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

static unsigned long long g_state = 0x9E3779B97F4A7C15ull;
static float rnd() {                       // uniform in (-1, 1)
  g_state ^= g_state << 13; g_state ^= g_state >> 7; g_state ^= g_state << 17;
  return (float)((double)(g_state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
template <typename T> static T* to_device(const std::vector<T>& v) {
  T* d = nullptr;
  if (hipMalloc(&d, v.size() * sizeof(T)) != hipSuccess) return nullptr;
  if (hipMemcpy(d, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return nullptr;
  return d;
}

int main() {
  const int L = 3, B = 2, H = 2, D = 64, P = 96, S = 5, hidden = 64;
  const int64_t T = (int64_t)B * P;
  // ---- layer importance (Algorithm 1 steps 1-4) and budgets (steps 5-11) -----------------------------------
  const float noise[L] = {2.0f, 0.3f, 1.5f};
  std::vector<float> h_in((size_t)L * T * hidden), h_out(h_in.size());
  for (int l = 0; l < L; ++l)
    for (size_t i = 0; i < (size_t)T * hidden; ++i) {
      const size_t at = (size_t)l * T * hidden + i;
      h_in[at] = rnd(); h_out[at] = h_in[at] + noise[l] * rnd();
    }
  float *d_hin = to_device(h_in), *d_hout = to_device(h_out), *d_cos = nullptr;
  CHECK(d_hin && d_hout);
  HIP_OK(hipMalloc(&d_cos, L * sizeof(float)));
  const size_t imp_bytes = sqa_layer_importance_workspace_bytes(L, T, hidden);
  void* d_impws = nullptr; HIP_OK(hipMalloc(&d_impws, imp_bytes ? imp_bytes : 8));
  SQA_CALL(sqa_layer_importance(d_hin, d_hout, SQA_F32, L, T, hidden, d_cos, d_impws, imp_bytes, nullptr));
  float cosv[L]; HIP_OK(hipMemcpy(cosv, d_cos, sizeof(cosv), hipMemcpyDeviceToHost));
  CHECK(cosv[1] > cosv[2] && cosv[2] > cosv[0] && cosv[0] > 0.f && cosv[1] < 1.f);   // less noise, more alike
  const int b_init = P / 5;
  int32_t budget[L]; int8_t group[L];
  SQA_CALL(sqa_allocate_budgets(cosv, L, (int64_t)L * b_init, 0.35, budget, group));
  CHECK(budget[0] + budget[1] + budget[2] == L * b_init && budget[1] < budget[0] && group[1] == 2);
  std::printf("cos %.4f %.4f %.4f -> budgets %d %d %d\n", cosv[0], cosv[1], cosv[2], budget[0], budget[1], budget[2]);

  // ---- caches, prompt scores, compression (step 12 with 16-17 on the prompt) --------------------------------
  sqa_layer_cache layers[L] = {};
  const size_t unit = (size_t)B * H;
  for (int l = 0; l < L; ++l) {
    const int cap = budget[l] < P + S ? budget[l] : P + S;
    layers[l].capacity = cap; layers[l].budget = budget[l];
    HIP_OK(hipMalloc(&layers[l].K, unit * cap * D * sizeof(float)));
    HIP_OK(hipMalloc(&layers[l].V, unit * cap * D * sizeof(float)));
    HIP_OK(hipMalloc((void**)&layers[l].score_acc, unit * cap * sizeof(float)));
    HIP_OK(hipMalloc((void**)&layers[l].pos, unit * cap * sizeof(int32_t)));
    HIP_OK(hipMalloc((void**)&layers[l].unit_state, unit * 4 * sizeof(int32_t)));
  }
  const size_t sc_ws_bytes = sqa_prefill_scores_workspace_bytes(B, H, H, P, D);
  void* d_scws = nullptr; HIP_OK(hipMalloc(&d_scws, sc_ws_bytes));
  float* d_scores = nullptr; HIP_OK(hipMalloc(&d_scores, unit * P * sizeof(float)));
  std::vector<float> q((size_t)unit * P * D), k(q.size()), v(q.size());
  for (int l = 0; l < L; ++l) {
    for (size_t i = 0; i < q.size(); ++i) { q[i] = rnd(); k[i] = rnd(); v[i] = rnd(); }
    float *dq = to_device(q), *dk = to_device(k), *dv = to_device(v);
    CHECK(dq && dk && dv);
    SQA_CALL(sqa_prefill_scores(dq, dk, SQA_F32, B, H, H, P, D, d_scores, d_scws, sc_ws_bytes, nullptr));
    SQA_CALL(sqa_prefill_compress(dk, dv, SQA_F32, d_scores, B, H, P, D, SQA_H2O, 4, &layers[l], nullptr));
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipFree(dq)); HIP_OK(hipFree(dk)); HIP_OK(hipFree(dv));
  }

  // ---- decode (steps 14-21): all layers in one launch per step ----------------------------------------------
  const size_t ws_bytes = sqa_decode_workspace_bytes(layers, L, B, H, H, D, SQA_H2O);
  CHECK(ws_bytes > 0);
  void* d_ws = nullptr; HIP_OK(hipMalloc(&d_ws, ws_bytes));
  SQA_CALL(sqa_decode_workspace_init(d_ws, ws_bytes, nullptr));
  sqa_decode_plan_info plan;
  SQA_CALL(sqa_decode_plan(layers, L, B, H, H, D, SQA_F32, SQA_H2O, &plan, nullptr));
  CHECK(plan.workgroups >= 1 && (size_t)plan.workspace_bytes <= ws_bytes);
  std::vector<float> step((size_t)L * unit * D), out(step.size());
  float *d_q = nullptr, *d_k = nullptr, *d_v = nullptr, *d_out = nullptr;
  HIP_OK(hipMalloc(&d_q, step.size() * 4)); HIP_OK(hipMalloc(&d_k, step.size() * 4));
  HIP_OK(hipMalloc(&d_v, step.size() * 4)); HIP_OK(hipMalloc(&d_out, step.size() * 4));
  for (int t = 0; t < S; ++t) {
    for (float* dst : {d_q, d_k, d_v}) {
      for (auto& x : step) x = rnd();
      HIP_OK(hipMemcpy(dst, step.data(), step.size() * 4, hipMemcpyHostToDevice));
    }
    SQA_CALL(sqa_decode_step(d_q, d_k, d_v, SQA_F32, B, H, H, D, P + t, SQA_H2O, 4, layers, nullptr, L, d_out, d_ws, ws_bytes, nullptr));
    int32_t dev_status = -1;
    SQA_CALL(sqa_read_device_status(d_ws, nullptr, &dev_status));
    CHECK(dev_status == 0);
    HIP_OK(hipMemcpy(out.data(), d_out, out.size() * 4, hipMemcpyDeviceToHost));
    for (float x : out) CHECK(std::isfinite(x) && std::fabs(x) <= 1.0f);      // a convex combination of V rows in (-1, 1)
  }
  for (int l = 0; l < L; ++l) {
    const int cap = layers[l].capacity;
    int32_t* d_sorted = nullptr; HIP_OK(hipMalloc((void**)&d_sorted, unit * cap * sizeof(int32_t)));
    SQA_CALL(sqa_kept_idx_sorted(&layers[l], B, H, d_sorted, nullptr));
    std::vector<int32_t> kept(unit * cap), st(unit * 4);
    HIP_OK(hipMemcpy(kept.data(), d_sorted, kept.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(st.data(), layers[l].unit_state, st.size() * 4, hipMemcpyDeviceToHost));
    const int want = budget[l] < P + S ? budget[l] : P + S;
    for (size_t u = 0; u < unit; ++u) {
      CHECK(st[u * 4 + SQA_ST_LEN] == want);
      for (int i = 1; i < want; ++i) CHECK(kept[u * cap + i] > kept[u * cap + i - 1]);     // ascending, unique
      CHECK(kept[u * cap] >= 0 && kept[u * cap + want - 1] == P + S - 1);                 // the newest token is there
      const int rec = budget[l] - budget[l] / 2;                                          // H2O: the recent half is the last `rec` positions
      CHECK(kept[u * cap + want - rec] == P + S - rec);
    }
  }

  // ---- a cache that never fills (Algorithm 1: compress only if len > b) is plain attention ------------------
  {
    const int cap = P + S;
    sqa_layer_cache full = {};
    full.capacity = cap; full.budget = cap;
    HIP_OK(hipMalloc(&full.K, (size_t)cap * D * 4)); HIP_OK(hipMalloc(&full.V, (size_t)cap * D * 4));
    HIP_OK(hipMalloc((void**)&full.pos, cap * 4)); HIP_OK(hipMalloc((void**)&full.unit_state, 16));
    std::vector<float> K((size_t)cap * D), V(K.size()), qv(D), o(D);
    for (size_t i = 0; i < (size_t)P * D; ++i) { K[i] = rnd(); V[i] = rnd(); }
    float *dK = to_device(std::vector<float>(K.begin(), K.begin() + (size_t)P * D)), *dV = to_device(std::vector<float>(V.begin(), V.begin() + (size_t)P * D));
    CHECK(dK && dV);
    SQA_CALL(sqa_prefill_compress(dK, dV, SQA_F32, nullptr, 1, 1, P, D, SQA_SLIDING, 0, &full, nullptr));
    const size_t wsb = sqa_decode_workspace_bytes(&full, 1, 1, 1, 1, D, SQA_SLIDING);
    void* w = nullptr; HIP_OK(hipMalloc(&w, wsb)); SQA_CALL(sqa_decode_workspace_init(w, wsb, nullptr));
    float *dq1 = nullptr, *dk1 = nullptr, *dv1 = nullptr, *do1 = nullptr;
    HIP_OK(hipMalloc(&dq1, D * 4)); HIP_OK(hipMalloc(&dk1, D * 4)); HIP_OK(hipMalloc(&dv1, D * 4)); HIP_OK(hipMalloc(&do1, D * 4));
    double worst = 0.0;
    for (int t = 0; t < S; ++t) {
      for (int d = 0; d < D; ++d) { qv[d] = rnd(); K[(size_t)(P + t) * D + d] = rnd(); V[(size_t)(P + t) * D + d] = rnd(); }
      HIP_OK(hipMemcpy(dq1, qv.data(), D * 4, hipMemcpyHostToDevice));
      HIP_OK(hipMemcpy(dk1, &K[(size_t)(P + t) * D], D * 4, hipMemcpyHostToDevice));
      HIP_OK(hipMemcpy(dv1, &V[(size_t)(P + t) * D], D * 4, hipMemcpyHostToDevice));
      SQA_CALL(sqa_decode_step(dq1, dk1, dv1, SQA_F32, 1, 1, 1, D, P + t, SQA_SLIDING, 0, &full, nullptr, 1, do1, w, wsb, nullptr));
      HIP_OK(hipMemcpy(o.data(), do1, D * 4, hipMemcpyDeviceToHost));
      const int n = P + t + 1;
      std::vector<double> s(n); double mx = -1e300, sum = 0.0;
      for (int j = 0; j < n; ++j) { double a = 0.0; for (int d = 0; d < D; ++d) a += (double)qv[d] * K[(size_t)j * D + d]; s[j] = a / std::sqrt((double)D); mx = s[j] > mx ? s[j] : mx; }
      for (int j = 0; j < n; ++j) { s[j] = std::exp(s[j] - mx); sum += s[j]; }
      double ref_max = 0.0, err = 0.0;
      for (int d = 0; d < D; ++d) {
        double a = 0.0; for (int j = 0; j < n; ++j) a += s[j] / sum * V[(size_t)j * D + d];
        ref_max = std::fabs(a) > ref_max ? std::fabs(a) : ref_max;
        err = std::fabs(a - o[d]) > err ? std::fabs(a - o[d]) : err;
      }
      worst = err / ref_max > worst ? err / ref_max : worst;
    }
    std::printf("uncompressed cache against textbook attention: worst relative error %.2e\n", worst);
    CHECK(worst < 1e-5);
  }
  std::printf("c_abi_demo ok\n");
  return 0;
}
