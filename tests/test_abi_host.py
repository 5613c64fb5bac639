"""CPU-side checks of the C-ABI library: it loads, exports every symbol that
include/sqa.h declares, validates arguments before touching the GPU, and its
host-side budget allocator agrees bit for bit with the oracle (Algorithm 1
steps 5-11)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import sqa_oracle as O
from paper_2404_04793_amd import binding as sqa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "sqa.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(sqa_[a-z_0-9]+)\s*\(", hdr))
    assert {"sqa_layer_importance", "sqa_allocate_budgets", "sqa_prefill_compress", "sqa_decode_step"} <= names
    lib = C.CDLL(sqa.LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), n


def test_struct_layout_matches_header():
    assert C.sizeof(sqa.LayerCacheStruct) == 72
    assert sqa.LayerCacheStruct.block_table.offset == 48 and sqa.LayerCacheStruct.capacity.offset == 56
    assert sqa.LayerCacheStruct.budget.offset == 60 and sqa.LayerCacheStruct.n_blocks.offset == 68


def test_batch_opts_layout_and_validation():
    assert C.sizeof(sqa.BatchOptsStruct) == 40 and sqa.BatchOptsStruct.order.offset == 32
    lib = sqa._lib
    p = C.c_void_p(0x1000)
    lc = sqa.LayerCacheStruct(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, None, None, 8, 4, 0, 0)
    bad = sqa.BatchOptsStruct(None, None, None, None, 2)
    base = [p, p, p, 1, 1, 1, 1, 128, -1, 2, 4, C.byref(lc), None, 1, p, C.c_void_p(0x1000), 1 << 20, None]
    assert lib.sqa_decode_step_ex(*base, C.byref(bad)) == 4                       # unknown order
    assert lib.sqa_decode_step_ex(*base, None) == 2                                # new_pos < 0 without per-sequence positions
    assert lib.sqa_layer_importance_seq(p, p, 1, 1, 4, 64, None, 1, p, p, 1 << 20, None) == 1
    assert lib.sqa_layer_importance_seq(p, p, 1, 1, 4, 64, p, 0, p, p, 1 << 20, None) == 2
    assert lib.sqa_layer_importance_seq(p, p, 1, 1, 4, 64, p, 3, p, p, 16, None) == 6    # needs n_seq times the plain workspace


def test_paper_worked_example_through_the_library():
    # Appendix A.2: 18 important / 14 unimportant layers, b_init 1000, p 0.3 -> 300 / 1544
    r = np.random.default_rng(0)
    cos = np.concatenate([0.4 + 0.05 * r.random(4), 0.7 + 0.04 * r.random(14), 0.94 + 0.02 * r.random(14)])
    cos = cos[r.permutation(32)].astype(np.float32)
    budget, group = sqa.allocate_budgets(cos, 32000, 0.3)
    assert sum(budget) == 32000
    assert {b for b, g in zip(budget, group) if g == 2} == {300}
    assert min(b for b, g in zip(budget, group) if g != 2) == 1544
    assert sum(1 for g in group if g == 2) == 14


@pytest.mark.parametrize("seed", range(40))
def test_budgets_bit_exact_vs_oracle(seed):
    r = np.random.default_rng(seed)
    L = int(r.integers(1, 100))
    kind = seed % 4
    if kind == 0:
        cos = r.random(L)
    elif kind == 1:
        cos = np.round(r.random(L), 1)                 # many equal values
    elif kind == 2:
        cos = 0.9 + 0.05 * r.standard_normal(L); cos[: L // 5] = 0.4 + 0.1 * r.random(L // 5)
    else:
        cos = np.arange(L) / max(L, 1)                 # evenly spaced: ties between splits
    cos = cos.astype(np.float32)
    total = int(r.integers(L * 3, L * 4000 + 1))
    p = float(r.choice([0.1, 0.25, 0.3, 0.35, 0.4, 0.5, 0.9, 1.0]))
    try:
        want = O.allocate_budgets(cos, total, p)
    except ValueError:
        with pytest.raises(sqa.SqaError) as e:
            sqa.allocate_budgets(cos, total, p)
        assert e.value.code == 5
        return
    got = sqa.allocate_budgets(cos, total, p)
    assert got[0] == want[0] and got[1] == want[1]


def test_budget_argument_errors():
    for cos, total, p, code in [([0.1, 0.5, 0.9], 2, 0.3, 5), ([0.1, 0.5, 0.9], 30, 0.0, 5),
                                ([0.1, 0.5, 0.9], 30, 1.01, 5), ([0.1, 0.5, 0.9], 3, 0.3, 5)]:
        with pytest.raises(sqa.SqaError) as e:
            sqa.allocate_budgets(cos, total, p)
        assert e.value.code == code
    lib = sqa._lib
    out = (C.c_int32 * 3)()
    assert lib.sqa_allocate_budgets(None, 3, 30, 0.3, out, None) == 1
    assert lib.sqa_allocate_budgets((C.c_float * 3)(0.1, 0.2, 0.3), 0, 30, 0.3, out, None) == 2


def test_device_entry_points_validate_before_any_gpu_call():
    """Bogus but non-NULL, aligned pointers: every call must fail in validation."""
    lib = sqa._lib
    p = C.c_void_p(0x1000)
    assert lib.sqa_layer_importance(None, p, 0, 1, 4, 64, p, p, 1 << 20, None) == 1
    assert lib.sqa_layer_importance(p, p, 7, 1, 4, 64, p, p, 1 << 20, None) == 3
    assert lib.sqa_layer_importance(p, p, 0, 1, 4, 60, p, p, 1 << 20, None) == 2
    assert lib.sqa_layer_importance(p, p, 0, 1, 4, 64, p, p, 0, None) == 6
    assert lib.sqa_residual_add_importance(p, p, None, 0, 1, 4, 64, p, p, 1 << 20, None) == 1
    assert lib.sqa_residual_add_importance(p, None, p, 0, 1, 4, 64, p, p, 1 << 20, None) == 1
    assert lib.sqa_residual_add_importance(p, p, C.c_void_p(0x1008), 0, 1, 4, 64, p, p, 1 << 20, None) == 2
    assert lib.sqa_residual_add_importance(p, p, p, 2, 1, 4, 64, p, p, 1 << 20, None) == 3
    assert lib.sqa_residual_add_importance(p, p, p, 1, 1, 4, 64, p, p, 0, None) == 6
    lc = sqa.LayerCacheStruct(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, None, None, 8, 4, 0, 0)
    args = lambda **kw: [kw.get("K", p), p, kw.get("dt", 1), kw.get("sc", p), 1, 1, kw.get("P", 16), kw.get("D", 128),
                         kw.get("pol", 2), kw.get("ns", 4), C.byref(kw.get("lc", lc)), None]
    assert lib.sqa_prefill_compress(*args(K=None)) == 1
    assert lib.sqa_prefill_compress(*args(dt=5)) == 3
    assert lib.sqa_prefill_compress(*args(pol=3)) == 4
    assert lib.sqa_prefill_compress(*args(D=96)) == 2
    assert lib.sqa_prefill_compress(*args(sc=None)) == 1                     # H2O needs scores
    assert lib.sqa_prefill_compress(*args(pol=1, ns=4)) == 5                 # streaming: budget 4 < n_sink+1
    small = sqa.LayerCacheStruct(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, None, None, 3, 4, 0, 0)
    assert lib.sqa_prefill_compress(*args(lc=small)) == 6                    # capacity 3 < min(P, budget)
    one = sqa.LayerCacheStruct(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, None, None, 8, 1, 0, 0)
    assert lib.sqa_prefill_compress(*args(lc=one)) == 5                      # H2O: budget 1 < 2

    def dec(**kw):
        return lib.sqa_decode_step(kw.get("q", p), p, p, kw.get("dt", 1), 1, kw.get("Hq", 4), kw.get("Hkv", 4),
                                   kw.get("D", 128), kw.get("pos", 5), kw.get("pol", 2), 4,
                                   C.byref(kw.get("lc", lc)), None, kw.get("nl", 1), p, C.c_void_p(0x10000), kw.get("ws", 1 << 20), None)
    assert dec(q=None) == 1
    assert dec(dt=9) == 3
    assert dec(pol=-1) == 4
    assert dec(Hq=6) == 2                      # Hq % Hkv != 0
    assert dec(Hq=12) == 2                     # group of 3 not supported
    assert dec(D=100) == 2
    assert dec(nl=1000) == 2
    assert dec(ws=8) == 6
    assert dec(lc=one) == 5
    # blocked allocation: the table row must cover the unit's slots, packed units and blocks do not mix,
    # the pools hold at least one block
    tblp, offp = 0x6000, 0x7000
    blk = lambda **kw: sqa.LayerCacheStruct(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, kw.get("off"), tblp,
                                            kw.get("cap", 40), kw.get("b", 40), kw.get("bpu", 3), kw.get("nb", 8))
    for call in (lambda c: dec(lc=c), lambda c: lib.sqa_prefill_compress(*args(lc=c, P=64))):
        assert call(blk(bpu=2)) == 2               # 2 x 16 rows < 40 slots
        assert call(blk(off=offp)) == 2
        assert call(blk(nb=0)) == 2
        assert call(blk(bpu=1025, cap=20000, b=20000)) == 2
    assert lib.sqa_prefill_compress(*args(lc=blk(cap=70000, b=70000, bpu=1024, nb=8), P=80000)) in (2, 6)
    assert lib.sqa_decode_workspace_bytes(C.byref(lc), 0, 1, 4, 4, 128, 2) == 0
    assert lib.sqa_decode_workspace_bytes(C.byref(lc), 1, 1, 4, 4, 128, 2) >= 256 + 64
    big = sqa.LayerCacheStruct(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, None, None, 5000, 5000, 0, 0)
    # 5000 slots -> several chunks per unit: partial records, logits and counters
    assert lib.sqa_decode_workspace_bytes(C.byref(big), 1, 2, 4, 4, 128, 2) > 2 * 4 * 5000 * 4
    assert lib.sqa_decode_workspace_init(None, 16, None) == 1
    assert lib.sqa_kept_idx_sorted(None, 1, 1, p, None) == 1
    assert lib.sqa_prefill_scores(p, p, 1, 1, 6, 4, 16, 128, p, p, 1 << 20, None) == 2
    lib.sqa_status_str.restype = C.c_char_p
    assert lib.sqa_status_str(5) == b"bad budget"


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: include/sqa.h must compile as strict C99, without a C++ or HIP compiler."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_header.c"
    src.write_text('#include "sqa.h"\n'
                   'int main(void) {\n'
                   '  sqa_batch_opts o = {0}; sqa_layer_cache c = {0};\n'
                   '  (void)o; (void)c;\n'
                   '  return sizeof(sqa_layer_cache) == 72 && SQA_ST_WORDS == 4 && SQA_BLOCK_SLOTS == 16 ? 0 : 1;\n'
                   '}\n')
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                        str(src), "-o", str(tmp_path / "use_header")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    assert subprocess.run([str(tmp_path / "use_header")]).returncode == 0


def test_host_entry_point_called_from_c(tmp_path):
    """A C program linked against libsqa.so reproduces the worked example of Appendix A.2
    (b_init 1000, p 0.3, 18 important layers of 32: 300 for the others, 1544 or 1545 for the important ones)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    libdir = os.path.dirname(sqa.LIB_PATH)
    src = tmp_path / "budgets.c"
    src.write_text(r'''
#include <stdio.h>
#include "sqa.h"
int main(void) {
  float cos[32]; int32_t budget[32]; int8_t group[32];
  /* 2 special layers near 0.4, 16 around 0.7, 14 around 0.96: the 14 form G3 */
  for (int i = 0; i < 32; ++i) cos[i] = i < 2 ? 0.40f + 0.01f * i : (i < 16 || i >= 30 ? 0.70f + 0.0005f * i : 0.95f + 0.0005f * i);
  sqa_status st = sqa_allocate_budgets(cos, 32, 32000, 0.3, budget, group);
  if (st != SQA_OK) { printf("status %s\n", sqa_status_str(st)); return 2; }
  long sum = 0; int n3 = 0;
  for (int i = 0; i < 32; ++i) { sum += budget[i]; n3 += group[i] == 2; }
  printf("%ld %d %d %d\n", sum, n3, (int)budget[20], (int)budget[5]);
  return sqa_allocate_budgets(cos, 32, 16, 0.3, budget, group) == SQA_ERR_BUDGET ? 0 : 3;
}
''')
    exe = tmp_path / "budgets"
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                        "-L", libdir, "-lsqa", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    run = subprocess.run([str(exe)], capture_output=True, text=True)
    assert run.returncode == 0, (run.stdout, run.stderr)
    total, n3, low, high = [int(x) for x in run.stdout.split()]
    assert total == 32000 and n3 == 14 and low == 300 and high in (1544, 1545)   # 14 x 300 + 18 x 1544.4 = 32000


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching any device."""
    import subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_host_allocator_under_address_and_undefined_sanitizers(tmp_path):
    """The host-only part of the library (clustering and budgets, Algorithm 1 steps 5-11) built from its
    source with AddressSanitizer and UndefinedBehaviorSanitizer, no GPU code involved: the seeded cases of
    test_budgets_bit_exact_vs_oracle plus degenerate inputs run through a small driver, then the block free
    list under a random sequence of take / give calls; any report ends the driver with a non-zero status.
    Results must still equal the oracle's."""
    import shutil
    import subprocess
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    driver = tmp_path / "driver.cpp"
    driver.write_text(r'''
#include <cstdio>
#include <vector>
#include "sqa.h"
int main() {
  int L; long long total; double p;
  while (std::scanf("%d %lld %lf", &L, &total, &p) == 3) {
    std::vector<float> cos(L > 0 ? L : 1);
    for (int i = 0; i < L; ++i) { double x; if (std::scanf("%lf", &x) != 1) return 9; cos[i] = (float)x; }
    std::vector<int32_t> budget(L > 0 ? L : 1);
    std::vector<int8_t> group(L > 0 ? L : 1);
    const sqa_status st = sqa_allocate_budgets(cos.data(), L, total, p, budget.data(), group.data());
    std::printf("%d", (int)st);
    if (st == SQA_OK) for (int i = 0; i < L; ++i) std::printf(" %d:%d", (int)budget[i], (int)group[i]);
    std::printf("\n");
  }
  // the block free list: sequences join and leave with different block counts; no block is ever held twice
  sqa_block_pool* pool = sqa_block_pool_create(97);
  if (!pool) return 8;
  std::vector<std::vector<int32_t>> held;
  std::vector<int> owner(97, -1);
  unsigned long long x = 88172645463325252ull;
  for (int step = 0; step < 5000; ++step) {
    x ^= x << 13; x ^= x >> 7; x ^= x << 17;
    if (!held.empty() && (x & 1)) {
      const size_t k = (size_t)((x >> 8) % held.size());
      if (sqa_block_pool_give(pool, held[k].data(), (int32_t)held[k].size()) != SQA_OK) return 7;
      for (int32_t id : held[k]) owner[id] = -1;
      if (sqa_block_pool_give(pool, held[k].data(), (int32_t)held[k].size()) != SQA_ERR_SHAPE && !held[k].empty()) return 6;   // twice
      held.erase(held.begin() + (long)k);
    } else {
      const int32_t n = (int32_t)((x >> 8) % 40);
      std::vector<int32_t> ids((size_t)n + 1, -7);
      const int32_t before = sqa_block_pool_free_count(pool);
      const sqa_status st = sqa_block_pool_take(pool, n, ids.data());
      if (st == SQA_ERR_CAPACITY) { if (n <= before || ids[0] != -7) return 5; continue; }
      if (st != SQA_OK || ids[(size_t)n] != -7) return 4;
      ids.resize((size_t)n);
      for (int32_t id : ids) { if (id < 0 || id >= 97 || owner[id] != -1) return 3; owner[id] = step; }
      held.push_back(ids);
    }
  }
  int32_t out_of_range[2] = {0, 97};
  if (sqa_block_pool_give(pool, out_of_range, 2) != SQA_ERR_SHAPE) return 2;
  sqa_block_pool_destroy(pool);
  std::printf("pool ok\n");
  return 0;
}
''')
    exe = tmp_path / "driver"
    host_src = os.path.join(ROOT, "paper_2404_04793_amd", "csrc", "sqa_host.cpp")
    r = subprocess.run([gxx, "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined",
                        "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
                        "-I", os.path.join(ROOT, "include"), str(driver), host_src, "-o", str(exe)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    cases = []
    for seed in range(40):
        r_ = np.random.default_rng(seed)
        L = int(r_.integers(1, 100))
        cos = [r_.random(L), np.round(r_.random(L), 1), 0.9 + 0.05 * r_.standard_normal(L), np.arange(L) / max(L, 1)][seed % 4]
        cases.append((cos.astype(np.float32), int(r_.integers(L * 3, L * 4000 + 1)), float(r_.choice([0.1, 0.3, 0.35, 0.5, 1.0]))))
    cases += [(np.array([0.5], dtype=np.float32), 1, 1.0), (np.full(128, 0.25, dtype=np.float32), 128, 0.01),
              (np.array([0.1, 0.9], dtype=np.float32), 2, 0.5), (np.array([0.1, 0.5, 0.9], dtype=np.float32), 2, 0.3)]
    text = "".join("%d %d %.17g %s\n" % (len(c), t, p, " ".join("%.9g" % float(x) for x in c)) for c, t, p in cases)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe)], input=text, capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stderr[-2000:]
    lines = run.stdout.strip().splitlines()
    assert lines[-1] == "pool ok"
    lines = lines[:-1]
    assert len(lines) == len(cases)
    for (c, t, p), line in zip(cases, lines):
        parts = line.split()
        try:
            want = O.allocate_budgets(c, t, p)
        except ValueError:
            assert parts == ["5"], (line, t, p)
            continue
        assert parts[0] == "0"
        got = [tuple(int(v) for v in x.split(":")) for x in parts[1:]]
        assert [b for b, _ in got] == want[0] and [g for _, g in got] == want[1]
