"""CPU-side checks of the boundary: the library loads, exports what the header declares, and
the host-only append planner follows the residual policy."""
import os
import re

from paper_2503_16163_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "specache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(specache_[a-z_]+)\s*\(", text))
    assert declared == set(binding.EXPORTS), declared ^ set(binding.EXPORTS)
    L = binding.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_plan_append_equals_token_by_token_simulation():
    import random
    rng = random.Random(5)
    for R, g in [(64, 32), (64, 64), (96, 32), (128, 64), (256, 32), (128, 128), (256, 128)]:
        for _ in range(500):
            r0, nq, n = rng.randrange(0, R), g * rng.randrange(0, 6), rng.randrange(0, 400)
            r, flushed = r0, 0
            for _ in range(n):
                r += 1
                if r == R:
                    flushed += 1
                    r -= g
            assert binding.plan_append(R, g, nq + r0, nq, n) == flushed


def test_plan_append_rejects_inconsistent_counts():
    import pytest
    for args in [(64, 32, 10, 20, 1), (64, 48, 0, 0, 1), (64, 32, 64, 0, 1), (64, 32, 0, 0, -1)]:
        with pytest.raises(binding.SpeCacheError):
            binding.plan_append(*args)


def test_config_struct_matches_header_field_order():
    text = open(os.path.join(ROOT, "include", "specache.h")).read()
    body = text[text.index("typedef struct specache_config {"):text.index("} specache_config;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(?:int32_t|float)\s+([a-z_]+)\s*;", body)
    assert fields == [f[0] for f in binding.Config._fields_]


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus N with N > 1 exits with a message that says so (before touching a GPU)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)


def test_arrangement_plan_on_the_benchmarks_shapes():
    """The stepping rule (host logic): what it picks for the shapes the benchmark and the full-size tests run, and
    its boundaries (one layer, non-speculative, shapes without the one-launch kernel)."""
    from paper_2503_16163_amd import arrangement as a
    p = a.plan(1, 32, 1, 32768, 256, 32)                       # 7B shape, k = 256: bound by the link
    assert (p["calls"], p["async_select"], p["side_streams"], p["carry_append"]) == ("one-pass", 2, 3, False)
    p = a.plan(1, 32, 1, 32768, 64, 32)                        # the paper's k: bound by compute
    assert (p["calls"], p["async_select"], p["side_streams"], p["carry_append"]) == ("one-pass", 2, 2, True)
    p = a.plan(1, 32, 1, 32768, 512, 32)                       # the link alone
    assert (p["calls"], p["async_select"], p["side_streams"]) == ("four", 1, 2)
    assert a.plan(16, 32, 1, 2048, 128, 4)["calls"] == "four"                      # config 3: 512 rows over the link
    assert a.plan(4, 8, 4, 32768, 512, 4)["calls"] == "split"                      # several query heads per KV head
    assert a.plan(1, 8, 4, 131072, 1024, 32, bits=1) == a.plan(4, 8, 4, 32768, 512, 4)
    assert a.plan(1, 32, 1, 32768, 64, 32, bits=1)["calls"] == "one-pass"          # 1-bit codes have the one-launch kernel
    assert a.plan(1, 32, 1, 32768, 64, 32, bits=4)["calls"] == "split"             # 4-bit codes do not
    assert a.plan(1, 32, 1, 32768, 64, 32, select_lowbit=False)["calls"] == "split"
    for p in (a.plan(1, 1, 1, 4096, 64, 1), a.plan(1, 32, 1, 32768, 256, 32, speculative=False)):
        assert (p["calls"], p["async_select"], p["side_streams"], p["carry_append"]) == ("four", 0, 1, False)
    assert abs(a.link_us(32, 256) - 72.9) < 0.1 and abs(a.main_us(32, 32768) - 42.8) < 0.1 and a.main_us(32, 4096) == 33.0


def test_kernel_source_hash_follows_the_kernels_own_sources():
    """Figures in profiles/*.json are tied to the sources of the kernel they were measured on: the .hip file that
    defines it and the headers it includes, nothing else."""
    import os
    from paper_2503_16163_amd import build, profile_summary
    names = lambda k: sorted(os.path.basename(f) for f in build.kernel_sources(k))
    assert names("topk_kernel") == ["kernels.h", "layout.h", "topk.hip"]
    assert "score_i8_wave.h" in names("attend_i8_kernel") and "attend.hip" not in names("attend_i8_kernel")
    assert build.kernel_sources("no_such_kernel") is None and build.kernel_source_hash("no_such_kernel") is None
    assert build.kernel_source_hash("topk_kernel") != build.kernel_source_hash("gather_kernel")
    full = "void specache::(anonymous namespace)::attend_i8_kernel<32, 2, false, true>(specache::LayerView, specache::(anonymous namespace)::AttendArgs, float, unsigned int*, unsigned long)"
    assert profile_summary.short_name(full) == "attend_i8_kernel+score"
    assert profile_summary.short_name(full.replace("false, true>", "false, false>")) == "attend_i8_kernel"
    assert profile_summary.short_name("void at::native::vectorized_elementwise_kernel<4>(int)") is None
    assert profile_summary.short_name("__amd_rocclr_copyBuffer") == profile_summary.COPY_KERNEL
