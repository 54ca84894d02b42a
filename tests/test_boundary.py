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
