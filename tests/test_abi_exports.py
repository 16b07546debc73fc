"""The C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "rapidgnn.h")
LIB = os.path.join(ROOT, "paper_2505_10806_amd", "librapidgnn.so")


def _declared_symbols():
    text = open(HEADER).read()
    return sorted(set(re.findall(r"RG_API\s+[\w\s\*]+?\b(rg_\w+)\s*\(", text)))


def test_header_declares_the_path_entry_points():
    syms = _declared_symbols()
    for name in ("rg_sample_blocks", "rg_access_histogram", "rg_build_cache", "rg_gather_features",
                 "rg_epoch_schedule", "rg_create", "rg_destroy"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} is not built; run __graft_entry__.build()")
    lib = ctypes.CDLL(LIB)
    for name in _declared_symbols():
        assert hasattr(lib, name), name


def test_binding_lists_every_declared_symbol_and_has_no_fallback():
    from paper_2505_10806_amd import binding
    assert sorted(binding.EXPORTED_SYMBOLS) == _declared_symbols()
    assert "gfx950" in binding.version()
    src = open(os.path.join(ROOT, "paper_2505_10806_amd", "binding.py")).read()
    assert "oracle" not in src.replace("no fallback", "")


def test_bounds_match_closed_form():
    from paper_2505_10806_amd import binding
    fub, eub = binding.blocks_bounds(10_000_000, 500_000_000, 4096, (15, 10, 5))
    assert fub == [4096, 65536, 720896, 4325376] and eub == [61440, 655360, 3604480]
    fub, eub = binding.blocks_bounds(10_000, 200_000, 256, (10, 5))
    assert fub == [256, 2816, 10_000] and eub == [2560, 14080]
    fub, eub = binding.blocks_bounds(100, 50, 10, (binding.RG_FANOUT_ALL, 3))
    assert eub == [50, 50] and fub == [10, 60, 100]
    with pytest.raises(binding.RgError):
        binding.blocks_bounds(100, 50, 10, (binding.RG_MAX_FANOUT + 1,))


def test_create_without_gpu_fails_loudly():
    import torch
    from paper_2505_10806_amd import binding
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(binding.RgError) as e:
        binding.Context(0)
    assert e.value.status == binding.RG_ERR_HIP


def test_pipeline_call_sizes_cover_every_batch_once():
    """Host logic of the epoch driver: the batches of an epoch are dealt to sampler calls of at most `group` batches;
    with one pull per call a period opens with a single batch and closes with calls of 2, 1 and 1."""
    import types
    from paper_2505_10806_amd.pipeline import EpochPipeline
    grouped = types.SimpleNamespace(group_pulls=True)
    plain = types.SimpleNamespace(group_pulls=False)
    for group in (1, 2, 8, 16):
        for n in list(range(1, 40)) + [245, 1000]:
            for first in (False, True):
                for last in (False, True):
                    sizes = EpochPipeline._call_sizes(grouped, n, group, first, last)
                    assert sum(sizes) == n and all(1 <= x <= group for x in sizes), (group, n, first, last, sizes)
                    if group > 1 and n > 1 and first:
                        assert sizes[0] == 1
                    if group > 1 and n >= 6 and last:
                        assert sizes[-3:] == [2, 1, 1]
            assert EpochPipeline._call_sizes(plain, n, group, True, True) == [group] * (n // group) + ([n % group] if n % group else [])
