"""CPU-side checks of the boundary: the library loads without a GPU, exports everything include/nexus.h declares,
and its host-only logic (split selection) agrees with the oracle's rule and with an exhaustive scan."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "nexus.h")


@pytest.fixture(scope="module")
def binding():
    from paper_2507_06608_amd import binding as b
    from paper_2507_06608_amd import build
    if build.stale():
        build.build()
    b.lib()
    return b


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(nexus_[a-z_0-9]+)\s*\(", src)))


def test_header_declares_the_five_entry_points():
    names = declared_functions()
    for n in ("nexus_mixed_step", "nexus_prefill_chunk", "nexus_decode_step", "nexus_set_cu_split",
              "nexus_profile_split"):
        assert n in names


def test_library_exports_every_declared_symbol(binding):
    lib = binding.lib()
    names = declared_functions()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), f"{n} declared in nexus.h but not exported"
    assert set(binding.EXPORTS) == set(names)


def test_struct_sizes_match_the_header_layout(binding):
    # field-by-field C layout: 7 int32 + 2 float; 4 int32; 7 pointers; 2 pointers + int64 + int32 (padded)
    assert ctypes.sizeof(binding.ModelDesc) == 36
    assert ctypes.sizeof(binding.Limits) == 16
    assert ctypes.sizeof(binding.LayerWeights) == 56
    assert ctypes.sizeof(binding.KVCache) == 32
    assert ctypes.sizeof(binding.PrefillBatchC) == 8 + 5 * 8 + 12 + 4
    assert ctypes.sizeof(binding.DecodeBatchC) == 8 + 4 * 8 + 8
    assert ctypes.sizeof(binding.StepTiming) == 12


def test_choose_split_matches_oracle_rule_and_exhaustive_scan(binding, oracle):
    r = np.random.default_rng(17)
    for trial in range(200):
        n = int(r.integers(1, 9))
        t_p = (r.random(n) * 3 + 0.5).astype(np.float32)
        t_d = (r.random(n) * 3 + 0.5).astype(np.float32)
        t_s = (np.maximum(t_p, t_d) + r.random(n)).astype(np.float32)
        tpa, tda = float(np.float32(t_p.min() * r.uniform(0.6, 1.1))), float(np.float32(t_d.min() * r.uniform(0.6, 1.1)))
        for pol in (0, 1, 2):
            a, b = float(np.float32(r.uniform(1.0, 1.6))), float(np.float32(r.uniform(1.0, 1.6)))
            got = binding.choose_split(t_p, t_d, t_s, tpa, tda, pol, a, b)
            assert got == oracle.choose_split(t_p, t_d, t_s, tpa, tda, pol, a, b)


def test_choose_split_rejects_bad_arguments(binding):
    t = np.ones(3, np.float32)
    with pytest.raises(binding.NexusError):
        binding.choose_split(t, t, t, 1.0, 1.0, 7, 1.3, 1.1)
    with pytest.raises(binding.NexusError):
        binding.choose_split(t[:0], t[:0], t[:0], 1.0, 1.0, 0, 1.3, 1.1)


def test_monotone_curves_pick_the_papers_operating_points(binding):
    # prefill time falls as 1/share; decode saturates early (flat beyond half the CUs): with slack 1.1 on decode the
    # prefill-prioritised rule hands prefill as much as decode tolerates, the decode-prioritised rule the reverse.
    share = np.arange(1, 8) / 8.0
    t_p = (1.0 / share).astype(np.float32)
    t_d = np.where(1 - share >= 0.5, 1.0, 1.0 + 2.0 * (0.5 - (1 - share))).astype(np.float32)
    t_s = np.maximum(t_p, t_d)
    assert binding.choose_split(t_p, t_d, t_s, 1.0, 1.0, 0, 1.3, 1.1) == 3      # 4/8: largest share with t_d <= 1.1
    assert binding.choose_split(t_p, t_d, t_s, 1.0, 1.0, 1, 1.3, 1.1) == 6      # only 7/8 keeps t_p <= 1.3
    assert binding.choose_split(t_p, t_d, t_s, 1.0, 1.0, 2, 1.3, 1.1) == int(np.argmin(t_s))


def test_token_order_of_the_per_token_kernels_is_a_permutation_in_xcd_runs(binding):
    """Workgroup b -> token: a permutation of [0, n) for every n (a token skipped or visited twice would go unnoticed
    by nothing but parity), and in whole groups the 8 XCDs (workgroup index modulo 8) get runs of consecutive tokens."""
    lib = binding.lib()
    order = lambda n: [lib.nexus_debug_token_order(b, n) for b in range(n)]
    for n in list(range(1, 140)) + [255, 256, 257, 320, 511, 512, 513, 1000, 8192]:
        o = order(n)
        assert sorted(o) == list(range(n)), n
        full256, full64 = n // 256 * 256, n // 64 * 64
        assert o[full64:] == list(range(full64, n))                     # the tail keeps its order
        for g0 in range(0, full256, 256):                                # 32 consecutive tokens per XCD
            for x in range(8):
                toks = sorted(o[b] for b in range(g0, g0 + 256) if b % 8 == x)
                assert toks == list(range(g0 + 32 * x, g0 + 32 * x + 32))
        for g0 in range(full256, full64, 64):                            # 8 consecutive tokens per XCD
            for x in range(8):
                toks = sorted(o[b] for b in range(g0, g0 + 64) if b % 8 == x)
                assert toks == list(range(g0 + 8 * x, g0 + 8 * x + 8))
    assert lib.nexus_debug_token_order(5, 5) < 0 and lib.nexus_debug_token_order(-1, 5) < 0
