"""CPU-side checks of the C-ABI library: it loads, exports what the header declares,
and its host-only entry points agree with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import sampler as S
from oracle import search as K
from paper_2203_05705_amd import binding as ard

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    with open(os.path.join(ROOT, "include", "ard.h")) as f:
        src = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    return sorted(set(re.findall(r"\b(ard_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 14
    handle = ctypes.CDLL(ard.LIB_PATH)
    for n in names:
        assert hasattr(handle, n), f"{n} declared in include/ard.h but not exported"
    assert sorted(ard.exported_symbols()) == names          # the binding covers the whole header
    assert ard.lib().ard_version() >= 100


@pytest.mark.parametrize("p", [0.3, 0.5, 0.7])
def test_search_k_matches_oracle(p):
    k, cdf = ard.search_k(p, 8)
    d, _ = K.search_k(p, 8)
    assert abs(sum(k) - 1) < 1e-12
    assert np.max(np.abs(np.array(k) - d)) < 5e-5
    assert cdf[-1] == 1 << 32 and all(cdf[i] <= cdf[i + 1] for i in range(7))
    # the library's own table is the fixed-point image of its own k
    assert [int(c) for c in K.fixed_point_cdf(np.array(k))] == cdf


def test_pattern_sample_bit_exact_against_oracle():
    d, _ = K.search_k(0.5, 8)
    cdf = [int(c) for c in K.fixed_point_cdf(d)]
    for seed in (0, 2, 12345678901234567):
        for stream_id in (0, 1, 7):
            for it in list(range(100)) + [1 << 40, (1 << 64) - 1]:
                assert ard.pattern_sample(cdf, seed, it, stream_id) == S.sample_pattern(cdf, seed, it, stream_id)
    edge = [0, 0, 5, 1 << 32]
    for it in range(200):
        assert ard.pattern_sample(edge, 9, it, 3) == S.sample_pattern(edge, 9, it, 3)


def test_host_side_argument_errors():
    lib = ard.lib()
    with pytest.raises(ard.ArdError) as e:
        ard.search_k(1.0, 8)
    assert e.value.code == -1
    with pytest.raises(ard.ArdError) as e:
        ard.search_k(0.5, 0)
    assert e.value.code == -2
    # argument checks run before anything touches the device: fake non-null pointers are never dereferenced
    fake = ctypes.c_void_p(0x1000)
    bad = ard.CPattern(ard.PAT_ROW, 3, 4, 0, 0, 0, None, None, None, None, None)      # b > dp
    code = lib.ard_drop_gemm_fwd(ard.F32, 4, 8, 8, fake, fake, fake, ctypes.byref(bad), None, 1.0, 0, 0, None, 0, None)
    assert code == -1 and b"b=4" in lib.ard_last_error()
    bad = ard.CPattern(ard.PAT_ROW, 9, 1, 0, 0, 0, None, None, None, None, None)      # dp > number of rows
    code = lib.ard_drop_gemm_fwd(ard.F32, 4, 8, 8, fake, fake, fake, ctypes.byref(bad), None, 1.0, 0, 0, None, 0, None)
    assert code == -1
    ok = ard.CPattern(ard.PAT_ROW, 2, 1, 0, 0, 0, None, None, None, None, None)
    assert lib.ard_drop_gemm_fwd(ard.F32, 0, 8, 8, fake, fake, fake, ctypes.byref(ok), None, 1.0, 0, 0, None, 0, None) == -2
    assert lib.ard_drop_gemm_fwd(7, 4, 8, 8, fake, fake, fake, ctypes.byref(ok), None, 1.0, 0, 0, None, 0, None) == -3
    assert lib.ard_drop_gemm_fwd(ard.F32, 4, 8, 8, None, fake, fake, ctypes.byref(ok), None, 1.0, 0, 0, None, 0, None) == -1
    tile = ard.CPattern(ard.PAT_TILE, 2, 1, 64, 64, 0, None, None, None, None, None)
    assert lib.ard_drop_gemm_fwd(ard.BF16, 4, 128, 128, fake, fake, fake, ctypes.byref(tile), None, 1.0, 0, 0, None, 0, None) == -4
    assert lib.ard_gemm_workspace_bytes(ard.BF16, 4, 128, 128, ctypes.byref(tile), None) > 0
    assert lib.ard_pattern_gen(ctypes.byref(ok), 0, 0, None, None, None, None, None, None, None) == -2
    assert lib.ard_pattern_gen(None, 8, 0, None, None, None, None, None, None, None) == -1
