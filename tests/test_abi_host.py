"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared symbol,
plans rows like the oracle, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "lowra.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lowra_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = lowra.lib()
    names = declared_symbols()
    assert set(names) == set(lowra.SYMBOLS)
    for name in names:
        assert getattr(L, name) is not None


def test_status_strings():
    assert lowra.status_string(0) == "ok"
    assert len({lowra.status_string(i) for i in range(6)}) == 6


def test_plan_rows_matches_oracle_and_rejects_bad_input():
    rng = np.random.default_rng(0)
    bits = rng.choice(np.array([1, 2, 4], np.uint8), size=1000)
    for K in (64, 4096, 13824):
        assert np.array_equal(lowra.lowra_plan_rows(K, bits), orc.row_offsets(K, bits))
    with pytest.raises(lowra.LowraError) as e:
        lowra.lowra_plan_rows(100, bits)
    assert e.value.status == lowra.UNSUPPORTED
    with pytest.raises(lowra.LowraError) as e:
        lowra.lowra_plan_rows(64, np.array([1, 3], np.uint8))
    assert e.value.status == lowra.UNSUPPORTED
    with pytest.raises(lowra.LowraError) as e:      # more than 4 GiB of codes
        lowra.lowra_plan_rows(1 << 20, np.full(1 << 13, 4, np.uint8))
    assert e.value.status == lowra.UNSUPPORTED


def test_layout_create_validates_on_host_first():
    """Every rejected argument is reported without a device; a valid one needs a device (HIP_ERROR here)."""
    _, _, cb_bits = synth.shared_codebooks()
    L = lowra.lib()
    h = C.c_void_p()

    def create(N, K, group, bits, cb, Cn, cbb):
        b = np.ascontiguousarray(bits, np.uint8); c = np.ascontiguousarray(cb, np.int32)
        q = np.ascontiguousarray(cbb, np.uint8)
        return L.lowra_layout_create(N, K, group, b.ctypes.data, c.ctypes.data, Cn, q.ctypes.data, C.byref(h))

    assert create(4, 128, 32, [1] * 4, [0] * 4, 3, cb_bits) == lowra.UNSUPPORTED      # group != 64
    assert create(4, 96, 64, [1] * 4, [0] * 4, 3, cb_bits) == lowra.UNSUPPORTED       # K % 64
    assert create(4, 128, 64, [1, 2, 8, 1], [0, 1, 2, 0], 3, cb_bits) == lowra.UNSUPPORTED
    assert create(4, 128, 64, [1] * 4, [0, 0, 3, 0], 3, cb_bits) == lowra.INVALID_ARG  # table index out of range
    assert create(4, 128, 64, [1, 2, 4, 1], [0, 1, 1, 0], 3, cb_bits) == lowra.INVALID_ARG  # width/table mismatch
    assert create(-1, 128, 64, [1], [0], 3, cb_bits) == lowra.INVALID_ARG
    assert L.lowra_layout_create(4, 128, 64, None, None, 3, None, C.byref(h)) == lowra.INVALID_ARG
    assert L.lowra_packed_bytes(None) == 0
    assert L.lowra_set_linear_path(7) == lowra.INVALID_ARG
    assert L.lowra_quantize(None, None, None, None, None, None) == lowra.INVALID_ARG
