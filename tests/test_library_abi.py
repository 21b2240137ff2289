"""The C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "zo2.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zo2_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_step_api():
    names = _declared()
    for must in ("zo2_init", "zo2_step", "zo2_set_resident_budget", "zo2_flush", "zo2_sync_to_host", "zo2_destroy"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2503_12668_amd import binding
    L = binding.lib()
    for name in _declared():
        assert hasattr(L, name), name
    assert sorted(binding.EXPORTED) == _declared()


def test_layout_helpers_and_argument_errors():
    from paper_2503_12668_amd import binding
    import synth_inputs as si
    L = binding.lib()
    assert [L.zo2_dtype_size(i) for i in range(6)] == [4, 2, 2, 1, 1, 0]
    cfg = si.opt_config("opt-125m")
    offs = binding.block_tensor_offsets(binding.make_config(cfg))
    d, f = 768, 3072
    sizes = [d, d, d * d, d, d * d, d, d * d, d, d * d, d, d, d, f * d, f, d * f, d]
    assert offs[0] == 0 and all(o % 256 == 0 for o in offs)
    for k in range(16):
        assert offs[k + 1] - offs[k] >= sizes[k] and offs[k + 1] - offs[k] < sizes[k] + 256
    bad = dict(cfg, d_model=770)
    with pytest.raises(binding.Zo2Error):
        binding.block_tensor_offsets(binding.make_config(bad))
    # NULL context
    assert L.zo2_flush(None) == 1 and L.zo2_step(None, None, None, 1, 1, 0, 1e-3, 0.0, None, None, None) == 1
