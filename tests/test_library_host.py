"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header
declares, and its weight layout / workspace arithmetic agree with the parameter inventory."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2408_05636_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "specdiff.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sd_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.lib()
    names = declared_functions()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


@pytest.mark.parametrize("name", ["tiny", "gpt2s", "gpt2xl", "llama8b"])
def test_weight_layout_matches_parameter_inventory(name):
    w = synth.workload(name)
    for cfg in (w["target"], w["drafter"]):
        layout = binding.sd_weight_layout(cfg)
        specs = synth.weight_specs(cfg)
        assert [l[0] for l in layout] == [s[0] for s in specs]
        end = 0
        for (lname, rows, cols, eb, off), (sname, shape, role) in zip(layout, specs):
            assert rows * cols == int(np.prod(shape)) and cols == shape[-1]
            assert eb == (4 if role in ("gain", "bias") or cfg.dtype == "f32" else 2)
            assert off % 256 == 0 and off >= end
            end = off + rows * cols * eb
        assert binding.sd_weight_bytes(cfg) >= end


def test_pack_weights_round_trip():
    cfg = synth.shrink(synth.workload("gpt2s")["drafter"], n_layer=1, vocab=300, n_ctx=64)
    W = synth.gen_weights(cfg, 1)
    buf = binding.pack_weights(cfg, W)
    for name, rows, cols, eb, off in binding.sd_weight_layout(cfg):
        raw = buf[off:off + rows * cols * eb]
        if eb == 2:
            back = (raw.view(np.uint16).astype(np.uint32) << 16).view(np.float32)
        else:
            back = raw.view(np.float32)
        assert np.array_equal(back, W[name].reshape(-1)), name


def test_workspace_bytes_and_config_validation():
    w = synth.workload("gpt2s")
    n1 = binding.sd_workspace_bytes(w["target"], w["drafter"], 1, 16)
    n2 = binding.sd_workspace_bytes(w["target"], w["drafter"], 2, 16)
    assert 0 < n1 < n2 < 2 ** 33
    assert binding.sd_workspace_bytes(w["drafter"], w["drafter"], 1, 16) == 0      # target must be causal
    assert binding.sd_workspace_bytes(w["target"], w["target"], 1, 16) == 0        # drafter must be bidirectional
    bad = synth.shrink(w["drafter"], vocab=1000)
    assert binding.sd_workspace_bytes(w["target"], bad, 1, 16) == 0                # vocabularies must agree
    assert binding.sd_workspace_bytes(w["target"], w["drafter"], 0, 16) == 0
    assert binding.sd_weight_bytes(synth.shrink(w["target"], n_head=7)) == 0       # d_model % n_head
    assert binding.sd_vocab_pad(50257) == 50432 and binding.sd_vocab_pad(512) == 512


def test_null_and_bad_arguments_are_reported_not_crashed():
    lib = binding.lib()
    out = C.c_void_p()
    cfg = binding.c_config(synth.workload("tiny")["target"])
    assert lib.sd_create(C.byref(cfg), C.byref(cfg), None, None, 1, 8, None, 0, None, C.byref(out)) == 1
    assert out.value is None
    assert lib.sd_prefill(None, 1, None, None) == 1
    assert lib.sd_last_error(None) == b"null handle"
    assert lib.sd_sampling_scratch_bytes(0, 100) == 0
    assert lib.sd_unmask_sample(None, 1, 1, 10, 1, 0, None, None, None, None, 0, None) == 1
    assert lib.sd_linear(0, None, None, None, None, 1, 1, 8, 1, 0, None, 0, None) == 1
    lib.sd_destroy(None)
