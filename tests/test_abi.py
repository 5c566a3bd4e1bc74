"""CPU-side checks of the boundary: the library loads and exports every symbol the header declares;
argument validation that needs no GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "rlhf_rollout.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:rlhf_|rollout_|score_)[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2403_17031_amd as P
    if not os.path.exists(P.LIB_PATH):
        from paper_2403_17031_amd.build import build
        build()
    lib = P.load_library()
    names = _declared_symbols()
    assert "rollout_generate" in names and "score_sequences" in names and len(names) >= 10
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in the header but not exported"
    assert set(names) == set(P.binding.EXPORTS)


def test_null_arguments_are_rejected_without_a_gpu():
    import paper_2403_17031_amd as P
    lib = P.load_library()
    out = C.c_void_p()
    assert lib.rlhf_create(None, None, None, 0, C.byref(out)) == -1
    assert out.value is None
    assert b"null" in lib.rlhf_last_error()
    sz = C.c_size_t()
    assert lib.rlhf_weight_image_bytes(None, C.byref(sz)) == -1
    assert lib.rlhf_refresh_weights(None, None) == -1
    assert lib.rlhf_workspace_bytes(None, 1, 1, 1, 1, C.byref(sz)) == -1
    assert lib.rollout_generate(None, None, None, 1, 1, 0, 0, 0.7, 1, None, None, None, None, None, 0, None) == -1
    assert lib.score_sequences(None, None, None, 1, 1, 0.7, None, None, None, 0, None) == -1
    lib.rlhf_destroy(None)  # no-op


def test_weight_image_size_is_the_fp16_copy_of_the_matrices():
    """The caller-owned image holds, per layer, W_qkv + its bias, W_fc1 and W_o | W_fc2, then the LM head, in fp16;
    an fp32 model needs none."""
    import paper_2403_17031_amd as P
    from paper_2403_17031_amd.binding import _Config
    lib = P.load_library()
    sz = C.c_size_t()
    L, d, F, V = 3, 64, 256, 1000
    c = _Config(L, d, 4, 16, 4, F, V, 1, 0, V - 1, 1e-5, 10000.0)
    assert lib.rlhf_weight_image_bytes(C.byref(c), C.byref(sz)) == 0
    assert sz.value == 2 * (L * (3 * d * d + 3 * d + d * d + 2 * d * F) + V * d)
    c.dtype = 0
    assert lib.rlhf_weight_image_bytes(C.byref(c), C.byref(sz)) == 0 and sz.value == 0


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    import paper_2403_17031_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(b.RlhfError, match="missing"):
        b.load_library()
