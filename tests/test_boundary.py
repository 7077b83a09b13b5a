"""The C boundary without a GPU: the library loads, exports what the header declares, and its
host-only entry points behave."""
import ctypes
import os
import re

import pytest

from paper_2511_20100_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2511_20100_amd", "libmtmc.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2511_20100_amd import build
        build.build(verbose=False)
    return ctypes.CDLL(LIB)


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mtmc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mtmc_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"mtmc_rollout", "mtmc_score", "mtmc_weights_create", "mtmc_weights_destroy"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_lists_the_same_entry_points():
    from paper_2511_20100_amd import mtmc
    assert sorted(mtmc.EXPORTS) == declared_symbols()
    for n in mtmc.EXPORTS:
        assert hasattr(mtmc, n) or n == "mtmc_last_error"


def test_binding_constants_match_the_header():
    from paper_2511_20100_amd import mtmc
    text = open(os.path.join(ROOT, "include", "mtmc.h")).read()
    defines = {k: v.strip("()") for k, v in re.findall(r"^#define\s+(MTMC_[A-Z0-9_]+)\s+(\(?-?\d+\)?)", text, flags=re.M)}
    assert {"MTMC_OK", "MTMC_EINVAL", "MTMC_BF16", "MTMC_MAX_DECODE_CONTEXT", "MTMC_OPT_HIP_GRAPH"} <= set(defines)
    for name, value in defines.items():
        assert getattr(mtmc, name) == int(value), name


@pytest.mark.parametrize("cfg", [inputs.TINY, inputs.POLICY_1P5B, inputs.POLICY_7B,
                                 inputs.TINY.with_(dtype="bf16", head_dim=128, n_q_heads=2, n_kv_heads=1)])
def test_blob_size_agrees_with_the_input_generator(cfg):
    from paper_2511_20100_amd import mtmc
    _, total = inputs.blob_layout(cfg)
    assert mtmc.mtmc_blob_bytes(mtmc.make_config(cfg, 4096)) == total


def test_invalid_configurations_are_rejected():
    from paper_2511_20100_amd import mtmc
    bad = [inputs.TINY.with_(head_dim=48), inputs.TINY.with_(n_q_heads=3), inputs.TINY.with_(d_model=250),
           inputs.TINY.with_(vocab=0)]
    for cfg in bad:
        assert mtmc.mtmc_blob_bytes(mtmc.make_config(cfg, 64)) == 0
        assert "invalid argument" in mtmc.mtmc_last_error()
    c = mtmc.make_config(inputs.TINY, 64)
    c.page_tokens = 8
    assert mtmc.mtmc_blob_bytes(c) == 0


def test_data_flag_text_names_each_cause():
    """What mtmc_poll_errors reports for each bit of the device's sticky data flag (host-only call)."""
    from paper_2511_20100_amd import mtmc
    assert mtmc.mtmc_data_error_string(0) == ""
    assert "token id" in mtmc.mtmc_data_error_string(mtmc.MTMC_DATA_TOKEN_ID)
    assert "length" in mtmc.mtmc_data_error_string(mtmc.MTMC_DATA_LENGTH)
    assert "weight" in mtmc.mtmc_data_error_string(mtmc.MTMC_DATA_WEIGHT)
    sat = mtmc.mtmc_data_error_string(mtmc.MTMC_DATA_FP16_RANGE)
    assert "fp16 range" in sat and "65504" in sat and "clamped" in sat and "token id" not in sat
    both = mtmc.mtmc_data_error_string(mtmc.MTMC_DATA_TOKEN_ID | mtmc.MTMC_DATA_FP16_RANGE)
    assert "token id" in both and "fp16 range" in both and "; " in both


def test_blob_roundtrip():
    w = inputs.make_weights(inputs.TINY.with_(n_layers=1), seed=3)
    blob = w.blob()
    w2 = inputs.weights_from_blob(w.cfg, blob)
    for n in w.names():
        assert (w.f32(n) == w2.f32(n)).all()
    wb = inputs.make_weights(inputs.TINY.with_(n_layers=1, dtype="bf16"), seed=3)
    # bf16 storage holds the nearest bf16 of the fp32 draw
    import numpy as np
    a, b = w.f32("lm_head"), wb.f32("lm_head")
    assert np.abs(a - b).max() <= np.abs(a).max() * 2.0 ** -8
    assert ((wb.tensors["lm_head"].astype(np.uint32) << 16).view(np.float32) == b).all()


def test_product_sources_never_touch_the_oracle():
    """The oracle is test infrastructure: nothing in the package (Python or HIP) or in the C header
    may import, include or name it, and the two sides share no source file."""
    import os
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    offenders = []
    for base in ("paper_2511_20100_amd", "include"):
        for dirpath, _, files in os.walk(os.path.join(root, base)):
            for f in files:
                if not f.endswith((".py", ".h", ".hip", ".cpp", ".c")):
                    continue
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                if f == "inputs.py":  # the seeded input generators serve both sides and import neither
                    assert not re.search(r"^\s*(import|from)\s+(mtmc_oracle|oracle|\.mtmc|paper_2511_20100_amd\.mtmc)", text, re.M)
                    continue
                if re.search(r"\boracle\b", text):
                    offenders.append(os.path.join(dirpath, f))
    assert offenders == []
    oracle_text = "".join(open(os.path.join(root, "oracle", f)).read() for f in os.listdir(os.path.join(root, "oracle"))
                          if f.endswith(".py"))
    assert "paper_2511_20100_amd" not in oracle_text and "libmtmc" not in oracle_text
