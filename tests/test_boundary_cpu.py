"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, exports every symbol
the public header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2504_00970_amd as skv
from paper_2504_00970_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "sentencekv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(skv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding._lib()
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(skv.EXPORTS) == names


def test_strerror_covers_every_status():
    lib = binding._lib()
    msgs = {lib.skv_strerror(c).decode() for c in (0, -1, -2, -3, -4)}
    assert len(msgs) == 5 and lib.skv_strerror(-99).decode() == "unknown status"


@pytest.mark.parametrize("field,value", [("head_dim", 64), ("n_q_heads", 30), ("kv_dtype", 7), ("max_budget", 0),
                                         ("n_kv_heads", 0), ("max_batch", 0), ("n_q_heads", 8 * 16), ("semvec_dtype", 3), ("kv_dtype", 2), ("max_batch", 4097)])
def test_create_rejects_bad_descriptors_before_touching_the_gpu(field, value):
    kw = dict(n_layers=1, n_q_heads=32, n_kv_heads=8, max_tokens=64, max_sentences=8, max_budget=16)
    kw[field] = value
    with pytest.raises(skv.SkvError) as e:
        skv.Context(skv.Desc(**kw))
    assert e.value.status == skv.SKV_EINVAL


def test_null_context_and_null_out_pointer_are_invalid_arguments():
    lib = binding._lib()
    assert lib.skv_create(None, None, None) == skv.SKV_EINVAL
    assert lib.skv_score(None, 0, None, None, 0, None) == skv.SKV_EINVAL
    assert lib.skv_attend(None, None, None, None, None, 0, None, None) == skv.SKV_EINVAL
    assert lib.skv_set_stream(None, None) == skv.SKV_EINVAL
    assert lib.skv_workspace_bytes(None) == 0
    assert lib.skv_query_update(None, 1, None, None, None, 8, None, None, None) == skv.SKV_EINVAL
    assert lib.skv_build_semvec_layers(None, None, 0, None, 0, None) == skv.SKV_EINVAL
    assert lib.skv_token_importance_work_bytes(None, 100, 8) == -1
    assert lib.skv_token_importance(None, None, None, 100, 8, None, None, 0) == skv.SKV_EINVAL
    assert lib.skv_retain(None, None, 1, 1, None, 1, None, None, None, None) == skv.SKV_EINVAL
    assert lib.skv_compact_pool(None, None, None, 1, None, 1, None, None, None) == skv.SKV_EINVAL
    assert lib.skv_merge_lse(None, 1, None, None, None, None, None, None) == skv.SKV_EINVAL
    lib.skv_destroy(None)      # no-op


def test_product_package_does_not_reach_into_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_00970_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower(), f
