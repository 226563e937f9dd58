"""The C-ABI library loads without a GPU and exports every function include/hashattn.h declares;
argument checks that come before any HIP call return status codes."""
import ctypes as C
import os
import re

import paper_2412_14468_amd as ha
from paper_2412_14468_amd.binding import Config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hashattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hashattn_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert {"hashattn_encode_keys", "hashattn_encode_query", "hashattn_score_topk",
            "hashattn_gather_attend", "hashattn_create", "hashattn_destroy"} <= set(names)
    lib = ha.load()
    for n in names:
        assert getattr(lib, n) is not None, n


def test_create_rejects_bad_shapes_before_touching_the_device():
    lib = ha.load()
    h = C.c_void_p()
    cases = [
        (Config(64, 32, 8, 32, 0, 1, 1024, 32), ha.UNSUPPORTED, "head_dim"),
        (Config(128, 32, 8, 48, 0, 1, 1024, 32), ha.UNSUPPORTED, "bits"),
        (Config(128, 32, 5, 32, 0, 1, 1024, 32), ha.INVALID_ARG, "multiple"),
        (Config(128, 48, 16, 32, 0, 1, 1024, 32), ha.UNSUPPORTED, "group"),
        (Config(128, 32, 8, 32, 8, 1, 1024, 32), ha.UNSUPPORTED, "page_size"),
        (Config(128, 32, 8, 32, 0, 0, 1024, 32), ha.INVALID_ARG, "max_batch"),
        (Config(128, 32, 8, 32, 0, 1, 0, 32), ha.INVALID_ARG, "max_context"),
        (Config(128, 32, 8, 32, 0, 1, 1024, 0), ha.INVALID_ARG, "max_k"),
    ]
    for cfg, status, word in cases:
        assert lib.hashattn_create(C.byref(h), C.byref(cfg)) == status
        assert word in lib.hashattn_last_error(None).decode()
        assert not h.value
    assert lib.hashattn_create(None, None) == ha.INVALID_ARG
    assert lib.hashattn_destroy(None) == ha.OK
    assert lib.hashattn_scratch_bytes(None) == 0


def test_null_context_is_rejected():
    lib = ha.load()
    assert lib.hashattn_encode_query(None, None, None, 1, None, None) == ha.INVALID_ARG
    assert lib.hashattn_score_topk(None, None, None, 1, None, 1, None, None, None, None) == ha.INVALID_ARG
    assert lib.hashattn_gather_attend(None, None, None, None, None, 1, 1, 1.0, None, None) == ha.INVALID_ARG
    assert lib.hashattn_dense_attend(None, None, None, 1, 1.0, None, None) == ha.INVALID_ARG
    assert lib.hashattn_encode_keys(None, None, None, None, 1, 1, None, None) == ha.INVALID_ARG
    assert lib.hashattn_encode_score_topk(None, None, None, None, 1, None, 1, 0, 0, None, None, None, None, None) == ha.INVALID_ARG
    assert lib.hashattn_decode_step(None, None, None, None, None, None, None, 1, None, 1, 0, 0, 1.0, None, None, None, None,
                                    None, None) == ha.INVALID_ARG
    assert lib.hashattn_selftest_set_topk_path(None, 0) == ha.INVALID_ARG
