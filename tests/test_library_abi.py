"""Host-side checks that need no GPU: the library loads and exports every declared symbol."""
import ctypes
import os
import re

from helpers import ROOT, load_binding


def declared_functions():
    """Every function that any header under include/ declares."""
    names = set()
    inc = os.path.join(ROOT, "include")
    headers = sorted(f for f in os.listdir(inc) if f.endswith(".h"))
    assert "cqa.h" in headers and "cqa_test.h" in headers
    for f in headers:
        text = open(os.path.join(inc, f)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(cqa_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_the_product_header_holds_no_test_hooks():
    text = open(os.path.join(ROOT, "include", "cqa.h")).read()
    for hook in ("cqa_set_splits", "cqa_set_kernel_variant", "cqa_set_stream_hint", "cqa_adaptive_state",
                 "cqa_time_", "cqa_profile_"):
        assert hook not in text, hook


def test_every_declared_symbol_is_exported_and_bound():
    cqa = load_binding()
    names = declared_functions()
    assert len(names) >= 15
    lib = ctypes.CDLL(cqa.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/*.h but not exported"
        assert n in cqa.EXPORTED, f"{n} has no ctypes signature in the binding"
        assert hasattr(cqa, n), f"{n} has no Python wrapper"
    assert cqa.cqa_version() == 100


def test_struct_layouts_match_the_header():
    cqa = load_binding()
    assert ctypes.sizeof(cqa.HeadCert) == 40
    assert ctypes.sizeof(cqa.Tolerances) == 48
    assert ctypes.sizeof(cqa.CacheDesc) == 40
    assert ctypes.sizeof(cqa.Selector) == 40
    assert cqa.CERT_BYTES == 40


def test_host_side_argument_checks_need_no_gpu():
    cqa = load_binding()
    d = cqa.CacheDesc(1, 1, 32, 8, 128, 16, 16, 0, 131072)
    dev, pin = cqa.cqa_workspace_bytes(d)
    # Tier-1 is 288.5 bytes per token per kv head; Tier-2 is 512
    assert dev >= 131072 * 8 * 288.5 and pin >= 131072 * 8 * 512
    # + fallback staging for one KV group (2 buffers x K, V) and the adaptive-precision scratch
    assert dev < 131072 * 8 * 288.5 * 1.8
    for bad in (cqa.CacheDesc(1, 1, 32, 8, 64, 16, 16, 0, 1024),      # head_dim
                cqa.CacheDesc(1, 1, 32, 8, 128, 32, 16, 0, 1024),     # block
                cqa.CacheDesc(1, 1, 32, 8, 128, 16, 32, 0, 1024),     # group
                cqa.CacheDesc(1, 1, 24, 8, 128, 16, 16, 0, 1024)):    # GQA 3
        try:
            cqa.cqa_workspace_bytes(bad)
            assert False, "expected an error"
        except cqa.CqaError as e:
            assert e.status == cqa.ERR_UNSUPPORTED
    try:
        cqa.cqa_workspace_bytes(cqa.CacheDesc(1, 1, 30, 8, 128, 16, 16, 0, 1024))
        assert False
    except cqa.CqaError as e:
        assert e.status == cqa.ERR_INVALID_ARG
    assert "Tier 2" in cqa.cqa_strerror(cqa.ERR_NO_TIER2)
