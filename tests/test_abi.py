"""The C-ABI library: it loads, exports every symbol the header declares, and rejects bad
descriptions on the host before touching the GPU.  No compute calls here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2603_17573_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build(force=False)
    return binding.load()


def declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names.update(re.findall(r"\b(heisd_[a-z_0-9]+)\s*\(", text))
    return names


def test_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert {"heisd_verify_init", "heisd_verify_step", "heisd_free", "heisd_verify_workspace_bytes",
            "heisd_last_error"} <= names
    for n in names:
        assert hasattr(lib, n), "library does not export %s" % n


def test_struct_layouts_match_header():
    from paper_2603_17573_amd import binding as B
    assert ctypes.sizeof(B.heisd_accept_desc) == 4 * 3 + 4 * 8 + 4 + 4
    assert ctypes.sizeof(B.heisd_kv_desc) == 4 * 8
    assert B.heisd_model_desc.tok_emb.offset == 56 and ctypes.sizeof(B.heisd_model_desc) == 56 + 8 * 14


def test_host_side_validation(lib):
    from paper_2603_17573_amd import binding as B
    shape = dict(n_layers=1, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1000, n_bins=256,
                 bin_token_base=744, rms_eps=1e-6, rope_base=1e4)
    fake = 0x1000   # never dereferenced: every check below fails before any device access
    ptrs = {k: [fake] for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "attn_norm", "ffn_norm")}
    ptrs.update(tok_emb=fake, lm_head=fake, final_norm=fake)
    desc, keep = B.make_model_desc(shape, ptrs, 2, 7, 80)
    need = B.heisd_verify_workspace_bytes(desc)
    assert need > 2 * 7 * (256 * 5 + 688 + 256) * 4
    rc, ctx = B.heisd_verify_init(desc)                       # workspace NULL
    assert rc == B.HEISD_EINVAL and ctx is None and "NULL" in B.heisd_last_error(None)
    desc.workspace, desc.workspace_bytes = 0x10000, need - 1
    assert B.heisd_verify_init(desc)[0] == B.HEISD_ENOMEM
    desc.workspace = 0x10010
    desc.workspace_bytes = need
    assert B.heisd_verify_init(desc)[0] == B.HEISD_EINVAL    # misaligned workspace
    bad = dict(shape, head_dim=32, n_heads=8)
    d2, k2 = B.make_model_desc(bad, ptrs, 2, 7, 80, 0x10000, 1 << 30)
    assert B.heisd_verify_init(d2)[0] == B.HEISD_EUNSUPPORTED
    bad = dict(shape, n_heads=3)
    d3, k3 = B.make_model_desc(bad, ptrs, 2, 7, 80, 0x10000, 1 << 30)
    assert B.heisd_verify_init(d3)[0] == B.HEISD_EINVAL and B.heisd_verify_workspace_bytes(d3) == 0
    bad = dict(shape, bin_token_base=800)
    d4, k4 = B.make_model_desc(bad, ptrs, 2, 7, 80, 0x10000, 1 << 30)
    assert B.heisd_verify_init(d4)[0] == B.HEISD_EINVAL
    assert lib.heisd_verify_step(None, None, None, 7, 1, None, None, None, None, None, None, None) == B.HEISD_EINVAL
    lib.heisd_free(None)
