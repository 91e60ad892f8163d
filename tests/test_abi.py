"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every function the
header declares, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

from paper_2502_14051_amd import rocketkv as rk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(rk.LIB_PATH):
        from paper_2502_14051_amd import build
        build.build()
    return rk.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "rocketkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rocketkv_[a-z_0-9]+)\s*\(", text)))


def test_exports_match_header(L):
    names = declared_functions()
    assert set(names) == set(rk.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_version_and_error_string(L):
    assert L.rocketkv_version() >= 100
    assert isinstance(rk.last_error(), str)


def fake_cache(**kw):
    d = dict(batch=2, n_q_heads=32, n_kv_heads=8, head_dim=128, page_size=16, pages_cap=256,
             n_phys_pages=512, stride_page=8 * 16 * 128, stride_head=16 * 128,
             seq_lens=0x1000, block_table=None, k_pool=0x10000, v_pool=0x20000)
    d.update(kw)
    return rk.CacheStruct(**d)


def test_workspace_query_needs_no_device(L):
    st = fake_cache()
    n = L.rocketkv_workspace_bytes(rk.OP_HSA_DECODE, C.byref(st), 1024, 0)
    assert n > 0 and n % 256 == 0
    assert L.rocketkv_workspace_bytes(rk.OP_DENSE_DECODE, C.byref(st), 0, 0) > 0
    assert L.rocketkv_workspace_bytes(rk.OP_SNAPKV, C.byref(st), 32, 1024) > 0
    assert L.rocketkv_workspace_bytes(rk.OP_ATTEND, C.byref(st), 64, 0) > 0
    assert L.rocketkv_workspace_bytes(99, C.byref(st), 0, 0) == 0 and "unknown op" in rk.last_error()
    assert L.rocketkv_workspace_bytes(rk.OP_HSA_DECODE, C.byref(st), 0, 0) == 0
    assert L.rocketkv_workspace_bytes(rk.OP_SNAPKV, C.byref(st), 32, 32) == 0


BAD_CACHES = [
    (dict(n_q_heads=30), rk.INVALID_ARG, "multiple"),
    (dict(head_dim=64), rk.UNSUPPORTED, "head_dim"),
    (dict(head_dim=0), rk.INVALID_ARG, "head_dim"),
    (dict(n_q_heads=8 * 32), rk.UNSUPPORTED, "group size"),
    (dict(page_size=0), rk.INVALID_ARG, "page_size"),
    (dict(pages_cap=250), rk.INVALID_ARG, "pages_cap"),
    (dict(batch=0), rk.INVALID_ARG, "positive"),
    (dict(k_pool=None), rk.INVALID_ARG, "NULL"),
    (dict(seq_lens=None), rk.INVALID_ARG, "NULL"),
    (dict(stride_head=100), rk.INVALID_ARG, "strides"),
    (dict(n_phys_pages=100), rk.INVALID_ARG, "identity block table"),
    (dict(k_pool=0x10004), rk.INVALID_ARG, "aligned"),
]


@pytest.mark.parametrize("kw,status,needle", BAD_CACHES)
def test_bad_cache_is_rejected_before_launch(L, kw, status, needle):
    st = fake_cache(**kw)
    r = L.rocketkv_build_page_summaries(C.byref(st), 0x100, 0x200, 0, -1, None)
    assert r == status, rk.last_error()
    assert needle in rk.last_error()


def test_null_and_range_arguments(L):
    st = fake_cache()
    q, kx, kn, out, ws = 0x1000, 0x2000, 0x3000, 0x4000, 0x5000
    assert L.rocketkv_build_page_summaries(None, kx, kn, 0, -1, None) == rk.INVALID_ARG
    assert L.rocketkv_build_page_summaries(C.byref(st), None, kn, 0, -1, None) == rk.INVALID_ARG
    assert L.rocketkv_build_page_summaries(C.byref(st), kx, kn, -1, -1, None) == rk.INVALID_ARG
    dec = lambda **k: L.rocketkv_hsa_decode(C.byref(st), k.get("q", q), kx, kn, k.get("k1", 32),
                                            k.get("T", 1024), k.get("nr", 0), k.get("out", out),
                                            None, None, None, k.get("ws", ws), k.get("wsb", 1 << 30),
                                            None)
    assert dec(q=None) == rk.INVALID_ARG
    assert dec(k1=0) == rk.INVALID_ARG and "channel_budget" in rk.last_error()
    assert dec(k1=129) == rk.INVALID_ARG
    assert dec(T=0) == rk.INVALID_ARG and "token_budget" in rk.last_error()
    assert dec(nr=-1) == rk.INVALID_ARG
    assert dec(out=None) == rk.INVALID_ARG
    assert dec(ws=None) == rk.WORKSPACE_TOO_SMALL
    assert dec(wsb=16) == rk.WORKSPACE_TOO_SMALL and "workspace" in rk.last_error()
    assert dec(ws=0x5010) == rk.INVALID_ARG and "aligned" in rk.last_error()
    st3 = fake_cache(page_size=3, stride_head=3 * 128, stride_page=8 * 3 * 128)
    assert L.rocketkv_attend(C.byref(st3), q, None, 0, out, None, ws, 1 << 30, None) == rk.UNSUPPORTED
    big = fake_cache(pages_cap=rk.MAX_PAGES + 8, n_phys_pages=4 * (rk.MAX_PAGES + 8))
    assert L.rocketkv_hsa_select(C.byref(big), q, kx, kn, 32, 1024, 0, 0x6000, 64, None, None,
                                 None) == rk.UNSUPPORTED
    assert L.rocketkv_hsa_select(C.byref(st), q, kx, kn, 32, 1024, 0, 0x6000, 8, None, None,
                                 None) == rk.INVALID_ARG and "pages_row_len" in rk.last_error()
    assert L.rocketkv_append_kv(C.byref(st), None, q, kx, kn, None) == rk.INVALID_ARG
    assert L.rocketkv_workspace_init(None, 1024, None) == rk.INVALID_ARG
    assert L.rocketkv_workspace_init(0x5010, 1024, None) == rk.INVALID_ARG


def test_snapkv_argument_checks(L):
    src = fake_cache(pages_cap=2048, n_phys_pages=4096)
    dst = fake_cache(k_pool=0x30000, v_pool=0x40000)
    call = lambda **k: L.rocketkv_snapkv_compress(k.get("qobs", 0x1000), C.byref(k.get("src", src)),
                                                  k.get("W", 32), k.get("ks", 63), k.get("N", 1024),
                                                  C.byref(k.get("dst", dst)), None, k.get("ws", 0x5000),
                                                  k.get("wsb", 1 << 40), None)
    assert call(qobs=None) == rk.INVALID_ARG
    assert call(ks=62) == rk.INVALID_ARG and "odd" in rk.last_error()
    assert call(W=0) == rk.INVALID_ARG
    assert call(W=24) == rk.UNSUPPORTED
    assert call(N=32) == rk.INVALID_ARG and "exceed" in rk.last_error()
    assert call(N=8192) == rk.INVALID_ARG and "dst holds" in rk.last_error()
    assert call(dst=fake_cache(n_kv_heads=4, k_pool=0x30000, v_pool=0x40000)) == rk.INVALID_ARG
    assert call(dst=src) == rk.INVALID_ARG and "distinct" in rk.last_error()
    assert call(wsb=1024) == rk.WORKSPACE_TOO_SMALL


def test_decompose_is_host_arithmetic_and_matches_oracle(L, oracle):
    """rocketkv_decompose launches nothing, so it is checked here against the oracle's own
    evaluation of Section 3.6 over a grid of sequence lengths and budgets."""
    g = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "decompose_c64.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            g[k] = float(v)
    got = rk.decompose(64 * 512, 512, 128)
    assert got["c"] == g["c"] and round(got["r"], 2) == g["r"]
    assert round(got["stage1"], 1) == g["stage1"] and round(got["stage2"], 1) == g["stage2"]
    assert got["page_size"] == g["page"] and round(got["head_ratio"], 1) == g["head_ratio"]
    for S in (1, 100, 4096, 32768, 131072, 1 << 20):
        for t in (1, 256, 512, 1024, 4096, 16384):
            for D in (64, 128):
                got = rk.decompose(S, t, D)
                ref = oracle.decompose(max(1.0, S / t))
                want = oracle.decompose_budget(S, t, D)
                for k_lib, k_or in (("r", "r"), ("stage1", "stage1"), ("stage2", "stage2"),
                                    ("head_ratio", "head_ratio")):
                    assert abs(got[k_lib] - ref[k_or]) <= 1e-12 * max(1.0, abs(ref[k_or]))
                assert (got["page_size"], got["keep_budget"], got["channel_budget"], got["attend_tokens"]) == \
                    (want["page"], want["keep"], want["channels"], want["attend_tokens"]), (S, t, D)
                cm = oracle.cost_model(max(1.0, S / t))
                for k in ("storage", "storage_mt", "traffic"):
                    assert abs(got[k] - cm[k]) <= 1e-12 * max(1.0, cm[k])
    out = rk.SplitStruct()
    assert L.rocketkv_decompose(0, 512, 128, C.byref(out)) == rk.INVALID_ARG
    assert L.rocketkv_decompose(4096, 0, 128, C.byref(out)) == rk.INVALID_ARG
    assert L.rocketkv_decompose(4096, 512, 128, None) == rk.INVALID_ARG


def test_layout_field_is_validated(L):
    st = fake_cache(v_layout=7)
    assert L.rocketkv_workspace_bytes(rk.OP_DENSE_DECODE, C.byref(st), 0, 0) == 0
    assert "v_layout" in rk.last_error()
    # token-major caches may have any page size up to 64; channel-major attention needs 16
    tm = fake_cache(page_size=3, stride_page=8 * 3 * 128, stride_head=3 * 128, v_layout=rk.V_TOKEN_MAJOR)
    assert L.rocketkv_workspace_bytes(rk.OP_HSA_DECODE, C.byref(tm), 256, 0) > 0


def test_multi_turn_argument_checks(L):
    tm = fake_cache(v_layout=rk.V_TOKEN_MAJOR)
    ix = rk.IndexStruct(0x3000, 0x4000, 4, 256)
    assert L.rocketkv_mt_workspace_bytes(C.byref(tm), C.byref(ix), 512) > 0
    assert L.rocketkv_mt_workspace_bytes(C.byref(tm), C.byref(ix), 0) == 0
    bad = rk.IndexStruct(0x3000, 0x4000, 4, 250)  # pages_cap not a multiple of 8
    assert L.rocketkv_mt_workspace_bytes(C.byref(tm), C.byref(bad), 512) == 0
    # the cache behind an index must be token-major; rejected before anything is launched
    cm = fake_cache()
    r = L.rocketkv_mt_build_page_summaries(C.byref(cm), C.byref(ix), 0x5000, 0x6000, 0, -1, None)
    assert r == rk.UNSUPPORTED and "token-major" in rk.last_error()
    r = L.rocketkv_mt_append_kv(C.byref(tm), None, 0x5000, 0x6000, 0x7000, 0x8000, None)
    assert r == rk.INVALID_ARG
    r = L.rocketkv_mt_hsa_decode(C.byref(tm), C.byref(ix), 0x5000, 0x6000, 0x7000, 32, 512, 0, None, None, None,
                                 None, 0x10000, 1 << 30, None)
    assert r == rk.INVALID_ARG and "out" in rk.last_error()
    small_ix = rk.IndexStruct(0x3000, 0x4000, 4, 8)  # 32 entries per row < keep budget
    r = L.rocketkv_snapkv_filter(0x5000, C.byref(tm), 32, 63, 1024, C.byref(small_ix), 0x10000, 1 << 30, None)
    assert r == rk.INVALID_ARG and "keep_budget" in rk.last_error()


def test_product_and_oracle_do_not_know_each_other():
    """The HIP path and the oracle share no code: nothing under the package imports, includes or opens
    anything of ``oracle/``, and the oracle includes none of the package's headers and imports none of its
    modules (the seeded input generators are handed to it as data by the tests)."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2502_14051_amd")
    for base, _, files in os.walk(pkg):
        if "_build" in base or "__pycache__" in base:
            continue
        for f in files:
            if not f.endswith((".py", ".hip", ".h", ".c", ".cpp")):
                continue
            text = open(os.path.join(base, f), encoding="utf-8").read()
            assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), f
            assert "rocketkv_oracle" not in text and "oracle/" not in text, f
    for f in os.listdir(os.path.join(root, "oracle")):
        if not f.endswith((".py", ".c", ".h")):
            continue
        text = open(os.path.join(root, "oracle", f), encoding="utf-8").read()
        assert "paper_2502_14051_amd" not in text and "csrc" not in text, f
        assert '#include "' not in text or "rocketkv.h" not in text, f
    entry = open(os.path.join(root, "include", "rocketkv.h"), encoding="utf-8").read()
    assert "oracle" not in entry.lower()


def test_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    """Without the built library every entry point of the binding raises: there is no CPU path behind it."""
    from paper_2502_14051_amd import rocketkv as rk

    monkeypatch.setattr(rk, "_lib", None)
    monkeypatch.setattr(rk, "LIB_PATH", str(tmp_path / "librocketkv.so"))
    with pytest.raises(ImportError, match="no fallback"):
        rk.lib()
    with pytest.raises(ImportError, match="no fallback"):
        rk.decompose(32768, 2048, 128)


def test_no_kernel_spills_registers():
    """The build writes what the compiler reports per kernel.  No kernel of the library may use scratch
    memory: a spill costs HBM traffic on every launch (12 bytes per lane in the fused decode kernel were
    1.5 % of its time and 2 MB per launch) and no numerical test would ever notice."""
    from paper_2502_14051_amd import build as b

    if not os.path.exists(b.RESOURCES):
        pytest.skip("no kernel_resources.txt: build the library first")
    rows = [l.split() for l in open(b.RESOURCES) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 40, "the report lists fewer kernels than the library has"
    names = " ".join(r[1] for r in rows)
    for must in ("hsa_decode_kernel", "hsa_decode_tok_kernel", "attend_mfma_kernel", "snap_score_kernel"):
        assert must in names, must
    spilling = [(r[0], r[1], r[5]) for r in rows if r[5] != "0"]
    assert not spilling, spilling
