"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2509_18085_amd import spiffy as sp, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    hdr = open(os.path.join(ROOT, "include", "spiffy.h")).read()
    declared = set(re.findall(r"\b(spiffy_[a-z_]+)\s*\(", hdr))
    declared -= {"spiffy_workspace_bytes(...)"}
    assert declared == set(sp.EXPORTS), declared ^ set(sp.EXPORTS)
    for name in declared:
        assert getattr(sp.lib, name) is not None


def test_header_is_plain_c(tmp_path):
    """The boundary is a C header: it compiles as C99 with no C++ or torch types."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "t.c"
    src.write_text('#include "spiffy.h"\nint main(void) { return (int)sizeof(spiffy_model_cfg) == 0; }\n')
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_status_strings():
    assert sp.status_str(0) == "ok"
    for s in (-1, -2, -3, -4, -5):
        assert sp.status_str(s) not in ("ok", "unknown status")


def _cfg(key="c3"):
    return sp.cfg_from_synth(synth.CONFIGS[key])


def test_kernel_choice_by_shape():
    assert sp.uses_mfma(_cfg("c3"), 32) == 1
    assert sp.uses_mfma(_cfg("c4"), 32) == 1
    assert sp.uses_mfma(_cfg("c5"), 4) == 1
    assert sp.uses_mfma(_cfg("c1"), 8) == 0


def test_workspace_bytes():
    c = synth.CONFIGS["c3"]
    n = sp.workspace_bytes(_cfg("c3"), c.G, c.B, c.P)
    M = c.G * c.B
    # at least the SwiGLU activation and the QKV buffer must fit
    assert n > M * c.F * 2 + M * 3 * c.d * 2
    assert n < 2 << 30
    assert sp.workspace_bytes(_cfg("c3"), 0, 32, 10) == 0
    assert sp.workspace_bytes(_cfg("c3"), 4, 32, -1) == 0
    bad = _cfg("c3")
    bad.n_kv_heads = 5
    assert sp.workspace_bytes(bad, 4, 32, 10) == 0
    # more prefix (more splits) never needs less
    assert sp.workspace_bytes(_cfg("c5"), 64, 4, 8192) >= sp.workspace_bytes(_cfg("c5"), 64, 4, 1024)


DUMMY = 0x10000  # non-null, 16-byte aligned, never dereferenced: every check fails before a launch


def _layer_structs():
    w = sp.LayerWeights(*([DUMMY] * 9 + [None] * 3))
    p = sp.PrefixKV(DUMMY, DUMMY, 64)
    return w, p


def test_verify_layer_argument_errors():
    cfg = _cfg("c3")
    w, p = _layer_structs()
    call = lambda **k: sp.lib.spiffy_verify_layer(
        C.byref(k.get("cfg", cfg)), C.byref(k.get("w", w)), C.byref(k.get("p", p)), k.get("hin", DUMMY),
        k.get("G", 4), k.get("B", 32), k.get("pos0", 64), k.get("hout", DUMMY), k.get("ws", 0x100000),
        k.get("wsn", 16), None)
    assert call() == sp.SPIFFY_EWORKSPACE                      # tiny workspace, everything else fine
    assert call(G=0) == sp.SPIFFY_EINVAL
    assert call(B=0) == sp.SPIFFY_EINVAL
    assert call(hin=None) == sp.SPIFFY_EINVAL
    assert call(ws=None) == sp.SPIFFY_EINVAL
    assert call(pos0=-1) == sp.SPIFFY_EINVAL
    assert call(hout=DUMMY + 2) == sp.SPIFFY_EALIGN
    assert call(ws=0x100010) == sp.SPIFFY_EALIGN
    assert call(G=4096, B=32) == sp.SPIFFY_ESHAPE               # more rows than SPIFFY_MAX_ROWS
    w2, _ = _layer_structs()
    w2.w_down = None
    assert call(w=w2) == sp.SPIFFY_EINVAL
    w3, _ = _layer_structs()
    w3.wq = DUMMY + 8
    assert call(w=w3) == sp.SPIFFY_EALIGN
    p2 = sp.PrefixKV(None, None, 64)
    assert call(p=p2) == sp.SPIFFY_EINVAL
    bad = _cfg("c3")
    bad.dtype = 7
    assert call(cfg=bad) == sp.SPIFFY_EINVAL
    bad = _cfg("c3")
    bad.head_dim = 100
    assert call(cfg=bad) == sp.SPIFFY_ESHAPE
    bad = _cfg("c3")
    bad.mask_id = bad.vocab
    assert call(cfg=bad) == sp.SPIFFY_EINVAL


def test_verify_layer_last_argument_errors():
    cfg = _cfg("c3")
    w, p = _layer_structs()
    call = lambda **k: sp.lib.spiffy_verify_layer_last(
        C.byref(cfg), C.byref(w), C.byref(p), k.get("hin", DUMMY), k.get("tok", DUMMY), None, k.get("G", 4), 32, 64,
        k.get("hout", DUMMY), k.get("ws", 0x100000), k.get("wsn", 16), None)
    assert call() == sp.SPIFFY_EWORKSPACE
    assert call(tok=None) == sp.SPIFFY_EINVAL
    assert call(hin=None) == sp.SPIFFY_EINVAL
    assert call(G=0) == sp.SPIFFY_EINVAL
    assert call(hout=DUMMY + 2) == sp.SPIFFY_EALIGN
    assert call(ws=0x100010) == sp.SPIFFY_EALIGN


def test_decode_head_argument_errors():
    cfg = _cfg("c3")
    call = lambda **k: sp.lib.spiffy_decode_head(
        C.byref(cfg), k.get("hid", DUMMY), DUMMY, DUMMY, k.get("tok", DUMMY), None, k.get("G", 4), 32,
        k.get("tau", 0.9), k.get("scale", 1.0), 1, k.get("amax", DUMMY), DUMMY, DUMMY, None, None,
        k.get("ws", 0x100000), k.get("wsn", 16), None)
    assert call() == sp.SPIFFY_EWORKSPACE
    assert call(tau=1.5) == sp.SPIFFY_EINVAL
    assert call(tau=-0.1) == sp.SPIFFY_EINVAL
    assert call(tau=float("nan")) == sp.SPIFFY_EINVAL
    assert call(scale=0.0) == sp.SPIFFY_EINVAL
    assert call(tok=None) == sp.SPIFFY_EINVAL
    assert call(amax=None) == sp.SPIFFY_EINVAL
    assert call(hid=DUMMY + 4) == sp.SPIFFY_EALIGN
    assert call(G=-3) == sp.SPIFFY_EINVAL


def test_matrix_core_head_refuses_what_its_32_bit_offsets_cannot_address():
    """V * d * 2 bytes >= 4 GiB, or more than 2048 chunk summaries per row (V > 262144): a shape error from the
    host checks of spiffy_decode_head and spiffy_head_topk, never a wrapped offset or a failed launch."""
    big = _cfg("c3")
    big.vocab, big.d, big.mask_id = 262144, 8192, 5
    wide = _cfg("c3")
    wide.vocab, wide.d, wide.mask_id = 300000, 1024, 5
    for cfg in (big, wide):
        assert sp.lib.spiffy_decode_head(C.byref(cfg), DUMMY, DUMMY, DUMMY, DUMMY, None, 4, 32, 0.9, 1.0, 1, DUMMY, DUMMY,
                                         DUMMY, None, None, 0x100000, 1 << 40, None) == sp.SPIFFY_ESHAPE
        assert sp.lib.spiffy_head_topk(C.byref(cfg), DUMMY, DUMMY, 4, 32, None, 0, 2, 1.0, 0, DUMMY, DUMMY, 0x100000,
                                       1 << 40, None) == sp.SPIFFY_ESHAPE
    ok = _cfg("c3")
    ok.vocab, ok.d, ok.mask_id = 262144, 4096, 5            # 2 GiB of vocabulary matrix, 2048 chunks: the largest that runs
    assert sp.lib.spiffy_decode_head(C.byref(ok), DUMMY, DUMMY, DUMMY, DUMMY, None, 4, 32, 0.9, 1.0, 1, DUMMY, DUMMY,
                                     DUMMY, None, None, 0x100000, 16, None) == sp.SPIFFY_EWORKSPACE


def test_graph_accept_argument_errors():
    call = lambda **k: sp.lib.spiffy_graph_accept(
        k.get("edges", DUMMY), k.get("E", 3), k.get("ds", DUMMY), k.get("ts", DUMMY), k.get("G", 4), 8,
        k.get("root", 0), k.get("res", DUMMY), None, None)
    assert call(G=65) == sp.SPIFFY_ESHAPE
    assert call(root=4) == sp.SPIFFY_EINVAL
    assert call(root=-1) == sp.SPIFFY_EINVAL
    assert call(E=-1) == sp.SPIFFY_EINVAL
    assert call(edges=None) == sp.SPIFFY_EINVAL
    assert call(ds=None) == sp.SPIFFY_EINVAL
    assert call(res=None) == sp.SPIFFY_EINVAL
    assert call(G=0) == sp.SPIFFY_EINVAL


def test_head_topk_argument_errors():
    cfg = sp.cfg_from_synth(synth.CONFIGS["c2"])
    big = 1 << 40
    def call(**k):
        return sp.lib.spiffy_head_topk(
            C.byref(k.get("cfg", cfg)), k.get("wv", DUMMY), k.get("tok", DUMMY), k.get("G", 4), 32,
            k.get("res", DUMMY), k.get("node", 0), k.get("K", 2), k.get("scale", 1.0), k.get("after", 0),
            k.get("ot", DUMMY), DUMMY, k.get("ws", 0x100000), k.get("wsb", big), None)
    assert call(wv=None) == sp.SPIFFY_EINVAL
    assert call(tok=None) == sp.SPIFFY_EINVAL
    assert call(ot=None) == sp.SPIFFY_EINVAL
    assert call(ws=None) == sp.SPIFFY_EINVAL
    assert call(scale=0.0) == sp.SPIFFY_EINVAL
    assert call(res=None, node=4) == sp.SPIFFY_EINVAL
    assert call(res=None, node=-1) == sp.SPIFFY_EINVAL
    assert call(K=0) == sp.SPIFFY_ESHAPE
    assert call(K=9) == sp.SPIFFY_ESHAPE
    assert call(wv=DUMMY + 2) == sp.SPIFFY_EALIGN
    assert call(ws=0x100010) == sp.SPIFFY_EALIGN
    assert call(wsb=1024) == sp.SPIFFY_EWORKSPACE
    assert call(wsb=1024, after=1) == sp.SPIFFY_EWORKSPACE


def test_draft_prune_argument_errors():
    def call(**k):
        return sp.lib.spiffy_draft_prune(
            k.get("state", DUMMY), k.get("B", 32), 99, k.get("tok", DUMMY), DUMMY, k.get("K", 2),
            k.get("off", DUMMY), k.get("pairs", DUMMY), k.get("D", 5), k.get("nnz", 9), k.get("edges", DUMMY),
            k.get("E", 4), k.get("d_star", 3), k.get("drafts", DUMMY), DUMMY, DUMMY, DUMMY, DUMMY, DUMMY,
            k.get("eout", DUMMY), k.get("counts", DUMMY), None)
    assert call(state=None) == sp.SPIFFY_EINVAL
    assert call(tok=None) == sp.SPIFFY_EINVAL
    assert call(off=None) == sp.SPIFFY_EINVAL
    assert call(pairs=None) == sp.SPIFFY_EINVAL
    assert call(edges=None) == sp.SPIFFY_EINVAL
    assert call(eout=None) == sp.SPIFFY_EINVAL
    assert call(drafts=None) == sp.SPIFFY_EINVAL
    assert call(counts=None) == sp.SPIFFY_EINVAL
    assert call(B=0) == sp.SPIFFY_ESHAPE
    assert call(B=4097) == sp.SPIFFY_ESHAPE
    assert call(K=0) == sp.SPIFFY_ESHAPE
    assert call(K=17) == sp.SPIFFY_ESHAPE
    assert call(D=64) == sp.SPIFFY_ESHAPE
    assert call(D=-1) == sp.SPIFFY_ESHAPE
    assert call(nnz=-1) == sp.SPIFFY_ESHAPE
    assert call(E=-1) == sp.SPIFFY_ESHAPE
    assert call(d_star=-1) == sp.SPIFFY_ESHAPE


def test_verify_step_argument_errors():
    cfg = _cfg("c3")
    w, p = _layer_structs()
    layers = (sp.LayerWeights * 1)(w)
    prefix = (sp.PrefixKV * 1)(p)
    call = lambda **k: sp.lib.spiffy_verify_step(
        C.byref(cfg), 1, layers, prefix, DUMMY, k.get("fn", DUMMY), DUMMY, DUMMY, k.get("G", 4), 32, 64,
        DUMMY, 2, k.get("root", 0), k.get("tau", 0.9), 1.0, 1, None, DUMMY, DUMMY, DUMMY, None, None,
        k.get("res", DUMMY), None, 0x100000, 16, None)
    assert call() == sp.SPIFFY_EWORKSPACE
    assert call(root=9) == sp.SPIFFY_EINVAL
    assert call(tau=2.0) == sp.SPIFFY_EINVAL
    assert call(fn=None) == sp.SPIFFY_EINVAL
    assert call(res=None) == sp.SPIFFY_EINVAL
    assert call(G=100) == sp.SPIFFY_ESHAPE                      # walk supports at most 64 nodes


def test_commit_block_argument_errors():
    cfg = _cfg("c3")
    w, _ = _layer_structs()
    layers = (sp.LayerWeights * 1)(w)
    def call(**k):
        prefix = (sp.PrefixKV * 1)(sp.PrefixKV(k.get("pk", DUMMY), DUMMY, k.get("P", 64), k.get("cap", 128)))
        return sp.lib.spiffy_commit_block(
            C.byref(cfg), k.get("L", 1), layers, prefix, k.get("we", DUMMY), k.get("tok", DUMMY), k.get("B", 32),
            k.get("pos0", 64), k.get("ws", 0x100000), k.get("wsb", 16), None)
    assert call() == sp.SPIFFY_EWORKSPACE                       # every argument check passed
    assert call(cap=95) == sp.SPIFFY_ESHAPE                     # 64 + 32 rows do not fit
    assert call(cap=0) == sp.SPIFFY_ESHAPE                      # capacity 0 means P: no room at all
    assert call(cap=32) == sp.SPIFFY_EINVAL                     # capacity below P
    assert call(pk=None) == sp.SPIFFY_EINVAL                    # a cache to append to is required
    assert call(L=0) == sp.SPIFFY_EINVAL
    assert call(we=None) == sp.SPIFFY_EINVAL
    assert call(tok=None) == sp.SPIFFY_EINVAL
    assert call(ws=None) == sp.SPIFFY_EINVAL
    assert call(pos0=-1) == sp.SPIFFY_EINVAL
    assert call(B=0) == sp.SPIFFY_EINVAL
    assert call(B=5000) == sp.SPIFFY_ESHAPE
    assert call(ws=0x100010) == sp.SPIFFY_EALIGN


def test_subgraph_search_argument_errors():
    assert sp.lib.spiffy_subgraph_search_workspace_bytes() > 0
    def call(**k):
        return sp.lib.spiffy_subgraph_search(
            k.get("count", DUMMY), k.get("level", DUMMY), k.get("N", 30), k.get("edges", DUMMY), k.get("E", 5),
            k.get("D", 5), k.get("mask", DUMMY), k.get("sum", DUMMY), k.get("n", DUMMY), None, k.get("ws", 0x100000),
            k.get("wsb", 16), None)
    assert call() == sp.SPIFFY_EWORKSPACE                       # every argument check passed
    assert call(count=None) == sp.SPIFFY_EINVAL
    assert call(level=None) == sp.SPIFFY_EINVAL
    assert call(edges=None) == sp.SPIFFY_EINVAL
    assert call(edges=None, E=0) == sp.SPIFFY_EWORKSPACE
    assert call(mask=None) == sp.SPIFFY_EINVAL
    assert call(sum=None) == sp.SPIFFY_EINVAL
    assert call(n=None) == sp.SPIFFY_EINVAL
    assert call(ws=None) == sp.SPIFFY_EINVAL
    assert call(N=0) == sp.SPIFFY_ESHAPE
    assert call(N=65) == sp.SPIFFY_ESHAPE
    assert call(D=0) == sp.SPIFFY_ESHAPE
    assert call(D=65) == sp.SPIFFY_ESHAPE
    assert call(E=-1) == sp.SPIFFY_ESHAPE
    assert call(N=64, D=32) == sp.SPIFFY_ESHAPE                 # 1.8e18 sets: refused
    assert call(N=64, D=12) == sp.SPIFFY_ESHAPE                 # 3.3e12 > 2^40
    assert call(N=64, D=11) == sp.SPIFFY_EWORKSPACE             # 7.4e11 sets: accepted
    assert call(N=64, D=64) == sp.SPIFFY_EWORKSPACE
    assert call(N=3, D=9) == sp.SPIFFY_EWORKSPACE               # more than there are nodes: an empty answer, not an error
    assert call(ws=0x100010) == sp.SPIFFY_EALIGN


def test_verify_step_seq_argument_errors():
    cfg = _cfg("c3")
    w, _ = _layer_structs()
    layers = (sp.LayerWeights * 1)(w)
    def call(**k):
        prefix = (sp.PrefixKV * 1)(sp.PrefixKV(k.get("pk", DUMMY), DUMMY, 64, k.get("cap", 1024), k.get("pS", 0)))
        return sp.lib.spiffy_verify_step_seq(
            C.byref(cfg), k.get("L", 1), layers, prefix, DUMMY, DUMMY, DUMMY, DUMMY, k.get("suf", DUMMY), k.get("G", 4), 32,
            k.get("S", 224), 64, DUMMY, 2, 0, 0.9, 1.0, 1, None, DUMMY, DUMMY, DUMMY, None, None, DUMMY, None,
            0x100000, k.get("wsb", 16), None)
    assert call() == sp.SPIFFY_EWORKSPACE                       # every argument check passed
    assert call(S=0, suf=None) == sp.SPIFFY_EWORKSPACE          # no suffix: the plain step
    assert call(suf=None) == sp.SPIFFY_EINVAL
    assert call(S=-1) == sp.SPIFFY_EINVAL
    assert call(S=5000) == sp.SPIFFY_ESHAPE
    assert call(cap=64 + 32 + 223) == sp.SPIFFY_ESHAPE          # no room behind the prefix for block and suffix
    assert call(pS=8) == sp.SPIFFY_EINVAL                       # a cached suffix and a computed one exclude each other
    assert call(pk=None) == sp.SPIFFY_EINVAL
    assert call(L=0) == sp.SPIFFY_EINVAL
    assert sp.lib.spiffy_workspace_bytes_seq(C.byref(cfg), 4, 32, 224, 64) > sp.lib.spiffy_workspace_bytes(C.byref(cfg), 4, 32, 64)
    assert sp.lib.spiffy_workspace_bytes_seq(C.byref(cfg), 4, 32, 0, 64) == sp.lib.spiffy_workspace_bytes(C.byref(cfg), 4, 32, 64)
    assert sp.lib.spiffy_workspace_bytes_seq(C.byref(cfg), 4, 32, 5000, 64) == 0


def test_verify_step_commit_argument_errors():
    cfg = _cfg("c3")
    w, _ = _layer_structs()
    layers = (sp.LayerWeights * 1)(w)
    def call(**k):
        prefix = (sp.PrefixKV * 1)(sp.PrefixKV(k.get("pk", DUMMY), DUMMY, 64, k.get("cap", 1024), k.get("pS", 0)))
        return sp.lib.spiffy_verify_step_commit(
            C.byref(cfg), k.get("L", 1), layers, prefix, DUMMY, DUMMY, DUMMY, k.get("prev", DUMMY), DUMMY, k.get("G", 4), 32,
            k.get("pos0", 96), DUMMY, 2, 0, 0.9, 1.0, 1, None, DUMMY, DUMMY, DUMMY, None, None, DUMMY, None,
            0x100000, k.get("wsb", 16), None)
    assert call() == sp.SPIFFY_EWORKSPACE                       # every argument check passed
    assert call(pS=64) == sp.SPIFFY_EWORKSPACE                  # with a cached suffix behind the finished block
    assert call(prev=None) == sp.SPIFFY_EINVAL
    assert call(pos0=31) == sp.SPIFFY_EINVAL                    # no room for the finished block in front of pos0
    assert call(cap=64 + 31) == sp.SPIFFY_ESHAPE                # no room for the finished block's rows
    assert call(pS=64, cap=64 + 32 + 63) == sp.SPIFFY_ESHAPE
    assert call(pk=None) == sp.SPIFFY_EINVAL
    assert call(L=0) == sp.SPIFFY_EINVAL
    assert call(G=0) == sp.SPIFFY_EINVAL
    assert call(G=512) == sp.SPIFFY_ESHAPE                      # (G + 1) * B rows exceed the row limit
    assert sp.lib.spiffy_workspace_bytes_commit(C.byref(cfg), 4, 32, 64) > sp.lib.spiffy_workspace_bytes(C.byref(cfg), 4, 32, 96)
    assert sp.lib.spiffy_workspace_bytes_commit(C.byref(cfg), 512, 32, 64) == 0


def test_probe_library_is_separate_and_checks_its_arguments():
    """The machine probes live in libspiffy_probe.so: the verification library does not export them."""
    from paper_2509_18085_amd import probe
    with pytest.raises(AttributeError):
        sp.lib.spiffy_probe_mfma
    flop = C.c_double(0)
    assert probe.lib.spiffy_probe_mfma(0, 0, DUMMY, C.byref(flop), None) == sp.SPIFFY_EINVAL
    assert probe.lib.spiffy_probe_mfma(1 << 25, 0, DUMMY, C.byref(flop), None) == sp.SPIFFY_EINVAL
    assert probe.lib.spiffy_probe_mfma(10, 0, None, C.byref(flop), None) == sp.SPIFFY_EINVAL
    assert probe.lib.spiffy_probe_mfma(10, 0, DUMMY, None, None) == sp.SPIFFY_EINVAL
    assert probe.lib.spiffy_probe_hbm_read(None, 1024, DUMMY, None) == sp.SPIFFY_EINVAL
    assert probe.lib.spiffy_probe_hbm_read(DUMMY, 8, DUMMY, None) == sp.SPIFFY_EINVAL
    assert probe.lib.spiffy_probe_hbm_read(DUMMY + 8, 1024, DUMMY, None) == sp.SPIFFY_EALIGN
    hdr = open(os.path.join(ROOT, "include", "spiffy_probe.h")).read()
    assert set(re.findall(r"\b(spiffy_probe_[a-z_]+)\s*\(", hdr)) == {"spiffy_probe_mfma", "spiffy_probe_hbm_read"}



def test_binding_fails_loudly_without_library(tmp_path, monkeypatch):
    import importlib
    monkeypatch.setattr(sp, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        sp._load()


def test_synth_graphs_follow_the_recipes():
    import numpy as np
    for key in ("c1", "c3", "c4", "c5"):
        cfg = synth.CONFIGS[key]
        st, e = synth.draft_graph(key, cfg)
        assert st.shape == (cfg.G, cfg.B), key
        assert len(e) > 0 and e.min() >= 0 and e.max() < cfg.G
        for p, c in e:            # child's unmasked set strictly contains the parent's (Eq. 6)
            up = set(np.nonzero(st[p] != cfg.mask_id)[0])
            uc = set(np.nonzero(st[c] != cfg.mask_id)[0])
            assert up < uc
    st, e = synth.draft_graph("c5", synth.CONFIGS["c5"])
    assert len({tuple(r) for r in st}) == 16          # 16 subsets, 4 copies each
    tgt, path = synth.planted_targets(*synth.draft_graph("c3", synth.CONFIGS["c3"]), synth.CONFIGS["c3"].V, 3, 5)
    assert len(path) >= 2


# ------------------------------------------------------------------ launch plans (host arithmetic of the GEMM dispatcher)

TILE_ROWS = {256, 128, 64, 32}


def _check_plan(epi, M, N, K, plan):
    unit = 2 if epi == sp.GEMM_SWIGLU else 1
    col = 0
    for l in plan["launches"]:
        bm, bn = l["tile"]
        assert bm in TILE_ROWS and bn in (192, 128, 96, 64, 32), (M, N, l)
        assert l["col0"] == col and l["n_cols"] > 0 and l["n_cols"] % (bn // unit) == 0, (M, N, l)
        assert l["workgroups"] == -(-M // bm) * (l["n_cols"] // (bn // unit)) * plan["k_slices"], (M, N, l)
        col += l["n_cols"]
    assert col == N, (M, N, plan)       # the launches cover every output column exactly once


def test_gemm_plans_cover_the_columns_once_and_slice_k_by_shape_only():
    """Every plan of the dispatcher covers [0, N) exactly once with tiles that divide their range, for the projection
    shapes of the three models and row counts from 1 to 2048; the K-slice count is the same for every row count."""
    shapes = [(sp.GEMM_STORE, 12288, 4096), (sp.GEMM_STORE, 4608, 3584), (sp.GEMM_RESID, 4096, 4096),
              (sp.GEMM_RESID, 4096, 12288), (sp.GEMM_RESID, 3584, 18944), (sp.GEMM_RESID, 3584, 3584),
              (sp.GEMM_RESID, 192, 512), (sp.GEMM_SWIGLU, 12288, 4096), (sp.GEMM_SWIGLU, 18944, 3584),
              (sp.GEMM_SWIGLU, 320, 640)]
    for epi, N, K in shapes:
        slices = set()
        for M in list(range(1, 300, 7)) + [256, 512, 640, 768, 1000, 1024, 1536, 2048]:
            for ws in (True, False):
                plan = sp.gemm_plan(epi, M, N, K, ws)
                _check_plan(epi, M, N, K, plan)
                if ws:
                    slices.add(plan["k_slices"])
                else:
                    assert plan["k_slices"] == 1
        assert len(slices) == 1, (epi, N, K, slices)


def test_gemm_plans_of_the_benchmark_shapes():
    """The schedules the design notes describe: two rounds of 256 x 192 tiles for the headline gate/up launch, the
    two-part schedule at 18944 features over 768 rows, three K slices for K = 18944, 96-column tiles for QKV over two
    rows of tiles."""
    assert sp.gemm_plan(sp.GEMM_SWIGLU, 1024, 12288, 4096) == {
        "k_slices": 1, "launches": [{"tile": (256, 192), "col0": 0, "n_cols": 12288, "workgroups": 512}]}
    assert sp.gemm_plan(sp.GEMM_SWIGLU, 768, 18944, 3584)["launches"] == [
        {"tile": (256, 192), "col0": 0, "n_cols": 16320, "workgroups": 510},
        {"tile": (128, 128), "col0": 16320, "n_cols": 2624, "workgroups": 246}]
    assert sp.gemm_plan(sp.GEMM_SWIGLU, 128, 18944, 3584)["launches"] == [        # four states of the same model
        {"tile": (128, 128), "col0": 0, "n_cols": 16384, "workgroups": 256},
        {"tile": (64, 64), "col0": 16384, "n_cols": 2560, "workgroups": 160}]
    assert sp.gemm_plan(sp.GEMM_RESID, 768, 3584, 18944) == {
        "k_slices": 3, "launches": [{"tile": (256, 128), "col0": 0, "n_cols": 3584, "workgroups": 252}]}
    assert sp.gemm_plan(sp.GEMM_RESID, 1024, 4096, 12288)["k_slices"] == 2
    assert sp.gemm_plan(sp.GEMM_STORE, 256, 12288, 4096)["launches"][0]["tile"] == (128, 96)
    assert sp.gemm_plan(sp.GEMM_STORE, 128, 12288, 4096)["launches"][0]["tile"] == (64, 96)
    assert sp.gemm_plan(sp.GEMM_STORE, 1024, 12288, 4096)["launches"][0] == {
        "tile": (256, 192), "col0": 0, "n_cols": 12288, "workgroups": 256}


def test_gemm_plan_errors():
    p = sp.GemmPlan()
    assert sp.lib.spiffy_gemm_plan(sp.GEMM_STORE, 64, 100, 256, 1, C.byref(p)) == sp.SPIFFY_ESHAPE     # N % 64
    assert sp.lib.spiffy_gemm_plan(sp.GEMM_STORE, 64, 128, 100, 1, C.byref(p)) == sp.SPIFFY_ESHAPE     # K % 64
    assert sp.lib.spiffy_gemm_plan(sp.GEMM_STORE, 0, 128, 128, 1, C.byref(p)) == sp.SPIFFY_ESHAPE
    assert sp.lib.spiffy_gemm_plan(7, 64, 128, 128, 1, C.byref(p)) == sp.SPIFFY_EINVAL
    assert sp.lib.spiffy_gemm_plan(sp.GEMM_STORE, 64, 128, 128, 1, None) == sp.SPIFFY_EINVAL


def test_layer_width_limit_is_a_host_check():
    """A bf16 model wider than 16384 would need more than 64 KB of on-chip memory per row in the reduction behind the
    split-K projections: refused on the host, nothing is launched."""
    cfg = sp.ModelCfg()
    cfg.d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn, cfg.vocab = 16512, 129, 129, 128, 4096, 1000
    cfg.dtype, cfg.rms_eps, cfg.rope_base, cfg.mask_id = sp.SPIFFY_BF16, 1e-5, 10000.0, 999
    w = sp.LayerWeights()
    for f in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm1", "norm2"):
        setattr(w, f, DUMMY)
    pf = sp.PrefixKV()
    assert sp.lib.spiffy_verify_layer(C.byref(cfg), C.byref(w), C.byref(pf), DUMMY, 2, 32, 0, DUMMY, DUMMY, 1 << 40, None) \
        == sp.SPIFFY_ESHAPE
    cfg.d, cfg.n_q_heads, cfg.n_kv_heads = 16384, 128, 128
    rc = sp.lib.spiffy_verify_layer(C.byref(cfg), C.byref(w), C.byref(pf), DUMMY, 2, 32, 0, DUMMY, DUMMY, 16, None)
    assert rc == sp.SPIFFY_EWORKSPACE      # the shape itself is accepted; the call stops at the next host check
