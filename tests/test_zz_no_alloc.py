"""The allocation-free entry point (spiffy_decode_head_static) against spiffy_decode_head through the C ABI:
same kernels on the library's own device scratch, so every output is bit-identical; two calls in a row, the
second on a smaller input (what the first call left in the shared scratch must not show)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2509_18085_amd import synth

DEV = "cuda:0"


@pytest.fixture(scope="module")
def sp():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2509_18085_amd import spiffy
    return spiffy


def _blank(sp, G, B):
    return dict(argmax=torch.full((G, B), -7, dtype=torch.int32, device=DEV),
                conf=torch.full((G, B), -7.0, dtype=torch.float32, device=DEV),
                unmask=torch.full((G, B), 9, dtype=torch.uint8, device=DEV),
                margin=torch.full((G, B), -7.0, dtype=torch.float32, device=DEV),
                target_states=torch.full((G, B), -7, dtype=torch.int32, device=DEV))


def _both(sp, cfg, G, seed, scale, tau):
    scfg = sp.cfg_from_synth(cfg)
    st = synth.random_states(G, cfg.B, cfg.V, 0.3, 0.9, seed)
    hidden = synth.hidden_states(cfg, seed, G=G).to(DEV)
    hw = {k: v.to(DEV) for k, v in synth.head_weights(cfg, seed).items()}
    d_st = torch.from_numpy(st).to(DEV)
    ws = sp.alloc_workspace(scfg, G, cfg.B, 0, DEV)
    ref = sp.decode_head(scfg, hidden, hw["final_norm"], hw["w_vocab"], d_st, tau, ws, logit_scale=scale)
    out = _blank(sp, G, cfg.B)                      # allocated before the call under test
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    sp.decode_head_static(scfg, hidden, hw["final_norm"], hw["w_vocab"], d_st, tau, out, logit_scale=scale)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for k in ref:
        assert torch.equal(out[k], ref[k]), (cfg.name, G, k)
    assert int((st == cfg.mask_id).sum()) > 0
    return out


@pytest.mark.gpu
@pytest.mark.parametrize("kind", ["mfma_bf16", "generic_f32"])
def test_static_head_equals_workspace_head_twice(sp, kind):
    if kind == "mfma_bf16":        # matrix-core head: vocabulary with a ragged last tile, four states then one
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=512, V=128 * 37 + 24, B=32, G=4)
    else:
        cfg = synth.CONFIGS["c1"].scaled(B=8, G=4)
    _both(sp, cfg, 4, 11, 30.0, 0.6)
    _both(sp, cfg, 1, 12, 30.0, 0.6)            # smaller input, same scratch
    _both(sp, cfg, 3, 13, 1.0, 0.9)


@pytest.mark.gpu
def test_static_head_limits(sp):
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=512, V=1280, B=32, G=4)
    scfg = sp.cfg_from_synth(cfg)
    out = _blank(sp, 5, 32)
    d = torch.zeros((5, 32, cfg.d), dtype=torch.bfloat16, device=DEV)
    t = torch.zeros((5, 32), dtype=torch.int32, device=DEV)
    hw = {k: v.to(DEV) for k, v in synth.head_weights(cfg).items()}
    with pytest.raises(sp.SpiffyError) as e:     # 160 rows: beyond SPIFFY_STATIC_MAX_ROWS
        sp.decode_head_static(scfg, d, hw["final_norm"], hw["w_vocab"], t, 0.9, out)
    assert e.value.status == sp.SPIFFY_ELIMIT
    torch.cuda.synchronize()
    assert (out["argmax"] == -7).all()           # nothing was launched


def test_static_head_limits_are_host_checks():
    """No GPU needed: sizes beyond the library's scratch are refused before anything touches the device."""
    from paper_2509_18085_amd import spiffy as sp
    DUMMY = 0x10000
    call = lambda cfg, G, B: sp.lib.spiffy_decode_head_static(C.byref(cfg), DUMMY, DUMMY, DUMMY, DUMMY, None, G, B, 0.9,
                                                              1.0, 1, DUMMY, DUMMY, DUMMY, None, None, None)
    c3 = sp.cfg_from_synth(synth.CONFIGS["c3"])
    assert call(c3, 5, 32) == sp.SPIFFY_ELIMIT                      # 160 rows
    assert call(c3, 0, 32) == sp.SPIFFY_EINVAL
    wide = sp.cfg_from_synth(synth.CONFIGS["c1"].scaled(d=16384))   # fp32 rows of 64 KB: 128 of them do not fit
    assert call(wide, 4, 32) == sp.SPIFFY_ELIMIT
    assert sp.status_str(sp.SPIFFY_ELIMIT) not in ("ok", "unknown status")
    assert sp.STATIC_SCRATCH_BYTES == 8 << 20 and sp.STATIC_MAX_ROWS == 128
