"""Ordinary inference of one model alone (the reference points of the paper's timing experiments,
Sec. 6.3 "Timing Experiments") through the C ABI against the oracle's reference_prefill."""
import numpy as np
import pytest
import torch

import kvp_synth as S
from oracle import kvp_oracle as O
from parity_util import TOL, slice_rel_err, argmax_report

pytestmark = pytest.mark.gpu


def _run(cfg, side, tokens, keep_cache=True, env=None):
    import paper_2410_08391_amd as K
    store = S.WeightStore(cfg)
    names = sorted(set(S.hot_path_tensor_names(cfg)) | set(S.reference_tensor_names(cfg, side)))
    store.prefetch(names)
    dev = {n: store.get(n).to("cuda").contiguous() for n in names}
    B, T = tokens.shape
    m = K.KVP(cfg, dev, max_batch=B, max_seq=T, T_cap=T)
    kc, vc = m.reference(torch.from_numpy(tokens).to("cuda"), K.MODEL_BASE if side == "base" else K.MODEL_AUX, keep_cache)
    torch.cuda.synchronize()
    got = {"logits": m.logits[:B].cpu().numpy(), "first": m.argmax[:B].cpu().numpy().astype(np.int64)}
    if keep_cache:
        got["K"], got["V"] = kc.float().cpu().numpy(), vc.float().cpu().numpy()
    ref = O.reference_prefill(cfg, store.f64, side, tokens)
    return got, ref


def _compare(cfg, got, ref, show=False):
    # The 2e-2 (bf16) / 1e-4 (fp32) bound is stated for the predicted cache, which sits behind
    # auxiliary stacks of 8 to 12 layers.  Every layer adds independent roundings of the same size
    # to the residual stream (h, q, k, v, P, attention output, SwiGLU activation), so the error of
    # a deeper stack grows like a random walk: the bound scales with sqrt(layers / 8).  The exponent
    # is measured, not assumed: `show` prints the worst slice error of every layer's keys and values
    # (configuration 1's 28-layer base model: the design notes hold the table and the fitted exponent).
    L, B = ref["K"].shape[:2]
    tol = TOL[cfg.dtype] * max(1.0, float(np.sqrt(L / 8.0)))
    per_layer = []
    for i in range(L):
        worst = 0.0
        for name in ("K", "V"):
            if name in got:
                for b in range(B):
                    e = slice_rel_err(got[name][i, b], ref[name][i, b])
                    assert e <= tol, f"{name} layer {i} sequence {b}: {e:.3e} > {tol}"
                    worst = max(worst, e)
        per_layer.append(worst)
    for b in range(B):
        e = slice_rel_err(got["logits"][b], ref["logits"][b])
        assert e <= tol, f"logits sequence {b}: {e:.3e} > {tol}"
    if show and "K" in got:
        print("\nworst K/V slice error by layer (1-based depth): " + " ".join(f"{i + 1}:{e:.4f}" for i, e in enumerate(per_layer)))
        d = np.arange(2, L + 1, dtype=np.float64)          # layer 1's keys carry no accumulated residual error yet
        slope = np.polyfit(np.log(d), np.log(np.asarray(per_layer[1:])), 1)[0]
        print(f"fitted exponent of error ~ depth^p over layers 2..{L}: p = {slope:.2f} (bound used: {tol:.3e} = {TOL[cfg.dtype]} * sqrt({L}/8))")
    return per_layer


@pytest.mark.parametrize("side", ["base", "aux"])
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_reference_prefill_tiny_odd_shapes(side, dtype):
    """Shape-generic kernels: odd sizes, grouped heads, ragged length."""
    cfg = S.tiny_config(dtype, base=(3, 72, 6, 2, 16, 104), aux=(2, 40, 4, 1, 8, 56), batch=3, seq_len=37, vocab=131, seed=61)
    tok = S.draw_tokens(cfg)
    got, ref = _run(cfg, side, tok)
    _compare(cfg, got, ref)
    if dtype == "fp32":
        np.testing.assert_array_equal(got["first"], ref["first"])


@pytest.mark.parametrize("side,group,T", [("base", 4, 200), ("aux", 4, 130), ("base", 3, 97), ("aux", 8, 64)])
def test_reference_prefill_mfma_path(side, group, T):
    """head_dim 128 stacks run the MFMA GEMMs and the flash attention kernels."""
    big = (3, 256, group, 1, 128, 320)
    small = (2, 128, 4, 2, 128, 192)
    cfg = S.tiny_config("bf16", base=big if side == "base" else small, aux=big if side == "aux" else small,
                        batch=2, seq_len=T, vocab=211, seed=67 + T)
    tok = S.draw_tokens(cfg)
    got, ref = _run(cfg, side, tok)
    _compare(cfg, got, ref)


def test_reference_prefill_without_cache_and_config0():
    cfg = S.CONFIGS[0]
    tok = S.draw_tokens(cfg)
    for side in ("base", "aux"):
        got, ref = _run(cfg, side, tok, keep_cache=False)
        _compare(cfg, got, ref)
        np.testing.assert_array_equal(got["first"], ref["first"])


def test_reference_prefill_config1_base():
    """Full-size configuration 1: the 1.1B-class base model, B = 1, T = 1024."""
    cfg = S.CONFIGS[1]
    tok = S.draw_tokens(cfg)
    got, ref = _run(cfg, "base", tok)
    _compare(cfg, got, ref, show=True)


def test_reference_prefill_identity_relation():
    """aux == base weights, j_i = i, identity predictors: the KV Prediction path and ordinary base
    inference are the same computation; the two device paths (predictor GEMM + decode step vs. one
    causal pass) must agree within the tolerance, cache and logits."""
    import paper_2410_08391_amd as K
    shape = (3, 256, 4, 2, 128, 320)
    cfg = S.tiny_config("bf16", base=shape, aux=shape, batch=2, seq_len=150, vocab=211, layer_map=range(3), seed=71)
    store = S.WeightStore(cfg)
    eye = torch.eye(cfg.base.kv_dim, dtype=torch.bfloat16)
    names = sorted(set(S.hot_path_tensor_names(cfg)) | set(S.reference_tensor_names(cfg, "base")))
    dev = {}
    for n in names:
        if n.startswith("pred."):
            dev[n] = eye.to("cuda").contiguous()
        elif n.startswith("aux."):
            dev[n] = store.get(n.replace("aux.", "base.")).to("cuda").contiguous()
        else:
            dev[n] = store.get(n).to("cuda").contiguous()
    tok = S.draw_tokens(cfg)
    B, T = tok.shape
    m = K.KVP(cfg, dev, max_batch=B, max_seq=T, T_cap=T)
    t = torch.from_numpy(tok).to("cuda")
    m.run(t)
    torch.cuda.synchronize()
    kh, vh = [x[:, :, :, :T].float().cpu().numpy() for x in m.caches(B)]
    lg = m.logits[:B].cpu().numpy().copy()
    kc, vc = m.reference(t, K.MODEL_BASE, True)
    torch.cuda.synchronize()
    lr = m.logits[:B].cpu().numpy()
    for i in range(3):
        for b in range(B):
            assert slice_rel_err(kh[i, b], kc[i, b].float().cpu().numpy().astype(np.float64)) <= 2e-2
            assert slice_rel_err(vh[i, b], vc[i, b].float().cpu().numpy().astype(np.float64)) <= 2e-2
    for b in range(B):
        assert slice_rel_err(lg[b], lr[b].astype(np.float64)) <= 2e-2


def test_reference_prefill_error_paths():
    import paper_2410_08391_amd as K
    cfg = S.tiny_config("fp32", batch=1, seq_len=8)
    store = S.WeightStore(cfg)
    names = S.hot_path_tensor_names(cfg)        # no base wk / wv, no aux head
    dev = {n: store.get(n).to("cuda").contiguous() for n in names}
    m = K.KVP(cfg, dev)
    tok = torch.from_numpy(S.draw_tokens(cfg)).to("cuda")
    with pytest.raises(K.KVPError) as e:
        m.reference(tok, K.MODEL_BASE)
    assert e.value.code == -1 and "wk" in str(e.value)
    with pytest.raises(K.KVPError) as e:
        m.reference(tok, K.MODEL_AUX)
    assert e.value.code == -1 and "lm_head" in str(e.value)
    assert K.kvp_reference_workspace_bytes(m.handle, 7, 1, 8) == 0
