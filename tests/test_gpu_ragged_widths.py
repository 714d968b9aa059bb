"""Stacks whose layers differ in head counts and feed-forward width (OpenELM's layer-wise scaling,
the models of the paper's experiments), against the oracle evaluated on the per-layer shapes:
(a) natively, every layer launched at its own width (per-layer arrays in kvp_model_shape; the
caches are blocks of the widest layer's size with each layer's dense array at the start);
(b) as a uniform model widened with zero rows / columns (kvp_synth.pad_to_uniform), which computes
the same function exactly."""
import numpy as np
import pytest
import torch

import kvp_synth as S
from oracle import kvp_oracle as O
from parity_util import TOL, run_gpu, slice_rel_err

pytestmark = pytest.mark.gpu


def _check(cfg, B, T):
    import paper_2410_08391_amd as K
    store = S.WeightStore(cfg)
    tok = S.draw_tokens(cfg)
    ucfg, padded = S.pad_to_uniform(cfg, store.get)
    dev = {n: padded(n).to("cuda").contiguous() for n in S.hot_path_tensor_names(ucfg)}
    model = K.KVP(ucfg, dev, max_batch=B, max_seq=T, T_cap=T)
    got = run_gpu(ucfg, None, tok, model=model)
    ref = O.kvp_prefill_predict(cfg, store.f64, tok)
    tol = TOL[cfg.dtype]
    assert isinstance(ref["K_hat"], list)
    for name in ("K_hat", "V_hat"):
        for i in range(cfg.base.n_layers):
            n_kv = cfg.base.widths(i)[1]
            for b in range(B):
                e = slice_rel_err(got[name][i, b, :n_kv], ref[name][i][b])
                assert e <= tol, f"{name} layer {i} sequence {b}: {e:.3e} > {tol}"
            assert np.all(got[name][i, :, n_kv:] == 0), f"{name} layer {i}: appended heads must be exactly zero"
    for b in range(B):
        e = slice_rel_err(got["logits"][b], ref["logits"][b])
        assert e <= tol, f"logits sequence {b}: {e:.3e} > {tol}"
    return got, ref


def test_ragged_widths_generic_kernels_fp32():
    cfg = S.tiny_config("fp32", base=(3, 48, 12, 3, 16, 88), aux=(2, 40, 4, 2, 16, 56), batch=2, seq_len=29, vocab=67, seed=131,
                        base_widths=[(8, 2, 72), (4, 1, 40), (12, 3, 88)], aux_widths=[(4, 2, 56), (2, 1, 24)])
    got, ref = _check(cfg, 2, 29)
    np.testing.assert_array_equal(got["first"], ref["first"])


@pytest.mark.parametrize("B,T,qk_norm", [(1, 150, False), (3, 97, True)])
def test_ragged_widths_mfma_kernels(B, T, qk_norm):
    cfg = S.tiny_config("bf16", base=(3, 256, 8, 2, 128, 448), aux=(3, 128, 4, 2, 128, 192), batch=B, seq_len=T, vocab=211,
                        seed=137 + T, qk_norm=qk_norm,
                        base_widths=[(4, 1, 320), (8, 2, 448), (4, 1, 192)], aux_widths=[(2, 1, 128), (4, 2, 192), (2, 1, 64)])
    _check(cfg, B, T)


def _check_native(cfg, B, T, n_new=0):
    """Every layer at its own width: whole path, then (n_new > 0) teacher-forced generation steps."""
    import paper_2410_08391_amd as K
    store = S.WeightStore(cfg)
    tok = S.draw_tokens(cfg)
    names = sorted(set(S.hot_path_tensor_names(cfg)) | set(S.reference_tensor_names(cfg, "base")))
    store.prefetch(names)
    dev = {n: store.get(n).to("cuda").contiguous() for n in names}
    m = K.KVP(cfg, dev, max_batch=B, max_seq=T + n_new, T_cap=T + n_new)
    m.run(torch.from_numpy(tok).to("cuda"))
    torch.cuda.synchronize()
    ref = [O.kvp_generate(cfg, store.f64, tok[b], max(1, n_new)) for b in range(B)]
    tol = TOL[cfg.dtype]

    def check_logits(step):
        lg = m.logits[:B].cpu().numpy()
        for b in range(B):
            e = slice_rel_err(lg[b], ref[b]["logits"][step])
            assert e <= tol, f"step {step} sequence {b}: logits {e:.3e} > {tol}"

    check_logits(0)
    # auxiliary cache, layer by layer (before the generation steps: they reuse the start of the workspace)
    for l in range(cfg.aux.n_layers):
        ka, va = m.aux_cache_layer(l, B, T)
        for b in range(B):
            KA, VA = O.aux_prefill(cfg, store.f64, tok[b])
            e = slice_rel_err(ka[b * T:(b + 1) * T].float().cpu().numpy(), O.merge_heads(KA[l]))
            assert e <= tol, f"K_A layer {l} sequence {b}: {e:.3e} > {tol}"
            e = slice_rel_err(va[b * T:(b + 1) * T].float().cpu().numpy(), O.merge_heads(VA[l]))
            assert e <= tol, f"V_A layer {l} sequence {b}: {e:.3e} > {tol}"
    for s in range(1, max(1, n_new)):
        fed = torch.tensor([int(ref[b]["tokens"][s - 1]) for b in range(B)], dtype=torch.int32, device="cuda")
        m.generation_step(fed, T + s - 1)
        torch.cuda.synchronize()
        check_logits(s)
    n_valid = T + max(1, n_new) - 1
    for i in range(cfg.base.n_layers):
        kc, vc = m.cache_layer(i, B)
        assert kc.shape[1] == cfg.base.widths(i)[1]
        for name, got in (("K", kc), ("V", vc)):
            g = got[:, :, :n_valid].float().cpu().numpy()
            for b in range(B):
                e = slice_rel_err(g[b], ref[b][name][i][:, :n_valid])
                assert e <= tol, f"{name} layer {i} sequence {b}: {e:.3e} > {tol}"
    return m, ref


def test_native_ragged_widths_generic_kernels_fp32():
    cfg = S.tiny_config("fp32", base=(3, 48, 12, 3, 16, 88), aux=(2, 40, 4, 2, 16, 56), batch=2, seq_len=29, vocab=67, seed=139,
                        base_widths=[(8, 2, 72), (4, 1, 40), (12, 3, 88)], aux_widths=[(4, 2, 56), (2, 1, 24)])
    _check_native(cfg, 2, 29, n_new=3)


@pytest.mark.parametrize("B,T,qk_norm", [(1, 150, False), (2, 64, True), (4, 97, False)])
def test_native_ragged_widths_mfma_kernels(B, T, qk_norm):
    """head_dim 128: MFMA prefill and predictor (one launch per run of equal widths), row kernels
    and matrix-core chain in the base step; base layers 1 and 2 share an auxiliary layer but
    differ in width, layers 2 and 3 share both."""
    cfg = S.tiny_config("bf16", base=(4, 256, 8, 2, 128, 448), aux=(3, 128, 4, 2, 128, 192), batch=B, seq_len=T, vocab=211,
                        seed=149 + T, qk_norm=qk_norm, layer_map=(0, 1, 1, 1),
                        base_widths=[(4, 1, 320), (8, 2, 448), (4, 1, 192), (4, 1, 256)],
                        aux_widths=[(2, 1, 128), (4, 2, 192), (2, 1, 64)])
    _check_native(cfg, B, T, n_new=3)


def test_native_ragged_widths_reference_prefill():
    import paper_2410_08391_amd as K
    cfg = S.tiny_config("bf16", base=(3, 256, 8, 2, 128, 448), aux=(2, 128, 4, 2, 128, 192), batch=2, seq_len=70, vocab=211,
                        seed=151, base_widths=[(4, 1, 320), (8, 2, 448), (4, 1, 192)], aux_widths=[(2, 1, 128), (4, 2, 192)])
    store = S.WeightStore(cfg)
    tok = S.draw_tokens(cfg)
    names = sorted(set(S.hot_path_tensor_names(cfg)) | set(S.reference_tensor_names(cfg, "base")))
    dev = {n: store.get(n).to("cuda").contiguous() for n in names}
    m = K.KVP(cfg, dev, max_batch=2, max_seq=70, T_cap=70)
    m.reference(torch.from_numpy(tok).to("cuda"), K.MODEL_BASE, keep_cache=False)
    torch.cuda.synchronize()
    ref = O.reference_prefill(cfg, store.f64, "base", tok)
    lg = m.logits[:2].cpu().numpy()
    for b in range(2):
        assert slice_rel_err(lg[b], ref["logits"][b]) <= TOL["bf16"]


def test_widths_that_are_not_the_maxima_are_refused():
    import paper_2410_08391_amd as K
    cfg = S.tiny_config("fp32", base=(3, 48, 12, 3, 16, 88), aux=(2, 40, 4, 2, 16, 56), batch=1, seq_len=8, vocab=67, seed=157,
                        base_widths=[(8, 2, 72), (4, 1, 40), (12, 3, 88)])
    store = S.WeightStore(cfg)
    dev = {n: store.get(n).to("cuda").contiguous() for n in S.hot_path_tensor_names(cfg)}
    import dataclasses
    bad = cfg.with_(base=dataclasses.replace(cfg.base, n_kv_heads=4))
    with pytest.raises(K.KVPError):
        K.KVP(bad, dev)
