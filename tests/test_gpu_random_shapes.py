"""Seeded random small configurations (head counts, widths, layer maps, batch and prompt lengths, cache capacity,
query / key norm, both element types and both kernel families) through the C ABI against the oracle: the whole path,
the absorbed base step where the library serves the shape, and on a handle sized larger than the call."""
import os
import random

import numpy as np
import pytest
import torch

import kvp_synth as S
from oracle import kvp_oracle as O
from parity_util import TOL, device_weights, slice_rel_err

pytestmark = pytest.mark.gpu


def _draw(rng, case):
    mfma = rng.random() < 0.7
    if mfma:      # auxiliary head_dim 128 and widths in multiples of 64: the matrix-core kernels
        hd, dtype = 128, "bf16"
        nkv_a, ga = rng.choice([1, 2, 4]), rng.choice([1, 2, 3, 4])
        nkv_b, gb = rng.choice([1, 2, 4, 8]), rng.choice([1, 2, 3, 4, 6, 8])
        da, db, fa, fb = (64 * rng.randint(2, 6) for _ in range(4))
    else:         # anything else: the shape-generic kernels
        hd, dtype = rng.choice([16, 32, 64]), rng.choice(["fp32", "bf16"])
        nkv_a, ga = rng.choice([1, 2, 3]), rng.choice([1, 2, 4])
        nkv_b, gb = rng.choice([1, 2, 3]), rng.choice([1, 2, 3, 4])
        da, db, fa, fb = (8 * rng.randint(3, 12) for _ in range(4))
    La, Lb = rng.randint(1, 4), rng.randint(1, 6)
    B = rng.choice([1, 2, 3, 4, 5, 8, 17])
    T = rng.choice([1, 2, 31, 64, 65, 100, 129, 257, 300, 511])
    if B * T > 3000:
        T = max(1, 3000 // B)
    lmap = tuple(rng.randrange(La) for _ in range(Lb))
    if rng.random() < 0.7:
        lmap = tuple(sorted(lmap))
    return S.tiny_config(dtype, base=(Lb, db, nkv_b * gb, nkv_b, hd, fb), aux=(La, da, nkv_a * ga, nkv_a, hd, fa),
                         batch=B, seq_len=T, vocab=rng.choice([50, 97, 300, 1000]), seed=1000 + case, layer_map=lmap,
                         qk_norm=rng.random() < 0.3)


# 16 cases by default; KVP_TEST_RANDOM_CASES=N draws the first N of the same seeded sequence for a longer sweep
N_CASES = int(os.environ.get("KVP_TEST_RANDOM_CASES", "16"))


@pytest.mark.parametrize("case", range(N_CASES))
def test_random_configuration(case):
    import paper_2410_08391_amd as K
    rng = random.Random(4000 + case)
    cfg = _draw(rng, case)
    B, T = cfg.batch, cfg.seq_len
    store = S.WeightStore(cfg)
    tok = S.draw_tokens(cfg)
    extra = rng.choice([0, 3, 40])
    m = K.KVP(cfg, device_weights(cfg, store), max_batch=B + rng.choice([0, 1]), max_seq=T + extra,
              T_cap=T + extra + rng.choice([0, 5]))
    tok_d = torch.from_numpy(tok).to("cuda")
    m.run(tok_d)
    torch.cuda.synchronize()
    ref = O.kvp_prefill_predict(cfg, store.f64, tok)
    kc, vc = m.caches(B)
    tol = TOL[cfg.dtype]
    for i in range(cfg.base.n_layers):
        for b in range(B):
            assert slice_rel_err(kc[i, b, :, :T].float().cpu().numpy(), ref["K_hat"][i, b]) <= tol, (cfg, i, b)
            assert slice_rel_err(vc[i, b, :, :T].float().cpu().numpy(), ref["V_hat"][i, b]) <= tol, (cfg, i, b)
    for b in range(B):
        assert slice_rel_err(m.logits[b].cpu().numpy(), ref["logits"][b]) <= tol, (cfg, b)
    if m.T_cap > T:
        assert float(kc[:, :, :, T:].abs().max()) == 0.0 and float(vc[:, :, :, T:].abs().max()) == 0.0
    if cfg.dtype == "fp32":
        np.testing.assert_array_equal(m.argmax[:B].cpu().numpy(), ref["first"])
    try:        # the absorbed base step: the same logits, or a refusal of the shape
        m.run(tok_d, K.STAGE_AUX | K.STAGE_BASE_ABSORBED)
        torch.cuda.synchronize()
        for b in range(B):
            assert slice_rel_err(m.logits[b].cpu().numpy(), ref["logits"][b]) <= tol, (cfg, b)
    except K.KVPError as e:
        assert e.code == -6, e
    m.close()
