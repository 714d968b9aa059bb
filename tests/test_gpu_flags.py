"""kvp_check_flags: a token id outside the vocabulary is clamped by the embedding kernels and the
clamp is reported through the handle's device-side flag word (the algorithm takes the token
sequence I as given, Sec. 4.1; a bad id is the caller's error and must not read out of bounds)."""
import numpy as np
import pytest
import torch

import kvp_synth as S
from oracle import kvp_oracle as O
from parity_util import compare, device_weights

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_clamped_token_sets_the_flag_and_equals_the_clamped_prompt(dtype):
    import paper_2410_08391_amd as K
    base, aux = ((3, 256, 8, 2, 128, 320), (2, 128, 4, 1, 128, 192)) if dtype == "bf16" else ((3, 64, 4, 2, 16, 88), (2, 32, 2, 1, 16, 40))
    cfg = S.tiny_config(dtype, base=base, aux=aux, batch=3, seq_len=40, vocab=97, seed=5)
    store = S.WeightStore(cfg)
    m = K.KVP(cfg, device_weights(cfg, store))
    tok = S.draw_tokens(cfg)
    m.run(torch.from_numpy(tok).to("cuda"))
    torch.cuda.synchronize()
    assert m.check_flags() == 0                               # in-range prompts leave the word clear
    bad = tok.copy()
    bad[1, 7] = cfg.vocab + 5                                 # mid-prompt: the auxiliary embedding clamps it
    bad[2, -1] = -3                                           # last token: the base embedding clamps it too
    m.run(torch.from_numpy(bad).to("cuda"))
    torch.cuda.synchronize()
    assert m.check_flags() == K.FLAG_TOKEN_CLAMPED
    assert m.check_flags(clear=True) == K.FLAG_TOKEN_CLAMPED  # reading does not clear unless asked
    assert m.check_flags() == 0
    # the result is that of the clamped prompt
    clamped = np.clip(bad, 0, cfg.vocab - 1)
    ref = O.kvp_prefill_predict(cfg, store.f64, clamped)
    B, T = tok.shape
    kc, vc = m.caches(B)
    got = {"K_hat": kc[:, :, :, :T].float().cpu().numpy(), "V_hat": vc[:, :, :, :T].float().cpu().numpy(),
           "logits": m.logits[:B].cpu().numpy()}
    compare(cfg, got, ref)
    m.close()
