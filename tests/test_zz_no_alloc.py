"""kvp_generation_step_static (the entry point for callers that cannot allocate: its scratch is a
static device array inside the library) against kvp_generation_step with a caller's workspace, through
the C ABI.  Same kernels on the same inputs, so the bar is bit equality of logits, first tokens and the
appended cache entries.  Two calls in a row share the static array, the second with a smaller input
(fewer sequences, shorter cache), so stale contents of the first call lie beyond and beside what the
second one uses."""
import numpy as np
import pytest
import torch

import kvp_synth as S

pytestmark = pytest.mark.gpu


def _setup(cfg, n_new):
    import paper_2410_08391_amd as K
    store = S.WeightStore(cfg)
    names = sorted(set(S.hot_path_tensor_names(cfg)) | set(S.reference_tensor_names(cfg, "base")))
    store.prefetch(names)
    dev = {n: store.get(n).to("cuda").contiguous() for n in names}
    tokens = S.draw_tokens(cfg)
    B, T = tokens.shape
    m = K.KVP(cfg, dev, max_batch=B, max_seq=T + n_new, T_cap=T + n_new)
    m.run(torch.from_numpy(tokens).to("cuda"))
    torch.cuda.synchronize()
    return K, m, B, T


def _step_both(K, m, fed, B, pos):
    """One generation step at `pos` through both entry points from the same cache state; returns
    (logits, argmax, appended K, appended V) of each."""
    stream = torch.cuda.current_stream().cuda_stream
    out = []
    for static in (False, True):
        # both write slot `pos`; poison it first so a call that skipped the append cannot pass
        m.k_cache[:, :, :, pos].fill_(float("nan"))
        m.v_cache[:, :, :, pos].fill_(float("nan"))
        m.logits.fill_(float("nan"))
        m.argmax.fill_(-1)
        if static:
            K.kvp_generation_step_static(m.handle, fed, B, pos, m.k_cache, m.v_cache, m.T_cap, m.logits, m.argmax, stream)
        else:
            K.kvp_generation_step(m.handle, fed, B, pos, m.k_cache, m.v_cache, m.T_cap, m.logits, m.argmax, m.workspace, stream)
        torch.cuda.synchronize()
        kc, vc = m.caches(B)
        out.append((m.logits[:B].clone(), m.argmax[:B].clone(), kc[:, :, :, pos].clone(), vc[:, :, :, pos].clone()))
    return out


@pytest.mark.parametrize("dtype,base,aux", [
    ("bf16", (3, 256, 8, 2, 128, 320), (2, 128, 4, 1, 128, 192)),     # matrix-core chain + MFMA decode attention
    ("fp32", (3, 72, 6, 2, 16, 104), (2, 40, 4, 1, 8, 56)),           # shape-generic kernels
])
def test_static_scratch_matches_workspace_two_calls(dtype, base, aux):
    cfg = S.tiny_config(dtype, base=base, aux=aux, batch=5, seq_len=150, vocab=211, seed=97)
    K, m, B, T = _setup(cfg, 3)
    assert K.kvp_static_scratch_bytes() == 8 << 20
    fed = torch.tensor([3, 1, 4, 1, 5], dtype=torch.int32, device="cuda")
    for (b, pos) in ((B, T), (2, T + 1)):                  # second call: fewer sequences (their own cache layout), one more entry
        # a batch of b sequences has its own cache layout [L][b][...]: refill it through the library
        if b != B:
            tok = torch.from_numpy(S.draw_tokens(cfg, batch=b)).to("cuda")
            m.run(tok)
            K.kvp_generation_step(m.handle, fed[:b].contiguous(), b, T, m.k_cache, m.v_cache, m.T_cap, m.logits, m.argmax,
                                  m.workspace, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
        (l0, a0, k0, v0), (l1, a1, k1, v1) = _step_both(K, m, fed[:b].contiguous(), b, pos)
        assert torch.isfinite(l0).all() and (a0 >= 0).all()
        assert torch.equal(l0, l1), f"logits differ at B={b}, pos={pos}: max |d| {(l0 - l1).abs().max().item()}"
        assert torch.equal(a0, a1)
        assert torch.equal(k0.view(torch.uint8), k1.view(torch.uint8)) and torch.equal(v0.view(torch.uint8), v1.view(torch.uint8))
        assert torch.isfinite(k1.float()).all() and torch.isfinite(v1.float()).all()
    m.close()


def test_static_scratch_config1_shape():
    """The 1.1B-class shapes at their benchmark batch and prompt length (two steps, then a shorter one)."""
    cfg = S.CONFIGS[1]
    K, m, B, T = _setup(cfg, 2)
    fed = torch.tensor([17], dtype=torch.int32, device="cuda")
    for pos in (T, T + 1):
        (l0, a0, k0, v0), (l1, a1, k1, v1) = _step_both(K, m, fed, B, pos)
        assert torch.isfinite(l0).all()
        assert torch.equal(l0, l1) and torch.equal(a0, a1)
        assert torch.equal(k0.view(torch.uint8), k1.view(torch.uint8)) and torch.equal(v0.view(torch.uint8), v1.view(torch.uint8))
    m.close()


def test_static_scratch_rejects_what_does_not_fit():
    """Sizes beyond the static array are an error, not a fault: a vocabulary whose logits alone exceed 8 MiB."""
    cfg = S.tiny_config("fp32", batch=9, seq_len=8, vocab=300000, base=(1, 64, 4, 2, 16, 88), aux=(1, 32, 2, 1, 16, 40))
    K, m, B, T = _setup(cfg, 1)
    fed = torch.zeros(B, dtype=torch.int32, device="cuda")
    assert K.kvp_generation_workspace_bytes(m.handle, B, T + 1) > K.kvp_static_scratch_bytes()
    with pytest.raises(K.KVPError) as e:
        K.kvp_generation_step_static(m.handle, fed, B, T, m.k_cache, m.v_cache, m.T_cap, m.logits, m.argmax, 0)
    assert e.value.code == -4 and "static" in str(e.value)
    # the workspace variant serves it
    K.kvp_generation_step(m.handle, fed, B, T, m.k_cache, m.v_cache, m.T_cap, m.logits, m.argmax, m.workspace, 0)
    torch.cuda.synchronize()
    assert torch.isfinite(m.logits[:B]).all()
    m.close()
