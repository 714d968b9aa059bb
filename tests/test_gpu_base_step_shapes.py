"""The base model's single-token step at widths where its GEMV kernels take their other routes:
whole rows of 5 to 12 pieces in flight and rows in several groups (one or two sequences), and the
coalesced weight route through LDS with 4, 2 or 1 steps per right-hand-side load and one or two row
tiles per block (three to sixteen sequences).  Small auxiliary model, short prompts, two base
layers: the oracle finishes in seconds."""
import numpy as np
import pytest

import kvp_synth as S
from oracle import kvp_oracle as O
from parity_util import compare, run_gpu
from test_gpu_generation import _generate

pytestmark = pytest.mark.gpu

AUX = (2, 128, 4, 1, 128, 192)


@pytest.mark.parametrize("B", [1, 2])
@pytest.mark.parametrize("d,heads,kv,ffn", [(2560, 20, 5, 3584), (2048, 16, 4, 6400), (3072, 24, 4, 4096)])
def test_row_kernels_wide_rows(B, d, heads, kv, ffn):
    """K = 2560 / 3584 (8 pieces in flight), 6400 (13 pieces: a group of 12 and a second trip),
    3072 and 4096; the output projection merges the attention splits at K = heads * 128."""
    cfg = S.tiny_config("bf16", base=(2, d, heads, kv, 128, ffn), aux=AUX, batch=B, seq_len=33, vocab=1000, seed=107 + d // 64)
    store = S.WeightStore(cfg)
    tok = S.draw_tokens(cfg)
    got = run_gpu(cfg, store, tok)
    compare(cfg, got, O.kvp_prefill_predict(cfg, store.f64, tok))


@pytest.mark.parametrize("B", [3, 4, 7, 8, 9, 16, 17, 37])
def test_chain_kernels_coalesced_route(B):
    """K = 2048 and 2176 (>= 64 steps, multiples of 128), N = 2048 (one row tile per block) and an
    LM head of 4112 rows (two row tiles per block).  17 and 37 sequences: grid rows of 16 right-hand
    sides in one launch (the last row ragged), which load the weights without the non-temporal hint."""
    cfg = S.tiny_config("bf16", base=(2, 2048, 16, 4, 128, 2176), aux=AUX, batch=B, seq_len=40, vocab=4112, seed=109 + B)
    store = S.WeightStore(cfg)
    tok = S.draw_tokens(cfg)
    got = run_gpu(cfg, store, tok)
    compare(cfg, got, O.kvp_prefill_predict(cfg, store.f64, tok))


def test_generation_wide_base_model():
    """Generation loop (own key / value projections on the same kernels) at K = 2048 / 2176, five sequences."""
    cfg = S.tiny_config("bf16", base=(2, 2048, 16, 4, 128, 2176), aux=AUX, batch=5, seq_len=40, vocab=4112, seed=127)
    _generate(cfg, 3)


@pytest.mark.parametrize("B,T", [(3, 500), (4, 700), (8, 300), (5, 1100), (16, 600)])
def test_chain_kernels_with_several_attention_splits(B, T):
    """Three to sixteen sequences at prompt lengths that give the decode attention 5 to 18 splits per
    (sequence, kv head): split kernel + combine launch feeding the matrix-core output projection."""
    cfg = S.tiny_config("bf16", base=(2, 2048, 16, 4, 128, 2176), aux=AUX, batch=B, seq_len=T, vocab=1000, seed=131 + B)
    store = S.WeightStore(cfg)
    tok = S.draw_tokens(cfg)
    got = run_gpu(cfg, store, tok)
    compare(cfg, got, O.kvp_prefill_predict(cfg, store.f64, tok))
