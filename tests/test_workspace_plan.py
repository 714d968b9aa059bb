"""The workspace plan, checked on the host: for the five benchmark configurations and a grid of
(B, T), every region the planner carves ends inside kvp_workspace_bytes, no two regions overlap,
and what the launch-side shape rules say a call touches fits what the planner reserved (the
split-partial region is sized from bounds of the planner's own: an under-sized one is a device
memory fault at run time).  kvp_debug_plan runs the library's own planner without a GPU."""
import pytest

import kvp_synth as S


@pytest.fixture(scope="module")
def K():
    import os
    import paper_2410_08391_amd as K
    if not os.path.exists(K.library_path()):
        from paper_2410_08391_amd import build
        build.build(verbose=False)
    return K


def _check_plan(K, cfg, B, T, max_batch, max_seq):
    regions, total = K.kvp_debug_plan(cfg, B, T, max_batch, max_seq)
    assert total > 0 and total % 256 == 0
    end = 0
    names = set()
    for name, off, nbytes, touched in regions:
        assert name not in names, f"{cfg.name} B={B} T={T}: region {name} carved twice"
        names.add(name)
        assert off % 256 == 0, f"{cfg.name} B={B} T={T}: region {name} is not 256-byte aligned"
        assert off >= end, f"{cfg.name} B={B} T={T}: region {name} at {off} overlaps the one before it (ends at {end})"
        assert touched <= nbytes, f"{cfg.name} B={B} T={T}: a call touches {touched} bytes of {name}, {nbytes} reserved"
        end = off + nbytes
        assert end <= total, f"{cfg.name} B={B} T={T}: region {name} ends at {end}, workspace has {total}"
    assert {"aux_k", "aux_v", "x", "part", "logits", "y"} <= names
    return total


@pytest.mark.parametrize("ci", range(5))
def test_regions_fit_and_do_not_overlap(K, ci):
    cfg = S.CONFIGS[ci]
    Bs = sorted({1, 2, 3, 4, 5, 8, 16, 17, 64, cfg.batch})
    Ts = sorted({1, 2, 31, 64, 65, 127, 128, 129, 1000, 1024, 2048, 4095, 4096, 4097, 8191, 8192, 8193, 8208, 8320,
                 16384, cfg.seq_len})
    max_seq = max(Ts)
    for B in Bs:
        prev = 0
        for T in Ts:
            if B * T > 1 << 20:
                continue
            total = _check_plan(K, cfg, B, T, max(Bs), max_seq)
            # a buffer sized for T also serves every shorter prompt of B sequences
            assert total >= prev, f"{cfg.name} B={B}: workspace shrinks from {prev} to {total} bytes at T={T}"
            prev = total


def test_every_prompt_length_up_to_a_tile_boundary(K):
    """Dense sweep of T around the points where split counts change (chunks of 64 / 128 / 256 keys)."""
    cfg = S.CONFIGS[4]
    for B in (1, 4):
        prev = 0
        for T in list(range(8000, 8400)) + list(range(1, 300)):
            total = _check_plan(K, cfg, B, T, 4, 8400)
            if T > 8000:
                assert total >= prev
                prev = total


def test_layers_of_different_width(K):
    cfg = S.tiny_config("bf16", batch=3, seq_len=200, base=(4, 256, 8, 4, 128, 512), aux=(2, 128, 4, 2, 128, 256),
                        base_widths=[(4, 2, 256), (8, 4, 512), (4, 4, 384), (8, 2, 512)],
                        aux_widths=[(2, 1, 128), (4, 2, 256)])
    for B in (1, 2, 3):
        for T in (1, 64, 100, 200):
            _check_plan(K, cfg, B, T, 3, 200)


def test_bad_arguments(K):
    from paper_2410_08391_amd.binding import KVPError
    cfg = S.CONFIGS[0]
    with pytest.raises(KVPError):
        K.kvp_debug_plan(cfg, 0, 16, 4, 128)
    with pytest.raises(KVPError):
        K.kvp_debug_plan(cfg, 2, 16, 1, 128)          # B > max_batch
    with pytest.raises(KVPError):
        K.kvp_debug_plan(cfg.with_(layer_map=(0, 0, 1, 2)), 1, 16, 4, 128)     # layer map out of range
