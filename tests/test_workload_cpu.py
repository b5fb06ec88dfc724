"""CPU checks of the synthetic input generator (paper_2403_17312_amd/workload.py): it holds none of the
method's arithmetic, but both the oracle and the GPU path are fed from it, and an index outside the prompt
in it is an out-of-bounds device access in the GPU tests."""
import torch

from paper_2403_17312_amd import workload as W


def test_planted_positions_lie_inside_the_prompt_and_outside_the_window():
    for w in (W_EVEN := -1, 0, 1, 5, 40, 100):
        for s in list(range(1, 70)) + [512, 2048]:
            wl = W.Workload("t_gen", 1, b=3, h=1, d=64, dtype="f16", prompt_lo=s, prompt_hi=s, steps=1, w=w,
                            sparsity_bp=5000, hh_frac=0.3)
            for seq in range(3):
                hh = W.heavy_hitter_positions(wl, seq, s)
                assert len(hh) >= 1 and len(set(hh.tolist())) == len(hh)
                assert 0 <= int(hh.min()) and int(hh.max()) < s, (w, s, hh.tolist())
                if 0 <= w < s:
                    assert int(hh.max()) < s - w, (w, s, hh.tolist())


def test_prompt_state_on_the_host_has_the_stated_shapes_and_padding():
    wl = W.Workload("t_gen2", 2, b=4, h=2, d=64, dtype="bf16", prompt_lo=1, prompt_hi=37, steps=5, w=-1,
                    sparsity_bp=8000, hh_frac=0.5)
    p = W.make_prompt(wl, "cpu", slack="nan")
    assert p["K"].shape == (4, 2, wl.cap, 64) and wl.cap % 64 == 0 and wl.cap >= 37 + 5 + 1
    for s_i, L in enumerate(p["lengths"]):
        assert 1 <= L <= 37
        assert bool(torch.isfinite(p["K"][s_i, :, :L].float()).all()) and bool(torch.isnan(p["K"][s_i, :, L:].float()).all())
        assert p["pos"][s_i, 0, :L].tolist() == list(range(L)) and bool((p["pos"][s_i, :, L:] == -1).all())
