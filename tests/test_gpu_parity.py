"""GPU parity tests: the HIP library (through its C ABI) against the fp64 oracle."""
import math
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' on CPU-only hosts)")
    from oracle import swa_oracle as O
    from paper_2403_17312_amd import binding as B
    from paper_2403_17312_amd import workload as W
    import lockstep as LS
    O.build()
    B.lib()
    return O, B, W, LS


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------------------------
# the five workloads, lock-step
# ------------------------------------------------------------------------------------
def test_c1_tiny_every_pair_every_step(env):
    O, B, W, LS = env
    _say("c1_tiny lockstep")
    rep = LS.run_lockstep(W.CONFIGS["c1_tiny"])
    _say(f"  {rep}")
    assert rep.steps == 16 and rep.evictions > 0


def test_c1_tiny_with_prefill_seed_fp32_mfma(env):
    O, B, W, LS = env
    wl = W.CONFIGS["c1_tiny"].replace(prefill_R=8)
    _say("c1_tiny lockstep with prefill seed (fp32 MFMA path)")
    rep = LS.run_lockstep(wl)
    _say(f"  {rep}")


def test_free_running_trajectories_part_only_at_near_ties(env):
    # no state adoption: the fp32 GPU path and the fp64 oracle each run on their own; they may only
    # part where the oracle's importance values are tied to within 2e-5 relative
    O, B, W, LS = env
    for name in ("c1_tiny", "c2_opt6p7b"):
        step, flipped = LS.run_free(W.CONFIGS[name])
        _say(f"  {name}: free-running, first divergent step {step} ({flipped} near-tie flips)")
    step, flipped = LS.run_free(W.CONFIGS["c1_tiny"].replace(prefill_R=8))
    _say(f"  c1_tiny with prefill seed: first divergent step {step} ({flipped} near-tie flips)")


def test_c1_tiny_without_compaction(env):
    # decode steps back to back with no compaction: every slot stays a candidate
    O, B, W, LS = env
    _say("c1_tiny lockstep, never compacted")
    rep = LS.run_lockstep(W.CONFIGS["c1_tiny"], compact_every=0)
    assert rep.steps == 16
    rep = LS.run_lockstep(W.CONFIGS["c1_tiny"], compact_every=5)
    assert rep.steps == 16


def test_lazy_compaction_at_full_size(env):
    # the cache keeps every token between compactions and the selection runs over all of them:
    # config 2 compacting every 8th step (every pair), config 3 never compacting (sampled pairs)
    O, B, W, LS = env
    _say("c2 lockstep, compaction every 8 steps")
    rep = LS.run_lockstep(W.CONFIGS["c2_opt6p7b"], compact_every=8, use_len_bound=True)
    _say(f"  {rep}")
    assert rep.steps == 32 and rep.evictions > 0
    _say("c3 lockstep, never compacted, sampled pairs")
    rep = LS.run_lockstep(W.CONFIGS["c3_opt13b"], compact_every=0, steps=12, seqs=[0, 31, 63],
                          heads=[0, 17, 39], use_len_bound=True)
    _say(f"  {rep}")
    assert rep.steps == 12


def test_c2_opt6p7b_every_pair_every_step(env):
    O, B, W, LS = env
    _say("c2 lockstep")
    rep = LS.run_lockstep(W.CONFIGS["c2_opt6p7b"])
    _say(f"  {rep}")
    assert rep.steps == 32
    # the launch configuration bench.py times: LDS sized from the host's length bound
    rep = LS.run_lockstep(W.CONFIGS["c2_opt6p7b"], use_len_bound=True)
    assert rep.steps == 32


def test_fused_compaction_matches_the_two_call_path(env):
    # swa_decode_step with SWA_FUSE_COMPACTION against the oracle's step + stable gather
    O, B, W, LS = env
    _say("c1 / c2 lockstep, fused compaction")
    rep = LS.run_lockstep(W.CONFIGS["c1_tiny"], fused=True)
    assert rep.steps == 16 and rep.evictions > 0
    rep = LS.run_lockstep(W.CONFIGS["c1_tiny"].replace(prefill_R=8, w=0), fused=True)
    rep = LS.run_lockstep(W.CONFIGS["c2_opt6p7b"], fused=True, use_len_bound=True)
    _say(f"  {rep}")
    assert rep.steps == 32
    for dtype, d in [("f32", 128), ("bf16", 64), ("f16", 64)]:
        wl = W.Workload(f"t_fc_{dtype}_{d}", 17, b=3, h=5, d=d, dtype=dtype, prompt_lo=2, prompt_hi=333,
                        steps=12, w=7, sparsity_bp=7000, hh_frac=0.02, prefill_R=5)
        LS.run_lockstep(wl, fused=True)
    # sparsity 0 (nothing ever evicted), and a budget that evicts several tokens per step
    LS.run_lockstep(W.Workload("t_fc_dense", 18, b=2, h=3, d=128, dtype="f16", prompt_lo=1, prompt_hi=90,
                               steps=9, w=4, sparsity_bp=0, hh_frac=0.02), fused=True)
    LS.run_lockstep(W.Workload("t_fc_w0", 19, b=2, h=3, d=128, dtype="f16", prompt_lo=50, prompt_hi=90,
                               steps=9, w=0, sparsity_bp=9000, hh_frac=0.02), fused=True)


def test_unordered_compaction_matches_the_oracle_as_a_set(env):
    # SWA_FUSE_COMPACTION | SWA_UNORDERED: holes are filled instead of shifting rows; the cache is
    # compared with the oracle after sorting by token position
    O, B, W, LS = env
    _say("c1 / c2 lockstep, unordered compaction")
    rep = LS.run_lockstep(W.CONFIGS["c1_tiny"], fused=True, unordered=True)
    assert rep.steps == 16 and rep.evictions > 0
    LS.run_lockstep(W.CONFIGS["c1_tiny"].replace(prefill_R=8, w=0), fused=True, unordered=True)
    # config 2, every pair, every step, with the twin state in the call form bench.py times
    rep = LS.run_lockstep(W.CONFIGS["c2_opt6p7b"], fused=True, unordered=True, use_len_bound=True, twin=True)
    _say(f"  {rep}")
    assert rep.steps == 32 and rep.twin_steps == 32
    for dtype, d in [("f32", 128), ("bf16", 64), ("f16", 64), ("bf16", 128)]:
        wl = W.Workload(f"t_un_{dtype}_{d}", 27, b=3, h=5, d=d, dtype=dtype, prompt_lo=2, prompt_hi=333,
                        steps=12, w=7, sparsity_bp=7000, hh_frac=0.02, prefill_R=5)
        LS.run_lockstep(wl, fused=True, unordered=True)
    LS.run_lockstep(W.Workload("t_un_dense", 28, b=2, h=3, d=128, dtype="f16", prompt_lo=1, prompt_hi=90,
                               steps=9, w=4, sparsity_bp=0, hh_frac=0.02), fused=True, unordered=True)
    LS.run_lockstep(W.Workload("t_un_w0", 29, b=2, h=3, d=128, dtype="f16", prompt_lo=50, prompt_hi=90,
                               steps=9, w=0, sparsity_bp=9000, hh_frac=0.02), fused=True, unordered=True)
    LS.run_lockstep(W.Workload("t_un_win", 30, b=2, h=3, d=128, dtype="f16", prompt_lo=5, prompt_hi=40,
                               steps=30, w=16, sparsity_bp=9999, hh_frac=0.02), fused=True, unordered=True)


def test_unordered_ties_go_to_the_earliest_token(env):
    # identical prompt keys => bitwise-equal importance among the old tokens at every step; once the
    # slots are no longer in token order the tie rule must follow pos, as the oracle's does
    O, B, W, LS = env
    for sp, w in [(5000, 3), (3000, 0), (8000, 5)]:
        wl = W.Workload("t_un_ties", 31, b=2, h=3, d=128, dtype="f16", prompt_lo=40, prompt_hi=70,
                        steps=25, w=w, sparsity_bp=sp, hh_frac=0.02)
        prompt = W.make_prompt(wl, "cuda", slack="nan")
        for s_i, L in enumerate(prompt["lengths"]):
            prompt["K"][s_i, :, :L] = prompt["K"][s_i, :, :1].clone()
        rep = LS.run_lockstep(wl, prompt=prompt, fused=True, unordered=True)
        assert rep.evictions > 0
        # a budget that tightens later: many evictions at once on a cache that is out of token
        # order and full of exact ties (radix select + rank-by-position path)
        prompt = W.make_prompt(wl, "cuda", slack="nan")
        for s_i, L in enumerate(prompt["lengths"]):
            prompt["K"][s_i, :, :L] = prompt["K"][s_i, :, :1].clone()
        rep = LS.run_lockstep(wl, prompt=prompt, fused=True, unordered=True,
                              sparsity_of_step=lambda t: 2000 if t < 12 else (8500 if t < 14 else 6000))
        assert rep.evictions > 0
        # the ordered mode on the same inputs (ties by slot) must agree with the oracle as well
        prompt = W.make_prompt(wl, "cuda", slack="nan")
        for s_i, L in enumerate(prompt["lengths"]):
            prompt["K"][s_i, :, :L] = prompt["K"][s_i, :, :1].clone()
        LS.run_lockstep(wl, prompt=prompt, fused=True)


def test_unordered_window_that_was_widened_keeps_exactly_the_budget(env):
    # The unordered form finds the window by token position.  When the caller widens w (and tightens
    # the budget) between two calls, some positions of the new window were evicted long ago: the step
    # must still keep exactly `keep` tokens - every present window token, and the best of the others
    # for the rest - and leave a dense cache whose rows are the kept tokens' rows.
    O, B, W, LS = env
    wl = W.Workload("t_un_grow", 37, b=3, h=4, d=128, dtype="f16", prompt_lo=60, prompt_hi=140, steps=12, w=4,
                    sparsity_bp=5000, hh_frac=0.02)
    prompt = W.make_prompt(wl, "cuda", slack="nan")
    st = LS.new_state(wl, prompt)
    st.score.zero_()
    st.params.flags = B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED
    for t in range(wl.steps):
        q, kn, vn = W.make_step(wl, t, prompt["mu"])
        st.seq_len += 1
        st.decode_compact_step(q, kn, vn)
    assert st.check_status() == 0
    # the widened step: w 4 -> 24, sparsity 50 % -> 80 %
    w2, sp2 = 24, 8000
    lens = st.cache_len.cpu().numpy()
    # a copy in the two-call form gives the weights and the new importance of every slot (same arithmetic)
    ref = LS.new_state(wl, dict(prompt, K=st.K.clone(), V=st.V.clone(), pos=st.pos.clone()))
    for name in ("score", "cache_len", "seq_len"):
        getattr(ref, name).copy_(getattr(st, name))
    ref.params.w, ref.params.sparsity_bp = w2, sp2
    st.params.w, st.params.sparsity_bp = w2, sp2
    q, kn, vn = W.make_step(wl, wl.steps, prompt["mu"])
    ref.seq_len += 1
    ref.decode_step(q, kn, vn)
    st.seq_len += 1
    st.decode_compact_step(q, kn, vn)
    assert st.check_status() == 0
    n = st.seq_len.cpu().numpy()
    snew, probs = LS._np64(ref.score), LS._np64(ref.probs)
    pos_all = ref.pos.cpu().numpy()                          # slot len holds the new token now
    Kall, Vall = LS._np64(ref.K), LS._np64(ref.V)
    got_len = st.cache_len.cpu().numpy()
    gpos, gK, gV, gS = st.pos.cpu().numpy(), LS._np64(st.K), LS._np64(st.V), LS._np64(st.score)
    out_g = LS._np64(st.out)
    grew = 0
    for s_i in range(wl.b):
        m = int(lens[s_i]) + 1
        keep, n_local, _ = O.budget(int(n[s_i]), m, w2, sp2)
        assert got_len[s_i] == keep < m
        wlo = int(n[s_i]) - n_local
        for hd in range(wl.h):
            p_ = pos_all[s_i, hd, :m]
            window = [i for i in range(m) if p_[i] >= wlo]
            grew += len(window) < n_local
            others = sorted((i for i in range(m) if p_[i] < wlo), key=lambda i: (-snew[s_i, hd, i], p_[i]))
            want = window + others[:keep - len(window)]
            want_pos = sorted(int(p_[i]) for i in want)
            got_pos = gpos[s_i, hd, :keep].tolist()
            assert sorted(got_pos) == want_pos, f"pair {s_i},{hd}: kept tokens"
            slot_of = {int(p_[i]): i for i in range(m)}
            for j, tp in enumerate(got_pos):                # the rows in the compacted cache are those tokens' rows
                i = slot_of[tp]
                assert np.array_equal(gK[s_i, hd, j], Kall[s_i, hd, i]) and np.array_equal(gV[s_i, hd, j], Vall[s_i, hd, i])
                assert gS[s_i, hd, j] == snew[s_i, hd, i]
            idx = np.array(sorted(want), dtype=np.int32)[None, None, :]
            out_o = O.sparse_attention(LS._np64(q[s_i:s_i + 1, hd:hd + 1]), Kall[s_i:s_i + 1, hd:hd + 1],
                                       Vall[s_i:s_i + 1, hd:hd + 1], idx, np.array([keep], dtype=np.int32), wl.scale)
            LS.check_out(out_g[s_i:s_i + 1, hd:hd + 1], out_o, wl.dtype, f"widened window, pair {s_i},{hd}")
    assert grew > 0, "the case must contain windows with evicted positions"


def test_a_budget_that_keeps_no_token_gives_a_zero_output_and_an_empty_cache(env):
    # no local window (w = 0, or the even split with k = 0) and n r below one half: keep = 0, the sum over
    # the kept set is empty, the output is zero (as the oracle's) and the cache is empty afterwards
    O, B, W, LS = env
    sched = [9900, 9900, 5000, 9999, 9999, 0, 9950, 9000]
    for form in ["split", "fused", "unordered", "shared", "q8", "window", "lazy"]:
        for w in (0, B.SWA_W_EVEN_SPLIT):
            wl = W.Workload("t_keep0", 91, b=3, h=2, d=64, dtype="f16" if form == "q8" else "bf16", prompt_lo=3,
                            prompt_hi=40, steps=8, w=w, sparsity_bp=9900, hh_frac=0.03)
            _say(f"  empty budget: {form} w={w}")
            sp = lambda t: sched[t]
            if form == "window":
                rep = LS.run_lockstep_window(wl, 5, sparsity_of_step=sp)
            elif form == "lazy":
                rep = LS.run_lockstep(wl, compact_every=3, sparsity_of_step=sp)
            else:
                rep = LS.run_lockstep(wl, fused=form != "split", unordered=form in ("unordered", "shared", "q8"),
                                      head_shared=form == "shared", kv_int8=form == "q8", sparsity_of_step=sp)
            assert rep.evictions > 0
    # the call itself: one step on a 5-token cache at 99.99 % sparsity
    wl = W.Workload("t_keep0_one", 92, b=2, h=2, d=128, dtype="f16", prompt_lo=5, prompt_hi=5, steps=1, w=0,
                    sparsity_bp=9999, hh_frac=0.03)
    prompt = W.make_prompt(wl, "cuda", slack="nan")
    for flags in (0, B.SWA_FUSE_COMPACTION, B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED):
        st = LS.new_state(wl, dict(prompt, K=prompt["K"].clone(), V=prompt["V"].clone(), pos=prompt["pos"].clone()))
        st.score.zero_()
        st.params.flags = flags
        st.out.fill_(7.0)
        q, kn, vn = W.make_step(wl, 0, prompt["mu"])
        st.seq_len += 1
        if flags:
            st.decode_compact_step(q, kn, vn)
        else:
            st.decode_step(q, kn, vn)
            assert st.kept_cnt.tolist() == [0, 0]
            st.compact()
        assert st.check_status() == 0
        assert st.cache_len.tolist() == [0, 0] and bool((st.out == 0).all())


def test_even_split_of_algorithm_1_in_every_step_mode(env):
    # w = SWA_W_EVEN_SPLIT: k = nint(n r / 2) local and k global tokens, recomputed per sequence and step
    O, B, W, LS = env
    for sp in (8000, 5000):
        wl = W.Workload("t_even", 33, b=4, h=3, d=128, dtype="f16", prompt_lo=30, prompt_hi=400,
                        steps=14, w=B.SWA_W_EVEN_SPLIT, sparsity_bp=sp, hh_frac=0.02, prefill_R=4)
        _say(f"even split sp={sp}")
        r0 = LS.run_lockstep(wl)
        r1 = LS.run_lockstep(wl, fused=True)
        r2 = LS.run_lockstep(wl, fused=True, unordered=True)
        assert r0.evictions == r1.evictions == r2.evictions > 0
    rep = LS.run_lockstep(W.CONFIGS["c2_opt6p7b"].replace(w=B.SWA_W_EVEN_SPLIT), fused=True, unordered=True,
                          use_len_bound=True)
    assert rep.steps == 32


def test_head_shared_selection_matches_the_oracle(env):
    # SWA_HEAD_SHARED: the local attention sum is reduced over the heads, one token set per sequence
    O, B, W, LS = env
    _say("head-shared selection")
    rep = LS.run_lockstep(W.CONFIGS["c1_tiny"], fused=True, unordered=True, head_shared=True)
    assert rep.steps == 16 and rep.evictions > 0
    for dtype, d, w in [("f16", 128, 7), ("bf16", 64, 0), ("f32", 128, B.SWA_W_EVEN_SPLIT)]:
        wl = W.Workload(f"t_sh_{dtype}", 35, b=3, h=5, d=d, dtype=dtype, prompt_lo=2, prompt_hi=333,
                        steps=12, w=w, sparsity_bp=7000, hh_frac=0.02, prefill_R=5)
        rep = LS.run_lockstep(wl, fused=True, unordered=True, head_shared=True)
        assert rep.evictions > 0
    # a budget that tightens later (many evictions at once on a cache out of token order)
    wl = W.Workload("t_sh_sched", 36, b=2, h=4, d=128, dtype="f16", prompt_lo=60, prompt_hi=90,
                    steps=20, w=4, sparsity_bp=3000, hh_frac=0.02)
    LS.run_lockstep(wl, fused=True, unordered=True, head_shared=True,
                    sparsity_of_step=lambda t: 3000 if t < 10 else (8500 if t < 12 else 6000))
    # config 2 at full size, every pair
    rep = LS.run_lockstep(W.CONFIGS["c2_opt6p7b"], fused=True, unordered=True, head_shared=True,
                          use_len_bound=True)
    _say(f"  {rep}")
    assert rep.steps == 32
    # every head of a sequence ends with the same tokens
    wl = W.CONFIGS["c2_opt6p7b"]
    prompt = W.make_prompt(wl, "cuda")
    st = LS.new_state(wl, prompt, debug_probs=False)
    st.params.flags = B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED | B.SWA_HEAD_SHARED
    st.workspace = torch.zeros((B.swa_workspace_bytes(st.params),), dtype=torch.uint8, device="cuda")
    B.swa_workspace_init(st.params, st.workspace)
    st.score.zero_()
    for t in range(6):
        q, kn, vn = W.make_step(wl, t, prompt["mu"])
        st.seq_len += 1
        st.decode_compact_step(q, kn, vn)
    L = int(st.cache_len[0])
    srt = st.pos[:, :, :L].sort(dim=-1).values
    assert torch.equal(srt, srt[:, :1].expand_as(srt))


def test_kv_int8_compressed_cache_matches_the_oracle(env):
    # Section V-B: 8-bit channel-wise codes in memory; parameters and codes bit-exact, the step
    # against the oracle on the de-quantised values, in every way the step can be issued
    O, B, W, LS = env
    _say("compressed cache, small shapes")
    for d, w, modes in [(128, 7, ("unordered", "fused", "split")), (64, 3, ("unordered", "split"))]:
        wl = W.Workload(f"t_q8_d{d}", 37, b=3, h=3, d=d, dtype="f16", prompt_lo=1, prompt_hi=300,
                        steps=14, w=w, sparsity_bp=7500, hh_frac=0.02, prefill_R=6)
        for mode in modes:
            _say(f"  d={d} {mode}")
            rep = LS.run_lockstep(wl, fused=mode != "split", unordered=mode == "unordered", kv_int8=True)
            assert rep.evictions > 0
    wl = W.Workload("t_q8_shared", 38, b=2, h=4, d=128, dtype="f16", prompt_lo=40, prompt_hi=200,
                    steps=10, w=SW_EVEN(B), sparsity_bp=6000, hh_frac=0.02)
    LS.run_lockstep(wl, fused=True, unordered=True, head_shared=True, kv_int8=True)
    _say("compressed cache, config 2 at full size, every pair")
    rep = LS.run_lockstep(W.CONFIGS["c2_opt6p7b"], fused=True, unordered=True, kv_int8=True, use_len_bound=True)
    _say(f"  {rep}")
    assert rep.steps == 32


def SW_EVEN(B):
    return B.SWA_W_EVEN_SPLIT


def test_strict_window_sum_matches_the_oracle(env):
    # Algorithm 1 line 2 to the letter: importance = sum of the last R attention rows (a ring)
    O, B, W, LS = env
    _say("strict window, small shapes")
    for dtype, d, R, w in [("f32", 64, 4, 8), ("f16", 128, 16, 7), ("bf16", 128, 5, 0), ("f16", 64, 1, 3)]:
        wl = W.Workload(f"t_win_{dtype}_{R}", 39, b=3, h=3, d=d, dtype=dtype, prompt_lo=2, prompt_hi=300,
                        steps=3 * R + 5, w=w, sparsity_bp=7000, hh_frac=0.02)
        _say(f"  {dtype} d={d} R={R}")
        rep = LS.run_lockstep_window(wl, R)
        assert rep.evictions > 0
    rep = LS.run_lockstep_window(W.CONFIGS["c1_tiny"], 8, seed_rows=False)
    assert rep.steps == 16
    # budget that tightens and relaxes: many evictions at once on a cache out of token order
    wl = W.Workload("t_win_sched", 40, b=2, h=4, d=128, dtype="f16", prompt_lo=60, prompt_hi=90,
                    steps=24, w=4, sparsity_bp=3000, hh_frac=0.02)
    LS.run_lockstep_window(wl, 6, sparsity_of_step=lambda t: 3000 if t < 10 else (8500 if t < 12 else 6000))
    wl = W.Workload("t_win_even", 41, b=2, h=2, d=128, dtype="f16", prompt_lo=100, prompt_hi=140,
                    steps=20, w=B.SWA_W_EVEN_SPLIT, sparsity_bp=8000, hh_frac=0.02)
    LS.run_lockstep_window(wl, 8)
    _say("strict window, config 2 at full size (R = w = 16), every pair")
    rep = LS.run_lockstep_window(W.CONFIGS["c2_opt6p7b"], 16, use_len_bound=True)
    _say(f"  {rep}")
    assert rep.steps == 32


def test_strict_window_on_the_compressed_cache_and_with_the_head_reduced_set(env):
    # Algorithm 1 line 2 (the ring of attention rows) combined with Section V-B (8-bit cache) and with
    # the note in Algorithm 1's header (importance summed over the heads), and all three together
    O, B, W, LS = env
    for dtype, d, R, w, q8, sh in [("f16", 128, 6, 5, True, False), ("f16", 64, 3, 0, True, False),
                                   ("f16", 128, 5, 4, False, True), ("bf16", 64, 4, 7, False, True),
                                   ("f32", 128, 2, B.SWA_W_EVEN_SPLIT, False, True), ("f16", 128, 7, 3, True, True)]:
        wl = W.Workload(f"t_winx_{dtype}_{R}", 47, b=3, h=4, d=d, dtype=dtype, prompt_lo=2, prompt_hi=260,
                        steps=2 * R + 6, w=w, sparsity_bp=7000, hh_frac=0.02)
        _say(f"  window x {'int8 ' if q8 else ''}{'head-shared ' if sh else ''}{dtype} d={d} R={R}")
        rep = LS.run_lockstep_window(wl, R, kv_int8=q8, head_shared=sh)
        assert rep.evictions > 0
    # a budget that tightens and relaxes, all three combined
    wl = W.Workload("t_winx_sched", 48, b=2, h=4, d=128, dtype="f16", prompt_lo=60, prompt_hi=90,
                    steps=24, w=4, sparsity_bp=3000, hh_frac=0.02)
    LS.run_lockstep_window(wl, 6, kv_int8=True, head_shared=True,
                           sparsity_of_step=lambda t: 3000 if t < 10 else (8500 if t < 12 else 6000))
    _say("  config 2 at full size, every pair: window x int8, window x head-shared")
    rep = LS.run_lockstep_window(W.CONFIGS["c2_opt6p7b"], 16, use_len_bound=True, kv_int8=True)
    assert rep.steps == 32
    rep = LS.run_lockstep_window(W.CONFIGS["c2_opt6p7b"], 16, use_len_bound=True, head_shared=True)
    _say(f"  {rep}")
    assert rep.steps == 32


def test_rows_split_over_workgroups_matches_the_oracle_and_the_one_workgroup_form(env):
    # SWA_SPLIT_ROWS: few pairs with long caches; the step runs as four launches
    O, B, W, LS = env
    for dtype, d, b, h, hi, ce in [("f16", 128, 1, 4, 2500, 0), ("bf16", 128, 2, 2, 2300, 3), ("f32", 64, 1, 3, 2100, 1),
                                   ("f16", 64, 2, 3, 900, 0), ("bf16", 64, 1, 1, 5000, 2)]:   # 900: the one-workgroup fall-back
        wl = W.Workload(f"t_split_{dtype}_{d}", 81, b=b, h=h, d=d, dtype=dtype, prompt_lo=hi // 2, prompt_hi=hi, steps=6,
                        w=16, sparsity_bp=8000, hh_frac=0.01, prefill_R=8)
        _say(f"  split rows: {dtype} d={d} b={b} h={h} prompts {hi // 2}..{hi}, compaction every {ce}")
        assert B.swa_workspace_bytes(B.make_params(b, h, d, wl.cap, 16, 8000, wl.torch_dtype, flags=B.SWA_SPLIT_ROWS)) > \
            2 * 4 * b * h * wl.cap
        rep = LS.run_lockstep(wl, compact_every=ce, split_rows=True, use_len_bound=True, twin=True)
        assert rep.steps == 6 and rep.evictions > 0
    # weights, importance and kept lists are bit-identical to the one-workgroup form; outputs within tolerance
    wl = W.Workload("t_split_same", 82, b=2, h=4, d=128, dtype="f16", prompt_lo=700, prompt_hi=3000, steps=5, w=32,
                    sparsity_bp=9000, hh_frac=0.01)
    prompt = W.make_prompt(wl, "cuda", slack="nan")
    states = []
    for flags in (0, B.SWA_SPLIT_ROWS):
        st = LS.new_state(wl, dict(prompt, K=prompt["K"].clone(), V=prompt["V"].clone(), pos=prompt["pos"].clone()))
        st.params.flags = flags
        st.workspace = torch.zeros((B.swa_workspace_bytes(st.params),), dtype=torch.uint8, device="cuda")
        B.swa_workspace_init(st.params, st.workspace)
        st.score.zero_()
        states.append(st)
    for t in range(wl.steps):
        q, kn, vn = W.make_step(wl, t, prompt["mu"])
        for st in states:
            st.seq_len += 1
            st.decode_step(q, kn, vn)
        a, b_ = states
        assert torch.equal(a.cache_len, b_.cache_len) and torch.equal(a.kept_cnt, b_.kept_cnt)
        for s_i, L in enumerate(a.cache_len.tolist()):
            c = int(a.kept_cnt[s_i])
            assert torch.equal(a.probs[s_i, :, :L], b_.probs[s_i, :, :L]), f"step {t}: weights"
            assert torch.equal(a.score[s_i, :, :L], b_.score[s_i, :, :L]), f"step {t}: importance"
            assert torch.equal(a.kept_idx[s_i, :, :c], b_.kept_idx[s_i, :, :c]), f"step {t}: kept list"
        assert float((a.out.float() - b_.out.float()).abs().max()) <= 2e-3
        if t % 2 == 1:
            for st in states:
                st.compact()
    # a full cache: the sequence is skipped by all four launches and reported
    b, h, d, cap = 2, 2, 128, 512
    params = B.make_params(b, h, d, cap, 4, 5000, torch.float16, flags=B.SWA_SPLIT_ROWS)
    st = B.DecodeState(params)
    st.K.normal_()
    st.V.normal_()
    st.cache_len.copy_(torch.tensor([512, 400], dtype=torch.int32))
    st.seq_len.copy_(torch.tensor([513, 401], dtype=torch.int32))
    st.out.fill_(7.0)
    st.kept_cnt.fill_(-7)
    x = torch.randn((b, h, d), device="cuda").half()
    st.decode_step(x, x, x)
    assert st.check_status() == B.SWA_ERR_CAPACITY
    assert st.cache_len.tolist() == [512, 401] and st.kept_cnt[0].item() == -7
    assert bool((st.out[0] == 7.0).all()) and not bool((st.out[1] == 7.0).any())


def test_c3_opt13b_full_size_sampled_pairs(env):
    O, B, W, LS = env
    wl = W.CONFIGS["c3_opt13b"]
    _say("c3 lockstep (full size on the GPU, sampled pairs checked)")
    rep = LS.run_lockstep(wl, seqs=[0, 1, 17, 31, 32, 63], heads=[0, 7, 20, 39], slack="zero",
                          use_len_bound=True)
    _say(f"  {rep}")
    rep = LS.run_lockstep(wl, seqs=[0, 1, 17, 31, 32, 63], heads=[0, 7, 20, 39], slack="zero",
                          use_len_bound=True, fused=True)
    _say(f"  {rep}")
    rep = LS.run_lockstep(wl, seqs=[0, 1, 17, 31, 32, 63], heads=[0, 7, 20, 39], slack="zero",
                          use_len_bound=True, fused=True, unordered=True, twin=True, twin_kv_every=8)
    _say(f"  {rep}")
    assert rep.steps == 64 and rep.twin_steps == 64


def test_c4_opt30b_full_size_sampled_pairs_with_mfma_prefill(env):
    O, B, W, LS = env
    wl = W.CONFIGS["c4_opt30b"]
    _say("c4 lockstep (full size, bf16, MFMA prefill seed)")
    rep = LS.run_lockstep(wl, seqs=[0, 13, 31], heads=[0, 28, 55], slack="zero", use_len_bound=True)
    _say(f"  {rep}")
    rep = LS.run_lockstep(wl, seqs=[0, 13, 31], heads=[0, 28, 55], slack="zero", use_len_bound=True,
                          fused=True)
    _say(f"  {rep}")
    rep = LS.run_lockstep(wl, seqs=[0, 13, 31], heads=[0, 28, 55], slack="zero", use_len_bound=True,
                          fused=True, unordered=True, twin=True, twin_kv_every=16)
    _say(f"  {rep}")
    _say(f"  bf16 outputs beyond the 2e-3 bar stated for fp16: {rep.out_over_2e3} of {rep.out_elems}")
    assert rep.steps == 128 and rep.twin_steps == 128


def test_full_size_sampled_pairs_in_the_other_step_forms(env):
    # configs 3-5 at full size on the GPU, in the launch configurations bench.py times with
    # --kv-int8, --step-mode window and --step-mode shared; sampled pairs checked
    O, B, W, LS = env
    c3, c4, c5 = W.CONFIGS["c3_opt13b"], W.CONFIGS["c4_opt30b"], W.CONFIGS["c5_llama7b_sp80"]
    _say("c3, compressed cache")
    rep = LS.run_lockstep(c3, seqs=[0, 17, 63], heads=[0, 20, 39], slack="zero", use_len_bound=True,
                          fused=True, unordered=True, kv_int8=True)
    _say(f"  {rep}")
    assert rep.steps == 64
    _say("c3, strict window (R = w = 32)")
    rep = LS.run_lockstep_window(c3, 32, seqs=[0, 17, 63], heads=[0, 20, 39], slack="zero", use_len_bound=True)
    _say(f"  {rep}")
    assert rep.steps == 64
    _say("c4, strict window (R = w = 64), first steps")
    rep = LS.run_lockstep_window(c4, 64, steps=6, seqs=[0, 31], heads=[0, 55], slack="zero", use_len_bound=True)
    _say(f"  {rep}")
    _say("c3, head-shared (all heads of two sequences)")
    rep = LS.run_lockstep(c3, steps=16, seqs=[5, 63], slack="zero", use_len_bound=True, fused=True,
                          unordered=True, head_shared=True)
    _say(f"  {rep}")
    lens = W.prompt_lengths(c5).tolist()
    seqs = sorted({int(np.argmin(lens)), int(np.argmax(lens)), 100})
    _say(f"c5 (80 %), compressed cache, seqs {seqs}")
    rep = LS.run_lockstep(c5, steps=24, seqs=seqs, heads=[0, 31], slack="zero", use_len_bound=True, fused=True,
                          unordered=True, kv_int8=True)
    _say(f"  {rep}")
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["c5_llama7b_sp50", "c5_llama7b_sp80", "c5_llama7b_sp90"])
def test_c5_llama7b_full_size_sampled_pairs(env, name):
    # the form bench.py times (one kernel, hole-filling compaction, per-step length bound), whole
    # trajectory, with the twin state that runs without debug outputs
    O, B, W, LS = env
    wl = W.CONFIGS[name]
    lens = W.prompt_lengths(wl).tolist()
    seqs = sorted({int(np.argmin(lens)), int(np.argmax(lens)), 0, 100, 255})
    _say(f"{name} lockstep (full size, mixed lengths {min(lens)}..{max(lens)}, seqs {seqs})")
    check = set(range(0, 256, 3)) | {1, 2, 254, 255}
    rep = LS.run_lockstep(wl, seqs=seqs, heads=[0, 15, 31], slack="zero", check_steps=check,
                          use_len_bound=True, fused=True, unordered=True, twin=True, twin_kv_every=32)
    _say(f"  {rep}")
    assert rep.steps == 256 and rep.twin_steps == 256
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name,form", [("c5_llama7b_sp50", "split"), ("c5_llama7b_sp90", "fused"),
                                       ("c5_llama7b_sp80", "split"), ("c5_llama7b_sp50", "fused")])
def test_c5_llama7b_full_size_in_the_token_ordered_forms(env, name, form):
    O, B, W, LS = env
    wl = W.CONFIGS[name]
    lens = W.prompt_lengths(wl).tolist()
    seqs = sorted({int(np.argmin(lens)), int(np.argmax(lens)), 7, 200})
    _say(f"{name} lockstep, {form}")
    check = set(range(0, 256, 5)) | {1, 2, 254, 255}
    rep = LS.run_lockstep(wl, seqs=seqs, heads=[0, 15, 31], slack="zero", check_steps=check,
                          use_len_bound=True, fused=(form == "fused"), twin=True, twin_kv_every=64)
    _say(f"  {rep}")
    assert rep.steps == 256
    torch.cuda.empty_cache()


EVERY_PAIR = [("c3_opt13b", 0, 64), ("c4_opt30b", 0, 16), ("c4_opt30b", 16, 32),
              ("c5_llama7b_sp80", 0, 128), ("c5_llama7b_sp80", 128, 256),
              ("c5_llama7b_sp50", 0, 128), ("c5_llama7b_sp50", 128, 256),
              ("c5_llama7b_sp90", 0, 128), ("c5_llama7b_sp90", 128, 256)]


@pytest.mark.parametrize("name,first,last", EVERY_PAIR)
def test_every_pair_on_the_first_and_the_first_steady_steps(env, name, first, last):
    # configs 3-5 at full size, in the form bench.py times: EVERY (sequence, head) pair of the
    # sequence range is checked against the oracle on the step right after the prompt (many
    # evictions: key pass, radix select, gather) and on the two steady steps that follow
    O, B, W, LS = env
    wl = W.CONFIGS[name]
    chunk = {3: 16, 4: 4, 5: 16}[wl.config_id]
    _say(f"{name}: every pair of sequences {first}..{last - 1}, steps 0-2")
    rep = LS.run_every_pair(wl, 3, chunk, first_seq=first, last_seq=last, fused=True, unordered=True)
    _say(f"  {rep}")
    assert rep.steps == 3 and rep.pairs == (last - first) * wl.h and rep.evictions > 0
    if wl.dtype == "bf16":
        _say(f"  bf16 outputs beyond the 2e-3 bar stated for fp16: {rep.out_over_2e3} of {rep.out_elems}")
    torch.cuda.empty_cache()


def test_prefill_attention_at_the_benchmarked_shape_sampled_pairs(env):
    # config 4's prompts (1792 pairs x 4096 tokens, bf16), the shape bench.py --prefill-attention
    # times: the kernel runs at full size, sampled pairs are compared with the oracle row by row
    # (tolerance as in test_prefill_attention_matches_the_oracle), the seed on the same pairs
    O, B, W, LS = env
    wl = W.CONFIGS["c4_opt30b"]
    prompt = W.make_prompt(wl, "cuda")
    g = torch.Generator(device="cuda").manual_seed(4096)
    Q = torch.randn((wl.b, wl.h, wl.cap, wl.d), generator=g, device="cuda", dtype=torch.float32).to(wl.torch_dtype)
    out = torch.full_like(Q, 7.0)
    score = torch.full((wl.b, wl.h, wl.cap), float("nan"), dtype=torch.float32, device="cuda")
    R = wl.prefill_R
    L = wl.prompt_hi
    params = B.make_params(wl.b, wl.h, wl.d, wl.cap, wl.w, wl.sparsity_bp, wl.torch_dtype, len_bound=L)
    ws = torch.zeros((B.swa_workspace_bytes(params),), dtype=torch.uint8, device="cuda")
    B.swa_prefill_attention(params, Q, prompt["K"], prompt["V"], prompt["cache_len"], out, R, score, ws)
    torch.cuda.synchronize()
    assert bool((out[:, :, L:] == 7.0).all()), "rows past the prompt must not be written"
    pairs = [(0, 0), (0, 55), (13, 28), (31, 0), (31, 55), (17, 3)]
    si = torch.tensor([p[0] for p in pairs], device="cuda")
    hi = torch.tensor([p[1] for p in pairs], device="cuda")
    pick = lambda x: np.ascontiguousarray(x[si, hi][:, None, :L].double().cpu().numpy())      # [pairs, 1, L, ...]
    Qn, Kn, Vn, og, S_g = pick(Q), pick(prompt["K"]), pick(prompt["V"]), pick(out), pick(score)
    ln = np.full((len(pairs),), L, dtype=np.int32)
    _say("  oracle: dense causal attention of the sampled pairs")
    ref = O.prefill_attention(Qn, Kn, Vn, ln, wl.scale)
    mag = O.prefill_attention(Qn, Kn, np.abs(Vn), ln, wl.scale)
    u = 2.0 ** -8
    err = np.abs(og - ref)
    bound = 1.5 * u * (mag + np.abs(ref)) + 1e-5
    assert np.all(np.isfinite(og))
    assert np.all(err <= bound), f"max excess {np.max(err - bound):.3e}"
    S_ref = O.prefill_scores(np.ascontiguousarray(Qn[:, :, L - R:]), Kn, ln, wl.scale)
    np.testing.assert_allclose(S_g, S_ref, rtol=1e-5, atol=1e-12)
    _say(f"  {len(pairs)} pairs x {L} rows: max |delta| {err.max():.3e}, max delta/bound {np.max(err / bound):.3f}")
    del Q, out, score, prompt
    torch.cuda.empty_cache()


# ------------------------------------------------------------------------------------
# shapes, dtypes, edge cases
# ------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("d", [64, 128])
def test_every_dtype_and_head_dim(env, dtype, d):
    O, B, W, LS = env
    wl = W.Workload(f"t_{dtype}_{d}", 11, b=3, h=5, d=d, dtype=dtype, prompt_lo=40, prompt_hi=333,
                    steps=12, w=7, sparsity_bp=7000, hh_frac=0.02, prefill_R=5)
    _say(f"dtype {dtype} d {d}")
    rep = LS.run_lockstep(wl)
    assert rep.steps == 12 and rep.evictions > 0


@pytest.mark.parametrize("w,sp,R", [(0, 5000, 1), (1, 9999, 33), (500, 8000, 64), (4, 0, 128),
                                    (16, 9000, 97)])
def test_window_and_sparsity_extremes(env, w, sp, R):
    # w = 0 (no window), sparsity ~1 (only the window survives), w larger than the
    # cache (nothing evicted), sparsity 0 (dense), prefill rows beyond the prompt start
    O, B, W, LS = env
    wl = W.Workload("t_ext", 12, b=4, h=3, d=128, dtype="f16", prompt_lo=1, prompt_hi=150,
                    steps=10, w=w, sparsity_bp=sp, hh_frac=0.02, prefill_R=R)
    _say(f"extremes w={w} sp={sp} R={R} lens={W.prompt_lengths(wl).tolist()}")
    rep = LS.run_lockstep(wl)
    assert rep.steps == 10


def test_workgroup_size_variants_and_large_cap(env):
    # pair counts that select the 1024-, 512- and 256-thread kernels; cap near the LDS limit
    O, B, W, LS = env
    for b, h, hi, steps in [(1, 2, 3000, 4), (8, 100, 300, 4), (16, 130, 200, 4)]:
        wl = W.Workload("t_wg", 13, b=b, h=h, d=128, dtype="bf16", prompt_lo=hi // 2, prompt_hi=hi,
                        steps=steps, w=9, sparsity_bp=8500, hh_frac=0.01)
        _say(f"workgroup variant b={b} h={h}")
        LS.run_lockstep(wl, seqs=list(range(min(b, 4))), heads=[0, h - 1])
    wl = W.Workload("t_cap", 14, b=1, h=2, d=64, dtype="f16", prompt_lo=12000, prompt_hi=12000,
                    steps=3, w=64, sparsity_bp=9000, hh_frac=0.001)
    assert wl.cap <= B.SWA_MAX_CAP
    _say("large cap")
    LS.run_lockstep(wl)


def test_decoding_from_an_empty_cache_in_every_form(env):
    # cache_len = 0: the first token attends to itself only; then the cache grows from nothing
    O, B, W, LS = env
    wl = W.Workload("t_empty", 45, b=3, h=2, d=128, dtype="f16", prompt_lo=1, prompt_hi=40, steps=12, w=2,
                    sparsity_bp=6000, hh_frac=0.02)
    for form in ("split", "fused", "unordered", "shared", "q8", "window"):
        prompt = W.make_prompt(wl, "cuda", slack="nan")
        prompt["cache_len"][1] = 0
        prompt["lengths"][1] = 0
        prompt["K"][1] = float("nan")
        prompt["V"][1] = float("nan")
        prompt["pos"][1] = -1
        _say(f"  empty cache, {form}")
        if form == "window":
            # run_lockstep_window builds its own prompt: emulate with a one-token prompt instead
            LS.run_lockstep_window(wl.replace(prompt_lo=1, prompt_hi=1), 4, seed_rows=False)
            continue
        rep = LS.run_lockstep(wl, prompt=prompt, fused=form != "split", unordered=form in ("unordered", "shared", "q8"),
                              head_shared=form == "shared", kv_int8=form == "q8")
        assert rep.steps == 12
    # the prefill calls leave an empty sequence alone
    params = B.make_params(wl.b, wl.h, wl.d, wl.cap, wl.w, wl.sparsity_bp, wl.torch_dtype)
    ws = torch.zeros((B.swa_workspace_bytes(params),), dtype=torch.uint8, device="cuda")
    prompt = W.make_prompt(wl, "cuda", slack="nan")
    prompt["cache_len"][1] = 0
    Q = torch.randn((wl.b, wl.h, wl.cap, wl.d), device="cuda").half()
    out = torch.full_like(Q, 7.0)
    score = torch.full((wl.b, wl.h, wl.cap), float("nan"), dtype=torch.float32, device="cuda")
    B.swa_prefill_attention(params, Q, prompt["K"], prompt["V"], prompt["cache_len"], out, 3, score, ws)
    assert torch.all(out[1] == 7.0) and torch.all(score[1] == 0.0)
    assert torch.isfinite(out[0, :, :int(prompt["cache_len"][0])].float()).all()


def test_exact_ties_go_to_the_lowest_slot(env):
    # identical keys => identical logits => bitwise-equal probabilities and scores
    O, B, W, LS = env
    b, h, d, cap, L, w = 2, 3, 128, 700, 600, 5
    params = B.make_params(b, h, d, cap, w, 6000, torch.float16)
    st = B.DecodeState(params, debug_probs=True)
    g = torch.Generator(device="cuda").manual_seed(5)
    key = torch.randn((d,), generator=g, device="cuda").half()
    st.K[:, :, :L] = key
    st.V[:, :, :L] = torch.randn((b, h, L, d), generator=g, device="cuda").half()
    st.cache_len.fill_(L)
    st.seq_len.fill_(L + 1)
    q = torch.randn((b, h, d), generator=g, device="cuda").half()
    kn = key.expand(b, h, d).contiguous()
    vn = torch.randn((b, h, d), generator=g, device="cuda").half()
    st.decode_step(q, kn, vn)
    keep, nl, ng = B.swa_budget(L + 1, L + 1, w, 6000)
    assert st.kept_cnt.tolist() == [keep] * b
    expect = list(range(ng)) + list(range(L + 1 - nl, L + 1))
    kept = st.kept_idx.cpu().numpy()
    for s in range(b):
        for hd in range(h):
            assert kept[s, hd, :keep].tolist() == expect
    p = st.probs.cpu().numpy()
    assert np.all(p[:, :, :L + 1] == p[:, :, :1])


def test_capacity_overflow_is_reported_and_nothing_is_written(env):
    O, B, W, LS = env
    b, h, d, cap = 3, 2, 64, 16
    params = B.make_params(b, h, d, cap, 2, 5000, torch.float32)
    st = B.DecodeState(params)
    st.K.normal_()
    st.V.normal_()
    st.cache_len.copy_(torch.tensor([5, 16, 15], dtype=torch.int32))   # sequence 1 is full
    st.seq_len.copy_(torch.tensor([6, 17, 16], dtype=torch.int32))
    K0, V0, s0 = st.K.clone(), st.V.clone(), st.score.clone()
    st.kept_cnt.fill_(-7)
    x = torch.randn((b, h, d), device="cuda")
    st.decode_step(x, x, x)
    assert st.check_status() == B.SWA_ERR_CAPACITY
    assert st.check_status() == 0                       # sticky bit is cleared by the read
    assert st.cache_len.tolist() == [6, 16, 16]
    assert st.kept_cnt[1].item() == -7
    assert torch.equal(st.K[1], K0[1]) and torch.equal(st.V[1], V0[1]) and torch.equal(st.score[1], s0[1])
    # a second step: arrival counters were reset, sequence 2 is now full as well
    st.seq_len += 1
    st.decode_step(x, x, x)
    assert st.cache_len.tolist() == [7, 16, 16]
    assert st.check_status() == B.SWA_ERR_CAPACITY


def test_compressed_cache_and_strict_window_edge_cases(env):
    O, B, W, LS = env
    # exact ties on a compressed cache: identical prompt keys give identical codes (flat channels
    # take the minimum range), so the tie rule decides every eviction
    wl = W.Workload("t_q8_ties", 42, b=2, h=3, d=128, dtype="f16", prompt_lo=40, prompt_hi=70,
                    steps=20, w=3, sparsity_bp=5000, hh_frac=0.02)
    prompt = W.make_prompt(wl, "cuda", slack="nan")
    for s_i, L in enumerate(prompt["lengths"]):
        prompt["K"][s_i, :, :L] = prompt["K"][s_i, :, :1].clone()
    rep = LS.run_lockstep(wl, prompt=prompt, fused=True, unordered=True, kv_int8=True)
    assert rep.evictions > 0
    # a full cache is skipped and reported by both new step entry points; nothing of it is written
    b, h, d, cap, R = 3, 2, 128, 32, 4
    for mode in ("q8", "window"):
        flags = B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED
        params = B.make_params(b, h, d, cap, 2, 5000, torch.float16, flags=flags)
        st = B.DecodeState(params)
        st.K.normal_()
        st.V.normal_()
        lens = torch.tensor([5, 32, 31], dtype=torch.int32, device="cuda")   # sequence 1 is full
        st.cache_len.copy_(lens)
        st.seq_len.copy_(lens + 1)
        st.pos[:] = torch.arange(cap, device="cuda", dtype=torch.int32)
        x = torch.randn((b, h, d), device="cuda").half()
        ring = torch.rand((b, h, R, cap), device="cuda")
        if mode == "q8":
            st.quantize()
        K0, V0, s0, r0 = st.K.clone(), st.V.clone(), st.score.clone(), ring.clone()
        if mode == "q8":
            st.decode_compact_step(x, x, x)
        else:
            B.swa_decode_step_window(st.params, x, x, x, st.K, st.V, ring, R, 1, st.score, st.pos, st.cache_len,
                                     st.seq_len, st.kept_idx, st.kept_cnt, st.out, None, st.workspace)
            st.cache_len, st.kept_cnt = st.kept_cnt, st.cache_len
        assert st.check_status() == B.SWA_ERR_CAPACITY
        keep0 = B.swa_budget(6, 6, 2, 5000)[0]
        keep2 = B.swa_budget(32, 32, 2, 5000)[0]
        assert st.cache_len.tolist() == [keep0, 32, keep2], mode
        assert torch.equal(st.K[1], K0[1]) and torch.equal(st.V[1], V0[1]) and torch.equal(st.score[1], s0[1])
        assert torch.equal(ring[1], r0[1])
    # both paths give the same bits on a second run
    wl = W.Workload("t_det2", 43, b=3, h=4, d=128, dtype="f16", prompt_lo=100, prompt_hi=300,
                    steps=6, w=8, sparsity_bp=8000, hh_frac=0.02)
    for mode in ("q8", "window"):
        results = []
        for _ in range(2):
            prompt = W.make_prompt(wl, "cuda", slack="nan")
            st = LS.new_state(wl, prompt, debug_probs=False)
            st.params.flags = B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED
            st.score.zero_()
            ring = torch.zeros((wl.b, wl.h, 8, wl.cap), device="cuda")
            if mode == "q8":
                st.quantize()
            outs = []
            for t in range(wl.steps):
                q, kn, vn = W.make_step(wl, t, prompt["mu"])
                st.seq_len += 1
                if mode == "q8":
                    st.decode_compact_step(q, kn, vn)
                else:
                    B.swa_decode_step_window(st.params, q, kn, vn, st.K, st.V, ring, 8, t % 8, st.score, st.pos,
                                             st.cache_len, st.seq_len, st.kept_idx, st.kept_cnt, st.out, None,
                                             st.workspace)
                    st.cache_len, st.kept_cnt = st.kept_cnt, st.cache_len
                outs.append(st.out.clone())
            assert not torch.isnan(torch.stack(outs)).any()
            L = st.cache_len.tolist()
            results.append((torch.stack(outs), [st.score[s, :, :L[s]].clone() for s in range(wl.b)],
                            [st.pos[s, :, :L[s]].clone() for s in range(wl.b)], L))
        a, b_ = results
        assert torch.equal(a[0], b_[0]) and a[3] == b_[3], mode
        for s in range(wl.b):
            assert torch.equal(a[1][s], b_[1][s]) and torch.equal(a[2][s], b_[2][s]), mode


def test_randomised_small_workloads_in_every_form(env):
    # seeded sweep: random shapes, windows, budgets that change from step to step (so the number of
    # evictions per step varies between none and most of the cache), every way of issuing the step
    O, B, W, LS = env
    rng = np.random.default_rng(20240317)
    forms = ["split", "fused", "unordered", "shared", "q8", "q8_fused", "window", "lazy"]
    for case in range(24):
        form = forms[case % len(forms)]
        d = int(rng.choice([64, 128]))
        dtype = "f16" if form.startswith("q8") else str(rng.choice(["f32", "f16", "bf16"]))
        hi = int(rng.integers(3, 420))
        lo = int(rng.integers(1, hi + 1))
        w = int(rng.choice([0, 1, 5, 17, B.SWA_W_EVEN_SPLIT]))
        steps = int(rng.integers(6, 20))
        sched = rng.integers(0, 9500, size=steps)
        sched[rng.integers(0, steps)] = 0                       # at least one step that keeps everything
        wl = W.Workload(f"t_rand_{case}", 50 + case, b=int(rng.integers(1, 4)), h=int(rng.integers(1, 5)), d=d,
                        dtype=dtype, prompt_lo=lo, prompt_hi=hi, steps=steps, w=w, sparsity_bp=int(sched[0]),
                        hh_frac=0.03, prefill_R=int(rng.choice([0, 0, 3, 9])))
        _say(f"  case {case}: {form} {dtype} d={d} prompts {lo}..{hi} w={w} steps={steps}")
        sp = lambda t, sched=sched: int(sched[t])
        if form == "window":
            LS.run_lockstep_window(wl.replace(prefill_R=0), int(rng.integers(1, 20)), sparsity_of_step=sp,
                                   seed_rows=bool(rng.integers(0, 2)))
        elif form == "lazy":
            LS.run_lockstep(wl, compact_every=int(rng.integers(0, 5)), sparsity_of_step=sp)
        else:
            LS.run_lockstep(wl, fused=form in ("fused", "unordered", "shared", "q8_fused", "q8"),
                            unordered=form in ("unordered", "shared", "q8"), head_shared=form == "shared",
                            kv_int8=form.startswith("q8"), sparsity_of_step=sp)


@pytest.mark.parametrize("form", ["two-call", "unordered", "q8", "window"])
def test_a_trajectory_resumed_from_a_saved_state_continues_bit_for_bit(env, form):
    # stop after a few steps, copy the state tensors the header names (cache, importance, positions,
    # lengths; the compression parameters; the ring) to the host, rebuild them in fresh device buffers
    # whose unused slots hold NaN / garbage, and go on: every later output and the final state must
    # equal the uninterrupted run's bits.  Nothing else (workspace, kept list, LDS) carries state.
    O, B, W, LS = env
    wl = W.Workload("t_resume", 47, b=3, h=5, d=128, dtype="f16", prompt_lo=90, prompt_hi=260, steps=12, w=8,
                    sparsity_bp=7500, hh_frac=0.02)
    fused = form != "two-call"
    flags = (B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED) if fused else 0
    R = 6
    prompt = W.make_prompt(wl, "cuda")
    inputs = [W.make_step(wl, t, prompt["mu"]) for t in range(wl.steps)]
    seq_lens = [(prompt["cache_len"] + (t + 1)).to(torch.int32) for t in range(wl.steps)]

    def fresh_state(src=None):
        params = B.make_params(wl.b, wl.h, wl.d, wl.cap, wl.w, wl.sparsity_bp, wl.torch_dtype, flags=flags)
        st = B.DecodeState(params, debug_probs=False)
        ring = torch.zeros((wl.b, wl.h, R, wl.cap), device="cuda")
        if src is None:
            st.K.copy_(prompt["K"])
            st.V.copy_(prompt["V"])
            st.pos.copy_(prompt["pos"])
            st.cache_len.copy_(prompt["cache_len"])
            if form == "q8":
                st.quantize()
        else:
            saved, L = src
            if form == "q8":
                st.quantize()                       # allocates the code tensors and the parameter array
                st.qparams.copy_(saved["qparams"].cuda())
            st.K.view(torch.uint8).fill_(0xFF)      # NaN in fp16, code 255: unused slots must never be read
            st.V.view(torch.uint8).fill_(0xFF)
            st.score.fill_(float("nan"))
            st.pos.fill_(-7)
            ring.fill_(float("nan"))
            for s_i in range(wl.b):
                n = L[s_i]
                st.K[s_i, :, :n].copy_(saved["K"][s_i, :, :n].cuda())
                st.V[s_i, :, :n].copy_(saved["V"][s_i, :, :n].cuda())
                st.score[s_i, :, :n].copy_(saved["score"][s_i, :, :n].cuda())
                st.pos[s_i, :, :n].copy_(saved["pos"][s_i, :, :n].cuda())
                ring[s_i, :, :, :n].copy_(saved["ring"][s_i, :, :, :n].cuda())
            st.cache_len.copy_(torch.tensor(L, dtype=torch.int32))
        return st, ring

    def run(st, ring, t0, t1, outs):
        cur, nxt = st.cache_len, st.kept_cnt
        for t in range(t0, t1):
            q, kn, vn = inputs[t]
            kidx = None if fused else st.kept_idx
            if form == "window":
                B.swa_decode_step_window(st.params, q, kn, vn, st.K, st.V, ring, R, t % R, st.score, st.pos, cur,
                                         seq_lens[t], kidx, nxt, st.out, None, st.workspace)
            elif form == "q8":
                B.swa_decode_step_q8(st.params, q, kn, vn, st.K, st.V, st.qparams, st.score, st.pos, cur, seq_lens[t],
                                     kidx, nxt, st.out, None, st.workspace)
            else:
                B.swa_decode_step(st.params, q, kn, vn, st.K, st.V, st.score, st.pos, cur, seq_lens[t], kidx, nxt,
                                  st.out, None, st.workspace)
            outs.append(st.out.clone())
            if fused:
                cur, nxt = nxt, cur
            else:
                B.swa_compact_kv(st.params, st.K, st.V, st.score, st.pos, st.kept_idx, st.kept_cnt, st.cache_len,
                                 st.workspace)
        return cur

    def valid(st, ring, lens_t):
        L = lens_t.tolist()
        host = lambda x: x.cpu()
        return ({"K": host(st.K), "V": host(st.V), "score": host(st.score), "pos": host(st.pos), "ring": host(ring),
                 "qparams": host(st.qparams) if form == "q8" else None}, L)

    def same(a, b_, L):
        for name in ("K", "V", "score", "pos"):
            for s_i in range(wl.b):
                x, y = a[name][s_i, :, :L[s_i]], b_[name][s_i, :, :L[s_i]]
                assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), f"{form}: {name} of sequence {s_i}"
        if form == "window":
            for s_i in range(wl.b):
                assert torch.equal(a["ring"][s_i, :, :, :L[s_i]], b_["ring"][s_i, :, :, :L[s_i]]), f"{form}: ring"

    stop = 5
    st, ring = fresh_state()
    outs_a = []
    lens_a = run(st, ring, 0, wl.steps, outs_a)
    final_a = valid(st, ring, lens_a)
    st2, ring2 = fresh_state()
    outs_b = []
    mid = valid(st2, ring2, run(st2, ring2, 0, stop, outs_b))
    del st2, ring2
    st3, ring3 = fresh_state(mid)
    lens_c = run(st3, ring3, stop, wl.steps, outs_b)
    final_c = valid(st3, ring3, lens_c)
    assert final_a[1] == final_c[1], f"{form}: lengths {final_a[1]} vs {final_c[1]}"
    assert len(outs_a) == len(outs_b) == wl.steps
    for t in range(wl.steps):
        assert torch.equal(outs_a[t], outs_b[t]), f"{form}: output of step {t}"
    same(final_a[0], final_c[0], final_a[1])
    for x in (st, st3):
        assert x.check_status() == 0


@pytest.mark.parametrize("form", ["unordered", "fused", "shared", "q8", "window"])
def test_hip_graph_replays_equal_the_eager_run(env, form):
    # bench.py times HIP-graph replays: a captured trajectory, replayed several times with the
    # state restored eagerly in between, must give the eager run's bits every time
    O, B, W, LS = env
    wl = W.Workload("t_graph", 46, b=4, h=6, d=128, dtype="f16", prompt_lo=100, prompt_hi=300, steps=8, w=8,
                    sparsity_bp=8000, hh_frac=0.02)
    flags = {"unordered": B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED, "fused": B.SWA_FUSE_COMPACTION,
             "shared": B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED | B.SWA_HEAD_SHARED,
             "q8": B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED, "window": B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED}[form]
    R = 8
    prompt = W.make_prompt(wl, "cuda")
    inputs = [W.make_step(wl, t, prompt["mu"]) for t in range(wl.steps)]
    seq_lens = [(prompt["cache_len"] + (t + 1)).to(torch.int32) for t in range(wl.steps)]
    params = B.make_params(wl.b, wl.h, wl.d, wl.cap, wl.w, wl.sparsity_bp, wl.torch_dtype, flags=flags)
    st = B.DecodeState(params, debug_probs=False)
    ring = torch.zeros((wl.b, wl.h, R, wl.cap), device="cuda")
    if form == "q8":
        st.K.copy_(prompt["K"])
        st.V.copy_(prompt["V"])
        st.cache_len.copy_(prompt["cache_len"])
        st.quantize()
        prompt = dict(prompt, K=st.K.clone(), V=st.V.clone())
    names = ["K", "V", "score", "pos", "cache_len", "kept_cnt"]

    def reset():
        st.K.copy_(prompt["K"])
        st.V.copy_(prompt["V"])
        st.pos.copy_(prompt["pos"])
        st.score.zero_()
        ring.zero_()
        lens["a"].copy_(prompt["cache_len"])
        lens["b"].zero_()

    lens = {"a": st.cache_len, "b": st.kept_cnt}
    outs = torch.zeros((wl.steps, wl.b, wl.h, wl.d), dtype=torch.float16, device="cuda")

    def trajectory():
        cur, nxt = lens["a"], lens["b"]
        for t in range(wl.steps):
            q, kn, vn = inputs[t]
            if form == "window":
                B.swa_decode_step_window(st.params, q, kn, vn, st.K, st.V, ring, R, t % R, st.score, st.pos, cur,
                                         seq_lens[t], None, nxt, st.out, None, st.workspace)
            elif form == "q8":
                B.swa_decode_step_q8(st.params, q, kn, vn, st.K, st.V, st.qparams, st.score, st.pos, cur,
                                     seq_lens[t], None, nxt, st.out, None, st.workspace)
            else:
                B.swa_decode_step(st.params, q, kn, vn, st.K, st.V, st.score, st.pos, cur, seq_lens[t], None, nxt,
                                  st.out, None, st.workspace)
            outs[t].copy_(st.out)
            cur, nxt = nxt, cur
        return cur                                    # the tensor that holds the final lengths

    def snapshot(final_len):
        L = final_len.tolist()
        return (outs.clone(), [st.K[s, :, :L[s]].clone() for s in range(wl.b)],
                [st.score[s, :, :L[s]].clone() for s in range(wl.b)],
                [st.pos[s, :, :L[s]].clone() for s in range(wl.b)], L,
                [ring[s, :, :, :L[s]].clone() for s in range(wl.b)])

    reset()
    final = trajectory()                              # eager reference (also warms every kernel up)
    torch.cuda.synchronize()
    ref = snapshot(final)
    assert all(0 < x < wl.cap for x in ref[4]) and not torch.isnan(ref[0].float()).any()
    reset()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        final_g = trajectory()
    assert final_g is final
    for rep in range(3):
        reset()
        outs.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = snapshot(final)
        assert torch.equal(got[0], ref[0]), f"{form}: outputs of replay {rep}"
        assert got[4] == ref[4]
        for k in (1, 2, 3, 5):
            for s_i in range(wl.b):
                assert torch.equal(got[k][s_i], ref[k][s_i]), f"{form}: state {k} of replay {rep}"
    assert st.check_status() == 0


def test_a_few_evictions_at_once_give_the_same_bits_on_every_run(env):
    # 2..8 evictions in one step take the subtractive output, which adds the evicted rows up in list
    # order: the list must come out in a fixed order (ascending slots), or the output's last bits depend
    # on which wave wrote first.  Four states step the same trajectory; a budget that tightens by a few
    # tokens every other step keeps the step on that path.
    O, B, W, LS = env
    for dtype, flags in [("f32", B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED), ("f16", B.SWA_FUSE_COMPACTION), ("bf16", 0)]:
        wl = W.Workload(f"t_det_few_{dtype}", 19, b=4, h=5, d=128, dtype=dtype, prompt_lo=73, prompt_hi=301, steps=14, w=5,
                        sparsity_bp=3000, hh_frac=0.02)
        sched = [3000, 3100, 3100, 3250, 3250, 3400, 3400, 3600, 3600, 3800, 3800, 4000, 4000, 4100]
        prompt = W.make_prompt(wl, "cuda", slack="nan")
        inputs = [W.make_step(wl, t, prompt["mu"]) for t in range(wl.steps)]
        runs, few = [], 0
        for rep in range(4):
            st = LS.new_state(wl, dict(prompt, K=prompt["K"].clone(), V=prompt["V"].clone(), pos=prompt["pos"].clone()),
                              debug_probs=(rep % 2 == 0))
            st.score.zero_()
            st.params.flags = flags
            outs = []
            for t in range(wl.steps):
                st.params.sparsity_bp = sched[t]
                q, kn, vn = inputs[t]
                st.seq_len += 1
                before = st.cache_len.clone()
                if flags:
                    st.decode_compact_step(q, kn, vn, want_idx=(rep < 2))
                else:
                    st.decode_step(q, kn, vn)
                    st.compact()
                if rep == 0:
                    ev = (before + 1 - st.cache_len)
                    few += int(((ev >= 2) & (ev <= 8)).sum())
                outs.append(st.out.clone())
            assert st.check_status() == 0
            runs.append((torch.stack(outs), st.cache_len.clone(), st.score.clone()))
        assert few >= 8, "the schedule must produce steps with 2..8 evictions"
        for r in runs[1:]:
            assert torch.equal(r[1], runs[0][1])
            assert torch.equal(r[0].view(torch.uint8), runs[0][0].view(torch.uint8)), f"{dtype}: outputs differ between runs"


def test_slack_slots_are_never_touched_and_runs_are_deterministic(env):
    O, B, W, LS = env
    wl = W.Workload("t_det", 15, b=4, h=6, d=128, dtype="f16", prompt_lo=100, prompt_hi=400,
                    steps=6, w=8, sparsity_bp=8000, hh_frac=0.02, prefill_R=16)
    results = []
    for rep in range(2):
        prompt = W.make_prompt(wl, "cuda", slack="nan")
        st = LS.new_state(wl, prompt, debug_probs=False)
        st.score.fill_(float("nan"))                    # prefill must overwrite every slot
        st.prefill_scores(W.make_q_tail(wl, prompt["mu"], wl.prefill_R))
        outs = []
        for t in range(wl.steps):
            q, kn, vn = W.make_step(wl, t, prompt["mu"])
            st.seq_len += 1
            st.decode_step(q, kn, vn)
            outs.append(st.out.clone())
            st.compact()
        lens = st.cache_len.tolist()
        for s, L in enumerate(lens):
            assert torch.isnan(st.K[s, :, wl.prompt_hi + wl.steps:]).all()   # beyond any append
        assert not torch.isnan(torch.stack(outs)).any()
        results.append((torch.stack(outs), st.score.clone(), st.kept_idx.clone(), st.K.clone(), lens))
    a, b_ = results
    assert torch.equal(a[0], b_[0]) and a[4] == b_[4]
    for s, L in enumerate(a[4]):
        assert torch.equal(a[1][s, :, :L], b_[1][s, :, :L])
        assert torch.equal(a[2][s, :, :L], b_[2][s, :, :L])
        assert torch.equal(a[3][s, :, :L], b_[3][s, :, :L])


@pytest.mark.parametrize("dtype,d,logits", [("f16", 128, "random"), ("bf16", 128, "random"), ("f16", 64, "random"),
                                            ("bf16", 64, "random"), ("f32", 128, "random"), ("f32", 64, "random"),
                                            ("f16", 128, "rising"), ("bf16", 128, "rising"), ("f32", 64, "rising")])
def test_prefill_attention_matches_the_oracle(env, dtype, d, logits):
    # dense causal attention over the prompt (Eq. 1-2) on MFMA, plus the importance seed.
    # Tolerance from the arithmetic: the weights are rounded once to the cache dtype before the
    # second product (unit roundoff u = 2^-11 fp16, 2^-8 bf16), values are exact, sums are fp32,
    # the output is rounded once: |delta_c| <= 1.5 u (sum_j p_j |v_jc| + |out_c|) + 1e-5.
    # (fp32: nothing is rounded below fp32; u = 2^-20 covers the fp32 sums over up to 417 keys and
    # the hardware exponential.)
    O, B, W, LS = env
    u = {"f16": 2.0 ** -11, "bf16": 2.0 ** -8, "f32": 2.0 ** -20}[dtype]
    lens = [1, 31, 32, 33, 127, 128, 129, 300, 417]
    wl = W.Workload(f"t_pf_{dtype}_{d}", 44, b=len(lens), h=2, d=d, dtype=dtype, prompt_lo=1, prompt_hi=417,
                    steps=2, w=4, sparsity_bp=8000, hh_frac=0.02)
    prompt = W.make_prompt(wl, "cuda", slack="nan")
    g = torch.Generator(device="cuda").manual_seed(77)
    # "rising": every query's logits grow with the key position, by about 40 powers of two over the longest
    # prompt and in steps of every size, so the running maximum of the streaming softmax moves at every tile
    axis = torch.nn.functional.normalize(torch.randn((wl.h, 1, d), generator=g, device="cuda"), dim=-1)
    for s_i, L in enumerate(lens):           # fixed lengths that straddle the tile and block sizes
        k = torch.randn((wl.h, L, d), generator=g, device="cuda")
        v = torch.randn((wl.h, L, d), generator=g, device="cuda")
        if logits == "rising":
            ramp = torch.arange(L, device="cuda", dtype=torch.float32) / 417.0
            k = 0.25 * k + (40.0 * math.log(2.0) / (4.0 * wl.scale)) * ramp[None, :, None] * axis
        prompt["K"][s_i] = float("nan")
        prompt["V"][s_i] = float("nan")
        prompt["K"][s_i, :, :L] = k.to(wl.torch_dtype)
        prompt["V"][s_i, :, :L] = v.to(wl.torch_dtype)
    cache_len = torch.tensor(lens, dtype=torch.int32, device="cuda")
    Q = torch.full((wl.b, wl.h, wl.cap, d), float("nan"), dtype=wl.torch_dtype, device="cuda")
    for s_i, L in enumerate(lens):
        qf = 1.5 * torch.randn((wl.h, L, d), generator=g, device="cuda")
        if logits == "rising":
            qf = 0.25 * qf + 4.0 * axis
        Q[s_i, :, :L] = qf.to(wl.torch_dtype)
    out = torch.full_like(Q, 7.0)
    R = 5
    score = torch.full((wl.b, wl.h, wl.cap), float("nan"), dtype=torch.float32, device="cuda")
    params = B.make_params(wl.b, wl.h, d, wl.cap, wl.w, wl.sparsity_bp, wl.torch_dtype)
    ws = torch.zeros((B.swa_workspace_bytes(params),), dtype=torch.uint8, device="cuda")
    B.swa_prefill_attention(params, Q, prompt["K"], prompt["V"], cache_len, out, R, score, ws)
    torch.cuda.synchronize()
    Kn, Vn, Qn = (np.nan_to_num(x.double().cpu().numpy(), nan=0.0) for x in (prompt["K"], prompt["V"], Q))
    ln = np.array(lens, dtype=np.int32)
    ref = O.prefill_attention(Qn, Kn, Vn, ln, wl.scale)
    mag = O.prefill_attention(Qn, Kn, np.abs(Vn), ln, wl.scale)
    og = out.double().cpu().numpy()
    for s_i, L in enumerate(lens):
        assert np.all(og[s_i, :, L:] == 7.0), "rows past the prompt must not be written"
        err = np.abs(og[s_i, :, :L] - ref[s_i, :, :L])
        bound = 1.5 * u * (mag[s_i, :, :L] + np.abs(ref[s_i, :, :L])) + 1e-5
        assert np.all(np.isfinite(og[s_i, :, :L]))
        assert np.all(err <= bound), f"len {L}: max excess {np.max(err - bound):.3e}"
    # the seed equals the seed routine fed with the last R query rows
    q_tail = np.zeros((wl.b, wl.h, R, d))
    for s_i, L in enumerate(lens):
        for r in range(R):
            if L - R + r >= 0:
                q_tail[s_i, :, r] = Qn[s_i, :, L - R + r]
    S_ref = O.prefill_scores(q_tail, Kn, ln, wl.scale)
    S_g = score.double().cpu().numpy()
    np.testing.assert_allclose(S_g, S_ref, rtol=1e-5, atol=1e-12)
    # R = 0: attention only
    out2 = torch.full_like(Q, 7.0)
    B.swa_prefill_attention(params, Q, prompt["K"], prompt["V"], cache_len, out2, 0, None, ws)
    assert torch.equal(out2, out)


def test_prefill_scores_edge_shapes(env):
    O, B, W, LS = env
    for dtype, d in [("f16", 128), ("bf16", 64), ("f32", 128)]:
        for R in [1, 31, 32, 64, 100, 128]:
            wl = W.Workload("t_pf", 16, b=5, h=2, d=d, dtype=dtype, prompt_lo=1, prompt_hi=260,
                            steps=1, w=4, sparsity_bp=5000, hh_frac=0.02)
            prompt = W.make_prompt(wl, "cuda", slack="nan")
            prompt["cache_len"][0] = 0                    # an empty cache
            st = LS.new_state(wl, prompt)
            st.score.fill_(float("nan"))
            qt = W.make_q_tail(wl, prompt["mu"], R)
            st.prefill_scores(qt)
            lens = st.cache_len.cpu().numpy()
            S_ref = O.prefill_scores(LS._np64(qt), np.nan_to_num(LS._np64(st.K)), lens, wl.scale)
            S_gpu = LS._np64(st.score)
            np.testing.assert_allclose(S_gpu, S_ref, rtol=1e-5, atol=1e-12,
                                       err_msg=f"{dtype} d={d} R={R} lens={lens.tolist()}")
            want = np.broadcast_to(np.minimum(R, lens[1:])[:, None].astype(np.float64), (4, 2))
            np.testing.assert_allclose(S_gpu.sum(-1)[1:], want, rtol=1e-5)


def test_full_size_sampled_single_step_matches_dense_definition(env):
    # At the largest shape, one step with sparsity 0: every sampled output must equal
    # plain dense attention (Eq. 1-2) computed by the oracle pair by pair.
    O, B, W, LS = env
    wl = W.CONFIGS["c5_llama7b_sp80"].replace(sparsity_bp=0, steps=1)
    rep = LS.run_lockstep(wl, seqs=[3, 77, 200], heads=[1, 30], slack="zero")
    assert rep.evictions == 0
    torch.cuda.empty_cache()
