"""swa_decode_step_static (the entry point that allocates nothing and takes no workspace) against
swa_decode_step on the same inputs: same kernels, so every output must agree bit for bit.  Each
case makes two calls in a row on the shared static scratch, the second with a smaller input."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' on CPU-only hosts)")
    from paper_2403_17312_amd import binding as B
    from paper_2403_17312_amd import workload as W
    B.lib()
    return B, W


def _twin_states(B, W, wl, flags):
    """Two identical device states after the prompt of workload wl."""
    prompt = W.make_prompt(wl, "cuda", slack="nan")
    states = []
    for _ in range(2):
        params = B.make_params(wl.b, wl.h, wl.d, wl.cap, wl.w, wl.sparsity_bp, wl.torch_dtype, flags=flags)
        st = B.DecodeState(params, debug_probs=True)
        st.K.copy_(prompt["K"])
        st.V.copy_(prompt["V"])
        st.pos.copy_(prompt["pos"])
        st.cache_len.copy_(prompt["cache_len"])
        st.seq_len.copy_(prompt["cache_len"])
        if flags & B.SWA_HEAD_SHARED:
            st.workspace = torch.zeros((B.swa_workspace_bytes(params),), dtype=torch.uint8, device="cuda")
            B.swa_workspace_init(params, st.workspace)
        states.append(st)
    return prompt, states


def _trajectory(B, W, wl, flags, steps):
    print(f"  static vs workspace: {wl.name} b={wl.b} h={wl.h} cap={wl.cap} flags={flags}", flush=True)
    prompt, (ref, sta) = _twin_states(B, W, wl, flags)
    fused = bool(flags & B.SWA_FUSE_COMPACTION)
    for t in range(steps):
        q, kn, vn = W.make_step(wl, t, prompt["mu"])
        for st in (ref, sta):
            st.seq_len += 1
        B.swa_decode_step(ref.params, q, kn, vn, ref.K, ref.V, ref.score, ref.pos, ref.cache_len, ref.seq_len,
                          ref.kept_idx, ref.kept_cnt, ref.out, ref.probs, ref.workspace)
        B.swa_decode_step_static(sta.params, q, kn, vn, sta.K, sta.V, sta.score, sta.pos, sta.cache_len,
                                 sta.seq_len, sta.kept_idx, sta.kept_cnt, sta.out, sta.probs)
        if fused:
            for st in (ref, sta):
                st.cache_len, st.kept_cnt = st.kept_cnt, st.cache_len
        else:
            for st in (ref, sta):
                st.compact()
        torch.cuda.synchronize()
        assert torch.equal(ref.cache_len, sta.cache_len), f"step {t}: cache_len"
        assert torch.equal(ref.kept_cnt, sta.kept_cnt), f"step {t}: kept_cnt"
        assert torch.equal(ref.out.view(torch.int16 if wl.elem_bytes == 2 else torch.int32),
                           sta.out.view(torch.int16 if wl.elem_bytes == 2 else torch.int32)), f"step {t}: out"
        lens = ref.cache_len.tolist()
        assert all(0 < L <= wl.cap for L in lens)
        for s, L in enumerate(lens):
            for name in ("K", "V", "score", "pos", "kept_idx", "probs"):
                a, b_ = getattr(ref, name)[s, :, :L], getattr(sta, name)[s, :, :L]
                assert torch.equal(a, b_), f"step {t} seq {s}: {name}"
            assert not torch.isnan(ref.out[s].float()).any()
    assert ref.check_status() == 0
    assert B.swa_check_status(sta.params, None) == 0


def test_static_entry_point_equals_the_workspace_one_two_calls_in_a_row(env):
    B, W = env
    B.swa_prepare()
    big = W.Workload("t_static_big", 61, b=6, h=5, d=128, dtype="f16", prompt_lo=40, prompt_hi=300, steps=4, w=6,
                     sparsity_bp=7000, hh_frac=0.02)
    small = W.Workload("t_static_small", 62, b=2, h=3, d=64, dtype="bf16", prompt_lo=5, prompt_hi=90, steps=4,
                       w=3, sparsity_bp=6000, hh_frac=0.02)
    shared = B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED | B.SWA_HEAD_SHARED
    for flags in (0, shared, B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED, B.SWA_FUSE_COMPACTION):
        _trajectory(B, W, big, flags, big.steps)        # leaves its counters and slabs in the scratch
        _trajectory(B, W, small, flags, small.steps)    # a smaller input right after it
    # once more in the two-call form, whose arrival counters the scratch carries from call to call
    _trajectory(B, W, big, 0, 2)
    _trajectory(B, W, small, 0, 2)


def test_static_entry_point_reports_a_full_cache_and_refuses_what_does_not_fit(env):
    B, W = env
    b, h, d, cap = 3, 2, 64, 16
    params = B.make_params(b, h, d, cap, 2, 5000, torch.float32)
    st = B.DecodeState(params)
    st.K.normal_()
    st.V.normal_()
    st.cache_len.copy_(torch.tensor([5, 16, 15], dtype=torch.int32))   # sequence 1 is full
    st.seq_len.copy_(torch.tensor([6, 17, 16], dtype=torch.int32))
    K0 = st.K.clone()
    x = torch.randn((b, h, d), device="cuda")
    B.swa_decode_step_static(params, x, x, x, st.K, st.V, st.score, st.pos, st.cache_len, st.seq_len, st.kept_idx,
                             st.kept_cnt, st.out, None)
    assert B.swa_check_status(params, None) == B.SWA_ERR_CAPACITY
    assert B.swa_check_status(params, None) == 0                      # cleared by the read
    assert st.cache_len.tolist() == [6, 16, 16] and torch.equal(st.K[1], K0[1])
    # a head-shared step whose slabs exceed the static scratch is refused on the host
    flags = B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED | B.SWA_HEAD_SHARED
    too_big = B.make_params(64, 40, 128, 1152, 32, 8000, torch.float16, flags=flags)
    assert B.swa_workspace_bytes(too_big) > B.SWA_STATIC_SCRATCH_BYTES
    with pytest.raises(B.SwaError) as e:
        B.swa_decode_step_static(too_big, x, x, x, st.K, st.V, st.score, st.pos, st.cache_len, st.seq_len,
                                 st.kept_idx, st.kept_cnt, st.out, None)
    assert e.value.code == B.SWA_ERR_CAPACITY
