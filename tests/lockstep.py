"""Lock-step parity harness: HIP path vs the fp64 oracle, with state adoption.

Selection is discontinuous: an fp32 GPU and an independent fp64 oracle order
near-tied importance scores differently, and one flipped eviction changes the
cache for good.  So before every step the oracle's importance vector is
overwritten with the GPU's fp32 values of the previous step (K, V, pos and the
lengths are identical by construction: compaction is a pure copy and is itself
checked bit-exactly).  Per step, on the sampled (sequence, head) pairs:
  (i)   attention weights and new importance, GPU vs oracle from the adopted
        state: |delta| <= 1e-5 * |oracle| (+ 1e-12);
  (ii)  kept indices: the oracle's selection routine applied to the GPU's own
        fp32 importance values must equal kept_idx / kept_cnt bit-exactly; the
        oracle's selection from its fp64 values may differ only in tokens whose
        fp64 importance is within 2e-5 relative of the cutoff (counted);
  (iii) output vs the oracle's sparse attention over that kept set, elementwise
        |delta| <= atol + rel_elem * |oracle| and per-pair relative L2 error <= rtol:
        fp16 2e-3, 0, 1e-2 (the stated bar); fp32 2e-5, 0, 1e-4; bf16 5e-4, 2^-8,
        1e-2 (the output is rounded once to bf16, whose half-ulp is up to 2^-8
        relative, so a pure absolute bar of 2e-3 cannot hold for |out| > 0.5);
  (iv)  after compaction: K, V, importance, pos, cache_len equal the oracle's
        stable gather bit-exactly.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Sequence

import numpy as np
import torch

from oracle import swa_oracle as O
from paper_2403_17312_amd import binding as B
from paper_2403_17312_amd import workload as W

TOL = {"f16": (2e-3, 0.0, 1e-2), "bf16": (5e-4, 2.0 ** -8, 1e-2), "f32": (2e-5, 0.0, 1e-4)}


@dataclasses.dataclass
class Report:
    steps: int = 0
    pairs: int = 0
    max_prob_rel: float = 0.0
    max_score_rel: float = 0.0
    max_out_abs: float = 0.0
    max_out_rel: float = 0.0
    near_tie_flips: int = 0
    evictions: int = 0
    moved_rows: int = 0
    out_elems: int = 0
    out_over_2e3: int = 0        # outputs whose |delta| exceeds the 2e-3 bar stated for fp16 (bf16 runs report it)
    twin_steps: int = 0          # steps on which the twin state (no debug outputs) was compared bit for bit


def _np64(t: torch.Tensor) -> np.ndarray:
    # widened on the device the tensor lives on (exact), then copied to the host
    return t.detach().to(torch.float64).to("cpu").numpy().copy()


def _same_bits(a: torch.Tensor, b: torch.Tensor) -> bool:
    """Bitwise equality (NaN-filled slack compares equal to itself)."""
    it = {1: torch.uint8, 2: torch.int16, 4: torch.int32}[a.element_size()]
    return a.dtype == b.dtype and torch.equal(a.view(it), b.view(it))


def _sub(t: torch.Tensor, seqs, heads) -> torch.Tensor:
    return t[seqs][:, heads]


def new_state(wl: W.Workload, prompt: dict, debug_probs: bool = True) -> B.DecodeState:
    params = B.make_params(wl.b, wl.h, wl.d, wl.cap, wl.w, wl.sparsity_bp, wl.torch_dtype)
    st = B.DecodeState(params, device=prompt["K"].device, debug_probs=debug_probs)
    st.K, st.V, st.pos = prompt["K"], prompt["V"], prompt["pos"]
    st.cache_len.copy_(prompt["cache_len"])
    st.seq_len.copy_(prompt["cache_len"])
    return st


def check_out(out_gpu: np.ndarray, out_ref: np.ndarray, dtype: str, what: str, rep=None):
    atol, rel_elem, rtol = TOL[dtype]
    err = np.abs(out_gpu - out_ref)
    assert np.all(np.isfinite(out_gpu)), f"{what}: non-finite output at {np.argwhere(~np.isfinite(out_gpu))[:8].tolist()}"
    rel = np.linalg.norm(out_gpu - out_ref, axis=-1) / np.maximum(np.linalg.norm(out_ref, axis=-1), 1e-30)
    excess = err - (atol + rel_elem * np.abs(out_ref))
    assert excess.max() <= 0, f"{what}: max abs {err.max():.3e} exceeds {atol} + {rel_elem:.2e}*|ref|"
    assert rel.max() <= rtol, f"{what}: rel L2 {rel.max():.3e} > {rtol}"
    if rep is not None:
        rep.out_elems += int(err.size)
        rep.out_over_2e3 += int(np.count_nonzero(err > 2e-3))
    return float(err.max()), float(rel.max())


def run_lockstep(wl: W.Workload, device="cuda", steps: Optional[int] = None,
                 seqs: Optional[Sequence[int]] = None, heads: Optional[Sequence[int]] = None,
                 compact_every: int = 1, slack: str = "nan", check_steps=None,
                 prompt: Optional[dict] = None, verbose: bool = False,
                 use_len_bound: bool = False, fused: bool = False, unordered: bool = False,
                 sparsity_of_step=None, head_shared: bool = False, kv_int8: bool = False,
                 twin: bool = False, twin_kv_every: int = 1, split_rows: bool = False) -> Report:
    """Runs the whole trajectory on the GPU; checks the sampled pairs every step.

    twin: a second full-size state is stepped beside the checked one in the call form that
    bench.py times - no debug weights and, in the fused forms, no kept_idx - and must stay
    bit-identical to it on EVERY pair (outputs, importance, positions and lengths every step; keys
    and values every twin_kv_every-th step and at the end).  The checked state is compared with
    the oracle, so the timed call form is tied to the oracle through it."""
    steps = wl.steps if steps is None else steps
    seqs = list(range(wl.b)) if seqs is None else list(seqs)
    heads = list(range(wl.h)) if heads is None else list(heads)
    prompt = W.make_prompt(wl, device, slack=slack) if prompt is None else prompt
    st = new_state(wl, prompt)
    rep = Report(pairs=len(seqs) * len(heads))
    if fused:
        # swa_decode_step with SWA_FUSE_COMPACTION: one kernel does the step and the compaction
        assert compact_every == 1
        st.params.flags = B.SWA_FUSE_COMPACTION | (B.SWA_UNORDERED if unordered else 0)
        if head_shared:
            # one token set per sequence from the head-summed importance: every head of a sampled
            # sequence is needed, and the workspace carries the slabs between the two launches
            assert unordered and len(heads) == wl.h
            st.params.flags |= B.SWA_HEAD_SHARED
            st.workspace = torch.zeros((B.swa_workspace_bytes(st.params),), dtype=torch.uint8, device=device)
            B.swa_workspace_init(st.params, st.workspace)
    else:
        assert not unordered
        if split_rows:
            # two-call form with one pair's rows split over several workgroups
            st.params.flags = B.SWA_SPLIT_ROWS
            st.workspace = torch.zeros((B.swa_workspace_bytes(st.params),), dtype=torch.uint8, device=device)
            B.swa_workspace_init(st.params, st.workspace)
    tw = None
    if twin:
        tw = new_state(wl, dict(prompt, K=prompt["K"].clone(), V=prompt["V"].clone(), pos=prompt["pos"].clone()),
                       debug_probs=False)
        tw.params.flags = st.params.flags
        tw.kept_idx.fill_(-7)                                  # must stay untouched in the fused forms
        if head_shared or split_rows:
            tw.workspace = torch.zeros((B.swa_workspace_bytes(tw.params),), dtype=torch.uint8, device=device)
            B.swa_workspace_init(tw.params, tw.workspace)
    # Unordered compaction keeps the cache as a set: every GPU tensor is brought into token order
    # (sorted by pos) before it is compared with the oracle, whose cache is always in token order.
    seqs_t = torch.tensor(seqs, device=device)
    heads_t = torch.tensor(heads, device=device)

    # oracle-side state of the sampled pairs
    K_o = _np64(_sub(st.K, seqs_t, heads_t))
    V_o = _np64(_sub(st.V, seqs_t, heads_t))
    pos_o = _sub(st.pos, seqs_t, heads_t).cpu().numpy().copy()
    len_o = st.cache_len[seqs_t].cpu().numpy().copy()
    n_o = len_o.copy()
    score_o = np.zeros(K_o.shape[:3])

    if wl.prefill_R > 0:
        q_tail = W.make_q_tail(wl, prompt["mu"], wl.prefill_R)
        st.prefill_scores(q_tail)
        S_ref = O.prefill_scores(_np64(_sub(q_tail, seqs_t, heads_t)), K_o, len_o, wl.scale)
        S_gpu = _np64(_sub(st.score, seqs_t, heads_t))
        np.testing.assert_allclose(S_gpu, S_ref, rtol=1e-5, atol=1e-12, err_msg="prefill seed")
        for i, L in enumerate(len_o):
            assert np.all(S_gpu[i, :, L:] == 0.0)
        score_o = S_gpu.copy()                                   # adopt
        if tw is not None:
            tw.prefill_scores(q_tail)
    else:
        st.score.zero_()
        if tw is not None:
            tw.score.zero_()

    qp = None
    if kv_int8:
        # Section V-B: the cache is compressed once the prompt (and its importance seed) is done.
        # Parameters and codes must equal the oracle's bit for bit; from here on the oracle's cache
        # holds the de-quantised values, which are what the compressed attention reads.
        st.quantize()
        if tw is not None:
            tw.quantize()
        qp_g = [_sub(st.qparams[k], seqs_t, heads_t).cpu().numpy() for k in range(4)]
        lamK, zK = O.kv_qparams(K_o, len_o)
        lamV, zV = O.kv_qparams(V_o, len_o)
        for g, o, nm in zip(qp_g, (lamK, zK, lamV, zV), ("lambda_K", "z_K", "lambda_V", "z_V")):
            assert np.array_equal(g, o), f"quantisation parameter {nm}"
        cK, cV = O.kv_quantize(K_o, len_o, lamK, zK), O.kv_quantize(V_o, len_o, lamV, zV)
        cK_g = _sub(st.K, seqs_t, heads_t).cpu().numpy()
        cV_g = _sub(st.V, seqs_t, heads_t).cpu().numpy()
        for i, L in enumerate(len_o):
            assert np.array_equal(cK_g[i, :, :L], cK[i, :, :L]), "key codes"
            assert np.array_equal(cV_g[i, :, :L], cV[i, :, :L]), "value codes"
        K_o, V_o = O.kv_dequantize(cK, len_o, lamK, zK), O.kv_dequantize(cV, len_o, lamV, zV)
        qp = (lamK, zK, lamV, zV)
        ones = np.ones_like(len_o)

        def through_codes(x, lam, zero):          # [S,H,d] new rows: quantise on arrival, de-quantise
            x4 = np.ascontiguousarray(x[:, :, None, :])
            return O.kv_dequantize(O.kv_quantize(x4, ones, lam, zero), ones, lam, zero)[:, :, 0, :]

    host_len = list(prompt["lengths"])          # host-side replay of every sequence's length
    for t in range(steps):
        q, kn, vn = W.make_step(wl, t, prompt["mu"])
        st.seq_len += 1
        n_o = n_o + 1
        sp_t = wl.sparsity_bp if sparsity_of_step is None else int(sparsity_of_step(t))
        st.params.sparsity_bp = sp_t          # the budget may change from call to call
        if use_len_bound:
            # exact bound: the longest cache of this step, from the host's replay of the budget
            st.params.len_bound = max(host_len) + 1
        if fused:
            score_prev32 = _sub(st.score, seqs_t, heads_t).cpu().numpy().astype(np.float32)
            pos_prev = _sub(st.pos, seqs_t, heads_t).cpu().numpy().copy()
            st.decode_compact_step(q, kn, vn)        # swaps cache_len / kept_cnt afterwards
        else:
            st.decode_step(q, kn, vn)
        if tw is not None:
            tw.seq_len += 1
            tw.params.sparsity_bp = sp_t
            tw.params.len_bound = st.params.len_bound
            if fused:
                tw.decode_compact_step(q, kn, vn, want_idx=False)
            else:
                tw.decode_step(q, kn, vn)
            assert _same_bits(tw.out, st.out), f"step {t}: twin output differs"
        for s_i in range(wl.b):
            m_i = host_len[s_i] + 1
            host_len[s_i] = (B.swa_budget(prompt["lengths"][s_i] + t + 1, m_i, wl.w, sp_t)[0]
                             if compact_every > 0 and (t + 1) % compact_every == 0 else m_i)
        do_check = check_steps is None or t in check_steps
        do_compact = compact_every > 0 and (t + 1) % compact_every == 0

        # ---- oracle step from the adopted state ---------------------------------
        q_o, kn_o, vn_o = (_np64(_sub(x, seqs_t, heads_t)) for x in (q, kn, vn))
        if kv_int8:
            kn_o, vn_o = through_codes(kn_o, qp[0], qp[1]), through_codes(vn_o, qp[2], qp[3])
        kept_o, cnt_o, out_o, p_o = O.decode_step(q_o, kn_o, vn_o, K_o, V_o, score_o, pos_o, len_o,
                                                  n_o, wl.w, sp_t, wl.scale, head_shared=head_shared)
        kept_g = _sub(st.kept_idx, seqs_t, heads_t).cpu().numpy()
        if fused:
            # the cache is already compacted: the new lengths are in cache_len (swapped in),
            # and the GPU's pre-compaction importance vector is rebuilt exactly as the kernel
            # formed it, fp32(old + p), from the adopted fp32 state and the fp32 weights
            cnt_g = st.cache_len[seqs_t].cpu().numpy()
            p32 = _sub(st.probs, seqs_t, heads_t).cpu().numpy().astype(np.float32)
            full32 = score_prev32.copy()
            for i, m in enumerate(len_o):
                full32[i, :, m - 1] = 0.0                      # the new token starts at zero
                full32[i, :, :m] = (full32[i, :, :m] + p32[i, :, :m]).astype(np.float32)
            score_g = full32.astype(np.float64)
            comp32 = _sub(st.score, seqs_t, heads_t).cpu().numpy()
            for i, c in enumerate(cnt_g):
                for hd in range(len(heads)):
                    assert np.array_equal(comp32[i, hd, :c], full32[i, hd, kept_g[i, hd, :c]]), \
                        f"step {t}: compacted importance is not fp32(old + p) of the kept slots"
            if unordered:
                # canonical (token-order) views: rank r of the pre-step cache <-> slot order[r]
                pos_post = _sub(st.pos, seqs_t, heads_t).cpu().numpy()
                p_can = np.zeros_like(p32)
                kept_can = np.full_like(kept_g, -1)
                orders = {}
                for i, m in enumerate(len_o):
                    for hd in range(len(heads)):
                        slot_pos = np.concatenate([pos_prev[i, hd, :m - 1], [n_o[i] - 1]])
                        order = np.argsort(slot_pos, kind="stable")
                        assert np.array_equal(slot_pos[order], pos_o[i, hd, :m]), \
                            f"step {t}: the cached token set differs from the oracle's"
                        inv = np.empty(m, dtype=np.int64)
                        inv[order] = np.arange(m)
                        c = cnt_g[i]
                        # kept_idx[j] is the pre-compaction slot of the token now in slot j
                        assert np.array_equal(slot_pos[kept_g[i, hd, :c]], pos_post[i, hd, :c]), \
                            f"step {t}: kept_idx does not describe the compacted cache"
                        kept_can[i, hd, :c] = np.sort(inv[kept_g[i, hd, :c]])
                        p_can[i, hd, :m] = p32[i, hd, order]
                        full32[i, hd, :m] = full32[i, hd, order]
                        orders[(i, hd)] = np.argsort(pos_post[i, hd, :c], kind="stable")
                kept_g = kept_can
                score_g = full32.astype(np.float64)
        else:
            score_g = _np64(_sub(st.score, seqs_t, heads_t))
            cnt_g = st.kept_cnt[seqs_t].cpu().numpy()
            assert np.array_equal(st.cache_len[seqs_t].cpu().numpy(), len_o), f"step {t}: cache_len"
        assert np.array_equal(cnt_g, cnt_o), f"step {t}: kept_cnt {cnt_g} vs {cnt_o}"

        if do_check:
            p_g = p_can.astype(np.float64) if unordered else _np64(_sub(st.probs, seqs_t, heads_t))
            out_g = _np64(_sub(st.out, seqs_t, heads_t))
            for i, m in enumerate(len_o):
                pe = np.abs(p_g[i, :, :m] - p_o[i, :, :m])
                assert np.all(pe <= 1e-5 * np.abs(p_o[i, :, :m]) + 1e-12), \
                    f"step {t} seq {seqs[i]}: probs rel err {np.max(pe / (p_o[i, :, :m] + 1e-300)):.3e}"
                assert np.all(p_g[i, :, m:] == 0.0)
                se = np.abs(score_g[i, :, :m] - score_o[i, :, :m])
                assert np.all(se <= 1e-5 * np.abs(score_o[i, :, :m]) + 1e-12), \
                    f"step {t} seq {seqs[i]}: score rel err"
                rep.max_prob_rel = max(rep.max_prob_rel, float(np.max(pe / (np.abs(p_o[i, :, :m]) + 1e-30))))
                rep.max_score_rel = max(rep.max_score_rel,
                                        float(np.max(se / (np.abs(score_o[i, :, :m]) + 1e-30))))
            # (ii) index sets: oracle selection on the GPU's own fp32 scores, bit-exact
            if head_shared:
                # the kernel sums the heads in fp32, head 0 first: take the decision in that precision
                tot32 = np.zeros((score_g.shape[0], score_g.shape[2]), dtype=np.float32)
                for hd in range(len(heads)):
                    tot32 = (tot32 + score_g[:, hd].astype(np.float32)).astype(np.float32)
                k1, cnt_ref = O.select(tot32[:, None, :].astype(np.float64), len_o, n_o, wl.w, sp_t)
                kept_ref = np.repeat(k1, len(heads), axis=1)
            else:
                kept_ref, cnt_ref = O.select(score_g, len_o, n_o, wl.w, sp_t)
            assert np.array_equal(cnt_ref, cnt_g)
            for i, c in enumerate(cnt_g):
                assert np.array_equal(kept_g[i, :, :c], kept_ref[i, :, :c]), \
                    f"step {t} seq {seqs[i]}: kept_idx differs from selection on the GPU's scores"
                # near-tie certificate against the oracle's own fp64 selection
                for hd in range(len(heads)):
                    a, b_ = set(kept_g[i, hd, :c].tolist()), set(kept_o[i, hd, :c].tolist())
                    diff = a ^ b_
                    if diff:
                        m = len_o[i]
                        nl = O.budget(int(n_o[i]), int(m), wl.w, sp_t)[1]
                        sel_o = score_o[i].sum(axis=0) if head_shared else score_o[i, hd]
                        cand = np.sort(sel_o[:m - nl])[::-1]
                        cutoff = cand[c - nl - 1]
                        for j in diff:
                            assert abs(sel_o[j] - cutoff) <= 2e-5 * abs(cutoff), \
                                f"step {t}: flipped token {j} is not a near tie"
                        rep.near_tie_flips += len(diff) // 2
            # (iii) output on the GPU's kept set
            out_ref = O.sparse_attention(q_o, K_o, V_o, kept_g, cnt_g, wl.scale)
            ea, er = check_out(out_g, out_ref, wl.dtype, f"step {t} out", rep)
            rep.max_out_abs, rep.max_out_rel = max(rep.max_out_abs, ea), max(rep.max_out_rel, er)

        # ---- adopt the GPU's importance values; compaction ----------------------------
        score_o = score_g.copy()
        for i, c in enumerate(cnt_g):
            rep.evictions += (int(len_o[i]) - int(c)) * len(heads)
        if do_compact:
            for i, c in enumerate(cnt_g):
                for hd in range(len(heads)):
                    rep.moved_rows += int(np.sum(kept_g[i, hd, :c] != np.arange(c)))
            if not fused:
                st.compact()
                if tw is not None:
                    tw.compact()
            O.compact(K_o, V_o, score_o, pos_o, kept_g, cnt_g, len_o)
            assert np.array_equal(st.cache_len[seqs_t].cpu().numpy(), len_o)
            if do_check:
                if kv_int8:
                    capc = np.full_like(len_o, st.K.shape[2])
                    K_g = O.kv_dequantize(_sub(st.K, seqs_t, heads_t).cpu().numpy(), capc, qp[0], qp[1])
                    V_g = O.kv_dequantize(_sub(st.V, seqs_t, heads_t).cpu().numpy(), capc, qp[2], qp[3])
                else:
                    K_g = _np64(_sub(st.K, seqs_t, heads_t))
                    V_g = _np64(_sub(st.V, seqs_t, heads_t))
                s_g = _np64(_sub(st.score, seqs_t, heads_t))
                pos_g = _sub(st.pos, seqs_t, heads_t).cpu().numpy().copy()
                if unordered:
                    for (i, hd), o2 in orders.items():
                        L = len_o[i]
                        K_g[i, hd, :L], V_g[i, hd, :L] = K_g[i, hd, o2], V_g[i, hd, o2]
                        s_g[i, hd, :L], pos_g[i, hd, :L] = s_g[i, hd, o2], pos_g[i, hd, o2]
                for i, L in enumerate(len_o):
                    assert np.array_equal(K_g[i, :, :L], K_o[i, :, :L]), f"step {t}: K after compaction"
                    assert np.array_equal(V_g[i, :, :L], V_o[i, :, :L]), f"step {t}: V after compaction"
                    assert np.array_equal(s_g[i, :, :L], score_o[i, :, :L]), f"step {t}: score after compaction"
                    assert np.array_equal(pos_g[i, :, :L], pos_o[i, :, :L]), f"step {t}: pos after compaction"
        if tw is not None:
            assert torch.equal(tw.cache_len, st.cache_len), f"step {t}: twin lengths differ"
            assert _same_bits(tw.score, st.score) and _same_bits(tw.pos, st.pos), f"step {t}: twin importance/pos"
            if (t + 1) % twin_kv_every == 0 or t == steps - 1:
                assert _same_bits(tw.K, st.K) and _same_bits(tw.V, st.V), f"step {t}: twin K/V differ"
            if fused:
                assert bool((tw.kept_idx == -7).all()), "kept_idx was written although not requested"
            rep.twin_steps += 1
        rep.steps += 1
        if verbose and (t % 16 == 0 or t == steps - 1):
            print(f"  [{wl.name}] step {t}: m={len_o.tolist()[:4]} ok", flush=True)
    assert st.check_status() == 0
    if tw is not None:
        assert tw.check_status() == 0
    return rep


def run_every_pair(wl: W.Workload, steps: int, chunk: int, device="cuda", first_seq: int = 0,
                   last_seq: Optional[int] = None, **kw) -> Report:
    """Lock-step check of EVERY (sequence, head) pair of sequences first_seq..last_seq-1 over the
    first `steps` decode steps (the step right after the prompt and the first steady ones), at
    full size on the GPU.  The sequences are checked `chunk` at a time to bound host memory; the
    GPU side is the same full-size trajectory for every chunk.  Stops at the first failure."""
    last_seq = wl.b if last_seq is None else last_seq
    prompt = W.make_prompt(wl, device, slack="zero")
    total = Report()
    for c0 in range(first_seq, last_seq, chunk):
        seqs = list(range(c0, min(last_seq, c0 + chunk)))
        pc = dict(prompt, K=prompt["K"].clone(), V=prompt["V"].clone(), pos=prompt["pos"].clone(),
                  cache_len=prompt["cache_len"].clone())
        rep = run_lockstep(wl, device=device, steps=steps, seqs=seqs, prompt=pc, slack="zero", use_len_bound=True, **kw)
        total.steps = rep.steps
        total.pairs += rep.pairs
        for f in ("max_prob_rel", "max_score_rel", "max_out_abs", "max_out_rel"):
            setattr(total, f, max(getattr(total, f), getattr(rep, f)))
        for f in ("near_tie_flips", "evictions", "moved_rows", "out_elems", "out_over_2e3"):
            setattr(total, f, getattr(total, f) + getattr(rep, f))
        print(f"  [{wl.name}] sequences {seqs[0]}..{seqs[-1]}: every head, {rep.steps} steps ok", flush=True)
        del pc
    return total


def run_lockstep_window(wl: W.Workload, R: int, device="cuda", steps: Optional[int] = None,
                        seqs: Optional[Sequence[int]] = None, heads: Optional[Sequence[int]] = None,
                        slack: str = "nan", use_len_bound: bool = False, seed_rows: bool = True,
                        sparsity_of_step=None, head_shared: bool = False, kv_int8: bool = False) -> Report:
    """Lock-step parity of swa_decode_step_window (strict local attention sum over a ring of R rows,
    unordered fused compaction) against the oracle's *_window routines.  The oracle's ring is the
    GPU's fp32 ring in token order (adopted row by row), so after every compaction the two rings
    must agree bit for bit; the importance is rebuilt from the GPU's own fp32 rows exactly as the
    kernel adds them (row order, fp32) and the selection is checked on those values."""
    steps = wl.steps if steps is None else steps
    seqs = list(range(wl.b)) if seqs is None else list(seqs)
    heads = list(range(wl.h)) if heads is None else list(heads)
    prompt = W.make_prompt(wl, device, slack=slack)
    st = new_state(wl, prompt)
    st.params.flags = B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED
    if head_shared:
        # one token set per sequence from the head-summed window sums: every head is needed
        assert len(heads) == wl.h
        st.params.flags |= B.SWA_HEAD_SHARED
        st.workspace = torch.zeros((B.swa_workspace_bytes(st.params),), dtype=torch.uint8, device=device)
        B.swa_workspace_init(st.params, st.workspace)
    rep = Report(pairs=len(seqs) * len(heads))
    seqs_t = torch.tensor(seqs, device=device)
    heads_t = torch.tensor(heads, device=device)
    K_o = _np64(_sub(st.K, seqs_t, heads_t))
    V_o = _np64(_sub(st.V, seqs_t, heads_t))
    pos_o = _sub(st.pos, seqs_t, heads_t).cpu().numpy().copy()
    len_o = st.cache_len[seqs_t].cpu().numpy().copy()
    n_o = len_o.copy()
    score_o = np.zeros(K_o.shape[:3])
    ring = torch.zeros((wl.b, wl.h, R, wl.cap), dtype=torch.float32, device=device)
    if seed_rows:
        q_tail = W.make_q_tail(wl, prompt["mu"], R)
        B.swa_prefill_rows(st.params, q_tail, R, st.K, st.cache_len, ring, st.workspace)
        ring_ref = O.prefill_rows(_np64(_sub(q_tail, seqs_t, heads_t)), K_o, len_o, wl.scale)
        ring_g = _np64(_sub(ring, seqs_t, heads_t))
        np.testing.assert_allclose(ring_g, ring_ref, rtol=1e-5, atol=1e-12, err_msg="prefill rows")
        assert np.all(ring_g[ring_ref == 0.0] == 0.0), "prefill rows: masked entries must be exactly 0"
        # their sum must agree with the seed of the running-sum path
        st.prefill_scores(q_tail)
        np.testing.assert_allclose(_np64(_sub(st.score, seqs_t, heads_t)), ring_g.sum(axis=2), rtol=2e-6, atol=1e-12)
        ring_o = ring_g.copy()
    else:
        ring_o = np.zeros((len(seqs), len(heads), R, wl.cap))
    # whatever sits in unused slots of the ring must never be read
    for s_i, L in enumerate(prompt["lengths"]):
        ring[s_i, :, :, L:] = float("nan")
    st.score.fill_(float("nan"))            # output only in this mode
    qp = None
    if kv_int8:
        # Section V-B after the prompt's rows are in the ring: parameters and codes bit-exact, then the
        # oracle's cache holds the de-quantised values
        st.quantize()
        qp_g = [_sub(st.qparams[k], seqs_t, heads_t).cpu().numpy() for k in range(4)]
        lamK, zK = O.kv_qparams(np.nan_to_num(K_o), len_o)
        lamV, zV = O.kv_qparams(np.nan_to_num(V_o), len_o)
        for g, o in zip(qp_g, (lamK, zK, lamV, zV)):
            assert np.array_equal(g, o), "quantisation parameters"
        cK, cV = O.kv_quantize(np.nan_to_num(K_o), len_o, lamK, zK), O.kv_quantize(np.nan_to_num(V_o), len_o, lamV, zV)
        cK_g = _sub(st.K, seqs_t, heads_t).cpu().numpy()
        for i, L in enumerate(len_o):
            assert np.array_equal(cK_g[i, :, :L], cK[i, :, :L]), "key codes"
        K_o, V_o = O.kv_dequantize(cK, len_o, lamK, zK), O.kv_dequantize(cV, len_o, lamV, zV)
        qp = (lamK, zK, lamV, zV)
        ones = np.ones_like(len_o)

        def through_codes(x, lam, zero):
            x4 = np.ascontiguousarray(x[:, :, None, :])
            return O.kv_dequantize(O.kv_quantize(x4, ones, lam, zero), ones, lam, zero)[:, :, 0, :]

    host_len = list(prompt["lengths"])
    for t in range(steps):
        row = t % R
        q, kn, vn = W.make_step(wl, t, prompt["mu"])
        st.seq_len += 1
        n_o = n_o + 1
        sp_t = wl.sparsity_bp if sparsity_of_step is None else int(sparsity_of_step(t))
        st.params.sparsity_bp = sp_t
        if use_len_bound:
            st.params.len_bound = max(host_len) + 1
        ring_prev = _sub(ring, seqs_t, heads_t).cpu().numpy()
        pos_prev = _sub(st.pos, seqs_t, heads_t).cpu().numpy().copy()
        if kv_int8:
            B.swa_decode_step_window_q8(st.params, q, kn, vn, st.K, st.V, st.qparams, ring, R, row, st.score,
                                        st.pos, st.cache_len, st.seq_len, st.kept_idx, st.kept_cnt, st.out,
                                        st.probs, st.workspace)
        else:
            B.swa_decode_step_window(st.params, q, kn, vn, st.K, st.V, ring, R, row, st.score, st.pos,
                                     st.cache_len, st.seq_len, st.kept_idx, st.kept_cnt, st.out, st.probs,
                                     st.workspace)
        st.cache_len, st.kept_cnt = st.kept_cnt, st.cache_len
        for s_i in range(wl.b):
            host_len[s_i] = B.swa_budget(prompt["lengths"][s_i] + t + 1, host_len[s_i] + 1, wl.w, sp_t)[0]

        q_o, kn_o, vn_o = (_np64(_sub(x, seqs_t, heads_t)) for x in (q, kn, vn))
        if kv_int8:
            kn_o, vn_o = through_codes(kn_o, qp[0], qp[1]), through_codes(vn_o, qp[2], qp[3])
        kept_o, cnt_o, out_o, p_o = O.decode_step_window(q_o, kn_o, vn_o, K_o, V_o, ring_o, row, score_o,
                                                         pos_o, len_o, n_o, wl.w, sp_t, wl.scale,
                                                         head_shared=head_shared)
        kept_g = _sub(st.kept_idx, seqs_t, heads_t).cpu().numpy()
        cnt_g = st.cache_len[seqs_t].cpu().numpy()
        assert np.array_equal(cnt_g, cnt_o), f"step {t}: kept_cnt {cnt_g} vs {cnt_o}"
        p32 = _sub(st.probs, seqs_t, heads_t).cpu().numpy().astype(np.float32)
        comp32 = _sub(st.score, seqs_t, heads_t).cpu().numpy()
        pos_post = _sub(st.pos, seqs_t, heads_t).cpu().numpy()
        ring_post = _sub(ring, seqs_t, heads_t).cpu().numpy()
        S32 = np.zeros(p32.shape, dtype=np.float32)
        p_can = np.zeros_like(p32)
        S_can = np.zeros_like(p32)
        kept_can = np.full_like(kept_g, -1)
        orders = {}
        for i, m in enumerate(len_o):
            # the kernel's sum: ring rows in index order, this step's weights in place of row `row`,
            # nothing from earlier rows for the token appended now (slot m-1)
            acc = np.zeros((len(heads), m), dtype=np.float32)
            for j in range(R):
                if j == row:
                    term = p32[i, :, :m]
                else:
                    term = ring_prev[i, :, j, :m].copy()
                    term[:, m - 1] = 0.0
                acc = (acc + term).astype(np.float32)
            S32[i, :, :m] = acc
            c = cnt_g[i]
            for hd in range(len(heads)):
                assert np.array_equal(comp32[i, hd, :c], S32[i, hd, kept_g[i, hd, :c]]), \
                    f"step {t}: compacted importance is not the fp32 row sum of the kept slots"
                slot_pos = np.concatenate([pos_prev[i, hd, :m - 1], [n_o[i] - 1]])
                order = np.argsort(slot_pos, kind="stable")
                assert np.array_equal(slot_pos[order], pos_o[i, hd, :m]), f"step {t}: cached token set"
                inv = np.empty(m, dtype=np.int64)
                inv[order] = np.arange(m)
                assert np.array_equal(slot_pos[kept_g[i, hd, :c]], pos_post[i, hd, :c]), \
                    f"step {t}: kept_idx does not describe the compacted cache"
                kept_can[i, hd, :c] = np.sort(inv[kept_g[i, hd, :c]])
                p_can[i, hd, :m] = p32[i, hd, order]
                S_can[i, hd, :m] = S32[i, hd, order]
                orders[(i, hd)] = np.argsort(pos_post[i, hd, :c], kind="stable")
        p_g, S_g = p_can.astype(np.float64), S_can.astype(np.float64)
        out_g = _np64(_sub(st.out, seqs_t, heads_t))
        for i, m in enumerate(len_o):
            pe = np.abs(p_g[i, :, :m] - p_o[i, :, :m])
            assert np.all(pe <= 1e-5 * np.abs(p_o[i, :, :m]) + 1e-12), f"step {t}: probs"
            se = np.abs(S_g[i, :, :m] - score_o[i, :, :m])
            assert np.all(se <= 1e-5 * np.abs(score_o[i, :, :m]) + 1e-12), f"step {t}: window sum"
            rep.max_prob_rel = max(rep.max_prob_rel, float(np.max(pe / (np.abs(p_o[i, :, :m]) + 1e-30))))
            rep.max_score_rel = max(rep.max_score_rel, float(np.max(se / (np.abs(score_o[i, :, :m]) + 1e-30))))
        if head_shared:
            # the kernel sums the heads in fp32, head 0 first: take the decision in that precision
            tot32 = np.zeros((S_g.shape[0], S_g.shape[2]), dtype=np.float32)
            for hd in range(len(heads)):
                tot32 = (tot32 + S_can[:, hd]).astype(np.float32)
            k1, cnt_ref = O.select(tot32[:, None, :].astype(np.float64), len_o, n_o, wl.w, sp_t)
            kept_ref = np.repeat(k1, len(heads), axis=1)
        else:
            kept_ref, cnt_ref = O.select(S_g, len_o, n_o, wl.w, sp_t)
        assert np.array_equal(cnt_ref, cnt_g)
        for i, c in enumerate(cnt_g):
            assert np.array_equal(kept_can[i, :, :c], kept_ref[i, :, :c]), \
                f"step {t} seq {seqs[i]}: kept_idx differs from selection on the GPU's window sums"
            for hd in range(len(heads)):
                diff = set(kept_can[i, hd, :c].tolist()) ^ set(kept_o[i, hd, :c].tolist())
                if diff:
                    m = len_o[i]
                    nl = O.budget(int(n_o[i]), int(m), wl.w, sp_t)[1]
                    sel_o = score_o[i].sum(axis=0) if head_shared else score_o[i, hd]
                    cutoff = np.sort(sel_o[:m - nl])[::-1][c - nl - 1]
                    for j in diff:
                        assert abs(sel_o[j] - cutoff) <= 2e-5 * abs(cutoff), f"step {t}: not a near tie"
                    rep.near_tie_flips += len(diff) // 2
            rep.evictions += (int(len_o[i]) - int(c)) * len(heads)
        out_ref = O.sparse_attention(q_o, K_o, V_o, kept_can, cnt_g, wl.scale)
        ea, er = check_out(out_g, out_ref, wl.dtype, f"step {t} out")
        rep.max_out_abs, rep.max_out_rel = max(rep.max_out_abs, ea), max(rep.max_out_rel, er)

        # adopt the GPU's row and sums, then compact both sides
        for i, m in enumerate(len_o):
            ring_o[i, :, row, :m] = p_g[i, :, :m]
        score_o = S_g.copy()
        O.compact_ring(ring_o, kept_can, cnt_g)
        O.compact(K_o, V_o, score_o, pos_o, kept_can, cnt_g, len_o)
        if kv_int8:
            capc = np.full_like(len_o, st.K.shape[2])
            K_g = O.kv_dequantize(_sub(st.K, seqs_t, heads_t).cpu().numpy(), capc, qp[0], qp[1])
            V_g = O.kv_dequantize(_sub(st.V, seqs_t, heads_t).cpu().numpy(), capc, qp[2], qp[3])
        else:
            K_g = _np64(_sub(st.K, seqs_t, heads_t))
            V_g = _np64(_sub(st.V, seqs_t, heads_t))
        for (i, hd), o2 in orders.items():
            L = len_o[i]
            assert np.array_equal(K_g[i, hd, o2], K_o[i, hd, :L]), f"step {t}: K after compaction"
            assert np.array_equal(V_g[i, hd, o2], V_o[i, hd, :L]), f"step {t}: V after compaction"
            assert np.array_equal(pos_post[i, hd, o2], pos_o[i, hd, :L]), f"step {t}: pos after compaction"
            assert np.array_equal(comp32[i, hd, o2].astype(np.float64), score_o[i, hd, :L])
            assert np.array_equal(ring_post[i, hd][:, o2].astype(np.float64), ring_o[i, hd, :, :L]), \
                f"step {t}: ring after compaction"
        rep.steps += 1
    assert st.check_status() == 0
    return rep


def run_free(wl: W.Workload, device="cuda", steps: Optional[int] = None):
    """Free-running comparison (no state adoption): the GPU and the fp64 oracle each follow their
    own trajectory from the same prompt.  While the kept sets agree, weights, importance and outputs
    must agree within the usual tolerances.  At the first step where they differ, every token of
    the symmetric difference must be a near tie in the oracle's own importance (within 2e-5
    relative of the cutoff): that is the only way an fp32 path may part from the fp64 one.
    Returns (first divergent step or None, flipped tokens at that step)."""
    steps = wl.steps if steps is None else steps
    prompt = W.make_prompt(wl, device, slack="nan")
    st = new_state(wl, prompt)
    K_o, V_o = np.nan_to_num(_np64(st.K)), np.nan_to_num(_np64(st.V))
    pos_o = st.pos.cpu().numpy().copy()
    len_o = st.cache_len.cpu().numpy().copy()
    n_o = len_o.copy()
    if wl.prefill_R > 0:
        q_tail = W.make_q_tail(wl, prompt["mu"], wl.prefill_R)
        st.prefill_scores(q_tail)
        score_o = O.prefill_scores(_np64(q_tail), K_o, len_o, wl.scale)
    else:
        st.score.zero_()
        score_o = np.zeros(K_o.shape[:3])
    for t in range(steps):
        q, kn, vn = W.make_step(wl, t, prompt["mu"])
        st.seq_len += 1
        n_o = n_o + 1
        st.decode_step(q, kn, vn)
        kept_o, cnt_o, out_o, p_o = O.decode_step(_np64(q), _np64(kn), _np64(vn), K_o, V_o, score_o, pos_o, len_o,
                                                  n_o, wl.w, wl.sparsity_bp, wl.scale)
        kept_g = st.kept_idx.cpu().numpy()
        cnt_g = st.kept_cnt.cpu().numpy()
        assert np.array_equal(cnt_g, cnt_o)
        p_g, s_g = _np64(st.probs), _np64(st.score)
        for i, m in enumerate(len_o):
            assert np.all(np.abs(p_g[i, :, :m] - p_o[i, :, :m]) <= 1e-5 * p_o[i, :, :m] + 1e-12), f"step {t}: probs"
            assert np.all(np.abs(s_g[i, :, :m] - score_o[i, :, :m]) <= 1e-5 * score_o[i, :, :m] + 1e-12), f"step {t}: score"
        flipped = 0
        for i, c in enumerate(cnt_g):
            m = len_o[i]
            nl = O.budget(int(n_o[i]), int(m), wl.w, wl.sparsity_bp)[1]
            for hd in range(wl.h):
                diff = set(kept_g[i, hd, :c].tolist()) ^ set(kept_o[i, hd, :c].tolist())
                if diff:
                    cutoff = np.sort(score_o[i, hd, :m - nl])[::-1][c - nl - 1]
                    for j in diff:
                        assert abs(score_o[i, hd, j] - cutoff) <= 2e-5 * abs(cutoff), \
                            f"step {t}: the paths part at token {j}, which is not a near tie"
                    flipped += len(diff) // 2
        if flipped:
            return t, flipped
        check_out(_np64(st.out), out_o, wl.dtype, f"free-running step {t} out")
        st.compact()
        O.compact(K_o, V_o, score_o, pos_o, kept_o, cnt_o, len_o)
    return None, 0
