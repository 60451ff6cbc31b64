"""Helpers that compare the HIP path with the CPU oracle on the same seeded inputs.

Decisions (token ids, accept bits) are compared bit-exactly wherever the oracle's decision is
stable under the measured logit difference: for a step whose GPU logits differ from the
oracle's by at most e per element, every score of the samplers moves by at most e/T (plus a few
fp32 rounding steps of the exp/log the kernels evaluate), and the oracle reports whether its
winner can change under such a move.  Unstable decisions are counted, never silently passed.
"""
import numpy as np

import pass_oracle as O

F32_ARITH = 3e-5  # fp32 exp/log/ln-sum-exp noise on scores of magnitude <~ 30

LOGIT_TOL = {0: 1e-4, 1: 2e-2}  # per row: max|diff| / max|logit|, fp32 / bf16 models


def logits_error(gpu, ref, tol, what=""):
    """Assert per-row max|diff| <= tol * max|ref| and return the largest absolute difference."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite logits"
    worst = 0.0
    for r in range(ref.shape[0]):
        diff = np.abs(gpu[r] - ref[r]).max()
        scale = np.abs(ref[r]).max()
        assert diff <= tol * scale, f"{what} row {r}: max|diff| {diff:.3e} > {tol:g} * {scale:.3e}"
        worst = max(worst, diff)
    return worst


class StepStats:
    def __init__(self):
        self.compared = 0
        self.unstable = 0
        self.iterations = 0
        self.accepted = 0
        self.resyncs = 0
        self.max_rel_err = 0.0

    def __repr__(self):
        return (f"iters={self.iterations} decisions={self.compared} unstable={self.unstable} "
                f"accepted={self.accepted} resyncs={self.resyncs} max_rel_err={self.max_rel_err:.2e}")


def _check_draft(st, it, k, temp, seed, seq_id, tol, top_k, ol, gl, o_first, o_drafts, g_first, g_drafts):
    """Drafting call of one sequence: logits within tolerance, every stable decision identical.
    Returns (all decisions identical, largest absolute logit difference)."""
    inv_t = 1.0 if temp == 0 else 1.0 / temp
    err_d = logits_error(gl, ol, tol, f"draft it={it}")
    st.max_rel_err = max(st.max_rel_err, err_d / np.abs(ol).max())
    tau = err_d * inv_t * 1.01 + (0.0 if temp == 0 else F32_ARITH)
    same = True
    for t in range(k + 1):
        tok, stable = O.sample_softmax(ol[t], temp, seed, seq_id, it, t, O.DRAFT, tau, top_k)
        o_tok = o_first if t == 0 else o_drafts[t - 1]
        g_tok = g_first if t == 0 else g_drafts[t - 1]
        assert tok == o_tok
        st.compared += 1
        if stable:
            assert g_tok == tok, f"draft it={it} row {t}: gpu {g_tok} != oracle {tok} on a stable decision"
        else:
            st.unstable += 1
            same &= g_tok == tok
    return same, err_d


def _check_verify(st, it, k, temp, seed, seq_id, tol, top_k, ol, pl, gpl, err_d, o_drafts, o_a, o_out, g_a, g_out):
    """Validation call of one sequence (g_out: the slot's k + 1 output entries).  Returns whether
    the two sides took the same decisions (a difference on a stable decision fails)."""
    inv_t = 1.0 if temp == 0 else 1.0 / temp
    err_v = logits_error(gpl, pl, tol, f"verify it={it}")
    st.max_rel_err = max(st.max_rel_err, err_v / np.abs(pl).max())
    tau = max(err_d, err_v) * inv_t * 1.01 + (0.0 if temp == 0 else F32_ARITH)
    a = 0
    chain_stable = True
    for t in range(1, k + 1):  # replay the accept chain with stability flags
        acc, stable = O.accept(pl[t - 1], ol[t], o_drafts[t - 1], temp, seed, seq_id, it, t, tau, top_k)
        st.compared += 1
        if not stable:
            st.unstable += 1
            chain_stable = False
        if not acc:
            break
        a += 1
    assert a == o_a
    if chain_stable:
        assert g_a == a, f"verify it={it}: gpu accepted {g_a}, oracle {a}"
    elif g_a != a:
        return False
    if a < k:
        y, stable, _ = O.sample_residual(pl[a], ol[a + 1], temp, seed, seq_id, it, a + 1, tau, top_k)
    else:
        y, stable = O.sample_softmax(pl[k], temp, seed, seq_id, it, k + 1, O.BONUS, tau, top_k)
    assert y == o_out[-1]
    st.compared += 1
    assert np.array_equal(g_out[:a], o_out[:a])
    if stable:
        assert g_out[a] == y, f"verify it={it}: final token gpu {g_out[a]} != oracle {y} (a={a})"
    else:
        st.unstable += 1
        if g_out[a] != y:
            return False
    assert np.all(g_out[a + 1:] == -1)
    st.accepted += a
    return True


def _one_iteration(gpu, oseq, slot, seq_id, it, temp, seed, tol, st, top_k=0):
    """One draft + verify on both sides.  Returns (tokens the oracle added, in_sync)."""
    k = getattr(gpu, "k_act", gpu.k)  # look-ahead rows of this call (buffers are sized for gpu.k)
    kv0 = oseq.kv_len
    o_first, o_drafts = oseq.draft(temp, seed, top_k=top_k)
    g_first, g_drafts = gpu.draft([slot], temp, seed, top_k)
    ol, gl = oseq.logits(0), gpu.get_logits(slot, 0)[:k + 1]
    same, err_d = _check_draft(st, it, k, temp, seed, seq_id, tol, top_k, ol, gl, o_first, o_drafts,
                               g_first[0], g_drafts[0])
    assert gpu.seq_len(slot)[0] == kv0 + 1 == oseq.kv_len
    o_a, o_out = oseq.verify(temp, seed, top_k=top_k)
    added = [o_first] + [int(x) for x in o_out]
    if not same:
        return added, False
    g_a, g_out = gpu.verify([slot], temp, seed, top_k)
    pl, gpl = oseq.logits(1), gpu.get_logits(slot, 1)[:k + 1]
    if not _check_verify(st, it, k, temp, seed, seq_id, tol, top_k, ol, pl, gpl, err_d, o_drafts, o_a, o_out,
                         int(g_a[0]), g_out[0]):
        return added, False
    assert gpu.seq_len(slot)[0] == kv0 + 2 + o_a == oseq.kv_len
    return added, True


def batch_parity(gpu, omodel, slots, seq_ids, prompts, sampled, n_iters, temp, seed, tol, max_len, top_k=0, one_call=False):
    """A batch of slots through draft / verify calls that carry every slot (the launch shapes of the
    batch), with the sequences of the `sampled` slots run alone through the oracle: a sequence's
    result does not depend on what shares its calls.  Every call's logits and decisions of the
    sampled slots are compared as in stepwise_parity.  A sampled slot that parts ways on an
    unstable decision is dropped from the comparison from then on (counted in `resyncs`).
    one_call: the prompts go through pass_prefill_batch instead of one pass_prefill each.
    Returns {slot: StepStats}."""
    k = getattr(gpu, "k_act", gpu.k)
    if one_call:
        gpu.prefill_batch(slots, prompts, seq_ids)
    else:
        for sl, sid, p in zip(slots, seq_ids, prompts):
            gpu.prefill(sl, p, seq_id=sid)
    oseqs, stats, live = {}, {}, set(sampled)
    for sl in sampled:
        i = list(slots).index(sl)
        oseqs[sl] = omodel.sequence(max_len, seq_id=seq_ids[i])
        oseqs[sl].prefill(prompts[i])
        stats[sl] = StepStats()
    for it in range(n_iters):
        g_first, g_drafts = gpu.draft(slots, temp, seed, top_k)
        g_kv = {sl: gpu.seq_len(sl)[0] for sl in live}
        pend = {}
        for sl in sorted(live):
            i, o, st = list(slots).index(sl), oseqs[sl], stats[sl]
            kv0 = o.kv_len
            o_first, o_drafts = o.draft(temp, seed, top_k=top_k)
            ol, gl = o.logits(0), gpu.get_logits(sl, 0)[:k + 1]
            same, err_d = _check_draft(st, it, k, temp, seed, seq_ids[i], tol, top_k, ol, gl, o_first, o_drafts,
                                       g_first[i], g_drafts[i])
            assert g_kv[sl] == kv0 + 1 == o.kv_len
            o_a, o_out = o.verify(temp, seed, top_k=top_k)
            pend[sl] = (same, err_d, ol, o_drafts, o_a, o_out, kv0)
        g_a, g_out = gpu.verify(slots, temp, seed, top_k)
        for sl in sorted(live):
            i, o, st = list(slots).index(sl), oseqs[sl], stats[sl]
            same, err_d, ol, o_drafts, o_a, o_out, kv0 = pend[sl]
            st.iterations += 1
            if same:
                pl, gpl = o.logits(1), gpu.get_logits(sl, 1)[:k + 1]
                same = _check_verify(st, it, k, temp, seed, seq_ids[i], tol, top_k, ol, pl, gpl, err_d, o_drafts,
                                     o_a, o_out, int(g_a[i]), g_out[i])
            if same:
                assert gpu.seq_len(sl)[0] == kv0 + 2 + o_a == o.kv_len
            else:
                st.resyncs += 1
                live.discard(sl)
    return stats


def stepwise_parity(gpu, omodel, slot, seq_id, prompt, n_iters, temp, seed, tol, max_len=256, stats=None,
                    top_k=0, first_oseq=None):
    """Drive one sequence through draft / verify on both sides, comparing the logits of every
    call and every decision.  A difference on a stable decision fails.  When an unstable decision
    differs, both sides restart from the oracle's token history (a resync, counted).
    first_oseq: an oracle sequence that already holds the prompt (same sequence id), used instead
    of a fresh prompt pass of the oracle for the first round."""
    st = stats or StepStats()
    hist = [int(t) for t in prompt]
    done = 0
    while done < n_iters:
        gpu.prefill(slot, hist, seq_id=seq_id)
        if first_oseq is not None:
            oseq, first_oseq = first_oseq, None
        else:
            oseq = omodel.sequence(max_len, seq_id=seq_id)
            oseq.prefill(hist)
        it = 0
        while done < n_iters:
            added, in_sync = _one_iteration(gpu, oseq, slot, seq_id, it, temp, seed, tol, st, top_k)
            hist += added
            done += 1
            it += 1
            st.iterations += 1
            if not in_sync:
                st.resyncs += 1
                break
    return st


# Bounds of check_stats: about twice what the seeded runs of the test suite measure on MI355X.
# fp32 models agree to 4e-7 of the row's largest logit; bf16 models of two or three layers to
# 2e-4 (weights and K/V are the only rounded values: the rest is fp32 against fp64), the 7B width
# with two layers to 5.5e-4, the 7B model at full depth to 1.3e-3.
ERR_F32 = 2e-6
ERR_BF16_SMALL = 4e-4
ERR_BF16_7B_2L = 1.2e-3


def check_stats(st, n_iters, max_err, max_unstable=2, max_resyncs=0):
    """The run did what it was asked, and stayed as close to the oracle as such runs measure."""
    assert st.iterations == n_iters, st
    assert st.max_rel_err <= max_err, st
    assert st.unstable <= max_unstable and st.resyncs <= max_resyncs, st


def sps_parity(gpu_t, gpu_d, om_t, om_d, slot, seq_id, prompt, n_iters, temp, seed, tol, max_len=256, top_k=0):
    """Two-model speculative sampling (Algorithm 2), one sequence, GPU target / drafter contexts
    against the oracle's: per iteration the drafter's logits rows and drafted tokens, the target's
    validation logits and every decision, as in stepwise_parity (resync on an unstable difference)."""
    st = StepStats()
    k = getattr(gpu_t, "k_act", gpu_t.k)
    inv_t = 1.0 if temp == 0 else 1.0 / temp
    hist = [int(t) for t in prompt]
    done = 0
    while done < n_iters:
        for g in (gpu_t, gpu_d):
            g.prefill(slot, hist, seq_id=seq_id)
        ot, od = om_t.sequence(max_len, seq_id=seq_id), om_d.sequence(max_len, seq_id=seq_id)
        ot.prefill(hist)
        od.prefill(hist)
        it = 0
        while done < n_iters:
            kv0 = ot.kv_len
            o_a, o_out, o_dl = ot.sps_iteration(od, temp, seed, top_k=top_k)
            g_drafts, g_a, g_out = gpu_t.sps_iteration(gpu_d, [slot], [slot], temp, seed, top_k)
            done += 1
            st.iterations += 1
            hist += [int(x) for x in o_out]
            in_sync = True
            # drafting: rows 1 .. k of the target slot's drafting logits hold the drafter's rows
            err_d = 0.0
            drafts = []
            if k:
                gl = gpu_t.get_logits(slot, 0)[1:k + 1]
                err_d = logits_error(gl, o_dl, tol, f"drafter it={it}")
                st.max_rel_err = max(st.max_rel_err, err_d / np.abs(o_dl).max())
            tau = err_d * inv_t * 1.01 + (0.0 if temp == 0 else F32_ARITH)
            for t in range(1, k + 1):
                tok, stable = O.sample_softmax(o_dl[t - 1], temp, seed, seq_id, it, t, O.DRAFT, tau, top_k)
                drafts.append(tok)
                st.compared += 1
                if stable:
                    assert g_drafts[0, t - 1] == tok, f"drafter it={it} row {t}: gpu {g_drafts[0, t - 1]} != oracle {tok}"
                else:
                    st.unstable += 1
                    in_sync &= g_drafts[0, t - 1] == tok
                if not in_sync:
                    break  # later drafter rows saw another token
            if in_sync:
                ol = np.concatenate([np.zeros((1, o_dl.shape[1]), np.float32), o_dl]) if k else np.zeros((1, gpu_t.vocab), np.float32)
                pl, gpl = ot.logits(1), gpu_t.get_logits(slot, 1)[:k + 1]
                in_sync = _check_verify(st, it, k, temp, seed, seq_id, tol, top_k, ol, pl, gpl, err_d, drafts, o_a, o_out,
                                        int(g_a[0]), g_out[0])
            if in_sync:
                assert gpu_t.seq_len(slot)[0] == kv0 + 1 + o_a == ot.kv_len == od.kv_len == gpu_d.seq_len(slot)[0]
            else:
                st.resyncs += 1
                break
            it += 1
    return st


def generate_parity(gpu_tokens, oracle_tokens, oracle_acc, oracle_stable):
    """Free-running comparison.  Returns the identical prefix length; a mismatch inside an
    iteration whose decisions the oracle reports stable (and with no unstable iteration before
    it) fails."""
    n = len(oracle_tokens)
    assert len(gpu_tokens) == n
    if np.array_equal(gpu_tokens, oracle_tokens):
        return n
    first_bad = int(np.nonzero(np.asarray(gpu_tokens) != np.asarray(oracle_tokens))[0][0])
    pos = 0
    for it, a in enumerate(oracle_acc):
        end = pos + a + 2
        if not oracle_stable[it]:
            return first_bad  # an unstable decision at or before the mismatch: allowed to part ways
        if first_bad < end:
            raise AssertionError(f"token {first_bad} differs inside iteration {it}, "
                                 "all of whose decisions are stable")
        pos = end
    raise AssertionError("mismatch beyond the recorded iterations")
