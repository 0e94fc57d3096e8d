"""The stored oracle trajectories under tests/golden/ obey what Alg. 2 / Alg. 3 fix for any model
(no GPU, no oracle call: only the files are read).  A file that was cut short, written by a broken
recorder, or generated for other decode arguments than its workload's fails here, before any GPU test
leans on it."""
import glob
import json
import os

import numpy as np
import pytest

from paper_2509_25188_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
FILES = sorted(glob.glob(os.path.join(GOLDEN, "traj_*.npz")))


def workload_of(meta):
    w = synth.WORKLOADS[meta["workload"]]
    return w


@pytest.mark.parametrize("path", FILES, ids=[os.path.basename(p) for p in FILES])
def test_stored_trajectory_obeys_the_decode_rule(path):
    z = np.load(path)
    meta = json.loads(str(z["meta"]))
    w = workload_of(meta)
    m, s, P, G = w.model, w.block_len, w.prompt_len, w.gen_len
    assert (meta["block_len"], meta["prompt_len"], meta["gen_len"], meta["threshold"]) == (s, P, G, w.threshold)
    assert meta["layers"] in (m.n_layers, 2) and meta["seed"] == 1234
    prompt = synth.make_prompt(1234, max(w.batch, meta["seq"] + 1), P, w.prompt_hi)[meta["seq"]].numpy()
    np.testing.assert_array_equal(z["prompt"], prompt)
    if "block" not in z:                      # result of a decode only (EoTP-off companion)
        assert not meta["eotp"] and int(z["decoded_len"]) == G and not np.any(z["tokens"] == m.mask_id)
        assert G // s <= int(z["steps"]) <= G
        on = path.replace("_eotp_off", "")
        if os.path.exists(on):
            # Alg. 3 changes nothing before it stops: the run with EoTP is a prefix of the run without, and shorter
            zo = np.load(on)
            dl = int(zo["decoded_len"])
            np.testing.assert_array_equal(zo["tokens"][:dl], z["tokens"][:dl])
            assert int(zo["steps"]) < int(z["steps"])
        return
    X, blk, sel, masked = z["X_before"], z["block"], z["sel"].astype(bool), z["masked"].astype(bool)
    conf, pre, p = z["conf"], z["pre"], z["p"]
    n = len(blk)
    assert X.shape == (n, P + G) and sel.shape == (n, s) == masked.shape == conf.shape == pre.shape == p.shape
    whole = "states_from" not in meta
    for i in range(n):
        lo = P + int(blk[i]) * s
        np.testing.assert_array_equal(X[i, :P], prompt)
        np.testing.assert_array_equal(masked[i], X[i, lo:lo + s] == m.mask_id)       # masked <=> holds the mask id
        assert masked[i].any() and not np.any(X[i, P:lo] == m.mask_id)               # earlier blocks are complete
        assert np.all(X[i, lo + s:] == m.mask_id)                                    # later blocks untouched
        assert not np.any(sel[i] & ~masked[i]) and sel[i].any()                      # only masked positions, at least one
        assert np.all(sel[i][masked[i] & (p[i] > np.float32(w.threshold))])          # everything above tau is taken
        top = int(np.argmax(np.where(masked[i], conf[i], -np.inf)))
        assert sel[i][top]                                                           # the forced position
        extra = sel[i] & ~(p[i] > np.float32(w.threshold))
        assert extra.sum() <= 1 and (not extra.any() or extra[top])                  # and nothing else below tau
        assert np.all(pre[i] != m.mask_id) and np.all((conf[i] > 0) & (conf[i] <= 1))
        if whole and i + 1 < n:
            after = X[i].copy()
            after[lo + np.nonzero(sel[i])[0]] = pre[i][sel[i]]
            np.testing.assert_array_equal(X[i + 1], after)                           # never remasked, nothing else moves
            assert blk[i + 1] == blk[i] + (0 if np.any(after[lo:lo + s] == m.mask_id) else 1)
    if whole:
        assert blk[0] == 0 and np.all(X[0, P:] == m.mask_id)
        per_block = np.bincount(blk)
        assert np.all(per_block >= 1) and np.all(per_block <= s)                     # at most block_len steps per block
        assert int(z["steps"]) == n
        last = X[-1].copy()
        lo = P + int(blk[-1]) * s
        last[lo + np.nonzero(sel[-1])[0]] = pre[-1][sel[-1]]
        np.testing.assert_array_equal(z["tokens"], last[P:])
        dlen = int(z["decoded_len"])
        if w.eotp:
            stop = w.bias_from // s                                                  # the block holding the first forced end-of-text
            assert int(blk[-1]) == stop and dlen == (stop + 1) * s
            assert np.all(z["tokens"][w.bias_from:dlen] == m.eos_id) and np.all(z["tokens"][dlen:] == m.mask_id)
            first = int(np.nonzero(z["tokens"] == m.eos_id)[0][0])
            assert first // s == stop                                                # no end-of-text in an earlier block
        else:
            assert dlen == G and int(blk[-1]) == G // s - 1 and not np.any(z["tokens"] == m.mask_id)
    # sampled steps: logit samples and the two comparison distances
    smp = z["smp_idx"]
    assert len(smp) >= 2 and np.all(np.diff(smp) > 0) and smp[-1] < n
    assert z["lg_fixed"].shape == (len(smp), s, len(z["cols_fixed"])) and z["lg_top"].shape == (len(smp), s, 8)
    assert np.all(np.diff(z["lg_top"], axis=-1) <= 0)                                # the oracle's largest logits, descending
    np.testing.assert_array_equal(z["cols_top"][:, :, 0], pre[smp])                  # the largest one is the greedy token
    np.testing.assert_allclose(z["gap"][smp], z["lg_top"][:, :, 0] - z["lg_top"][:, :, 1], rtol=0, atol=1e-5)
    assert np.all(z["absmax"][smp] >= np.max(np.abs(z["lg_top"]), axis=(1, 2)) - 1e-6)
    floor = z["floor_abs"][np.isfinite(z["floor_abs"])]
    assert len(floor) >= 1 and np.all(floor > 0) and np.all(z["fmt_abs"] > 0)
    assert floor.max() < z["fmt_abs"].max()          # the format's error exceeds the accumulation noise
    assert z["fmt_abs"].max() < 0.05 * z["absmax"].max()
