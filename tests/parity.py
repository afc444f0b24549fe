"""GPU-vs-oracle comparison rule (not collected by pytest).

Labels and emission frames must be identical and scores within 1e-3, except for
hypotheses where a different rounding order flipped a decision whose top-2 logit
margin is below 1e-3.  Such a hypothesis is accepted only if the oracle's replay
check confirms that the GPU's (labels, frames) is a greedy decode under an argmax
tolerant to 1e-3, with the score re-computed along that path; the number of
hypotheses and of near-tie choices accepted this way is returned and bounded by
the caller.
"""
from __future__ import annotations

import os
import sys

import numpy as np

TOL_MARGIN = 1e-3
TOL_SCORE = 1e-3


_CASE_LOG = os.environ.get("TDT_CASE_LOG", "")   # optional file that also receives the case names


def announce(msg: str) -> None:
    """Name the case before a GPU step: on the real stderr, and -- if TDT_CASE_LOG names a file --
    appended there and flushed to disk, so that its last line names the case if the process dies."""
    sys.__stderr__.write("[gpu-case] " + msg + "\n")
    sys.__stderr__.flush()
    if not _CASE_LOG:
        return
    try:
        os.makedirs(os.path.dirname(os.path.abspath(_CASE_LOG)), exist_ok=True)
        with open(_CASE_LOG, "a") as f:
            f.write(msg + "\n")
            f.flush()
            os.fsync(f.fileno())
    except OSError:
        pass


def compare(oracle, omodel, cfg, enc, enc_len, gpu: dict, u_cap: int, rows=None,
            max_symbols=None, orc: dict = None) -> dict:
    """Compare rows (default: all) of a GPU result against the oracle."""
    S = cfg.max_symbols if max_symbols is None else max_symbols
    rows = list(range(len(enc_len))) if rows is None else list(rows)
    lens_clamped = np.clip(enc_len, 0, cfg.T)
    if orc is None:
        sub_enc = enc[rows]
        orc = oracle.decode_batch(omodel, sub_enc, lens_clamped[rows], S, u_cap)
        orc_rows = {b: i for i, b in enumerate(rows)}
    else:
        orc_rows = {b: b for b in rows}
    n_exact = n_replayed = n_tie = 0
    score_err = 0.0
    for b in rows:
        i = orc_rows[b]
        n, no = int(gpu["len"][b]), int(orc["len"][i])
        gl, gf = gpu["labels"][b, :n], gpu["frames"][b, :n]
        same = n == no and (gl == orc["labels"][i, :no]).all() and (gf == orc["frames"][i, :no]).all()
        if same:
            score_err = max(score_err, abs(float(gpu["score"][b]) - float(orc["score"][i])))
            assert abs(float(gpu["score"][b]) - float(orc["score"][i])) <= TOL_SCORE, \
                f"row {b}: score {gpu['score'][b]} vs oracle {orc['score'][i]}"
            assert bool(gpu["status"][b] & 1) == bool(orc["status"][i]), f"row {b}: status"
            n_exact += 1
            continue
        rp = oracle.replay_utt(omodel, enc[b], int(lens_clamped[b]), S, u_cap, gl, gf, tol=TOL_MARGIN)
        first = next((j for j in range(min(n, no))
                      if gl[j] != orc["labels"][i, j] or gf[j] != orc["frames"][i, j]), min(n, no))
        assert rp["ok"], (f"row {b}: GPU hypothesis (len {n}) differs from the oracle's (len {no}) "
                          f"at label {first} and is not a greedy decode within {TOL_MARGIN}")
        assert rp["n_tie"] >= 1
        score_err = max(score_err, abs(float(gpu["score"][b]) - rp["score"]))
        assert abs(float(gpu["score"][b]) - rp["score"]) <= TOL_SCORE, f"row {b}: replayed score"
        n_replayed += 1
        n_tie += rp["n_tie"]
    return dict(exact=n_exact, replayed=n_replayed, ties=n_tie, rows=len(rows), max_score_err=score_err)
