"""Comparison rules between the HIP path and the CPU oracle.

Bars (from the build's contract): noise bits, indices and flags bit-exact, except where
floating point decides them and the oracle's own gap is below 1e-6 relative (those are
excused AND counted); fp32 margins, CDF values and distances within 1e-4 absolute.
"""
import numpy as np
import torch

import oracle

ABS_TOL = 1e-4          # fp32 margins, interval ends, distances
TIE_REL = 1e-6          # oracle gap below this (relative) => either answer is accepted


def to_host_logits(t: torch.Tensor) -> np.ndarray:
    """Device or host logits tensor -> numpy array the oracle accepts (uint16 bf16 bits / float32)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    assert t.dtype == torch.float32
    return t.numpy()


def seeds_u64(seeds: torch.Tensor) -> np.ndarray:
    return seeds.cpu().numpy().view(np.uint64)


def positions_u32(pos: torch.Tensor) -> np.ndarray:
    return pos.cpu().numpy().view(np.uint32)


def _np(d):
    return {k: (v.detach().cpu().numpy() if isinstance(v, torch.Tensor) else v) for k, v in d.items()}


def _close(gpu, ref, tol, what):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    both_nan = np.isnan(gpu) & np.isnan(ref)
    both_inf = np.isinf(gpu) & np.isinf(ref) & (np.sign(gpu) == np.sign(ref))
    err = np.where(both_nan | both_inf, 0.0, np.abs(gpu - ref))
    bad = ~(err <= tol)
    assert not bad.any(), "%s: %d rows beyond %g, worst %g at row %d (gpu %r, oracle %r)" % (
        what, int(bad.sum()), tol, float(np.nanmax(err)), int(np.argmax(np.nan_to_num(err, nan=np.inf))),
        gpu[np.argmax(np.nan_to_num(err, nan=np.inf))], ref[np.argmax(np.nan_to_num(err, nan=np.inf))])
    return float(err.max()) if err.size else 0.0


def compare_gumbel(gpu: dict, ref: dict, tie_rel: float = TIE_REL):
    """gpu: outputs of the binding (torch), ref: outputs of oracle.gumbel_score (numpy).
    Returns a dict of counters (near ties that were excused, worst errors).
    tie_rel: oracle gap (relative to max(1, |max score|)) below which either argmax is accepted; callers
    whose logits themselves carry rounding error (the fused LM head) pass that error's size."""
    g = _np(gpu)
    n = ref["margin"].shape[0]
    scale = np.maximum(1.0, np.abs(ref["max_score"]))
    near_tie = ref["gap2"] < tie_rel * scale
    stats = {"rows": n, "near_ties": int(near_tie.sum())}
    stats["margin_err"] = _close(g["margin"], ref["margin"], ABS_TOL, "margin")
    if "max_score" in g:
        stats["max_err"] = _close(g["max_score"], ref["max_score"], ABS_TOL, "max_score")
        stats["claimed_err"] = _close(g["claimed_score"], ref["claimed_score"], ABS_TOL, "claimed_score")
    diff = g["argmax"] != ref["argmax"]
    assert not (diff & ~near_tie).any(), "argmax differs on %d rows that are not near ties: rows %s" % (
        int((diff & ~near_tie).sum()), np.nonzero(diff & ~near_tie)[0][:10])
    stats["argmax_excused"] = int(diff.sum())
    fdiff = (g["flags"] ^ ref["flags"]).astype(np.uint8)
    assert not (fdiff & ~np.uint8(1)).any(), "non-MATCH flag bits differ on rows %s" % np.nonzero(fdiff & 0xFE)[0][:10]
    assert not ((fdiff & 1).astype(bool) & ~near_tie).any(), "MATCH differs outside near ties"
    stats["match_excused"] = int((fdiff & 1).sum())
    assert (g["margin"][~np.isnan(g["margin"])] >= 0).all()
    return stats


def compare_ipt(gpu: dict, ref: dict, logits_host=None, V=None, row_args=None, log_mass_sigma=None,
                tie_rel: float = TIE_REL):
    """ref: outputs of oracle.ipt_score.  If tokens are compared and some differ, `logits_host`
    (numpy, as given to the oracle), `V` and `row_args` (T or per-row temps, seeds, seq_ids,
    positions as numpy) let the near-tie rule look at the oracle interval of the GPU's token."""
    g = _np(gpu)
    n = ref["dist"].shape[0]
    stats = {"rows": n}
    stats["dist_err"] = _close(g["dist"], ref["dist"], ABS_TOL, "dist")
    if "cdf_lo" in g:
        stats["cdf_err"] = max(_close(g["cdf_lo"], ref["cdf_lo"], ABS_TOL, "cdf_lo"),
                               _close(g["cdf_hi"], ref["cdf_hi"], ABS_TOL, "cdf_hi"))
        ok = ~np.isnan(g["u"])
        assert np.array_equal(g["u"][ok].astype(np.float64), ref["u"][ok]), "regenerated uniform differs"
    near_edge = np.nan_to_num(ref["edge"], nan=np.inf) < tie_rel
    stats["near_edges"] = int(near_edge.sum())
    slow = np.uint8(8)
    fdiff = ((g["flags"] & ~slow) ^ ref["flags"]).astype(np.uint8)
    assert not (fdiff & ~np.uint8(1)).any(), "non-MATCH flag bits differ on rows %s" % np.nonzero(fdiff & 0xFE)[0][:10]
    assert not ((fdiff & 1).astype(bool) & ~near_edge).any(), "MATCH differs outside near ties: rows %s" % (
        np.nonzero((fdiff & 1).astype(bool) & ~near_edge)[0][:10])
    stats["match_excused"] = int((fdiff & 1).sum())
    if "ipt_token" in g:
        diff = np.nonzero(g["ipt_token"] != ref["ipt_token"])[0]
        excused = 0
        for r in diff:
            assert logits_host is not None, "ipt_token differs on row %d" % r
            T, seeds, seq_ids, positions = row_args
            Tr = float(T[r]) if np.ndim(T) else float(T)
            x = oracle.decode_row(np.ascontiguousarray(logits_host[r, :V]))
            alt = oracle.ipt_row(x, Tr, int(seeds[seq_ids[r]]), int(seq_ids[r]), int(positions[r]),
                                 int(g["ipt_token"][r]))
            # the GPU's token must own an interval that touches u within the tie width
            assert alt["dist"] < TIE_REL and alt["cdf_hi"] > alt["cdf_lo"], \
                "ipt_token differs on row %d beyond a near tie (oracle %d, gpu %d, dist %g)" % (
                    r, ref["ipt_token"][r], g["ipt_token"][r], alt["dist"])
            excused += 1
        stats["token_excused"] = excused
    if "log_mass" in g and log_mass_sigma is not None:
        # The bar is the reading taken for the printed score: |dS| <= 1e-4 max(1, |S|).  The log-mass is evaluated
        # in fp64 from the kernel's fp64 interval, whose position carries the error of the fp32 exponentials (da, a
        # few 1e-8 absolute) and whose width carries the relative error dw of one fp32 exponential; to first order
        #   dS = (phi(z_b) db - phi(z_a) da) / (sigma (mass + eps))  <~  dw + 4 da (1 + dist/sigma + width/sigma) / sigma.
        # A row beyond the bar is accepted only if that first-order error alone can exceed the bar there (a sigma
        # so small that the interval's fp32 position error shows), stays within it, and is counted.
        # One more term belongs to the definition itself: a and b are CDF values (the appendix takes them from
        # F = concat(0, cumsum p)), doubles of size up to 1 whose spacing is 1.1e-16; a claimed token of probability
        # 1e-14 has an interval that is a hundred such steps wide on either side of the comparison, so its width -
        # and with it the mass - is only good to a per cent, in the oracle as much as in the kernel.
        da, dw = 1e-7, 4e-6
        z = np.nan_to_num(ref["dist"], nan=0.0) / log_mass_sigma
        width = np.nan_to_num(ref["cdf_hi"] - ref["cdf_lo"], nan=0.0)
        zin = np.minimum(1.0, width) / log_mass_sigma
        # (a step on either end, on either side, and as much again where the two normal CDF values are subtracted)
        quant = np.where(width > 0.0, 4.5e-16 / np.maximum(width, 1e-300), 0.0)
        quant = np.where(width < 2e-15, np.inf, quant)  # under twenty steps wide: either side's width may round to 0
        first_order = dw + quant + 4.0 * da * (1.0 + z + zin) / log_mass_sigma
        gl, rl = g["log_mass"].astype(np.float64), ref["log_mass"]
        ok = ~(np.isnan(gl) & np.isnan(rl))
        err = np.where(ok, np.abs(gl - rl), 0.0)
        bar = 1e-4 * np.maximum(1.0, np.abs(np.nan_to_num(rl)))
        beyond = ~(err <= bar)
        allowed = (first_order > bar) & (err <= 1e-4 + first_order)
        worst = int(np.argmax(err - np.where(allowed, 1e-4 + first_order, bar)))
        assert not (beyond & ~allowed).any(), (
            "log_mass beyond its bar at row %d: gpu S %.9g oracle S %.9g bar %.3g; gpu a %.9g b %.9g u %.9g; "
            "oracle a %.12g b %.12g dist %.6g" % (worst, gl[worst], rl[worst], bar[worst], g["cdf_lo"][worst],
                                                   g["cdf_hi"][worst], g["u"][worst], ref["cdf_lo"][worst],
                                                   ref["cdf_hi"][worst], ref["dist"][worst]))
        stats["log_mass_beyond_bar"] = int(beyond.sum())
        stats["log_mass_interval_below_fp64_spacing"] = int(np.isinf(quant).sum())
        err = err[ok]
        stats["log_mass_err"] = float(err.max()) if err.size else 0.0
    d = g["dist"][~np.isnan(g["dist"])]
    assert (d >= 0).all() and (d < 1).all()
    return stats


def compare_seq(gpu: dict, ref: dict, tau: float, mismatch_slack: int = 0):
    """mismatch_slack: number of MATCH bits that the row comparison excused as near ties; the
    per-sequence mismatch counts may differ by that many in total."""
    g = _np(gpu)
    stats = {"seqs": ref["seq_mean"].shape[0]}
    stats["mean_err"] = _close(g["seq_mean"], ref["seq_mean"], ABS_TOL, "seq_mean")
    _close(g["seq_max"], ref["seq_max"], ABS_TOL, "seq_max")
    assert int(np.abs(g["seq_mismatch"].astype(np.int64) - ref["seq_mismatch"]).sum()) <= mismatch_slack
    near = np.abs(np.nan_to_num(ref["seq_mean"], nan=np.inf) - tau) <= TIE_REL * max(1.0, abs(tau))
    diff = g["seq_flag"] != ref["seq_flag"]
    assert not (diff & ~near).any(), "seq_flag differs outside near ties"
    stats["flag_excused"] = int(diff.sum())
    return stats
