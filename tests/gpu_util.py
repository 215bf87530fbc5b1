"""Helpers shared by the GPU parity tests: run a campaign through the C-ABI binding and
through the oracle on the same seeded inputs."""
import numpy as np

from oracle import pyoracle as orc
from paper_2311_05782_amd import fi


def make_plan(Aw, Bw, kb, fmt, cfg=None, group=None, **kw):
    M, K = Aw.shape
    N = Bw.shape[1] if kw.get("b_layout", 0) == 1 else Bw.shape[0]
    d_A, d_B = fi.words_to_device(Aw), fi.words_to_device(Bw)
    desc = fi.plan_desc(M, N, K, kb, fmt, **kw)
    plan = fi.Plan(desc, d_A, d_B)
    if cfg is not None or group is not None:
        plan.tune(-1 if cfg is None else cfg, -1 if group is None else group)
    return plan


def gpu_campaign(plan, faults, policy, want_c=False):
    import torch
    n = len(faults)
    d = plan.desc
    d_f = fi.to_device(faults)
    d_r = fi.empty_results(n)
    d_c = torch.empty((n, d.M, d.N), dtype=torch.float32, device="cuda") if want_c else None
    plan.fi_gemm_inject_batch(d_f, n, policy, d_r, d_c)
    recs = fi.results_to_host(d_r)
    return (recs, d_c.cpu().numpy()) if want_c else recs


def gpu_classify(plan, recs_dev, n):
    import torch
    d_cls = torch.empty(n, dtype=torch.uint8, device="cuda")
    d_cnt = torch.empty(3, dtype=torch.int64, device="cuda")
    plan.fi_classify(recs_dev, n, d_cls, d_cnt)
    torch.cuda.synchronize()
    return d_cls.cpu().numpy(), d_cnt.cpu().numpy().astype(np.uint64)


def cls_of(recs):
    return np.where(recs["n_flagged"] > 0, 2, np.where(recs["n_dev_pre"] > 0, 1, 0)).astype(np.uint8)


def to_orc_faults(f):
    out = np.zeros(len(f), orc.FAULT_DTYPE)
    for k in ("kind", "row", "col", "kblock", "xor_mask"):
        out[k] = f[k]
    return out


def class_is_certain(o):
    """True if the borderline elements the oracle counted cannot change the trial's class: enough
    flags stand outside the band around T, or nothing is near T and the count of deviating
    elements cannot reach or leave zero."""
    if int(o["n_flagged"]) > int(o["n_border_T"]):
        return True                                          # detected whatever the band holds
    if int(o["n_flagged"]) == 0 and int(o["n_border_T"]) == 0:
        if int(o["n_dev_pre"]) > int(o["n_border_tau"]):
            return True                                      # SDC for sure
        if int(o["n_dev_pre"]) == 0 and int(o["n_border_tau"]) == 0:
            return True                                      # masked for sure
    return False


def site_tolerances(faults, Af, Bf):
    """Per trial, 2^-12 * sum_k |a_ik b_kj| of the faulted output element (accumulator and
    product-term faults; 0 elsewhere), in float64 from the decoded operands Af [M][K], Bf [N][K]."""
    tol = np.zeros(len(faults))
    for t in range(len(faults)):
        if int(faults["kind"][t]) in (1, 4):
            i, j = int(faults["row"][t]), int(faults["col"][t])
            if i < Af.shape[0] and j < Bf.shape[0]:
                tol[t] = 2.0 ** -12 * float(np.abs(Af[i].astype(np.float64)) @ np.abs(Bf[j].astype(np.float64)))
    return tol


def _f32(word):
    return float(np.array([word], np.uint32).view(np.float32)[0])


def compare_records(gpu, ora, faults, exact_words=False, site_tol=0.0, operands=None):
    """The parity rule: outside the oracle's guard bands, class and counters are equal; inside,
    they may differ by at most the number of borderline elements; the class is compared for every
    trial whose borderline elements cannot change it.  With `operands` = (Af, Bf), the decoded
    operands, the accumulator word at the site is compared within ITS element's tolerance
    2^-12 * S_ij (else within the scalar site_tol) and the largest deviations are compared too.
    Returns a summary dict."""
    n = len(gpu)
    assert len(ora) == n
    clean = (ora["n_border_T"] == 0) & (ora["n_border_tau"] == 0)
    tols = site_tolerances(faults, *operands) if operands is not None else np.full(n, float(site_tol))
    bad = []
    n_certain = 0
    for t in range(n):
        g, o = gpu[t], ora[t]
        stol = float(tols[t])
        if int(g["status"]) != (0 if o["valid"] else 1):
            bad.append((t, "status", int(g["status"]), int(o["valid"])))
        dT, dtau = int(o["n_border_T"]), int(o["n_border_tau"])
        if abs(int(g["n_flagged"]) - int(o["n_flagged"])) > dT:
            bad.append((t, "n_flagged", int(g["n_flagged"]), int(o["n_flagged"])))
        if abs(int(g["n_dev_pre"]) - int(o["n_dev_pre"])) > dtau:
            bad.append((t, "n_dev_pre", int(g["n_dev_pre"]), int(o["n_dev_pre"])))
        if abs(int(g["n_dev_post"]) - int(o["n_dev_post"])) > dtau + dT:
            bad.append((t, "n_dev_post", int(g["n_dev_post"]), int(o["n_dev_post"])))
        if class_is_certain(o):
            n_certain += 1
            if cls_of(gpu[t:t + 1])[0] != int(o["cls"]):
                bad.append((t, "cls", int(cls_of(gpu[t:t + 1])[0]), int(o["cls"])))
        kind = int(faults["kind"][t])
        if operands is not None and clean[t] and o["valid"] and kind in (1, 4):
            # Largest deviation of a one-element fault: both sides subtract their own fault-free
            # value from their own faulty one; the two pairs differ by the element's tolerance
            # each, and a flipped exponent bit scales the difference of the accumulators at the
            # site by what it scaled the accumulator by.
            before, after = abs(_f32(o["site_word_before"])), abs(_f32(o["site_word_after"]))
            scale = after / before if before > 0 and np.isfinite(after) else 1.0
            # two accumulators that may sit on either side of a power of two react differently to
            # a flipped exponent bit: nothing to compare then
            straddle = before > 0 and np.frexp(max(before - 2 * stol, 1e-300))[1] != np.frexp(before + 2 * stol)[1]
            for k in (() if straddle else ("max_dev_pre", "max_dev_post")):
                gv, ov = float(g[k]), float(o[k])
                if np.isfinite(ov) and np.isfinite(scale):
                    if not abs(gv - ov) <= 2.0 * stol * (1.0 + scale) + 2.0 ** -20 * abs(ov):
                        bad.append((t, k, gv, ov, stol, scale))
                elif np.isfinite(gv) and not np.isfinite(ov):
                    bad.append((t, k, gv, ov))
        if o["valid"] and kind != 0:
            if kind == 4:
                # product-term fault: the site words are the accumulator before and after the
                # write-back (acc - re) + re_err, with the same re and re_err on both sides
                gb, ob, ga, oa = [_f32(x) for x in (g["site_word_before"], o["site_word_before"],
                                                    g["site_word_after"], o["site_word_after"])]
                if exact_words:
                    if int(g["site_word_before"]) != int(o["site_word_before"]) or not (
                            int(g["site_word_after"]) == int(o["site_word_after"]) or (np.isnan(ga) and np.isnan(oa))):
                        bad.append((t, "site_words", gb, ob, ga, oa))
                else:
                    if not abs(gb - ob) <= stol:
                        bad.append((t, "site_word_before", gb, ob))
                    same_after = (np.isnan(ga) and np.isnan(oa)) or ga == oa or \
                        abs(ga - oa) <= stol + 1e-6 * max(1.0, abs(oa), abs(ob))
                    if not same_after:
                        bad.append((t, "site_word_after", ga, oa))
                continue
            if kind == 1 and not exact_words:
                # the two accumulators followed different summation orders: same value to within
                # the unfaulted tolerance of the element, not the same bits
                gv, ov = _f32(g["site_word_before"]), _f32(o["site_word_before"])
                if not abs(gv - ov) <= stol:
                    bad.append((t, "site_word_before", gv, ov, stol))
            else:
                if int(g["site_word_before"]) != int(o["site_word_before"]) or \
                        int(g["site_word_after"]) != int(o["site_word_after"]):
                    bad.append((t, "site_words", hex(int(g["site_word_before"])), hex(int(o["site_word_before"]))))
            if (int(g["site_word_before"]) ^ int(g["site_word_after"])) != \
                    (int(faults["xor_mask"][t]) & (0xFFFFFFFF if kind == 1 else 0xFFFF)):
                bad.append((t, "xor", hex(int(g["site_word_before"])), hex(int(g["site_word_after"]))))
    gc, oc = cls_of(gpu), ora["cls"].astype(np.uint8)
    return dict(n=n, borderline=int((~clean).sum()), certain=n_certain, mismatches=bad,
                gpu_counts=[int((gc == c).sum()) for c in range(3)],
                oracle_counts=[int((oc == c).sum()) for c in range(3)])
