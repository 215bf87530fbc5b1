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


def compare_records(gpu, ora, faults, exact_words=False, site_tol=0.0):
    """The parity rule: outside the oracle's guard bands, class and counters are equal; inside,
    they may differ by at most the number of borderline elements.  Returns a summary dict."""
    n = len(gpu)
    assert len(ora) == n
    clean = (ora["n_border_T"] == 0) & (ora["n_border_tau"] == 0)
    bad = []
    for t in range(n):
        g, o = gpu[t], ora[t]
        if int(g["status"]) != (0 if o["valid"] else 1):
            bad.append((t, "status", int(g["status"]), int(o["valid"])))
        dT, dtau = int(o["n_border_T"]), int(o["n_border_tau"])
        if abs(int(g["n_flagged"]) - int(o["n_flagged"])) > dT:
            bad.append((t, "n_flagged", int(g["n_flagged"]), int(o["n_flagged"])))
        if abs(int(g["n_dev_pre"]) - int(o["n_dev_pre"])) > dtau:
            bad.append((t, "n_dev_pre", int(g["n_dev_pre"]), int(o["n_dev_pre"])))
        if abs(int(g["n_dev_post"]) - int(o["n_dev_post"])) > dtau + dT:
            bad.append((t, "n_dev_post", int(g["n_dev_post"]), int(o["n_dev_post"])))
        if clean[t] and cls_of(gpu[t:t + 1])[0] != int(o["cls"]):
            bad.append((t, "cls", int(cls_of(gpu[t:t + 1])[0]), int(o["cls"])))
        kind = int(faults["kind"][t])
        if o["valid"] and kind != 0:
            if kind == 4:
                # product-term fault: the site words are the accumulator before and after the
                # write-back (acc - re) + re_err, with the same re and re_err on both sides
                w = [np.array([x], np.uint32).view(np.float32)[0] for x in
                     (g["site_word_before"], o["site_word_before"], g["site_word_after"], o["site_word_after"])]
                gb, ob, ga, oa = [float(x) for x in w]
                if exact_words:
                    if int(g["site_word_before"]) != int(o["site_word_before"]) or not (
                            int(g["site_word_after"]) == int(o["site_word_after"]) or (np.isnan(ga) and np.isnan(oa))):
                        bad.append((t, "site_words", gb, ob, ga, oa))
                else:
                    if not abs(gb - ob) <= site_tol:
                        bad.append((t, "site_word_before", gb, ob))
                    same_after = (np.isnan(ga) and np.isnan(oa)) or ga == oa or \
                        abs(ga - oa) <= site_tol + 1e-6 * max(1.0, abs(oa), abs(ob))
                    if not same_after:
                        bad.append((t, "site_word_after", ga, oa))
                continue
            if kind == 1 and not exact_words:
                # the two accumulators followed different summation orders: same value to within
                # the unfaulted tolerance, not the same bits
                gv = float(np.array([g["site_word_before"]], np.uint32).view(np.float32)[0])
                ov = float(np.array([o["site_word_before"]], np.uint32).view(np.float32)[0])
                if not abs(gv - ov) <= site_tol:
                    bad.append((t, "site_word_before", gv, ov))
            else:
                if int(g["site_word_before"]) != int(o["site_word_before"]) or \
                        int(g["site_word_after"]) != int(o["site_word_after"]):
                    bad.append((t, "site_words", hex(int(g["site_word_before"])), hex(int(o["site_word_before"]))))
            if (int(g["site_word_before"]) ^ int(g["site_word_after"])) != \
                    (int(faults["xor_mask"][t]) & (0xFFFFFFFF if kind == 1 else 0xFFFF)):
                bad.append((t, "xor", hex(int(g["site_word_before"])), hex(int(g["site_word_after"]))))
    gc, oc = cls_of(gpu), ora["cls"].astype(np.uint8)
    return dict(n=n, borderline=int((~clean).sum()), mismatches=bad,
                gpu_counts=[int((gc == c).sum()) for c in range(3)],
                oracle_counts=[int((oc == c).sum()) for c in range(3)])
