"""A second, independent statement of one trial, in NumPy float32 scalar steps.

Used only on tiny shapes to cross-check the C oracle by brute force.  It is
written against the paper (Sec. II-A formats, Sec. IV-C fault model, Sec. VI-A
range argument) and deliberately shares nothing with oracle/: operands are
decoded with NumPy's own float16 type and the "bfloat16 is the top half of a
binary32" identity, accumulation uses np.float32 scalars, the accumulator word
is flipped through a uint32 view.  Product-term faults (Sec. III-E write-back)
round the product to the operand format with NumPy's own float32 -> float16
conversion, or for BF16 with the add-half-then-truncate integer identity.
"""
import numpy as np

FP16, BF16 = 0, 1
NONE, ACC, SITE_A, SITE_B, PRODUCT = 0, 1, 2, 3, 4
C_NONE, C_ZERO, C_RECOMPUTE = 0, 1, 2


def decode(words, fmt):
    words = np.asarray(words, np.uint16)
    if fmt == FP16:
        return words.view(np.float16).astype(np.float32)
    return (words.astype(np.uint32) << 16).view(np.float32)


def flip(x, mask):
    w = np.array([x], np.float32).view(np.uint32)
    before = int(w[0])
    w[0] ^= np.uint32(mask)
    return w.view(np.float32)[0], before, int(w[0])


def to_format(x, fmt):
    """float32 scalar -> 16-bit word of the operand format, round to nearest even."""
    x = np.float32(x)
    with np.errstate(all="ignore"):
        if fmt == FP16:
            return int(np.array([x], np.float32).astype(np.float16).view(np.uint16)[0])
        bits = int(np.array([x], np.float32).view(np.uint32)[0])
        if np.isnan(x):
            return ((bits >> 16) & 0x8000) | 0x7FC0
        return ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) & 0xFFFF


def dot(a, b, kb, fault_s=-1, mask=0, prod_k=-1, prod_mask=0, fmt=FP16):
    """a, b: float32 vectors.  Returns (value, word_before, word_after).
    prod_k >= 0: product-term fault - after the 16-term step holding prod_k the accumulator
    becomes (acc - re) + re_err, re = the product in the operand format."""
    acc = np.float32(0.0)
    wb = wa = 0
    with np.errstate(all="ignore"):
        for s in range(len(a) // kb):
            for k in range(s * kb, (s + 1) * kb):
                acc = np.float32(acc + np.float32(a[k] * b[k]))
                if prod_k >= 0 and k == 16 * (prod_k // 16) + 15:
                    w = to_format(np.float32(a[prod_k] * b[prod_k]), fmt)
                    re = decode(np.array([w], np.uint16), fmt)[0]
                    re_err = decode(np.array([w ^ (prod_mask & 0xFFFF)], np.uint16), fmt)[0]
                    wb = int(np.array([acc], np.float32).view(np.uint32)[0])
                    acc = np.float32(np.float32(acc - re) + re_err)
                    wa = int(np.array([acc], np.float32).view(np.uint32)[0])
            if s == fault_s:
                acc, wb, wa = flip(acc, mask)
    return acc, wb, wa


def run_trial(Aw, Bw, fmt, kb, fault, policy, gamma=np.float32(1 + 2.0 ** -11), bound_global=False):
    """Aw [M,K], Bw [N,K] uint16 words.  fault = (kind,row,col,kblock,mask).
    Returns dict with C_star, C_f, C_c, flags and the counters."""
    kind, row, col, s, mask = fault
    A = decode(Aw, fmt)
    Bt = decode(Bw, fmt)
    M, K = A.shape
    N = Bt.shape[0]
    ra = np.abs(A).max(axis=1)
    cb = np.abs(Bt).max(axis=1)
    Af, Btf = A.copy(), Bt.copy()
    wb = wa = 0
    if kind == SITE_A:
        w = int(Aw[row, col]); wb, wa = w, w ^ (mask & 0xFFFF)
        Af[row, col] = decode(np.array([wa], np.uint16), fmt)[0]
    elif kind == SITE_B:
        w = int(Bw[col, row]); wb, wa = w, w ^ (mask & 0xFFFF)
        Btf[col, row] = decode(np.array([wa], np.uint16), fmt)[0]
    Cs = np.zeros((M, N), np.float32)
    Cf = np.zeros((M, N), np.float32)
    S = np.zeros((M, N), np.float64)
    for i in range(M):
        for j in range(N):
            Cs[i, j] = dot(A[i], Bt[j], kb)[0]
            if kind == ACC and i == row and j == col:
                Cf[i, j], wb, wa = dot(Af[i], Btf[j], kb, s, mask)
            elif kind == PRODUCT and i == row and j == col:
                Cf[i, j], wb, wa = dot(Af[i], Btf[j], kb, prod_k=s, prod_mask=mask, fmt=fmt)
            else:
                Cf[i, j] = dot(Af[i], Btf[j], kb)[0]
            S[i, j] = np.abs(A[i].astype(np.float64) * Bt[j].astype(np.float64)).sum()
    Kf = np.float32(K)
    if bound_global:
        T = np.full((M, N), np.float32(np.float32(np.float32(Kf * ra.max()) * cb.max()) * gamma), np.float32)
    else:
        T = ((Kf * ra).astype(np.float32)[:, None] * cb[None, :]).astype(np.float32)
        T = (T * np.float32(gamma)).astype(np.float32)
    with np.errstate(all="ignore"):
        flags = ~(np.abs(Cf) <= T)
        Cc = Cf.copy()
        if policy == C_ZERO:
            Cc[flags] = np.float32(0)
        elif policy == C_RECOMPUTE:
            Cc[flags] = Cs[flags]
        tau = S * 2.0 ** -12
        dpre = np.abs(Cf.astype(np.float64) - Cs.astype(np.float64))
        dpost = np.abs(Cc.astype(np.float64) - Cs.astype(np.float64))
        dpre[~np.isfinite(dpre)] = np.inf
        dpost[~np.isfinite(dpost)] = np.inf
    out = dict(C_star=Cs, C_f=Cf, C_c=Cc, flags=flags, T=T, tau=tau,
               n_flagged=int(flags.sum()),
               n_bitdiff=int((Cf.view(np.uint32) != Cs.view(np.uint32)).sum()),
               n_dev_pre=int((~(dpre <= tau)).sum()),
               n_dev_post=int((~(dpost <= tau)).sum()),
               max_dev_pre=float(dpre.max()), max_dev_post=float(dpost.max()),
               site_word_before=wb, site_word_after=wa)
    out["cls"] = 2 if out["n_flagged"] else (1 if out["n_dev_pre"] else 0)
    return out
