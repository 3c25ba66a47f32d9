"""A float (binary64) Swin block written with numpy, independent of the oracle.

It is the textbook the oracle is pinned to: attention is taken DENSELY over all
tokens of the padded map with an explicit "may attend" predicate instead of
going through window partition / roll / mask tables, and nothing is quantized
(weights are the dequantized int8 codes).  Per-window branch parameters are
honoured (the LayerNorms and biases of the branch a window belongs to).
"""
import numpy as np
from scipy.special import erf


def _ln(v, g, b, eps):
    mu = v.mean(-1, keepdims=True)
    var = ((v - mu) ** 2).mean(-1, keepdims=True)
    return (v - mu) / np.sqrt(var + eps) * g + b


def float_block(inp, x, branch_of_window, shift=None, return_intermediates=False):
    """x [B,H,W,C]; branch_of_window [B,nW] in {0,1}, indexed by window number of
    the (rolled) grid.  Returns y [B,H,W,C] float64."""
    spec, sh = inp.spec, inp.shared
    s = spec.shift if shift is None else shift
    ws, Cc, nh = spec.window, spec.C, spec.heads
    hd = Cc // nh
    Hp, Wp = spec.Hp, spec.Wp
    Wq = sh.w_qkv.astype(np.float64) * sh.s_qkv[:, None].astype(np.float64)
    Wo = sh.w_proj.astype(np.float64) * sh.s_proj[:, None].astype(np.float64)
    W1 = sh.w_fc1.astype(np.float64) * sh.s_fc1[:, None].astype(np.float64)
    W2 = sh.w_fc2.astype(np.float64) * sh.s_fc2[:, None].astype(np.float64)
    rr, cc = np.meshgrid(np.arange(Hp), np.arange(Wp), indexing="ij")
    rr, cc = rr.ravel(), cc.ravel()                       # original padded coordinates of every token
    ro, co = (rr - s) % Hp, (cc - s) % Wp                 # coordinates after rolling by -s
    win = (ro // ws) * (Wp // ws) + (co // ws)            # window of the rolled grid
    tok = (ro % ws) * ws + (co % ws)                      # index inside that window
    inside = (rr < spec.H) & (cc < spec.W)
    allowed = (win[:, None] == win[None, :]) & (np.abs(rr[:, None] - rr[None, :]) < ws) & \
              (np.abs(cc[:, None] - cc[None, :]) < ws)
    same_window = win[:, None] == win[None, :]
    ys = np.zeros((spec.B, spec.H, spec.W, Cc))
    inter = []
    for b in range(spec.B):
        xp = np.zeros((Hp, Wp, Cc))
        xp[:spec.H, :spec.W] = x[b].astype(np.float64)
        xt = xp.reshape(-1, Cc)
        br = np.asarray(branch_of_window[b])[win]         # branch of every token
        P = [inp.branches[0], inp.branches[1]]
        pick = lambda name: np.where(br[:, None] == 0, getattr(P[0], name)[None, :].astype(np.float64),
                                     getattr(P[1], name)[None, :].astype(np.float64))
        ln1 = _ln(xt, pick("ln1_gamma"), pick("ln1_beta"), spec.ln_eps) * inside[:, None]
        qkv = ln1 @ Wq.T + pick("b_qkv")
        q, k, v = qkv[:, :Cc], qkv[:, Cc:2 * Cc], qkv[:, 2 * Cc:]
        att = np.zeros_like(q)
        probs = []
        for h in range(nh):
            sl = slice(h * hd, (h + 1) * hd)
            lg = q[:, sl] @ k[:, sl].T / np.sqrt(hd) + sh.rel_pos_bias[h].astype(np.float64)[tok[:, None], tok[None, :]]
            lg = np.where(allowed, lg, np.where(same_window, lg - 100.0, -np.inf))
            lg -= lg.max(-1, keepdims=True)
            e = np.exp(lg)
            p = e / e.sum(-1, keepdims=True)
            att[:, sl] = p @ v[:, sl]
            probs.append(p)
        hres = att @ Wo.T + pick("b_proj") + xt
        ln2 = _ln(hres, pick("ln2_gamma"), pick("ln2_beta"), spec.ln_eps)
        f1 = ln2 @ W1.T + pick("b_fc1")
        gl = 0.5 * f1 * (1.0 + erf(f1 / np.sqrt(2.0)))
        out = gl @ W2.T + pick("b_fc2") + hres
        ys[b] = out.reshape(Hp, Wp, Cc)[:spec.H, :spec.W]
        inter.append(dict(ln1=ln1, q=q, k=k, v=v, p=np.stack(probs), att=att, hres=hres, ln2=ln2, f1=f1, gelu=gl,
                          inside=inside, br=br))
    return (ys, inter) if return_intermediates else ys


def sqnr_db(ref, test):
    ref = np.asarray(ref, dtype=np.float64)
    err = ref - np.asarray(test, dtype=np.float64)
    return 10.0 * np.log10((ref ** 2).sum() / max((err ** 2).sum(), 1e-300))
