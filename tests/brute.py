"""Literal nested-loop evaluation of the gated layer for tiny shapes.

Written independently of ``oracle/cg_ref.c`` (pure Python scalars, fractions for
the float path so that no rounding order is involved) and used only to pin it.
Follows Eq. 1 and the merged gate of Sec. 3.2 of the channel-gating paper.
"""
from fractions import Fraction


def gated_conv_brute(x, w_base, w_cond, stride, pad, thr, exact=True, groups=1, tau_c=0):
    """x: nested list [N][H][W][C]; w_base [CO][KH][KW][CP]; w_cond [CO][KH][KW][CR];
    thr: per-channel threshold on the raw partial sum (gate fires iff P >= thr[co]).
    groups > 1 (Sec. 3.3): the output channels are cut into `groups` equal runs; run i reads
    input channels [i*CP, (i+1)*CP) on the base path and all the others, in order, on the
    conditional path.
    tau_c > 0 (channel-wise gate of Sec. 3.2): an output channel of an image whose fired count is
    below tau_c * HO * WO loses its conditional path altogether.
    Returns P, R, d, S as nested lists [N][HO][WO][CO] (Fractions if exact)."""
    conv = Fraction if exact else (lambda v: v)
    N, H, W = len(x), len(x[0]), len(x[0][0])
    CO, KH, KW = len(w_base), len(w_base[0]), len(w_base[0][0])
    CP = len(w_base[0][0][0])
    CR = len(w_cond[0][0][0]) if w_cond is not None else 0
    HO = (H + 2 * pad - KH) // stride + 1
    WO = (W + 2 * pad - KW) // stride + 1
    P = [[[[0] * CO for _ in range(WO)] for _ in range(HO)] for _ in range(N)]
    R = [[[[0] * CO for _ in range(WO)] for _ in range(HO)] for _ in range(N)]
    D = [[[[0] * CO for _ in range(WO)] for _ in range(HO)] for _ in range(N)]
    S = [[[[0] * CO for _ in range(WO)] for _ in range(HO)] for _ in range(N)]
    for n in range(N):
        for oh in range(HO):
            for ow in range(WO):
                for co in range(CO):
                    own = co // (CO // groups) if groups > 1 else 0
                    base_ch = [own * CP + c for c in range(CP)]
                    cond_ch = [c for c in range(CP + CR) if c not in base_ch]
                    p = conv(0)
                    q = conv(0)
                    for kh in range(KH):
                        for kw in range(KW):
                            ih = oh * stride + kh - pad
                            iw = ow * stride + kw - pad
                            if not (0 <= ih < H and 0 <= iw < W):
                                continue
                            for c, ch in enumerate(base_ch):
                                p += conv(x[n][ih][iw][ch]) * conv(w_base[co][kh][kw][c])
                            for c, ch in enumerate(cond_ch):
                                q += conv(x[n][ih][iw][ch]) * conv(w_cond[co][kh][kw][c])
                    fire = 1 if (CR == 0 or p >= thr[co]) else 0
                    P[n][oh][ow][co] = p
                    R[n][oh][ow][co] = q
                    D[n][oh][ow][co] = fire if CR else 0
                    S[n][oh][ow][co] = p + q if fire else p
    if tau_c and CR:
        for n in range(N):
            for co in range(CO):
                fired = sum(D[n][oh][ow][co] for oh in range(HO) for ow in range(WO))
                if fired < Fraction(tau_c) * HO * WO:
                    for oh in range(HO):
                        for ow in range(WO):
                            D[n][oh][ow][co] = 0
                            S[n][oh][ow][co] = P[n][oh][ow][co]
    return P, R, D, S
