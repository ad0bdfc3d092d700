"""A numpy model of the sweep kernel's arithmetic (test helper, CPU only; shares no code with the HIP library).

It replays the column sweep with the ORACLE's codes, scales and zero-points forced, so that rows never diverge, in the
precision the kernel works in, and returns the value before rounding, t = w / s + z, for every entry; the deviation
from the float64 oracle's t is what decides how often a code falls the other way at a near-tie (probability about
twice the mean absolute deviation per entry).  Two designs:
  "w32"   the compensated weight itself is held in fp32: the working copy in memory, the accumulators of the MFMA
          chains (initialized with it) and the registers of the sequential part;
  "split" what the library does: the original weight and the feedback sum c are kept apart, c in fp32, every MFMA chain
          accumulates from zero and is added to c once, and inside a 32-column inner block w = w0 + c, the decision and
          the feedback are fp64.
MFMA accumulation as measured on gfx950 with an in-bounds probe: v_mfma_f32_32x32x16_f16 adds the products of k 0..7
and of k 8..15 to the accumulator in two steps, each rounded to fp32 (half to even); v_mfma_f32_32x32x2_f32 rounds
after each k.  Operands across blocks are two fp16 halves (hi = rne(x), lo = rne(x - hi)) of the residual and of
U_jk / U_jj after power-of-two scalings, three products (lo*hi, hi*lo, hi*hi)."""
import numpy as np

f32 = np.float32
OPT = {"split": True, "mfma_round": True, "c_round": True, "third": False}


def split16(x):
    x = np.clip(x.astype(f32), -60000, 60000)
    if not OPT["split"]:
        return x.astype(np.float64), np.zeros(x.shape)
    h = x.astype(np.float16)
    l = (x - h.astype(f32)).astype(np.float16)
    return h.astype(np.float64), l.astype(np.float64)


def mfma16(acc, A_h, A_l, B_h, B_l):
    """acc (rows x cols, f32) += sum over k (multiple of 16) of the three split products, two roundings per 16-k step and product."""
    K = A_h.shape[1]
    if not OPT["mfma_round"]:
        return (acc.astype(np.float64) + A_l @ B_h + A_h @ B_l + A_h @ B_h + (A_l @ B_l if OPT["third"] else 0.0))
    for k0 in range(0, K, 16):
        for (A, B) in ((A_l, B_h), (A_h, B_l), (A_h, B_h)):
            for h in (0, 8):
                acc = (acc.astype(np.float64) + A[:, k0 + h:k0 + h + 8] @ B[k0 + h:k0 + h + 8, :]).astype(f32)
    return acc


def run(W, U, bits, G, o, design, SB=128, SBIG=512):
    rows, d_in = W.shape
    qmax = 2 ** bits - 1
    Q = o["Q"].astype(np.float64)
    S = o["scales"]; Z = o["zeros"]
    T = np.zeros((rows, d_in))
    maxw = np.abs(W).max()
    Un = np.triu(U, 1) / np.diag(U)[:, None]
    maxu = np.abs(Un).max()
    ew = np.frexp(maxw)[1]; eu = np.frexp(maxu)[1]
    f_d = 2.0 ** (13 - ew); f_u = 2.0 ** (14 - eu); f_all = f_d * f_u; f_inv = 1.0 / f_all
    Unf = (U.astype(f32) / np.diag(U).astype(f32)[:, None] * f32(f_u)).astype(f32)   # fp32 division then scale, as the kernel
    Uh, Ul = split16(np.triu(Unf, 1))
    if design == "w32":
        C = W.astype(f32).copy()           # working copy holds w itself
    else:
        C = np.zeros((rows, d_in), dtype=f32)
    U32 = U.astype(f32)
    for s0 in range(0, d_in, SBIG):
        s1 = min(d_in, s0 + SBIG)
        Dh = np.zeros((rows, s1 - s0)); Dl = np.zeros((rows, s1 - s0))
        for j0 in range(s0, s1, SB):
            # near update from the earlier blocks of the super-block
            if design == "w32":
                acc = (C[:, j0:j0 + SB].astype(np.float64) * f_all).astype(f32)
            else:
                acc = np.zeros((rows, SB), dtype=f32)
            if j0 > s0:
                acc = mfma16(acc, Dh[:, :j0 - s0], Dl[:, :j0 - s0], Uh[s0:j0, j0:j0 + SB], Ul[s0:j0, j0:j0 + SB])
            if design == "w32":
                sW = (acc.astype(np.float64) * f_inv).astype(f32) if j0 > s0 else C[:, j0:j0 + SB].copy()
            else:
                sC = (acc.astype(np.float64) * f_inv + C[:, j0:j0 + SB].astype(np.float64)).astype(f32)
            E32 = np.zeros((rows, SB), dtype=f32)
            for jb in range(0, SB, 32):
                if design == "w32":
                    w = sW[:, jb:jb + 32].copy()       # f32 registers
                else:
                    w = W[:, j0 + jb:j0 + jb + 32] + sC[:, jb:jb + 32].astype(np.float64)
                for j in range(32):
                    col = j0 + jb + j
                    g = col // G
                    s = S[:, g]; z = Z[:, g]
                    q = Q[:, col]
                    if design == "w32":
                        s32 = s.astype(f32); rs = (f32(1) / s32).astype(f32)
                        T[:, col] = (w[:, j] * rs).astype(np.float64) + z
                        wh = (s32 * (q - z).astype(f32)).astype(f32)
                        rd = (f32(1) / U32[col, col]).astype(f32)
                        e = ((w[:, j] - wh).astype(f32) * rd).astype(f32)
                        # fp32 FMA: one rounding
                        w[:, j + 1:] = (w[:, j + 1:].astype(np.float64) - e.astype(np.float64)[:, None] * U[col, col + 1:j0 + jb + 32][None, :]).astype(f32)
                        E32[:, jb + j] = e
                    else:
                        T[:, col] = w[:, j] * (1.0 / s) + z
                        resid = w[:, j] - s * (q - z)
                        e = resid * (1.0 / U[col, col])
                        w[:, j + 1:] -= e[:, None] * U[col, col + 1:j0 + jb + 32][None, :]
                        E32[:, jb + j] = e.astype(f32)
                # inner update of the rest of the block: fp32 MFMA, one rounding per k
                cs = jb + 32
                if cs < SB:
                    if design == "w32":
                        acc2 = sW[:, cs:].copy()
                    else:
                        acc2 = np.zeros((rows, SB - cs), dtype=f32)
                    for k in range(32):
                        acc2 = (acc2.astype(np.float64) - E32[:, jb + k].astype(np.float64)[:, None] * U[j0 + jb + k, j0 + cs:j0 + SB][None, :]).astype(f32)
                    if design == "w32":
                        sW[:, cs:] = acc2
                    else:
                        sC[:, cs:] = (sC[:, cs:].astype(np.float64) + acc2.astype(np.float64)).astype(f32)
            # residual panel of the block: -(e U_jj) f_d split
            ujj = (np.diag(U32)[j0:j0 + SB] * f32(f_d)).astype(f32)
            x = (-(E32 * ujj[None, :])).astype(f32)
            h, l = split16(x)
            Dh[:, j0 - s0:j0 - s0 + SB] = h; Dl[:, j0 - s0:j0 - s0 + SB] = l
        # far update of everything beyond the super-block
        if s1 < d_in:
            if design == "w32":
                acc = (C[:, s1:].astype(np.float64) * f_all).astype(f32)
                acc = mfma16(acc, Dh, Dl, Uh[s0:s1, s1:], Ul[s0:s1, s1:])
                C[:, s1:] = (acc.astype(np.float64) * f_inv).astype(f32)
            else:
                acc = np.zeros((rows, d_in - s1), dtype=f32)
                acc = mfma16(acc, Dh, Dl, Uh[s0:s1, s1:], Ul[s0:s1, s1:])
                C[:, s1:] = (C[:, s1:].astype(np.float64) + acc.astype(np.float64) * f_inv).astype(f32)
    return T


