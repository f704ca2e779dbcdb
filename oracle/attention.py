"""FP8 dot-product attention, forward and backward, one (batch, head) at a time.

Appendix B defines a head as selfattn = P V with P = Softmax(s Q K^T + M)
(M the causal mask); the table of FP8 methods in Appendix E says that under
FP8DPA both Q K^T and P V are FP8 products, and Section 2 assigns E4M3 to
forward tensors and E5M2 to backward tensors.  The paper gives no kernel-level
detail; the steps below fix the readings (each listed in the design notes):

  * logits are taken in the log2 domain, x = s * log2(e) * (Q K^T);
  * forward: the row reference is the INTEGER M_i = ceil(max_j x_ij); the
    un-normalised p_ij = 2^(x_ij - M_i) is what is cast to E4M3 (times rho_P);
    the row sum l_i uses the un-quantised p;
  * backward: the normalised P_ij = 2^(x_ij - LSE_i) is cast to E4M3 for the dV
    product; dS = P o (dP - D) uses the un-quantised P and is cast to E5M2;
    D_i = sum_d dO_id O_id from the bf16 tensors.

With fp8_p=False / fp8_ds=False the casts of P and dS are skipped: that mode is
plain softmax attention on the decoded operands and pins the formulas.
"""
import numpy as np

from . import bf16, fp8

LOG2E = 1.4426950408889634


def logits(Q8, K8, sinv_q, sinv_k, softmax_scale, causal):
    """x = s log2(e) sinv_q sinv_k (Q~ K~^T) in float64, masked entries -inf (Appendix B: s Q K^T + M)."""
    q = fp8.decode(Q8, fp8.E4M3)
    k = fp8.decode(K8, fp8.E4M3)
    c = np.float64(softmax_scale) * LOG2E * np.float64(sinv_q) * np.float64(sinv_k)
    x = c * (q @ k.T)
    if causal:
        S = x.shape[0]
        i = np.arange(S)[:, None]
        j = np.arange(x.shape[1])[None, :]
        x = np.where(j > i, -np.inf, x)
    return x


def attn_fwd_head(Q8, K8, V8, sinv_q, sinv_k, sinv_v, softmax_scale, scale_p, causal=True, fp8_p=True):
    """Returns (O float64 [S,D], LSE float64 [S] in the log2 domain, amax of p)."""
    x = logits(Q8, K8, sinv_q, sinv_k, softmax_scale, causal)
    M = np.ceil(x.max(axis=1, keepdims=True))
    p = np.exp2(x - M)
    l = p.sum(axis=1, keepdims=True)
    v = fp8.decode(V8, fp8.E4M3)
    rho_p = np.float64(scale_p)
    if fp8_p:
        t = (rho_p * p).astype(np.float32)           # one binary32 rounding of rho_P * p
        pq = fp8.decode(fp8.encode_sat(t, fp8.E4M3), fp8.E4M3)
    else:
        pq = rho_p * p
    O = np.float64(sinv_v) * (pq @ v) / (rho_p * l)
    lse = (M + np.log2(l))[:, 0]
    return O, lse, np.float32(p.max())


def attn_bwd_head(Q8, K8, V8, sinv_q, sinv_k, sinv_v, O_bits, dO_bits, dO8, sinv_do, lse,
                  softmax_scale, scale_p, scale_ds, causal=True, fp8_p=True, fp8_ds=True):
    """Returns (dQ, dK, dV float64 [S,D], amax of dS)."""
    x = logits(Q8, K8, sinv_q, sinv_k, softmax_scale, causal)
    P = np.exp2(x - np.asarray(lse, dtype=np.float64)[:, None])
    o = bf16.bits_to_f64(O_bits)
    do_hi = bf16.bits_to_f64(dO_bits)
    Dv = (do_hi * o).sum(axis=1, keepdims=True)
    q = fp8.decode(Q8, fp8.E4M3)
    k = fp8.decode(K8, fp8.E4M3)
    v = fp8.decode(V8, fp8.E4M3)
    do = fp8.decode(dO8, fp8.E5M2)
    rho_p, rho_ds = np.float64(scale_p), np.float64(scale_ds)
    if fp8_p:
        pq = fp8.decode(fp8.encode_sat((rho_p * P).astype(np.float32), fp8.E4M3), fp8.E4M3)
    else:
        pq = rho_p * P
    dV = (np.float64(sinv_do) / rho_p) * (pq.T @ do)
    dP = np.float64(sinv_do) * np.float64(sinv_v) * (do @ v.T)
    dS = P * (dP - Dv)                               # masked entries have P = 0
    if fp8_ds:
        dsq = fp8.decode(fp8.encode_sat((rho_ds * dS).astype(np.float32), fp8.E5M2), fp8.E5M2)
    else:
        dsq = rho_ds * dS
    s = np.float64(softmax_scale)
    dQ = (s * np.float64(sinv_k) / rho_ds) * (dsq @ k)
    dK = (s * np.float64(sinv_q) / rho_ds) * (dsq.T @ q)
    return dQ, dK, dV, np.float32(np.abs(dS).max())
