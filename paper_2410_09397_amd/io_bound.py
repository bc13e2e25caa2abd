"""The paper's I/O bounds evaluated for a workload: the yardstick for measured HBM bytes.

arXiv 2410.09397: Theorem 1.1 / Table 1 (Q, K, V form, n >= d): the backward (and forward) I/O
complexity is Theta(n^2 d^2 / M) for a cache of M = Omega(d^2) items and Theta(n^2 d / sqrt(M))
for M = o(d^2); Theorem 4.5 (sparse): Omega(min{Z_in^2 / M, Z_in sqrt(Z_QK) / sqrt(M)}).
M counts items, so a byte budget is divided by the element size.  The constant inside Theta is
taken as 1, the causal mask counts half of n^2, and the bound is floored by the compulsory
traffic (with a cache of Theta(nd) the I/O is the input plus output size, Sec. 5).
"""
import math

# Candidate "cache" sizes on MI355X, in bytes.
M_EFF_BYTES = {"lds_160KB": 160 * 1024, "lds_plus_vgpr_672KB": 672 * 1024, "l2_xcd_4MB": 4 * 1024 * 1024}


def element_size(dtype):
    return {"bf16": 2, "f32": 4}[dtype]


def compulsory_bytes(w, backward=True):
    """Read Q, K, V (+ O, dO, LSE) once and write the outputs once."""
    es, bh = element_size(w.dtype), w.batch * w.heads
    if backward:
        return bh * (8 * w.n * w.d * es + 4 * w.n)
    return bh * (4 * w.n * w.d * es + 4 * w.n)


def theta_bytes(w, m_bytes):
    """es * min{large-cache term, small-cache term} summed over heads (constant 1)."""
    es, bh = element_size(w.dtype), w.batch * w.heads
    M = m_bytes / es
    n, d = float(w.n), float(w.d)
    if w.sparse:
        z_in, z_qk = n * d, w.kept_fraction() * n * n
        items = min(z_in * z_in / M, z_in * math.sqrt(z_qk) / math.sqrt(M))
    else:
        items = min(n * n * d * d / M, n * n * d / math.sqrt(M)) * w.kept_fraction()
    return bh * es * items


def regime(w, m_bytes):
    """'large' if the cache holds a d x d block (M >= d^2; sparse: M >= Z_in^2 / Z_QK), else 'small'."""
    M = m_bytes / element_size(w.dtype)
    if w.sparse:
        return "large" if M >= (w.n * w.d) ** 2 / (w.kept_fraction() * w.n * w.n) else "small"
    return "large" if M >= w.d * w.d else "small"


def yardstick(w, m_bytes=M_EFF_BYTES["lds_160KB"], backward=True):
    """max{compulsory, Theta-term}: what measured HBM bytes are compared with."""
    return max(compulsory_bytes(w, backward), theta_bytes(w, m_bytes))


def report(w):
    out = {"compulsory_bwd_bytes": compulsory_bytes(w), "regime_at_lds": regime(w, M_EFF_BYTES["lds_160KB"])}
    for k, m in M_EFF_BYTES.items():
        out["theta_bytes_" + k] = theta_bytes(w, m)
    out["yardstick_bytes"] = yardstick(w)
    return out
