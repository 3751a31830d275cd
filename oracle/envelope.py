"""Ideal sparse-serving envelope: the paper's byte and time model (test
infrastructure; Section 3.1, Eq. 1-3).

B requests, L layers, H KV heads, head dimension d, e bytes per element,
context N; alpha = summary bytes relative to the full KV cache as the paper
uses it in Eq. 1 (summary bytes = B L H d e alpha N); beta = attended fraction;
rho = fraction of attended bytes that miss HBM.
"""


def qk_score_bytes(B, L, H, d, e, alpha, N):
    """Eq. 1: HBM bytes read by scoring."""
    return B * L * H * d * e * alpha * N


def kv_topk_bytes(B, L, H, d, e, beta, N):
    """Eq. 2: HBM bytes read by attention over the selected KV (K and V)."""
    return 2 * B * L * H * d * e * beta * N


def tpot_seconds(score_bytes, topk_bytes, bw_hbm, rho=0.0, bw_pcie=float("inf"), t_mlp=0.0):
    """Eq. 3."""
    return (score_bytes + topk_bytes) / bw_hbm + rho * topk_bytes / bw_pcie + t_mlp


def kv_cache_bytes(layers, kv_heads, head_dim, bytes_per_el, tokens):
    """Full KV footprint of one request (K and V)."""
    return 2 * layers * kv_heads * head_dim * bytes_per_el * tokens
