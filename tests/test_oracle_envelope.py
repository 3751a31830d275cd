"""The byte model (Eq. 1-3) against the figures the paper prints."""
from oracle import envelope
from golden_util import load_golden


def test_eq1_eq2_headline_workload():
    g = load_golden()
    # min + max vector per 16-token page: 2*d*e bytes per 16 tokens of K+V... the
    # paper's Eq. 1 counts summary bytes as B L H d e (alpha N): alpha N = number
    # of summary vectors = 2 per page = N/8.
    assert envelope.qk_score_bytes(16, 1, 8, 128, 2, 1 / 8, 32768) == g["eq1_score_bytes_cfg1"]
    assert envelope.kv_topk_bytes(16, 1, 8, 128, 2, 1 / 16, 32768) == g["eq2_topk_bytes_cfg1"]
    # the same numbers from first principles: 512 B per partition, 8 KiB per page
    assert 16 * 8 * 2048 * 512 == g["eq1_score_bytes_cfg1"]
    assert 16 * 8 * 128 * 8192 == g["eq2_topk_bytes_cfg1"]


def test_intro_kv_footprint_example():
    g = load_golden()
    full = envelope.kv_cache_bytes(36, 8, 128, 2, int(g["kv_request_tokens"]))
    assert abs(full / 1e9 - g["kv_request_gb_approx"]) < 0.5
    per_step = envelope.kv_topk_bytes(1, 36, 8, 128, 2, 1 - g["sparsity"], int(g["kv_request_tokens"]))
    assert per_step / 1e9 < g["kv_sparse_step_gb_upper"]
    assert abs(per_step - (1 - g["sparsity"]) * full) < 1.0


def test_eq3_terms():
    t = envelope.tpot_seconds(134217728, 134217728, 8e12)
    assert abs(t * 1e6 - 33.554432) < 1e-9
    t2 = envelope.tpot_seconds(100.0, 200.0, 10.0, rho=0.5, bw_pcie=5.0, t_mlp=1.0)
    assert t2 == 30.0 + 20.0 + 1.0
