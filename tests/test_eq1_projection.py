"""Host check of the benchmark's Eq. (1) projection: the paper's speed-up model
T_sd / T_t = (d T_d / T_t + T_v(n) / T_t) / tau(n, d) evaluated by hand on made-up layer times."""
import bench


def test_projection_formula_by_hand():
    layer_ms = {1: 0.100, 24: 0.130, 32: 0.140, 40: 0.160, 48: 0.170}     # ms per decoder layer
    read_GBps = 6000.0
    out = bench.eq1_projection(layer_ms, read_GBps)
    H, V = 8192, 128256
    lm_head_ms = V * H * 2 / (read_GBps * 1e6)
    layer_params = 8192 * 10240 + 8192 * 8192 + 8192 * 57344 + 28672 * 8192
    draft_ms = (layer_params * 2 + 2 * H * H * 2) / (read_GBps * 1e6) + lm_head_ms
    t_t = 80 * 0.100 + lm_head_ms
    assert abs(out["inputs"]["T_t_ms"] - t_t) < 1e-12 and abs(out["inputs"]["T_d_ms_estimated"] - draft_ms) < 1e-12
    assert out["inputs"]["lm_head"] == "estimated from bytes"
    for n, (d, tau) in bench.PAPER_TAU_70B_W4A16.items():
        ratio = (80 * layer_ms[n] + lm_head_ms) / t_t
        row = out[str(n)]
        assert row["d"] == d and row["tau_paper"] == tau
        assert abs(row["T_v_over_T_t"] - ratio) < 1e-12
        assert abs(row["speedup_over_own_autoregressive_no_draft_cost"] - tau / ratio) < 1e-12
        # Eq. (1): expected latency per token relative to plain decoding, inverted into a speed-up
        rel_latency = (d * draft_ms / t_t + ratio) / tau
        assert abs(row["speedup_over_own_autoregressive_estimated_draft"] - 1.0 / rel_latency) < 1e-12
    # the paper's figure: accepted length grows with the tree, so does the A100 verification ratio
    taus = [bench.PAPER_TAU_70B_W4A16[n][1] for n in (24, 32, 40, 48)]
    assert taus == sorted(taus) and all(3.2 < t < 4.0 for t in taus)
    ratios = [bench.PAPER_RATIO_70B_W4A16_A100[n] for n in (24, 32, 40, 48)]
    assert ratios == sorted(ratios) and ratios[-1] == 1.58


def test_projection_with_measured_heads_and_the_8b_tables():
    from paper_2505_22179_amd import inputs as I
    layer_ms = {1: 0.040, 30: 0.050, 40: 0.060, 50: 0.066, 60: 0.070}
    out = bench.eq1_projection(layer_ms, 6500.0, shapes=I.LLAMA3_8B, n_layers=32, tau=bench.PAPER_TAU_8B_W4A16,
                               paper_ratio=bench.PAPER_RATIO_8B_W4A16_A100, lm_head_ms=0.175, draft_lm_head_ms=0.200)
    t_t = 32 * 0.040 + 0.175
    layer_params = 4096 * 6144 + 4096 * 4096 + 4096 * 28672 + 14336 * 4096
    draft_ms = (layer_params * 2 + 2 * 4096 * 4096 * 2) / (6500.0 * 1e6) + 0.200
    assert abs(out["inputs"]["T_t_ms"] - t_t) < 1e-12 and abs(out["inputs"]["T_d_ms_estimated"] - draft_ms) < 1e-12
    row = out["60"]
    ratio = (32 * 0.070 + 0.175) / t_t
    assert row["d"] == 6 and abs(row["T_v_over_T_t"] - ratio) < 1e-12 and row["T_v_over_T_t_paper_A100"] == 1.803
    assert abs(row["speedup_over_own_autoregressive_estimated_draft"] - 4.046 / (6 * draft_ms / t_t + ratio)) < 1e-12


def test_projection_from_whole_model_passes():
    model_ms = {1: 9.0, 24: 11.7, 32: 12.6, 40: 14.4, 48: 14.4 * 1.1}
    out = bench.eq1_projection({}, 6500.0, lm_head_ms=0.33, draft_lm_head_ms=0.35, model_ms=model_ms)
    assert out["inputs"]["T_t_ms"] == 9.0
    assert abs(out["24"]["T_v_over_T_t"] - 11.7 / 9.0) < 1e-12
    d, tau = bench.PAPER_TAU_70B_W4A16[48]
    draft = out["inputs"]["T_d_ms_estimated"]
    assert abs(out["48"]["speedup_over_own_autoregressive_estimated_draft"] - tau / (d * draft / 9.0 + model_ms[48] / 9.0)) < 1e-12
