"""What the dynamic per-token FP8 scale of the cache buys (Opt-KV, Eq. 6 and the FP8 storage of
Alg. 1) against the schemes it stands against -- a static per-head scale, a per-block scale, and
E5M2 codes -- measured as attention error on a long context with outlier keys (1 % of the tokens'
K rows scaled by 20), CPU only.  The figures are printed (pytest -s) and quoted in the design notes."""
import numpy as np

import workloads
from oracle import variants


def _workload(outliers: bool):
    return workloads.make_custom("variants", seed=9326, S=6, H_q=10, H_k=2, d=128, B=16, NB=1024,
                                 context_lens=[1500, 2048, 1024, 1777, 1300, 2000],
                                 k_outlier_frac=0.01 if outliers else 0.0)


def test_rounding_grids():
    e4 = variants._round_e4m3(np.array([0.0, 1.0, 1.0625, 1.1875, 447.0, 1e9, -3.3], np.float32))
    assert e4.tolist() == [0.0, 1.0, 1.0, 1.25, 448.0, 448.0, -3.25]       # ties to even, saturation
    e5 = variants._round_e5m2(np.array([0.0, 1.0, 1.125, 1.375, 1.2, 60000.0, -2.6, 2.0 ** -16]))
    assert e5.tolist() == [0.0, 1.0, 1.0, 1.5, 1.25, 57344.0, -2.5, 2.0 ** -16]
    x = np.random.default_rng(0).standard_normal(4096).astype(np.float32) * 3
    assert np.all(np.abs(variants._round_e4m3(x) - x) <= np.abs(x) * 2.0 ** -4 + 2.0 ** -10)
    assert np.all(np.abs(variants._round_e5m2(x) - x) <= np.abs(x) * 2.0 ** -3 + 2.0 ** -17)


def test_per_token_scheme_is_the_cache_the_write_path_builds(oracle_mod):
    """quantise_rows('per_token', 'e4m3') reproduces, value for value, what the oracle's cache
    write stores and its attention reads (so the comparison below is about THIS build's cache)."""
    from helpers import gather_dequant, oracle_fill
    w = workloads.make_custom("v", seed=3, S=1, H_q=4, H_k=2, d=64, B=16, NB=8, context_lens=[100])
    K, V = gather_dequant(w, oracle_fill(oracle_mod, w), 0)
    assert np.array_equal(K, variants.quantise_rows(w.k_ctx, "per_token", "e4m3"))
    assert np.array_equal(V, variants.quantise_rows(w.v_ctx, "per_token", "e4m3"))


def _errors(w):
    G = w.H_q // w.H_k
    rows = {}
    for scheme in ("static", "per_block", "per_token"):
        for fmt in ("e4m3", "e5m2"):
            worst, sq = 0.0, []
            for s in range(w.S):
                a, b = int(w.seq_start[s]), int(w.seq_start[s + 1])
                K, V = w.k_ctx[a:b], w.v_ctx[a:b]
                # a static scale is fixed in advance, here from the first 256 tokens of the sequence
                Kq = variants.quantise_rows(K, scheme, fmt, calib=K[:256])
                Vq = variants.quantise_rows(V, scheme, fmt, calib=V[:256])
                mx, r = variants.attention_error(w.q[s], K, V, Kq, Vq, G, w.softmax_scale)
                worst = max(worst, mx); sq.append(r * r)
            rows[(scheme, fmt)] = (worst, float(np.sqrt(np.mean(sq))))
    return rows


def test_dynamic_scale_against_the_alternatives():
    plain, outl = _errors(_workload(False)), _errors(_workload(True))
    for name, rows in (("N(0,1) keys", plain), ("1 % of key rows x20", outl)):
        for (scheme, fmt), (worst, rms) in rows.items():
            print(f"{name:20s} {scheme:9s} {fmt}: attention error max-abs {worst:.3e}  rms {rms:.3e}")
    for rows in (plain, outl):
        for scheme in ("per_block", "per_token"):
            # one more mantissa bit: E4M3 beats E5M2 whenever the scale keeps values in range
            assert rows[(scheme, "e4m3")][1] < rows[(scheme, "e5m2")][1]
    # a scale fixed before the outliers arrive saturates them; a dynamic one (per block or per
    # token) follows them -- with a floating-point code the two dynamic granularities are close
    dyn = min(outl[("per_block", "e4m3")][1], outl[("per_token", "e4m3")][1])
    assert outl[("static", "e4m3")][1] > 1.25 * max(outl[("per_block", "e4m3")][1], outl[("per_token", "e4m3")][1])
    assert plain[("per_token", "e4m3")][1] < 5e-3 and dyn > plain[("per_token", "e4m3")][1]
