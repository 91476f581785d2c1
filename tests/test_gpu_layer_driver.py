"""The layer driver runs the recipes of the paper's efficiency table and orders them sensibly (GPU)."""
import pytest

from paper_2512_10411_amd import layer_driver

pytestmark = pytest.mark.gpu


def test_layer_driver_orders_the_recipes():
    rows = layer_driver.run(n=16384, gen=64, layers=8, reps=3, quiet=True)
    by = {(r["window"], r["keep_first"], r["fa_decode"], r["fa_layers"]): r for r in rows}
    full = by[("Full", 0, False, "all")]
    swa = by[("2k", 0, False, "none")]
    half = by[("2k", 0, False, "1/2")]
    fa_dec = by[("2k", 0, True, "none")]
    assert len(rows) == len(layer_driver.TABLE) and all(r["request_s"] > 0 for r in rows)
    assert swa["prefill_s"] < half["prefill_s"] < full["prefill_s"]      # fewer full-attention layers, less work
    assert abs(fa_dec["prefill_s"] - swa["prefill_s"]) < 0.2 * swa["prefill_s"]  # FA Decode leaves prefill alone
    assert fa_dec["decode_s_per_token"] > swa["decode_s_per_token"]      # and pays for it while decoding
    assert full["speedup_vs_full"] == 1.0 and swa["speedup_vs_full"] > 1.5
