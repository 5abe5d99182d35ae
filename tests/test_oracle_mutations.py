"""The pins must be able to see a mistake: plant plausible errors in a copy of
the oracle's C source (CPU only) and check that the pin suite fails on each."""
import os
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parents[1]
SRC = ROOT / "oracle" / "dvp_oracle.c"

MUTATIONS = {
    "exclusive_boundary": ("int s = zrow[k] >= tau;", "int s = zrow[k] > tau;"),
    "gradient_sign": ("(k == y ? 1.0 : 0.0) - p", "p - (k == y ? 1.0 : 0.0)"),
    "unmasked_sum": ("if (zrow[k] >= tau) nsum_add(&S_safe, e);", "nsum_add(&S_safe, e);"),
    "unrounded_threshold": ("const double tau = (double)(float)tau_ideal;", "const double tau = tau_ideal;"),
    "full_normaliser": ("logp = zrow[y] - lse_safe;", "logp = zrow[y] - lse_full;"),
    "gradient_on_pruned_token_rows": ("if (y_safe && zrow[k] >= tau) {", "if (zrow[k] >= tau) {"),
    "gradient_scale_dropped": ("d[k] = g * (", "d[k] = ("),
    "threshold_sign": ("const double tau_ideal = m + (double)J->log_rho;",
                       "const double tau_ideal = m - (double)J->log_rho;"),
    "onehot_index": ("(k == y ? 1.0 : 0.0)", "(k == y + 1 ? 1.0 : 0.0)"),
    "weight_ratio_direction": ("else                 l = lt - li;", "else                 l = li - lt;"),
    "veto_inclusive": ("if (l32 < log_threshold ||", "if (l32 <= log_threshold ||"),
    "pruned_token_weight_not_zero": ("if (lt == -INFINITY) l = -INFINITY;", "if (0) l = -INFINITY;"),
    "sequence_min_never_updated": ("else if (w < wmin) wmin = w;", "else if (w > wmin) wmin = w;"),
    "e4m3_bias": ("ldexp(1.0 + (double)mant / 8.0, expo - 7)", "ldexp(1.0 + (double)mant / 8.0, expo - 8)"),
    "e4m3_subnormals_flushed": ("if (expo == 0) v = ldexp((double)mant, -9);", "if (expo == 0) v = 0.0;"),
    "e4m3_has_infinity": ("if (expo == 15 && mant == 7) return NAN;",
                          "if (expo == 15) return mant ? NAN : (sign ? -INFINITY : INFINITY);"),
    "e4m3_mantissa_width": ("(double)mant / 8.0, expo", "(double)mant / 16.0, expo"),
    "entropy_sign": ("nsum_add(&H, -exp(lp) * lp);", "nsum_add(&H, exp(lp) * lp);"),
    "entropy_over_all_tokens": ("""            if (zrow[k] >= tau) {
                double lp = zrow[k] - lse_safe;""", """            if (1) {
                double lp = zrow[k] - lse_safe;"""),
    "finite_mask_threshold_not_rounded": ("if (dtype == DVP_ORACLE_BF16) t32 = bf16_round_nearest_even(t32);", ""),
    "finite_mask_pruned_mass_dropped": ("nsum_add(&S, exp((pruned ? mask_value : zrow[k]) - ref));",
                                        "if (!pruned) nsum_add(&S, exp(zrow[k] - ref));"),
    "finite_mask_pruned_token_minus_inf": ("((y_pruned ? mask_value : zrow[y]) - lse)",
                                           "(y_pruned ? -INFINITY : zrow[y] - lse)"),
    "finite_mask_gradient_reaches_pruned": ("if (!in_range || zrow[k] < tau) dz[i * V + k] = 0.0;",
                                            "if (!in_range) dz[i * V + k] = 0.0;"),
    "finite_mask_inclusive_pruning": ("const int pruned = zrow[k] < tau;", "const int pruned = zrow[k] <= tau;"),
    "infinite_weight_not_vetoed": ("|| l32 == INFINITY) veto = 1;", ") veto = 1;"),
}


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTATIONS[name]
    text = SRC.read_text()
    assert text.count(old) >= 1, "mutation site not found: " + name
    mutated = tmp_path / ("oracle_%s.c" % name)
    mutated.write_text(text.replace(old, new, 1))
    env = dict(os.environ, DVP_ORACLE_SRC=str(mutated))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        str(ROOT / "tests" / "test_oracle_pins.py")],
                       cwd=str(ROOT), env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode != 0, "the pins did not notice: " + name
    assert "failed" in r.stdout
