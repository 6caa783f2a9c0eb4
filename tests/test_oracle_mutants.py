"""The pins must notice a plausible mistake anywhere in the oracle.  Each mutant below plants one
(dropped term, wrong sign or index, transposed operand, wrong constant) into the oracle module on the CPU;
the pin tests are then re-run against the mutated module and at least one of them has to fail."""
import math
import os

import numpy as np
import pytest

from oracle import flashdp_oracle as O
import test_oracle_definition as TD
import test_oracle_gaussian as TG
import test_oracle_philox as TP

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def pins():
    """Callables that run the pin tests against whatever the oracle module currently holds."""
    return [
        lambda: TP.test_philox_known_answers(GOLDEN),
        lambda: TP.test_field_keying_seed_layer_element(),
        lambda: TG.test_uniform24_range_and_grid(),
        lambda: TG.test_box_muller_closed_form_points(),
        lambda: TG.test_field_is_standard_normal(),
        lambda: TD.test_widen_bf16_bit_patterns(),
        lambda: TD.test_hand_worked_2x2(GOLDEN),
        lambda: TD.test_brute_force_small_integers((3, 5, 4, 3)),
        lambda: TD.test_ghost_norm_identity_is_an_independent_route(),
        lambda: TD.test_closed_forms(),
        lambda: TD.test_invariants_of_clipping_and_aggregation(),
        lambda: TD.test_sum_not_mean_over_batch(),
    ]


def caught():
    for p in pins():
        try:
            p()
        except AssertionError:
            return True
        except Exception:      # a shape error etc. also exposes the mutant
            return True
    return False


def _philox_with(m0=0xD2511F53, m1=0xCD9E8D57, w0=0x9E3779B9, w1=0xBB67AE85, rounds=10, swap=False, bump_first=False):
    def f(counter, key):
        c = np.asarray(counter, dtype=np.uint32)
        c0, c1, c2, c3 = (c[..., j].astype(np.uint64) for j in range(4))
        k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
        for r in range(rounds):
            if r > 0 or bump_first:
                k0 = (k0 + w0) & 0xFFFFFFFF
                k1 = (k1 + w1) & 0xFFFFFFFF
            p0 = np.uint64(m0) * c0
            p1 = np.uint64(m1) * c2
            hi0, lo0 = p0 >> np.uint64(32), p0 & np.uint64(0xFFFFFFFF)
            hi1, lo1 = p1 >> np.uint64(32), p1 & np.uint64(0xFFFFFFFF)
            if swap:
                c0, c1, c2, c3 = (hi0 ^ c1 ^ np.uint64(k0)), lo0, (hi1 ^ c3 ^ np.uint64(k1)), lo1
            else:
                c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0)), lo1, (hi0 ^ c3 ^ np.uint64(k1)), lo0
        out = np.empty(c.shape, dtype=np.uint32)
        out[..., 0], out[..., 1], out[..., 2], out[..., 3] = c0, c1, c2, c3
        return out
    return f


def _gauss(swap_trig=False, no_minus2=False, angle_from_first=False, second_pair_reuses_first=False, two_pi=2.0 * np.pi):
    def f(r):
        u = [O.uniform24(r[..., k]) for k in range(4)]
        if angle_from_first:
            u[0], u[1] = u[1], u[0]
        if second_pair_reuses_first:
            u[2], u[3] = u[0], u[1]
        ra = np.sqrt((-1.0 if no_minus2 else -2.0) * np.log(u[0]))
        rb = np.sqrt((-1.0 if no_minus2 else -2.0) * np.log(u[2]))
        z = np.empty(r.shape, dtype=np.float64)
        t0, t1 = (np.sin, np.cos) if swap_trig else (np.cos, np.sin)
        z[..., 0], z[..., 1] = ra * t0(two_pi * u[1]), ra * t1(two_pi * u[1])
        z[..., 2], z[..., 3] = rb * t0(two_pi * u[3]), rb * t1(two_pi * u[3])
        return z
    return f


def _linear(mean=False, noise_per_sample=False, noise_without_C=False, norm_of_clipped=False):
    def f(X, dY, C, sigma, seed, layer=0):
        X, dY = np.asarray(X), np.asarray(dY)
        B, D, P = X.shape[0], dY.shape[2], X.shape[2]
        out = np.zeros((D, P))
        norms = np.zeros(B)
        for i in range(B):
            G = O.per_sample_gradient(X[i], dY[i])
            norms[i] = O.frobenius_norm(G)
            c = O.clip_factor(norms[i], float(C))
            out += c * G
            if norm_of_clipped:
                norms[i] *= c
        if mean:
            out /= B
        if sigma != 0.0:
            scale = float(sigma) * (1.0 if noise_without_C else float(C)) * (B if noise_per_sample else 1)
            out += scale * O.noise_field(seed, layer, D * P).reshape(D, P)
        return out, norms
    return f


MUTANTS = {
    # Philox
    "philox_multiplier0": ("philox4x32_10", _philox_with(m0=0xD2511F55)),
    "philox_multiplier1": ("philox4x32_10", _philox_with(m1=0xCD9E8D59)),
    "philox_weyl0": ("philox4x32_10", _philox_with(w0=0x9E3779B1)),
    "philox_weyl1": ("philox4x32_10", _philox_with(w1=0xBB67AE87)),
    "philox_9_rounds": ("philox4x32_10", _philox_with(rounds=9)),
    "philox_11_rounds": ("philox4x32_10", _philox_with(rounds=11)),
    "philox_products_not_crossed": ("philox4x32_10", _philox_with(swap=True)),
    "philox_key_bumped_before_first_round": ("philox4x32_10", _philox_with(bump_first=True)),
    # keying of the field
    "field_layer_in_word3": ("_group_counters", lambda g, layer: np.stack(
        [(np.asarray(g, np.uint64) & np.uint64(0xFFFFFFFF)).astype(np.uint32),
         (np.asarray(g, np.uint64) >> np.uint64(32)).astype(np.uint32),
         np.zeros(np.shape(g), np.uint32), np.full(np.shape(g), layer, np.uint32)], axis=-1)),
    "field_key_words_swapped": ("_key", lambda seed: ((int(seed) >> 32) & 0xFFFFFFFF, int(seed) & 0xFFFFFFFF)),
    "field_seed_truncated_to_32_bits": ("_key", lambda seed: (int(seed) & 0xFFFFFFFF, 0)),
    # uniform and Box-Muller
    "uniform_without_half_step": ("uniform24", lambda r: (np.asarray(r, np.uint32) >> np.uint32(8)).astype(np.float64) / 16777216.0 + 1e-300),
    "uniform_keeps_low_bits": ("uniform24", lambda r: (np.asarray(r, np.uint32).astype(np.float64) + 0.5) / 4294967296.0),
    "box_muller_sin_cos_swapped": ("gaussians_from_words", _gauss(swap_trig=True)),
    "box_muller_missing_factor_2": ("gaussians_from_words", _gauss(no_minus2=True)),
    "box_muller_angle_from_first_word": ("gaussians_from_words", _gauss(angle_from_first=True)),
    "box_muller_second_pair_reuses_first": ("gaussians_from_words", _gauss(second_pair_reuses_first=True)),
    "box_muller_pi_instead_of_two_pi": ("gaussians_from_words", _gauss(two_pi=np.pi)),
    # stages 1-4
    "widen_shift_15": ("widen", lambda a: (np.asarray(a).astype(np.uint32) << np.uint32(15)).view(np.float32).astype(np.float64)
                       if np.asarray(a).dtype == np.uint16 else np.asarray(a).astype(np.float64)),
    "gradient_transposed": ("per_sample_gradient", lambda X_i, dY_i: (O.widen(X_i).T @ O.widen(dY_i))),
    "gradient_drops_last_token": ("per_sample_gradient", lambda X_i, dY_i: O.widen(dY_i)[:-1].T @ O.widen(X_i)[:-1]
                                  if len(X_i) > 1 else O.widen(dY_i).T @ O.widen(X_i)),
    "norm_without_square": ("frobenius_norm", lambda G: float(np.sqrt(np.abs(np.sum(G))))),
    "norm_without_root": ("frobenius_norm", lambda G: float(np.sum(np.square(G)))),
    "norm_max_abs": ("frobenius_norm", lambda G: float(np.max(np.abs(G)))),
    "clip_always": ("clip_factor", lambda n, C: C / n if n > 0 else 1.0),
    "clip_inverted": ("clip_factor", lambda n, C: 1.0 / max(1.0, C / n) if n > 0 else 1.0),
    "clip_squared_norm": ("clip_factor", lambda n, C: 1.0 / max(1.0, n * n / C)),
    "mean_over_batch": ("linear_dp_grad", _linear(mean=True)),
    "noise_once_per_sample": ("linear_dp_grad", _linear(noise_per_sample=True)),
    "noise_scale_without_C": ("linear_dp_grad", _linear(noise_without_C=True)),
    "norms_reported_after_clipping": ("linear_dp_grad", _linear(norm_of_clipped=True)),
}


def test_unmutated_oracle_passes_every_pin():
    assert not caught()


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_mutant(name, monkeypatch):
    attr, repl = MUTANTS[name]
    monkeypatch.setattr(O, attr, repl)
    assert caught(), f"no pin notices the mutant {name}"
