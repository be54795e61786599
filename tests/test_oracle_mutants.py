"""The pins must be able to fail: plausible mistakes are planted in the oracle (on the CPU) and each must be caught.

Every mutant replaces one elementary piece of oracle/decoder_layer.py with a subtly wrong version (wrong sign, wrong
pairing, dropped term, off-by-one mask, wrong head mapping, ...).  With the mutant in place at least one of the pin
tests in test_oracle_pins.py has to raise.  The unmutated oracle passes all of them (that is test_oracle_pins itself).
"""
import importlib

import numpy as np
import pytest

import oracle.decoder_layer as dl

pins = importlib.import_module("test_oracle_pins")
F64 = np.float64


def rope_wrong_sign(v, positions, theta):
    v = np.asarray(v, dtype=F64)
    half = v.shape[-1] // 2
    phi = dl.rope_angles(positions, v.shape[-1], theta)
    c, s = np.cos(phi)[:, None, :], np.sin(phi)[:, None, :]
    lo, hi = v[..., :half], v[..., half:]
    return np.concatenate([lo * c + hi * s, hi * c - lo * s], axis=-1)


def rope_interleaved_pairs(v, positions, theta):
    v = np.asarray(v, dtype=F64)
    phi = dl.rope_angles(positions, v.shape[-1], theta)
    c, s = np.cos(phi)[:, None, :], np.sin(phi)[:, None, :]
    out = np.empty_like(v)
    ev, od = v[..., 0::2], v[..., 1::2]
    out[..., 0::2] = ev * c - od * s
    out[..., 1::2] = od * c + ev * s
    return out


def rope_angles_wrong_exponent(positions, head_dim, theta):
    j = np.arange(head_dim // 2, dtype=F64)
    return np.asarray(positions, dtype=F64)[:, None] * (theta ** (-j / head_dim))[None, :]


def rmsnorm_eps_outside(x, g, eps):
    x = np.asarray(x, dtype=F64)
    return x / (np.sqrt(np.mean(x * x, axis=-1, keepdims=True)) + eps) * np.asarray(g, dtype=F64)


def rmsnorm_subtracts_mean(x, g, eps):
    x = np.asarray(x, dtype=F64)
    x = x - np.mean(x, axis=-1, keepdims=True)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * np.asarray(g, dtype=F64)


def silu_as_sigmoid(z):
    return 1.0 / (1.0 + np.exp(-np.asarray(z, dtype=F64)))


def _attention_variant(scale_fn, visible_fn, head_fn):
    def attn(q, k, v, *, row_block=1024, return_probs=False):
        n, hq, d = q.shape
        hkv = k.shape[1]
        g = hq // hkv
        out = np.empty((n, hq, d), dtype=F64)
        probs = np.zeros((hq, n, n), dtype=F64)
        idx = np.arange(n)
        for h in range(hq):
            c = head_fn(h, g, hkv)
            s = (q[:, h, :] @ k[:, c, :].T) * scale_fn(d)
            s = np.where(visible_fn(idx[None, :], idx[:, None]), s, -np.inf)
            s[np.all(np.isinf(s), axis=1), 0] = 0.0
            p = dl._softmax_rows(s)
            out[:, h, :] = p @ v[:, c, :]
            probs[h] = p
        return (out, probs) if return_probs else out
    return attn


attn_no_scale = _attention_variant(lambda d: 1.0, lambda m, n: m <= n, lambda h, g, hkv: h // g)
attn_scale_by_d = _attention_variant(lambda d: 1.0 / d, lambda m, n: m <= n, lambda h, g, hkv: h // g)
attn_strict_mask = _attention_variant(lambda d: 1.0 / np.sqrt(d), lambda m, n: m < n, lambda h, g, hkv: h // g)
attn_no_mask = _attention_variant(lambda d: 1.0 / np.sqrt(d), lambda m, n: m <= n + 10 ** 9, lambda h, g, hkv: h // g)
attn_head_modulo = _attention_variant(lambda d: 1.0 / np.sqrt(d), lambda m, n: m <= n, lambda h, g, hkv: h % hkv)


def mlp_swapped_gate_up(r, p):
    h2 = dl.rmsnorm(r, p.g2, p.rms_eps)
    return r + (dl.silu(h2 @ p.wu.T) * (h2 @ p.wg.T)) @ p.wd.T


def mlp_without_residual(r, p):
    h2 = dl.rmsnorm(r, p.g2, p.rms_eps)
    return (dl.silu(h2 @ p.wg.T) * (h2 @ p.wu.T)) @ p.wd.T


def mlp_norm_gain_of_first_norm(r, p):
    h2 = dl.rmsnorm(r, p.g1, p.rms_eps)
    return r + (dl.silu(h2 @ p.wg.T) * (h2 @ p.wu.T)) @ p.wd.T


def project_qkv_swaps_k_and_v(h, p):
    q, k, v = _orig_project(h, p)
    return q, v, k


_orig_project = dl._project_qkv


def _rows_form_variant(old, new):
    """layer_forward_rows with one expression of its source replaced (the planted mistake)."""
    import inspect
    src = inspect.getsource(dl.layer_forward_rows)
    assert src.count(old) == 1, old
    scope = dict(vars(dl))
    exec(src.replace(old, new), scope)
    fn = scope["layer_forward_rows"]
    fn.__name__ = "rows_form_" + "".join(ch if ch.isalnum() else "_" for ch in new)[:40]
    return fn


rows_form_strict_mask = _rows_form_variant("<= pos[:, None]", "< pos[:, None]")
rows_form_sorted_output = _rows_form_variant("o[sel, hh, :] =", "o[np.arange(a, a + len(sel)), hh, :] =")
rows_form_wrong_kv_head = _rows_form_variant("c = hh // p.group", "c = hh % p.n_kv_heads")
rows_form_query_position = _rows_form_variant("p.head_dim), rows, p.rope_theta)", "p.head_dim), np.arange(len(rows)), p.rope_theta)")

MUTANTS = [
    ("rope", rope_wrong_sign), ("rope", rope_interleaved_pairs), ("rope_angles", rope_angles_wrong_exponent),
    ("rmsnorm", rmsnorm_eps_outside), ("rmsnorm", rmsnorm_subtracts_mean), ("silu", silu_as_sigmoid),
    ("causal_gqa_attention", attn_no_scale), ("causal_gqa_attention", attn_scale_by_d),
    ("causal_gqa_attention", attn_strict_mask), ("causal_gqa_attention", attn_no_mask),
    ("causal_gqa_attention", attn_head_modulo),
    ("_mlp_residual", mlp_swapped_gate_up), ("_mlp_residual", mlp_without_residual),
    ("_mlp_residual", mlp_norm_gain_of_first_norm), ("_project_qkv", project_qkv_swaps_k_and_v),
    ("layer_forward_rows", rows_form_strict_mask), ("layer_forward_rows", rows_form_sorted_output),
    ("layer_forward_rows", rows_form_wrong_kv_head), ("layer_forward_rows", rows_form_query_position),
]

PIN_CALLS = [
    lambda: pins.test_attention_matches_scalar_loops(19, 6, 2, 8),
    lambda: pins.test_attention_matches_library_sdpa(),
    lambda: pins.test_attention_closed_forms(),
    lambda: pins.test_attention_is_causal_and_rows_sum_to_one(),
    lambda: pins.test_gqa_equals_expanded_mha_and_head_mapping(),
    lambda: pins.test_scale_is_inverse_sqrt_head_dim(),
    lambda: pins.test_rope_properties(),
    lambda: pins.test_rope_scores_depend_on_relative_position_only(),
    lambda: pins.test_rope_frequency_of_second_pair(),
    lambda: pins.test_rmsnorm_pins(),
    lambda: pins.test_silu_matches_library_and_hand_values(),
    lambda: pins.test_layer_matches_library_composition(True),
    lambda: pins.test_layer_residual_special_cases(),
    lambda: pins.test_chunked_equals_unchunked(1),
    lambda: pins.test_chunk_attention_matches_scalar_loops_with_prefix(),
    lambda: pins.test_rows_form_equals_full_form(),
]


@pytest.mark.parametrize("name,mutant", MUTANTS, ids=[f"{n}:{f.__name__}" for n, f in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, name, mutant):
    monkeypatch.setattr(dl, name, mutant)
    if hasattr(pins, name):
        monkeypatch.setattr(pins, name, mutant)
    import oracle as pkg
    if hasattr(pkg, name):
        monkeypatch.setattr(pkg, name, mutant)
    caught = []
    for i, call in enumerate(PIN_CALLS):
        try:
            call()
        except AssertionError:
            caught.append(i)
        except Exception as e:  # a mutant may also break shapes; that counts as caught
            caught.append((i, type(e).__name__))
    assert caught, f"no pin noticed the planted mistake {mutant.__name__} in {name}"
