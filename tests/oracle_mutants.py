"""pytest plugin used only by test_oracle_pin_strength.py: plants ONE mistake in the CPU oracle (never in
the HIP path) before the pin tests are collected, so that the meta-test can check that the pins notice.

Activated with `-p oracle_mutants` and the environment variable SDLLM_ORACLE_MUTANT=<name>.  A mutant is the
oracle module's own source with one textual replacement, executed as a fresh module whose public names
replace the originals in the `oracle` package."""
import importlib
import os
import sys
import types

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# name -> (oracle submodule, text to replace, replacement)
MUTANTS = {
    # attention (Eq. 8 and the paragraph after it)
    "attn_scale_dropped": ("attention", "Sc = scale * (", "Sc = 1.0 * ("),
    "attn_scores_from_values": ("attention", "@ Kr.astype(np.float64).T", "@ Vr.astype(np.float64).T"),
    "attn_gqa_map": ("attention", "kvh = hq // g", "kvh = hq % Hkv"),
    "attn_prefix_one_short": ("attention", "parts.append(cache[:P])", "parts.append(cache[:max(P - 1, 0)])"),
    "attn_prefix_one_long": ("attention", "parts.append(cache[:P])", "parts.append(cache[:P + 1])"),
    "attn_gather_ignored": ("attention", "parts.append(suffix[keep_idx])", "parts.append(suffix[:len(keep_idx)])"),
    "attn_softmax_wrong_axis": ("attention", "E.sum(axis=1, keepdims=True)", "E.sum(axis=0, keepdims=True)"),
    "attn_causal_mask": ("attention", "Sc = Sc - Sc.max(axis=1, keepdims=True)",
                         "Sc = np.where(np.arange(Sc.shape[1])[None, :] > np.arange(Sc.shape[0])[:, None] + "
                         "(Sc.shape[1] - Sc.shape[0]), -1e300, Sc); Sc = Sc - Sc.max(axis=1, keepdims=True)"),
    "attn_output_transposed_operand": ("attention", "out[b, hq] = Pm @ Vr.astype(np.float64)",
                                       "out[b, hq] = Pm @ Kr.astype(np.float64)"),
    # unmask (Eq. 4, 5, 9, 10, termination, early exit)
    "unmask_strict_threshold": ("unmask", "if conf[b, i] >= tau[b]]", "if conf[b, i] > tau[b]]"),
    "unmask_threshold_sign": ("unmask", "tau0 * (1.0 - alpha * (1.0 - r_mask))", "tau0 * (1.0 + alpha * (1.0 - r_mask))"),
    "unmask_ratio_inverted": ("unmask", "tau0 * (1.0 - alpha * (1.0 - r_mask))", "tau0 * (1.0 - alpha * r_mask)"),
    "unmask_no_fallback": ("unmask", "C = [best]", "C = []"),
    "unmask_fallback_highest_position": ("unmask", "if conf[b, i] > conf[b, best]:", "if conf[b, i] >= conf[b, best]:"),
    "unmask_argmax_last_on_ties": ("unmask", "xhat = int(np.argmax(z))", "xhat = int(len(z) - 1 - np.argmax(z[::-1]))"),
    "unmask_no_max_shift": ("unmask", "e = np.exp(z - z[xhat])", "e = np.exp(z)"),
    "unmask_eos_unconditional": ("unmask", "and conf[b, i] >= tau_eos", "and True"),
    "unmask_block_done_early": ("unmask", "block_done[b] = 1 if (m - len(C)) == 0 else 0", "block_done[b] = 1 if len(C) > 0 else 0"),
    "unmask_ratio_after_commit": ("unmask", "tau[b] = dynamic_threshold(tau0, alpha, m, K, extra_masked, extra_total)",
                                  "tau[b] = dynamic_threshold(tau0, alpha, max(m - 1, 0), K, extra_masked, extra_total)"),
    # kv append
    "append_row_offset": ("kv_append", "k_out[:, b, :, P:P + K, :] = k_blocks[:, b]", "k_out[:, b, :, P - 1:P + K - 1, :] = k_blocks[:, b]"),
    "append_v_from_k": ("kv_append", "v_out[:, b, :, P:P + K, :] = v_blocks[:, b]", "v_out[:, b, :, P:P + K, :] = k_blocks[:, b]"),
    "append_flags_ignored": ("kv_append", "if do_append is not None and do_append[b] == 0:", "if False:"),
    # suffix rule (Eq. 7)
    "suffix_window_from_current_block": ("suffix", "for n in range(c + 1, min(c + w, N - 1) + 1):", "for n in range(c, min(c + w, N - 1) + 1):"),
    "suffix_window_one_block_short": ("suffix", "for n in range(c + 1, min(c + w, N - 1) + 1):", "for n in range(c + 1, min(c + w, N - 1)):"),
    "suffix_no_trailing": ("suffix", "if keep_trailing and last >= suffix_start:", "if False:"),
    # rope (section 3.3, sentence before Eq. 7)
    "rope_one_sign": ("rope", "out[..., t, a] = x[..., t, a] * c - x[..., t, b] * s", "out[..., t, a] = x[..., t, a] * c + x[..., t, b] * s"),
    "rope_direction": ("rope", "c, s = np.cos(p * theta), np.sin(p * theta)", "c, s = np.cos(p * theta), -np.sin(p * theta)"),
    "rope_frequency": ("rope", "theta = float(base) ** (-2.0 * i / D)", "theta = float(base) ** (-1.0 * i / D)"),
    "rope_pair_layout": ("rope", "if interleaved else (i, i + D // 2)", "if not interleaved else (i, i + D // 2)"),
    "rope_positions_shift_with_pruning": ("rope", "pos0 + K + keep_idx])", "pos0 + K + np.arange(len(keep_idx))])"),
    # vocabulary projection (last map of Eq. 3)
    "lm_head_transposed_weight": ("lm_head", "z[:, v0:v0 + Wc.shape[0]] = h2 @ Wc.T",
                                  "z[:, v0:v0 + Wc.shape[0]] = (h2 @ Wc) if Wc.shape[0] == Wc.shape[1] else (h2 @ Wc.T)"),
    "lm_head_slice_misplaced": ("lm_head", "z[:, v0:v0 + Wc.shape[0]] = h2 @ Wc.T", "z[:, V - v0 - Wc.shape[0]:V - v0] = h2 @ Wc.T"),
    "lm_head_projects_unmasked_rows_only": ("lm_head", "m = np.asarray(masked) != 0", "m = np.asarray(masked) == 0"),
    "lm_head_logits_rounded_to_bf16_grid": ("lm_head", "logits[m] = lm_head_logits(hidden[m], weight)",
                                            "logits[m] = np.round(lm_head_logits(hidden[m], weight) * 8.0) / 8.0"),
}

# the pin files that must notice a mistake in the given oracle submodule
PIN_FILES = {
    "attention": ["test_oracle_attention.py"],
    "unmask": ["test_oracle_unmask.py"],
    "kv_append": ["test_oracle_kv_append.py"],
    "suffix": ["test_suffix_rule.py"],
    "rope": ["test_oracle_rope.py"],
    "lm_head": ["test_oracle_lm_head.py"],
}


def plant(name: str) -> None:
    sub, old, new = MUTANTS[name]
    import oracle
    mod = importlib.import_module("oracle." + sub)
    src = open(mod.__file__).read()
    assert src.count(old) == 1, f"mutant {name}: the text to replace must occur exactly once in oracle/{sub}.py"
    mutant = types.ModuleType("oracle." + sub)
    mutant.__file__ = mod.__file__
    exec(compile(src.replace(old, new), mod.__file__ + "<mutant " + name + ">", "exec"), mutant.__dict__)
    for k, v in mutant.__dict__.items():
        if callable(v) and getattr(v, "__module__", None) == "oracle." + sub:
            setattr(mod, k, v)
            if hasattr(oracle, k):
                setattr(oracle, k, v)


def pytest_configure(config):
    name = os.environ.get("SDLLM_ORACLE_MUTANT")
    if name:
        plant(name)
