"""Are the oracle's pins sharp?  Each case plants ONE plausible mistake in a copy of the oracle's C
source (a dropped term, a wrong sign or comparison, a swapped index, a misplaced constant), builds
it, and runs the pin tests against the copy: at least one pin must fail.  Everything here runs on
the CPU; the HIP library is not involved.

A planted snippet that no longer occurs in dc_oracle.c fails the case loudly: the list has to be
kept in step with the source.
"""
import ctypes as C
import os
import subprocess

import pytest

import oracle
import test_oracle_advantage as T_adv
import test_oracle_balance as T_bal
import test_oracle_gae as T_gae
import test_oracle_plan_gather as T_pg

SRC = os.path.join(os.path.dirname(oracle.__file__), "dc_oracle.c")


def _balance_pins():
    T_bal.test_hand_traces()
    for seed in range(6):
        T_bal.test_scan_equals_priority_queue(seed)
    T_bal.test_constraint_changes_the_answer()
    T_bal.test_structure_on_all_workloads()
    for K, N in ((2, 8), (3, 9), (4, 12)):
        T_bal.test_graham_bound_unconstrained(K, N)
        T_bal.test_constrained_vs_constrained_opt(K, N)


def _advantage_pins():
    T_adv.test_closed_form_binary_rewards()
    T_adv.test_printed_value_g8_k1()
    for ddof in (0, 1):
        T_adv.test_reduces_to_library_std(ddof)
    T_adv.test_group_sum_zero_and_identical_groups()
    T_adv.test_identical_rewards_any_group_size()
    T_adv.test_singleton_group_and_empty_group()
    T_adv.test_shift_scale_invariance_and_permutation()
    T_adv.test_unit_sample_variance()
    T_adv.test_broadcast_selects_on_mask()


def _plan_pins():
    for cfg in (1, 2):
        for align in (1, 64):
            T_pg.test_plan_matches_rederivation(cfg, align)
    T_pg.test_plan_hand_example()
    T_pg.test_next_fit_properties()


def _gather_pins():
    for align in (1, 16):
        T_pg.test_every_token_exactly_once_and_inverse(1, align)
        T_pg.test_every_token_exactly_once_and_inverse(2, align)
    T_pg.test_identity_case()
    T_pg.test_gather_preserves_nan_payload_bits()


def _scatter_pins():
    import numpy as np
    for dt in (np.uint8, np.uint16, np.int32):
        T_pg.test_scatter_undoes_gather(dt)
    T_pg.test_scatter_against_index_formulation()
    T_pg.test_scatter_hand_example()


def _gae_pins():
    T_gae.test_hand_worked_example()
    T_gae.test_lambda_one_gamma_one_gives_the_score_as_every_return()
    T_gae.test_lambda_zero_is_the_td_residual()
    T_gae.test_zero_values_give_a_geometric_tail()
    T_gae.test_constant_values_gamma_one()
    T_gae.test_explicit_double_sum_with_kl_penalty()
    T_gae.test_tokens_without_loss_are_transparent()
    T_gae.test_all_masked_sequence_and_sequence_independence()
    T_gae.test_two_rollout_shards_and_padded_rows()


# (what is planted, text in dc_oracle.c, its replacement, pins that must notice)
MISTAKES = [
    # ---- Algorithm 1
    ("equal loads resolved to the LARGEST worker id",
     "if (to < 0 || shard_load[k] < shard_load[to]) to = k;", "if (to < 0 || shard_load[k] <= shard_load[to]) to = k;",
     _balance_pins),
    ("ascending instead of descending lengths",
     "return g_len_of[a] > g_len_of[b] ? -1 : 1;", "return g_len_of[a] < g_len_of[b] ? -1 : 1;", _balance_pins),
    ("equal lengths in descending index order",
     "return a < b ? -1 : (a > b);", "return a > b ? -1 : (a < b);", _balance_pins),
    ("cardinality test off by one (a worker may take C + 1 items)",
     "if (held[k] >= C) continue;", "if (held[k] > C) continue;", _balance_pins),
    ("cardinality constraint dropped",
     "if (held[k] >= C) continue;", ";", _balance_pins),
    ("the load of a worker is not advanced by the item's length",
     "shard_load[to] += S[order[t]];", "shard_load[to] += 1;", _balance_pins),
    ("the most loaded worker takes the item",
     "if (to < 0 || shard_load[k] < shard_load[to]) to = k;", "if (to < 0 || shard_load[k] > shard_load[to]) to = k;",
     _balance_pins),
    # ---- group-relative advantage
    ("eps inside the square root",
     "double sd = sqrt(ss / (double)(G - ddof));", "double sd = sqrt(ss / (double)(G - ddof) + eps); eps = 0;",
     _advantage_pins),
    ("ddof ignored (always the population std)",
     "double sd = sqrt(ss / (double)(G - ddof));", "double sd = sqrt(ss / (double)G);", _advantage_pins),
    ("mean not subtracted in the numerator",
     "adv_seq[i] = (float)(((double)reward[i] - mean) / (sd + eps));",
     "adv_seq[i] = (float)(((double)reward[i]) / (sd + eps));", _advantage_pins),
    ("sign of the advantage flipped",
     "adv_seq[i] = (float)(((double)reward[i] - mean) / (sd + eps));",
     "adv_seq[i] = (float)((mean - (double)reward[i]) / (sd + eps));", _advantage_pins),
    ("no special case for a group of identical rewards",
     "if (all_same || G - ddof <= 0) {", "if (G - ddof <= 0) {", _advantage_pins),
    ("broadcast multiplies by the mask byte instead of selecting",
     "adv_tok[base + t] = mask[base + t] ? adv_seq[i] : 0.0f;", "adv_tok[base + t] = mask[base + t] * adv_seq[i];",
     _advantage_pins),
    ("broadcast ignores the mask",
     "adv_tok[base + t] = mask[base + t] ? adv_seq[i] : 0.0f;", "adv_tok[base + t] = adv_seq[i];", _advantage_pins),
    # ---- plan
    ("a slot that fills the budget exactly opens a new micro-batch",
     "in_mb + len > budget) {", "in_mb + len >= budget) {", _plan_pins),
    ("micro-batches run on across shards",
     "if (j == shard_seq_off[p] || in_mb + len > budget) {", "if (j == 0 || in_mb + len > budget) {", _plan_pins),
    ("shard starts rounded down instead of up",
     "pos = (pos + align - 1) / align * align;", "pos = pos / align * align;", _plan_pins),
    ("cu_seqlens holds lengths, not running totals",
     "cu_seqlens[cu_at] = (int32_t)in_mb;", "cu_seqlens[cu_at] = (int32_t)len;", _plan_pins),
    ("slices of cu_seqlens do not leave room for their leading zero",
     "cu_at = j + M;", "cu_at = j;", _plan_pins),
    # ---- gather / scatter
    ("gather drops the last element of every sequence",
     "memcpy(to, from, (size_t)S[i] * (size_t)elem_bytes);\n    }\n    return DCO_OK;\n}\n\n/*\n * Reverse",
     "memcpy(to, from, (size_t)(S[i] - 1) * (size_t)elem_bytes);\n    }\n    return DCO_OK;\n}\n\n/*\n * Reverse", _gather_pins),
    ("gather copies elements, not bytes, of a multi-byte field",
     "memcpy(to, from, (size_t)S[i] * (size_t)elem_bytes);\n    }\n    return DCO_OK;\n}\n\n/*\n * Reverse",
     "memcpy(to, from, (size_t)S[i]);\n    }\n    return DCO_OK;\n}\n\n/*\n * Reverse", _gather_pins),
    ("scatter copies in the gather's direction",
     "const char* from = (const char*)arena + dst_tok_off[j] * elem_bytes;\n        memcpy(to, from,",
     "const char* from = (const char*)arena + dst_tok_off[j] * elem_bytes;\n        memcpy((void*)from, to,", _scatter_pins),
    ("scatter drops the first element of every sequence",
     "const char* from = (const char*)arena + dst_tok_off[j] * elem_bytes;\n        memcpy(to, from, (size_t)S[i] * (size_t)elem_bytes);",
     "const char* from = (const char*)arena + dst_tok_off[j] * elem_bytes;\n        memcpy(to + elem_bytes, from + elem_bytes, (size_t)(S[i] - 1) * (size_t)elem_bytes);",
     _scatter_pins),
    # ---- generalized advantage estimation
    ("lambda applied to the value term as well",
     "const double delta = r + gamma * next_V - V;", "const double delta = r + gamma * lambda * next_V - V;", _gae_pins),
    ("gamma missing from the recursion",
     "const double A = delta + gamma * lambda * next_A;", "const double A = delta + lambda * next_A;", _gae_pins),
    ("value of the NEXT token (masked or not) instead of the next loss-bearing one",
     "if (!mask[x]) { adv_tok[x] = 0.0f; ret_tok[x] = 0.0f; continue; }",
     "if (!mask[x]) { adv_tok[x] = 0.0f; ret_tok[x] = 0.0f; next_V = (double)value[x]; continue; }", _gae_pins),
    ("KL penalty with the wrong sign",
     "r = -kl_coef * ((double)logp[x] - (double)ref_logp[x]);", "r = kl_coef * ((double)logp[x] - (double)ref_logp[x]);",
     _gae_pins),
    ("return without the value",
     "ret_tok[x] = (float)(A + V);", "ret_tok[x] = (float)A;", _gae_pins),
    ("score added on every loss-bearing token",
     "if (!seen_last) { r += (double)reward[i]; seen_last = 1; }", "r += (double)reward[i]; (void)seen_last;", _gae_pins),
]


@pytest.fixture
def planted(tmp_path):
    """Builds a mutated oracle and swaps it in; restores the real one afterwards."""
    real = oracle._load()

    def plant(old, new):
        text = open(SRC).read()
        assert text.count(old) == 1, f"snippet not found exactly once in dc_oracle.c: {old!r}"
        c_file, so_file = tmp_path / "mutant.c", tmp_path / "mutant.so"
        c_file.write_text(text.replace(old, new))
        subprocess.check_call(["gcc", "-O1", "-std=c11", "-w", "-shared", "-fPIC", "-o", str(so_file), str(c_file), "-lm"])
        lib = C.CDLL(str(so_file))
        for name in ("dco_balance", "dco_group_advantage", "dco_adv_broadcast", "dco_plan", "dco_gather",
                     "dco_scatter", "dco_gae"):
            getattr(lib, name).restype = C.c_int
        oracle._lib = lib

    yield plant
    oracle._lib = real


@pytest.mark.parametrize("what,old,new,pins", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_a_planted_mistake_fails_a_pin(planted, what, old, new, pins):
    pins()                                           # the pins pass on the real oracle ...
    planted(old, new)
    with pytest.raises((AssertionError, oracle.OracleError)):
        pins()                                       # ... and not on the mutated one
