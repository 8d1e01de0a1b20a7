"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's source (text
substitution, compiled to a temporary library, CPU only) and checks that a pin which passes on the
real oracle fails on the mutant.  If a snippet no longer occurs in the source the case fails loudly, so
the list cannot silently rot.  (Letting the partial tail block be a candidate is not in the list: it is
an equivalent mutant, the tail is always a window block because Nw >= 1.)"""
import ctypes
import os
import subprocess
import tempfile

import numpy as np
import pytest

import oracle
import test_oracle_attention as t_att
import test_oracle_load as t_load
import test_oracle_select as t_sel
import test_oracle_append as t_app
import test_oracle_evict as t_ev

SRC = os.path.join(os.path.dirname(oracle.__file__), "nosa_oracle.c")

MUTANTS = [
    # (name, original snippet, planted mistake, pin that must now fail)
    ("bias dropped from the logit", "if (pool_bias) zz += (double)pool_bias[((int64_t)u * C + s) * nb + r];", "",
     lambda: t_att.test_brute_force_masked_dense_attention("bf16", 17)),
    ("scale also applied to the bias", "double zz = p->softmax_scale * dot;\n          if (pool_bias) zz += (double)pool_bias[((int64_t)u * C + s) * nb + r];",
     "double zz = dot;\n          if (pool_bias) zz += (double)pool_bias[((int64_t)u * C + s) * nb + r];\n          zz *= p->softmax_scale;",
     lambda: t_att.test_brute_force_masked_dense_attention("fp32", 0)),
    ("tail mask off by one", "if (t >= T) break;", "if (t > T) break;",
     lambda: t_att.test_brute_force_masked_dense_attention("fp32", 63)),
    ("slot indirection ignored (block index used as slot)", "const int J = sel[i], s = sob[J];\n        if (s < 0) { ++bad; continue; }\n        for (int r = 0; r < nb; ++r) {\n          const int t = J * nb + r;",
     "const int J = sel[i], s = sob[J] < 0 ? -1 : (J % C);\n        if (s < 0) { ++bad; continue; }\n        for (int r = 0; r < nb; ++r) {\n          const int t = J * nb + r;",
     lambda: t_att.test_brute_force_masked_dense_attention("bf16", 0)),
    ("value read from the key pool", "o[e] += w * load_elem(pool_v, vb + e, p->dtype);", "o[e] += w * load_elem(pool_k, vb + e, p->dtype);",
     lambda: t_att.test_select_all_no_bias_is_textbook_attention("fp32")),
    ("lse without the max", "lse[(int64_t)b * p->n_q_heads + hq] = zmax + log(denom);", "lse[(int64_t)b * p->n_q_heads + hq] = log(denom);",
     lambda: t_att.test_chunked_lse_merge_equals_one_shot()),
    ("ties go to the higher index", "if (best < 0 || s[J] > s[best]) best = J;", "if (best < 0 || s[J] >= s[best]) best = J;",
     lambda: t_sel.test_single_pass_infinity_form(False)),
    ("window forgets the tail block", "const int window = J >= N - p->window_blocks;", "const int window = J >= N - p->window_blocks && J < N - 1;",
     lambda: t_sel.test_per_batch_token_counts()),
    ("query-agnostic fill ranks by the query-aware score", "const int J = arg_best(se, elig, Nc);", "const int J = arg_best(sq, elig, Nc);",
     lambda: t_sel.test_exhaustive_subset_search(64 * 12, 6, 2, 1, 1)),
    ("Ke forgets the forced blocks", "int ke = K - nF - p->kq_blocks;", "int ke = K - p->kq_blocks;",
     lambda: t_sel.test_invariants_and_best_agnostic_always_selected()),
    ("group sum replaced by the last head", "sgroup += dot;", "sgroup = dot;",
     lambda: t_sel.test_pooled_key_score_equals_pooled_token_scores("fp32")),
    ("sub-block crossing a block edge is kept", "if (hi > (J + 1) * nb || J >= p->max_blocks) continue;", "if (J >= p->max_blocks) continue;",
     lambda: t_sel.test_two_stage_pooling_geometry(32, 16)),
    ("mean divides by lk + 1", "s /= (double)lk;", "s /= (double)(lk + 1);",
     lambda: t_sel.test_pool_rounds_to_nearest_even_bf16()),
    ("victim may hold a selected block", "while (s < C && bos[s] >= 0 && in_gamma[bos[s]]) ++s;   /* next victim */", "while (0) ++s;",
     lambda: t_load.test_theorem1_locality_bound_over_steps(8, 2, 1, 1, 8, 32)),
    ("evicted block keeps its stale map entry", "if (bos[s] >= 0) sob[bos[s]] = -1;\n      bos[s] = J; sob[J] = s;\n      ll[2 * nl] = J; ll[2 * nl + 1] = s;\n      ++nl; ++s;",
     "bos[s] = J; sob[J] = s;\n      ll[2 * nl] = J; ll[2 * nl + 1] = s;\n      ++nl; ++s;",
     lambda: t_load.test_theorem1_locality_bound_over_steps(8, 2, 1, 1, 8, 32)),
    ("fetch forgets the bias", "if (host_bias && pool_bias) memcpy(pool_bias + dst * nb, host_bias + src * nb, (size_t)nb * 4);", "",
     lambda: t_load.test_full_step_through_pool_equals_bruteforce_on_host_cache()),
    ("appended token goes to the wrong row of the slot", "const size_t prow = ((size_t)u * C + sob[J]) * nb + row;", "const size_t prow = ((size_t)u * C + sob[J]) * nb + (row + 1) % nb;",
     lambda: t_app.test_append_places_tokens_and_keeps_attention_and_fetch_bound()),
    ("new block evicts the most important resident block", "< se_blk[(int64_t)u * p->max_blocks + bos[best]]) best = s;", "> se_blk[(int64_t)u * p->max_blocks + bos[best]]) best = s;",
     lambda: t_app.test_append_places_tokens_and_keeps_attention_and_fetch_bound()),
    ("the block that leaves the window may not give up its slot", "const int protect = p->window_blocks;", "const int protect = p->window_blocks > 2 ? p->window_blocks : 2;",
     lambda: t_app.test_fetch_bound_holds_across_block_boundaries_for_tight_budgets(1, 1, 0, 1)),
    ("token fetch reads the host row at the pool's row index", "const size_t src = (size_t)u * p->max_blocks * nb + t, dst = (size_t)u * C * nb + r;",
     "const size_t src = (size_t)u * p->max_blocks * nb + r, dst = (size_t)u * C * nb + r;",
     lambda: t_load.test_token_fetch_is_a_row_gather("bf16")),
    ("token fetch copies the key row into the value pool", "memcpy((char *)pool_v + dst * rowb, (const char *)host_v + src * rowb, rowb);",
     "memcpy((char *)pool_v + dst * rowb, (const char *)host_k + src * rowb, rowb);",
     lambda: t_load.test_token_fetch_of_whole_blocks_equals_block_fetch()),
    ("softplus without the linear part", "return (x > 0 ? x : 0) + log1p(exp(-fabs(x)));", "return log1p(exp(-fabs(x)));",
     lambda: t_ev.test_softplus_closed_forms_through_the_head()),
    ("eviction head reads the key instead of the value", "const int64_t vb = (int64_t)b * row + (int64_t)(Hq + Hkv + h) * d;", "const int64_t vb = (int64_t)b * row + (int64_t)(Hq + h) * d;",
     lambda: t_ev.test_eviction_head_against_torch_softplus("fp32", 0)),
]


@pytest.fixture()
def real_oracle():
    keep = oracle._lib
    yield
    oracle._lib = keep


@pytest.mark.parametrize("name,old,new,pin", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pin_catches_planted_mistake(name, old, new, pin, real_oracle):
    src = open(SRC).read()
    assert src.count(old) == 1, f"snippet for '{name}' not found exactly once in the oracle source"
    pin()                                                    # passes on the real oracle
    with tempfile.TemporaryDirectory() as tmp:
        c, so = os.path.join(tmp, "mutant.c"), os.path.join(tmp, "mutant.so")
        open(c, "w").write(src.replace(old, new))
        subprocess.run(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-w", "-o", so, c, "-lm"], check=True)
        lib = ctypes.CDLL(so)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_attention.restype = ctypes.c_int
        oracle._lib = lib
        with pytest.raises((AssertionError, RuntimeError)):
            pin()
