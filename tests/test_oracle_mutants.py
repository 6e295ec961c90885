"""The pins are sharp: plausible mistakes planted in the oracle (on the CPU, in a
temporary copy of its source) each make at least one pin fail."""
import os
import subprocess
import tempfile

import pytest

import oracle
import test_oracle_alias as t_alias
import test_oracle_counts_loglik as t_counts
import test_oracle_mh as t_mh
import test_oracle_philox as t_philox
import test_oracle_doc_refresh as t_refresh

SRC = os.path.join(os.path.dirname(oracle.__file__), "ldaref.c")


def pins_mh(mod):
    doff, words = t_mh.tiny_corpus()
    o = mod.Oracle(doff, words, t_mh.V, t_mh.K, t_mh.ALPHA, t_mh.BETA, seed=42)
    o.build_alias()
    setup = (o, doff, words)
    t_mh.test_detailed_balance_of_coded_acceptance(mod, setup, 6)
    t_mh.test_word_table_is_word_proposal(mod, setup)
    t_mh.test_chain_matches_exact_m_step_distribution(mod, setup, 0, 1)
    t_mh.test_chain_matches_exact_m_step_distribution(mod, setup, 6, 2)
    t_mh.test_doc_draw_histogram(mod)


def pins_alias(mod):
    t_alias.test_adversarial_shapes(mod)
    t_alias.test_dense_row_matches_word_proposal(mod)


def pins_counts(mod):
    t_counts.test_counts_invariants_and_recount(mod)
    t_counts.test_initial_assignment_rule(mod)
    t_counts.test_loglik_matches_scipy(mod)
    t_counts.test_incremental_update_equals_recount(mod)


def pins_refresh(mod):
    t_refresh.test_sweep_is_the_fold_of_chains_in_token_order(mod)


def pins_philox(mod):
    t_philox.test_known_answer_vectors(mod)


# (name, text in ldaref.c, replacement, pins expected to catch it)
MUTANTS = [
    ("dropped factor in Eq. 8", "        num = num * ((double)nk_t + betabar);\n", "", pins_mh),
    ("wrong sign of the exclusion", "double num = ((double)(ndk_t - mt) + alpha);",
     "double num = ((double)(ndk_t + mt) + alpha);", pins_mh),
    ("no exclusion of the token itself", "const int32_t ms = (s == z0) ? 1 : 0;",
     "const int32_t ms = 0;", pins_mh),
    ("transposed proposal factors (word)", "        num = num * ((double)nkw_s + beta);\n",
     "        num = num * ((double)nkw_t + beta);\n", pins_mh),
    ("transposed proposal factors (doc)", "        den = den * ((double)ndk_t + alpha);\n",
     "        den = den * ((double)ndk_s + alpha);\n", pins_mh),
    ("doc-proposal mixture weight", "if (u0 * ((double)L + alphabar) < (double)L) {",
     "if (u0 * ((double)L + alphabar) < alphabar) {", pins_mh),
    ("doc-proposal before word-proposal", "((j & 1) == 0) : (c->proposal_mode == 1);",
     "((j & 1) == 1) : (c->proposal_mode == 1);", pins_mh),
    ("accept uses the wrong random word", "c->nk[t], c->alpha, c->beta, c->betabar, x[2]))",
     "c->nk[t], c->alpha, c->beta, c->betabar, x[1]))", pins_mh),
    ("alias residual update", "            r -= C - m[li];\n", "            r -= C;\n", pins_alias),
    ("alias borrows from the wrong bin", "alias[h] = (r == C) ? (uint32_t)h : (uint32_t)hi;",
     "alias[h] = (uint32_t)h;", pins_alias),
    ("word-proposal numerator", "double a = ((double)nkw_row[k] + beta) / ((double)nk[k] + betabar);",
     "double a = ((double)nk[k] + beta) / ((double)nkw_row[k] + betabar);", pins_alias),
    ("Philox Weyl constant", "k1 += 0xBB67AE85u;", "k1 += 0xBB67AE86u;", pins_philox),
    ("Philox output order", "uint32_t n1 = (uint32_t)p1;", "uint32_t n1 = (uint32_t)p0;",
     pins_philox),
    ("n_k not counted per token", "        c->nk[c->z[g]] += 1;\n", "        c->nk[c->z[g]] = 1;\n",
     pins_counts),
    ("incremental update moves the count the wrong way", "        c->nk[a] -= 1;\n",
     "        c->nk[a] += 1;\n", pins_counts),
    ("doc side not refreshed after a token", "                zcur[g - b] = s;\n", "", pins_refresh),
    ("initial topic from the wrong counter", "token_random(seed, (uint64_t)g, 0xFFFFFFFFu, 0u, x);",
     "token_random(seed, (uint64_t)g, 0u, 0u, x);", pins_counts),
    ("log-likelihood misses lgamma(alpha)", "kadd(&sd, lgamma((double)ndk[k] + c->alpha) - lga);",
     "kadd(&sd, lgamma((double)ndk[k] + c->alpha));", pins_counts),
]


class Shim:
    """The oracle module with its library swapped for a mutant."""

    def __init__(self, lib):
        self._lib = lib

    def __getattr__(self, name):
        return getattr(oracle, name)


@pytest.fixture()
def swap_lib():
    saved = oracle._lib
    yield
    oracle._lib = saved


@pytest.mark.parametrize("name,old,new,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, old, new, pins, swap_lib, tmp_path):
    oracle.lib()
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site not unique: %r" % old
    c_path = tmp_path / "mutant.c"
    so_path = tmp_path / "libmutant.so"
    c_path.write_text(text.replace(old, new))
    subprocess.run(["gcc", *oracle.CFLAGS, "-Wno-unused-variable", "-Wno-unused-parameter",
                    "-o", str(so_path), str(c_path), "-lm"], check=True)
    oracle._lib = oracle.bind(str(so_path))
    with pytest.raises((AssertionError, oracle.OracleError)):
        pins(oracle)


def test_pins_pass_on_the_real_oracle(swap_lib):
    oracle._lib = oracle.bind(oracle.build_oracle())
    for pins in (pins_mh, pins_alias, pins_counts, pins_philox, pins_refresh):
        pins(oracle)
