"""Are the oracle's pins strong enough?  Each case plants one plausible mistake
in a copy of the oracle's C source (on the CPU, in a temporary directory),
builds it, and runs the pin tests of test_oracle_attention.py,
test_oracle_logprob_kl.py, test_oracle_sampling.py and test_oracle_prefill.py against the copy.  Every planted mistake must make at
least one pin fail; the unmodified source must pass them all."""
import inspect
import os

import pytest

import oracle as oracle_pkg
import test_oracle_attention as pins_attention
import test_oracle_logprob_kl as pins_logprob
import test_oracle_prefill as pins_prefill
import test_oracle_sampling as pins_sampling

SRC = os.path.join(os.path.dirname(oracle_pkg.__file__), "rollout_oracle.c")

# (name, text to find exactly once or n times, replacement, which pin module exposes it)
MUTANTS = [
    ("attention: scale dropped",
     "                s *= scale;\n                const double w = exp(s - m);",
     "                const double w = exp(s - m);", "attention"),
    ("attention: wrong kv head for a query head", "const int hkv = hq / G;", "const int hkv = hq % Hkv;",
     "attention"),
    ("attention: slot index off by one", "((size_t)hkv * P + j % P) * D;\n                double s = 0.0;\n"
     "                for (int d = 0; d < D; ++d)\n                    s += load_elem(q, qbase + d, dtype) * "
     "load_elem(k_pages, row + d, dtype);\n                s *= scale;\n                const double w",
     "((size_t)hkv * P + (j + 1) % P) * D;\n                double s = 0.0;\n"
     "                for (int d = 0; d < D; ++d)\n                    s += load_elem(q, qbase + d, dtype) * "
     "load_elem(k_pages, row + d, dtype);\n                s *= scale;\n                const double w",
     "attention"),
    ("attention: page table ignored",
     "const size_t page = (size_t)page_table[(size_t)b * max_pages + j / P];\n"
     "                const size_t row = page * page_elems + ((size_t)hkv * P + j % P) * D;\n"
     "                double s = 0.0;\n                for (int d = 0; d < D; ++d)\n"
     "                    s += load_elem(q, qbase + d, dtype) * load_elem(k_pages, row + d, dtype);\n"
     "                s *= scale;\n                const double w",
     "const size_t page = (size_t)(j / P) + 0 * (size_t)page_table[(size_t)b * max_pages];\n"
     "                const size_t row = page * page_elems + ((size_t)hkv * P + j % P) * D;\n"
     "                double s = 0.0;\n                for (int d = 0; d < D; ++d)\n"
     "                    s += load_elem(q, qbase + d, dtype) * load_elem(k_pages, row + d, dtype);\n"
     "                s *= scale;\n                const double w", "attention"),
    ("attention: weights not normalised", "                o[d] /= denom;", "                o[d] /= 1.0;",
     "attention"),
    ("attention: value rows read from K", "o[d] += w * load_elem(v_pages, row + d, dtype);",
     "o[d] += w * load_elem(k_pages, row + d, dtype);", "attention"),
    ("attention: exponent sign", "const double w = exp(s - m);", "const double w = exp(m - s);", "attention"),
    ("attention: query read backwards in the weight pass",
     "s += load_elem(q, qbase + d, dtype) * load_elem(k_pages, row + d, dtype);\n                s *= scale;\n"
     "                const double w",
     "s += load_elem(q, qbase + (D - 1 - d), dtype) * load_elem(k_pages, row + d, dtype);\n"
     "                s *= scale;\n                const double w", "attention"),
    ("widening: bfloat16 shift", "uint32_t u = (uint32_t)b << 16;", "uint32_t u = (uint32_t)b << 15;", "both"),
    ("widening: binary16 exponent bias", "v = ldexp((double)(f | 0x400), e - 25);",
     "v = ldexp((double)(f | 0x400), e - 24);", "both"),
    ("widening: binary16 subnormals", "v = ldexp((double)f, -24);", "v = 0.0;", "both"),
    ("kl: direction swapped", "acc += p * (la - lr);", "acc += exp(lr) * (lr - la);", "logprob"),
    ("kl: reference not normalised", "const double lr = load_elem(ref, base + v, dtype) - lse_r;",
     "const double lr = load_elem(ref, base + v, dtype) - lse_a;", "logprob"),
    ("kl: weights from the reference", "const double p = exp(la);", "const double p = exp(lr);", "logprob"),
    ("kl: term dropped", "acc += p * (la - lr);", "acc += p * la;", "logprob"),
    ("logp: gathered at the wrong token", "*logp_actor = load_elem(actor, base + (size_t)tok, dtype) - lse_a;",
     "*logp_actor = load_elem(actor, base + (size_t)(tok > 0 ? tok - 1 : 0), dtype) - lse_a;", "logprob"),
    ("logp: sign", "*logp_actor = load_elem(actor, base + (size_t)tok, dtype) - lse_a;",
     "*logp_actor = lse_a - load_elem(actor, base + (size_t)tok, dtype);", "logprob"),
    ("ref logp: normalised with the actor's lse", "*logp_ref = load_elem(ref, base + (size_t)tok, dtype) - lse_r;",
     "*logp_ref = load_elem(ref, base + (size_t)tok, dtype) - lse_a;", "logprob"),
    ("ref logp: gathered from the actor row", "*logp_ref = load_elem(ref, base + (size_t)tok, dtype) - lse_r;",
     "*logp_ref = load_elem(actor, base + (size_t)tok, dtype) - lse_r;", "logprob"),
    ("reward: penalty sign", "reward[i] = -kl_coef * penalty + (terminal ? terminal[i] : 0.0);",
     "reward[i] = kl_coef * penalty + (terminal ? terminal[i] : 0.0);", "logprob"),
    ("reward: terminal score dropped", "reward[i] = -kl_coef * penalty + (terminal ? terminal[i] : 0.0);",
     "reward[i] = -kl_coef * penalty;", "logprob"),
    ("reward: sampled penalty swapped", "const double penalty = sampled_penalty ? lpa - lpr : kl;",
     "const double penalty = sampled_penalty ? lpr - lpa : kl;", "logprob"),
    ("reward: penalty modes exchanged", "const double penalty = sampled_penalty ? lpa - lpr : kl;",
     "const double penalty = sampled_penalty ? kl : lpa - lpr;", "logprob"),
    ("reward: stride ignored", "score_row(actor, ref, (size_t)i * (size_t)stride, V, dtype, tok, &lpa, &lpr, &kl);",
     "score_row(actor, ref, (size_t)i * (size_t)V, V, dtype, tok, &lpa, &lpr, &kl);", "logprob"),
    ("logp: base-2 logarithm", "const double lse_a = ma + log(sa);", "const double lse_a = ma + log2(sa);",
     "logprob"),
    ("logp: maximum not added back", "const double lse_a = ma + log(sa);", "const double lse_a = log(sa);",
     "logprob"),
    ("rows: stride ignored", "const size_t base = (size_t)i * (size_t)stride;",
     "const size_t base = (size_t)i * (size_t)V;", "logprob"),
    ("philox: nine rounds", "for (int round = 0; round < 10; ++round) {", "for (int round = 0; round < 9; ++round) {",
     "sampling"),
    ("philox: multipliers exchanged", "const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;",
     "const uint64_t M0 = 0xCD9E8D57u, M1 = 0xD2511F53u;", "sampling"),
    ("philox: key not advanced", "        k1 += 0xBB67AE85u;\n", "", "sampling"),
    ("sampling: wrong word of the block", "return ((double)(r[v % 4] >> 9) + 0.5)",
     "return ((double)(r[(v + 1) % 4] >> 9) + 0.5)", "sampling"),
    ("sampling: row not in the counter", "(uint32_t)(v / 4), (uint32_t)row, (uint32_t)offset",
     "(uint32_t)(v / 4), 0u, (uint32_t)offset", "sampling"),
    ("sampling: noise sign", "z += -log(-log(sampling_uniform(i, v, seed, offset)));",
     "z += log(-log(sampling_uniform(i, v, seed, offset)));", "sampling"),
    ("sampling: temperature ignored", "const double inv_t = temperature > 0.0 ? 1.0 / temperature : 1.0;",
     "const double inv_t = 1.0 + 0.0 * temperature;", "sampling"),
    ("sampling: ties to the last index", "            if (z > best_z) {", "            if (z >= best_z) {",
     "sampling"),
    ("sampling: logp without the temperature", "s += exp(load_elem(logits, base + v, dtype) * inv_t - m);",
     "s += exp(load_elem(logits, base + v, dtype) - m);", "sampling"),
    ("prefill: query cannot see itself", "                for (int j = 0; j <= p; ++j) {\n                    const size_t page = (size_t)page_table[(size_t)b * max_pages + j / P];\n                    const size_t row = page * page_elems + ((size_t)hkv * P + j % P) * D;\n                    double s = 0.0;\n                    for (int d = 0; d < D; ++d)\n                        s += load_elem(q, qbase + d, dtype) * load_elem(k_pages, row + d, dtype);\n                    const double w",
     "                for (int j = 0; j < p + (p == 0); ++j) {\n                    const size_t page = (size_t)page_table[(size_t)b * max_pages + j / P];\n                    const size_t row = page * page_elems + ((size_t)hkv * P + j % P) * D;\n                    double s = 0.0;\n                    for (int d = 0; d < D; ++d)\n                        s += load_elem(q, qbase + d, dtype) * load_elem(k_pages, row + d, dtype);\n                    const double w", "prefill"),
    ("prefill: no causal mask", "const int p = first + i;          /* last key this query may see */",
     "const int p = seq_lens[b] - 1 + 0 * (first + i);", "prefill"),
    ("prefill: block placed at the start of the cache", "const int first = seq_lens[b] - n;\n#pragma omp",
     "const int first = 0 * (seq_lens[b] - n);\n#pragma omp", "prefill"),
    ("prefill: wrong head group", "const int p = first + i;          /* last key this query may see */\n                const int hkv = hq / G;",
     "const int p = first + i;          /* last key this query may see */\n                const int hkv = hq % Hkv;", "prefill"),
    ("prefill: scale dropped", "const double w = exp(s * scale - m);", "const double w = exp(s - m);", "prefill"),
    ("top-k: threshold one rank too low", "const double tau = sorted[k - 1];", "const double tau = sorted[k < V ? k : V - 1];",
     "sampling"),
    ("top-k: sorted upwards", "return (x < y) - (x > y);", "return (x > y) - (x < y);", "sampling"),
    ("top-k: ties at the threshold dropped", "            const int kept = a >= tau;", "            const int kept = a > tau || v == 0;",
     "sampling"),
    ("top-k: log-prob normalised over the whole row", "            if (a >= tau)\n                s += exp(a * inv_t - m);",
     "            s += exp(a * inv_t - m);", "sampling"),
    ("top-k: noise of another entry", "z += -log(-log(sampling_uniform(i, v, seed, offset)));\n                ++count;",
     "z += -log(-log(sampling_uniform(i, count, seed, offset)));\n                ++count;", "sampling"),
    ("top-k: best score not restricted to survivors", "            double z = -INFINITY;\n            if (kept) {",
     "            double z = -INFINITY;\n            if (kept || a >= tau - 1.0) {", "sampling"),
    ("padding: not zeroed", "            logp[i] = 0.0;\n            kl[i] = 0.0;\n            continue;",
     "            logp[i] = -1.0;\n            kl[i] = 0.0;\n            continue;", "logprob"),
]


def _pins(which):
    mods = {"attention": [pins_attention], "logprob": [pins_logprob], "sampling": [pins_sampling],
            "prefill": [pins_prefill],
            "both": [pins_attention, pins_logprob], "all": [pins_attention, pins_logprob, pins_sampling, pins_prefill]}[which]
    out = []
    for mod in mods:
        for name, fn in sorted(vars(mod).items()):
            if name.startswith("test_") and list(inspect.signature(fn).parameters) == ["oracle"]:
                out.append(fn)
    return out


def _build_variant(tmp_path, text, tag):
    src = tmp_path / f"oracle_{tag}.c"
    src.write_text(text)
    lib = str(tmp_path / f"liboracle_{tag}.so")
    oracle_pkg.build(force=True, src=str(src), lib=lib)
    return oracle_pkg.OracleLib(lib)


def _first_failure(lib, pins):
    for fn in pins:
        try:
            fn(lib)
        except AssertionError as e:
            return f"{fn.__name__}: {str(e)[:80]}"
    return None


def test_unmodified_copy_passes_every_pin(tmp_path):
    lib = _build_variant(tmp_path, open(SRC).read(), "clean")
    assert len(_pins("all")) >= 40
    assert _first_failure(lib, _pins("all")) is None


@pytest.mark.parametrize("name,find,replace,which", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, find, replace, which):
    text = open(SRC).read()
    assert text.count(find) >= 1, "mutation pattern no longer matches the oracle source"
    lib = _build_variant(tmp_path, text.replace(find, replace), "mutant")
    failure = _first_failure(lib, _pins(which))
    assert failure is not None, f"no pin noticed: {name}"
