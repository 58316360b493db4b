"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source
(a dropped check, a wrong index, a wrong shift, a flipped comparison), compiles it on the CPU and
runs the same pin functions against it: at least one pin must fail.  The untouched source must
pass them all.  Nothing here runs on a GPU."""
import functools
import os
import subprocess

import pytest

import oracle
from oracle import hps_oracle

import test_oracle_dedup as dedup_pins
import test_oracle_lookup as lookup_pins
import test_oracle_lru as lru_pins
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "hps_oracle.c")

MUTANTS = [
    ("hash: wrong first shift", "x ^= x >> 30;", "x ^= x >> 31;"),
    ("hash: wrong multiplier", "0x94D049BB133111EBULL", "0x94D049BB133111EDULL"),
    ("hash: last xor-shift dropped", "    x ^= x >> 31;\n    return x;", "    return x;"),
    ("set: lower instead of upper hash half", "(uint32_t)(hpso_mix64((uint64_t)key) >> 32)", "(uint32_t)(hpso_mix64((uint64_t)key))"),
    ("set: off by one before the modulo", "return (uint64_t)h % c->S;", "return ((uint64_t)h + 1) % c->S;"),
    ("search: last way never looked at", "for (uint32_t w = 0; w < c->W; ++w)\n        if (c->K[s * c->W + w] == key)", "for (uint32_t w = 0; w + 1 < c->W || w == 0; ++w)\n        if (c->K[s * c->W + w] == key)"),
    ("query: miss index off by one", "miss_idx[n_miss] = (uint32_t)i;", "miss_idx[n_miss] = (uint32_t)i + 1;"),
    ("query: miss rows zeroed", "            miss_keys[n_miss] = q;\n            ++n_miss;", "            miss_keys[n_miss] = q;\n            ++n_miss;\n            memset(out + i * c->d, 0, sizeof(uint32_t) * c->d);"),
    ("query: row copied one word short", "            memcpy(out + i * c->d, c->V + (s * c->W + (uint64_t)w) * c->d,\n                   sizeof(uint32_t) * c->d);", "            memcpy(out + i * c->d, c->V + (s * c->W + (uint64_t)w) * c->d,\n                   sizeof(uint32_t) * (c->d - 1));"),
    ("query: reserved keys searched like others", "        if (!is_reserved(q)) {\n            s = hpso_set_of(c, q);\n            w = find_way(c, s, q);\n        }", "        {\n            s = hpso_set_of(c, q);\n            w = find_way(c, s, q);\n        }"),
    ("insert: cached keys inserted again", "        if (f >= 0) {                                   /* already cached: row ignored */", "        if (0) {"),
    ("insert: victim counter starts one too far", "w = c->C[s] % c->W;", "w = (c->C[s] + 1) % c->W;"),
    ("insert: victim counter never advances", "        c->C[s] += 1;\n        c->K[s * c->W + w] = q;", "        c->K[s * c->W + w] = q;"),
    ("insert: row of the previous batch element stored", "memcpy(c->V + (s * c->W + w) * c->d, vals + i * c->d, sizeof(uint32_t) * c->d);", "memcpy(c->V + (s * c->W + w) * c->d, vals + (i ? i - 1 : 0) * c->d, sizeof(uint32_t) * c->d);"),
    ("insert: reserved keys stored", "        if (is_reserved(q)) continue;\n        uint64_t s = hpso_set_of(c, q);\n        int f = find_way(c, s, q);", "        uint64_t s = hpso_set_of(c, q);\n        int f = find_way(c, s, q);"),
    ("update: absent keys inserted at way 0", "        int w = find_way(c, s, q);\n        if (w < 0) continue;\n        memcpy(c->V", "        int w = find_way(c, s, q);\n        if (w < 0) { w = 0; c->K[s * c->W] = q; }\n        memcpy(c->V"),
    ("update: cached rows left alone", "        if (w < 0) continue;\n        memcpy(c->V + (s * c->W + (uint64_t)w) * c->d, vals + i * c->d,\n               sizeof(uint32_t) * c->d);\n    }\n}\n\n/* Dump", "        if (w < 0) continue;\n    }\n}\n\n/* Dump"),
    ("dump: empty slots reported", "        if (c->K[i] != HPSO_EMPTY)\n            keys_out[m++] = c->K[i];", "        keys_out[m++] = c->K[i];"),
    ("lru: iteration count not advanced by query", "if (c->policy == 1) c->g += 1;", "if (c->policy == 2) c->g += 1;"),
    ("lru: query hit does not refresh the stamp", "if (c->policy == 1) c->T[s * c->W + (uint64_t)w] = c->g;   /* refresh the counter */", ""),
    ("lru: cached key in a Replace call not refreshed", "            if (c->policy == 1) c->T[s * c->W + (uint64_t)f] = c->g;\n            continue;", "            continue;"),
    ("lru: empty slots not taken first", "            int e = find_way(c, s, HPSO_EMPTY);         /* empty slots first */", "            int e = -1;"),
    ("lru: youngest instead of oldest evicted", "(uint32_t)(c->g - c->T[s * c->W + x]) > (uint32_t)(c->g - c->T[s * c->W + w])", "(uint32_t)(c->g - c->T[s * c->W + x]) < (uint32_t)(c->g - c->T[s * c->W + w])"),
    ("lru: ties go to the highest way", "(uint32_t)(c->g - c->T[s * c->W + x]) > (uint32_t)(c->g - c->T[s * c->W + w])", "(uint32_t)(c->g - c->T[s * c->W + x]) >= (uint32_t)(c->g - c->T[s * c->W + w])"),
    ("lru: stamps compared without wrap-around", "(uint32_t)(c->g - c->T[s * c->W + x]) > (uint32_t)(c->g - c->T[s * c->W + w])", "c->T[s * c->W + x] < c->T[s * c->W + w]"),
    ("dedup: only the previous distinct key is compared", "        uint64_t j = 0;\n        while (j < u && unique_out[j] != keys[i]) ++j;", "        uint64_t j = u ? u - 1 : 0;\n        while (j < u && unique_out[j] != keys[i]) ++j;"),
    ("dedup: place counted from one", "        inverse_out[i] = (uint32_t)j;", "        inverse_out[i] = (uint32_t)j + 1;"),
    ("dedup: a repeated key is listed again", "        if (j == u) unique_out[u++] = keys[i];", "        if (j == u || j == 0) unique_out[u++] = keys[i];"),
    ("expand: position used instead of the map", "memcpy(out + i * d, rows + (uint64_t)inverse[i] * d, sizeof(uint32_t) * d);", "memcpy(out + i * d, rows + (i < 37 ? i : 0) * d, sizeof(uint32_t) * d);"),
    ("lookup: hit rate divides by the cache size", "float rate = 1.0f - (float)m / (float)n;", "float rate = 1.0f - (float)m / (float)(c->S * c->W);"),
    ("lookup: a hit rate equal to the threshold counts as below it", "        if (rate < t) {", "        if (rate <= t) {"),
    ("lookup: decision taken in double precision", "float rate = 1.0f - (float)m / (float)n;", "double rate = 1.0 - (double)m / (double)n;"),
    ("lookup: default vector handed out in synchronous mode", "memcpy(out + (uint64_t)miss_idx[j] * c->d, lower + (uint64_t)miss_idx[j] * c->d,", "memcpy(out + (uint64_t)miss_idx[j] * c->d, default_row,"),
    ("lookup: a repeated missing key is fetched again", "while (e < u && ins_keys[e] != miss_keys[j]) ++e;", "e = u;"),
    ("lookup: fetched row taken by list index instead of position", "memcpy(ins_rows + u * c->d, lower + (uint64_t)miss_idx[j] * c->d,", "memcpy(ins_rows + u * c->d, lower + j * c->d,"),
    ("lookup: nothing inserted in asynchronous mode", "if (do_insert) hpso_insert(c, ins_keys, ins_rows, u);", "if (do_insert && *synchronous) hpso_insert(c, ins_keys, ins_rows, u);"),
    ("lookup: cached rows replaced by the lower tiers' rows", "    uint64_t m = hpso_query(c, keys, n, out, miss_idx, miss_keys);", "    uint64_t m = hpso_query(c, keys, n, out, miss_idx, miss_keys);\n    memcpy(out, lower, sizeof(uint32_t) * n * c->d);"),
    ("lru: new key not stamped", "            c->T[s * c->W + w] = c->g;\n        }\n        c->C[s] += 1;", "        }\n        c->C[s] += 1;"),
]


def build(tmp_path, name, text):
    src = tmp_path / f"{name}.c"
    lib = tmp_path / f"lib{name}.so"
    src.write_text(text)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", str(src), "-o", str(lib)], check=True)
    return hps_oracle.load_library(str(lib))


def battery(lib, monkeypatch):
    """Runs the pins against `lib`; returns the name of the first pin that fails, or None."""
    cache = functools.partial(hps_oracle.OracleCache, lib=lib)
    for mod in (pins, lru_pins, lookup_pins):
        monkeypatch.setattr(mod, "OracleCache", cache)
    monkeypatch.setattr(pins, "mix64", functools.partial(hps_oracle.mix64, lib=lib))
    monkeypatch.setattr(oracle, "set_of", functools.partial(hps_oracle.set_of, lib=lib))
    monkeypatch.setattr(oracle, "dedup", functools.partial(hps_oracle.dedup, lib=lib))
    monkeypatch.setattr(oracle, "expand", functools.partial(hps_oracle.expand, lib=lib))
    checks = [
        ("published hash vectors", pins.test_mix64_published_vectors),
        ("hash vs big integers", pins.test_mix64_against_bigint_many_keys),
        ("set mapping S=25", lambda: pins.test_set_of_uses_upper_32_bits_mod_S(25)),
        ("set mapping S=4096", lambda: pins.test_set_of_uses_upper_32_bits_mod_S(4096)),
        ("contract details: query", pins.test_duplicates_and_reserved_keys_in_query),
        ("contract details: insert/update", pins.test_insert_ignores_existing_and_duplicates_take_first),
        ("empty batches", pins.test_empty_batches_and_bad_geometry),
        ("dict", pins.test_no_overflow_behaves_like_dict),
        ("deque W=2", lambda: pins.test_one_set_is_a_fifo_deque(2)),
        ("deque W=8", lambda: pins.test_one_set_is_a_fifo_deque(8)),
        ("direct mapped", pins.test_direct_mapped_last_writer_of_set_wins),
        ("fully associative", pins.test_single_set_fully_associative_fifo),
        ("brute force 3x2", lambda: pins.test_brute_force_random_op_sequences(3, 2)),
        ("brute force 7x8", lambda: pins.test_brute_force_random_op_sequences(7, 8)),
        ("lru textbook W=4", lambda: lru_pins.test_single_key_calls_are_textbook_lru(4)),
        ("lru per set", lru_pins.test_each_set_is_its_own_lru),
        ("lru batched model 3x2", lambda: lru_pins.test_batched_calls_match_independent_model(3, 2)),
        ("lru batched model 7x8", lambda: lru_pins.test_batched_calls_match_independent_model(7, 8)),
        ("lru touched keys survive", lru_pins.test_keys_touched_by_a_call_outlive_untouched_ones),
        ("policy 0 ignores stamps", lru_pins.test_policy0_is_unaffected_by_stamps),
        ("dedup worked example", dedup_pins.test_worked_example),
        ("dedup degenerate batches", dedup_pins.test_degenerate_batches),
        ("dedup vs set/dict/numpy", lambda: dedup_pins.test_against_set_dict_and_numpy_unique(1, 1.05)),
        ("dedup brute force", dedup_pins.test_brute_force_small_alphabets),
        ("expand is a gather", dedup_pins.test_expand_is_a_row_gather),
        ("alg 1 worked batch", lookup_pins.test_worked_batch_at_and_above_the_threshold),
        ("alg 1 degenerate batches", lookup_pins.test_degenerate_batches),
        ("alg 1 single precision", lookup_pins.test_decision_is_taken_in_single_precision),
        ("alg 1 over a dict", lambda: lookup_pins.test_against_alg1_over_a_dict(3, 0.6)),
    ]
    for name, fn in checks:
        try:
            fn()
        except (AssertionError, ValueError, IndexError, KeyError):
            return name
    return None


def test_untouched_source_passes_the_battery(tmp_path, monkeypatch):
    lib = build(tmp_path, "pristine", open(SRC).read())
    assert battery(lib, monkeypatch) is None


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"pattern for '{name}' must occur exactly once in the oracle source"
    lib = build(tmp_path, "mutant", text.replace(old, new))
    caught_by = battery(lib, monkeypatch)
    assert caught_by is not None, f"no pin notices: {name}"
