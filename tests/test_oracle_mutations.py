"""The pins must be able to see a mistake: each plausible bug, planted in a copy of the oracle's C source (on the
CPU, in a temporary library), has to make at least one pin of test_oracle_pins.py fail.  The oracle that ships is
never touched; the HIP path is not involved."""
import ctypes
import os
import subprocess

import pytest

from oracle import treeattn_oracle as O

from . import test_oracle_pins as pins

# (name, text in tree_attn_oracle.c, replacement)
MUTATIONS = [
    ("node does not attend to itself", "    int n = 0, cur = i;\n", "    int n = 0, cur = parent[i];\n"),
    ("siblings visible (flattened-order causal mask)", "        cur = parent[cur];\n", "        cur = cur - 1;\n"),
    ("query head h reads KV head h mod Hkv", "const int g = h / (p->Hq / p->Hkv);", "const int g = h % p->Hkv;"),
    ("tree token at the wrong cache position", "int64_t pos = t < W ? S + t : L + path[t - W];\n        int64_t ko",
     "int64_t pos = t < L ? t : L + (path[t - L] + 1) % p->T;\n        int64_t ko"),
    ("value row of another key", "int64_t pos = t < W ? S + t : L + path[t - W];\n        int64_t vo",
     "int64_t pos = t < L ? (L - 1 - t) : L + path[t - L];\n        int64_t vo"),
    ("scale dropped", "scores[t] = p->scale * dot;", "scores[t] = dot;"),
    ("page table ignored", "page = p->page_table[(int64_t)b * p->max_pages + pos / p->page_size];",
     "page = (int64_t)b * p->max_pages + pos / p->page_size;"),
    ("slot inside the page off by one", "slot = pos % p->page_size;", "slot = (pos + 1) % p->page_size;"),
    ("log-sum-exp without the subtracted maximum", "*lse_out = smax + log(denom);", "*lse_out = log(denom);"),
    ("last prefix token dropped", "        scores[t] = p->scale * dot;\n",
     "        scores[t] = (t == L - 1) ? -INFINITY : p->scale * dot;\n"),
    ("window start ignored", "const int64_t S = p->kv_start ? p->kv_start[b] : 0;", "const int64_t S = 0;"),
    ("window off by one", "const int64_t W = L - S;", "const int64_t W = L - S + (S > 0);"),
    ("query range starts at node 0 whatever the offset", "root_path(par, p->T, p->q_off + i, path);",
     "root_path(par, p->T, i, path);"),
]


def _battery():
    """Calls the pins one by one; returns the names of those that fail."""
    calls = [(pins.test_chain_tree_is_causal_attention, dict(dtype="bf16", L=37)),
             (pins.test_chain_tree_is_causal_attention, dict(dtype="f32", L=0)),
             (pins.test_single_node_is_decode_attention, dict(paged=True)),
             (pins.test_brute_force_every_tree_shape, dict(T=4)),
             (pins.test_brute_force_gqa_and_seven_node_binary_tree, {}),
             (pins.test_zero_query_counts_attended_keys, {}),
             (pins.test_non_ancestors_are_invisible_and_ancestors_are_not, {}),
             (pins.test_planted_key_selects_its_value_row, {}),
             (pins.test_path_unrolling_equals_causal_prefill, {}),
             (pins.test_relabelling_nodes_permutes_outputs, {}),
             (pins.test_page_permutation_and_layout_do_not_matter, {}),
             (pins.test_query_head_reads_kv_head_h_div_g, {}),
             (pins.test_constant_values_and_no_garbage_leak, {}),
             (pins.test_scale_is_applied_to_scores, {}),
             (pins.test_window_start_equals_a_cache_that_begins_there, {}),
             (pins.test_window_start_zero_query_counts_keys_and_hides_what_lies_before, {}),
             (pins.test_query_subset_equals_those_rows_of_the_whole_tree, {})]
    failed = []
    for fn, kw in calls:
        try:
            fn(**kw)
        except AssertionError:
            failed.append(fn.__name__)
    return failed


def test_the_unmutated_oracle_passes_the_battery():
    assert _battery() == []


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, old, new, tmp_path, monkeypatch):
    src = open(O._SRC).read()
    assert src.count(old) == 1, "mutation anchor not unique: %r" % old
    mutated = tmp_path / "oracle_mutant.c"
    mutated.write_text(src.replace(old, new))
    lib_path = str(tmp_path / "liboracle_mutant.so")
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-std=c99", str(mutated), "-o", lib_path, "-lm"])
    real = O._load()
    lib = ctypes.CDLL(lib_path)
    for fn in ("tree_attn_oracle", "tree_attn_oracle_sample", "tree_attn_oracle_threads"):
        getattr(lib, fn).restype = getattr(real, fn).restype
        getattr(lib, fn).argtypes = getattr(real, fn).argtypes
    monkeypatch.setattr(O, "_lib", lib)
    failed = _battery()
    assert failed, "no pin noticed: " + name
