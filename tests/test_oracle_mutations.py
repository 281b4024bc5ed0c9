"""The pins must bite: plant one plausible mistake at a time in a COPY of the oracle (on the CPU) and check
that the pin suite fails for it.  The real oracle is never touched."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTATIONS = {
    # name: (text in the oracle source, replacement[, file under oracle/ if not symph_oracle.c])
    "kv_order_swapped_in_buffer": ("((int64_t)2 * l + kv) * prefix_lens[s]", "((int64_t)2 * l + 1 - kv) * prefix_lens[s]"),
    "buffer_token_major_instead_of_layer_major": ("(offsets[s] * 2 * n_layers + ((int64_t)2 * l + kv) * prefix_lens[s] + t) * row",
                                                  "((offsets[s] + t) * 2 * n_layers + ((int64_t)2 * l + kv)) * row"),
    "slot_index_wrong": ("const int64_t o = t % block_size;\n  *pool_elem = (int64_t)l * layer_stride + b * block_stride + o * row;\n  *buf_elem = (offsets[s] * 2 * n_layers",
                         "const int64_t o = (t + 1) % block_size;\n  *pool_elem = (int64_t)l * layer_stride + b * block_stride + o * row;\n  *buf_elem = (offsets[s] * 2 * n_layers"),
    "slot_index_wrong_batch_layers": ("const int64_t o = t % block_size;\n  *pool_elem = (int64_t)l * layer_stride + b * block_stride + o * row;\n  *buf_elem = ((int64_t)l * 2 * total",
                                      "const int64_t o = (t + 1) % block_size;\n  *pool_elem = (int64_t)l * layer_stride + b * block_stride + o * row;\n  *buf_elem = ((int64_t)l * 2 * total"),
    "gqa_head_modulo": ("const int32_t g = h / G;", "const int32_t g = h % n_kv_heads;"),
    "causal_excludes_self": ("const int64_t n_keys = (int64_t)P + i + 1;", "const int64_t n_keys = (int64_t)P + i;"),
    "causal_sees_future": ("const int64_t n_keys = (int64_t)P + i + 1;", "const int64_t n_keys = (int64_t)P + i + 2;"),
    "scale_dropped": ("x[j] = scale * dot;", "x[j] = dot;"),
    "no_normalisation": ("const double p = x[j] / Z;", "const double p = x[j];"),
    "v_read_from_k": ("const void* vb = in_pool ? v_base : v_new;", "const void* vb = in_pool ? k_base : k_new;"),
    "new_keys_offset_wrong": ("*elem = (((int64_t)cu_s + (j - P)) * n_kv_heads + g) * head_dim;",
                              "*elem = (((int64_t)(j - P)) * n_kv_heads + g) * head_dim;"),
    "bf16_widen_shift": ("<< 16;\n    float f;", "<< 15;\n    float f;"),
    "tail_starts_at_token_zero": ("const int64_t t = tail_begin[s] + i;", "const int64_t t = i;"),
    "tail_plane_stride_is_the_whole_length": ("((int64_t)2 * l + kv) * T + i) * row", "((int64_t)2 * l + kv) * prefix_lens[s] + i) * row"),
    "unit_v_rows_not_behind_the_k_rows": ("(chunk_rows[u] + (int64_t)kv * unit_lens[u] + t) * row", "(chunk_rows[u] + t) * row"),
    "unit_chunk_of_the_first_unit": ("(chunk_rows[u] + (int64_t)kv * unit_lens[u] + t) * row", "(chunk_rows[0] + (int64_t)kv * unit_lens[u] + t) * row"),
    "unit_slot_from_the_first_table_row": ("table[(int64_t)u * table_stride + t / block_size];", "table[t / block_size];"),
    "batch_layer_major_with_v_before_k": ("offsets[s] * 2 + (int64_t)kv * prefix_lens[s] + t) * row",
                                          "offsets[s] * 2 + (int64_t)(1 - kv) * prefix_lens[s] + t) * row"),
    "batch_layer_major_layer_stride_of_one_session": ("*buf_elem = ((int64_t)l * 2 * total + offsets[s] * 2",
                                                      "*buf_elem = ((int64_t)l * 2 * prefix_lens[s] + offsets[s] * 2"),
    "row_map_names_the_other_pool": ("kv_of_row[be / row] = (uint8_t)kv;", "kv_of_row[be / row] = (uint8_t)(1 - kv);"),
    # the residency oracle (priority.py)
    "admits_later_layers_first": ("keyed.append((layer, -blocks_of(n_tokens, block_size), sid))",
                                  "keyed.append((-layer, -blocks_of(n_tokens, block_size), sid))", "priority.py"),
    "admits_smallest_caches_first": ("keyed.append((layer, -blocks_of(n_tokens, block_size), sid))",
                                     "keyed.append((layer, blocks_of(n_tokens, block_size), sid))", "priority.py"),
    "stops_at_the_first_unit_that_does_not_fit": ("            r[sid] += 1\n            used += b\n",
                                                  "            r[sid] += 1\n            used += b\n        else:\n            break\n",
                                                  "priority.py"),
    "gives_up_largest_caches_first": ("keyed.append((-layer, blocks_of(sessions[sid], block_size), -sid))",
                                      "keyed.append((-layer, -blocks_of(sessions[sid], block_size), -sid))", "priority.py"),
    "gives_up_lower_layers_first": ("return [(-neg_layer, -neg_sid) for neg_layer, _, neg_sid in keyed]",
                                    "return [(-neg_layer, -neg_sid) for neg_layer, _, neg_sid in keyed[::-1]]", "priority.py"),
    "partial_last_block_not_counted": ("return -(-n_tokens // block_size)", "return max(1, n_tokens // block_size)", "priority.py"),
    "eviction_frees_one_slot_per_unit": ("        free_now += blocks_of(sessions[sid], block_size)\n", "        free_now += 1\n", "priority.py"),
}


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pins_fail_on_planted_mistake(tmp_path, name):
    old, new, *where = MUTATIONS[name]
    target = where[0] if where else "symph_oracle.c"
    src = open(os.path.join(ROOT, "oracle", target)).read()
    assert src.count(old) == 1, f"mutation anchor for {name} not found exactly once"
    mroot = tmp_path / "root"
    (mroot / "oracle").mkdir(parents=True)
    for f in ("__init__.py", "priority.py", "symph_oracle.c"):
        shutil.copy(os.path.join(ROOT, "oracle", f), mroot / "oracle" / f)
    (mroot / "oracle" / target).write_text(src.replace(old, new))
    shutil.copytree(os.path.join(ROOT, "workloads"), mroot / "workloads")
    (mroot / "tests").mkdir()
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), mroot / "tests" / "golden")
    pins = "test_oracle_priority_pins.py" if target == "priority.py" else "test_oracle_pins.py"
    for f in ("conftest.py", pins):
        shutil.copy(os.path.join(ROOT, "tests", f), mroot / "tests" / f)
    env = dict(os.environ, PYTHONPATH=str(mroot), OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/" + pins],
                       cwd=str(mroot), env=env, capture_output=True, text=True, timeout=300)
    # 1 = a pin failed; a negative code = the mutant ran off its own scratch array and was aborted: caught too
    assert r.returncode != 0, f"pins did not catch {name}:\n{r.stdout[-2000:]}\n{r.stderr[-2000:]}"
