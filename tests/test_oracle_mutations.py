"""Are the oracle's pins sharp?  Plant one plausible mistake at a time in a copy of the oracle's source (on the CPU, in a
temporary build) and require that the pin suite notices every one of them.  The unmutated build must pass the same battery."""
import os
import subprocess

import numpy as np
import pytest

import oracle as O
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.abspath(O.__file__)), "harvest_oracle.c")

# (what the mistake is, text to find, text to put)
MUTATIONS = [
    ("transposed pool indexing (slot-major instead of layer-major)",
     "return plane + ((uint64_t)layer * n_slots + slot) * c->chunk_bytes;",
     "return plane + ((uint64_t)slot * c->n_layers + layer) * c->chunk_bytes;"),
    ("cache-tier objects resolved through their host slot number",
     "case T_CACHE: return cache_at(c, plane, layer, (uint64_t)c->slot[id]);",
     "case T_CACHE: return cache_at(c, plane, layer, (uint64_t)c->host_slot[id] % c->n_cache_slots);"),
    ("host copy looked up by object number instead of host slot",
     "case T_HOST:  return at(c->host[plane], c, c->n_host_slots, layer, (uint64_t)c->host_slot[id]);",
     "case T_HOST:  return at(c->host[plane], c, c->n_host_slots, layer, (uint64_t)id);"),
    ("K and V destinations swapped in the KV fetch",
     "if (src) memcpy(dst[p] + (seq_dst_block[s] + j) * c->chunk_bytes, src, c->chunk_bytes);",
     "if (src) memcpy(dst[c->n_planes - 1 - p] + (seq_dst_block[s] + j) * c->chunk_bytes, src, c->chunk_bytes);"),
    ("sequence offset dropped from the destination index",
     "if (src) memcpy(dst[p] + (seq_dst_block[s] + j) * c->chunk_bytes, src, c->chunk_bytes);",
     "if (src) memcpy(dst[p] + (uint64_t)j * c->chunk_bytes, src, c->chunk_bytes);"),
    ("placement copies only the first layer",
     "for (uint32_t l = 0; l < c->n_layers; ++l)\n                        memcpy(cache_at(c, p, l, (uint64_t)s),",
     "for (uint32_t l = 0; l < 1; ++l)\n                        memcpy(cache_at(c, p, l, (uint64_t)s),"),
    ("placement takes the highest free slot",
     "int64_t s = lowest_free(c->cache_used, c->n_cache_slots);\n    if (s >= 0) c->cache_used[s] = 1;",
     "int64_t s = -1; for (int64_t q = (int64_t)c->n_cache_slots - 1; q >= 0; --q) if (!c->cache_used[q]) { s = q; break; }\n    if (s >= 0) c->cache_used[s] = 1;"),
    ("a full cache tier reported as success",
     "if (s < 0) st = ORC_ENOSPC;", "if (s < 0) st = ORC_OK;"),
    ("revocation forgets the generation",
     "c->slot[id] = -1; c->gen[id] += 1;\n    }\n    for (uint32_t i = 0; i < n; ++i) {               /* free (+ poison) */",
     "c->slot[id] = -1;\n    }\n    for (uint32_t i = 0; i < n; ++i) {               /* free (+ poison) */"),
    ("revocation never frees the slot",
     "cache_release(c, old[i]);", ";"),
    ("revoked lossy objects fall back to a host copy they do not have",
     "c->tier[id] = c->host_slot[id] >= 0 ? T_HOST : T_NONE;", "c->tier[id] = T_HOST;"),
    ("write-back skips the cache-tier copy",
     "if (c->tier[id] == T_CACHE)\n                    memcpy(cache_at(c, p, l, (uint64_t)c->slot[id]), s, c->chunk_bytes);",
     "if (0)\n                    memcpy(cache_at(c, p, l, (uint64_t)c->slot[id]), s, c->chunk_bytes);"),
    ("write-back skips the host copy",
     "if (c->host_slot[id] >= 0)\n                    memcpy(at(c->host[p], c, c->n_host_slots, l, (uint64_t)c->host_slot[id]), s, c->chunk_bytes);",
     "if (0)\n                    memcpy(at(c->host[p], c, c->n_host_slots, l, (uint64_t)c->host_slot[id]), s, c->chunk_bytes);"),
    ("all-layer write-back reads every layer from the first source layer",
     "uint64_t li = layer < 0 ? l : 0;", "uint64_t li = 0;"),
    ("demotion keeps the local slot",
     "c->local_used[c->slot[id]] = 0;", ""),
    ("cache hits listed as misses",
     "case T_CACHE: k.n_cache++; break;", "case T_CACHE: k.n_cache++; if (miss_idx) miss_idx[nm] = r; nm++; break;"),
    ("local experts consume a staging slot",
     "kind[e] = 1; where[e] = c->slot[id]; kc.n_local++;", "kind[e] = 1; where[e] = c->slot[id]; kc.n_local++; rank++;"),
    ("expert object number ignores the layer",
     "uint32_t id = layer * n_experts + e;", "uint32_t id = e;"),
    ("lossy objects demoted to the host tier, where they have no copy",
     "if (to_cache >= 0) { c->tier[id] = T_CACHE; c->slot[id] = to_cache; }\n            else { c->tier[id] = T_HOST; c->slot[id] = -1; }",
     "{ c->tier[id] = T_HOST; c->slot[id] = -1; }"),
    ("head-major fetch reads the block as if it were head-major already",
     "src + ((uint64_t)tok * n_heads + h) * head_bytes, head_bytes);",
     "src + ((uint64_t)h * block_tokens + tok) * head_bytes, head_bytes);"),
    ("head-major fetch forgets the block's position in the sequence",
     "memcpy(seq_base + h * strip + ((uint64_t)j * block_tokens + tok) * head_bytes,",
     "memcpy(seq_base + h * strip + ((uint64_t)tok) * head_bytes,"),
    ("head strips sized by the current length instead of the capacity",
     "uint64_t strip = (uint64_t)seq_cap_blocks[s] * block_tokens * head_bytes;",
     "uint64_t strip = (uint64_t)nb * block_tokens * head_bytes;"),
    ("duplicate ids accepted by the write-back",
     "if (ids[j] == ids[i]) return ORC_EINVAL;\n    }\n    /* room for", "if (0) return ORC_EINVAL;\n    }\n    /* room for"),
    ("a restored object keeps its old generation",
     "c->tier[ids[i]] = T_LOCAL; c->slot[ids[i]] = s; c->gen[ids[i]] += 1;", "c->tier[ids[i]] = T_LOCAL; c->slot[ids[i]] = s;"),
    ("restore accepts objects that are not lost",
     "if (c->tier[ids[i]] != T_NONE) return ORC_EINVAL;", ""),
    ("restore does not claim the local slot it hands out",
     "c->local_used[s] = 1;\n        c->tier[ids[i]] = T_LOCAL;", "c->tier[ids[i]] = T_LOCAL;"),
    ("first-fit instead of best-fit",
     "(best < 0 || g->run_len[i] < g->run_len[best])", "(best < 0)"),
    ("worst-fit instead of best-fit",
     "(best < 0 || g->run_len[i] < g->run_len[best])", "(best < 0 || g->run_len[i] > g->run_len[best])"),
    ("equally good runs: the highest taken instead of the lowest",
     "(best < 0 || g->run_len[i] < g->run_len[best])", "(best < 0 || g->run_len[i] <= g->run_len[best])"),
    ("segment carved from the high end of its run",
     "} else { g->run_off[best] += need; g->run_len[best] -= need; }",
     "} else { off = g->run_off[best] + g->run_len[best] - need; g->run_len[best] -= need; }"),
    ("a freed segment never joins the run before it",
     "int joins_prev = i > 0 && g->run_off[i - 1] + g->run_len[i - 1] == off;", "int joins_prev = 0;"),
    ("a freed segment never joins the run after it",
     "int joins_next = i < g->n_runs && off + len == g->run_off[i];", "int joins_next = 0;"),
    ("segment laid out plane-major",
     "+ ((uint64_t)layer * c->n_planes + plane) * c->chunk_bytes;", "+ ((uint64_t)plane * c->n_layers + layer) * c->chunk_bytes;"),
    ("object size rounded down to whole granules",
     "return (object_bytes(c) + c->seg->granule - 1) / c->seg->granule;", "return object_bytes(c) / c->seg->granule;"),
    ("a failed demotion keeps the segments it had taken",
     "while (k > 0) cache_release(c, room[--k]);", ""),
    ("placement from a device copy reads the host copy instead",
     "const uint8_t *from = src[p] + ((uint64_t)l * src_layer_stride + src_block[i]) * c->chunk_bytes;",
     "const uint8_t *from = at(c->host[p], c, c->n_host_slots, l, (uint64_t)c->host_slot[id]);"),
    ("placement from a device copy takes the i-th source block instead of the named one",
     "const uint8_t *from = src[p] + ((uint64_t)l * src_layer_stride + src_block[i]) * c->chunk_bytes;",
     "const uint8_t *from = src[p] + ((uint64_t)l * src_layer_stride + i) * c->chunk_bytes;"),
    ("placement from a device copy reads every layer from the first source layer",
     "const uint8_t *from = src[p] + ((uint64_t)l * src_layer_stride + src_block[i]) * c->chunk_bytes;",
     "const uint8_t *from = src[p] + ((uint64_t)0 * src_layer_stride + src_block[i]) * c->chunk_bytes;"),
    ("placement from a device copy forgets the generation",
     "c->slot[id] = room; c->gen[id] = c->gen[id] + 1;", "c->slot[id] = room;"),
    ("placement from a device copy overwrites objects that are in HBM already",
     "else if (c->tier[id] == T_CACHE || c->tier[id] == T_LOCAL) st = ORC_OK;      /* in HBM already: not written */",
     "else if (c->tier[id] == T_LOCAL) st = ORC_OK;"),
    ("placement from a device copy reports a full cache tier as success",
     "if (room < 0) st = ORC_ENOSPC;", "if (room < 0) st = ORC_OK;"),
    ("placement from a device copy also rewrites the host copy",
     "memcpy(cache_at(c, p, l, (uint64_t)room), from, c->chunk_bytes);",
     "memcpy(cache_at(c, p, l, (uint64_t)room), from, c->chunk_bytes); memcpy(at(c->host[p], c, c->n_host_slots, l, (uint64_t)c->host_slot[id]), from, c->chunk_bytes);"),
    ("revocation poisons whole granules instead of the object",
     "memset(cache_at(c, p, l, (uint64_t)old[i]), ORC_POISON, c->chunk_bytes);",
     "memset(cache_at(c, p, l, (uint64_t)old[i]), ORC_POISON, c->chunk_bytes + (c->seg ? 16 : 0));"),
]


def battery():
    """The pin suite, called directly (parametrised tests with their parameter sets)."""
    for p in (0.0, 0.3, 0.6, 1.0):
        for seed in (0, 1, 2):
            pins.test_fetch_kv_every_destination_word_names_its_request(p, seed)
    pins.test_fetch_is_identical_for_every_residency_assignment()
    pins.test_fetch_equals_numpy_take_on_the_host_plane()
    pins.test_torch_index_select_reproduces_the_gather()
    pins.test_all_cached_identity_table_is_one_memcpy()
    pins.test_brute_force_three_blocks_all_tables_residencies_and_revocations()
    pins.test_evict_of_fetched_bytes_is_identity_and_evict_of_new_bytes_is_returned()
    pins.test_evict_all_layers_layout_and_duplicate_rejection()
    for poison in (False, True):
        pins.test_revocation_falls_back_to_host_and_grows_the_miss_set_exactly(poison)
    pins.test_miss_list_is_exactly_the_host_and_lost_requests_in_request_order()
    pins.test_place_takes_lowest_free_slot_copies_the_host_bytes_and_reports_enospc()
    pins.test_place_from_a_copy_in_device_memory_writes_those_bytes_and_never_touches_the_host()
    pins.test_place_from_the_host_bytes_is_place()
    pins.test_fetch_never_changes_the_directory_or_any_tier()
    pins.test_local_objects_append_evict_demote_then_place()
    pins.test_invalid_requests_are_skipped_and_counted()
    pins.test_expert_fetch_union_ranks_and_bytes()
    pins.test_expert_fetch_staging_overflow_invalid_ids_and_revocation()
    pins.test_lossy_object_is_lost_after_revocation_and_leaves_dst_untouched()
    for seed in range(3):
        pins.test_random_operation_sequences_keep_tiered_and_plain_fetch_equal(seed)
    for heads, bt, hb in ((8, 16, 256), (3, 4, 48), (1, 16, 32), (5, 1, 16)):
        pins.test_head_major_fetch_is_the_transpose_of_the_token_major_fetch(heads, bt, hb)
    pins.test_head_major_fetch_rejects_what_does_not_fit()
    pins.test_restore_is_all_or_nothing_when_local_hbm_is_full()
    pins.test_best_fit_worked_example()
    for seed in range(5):
        pins.test_best_fit_agrees_with_the_bitmap_definition_on_random_sequences(seed)
    pins.test_two_classes_share_one_segment_pool()
    pins.test_lossy_demotion_into_segments_is_all_or_nothing()


def test_the_unmutated_oracle_passes_the_battery():
    O.use_library(None)
    battery()


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_every_planted_mistake_is_caught(what, old, new, tmp_path):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site not found exactly once: {what}"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-w", "-o", str(lib), str(src)])
    O.use_library(str(lib))
    try:
        with pytest.raises((AssertionError, O.OracleError, pytest.fail.Exception)):
            battery()
    finally:
        O.use_library(None)
