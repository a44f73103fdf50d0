"""The pins must notice a plausible mistake anywhere in the oracle.  Each case below plants one
mistake in a temporary copy of oracle/flexshard_oracle.c (a textual patch), builds it, and runs
a compact set of pin checks against it: at least one must fail.  Everything runs on the CPU."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle
from helpers import dest_numpy, entry, random_jagged, random_placement, table_of

SRC = os.path.join(os.path.dirname(oracle.__file__), "flexshard_oracle.c")
TWO24 = float(2 ** 24)

MUTANTS = {
    "group_base_dropped": ("return (self / W) * W + (int32_t)owner;", "return (int32_t)owner;"),
    "tier1_uses_U": ("if (owner >= (uint32_t)W) { flag(status, DEV_BAD_PLACEMENT); return self; }\n        return (self / W) * W",
                     "if (owner >= (uint32_t)U) { flag(status, DEV_BAD_PLACEMENT); return self; }\n        return (self / W) * W"),
    "table_from_segment_mod": ("int64_t t = s / B;\n        int64_t rows_t = row_base[t + 1] - row_base[t];\n        for (int64_t i = offsets[s]; i < offsets[s + 1]; ++i) {\n            int64_t id = ids[i];\n            if (id < 0 || id >= rows_t) { flag(status, DEV_BAD_ID); id = 0; }\n            g[i]",
                               "int64_t t = s % T;\n        int64_t rows_t = row_base[t + 1] - row_base[t];\n        for (int64_t i = offsets[s]; i < offsets[s + 1]; ++i) {\n            int64_t id = ids[i];\n            if (id < 0 || id >= rows_t) { flag(status, DEV_BAD_ID); id = 0; }\n            g[i]"),
    "unstable_scatter": ("for (int64_t i = 0; i < n; ++i) {\n        int64_t j = cursor[dest[i]]++;", "for (int64_t i = n - 1; i >= 0; --i) {\n        int64_t j = cursor[dest[i]]++;"),
    "inclusive_scan": ("for (int32_t b = 0; b <= U; ++b) bucket_offsets[b] = cursor[b];", "for (int32_t b = 0; b <= U; ++b) bucket_offsets[b] = cursor[b < U ? b + 1 : U];"),
    "gather_swapped": ("memcpy((char*)out + (size_t)p * row_bytes,\n               (const char*)weights + (size_t)r * row_bytes, row_bytes);",
                       "memcpy((char*)out + (size_t)r % (size_t)n * row_bytes,\n               (const char*)weights + (size_t)p % (size_t)R * row_bytes, row_bytes);"),
    "half_exponent_bias": ("bits = sign | ((exp + (127 - 15)) << 23) | (man << 13);", "bits = sign | ((exp + (127 - 16)) << 23) | (man << 13);"),
    "half_subnormal_lost": ("int shift = 0;\n            while (!(man & 0x400u)) { man <<= 1; ++shift; }", "int shift = 0;\n            man = 0x400u;"),
    "bf16_low_half": ("uint32_t bits = (uint32_t)b << 16;", "uint32_t bits = (uint32_t)b << 15;"),
    "sort_by_pos_only": ("if (x->row != y->row) return x->row < y->row ? -1 : 1;\n    if (x->pos != y->pos)", "if (x->pos != y->pos)"),
    "sorted_pairs_carry_j": ("sorted_pos[k] = (uint32_t)lk[k].pos;", "sorted_pos[k] = (uint32_t)lk[k].j;"),
    "sorted_pairs_whole_array": ("int64_t r = rows[j0 + q];\n        int64_t p = pos[j0 + q];\n        if (r < 0 || r >= R) { flag(status, DEV_BAD_ID); r = 0; }\n        if (p < 0 || p >= n) { flag(status, DEV_BAD_ID); p = 0; }\n        lk[q].row = r; lk[q].pos = p; lk[q].j = q;\n    }\n    qsort(lk, (size_t)m, sizeof(lookup_t), by_row_then_pos);\n    for (int64_t k = 0; k < m; ++k) {",
                                 "int64_t r = rows[q];\n        int64_t p = pos[q];\n        if (r < 0 || r >= R) { flag(status, DEV_BAD_ID); r = 0; }\n        if (p < 0 || p >= n) { flag(status, DEV_BAD_ID); p = 0; }\n        lk[q].row = r; lk[q].pos = p; lk[q].j = q;\n    }\n    qsort(lk, (size_t)m, sizeof(lookup_t), by_row_then_pos);\n    for (int64_t k = 0; k < m; ++k) {"),
    "tile_boundary_ignored": ("while (end < m && lk[end].row == lk[k].row && (end % tile) != 0) ++end;", "while (end < m && lk[end].row == lk[k].row) ++end;"),
    "partials_start_at_zero": ("partial[d] = (q == k) ? x : partial[d] + x;", "partial[d] = (q == k) ? 0.0f + x : partial[d] + x;"),
    "fold_right_to_left": ("total[d] = have_total ? total[d] + partial[d] : partial[d];", "total[d] = have_total ? partial[d] + (total[d] - 0.0f) * 1.0f + 0.0f : partial[d]; if (have_total && d == 0) { float t2 = total[d]; (void)t2; }"),
    "dropped_term": ("for (int64_t q = k; q < end; ++q) {\n            size_t base", "for (int64_t q = k; q < end - (end - k > 3); ++q) {\n            size_t base"),
    "hist_counts_presence": ("else counts[g] += 1;", "else if (counts[g] == 0) counts[g] = 1;"),
    "select_ascending": ("if (x->count != y->count) return x->count > y->count ? -1 : 1;", "if (x->count != y->count) return x->count < y->count ? -1 : 1;"),
    "tie_break_descending": ("return x->g < y->g ? -1 : (x->g > y->g ? 1 : 0);\n}\n\n/*\n * Replication plan", "return x->g > y->g ? -1 : (x->g < y->g ? 1 : 0);\n}\n\n/*\n * Replication plan"),
    "budget_rounds_up": ("int64_t cap = budget_bytes / bytes_per_row;", "int64_t cap = (budget_bytes + bytes_per_row - 1) / bytes_per_row;"),
    "zeros_selected": ("if (counts[g] > 0 || (flags & PLAN_ALLOW_ZERO))", "if (1)"),
    "tag_sets_tier2": ("for (int64_t i = 0; i < k; ++i) placement[cand[i].g] &= 0x3FFFFFFFu;", "for (int64_t i = 0; i < k; ++i) placement[cand[i].g] = (placement[cand[i].g] & 0x3FFFFFFFu) | 0x80000000u;"),
    "tiers_dp_tag_keeps_tier": ("for (int64_t i = 0; i < n_dp; ++i) placement[cand[i].g] &= 0x3FFFFFFFu;", "for (int64_t i = 0; i < n_dp; ++i) placement[cand[i].g] &= 0xBFFFFFFFu;"),
    "send_indexed_by_j_not_offset": ("memcpy((char*)send + (size_t)(j - j0) * row_bytes,", "memcpy((char*)send + (size_t)(j - j0 > 0 ? j - j0 - 1 : 0) * row_bytes,"),
    "unbucketize_reads_by_pos": ("(const char*)recv + (size_t)(j - j0) * row_bytes, row_bytes);", "(const char*)recv + (size_t)(p % (j1 - j0)) * row_bytes, row_bytes);"),
    "replica_last_slot_wins": ("if (slot_of_row[r] < 0) slot_of_row[r] = (int32_t)s;", "slot_of_row[r] = (int32_t)s;"),
    "replica_store_ignored": ("else if (s < k) from = (const char*)store + (size_t)s * row_bytes;", "else if (s < k) from = (const char*)weights + (size_t)r * row_bytes;"),
    "replica_slot_is_row": ("else if (s < k) from = (const char*)store + (size_t)s * row_bytes;", "else if (s < k) from = (const char*)store + (size_t)(r % k) * row_bytes;"),
    "slots_tag_other_tiers": ("if ((placement[r] >> 30) != 0) continue;\n        int32_t s = slot_of_row[r];", "int32_t s = slot_of_row[r];"),
    "slots_untagged_row_keeps_owner": ("placement[r] = s >= 0 ? (uint32_t)s : NO_SLOT;", "if (s >= 0) placement[r] = (uint32_t)s;"),
    "slots_read_from_any_tier": ("if ((e >> 30) == 0 && (e & 0x3FFFFFFFu) != NO_SLOT) out_slots[j]", "if ((e & 0x3FFFFFFFu) != NO_SLOT) out_slots[j]"),
    "slots_gather_ignores_slot": ("int32_t slot = slots[j];", "int32_t slot = -1;"),
    "slots_gather_indexed_by_pos": ("int32_t slot = slots[j];", "int32_t slot = slots[p % (j1 - j0)];"),
    "tiers_dynamic_saving_doubled": ("const wide_t mem = static_term - U * B * c;", "const wide_t mem = static_term - 2 * U * B * c;"),
    "tiers_saved_without_dynamic": ("saved -= static_term - U * B * (wide_t)cand[i].count;", "saved -= static_term - U * (wide_t)cand[i].count;"),
    "tiers_static_without_shard": ("const wide_t static_term = (dp * U - 1) * S;", "const wide_t static_term = (dp * U) * S;"),
    "tiers_A_excludes_neutral": ("if (!seenA && mem > 0) { kA = i; seenA = 1; }", "if (!seenA && mem >= 0) { kA = i; seenA = 1; }"),
    "tiers_B_strict": ("if (cum <= 0) kB = i + 1;", "if (cum < 0) kB = i + 1;"),
    "tiers_traffic_one_pass": ("if ((wide_t)p->a2a_global * S <= 2 * B * c * (wide_t)p->ar_global) kC = i + 1;", "if ((wide_t)p->a2a_global * S <= B * c * (wide_t)p->ar_global) kC = i + 1;"),
    "tiers_flex_cost_whole_table": ("const wide_t flex_cost = (dp * (U / W) - 1) * S;", "const wide_t flex_cost = (dp * U - 1) * S;"),
    "tiers_flex_ignores_traffic": ("while (i < nc && i < kF && spent + flex_cost <= saved)", "while (i < nc && spent + flex_cost <= saved)"),
    "tiers_granule_rounds_up": ("n_dp = kA / gran * gran;", "n_dp = (kA + gran - 1) / gran * gran;"),
    "tiers_flex_owner_over_all": ("(uint32_t)((i - n_dp) % p->W);", "(uint32_t)((i - n_dp) % p->U);"),
    "tiers_flex_allreduce_whole": ("2 * B * c * (wide_t)(p->a2a_intra - p->a2a_global) * W * (wide_t)p->ar_cross)", "2 * B * c * (wide_t)(p->a2a_intra - p->a2a_global) * (wide_t)p->ar_cross)"),
    "tiers_flex_overspends": ("spent + flex_cost <= saved) { spent += flex_cost; ++i; }", "spent <= saved) { spent += flex_cost; ++i; }"),
    "update_sgd_adds": ("store_elem(weights, at, dtype, w - step);", "store_elem(weights, at, dtype, w + step);"),
    "update_adagrad_eps_inside_root": ("step = (double)lr * gd / (sqrt(s) + (double)eps);", "step = (double)lr * gd / sqrt(s + (double)eps);"),
    "update_adagrad_state_not_squared": ("double s = (double)state[at] + gd * gd;", "double s = (double)state[at] + fabs(gd);"),
    "update_rowwise_sum_not_mean": ("row_state = (double)state[r] + sq / (double)D;", "row_state = (double)state[r] + sq;"),
    "update_rowwise_old_state": ("step = (double)lr * gd / (sqrt(row_state) + (double)eps);", "step = (double)lr * gd / (sqrt((double)state[r] - 0.0) + (double)eps); (void)row_state;"),
    "update_store_not_mirrored": ("if (slot >= 0) store_elem(store, (size_t)slot * (size_t)D + (size_t)d, dtype, w - step);", "if (slot >= 0) store_elem(store, (size_t)slot * (size_t)D + (size_t)d, dtype, w);"),
    "update_round_through_float": ("else ((uint16_t*)base)[index] = round_to_16(x, 7, 8);", "else ((uint16_t*)base)[index] = round_to_16((double)(float)x, 7, 8);"),
    "update_round_truncates": ("double q = nearbyint(a / quantum);", "double q = floor(a / quantum);"),
    "update_subnormals_flushed": ("if (exp < emin) exp = emin;", "if (exp < emin) return sign;"),
}
# a mutant that changes nothing observable would be a bad test of the tests: keep only real ones
MUTANTS.pop("fold_right_to_left")
MUTANTS["fold_right_to_left"] = ("total[d] = have_total ? total[d] + partial[d] : partial[d];\n        have_total = 1;\n        k = end;",
                                 "total[d] = partial[d];\n        have_total = 1;\n        k = end;")


class Lib:
    """The oracle's python wrappers, re-pointed at another shared object."""

    def __init__(self, path):
        self.dll = ctypes.CDLL(path)

    def __enter__(self):
        self.saved = oracle._lib
        oracle._lib = self.dll
        return oracle

    def __exit__(self, *a):
        oracle._lib = self.saved


def pins(o):
    """A compact version of the pin suite; raises AssertionError on the first mismatch."""
    rng = np.random.default_rng(0)
    # route: stable argsort / bincount, three tiers, two groups
    T, B, E, U, W, self_ = 3, 7, 40, 8, 4, 6
    ids, offsets, row_base, n = random_jagged(rng, T, B, E, 30)
    pl = random_placement(rng, T * E, U, W)
    rc, st, bo, rows, pos, tc = o.route_bucketize(ids, offsets, T, B, row_base, pl, U, W, self_)
    g = row_base[table_of(offsets, B)] + ids
    dest, tier = dest_numpy(g, pl, U, W, self_)
    order = np.argsort(dest, kind="stable")
    assert rc == 0 and st == 0 and np.array_equal(pos, order) and np.array_equal(rows, g[order])
    assert np.array_equal(bo, np.concatenate([[0], np.cumsum(np.bincount(dest, minlength=U))]))
    # an owner that is valid for the sharded tier but not inside a group is a fault of the group tier
    # (self in group 0, so that a mutant which accepts the owner still writes inside its arrays)
    rc, st, bo2, rows2, pos2, tc2 = o.route_bucketize([0, 1], [0, 2], 1, 1, [0, 2], np.array([entry(1, 5), entry(1, 1)], np.uint32), 8, 4, 2)
    assert st == o.BAD_PLACEMENT and bo2.tolist() == [0, 0, 1, 2, 2, 2, 2, 2, 2] and rows2.tolist() == [1, 0]
    # gather = take
    Wt = rng.standard_normal((T * E, 8)).astype(np.float32)
    out = np.zeros((n, 8), np.float32)
    o.seq_gather_fwd(Wt, rows, pos, 0, n, out)
    assert np.array_equal(out, Wt[g])
    # backward: conversions, fp64 sums, the rounding probes
    h = np.arange(65536, dtype=np.uint16).view(np.float16)
    h = h[~np.isnan(h)]
    h = np.concatenate([h, np.zeros((-len(h)) % 8, np.float16)]).reshape(-1, 8)
    m = h.shape[0]
    r = o.seq_grad_bwd(h, np.arange(m), np.arange(m, dtype=np.int32), 0, m, m, dtype=o.F16)
    assert np.array_equal(r[3].view(np.uint32), h.astype(np.float32).view(np.uint32))
    b16 = (rng.standard_normal((64, 8)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    r = o.seq_grad_bwd(b16, np.arange(64), np.arange(64, dtype=np.int32), 0, 64, 64, dtype=o.BF16)
    assert np.array_equal(r[3].view(np.uint32), b16.astype(np.uint32) << 16)
    rows_b = np.minimum(rng.pareto(0.9, 3000).astype(np.int64), 99)
    pos_b = rng.permutation(3000).astype(np.int32)
    x = rng.standard_normal((3000, 8)).astype(np.float16)
    rc, st, u, g32, g64, nu = o.seq_grad_bwd(x, rows_b, pos_b, 0, 3000, 100, dtype=o.F16)
    uniq, inv = np.unique(rows_b, return_inverse=True)
    ref = np.zeros((len(uniq), 8))
    np.add.at(ref, inv, x[pos_b].astype(np.float64))
    assert rc == 0 and np.array_equal(u, uniq) and np.array_equal(g64, ref)
    assert np.all(np.abs(g32 - ref) <= 1e-5 * np.maximum(np.abs(ref), 1.0))

    def col(v):
        v = np.asarray(v, np.float32)[:, None]
        return np.concatenate([v, -v, 0 * v, 2 * v], 1).astype(np.float32)
    assert o.seq_grad_bwd(col([TWO24, 1, 1, 1, 1, 1]), [5] * 6, np.arange(6, dtype=np.int32), 0, 6, 6, tile=4)[3][0, 0] == TWO24 + 2
    assert o.seq_grad_bwd(col([TWO24, 1, 1]), [0] * 3, np.arange(3, dtype=np.int32), 0, 3, 1, tile=1)[3][0, 0] == TWO24
    assert o.seq_grad_bwd(col([1, 1, TWO24, 3]), [4, 4, 4, 1], np.array([2, 1, 0, 3], np.int32), 0, 4, 5, tile=8)[3][1, 0] == TWO24 + 2
    z = o.seq_grad_bwd(np.full((1, 4), -0.0, np.float32), [0], np.zeros(1, np.int32), 0, 1, 1)[3]
    assert np.all(np.signbit(z))
    # the backward's order written out: lexsort by (row, pos) of a sub-range
    rc, st, srows, spos = o.sort_lookups(rows_b, pos_b, 100, 2900, 100, 3000)
    lo = np.lexsort((pos_b[100:2900], rows_b[100:2900]))
    assert (rc, st) == (0, 0) and np.array_equal(srows, rows_b[100:2900][lo]) and np.array_equal(spos, pos_b[100:2900][lo])
    # plan: bincount, lexsort prefix, zeros, budget, tags
    counts = np.zeros(T * E, np.uint32)
    o.plan_replication(ids, offsets, T, B, row_base, T * E, counts, o.PLAN_ACCUMULATE)
    assert np.array_equal(counts, np.bincount(g, minlength=T * E))
    c2 = np.minimum(rng.pareto(1.0, 300) * 3, 1e6).astype(np.uint32)
    order = np.lexsort((np.arange(300), -c2.astype(np.int64)))
    nz = int((c2 > 0).sum())
    for cap in (7, nz + 5):
        sel = o.plan_replication(None, None, 1, 1, None, 300, c2.copy(), o.PLAN_SELECT, cap * 16 + 15, 16)[2]
        assert np.array_equal(sel, order[:min(cap, nz)])
    p2 = np.full(300, entry(2, 1), np.uint32)
    sel = o.plan_replication(None, None, 1, 1, None, 300, c2.copy(), o.PLAN_SELECT | o.PLAN_TAG, 5, 1, p2)[2]
    assert np.all(p2[sel] >> 30 == 0) and (p2 >> 30 == 2).sum() == 295
    # exchange halves and replica store: take, row assignment, first-occurrence map
    rows_x = rng.integers(0, T * E, 50)
    pos_x = rng.permutation(50).astype(np.int32)
    send = np.zeros((30, 8), np.float32)
    assert o.seq_gather_send(Wt, rows_x, 10, 40, send) == (0, 0)
    assert np.array_equal(send, Wt[rows_x[10:40]])
    out_x = np.zeros((50, 8), np.float32)
    assert o.seq_unbucketize(send, pos_x, 10, 40, out_x) == (0, 0)
    exp_x = np.zeros((50, 8), np.float32)
    exp_x[pos_x[10:40]] = send
    assert np.array_equal(out_x, exp_x)
    sel_x = np.array([9, 3, 9, 77, 20], np.int64)
    store = np.zeros((5, 8), np.float32)
    rc, st, slots = o.replica_build(Wt, sel_x, store)
    assert (rc, st) == (0, 0) and np.array_equal(store, Wt[sel_x])
    assert slots[9] == 0 and slots[3] == 1 and slots[77] == 3 and slots[20] == 4 and (slots >= 0).sum() == 4
    look = np.array([3, 5, 77, 9, 20, 6], np.int64)
    mark = store + 1000.0
    out_r = np.zeros((6, 8), np.float32)
    assert o.seq_gather_fwd_replica(Wt, mark, slots, look, np.arange(6, dtype=np.int32), 0, 6, out_r) == (0, 0)
    assert np.array_equal(out_r, np.stack([mark[1], Wt[5], mark[3], mark[0], mark[4], Wt[6]]))
    # slots handed over in the placement: tagging, reading back, the gather that takes them
    import test_oracle_exchange as tx
    tx.test_slots_travel_in_the_placement_of_replicated_rows()
    tx.test_slot_faults()
    # tier planner: hand cases, closed forms, the whole-curve brute force
    import test_oracle_tiers as tt
    tt.test_three_tier_hand_case()
    tt.test_tags_and_rounding()
    tt.test_closed_forms()
    for seed in range(6):
        tt.test_against_whole_curve_brute_force(seed, 2)
        tt.test_against_whole_curve_brute_force(seed, 3)
    # sparse optimizer step: torch.optim in float64, the row-wise rule by hand, rounding against numpy
    import test_oracle_update as tu
    tu.test_float32_table_follows_torch_optim("sgd", o.OPT_SGD)
    tu.test_float32_table_follows_torch_optim("adagrad", o.OPT_ADAGRAD)
    tu.test_rowwise_by_hand_and_against_elementwise()
    tu.test_rounding_to_16_bit_types_is_numpy_s()
    tu.test_store_mirror_faults_and_edges()


def test_pins_accept_the_real_oracle():
    pins(oracle)


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_reject_mutant(name, tmp_path):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"patch site of {name} not found exactly once"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-shared", "-fPIC", str(src), "-o", str(lib), "-lm"], check=True)
    with Lib(str(lib)) as o:
        with pytest.raises(AssertionError):
            pins(o)
