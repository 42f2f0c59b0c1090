"""The pins must bite: plant a plausible mistake in the oracle (on the CPU, by
monkeypatching one of its functions) and check that at least one pin fails."""

import numpy as np
import pytest

from oracle import s2r_oracle as orc
from tests import test_oracle_pins as pins


def _fails(fn, *args):
    try:
        fn(*args)
    except AssertionError:
        return True
    except Exception:           # a crash also counts as "noticed"
        return True
    return False


def _some_pin_fails():
    checks = [
        (pins.test_algorithm1_matches_pure_python, (3, 16, 1)),
        (pins.test_algorithm1_matches_pure_python, (4, 32, 2)),
        (pins.test_insert_and_query_equal_mapping_matrix_form, ()),
        (pins.test_exact_recovery_when_collision_free, (3,)),
        (pins.test_bitmap_and_sparse_match_elementwise_definition, (127,)),
        (pins.test_median_brute_force_and_permutation_invariance, (5,)),
        (pins.test_median_brute_force_and_permutation_invariance, (4,)),
        (pins.test_bucket_and_sign_match_bigint, (1 << 14,)),
        (pins.test_merged_bitmap_popcount_is_union_size, ()),
        (pins.test_single_element_gradient, ()),
        (pins.test_hash_params_order_and_oddness, ()),
        (pins.test_mass_table_and_decode_tolerance_mass_match_pure_python, (3, 16, 1)),
        (pins.test_mass_table_and_decode_tolerance_mass_match_pure_python, (5, 4, 3)),
        (pins.test_single_row_error_variance_is_the_others_energy_over_the_width, ()),
        (pins.test_block_algorithm_matches_pure_python, (7, 4, 32, 2)),
        (pins.test_block_sketch_equals_element_sketch_and_values_agree_on_the_union, ()),
        (pins.test_topk_blocks_matches_pure_python, (4, 3)),
        (pins.test_topk_blocks_matches_pure_python, (16, 13)),
        (pins.test_topk_ties_go_to_the_lower_block_and_extremes, ()),
        (pins.test_topk_is_a_delta_approximate_compressor_and_loses_nothing, ()),
        (pins.test_decode_blocks_update_against_pure_python_and_the_element_update, ()),
        (pins.test_topk_encode_blocks_matches_pure_python, (4, 3)),
        (pins.test_topk_encode_blocks_is_topk_then_encode_blocks_unless_a_kept_block_is_zero, ()),
        (pins.test_topk_encode_blocks_round_trip_without_collisions_returns_acc_in_the_kept_blocks, ()),
    ]
    return any(_fails(fn, *a) for fn, a in checks)


def test_unmutated_oracle_passes_the_same_checks():
    assert not _some_pin_fails()


def _mut_sign_dropped_in_query(monkeypatch):
    real = orc.estimates

    def bad(S, idx, seed):
        d, w = S.shape
        est = np.empty((d, idx.shape[0]))
        for j, (a, b, c, e) in enumerate(orc.hash_params(seed, d)):
            est[j] = S[j, orc.bucket_hash(idx, a, b, w)]
        return est
    monkeypatch.setattr(orc, "estimates", bad)
    return real


def _mut_msb_first_bitmap(monkeypatch):
    def bad(mask):
        n = mask.shape[0]
        words = (n + 63) // 64
        by = np.packbits(mask.astype(np.uint8), bitorder="big")
        buf = np.zeros(words * 8, dtype=np.uint8)
        buf[: by.shape[0]] = by
        return buf.view("<u8").astype(np.uint64)
    monkeypatch.setattr(orc, "pack_bitmap", bad)


def _mut_median_off_by_one(monkeypatch):
    def bad(est):
        srt = np.sort(est, axis=0)
        return srt[max(0, est.shape[0] // 2 - 1)]
    monkeypatch.setattr(orc, "median_rows", bad)


def _mut_low_bits_bucket(monkeypatch):
    def bad(idx, a, b, w):
        i = idx.astype(np.uint64)
        with np.errstate(over="ignore"):
            u = i * np.uint64(a) + np.uint64(b)
        return (u & np.uint64(w - 1)).astype(np.int64)
    monkeypatch.setattr(orc, "bucket_hash", bad)


def _mut_sign_uses_bucket_multiplier(monkeypatch):
    real = orc.hash_params

    def bad(seed, d):
        return [(a, b, a, b) for (a, b, c, e) in real(seed, d)]
    monkeypatch.setattr(orc, "hash_params", bad)


def _mut_merge_xor(monkeypatch):
    def bad(sketches, bitmaps):
        S = np.sum(sketches, axis=0)
        C = np.zeros_like(bitmaps[0])
        for Ck in bitmaps:
            C = C ^ Ck
        return S, C
    monkeypatch.setattr(orc, "merge", bad)


def _mut_merge_drops_last_worker(monkeypatch):
    def bad(sketches, bitmaps):
        S = np.sum(sketches[:-1], axis=0) if len(sketches) > 1 else sketches[0]
        C = np.zeros_like(bitmaps[0])
        for Ck in bitmaps:
            C = C | Ck
        return S, C
    monkeypatch.setattr(orc, "merge", bad)


def _mut_negative_zero_counts(monkeypatch):
    def bad(g):
        g = np.ascontiguousarray(g, dtype=np.float32)
        return g.view(np.uint32) != 0
    monkeypatch.setattr(orc, "nonzero_mask", bad)


def _mut_insert_assign_not_accumulate(monkeypatch):
    def bad(idx, val, d, w, seed):
        S = np.zeros((d, w))
        M = np.zeros((d, w))
        v = val.astype(np.float64)
        for j, (a, b, c, e) in enumerate(orc.hash_params(seed, d)):
            h = orc.bucket_hash(idx, a, b, w)
            S[j, h] += orc.sign_hash(idx, c, e) * v      # buffered: last write wins
            M[j, h] += np.abs(v)
        return S, M
    monkeypatch.setattr(orc, "insert", bad)


def _mut_block_needs_all_elements(monkeypatch):
    real = orc.block_mask
    def bad(g, B):
        nz = orc.nonzero_mask(np.ascontiguousarray(g, dtype=np.float32))
        nb = (nz.shape[0] + B - 1) // B
        padded = np.ones(nb * B, dtype=bool)
        padded[: nz.shape[0]] = nz
        return padded.reshape(nb, B).all(axis=1)
    monkeypatch.setattr(orc, "block_mask", bad)


def _mut_block_boundary_shifted(monkeypatch):
    def bad(g, B):
        nz = orc.nonzero_mask(np.ascontiguousarray(g, dtype=np.float32))
        nz = np.concatenate([[False], nz[:-1]])                     # element i counted in the block of i + 1
        nb = (nz.shape[0] + B - 1) // B
        padded = np.zeros(nb * B, dtype=bool)
        padded[: nz.shape[0]] = nz
        return padded.reshape(nb, B).any(axis=1)
    monkeypatch.setattr(orc, "block_mask", bad)


def _mut_block_decode_skips_zero_elements(monkeypatch):
    real = orc.decode_blocks
    def bad(S, bitmap, n, B, seed):
        out = real(S, bitmap, n, B, seed)
        out["val"] = np.where(np.abs(out["val"]) < 1e-3, 0.0, out["val"])      # as if only "large" entries were queried
        return out
    monkeypatch.setattr(orc, "decode_blocks", bad)


def _mut_topk_scores_by_abs_sum(monkeypatch):
    def bad(acc, B):
        acc = np.ascontiguousarray(acc, dtype=np.float32)
        nb = (acc.shape[0] + B - 1) // B
        padded = np.zeros(nb * B, dtype=np.float64)
        padded[: acc.shape[0]] = np.abs(acc.astype(np.float64))                  # l1 instead of l2
        return np.sum(padded.reshape(nb, B), axis=1).astype(np.float32)
    monkeypatch.setattr(orc, "block_scores", bad)


def _mut_topk_keeps_smallest(monkeypatch):
    real = orc.block_scores
    monkeypatch.setattr(orc, "block_scores", lambda acc, B: (-real(acc, B)).astype(np.float32))


def _mut_topk_residual_forgets_old_error(monkeypatch):
    real = orc.topk_blocks
    monkeypatch.setattr(orc, "topk_blocks", lambda g, e, B, K: real(g, None, B, K))


def _mut_fused_step_marks_only_nonzero_blocks(monkeypatch):
    real = orc.topk_encode_blocks
    def bad(g, e, B, K, d, w, seed):
        out = real(g, e, B, K, d, w, seed)
        out["bitmap"] = orc.pack_bitmap(orc.block_mask(out["sparse"], B))        # looks at the values again
        return out
    monkeypatch.setattr(orc, "topk_encode_blocks", bad)


def _mut_fused_step_sketches_the_gradient_without_the_residual(monkeypatch):
    real = orc.topk_encode_blocks
    def bad(g, e, B, K, d, w, seed):
        out = real(g, e, B, K, d, w, seed)
        elems = orc.block_elements(out["blocks"], B, len(g))
        only_g = np.zeros(len(g), dtype=np.float32)
        only_g[elems] = np.asarray(g, dtype=np.float32)[elems]
        idx, val = orc.sparse_of(only_g)
        out["S"], out["M"] = orc.insert(idx, val, d, w, seed)
        return out
    monkeypatch.setattr(orc, "topk_encode_blocks", bad)


def _mut_fused_step_keeps_the_residual_of_sent_blocks(monkeypatch):
    real = orc.topk_encode_blocks
    def bad(g, e, B, K, d, w, seed):
        out = real(g, e, B, K, d, w, seed)
        out["residual"] = (out["residual"] + out["sparse"]).astype(np.float32)   # sent blocks not cleared
        return out
    monkeypatch.setattr(orc, "topk_encode_blocks", bad)


def _mut_block_update_runs_past_the_end_of_the_block(monkeypatch):
    real = orc.block_elements
    def bad(blocks, B, n):
        e = real(blocks, B, n)
        return np.minimum(e + 1, n - 1)                                          # every element shifted by one
    monkeypatch.setattr(orc, "block_elements", bad)


def _mut_block_update_ignores_the_scale(monkeypatch):
    real = orc.decode_blocks_update
    monkeypatch.setattr(orc, "decode_blocks_update", lambda S, bm, n, B, seed, p, scale: real(S, bm, n, B, seed, p, 1.0))


def _mut_mass_table_inflated(monkeypatch):
    real = orc.insert

    def bad(idx, val, d, w, seed):
        S, M = real(idx, val, d, w, seed)
        return S, 100.0 * M                                                     # every tolerance 100 times too wide
    monkeypatch.setattr(orc, "insert", bad)


def _mut_tolerance_mass_sums_the_rows(monkeypatch):
    def bad(M, idx, seed):
        d, w = M.shape
        m = np.zeros(idx.shape[0])
        for j, (a, b, _c, _e) in enumerate(orc.hash_params(seed, d)):
            m = m + M[j, orc.bucket_hash(idx, a, b, w)]                        # sum over the rows, not the largest
        return m
    monkeypatch.setattr(orc, "decode_tolerance_mass", bad)


def _mut_mass_table_signed(monkeypatch):
    def bad(idx, val, d, w, seed):
        S = np.zeros((d, w))
        M = np.zeros((d, w))
        v = val.astype(np.float64)
        for j, (a, b, c, e) in enumerate(orc.hash_params(seed, d)):
            h = orc.bucket_hash(idx, a, b, w)
            np.add.at(S[j], h, orc.sign_hash(idx, c, e) * v)
            np.add.at(M[j], h, v)                                               # signs cancel inside the mass
        return S, np.abs(M)
    monkeypatch.setattr(orc, "insert", bad)


@pytest.mark.parametrize("mutant", [
    _mut_mass_table_inflated, _mut_tolerance_mass_sums_the_rows, _mut_mass_table_signed,
    _mut_sign_dropped_in_query, _mut_msb_first_bitmap, _mut_median_off_by_one,
    _mut_low_bits_bucket, _mut_sign_uses_bucket_multiplier, _mut_merge_xor,
    _mut_merge_drops_last_worker, _mut_negative_zero_counts,
    _mut_insert_assign_not_accumulate,
    _mut_block_needs_all_elements, _mut_block_boundary_shifted, _mut_block_decode_skips_zero_elements,
    _mut_topk_scores_by_abs_sum, _mut_topk_keeps_smallest, _mut_topk_residual_forgets_old_error,
    _mut_fused_step_marks_only_nonzero_blocks, _mut_fused_step_sketches_the_gradient_without_the_residual,
    _mut_fused_step_keeps_the_residual_of_sent_blocks,
    _mut_block_update_runs_past_the_end_of_the_block, _mut_block_update_ignores_the_scale,
], ids=lambda f: f.__name__)
def test_planted_mistake_is_caught(monkeypatch, mutant):
    mutant(monkeypatch)
    assert _some_pin_fails()
