"""The pins are only worth something if a plausible mistake in the checker
fails one of them.  Each case below plants one mistake in the CPU checker
(monkeypatched, CPU only) and asserts that the named pin then fails."""
import numpy as np
import pytest

import oracle
import test_oracle_arith as arith
import test_oracle_plan as plan_pins
import test_oracle_sampler as sampler_pins


def expect_pin_fails(pin, *args):
    with pytest.raises((AssertionError, ValueError, ArithmeticError, IndexError)):
        pin(*args)


def test_reduce_mistakes_are_caught(monkeypatch):
    good = oracle.weighted_reduce

    def drop_last_term(peers, w, dtype, mode="D"):
        w2 = np.array(w, dtype=np.float32).copy()
        if len(w2) > 1:
            w2[-1] = 0.0
        return good(peers, w2, dtype, mode)

    def reversed_weights(peers, w, dtype, mode="D"):
        return good(peers, np.array(w, dtype=np.float32)[::-1].copy(), dtype, mode)

    def shifted_peer_index(peers, w, dtype, mode="D"):
        return good(list(peers[1:]) + list(peers[:1]), w, dtype, mode)

    def wrong_sign(peers, w, dtype, mode="D"):
        w2 = np.array(w, dtype=np.float32).copy()
        w2[0] = -w2[0]
        return good(peers, w2, dtype, mode)

    for mutant in (drop_last_term, reversed_weights, shifted_peer_index, wrong_sign):
        monkeypatch.setattr(oracle, "weighted_reduce", mutant)
        expect_pin_fails(arith.test_reduce_integer_sums_exact)
        expect_pin_fails(arith.test_reduce_bruteforce_exact_rationals)
    for mutant in (reversed_weights, shifted_peer_index):
        monkeypatch.setattr(oracle, "weighted_reduce", mutant)
        expect_pin_fails(arith.test_reduce_one_hot_and_copy)
    monkeypatch.setattr(oracle, "weighted_reduce", drop_last_term)
    expect_pin_fails(arith.test_reduce_identical_peers_returns_input)
    expect_pin_fails(arith.test_reduce_mean_special_case_matches_library)


def test_pack_and_scale_mistakes_are_caught(monkeypatch):
    good_pack = oracle.pack

    def off_by_one(layout, tensors, dtype):
        lay = dict(layout)
        lay["tensor_offset"] = [o + (1 if i == 1 else 0) for i, o in enumerate(layout["tensor_offset"])]
        return good_pack(lay, tensors, dtype)

    monkeypatch.setattr(oracle, "pack", off_by_one)
    expect_pin_fails(arith.test_pack_unpack_bruteforce, "f32", 16)
    monkeypatch.setattr(oracle, "pack", good_pack)

    good_scale = oracle.scale_array
    monkeypatch.setattr(oracle, "scale_array", lambda x, s, dtype, mode="D": good_scale(x, s * (1 + 2.0 ** -20), dtype, mode))
    expect_pin_fails(arith.test_scale_pins)


def test_bf16_rounding_mistakes_are_caught(monkeypatch):
    good = oracle.bf16_round

    def truncate(x):
        u = np.array([x], dtype=np.float32).view(np.uint32)[0]
        return int(u >> 16)

    def half_up(x):           # ties away from zero instead of to even
        f = np.float32(x)
        u = int(np.array([f], dtype=np.float32).view(np.uint32)[0])
        if np.isnan(f):
            return good(x)
        return ((u + 0x8000) >> 16) & 0xFFFF

    for mutant in (truncate, half_up):
        monkeypatch.setattr(oracle, "bf16_round", mutant)
        expect_pin_fails(arith.test_bf16_round_against_library_and_integer_rule)


def test_share_mistakes_are_caught(monkeypatch):
    good = oracle.plan_shares

    def plain_rounding(thr, B):
        S = sum(thr)
        return [int(round(t / S * B)) for t in thr]

    def remainder_to_first(thr, B):
        S = sum(thr)
        b = [int(t / S * B) for t in thr]
        b[0] += B - sum(b)
        return b

    def ties_to_last(thr, B):
        b = good(list(reversed(thr)), B)
        return list(reversed(b))

    monkeypatch.setattr(oracle, "plan_shares", plain_rounding)
    expect_pin_fails(plan_pins.test_shares_golden, 2048, "1.0 1.0 0.7 0.7 0.5 0.5 0.3 0.3".split(),
                     [409, 409, 287, 287, 205, 205, 123, 123])
    monkeypatch.setattr(oracle, "plan_shares", remainder_to_first)
    expect_pin_fails(plan_pins.test_shares_bruteforce_minimises_deviation)
    monkeypatch.setattr(oracle, "plan_shares", ties_to_last)
    expect_pin_fails(plan_pins.test_shares_golden, 3, ["1", "1"], [2, 1])


def test_layout_and_sampler_mistakes_are_caught(monkeypatch):
    good = oracle.assign_buckets

    def never_close(numels, es, cap, align):
        return good(numels, es, 0, align)

    def unaligned(numels, es, cap, align):
        return good(numels, es, cap, es)

    monkeypatch.setattr(oracle, "assign_buckets", never_close)
    expect_pin_fails(plan_pins.test_bucket_layout_hand_example)
    expect_pin_fails(plan_pins.test_bucket_layout_workloads)
    monkeypatch.setattr(oracle, "assign_buckets", unaligned)
    expect_pin_fails(plan_pins.test_bucket_layout_hand_example)
    monkeypatch.setattr(oracle, "assign_buckets", good)

    class BadMix(oracle.SplitMix64):
        def next(self):
            return (super().next() >> 1)

    monkeypatch.setattr(oracle, "SplitMix64", BadMix)
    expect_pin_fails(sampler_pins.test_splitmix64_published_values)
    monkeypatch.undo()
    good_epoch = oracle.sampler_epoch

    def strided(N, B, shares, seed, epoch, rank, shuffle=True, drop_last=False):
        out = good_epoch(N, B, shares, seed, epoch, rank, shuffle, drop_last)
        return out[::-1]

    monkeypatch.setattr(oracle, "sampler_epoch", strided)
    expect_pin_fails(sampler_pins.test_partition_equal_devices_is_plain_split)


def test_master_model_copy_mistakes_are_caught(monkeypatch):
    good = oracle.unpack_sgd_master

    def truncates_instead_of_rounding(*a, **k):
        p, v, m = good(*a, **k)
        return p, v, [(x.view(np.uint32) >> np.uint32(16)).astype(np.uint16) for x in p]

    def copies_the_old_parameters(layout, buckets, numels, scale, masters, *rest, **k):
        p, v, _ = good(layout, buckets, numels, scale, masters, *rest, **k)
        _, _, m = good(layout, buckets, numels, 0.0, masters, rest[0], 0.0, 0.0, 0.0, True, *rest[5:], **k)
        return p, v, m

    for mutant in (truncates_instead_of_rounding, copies_the_old_parameters):
        monkeypatch.setattr(oracle, "unpack_sgd_master", mutant)
        expect_pin_fails(arith.test_sgd_master_model_copy_is_the_library_bf16_rounding)
