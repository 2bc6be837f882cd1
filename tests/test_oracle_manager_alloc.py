"""Pins for the integer oracles: CU-split choice (section 4.5.3) and block allocator (4.5.1)."""
import pytest

from oracle.kv_alloc import KVAllocator, NoBlocks
from oracle.manager import Profile, choose_split

# Hand-built profile with known answers.  batch buckets 8/64/256, ctx buckets 10k/100k/1M.
# Distinct-split decode CU options 32..224; latencies fall with more CUs.
CUS = [32, 64, 96, 128, 160, 192, 224]


def _row(base):
    return [base * 256 // c for c in CUS]


PROF = Profile(
    batch_edges=[8, 64, 256], ctx_edges=[10_000, 100_000, 1_000_000], decode_cus=CUS,
    lat_distinct_us=[[_row(b * c) for c in (10, 40, 160)] for b in (10, 40, 100)],
    lat_over_us=[[b * c * 3 for c in (10, 40, 160)] for b in (10, 40, 100)],
)


def test_no_prefill_gives_decode_everything():
    assert choose_split(64, 50_000, False, PROF, 1000) == (0, 256)


def test_no_decode_gives_prefill_everything():
    assert choose_split(0, 0, True, PROF, 1000) == (256, 0)


def test_light_load_over_allocates():
    # bucket (8, 10k): over-allocation latency 10*10*3 = 300us <= 1000us
    assert choose_split(4, 5_000, True, PROF, 1000) == (256, 256)


def test_heavy_load_takes_min_cus_meeting_slo_and_remainder_goes_to_prefill():
    # bucket (64, 100k): base 40*40 = 1600; over = 4800 > 2000; distinct: 1600*256/c <= 2000
    # -> c >= 204.8 -> first option 224
    assert choose_split(33, 60_000, True, PROF, 2000) == (32, 224)
    # looser objective 4000us: c >= 102.4 -> 128
    assert choose_split(33, 60_000, True, PROF, 4000) == (128, 128)


def test_load_is_rounded_up_to_next_bucket():
    # batch 9 falls in the 64 bucket, not the 8 bucket
    assert choose_split(9, 5_000, True, PROF, 400) != choose_split(8, 5_000, True, PROF, 400)
    assert choose_split(8, 5_000, True, PROF, 400) == (256, 256)       # 300 <= 400
    # (64,10k): over 1200 > 400; distinct base 400: 400*256/c <= 400 -> c=256 not offered
    # -> nothing meets: fastest split = 224
    assert choose_split(9, 5_000, True, PROF, 400) == (32, 224)


def test_beyond_last_bucket_uses_last_bucket():
    assert choose_split(1000, 10**9, True, PROF, 10**9) == (256, 256)
    assert choose_split(1000, 10**9, True, PROF, 1) == (32, 224)


def test_monotone_in_load_and_conserves_cus():
    prev = 0
    for b, c in [(4, 5000), (32, 5000), (32, 90_000), (200, 90_000), (200, 900_000)]:
        p, d = choose_split(b, c, True, PROF, 3000)
        if (p, d) != (256, 256):
            assert p + d == 256
            assert d >= prev
            prev = d


def test_allocator_block_count_is_ceil_of_length_over_16():
    a = KVAllocator(100)
    for n, want in [(1, 1), (16, 1), (17, 2), (2048, 128 if False else 128)]:
        a2 = KVAllocator(200)
        assert len(a2.alloc(0, n)) == want
    assert a.alloc(7, 33) == [0, 1, 2]


def test_allocator_growth_keeps_prefix_and_failure_changes_nothing():
    a = KVAllocator(4)
    assert a.alloc(1, 16) == [0]
    assert a.alloc(2, 20) == [1, 2]
    with pytest.raises(NoBlocks):            # one block is free, three more are needed: nothing may be taken
        a.alloc(2, 80)
    assert a.n_free() == 1 and a.owned[2] == [1, 2] and a.free == [3]
    assert a.alloc(1, 17) == [0, 3]
    with pytest.raises(NoBlocks):
        a.alloc(2, 49)
    assert a.n_free() == 0 and a.owned[2] == [1, 2]
    a.release(2)
    assert a.n_free() == 2
    assert a.alloc(3, 32) == [1, 2]          # LIFO: same ids, same order
    a.release(1); a.release(3)
    assert sorted(a.free) == [0, 1, 2, 3]
