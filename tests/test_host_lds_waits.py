"""The hand-placed LDS waits of the fused dK/dV kernel, checked on the compiler's listing (no GPU).

The kernel's operand reads are explicit instructions whose results the compiler does not track; the checker models
the LDS counter and flags any instruction that touches a register of a read still in flight.  The model itself is
pinned on small listings written here: a correct sequence, one with a wait count one too large, one where the
compiler would have moved a copy in front of the wait.
"""
import os

import pytest

from paper_2409_15373_amd import build, check_lds_waits

GOOD = """
    ds_read_b128 v[4:7], v1
    ds_read_b128 v[8:11], v1 offset:32
    ds_read_b128 v[12:15], v1 offset:64
    s_waitcnt lgkmcnt(2)
    v_mfma_f32_32x32x16_bf16 v[20:35], v[4:7], v[40:43], v[20:35]
    s_waitcnt lgkmcnt(1)
    v_mfma_f32_32x32x16_bf16 v[20:35], v[8:11], v[44:47], v[20:35]
    s_waitcnt lgkmcnt(0)
    v_mfma_f32_32x32x16_bf16 v[20:35], v[12:15], v[48:51], v[20:35]
"""


def test_a_correct_sequence_passes():
    r = check_lds_waits.scan(GOOD)
    assert r["violations"] == [] and r["lds_reads"] == 3 and r["lgkmcnt_waits"] == 3 and r["deepest_queue"] == 3


def test_a_count_one_too_large_is_found():
    r = check_lds_waits.scan(GOOD.replace("s_waitcnt lgkmcnt(1)", "s_waitcnt lgkmcnt(2)"))
    assert len(r["violations"]) == 1 and "v[8:11]" in r["violations"][0][1]


def test_a_copy_of_a_pending_register_is_found():
    r = check_lds_waits.scan(GOOD.replace("    s_waitcnt lgkmcnt(2)\n", "    v_mov_b32_e32 v60, v13\n    s_waitcnt lgkmcnt(2)\n"))
    assert len(r["violations"]) == 1 and "v_mov_b32" in r["violations"][0][1]


def test_a_store_in_the_queue_counts():
    # operations complete in order: with a write issued after the read, lgkmcnt(1) is enough for the read; without it, it is not
    with_store = "    ds_read_b128 v[4:7], v1\n    ds_write_b32 v2, v3\n    s_waitcnt lgkmcnt(1)\n    v_mov_b32_e32 v9, v4\n"
    assert check_lds_waits.scan(with_store)["violations"] == []
    assert len(check_lds_waits.scan(with_store.replace("    ds_write_b32 v2, v3\n", ""))["violations"]) == 1


def test_scalar_loads_are_ignored_and_overwrites_are_found():
    r = check_lds_waits.scan("    ds_read_b64_tr_b16 v[4:5], v1\n    s_load_dword s4, s[0:1], 0x0\n    v_mov_b32_e32 v5, 0\n    s_waitcnt lgkmcnt(0)\n")
    assert len(r["violations"]) == 1


@pytest.mark.skipif(not os.path.exists(build.HIPCC), reason="needs hipcc")
def test_the_fused_kernel_reads_no_register_in_flight():
    r = check_lds_waits.scan(check_lds_waits.listing_of(os.path.join(build.CSRC, "jfa_bwd_dkv_dma.hip")))
    assert r["lds_reads"] > 1000 and r["violations"] == [], r["violations"][:5]
    assert r["deepest_queue"] <= 15   # the counter has four bits


def test_partial_vmcnt_model_counts_what_follows_a_wait():
    text = """
        s_waitcnt vmcnt(2) lgkmcnt(0)
        global_load_lds_dwordx4 v1, s[2:3]
        global_store_dwordx4 v[2:3], v[4:7], off
        scratch_load_dword v9, off, off
        global_store_dwordx4 v[2:3], v[4:7], off
        s_barrier
        global_store_dwordx4 v[2:3], v[4:7], off
    """
    assert check_lds_waits.behind_partial_vmcnt_wait(text, 2) == [(1, 2, 1)]
    assert check_lds_waits.behind_partial_vmcnt_wait(text, 3) == []


def test_the_few_query_backward_leaves_exactly_its_stores_in_flight():
    """Its wait for a block's K and V rows is vmcnt(16): sixteen copies of the next block, then the sixteen stores of
    dK and dV that may stay in flight, and no other vector-memory instruction (no scratch) in the block loop."""
    listing = check_lds_waits.listing_of(os.path.join(build.CSRC, "jfa_bwd_cross_fewq.hip"))
    assert check_lds_waits.behind_partial_vmcnt_wait(listing, 16) == [(16, 16, 0)]
