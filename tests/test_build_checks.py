"""The build-time check of the generated kernels (no register copy while an inline LDS read into
the source is pending) on hand-written assembly: it must flag the hazard and pass the safe forms."""

from paper_2601_11590_amd import check_lds_waits as C

HEAD = "\t.type\tk,@function\nk:\n"
TAIL = "\ts_endpgm\n.Lfunc_end0:\n"


def errs(body):
    return C.check_asm(HEAD + body + TAIL, ("k",))


def test_copy_before_the_wait_is_flagged_and_after_it_is_not():
    bad = "\tds_read_b128 v[4:7], v1\n\tv_mov_b64_e32 v[8:9], v[4:5]\n\ts_waitcnt lgkmcnt(0)\n"
    good = "\tds_read_b128 v[4:7], v1\n\ts_waitcnt lgkmcnt(0)\n\tv_mov_b64_e32 v[8:9], v[4:5]\n"
    assert len(errs(bad)) == 1 and "v4" in errs(bad)[0]
    assert errs(good) == []


def test_counted_wait_retires_the_oldest_reads_only():
    body = ("\tds_read_b128 v[4:7], v1\n\tds_read_b128 v[8:11], v1\n\ts_waitcnt lgkmcnt(1)\n"
            "\tv_mov_b32_e32 v20, v5\n")                       # first read done: fine
    assert errs(body) == []
    body2 = body + "\tv_mov_b32_e32 v21, v9\n"                 # second read still pending
    assert len(errs(body2)) == 1 and "v9" in errs(body2)[0]
    # a scalar load in the queue may take the completion the wait guarantees
    body3 = ("\tds_read_b128 v[4:7], v1\n\ts_load_dword s4, s[0:1], 0x0\n\tds_read_b128 v[8:11], v1\n"
             "\ts_waitcnt lgkmcnt(2)\n\tv_mov_b32_e32 v20, v5\n")
    assert len(errs(body3)) == 1


def test_pending_reads_are_followed_around_a_loop_and_across_a_branch():
    # the read is issued at the end of the loop body; the copy at its top comes before the wait
    loop = (".LBB0_1:\n\tv_mov_b32_e32 v20, v4\n\ts_waitcnt lgkmcnt(0)\n\tv_mfma_f32_32x32x16_bf16 v[30:45], v[4:7], v[4:7], v[30:45]\n"
            "\tds_read_b128 v[4:7], v1\n\ts_cbranch_scc1 .LBB0_1\n")
    assert len(errs(loop)) == 1
    # one path waits, the other does not: the copy behind the join is flagged
    branch = ("\tds_read_b128 v[4:7], v1\n\ts_cbranch_scc1 .LBB0_2\n\ts_waitcnt lgkmcnt(0)\n.LBB0_2:\n\tv_mov_b32_e32 v20, v4\n")
    assert len(errs(branch)) == 1
    # spills count as copies; ordinary arithmetic on the path-insensitive walk does not
    assert len(errs("\tds_read_b128 v[4:7], v1\n\tscratch_store_dword off, v4, off\n\ts_waitcnt lgkmcnt(0)\n")) == 1
    assert errs("\tds_read_b128 v[4:7], v1\n\tv_add_u32_e32 v20, v4, v3\n\ts_waitcnt lgkmcnt(0)\n") == []


def test_a_file_without_the_kernel_is_an_error():
    assert C.check_asm("\t.text\n", ("gemm_bf16_kernel",)) != []


def test_an_overwritten_register_is_no_longer_awaited():
    # the read is pending only on the path that skips the wait; the register then gets a new
    # value (an accumulator read back), and copying THAT is not a hazard
    body = ("\tds_read_b128 v[4:7], v1\n\ts_cbranch_scc1 .LBB0_2\n\ts_waitcnt lgkmcnt(0)\n.LBB0_2:\n"
            "\tv_accvgpr_read_b32 v4, a3\n\tv_mov_b32_e32 v20, v4\n\tv_mov_b32_e32 v21, v5\n")
    e = errs(body)
    assert len(e) == 1 and "v5" in e[0]                        # v5 was not overwritten: still flagged


def test_overwriting_a_register_with_a_read_in_flight_in_the_same_block_is_flagged():
    bad = "\tds_read_b128 v[4:7], v1\n\tv_add_u32_e32 v5, v2, v3\n\ts_waitcnt lgkmcnt(0)\n"
    e = errs(bad)
    assert len(e) == 1 and "overwrites v5" in e[0]
    good = "\tds_read_b128 v[4:7], v1\n\ts_waitcnt lgkmcnt(0)\n\tv_add_u32_e32 v5, v2, v3\n"
    assert errs(good) == []
    # counted wait: the older read has landed, the younger has not
    two = ("\tds_read_b128 v[4:7], v1\n\tds_read_b128 v[8:11], v1\n\ts_waitcnt lgkmcnt(1)\n"
           "\tv_mov_b32_e32 v4, v20\n\tv_mov_b32_e32 v9, v20\n")
    e = errs(two)
    assert len(e) == 1 and "overwrites v9" in e[0]
