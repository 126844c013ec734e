"""The build-time scan of the fast encoder's assembly (paper_2601_17702_amd/asm_check.py) on hand-written snippets:
it has to flag each of the five patterns it exists for, and to accept the shapes the kernel really has."""
from paper_2601_17702_amd import asm_check

MFMA = "v_mfma_f32_32x32x16_bf16 v[16:31], v[40:43], v[44:47], v[16:31]"


def test_accepts_chain_and_distant_read():
    ok = [MFMA, MFMA, "v_sub_f32 v2, v3, v100", MFMA] + ["v_add_u32 v2, v2, v3"] * 9 + ["s_nop 1", "v_mov_b32 v60, v16"]
    assert asm_check.scan_kernel(ok) == []


def test_flags_early_read_of_mfma_result():
    bad = [MFMA, "s_nop 0", "v_mov_b64_e32 v[124:125], v[30:31]"]
    assert any("MFMA result" in f for f in asm_check.scan_kernel(bad))
    # ten other instructions are not enough, eleven are
    assert asm_check.scan_kernel([MFMA] + ["s_mov_b32 s0, s1"] * 10 + ["v_mov_b32 v1, v16"])
    assert asm_check.scan_kernel([MFMA] + ["s_mov_b32 s0, s1"] * 11 + ["v_mov_b32 v1, v16"]) == []


def test_flags_register_of_lds_read_in_flight():
    bad = ["ds_read_b128 v[4:7], v200 offset:128", "v_mov_b64_e32 v[198:199], v[4:5]", "s_waitcnt lgkmcnt(0)"]
    assert any("in flight" in f for f in asm_check.scan_kernel(bad))
    ok = ["ds_read_b128 v[4:7], v200 offset:128", "v_add_u32 v9, v9, v10", "s_waitcnt lgkmcnt(0)", "v_mov_b64_e32 v[198:199], v[4:5]"]
    assert asm_check.scan_kernel(ok) == []
    # reads complete in order: lgkmcnt(1) covers all but the last one
    part = ["ds_read_b32 v4, v200", "ds_read_b32 v5, v200 offset:4", "s_waitcnt lgkmcnt(1)", "v_add_u32 v6, v4, v4"]
    assert asm_check.scan_kernel(part) == []
    assert any("in flight" in f for f in asm_check.scan_kernel(part + ["v_add_u32 v7, v5, v5"]))
    call = ["ds_read_b128 v[4:7], v200", "s_swappc_b64 s[30:31], s[0:1]"]
    assert any("call" in f for f in asm_check.scan_kernel(call))


def test_flags_vector_write_right_before_mfma_source():
    bad = ["v_accvgpr_read_b32 v40, a3", MFMA]
    assert any("source written" in f for f in asm_check.scan_kernel(bad))
    assert asm_check.scan_kernel(["v_accvgpr_read_b32 v40, a3", "s_nop 1", MFMA]) == []


def test_flags_partial_wait_with_scalar_load_in_flight():
    # the chain's own shape: reads issued in a block, each MFMA behind the partial wait that covers its fragment
    chain = ["s_waitcnt lgkmcnt(0)", "ds_read_b128 v[40:43], v200", "ds_read_b128 v[48:51], v201",
             "s_waitcnt lgkmcnt(1)", MFMA, "s_waitcnt lgkmcnt(0)",
             "v_mfma_f32_32x32x16_bf16 v[16:31], v[48:51], v[44:47], v[16:31]"]
    assert asm_check.scan_kernel(chain) == []
    # scalar loads count on the same counter and return out of order: a partial wait then proves nothing
    bad = ["s_load_dwordx2 s[4:5], s[0:1], 0x0"] + chain[1:]
    assert any("scalar-memory" in f for f in asm_check.scan_kernel(bad))
    # a fragment consumed before its wait
    early = chain[:3] + [MFMA]
    assert any("in flight" in f for f in asm_check.scan_kernel(early))


def test_flags_scc_kept_across_an_asm_statement_that_writes_it():
    blk = ["#asm_begin", "v_cmp_eq_u32 vcc, v1, v2", "s_or_b64 s[0:1], s[0:1], vcc", "#asm_end"]
    bad = ["s_cmp_eq_u32 s4, 0"] + blk + ["s_cselect_b64 vcc, -1, 0"]
    assert any("SCC" in f for f in asm_check.scan_kernel(bad))
    # the compiler compares again behind the statement: fine
    assert asm_check.scan_kernel(["s_cmp_eq_u32 s4, 0"] + blk + ["s_cmp_eq_u32 s4, 0", "s_cselect_b64 vcc, -1, 0"]) == []
    # a statement that leaves SCC alone
    ok = ["s_cmp_eq_u32 s4, 0", "#asm_begin", "v_add_u32 v1, v1, v2", "#asm_end", "s_cbranch_scc1 .LBB0_2"]
    assert asm_check.scan_kernel(ok) == []


def test_scan_file_splits_kernels(tmp_path):
    p = tmp_path / "k.s"
    p.write_text("\n".join([
        "\t.text", "_Z3foo_sae_encode_topk_x:", "; comment", "\t" + MFMA, "\ts_nop 0", "\tv_mov_b32 v1, v16", "\ts_endpgm",
        "_Z5other:", "\t" + MFMA, "\tv_mov_b32 v1, v16", "\ts_endpgm", ""]))
    res = asm_check.scan_file(str(p), "sae_encode_topk_")
    assert list(res) == ["_Z3foo_sae_encode_topk_x"] and len(res["_Z3foo_sae_encode_topk_x"]) == 1
