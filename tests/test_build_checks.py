"""The build inspects the assembly of the attention kernels (their matrix instructions are inline
assembly that updates accumulator registers behind the compiler's back).  These tests plant each
kind of violation in a small fake assembly text and make sure the checker objects; no GPU needed."""
from paper_2410_02367_amd.build import check_attention_asm

KERNELS = ["_ZN4sage16sage_attn_kernelILi%dELi%dELb%dELb%dELb%dEEEvPKa" % (d, nw, c, dump, ktok)
           for d in (64, 128) for nw in (4, 8)
           for c, dump, ktok in ((0, 1, 0), (1, 0, 0), (0, 0, 0), (1, 0, 1), (0, 0, 1))
           if not (d == 128 and nw == 4 and ktok)]
# the two measurement builds (clock counters): D = 128, 8 wavefronts, causal / full
KERNELS += ["_ZN4sage16sage_attn_kernelILi128ELi8ELb%dELb0ELb0ELb1EEEvPKa" % c for c in (1, 0)]


def fake(body_of_first: str) -> str:
    parts = []
    for i, k in enumerate(KERNELS):
        body = body_of_first if i == 0 else "\ts_endpgm\n"
        parts.append(f"{k}:\n{body}.Lfunc_end{i}:\n")
    return "\n".join(parts)


CLEAN = """\tv_accvgpr_mov_b32 a16, a0
\ts_cbranch_scc1 .LBB0_2
.LBB0_1:
\t;;#ASMSTART
\tv_mfma_f32_32x32x16_f16 a[0:15], v[0:3], v[4:7], a[0:15]
\t;;#ASMEND
\tv_fma_f32 v1, v2, v3, v4
\ts_cbranch_scc1 .LBB0_1
.LBB0_2:
\t;;#ASMSTART
\ts_nop 11
\t;;#ASMEND
\tv_accvgpr_read_b32 v9, a3
\ts_endpgm
"""


def test_clean_text_passes():
    assert check_attention_asm(fake(CLEAN)) == []


def test_missing_kernel_is_reported():
    text = fake(CLEAN).split(KERNELS[-1])[0]
    assert any("expected 20" in p for p in check_attention_asm(text))


def test_accumulator_copy_after_first_matrix_instruction_is_reported():
    bad = CLEAN.replace("\tv_fma_f32 v1, v2, v3, v4\n", "\tv_fma_f32 v1, v2, v3, v4\n\tv_accvgpr_mov_b32 a20, a4\n")
    assert any("accumulator-to-accumulator copy" in p for p in check_attention_asm(fake(bad)))


def test_accumulator_read_beside_matrix_instructions_is_reported():
    bad = CLEAN.replace("\tv_fma_f32 v1, v2, v3, v4\n", "\tv_accvgpr_read_b32 v1, a4\n")
    assert any("accumulator read next to matrix instructions" in p for p in check_attention_asm(fake(bad)))


def test_registers_that_no_matrix_instruction_names_are_the_compilers_to_use():
    ok = CLEAN.replace("\tv_fma_f32 v1, v2, v3, v4\n", "\tv_accvgpr_read_b32 v1, a40\n\tv_accvgpr_mov_b32 a41, a42\n")
    assert check_attention_asm(fake(ok)) == []


def test_scratch_and_m0_are_reported():
    bad = CLEAN.replace("\tv_fma_f32 v1, v2, v3, v4\n", "\tscratch_store_dword off, v1, off\n\ts_mov_b32 m0, s4\n")
    problems = check_attention_asm(fake(bad))
    assert any("scratch access" in p for p in problems)
    assert any("use of m0" in p for p in problems)


def test_m0_inside_the_sources_own_assembly_is_allowed():
    ok = CLEAN.replace("\ts_nop 11\n", "\ts_mov_b32 m0, s4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 v[0:1], off\n")
    assert check_attention_asm(fake(ok)) == []


def test_touching_a_matrix_result_too_early_is_reported():
    early = CLEAN.replace("\tv_fma_f32 v1, v2, v3, v4\n",
                          "\t;;#ASMSTART\n\tv_mfma_i32_32x32x32_i8 v[8:23], v[0:3], a[0:3], v[8:23]\n\t;;#ASMEND\n"
                          "\tv_add_f32_e32 v30, v31, v32\n\tv_exp_f32_e32 v9, v30\n")
    assert any("touches the result" in p for p in check_attention_asm(fake(early)))
    # the same access after a long enough pause is fine, and so is the next instruction of the chain
    late = early.replace("\tv_add_f32_e32 v30, v31, v32\n", "\ts_nop 11\n")
    assert check_attention_asm(fake(late)) == []
    chain = CLEAN.replace("\tv_fma_f32 v1, v2, v3, v4\n",
                          "\t;;#ASMSTART\n\tv_mfma_i32_32x32x32_i8 v[8:23], v[0:3], a[0:3], v[8:23]\n\t;;#ASMEND\n"
                          "\t;;#ASMSTART\n\tv_mfma_i32_32x32x32_i8 v[8:23], v[4:7], a[4:7], v[8:23]\n\t;;#ASMEND\n\ts_nop 11\n")
    assert check_attention_asm(fake(chain)) == []


def test_matrix_instruction_reading_a_fresh_valu_result_is_reported():
    bad = CLEAN.replace("\t;;#ASMSTART\n\tv_mfma_f32_32x32x16_f16 a[0:15], v[0:3], v[4:7], a[0:15]\n",
                        "\tv_cvt_pk_f16_f32 v5, v20, v21\n\t;;#ASMSTART\n\tv_mfma_f32_32x32x16_f16 a[0:15], v[0:3], v[4:7], a[0:15]\n")
    assert any("less than 2 wait states" in p for p in check_attention_asm(fake(bad)))
    ok = bad.replace("\tv_cvt_pk_f16_f32 v5, v20, v21\n", "\tv_cvt_pk_f16_f32 v5, v20, v21\n\tv_mov_b32_e32 v40, v41\n\tv_mov_b32_e32 v42, v41\n")
    assert check_attention_asm(fake(ok)) == []


# ------------------------------------------------------------------ INT8-P~V kernels (compiler-scheduled)

from paper_2410_02367_amd.build import check_pv8_asm  # noqa: E402

PV8_KERNELS = ["_ZN4sage20sage_attn_pv8_kernelILi%dELb%dELb%dELb%dEEEvPKa" % (d, c, k, sp)
               for d in (64, 128) for c in (0, 1) for k in (0, 1) for sp in (0, 1)]


def fake_pv8(body_of_first: str, kernels=PV8_KERNELS) -> str:
    return "\n".join(f"{k}:\n{body_of_first if i == 0 else chr(9) + 's_endpgm' + chr(10)}.Lfunc_end{i}:\n"
                     for i, k in enumerate(kernels))


PV8_CLEAN = """\t;;#ASMSTART
\ts_mov_b32 m0, s4
\ts_nop 0
\tbuffer_load_dwordx4 v1, s[8:11], 0 offen lds
\t;;#ASMEND
\tv_mfma_i32_32x32x32_i8 v[0:15], v[16:19], v[20:23], v[0:15]
\ts_endpgm
"""


def test_pv8_clean_text_passes_and_a_missing_kernel_is_reported():
    assert check_pv8_asm(fake_pv8(PV8_CLEAN)) == []
    assert any("expected 16" in p for p in check_pv8_asm(fake_pv8(PV8_CLEAN, PV8_KERNELS[:-1])))


def test_pv8_scratch_and_compiler_use_of_m0_are_reported():
    bad = PV8_CLEAN.replace("\ts_endpgm\n", "\tscratch_load_dword v1, off, off\n\ts_mov_b32 m0, s9\n\ts_endpgm\n")
    problems = check_pv8_asm(fake_pv8(bad))
    assert any("scratch access" in p for p in problems) and any("use of m0" in p for p in problems)


def test_spill_check_names_the_kernel_that_touches_scratch():
    from paper_2410_02367_amd.build import check_no_spills
    clean = "_ZN4sage15k_colsum_kernelILi64EEEv:\n\tv_add_u32 v0, v1, v2\n\ts_endpgm\n.Lfunc_end0:\n"
    assert check_no_spills(clean) == []
    spilling = clean.replace("\tv_add_u32 v0, v1, v2\n", "\tscratch_store_dword off, v3, off offset:4\n")
    problems = check_no_spills(clean + spilling.replace("k_colsum", "k_small").replace("func_end0", "func_end1"))
    assert len(problems) == 1 and "k_small" in problems[0]


def test_source_hash_guard_tells_a_foreign_binary_from_ours(tmp_path):
    """The library carries the hash of the sources it was built from; a file without the marker, or with
    another hash, is not ours."""
    from paper_2410_02367_amd import build
    h = build.source_hash()
    assert len(h) == 64 and h == build.source_hash()
    good = tmp_path / "good.so"
    good.write_bytes(b"\x7fELF junk " + build.HASH_MARKER + h.encode() + b"\0 more")
    assert build.built_hash(str(good)) == h
    other = tmp_path / "other.so"
    other.write_bytes(b"\x7fELF junk " + build.HASH_MARKER + (b"0" * 64) + b"\0")
    assert build.built_hash(str(other)) == "0" * 64 != h
    assert build.built_hash(str(tmp_path / "missing.so")) is None
    bare = tmp_path / "bare.so"
    bare.write_bytes(b"\x7fELF no marker here")
    assert build.built_hash(str(bare)) is None
    # the library in the tree belongs to the sources in the tree (load() would rebuild or refuse otherwise)
    from paper_2410_02367_amd import binding
    binding.load()
    assert not build.is_stale() and binding.sage_source_hash() == h
