"""Compile-time properties of the hot kernels, checked without a GPU: the gfx950 code object
must keep the tiled and skinny GEMM kernels free of scratch spills (a spill in the K loop costs
~30 % on an MI355X) and inside the LDS and register budgets their launch configuration assumes."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


@pytest.fixture(scope="module")
def asm(tmp_path_factory):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    out = tmp_path_factory.mktemp("asm") / "fle_kernels.s"
    subprocess.check_call([HIPCC, "-O3", "--offload-arch=gfx950", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-S", "--cuda-device-only",
                           "-o", str(out), os.path.join(ROOT, "paper_2511_16964_amd", "csrc", "fle_kernels.hip")],
                          stderr=subprocess.DEVNULL)
    return out.read_text()


def kernel_props(asm):
    props = {}
    for m in re.finditer(r"\.amdhsa_kernel (\S+)(.*?)\.end_amdhsa_kernel", asm, flags=re.S):
        body = m.group(2)
        get = lambda key: int(re.search(r"\.amdhsa_%s (\d+)" % key, body).group(1))
        props[m.group(1)] = dict(lds=get("group_segment_fixed_size"), scratch=get("private_segment_fixed_size"),
                                 vgpr=get("next_free_vgpr"))
    return props


def test_hot_kernels_do_not_spill_and_fit_their_budgets(asm):
    props = kernel_props(asm)
    names = {k: v for k, v in props.items() if "gemm_bf16_skinny" in k or "gemm_tiled_" in k}
    assert len(names) == 17 + 20 + 24, sorted(props)   # skinny: 7 shapes x 2 dtypes and 3 K steps in fp32; tiled: 2 tiles x 4 dtypes (fp8 among them) x 2 epilogues, and the block-scaled fp8 form of each tile and epilogue; grouped: the same 4 dtypes plus the 128 tile with streamed W
    for name, p in names.items():
        assert p["scratch"] == 0, "%s spills %d bytes of scratch" % (name, p["scratch"])
        assert p["lds"] <= 160 * 1024, name
        assert p["vgpr"] <= 512, name
    for t128 in [v for k, v in names.items() if "tiled_128" in k or "grouped_128" in k]:
        assert t128["lds"] <= 80 * 1024 and t128["vgpr"] <= 256  # two workgroups per CU
    for t256 in [v for k, v in names.items() if "tiled_256" in k or "grouped_256" in k]:
        assert t256["lds"] == 160 * 1024


def test_thin_kernels_do_not_spill(asm):
    props = kernel_props(asm)
    thin = {k: v for k, v in props.items() if "gemm_thin" in k or "gemm_gemv" in k}
    assert len(thin) == 6 + 13 + 12, sorted(thin)   # MFMA form: 3 dtypes x 2 row counts; dot-product form: 1, 2, 4 rows and the 16-wave form x 3 dtypes, 8 rows in fp32; the same again, up to 4 rows, with the LayerNorm of x folded in
    for name, p in thin.items():
        assert p["scratch"] == 0 and p["vgpr"] <= 256, (name, p)   # at least two waves per SIMD


def test_attention_kernels_keep_two_waves_per_simd(asm):
    props = kernel_props(asm)
    att = {k: v for k, v in props.items() if "flash_attention" in k}
    assert len(att) == 8, sorted(att)   # bf16 / fp16 x head dimension 32 / 64 / 128 / 256
    for name, p in att.items():
        assert p["scratch"] == 0, (name, p)
        if "Li256ELi1E" in name:        # head dimension 256: one wave per SIMD, one workgroup per CU
            assert p["vgpr"] <= 512 and p["lds"] == 128 * 1024, (name, p)
        else:
            assert p["vgpr"] <= 256 and p["lds"] <= 64 * 1024, (name, p)
    assert "ds_read_b64_tr_b16" in asm   # V is transposed by the LDS read itself


def test_chain_kernel_leaves_room_for_all_workgroups(asm):
    """The persistent perceptron kernel waits at a grid barrier, so every workgroup must be resident: 16 waves of
    at most 128 registers and next to no LDS let a CU hold two of them while the launch asks for one per CU."""
    props = kernel_props(asm)
    chain = {k: v for k, v in props.items() if "mlp_chain" in k}
    assert len(chain) == 5, sorted(chain)   # three dtypes, and bf16 / fp16 weights under fp32 activations
    for name, p in chain.items():
        # (the only LDS is the few words through which a workgroup agrees on whether its barrier wait was given up)
        assert p["scratch"] == 0 and p["vgpr"] <= 128 and p["lds"] <= 1024, (name, p)
    assert "buffer_wbl2" not in asm and "buffer_inv" not in asm   # no kernel flushes or invalidates a cache


def test_streaming_finalize_keeps_its_occupancy(asm):
    """The LayerNorm finalize pass is a streaming kernel: it needs several waves per SIMD, so its register count
    must stay bounded (a shared code path once pushed it to 149 and cost 40 % of its speed; holding a whole item's
    loads as one batch takes 116, four waves per SIMD, and measured faster than 79 with the loads one by one)."""
    props = kernel_props(asm)
    ln = [v for k, v in props.items() if "finalize_rowsILb1ELb1" in k]
    assert len(ln) == 3 and all(v["vgpr"] <= 128 and v["scratch"] == 0 for v in ln), ln   # one per storage dtype


def test_main_loop_uses_the_intended_instructions(asm):
    body = asm
    assert re.search(r"buffer_load_dwordx4 .* lds", body)          # direct-to-LDS copies
    assert "v_mfma_f32_16x16x4_f32" in asm                         # fp32 path stays on fp32 MFMA
    m = re.search(r"^_ZN3fle14gemm_tiled_256ILi0ELb0ELi32ELin1ELb0EEEvNS_8GemmArgsE:(.*?)s_endpgm", asm, flags=re.S | re.M)   # fp32 operands
    assert m and "v_mfma_f32_32x32x2_f32" in m.group(1) and "_bf16" not in m.group(1) and "x16_f16" not in m.group(1) and "x32_f16" not in m.group(1)
    # 2-byte operands: the tiled loop runs on the 16x16x32 shape, whose accumulators stay where they are (no
    # accumulator moves between register files inside the K loop) and nothing spills
    for dt, mn in ((1, "v_mfma_f32_16x16x32_bf16"), (2, "v_mfma_f32_16x16x32_f16")):
        for kern in ("gemm_tiled_256", "gemm_tiled_128"):
            m = re.search(r"^_ZN3fle14%sILi%dELb0ELi16ELin1ELb0EEEvNS_8GemmArgsE:(.*?)s_endpgm" % (kern, dt), asm, flags=re.S | re.M)
            assert m, (kern, dt)
            text = m.group(1)
            first, last = text.index(mn), text.rindex(mn)
            assert text.count(mn) >= 128 and "32x32x16" not in text
            # (the only accumulator moves allowed between the matrix instructions are the one-time zero fill,
            # which the compiler places between its copies of the K step)
            assert text[first:last].count("v_accvgpr") <= 256 and "v_accvgpr_read" not in text[first:last] and "scratch_" not in text
    assert "v_mfma_f32_16x16x16_bf16" in asm and "v_mfma_f32_16x16x16_f16" in asm   # general kernel on 2-byte operands
    assert "v_pk_fma_f32" not in asm and "v_pk_mul_f32" not in asm and "v_pk_add_f32" not in asm
