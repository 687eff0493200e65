"""The C-ABI library loads, exports every symbol include/ssmm.h declares, and its
host-side checks answer without touching a GPU."""
import ctypes
import os
import re

import pytest

from paper_2503_10725_amd import binding as B
from oracle import ssmm_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ssmm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ssmm_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_functions()
    assert len(names) >= 9
    lib = B.lib()
    for n in names:
        assert getattr(lib, n) is not None
        assert n in B.EXPORTS, f"{n} is declared in the header but has no ctypes signature"
    assert sorted(B.EXPORTS) == names


def test_strerror():
    assert B.strerror(0) == "ok"
    for code in (B.SSMM_EINVAL, B.SSMM_ESHAPE, B.SSMM_EWORKSPACE, B.SSMM_EHIP, B.SSMM_ELIMIT, -99):
        assert isinstance(B.strerror(code), str) and B.strerror(code)


@pytest.mark.parametrize("rows,K,fmt", [(64, 128, (1, 1, 0)), (64, 128, (1, 2, 8)), (14336, 4096, (1, 2, 8)), (32, 96, (4, 8, 32)),
                                        (128, 256, (1, 2, 16)), (128, 256, (1, 2, 32)), (64, 192, (1, 2, 12)),
                                        (128, 256, (4, 8, 32)), (256, 128, (8, 16, 32)), (64, 128, (2, 4, 64)), (128, 128, (1, 4, 32)),
                                        (128, 256, (4, 8, 16)), (96, 128, (3, 4, 32)), (32, 128, (4, 8, 32)),
                                        (6, 20, (1, 1, 0)), (1024, 512, (1, 1, 0)), (14336, 4096, (1, 1, 0))])
def test_compressed_sizes_match_closed_forms_and_oracle(rows, K, fmt):
    vb, mb, ib, tb = B.compressed_sizes(rows, K, fmt)
    assert (vb, mb, ib) == O.compressed_sizes(rows, K, O.Format(*fmt))
    N, M, V = fmt
    rc = rows * N // M if N < M else rows
    assert vb == rc * (K // 2) * 2                      # (m N/M) x (k/2) bf16
    if K % 32 == 0:
        assert mb * 8 == rc * (K // 2) * 2              # 2 bits per kept value
    assert ib == (rc * (K // V) if N < M else 0)        # (m N/M) x (k/V) bytes
    pow2 = lambda v: v > 0 and v & (v - 1) == 0
    masked = N == 1 and M == 2 and V % 8 == 0                  # every stored operand multiplied once per source row
    gathered = N < M and not masked and pow2(M) and M <= 32 and M % N == 0 and pow2(M // N) and V % 32 == 0
    tileable = (N == M or masked or (gathered and rows % 32 == 0)) and rc % 32 == 0 and K % 64 == 0
    vidx = 0
    if masked:
        vidx = (rc // 32) * (K // 64) * 64 * 2                 # 2 source-row bits per lane and k block
    if gathered:
        vidx = rows * (K // 32)                                # one byte per dense row and k block
    assert tb == (vb + mb + vidx if tileable else 0)


def test_host_side_argument_checks():
    lib = B.lib()
    f24 = B.Format(1, 1, 0)
    sz = ctypes.c_size_t(0)
    assert lib.ssmm_compressed_sizes(64, 126, f24, ctypes.byref(sz), None, None, None) == B.SSMM_ESHAPE
    assert lib.ssmm_compressed_sizes(63, 128, B.Format(1, 2, 8), None, None, None, None) == B.SSMM_ESHAPE
    assert lib.ssmm_compressed_sizes(64, 132, B.Format(1, 2, 8), None, None, None, None) == B.SSMM_ESHAPE
    assert lib.ssmm_compressed_sizes(64, 128, B.Format(2, 1, 8), None, None, None, None) == B.SSMM_EINVAL
    assert lib.ssmm_compressed_sizes(64, 128, B.Format(1, 2, 6), None, None, None, None) == B.SSMM_EINVAL
    assert lib.ssmm_compress_weights(None, 1, 64, 128, f24, None, None, None, None, None) == B.SSMM_EINVAL
    one = ctypes.c_void_p(256)   # never dereferenced: the calls below fail before any launch
    assert lib.ssmm_compress_weights(one, 1, 64, 126, f24, one, one, None, None, None) == B.SSMM_ESHAPE
    assert lib.ssmm_compress_weights(one, 1, 48, 128, f24, None, None, None, one, None) == B.SSMM_ESHAPE
    assert lib.ssmm_compress_weights(one, 1, 64, 128, f24, one, None, None, None, None) == B.SSMM_EINVAL
    assert lib.ssmm_decompress_weights(None, one, None, 1, 64, 128, f24, one, None) == B.SSMM_EINVAL
    assert lib.ssmm_untile_weights(one, 1, 64, 96, f24, one, one, None, None) == B.SSMM_ESHAPE
    # expansion to plain 2:4 operands: gathered formats only, tileable shapes, pointers; no expert is a no-op
    g48 = B.Format(4, 8, 32)
    assert lib.ssmm_expand_tiled_weights(one, 1, 64, 128, f24, one, None) == B.SSMM_ESHAPE
    assert lib.ssmm_expand_tiled_weights(one, 1, 64, 128, B.Format(1, 2, 8), one, None) == B.SSMM_ESHAPE
    assert lib.ssmm_expand_tiled_weights(one, 1, 48, 128, g48, one, None) == B.SSMM_ESHAPE
    assert lib.ssmm_expand_tiled_weights(one, 1, 64, 96, g48, one, None) == B.SSMM_ESHAPE
    assert lib.ssmm_expand_tiled_weights(None, 1, 64, 128, g48, one, None) == B.SSMM_EINVAL
    assert lib.ssmm_expand_tiled_weights(one, 0, 64, 128, g48, one, None) == B.SSMM_OK
    # routing: top-k out of range, too many experts, missing pointers, small workspace
    args = lambda T, E, k, S, ws: (one, T, E, k, S, 1, one, one, one, one, one, one, one, ws, None)
    assert lib.ssmm_route_bucket(*args(8, 4, 5, 0, 1 << 20)) == B.SSMM_ESHAPE
    assert lib.ssmm_route_bucket(*args(8, 4, 0, 0, 1 << 20)) == B.SSMM_ESHAPE
    assert lib.ssmm_route_bucket(*args(8, 255, 2, 2, 1 << 20)) == B.SSMM_ESHAPE
    assert lib.ssmm_route_bucket(*args(8, 64, 17, 0, 1 << 20)) == B.SSMM_ESHAPE
    assert lib.ssmm_route_bucket(*args(-1, 4, 2, 0, 1 << 20)) == B.SSMM_EINVAL
    assert lib.ssmm_route_bucket(*args(8, 4, 2, 0, 16)) == B.SSMM_EWORKSPACE
    assert lib.ssmm_route_bucket(None, 8, 4, 2, 0, 1, one, one, one, one, one, one, one, 1 << 20, None) == B.SSMM_EINVAL
    assert B.route_workspace_bytes(8192, 64, 6, 2) >= 32 * 64 * 4
    # router: reduction length, expert count, missing pointers; no tokens is a legal no-op
    assert lib.ssmm_router_logits(one, 8, 24, one, 4, one, None) == B.SSMM_ESHAPE
    assert lib.ssmm_router_logits(one, 8, 32, one, 257, one, None) == B.SSMM_ESHAPE
    assert lib.ssmm_router_logits(None, 8, 32, one, 4, one, None) == B.SSMM_EINVAL
    assert lib.ssmm_router_logits(one, 0, 32, one, 4, one, None) == B.SSMM_OK
    # FFN: untileable shapes, formats without a kernel-ready form, workspace
    ffn = lambda T, H, F, E, fmt, ws: (one, T, H, F, E, fmt, one, one, one, one, one, one, one, 2, one, one, ws, None)
    assert lib.ssmm_expert_ffn(*ffn(16, 96, 128, 4, f24, 1 << 30)) == B.SSMM_ESHAPE
    assert lib.ssmm_expert_ffn(*ffn(16, 128, 112, 4, f24, 1 << 30)) == B.SSMM_ESHAPE
    # stand-alone product: untileable shape, B too large for 32-bit offsets, missing pointers, workspace
    mm = lambda rows, K, fmt, n_b, n, ws, ptr=one: (ptr, rows, K, fmt, ptr, n_b, None, n, ptr, ptr, ws, None)
    assert lib.ssmm_matmul(*mm(48, 128, f24, 8, 8, 256)) == B.SSMM_ESHAPE
    assert lib.ssmm_matmul(*mm(64, 128, f24, 1 << 25, 8, 256)) == B.SSMM_ESHAPE
    assert lib.ssmm_matmul(*mm(64, 128, f24, 8, 9, 256)) == B.SSMM_EINVAL          # identity selection beyond B
    assert lib.ssmm_matmul(*mm(64, 128, f24, 8, 8, 256, None)) == B.SSMM_EINVAL
    assert lib.ssmm_matmul(*mm(64, 128, f24, 8, 8, 16)) == B.SSMM_EWORKSPACE
    assert lib.ssmm_matmul(*mm(64, 128, f24, 8, 0, 256)) == B.SSMM_OK               # nothing selected: no launch
    assert B.lib().ssmm_matmul_workspace_bytes(4096, 4096, 4096, f24) == 256              # enough tiles: no split
    assert B.lib().ssmm_matmul_workspace_bytes(256, 16384, 256, f24) == 256 + 8 * 256 * 256 * 4   # two tiles: 8 slices of fp32 partial sums
    assert lib.ssmm_matmul(*mm(256, 16384, f24, 256, 256, 256)) == B.SSMM_EWORKSPACE
    assert lib.ssmm_expert_ffn(*ffn(16, 128, 128, 4, B.Format(2, 4, 8), 1 << 30)) == B.SSMM_ESHAPE
    assert lib.ssmm_expert_ffn(*ffn(16, 128, 128, 4, B.Format(1, 2, 12), 1 << 30)) == B.SSMM_ESHAPE
    assert lib.ssmm_expert_ffn(*ffn(16, 128, 96, 4, B.Format(1, 2, 8), 1 << 30)) == B.SSMM_ESHAPE
    assert lib.ssmm_expert_ffn(*ffn(16, 128, 128, 4, f24, 64)) == B.SSMM_EWORKSPACE
    assert lib.ssmm_expert_ffn(*ffn(16, 128, 128, 0, f24, 1 << 30)) == B.SSMM_EINVAL
    assert lib.ssmm_expert_ffn(*ffn(16, 128, 128, 513, f24, 1 << 30)) == B.SSMM_ESHAPE    # more buckets than the kernels' table holds
    assert lib.ssmm_expert_ffn(*ffn(0, 128, 128, 4, f24, 0)) == B.SSMM_OK      # no tokens: legal no-op
    assert B.ffn_workspace_bytes(128, 512, 1024, 8, 2, f24) >= 256 * (1024 + 512) * 2


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libssmm.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()


def test_build_rejects_matrix_kernels_that_use_scratch_memory():
    """The build reads the compiler's per-kernel resource report: an SSMM kernel that spills is an error
    (its asm MFMAs and loads complete long after the compiler believes), other kernels may."""
    from paper_2503_10725_amd import build
    tag = " [-Rpass-analysis=kernel-resource-usage]"
    report = [
        "a.hip:1:1: remark: Function Name: _ZN4ssmm12ssmm_kernel2ILb1EEEvNS_8SsmmArgsE" + tag,
        "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 0" + tag,
        "a.hip:1:1: remark: Function Name: _ZN4ssmm11ssmm_kernelILb0EEEvNS_8SsmmArgsE" + tag,
        "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 68" + tag,
        "a.hip:1:1: remark: Function Name: _ZN4ssmm14combine_kernelEPKt" + tag,
        "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 16" + tag,
    ]
    assert build.scratch_users(report) == ["_ZN4ssmm11ssmm_kernelILb0EEEvNS_8SsmmArgsE"]
    assert build.scratch_users(report[:2]) == []


def test_build_rejects_hand_scheduled_kernels_that_park_registers_in_accumulation_registers():
    """Under register pressure the compiler parks VGPRs in unused AGPRs (no scratch involved); in a kernel whose
    loads are asm that can be the destination of a load still in flight.  The build compares each
    hand-scheduled instance's AGPR count with what its accumulators need."""
    from paper_2503_10725_amd import build
    tag = " [-Rpass-analysis=kernel-resource-usage]"
    ok = "_ZN4ssmm12ssmm_kernel2ILb1ELb0ELi1ELi1ELi4ELi1ELi4ELi2ELb0ELb0EEEvNS_8SsmmArgsE"     # gate+up, MT 1, NT 1: 32
    bad = "_ZN4ssmm12ssmm_kernel2ILb1ELb0ELi1ELi1ELi4ELi1ELi4ELi3ELb0ELb0EEEvNS_8SsmmArgsE"
    big = "_ZN4ssmm12ssmm_kernel2ILb1ELb0ELi2ELi5ELi4ELi1ELi3ELi1ELb0ELb0EEEvNS_8SsmmArgsE"    # 320 accumulators: capped at 256
    vec = "_ZN4ssmm12ssmm_kernel2ILb0ELb1ELi1ELi4ELi4ELi1ELi4ELi1ELb1ELb0EEEvNS_8SsmmArgsE"    # two passes: 128
    assert build.accumulator_registers(ok) == 32 and build.accumulator_registers(big) == 256
    assert build.accumulator_registers(vec) == 128
    assert build.accumulator_registers("_ZN4ssmm11ssmm_kernelILb0EEEvNS_8SsmmArgsE") is None
    report = []
    for name, agprs in ((ok, 32), (bad, 78), (big, 256), (vec, 132), ("_ZN4ssmm14combine_kernelEPKt", 0)):
        report += ["a.hip:1:1: remark: Function Name: " + name + tag, "a.hip:1:1: remark:     AGPRs: %d" % agprs + tag]
    assert build.agpr_parkers(report) == [bad]


def test_assembly_check_finds_every_access_to_a_register_whose_load_is_in_flight():
    """The build scans the device assembly of the hand-scheduled kernels (build.in_flight_hazards); here on
    hand-written snippets: a copy, a save to an accumulation register, a spill, an MFMA behind a wait that
    counts one load too few, and a use that is only wrong along the loop's back edge."""
    from paper_2503_10725_amd import build
    k2 = "_ZN4ssmm12ssmm_kernel2ILb1ELb0ELi1ELi1ELi4ELi1ELi4ELi2ELb0ELb0EEEvNS_8SsmmArgsE"
    asm = (k2 + """:
	;;#ASMSTART
	global_load_dwordx4 v[40:43], v0, s[34:35] offset:0x400
	;;#ASMEND
	v_accvgpr_write_b32 a40, v41
	v_accvgpr_write_b32 a41, v7
	v_mov_b32_e32 v50, v43
	scratch_store_dword off, v40, s32
	v_add_u32_e32 v9, v8, v7
	s_waitcnt vmcnt(0)
	v_accvgpr_write_b32 a42, v42
	v_mov_b32_e32 v51, v43
	s_endpgm
.Lfunc_end0:
_ZN4ssmm11ssmm_kernelILb0EEEvNS_8SsmmArgsE:
	;;#ASMSTART
	global_load_dwordx4 v[40:43], v0, s[34:35]
	;;#ASMEND
	v_accvgpr_write_b32 a40, v41
	s_endpgm
""").split("\n")
    found = build.in_flight_hazards(asm)
    assert [(t, r) for _, _, t, r in found] == [("v_accvgpr_write_b32 a40, v41", 41), ("v_mov_b32_e32 v50, v43", 43),
                                               ("scratch_store_dword off, v40, s32", 40)]
    assert all(k == k2 for k, _, _, _ in found)

    # loads return in order: vmcnt(N) covers a load once N or fewer were issued behind it
    counts = (k2 + """:
	;;#ASMSTART
	global_load_dwordx4 v[10:13], v0, s[34:35]
	;;#ASMEND
	;;#ASMSTART
	global_load_dwordx4 v[14:17], v0, s[34:35]
	;;#ASMEND
	;;#ASMSTART
	global_load_lds_dwordx4 v1, s[36:37]
	;;#ASMEND
	;;#ASMSTART
	s_waitcnt vmcnt(2)
	;;#ASMEND
	;;#ASMSTART
	v_smfmac_f32_32x32x32_bf16 a[0:15], v[10:13], v[20:27], v30
	;;#ASMEND
	;;#ASMSTART
	v_smfmac_f32_32x32x32_bf16 a[0:15], v[14:17], v[20:27], v30
	;;#ASMEND
	;;#ASMSTART
	s_waitcnt vmcnt(1)
	;;#ASMEND
	;;#ASMSTART
	v_smfmac_f32_32x32x32_bf16 a[0:15], v[14:17], v[20:27], v30
	;;#ASMEND
	s_endpgm
""").split("\n")
    found = build.in_flight_hazards(counts)
    assert sorted({r for _, _, _, r in found}) == [14, 15, 16, 17] and len({n for _, n, _, _ in found}) == 1

    # a load at the end of a loop body is still in flight at the top of the next pass
    loop = (k2 + """:
	s_mov_b32 s0, 0
.LBB0_1:
	v_add_u32_e32 v5, v12, v6
	;;#ASMSTART
	s_waitcnt vmcnt(0)
	;;#ASMEND
	v_add_u32_e32 v5, v13, v6
	;;#ASMSTART
	global_load_dwordx4 v[10:13], v0, s[34:35]
	;;#ASMEND
	s_add_i32 s0, s0, 1
	s_cmp_lt_i32 s0, 8
	s_cbranch_scc1 .LBB0_1
	s_waitcnt vmcnt(0)
	v_add_u32_e32 v5, v13, v6
	s_endpgm
""").split("\n")
    found = build.in_flight_hazards(loop)
    assert [(t, r) for _, _, t, r in found] == [("v_add_u32_e32 v5, v12, v6", 12)]
