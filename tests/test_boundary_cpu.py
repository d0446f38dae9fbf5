"""CPU-only checks of the C-ABI library: it loads, exports every declared entry
point, its host-side packer and tile layout are bit-exact, and every argument
error is reported before any GPU call.  No kernel is launched here.
"""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2505_11076_amd import binding as B
from paper_2505_11076_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "dbf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dbf_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared_symbols()
    assert len(names) >= 18
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTS) == names


def test_strerror_covers_all_codes():
    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -6):
        msg = B.strerror(code)
        assert msg and msg != "unknown error code"
        seen.add(msg)
    assert len(seen) == 7
    assert B.strerror(-99) == "unknown error code"


# ---- sign -> bit conversion -----------------------------------------------------------------------


def _bits_by_hand(S):
    """Canonical words by Python integer arithmetic (independent of both packers)."""
    rows, cols = S.shape
    out = np.zeros((rows, (cols + 31) // 32), dtype=np.uint32)
    for r in range(rows):
        for c in range(cols):
            if S[r, c] == 1:
                out[r, c // 32] |= np.uint32(1 << (c % 32))
    return out


@pytest.mark.parametrize("cols", [1, 31, 32, 33, 64, 100, 256])
def test_signs_to_bits_host(cols):
    rng = np.random.default_rng(cols)
    S = I.random_signs(rng, 7, cols)
    got = B.dbf_signs_to_bits_host(S)
    assert np.array_equal(got, _bits_by_hand(S))


def test_signs_to_bits_rejects_non_signs():
    for bad in (0, 2, -2, 127):
        S = np.ones((3, 40), dtype=np.int8)
        S[2, 39] = bad
        with pytest.raises(B.DbfError) as e:
            B.dbf_signs_to_bits_host(S)
        assert e.value.code == B.DBF_ENOTSIGN


# ---- tile layout --------------------------------------------------------------------------------------


def _tile_by_formula(rows, cols, bits):
    """The documented layout, element by element: byte 256g+16r+j, bit s of tile
    (rt, ct) is the sign at (128rt + 16s + r, 64ct + 16g + j)."""
    n_rt, n_ct = (rows + 127) // 128, (cols + 63) // 64
    out = np.zeros(n_rt * n_ct * 1024, dtype=np.uint8)
    for row in range(rows):
        rt, s, r = row // 128, (row % 128) // 16, row % 16
        for col in range(cols):
            if (int(bits[row, col // 32]) >> (col % 32)) & 1:
                ct, g, j = col // 64, (col % 64) // 16, col % 16
                out[(rt * n_ct + ct) * 1024 + 256 * g + 16 * r + j] |= np.uint8(1 << s)
    return out


@pytest.mark.parametrize("shape", [(1, 1), (16, 64), (128, 64), (129, 65), (200, 130), (300, 97), (17, 200)])
def test_tile_host_matches_documented_layout(shape):
    rows, cols = shape
    rng = np.random.default_rng(rows * 1000 + cols)
    bits = I.random_sign_words(rng, rows, cols)
    tiled = B.dbf_tile_host(rows, cols, bits)
    assert tiled.size == B.dbf_tiled_bytes(rows, cols) == ((rows + 127) // 128) * ((cols + 63) // 64) * 1024
    assert np.array_equal(tiled, _tile_by_formula(rows, cols, bits))


@pytest.mark.parametrize("shape", [(1, 1), (5, 31), (128, 64), (2985, 100), (100, 2985), (256, 5970), (513, 4096)])
def test_tile_round_trip(shape):
    rows, cols = shape
    rng = np.random.default_rng(rows * 7 + cols)
    bits = I.random_sign_words(rng, rows, cols)
    tiled = B.dbf_tile_host(rows, cols, bits)
    back = B.dbf_untile_host(rows, cols, tiled)
    assert np.array_equal(back, bits)


def test_tile_host_padding_is_zero():
    rows, cols = 130, 70
    bits = np.full((rows, 3), 0xFFFFFFFF, dtype=np.uint32)
    bits[:, 2] = (1 << (cols - 64)) - 1
    tiled = B.dbf_tile_host(rows, cols, bits)
    total_set = int(np.unpackbits(tiled).sum())
    assert total_set == rows * cols


def test_tile_host_rejects_dirty_tail():
    bits = np.zeros((4, 2), dtype=np.uint32)
    bits[3, 1] = 1 << 20  # column 52 of a 40-column matrix
    lib = B.lib()
    out = np.zeros(B.dbf_tiled_bytes(4, 40), dtype=np.uint8)
    assert lib.dbf_tile_host(4, 40, bits.ctypes.data, out.ctypes.data) == B.DBF_ENOTSIGN


def test_tiled_bytes_out_of_range():
    assert B.dbf_tiled_bytes(0, 5) == 0
    assert B.dbf_tiled_bytes(5, -1) == 0
    assert B.dbf_tiled_bytes(1 << 21, 5) == 0


# ---- argument errors of the GPU entry points (reported with no GPU present) ------------------


def _small_operands():
    L = I.make_layer(n_in=40, n_out=24, k=33, seed=5)
    return L


def test_pack_argument_errors():
    lib = B.lib()
    L = _small_operands()
    h = C.c_void_p(123)
    p = lambda arr: arr.ctypes.data
    # null pointers
    assert lib.dbf_pack_bits(40, 24, 33, None, p(L.B_bits), p(L.a), p(L.m), p(L.b), C.byref(h)) == B.DBF_EINVAL
    assert h.value is None
    assert lib.dbf_pack_bits(40, 24, 33, p(L.A_bits), p(L.B_bits), p(L.a), p(L.m), p(L.b), None) == B.DBF_EINVAL
    assert lib.dbf_pack(40, 24, 33, None, None, p(L.a), p(L.m), p(L.b), C.byref(h)) == B.DBF_EINVAL
    # shapes
    for bad in ((0, 24, 33), (40, 0, 33), (40, 24, 0), (-1, 24, 33), ((1 << 20) + 1, 24, 33)):
        assert lib.dbf_pack_bits(*bad, p(L.A_bits), p(L.B_bits), p(L.a), p(L.m), p(L.b), C.byref(h)) == B.DBF_ESHAPE
    # non-sign entries are found before the GPU is touched
    A = np.ones((24, 33), dtype=np.int8)
    Bm = np.ones((33, 40), dtype=np.int8)
    Bm[32, 39] = 0
    assert lib.dbf_pack(40, 24, 33, p(A), p(Bm), p(L.a), p(L.m), p(L.b), C.byref(h)) == B.DBF_ENOTSIGN
    # dirty tail bits in canonical words
    Ab = L.A_bits.copy()
    Ab[0, -1] |= np.uint32(1 << 31)
    assert lib.dbf_pack_bits(40, 24, 33, p(Ab), p(L.B_bits), p(L.a), p(L.m), p(L.b), C.byref(h)) == B.DBF_ENOTSIGN


def test_launch_argument_errors():
    lib = B.lib()
    assert lib.dbf_gemv(None, 1, 1, 1, None) == B.DBF_EINVAL
    assert lib.dbf_gemv_kind(None, 1, 1, 1, 0, None) == B.DBF_EINVAL
    assert lib.dbf_gemm(None, 1, 1, 1, 1, 1, None) == B.DBF_EINVAL
    assert lib.dbf_gemm_workspace_bytes(None, 5) == 0
    assert lib.dbf_unpack_bits(None, None, None, None, None, None) == B.DBF_EINVAL
    assert lib.dbf_dims(None, None, None, None, None) == B.DBF_EINVAL
    h = C.c_void_p(0)
    assert lib.dbf_stack_create(None, 1, C.byref(h)) == B.DBF_EINVAL
    arr = (C.c_void_p * 1)(None)
    assert lib.dbf_stack_create(arr, 1, C.byref(h)) == B.DBF_EINVAL
    assert lib.dbf_stack_create(arr, 0, C.byref(h)) == B.DBF_EINVAL
    assert lib.dbf_stack_create_grouped(None, 1, None, 0, C.byref(h)) == B.DBF_EINVAL
    assert lib.dbf_prune_middle(None, None, 1, C.byref(h)) == B.DBF_EINVAL
    assert lib.dbf_svid(None, 4, 4, 1, None, None, None, None, 0, None) == B.DBF_EINVAL
    assert lib.dbf_svid_workspace_bytes(0, 4) == 0 and lib.dbf_svid_workspace_bytes(64, 64) > 0
    assert lib.dbf_admm_step(None, None, 4, 4, 1.0, 1, None, None, None, None, None, 0, None) == B.DBF_EINVAL
    assert lib.dbf_admm_workspace_bytes(0, 4) == 0 and lib.dbf_admm_workspace_bytes(64, 64) >= 2 * 4 * 64 * 64
    assert lib.dbf_stack_create_grouped(arr, 1, None, 0, C.byref(h)) == B.DBF_EINVAL
    assert lib.dbf_stack_gemv(None, 1, 1, 1, 0, None) == B.DBF_EINVAL
    assert lib.dbf_stack_offsets(None, 0, 1, None, None) == B.DBF_EINVAL
    lib.dbf_free(None)
    lib.dbf_stack_free(None)


def test_binding_rejects_wrong_host_sizes():
    L = _small_operands()
    with pytest.raises(B.DbfError) as e:
        B.dbf_pack_bits(40, 24, 33, L.A_bits[:-1], L.B_bits, L.a, L.m, L.b)
    assert e.value.code == B.DBF_ESHAPE


def test_pack_without_gpu_reports_hip_error():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present; covered by the gpu tests")
    L = _small_operands()
    with pytest.raises(B.DbfError) as e:
        B.dbf_pack_bits(40, 24, 33, L.A_bits, L.B_bits, L.a, L.m, L.b)
    assert e.value.code == B.DBF_EHIP


def test_second_workload_middle_sizes_follow_the_storage_formula():
    """The Table-4 shapes of the input recipe take k = floor(bits n m / (n + m)) (section 3, "Middle
    dimension size"): checked against the oracle's own formula, and k is the largest size within the budget."""
    from oracle import dbf_oracle as O
    from paper_2505_11076_amd import inputs as I
    cfgs = I.table4_configs()
    assert len(cfgs) == 20
    for cfg in cfgs:
        n, m, k = cfg["n_out"], cfg["n_in"], cfg["k"]
        assert k == O.middle_dim_for_bits(cfg["bits"], n, m)
        assert O.bits_per_weight(n, m, k) <= cfg["bits"] < O.bits_per_weight(n, m, k + 1)
    # (the sizes the pruning benchmark cuts the prefill shapes down to, and those of the 224-layer stack: 1.5 bits)
    for (n, m), k in I.CONFIG4_PRUNED_K.items():
        assert k == O.middle_dim_for_bits(1.5, n, m)
    assert {(c["n_out"], c["n_in"], c["k"]) for c in I.llama2_7b_stack_shapes(1)} == {
        (n, m, O.middle_dim_for_bits(1.5, n, m)) for (n, m) in ((4096, 4096), (11008, 4096), (4096, 11008))}


def test_bench_refuses_more_than_one_gpu():
    """The path uses no collectives: bench.py --gpus N with N > 1 must exit with a message, before it
    touches a GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert res.returncode == 2
    assert "one GPU" in res.stderr and res.stdout.strip() == ""


def test_tuning_hooks_have_defaults_ranges_and_a_reset():
    """The tuning / test hooks of the header: defaults as documented, values outside the stated range and
    unknown knobs are refused, reset restores the defaults.  (No GPU involved.)"""
    lib = B.lib()
    B.dbf_tuning_reset()
    defaults = {B.TUNE_COL_PIECES: -1, B.TUNE_PIECE_TARGET: 0, B.TUNE_PIECE_MIN_TILES: 24, B.TUNE_PIECE_NEVER_TILES: 64,
                B.TUNE_PIECE_MAX_ROW_TILES: 768, B.TUNE_STACK_SPAN_B: 0, B.TUNE_STACK_SPAN_A: 0, B.TUNE_SHARED_Q: -1,
                B.TUNE_SHARED_MIN_BATCH: 2, B.TUNE_SHARED_LDS_KB: 52, B.TUNE_WAIT_LIMIT_US: 250000,
                B.TUNE_LONG_ROWS: -1, B.TUNE_GEMM_SPLITS: -1, B.TUNE_FUSED_MIN_B_ITEMS: 1024,
                B.TUNE_WIDE_WG_MAX_ITEMS: 256, B.TUNE_FP4_MAX_ITEMS: 256}
    assert len(defaults) == 16
    for knob, val in defaults.items():
        assert B.dbf_tuning_get(knob) == val
    for knob, bad in ((B.TUNE_COL_PIECES, -2), (B.TUNE_COL_PIECES, 65), (B.TUNE_STACK_SPAN_B, 17), (B.TUNE_SHARED_Q, 4),
                      (B.TUNE_SHARED_MIN_BATCH, 0), (B.TUNE_SHARED_LDS_KB, 65), (B.TUNE_WAIT_LIMIT_US, -1),
                      (B.TUNE_PIECE_MIN_TILES, 0), (B.TUNE_LONG_ROWS, 2), (B.TUNE_GEMM_SPLITS, 1025), (B.TUNE_GEMM_SPLITS, -2), (B.TUNE_FUSED_MIN_B_ITEMS, -1), (B.TUNE_WIDE_WG_MAX_ITEMS, -1), (B.TUNE_FP4_MAX_ITEMS, -1), (16, 0), (-1, 0)):
        assert lib.dbf_tuning_set(knob, bad) == B.DBF_EINVAL
    assert B.dbf_tuning_get(16) == -2 ** 31 and B.dbf_tuning_get(-1) == -2 ** 31
    B.dbf_tuning_set(B.TUNE_WAIT_LIMIT_US, 0)
    B.dbf_tuning_set(B.TUNE_COL_PIECES, 3)
    assert B.dbf_tuning_get(B.TUNE_WAIT_LIMIT_US) == 0 and B.dbf_tuning_get(B.TUNE_COL_PIECES) == 3
    B.dbf_tuning_reset()
    for knob, val in defaults.items():
        assert B.dbf_tuning_get(knob) == val


def test_the_library_reads_no_environment_variables():
    """Plans and launches are steered by the documented hooks only: no getenv in the product sources."""
    csrc = os.path.join(ROOT, "paper_2505_11076_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name)) as fh:
            assert "getenv" not in fh.read(), name


def test_host_code_is_clean_under_address_and_undefined_behaviour_sanitizers():
    """The host packer / tile layout and the argument-validation paths of the C ABI, built with
    -fsanitize=address,undefined (host code only) and exercised on exact-size heap buffers by
    tests/sanitize_host.cpp: any out-of-bounds access, bad shift or misaligned access in the host code
    ends that program with a report and a non-zero status."""
    import subprocess
    from paper_2505_11076_amd import build as _build
    exe = _build.build_sanitize_check(os.path.join(ROOT, "tests", "sanitize_host.cpp"))
    env = dict(os.environ)
    # (leak checking off: the HIP runtime keeps process-lifetime allocations; link order: other preloaded
    # libraries may come first)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "sanitize_host: ok" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr


def test_build_refuses_ring_slots_with_two_register_homes():
    """A slot of the hand-issued tile ring must keep one set of registers: with two, the compiler copies between them
    at loop ends while the slot's load is in flight (wrong sums, no fault).  The build counts the destination register
    sets of the ring's loads per kernel in the assembly; this checks the counter on a kernel with four homes for four
    slots, on one with five, and on one whose operand travels in the ring (four tile and four operand slots)."""
    from paper_2505_11076_amd import build as Bd

    def kernel(args, sets):
        loads = "".join("\tbuffer_load_dwordx4 %s, v1, s[28:31], 0 offen nt\n" % r for r in sets)
        return "_ZN12_GLOBAL__N_121dbf_items_mfma_kernelI%sEEvPK7DbfItemPyiiPKtPtiii:\n%s\ts_endpgm\n" % (args, loads + loads)

    four = ["v[2:5]", "v[6:9]", "v[10:13]", "v[14:17]"]
    ok = kernel("Li1ELb0ELi0ELb1ELi4ELb0", four) + kernel("Li1ELb0ELi2ELb0ELi4ELb0", four + ["v[18:21]", "v[22:25]", "v[26:29]", "v[30:33]"])
    assert Bd._ring_homes_report(ok, 4, 4) == (2, [])
    seen, bad = Bd._ring_homes_report(ok + kernel("Li1ELb0ELi0ELb0ELi4ELb0", four + ["v[54:57]"]), 4, 4)
    assert seen == 3 and len(bad) == 1 and "5 register sets for 4 ring slots" in bad[0]
    assert Bd._ring_homes_report("nothing here", 4, 4) == (0, [])


def test_build_refuses_spills_in_kernels_with_hand_issued_loads():
    """Kernels that issue loads by inline assembly must be built without spilled vector registers (an in-flight
    load would land in a register the compiler has already reused: a GPU memory fault).  The build reads the
    compiler's resource report; this checks the reader on a report with and without spills."""
    from paper_2505_11076_amd import build as Bd
    ok = ("x.hip:1:1: remark: Function Name: _ZN1a21dbf_items_mfma_kernelILi1EEEvv [-Rpass-analysis=kernel-resource-usage]\n"
          "x.hip:1:1: remark:     VGPRs: 109 [-Rpass-analysis=kernel-resource-usage]\n"
          "x.hip:1:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]\n"
          "x.hip:1:1: remark: Function Name: _ZN1a26dbf_quantise_inputs_kernelILb1EEEvv [-Rpass-analysis=kernel-resource-usage]\n"
          "x.hip:1:1: remark:     VGPRs Spill: 7 [-Rpass-analysis=kernel-resource-usage]\n")
    Bd._check_no_spills("dbf_gemv_mfma.hip", ok)   # (a kernel without hand-issued loads may spill)
    bad = ok.replace("VGPRs Spill: 0", "VGPRs Spill: 12")
    with pytest.raises(RuntimeError, match="12 spilled vector registers"):
        Bd._check_no_spills("dbf_gemv_mfma.hip", bad)
    assert set(Bd.NO_SPILL) == {"dbf_gemv_mfma.hip", "dbf_gemm_i8.hip"}
