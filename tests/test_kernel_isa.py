"""Static checks on the generated gfx950 code of the slice GEMM and of the FP64 fallback GEMM (no GPU needed:
hipcc cross-compiles).

The kernel issues its tile transfers and epilogue stores from asm blocks whose base address is a
scalar register pair.  Inside an asm block the compiler does not insert the wait states the
hardware needs between a vector-ALU write of a scalar register (v_readlane / v_readfirstlane, e.g. a
register-allocator reload) and a memory instruction that reads it; a store issued too early uses the
stale register as its address.  These tests read the compiler's assembly of this repository's own
kernel and check that no such pair is closer than the required distance, and that the MFMA loop
itself is free of register spills."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_13778_amd", "csrc")
WAIT_STATES = 5


@pytest.fixture(scope="module")
def gemm_asm(tmp_path_factory):
    from paper_2511_13778_amd.build import FLAGS
    out = tmp_path_factory.mktemp("isa") / "oz_gemm_i8.s"
    cmd = ["hipcc", *FLAGS, "-S", "--cuda-device-only", os.path.join(CSRC, "oz_gemm_i8.hip"), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return [ln for ln in open(out).read().splitlines() if ln.strip() and not ln.strip().startswith(";")]


def test_asm_memory_ops_never_read_a_freshly_valu_written_scalar(gemm_asm):
    written = {}           # scalar register -> wait-state position of its last vector-ALU write
    pos = 0
    checked = 0
    for ln in gemm_asm:
        pos += 1
        t = ln.split()
        if t[0] in ("v_readlane_b32", "v_readfirstlane_b32"):
            written[t[1].rstrip(",")] = pos
        elif t[0] == "s_nop":
            pos += int(t[1])
        elif t[0] in ("global_store_dword", "global_load_lds_dwordx4"):
            m = re.search(r"s\[(\d+):(\d+)\]", ln)
            if not m:
                continue
            checked += 1
            for x in range(int(m.group(1)), int(m.group(2)) + 1):
                reg = "s%d" % x
                assert pos - written.get(reg, -10 ** 9) > WAIT_STATES, "%s read %d wait states after a vector-ALU write: %s" % (
                    reg, pos - written[reg], ln)
    assert checked > 100          # the kernel's transfers and stores were actually seen


def test_mfma_loop_has_no_spills(gemm_asm):
    # basic blocks (label to label) that hold the K-step MFMAs must not touch scratch memory
    block, blocks = [], []
    for ln in gemm_asm:
        if re.match(r"^\.LBB\d+_\d+:", ln):
            blocks.append(block)
            block = []
        block.append(ln)
    blocks.append(block)
    hot = [b for b in blocks if sum("v_mfma_i32_32x32x32_i8" in ln for ln in b) >= 8
           and any("global_load_lds" in ln or "ds_read_b128" in ln for ln in b)]
    assert hot
    for b in hot:
        assert not any("scratch_" in ln for ln in b)


@pytest.fixture(scope="module")
def dgemm_asm(tmp_path_factory):
    from paper_2511_13778_amd.build import FLAGS
    out = tmp_path_factory.mktemp("isa") / "oz_dgemm_f64.s"
    cmd = ["hipcc", *FLAGS, "-S", "--cuda-device-only", os.path.join(CSRC, "oz_dgemm_f64.hip"), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return [ln for ln in open(out).read().splitlines() if ln.strip() and not ln.strip().startswith(";")]


def _kernel_body(asm, mangled_prefix):
    start = next(i for i, ln in enumerate(asm) if ln.startswith(mangled_prefix) and ":" in ln)
    end = next(i for i in range(start, len(asm)) if asm[i].split()[0] == "s_endpgm")
    return asm[start:end]


@pytest.mark.parametrize("mode", [0, 1])
def test_fp64_gemm_k_loop_has_no_vector_address_arithmetic(dgemm_asm, mode):
    # The K loop of the FP64 fallback GEMM (128 x 128 tiles, interior and ragged modes) loads its tiles
    # through a buffer descriptor: 16 buffer loads and 64 MFMAs per K step, and no 64-bit vector adds.  With
    # plain pointer loads the compiler rebuilt sixteen 64-bit per-lane addresses in every K step, which
    # cost the matrix unit 4 % of its issue slots; this guards the code generation the speed depends on.
    body = _kernel_body(dgemm_asm, "_ZN2oz16dgemm_f64_kernelILb1ELb0ELi%dELi128EEE" % mode)
    block, blocks = [], []
    for ln in body:
        if re.match(r"^\.LBB\d+_\d+:", ln):
            blocks.append(block)
            block = []
        block.append(ln)
    blocks.append(block)
    # the K loop: the block that branches back to its own label (a peeled first K step may precede it);
    # what follows the back branch belongs to the code after the loop
    loops = []
    for b in blocks:
        label = b[0].split(":")[0] if b and b[0].startswith(".LBB") else None
        back = [i for i, ln in enumerate(b) if label and ln.split()[0].startswith("s_cbranch") and ln.split()[1] == label]
        if back:
            loops.append(b[:back[0] + 1])
    loops = [b for b in loops if sum("v_mfma_f64_16x16x4" in ln for ln in b) == 64]
    assert len(loops) == 1
    loop = loops[0]
    assert sum("buffer_load_dwordx2" in ln for ln in loop) == 16
    assert not any(ln.split()[0].startswith(("v_lshl_add_u64", "v_add_co_u32", "v_addc_co_u32", "global_load")) for ln in loop)
    assert not any("scratch_" in ln for ln in loop)
