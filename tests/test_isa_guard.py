"""Guard on the generated code of the two dominant kernels (y = x W_eff^T and dx = dy W_eff on 256x256 tiles).

Their main loop uses all 512 vector registers of a lane (256 accumulators, the double-buffered fragments, the
load offsets), and the instruction order inside it is fixed by hand.  A harmless-looking change elsewhere in the
kernel can tip the register allocator into moving the accumulators between the two register files, or into
spilling, inside that loop: every result stays correct and the kernel runs 40 % slower.  No parity test sees that,
so this one compiles the kernel source to assembly (own source, device code only) and checks the loop blocks.
Needs hipcc, not a GPU; takes about a minute."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

KERNELS = {
    # the variants for contractions of whole k-tiles (plain loads) and the general ones (masked loads)
    "gemm_y  <256,256,bf16,A rows x K, B rows x K, whole k-tiles>": "nt_gemm_kernelILi256ELi256ELi0ELb0ELb0ELi2ELb1E",
    "gemm_dx <256,256,bf16,A rows x K, B K x rows, whole k-tiles>": "nt_gemm_kernelILi256ELi256ELi0ELb0ELb1ELi2ELb1E",
    "gemm_y  <256,256,bf16,A rows x K, B rows x K>": "nt_gemm_kernelILi256ELi256ELi0ELb0ELb0ELi2ELb0E",
    "gemm_dx <256,256,bf16,A rows x K, B K x rows>": "nt_gemm_kernelILi256ELi256ELi0ELb0ELb1ELi2ELb0E",
}


@pytest.fixture(scope="module")
def assembly(tmp_path_factory):
    from paper_2405_16528_amd import build as B
    out = tmp_path_factory.mktemp("isa") / "gemm_nt.s"
    flags = [f for f in B.FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [B.hipcc(), *flags, "-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"),
           os.path.join(B.PKG, "csrc", "gemm_nt.hip"), "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    return out.read_text()


def _loop_blocks(asm, mangled_part):
    start = asm.index(mangled_part)
    start = asm.index("\n", start)
    body = asm[start:asm.index(".Lfunc_end", start)]  # (a function may hold more than one s_endpgm)
    blocks, label, lines = [], "entry", []
    for line in body.split("\n"):
        if re.match(r"^\.LBB\d+_\d+:", line):
            blocks.append((label, lines))
            label, lines = line, []
        else:
            lines.append(line)
    blocks.append((label, lines))
    # LLVM marks the blocks of a loop in the label's comment
    return [(lab, ls) for (lab, ls) in blocks if "Loop" in lab and any("v_mfma" in x for x in ls)]


@pytest.mark.parametrize("name", list(KERNELS))
def test_main_loop_has_no_register_file_traffic(assembly, name):
    loops = _loop_blocks(assembly, KERNELS[name])
    assert loops, "main loop not found"
    text = [x for (_, ls) in loops for x in ls]
    n_mfma = sum("v_mfma_f32_16x16x32_bf16" in x for x in text)
    assert n_mfma == 128, f"{name}: {n_mfma} MFMAs in the loop blocks, expected the 128 of one k-tile"
    moved = [x.strip() for x in text if "v_accvgpr" in x]
    assert not moved, f"{name}: accumulators moved between register files inside the loop: {moved[:3]} ..."
    spilled = [x.strip() for x in text if "scratch_" in x]
    assert not spilled, f"{name}: spills inside the loop: {spilled[:3]} ..."
    # the k-tile's memory instructions: 32 fragment reads (twice as many when B is read transposed) and 16 loads
    n_loads = sum("global_load_lds_dwordx4" in x for x in text)
    assert n_loads == 16, f"{name}: {n_loads} direct loads in the loop blocks, expected 16"
    # M0 is written by the hand-written load sequence only (it cannot be declared as a clobber): every write of M0 in
    # the loop is the s_mov of that sequence, directly followed by the EXEC set-up and the load it serves
    for i, x in enumerate(text):
        if re.search(r"\bm0\b", x) and "s_mov_b32 m0" not in x:
            raise AssertionError(f"{name}: M0 used outside the direct-load sequence: {x.strip()}")
        if "s_mov_b32 m0" in x:
            nxt = [y.strip() for y in text[i + 1:i + 4]]
            masked = nxt[0].startswith("s_mov_b32 exec_lo") and nxt[2].startswith("global_load_lds_dwordx4")
            plain = nxt[0].startswith("global_load_lds_dwordx4")
            assert masked or plain, (name, nxt)
