"""Host-side check of a hardware rule the hand-written DPP multiply-adds rely on.

gfx9-family hardware needs two wait states between a VALU write of a VGPR and a DPP read
of the same VGPR.  The compiler enforces that for its own instructions but cannot look
inside inline asm, so this test compiles the small-matrix kernels to ISA text (no GPU
needed) and checks the spacing for every DPP instruction in it.
"""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _functions(text):
    """name -> instruction list; a branch target stays in the list as its label text ('.LBB0_3:')."""
    out = {}
    for f in re.split(r"\n(?=_Z\w+:)", text):
        m = re.match(r"(_Z\w+):", f)
        if not m:
            continue
        body = f.split("s_endpgm")[0]
        ins = []
        for l in body.split("\n")[1:]:
            l = l.split(";")[0].split("//")[0].strip()
            if not l or (l.startswith(".") and not l.endswith(":")):
                continue
            ins.append(l)
        out[m.group(1)] = ins
    return out


def _regs(tok):
    tok = tok.strip().lstrip("-|").rstrip("|,")
    m = re.match(r"v(\d+)$", tok)
    if m:
        return {int(m.group(1))}
    m = re.match(r"v\[(\d+):(\d+)\]$", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    return set()


def _wait_states(ins):
    if ins.split()[0] == "s_nop":
        return int(ins.split()[1], 0) + 1
    return 1


def _is_label(l):
    return l.endswith(":")


def find_hazards(text):
    """Two rules of the gfx9 family that nothing checks inside inline asm:
      * a VALU write of a VGPR needs two wait states before a DPP read of it;
      * a VALU write of EXEC (v_cmpx) needs five wait states before any DPP instruction.
    The instructions that can run before a DPP read are followed backwards through the control flow:
    at a branch target both the fall-through predecessor and every branch to that label are walked."""
    hazards, n_dpp = [], 0
    for name, ins in _functions(text).items():
        targets = {}
        for idx, l in enumerate(ins):
            if not _is_label(l) and l.split()[0].startswith(("s_cbranch", "s_branch")):
                targets.setdefault(l.split()[1] + ":", []).append(idx)

        def walk(j, ws, src, dpp, seen):
            """instructions before position j (exclusive), ws wait states already between them and the DPP read"""
            while j >= 0 and ws < 5:
                p = ins[j]
                if _is_label(p):
                    for b in targets.get(p, []):  # the branch itself is one wait state
                        if (b, ws) not in seen:
                            seen.add((b, ws))
                            walk(b - 1, ws + 1, src, dpp, seen)
                    j -= 1
                    if j >= 0 and not _is_label(ins[j]) and ins[j].split()[0] in ("s_branch", "s_setpc_b64"):
                        return  # no fall-through into the label
                    continue
                op = p.split()[0]
                if ws < 2 and op.startswith("v_") and not op.startswith("v_cmp"):
                    if _regs(p.split(None, 1)[1].split(",")[0]) & src:
                        hazards.append((name, p, dpp))
                if op.startswith("v_cmpx"):
                    hazards.append((name, p, dpp))
                ws += _wait_states(p)
                j -= 1

        for idx, l in enumerate(ins):
            if _is_label(l) or "_dpp" not in l.split()[0]:
                continue
            n_dpp += 1
            src = _regs(l.split(None, 1)[1].split(",")[1].split()[0])  # src0 is the DPP operand
            walk(idx - 1, 0, src, l, set())
    return hazards, n_dpp


def test_checker_sees_a_planted_hazard():
    bad = "_Zk:\n v_mul_f32_e32 v4, v1, v2\n s_nop 0\n v_fmac_f32_dpp v4, -v4, v9 row_newbcast:4 row_mask:0xf bank_mask:0xf\n s_endpgm\n"
    ok = "_Zk:\n v_mul_f32_e32 v4, v1, v2\n s_nop 1\n v_fmac_f32_dpp v4, -v4, v9 row_newbcast:4 row_mask:0xf bank_mask:0xf\n s_endpgm\n"
    assert len(find_hazards(bad)[0]) == 1
    assert find_hazards(ok) == ([], 1)


def test_checker_follows_branches_and_sees_an_exec_write_before_a_dpp_read():
    dpp = " v_fmac_f32_dpp v4, -v4, v9 row_newbcast:4 row_mask:0xf bank_mask:0xf\n s_endpgm\n"
    # the write sits in the block that falls through into the label
    fall = "_Zk:\n v_mul_f32_e32 v4, v1, v2\n.LBB0_2:\n" + dpp
    # the write is the last instruction before a branch to the label: one wait state (the branch) is not enough
    jump = "_Zk:\n v_mul_f32_e32 v4, v1, v2\n s_cbranch_scc1 .LBB0_2\n v_mov_b32_e32 v7, v1\n s_nop 4\n.LBB0_2:\n" + dpp
    # same, but the loop body writes another register last and the source two instructions earlier
    safe = "_Zk:\n v_mul_f32_e32 v4, v1, v2\n v_mov_b32_e32 v8, v1\n s_cbranch_scc1 .LBB0_2\n s_nop 4\n.LBB0_2:\n" + dpp
    # a loop: the back edge brings the write of the last iteration
    loop = "_Zk:\n s_nop 4\n.LBB0_2:\n" + dpp.replace(" s_endpgm\n", "") + " v_mul_f32_e32 v4, v1, v2\n s_cbranch_scc1 .LBB0_2\n s_endpgm\n"
    # an unconditional branch right before the label: nothing falls through
    nofall = "_Zk:\n s_cbranch_scc1 .LBB0_2\n v_mul_f32_e32 v4, v1, v2\n s_branch .LBB0_3\n.LBB0_2:\n" + dpp.replace(" s_endpgm\n", "") + ".LBB0_3:\n s_endpgm\n"
    assert len(find_hazards(fall)[0]) == 1
    assert len(find_hazards(jump)[0]) == 1
    assert find_hazards(safe) == ([], 1)
    assert len(find_hazards(loop)[0]) == 1
    assert find_hazards(nofall) == ([], 1)
    cmpx = "_Zk:\n v_cmpx_gt_f32_e32 v1, v2\n v_mov_b32_e32 v7, v1\n v_mov_b32_e32 v8, v1\n" + dpp
    cmpx_far = "_Zk:\n v_cmpx_gt_f32_e32 v1, v2\n s_nop 4\n" + dpp
    assert len(find_hazards(cmpx)[0]) == 1
    assert find_hazards(cmpx_far) == ([], 1)


def _compile_isa(name):
    from paper_1710_08717_amd import build

    src = os.path.join(build.CSRC, name)
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "out.s")
        cmd = ["hipcc", *build.FLAGS, "--cuda-device-only", "-S", "-o", out, src]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            return None, r.stderr[-2000:]
        return open(out).read(), ""


_ISA_FILES = ["leaf.hip", "tiny.hip", "tiny_ops.hip", "kalman.hip", "trsm_stream.hip", "tiny_rows.hip"]
_isa_cache = {}


def _isa_text(name):
    """ISA text of one source; all four files with hand-written DPP are compiled side by side on first use."""
    if not _isa_cache:
        from concurrent.futures import ThreadPoolExecutor

        with ThreadPoolExecutor(max_workers=6) as ex:
            for f, res in zip(_ISA_FILES, ex.map(_compile_isa, _ISA_FILES)):
                _isa_cache[f] = res
    text, err = _isa_cache[name]
    if text is None:
        pytest.fail("hipcc -S failed:\n" + err)
    return text


def test_checker_handles_64_bit_operands():
    bad = "_Zk:\n v_fma_f64 v[4:5], v[0:1], v[2:3], v[4:5]\n v_fmac_f64_dpp v[8:9], -v[4:5], v[6:7] row_newbcast:4 row_mask:0xf bank_mask:0xf\n s_endpgm\n"
    ok = "_Zk:\n v_fma_f64 v[4:5], v[0:1], v[2:3], v[4:5]\n s_nop 1\n v_fmac_f64_dpp v[8:9], -v[4:5], v[6:7] row_newbcast:4 row_mask:0xf bank_mask:0xf\n s_endpgm\n"
    assert len(find_hazards(bad)[0]) == 1
    assert find_hazards(ok) == ([], 1)


def test_diagonal_block_leaf_respects_dpp_spacing():
    text = _isa_text("leaf.hip")
    hazards, n_dpp = find_hazards(text)
    # per element type two inlined copies of the 16 x 16 factor-and-invert routine, 192 broadcast
    # multiply-adds each
    assert text.count("v_fmac_f32_dpp") >= 384
    assert text.count("v_fmac_f64_dpp") >= 384
    assert n_dpp >= 768
    assert hazards == []


def test_small_matrix_kernels_respect_dpp_spacing():
    text = _isa_text("tiny.hip")
    hazards, n_dpp = find_hazards(text)
    assert n_dpp > 600  # the fused v_fmac_f32_dpp of the fp32 16-lane kernels are really there
    assert text.count("v_fmac_f32_dpp") >= 600
    assert hazards == []


def test_small_matrix_operator_kernels_respect_dpp_spacing():
    text = _isa_text("tiny_ops.hip")
    hazards, n_dpp = find_hazards(text)
    # trsm / trmm, syrk and outer products, gemm2, syrk backward, potri in 4, 8 and 16 lanes per matrix
    assert text.count("v_fmac_f32_dpp") >= 2000
    assert text.count("v_fmac_f64_dpp") >= 1000
    assert hazards == []


def test_kalman_filter_kernel_respects_dpp_spacing():
    text = _isa_text("kalman.hip")
    hazards, n_dpp = find_hazards(text)
    # nine 16 x 16 products of 256 broadcast multiply-adds each per step and element type, plus the solves
    assert text.count("v_fmac_f32_dpp") >= 2000
    assert text.count("v_fmac_f64_dpp") >= 2000
    assert hazards == []


def test_streamed_solve_kernel_respects_dpp_spacing():
    text = _isa_text("trsm_stream.hip")
    hazards, n_dpp = find_hazards(text)
    assert n_dpp >= 100  # the in-register inverses of the diagonal tiles, per element type and row slot
    assert hazards == []


def test_two_rows_per_lane_operator_kernels_respect_dpp_spacing():
    text = _isa_text("tiny_rows.hip")
    hazards, n_dpp = find_hazards(text)
    assert text.count("v_fmac_f32_dpp") >= 1000 and text.count("v_fmac_f64_dpp") >= 1000
    assert hazards == []
