"""Host-side check of the generated instruction stream of attn_fwd128x2_kernel.

The stream is written by paper_2407_20485_amd/csrc/gen_attn_fwd128x2.py and assembled as is:
no compiler pass inserts the wait states that gfx950 does not interlock in hardware.  The
generator keeps the dependent instructions apart by construction; this test re-derives the
distances from the text of the stream, in fall-through order, and fails if a producer and a
consumer come closer than the margin used here (one instruction = at least one wait state,
`s_nop N` = N + 1).  Margins (at or above what the 8-pass matrix ops need):

  matrix op writes a register      -> vector / LDS / memory instruction reads or writes it : 12
  matrix op reads its accumulator  -> vector instruction overwrites it                     : 12
  vector op writes an AccVGPR      -> matrix op reads it as accumulator                    : 3
  transcendental writes a register -> next instruction must not read it                    : 1 between
  vector op writes a register      -> v_permlane32_swap reads it                           : 2 between
  scalar op writes M0              -> direct-to-LDS load                                   : 1 between

It also checks what the launch relies on: every register named lies inside the clobber list,
the matrix ops only accumulate in place (C == D) and never take a matrix-op result as A or B.
"""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GEN = os.path.join(ROOT, "paper_2407_20485_amd", "csrc", "gen_attn_fwd128x2.py")

REG = re.compile(r"\b([va])(\d+)\b|\b([va])\[(\d+):(\d+)\]")


def regs(text):
    out = set()
    for m in REG.finditer(text):
        if m.group(1):
            out.add((m.group(1), int(m.group(2))))
        else:
            out.update((m.group(3), i) for i in range(int(m.group(4)), int(m.group(5)) + 1))
    return out


def split_operands(line):
    op, _, rest = line.partition(" ")
    ops = [o.strip() for o in rest.split(",")] if rest else []
    return op, ops


@pytest.fixture(scope="module")
def stream(tmp_path_factory):
    path = tmp_path_factory.mktemp("gen") / "body.inc"
    subprocess.run([sys.executable, GEN, str(path)], check=True, capture_output=True)
    text = path.read_text()
    lines = re.findall(r'^\s+"([^"\\]*)\\n" \\$', text, flags=re.M)
    clob = re.search(r"#define A2SF_FWD128X2_CLOBBERS (.*)", text).group(1)
    return [ln.strip() for ln in lines if ln.strip() and not ln.strip().startswith(";")], clob


def classify(op):
    if op.startswith("v_mfma"):
        return "mfma"
    if op.startswith("v_"):
        return "valu"
    if op.startswith("ds_"):
        return "lds"
    if op.startswith("global_"):
        return "vmem"
    return "salu"


def reads_writes(line):
    """(registers read, registers written) of one instruction, operand text only."""
    op, ops = split_operands(line)
    kind = classify(op)
    if not ops or kind == "salu":
        return set(), set()
    if op.startswith("ds_read") or op.startswith("global_load_dword"):
        return regs(" ".join(ops[1:])), regs(ops[0])
    if op.startswith("ds_write") or op.startswith("global_store") or op.startswith("global_load_lds"):
        return regs(" ".join(ops)), set()
    if op == "v_permlane32_swap_b32":
        both = regs(" ".join(ops))
        return both, both
    if op.startswith("v_cmp"):
        return regs(" ".join(ops[1:])), set()
    return regs(" ".join(ops[1:])), regs(ops[0])


def hazards(lines):
    last_mfma_write, last_mfma_cread, last_valu_awrite, last_valu_write = {}, {}, {}, {}
    prev_trans_dst, clock, m0_written_at = set(), 0, -10
    problems = []
    for ln in lines:
        if ln.endswith(":"):
            continue
        op, ops = split_operands(ln)
        kind = classify(op)
        r, w = reads_writes(ln)
        if kind == "mfma":
            d, a, b, c = ops[0], ops[1], ops[2], ops[3]
            assert c == d or c == "0", f"matrix op does not accumulate in place: {ln}"
            for reg in regs(a) | regs(b):
                if clock - last_mfma_write.get(reg, -100) < 12:
                    problems.append(f"matrix-op result used as A/B too early: {ln}")
            for reg in regs(c):
                if reg[0] == "a" and clock - last_valu_awrite.get(reg, -100) < 3:
                    problems.append(f"accumulator written by a vector op right before: {ln}")
        else:
            if kind in ("valu", "lds", "vmem"):
                for reg in r | w:
                    if clock - last_mfma_write.get(reg, -100) < 12:
                        problems.append(f"reads/writes a matrix-op result after {clock - last_mfma_write[reg]} states: {ln}")
            if kind == "valu":
                for reg in w:
                    if clock - last_mfma_cread.get(reg, -100) < 12:
                        problems.append(f"overwrites an accumulator a matrix op is still reading: {ln}")
        if r & prev_trans_dst:
            problems.append(f"consumes a transcendental result in the next instruction: {ln}")
        if op == "v_permlane32_swap_b32":
            for reg in r:
                if clock - last_valu_write.get(reg, -100) < 3:
                    problems.append(f"v_permlane32_swap right after a vector write: {ln}")
        if op.startswith("global_load_lds") and clock - m0_written_at < 2:
            problems.append(f"direct-to-LDS load right after the M0 write: {ln}")
        # ---- bookkeeping
        if kind == "mfma":
            for reg in regs(ops[0]):
                last_mfma_write[reg] = clock
            if ops[3] != "0":
                for reg in regs(ops[3]):
                    last_mfma_cread[reg] = clock
        elif kind == "valu":
            for reg in w:
                last_valu_write[reg] = clock
                if reg[0] == "a":
                    last_valu_awrite[reg] = clock
        prev_trans_dst = w if op in ("v_exp_f32", "v_log_f32", "v_rcp_f32") else set()
        if kind == "salu" and ops and ops[0] == "m0":
            m0_written_at = clock
        clock += int(ops[0]) + 1 if op == "s_nop" else 1
    return problems


def test_stream_hazard_distances(stream):
    lines, _ = stream
    problems = hazards(lines)
    assert not problems, "\n".join(problems[:20])


@pytest.mark.parametrize("bad", [
    ["v_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], 0", "s_nop 7", "v_add_f32 v40, v3, v41"],
    ["v_mfma_f32_32x32x16_bf16 a[0:15], v[16:19], v[20:23], a[0:15]", "s_nop 3", "v_accvgpr_read_b32 v40, a7"],
    ["v_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], v[0:15]", "v_mov_b32 v9, v40"],
    ["v_accvgpr_write_b32 a3, v40", "v_mfma_f32_32x32x16_bf16 a[0:15], v[16:19], v[20:23], a[0:15]"],
    ["v_exp_f32 v5, v5", "v_add_f32 v6, v6, v5"],
    ["v_mov_b32 v5, v6", "v_permlane32_swap_b32 v7, v5"],
    ["s_add_u32 m0, s60, 4096", "global_load_lds_dwordx4 v188, s[62:63]"],
    ["v_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], 0",
     "v_mfma_f32_32x32x16_bf16 v[32:47], v[0:3], v[20:23], 0"],
])
def test_checker_sees_planted_hazards(bad):
    assert hazards(bad)


def test_checker_accepts_spaced_stream():
    ok = ["v_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], 0", "s_nop 7", "s_nop 7",
          "v_add_f32 v40, v3, v41", "v_exp_f32 v5, v5", "v_mov_b32 v50, v51", "v_add_f32 v6, v6, v5",
          "s_add_u32 m0, s60, 4096", "s_nop 0", "global_load_lds_dwordx4 v188, s[62:63]"]
    assert not hazards(ok)


def test_stream_registers_are_declared(stream):
    lines, clob = stream
    declared = set(re.findall(r'"([vas]\d+)"', clob))
    used = set()
    for ln in lines:
        for kind, idx in regs(ln):
            used.add(f"{kind}{idx}")
        for m in re.finditer(r"\bs(\d+)\b|\bs\[(\d+):(\d+)\]", ln):
            if m.group(1):
                used.add(f"s{m.group(1)}")
            else:
                used.update(f"s{i}" for i in range(int(m.group(2)), int(m.group(3)) + 1))
    assert used <= declared, sorted(used - declared)[:10]


def test_stream_special_registers(stream):
    """Special registers the stream writes: vcc and scc are declared; exec is restored to all
    ones wherever it is narrowed; M0 is written before the direct-to-LDS loads and is left out of
    the clobber list on purpose (a reserved register: the compiler keeps nothing in it across a
    statement and rejects it in a clobber list).  Nothing else may appear as a destination."""
    lines, clob = stream
    named = set(re.findall(r'"([a-z0-9]+)"', clob))
    assert {"vcc", "scc", "memory"} <= named and "m0" not in named
    written = set()
    for ln in lines:
        op, ops = split_operands(ln)
        if not ops or op.startswith(("s_cmp", "s_cbranch", "s_branch", "s_waitcnt", "s_nop", "s_barrier")):
            continue
        if op.startswith("v_cmp") and not op.startswith("v_cmpx"):
            written.add(ops[0])
            continue
        if classify(op) == "salu":
            written.add(ops[0])
    special = {w for w in written if not re.match(r"^s\d+$|^s\[\d+:\d+\]$", w)}
    assert special <= {"m0", "vcc", "exec", "vcc_lo", "vcc_hi"}, sorted(special)
    if "exec" in special:     # every narrowing of exec is undone before the stream ends
        last = max(i for i, ln in enumerate(lines) if split_operands(ln)[1][:1] == ["exec"])
        assert lines[last].replace(" ", "") in ("s_mov_b64exec,-1",), lines[last]


def test_stream_barriers_are_wave_uniform(stream):
    """Every s_barrier sits in code all four waves of a workgroup run the same number of times:
    none may lie between a conditional branch on a per-wave quantity and its target.  The only
    per-wave branches are the ones on a block's last tile (targets Lspe / Lspo / Lfe / Lfo)
    and the out-of-line slow paths; the barriers are in the iteration tops, the prologue and
    the epilogue, which every wave passes once per tile / once."""
    lines, _ = stream
    assert sum(1 for ln in lines if ln == "s_barrier") >= 4
    in_slow = False
    for ln in lines:
        if ln.startswith("Lslow"):
            in_slow = True
        elif ln.startswith("s_branch Lback"):
            in_slow = False
        assert not (in_slow and ln == "s_barrier")


def test_stream_scc_consumers_see_their_producer(stream):
    """s_addc_u32 must read the carry of the s_add_u32 just before it, s_cbranch_scc* and
    s_cselect_* the result of an s_cmp_*: no other scalar op that writes SCC may have slipped in
    between when instruction lists were interleaved."""
    lines, _ = stream
    writes_scc = ("s_add", "s_sub", "s_and", "s_or", "s_xor", "s_lshl", "s_lshr", "s_min", "s_max", "s_cmp")
    last = None
    for ln in lines:
        if ln.endswith(":"):
            continue   # a label: control may arrive from a branch, whose producer was checked there
        op = ln.split()[0]
        if op == "s_addc_u32":
            assert last is not None and last.startswith("s_add_u32"), (last, ln)
        elif op.startswith("s_cbranch_scc") or op.startswith("s_cselect"):
            assert last is not None and last.startswith("s_cmp"), (last, ln)
        if op.startswith(writes_scc):
            last = ln
