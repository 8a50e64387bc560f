"""Host-side execution model of the generated instruction stream of attn_fwd128x2_kernel.

The stream (paper_2407_20485_amd/csrc/gen_attn_fwd128x2.py) is hand-scheduled: scalar code
steers a persistent loop over 256-row blocks, direct-to-LDS loads fill a ring of four stages,
`s_waitcnt vmcnt(N)` plus one barrier per tile publish the tiles, and nothing in hardware checks
any of it.  This test runs the scalar side of the stream for the four waves of a workgroup on
the CPU -- vector arithmetic is skipped, memory instructions are recorded -- and checks what a
mistake there would break:

  * every wave reaches the end, all four pass the same number of barriers (no deadlock);
  * every global access lies inside its tensor, and the K / V tile, Q rows, O rows and
    log-sum-exp rows it touches are the ones the block needs;
  * every LDS operand read sees the tile the schedule wants (phase X of tile t: K(t+1) and the
    first V(t) fragments; phase Y: V(t), then the first K(t+2) fragments), that tile's
    direct-to-LDS loads have been waited for by every wave before the barrier the reader
    passed last, and no wave may have started to overwrite it (a load issued in a barrier
    epoch <= the reader's is a race);
  * a block's Q rows have arrived before its first matrix op;
  * each output row of the workgroup's blocks is written exactly once.

The fast path of the softmax is taken unless a seeded coin sends the wave through the
out-of-line rescale path (which must come back to where it left).
"""
import os
import random
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GEN = os.path.join(ROOT, "paper_2407_20485_amd", "csrc", "gen_attn_fwd128x2.py")

QBASE, KBASE, VBASE, OBASE, LBASE = (i << 36 for i in range(1, 6))
RING = 4 * 32768
M32 = 0xFFFFFFFF


@pytest.fixture(scope="module")
def program(tmp_path_factory):
    path = tmp_path_factory.mktemp("gen") / "body.inc"
    subprocess.run([sys.executable, GEN, str(path)], check=True, capture_output=True)
    text = path.read_text()
    lines = [ln.strip() for ln in re.findall(r'^\s+"([^"\\]*)\\n" \\$', text, flags=re.M)]
    prog, labels = [], {}
    for ln in lines:
        if not ln:
            continue
        if ln.endswith(":"):
            labels[ln[:-1]] = len(prog)
        elif ln.startswith(";"):
            prog.append(("marker", ln))
        else:
            op, _, rest = ln.partition(" ")
            prog.append((op, [a.strip() for a in rest.split(",")] if rest else []))
    return prog, labels


class Wave:
    """One wave: scalar registers, the vmcnt queue, the recorded memory events."""

    def __init__(self, prog, labels, operands, wave, coin):
        self.prog, self.labels, self.ops, self.wave, self.coin = prog, labels, operands, wave, coin
        self.s = {}            # scalar registers (32-bit), "vcc" and "m0" as 64 / 32-bit values
        self.scc = 0
        self.toggle = {}       # bit 16 of the K / V fragment address registers
        self.pc = 0
        self.epoch = 0         # barriers passed
        self.vm = []           # outstanding vector-memory instructions, oldest first
        self.phase = "setup"
        self.dma, self.reads, self.stores, self.qloads, self.qevents = [], [], [], [], []
        self.steps = 0

    # ---- operand access
    def val(self, a):
        a = a.split()[0] if " " in a and not a.startswith("s[") else a
        if a.startswith("%["):
            return self.ops[a[2:-1]] & M32
        if a.startswith("s["):
            lo = int(a[2:a.index(":")])
            return (self.s.get(lo, 0) | (self.s.get(lo + 1, 0) << 32))
        if a.startswith("s") and a[1:].isdigit():
            return self.s.get(int(a[1:]), 0)
        if a in ("vcc", "m0", "exec"):
            return self.s.get(a, 0)
        return int(a, 0) & 0xFFFFFFFFFFFFFFFF

    def put(self, a, v):
        if a.startswith("s["):
            lo = int(a[2:a.index(":")])
            self.s[lo], self.s[lo + 1] = v & M32, (v >> 32) & M32
        elif a.startswith("s") and a[1:].isdigit():
            self.s[int(a[1:])] = v & M32
        else:
            self.s[a] = v

    # ---- run to the next barrier (True) or to the end (False)
    def run(self):
        prog = self.prog
        while self.pc < len(prog):
            op, a = prog[self.pc]
            self.pc += 1
            self.steps += 1
            assert self.steps < 4_000_000, "wave does not terminate"
            if op[0] == "v":
                if op.startswith("v_mfma") and self.phase == "block":
                    # the block's first matrix ops read the Q registers: their loads must be back
                    assert all(ev["retired"] is not None for ev in self.qevents), "Q rows still in flight"
                elif op.startswith("v_cmp") and a[0] == "vcc":
                    # data-dependent: the tile-sum test of the softmax decides by coin, the rest is quiet
                    self.s["vcc"] = 1 if (op == "v_cmp_nge_f32" and self.coin()) else 0
                elif op == "v_xor_b32" and a[1] == "0x10000":
                    self.toggle[a[0]] = self.toggle.get(a[0], 0) ^ 1
                elif op == "v_xor_b32" and a[2] in ("%[hx16]", "%[clvs16]"):
                    self.toggle[a[0]] = 0      # address register initialised at block start
                continue
            if op == "marker":
                m = re.match(r"; ---- (\w+)", a)
                self.phase = m.group(1)
                continue
            if op == "s_barrier":
                self.epoch += 1
                return True
            getattr(self, op)(a)
        return False

    # ---- scalar ALU
    def s_nop(self, a): pass
    def s_sleep(self, a): pass
    def s_mov_b32(self, a): self.put(a[0], self.val(a[1]) & M32)
    def s_mov_b64(self, a): self.put(a[0], self.val(a[1]) if a[1] != "-1" else (1 << 64) - 1)

    def s_add_u32(self, a):
        r = (self.val(a[1]) & M32) + (self.val(a[2]) & M32)
        self.scc = r >> 32
        self.put(a[0], r & M32)

    def s_addc_u32(self, a):
        r = (self.val(a[1]) & M32) + (self.val(a[2]) & M32) + self.scc
        self.scc = r >> 32
        self.put(a[0], r & M32)

    def s_sub_u32(self, a):
        x, y = self.val(a[1]) & M32, self.val(a[2]) & M32
        self.scc = 1 if y > x else 0
        self.put(a[0], (x - y) & M32)

    def s_mul_i32(self, a): self.put(a[0], (self.val(a[1]) * self.val(a[2])) & M32)
    def s_mul_hi_u32(self, a): self.put(a[0], ((self.val(a[1]) & M32) * (self.val(a[2]) & M32)) >> 32)

    def _logic(self, a, f, mask):
        r = f(self.val(a[1]), self.val(a[2])) & mask
        self.scc = 1 if r else 0
        self.put(a[0], r)

    def s_and_b32(self, a): self._logic(a, lambda x, y: x & y, M32)
    def s_and_b64(self, a): self._logic(a, lambda x, y: x & y, (1 << 64) - 1)
    def s_lshl_b32(self, a): self._logic(a, lambda x, y: x << (y & 31), M32)
    def s_lshr_b32(self, a): self._logic(a, lambda x, y: (x & M32) >> (y & 31), M32)
    def s_cmp_eq_u32(self, a): self.scc = int((self.val(a[0]) & M32) == (self.val(a[1]) & M32))
    def s_cmp_lt_u32(self, a): self.scc = int((self.val(a[0]) & M32) < (self.val(a[1]) & M32))
    def s_cmp_lg_u64(self, a): self.scc = int(self.val(a[0]) != self.val(a[1]))
    def s_cselect_b32(self, a): self.put(a[0], self.val(a[1]) if self.scc else self.val(a[2]))

    def s_cselect_b64(self, a):
        pick = a[1] if self.scc else a[2]
        self.put(a[0], (1 << 64) - 1 if pick == "-1" else self.val(pick))

    def s_branch(self, a): self.pc = self.labels[a[0]]

    def s_cbranch_scc0(self, a):
        if not self.scc:
            self.pc = self.labels[a[0]]

    def s_cbranch_scc1(self, a):
        if self.scc:
            self.pc = self.labels[a[0]]

    def s_waitcnt(self, a):
        m = re.search(r"vmcnt\((\d+)\)", " ".join(a))
        if m:
            keep = int(m.group(1))
            while len(self.vm) > keep:
                ev = self.vm.pop(0)
                if ev is not None:
                    ev["retired"] = self.epoch
    def s_memtime(self, a): pass

    # ---- memory
    @staticmethod
    def _offset(a):
        for x in a:
            m = re.search(r"offset:(-?\d+)", x)
            if m:
                return int(m.group(1))
        return 0

    def global_load_lds_dwordx4(self, a):
        # a[0]: per-lane offsets KL+u / VL+u = u * 4096 + [1024 wave, 1024 wave + 1024)
        u = (int(a[0][1:]) - 188) % 4
        off = self._offset(a)
        g0 = self.val(a[1].split()[0]) + off + u * 4096 + 1024 * self.wave
        l0 = (self.s["m0"] + off) & M32
        ev = {"wave": self.wave, "issued": self.epoch, "retired": None, "global": g0, "lds": l0}
        self.dma.append(ev)
        self.vm.append(ev)

    def global_load_dwordx4(self, a):
        self.qloads.append((self.val(a[2].split()[0]) + self._offset(a), self.s[50]))
        self.qevents.append({"retired": None})
        self.vm.append(self.qevents[-1])

    def global_store_dword(self, a):
        self.stores.append(("lse", self.val(a[2].split()[0]), 128))
        self.vm.append(None)

    def global_store_dwordx4(self, a):
        self.stores.append(("o", self.val(a[2].split()[0]) + self._offset(a), 1024))
        self.vm.append(None)

    def _ds_read(self, a, size):
        name = a[1].split()[0]
        reg = int(name[1:])
        if 176 <= reg < 184:
            kind = "K"
        elif 184 <= reg < 188:
            kind = "V"
        else:
            return                                    # the epilogue's private strip
        addr = (self.toggle.get(name, 0) << 16) + self._offset(a)
        self.reads.append({"wave": self.wave, "epoch": self.epoch, "kind": kind, "stage": addr >> 15,
                           "phase": self.phase, "t": self.s.get(44, 0), "round": self.s.get(50, 0)})

    def ds_read_b128(self, a): self._ds_read(a, 16)
    def ds_read_b64_tr_b16(self, a): self._ds_read(a, 8)
    def ds_write_b64(self, a): pass


def kv_division(r):
    """(kvs, kvm) operands for r query heads per K/V head, as the launcher forms them."""
    if r & (r - 1) == 0:
        return r.bit_length() - 1, 0
    return 31, (1 << 32) // r + 1


def run_workgroup(program, n, G, rounds, block_x, seed=None, kvr=1):
    """Runs one workgroup of a launch over G heads of n rows; returns its four waves."""
    prog, labels = program
    nqb = n // 256
    ids = G * nqb
    if rounds > 1:
        assert ids % 512 == 0 and ids // 256 == rounds and nqb & (nqb - 1) == 0
        vid0 = (block_x % 8) * (ids // 8) + block_x // 8
    else:
        vid0 = block_x
    rng = random.Random(seed)
    coin = (lambda: rng.random() < 0.15) if seed is not None else (lambda: False)
    waves = []
    for w in range(4):
        operands = dict(qlo=QBASE & M32, qhi=QBASE >> 32, klo=KBASE & M32, khi=KBASE >> 32,
                        vlo=VBASE & M32, vhi=VBASE >> 32, olo=OBASE & M32, ohi=OBASE >> 32,
                        llo=LBASE & M32, lhi=LBASE >> 32, n=n, g0=vid0 // nqb, qb0=nqb - 1 - vid0 % nqb,
                        vid0=vid0, rounds=rounds, lgnqb=nqb.bit_length() - 1, nqbm1=nqb - 1,
                        kvs=kv_division(kvr)[0], kvm=kv_division(kvr)[1],
                        w32a=32 * w, w32b=32 * (7 - w), wodd=w & 1, wave_lds=1024 * w, scale=0,
                        hx16=0, krow=0, clvs16=0, vrow=0, kl0=0, vl0=0, qoff=0, lv=0, l32x4=0,
                        lanex16=0, strip_w=0, x16=0, crr16=0, strip_r=0)
        waves.append(Wave(prog, labels, operands, w, coin))
    live = [True] * 4
    while any(live):
        live = [wv.run() for wv in waves]
        assert all(live) or not any(live), "the waves of a workgroup pass different numbers of barriers"
    return waves, vid0


def block_of(vid0, j, nqb):
    """(head, row block) of round j for the workgroup that starts at id vid0."""
    vid = vid0 + 32 * j
    pos = vid % nqb
    return vid // nqb, (pos if j & 1 else nqb - 1 - pos)


def check_workgroup(waves, vid0, n, G, rounds, kvr=1):
    nqb = n // 256
    blocks = [block_of(vid0, j, nqb) for j in range(rounds)]
    assert len({wv.epoch for wv in waves}) == 1
    # ---- direct-to-LDS loads: label every load with the tile it brings and the LDS slot it fills
    fills = {}   # (kind, stage) -> per wave, list of loads in issue order
    for wv in waves:
        for ev in wv.dma:
            for kind, base in (("K", KBASE), ("V", VBASE)):
                if base <= ev["global"] < base + -(-G // kvr) * n * 256:
                    rel = ev["global"] - base
                    head, inside = divmod(rel, n * 256)
                    tile, within = divmod(inside, 16384)
                    assert within % 4096 == 1024 * wv.wave and ev["global"] + 1024 <= base + -(-G // kvr) * n * 256
                    stage, slot = divmod(ev["lds"], 32768)
                    assert 0 <= ev["lds"] < RING, "direct-to-LDS load outside the stage ring"
                    assert (slot >= 16384) == (kind == "V") and slot % 16384 == within, (kind, slot, within)
                    ev.update(kind=kind, head=head, tile=tile, stage=stage)
                    fills.setdefault((kind, stage), {}).setdefault(wv.wave, []).append(ev)
                    break
            else:
                raise AssertionError(f"direct-to-LDS load from {ev['global']:#x}: outside K and V")
    # ---- operand reads
    for wv in waves:
        for rd in wv.reads:
            g, qb = blocks[rd["round"]]
            nt = 4 * qb + 4
            t = rd["t"]
            if rd["phase"] == "block":
                want = rd["stage"]                      # K(0) twice, then K(1)'s first fragments
                assert rd["kind"] == "K" and want in (0, 1)
            elif rd["phase"] == "X":
                want = t + 1 if rd["kind"] == "K" else t
            elif rd["phase"] == "Y":
                want = t if rd["kind"] == "V" else t + 2
            else:
                assert rd["phase"] == "final" and rd["kind"] == "V"
                want = t
            assert want % 4 == rd["stage"], (rd, want)
            head, tile = (g, want) if want < nt else blocks[min(rd["round"] + 1, rounds - 1)][:1] + (want - nt,)
            for w2 in range(4):
                mine = [ev for ev in fills[(rd["kind"], rd["stage"])][w2] if ev["issued"] <= rd["epoch"]]
                assert mine, (rd, "nothing fetched yet")
                last = mine[-1]
                if want >= nt and rd["round"] + 1 >= rounds:
                    continue        # run-ahead fragments past the last block: never used
                assert (last["head"], last["tile"]) == (head // kvr, tile), (rd, last)   # K/V head of the query head
                assert last["retired"] is not None and last["retired"] < rd["epoch"], (rd, last)
    # ---- Q rows, O rows, log-sum-exp rows
    for wv in waves:
        seen = {}
        for addr, j in wv.qloads:
            seen.setdefault(j, []).append(addr)
        written = {"o": [], "lse": []}
        for kind, addr, size in wv.stores:
            written[kind].append(addr)
        exp_o, exp_l, exp_q = [], [], {}
        for j, (g, qb) in enumerate(blocks):
            for b, first in ((0, 32 * wv.wave), (1, 32 * (7 - wv.wave))):
                row = g * n + 256 * qb + first
                exp_o += [OBASE + (row + 4 * u) * 256 for u in range(8)]
                exp_l.append(LBASE + row * 4)
                exp_q.setdefault(j, []).extend(QBASE + row * 256 + 32 * kk for kk in range(8))
        assert sorted(written["o"]) == sorted(exp_o)
        assert sorted(written["lse"]) == sorted(exp_l)
        # Q: setup loads round 0, each last tile loads the next round (the last one its own block again)
        loads = sorted(a for v in seen.values() for a in v)
        want_q = sorted(exp_q[0] + [a for j in range(rounds) for a in exp_q[min(j + 1, rounds - 1)]])
        assert loads == want_q


CASES = [  # n, G, rounds, workgroup
    (2048, 1, 1, 7), (2048, 1, 1, 0), (256, 2, 1, 1), (768, 1, 1, 2),
    (1024, 256, 4, 0), (1024, 256, 4, 37), (1024, 256, 4, 255),
    (512, 512, 4, 8), (512, 512, 4, 129), (2048, 128, 4, 64), (4096, 32, 2, 250),
]


@pytest.mark.parametrize("n,G,rounds,block_x", CASES)
def test_stream_model(program, n, G, rounds, block_x):
    waves, vid0 = run_workgroup(program, n, G, rounds, block_x)
    check_workgroup(waves, vid0, n, G, rounds)


@pytest.mark.parametrize("n,G,rounds,block_x,kvr", [(1024, 256, 4, 37, 4), (2048, 8, 1, 13, 8), (512, 512, 4, 129, 2),
                                                    (1024, 256, 4, 37, 7), (2048, 8, 1, 6, 3), (512, 512, 4, 250, 5),
                                                    (512, 512, 4, 129, 6)])
def test_stream_model_grouped_query_heads(program, n, G, rounds, block_x, kvr):
    """kvr query heads share a K/V head: Q rows, outputs and log-sum-exp rows go by the query
    head, every K/V tile by the K/V head query head / kvr (a shift for powers of two, a
    multiplication by the reciprocal otherwise)."""
    waves, vid0 = run_workgroup(program, n, G, rounds, block_x, kvr=kvr)
    check_workgroup(waves, vid0, n, G, rounds, kvr=kvr)


def test_reciprocal_division_is_exact():
    """mulhi(head, floor(2^32 / r) + 1) = head // r for every head a launch can have."""
    for r in (3, 5, 6, 7):
        kvs, kvm = kv_division(r)
        assert kvs == 31
        for head in list(range(0, 70000)) + [2 ** 24 - 1, 2 ** 24, 2 ** 27 + 12345, 2 ** 28 - 1]:
            assert ((head * kvm) >> 32) + (head >> kvs) == head // r, (r, head)


def test_model_catches_a_wrong_kv_head(program):
    """Planted mistake: the K/V head is taken to be the query head although four of them share one."""
    waves, vid0 = run_workgroup(program, 1024, 256, 4, 37, kvr=1)
    with pytest.raises(AssertionError):
        check_workgroup(waves, vid0, 1024, 256, 4, kvr=4)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_stream_model_with_rescale_paths(program, seed):
    """The out-of-line maximum / rescale paths are entered at random: control must come back to
    the instruction after the one that left, so everything above still holds."""
    waves, vid0 = run_workgroup(program, 1024, 256, 4, 5 * seed, seed=seed)
    check_workgroup(waves, vid0, 1024, 256, 4)


def test_model_catches_a_missing_wait(program):
    """Planted mistake: the waits at the tops of the iterations let one more tile group stay in
    flight than the schedule allows (one more V tile would in fact still be safe, one more K tile
    is not)."""
    prog, labels = program
    bad = [(op, ["vmcnt(16)"]) if op == "s_waitcnt" and a == ["vmcnt(8)"] else (op, a) for op, a in prog]
    waves, vid0 = run_workgroup((bad, labels), 2048, 1, 1, 7)
    with pytest.raises(AssertionError):
        check_workgroup(waves, vid0, 2048, 1, 1)


def test_model_catches_q_rows_in_flight(program):
    """Planted mistake: the wait at block start leaves the Q loads out as well as the stores."""
    prog, labels = program
    bad = [(op, ["vmcnt(34)"]) if op == "s_waitcnt" and a == ["vmcnt(18)"] else (op, a) for op, a in prog]
    with pytest.raises(AssertionError):
        run_workgroup((bad, labels), 1024, 256, 4, 3)


def test_model_catches_a_stale_pointer(program):
    """Planted mistake: a block of four tiles does not move its K stream on to the next block."""
    prog, labels = program
    bad = list(prog)
    hits = [i for i, (op, a) in enumerate(prog)
            if op == "s_cselect_b64" and prog[i - 1] == ("s_cmp_eq_u32", ["s46", "4"])]
    assert len(hits) == 1
    bad[hits[0]] = ("s_nop", ["0"])
    waves, vid0 = run_workgroup((bad, labels), 512, 512, 4, 8)
    with pytest.raises(AssertionError):
        check_workgroup(waves, vid0, 512, 512, 4)
