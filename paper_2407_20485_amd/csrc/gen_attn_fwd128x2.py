#!/usr/bin/env python3
"""Writes attn_fwd128x2_body.inc: the gfx950 instruction stream of attn_fwd128x2_kernel.

The kernel computes the masked attention rows of the prompt (Section 1 and Section 3.1 Eq.3
of the paper) for d = 128 in bf16, 64 query rows per wave (two 32-row blocks, "block 0" and
"block 1") and 256 per workgroup, one wave per SIMD with the whole 512-register file.
Holding two query blocks per wave halves the LDS operand traffic per matrix op, which is
what bounds the one-block kernel; with a single wave per SIMD the overlap of matrix ops and
softmax arithmetic has to come from the instruction order inside the wave, and the register
file has to be laid out by hand (accumulators and Q in AccVGPRs), which is why the stream is
written out here instead of being left to the compiler.

Schedule for K/V tile t of 64 keys (S = logits, P = probabilities, O = output accumulator):

    phase X(t):  matrix ops  S0(t+1), S1(t+1) = K(t+1) Q^T       (one K fragment feeds both blocks)
                 vector ops  softmax of S1(t) -> P1(t)
    phase Y(t):  matrix ops  O0 += V(t)^T P0(t), O1 += V(t)^T P1(t)  (one V fragment feeds both)
                 vector ops  softmax of S0(t+1) -> P0(t+1)

so every phase pairs 32 matrix ops with one block's softmax, and nothing a phase's vector
ops touch is written by the matrix ops of the same phase (S1 and P0 are double-buffered; the
rare rescale of O by the running-maximum correction is deferred to the end of the phase).

K/V tiles arrive by global_load_lds DMA into a ring of four LDS stages; the barrier at the
top of iteration t publishes the tiles of iteration t+1, so fragment reads may run ahead
across phase and iteration boundaries.  A workgroup of the persistent launch works through
several 256-row blocks, and the tile stream runs on across them: the last four iterations of
a block fetch the first tiles of the next one, whose Q rows are loaded during the block's
last tile.

Hazards the hardware does not interlock are kept apart by construction: a vector op reads a
matrix-op result only after two later matrix ops have been issued plus explicit s_nop, a
transcendental result is never consumed by the next instruction, and M0 writes are followed
by s_nop before the DMA instruction.

Usage: python gen_attn_fwd128x2.py [output path]
"""
import os
import sys

PF = 4  # operand fragments in flight ahead of their matrix ops

# ---- vector registers ----------------------------------------------------------------
S0 = 0                  # logits of block 0 (32 registers: key sub-block 0, then 1)
S1 = (32, 64)           # logits of block 1, double-buffered by tile parity
P0 = (96, 112)          # bf16 probabilities of block 0, double-buffered
P1 = 128                # bf16 probabilities of block 1
RING = 144              # 8 operand fragments x 4 registers
KADDR = 176             # 8 LDS addresses of the K fragments (one per 16 d)
VADDR = 184             # 4 LDS addresses of the V fragments (one per 32 d)
KL = 188                # 4 per-lane global offsets of the K DMA
VL = 192                # 4 per-lane global offsets of the V DMA
M = (196, 197)          # running maximum (log2 units), per block
L = (198, 199)          # running sum, per block
CORR = (200, 201)       # correction factor of the last softmax, per block
MX, T1, T2, NEGINF = 202, 203, 204, 205
TMP = 206               # 16 temporaries
RS = 222                # sum of the current tile's probabilities (per lane)
NV = 230                # v0 .. v229 are used (and clobbered)
# ---- accumulation registers -----------------------------------------------------------
O = (0, 64)             # O^T accumulators: 4 blocks of 32 d x 16 registers each
Q = (128, 160)          # Q fragments: 8 x 4 registers each
NA = 192
# ---- scalar registers -----------------------------------------------------------------
KP, VP = 40, 42         # global pointers of the next K / V tile to fetch
T, TF0, NTMAX = 44, 45, 46   # iteration, block 0's last tile, tiles the workgroup streams
TF1 = 53                      # block 1's last tile
KJ, VJ = 47, 48         # index of the next K / V tile to fetch
FLAG = (56, 58)         # per block: all ones when the running maximum moved
FLAGO = (54, 66)        # per block: nonzero when O has to be rescaled (moved, and not from -inf)
ST0, ST1 = 60, 61
PAIR = 62               # scratch pair
OB = 64                 # output base pair
SHEAD, J, HASNEXT, SG, SQB = 49, 50, 51, 52, 69   # head * n (scratch), round, 1 if another block follows, head, row block
QW = (86, 88)           # Q row pointers of the two 32-row blocks
OW = (90, 92)           # O row pointers
LSEW = (94, 96)         # log-sum-exp pointers
KPN, VPN = 98, 82       # K / V pointers of the block after this one (this one again after the last)
SGN, SQBN = 84, 85      # its head and row block
SLO, SHI = 40, 99

STAGE = 32768           # one LDS stage: K tile (16 KB) then V tile (16 KB)
NSTAGE = 4


def v(n):
    return f"v{n}"


def vr(n, c):
    return f"v[{n}:{n + c - 1}]"


def ar(n, c):
    return f"a[{n}:{n + c - 1}]"


def sp(n):
    return f"s[{n}:{n + 1}]"


class Out:
    def __init__(self):
        self.lines = []
        self.far = []       # out-of-line code, appended after the main stream
        self.nlabel = 0

    def e(self, line):
        self.lines.append(line)

    def ext(self, lines):
        self.lines.extend(lines)

    def label(self, stem):
        self.nlabel += 1
        return f"L{stem}{self.nlabel}_%="


class Fifo:
    """Outstanding LDS reads, in issue order; they return in order."""

    def __init__(self, tags=()):
        self.q = list(tags)

    def push(self, tag):
        self.q.append(tag)

    def wait(self, tag):
        """Instruction that waits until every read tagged `tag` has returned."""
        idx = max(i for i, t in enumerate(self.q) if t == tag)
        left = len(self.q) - 1 - idx
        self.q = self.q[idx + 1:]
        assert left <= 15
        return f"s_waitcnt lgkmcnt({left})"


def slot(f):
    return RING + 4 * (f % 8)


# Tile j lives in LDS stage j % 4.  Bit 0 of the stage is known where the code is generated (the
# loop is unrolled by two) and goes into the instruction's immediate offset; bit 1 is bit 16 of
# the fragment address registers, toggled once every second iteration.
def k_read(f, odd):
    kk, kb = f >> 1, f & 1
    return [f"ds_read_b128 {vr(slot(f), 4)}, {v(KADDR + kk)} offset:{odd * STAGE + kb * 8192}"]


def v_read(j, odd):
    g, db = j >> 2, j & 3
    o = odd * STAGE + g * 4096
    return [f"ds_read_b64_tr_b16 {vr(slot(j), 2)}, {v(VADDR + db)} offset:{o}",
            f"ds_read_b64_tr_b16 {vr(slot(j) + 2, 2)}, {v(VADDR + db)} offset:{o + 2048}"]


def toggle(addr, count):
    return [f"v_xor_b32 {v(addr + i)}, 0x10000, {v(addr + i)}" for i in range(count)]


def mask_partial(base):
    """Causal mask of the 32 x 32 sub-block that holds the diagonal: local key
    8 (i/4) + 4 h + i%4 against local query l32, with %[lv] = l32 - 4 h."""
    out = []
    for i in range(16):
        c = 8 * (i >> 2) + (i & 3)
        out.append(f"v_cmp_gt_i32 vcc, {c}, %[lv]")
        out.append(f"v_cndmask_b32 {v(base + i)}, {v(base + i)}, {v(NEGINF)}, vcc")
    return out


def mask_full(base):
    return [f"v_mov_b32 {v(base + i)}, {v(NEGINF)}" for i in range(16)]


RESCALE_AT = 0x4e800000  # 2^30


def softmax(out, b, s, p):
    """Vector ops of one block's softmax over a 64-key tile, common case: the running maximum
    m is left alone and p = exp2(s * scale - m) is formed directly (logits in v[s..s+31] stay
    intact, bf16 probabilities go to v[p..p+15]).  Floating point keeps full relative
    precision while p stays far from overflow, so m only has to move when the tile's sum
    passes 2^30 (or is not a number, which is how the first tile, with m = -inf, announces
    itself); then the out-of-line slow path redoes the tile with a fresh maximum.  Returns
    (vector-op list, slow-path lines to be placed out of line)."""
    m, l, flag = M[b], L[b], FLAG[b]
    slow, back = out.label("slow"), out.label("back")
    t = [TMP + i for i in range(8)]
    o = [f"s_mov_b64 {sp(FLAGO[b])}, 0"]

    def fma(i):
        return f"v_fma_f32 {v(t[i % 8])}, {v(s + i)}, %[scale], -{v(m)}"

    def ex(i):
        return f"v_exp_f32 {v(t[i % 8])}, {v(t[i % 8])}"

    def add(i):
        if i == 0:
            return f"v_mov_b32 {v(RS)}, {v(t[0])}"
        return f"v_add_f32 {v(RS)}, {v(RS)}, {v(t[i % 8])}"

    def cvt(j):
        return f"v_cvt_pk_bf16_f32 {v(p + j)}, {v(t[(2 * j) % 8])}, {v(t[(2 * j + 1) % 8])}"

    # software-pipelined so that no instruction reads what the one before it wrote
    for i in range(34):
        if i < 32:
            o.append(fma(i))
        if 0 <= i - 1 < 32:
            o.append(ex(i - 1))
        if 0 <= i - 2 < 32:
            o.append(add(i - 2))
            if (i - 2) & 1:
                o.append(cvt((i - 2) // 2))
    o += [f"v_cmp_nge_f32 vcc, {RESCALE_AT:#x}, {v(RS)}",
          "s_cmp_lg_u64 vcc, 0",
          f"s_cbranch_scc1 {slow}",
          f"{back}:",
          f"v_add_f32 {v(l)}, {v(l)}, {v(RS)}"]
    far = [f"{slow}:"] + softmax_slow(b, s, p) + [f"v_mov_b32 {v(RS)}, 0", f"s_branch {back}"]
    return o, far


def softmax_slow(b, s, p):
    """One block's online softmax over a 64-key tile with a new running maximum: logits in
    v[s..s+31] become probabilities in place and, rounded to bf16, in v[p..p+15]; m, l and
    the correction factor are updated and the block's flag is raised."""
    m, l, corr, flag = M[b], L[b], CORR[b], FLAG[b]
    o = [f"v_max3_f32 {v(MX)}, {v(s)}, {v(s + 1)}, {v(s + 2)}"]
    for k in range(3, 31, 2):
        o.append(f"v_max3_f32 {v(MX)}, {v(MX)}, {v(s + k)}, {v(s + k + 1)}")
    o += [f"v_max_f32 {v(MX)}, {v(MX)}, {v(s + 31)}",
          f"v_mov_b32 {v(T1)}, {v(MX)}",
          "s_nop 1",
          f"v_permlane32_swap_b32 {v(MX)}, {v(T1)}",  # the two lanes of a query exchange halves
          "s_nop 1",
          f"v_max_f32 {v(MX)}, {v(MX)}, {v(T1)}",
          f"v_mul_f32 {v(MX)}, %[scale], {v(MX)}",
          f"v_max_f32 {v(MX)}, 0xf149f2ca, {v(MX)}",          # -1e30 floor
          f"v_add_f32 {v(T1)}, 0x41000000, {v(m)}",            # lazy rescale: only past m + 8
          f"v_cmp_gt_f32 vcc, {v(MX)}, {v(T1)}",
          "s_cmp_lg_u64 vcc, 0",
          f"s_cselect_b64 {sp(flag)}, -1, 0",
          f"v_cmp_lg_f32 vcc, {v(m)}, {v(NEGINF)}",            # O is still all zero on the first tile
          f"s_and_b64 {sp(FLAGO[b])}, vcc, {sp(flag)}",
          f"v_max_f32 {v(T1)}, {v(m)}, {v(MX)}",
          f"v_cndmask_b32 {v(T1)}, {v(m)}, {v(T1)}, {sp(flag)}",
          f"v_sub_f32 {v(T2)}, {v(m)}, {v(T1)}",
          f"v_exp_f32 {v(corr)}, {v(T2)}",
          f"v_mov_b32 {v(m)}, {v(T1)}",
          f"v_mul_f32 {v(l)}, {v(l)}, {v(corr)}"]

    def fma(i):
        return f"v_fma_f32 {v(s + i)}, {v(s + i)}, %[scale], -{v(m)}"

    def ex(i):
        return f"v_exp_f32 {v(s + i)}, {v(s + i)}"

    def add(i):
        return f"v_add_f32 {v(l)}, {v(l)}, {v(s + i)}"

    def cvt(j):
        return f"v_cvt_pk_bf16_f32 {v(p + j)}, {v(s + 2 * j)}, {v(s + 2 * j + 1)}"

    o += [fma(0), ex(0)]
    for i in range(1, 32):
        o += [fma(i), ex(i), add(i - 1)]
        if (i - 1) & 1:
            o.append(cvt((i - 1) // 2))
    o += ["s_nop 0", add(31), cvt(15)]
    return o


def rescale(out, b, settle):
    """O_b *= corr_b when block b's running maximum moved (rare after the first tiles)."""
    skip = out.label("nr")
    out.e(f"s_cmp_lg_u64 {sp(FLAGO[b])}, 0")
    out.e(f"s_cbranch_scc0 {skip}")
    if settle:
        out.ext(["s_nop 7", "s_nop 7", "s_nop 7"])
    for j in range(0, 64, 16):
        for k in range(16):
            out.e(f"v_accvgpr_read_b32 {v(TMP + k)}, a{O[b] + j + k}")
        for k in range(16):
            out.e(f"v_mul_f32 {v(TMP + k)}, {v(TMP + k)}, {v(CORR[b])}")
        for k in range(16):
            out.e(f"v_accvgpr_write_b32 a{O[b] + j + k}, {v(TMP + k)}")
    out.e("s_nop 7")
    out.e(f"{skip}:")


def merge(out, steps, valu, lead=0, lead_lines=()):
    """Interleave one phase: every matrix op is followed by its share of the vector-op list
    and by its share of the NEXT step's operand requests, so that the issue stream between
    two matrix ops is short and even (a lone wave issues about one instruction per 4.5
    cycles; a matrix op occupies its pipe for 32).  `lead` matrix ops are issued before any
    vector op (then `lead_lines`)."""
    mf = sum(len(s[2]) for s in steps)
    slots = max(mf - lead, 1)
    done_v, seen = 0, 0
    out.ext(steps[0][0])
    for k, (pre, wait, mfmas) in enumerate(steps):
        nxt = steps[k + 1][0] if k + 1 < len(steps) else []
        done_n = 0
        if wait:
            out.e(wait)
        for j, m in enumerate(mfmas):
            out.e(m)
            seen += 1
            if seen == lead:
                out.ext(lead_lines)
            if seen > lead or lead == 0:
                upto = (len(valu) * (seen - lead) + slots - 1) // slots
                out.ext(valu[done_v:upto])
                done_v = upto
            upto_n = (len(nxt) * (j + 1)) // len(mfmas)
            out.ext(nxt[done_n:upto_n])
            done_n = upto_n
    out.ext(valu[done_v:])


def qk_steps(fifo, s0, s1, odd, flip, next_reads, extra=None, blocks=(0, 1)):
    """Matrix side of S0, S1 = K Q^T over the 16 K fragments of a tile (fragments 0..PF-1
    already requested), two fragments = four matrix ops per step.  next_reads(i) = reads to
    request once the K reads ran out; extra[i] = further lines ahead of step i."""
    steps = []
    for f in range(0, 16, 2):
        pre = list((extra or {}).get(f // 2, []))
        for g in (f, f + 1):
            if g + PF < 16:
                pre += k_read(g + PF, odd)
                fifo.push(("K", g + PF))
            else:
                if g + PF == 16 and flip:
                    pre += toggle(KADDR, 8)
                pre += next_reads(g + PF - 16)
        wait = fifo.wait(("K", f + 1))
        mf = []
        for g in (f, f + 1):
            kk, kb = g >> 1, g & 1
            for b, sb in ((0, s0), (1, s1)):
                if b not in blocks:
                    continue
                d = vr(sb + 16 * kb, 16)
                c = "0" if kk == 0 else d
                mf.append(f"v_mfma_f32_32x32x16_bf16 {d}, {vr(slot(g), 4)}, {ar(Q[b] + 4 * kk, 4)}, {c}")
        steps.append((pre, wait, mf))
    return steps


def pv_steps(fifo, p0, p1, odd, flip, next_reads, blocks=(0, 1), extra=None):
    """Matrix side of O0, O1 += V^T P^T over the 16 V fragments of a tile."""
    steps = []
    for j in range(0, 16, 2):
        pre = list((extra or {}).get(j // 2, []))
        for i in (j, j + 1):
            if i + PF < 16:
                pre += v_read(i + PF, odd)
                fifo.push(("V", i + PF))
                fifo.push(("V", i + PF))
            else:
                if i + PF == 16 and flip:
                    pre += toggle(VADDR, 4)
                pre += next_reads(i + PF - 16)
        wait = fifo.wait(("V", j + 1))
        mf = []
        for i in (j, j + 1):
            g, db = i >> 2, i & 3
            for b, pb in ((0, p0), (1, p1)):
                if b not in blocks:
                    continue
                d = ar(O[b] + 16 * db, 16)
                mf.append(f"v_mfma_f32_32x32x16_bf16 {d}, {vr(slot(i), 4)}, {vr(pb + 4 * g, 4)}, {d}")
        steps.append((pre, wait, mf))
    return steps


def dma_lines(which):
    """Fetch of the next K (or V) tile into LDS stage (tile number) % NSTAGE.  The tile stream
    does not stop at the end of a 256-row block: after the block's last tile come the first
    tiles of the next block (pointer s[KPN] / s[VPN]), whose tile 0 falls on stage 0 again
    because a block always has a multiple of four tiles; so the fetch is the same instruction
    sequence in every iteration, the vmcnt bookkeeping is uniform and the next block finds its
    first tiles in LDS."""
    j, p, pn, lo, off = (KJ, KP, KPN, KL, 0) if which == "K" else (VJ, VP, VPN, VL, 16384)
    ln = [f"s_and_b32 s{ST1}, s{j}, {NSTAGE - 1}",
          f"s_lshl_b32 s{ST1}, s{ST1}, 15",
          f"s_add_u32 s{ST1}, s{ST1}, %[wave_lds]"]
    # the instruction's immediate offset moves the global and the LDS address alike, and the
    # four loads of a wave sit 4 KB apart in both: one M0 value serves two loads
    for u in (1, 3):
        ln += [f"s_add_u32 m0, s{ST1}, {off + u * 4096}", "s_nop 0",
               f"global_load_lds_dwordx4 {v(lo + u)}, {sp(p)} offset:-4096",
               f"global_load_lds_dwordx4 {v(lo + u)}, {sp(p)}"]
    ln += [f"s_add_u32 s{p}, s{p}, 16384", f"s_addc_u32 s{p + 1}, s{p + 1}, 0",
           f"s_add_u32 s{j}, s{j}, 1",
           f"s_cmp_eq_u32 s{j}, s{NTMAX}",
           f"s_cselect_b64 {sp(p)}, {sp(pn)}, {sp(p)}"]
    return ln


def dma_pieces(which):
    """The fetch of K(t+4) (phase X) / V(t+3) (phase Y), to ride between the phase's first
    matrix ops."""
    return {1: dma_lines(which)}


def dma(out, which):
    out.ext(dma_lines(which))


def top_drain(out):
    """Top of an iteration for a wave that has finished its rows: besides the newest tile
    group, the last tile's fetches and the next block's Q loads may stay in flight."""
    out.e(f"s_waitcnt vmcnt({8 + 8 + Q_LOADS})")
    out.e("s_barrier")
    dma(out, "K")
    dma(out, "V")


def top(out):
    """Top of iteration t: the group {K(t+2), V(t+1)} has landed for every wave (only the
    group fetched during iteration t-1 may still be in flight); the fetch of {K(t+4), V(t+3)},
    into the stages that held K(t) and V(t-1), follows inside the iteration."""
    out.e("s_waitcnt vmcnt(8)")
    out.e("s_barrier")


def k_prefetch_tags():
    return [("K", i) for i in range(PF)]


def mask_block(out, b, s):
    """Causal mask of block b's diagonal tile.  A block whose index inside the 256-row
    workgroup block is even starts a 64-key tile (first key sub-block partial, second fully
    masked); an odd one sits in the tile's second half (second sub-block partial).  Block 0
    of wave w has index w, block 1 index 7 - w."""
    up, done = out.label("mu"), out.label("md")
    return ([f"s_cmp_eq_u32 %[wodd], {b}", f"s_cbranch_scc0 {up}"]
            + mask_partial(s) + mask_full(s + 16) + [f"s_branch {done}", f"{up}:"]
            + mask_partial(s + 16) + [f"{done}:"])


def reader(fifo, kind, odd):
    def nxt(i):
        if kind == "K":
            fifo.push(("K", i))
            return k_read(i, odd)
        fifo.push(("V", i))
        fifo.push(("V", i))
        return v_read(i, odd)
    return nxt


def phase_x(out, fifo, par, blocks):
    """Matrix ops: logits of tile t+1 for `blocks` | vector ops: softmax of S1(t)."""
    out.e(f"; ---- X phase, parity {par}, blocks {blocks}")
    # K(t+1) now; K address bit 16 flips after the last read when t+2 has another bit 1 than t+1;
    # then the first V(t) fragments
    steps = qk_steps(fifo, S0, S1[1 - par], 1 - par, par == 0, reader(fifo, "V", par),
                     extra=dma_pieces("K"), blocks=blocks)
    valu, far = softmax(out, 1, S1[par], P1)
    out.far += far
    merge(out, steps, valu)
    rescale(out, 1, settle=False)


def phase_y(out, fifo, par, blocks, sm0):
    """Matrix ops: O += V(t)^T P(t) for `blocks` | vector ops: softmax of S0(t+1) (if sm0)."""
    out.e(f"; ---- Y phase, parity {par}, blocks {blocks}")
    # V(t) now, then the first K(t+2) fragments
    steps = pv_steps(fifo, P0[par], P1, par, par == 1, reader(fifo, "K", par), blocks=blocks,
                     extra=dma_pieces("V"))
    if not sm0:
        merge(out, steps, [])
        return
    nomask = out.label("nm")
    lead = (["s_nop 7", f"s_add_u32 s{ST0}, s{T}, 1", f"s_cmp_eq_u32 s{ST0}, s{TF0}",
             f"s_cbranch_scc0 {nomask}"] + mask_block(out, 0, S0) + [f"{nomask}:"])
    valu, far = softmax(out, 0, S0, P0[1 - par])
    out.far += far
    merge(out, steps, valu, lead=2, lead_lines=lead)
    rescale(out, 0, settle=True)


def iteration(out, par, kind):
    """Iteration t of parity par.  kind: "both" (t before block 0's last tile), "split" (t is
    block 0's last tile: its logits are complete, only its last O update remains), "one"
    (only block 1 is still running)."""
    fifo = Fifo(k_prefetch_tags())
    phase_x(out, fifo, par, (0, 1) if kind == "both" else (1,))
    phase_y(out, fifo, par, (1,) if kind == "one" else (0, 1), sm0=(kind == "both"))
    assert fifo.q == k_prefetch_tags()


def final(out, par):
    """Block 1's last tile (the one holding its diagonal): softmax of S1, then O1 += V^T P1."""
    out.e(f"; ---- final, parity {par}")
    dma(out, "K")
    dma(out, "V")
    # the Q registers are free from here on: the next block's Q rows are fetched between the
    # instructions of this last tile
    out.ext(next_block())
    out.e("s_waitcnt lgkmcnt(0)")
    out.ext(mask_block(out, 1, S1[par]))
    fifo = Fifo()
    pre = []
    for j in range(PF):
        pre += v_read(j, par)
        fifo.push(("V", j))
        fifo.push(("V", j))
    out.ext(pre)
    valu, far = softmax(out, 1, S1[par], P1)
    out.far += far
    out.ext(weave(valu, q_loads()))
    rescale(out, 1, settle=False)
    steps = pv_steps(fifo, P0[par], P1, par, False, lambda i: [], blocks=(1,))
    merge(out, steps, [])
    assert not fifo.q


def pointer(dst, base, t, shift):
    """s[dst:dst+1] = %[base_lo]:%[base_hi] + (s[t] << shift), s[t] < 2^31."""
    return [f"s_lshr_b32 s{OB}, s{t}, {32 - shift}", f"s_lshl_b32 s{OB + 1}, s{t}, {shift}",
            f"s_add_u32 s{dst}, %[{base}lo], s{OB + 1}", f"s_addc_u32 s{dst + 1}, %[{base}hi], s{OB}"]


def block_rows():
    """From head s[SG] and 256-row block s[SQB]: s[SHEAD] = head * n, s[ST0] = first row of the
    block, s[ST1] / s[PAIR] = head * n + first row of this wave's block 0 / block 1."""
    return [f"s_mul_i32 s{SHEAD}, s{SG}, %[n]",
            f"s_lshl_b32 s{ST0}, s{SQB}, 8",
            f"s_add_u32 s{ST1}, s{ST0}, %[w32a]", f"s_add_u32 s{PAIR}, s{ST0}, %[w32b]",
            f"s_add_u32 s{ST1}, s{ST1}, s{SHEAD}", f"s_add_u32 s{PAIR}, s{PAIR}, s{SHEAD}"]


Q_LOADS = 16   # memory instructions q_loads() issues
STORES = 18    # memory instructions the epilogue issues


def q_pointers():
    """Pointers of this wave's Q rows for the block (s[SG], s[SQB])."""
    return block_rows() + pointer(QW[0], "q", ST1, 8) + pointer(QW[1], "q", PAIR, 8)


def q_loads():
    """Q straight into the accumulation registers (B-operand fragments)."""
    return [f"global_load_dwordx4 {ar(Q[b] + 4 * kk, 4)}, %[qoff], {sp(QW[b])} offset:{kk * 32}"
            for b in (0, 1) for kk in range(8)]


def look_ahead():
    """s[SGN], s[SQBN] = the block of round s[J] + 1 (persistent launch: work id = vid0 + 32
    round, the row blocks of a head in turn from the long end and from the short end, so that
    two rounds together cost every workgroup the same) and s[HASNEXT] = 1; after the last round
    they are the current block again (whose first tiles are then simply fetched once more) and
    s[HASNEXT] = 0.  s[KPN], s[VPN] = that block's K and V."""
    return [f"s_add_u32 s{ST0}, s{J}, 1",
            f"s_lshl_b32 s{ST1}, s{ST0}, 5",
            f"s_add_u32 s{ST1}, s{ST1}, %[vid0]",
            f"s_lshr_b32 s{PAIR}, s{ST1}, %[lgnqb]",
            f"s_and_b32 s{ST1}, s{ST1}, %[nqbm1]",
            f"s_sub_u32 s{OB}, %[nqbm1], s{ST1}",
            f"s_and_b32 s{OB + 1}, s{ST0}, 1",
            f"s_cmp_eq_u32 s{OB + 1}, 1",                     # odd round: from the short end
            f"s_cselect_b32 s{ST1}, s{ST1}, s{OB}",
            f"s_cmp_lt_u32 s{ST0}, %[rounds]",
            f"s_cselect_b32 s{HASNEXT}, 1, 0",
            f"s_cselect_b32 s{SGN}, s{PAIR}, s{SG}",
            f"s_cselect_b32 s{SQBN}, s{ST1}, s{SQB}",
            ] + kv_head(SGN) + [
            f"s_mul_i32 s{SHEAD}, s{SHEAD}, %[n]"] + pointer(KPN, "k", SHEAD, 8) + pointer(VPN, "v", SHEAD, 8)


def kv_head(head):
    """s[SHEAD] = K/V head of query head s[head] = head / r for r query heads per K/V head
    (grouped-query heads): for r a power of two %[kvm] = 0 and %[kvs] = log2 r; otherwise
    %[kvs] = 31 (the shift gives 0) and %[kvm] = floor(2^32 / r) + 1, whose high product with the
    head is the quotient for every head below 2^32 / r.  s[OB] is scratch."""
    return [f"s_mul_hi_u32 s{SHEAD}, s{head}, %[kvm]",
            f"s_lshr_b32 s{OB}, s{head}, %[kvs]",
            f"s_add_u32 s{SHEAD}, s{SHEAD}, s{OB}"]


def next_block():
    """Scalar part of the early Q fetch: the next block becomes the current one."""
    return [f"s_mov_b32 s{SG}, s{SGN}", f"s_mov_b32 s{SQB}, s{SQBN}"] + q_pointers()


def weave(base, extra, tail=8):
    """`extra` spread evenly through `base`, none of it among the last `tail` lines."""
    body = base[:len(base) - tail]
    out, done = [], 0
    for i, ln in enumerate(body):
        out.append(ln)
        upto = (len(extra) * (i + 1)) // len(body)
        out += extra[done:upto]
        done = upto
    return out + base[len(base) - tail:]


def setup(out):
    """Once per launch: constants, the first block's Q and its first tiles."""
    out.e("; ---- setup")
    out.e(f"v_mov_b32 {v(NEGINF)}, 0xff800000")
    for u in range(4):
        out.e(f"v_add_u32 {v(KL + u)}, {u * 4096}, %[kl0]")
        out.e(f"v_add_u32 {v(VL + u)}, {u * 4096}, %[vl0]")
    out.e(f"s_mov_b32 s{J}, 0")
    out.e(f"s_mov_b32 s{SG}, %[g0]")
    out.e(f"s_mov_b32 s{SQB}, %[qb0]")
    out.ext(q_pointers() + q_loads())
    out.ext(kv_head(SG))
    out.e(f"s_mul_i32 s{SHEAD}, s{SHEAD}, %[n]")
    out.ext(pointer(KP, "k", SHEAD, 8) + pointer(VP, "v", SHEAD, 8))
    out.ext(look_ahead())
    out.e(f"s_lshl_b32 s{NTMAX}, s{SQB}, 2")
    out.e(f"s_add_u32 s{NTMAX}, s{NTMAX}, 4")
    out.e(f"s_mov_b32 s{KJ}, 0")
    out.e(f"s_mov_b32 s{VJ}, 0")
    for which in "KKVKVKV":
        dma(out, which)


def prologue(out):
    """Start of a 256-row block: its Q rows and its first tiles (K(0..3), V(0..2)) were
    requested during the block before (or by setup)."""
    out.e("; ---- block start")
    out.ext(block_rows())
    out.ext(pointer(OW[0], "o", ST1, 8) + pointer(OW[1], "o", PAIR, 8))
    out.ext(pointer(LSEW[0], "l", ST1, 2) + pointer(LSEW[1], "l", PAIR, 2))
    out.e(f"s_sub_u32 s{ST1}, s{ST1}, s{SHEAD}")
    out.e(f"s_sub_u32 s{PAIR}, s{PAIR}, s{SHEAD}")
    out.e(f"s_lshr_b32 s{TF0}, s{ST1}, 6")
    out.e(f"s_lshr_b32 s{TF1}, s{PAIR}, 6")
    out.e(f"s_lshr_b32 s{NTMAX}, s{ST0}, 6")
    out.e(f"s_add_u32 s{NTMAX}, s{NTMAX}, 4")
    out.e(f"s_mov_b32 s{T}, 0")
    out.e(f"s_mov_b32 s{KJ}, 4")      # K(0..3) and V(0..2) came with the tile stream
    out.e(f"s_mov_b32 s{VJ}, 3")
    out.ext(look_ahead())
    # a block of four tiles has nothing left to fetch for itself: its K stream moves on to the
    # next block right away (V still has tile 3 to go and switches in dma_lines)
    out.e(f"s_cmp_eq_u32 s{NTMAX}, 4")
    out.e(f"s_cselect_b64 {sp(KP)}, {sp(KPN)}, {sp(KP)}")
    for b in (0, 1):
        out.e(f"v_mov_b32 {v(M[b])}, {v(NEGINF)}")
        out.e(f"v_mov_b32 {v(L[b])}, 0")
    for kk in range(8):
        out.e(f"v_xor_b32 {v(KADDR + kk)}, {kk * 32}, %[hx16]")
        out.e(f"v_add_u32 {v(KADDR + kk)}, {v(KADDR + kk)}, %[krow]")
    for db in range(4):
        out.e(f"v_xor_b32 {v(VADDR + db)}, {db * 64}, %[clvs16]")
        out.e(f"v_add_u32 {v(VADDR + db)}, {v(VADDR + db)}, %[vrow]")
    for i in range(128):
        out.e(f"v_accvgpr_write_b32 a{i}, 0")
    # this block's Q rows (and, long before them, its first tiles) have arrived; only the last
    # block's output stores, which were issued after them, may still be under way
    out.e(f"s_waitcnt vmcnt({STORES})")
    out.e("s_barrier")             # also: every wave has left the last block's tiles
    # S0(0), then S1(0) with block 0's first softmax (the one that has to find a maximum)
    # riding between its matrix ops.  K(0)'s fragments are read once per pass, i.e. twice per
    # block, here: LDS is idle anyway.
    fifo = Fifo()
    for f in range(PF):
        out.ext(k_read(f, 0))
        fifo.push(("K", f))
    merge(out, qk_steps(fifo, S0, S1[0], 0, False, reader(fifo, "K", 0), blocks=(0,)), [])
    nomask = out.label("nm")
    lead = (["s_nop 7", f"s_cmp_eq_u32 s{TF0}, 0", f"s_cbranch_scc0 {nomask}"]
            + mask_block(out, 0, S0) + [f"{nomask}:"])
    merge(out, qk_steps(fifo, S0, S1[0], 0, False, reader(fifo, "K", 1), blocks=(1,)),
          softmax_slow(0, S0, P0[0]), lead=2, lead_lines=lead)
    assert fifo.q == k_prefetch_tags()


def epilogue(out):
    """Normalise, round to bf16 and store O; store the base-2 log-sum-exp.  A lane holds four
    consecutive d of one row at a time, so each 32 x 128 block of the wave is transposed
    through the wave's own 8 KB strip of LDS (above the stage ring; 16-byte chunks
    XOR-swizzled by the row) and leaves as whole 256-byte rows, four rows per store
    instruction.  No barrier: the strip is private, the next block's start has one."""
    out.e("; ---- epilogue")
    out.ext(["s_nop 7", "s_nop 7", "s_nop 7"])
    inv, lg, adr = TMP + 12, TMP + 13, TMP + 14
    n = 0
    for b in (0, 1):
        l, m = L[b], M[b]
        out.ext([f"v_mov_b32 {v(T1)}, {v(l)}", "s_nop 1",
                 f"v_permlane32_swap_b32 {v(l)}, {v(T1)}", "s_nop 1",
                 f"v_add_f32 {v(l)}, {v(l)}, {v(T1)}",
                 f"v_log_f32 {v(lg)}, {v(l)}",
                 f"v_rcp_f32 {v(inv)}, {v(l)}",
                 "s_nop 0",
                 f"v_add_f32 {v(lg)}, {v(lg)}, {v(m)}",
                 f"global_store_dword %[l32x4], {v(lg)}, {sp(LSEW[b])}"])
        for db in range(4):
            for i4 in range(4):
                t = TMP + 4 * (n % 2)          # two sets of four temporaries
                w = S0 + 2 * (n % 8)           # eight result pairs (the logit registers are free now)
                src = O[b] + 16 * db + 4 * i4
                for k in range(4):
                    out.e(f"v_accvgpr_read_b32 {v(t + k)}, a{src + k}")
                for k in range(4):
                    out.e(f"v_mul_f32 {v(t + k)}, {v(t + k)}, {v(inv)}")
                out.e(f"v_cvt_pk_bf16_f32 {v(w)}, {v(t)}, {v(t + 1)}")
                out.e(f"v_cvt_pk_bf16_f32 {v(w + 1)}, {v(t + 2)}, {v(t + 3)}")
                out.e(f"v_xor_b32 {v(adr)}, {(4 * db + i4) * 16}, %[x16]")
                out.e(f"v_add_u32 {v(adr)}, {v(adr)}, %[strip_w]")
                out.e(f"ds_write_b64 {v(adr)}, {vr(w, 2)}")
                n += 1
        out.e("s_waitcnt lgkmcnt(0)")
        for u in range(8):
            out.e(f"v_xor_b32 {v(adr)}, {64 * (u & 3)}, %[crr16]")
            out.e(f"v_add_u32 {v(adr)}, {v(adr)}, %[strip_r]")
            out.e(f"ds_read_b128 {vr(S1[b] + 4 * u, 4)}, {v(adr)} offset:{u * 1024}")
        out.e("s_waitcnt lgkmcnt(0)")
        out.e(f"s_mov_b64 {sp(OB)}, {sp(OW[b])}")
        for u in range(8):
            if u == 4:
                out.e(f"s_add_u32 s{OB}, s{OB}, 4096")
                out.e(f"s_addc_u32 s{OB + 1}, s{OB + 1}, 0")
            out.e(f"global_store_dwordx4 %[lanex16], {vr(S1[b] + 4 * u, 4)}, {sp(OB)} offset:{(u & 3) * 1024}")


def generate():
    out = Out()
    setup(out)
    block = out.label("blk")
    out.e(f"{block}:")
    prologue(out)
    la, lb_e, lb_o, sp_e, sp_o, fin_e, fin_o, drain, epi = (
        out.label(x) for x in ("la", "lbe", "lbo", "spe", "spo", "fe", "fo", "dr", "ep"))

    def step(kind, par, last, target):
        top(out)
        out.e(f"s_cmp_eq_u32 s{T}, s{last}")
        out.e(f"s_cbranch_scc1 {target}")
        iteration(out, par, kind)
        out.e(f"s_add_u32 s{T}, s{T}, 1")

    # both blocks running: until block 0 reaches its last tile
    out.e(f"{la}:")
    step("both", 0, TF0, sp_e)
    step("both", 1, TF0, sp_o)
    out.e(f"s_branch {la}")
    # block 0's last tile (no barrier here: the branch came from a top)
    out.e(f"{sp_e}:")
    iteration(out, 0, "split")
    out.e(f"s_add_u32 s{T}, s{T}, 1")
    out.e(f"s_branch {lb_o}")
    out.e(f"{sp_o}:")
    iteration(out, 1, "split")
    out.e(f"s_add_u32 s{T}, s{T}, 1")
    # only block 1 running: until its last tile
    out.e(f"{lb_e}:")
    step("one", 0, TF1, fin_e)
    out.e(f"{lb_o}:")
    step("one", 1, TF1, fin_o)
    out.e(f"s_branch {lb_e}")
    out.e(f"{fin_e}:")
    final(out, 0)
    out.e(f"s_branch {drain}")
    out.e(f"{fin_o}:")
    final(out, 1)
    out.e(f"{drain}:")
    out.e(f"s_add_u32 s{T}, s{T}, 1")
    out.e(f"s_cmp_lt_u32 s{T}, s{NTMAX}")
    out.e(f"s_cbranch_scc0 {epi}")
    top_drain(out)
    out.e(f"s_branch {drain}")
    out.e(f"{epi}:")
    epilogue(out)
    out.e(f"s_add_u32 s{J}, s{J}, 1")
    out.e(f"s_cmp_eq_u32 s{HASNEXT}, 1")
    out.e(f"s_cbranch_scc1 {block}")
    done = out.label("done")
    out.e(f"s_branch {done}")
    out.ext(out.far)
    out.e(f"{done}:")
    return out.lines


def clobbers():
    # M0 is written by the stream (before every direct-to-LDS load) but cannot be declared:
    # it is a reserved register, which the compiler never keeps a value in across a statement
    # -- it writes M0 itself right before each of its own uses -- and listing it only draws
    # "clobber list contains reserved registers".  The stream is also the kernel's last statement.
    c = [f"v{i}" for i in range(NV)] + [f"a{i}" for i in range(NA)]
    c += [f"s{i}" for i in range(SLO, SHI + 1)] + ["vcc", "scc", "memory"]
    return ", ".join(f'"{x}"' for x in c)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    args = sys.argv[1:]
    path = args[0] if args else os.path.join(here, "attn_fwd128x2_body.inc")
    lines = generate()
    with open(path, "w") as f:
        f.write("// Written by gen_attn_fwd128x2.py; edit the generator, not this file.\n")
        f.write("#define A2SF_FWD128X2_ASM \\\n")
        for ln in lines:
            assert '"' not in ln and "\\" not in ln
            f.write(f'  "{ln}\\n" \\\n')
        f.write('  ""\n')
        f.write(f"#define A2SF_FWD128X2_CLOBBERS {clobbers()}\n")
    print(f"{path}: {len(lines)} lines")


if __name__ == "__main__":
    main()
