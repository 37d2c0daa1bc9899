#!/usr/bin/env python3
"""Generates fisher_gram_bf16_wide_loop.inc: the token loop of the wide bf16 Gram kernel
(GuidedQuant, Algorithm 1, line 4) as ONE inline-assembly statement for gfx950.

Why assembly: a wave keeps a 96 x 256 block of one group's H in 384 accumulator registers
(24 tiles of 32 x 32), 256 of them in the accumulation registers and 128 in ordinary
vector registers.  The compiler only ever places matrix-core results in one of the two
files, so C++ stops at 256 (a 64 x 256 block).  The larger block needs 27 % fewer LDS
operand reads and direct loads per matrix instruction, which is what bounds the kernel.

What the statement does, for one run of token steps [k0, k0 + count) of one work item:
  * direct global->LDS loads (6 per wave and stage of 32 tokens) into a ring of 6 stages,
    addressed as scalar stage base + 32-bit lane offset;
  * per 16-token sub-step 24 matrix instructions v_mfma_f32_32x32x16_bf16 on a scaled
    operand (3 fragments of 32 rows, s[i,k] applied in registers: bf16 -> fp32, multiply,
    round to nearest even) and a raw operand (8 fragments of 32 columns);
  * between the matrix instructions: the transposing LDS reads of the next sub-step's
    operands (a raw fragment is re-read into its own registers right after its last use),
    the scaling, and the stage's direct loads, in a fixed issue order;
  * LDS waits (`lgkmcnt`) are derived here from the issue order by a small scoreboard.
The first sub-step starts the accumulators from the constant 0, so no register is cleared.

Two variants are generated.  fisher_gram_bf16_wide_loop.inc: a workgroup's four waves are four groups on one
row block of 96 rows (group counts divisible by 4).  fisher_gram_bf16_wide2_loop.inc: two groups on two row
blocks (even group counts): the stage holds two tiles of the scaled operand (its lane address is what tells a
wave's tile), so a stage is 6 KiB larger, the ring has five stages instead of six and a wave issues eight direct
loads per stage, the last one the weights.  The statements are otherwise the same.

Run by build.py before compiling; the output is committed next to this file.
"""
import os
import sys

NS = 6                  # ring stages
LOADS = 6               # direct loads per wave and stage
STAGE = 23552           # bytes per ring stage: A 6144 + B 16384 + weights 1024
A_ROW, B_ROW = 192, 512  # bytes per token row of the two staged tiles
OUT_NAME = "fisher_gram_bf16_wide_loop.inc"


def configure(row_blocks):
    """Sets the constants of a variant: `row_blocks` row blocks of the scaled operand per workgroup."""
    global NS, LOADS, STAGE, DMA_SLOTS, OUT_NAME
    if row_blocks == 1:
        NS, LOADS, STAGE, OUT_NAME = 6, 6, 23552, "fisher_gram_bf16_wide_loop.inc"
        DMA_SLOTS = [int(v) for v in os.environ.get("GQW_DMASLOTS", "4,13,22").split(",")]
    else:
        NS, LOADS, STAGE, OUT_NAME = 5, 8, 2 * 6144 + 16384 + 1024, "fisher_gram_bf16_wide2_loop.inc"
        DMA_SLOTS = [int(v) for v in os.environ.get("GQW_DMASLOTS2", "3,9,15,21").split(",")]
MA, NB = 3, 8           # fragments of the scaled / raw operand per wave

# ---- fixed vector registers (all listed as clobbers) -------------------------------------------
A_SET = [0, 12]         # two sets of scaled fragments, 3 x 4 registers each
RAW = 24                # raw fragments of the scaled operand as read, 3 x 4
WREG = 36               # 8 token weights of the lane
BREG = 44               # raw fragments, 8 x 4
TMP = 76                # 2 scratch registers of the scaling
BASE = 78               # 6 LDS byte addresses of the stage being read: A, B0..B3, S
N_VGPR = 84
# ---- fixed scalar registers (clobbers) ----------------------------------------------------------
S_SI, S_CNT, S_T, S_LO, S_HI = 84, 85, 86, 87, 88
S_XB, S_WB, S_B5 = 90, 92, 94       # 64-bit pairs
S_FIRST, S_LAST = 84, 95


# ---- the issue order inside a sub-step of 24 matrix instructions (slots 0..23) --------------------
# Defaults = the fastest of the orders timed on an MI355X (X[65536,4096] and X[32768,8192], G = 4): the scaling
# pieces one per slot in the slots that issue no LDS read (a raw fragment is re-read after slots 2, 5, 8, ...);
# two pieces per slot, batched re-reads (2 or 4 fragments at once) or split re-reads were 1-3 % slower.
A_SLOTS = [int(v) for v in os.environ.get("GQW_ASLOTS", "0,1").split(",")]          # weights + scaled-operand reads
DMA_SLOTS = [int(v) for v in os.environ.get("GQW_DMASLOTS", "4,13,22").split(",")]  # M0 set here, the load one slot later
SCALE_SLOTS = [int(v) for v in os.environ.get("GQW_SCALESLOTS", "6,7,9,10,12,13,15,16,18,19,21,22").split(",")]
NO_BARRIER = os.environ.get("GQW_NOBARRIER") == "1"          # timing experiments only: results are wrong without it


class Emitter:
    def __init__(self):
        self.lines = []
        self.issued = 0                 # LDS reads issued so far
        self.done = 0                   # LDS reads known complete (sequence numbers < done)
        self.pending = {}               # register -> sequence number of the read that writes it

    def raw(self, text):
        self.lines.append(text)

    def lds_read(self, op, dst_lo, width, addr, offset):
        regs = "v[%d:%d]" % (dst_lo, dst_lo + width - 1)
        self.raw("%s %s, v%d offset:%d" % (op, regs, addr, offset))
        for r in range(dst_lo, dst_lo + width):
            self.pending[r] = self.issued
        self.issued += 1

    def need(self, regs):
        """Wait until the LDS reads that write `regs` have returned (reads return in order)."""
        seq = max([self.pending.get(r, -1) for r in regs])
        if seq >= self.done:
            outstanding_allowed = self.issued - seq - 1
            if outstanding_allowed < 15:                     # the counter holds at most 15
                self.raw("s_waitcnt lgkmcnt(%d)" % outstanding_allowed)
            self.done = seq + 1

    def state(self):
        """Scoreboard relative to the number of reads issued (what must agree where control flow joins)."""
        return (self.issued - self.done, tuple(sorted((r, self.issued - q) for r, q in self.pending.items()
                                                      if q >= self.done)))

    def wait_all_lds(self):
        self.raw("s_waitcnt lgkmcnt(0)")
        self.done = self.issued


def acc(x, y):
    return "%%[acc%d]" % (x * NB + y)


def frag(base, x):
    return "v[%d:%d]" % (base + 4 * x, base + 4 * x + 3)


def fetch_reads(ks):
    """LDS reads of one sub-step's operands from the stage BASE points at: list of closures."""
    out = []
    # weights of the lane's 8 tokens
    out.append(("w", lambda e: e.lds_read("ds_read_b128", WREG, 4, BASE + 5, ks * 64)))
    out.append(("w", lambda e: e.lds_read("ds_read_b128", WREG + 4, 4, BASE + 5, ks * 64 + 16)))
    for x in range(MA):
        for half in range(2):
            off = 64 * x + (ks * 16 + 4 * half) * A_ROW
            out.append(("a", lambda e, x=x, half=half, off=off:
                        e.lds_read("ds_read_b64_tr_b16", RAW + 4 * x + 2 * half, 2, BASE, off)))
    return out


def b_reads(ks, y):
    out = []
    for half in range(2):
        off = 256 * (y // 4) + (ks * 16 + 4 * half) * B_ROW
        out.append(lambda e, half=half, off=off:
                   e.lds_read("ds_read_b64_tr_b16", BREG + 4 * y + 2 * half, 2, BASE + 1 + y % 4, off))
    return out


def scale_piece(e, x, q, dst_set):
    """One dword (two tokens) of scaled fragment x: bf16 -> fp32, times the token weights, RNE -> bf16."""
    src = RAW + 4 * x + q
    e.need([src, WREG + 2 * q, WREG + 2 * q + 1])
    e.raw("v_lshlrev_b32 v%d, 16, v%d" % (TMP, src))
    e.raw("v_and_b32 v%d, 0xffff0000, v%d" % (TMP + 1, src))
    e.raw("v_mul_f32 v%d, v%d, v%d" % (TMP, WREG + 2 * q, TMP))
    e.raw("v_mul_f32 v%d, v%d, v%d" % (TMP + 1, WREG + 2 * q + 1, TMP + 1))
    e.raw("v_cvt_pk_bf16_f32 v%d, v%d, v%d" % (A_SET[dst_set] + 4 * x + q, TMP, TMP + 1))


def stage_setup(e, slot_fill):
    """Scalar set-up of the direct loads of token step s_SI (clamped to the last step; the last step
    reads its own, shifted copy of tokens and weights so that no row past the last token is touched)."""
    e.raw("s_min_u32 s%d, s%d, %%[last]" % (S_T, S_SI))
    e.raw("s_mul_i32 s%d, s%d, %%[stepbytes]" % (S_LO, S_T))
    e.raw("s_mul_hi_u32 s%d, s%d, %%[stepbytes]" % (S_HI, S_T))
    e.raw("s_add_u32 s%d, %%[xlo], s%d" % (S_XB, S_LO))
    e.raw("s_addc_u32 s%d, %%[xhi], s%d" % (S_XB + 1, S_HI))
    e.raw("s_lshl_b32 s%d, s%d, 7" % (S_LO, S_T))                       # 32 tokens x 4 bytes of weights per step
    e.raw("s_cmp_eq_u32 s%d, %%[last]" % S_T)
    e.raw("s_cselect_b32 s%d, %%[xtlo], s%d" % (S_XB, S_XB))
    e.raw("s_cselect_b32 s%d, %%[xthi], s%d" % (S_XB + 1, S_XB + 1))
    e.raw("s_cselect_b32 s%d, %%[wtail], s%d" % (S_LO, S_LO))
    e.raw("s_add_u32 s%d, %%[wlo], s%d" % (S_WB, S_LO))
    e.raw("s_addc_u32 s%d, %%[whi], 0" % (S_WB + 1))
    e.raw("s_cmp_lg_u32 %[sel5], 0")                                     # load 5 of waves 2, 3 is the weights
    e.raw("s_cselect_b32 s%d, s%d, s%d" % (S_B5, S_WB, S_XB))
    e.raw("s_cselect_b32 s%d, s%d, s%d" % (S_B5 + 1, S_WB + 1, S_XB + 1))
    e.raw("s_add_u32 s%d, s%d, 1" % (S_SI, S_SI))


def dma_m0(e, k, slot_fill):
    e.raw("s_add_u32 m0, %%[dst%d], %d" % (k, slot_fill * STAGE))


def dma_load(e, k):
    base = S_B5 if k == LOADS - 1 else S_XB
    e.raw("global_load_lds_dwordx4 %%[vo%d], s[%d:%d]" % (k, base, base + 1))


def sub_step(e, cur_set, nxt_set, fetch_ks, dma, slot_fill, first=False, fetch=True, nb=NB):
    """3 * nb matrix instructions on (A set cur_set, raw fragments 0 .. nb-1); in between: fetch of the next
    sub-step's operands from the stage BASE points at (sub-step fetch_ks of it), their scaling into A set
    nxt_set, and the direct loads `dma` (indices) of the stage in ring slot slot_fill.  The issue order is
    given for the full sub-step (slots 0..23); with fewer live fragments every slot maps proportionally onto
    the matrix instructions that remain."""
    n_live = MA * nb

    def pos(s):
        return min(n_live - 1, (s * n_live) // (MA * NB))

    extras = [[] for _ in range(n_live)]
    if fetch:
        reads = fetch_reads(fetch_ks)
        extras[pos(A_SLOTS[0])] += [r for _, r in reads[:4]]
        extras[pos(A_SLOTS[1])] += [r for _, r in reads[4:]]
        for y in range(nb):                                   # a raw fragment is re-read right after its last use
            extras[MA * y + MA - 1] += b_reads(fetch_ks, y)
    for idx, k in enumerate(dma):                             # M0 one slot ahead of its load
        extras[pos(DMA_SLOTS[idx])].append(lambda e, k=k: (dma_m0(e, k, slot_fill), e.raw("s_nop 0")))
        extras[pos(DMA_SLOTS[idx] + 1)].append(lambda e, k=k: dma_load(e, k))
    if fetch:
        pieces = [(x, q) for x in range(MA) for q in range(4)]
        for s, (px, pq) in zip(SCALE_SLOTS, pieces):
            extras[pos(s)].append(lambda e, px=px, pq=pq: scale_piece(e, px, pq, nxt_set))
    for i in range(n_live):
        y, x = divmod(i, MA)
        e.need(list(range(BREG + 4 * y, BREG + 4 * y + 4)))
        c = "0" if first else acc(x, y)
        e.raw("v_mfma_f32_32x32x16_bf16 %s, %s, %s, %s" % (acc(x, y), frag(A_SET[cur_set], x), frag(BREG, y), c))
        for fn in extras[i]:
            fn(e)


def build(nb=NB):
    """The statement for work items of which only the first nb raw fragments (32 columns each) are live."""
    e = Emitter()
    # ---------------- prologue: fill the ring, fetch and scale the first sub-step --------------
    # Scalar loads of the surrounding code must not be counted against the LDS reads below.  Its vector
    # memory operations (the stores of the previous item's results) may stay in flight: the counter retires
    # in issue order, so every wait below also covers them.
    e.raw("s_waitcnt lgkmcnt(0)")
    e.raw("s_mov_b32 s%d, %%[k0]" % S_SI)
    e.raw("s_mov_b32 s%d, %%[count]" % S_CNT)
    for t in range(NS - 1):
        stage_setup(e, t)
        for k in range(LOADS):
            dma_m0(e, k, t)
            e.raw("s_nop 0")
            dma_load(e, k)
    e.raw("s_waitcnt vmcnt(%d)" % ((NS - 2) * LOADS))
    e.raw("s_barrier")
    bases = ["%[laneA]", "%[laneB0]", "%[laneB1]", "%[laneB2]", "%[laneB3]", "%[laneS]"]

    def set_base(slot):
        for k, b in enumerate(bases):
            if slot == 0:
                e.raw("v_mov_b32 v%d, %s" % (BASE + k, b))
            else:
                e.raw("v_add_u32 v%d, %d, %s" % (BASE + k, slot * STAGE, b))

    set_base(0)
    for _, r in fetch_reads(0):
        r(e)
    for y in range(nb):
        for r in b_reads(0, y):
            r(e)
    e.wait_all_lds()
    for x in range(MA):
        for q in range(4):
            scale_piece(e, x, q, 0)
    e.raw("s_nop 7")
    # first sub-step: tokens 0..15 of the first stage, accumulators start from 0; fetches tokens 16..31
    sub_step(e, 0, 1, 1, [], 0, first=True, nb=nb)
    join_state = e.state()
    e.raw("s_sub_u32 s%d, s%d, 1" % (S_CNT, S_CNT))
    e.raw("s_cmp_eq_u32 s%d, 0" % S_CNT)
    e.raw("s_cbranch_scc1 GQW_TAIL%=")
    # ---------------- the loop: iteration m enters stage k0 + m (ring slot m % NS) -------------
    e.raw("GQW_LOOP%=:")
    for j in range(NS):
        m = (j + 1) % NS                          # slot that is entered
        slot_fill = (m + NS - 2) % NS             # slot of the stage two back, refilled with stage k0 + m + NS - 2
        e.raw("s_waitcnt vmcnt(%d)" % ((NS - 3) * LOADS))
        e.raw("s_nop 0" if NO_BARRIER else "s_barrier")
        stage_setup(e, slot_fill)
        # tokens 16..31 of the previous stage (operands already in registers); fetches tokens 0..15 of the
        # stage entered: its addresses are formed first
        set_base(m)
        sub_step(e, 1, 0, 0, list(range(LOADS // 2)), slot_fill, nb=nb)
        # tokens 0..15 of the stage entered; fetches its tokens 16..31
        sub_step(e, 0, 1, 1, list(range(LOADS // 2, LOADS)), slot_fill, nb=nb)
        assert e.state() == join_state, "LDS scoreboard differs between the paths that meet at a label"
        e.raw("s_sub_u32 s%d, s%d, 1" % (S_CNT, S_CNT))
        e.raw("s_cmp_eq_u32 s%d, 0" % S_CNT)
        if j < NS - 1:
            e.raw("s_cbranch_scc1 GQW_TAIL%=")
        else:
            e.raw("s_cbranch_scc0 GQW_LOOP%=")
    # ---------------- tail: tokens 16..31 of the last stage -------------------------------------
    e.raw("GQW_TAIL%=:")
    sub_step(e, 1, 0, 0, [], 0, fetch=False, nb=nb)
    e.raw("s_waitcnt vmcnt(0)")
    e.raw("s_nop 15")
    e.raw("s_nop 15")
    return e.lines


HEADER = """// GENERATED by gen_gram_wide_loop.py -- do not edit.  The token loop of the wide bf16 Gram kernel
// (one run of token steps of one work item) as inline-assembly statements, one per number of live
// raw fragments (work items that cross the diagonal or the right edge skip the matrix instructions of
// the 32-column fragments that lie wholly outside the upper triangle); the variables named in the
// operand lists are those of fisher_gram_bf16_wide.hip.
"""


def statement(nb):
    lines = build(nb)
    out = ["asm volatile("]
    for l in lines:
        out.append('    "%s\\n"' % l)
    outs = ", ".join('[acc%d] "=%s"(acc[%d])' % (i, "a" if i < 16 else "&v", i) for i in range(MA * NB))
    ins = []
    for k in range(LOADS):
        ins.append('[vo%d] "v"(vo[%d])' % (k, k))
    ins += ['[laneA] "v"(laneA)', '[laneB0] "v"(laneB[0])', '[laneB1] "v"(laneB[1])', '[laneB2] "v"(laneB[2])',
            '[laneB3] "v"(laneB[3])', '[laneS] "v"(laneS)']
    for k in range(LOADS):
        ins.append('[dst%d] "s"(dst[%d])' % (k, k))
    ins += ['[xlo] "s"(x_lo)', '[xhi] "s"(x_hi)', '[xtlo] "s"(xt_lo)', '[xthi] "s"(xt_hi)', '[wlo] "s"(w_lo)',
            '[whi] "s"(w_hi)', '[wtail] "s"(w_tail)', '[stepbytes] "s"(step_bytes32)', '[last] "s"(last_step)',
            '[k0] "s"(k0_32)', '[count] "s"(count32)', '[sel5] "s"(sel5)']
    clob = ['"v%d"' % r for r in range(N_VGPR)] + ['"s%d"' % r for r in range(S_FIRST, S_LAST + 1)] + ['"memory"', '"scc"']
    out.append("    : " + outs)
    out.append("    : " + ", ".join(ins))
    out.append("    : " + ", ".join(clob) + ");")
    return out, sum(1 for l in lines if l.startswith("v_mfma"))


def main():
    out = [HEADER, "switch (nb_live) {"]
    total = 0
    for nb in range(NB, 0, -1):
        body, n_mfma = statement(nb)
        total += n_mfma
        out.append("  case %d:   // the first %d raw fragments are live (%d columns)" % (nb, nb, 32 * nb))
        out += ["  " + l for l in body]
        out.append("    break;")
    out.append("  default:\n    __builtin_unreachable();\n}")
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), OUT_NAME)
    with open(path, "w") as f:
        f.write("\n".join(out) + "\n")
    print("wrote %s: %d statements, %d matrix instructions" % (path, NB, total), file=sys.stderr)


if __name__ == "__main__":
    for rb in (1, 2):
        configure(rb)
        main()
