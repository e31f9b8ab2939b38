#!/usr/bin/env python3
"""Writes wk_attn_loop_gfx950.inc: the steady-state loop of k_attn_bf16 (8 waves x 32 queries, 64-key tiles) as
one hand-scheduled inline-assembly body for gfx950.

    python gen_attn_loop.py [output file]      (default: wk_attn_loop_gfx950.inc beside this script)

The loop does exactly what four consecutive `step`s of the C++ kernel do -- the same ring protocol, the same
arithmetic in the same order, bit-identical results -- but with the schedule fixed by hand:

  * K fragments are requested two pairs of reads ahead of the matrix instructions that consume them, V^T
    fragments six matrix instructions ahead; every wait on the LDS counter is partial (LDS reads return in
    order, so "at most n outstanding" names the read that has landed);
  * the softmax arithmetic of the tile being consumed (scale, exp2, round to bf16, row sum) is dealt between the
    16 matrix instructions that form S^T of the next tile, software-pipelined so that no instruction waits for
    its producer; the 16 value products follow with the next tile's row maximum between them;
  * the last three value products of a step are kept back past the workgroup barrier and issued behind the next
    step's first K reads: they cover the latency of those reads, which cannot be requested before the barrier;
  * tile loads (global memory -> LDS) are issued from here, so the compiler's wait-count pass never sees them.

Hazards the assembler does not resolve, and how the schedule respects them: a register written by a matrix
instruction is read by vector instructions only many matrix instructions later (the row maximum starts seven
instructions behind the last S^T product; the rare rescale of O^T waits 16 states first); a v_exp result is
consumed at least four instructions later; v_mov -> v_permlane32_swap has two wait states between.

Register map (VGPR), fixed through operand constraints in the kernel source:
  O   v[0:63]     o[b] = v[16b : 16b+15]
  SA  v[64:95]    S^T tile at even ring positions (two 32-key blocks of 16 registers)
  SB  v[96:127]   ... at odd ring positions
  Q   v[128:159]  qb[st] = v[128+4st : 131+4st]
  P   v[160:175]  pb[ks] = v[160+4ks : 163+4ks]
  KF  v[176:199]  six K fragment buffers
  VF  v[200:223]  six V^T fragment buffers (two 8-byte transpose reads each)
  KAD v[224:231]  LDS address of K operand read st
  VAD v[232:235]  LDS address of V^T operand read blk (V ring base included)
  KSRC v[236:237] VSRC v[238:239]   per-lane source offsets of this wave's tile loads
  M v240  L v241  MT v243   running max (log2 units), row sum, scaled max of the next tile
  T   v[244:246]  temporaries
SGPR:
  s[36:37] K rows of this head, s[38:39] V rows, s40 byte offset of the K tile requested next, s41 same for V,
  s42 LDS address of this wave's share of K ring slot 0, s43 scale*log2(e), s44 groups left, s45 the caller's m0
"""
import os
import sys

TILE = 16384          # bytes of one 64-key K or V tile
VRING = 65536         # the V ring sits behind the four K slots
DEFER = 3             # value products kept back past the barrier

S = {0: 64, 1: 96}


def Q(st):
    return 128 + 4 * st


def P(ks):
    return 160 + 4 * ks


def KF(i):
    return 176 + 4 * i


def VF(i):
    return 200 + 4 * i


def KAD(st):
    return 224 + st


def VAD(b):
    return 232 + b


KSRC, VSRC = (236, 237), (238, 239)
M, L, MT = 240, 241, 243
T0, T1, T2 = 244, 245, 246
ONES = "0x3f803f80"    # two bf16 ones


def rng(a, n):
    return f"v[{a}:{a + n - 1}]"


class Emitter:
    """Collects instructions and keeps the queue of outstanding LDS reads, from which the partial waits follow."""

    def __init__(self):
        self.lines = []
        self.lds = []
        self.next_id = 0
        self.deferred = []

    def emit(self, s):
        self.lines.append(s)

    def lds_read(self, text):
        self.emit(text)
        self.lds.append(self.next_id)
        self.next_id += 1
        assert len(self.lds) <= 15, "the 4-bit LDS counter would saturate"
        return self.next_id - 1

    def wait_for(self, rid):
        if rid in self.lds:
            k = self.lds.index(rid)
            self.emit(f"s_waitcnt lgkmcnt({len(self.lds) - 1 - k})")
            self.lds = self.lds[k + 1:]


def head(E, pos):
    """The first three pairs of K fragment reads of a step (tile j+1, ring slot pos+1)."""
    koff = ((pos + 1) & 3) * TILE
    kreads = {}
    for st in range(3):
        for b in range(2):
            buf = (2 * st + b) % 6
            rid = E.lds_read(f"ds_read_b128 {rng(KF(buf), 4)}, v{KAD(st)} offset:{koff + b * 8192}")
            kreads[(st, b)] = (buf, rid)
    return kreads


def step(E, pos, kreads=None):
    cur = S[pos & 1]            # S^T of the tile consumed in this step (ring slot pos)
    nxt = S[(pos + 1) & 1]      # S^T of the next tile, formed in this step
    koff = ((pos + 1) & 3) * TILE
    voff = pos * TILE

    if kreads is None:
        kreads = head(E, pos)
        for txt in E.deferred:   # the value products kept back by the previous step
            E.emit(txt)
        E.deferred = []

    def issue_k(st):
        for b in range(2):
            buf = (2 * st + b) % 6
            rid = E.lds_read(f"ds_read_b128 {rng(KF(buf), 4)}, v{KAD(st)} offset:{koff + b * 8192}")
            kreads[(st, b)] = (buf, rid)

    # this wave's share of K tile j+4 (into the K slot whose tile went into S^T one step ago) and of V tile j+3
    for i in range(2):
        E.emit(f"s_add_u32 m0, s42, {pos * TILE + i * 1024}")
        E.emit(f"v_add_u32_e32 v{T0}, s40, v{KSRC[i]}")
        E.emit(f"global_load_lds_dwordx4 v{T0}, s[36:37]")
    for i in range(2):
        E.emit(f"s_add_u32 m0, s42, {VRING + ((pos + 3) & 3) * TILE + i * 1024}")
        E.emit(f"v_add_u32_e32 v{T0}, s41, v{VSRC[i]}")
        E.emit(f"global_load_lds_dwordx4 v{T0}, s[38:39]")
    E.emit(f"s_add_u32 s40, s40, {TILE}")
    E.emit(f"s_add_u32 s41, s41, {TILE}")

    # lazy rescale: only when some row's maximum grew by more than 2^8
    lab = f"L_norescale_{pos}_%="
    E.emit(f"v_add_f32_e32 v{T0}, 0x41000000, v{M}")
    E.emit(f"v_cmp_gt_f32_e32 vcc, v{MT}, v{T0}")
    E.emit(f"s_cbranch_vccz {lab}")
    E.emit("s_nop 7")
    E.emit("s_nop 7")
    E.emit(f"v_max_f32_e32 v{T0}, v{M}, v{MT}")
    E.emit(f"v_sub_f32_e32 v{T1}, v{M}, v{T0}")
    E.emit(f"v_exp_f32_e32 v{T1}, v{T1}")
    E.emit(f"v_mov_b32_e32 v{M}, v{T0}")
    E.emit("s_nop 1")
    E.emit(f"v_mul_f32_e32 v{L}, v{L}, v{T1}")
    for r in range(64):
        E.emit(f"v_mul_f32_e32 v{r}, v{T1}, v{r}")
    E.emit(f"{lab}:")

    # softmax arithmetic of the tile consumed, in place in its registers; element e is register cur + e.
    # Slot i: scale elements 2i, 2i+1; exp2 of the pair scaled one slot ago; round the pair exponentiated one slot
    # ago into P; add the pair rounded one slot ago to the row sum.
    stream = []
    for i in range(16 + 3):
        ops = []
        if i < 16:
            ops += [f"v_fma_f32 v{cur + 2 * i}, v{cur + 2 * i}, s43, -v{M}",
                    f"v_fma_f32 v{cur + 2 * i + 1}, v{cur + 2 * i + 1}, s43, -v{M}"]
        if 1 <= i < 17:
            k = i - 1
            ops += [f"v_exp_f32_e32 v{cur + 2 * k}, v{cur + 2 * k}", f"v_exp_f32_e32 v{cur + 2 * k + 1}, v{cur + 2 * k + 1}"]
        if 2 <= i < 18:
            k = i - 2
            ops += [f"v_cvt_pk_bf16_f32 v{P(0) + k}, v{cur + 2 * k}, v{cur + 2 * k + 1}"]
        if 3 <= i < 19:
            ops += [f"v_dot2c_f32_bf16_e32 v{L}, {ONES}, v{P(0) + i - 3}"]
        stream.append(ops)

    vreads = {}

    def issue_v(n):
        ks, b = n // 4, n % 4
        buf = n % 6
        E.lds_read(f"ds_read_b64_tr_b16 {rng(VF(buf), 2)}, v{VAD(b)} offset:{voff + ks * 4096}")
        rid = E.lds_read(f"ds_read_b64_tr_b16 {rng(VF(buf) + 2, 2)}, v{VAD(b)} offset:{voff + ks * 4096 + 2048}")
        vreads[n] = (buf, rid)

    # S^T of the next tile: K block b (32 keys) x 16 features of step st, the two blocks' chains alternating
    slot = 0
    for st in range(8):
        for b in range(2):
            buf, rid = kreads[(st, b)]
            E.wait_for(rid)
            c = "0" if st == 0 else rng(nxt + 16 * b, 16)
            E.emit(f"v_mfma_f32_32x32x16_bf16 {rng(nxt + 16 * b, 16)}, {rng(KF(buf), 4)}, {rng(Q(st), 4)}, {c}")
            for op in stream[slot]:
                E.emit(op)
            slot += 1
        if st + 3 < 8:
            issue_k(st + 3)
        if st >= 5:   # the first V^T fragments, while the last K fragments are consumed
            issue_v(2 * (st - 5))
            issue_v(2 * (st - 5) + 1)
    for ops in stream[16:]:
        for op in ops:
            E.emit(op)

    # row maximum of the next tile (two chains over its 32 registers, then across the two lane halves), scaled
    mx = [f"v_max3_f32 v{T1}, v{nxt}, v{nxt + 1}, v{nxt + 2}", f"v_max3_f32 v{T2}, v{nxt + 3}, v{nxt + 4}, v{nxt + 5}"]
    for n, i in enumerate(range(6, 32, 2)):
        t = T1 if n % 2 == 0 else T2
        mx.append(f"v_max3_f32 v{t}, v{t}, v{nxt + i}, v{nxt + i + 1}")
    mx += [f"v_max_f32_e32 v{T1}, v{T1}, v{T2}", f"v_mov_b32_e32 v{T2}, v{T1}", "s_nop 1",
           f"v_permlane32_swap_b32_e32 v{T1}, v{T2}", "s_nop 0", f"v_max_f32_e32 v{T1}, v{T1}, v{T2}",
           f"v_mul_f32_e32 v{MT}, s43, v{T1}"]

    # O^T += V^T P^T: feature block b x 16 keys of step ks
    mi = 0
    for n in range(16):
        ks, b = n // 4, n % 4
        buf, rid = vreads[n]
        E.wait_for(rid)
        txt = f"v_mfma_f32_32x32x16_bf16 {rng(16 * b, 16)}, {rng(VF(buf), 4)}, {rng(P(ks), 4)}, {rng(16 * b, 16)}"
        if n >= 16 - DEFER:
            E.deferred.append(txt)
        else:
            E.emit(txt)
        if n + 6 < 16:
            issue_v(n + 6)
        if n >= 6:
            for op in mx[mi:mi + 3]:
                E.emit(op)
            mi += 3
    for op in mx[mi:]:
        E.emit(op)
    assert not E.lds
    E.emit("s_waitcnt vmcnt(8)")   # all but the tile loads of this step and the one before have landed
    E.emit("s_barrier")


def generate():
    # what position 3 keeps back is the same text in every iteration: find it with a dry run
    dry = Emitter()
    for pos in range(4):
        step(dry, pos)
    carried = list(dry.deferred)

    E = Emitter()
    E.emit("s_mov_b32 s45, m0")   # m0 is the compiler's to manage: hand it back as it was
    # entry: the first reads of position 0 with nothing kept back (the C++ step before finished its tile)
    kr = head(E, 0)
    E.emit("s_branch L_body_%=")
    state = (list(E.lds), E.next_id)
    E.emit("L_group_%=:")
    E.lds, E.next_id = [], 0
    assert head(E, 0) == kr and (list(E.lds), E.next_id) == state
    for txt in carried:
        E.emit(txt)
    E.emit("L_body_%=:")
    step(E, 0, kreads=kr)
    for pos in range(1, 4):
        step(E, pos)
    assert E.deferred == carried
    E.emit("s_sub_u32 s44, s44, 1")
    E.emit("s_cmp_lg_u32 s44, 0")
    E.emit("s_cbranch_scc1 L_group_%=")
    for txt in carried:
        E.emit(txt)
    E.emit("s_nop 7")    # the compiler's code behind the block may read O^T at once
    E.emit("s_nop 7")
    E.emit("s_mov_b32 m0, s45")
    return E.lines


def render():
    out = ["// Written by gen_attn_loop.py: the hand-scheduled steady-state loop of k_attn_bf16 (see that script).\n"]
    out += ['"' + ln + '\\n\\t"\n' for ln in generate()]
    return "".join(out)


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    path = sys.argv[1] if len(sys.argv) > 1 else os.path.join(here, "wk_attn_loop_gfx950.inc")
    with open(path, "w") as f:
        f.write(render())
    print(path)
