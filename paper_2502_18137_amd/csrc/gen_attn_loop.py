#!/usr/bin/env python3
"""Writes attn_loop_gfx950.inc: the iterations of the sparse flash loop (Alg. 1 lines 9-17 of
arXiv 2502.18137) as one hand-scheduled gfx950 assembly block per (head dimension, 16-bit type, LDS
stages), wrapped in a C++ function that attn.hip includes.

    python gen_attn_loop.py            # rewrites attn_loop_gfx950.inc next to this file

Why assembly: the matrix pipe and the vector ALU of a SIMD only overlap when MFMA and vector
instructions alternate at fine grain inside a wave, and one wave alone cannot issue vector
instructions back to back, so the kernel runs two waves per SIMD with 256 registers each; the
instruction order and the register assignment are the design.  The block is entered once per row
group, after the kernel has computed the scores of the row's first kept tile, and runs every
iteration including the last one and the drain; C++ keeps the list building, that first tile and the
epilogue.

A wave owns one 32-row group.  The loop is skewed by one tile; tiles are positions in the row's list
of kept key blocks.  State at the boundary "top of iteration u" (u >= 1):
  S[u & 1]        biased scores of tile u; the row statistics already include tile u
                  (scx = its dequantization scale, exec = its stage-2 decision),
  P[(u - 1) & 1]  P~ of tile u-1, waiting for its P~V product (execp = its stage-2 decision),
  LDS             K_hat(u+1) and V(u-1) have been requested NST-1 iterations ago.
Iteration u: wait for own copies, barrier, request K_hat(u+NST) and V(u+NST-2) (as far as the list
goes; a partial last K_hat block is copied with clamped rows); then one "step":
  vector ALU: softmax of tile u  ->  P[u & 1], row sum
  MFMA:       scores of tile u+1 -> S[(u + 1) & 1];  O += P~(u-1) V(u-1)
as a sequence of slots: operand read (LDS, three slots ahead), one MFMA, a chunk of the softmax.
The row maximum of the fresh scores, the stage-2 test (Alg. 1 line 15) and the test whether the
reference maximum must move follow at the end of the step.  A move takes effect at once for l and
m_ref; O is multiplied one iteration later, after the P~V product that was computed against the old
reference has been added (havefo / fo carry that debt, also across the block's boundary).

Every body exists with and without the P~V product (execp: the stage-2 decision of tile u-1).
Two kinds of iteration bodies exist.  "fast": tile u+1 needs no element masks.  "masked": the scores
of tile u+1 are overwritten in place with -inf where the key lies past N or (causal) past the row,
before their row maximum is taken, so the softmax of the following iteration needs no mask; a tile
u+1 that does not exist counts as fully masked, which makes the last iteration (u = cnt-1, nothing to
score) and the drain (u = cnt: only P~V of the last tile) ordinary masked iterations.  Iteration 0
enters with execp = 0: nothing is pending.
"""
import math
import os

MAGIC_NEG = 0xCB400000  # bit pattern of -12582912.0f = -(1.5 * 2^23)
RESCALE_T = {8: 0x41000000, 2: 0x40000000}  # 8.0f, 2.0f
LA = 4                  # operand reads run this many slots ahead; they are issued and awaited in pairs
RING = LA + 2
PRE_UNITS = 10          # vector work placed before the first MFMA of a step (covers the LDS latency)
NWAVE = 4               # waves per workgroup sharing the tile copies


class Cfg:
    def __init__(self, D, dt, qk16=False):
        self.D, self.dt, self.qk16 = D, dt, qk16
        # Q K^T: INT8 32x32x32 MFMAs on quantized operands, or (qk16) 32x32x16 MFMAs on the 16-bit tensors
        # themselves: twice the steps along d, twice the bytes per K row, fp32 scores
        self.NSTEP = D // 16 if qk16 else D // 32
        self.NDT = D // 32
        self.KROW = D * (2 if qk16 else 1)       # bytes of one K row in LDS
        self.fp8 = dt == "fp8"
        assert not (self.fp8 and qk16)
        # P~V: 16-bit 32x32x16 MFMAs (4 key steps per channel tile) or one FP8 32x32x64 MFMA per channel tile
        self.NQK, self.NPV = 2 * self.NSTEP, (self.NDT if self.fp8 else 4 * self.NDT)
        self.NSLOT = self.NQK + self.NPV
        self.NUNIT = self.NQK + (2 * self.NDT if self.fp8 else self.NPV)   # 16-byte operand reads per step
        self.K_BYTES, self.V_BYTES = 64 * self.KROW, (D * 64 if self.fp8 else D * 128)
        self.NP = 2 if self.fp8 else 4           # registers quads of one P~ tile
        # how far the row maximum may run ahead of the reference (log2 units); with FP8 P~ is scaled by
        # 448 / 2^T so that its largest possible value is the largest E4M3 number
        self.T_LOG2 = 2 if self.fp8 else 8
        self.KD, self.VD = self.K_BYTES // (1024 * NWAVE), self.V_BYTES // (1024 * NWAVE)  # copies per wave
        self.NDMA = self.KD + self.VD
        # ---- VGPRs (pinned; the kernel uses no AGPRs, so all 256 registers of a wave are VGPRs) ----
        self.S = (0, 32)
        self.P = (64, 80)
        # accumulator start value of the INT8 products (qk16 starts from the constant 0); ring of operand registers
        self.MG, self.RG = (None, 96) if qk16 else (96, 112)
        nxt = self.RG + 4 * RING
        (self.MT, self.MR, self.L, self.INV, self.CX) = range(nxt, nxt + 5)
        nxt += 5
        self.T = nxt                              # 3 temporaries
        self.L0, self.L1, self.L2 = nxt, nxt + 1, nxt + 2  # list prefetch: read back before the temporaries are used
        self.MLOC = nxt + 2
        nxt += 3
        self.KA, self.VA = nxt, nxt + self.NSTEP  # per-lane LDS addresses of the operand reads in buffer 0
        nxt += self.NSTEP + 4
        self.KSRC = nxt                           # KD registers: global offsets of this wave's K_hat copy pieces
        self.VSRC = nxt + self.KD                 # VD registers: the same for V
        self.KSRCC = self.VSRC + self.VD          # KD registers: K_hat pieces of a partial last block (rows clamped)
        nxt = self.KSRCC + self.KD
        self.L3, self.ROWLIM = nxt, nxt + 1       # masked bodies: list prefetch of tile u+1; last visible key per lane
        self.FO = nxt + 2                         # factor O still has to be multiplied by (the reference maximum moved)
        self.PJ, self.PS = nxt + 3, nxt + 4       # LDS addresses of the list entries of iteration u (blocks, scales)
        nxt += 5
        self.O = nxt + (nxt & 1)                  # tuples start at even registers
        self.Q = self.O + 16 * self.NDT
        self.NVGPR = self.Q + 4 * self.NSTEP
        assert self.NVGPR <= 256
        # ---- SGPRs (pinned) ----
        names = ("u jpart kb0 kb1 vb0 vb1 ldskd ldsvd ldsjl ldsscl lam2 exec pv scx scn jk jv negmagic rt scnn "
                 "t0 t1 a0 a1 b0 b1 cnt ufull jn mlim ex0 ex1 exp0 exp1 hf0 hf1 ktile").split()
        self.sg = {n: 36 + i for i, n in enumerate(names)}
        for n in "kb0 vb0 a0 b0 ex0 exp0 hf0".split():
            assert self.sg[n] % 2 == 0, (n, self.sg)


def sp(s, n):
    """An aligned SGPR pair by the name of its first register."""
    return f"s[{s[n]}:{s[n] + 1}]"


def vr(b, n=1):
    return f"v{b}" if n == 1 else f"v[{b}:{b + n - 1}]"


def gen_step(c, o, cur, NST, kbuf, vbuf, masked, pv, dkbuf, dvbuf, label, late):
    """One iteration body: softmax of S[cur] -> P[cur]; scores of the next tile -> S[1-cur];
    O += P[1-cur] V unless that product was voted out (pv = False: Alg. 1 line 15 said skip); then the
    row maximum of the fresh scores and the two decisions."""
    s = c.sg
    nxt = 1 - cur
    XS, XP, YS, YP = c.S[cur], c.P[cur], c.S[nxt], c.P[nxt]
    T0, T1, T2 = c.T, c.T + 1, c.T + 2

    NSLOT = c.NSLOT if pv else c.NQK  # without the P~V product only the score MFMAs remain
    NUNIT = c.NUNIT if pv else c.NQK  # operand reads (16 bytes per lane each)
    # MFMA slot -> (first operand unit, units): an FP8 P~V MFMA takes two
    if c.fp8:
        slot_units = [(sl, 1) for sl in range(c.NQK)] + [(c.NQK + 2 * dt, 2) for dt in range(c.NDT)]
    else:
        slot_units = [(sl, 1) for sl in range(c.NSLOT)]

    def read(un):
        dst = c.RG + 4 * (un % RING)
        if un < c.NQK:
            kh, st = un % 2, un // 2
            o(f"ds_read_b128 {vr(dst, 4)}, v{c.KA + st} offset:{kbuf * c.K_BYTES + kh * 32 * c.KROW}")
        elif c.fp8:
            dt, h2 = divmod(un - c.NQK, 2)
            o(f"ds_read_b128 {vr(dst, 4)}, v{c.VA} offset:{vbuf * c.V_BYTES + dt * 2048 + h2 * 1024}")
        else:
            ks, dt = divmod(un - c.NQK, c.NDT)
            o(f"ds_read_b128 {vr(dst, 4)}, v{c.VA + ks} offset:{vbuf * c.V_BYTES + dt * 4096}")

    def mfma(sl):
        un, _ = slot_units[sl]
        src = c.RG + 4 * (un % RING)
        if sl < c.NQK:
            kh, st = sl % 2, sl // 2
            d = YS + 16 * kh
            if c.qk16:
                acc = "0" if st == 0 else vr(d, 16)
                o(f"v_mfma_f32_32x32x16_{c.dt} {vr(d, 16)}, {vr(src, 4)}, {vr(c.Q + 4 * st, 4)}, {acc}")
            else:
                acc = vr(c.MG, 16) if st == 0 else vr(d, 16)
                o(f"v_mfma_i32_32x32x32_i8 {vr(d, 16)}, {vr(src, 4)}, {vr(c.Q + 4 * st, 4)}, {acc}")
        elif c.fp8:
            dt = sl - c.NQK
            a = c.O + 16 * dt
            o(f"v_mfma_f32_32x32x64_f8f6f4 {vr(a, 16)}, {vr(src, 8)}, {vr(YP, 8)}, {vr(a, 16)}")
        else:
            ks, dt = divmod(sl - c.NQK, c.NDT)
            a = c.O + 16 * dt
            o(f"v_mfma_f32_32x32x16_{c.dt} {vr(a, 16)}, {vr(src, 4)}, {vr(YP + 4 * ks, 4)}, {vr(a, 16)}")

    # ---- the vector instruction stream of the step: (text, issue units) ----
    ops = []
    x = lambda e: XS + e
    F = lambda e: ops.append((f"v_fma_f32 v{x(e)}, v{x(e)}, s{s['scx']}, v{c.CX}", 1))
    E = lambda e: ops.append((f"v_exp_f32 v{x(e)}, v{x(e)}", 2))
    A = lambda e: ops.append((f"v_add_f32 v{c.L}, v{c.L}, v{x(e)}", 1))
    if c.fp8:   # two E4M3 values into the low or the high half of a register
        C = lambda w: ops.append((f"v_cvt_pk_fp8_f32 v{XP + w // 2}, v{x(2 * w)}, v{x(2 * w + 1)}"
                                  + (" op_sel:[0,0,1]" if w % 2 else ""), 1))
    else:
        C = lambda w: ops.append((f"v_cvt_pk_{c.dt}_f32 v{XP + w}, v{x(2 * w)}, v{x(2 * w + 1)}", 1))
    for k in range(16):
        F(2 * k); F(2 * k + 1); E(2 * k); E(2 * k + 1)
        if k:
            A(2 * k - 2); A(2 * k - 1); C(k - 1)
    A(30); A(31); C(15)
    first_max = len(ops)  # index of the first instruction that touches the fresh scores
    y = lambda e: YS + e
    if masked:
        # -inf over the scores of keys this lane's row must not see: key offset inside the tile >
        # ROWLIM - 64 j (a tile that does not exist has everything masked); -inf is a negative integer,
        # so the integer maximum below ignores it
        ops.append((f"v_subrev_u32 v{T1}, s{s['mlim']}, v{c.ROWLIM}", 1))
        ops.append((f"v_mov_b32 v{T2}, 0xff800000", 1))
        for e in range(32):
            koff = (e >> 4) * 32 + 8 * ((e & 15) >> 2) + (e & 3)
            ops.append((f"v_cmp_le_i32 vcc, {koff}, v{T1}", 1))
            ops.append((f"v_cndmask_b32 v{y(e)}, v{T2}, v{y(e)}, vcc", 1))
    # row maximum of the fresh scores (biased integers compare like the scores themselves; fp32 scores of
    # the 16-bit product can be negative and take the float comparison)
    mx = "f32" if c.qk16 else "i32"
    chains = []
    for t, base in ((T0, y(0)), (T1, y(16))):
        ch = [f"v_max3_{mx} v{t}, v{base}, v{base + 1}, v{base + 2}"]
        ch += [f"v_max3_{mx} v{t}, v{t}, v{base + i}, v{base + i + 1}" for i in range(3, 15, 2)]
        ch += [f"v_max_{mx} v{t}, v{t}, v{base + 15}"]
        chains.append(ch)
    for a_, b_ in zip(*chains):
        ops.append((a_, 1)); ops.append((b_, 1))
    tail = [f"v_max_{mx} v{T0}, v{T0}, v{T1}"]
    if not c.qk16:
        tail += [f"v_add_f32 v{T0}, s{s['negmagic']}, v{T0}"]  # biased integer (as float) -> integer score
    tail += [f"v_mul_f32 v{T0}, s{s['scn']}, v{T0}",           # -> log2-domain score
            f"v_mov_b32 v{T1}, v{T0}",
            "s_nop 1",
            f"v_permlane32_swap_b32 v{T0}, v{T1}",            # exchange with the lane holding the other 16 keys
            "s_nop 1",
            f"v_max_f32 v{c.MLOC}, v{T0}, v{T1}",
            f"v_max_f32 v{c.MT}, v{c.MT}, v{c.MLOC}",         # new running maximum
            f"v_sub_f32 v{T0}, v{c.MLOC}, v{c.MT}",
            f"v_sub_f32 v{T1}, v{c.MT}, v{c.MR}",
            f"v_add_f32 v{T0}, v{T0}, v{c.INV}",              # rows past N: -inf
            f"v_add_f32 v{T1}, v{T1}, v{c.INV}"]
    assert all(isinstance(t, str) for t in tail)

    # chunk 0 runs before the first MFMA, chunk sl + 1 after MFMA sl
    if pv:
        def spread(part, weights, pre):
            """part's instructions over len(weights) + 1 consecutive chunks: `pre` issue units in the first
            one, the rest behind the MFMAs in proportion to the time each MFMA occupies the matrix pipe."""
            total = sum(u for _, u in part)
            wsum = max(sum(weights), 1)
            out, acc_u, idx, wacc = [], 0.0, 0, 0
            for k in range(len(weights) + 1):
                target = pre + (total - pre) * wacc / wsum
                ch = []
                while idx < len(part) and (acc_u + part[idx][1] / 2 <= target or k == len(weights)):
                    ch.append(part[idx][0]); acc_u += part[idx][1]
                    idx += 1
                out.append(ch)
                if k < len(weights):
                    wacc += weights[k]
            return out
        # an FP8 32x32x64 MFMA runs twice as long as the others
        wts = [2 if (c.fp8 and sl >= c.NQK) else 1 for sl in range(NSLOT)]
        # the fresh scores are complete a few slots after the last Q K^T MFMA: nothing that reads them
        # comes before chunk kmin
        kmin = c.NQK + (1 if c.fp8 else 2)
        chunks = spread(ops, wts, PRE_UNITS)
        if sum(len(ch) for ch in chunks[:kmin]) > first_max:
            chunks = spread(ops[:first_max], wts[:kmin - 1], PRE_UNITS) + spread(ops[first_max:], wts[kmin:], 0)
        assert sum(len(ch) for ch in chunks[:kmin]) <= first_max and len(chunks) == NSLOT + 1
    else:
        # the score MFMAs are the only ones: the softmax stream is spread over their slots, at least 20
        # of its instructions stay behind the last MFMA, and the work on the fresh scores follows them
        soft, fresh = ops[:first_max], ops[first_max:]
        keep_last = 20
        head = soft[:len(soft) - keep_last]
        total = sum(u for _, u in head)
        per_slot = total / NSLOT
        chunks, acc_u, idx = [], 0.0, 0
        for k in range(NSLOT):
            target = per_slot * (k + 1)
            ch = []
            while idx < len(head) and (acc_u + head[idx][1] / 2 <= target or k == NSLOT - 1):
                ch.append(head[idx][0]); acc_u += head[idx][1]
                idx += 1
            chunks.append(ch)
        chunks.append([t for t, _ in soft[len(soft) - keep_last:]] + [t for t, _ in fresh])
    chunks[-1] += tail
    assert len(chunks[-1]) >= 12, "too little vector work behind the last MFMA"

    o(f"; ---- {'masked' if masked else 'fast'} step: softmax S{cur} -> P{cur} | scores -> S{nxt}"
      + (f", O += P{nxt} V" if pv else " (P~V voted out)"))
    # list entries the next iteration needs (older than every operand read of this step)
    o(f"ds_read_u16 v{c.L1}, v{c.PJ} offset:{2 * (NST - 1)}")   # key block of V(u+1+NST-2)
    o(f"ds_read_u16 v{c.L0}, v{c.PJ} offset:{2 * (NST + 1)}")   # key block of K_hat(u+1+NST)
    o(f"ds_read_b32 v{c.L2}, v{c.PS} offset:8")                 # scale of tile u+2
    if masked:
        o(f"ds_read_u16 v{c.L3}, v{c.PJ} offset:2")             # key block of tile u+1
    for un in range(LA):
        read(un)
    o(f"v_add_u32 v{c.PJ}, 2, v{c.PJ}")
    o(f"v_add_u32 v{c.PS}, 4, v{c.PS}")
    o(f"v_mov_b32 v{c.CX}, s{s['negmagic']}")
    o(f"v_fma_f32 v{c.CX}, v{c.CX}, s{s['scx']}, -v{c.MR}")   # -(bias * scale) - reference maximum
    if c.fp8:  # P~ is scaled by 448 / 2^T onto the E4M3 range
        import struct
        bits = struct.unpack("<I", struct.pack("<f", math.log2(448.0) - c.T_LOG2))[0]
        o(f"v_add_f32 v{c.CX}, 0x{bits:08x}, v{c.CX}")
    if masked:  # a row that has not seen a key yet (reference -inf) only has masked scores here
        o(f"v_cmp_eq_f32 vcc, 0xff800000, v{c.MR}")
        o(f"v_cndmask_b32_e64 v{c.CX}, v{c.CX}, 0, vcc")
    if pv:
        o(f"s_add_u32 s{s['pv']}, s{s['pv']}, 1")
    for t in chunks[0]:
        o(t)
    tag = f"{label}"
    for sl in range(NSLOT):
        un, nu = slot_units[sl]
        if un % 2 == 0:   # a new pair of operand units begins: request the pair LA units ahead, wait for this one
            issued = min(NUNIT, un + LA + 2)
            for t in range(un + LA, issued):
                read(t)
            o(f"s_waitcnt lgkmcnt({issued - (un + 2)})")
        if sl == 0:   # while its MFMAs are being issued the wave goes first at the SIMD's arbiter; the other
            o("s_setprio 2")   # wave of the SIMD fills in from its MFMA-free stretch (measured: +3 % at d = 64)
        mfma(sl)
        if sl == NSLOT - 1:
            o("s_setprio 0")
        ch = list(chunks[sl + 1])
        if sl == 0:
            # this wave's pieces of K_hat(jk) and V(jv): group u+NST-1 = {K_hat(u+NST), V(u+NST-2)}.  The
            # lists are padded with their last entry, so the copies near the end of the list fetch a tile
            # nobody reads instead of being skipped, and every iteration issues the same number of loads.
            o(f"s_mul_i32 s{s['t0']}, s{s['jk']}, s{s['ktile']}")   # bytes between K tiles in memory
            o(f"s_add_u32 s{s['a0']}, s{s['kb0']}, s{s['t0']}")
            o(f"s_addc_u32 s{s['a1']}, s{s['kb1']}, 0")
            o(f"s_mul_i32 s{s['t1']}, s{s['jv']}, {c.V_BYTES}")
            o(f"s_add_u32 s{s['b0']}, s{s['vb0']}, s{s['t1']}")
            o(f"s_addc_u32 s{s['b1']}, s{s['vb1']}, 0")
            # the partial last key block is copied with its rows clamped to the last valid one
            o(f"s_cmp_eq_u32 s{s['jk']}, s{s['jpart']}")
            o(f"s_cbranch_scc1 L_kclamp{tag}_%=")
            ins = []
            for n in range(c.KD):
                piece = [f"s_add_u32 m0, s{s['ldskd']}, {dkbuf * c.K_BYTES + n * 1024 * NWAVE}", "s_nop 0"]
                for x in piece:
                    o(x)
                o(f"global_load_lds_dwordx4 v{c.KSRC + n}, {sp(s, 'a0')}")
                ins += piece + [f"global_load_lds_dwordx4 v{c.KSRCC + n}, {sp(s, 'a0')}"]
            o(f"L_kdone{tag}_%=:")
            late.append((f"L_kclamp{tag}_%=", ins + [f"s_branch L_kdone{tag}_%="]))
        if sl == 1:  # the list entries (older than the operand reads) have arrived
            o(f"v_readfirstlane_b32 s{s['jk']}, v{c.L0}")
            o(f"v_readfirstlane_b32 s{s['jv']}, v{c.L1}")
            o(f"v_readfirstlane_b32 s{s['scnn']}, v{c.L2}")
            if masked:
                o(f"v_readfirstlane_b32 s{s['jn']}, v{c.L3}")
                o(f"s_lshl_b32 s{s['mlim']}, s{s['jn']}, 6")
                o(f"s_add_u32 s{s['t1']}, s{s['u']}, 1")
                o(f"s_cmp_lt_u32 s{s['t1']}, s{s['cnt']}")
                o(f"s_cselect_b32 s{s['mlim']}, s{s['mlim']}, 0x40000000")   # no tile u+1: mask everything
                o(f"s_cselect_b32 s{s['scn']}, s{s['scn']}, 1.0")            # and do not use a scale from past the list
        if 2 <= sl < 2 + c.VD:
            # one V piece per slot; the vector instruction between the M0 write and the copy is the wait
            # state that write needs
            n = sl - 2
            o(f"s_add_u32 m0, s{s['ldsvd']}, {dvbuf * c.V_BYTES + n * 1024 * NWAVE}")
            o(ch.pop(0) if ch else "s_nop 0")
            o(f"global_load_lds_dwordx4 v{c.VSRC + n}, {sp(s, 'b0')}")
        for t in ch:
            o(t)
    assert NSLOT >= 2 + c.VD
    # stage-2 decision of the new tile (kept as a lane mask); has the maximum run away from the reference?
    o(f"s_mov_b64 {sp(s, 'exp0')}, {sp(s, 'ex0')}")   # the tile whose P~ was just made keeps its decision
    o(f"v_cmp_lt_f32_e64 {sp(s, 'ex0')}, s{s['lam2']}, v{T0}")
    o(f"v_cmp_lt_f32 vcc, s{s['rt']}, v{T1}")
    o(f"s_add_u32 s{s['u']}, s{s['u']}, 1")
    o(f"s_mov_b32 s{s['scx']}, s{s['scn']}")
    o(f"s_mov_b32 s{s['scn']}, s{s['scnn']}")
    # Rare, out of line: O *= fO if a move of the reference maximum is still owed to O (the P~V product
    # that was pending when the reference moved has now been added), then the move this step asks for:
    # l and m_ref at once, O one iteration later.
    o(f"s_or_b64 vcc, vcc, {sp(s, 'hf0')}")
    o(f"s_cbranch_scc1 L_slow{tag}_%=")
    o(f"L_after{tag}_%=:")
    ins = [f"s_cmp_eq_u64 {sp(s, 'hf0')}, 0",
           f"s_cbranch_scc1 L_slowb{tag}_%=",
           "s_nop 7", "s_nop 7", "s_nop 7"]               # the step's last MFMA results have landed
    ins += [f"v_mul_f32 v{c.O + i}, v{c.O + i}, v{c.FO}" for i in range(16 * c.NDT)]
    ins += [f"s_mov_b64 {sp(s, 'hf0')}, 0",
            f"L_slowb{tag}_%=:",
            f"v_cmp_lt_f32 vcc, s{s['rt']}, v{T1}",
            "s_cmp_eq_u64 vcc, 0",
            f"s_cbranch_scc1 L_after{tag}_%=",
            f"v_sub_f32 v{T0}, v{c.MR}, v{c.MT}",
            f"v_exp_f32 v{T0}, v{T0}",
            f"v_mov_b32 v{c.MR}, v{c.MT}",
            "s_nop 0",
            f"v_mul_f32 v{c.L}, v{c.L}, v{T0}",
            f"v_mov_b32 v{c.FO}, v{T0}",
            f"s_mov_b64 {sp(s, 'hf0')}, -1",
            "s_nop 3",
            f"s_branch L_after{tag}_%="]
    late.append((f"L_slow{tag}_%=", ins))


def gen_top(c, o, NST):
    """Top of an iteration: the wave's own copy pieces of the group this iteration reads (everything but
    the NST-2 youngest groups) have landed; the barrier makes every wave's pieces visible and frees the
    buffers the previous iteration read."""
    o(f"s_waitcnt vmcnt({c.NDMA * (NST - 2)})")
    o("s_barrier")


def gen_loop(c, NST):
    s = c.sg
    lines = []
    o = lines.append
    period = 2 * NST if NST % 2 else NST  # bodies: one set per value of u mod lcm(2, NST)
    # The loop's position relative to the 32-byte instruction fetch lines must not depend on the size of the
    # code the compiler puts in front of it: at d = 64 (bf16, three stages) a start 20 or 24 bytes into a line
    # is 2-3 % faster than any other multiple of 4 (measured over all eight of them, twice; d = 128 shows
    # no difference).  The padding runs once per item.
    o(".p2align 5")
    for _ in range(5):
        o("s_nop 0")
    o(f"s_mov_b32 s{s['negmagic']}, 0x{0 if c.qk16 else MAGIC_NEG:08x}")   # fp32 scores carry no bias
    o(f"s_mov_b32 s{s['rt']}, 0x{RESCALE_T[c.T_LOG2]:08x}")
    o(f"s_cmp_lg_u32 s{s['exec']}, 0")                 # stage-2 decision of tile 0 as a lane mask
    o(f"s_cselect_b64 {sp(s, 'ex0')}, -1, 0")
    o(f"s_mov_b64 {sp(s, 'exp0')}, 0")                 # nothing is pending: iteration 0 has no P~V
    o(f"s_mov_b64 {sp(s, 'hf0')}, 0")
    o(f"v_mov_b32 v{c.PJ}, s{s['ldsjl']}")
    o(f"v_mov_b32 v{c.PS}, s{s['ldsscl']}")
    o("s_waitcnt vmcnt(0) lgkmcnt(0)")
    late = []  # out-of-line pieces: (label, instructions)

    def body(r, masked, pv, kind):
        # iteration u = r (mod period): K_hat(u+1) in buffer (u+1) % NST, V(u-1) in (u-1) % NST;
        # the new copies go to u % NST (K_hat) and (u-2) % NST (V)
        gen_top(c, o, NST)
        gen_step(c, o, r & 1, NST, (r + 1) % NST, (r - 1) % NST, masked, pv, r % NST, (r - 2) % NST,
                 f"{kind}{r}", late)

    for r in range(period):
        # which body runs iteration u = r (mod period), if any; u has been counted up already
        o(f"L_go{r}_%=:")
        o(f"s_add_u32 s{s['t0']}, s{s['u']}, 1")
        o(f"s_cmp_lt_u32 s{s['t0']}, s{s['ufull']}")
        o(f"s_cbranch_scc0 L_tomask{r}_%=")
        o(f"s_cmp_eq_u64 {sp(s, 'exp0')}, 0")
        o(f"s_cbranch_scc1 L_fastnopv{r}_%=")
        body(r, False, True, "f")
        if r == period - 1:
            o("s_branch L_go0_%=")
    for r in range(period):
        nxt = f"s_branch L_go{(r + 1) % period}_%="
        o(f"L_fastnopv{r}_%=:")
        body(r, False, False, "g")
        o(nxt)
        o(f"L_tomask{r}_%=:")
        o(f"s_cmp_ge_u32 s{s['u']}, s{s['cnt']}")
        o(f"s_cbranch_scc0 L_tomaskb{r}_%=")
        # the drain (u = cnt) runs the pending P~V of the last tile if it was voted in; then the block is done
        o(f"s_cmp_eq_u32 s{s['u']}, s{s['cnt']}")
        o("s_cbranch_scc0 L_exit_%=")
        o(f"s_cmp_eq_u64 {sp(s, 'exp0')}, 0")
        o("s_cbranch_scc1 L_exit_%=")
        o(f"L_tomaskb{r}_%=:")
        o(f"s_cmp_eq_u64 {sp(s, 'exp0')}, 0")
        o(f"s_cbranch_scc1 L_masknopv{r}_%=")
        body(r, True, True, "m")
        o(nxt)
        o(f"L_masknopv{r}_%=:")
        body(r, True, False, "n")
        o(nxt)
    for label, ins in late:
        o(label + ":")
        for i in ins:
            o(i)
    o("L_exit_%=:")
    o("s_waitcnt vmcnt(0)")                    # no copy of this wave may still be writing LDS
    o("s_nop 7"); o("s_nop 7"); o("s_nop 7")   # the last MFMA results have landed
    return lines


def clobbers(c):
    v = list(range(c.RG, c.RG + 4 * RING)) + list(range(c.T, c.T + 3)) + [c.CX, c.L3, c.PJ, c.PS]
    sg = [c.sg[n] for n in ("negmagic rt scnn t0 t1 a0 a1 b0 b1 jn mlim ex0 ex1 exp0 exp1 hf0 hf1").split()]
    return [f"v{i}" for i in v] + [f"s{i}" for i in sg] + ["vcc", "scc", "memory"]


def gen_function(c, NST):
    s = c.sg
    body = gen_loop(c, NST)
    dtn = {"bf16": "SPARGE_BF16", "f16": "SPARGE_F16", "fp8": "PV_FP8"}[c.dt]
    qkn = "true" if c.qk16 else "false"
    io_names = "u jk jv scn scx pv".split()                       # read and written by the block
    in_names = "exec jpart cnt ufull ldskd ldsvd ldsjl ldsscl lam2 ktile".split()
    floats = {"scn", "scx", "lam2"}
    out = []
    w = out.append
    w(f"// head dimension {c.D}, {c.dt}{', 16-bit Q K^T' if c.qk16 else ''}, {NST} LDS stages: {c.NVGPR} VGPRs pinned, no AGPRs")
    w(f"template <> struct FastLoop<{c.D}, {dtn}, {NST}, {qkn}> {{")
    w("    template <class St>")
    w("    static __device__ __forceinline__ void run(St& w, const v16i& magic, FastLoopArgs& p) {")
    # scalar operands go through readfirstlane copies: the register allocator then knows they are uniform
    for n in io_names + in_names:
        if n in floats:
            w(f"        float {n}_ = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(p.{n})));")
        else:
            w(f"        int {n}_ = __builtin_amdgcn_readfirstlane(static_cast<int>(p.{n}));")
    w("        asm volatile(")
    for l in body:
        w(f'            "{l}\\n"')
    outs, ins = [], []
    for dt in range(c.NDT):
        outs.append(f'"+{{{vr(c.O + 16 * dt, 16)}}}"(w.O[{dt}])')
    for b in range(2):
        for kh in range(2):
            outs.append(f'"+{{{vr(c.S[b] + 16 * kh, 16)}}}"(w.S[{b}][{kh}])')
        for ks in range(c.NP):
            outs.append(f'"+{{{vr(c.P[b] + 4 * ks, 4)}}}"(w.P[{b}][{ks}])')
    for reg, expr in ((c.MT, "w.m_true"), (c.MR, "w.m_ref"), (c.L, "w.l")):
        outs.append(f'"+{{v{reg}}}"({expr})')
    outs.append(f'"+{{v{c.FO}}}"(p.fo)')
    for n in io_names:
        outs.append(f'"+{{s{s[n]}}}"({n}_)')
    for st in range(c.NSTEP):
        ins.append(f'"{{{vr(c.Q + 4 * st, 4)}}}"(w.qf[{st}])')
    if not c.qk16:
        ins.append(f'"{{{vr(c.MG, 16)}}}"(magic)')
    ins.append(f'"{{v{c.INV}}}"(p.inval)')
    ins.append(f'"{{v{c.ROWLIM}}}"(p.rowlim)')
    for st in range(c.NSTEP):
        ins.append(f'"{{v{c.KA + st}}}"(p.k_adr[{st}])')
    for ks in range(4):
        ins.append(f'"{{v{c.VA + ks}}}"(p.v_adr[{ks}])')
    for n in range(c.KD):
        ins.append(f'"{{v{c.KSRC + n}}}"(p.k_src[{n}])')
        ins.append(f'"{{v{c.KSRCC + n}}}"(p.k_src_clamped[{n}])')
    for n in range(c.VD):
        ins.append(f'"{{v{c.VSRC + n}}}"(p.v_src[{n}])')
    ins.append(f'"{{{sp(s, "kb0")}}}"(p.kbase)')
    ins.append(f'"{{{sp(s, "vb0")}}}"(p.vbase)')
    for n in in_names:
        ins.append(f'"{{s{s[n]}}}"({n}_)')
    w("            : " + ",\n              ".join(outs))
    w("            : " + ",\n              ".join(ins))
    w("            : " + ", ".join(f'"{x}"' for x in clobbers(c)) + ");")
    for n in ("u", "pv"):
        w(f"        p.{n} = {n}_;")
    w("    }")
    w("};")
    w("")
    return out


def generate():
    """The text of attn_loop_gfx950.inc."""
    out = ["// GENERATED by gen_attn_loop.py -- do not edit; edit the generator and run it again.",
           "// Steady-state iterations of the sparse flash loop as hand-scheduled gfx950 assembly.", ""]
    for D in (64, 128):
        for dt in ("f16", "bf16", "fp8"):
            for NST in (2, 3):
                out += gen_function(Cfg(D, dt), NST)
        for dt in ("f16", "bf16"):
            for NST in (2, 3):
                out += gen_function(Cfg(D, dt, qk16=True), NST)
    return "\n".join(out)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    text = generate()
    with open(os.path.join(here, "attn_loop_gfx950.inc"), "w") as f:
        f.write(text)
    print(f"wrote attn_loop_gfx950.inc ({text.count(chr(10)) + 1} lines)")


if __name__ == "__main__":
    main()
