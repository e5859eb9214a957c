#!/usr/bin/env python3
"""Writes attn_loop_gfx950.inc: the steady-state iterations of the sparse flash loop (Alg. 1 lines
9-17 of arXiv 2502.18137 on full, unmasked tiles) as one hand-scheduled gfx950 assembly block per
(head dimension, 16-bit type), wrapped in a C++ function that attn.hip includes.

    python gen_attn_loop.py            # rewrites attn_loop_gfx950.inc next to this file

Why assembly: the matrix pipe and the vector ALU of a SIMD only overlap when MFMA and vector
instructions alternate at fine grain inside one wave, and the wave owns its SIMD alone (512
registers), so the instruction order and the register assignment are the design.  The block is
entered at an iteration boundary of the kernel's main loop and leaves at one; everything irregular
(first and last tiles, tiles that need element masks, skipped P~V products) stays in C++.

State at the boundary "top of iteration u" (u >= 1; tiles are positions in the row's kept list):
  group A: P~ of tile u-1 waits for its P~V product (execA = its stage-2 decision);
  group B: biased scores S of tile u-1 wait for their softmax (scB = their dequantization scale,
           execB = their stage-2 decision); all row statistics are up to date;
  LDS:     K_hat(u) and V(u-1) have been requested NST-1 iterations ago.
Iteration u:  wait for own copies, barrier, request K_hat(u+NST-1) and V(u+NST-2), then
  step 1: softmax of (B, u-1) on the vector ALU  |  MFMA: scores of (A, u), P~V of (A, u-1)
  step 2: softmax of (A, u)                      |  MFMA: scores of (B, u), P~V of (B, u-1)
Each step is a sequence of slots: operand read (LDS, three slots ahead), one MFMA, a chunk of the
softmax.  The row maximum of the fresh scores, the stage-2 test (Alg. 1 line 15) and the test
whether the reference maximum must move follow at the end of the step.
"""
import os

MAGIC_NEG = 0xCB400000  # bit pattern of -12582912.0f = -(1.5 * 2^23)
RESCALE_T = 0x41000000  # 8.0f
LA = 3                  # operand reads run this many slots ahead
RING = LA + 1
PRE_UNITS = 14          # vector work placed before the first MFMA of a step (covers the LDS latency)


class Cfg:
    def __init__(self, D, dt):
        self.D, self.dt = D, dt
        self.NSTEP = self.NDT = D // 32
        self.NQK, self.NPV = 2 * self.NSTEP, 4 * self.NDT
        self.NSLOT = self.NQK + self.NPV
        self.K_BYTES, self.V_BYTES = 64 * D, D * 128
        self.KD, self.VD = self.K_BYTES // 2048, self.V_BYTES // 2048  # copies per wave and tile
        self.NDMA = self.KD + self.VD
        # ---- AGPRs ----
        self.AO, self.BO = 0, 16 * self.NDT
        self.AQ = 32 * self.NDT
        self.BQ = self.AQ + 4 * self.NSTEP
        # ---- VGPRs (pinned) ----
        self.BS, self.AS, self.AP, self.BP, self.MG, self.RG = 32, 64, 96, 112, 128, 144
        (self.A_MT, self.A_MR, self.A_L, self.B_MT, self.B_MR, self.B_L, self.A_INV, self.B_INV) = range(160, 168)
        self.KOFF, self.KA, self.VOFF, self.VA = 168, 172, 176, 180
        self.KSRC, self.VSRC = 184, 188
        self.T = 196          # 8 temporaries
        self.CX, self.MLOC, self.L0, self.L1 = 204, 205, 206, 207
        # ---- SGPRs (pinned) ----
        names = ("u uend kb0 kb1 vb0 vb1 ldsk ldskd ldsv ldsvd ldsjl ldsscl lam2 execA execB pvA pvB scB "
                 "jk jv scn bk negmagic rt jkn scnn t0 t1 t2 t3 kcur vcur dk dv a0 a1").split()
        self.S = {n: 36 + i for i, n in enumerate(names)}


class Group:
    def __init__(self, c, which):
        a = which == "A"
        self.S, self.P = (c.AS, c.AP) if a else (c.BS, c.BP)
        self.O, self.Q = (c.AO, c.AQ) if a else (c.BO, c.BQ)
        self.mt, self.mr, self.l, self.inv = (c.A_MT, c.A_MR, c.A_L, c.A_INV) if a else (c.B_MT, c.B_MR, c.B_L, c.B_INV)
        self.pv = c.S["pvA" if a else "pvB"]
        self.ex = c.S["execA" if a else "execB"]
        self.name = which


def vr(b, n=1):
    return f"v{b}" if n == 1 else f"v[{b}:{b + n - 1}]"


def ar(b, n=1):
    return f"a{b}" if n == 1 else f"a[{b}:{b + n - 1}]"


def gen_step(c, o, X, Y, scx, lbl, prefetch):
    """Softmax of X's pending scores | scores of Y's next tile and Y's pending P~V; then Y's row maximum."""
    s = c.S
    T0, T1, T2 = c.T, c.T + 1, c.T + 2

    def read(sl):
        dst = c.RG + 4 * (sl % RING)
        if sl < c.NQK:
            kh, st = sl % 2, sl // 2
            o(f"ds_read_b128 {vr(dst, 4)}, v{c.KA + st} offset:{kh * 32 * c.D}")
        else:
            ks, dt = divmod(sl - c.NQK, c.NDT)
            o(f"ds_read_b128 {vr(dst, 4)}, v{c.VA + ks} offset:{dt * 4096}")

    def mfma(sl):
        src = c.RG + 4 * (sl % RING)
        if sl < c.NQK:
            kh, st = sl % 2, sl // 2
            d = Y.S + 16 * kh
            acc = vr(c.MG, 16) if st == 0 else vr(d, 16)
            o(f"v_mfma_i32_32x32x32_i8 {vr(d, 16)}, {vr(src, 4)}, {ar(Y.Q + 4 * st, 4)}, {acc}")
        else:
            ks, dt = divmod(sl - c.NQK, c.NDT)
            a = Y.O + 16 * dt
            o(f"v_mfma_f32_32x32x16_{c.dt} {ar(a, 16)}, {vr(src, 4)}, {vr(Y.P + 4 * ks, 4)}, {ar(a, 16)}")

    # ---- the vector instruction stream of the step: (text, issue units) ----
    ops = []
    x = lambda e: X.S + e
    F = lambda e: ops.append((f"v_fma_f32 v{x(e)}, v{x(e)}, s{scx}, v{c.CX}", 1))
    E = lambda e: ops.append((f"v_exp_f32 v{x(e)}, v{x(e)}", 2))
    A = lambda e: ops.append((f"v_add_f32 v{X.l}, v{X.l}, v{x(e)}", 1))
    C = lambda w: ops.append((f"v_cvt_pk_{c.dt}_f32 v{X.P + w}, v{x(2 * w)}, v{x(2 * w + 1)}", 1))
    for k in range(16):
        F(2 * k); F(2 * k + 1); E(2 * k); E(2 * k + 1)
        if k:
            A(2 * k - 2); A(2 * k - 1); C(k - 1)
    A(30); A(31); C(15)
    n_exp_ops = len(ops)
    # row maximum of Y's fresh scores (biased integers compare like the scores themselves)
    y = lambda e: Y.S + e
    chains = []
    for t, base in ((T0, y(0)), (T1, y(16))):
        ch = [f"v_max3_i32 v{t}, v{base}, v{base + 1}, v{base + 2}"]
        ch += [f"v_max3_i32 v{t}, v{t}, v{base + i}, v{base + i + 1}" for i in range(3, 15, 2)]
        ch += [f"v_max_i32 v{t}, v{t}, v{base + 15}"]
        chains.append(ch)
    for a_, b_ in zip(*chains):
        ops.append((a_, 1)); ops.append((b_, 1))
    ops += [(f"v_max_i32 v{T0}, v{T0}, v{T1}", 1),
            (f"v_add_f32 v{T0}, s{s['negmagic']}, v{T0}", 1),      # biased integer (as float) -> score sum
            (f"v_mul_f32 v{T0}, s{s['scn']}, v{T0}", 1),           # -> log2-domain score
            (f"v_mov_b32 v{T1}, v{T0}", 1),
            ("s_nop 1", 1),
            (f"v_permlane32_swap_b32 v{T0}, v{T1}", 1),            # exchange with the lane holding the other 16 keys
            ("s_nop 1", 1),
            (f"v_max_f32 v{c.MLOC}, v{T0}, v{T1}", 1),
            (f"v_max_f32 v{Y.mt}, v{Y.mt}, v{c.MLOC}", 1),         # new running maximum
            (f"v_sub_f32 v{T0}, v{c.MLOC}, v{Y.mt}", 1),
            (f"v_sub_f32 v{T1}, v{Y.mt}, v{Y.mr}", 1),
            (f"v_add_f32 v{T0}, v{T0}, v{Y.inv}", 1),              # rows past N: -inf
            (f"v_add_f32 v{T1}, v{T1}, v{Y.inv}", 1)]
    first_max = n_exp_ops  # index of the first instruction that reads Y's fresh scores
    NTAIL = 13             # the dependent chain at the end stays behind the last MFMA

    body = ops[:-NTAIL]
    total = sum(u for _, u in body)
    per_slot = (total - PRE_UNITS) / c.NSLOT
    # chunk 0 runs before the first MFMA, chunk sl + 1 after MFMA sl
    chunks, acc_u, idx = [], 0.0, 0
    for k in range(c.NSLOT + 1):
        target = PRE_UNITS + per_slot * k
        ch = []
        while idx < len(body) and (acc_u + body[idx][1] / 2 <= target or k == c.NSLOT):
            ch.append(idx); acc_u += body[idx][1]; idx += 1
        chunks.append(ch)
    chunks[-1] += list(range(len(body), len(ops)))
    # the scores of Y are complete a few slots after the last Q K^T MFMA
    for k, ch in enumerate(chunks):
        if any(i >= first_max for i in ch):
            assert k - 1 >= c.NQK + 1, "row-maximum work scheduled too early"
            break
    assert len(chunks[-1]) >= 12, "too little vector work behind the last MFMA"

    o(f"; ---- {lbl}: softmax of group {X.name} | MFMAs for group {Y.name}")
    if prefetch:  # list entries of the next iteration (older than every operand read of this step)
        o(f"s_add_u32 s{s['t0']}, s{s['u']}, {prefetch}")
        o(f"s_lshl_b32 s{s['t0']}, s{s['t0']}, 1")
        o(f"s_add_u32 s{s['t0']}, s{s['t0']}, s{s['ldsjl']}")
        o(f"s_lshl_b32 s{s['t1']}, s{s['u']}, 2")
        o(f"s_add_u32 s{s['t1']}, s{s['t1']}, s{s['ldsscl']}")
        o(f"v_mov_b32 v{c.L0}, s{s['t0']}")
        o(f"v_mov_b32 v{c.L1}, s{s['t1']}")
        o(f"ds_read_u16 v{c.L0}, v{c.L0}")
        o(f"ds_read_b32 v{c.L1}, v{c.L1} offset:4")
    for sl in range(LA):
        read(sl)
    o(f"v_mov_b32 v{T2}, s{s['negmagic']}")
    o(f"v_fma_f32 v{c.CX}, v{T2}, s{scx}, -v{X.mr}")   # -(bias * scale) - reference maximum
    o(f"s_add_u32 s{Y.pv}, s{Y.pv}, 1")
    for i in chunks[0]:
        o(ops[i][0])
    for sl in range(c.NSLOT):
        if sl + LA < c.NSLOT:
            read(sl + LA)
        o(f"s_waitcnt lgkmcnt({min(LA, c.NSLOT - 1 - sl)})")
        mfma(sl)
        for i in chunks[sl + 1]:
            o(ops[i][0])
    # stage-2 decision of Y's new tile and "has the maximum run away from the reference"
    o(f"v_cmp_lt_f32 vcc, s{s['lam2']}, v{T0}")
    o(f"s_cmp_lg_u64 vcc, 0")
    o(f"s_cselect_b32 s{Y.ex}, 1, 0")
    if prefetch:
        o(f"v_readfirstlane_b32 s{s['jkn']}, v{c.L0}")
        o(f"v_readfirstlane_b32 s{s['scnn']}, v{c.L1}")
    o(f"v_cmp_lt_f32 vcc, s{s['rt']}, v{T1}")
    o(f"s_cbranch_vccnz L_rescale{Y.name}_%=")
    o(f"L_after{Y.name}_%=:")


def gen_rescale(c, o, G, cont):
    """Move the reference maximum of group G up to its running maximum: O, l *= 2^(m_ref - m)."""
    T = c.T
    F = c.T + 7
    o(f"L_rescale{G.name}_%=:")
    o("s_nop 7"); o("s_nop 7"); o("s_nop 7")   # the group's last MFMA results have landed
    o(f"v_sub_f32 v{F}, v{G.mr}, v{G.mt}")
    o(f"v_exp_f32 v{F}, v{F}")
    o("s_nop 1")
    n = 16 * c.NDT
    for i0 in range(0, n, 4):
        for j in range(4):
            o(f"v_accvgpr_read_b32 v{T + j}, a{G.O + i0 + j}")
        for j in range(4):
            o(f"v_mul_f32 v{T + j}, v{T + j}, v{F}")
        for j in range(4):
            o(f"v_accvgpr_write_b32 a{G.O + i0 + j}, v{T + j}")
    o(f"v_mul_f32 v{G.l}, v{G.l}, v{F}")
    o(f"v_mov_b32 v{G.mr}, v{G.mt}")
    o("s_nop 3")
    o(f"s_branch {cont}")


def gen_loop(c, NST):
    s = c.S
    lines = []
    o = lines.append
    A, B = Group(c, "A"), Group(c, "B")
    wait = c.NDMA * (NST - 2)

    def mod_nst(dst, src, add):
        o(f"s_add_u32 s{dst}, s{src}, {add}")
        o(f"s_cmp_ge_u32 s{dst}, {NST}")
        o(f"s_cselect_b32 s{s['t3']}, {NST}, 0")
        o(f"s_sub_u32 s{dst}, s{dst}, s{s['t3']}")

    o(f"s_mov_b32 s{s['negmagic']}, 0x{MAGIC_NEG:08x}")
    o(f"s_mov_b32 s{s['rt']}, 0x{RESCALE_T:08x}")
    o("s_waitcnt vmcnt(0) lgkmcnt(0)")
    o("s_branch L_check_%=")
    o("L_top_%=:")
    o(f"s_waitcnt vmcnt({wait})")
    o("s_barrier")
    # ---- buffers of this iteration: K_hat(u) in bk, V(u-1) in bk-1; copies go to bk-1 (K) and bk-2 (V)
    mod_nst(s['t0'], s['bk'], NST - 1)
    mod_nst(s['t1'], s['bk'], NST - 2 if NST > 2 else 0)
    o(f"s_mul_i32 s{s['kcur']}, s{s['bk']}, {c.K_BYTES}")
    o(f"s_add_u32 s{s['kcur']}, s{s['kcur']}, s{s['ldsk']}")
    o(f"s_mul_i32 s{s['vcur']}, s{s['t0']}, {c.V_BYTES}")
    o(f"s_add_u32 s{s['vcur']}, s{s['vcur']}, s{s['ldsv']}")
    o(f"s_mul_i32 s{s['dk']}, s{s['t0']}, {c.K_BYTES}")
    o(f"s_add_u32 s{s['dk']}, s{s['dk']}, s{s['ldskd']}")
    o(f"s_mul_i32 s{s['dv']}, s{s['t1']}, {c.V_BYTES}")
    o(f"s_add_u32 s{s['dv']}, s{s['dv']}, s{s['ldsvd']}")
    # ---- LDS-DMA: this wave's pieces of K_hat(jk) and V(jv)
    o(f"s_mul_i32 s{s['t0']}, s{s['jk']}, {c.K_BYTES}")
    o(f"s_add_u32 s{s['a0']}, s{s['kb0']}, s{s['t0']}")
    o(f"s_addc_u32 s{s['a1']}, s{s['kb1']}, 0")
    for n in range(c.KD):
        o(f"s_add_u32 m0, s{s['dk']}, {n * 2048}")
        o("s_nop 0")
        o(f"global_load_lds_dwordx4 v{c.KSRC + n}, s[{s['a0']}:{s['a1']}]")
    o(f"s_mul_i32 s{s['t0']}, s{s['jv']}, {c.V_BYTES}")
    o(f"s_add_u32 s{s['a0']}, s{s['vb0']}, s{s['t0']}")
    o(f"s_addc_u32 s{s['a1']}, s{s['vb1']}, 0")
    for n in range(c.VD):
        o(f"s_add_u32 m0, s{s['dv']}, {n * 2048}")
        o("s_nop 0")
        o(f"global_load_lds_dwordx4 v{c.VSRC + n}, s[{s['a0']}:{s['a1']}]")
    # ---- operand addresses of this iteration
    for st in range(c.NSTEP):
        o(f"v_add_u32 v{c.KA + st}, s{s['kcur']}, v{c.KOFF + st}")
    for ks in range(4):
        o(f"v_add_u32 v{c.VA + ks}, s{s['vcur']}, v{c.VOFF + ks}")
    gen_step(c, o, B, A, s['scB'], "step 1", 0)
    gen_step(c, o, A, B, s['scn'], "step 2", NST)
    # ---- next iteration
    o(f"s_add_u32 s{s['u']}, s{s['u']}, 1")
    o(f"s_mov_b32 s{s['scB']}, s{s['scn']}")
    o(f"s_mov_b32 s{s['scn']}, s{s['scnn']}")
    o(f"s_mov_b32 s{s['jv']}, s{s['jk']}")
    o(f"s_mov_b32 s{s['jk']}, s{s['jkn']}")
    mod_nst(s['bk'], s['bk'], 1)
    o("L_check_%=:")
    o(f"s_cmp_ge_u32 s{s['u']}, s{s['uend']}")
    o("s_cbranch_scc1 L_exit_%=")
    o(f"s_and_b32 s{s['t0']}, s{s['execA']}, s{s['execB']}")
    o(f"s_cmp_eq_u32 s{s['t0']}, 0")
    o("s_cbranch_scc0 L_top_%=")
    o("s_branch L_exit_%=")
    gen_rescale(c, o, A, "L_afterA_%=")
    gen_rescale(c, o, B, "L_afterB_%=")
    o("L_exit_%=:")
    o("s_nop 7"); o("s_nop 7"); o("s_nop 7")
    return lines


def clobbers(c):
    v = list(range(c.AS, c.AS + 32)) + list(range(c.BP, c.BP + 16)) + list(range(c.RG, c.RG + 16))
    v += list(range(c.KA, c.KA + 4)) + list(range(c.VA, c.VA + 4)) + list(range(c.T, c.T + 8))
    v += [c.CX, c.MLOC, c.L0, c.L1]
    sg = [c.S[n] for n in "negmagic rt jkn scnn t0 t1 t2 t3 kcur vcur dk dv a0 a1".split()]
    return [f"v{i}" for i in v] + [f"s{i}" for i in sg] + ["vcc", "scc", "memory"]


def gen_function(c, NST):
    s = c.S
    body = gen_loop(c, NST)
    dtn = "SPARGE_BF16" if c.dt == "bf16" else "SPARGE_F16"
    out = []
    w = out.append
    w(f"// head dimension {c.D}, {c.dt}, {NST} LDS stages")
    w(f"template <> struct FastLoop<{c.D}, {dtn}, {NST}> {{")
    w("    template <class Grp>")
    w("    static __device__ __forceinline__ void run(Grp& A, Grp& B, const v16i& magic, FastLoopArgs& p) {")
    w("        asm volatile(")
    for l in body:
        w(f'            "{l}\\n"')
    # operands
    outs, ins = [], []
    for dt in range(c.NDT):
        outs.append(f'"+{{{ar(c.AO + 16 * dt, 16)}}}"(A.O[{dt}])')
        outs.append(f'"+{{{ar(c.BO + 16 * dt, 16)}}}"(B.O[{dt}])')
    for kh in range(2):
        outs.append(f'"+{{{vr(c.BS + 16 * kh, 16)}}}"(B.S[{kh}])')
    for ks in range(4):
        outs.append(f'"+{{{vr(c.AP + 4 * ks, 4)}}}"(A.P[{ks}])')
    for reg, expr in ((c.A_MT, "A.m_true"), (c.A_MR, "A.m_ref"), (c.A_L, "A.l"), (c.B_MT, "B.m_true"),
                      (c.B_MR, "B.m_ref"), (c.B_L, "B.l")):
        outs.append(f'"+{{v{reg}}}"({expr})')
    for n in "u bk jk jv scn scB execA execB pvA pvB".split():
        outs.append(f'"+{{s{s[n]}}}"(p.{n})')
    for st in range(c.NSTEP):
        ins.append(f'"{{{ar(c.AQ + 4 * st, 4)}}}"(A.qf[{st}])')
        ins.append(f'"{{{ar(c.BQ + 4 * st, 4)}}}"(B.qf[{st}])')
    ins.append(f'"{{{vr(c.MG, 16)}}}"(magic)')
    ins.append(f'"{{v{c.A_INV}}}"(p.invalA)')
    ins.append(f'"{{v{c.B_INV}}}"(p.invalB)')
    for st in range(c.NSTEP):
        ins.append(f'"{{v{c.KOFF + st}}}"(p.k_off[{st}])')
    for ks in range(4):
        ins.append(f'"{{v{c.VOFF + ks}}}"(p.v_off[{ks}])')
    for n in range(c.KD):
        ins.append(f'"{{v{c.KSRC + n}}}"(p.k_src[{n}])')
    for n in range(c.VD):
        ins.append(f'"{{v{c.VSRC + n}}}"(p.v_src[{n}])')
    ins.append(f'"{{s[{s["kb0"]}:{s["kb1"]}]}}"(p.kbase)')
    ins.append(f'"{{s[{s["vb0"]}:{s["vb1"]}]}}"(p.vbase)')
    for n in "uend ldsk ldskd ldsv ldsvd ldsjl ldsscl lam2".split():
        ins.append(f'"{{s{s[n]}}}"(p.{n})')
    w("            : " + ",\n              ".join(outs))
    w("            : " + ",\n              ".join(ins))
    w("            : " + ", ".join(f'"{x}"' for x in clobbers(c)) + ");")
    w("    }")
    w("};")
    w("")
    return out


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    out = ["// GENERATED by gen_attn_loop.py -- do not edit; edit the generator and run it again.",
           "// Steady-state iterations of the sparse flash loop as hand-scheduled gfx950 assembly.", ""]
    for D in (64, 128):
        for dt in ("f16", "bf16"):
            for NST in (2, 3):
                out += gen_function(Cfg(D, dt), NST)
    with open(os.path.join(here, "attn_loop_gfx950.inc"), "w") as f:
        f.write("\n".join(out))
    print(f"wrote attn_loop_gfx950.inc ({len(out)} lines)")


if __name__ == "__main__":
    main()
