#!/usr/bin/env python3
"""Writes attn_pipe_asm.h: the instruction streams of the pipelined attention kernel.

Run after changing anything here:  python3 gen_pipe_asm.py   (the header is
committed; the build does not run this script).

The pipelined kernel keeps its large operands in registers the compiler is told
never to touch (the kernel is compiled with a cap of 64 vector registers), so
every instruction that reads or writes them is emitted here with literal
register names:

  v[64:127]   S of even tiles   S[t][kb][v]: 4 key sub-blocks x 16 accumulators
  v[128:191]  S of odd tiles
  v[192:223]  P of even tiles   32 registers = 32 bf16 pairs, pair pi = logits 2pi, 2pi+1
  v[224:255]  P of odd tiles
  a[64:95]    K operands of one k-slab, two stages of 4 key sub-blocks x 4 registers
  a[96:127]   V^T operands of one 16-key slab, two stages of 4 d blocks x 4 registers
  a[128:191]  O^T: 4 d blocks x 16 accumulators
  a[192:223]  Q^T: 8 k-slabs x 4 registers

Hazards the assembler does not check and that the streams below respect:
  * a transcendental result is not read by the next instruction;
  * MFMA results are read by other instructions only after >= 11 issue slots;
  * one instruction sits between a write of M0 and the LDS-DMA that uses it;
  * the result of a dot instruction is not touched by an instruction of another
    kind in the next 4 issue slots (also not by what the compiler places after a block).
"""
import os

FB_PAIRS = 12  # pairs of a tile's logits whose softmax rides on the PV product (the rest rides on QK)


def S(t, idx):
    return f"v{64 + 64 * t + idx}"


def St(t, kb):
    b = 64 + 64 * t + 16 * kb
    return f"v[{b}:{b + 15}]"


def Pr(t, pi):
    return f"v{192 + 32 * t + pi}"


def Pt(t, j):  # B operand of 16-key slab j
    b = 192 + 32 * t + 4 * j
    return f"v[{b}:{b + 3}]"


def Ka(st, kb):
    b = 64 + 16 * st + 4 * kb
    return f"a[{b}:{b + 3}]"


def Va(st, db, half):
    b = 96 + 16 * st + 4 * db + 2 * half
    return f"a[{b}:{b + 1}]"


def Vt(st, db):
    b = 96 + 16 * st + 4 * db
    return f"a[{b}:{b + 3}]"


def Ot(db):
    b = 128 + 16 * db
    return f"a[{b}:{b + 15}]"


def Qt(s):
    b = 192 + 4 * s
    return f"a[{b}:{b + 3}]"


class Op:
    def __init__(self, text, slots=1, trans_dst=None, reads=()):
        self.text, self.slots, self.trans_dst, self.reads = text, slots, trans_dst, tuple(reads)


def softmax_ops(t, pairs):
    """exp2(sc * s - m) of the given logit pairs of tile t, rounded to bf16 into P,
    row sums of the rounded values into l0 / l1.  Software-pipelined by one pair."""
    ops = []
    prev = None
    for n, pi in enumerate(pairs):
        ta, tb = f"%[t{2 * (n % 2)}]", f"%[t{2 * (n % 2) + 1}]"
        ops.append(Op(f"v_fma_f32 {ta}, {S(t, 2 * pi)}, %[sc], -%[m]"))
        ops.append(Op(f"v_fma_f32 {tb}, {S(t, 2 * pi + 1)}, %[sc], -%[m]"))
        if prev:
            ops += finish_pair(t, *prev)
        ops.append(Op(f"v_exp_f32 {ta}, {ta}", 2, trans_dst=ta))
        ops.append(Op(f"v_exp_f32 {tb}, {tb}", 2, trans_dst=tb))
        prev = (pi, ta, tb)
    if prev:
        ops.append(Op("s_nop 0"))
        ops += finish_pair(t, *prev)
        ops.append(Op("s_nop 3"))  # the compiler may touch l0 / l1 right after the block
    return ops


def finish_pair(t, pi, ta, tb):
    return [Op(f"v_cvt_pk_bf16_f32 {Pr(t, pi)}, {ta}, {tb}", reads=(ta, tb)),
            Op(f"v_dot2c_f32_bf16 %[l{pi % 2}], 0x3f803f80, {Pr(t, pi)}")]


def max_ops(t):
    """Maximum of this lane's 64 logits of tile t into %[mx] (uses %[t0])."""
    ops = [Op(f"v_max3_f32 %[mx], {S(t, 0)}, {S(t, 1)}, {S(t, 2)}"),
           Op(f"v_max3_f32 %[t0], {S(t, 3)}, {S(t, 4)}, {S(t, 5)}")]
    acc = ["%[mx]", "%[t0]"]
    i, k = 6, 0
    while i < 64:
        ops.append(Op(f"v_max3_f32 {acc[k]}, {S(t, i)}, {S(t, i + 1)}, {acc[k]}"))
        i += 2
        k ^= 1
    ops.append(Op("v_max_f32 %[mx], %[mx], %[t0]"))
    return ops


def check_trans(ops):
    """No VALU instruction reads a transcendental result in the slot right after it."""
    for a, b in zip(ops, ops[1:]):
        if a.trans_dst and a.trans_dst in b.reads:
            raise SystemExit(f"trans hazard: {a.text} -> {b.text}")


def weave(anchors, valu, pre=0):
    """anchors: list of (lines before the MFMA, MFMA line, lines after it); valu: Ops spread
    by issue slots over the gaps after the MFMAs; the first `pre` Ops go before everything."""
    lines = [o.text for o in valu[:pre]]
    rest = valu[pre:]
    total = sum(o.slots for o in rest)
    n = len(anchors)
    done = 0
    k = 0
    for a, (before, mfma, after) in enumerate(anchors):
        lines += before
        lines.append(mfma)
        goal = total * (a + 1) / n
        while k < len(rest) and (done + rest[k].slots / 2 <= goal or a == n - 1):
            lines.append(rest[k].text)
            done += rest[k].slots
            k += 1
        lines += after
    check_trans(valu)  # MFMAs and other instructions in between only add distance
    return lines


def dma(j):
    return [f"s_add_u32 m0, %[dl], {j * 4096}", f"s_add_u32 %[st], %[ds], {j * 4096}",
            "buffer_load_dwordx4 %[dv], %[dr], %[st] offen lds"]


def k_reads(st, s, koff):
    return [f"ds_read_b128 {Ka(st, kb)}, %[ka{s}] offset:{koff + kb * 8192}" for kb in range(4)]


def v_reads(st, j, voff):
    out = []
    for db in range(4):
        out.append(f"ds_read_b64_tr_b16 {Va(st, db, 0)}, %[va{db}] offset:{voff + j * 4096}")
        out.append(f"ds_read_b64_tr_b16 {Va(st, db, 1)}, %[va{db}] offset:{voff + j * 4096 + 1024}")
    return out


def qk_anchors(ty, koff, with_dma):
    """8 k-slabs of S_ty = K Q^T; operands of slab s+1 are read while slab s multiplies."""
    anchors = []
    for s in range(8):
        st = s & 1
        for kb in range(4):
            before, after = [], []
            if kb == 0:
                if s < 7:
                    before += k_reads(1 - st, s + 1, koff)
                    before.append("s_waitcnt lgkmcnt(4)")
                else:
                    before.append("s_waitcnt lgkmcnt(0)")
            c = "0" if s == 0 else St(ty, kb)
            mfma = f"v_mfma_f32_32x32x16_bf16 {St(ty, kb)}, {Ka(st, kb)}, {Qt(s)}, {c}"
            if with_dma and kb == 1:
                after += dma(s)
            anchors.append((before, mfma, after))
    return anchors


def pv_anchors(tx, voff, slabs, dma_plan=None):
    """16-key slabs of O^T += V^T P_tx; operands of slab j+2 are read once slab j has issued."""
    anchors = []
    for j in slabs:
        st = j & 1
        for db in range(4):
            before, after = [], []
            if db == 0:
                before.append("s_waitcnt lgkmcnt(8)" if j < 7 else "s_waitcnt lgkmcnt(0)")
            mfma = f"v_mfma_f32_32x32x16_bf16 {Ot(db)}, {Vt(st, db)}, {Pt(tx, j)}, {Ot(db)}"
            if dma_plan and (j, db) in dma_plan:
                after += dma(dma_plan[(j, db)])
            if db == 3 and j + 2 < 8:
                after += v_reads(st, j + 2, voff)
            anchors.append((before, mfma, after))
    return anchors


ALL_CLOBBERS = ", ".join([f'"v{i}"' for i in range(64, 256)] + [f'"a{i}"' for i in range(64, 224)])

T4_OUT = '[t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3)'
SM_OUT = f'{T4_OUT}, [l0] "+v"(l0), [l1] "+v"(l1)'
SM_IN = '[sc] "v"(sc), [m] "v"(m)'
DMA_OUT = '[st] "=&s"(st)'
DMA_IN = '[dr] "s"(rsrc), [dv] "v"(lane_off), [ds] "s"(soff), [dl] "s"(lds)'
DMA_SIG = "const u32x4 &rsrc, uint32_t lane_off, uint32_t soff, uint32_t lds"


def emit(lines, outs, ins, extra_clobbers=""):
    body = "\n".join(f'        "{l}\\n\\t"' for l in lines)
    return f"    asm volatile(\n{body}\n        : {outs}\n        : {ins}\n        : PIPE_PINNED{extra_clobbers});\n"


def by_parity(sig, pre, make):
    out = f"template <int PAR>\n__device__ __forceinline__ void {sig} {{\n{pre}"
    out += "  if constexpr (PAR == 0) {\n" + make(0) + "  } else {\n" + make(1) + "  }\n}\n\n"
    return out


def main():
    o = []
    o.append("// Instruction streams of the pipelined attention kernel.  GENERATED by gen_pipe_asm.py\n"
             "// (same directory): edit the script, not this file.  Register map and the hazards\n"
             "// respected are described at the top of the script and in attn_kernel_pipe.h.\n"
             "#pragma once\n#include \"attn_common.h\"\n\nnamespace calibatt_dev {\n\n")
    o.append(f"#define PIPE_PINNED {ALL_CLOBBERS}\n\n")
    o.append(f"constexpr int PIPE_FB_PAIRS = {FB_PAIRS};\n\n")

    # ---- O = 0
    lines = [f"v_accvgpr_write_b32 a{128 + i}, 0" for i in range(64)]
    o.append("__device__ __forceinline__ void pipe_zero_o() {\n" + emit(lines, "", "")  + "}\n\n")

    # ---- Q^T -> a[192:223], four k-slabs per call
    def loadq(half):
        lines = []
        for s in range(4):
            for e in range(4):
                lines.append(f"v_accvgpr_write_b32 a{192 + 16 * half + 4 * s + e}, %[q{s}{e}]")
        ins = ", ".join(f'[q{s}{e}] "v"(q{s}[{e}])' for s in range(4) for e in range(4))
        return emit(lines, "", ins)
    o.append("template <int PAR>\n__device__ __forceinline__ void pipe_load_q(const u32x4 &q0, const u32x4 &q1, const u32x4 &q2, const u32x4 &q3) {\n"
             "  if constexpr (PAR == 0) {\n" + loadq(0) + "  } else {\n" + loadq(1) + "  }\n}\n\n")

    # ---- O *= alpha
    lines = ["s_nop 15"]
    for i in range(0, 64, 4):
        lines += [f"v_accvgpr_read_b32 %[t{e}], a{128 + i + e}" for e in range(4)]
        lines += [f"v_mul_f32 %[t{e}], %[al], %[t{e}]" for e in range(4)]
        lines += [f"v_accvgpr_write_b32 a{128 + i + e}, %[t{e}]" for e in range(4)]
    lines.append("s_nop 7")
    o.append("__device__ __forceinline__ void pipe_rescale_o(float alpha) {\n  float t0, t1, t2, t3;\n" +
             emit(lines, T4_OUT, '[al] "v"(alpha)') + "}\n\n")

    # ---- O / l -> bf16 -> LDS staging row (lane: query row, 8-byte pieces at 64 db + 16 a)
    lines = ["s_nop 15"]
    for db in range(4):
        for a in range(4):
            lines += [f"v_accvgpr_read_b32 %[t{e}], a{128 + 16 * db + 4 * a + e}" for e in range(4)]
            lines += [f"v_mul_f32 %[t{e}], %[inv], %[t{e}]" for e in range(4)]
            w = 64 + 2 * ((4 * db + a) % 8)  # S registers are free by now; a pair is reused 8 stores later
            lines += [f"v_cvt_pk_bf16_f32 v{w}, %[t0], %[t1]", f"v_cvt_pk_bf16_f32 v{w + 1}, %[t2], %[t3]",
                      f"ds_write_b64 %[ad], v[{w}:{w + 1}] offset:{64 * db + 16 * a}"]
    lines.append("s_waitcnt lgkmcnt(0)")
    o.append("__device__ __forceinline__ void pipe_store_o(float inv, uint32_t ad) {\n  float t0, t1, t2, t3;\n" +
             emit(lines, T4_OUT, '[inv] "v"(inv), [ad] "v"(ad)') + "}\n\n")

    # ---- row maximum of tile T without a partner product (first tile)
    o.append(by_parity("pipe_max_plain(float &mx)", "  float t0;\n",
                       lambda t: emit(["s_nop 15"] + [x.text for x in max_ops(t)], '[mx] "=&v"(mx), [t0] "=&v"(t0)', "")))

    # ---- ragged last kv block: S = key < N ? S * sc : -inf  (lim = N - first key of this lane's group)
    def mask(t):
        lines = ["s_nop 15"]
        for kb in range(4):
            for v in range(16):
                kidx = 32 * kb + 16 * (v >> 3) + (v & 7)
                r = S(t, 16 * kb + v)
                lines += [f"v_mul_f32 {r}, %[sc], {r}", f"v_cmp_lt_i32 vcc, {kidx}, %[lim]", f"v_cndmask_b32 {r}, %[ninf], {r}, vcc"]
        return emit(lines, "", '[sc] "v"(sc), [lim] "v"(lim), [ninf] "v"(ninf)', ', "vcc"')
    o.append(by_parity("pipe_mask_tail(float sc, int lim, float ninf)", "", mask))

    # ---- softmax of part of tile T without a partner product (first and last tile)
    for part, (lo, hi) in enumerate([(0, FB_PAIRS), (FB_PAIRS, 32)]):
        def sm(t, lo=lo, hi=hi):
            ops = softmax_ops(t, range(lo, hi))
            check_trans(ops)
            lines = [x.text for x in ops]
            return emit(lines, SM_OUT, SM_IN)
        o.append(by_parity(f"pipe_softmax_part{part}(float sc, float m, float &l0, float &l1)", "  float t0, t1, t2, t3;\n", sm))

    # ---- S_0 = K_0 Q^T (first tile, K buffer 0)
    lines = k_reads(0, 0, 0) + weave(qk_anchors(0, 0, False), []) + ["s_nop 15"]
    ka_in = ", ".join(f'[ka{s}] "v"(ka[{s}])' for s in range(8))
    o.append("__device__ __forceinline__ void pipe_qk_first(const uint32_t (&ka)[8]) {\n" + emit(lines, "", ka_in) + "}\n\n")

    # ---- phase A(i), PAR = i & 1: S_{i+1} = K_{i+1} Q^T | softmax of the later pairs of tile i | DMA of V_{i+1}
    def phase_a(par):
        x, y = par, 1 - par
        koff = (1 - par) * 32768
        valu = softmax_ops(x, range(FB_PAIRS, 32))
        lines = k_reads(0, 0, koff) + weave(qk_anchors(y, koff, True), valu, pre=10)
        return emit(lines, f"{SM_OUT}, {DMA_OUT}", f"{ka_in}, {SM_IN}, {DMA_IN}", ', "m0", "scc"')
    o.append(by_parity(f"pipe_phase_a(const uint32_t (&ka)[8], float sc, float m, float &l0, float &l1, {DMA_SIG})",
                       "  float t0, t1, t2, t3;\n  uint32_t st;\n", phase_a))

    va_in = ", ".join(f'[va{d}] "v"(va[{d}])' for d in range(4))

    # ---- phase B1(i): first two slabs of O += V_i^T P_i | row maximum of S_{i+1}
    def phase_b1(par):
        x, y = par, 1 - par
        voff = par * 32768
        lines = v_reads(0, 0, voff) + v_reads(1, 1, voff) + weave(pv_anchors(x, voff, (0, 1)), max_ops(y))
        return emit(lines, '[mx] "=&v"(mx), [t0] "=&v"(t0)', va_in)
    o.append(by_parity("pipe_phase_b1(const uint32_t (&va)[4], float &mx)", "  float t0;\n", phase_b1))

    # ---- phase B2(i): remaining slabs | softmax of the first pairs of tile i+1 | DMA of K_{i+3}
    def phase_b2(par, with_k):
        x, y = par, 1 - par
        voff = par * 32768
        plan = {(2, 1): 0, (2, 2): 1, (3, 1): 2, (3, 2): 3, (4, 1): 4, (5, 1): 5, (6, 1): 6, (7, 1): 7} if with_k else None
        lines = weave(pv_anchors(x, voff, range(2, 8), plan), softmax_ops(y, range(0, FB_PAIRS)))
        if with_k:
            return emit(lines, f"{SM_OUT}, {DMA_OUT}", f"{va_in}, {SM_IN}, {DMA_IN}", ', "m0", "scc"')
        return emit(lines, SM_OUT, f"{va_in}, {SM_IN}")
    o.append(by_parity(f"pipe_phase_b2_k(const uint32_t (&va)[4], float sc, float m, float &l0, float &l1, {DMA_SIG})",
                       "  float t0, t1, t2, t3;\n  uint32_t st;\n", lambda p: phase_b2(p, True)))
    o.append(by_parity("pipe_phase_b2(const uint32_t (&va)[4], float sc, float m, float &l0, float &l1)",
                       "  float t0, t1, t2, t3;\n", lambda p: phase_b2(p, False)))

    # ---- O += V_i^T P_i without a partner (last tile)
    def pv_plain(par):
        voff = par * 32768
        lines = v_reads(0, 0, voff) + v_reads(1, 1, voff) + weave(pv_anchors(par, voff, range(8)), [])
        return emit(lines, "", va_in)
    o.append(by_parity("pipe_pv_plain(const uint32_t (&va)[4])", "", pv_plain))

    o.append("}  // namespace calibatt_dev\n")
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "attn_pipe_asm.h")
    with open(path, "w") as f:
        f.write("".join(o))


if __name__ == "__main__":
    main()
