#!/usr/bin/env python3
"""Writes attn_pipe_asm.h: the instruction streams of the pipelined attention kernel.

Run after changing anything here:  python3 gen_pipe_asm.py   (the header is
committed; the build does not run this script).

A wavefront of the pipelined kernel owns 64 queries (two groups qg of 32) and
works on kv sub-tiles of 64 keys (two sub-blocks kb of 32).  Its large operands
live in registers the compiler is told never to touch (the kernel is compiled
with a cap of 64 vector registers and must not spill beyond a7, which the
build checks), so every instruction that reads or writes them is emitted here
with literal register names:

  v[64:127]   S of even sub-tiles  S[t][kb][qg][16 accumulators]
  v[128:191]  S of odd sub-tiles
  v[192:223]  P of even sub-tiles  P[t][kb][qg][8]: register r = bf16 pair of logits 2r, 2r+1
  v[224:255]  P of odd sub-tiles
  a[8:31]     K operands of one k-slab, three stages of 2 key sub-blocks x 4 registers
  a[32:63]    V^T operands of one 16-key slab, two stages of 4 d blocks x 4 registers
  a[64:127]   Q^T: 8 k-slabs x 2 query groups x 4 registers
  a[128:255]  O^T: 4 d blocks x 2 query groups x 16 accumulators

Hazards the assembler does not check and that the streams below respect:
  * a transcendental result is not read by the next instruction;
  * MFMA results are read by other instructions only after >= 11 issue slots;
  * one instruction sits between a write of M0 and the LDS-DMA that uses it;
  * dot instructions are not used: they and a second transcendental between two
    MFMAs stall the matrix pipeline, measured at about 20 cycles each, while one
    transcendental plus up to four or five plain VALU instructions per MFMA hide
    behind it.  The softmax is therefore laid out with exactly one v_exp_f32
    behind every MFMA, and the row sums are plain additions of the bf16-rounded
    probabilities, unpacked again (the sums must add exactly what the PV product
    multiplies, or a row with one dominant key is off by the rounding of that key).
"""
import os

EXP = set(os.environ.get("PIPE_GEN_EXP", "").split(","))  # timing experiments only: nolds, novalu, nodma
# Softmax of a sub-tile's 32 logit pairs, by the block whose MFMAs it hides behind (one exp per MFMA):
PAIRS_B2 = range(0, 8)    # 16 MFMAs of the previous sub-tile's PV slabs 2-3 (these pairs feed PV slab 0)
PAIRS_A = range(8, 24)    # 32 MFMAs of the next sub-tile's QK
PAIRS_B1 = range(24, 32)  # 16 MFMAs of this sub-tile's PV slabs 0-1 (these pairs feed PV slab 3)


def S(t, kb, qg, v):
    return f"v{64 + 64 * t + 32 * kb + 16 * qg + v}"


def St(t, kb, qg):
    b = 64 + 64 * t + 32 * kb + 16 * qg
    return f"v[{b}:{b + 15}]"


def Pr(t, kb, qg, r):
    return f"v{192 + 32 * t + 16 * kb + 8 * qg + r}"


def Pt(t, j, qg):  # B operand of 16-key slab j
    b = 192 + 32 * t + 16 * (j >> 1) + 8 * qg + 4 * (j & 1)
    return f"v[{b}:{b + 3}]"


def Ka(st, kb):
    b = 8 + 8 * st + 4 * kb
    return f"a[{b}:{b + 3}]"


def Va(st, db, half):
    b = 32 + 16 * st + 4 * db + 2 * half
    return f"a[{b}:{b + 1}]"


def Vt(st, db):
    b = 32 + 16 * st + 4 * db
    return f"a[{b}:{b + 3}]"


def Qt(s, qg):
    b = 64 + 8 * s + 4 * qg
    return f"a[{b}:{b + 3}]"


def O(db, qg, i=0):
    return 128 + 32 * db + 16 * qg + i


def Ot(db, qg):
    return f"a[{O(db, qg)}:{O(db, qg) + 15}]"


class Op:
    def __init__(self, text, trans_dst=None, reads=()):
        self.text, self.trans_dst, self.reads = text, trans_dst, tuple(reads)


def pair(p):
    """Pair p of a sub-tile in the order the PV slabs consume them: (kb, qg, r)."""
    j, qg, r4 = p // 8, (p % 8) // 4, p % 4
    return j >> 1, qg, 4 * (j & 1) + r4


def softmax_groups(t, pairs):
    """exp2(sc * s - m) of the given logit pairs of sub-tile t, rounded to bf16 into P, row sums
    into l<qg>0 / l<qg>1.  Returns (pre, groups, tail): two groups per pair, each starting with
    the one transcendental it holds; pre goes before the first group, tail after the last."""
    pairs = list(pairs)
    n = len(pairs)

    def tmp(k, w):
        return f"%[t{2 * (k % 3) + w}]"

    def fma(k, w):
        kb, qg, r = pair(pairs[k])
        return Op(f"v_fma_f32 {tmp(k, w)}, {S(t, kb, qg, 2 * r + w)}, %[sc], -%[mq{qg}]")

    def exp(k, w):
        return Op(f"v_exp_f32 {tmp(k, w)}, {tmp(k, w)}", trans_dst=tmp(k, w))

    def cvt(k):
        kb, qg, r = pair(pairs[k])
        return Op(f"v_cvt_pk_bf16_f32 {Pr(t, kb, qg, r)}, {tmp(k, 0)}, {tmp(k, 1)}", reads=(tmp(k, 0), tmp(k, 1)))

    def unpack(k, w):  # the rounded value back as fp32: the row sums add exactly what the PV product multiplies
        kb, qg, r = pair(pairs[k])
        if w == 0:
            return Op(f"v_lshlrev_b32 {tmp(k, 0)}, 16, {Pr(t, kb, qg, r)}")
        return Op(f"v_and_b32 {tmp(k, 1)}, 0xffff0000, {Pr(t, kb, qg, r)}")

    def add(k, w):
        kb, qg, r = pair(pairs[k])
        return Op(f"v_add_f32 %[l{qg}{w}], %[l{qg}{w}], {tmp(k, w)}", reads=(tmp(k, w),))

    pre = [fma(0, 0), fma(0, 1)]
    groups = []
    for k in range(n):
        g0, g1 = [exp(k, 0)], [exp(k, 1)]
        if k >= 1:
            g0 += [cvt(k - 1), unpack(k - 1, 0)]
            g1 += [unpack(k - 1, 1), add(k - 1, 0), add(k - 1, 1)]
        if k + 1 < n:
            g0.append(fma(k + 1, 0))
            g1.append(fma(k + 1, 1))
        groups += [g0, g1]
    tail = [Op("s_nop 0"), cvt(n - 1), unpack(n - 1, 0), unpack(n - 1, 1), add(n - 1, 0), add(n - 1, 1)]
    return pre, groups, tail


def max_ops(t):
    """Maxima of this lane's 32 logits per query group of sub-tile t into %[mx0], %[mx1] (use %[xa0], %[xa1])."""
    ops = []
    for qg in range(2):
        vals = [S(t, kb, qg, v) for kb in range(2) for v in range(16)]
        acc = [f"%[mx{qg}]", f"%[xa{qg}]"]
        ops.append(Op(f"v_max3_f32 {acc[0]}, {vals[0]}, {vals[1]}, {vals[2]}"))
        ops.append(Op(f"v_max3_f32 {acc[1]}, {vals[3]}, {vals[4]}, {vals[5]}"))
        i, k = 6, 0
        while i < 32:
            ops.append(Op(f"v_max3_f32 {acc[k]}, {vals[i]}, {vals[i + 1]}, {acc[k]}"))
            i += 2
            k ^= 1
        ops.append(Op(f"v_max_f32 {acc[0]}, {acc[0]}, {acc[1]}"))
    return ops


def combine_ops():
    """Scale the lane maxima by %[sy] and take the maximum with the other half-wave (lane ^ 32)."""
    return [Op("v_mul_f32 %[mx0], %[sy], %[mx0]"), Op("v_mul_f32 %[mx1], %[sy], %[mx1]"),
            Op("v_mov_b32 %[xa0], %[mx0]"), Op("v_mov_b32 %[xa1], %[mx1]"), Op("s_nop 1"),
            Op("v_permlane32_swap_b32 %[mx0], %[xa0]"), Op("v_permlane32_swap_b32 %[mx1], %[xa1]"),
            Op("v_max_f32 %[mx0], %[mx0], %[xa0]"), Op("v_max_f32 %[mx1], %[mx1], %[xa1]")]


def check_trans(ops):
    """No VALU instruction reads a transcendental result in the slot right after it."""
    for a, b in zip(ops, ops[1:]):
        if a.trans_dst and a.trans_dst in b.reads:
            raise SystemExit(f"trans hazard: {a.text} -> {b.text}")


def weave(anchors, pre, groups, tail, extras=()):
    """anchors: list of (lines before the MFMA, MFMA line, lines after it).  Gap g (behind MFMA g)
    receives groups[g] and an even share of extras; pre goes before everything, tail at the end."""
    n = len(anchors)
    assert len(groups) <= n, (len(groups), n)
    extras = list(extras)
    seq = list(pre)
    lines = [o.text for o in pre]
    k = 0
    for a, (before, mfma, after) in enumerate(anchors):
        lines += before
        lines.append(mfma)
        gap = list(groups[a]) if a < len(groups) else []
        goal = (len(extras) * (a + 1)) // n
        gap += extras[k:goal]
        k = goal
        if a == n - 1:
            gap += list(tail)
        seq += gap
        lines += [o.text for o in gap]
        lines += after
    check_trans(seq)  # MFMAs and other instructions in between only add distance
    return lines


def flat(pre, groups, tail):
    ops = list(pre) + [o for g in groups for o in g] + list(tail)
    check_trans(ops)
    return [o.text for o in ops]


def dma_pair(j):
    """Two 1 KB direct-to-LDS loads of a wave (instructions 2j and 2j+1 of its 8 per sub-tile): 8 rows.
    The instruction offset moves the global and the LDS address alike, so one M0 serves both."""
    return [f"s_add_u32 m0, %[dl], {j * 4096}", f"s_add_u32 %[st], %[ds], {j * 4096}",
            "buffer_load_dwordx4 %[dv0], %[dr], %[st] offen lds",
            "buffer_load_dwordx4 %[dv1], %[dr], %[st] offen offset:2048 lds"]


def k_reads(s, koff):
    return [f"ds_read_b128 {Ka(s % 3, kb)}, %[ka{s}] offset:{koff + kb * 8192}" for kb in range(2)]


def v_reads(st, j, voff):
    out = []
    for db in range(4):
        out.append(f"ds_read_b64_tr_b16 {Va(st, db, 0)}, %[va{db}] offset:{voff + j * 4096}")
        out.append(f"ds_read_b64_tr_b16 {Va(st, db, 1)}, %[va{db}] offset:{voff + j * 4096 + 1024}")
    return out


def qk_anchors(ty, koff, dma_at=(), sync=()):
    """8 k-slabs of S_ty = K Q^T; operands of slab s+2 are read while slab s multiplies (the
    reads of slabs 0 and 1 are issued before).  sync: instructions placed in front of the last
    slab once its operands have arrived (the workgroup barrier and what follows it)."""
    anchors = []
    for s in range(8):
        for n, (kb, qg) in enumerate(((0, 0), (0, 1), (1, 0), (1, 1))):
            before, after = [], []
            if n == 0:
                if s + 2 < 8:
                    before += k_reads(s + 2, koff)
                before.append(f"s_waitcnt lgkmcnt({2 * min(2, 7 - s)})")
                if s == 7:
                    before += list(sync)
            c = "0" if s == 0 else St(ty, kb, qg)
            mfma = f"v_mfma_f32_32x32x16_bf16 {St(ty, kb, qg)}, {Ka(s % 3, kb)}, {Qt(s, qg)}, {c}"
            anchors.append((before, mfma, after))
    for d, a in enumerate(dma_at):
        anchors[a][2].extend(dma_pair(d))
    return anchors


def pv_anchors(tx, voff, slabs, dma_at=(), sync=(), first_read=True):
    """16-key slabs of O^T += V^T P_tx; operands of slab j+1 are read while slab j multiplies.
    sync: as in qk_anchors, in front of slab 3."""
    anchors = []
    for j in slabs:
        st = j & 1
        for n, (db, qg) in enumerate((db, qg) for db in range(4) for qg in range(2)):
            before, after = [], []
            if n == 0:
                if j < 3:
                    before += v_reads(1 - st, j + 1, voff)
                    before.append("s_waitcnt lgkmcnt(8)")
                else:
                    before.append("s_waitcnt lgkmcnt(0)")
                    before += list(sync)
            mfma = f"v_mfma_f32_32x32x16_bf16 {Ot(db, qg)}, {Vt(st, db)}, {Pt(tx, j, qg)}, {Ot(db, qg)}"
            anchors.append((before, mfma, after))
    for d, a in enumerate(dma_at):
        anchors[a][2].extend(dma_pair(d))
    return anchors


SYNC = ["s_waitcnt vmcnt(16)", "s_barrier"]  # all but the two youngest sub-tile loads have landed, in both waves

ALL_CLOBBERS = ", ".join([f'"v{i}"' for i in range(64, 256)] + [f'"a{i}"' for i in range(8, 256)])

T4_OUT = '[t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3)'
T6_OUT = T4_OUT + ', [t4] "=&v"(t4), [t5] "=&v"(t5)'
T6_DECL = "  float t0, t1, t2, t3, t4, t5;\n"
L_OUT = '[l00] "+v"(l[0][0]), [l01] "+v"(l[0][1]), [l10] "+v"(l[1][0]), [l11] "+v"(l[1][1])'
SM_OUT = f'{T6_OUT}, {L_OUT}'
SM_IN = '[sc] "v"(sc), [mq0] "v"(m[0]), [mq1] "v"(m[1])'
SM_SIG = "float sc, const float (&m)[2], float (&l)[2][2]"
DMA_OUT = '[st] "=&s"(st)'
DMA_IN = '[dr] "s"(rsrc), [dv0] "v"(lane_off0), [dv1] "v"(lane_off1), [ds] "s"(soff), [dl] "s"(lds)'
DMA_SIG = "const u32x4 &rsrc, uint32_t lane_off0, uint32_t lane_off1, uint32_t soff, uint32_t lds"
MX_OUT = '[mx0] "=&v"(mx[0]), [mx1] "=&v"(mx[1]), [xa0] "=&v"(xa0), [xa1] "=&v"(xa1)'
MX_DECL = "  float xa0, xa1;\n"
VALU_PREFIXES = ("v_fma", "v_exp", "v_cvt", "v_add_f32", "v_max", "v_mul", "v_mov", "v_permlane", "v_lshlrev", "v_and")


def emit(lines, outs, ins, extra_clobbers="", tag=""):
    if f"novalu_{tag}" in EXP or "novalu" in EXP:
        lines = [l for l in lines if not l.startswith(VALU_PREFIXES)]
    if "noexp" in EXP:
        lines = [l for l in lines if not l.startswith("v_exp")]
    if "nolds" in EXP:
        lines = [l for l in lines if not l.startswith("ds_read")]
    if "nodma" in EXP:
        lines = [l for l in lines if not l.startswith("buffer_load")]
    body = "\n".join(f'        "{l}\\n\\t"' for l in lines)
    return f"    asm volatile(\n{body}\n        : {outs}\n        : {ins}\n        : PIPE_PINNED{extra_clobbers});\n"


def by_index(tparam, count, sig, pre, make):
    out = f"template <int {tparam}>\n__device__ __forceinline__ void {sig} {{\n{pre}"
    for i in range(count):
        kw = "if" if i == 0 else "} else if"
        out += f"  {kw} constexpr ({tparam} == {i}) {{\n" + make(i)
    out += "  }\n}\n\n"
    return out


def by_parity(sig, pre, make):
    return by_index("PAR", 2, sig, pre, make)


def main():
    o = []
    o.append("// Instruction streams of the pipelined attention kernel.  GENERATED by gen_pipe_asm.py\n"
             "// (same directory): edit the script, not this file.  Register map and the hazards\n"
             "// respected are described at the top of the script and in attn_kernel_pipe.h.\n"
             "#pragma once\n#include \"attn_common.h\"\n\nnamespace calibatt_dev {\n\n")
    o.append(f"#define PIPE_PINNED {ALL_CLOBBERS}\n\n")

    # ---- O = 0
    lines = [f"v_accvgpr_write_b32 a{128 + i}, 0" for i in range(128)]
    o.append("__device__ __forceinline__ void pipe_zero_o() {\n" + emit(lines, "", "") + "}\n\n")

    # ---- Q^T -> a[64:127], two k-slabs (x two query groups) per call
    def loadq(part):
        lines = []
        for n, (s, qg) in enumerate((s, qg) for s in (2 * part, 2 * part + 1) for qg in range(2)):
            for e in range(4):
                lines.append(f"v_accvgpr_write_b32 a{64 + 8 * s + 4 * qg + e}, %[q{n}{e}]")
        ins = ", ".join(f'[q{n}{e}] "v"(q{n}[{e}])' for n in range(4) for e in range(4))
        return emit(lines, "", ins)
    o.append(by_index("PART", 4, "pipe_load_q(const u32x4 &q0, const u32x4 &q1, const u32x4 &q2, const u32x4 &q3)", "", loadq))

    # ---- O *= alpha, one query group
    def rescale(qg):
        lines = ["s_nop 15"]
        regs = [O(db, qg, i) for db in range(4) for i in range(16)]
        for i in range(0, 64, 4):
            lines += [f"v_accvgpr_read_b32 %[t{e}], a{regs[i + e]}" for e in range(4)]
            lines += [f"v_mul_f32 %[t{e}], %[al], %[t{e}]" for e in range(4)]
            lines += [f"v_accvgpr_write_b32 a{regs[i + e]}, %[t{e}]" for e in range(4)]
        lines.append("s_nop 7")
        return emit(lines, T4_OUT, '[al] "v"(alpha)')
    o.append(by_index("QG", 2, "pipe_rescale_o(float alpha)", "  float t0, t1, t2, t3;\n", rescale))

    # ---- O / l -> bf16 -> LDS staging row of one query group (8-byte pieces at 64 db + 16 a)
    def store(qg):
        lines = ["s_nop 15"]
        for db in range(4):
            for a in range(4):
                lines += [f"v_accvgpr_read_b32 %[t{e}], a{O(db, qg, 4 * a + e)}" for e in range(4)]
                lines += [f"v_mul_f32 %[t{e}], %[inv], %[t{e}]" for e in range(4)]
                w = 64 + 2 * ((4 * db + a) % 8)  # S registers are free by now; a pair is reused 8 stores later
                lines += [f"v_cvt_pk_bf16_f32 v{w}, %[t0], %[t1]", f"v_cvt_pk_bf16_f32 v{w + 1}, %[t2], %[t3]",
                          f"ds_write_b64 %[ad], v[{w}:{w + 1}] offset:{64 * db + 16 * a}"]
        lines.append("s_waitcnt lgkmcnt(0)")
        return emit(lines, T4_OUT, '[inv] "v"(inv), [ad] "v"(ad)')
    o.append(by_index("QG", 2, "pipe_store_o(float inv, uint32_t ad)", "  float t0, t1, t2, t3;\n", store))

    # ---- row maxima (scaled, combined over both half-waves) of sub-tile PAR without a partner product
    o.append(by_parity("pipe_max_plain(float sy, float (&mx)[2])", MX_DECL,
                       lambda t: emit(["s_nop 15"] + [x.text for x in max_ops(t) + combine_ops()], MX_OUT, '[sy] "v"(sy)')))

    # ---- ragged end of the sequence: S = key < N ? S * sc : -inf  (lim = N - first key of this lane's group)
    def mask(t):
        lines = ["s_nop 15"]
        for kb in range(2):
            for qg in range(2):
                for v in range(16):
                    kidx = 32 * kb + 16 * (v >> 3) + (v & 7)
                    r = S(t, kb, qg, v)
                    lines += [f"v_mul_f32 {r}, %[sc], {r}", f"v_cmp_lt_i32 vcc, {kidx}, %[lim]", f"v_cndmask_b32 {r}, %[ninf], {r}, vcc"]
        return emit(lines, "", '[sc] "v"(sc), [lim] "v"(lim), [ninf] "v"(ninf)', ', "vcc"')
    o.append(by_parity("pipe_mask_tail(float sc, int lim, float ninf)", "", mask))

    # ---- softmax of part of sub-tile PAR without a partner product (first and last sub-tile)
    for part, prs in enumerate([PAIRS_B2, list(PAIRS_A) + list(PAIRS_B1)]):
        o.append(by_parity(f"pipe_softmax_part{part}({SM_SIG})", T6_DECL,
                           lambda t, prs=prs: emit(flat(*softmax_groups(t, prs)), SM_OUT, SM_IN)))

    # ---- S_0 = K_0 Q^T (first sub-tile, K buffer 0)
    lines = k_reads(0, 0) + k_reads(1, 0) + weave(qk_anchors(0, 0), [], [], []) + ["s_nop 15"]
    ka_in = ", ".join(f'[ka{s}] "v"(ka[{s}])' for s in range(8))
    o.append("__device__ __forceinline__ void pipe_qk_first(const uint32_t (&ka)[8]) {\n" + emit(lines, "", ka_in) + "}\n\n")

    va_in = ", ".join(f'[va{d}] "v"(va[{d}])' for d in range(4))

    # ---- K operand reads of the first two k-slabs of K buffer KBUF (before the first phase A; later ones
    #      are issued by the phase B2 in front)
    o.append(by_index("KBUF", 2, "pipe_k_preread(const uint32_t (&ka)[8])", "",
                      lambda kbuf: emit(k_reads(0, kbuf * 16384) + k_reads(1, kbuf * 16384), "", '[ka0] "v"(ka[0]), [ka1] "v"(ka[1])')))

    # ---- phase A(i), PAR = i & 1: S_{i+1} = K_{i+1} Q^T | softmax of pairs PAIRS_A of sub-tile i | DMA of V_{i+1}.
    #      In front of the last k-slab: barrier (V_i has landed, K_{i+1} is read) and the first V operand reads.
    def phase_a(par):
        x, y = par, 1 - par
        koff = (1 - par) * 16384
        sync = SYNC + v_reads(0, 0, par * 16384)
        lines = weave(qk_anchors(y, koff, (1, 9, 17, 25), sync), *softmax_groups(x, PAIRS_A))
        return emit(lines, f"{SM_OUT}, {DMA_OUT}", f"{ka_in}, {va_in}, {SM_IN}, {DMA_IN}", ', "m0", "scc"', tag="a")
    o.append(by_parity(f"pipe_phase_a(const uint32_t (&ka)[8], const uint32_t (&va)[4], {SM_SIG}, {DMA_SIG})", T6_DECL + "  uint32_t st;\n", phase_a))

    # ---- phase B1(i): slabs 0-1 of O += V_i^T P_i | softmax of pairs PAIRS_B1 of sub-tile i | row maxima of S_{i+1}
    def phase_b1(par):
        x, y = par, 1 - par
        voff = par * 16384
        pre, groups, tail = softmax_groups(x, PAIRS_B1)
        mx = max_ops(y)
        lines = weave(pv_anchors(x, voff, (0, 1)), pre, groups, tail, mx + combine_ops())
        return emit(lines, f"{SM_OUT}, {MX_OUT}", f"{va_in}, {SM_IN}, [sy] \"v\"(sy)", tag="b1")
    o.append(by_parity(f"pipe_phase_b1(const uint32_t (&va)[4], {SM_SIG}, float sy, float (&mx)[2])", T6_DECL + MX_DECL, phase_b1))

    # ---- phase B2(i): slabs 2-3 | softmax of pairs PAIRS_B2 of sub-tile i+1 | DMA of K_{i+3}.
    #      In front of the last slab: barrier (K_{i+2} has landed, V_i is read) and the K operand reads of
    #      the first two k-slabs of the next phase A.
    def phase_b2(par):
        x, y = par, 1 - par
        voff = par * 16384
        sync = SYNC + k_reads(0, par * 16384) + k_reads(1, par * 16384)
        lines = weave(pv_anchors(x, voff, (2, 3), (1, 3, 5, 7), sync), *softmax_groups(y, PAIRS_B2))
        return emit(lines, f"{SM_OUT}, {DMA_OUT}", f"{va_in}, [ka0] \"v\"(ka[0]), [ka1] \"v\"(ka[1]), {SM_IN}, {DMA_IN}", ', "m0", "scc"', tag="b2")
    o.append(by_parity(f"pipe_phase_b2(const uint32_t (&va)[4], const uint32_t (&ka)[8], {SM_SIG}, {DMA_SIG})", T6_DECL + "  uint32_t st;\n", phase_b2))

    # ---- O += V_i^T P_i without a partner (last sub-tile)
    def pv_plain(par):
        voff = par * 16384
        lines = v_reads(0, 0, voff) + weave(pv_anchors(par, voff, range(4)), [], [], [])
        return emit(lines, "", va_in)
    o.append(by_parity("pipe_pv_plain(const uint32_t (&va)[4])", "", pv_plain))

    o.append("}  // namespace calibatt_dev\n")
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "attn_pipe_asm.h")
    with open(path, "w") as f:
        f.write("".join(o))


if __name__ == "__main__":
    main()
