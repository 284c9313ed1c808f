#!/usr/bin/env python3
"""Generator of gemm_step_asm.inc: the hand-scheduled inner step of gemm_fast_kernel.

Why assembly.  The fast GEMM kernel runs ONE wavefront per SIMD (its 512 x 32
int32 accumulators fill the 256 accumulation registers), and a lone wavefront
issues one instruction every 4 cycles.  A v_mfma_i32_32x32x32_i8 occupies the
matrix core for 8 such slots, so about 5 other instructions fit in the shadow
of each MFMA -- but only if they are placed between the MFMAs, in program
order.  The compiler's scheduler does not keep such an order, so the step is
emitted here, slot by slot:

  slot k (k = 0..31):   s_waitcnt lgkmcnt(n)          A fragment k has arrived from LDS
                        v_mfma acc[k % 16] += A_frag[k] * B[k / 16]
                        ds_read_b128  A fragment k + 8 (prefetch distance 8)
                        one piece (two instructions) of the expansion of the next
                        pair's W codes to int8          (28 of the 32 slots)
                        one direct global->LDS load of the pair three steps ahead
                        (10 of the 32 slots)

Registers are fixed (physical) so that values written asynchronously by LDS
reads never pass through compiler-chosen copies:
  a[0:255]      accumulators, group g in a[16g : 16g+15]
  v[128:135]    B operands (int8) set A: t = 0 in v[128:131], t = 1 in v[132:135]
  v[136:143]    B operands set B
  v[144:147]    W codes of the next pair, v[148:151] its table, v152 table offset, v153 table address
  v[156:191]    9 A-fragment buffers
  v[192:223]    temporaries of the W expansion (8 per code dword)
Variant X of the step multiplies by set A and writes set B, variant Y the reverse.

Run `python gen_gemm_step.py` in this directory to rewrite gemm_step_asm.inc
(the build does it, and the file is committed).
"""
import os

B_SETS = {"A": 128, "B": 136}
C0, TAB0, META, TABADDR = 144, 148, 152, 153
AF0, NBUF, DEPTH = 156, 9, 8
TMP0 = 192
NSLOT, NGROUP = 32, 16
A_STAGE_FRAG = 1024          # bytes per (group, t) fragment in an LDS stage


def vr(n, cnt=1):
    return f"v{n}" if cnt == 1 else f"v[{n}:{n + cnt - 1}]"


def af(i):
    return vr(AF0 + 4 * (i % NBUF), 4)


def frag_offset(k):
    g, t = k % NGROUP, k // NGROUP
    return (g * 2 + t) * A_STAGE_FRAG


class Lgkm:
    """In-order queue of outstanding LDS reads, to compute s_waitcnt lgkmcnt(n)."""

    def __init__(self):
        self.q = []

    def issue(self, tag):
        self.q.append(tag)

    def need(self, tag):
        if tag not in self.q:
            return None
        i = self.q.index(tag)
        n = len(self.q) - i - 1
        self.q = self.q[i + 1:]
        return f"s_waitcnt lgkmcnt({n})"


def expansion_pieces(bn):
    """The 28 two-instruction pieces that expand the four code dwords (see unpack8 in
    gemm.hip): 16 that need only the codes, then 12 that need the dialect table."""
    first, second = [], []
    for d in range(4):
        c = vr(C0 + d)
        t = [vr(TMP0 + 8 * d + i) for i in range(8)]
        ie, io, c4, c8, c12, mo, me, pe = t
        ne, po, no = c4, c8, c12                  # reuse once the masks are built
        first += [
            [f"v_and_b32 {ie}, 0x07070707, {c}", f"v_lshlrev_b32 {c4}, 4, {c}"],
            [f"v_lshrrev_b32 {io}, 4, {c}", f"v_lshlrev_b32 {c8}, 8, {c}"],
            [f"v_and_b32 {io}, 0x07070707, {io}", f"v_lshlrev_b32 {c12}, 8, {c4}"],
            [f"v_perm_b32 {mo}, {c8}, {c}, %[sel]", f"v_perm_b32 {me}, {c12}, {c4}, %[sel]"],
        ]
        plo, phi, nlo, nhi = (vr(TAB0 + i) for i in range(4))
        second += [
            [f"v_perm_b32 {pe}, {phi}, {plo}, {ie}", f"v_perm_b32 {ne}, {nhi}, {nlo}, {ie}"],
            [f"v_perm_b32 {po}, {phi}, {plo}, {io}", f"v_perm_b32 {no}, {nhi}, {nlo}, {io}"],
            [f"v_bfi_b32 {vr(bn + 2 * d)}, {me}, {ne}, {pe}", f"v_bfi_b32 {vr(bn + 2 * d + 1)}, {mo}, {no}, {po}"],
        ]
    return first, second


def dma_ops():
    """(m0 setup, load) of the 10 direct global->LDS loads of one step."""
    ops = []
    for j in range(8):                            # A: fragments (g, t) of this wave's 4 groups
        ops.append((f"s_add_u32 m0, %[m0a], {j * A_STAGE_FRAG}", f"global_load_lds_dwordx4 %[voff], %[a{j}]"))
    ops.append(("s_mov_b32 m0, %[m0w]", "global_load_lds_dwordx4 %[vcoff], %[wc]"))
    ops.append(("s_mov_b32 m0, %[m0m]", "global_load_lds_dword %[vmoff], %[wm]"))
    return ops


def step(cur, nxt):
    bc, bn = B_SETS[cur], B_SETS[nxt]
    out = []
    lg = Lgkm()
    # loads complete in order: all but the 10 issued during the previous step (pair vc+2)
    # have landed, in particular pair vc+1 (fetched two steps ago)
    out.append("s_waitcnt vmcnt(10)")
    out.append(f"ds_read_b128 {vr(C0, 4)}, %[swc]")
    lg.issue("c")
    out.append(f"ds_read_b32 {vr(META)}, %[swm]")
    lg.issue("meta")
    for k in range(DEPTH):
        out.append(f"ds_read_b128 {af(k)}, %[sa] offset:{frag_offset(k)}")
        lg.issue(f"af{k}")
    out.append(lg.need("meta"))
    out.append(f"v_add_u32 {vr(TABADDR)}, %[tabb], {vr(META)}")
    out.append(f"ds_read_b128 {vr(TAB0, 4)}, {vr(TABADDR)}")
    lg.issue("tab")
    first, second = expansion_pieces(bn)
    dmas = dma_ops()
    for k in range(NSLOT):
        w = lg.need(f"af{k}")
        if w:
            out.append(w)
        g, t = k % NGROUP, k // NGROUP
        acc = f"a[{16 * g}:{16 * g + 15}]"
        out.append(f"v_mfma_i32_32x32x32_i8 {acc}, {af(k)}, {vr(bc + 4 * t, 4)}, {acc}")
        dma = dmas[k // 2] if (k % 2 == 1 and k // 2 < len(dmas)) else None
        if dma:
            out.append(dma[0])
        if k + DEPTH < NSLOT:
            out.append(f"ds_read_b128 {af(k + DEPTH)}, %[sa] offset:{frag_offset(k + DEPTH)}")
            lg.issue(f"af{k + DEPTH}")
        piece = first[k] if k < 16 else (second[k - 16] if k - 16 < len(second) else None)
        if piece and k == 16:
            w = lg.need("tab")
            if w:
                out.append(w)
        if piece:
            out.append(piece[0])
        elif dma:
            out.append("s_nop 0")
        if dma:
            out.append(dma[1])
        if piece:
            out.append(piece[1])
    out.append("s_barrier")                      # the next pair's A fragments are visible to all waves
    return [o for o in out if o]


def c_string(lines):
    return "\n".join(f'    "{l}\\n\\t"' for l in lines)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    parts = ["// Generated by gen_gemm_step.py -- do not edit; see that file for the register map.\n"]
    for name, (cur, nxt) in (("X", ("A", "B")), ("Y", ("B", "A"))):
        parts.append(f"#define DFP4_STEP_ASM_{name} \\\n" + " \\\n".join(c_string(step(cur, nxt)).split("\n")) + "\n")
    zero = [f"v_accvgpr_write_b32 a{n}, 0" for n in range(256)]
    parts.append("#define DFP4_ACC_ZERO_ASM \\\n" + " \\\n".join(c_string(zero).split("\n")) + "\n")
    # all MFMAs have retired before the accumulators are read by the vector ALU
    drain = ["s_nop 15", "s_nop 15", "s_nop 15"]
    parts.append("#define DFP4_ACC_DRAIN_ASM \\\n" + " \\\n".join(c_string(drain).split("\n")) + "\n")
    shift = list(drain)
    for n0 in range(0, 256, 8):
        shift += [f"v_accvgpr_read_b32 {vr(TMP0 + i)}, a{n0 + i}" for i in range(8)]
        shift += [f"v_lshlrev_b32 {vr(TMP0 + i)}, 4, {vr(TMP0 + i)}" for i in range(8)]
        shift += [f"v_accvgpr_write_b32 a{n0 + i}, {vr(TMP0 + i)}" for i in range(8)]
    shift += ["s_nop 4"]
    parts.append("#define DFP4_ACC_SHIFT4_ASM \\\n" + " \\\n".join(c_string(shift).split("\n")) + "\n")
    for g in range(NGROUP):
        rd = [f"v_accvgpr_read_b32 %{i}, a{16 * g + i}" for i in range(16)]
        parts.append(f"#define DFP4_ACC_READ_ASM_{g} \\\n" + " \\\n".join(c_string(rd).split("\n")) + "\n")
    vclob = ", ".join(f'"v{n}"' for n in range(C0, TMP0 + 32))
    aclob = ", ".join(f'"a{n}"' for n in range(256))
    parts.append(f"#define DFP4_STEP_VGPR_CLOBBERS {vclob}\n")
    parts.append(f"#define DFP4_ACC_CLOBBERS {aclob}\n")
    tclob = ", ".join(f'"v{n}"' for n in range(TMP0, TMP0 + 8))
    parts.append(f"#define DFP4_SHIFT_VGPR_CLOBBERS {tclob}\n")
    path = os.path.join(here, "gemm_step_asm.inc")
    text = "\n".join(parts)
    if not os.path.exists(path) or open(path).read() != text:
        with open(path, "w") as f:
            f.write(text)
    return path


if __name__ == "__main__":
    print(main())
