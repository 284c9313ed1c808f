#!/usr/bin/env python3
"""Generator of gemm_native_asm.inc: main loop of gemm_native_kernel (block-scaled
v_mfma_scale_f32_32x32x64_f8f6f4 on FP4 or FP6 operands, see gemm_native.hip).

A workgroup computes 256 x 256 outputs with four waves as 2 x 2, each wave 128 x 128
(4 x 4 tiles of 32 x 32, accumulator tile (i, j) in a[16 (4 i + j) : +15]).  One step =
one pair of blocks (K = 64) = 16 MFMAs per wave.  Both operands arrive pre-arranged in the
instruction's register order (native_pack_kernel), so a (tile, step) chunk is 64 lanes x
16 bytes (FP4), followed for FP6 by 64 lanes x 12 bytes (8 used: registers 4 and 5), and the loop only moves data:

  global -> LDS  direct loads (global_load_lds_dwordx4 / dwordx3; a lane's 12 bytes land
                 at a 16-byte lane stride), three (FP6) or seven (FP4) steps ahead, four or eight LDS
                 stages in rotation;
                 wave w fetches A tiles 2w, 2w+1, B tiles 2w, 2w+1 and scale chunk w;
  LDS -> regs    the wave's 4 A and 4 B tiles and two scale dwords of step s + 1 are read
                 during step s (two register sets used alternately);
  one barrier per step, in the middle of the MFMA stream: after it every wave's loads of
  step s + 1 have landed and nobody reads the stage that this step's loads overwrite.

LDS stage: 16 tiles x TILE bytes (A tiles 0..7, B tiles 0..7; TILE = 1 KiB for FP4, 2 KiB
for FP6: two 1 KiB halves) + 4 x 256 bytes of scales (A groups 0, 1, B groups 0, 1).

Registers (fixed): a[0:255] accumulators; v[40:87] / v[88:135] operand sets (A tile i at
+6 i, B tile j at +24 + 6 j); v136..v139 scale dwords (A, B of set 0; A, B of set 1);
v140..v143 LDS read addresses (A, B, scales A, B), v144 / v145 / v146 global offsets (operands, scales, second
halves); s[60:69] global bases of the wave's five chunks, s70 step, s72 / s73 LDS address
of the stage read next / loaded next, s74..s76 scratch, s77..s83 the wave's offsets inside
a stage.
"""
import os

FR = [40, 88]
SA = [136, 138]
SB = [137, 139]
VA, VB, VSA, VSB, VOFF, VSOFF, VOFF2 = 140, 141, 142, 143, 144, 145, 146
S_BASE, S_VC, S_RD, S_LD, S_T0, S_T1, S_T2 = 60, 70, 72, 73, 74, 75, 76
S_RA, S_RB, S_RSA, S_RSB, S_DA, S_DB, S_DS = 77, 78, 79, 80, 81, 82, 83


def vr(n, cnt=1):
    return f"v{n}" if cnt == 1 else f"v[{n}:{n + cnt - 1}]"


def sr(n, cnt=1):
    return f"s{n}" if cnt == 1 else f"s[{n}:{n + cnt - 1}]"


class Fmt:
    def __init__(self, fp6):
        self.fp6 = fp6
        self.regs = 6 if fp6 else 4
        self.tile = 2048 if fp6 else 1024            # LDS bytes per tile and stage
        self.stage = 16 * self.tile + 1024
        self.gstride = 1792 if fp6 else 1024         # global bytes per (tile, step): 1024 + 768
        self.code = 2 if fp6 else 4                  # cbsz / blgp
        self.per_step = 9 if fp6 else 5              # direct loads per wave and step
        self.nst = 4 if fp6 else 8                   # LDS stages (FP6: 4 x 33 KiB, FP4: 8 x 17 KiB)
        self.dist = self.nst - 1                     # loads run this many steps ahead


def frag_reads(f, p):
    """LDS reads of a step's operands into register set p (addresses VA, VB, VSA, VSB)."""
    o = []
    for side, va in ((0, VA), (1, VB)):
        for t in range(4):
            r = FR[p] + 24 * side + 6 * t
            if f.fp6:
                o.append(f"ds_read_b128 {vr(r, 4)}, {vr(va)} offset:{t * f.tile}")
                o.append(f"ds_read_b64 {vr(r + 4, 2)}, {vr(va)} offset:{t * f.tile + 1024}")
            else:
                o.append(f"ds_read_b128 {vr(r, 4)}, {vr(va)} offset:{t * f.tile}")
    o.append(f"ds_read_b32 {vr(SA[p])}, {vr(VSA)}")
    o.append(f"ds_read_b32 {vr(SB[p])}, {vr(VSB)}")
    return o


def dma_ops(f):
    """(m0 setup, load) pairs of one step's direct loads of this wave; S_T0 / S_T1 / S_T2 hold
    the LDS addresses of its A, B and scale destinations in the stage being loaded."""
    o = []
    for side, dst in ((0, S_T0), (1, S_T1)):
        for k in range(2):
            base = sr(S_BASE + 4 * side + 2 * k, 2)
            if f.fp6:
                o.append((f"s_add_u32 m0, {sr(dst)}, {k * f.tile}", f"global_load_lds_dwordx4 {vr(VOFF)}, {base}"))
                o.append((f"s_add_u32 m0, {sr(dst)}, {k * f.tile + 1024}",
                          f"global_load_lds_dwordx3 {vr(VOFF2)}, {base}"))
            else:
                o.append((f"s_add_u32 m0, {sr(dst)}, {k * f.tile}", f"global_load_lds_dwordx4 {vr(VOFF)}, {base}"))
    o.append((f"s_mov_b32 m0, {sr(S_T2)}", f"global_load_lds_dword {vr(VSOFF)}, {sr(S_BASE + 8, 2)}"))
    return o


def dst_setup():
    return [f"s_add_u32 {sr(S_T0)}, {sr(S_LD)}, {sr(S_DA)}", f"s_add_u32 {sr(S_T1)}, {sr(S_LD)}, {sr(S_DB)}",
            f"s_add_u32 {sr(S_T2)}, {sr(S_LD)}, {sr(S_DS)}"]


def advance_load_stage(f):
    """next LDS stage to load (wraps), next global step"""
    return [f"s_add_u32 {sr(S_LD)}, {sr(S_LD)}, {f.stage}", f"s_cmp_lt_u32 {sr(S_LD)}, %[ldsend]",
            f"s_cselect_b32 {sr(S_LD)}, {sr(S_LD)}, %[lds]",
            f"v_add_u32 {vr(VOFF)}, {f.gstride}, {vr(VOFF)}", f"v_add_u32 {vr(VSOFF)}, 0x100, {vr(VSOFF)}"] + (
                [f"v_add_u32 {vr(VOFF2)}, {f.gstride}, {vr(VOFF2)}"] if f.fp6 else [])


def read_addr(f):
    return [f"s_add_u32 {sr(S_RD)}, {sr(S_RD)}, {f.stage}", f"s_cmp_lt_u32 {sr(S_RD)}, %[ldsend]",
            f"s_cselect_b32 {sr(S_RD)}, {sr(S_RD)}, %[lds]",
            f"s_add_u32 {sr(S_T0)}, {sr(S_RD)}, {sr(S_RA)}", f"v_add_u32 {vr(VA)}, {sr(S_T0)}, %[l16]",
            f"s_add_u32 {sr(S_T0)}, {sr(S_RD)}, {sr(S_RB)}", f"v_add_u32 {vr(VB)}, {sr(S_T0)}, %[l16]",
            f"s_add_u32 {sr(S_T0)}, {sr(S_RD)}, {sr(S_RSA)}", f"v_add_u32 {vr(VSA)}, {sr(S_T0)}, %[l4]",
            f"s_add_u32 {sr(S_T0)}, {sr(S_RD)}, {sr(S_RSB)}", f"v_add_u32 {vr(VSB)}, {sr(S_T0)}, %[l4]"]


def mfma(f, p, k):
    i, j = k // 4, k % 4
    acc = f"a[{16 * k}:{16 * k + 15}]"
    a = vr(FR[p] + 6 * i, f.regs)
    b = vr(FR[p] + 24 + 6 * j, f.regs)
    return (f"v_mfma_scale_f32_32x32x64_f8f6f4 {acc}, {a}, {b}, {acc}, {vr(SA[p])}, {vr(SB[p])} "
            f"op_sel:[{i & 1},{j & 1},0] op_sel_hi:[{i >> 1},{j >> 1},0] cbsz:{f.code} blgp:{f.code}")


def step(f, p):
    o = [f"s_cmp_lt_u32 {sr(S_VC)}, %[steps]", "s_cbranch_scc0 99f"]
    o += read_addr(f)                                       # LDS addresses of step s + 1's operands
    reads = frag_reads(f, 1 - p)
    dmas = dma_ops(f)
    for k in range(16):
        o.append(mfma(f, p, k))
        if k == 2:
            # the loads of step s + 1 have landed; those of the steps after it may be pending
            o += [f"s_waitcnt vmcnt({(f.dist - 2) * f.per_step})", "s_barrier"] + dst_setup()
        if k >= 3:
            n_r = (len(reads) + 12) // 13
            o += reads[(k - 3) * n_r:(k - 2) * n_r]
            n_d = (len(dmas) + 12) // 13
            for m0, ld in dmas[(k - 3) * n_d:(k - 2) * n_d]:
                o += [m0, "s_nop 0", ld]
    o += advance_load_stage(f)
    o += [f"s_add_u32 {sr(S_VC)}, {sr(S_VC)}, 1", "s_waitcnt lgkmcnt(0)"]
    return o


def entry(f):
    o = [f"v_accvgpr_write_b32 a{n}, 0" for n in range(256)]
    # global bases: A tiles 2w, 2w+1; B tiles 2w, 2w+1 (each tile holds `tstride` bytes); scale chunk
    o += [f"s_mov_b32 {sr(S_BASE)}, %[alo]", f"s_mov_b32 {sr(S_BASE + 1)}, %[ahi]",
          f"s_add_u32 {sr(S_BASE + 2)}, %[alo], %[tstride]", f"s_addc_u32 {sr(S_BASE + 3)}, %[ahi], 0",
          f"s_mov_b32 {sr(S_BASE + 4)}, %[blo]", f"s_mov_b32 {sr(S_BASE + 5)}, %[bhi]",
          f"s_add_u32 {sr(S_BASE + 6)}, %[blo], %[tstride]", f"s_addc_u32 {sr(S_BASE + 7)}, %[bhi], 0",
          f"s_mov_b32 {sr(S_BASE + 8)}, %[slo]", f"s_mov_b32 {sr(S_BASE + 9)}, %[shi]"]
    # the wave's offsets inside a stage: wm = wv >> 1, wn = wv & 1
    o += [f"s_lshr_b32 {sr(S_T0)}, %[wv], 1", f"s_and_b32 {sr(S_T1)}, %[wv], 1",
          f"s_mul_i32 {sr(S_RA)}, {sr(S_T0)}, {4 * f.tile}",
          f"s_mul_i32 {sr(S_RB)}, {sr(S_T1)}, {4 * f.tile}", f"s_add_u32 {sr(S_RB)}, {sr(S_RB)}, {8 * f.tile}",
          f"s_lshl_b32 {sr(S_RSA)}, {sr(S_T0)}, 8", f"s_add_u32 {sr(S_RSA)}, {sr(S_RSA)}, {16 * f.tile}",
          f"s_lshl_b32 {sr(S_RSB)}, {sr(S_T1)}, 8", f"s_add_u32 {sr(S_RSB)}, {sr(S_RSB)}, {16 * f.tile + 512}",
          f"s_mul_i32 {sr(S_DA)}, %[wv], {2 * f.tile}", f"s_add_u32 {sr(S_DB)}, {sr(S_DA)}, {8 * f.tile}",
          f"s_lshl_b32 {sr(S_DS)}, %[wv], 8", f"s_add_u32 {sr(S_DS)}, {sr(S_DS)}, {16 * f.tile}"]
    o += [f"s_mov_b32 {sr(S_VC)}, 0", f"s_mov_b32 {sr(S_LD)}, %[lds]",
          f"v_mov_b32 {vr(VOFF)}, %[g16]", f"v_mov_b32 {vr(VSOFF)}, %[g4]", f"v_mov_b32 {vr(VOFF2)}, %[g12]"]
    # pipeline fill: steps 0, 1, 2 into stages 0, 1, 2
    for _ in range(f.dist):
        o += dst_setup()
        for m0, ld in dma_ops(f):
            o += [m0, "s_nop 0", ld]
        o += advance_load_stage(f)
    # step 0's operands into set 0 (S_RD is advanced before use: start one stage "before" stage 0)
    o += [f"s_waitcnt vmcnt({(f.dist - 1) * f.per_step})", "s_barrier",
          f"s_add_u32 {sr(S_RD)}, %[lds], {(f.nst - 1) * f.stage}"]
    o += read_addr(f) + frag_reads(f, 0) + ["s_waitcnt lgkmcnt(0)"]
    return o


def main_loop(f):
    o = entry(f)
    o.append("80:")
    for p in range(2):
        o += step(f, p)
    o.append("s_branch 80b")
    o += ["99:", "s_waitcnt vmcnt(0) lgkmcnt(0)", "s_nop 15", "s_nop 15", "s_nop 15", "s_nop 15"]
    return o


def c_string(lines):
    return " \\\n".join(f'    "{l}\\n\\t"' for l in lines)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    parts = ["// Generated by gen_native_loop.py -- do not edit; see that file for the register map.\n"]
    parts.append("#define DFP4_NATIVE_LOOP_FP4 \\\n" + c_string(main_loop(Fmt(False))) + "\n")
    parts.append("#define DFP4_NATIVE_LOOP_FP6 \\\n" + c_string(main_loop(Fmt(True))) + "\n")
    for g in range(16):
        rd = [f"v_accvgpr_read_b32 %{i}, a{16 * g + i}" for i in range(16)]
        parts.append(f"#define DFP4_NATIVE_ACC_READ_{g} \\\n" + c_string(rd) + "\n")
    vclob = ", ".join(f'"v{n}"' for n in range(40, 148))
    aclob = ", ".join(f'"a{n}"' for n in range(256))
    sclob = ", ".join(f'"s{n}"' for n in range(S_BASE, S_DS + 1))
    parts.append(f"#define DFP4_NATIVE_VGPR_CLOBBERS {vclob}\n")
    parts.append(f"#define DFP4_NATIVE_ACC_CLOBBERS {aclob}\n")
    parts.append(f"#define DFP4_NATIVE_SGPR_CLOBBERS {sclob}\n")
    path = os.path.join(here, "gemm_native_asm.inc")
    text = "\n".join(parts)
    if not os.path.exists(path) or open(path).read() != text:
        with open(path, "w") as fh:
            fh.write(text)
    return path


if __name__ == "__main__":
    print(main())
