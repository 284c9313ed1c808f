#!/usr/bin/env python3
"""Generator of gemm_native_asm.inc: main loop of gemm_native_kernel (block-scaled
v_mfma_scale_f32_32x32x64_f8f6f4 on FP4 or FP6 operands, see gemm_native.hip).

A workgroup computes 256 x 256 outputs with four waves as 2 x 2, each wave 128 x 128
(4 x 4 tiles of 32 x 32, accumulator tile (i, j) in a[16 (4 i + j) : +15]).  One step =
one pair of blocks (K = 64) = 16 MFMAs per wave.  A second form (suffix _H) halves the rows:
128 x 256 per workgroup, 64 x 128 per wave, 8 MFMAs per step, for products with few tiles.  Both operands arrive pre-arranged in the
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
v144 / v145 / v146 global offsets (operands, scales, second halves), v150.. LDS read bases
(the loop is unrolled over the stages, so a stage is a base register plus an immediate);
s[60:69] global bases of the wave's five chunks, s70 step, s74 / s75 scratch, s77..s83 the
wave's LDS addresses inside stage 0 (reads: A, B, scales A, B; loads: A, B, scales).
"""
import os

FR = [40, 88]
SA = [136, 138]
SB = [137, 139]
VOFF, VSOFF, VOFF2 = 144, 145, 146
VBASE = 150                      # LDS read bases: group q at VBASE + 4 q: operands A, B, scales A, B
S_BASE, S_VC = 60, 70
S_T0, S_T1 = 74, 75
S_RA, S_RB, S_RSA, S_RSB, S_DA, S_DB, S_DS = 77, 78, 79, 80, 81, 82, 83


def vr(n, cnt=1):
    return f"v{n}" if cnt == 1 else f"v[{n}:{n + cnt - 1}]"


def sr(n, cnt=1):
    return f"s{n}" if cnt == 1 else f"s[{n}:{n + cnt - 1}]"


class Fmt:
    def __init__(self, fp6, ta=4):
        self.fp6 = fp6
        self.ta = ta                                 # A tiles (of 32 rows) per wave: 4 (256-row workgroup) or 2 (128)
        self.regs = 6 if fp6 else 4
        self.tile = 2048 if fp6 else 1024            # LDS bytes per tile and stage
        self.stage = (2 * ta + 8) * self.tile + 1024
        self.gstride = 1792 if fp6 else 1024         # global bytes per (tile, step): 1024 + 768
        self.code = 2 if fp6 else 4                  # cbsz / blgp
        a_tiles = ta // 2                            # A tiles this wave fetches per step (B: always 2)
        self.per_step = (a_tiles + 2) * (2 if fp6 else 1) + 1     # direct loads per wave and step
        self.nst = 4 if fp6 else 8                   # LDS stages (FP6: 4 x 33 KiB, FP4: 8 x 17 KiB)
        self.dist = self.nst - 1                     # loads run this many steps ahead
        # LDS reads address a stage as (base register of its group) + immediate (< 64 KiB)
        self.per_group = max(1, (65535 - (3 * self.tile + 1024 + 16)) // self.stage)
        self.groups = (self.nst + self.per_group - 1) // self.per_group


def frag_reads(f, p, stage):
    """LDS reads of the operands held in `stage` into register set p."""
    q, off = stage // f.per_group, (stage % f.per_group) * f.stage
    va, vb, vsa, vsb = (VBASE + 4 * q + i for i in range(4))
    o = []
    for side, v in ((0, va), (1, vb)):
        for t in range(f.ta if side == 0 else 4):
            r = FR[p] + 24 * side + 6 * t
            o.append(f"ds_read_b128 {vr(r, 4)}, {vr(v)} offset:{off + t * f.tile}")
            if f.fp6:
                o.append(f"ds_read_b64 {vr(r + 4, 2)}, {vr(v)} offset:{off + t * f.tile + 1024}")
    o.append(f"ds_read_b32 {vr(SA[p])}, {vr(vsa)} offset:{off}")
    o.append(f"ds_read_b32 {vr(SB[p])}, {vr(vsb)} offset:{off}")
    return o


def dma_groups(f, stage):
    """Direct loads of one step of this wave into `stage`, as groups (m0 setup, [loads that use it]).
    An instruction offset applies to the global and to the LDS address alike, and the second half of an
    FP6 chunk sits 1024 bytes behind the first in both, so the two halves share one m0."""
    o = []
    for side, dst in ((0, S_DA), (1, S_DB)):
        for k in range(f.ta // 2 if side == 0 else 2):
            base = sr(S_BASE + 4 * side + 2 * k, 2)
            loads = [f"global_load_lds_dwordx4 {vr(VOFF)}, {base}"]
            if f.fp6:
                loads.append(f"global_load_lds_dwordx3 {vr(VOFF2)}, {base} offset:1024")
            o.append((f"s_add_u32 m0, {sr(dst)}, {stage * f.stage + k * f.tile}", loads))
    o.append((f"s_add_u32 m0, {sr(S_DS)}, {stage * f.stage}", [f"global_load_lds_dword {vr(VSOFF)}, {sr(S_BASE + 8, 2)}"]))
    return o


def advance_global(f):
    return [f"v_add_u32 {vr(VOFF)}, {f.gstride}, {vr(VOFF)}", f"v_add_u32 {vr(VSOFF)}, 0x100, {vr(VSOFF)}"] + (
        [f"v_add_u32 {vr(VOFF2)}, {f.gstride}, {vr(VOFF2)}"] if f.fp6 else [])


def mfma(f, p, k):
    i, j = k // 4, k % 4
    acc = f"a[{16 * k}:{16 * k + 15}]"
    a = vr(FR[p] + 6 * i, f.regs)
    b = vr(FR[p] + 24 + 6 * j, f.regs)
    return (f"v_mfma_scale_f32_32x32x64_f8f6f4 {acc}, {a}, {b}, {acc}, {vr(SA[p])}, {vr(SB[p])} "
            f"op_sel:[{i & 1},{j & 1},0] op_sel_hi:[{i >> 1},{j >> 1},0] cbsz:{f.code} blgp:{f.code}")


def step(f, u):
    """Step number u (mod the number of stages): multiplies register set u % 2, reads the operands of
    the next step from stage (u + 1) % nst, loads stage (u + dist) % nst = (u - 1) % nst."""
    p = u % 2
    o = [f"s_cmp_lt_u32 {sr(S_VC)}, %[steps]", "s_cbranch_scc0 99f"]
    reads = frag_reads(f, 1 - p, (u + 1) % f.nst)
    dmas = dma_groups(f, (u + f.dist) % f.nst)
    # after the barrier: every m0 setup is followed by an LDS read (m0 needs one instruction before its use)
    tail = []
    for m0, loads in dmas:
        tail.append([m0] + ([reads.pop(0)] if reads else ["s_nop 0"]) + loads)
    while reads:
        tail.append([reads.pop(0)] + ([reads.pop(0)] if reads else []))
    nm = 4 * f.ta                     # MFMAs per step
    per = (len(tail) + nm - 5) // (nm - 4)      # spread evenly: bunching the memory instructions is slower
    for k in range(nm):
        o.append(mfma(f, p, k))
        if k == 2:
            # the loads of step s + 1 have landed; those of the steps after it may be pending
            o += [f"s_waitcnt vmcnt({(f.dist - 2) * f.per_step})", "s_barrier"]
        if k >= 3:
            for grp in tail[(k - 3) * per:(k - 2) * per]:
                o += grp
        if k == nm - 1:
            o += advance_global(f)
    o += [f"s_add_u32 {sr(S_VC)}, {sr(S_VC)}, 1", "s_waitcnt lgkmcnt(0)"]
    if f.ta == 2:                     # both row halves of the workgroup share one scale dword: bytes 2 wm, 2 wm + 1
        o.append(f"v_lshrrev_b32 {vr(SA[1 - p])}, {sr(S_T1)}, {vr(SA[1 - p])}")
    return o


def entry(f):
    o = [f"v_accvgpr_write_b32 a{n}, 0" for n in range(256)]
    # global bases: A tiles 2w, 2w+1; B tiles 2w, 2w+1 (each tile holds `tstride` bytes); scale chunk
    o += [f"s_mov_b32 {sr(S_BASE)}, %[alo]", f"s_mov_b32 {sr(S_BASE + 1)}, %[ahi]",
          f"s_add_u32 {sr(S_BASE + 2)}, %[alo], %[tstride]", f"s_addc_u32 {sr(S_BASE + 3)}, %[ahi], 0",
          f"s_mov_b32 {sr(S_BASE + 4)}, %[blo]", f"s_mov_b32 {sr(S_BASE + 5)}, %[bhi]",
          f"s_add_u32 {sr(S_BASE + 6)}, %[blo], %[tstride]", f"s_addc_u32 {sr(S_BASE + 7)}, %[bhi], 0",
          f"s_mov_b32 {sr(S_BASE + 8)}, %[slo]", f"s_mov_b32 {sr(S_BASE + 9)}, %[shi]"]
    # the wave's LDS addresses inside stage 0: wm = wv >> 1, wn = wv & 1
    offb, offs = 2 * f.ta * f.tile, (2 * f.ta + 8) * f.tile
    o += [f"s_lshr_b32 {sr(S_T0)}, %[wv], 1", f"s_and_b32 {sr(S_T1)}, %[wv], 1",
          f"s_mul_i32 {sr(S_RA)}, {sr(S_T0)}, {f.ta * f.tile}", f"s_add_u32 {sr(S_RA)}, {sr(S_RA)}, %[lds]",
          f"s_mul_i32 {sr(S_RB)}, {sr(S_T1)}, {4 * f.tile}", f"s_add_u32 {sr(S_RB)}, {sr(S_RB)}, {offb}",
          f"s_add_u32 {sr(S_RB)}, {sr(S_RB)}, %[lds]"]
    if f.ta == 4:
        o += [f"s_lshl_b32 {sr(S_RSA)}, {sr(S_T0)}, 8", f"s_add_u32 {sr(S_RSA)}, {sr(S_RSA)}, {offs}"]
    else:
        o += [f"s_mov_b32 {sr(S_RSA)}, {offs}"]
    o += [f"s_add_u32 {sr(S_RSA)}, {sr(S_RSA)}, %[lds]",
          f"s_lshl_b32 {sr(S_RSB)}, {sr(S_T1)}, 8", f"s_add_u32 {sr(S_RSB)}, {sr(S_RSB)}, {offs + 512}",
          f"s_add_u32 {sr(S_RSB)}, {sr(S_RSB)}, %[lds]",
          f"s_mul_i32 {sr(S_DA)}, %[wv], {(f.ta // 2) * f.tile}", f"s_add_u32 {sr(S_DA)}, {sr(S_DA)}, %[lds]",
          f"s_mul_i32 {sr(S_DB)}, %[wv], {2 * f.tile}", f"s_add_u32 {sr(S_DB)}, {sr(S_DB)}, {offb}",
          f"s_add_u32 {sr(S_DB)}, {sr(S_DB)}, %[lds]"]
    if f.ta == 4:
        o += [f"s_lshl_b32 {sr(S_DS)}, %[wv], 8"]
    else:                             # scale chunks: wave 0 and 1 -> the A group (slot 0), waves 2, 3 -> B groups (slots 2, 3)
        o += [f"s_cmp_lt_u32 %[wv], 2", f"s_cselect_b32 {sr(S_DS)}, 0, %[wv]", f"s_lshl_b32 {sr(S_DS)}, {sr(S_DS)}, 8"]
    o += [f"s_add_u32 {sr(S_DS)}, {sr(S_DS)}, {offs}", f"s_add_u32 {sr(S_DS)}, {sr(S_DS)}, %[lds]",
          f"s_lshl_b32 {sr(S_T1)}, {sr(S_T0)}, 4"]              # S_T1 = 16 wm: shift of the A scale dword (128-row form)
    for q in range(f.groups):
        goff = q * f.per_group * f.stage
        for i, (s, lane) in enumerate(((S_RA, "%[l16]"), (S_RB, "%[l16]"), (S_RSA, "%[l4]"), (S_RSB, "%[l4]"))):
            o += [f"s_add_u32 {sr(S_T0)}, {sr(s)}, {goff}", f"v_add_u32 {vr(VBASE + 4 * q + i)}, {sr(S_T0)}, {lane}"]
    o += [f"s_mov_b32 {sr(S_VC)}, 0",
          f"v_mov_b32 {vr(VOFF)}, %[g16]", f"v_mov_b32 {vr(VSOFF)}, %[g4]", f"v_mov_b32 {vr(VOFF2)}, %[g12]"]
    # pipeline fill: steps 0 .. dist-1 into stages 0 .. dist-1
    for st in range(f.dist):
        for m0, loads in dma_groups(f, st):
            o += [m0, "s_nop 0"] + loads
        o += advance_global(f)
    # step 0's operands into set 0
    o += [f"s_waitcnt vmcnt({(f.dist - 1) * f.per_step})", "s_barrier"]
    o += frag_reads(f, 0, 0) + ["s_waitcnt lgkmcnt(0)"]
    if f.ta == 2:
        o.append(f"v_lshrrev_b32 {vr(SA[0])}, {sr(S_T1)}, {vr(SA[0])}")
    return o


def main_loop(f):
    o = entry(f)
    o.append("80:")
    for u in range(f.nst):
        o += step(f, u)
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
    parts.append("#define DFP4_NATIVE_LOOP_FP4_H \\\n" + c_string(main_loop(Fmt(False, 2))) + "\n")
    parts.append("#define DFP4_NATIVE_LOOP_FP6_H \\\n" + c_string(main_loop(Fmt(True, 2))) + "\n")
    for g in range(16):
        rd = [f"v_accvgpr_read_b32 %{i}, a{16 * g + i}" for i in range(16)]
        parts.append(f"#define DFP4_NATIVE_ACC_READ_{g} \\\n" + c_string(rd) + "\n")
    vclob = ", ".join(f'"v{n}"' for n in range(40, 170))
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
