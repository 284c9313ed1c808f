#!/usr/bin/env python3
"""Generator of gemm_step_asm.inc: the hand-scheduled main loop of gemm_fast_kernel.

Why assembly.  The fast GEMM kernel runs ONE wavefront per SIMD (its 128 x 128
int32 accumulators fill the 256 accumulation registers), and a lone wavefront
issues one instruction every 4 cycles or so.  A v_mfma_i32_32x32x32_i8 occupies
the matrix core for 8 such slots, so about 5 other instructions fit in the shadow
of each MFMA -- but only if they are placed between the MFMAs, in program order.
The compiler's scheduler does not keep such an order, and operands prefetched for
the next step must stay in fixed registers from one step to the next, so the
whole loop (with its own loop control) is emitted here.

One step = one pair of (block, class) visits = 32 MFMAs per wave:
  wave w owns rows 128w .. 128w+127 of the 512 x 128 tile (groups gi = 0..3 of 32
  rows) and all four 32-column tiles n = 0..3; accumulator tile (gi, n) is
  a[16*(4*gi+n) : +15].  MFMA slot k: t = k / 16 (which half of the pair's
  operands), gi = (k % 16) / 4, n = k % 4:  acc[gi][n] += A[gi][t] * B[n][t].

  A operands (pre-expanded int8 fragments in global memory) are private to the
  wave: 8 global loads per step straight into registers, two steps ahead, three
  register sets used in rotation (step s uses set s % 3).
  B operands: every wave expands the 4-bit codes of ITS 32 rows of W (two steps
  ahead, v_perm_b32 lookups, 28 two-instruction pieces spread over the slots),
  writes the int8 result to LDS, and all four waves read the 8 fragments of a
  step from there (three LDS buffers in rotation, one barrier per step).
  The codes and table offsets come by global loads four steps ahead (three
  register sets in rotation).
  The list of visits sits in LDS (uint16: block | class of A << 10 | class of W << 12); the load offsets
  of the next step are computed at the end of each step.

The loop is unrolled three times (register sets); after every step the step
counter is compared with the end of the current class segment and a small
subroutine (s_call_b64) shifts the accumulators left by 4 between classes
(Horner's scheme) or leaves the loop after the last one.

Registers (all fixed):
  a[0:255]                accumulators
  v[40:135]               A sets 0..2: fragment f = 4*t + gi at set + 4*f
  v[136:151], v[152:167]  B fragments of phase t = 0 / 1: n at + 4*n
  v[168:179], v[180:182]  W codes sets 0..2 (4 registers each), table offsets 0..2
  v[184:187], v188        dialect table of the current expansion, its LDS address
  v[192:223]              temporaries of the W expansion (8 per code dword)
  v[224:231]              expanded int8 operands (t = 0: 224..227, t = 1: 228..231)
  v232 .. v243            visit entries, load offsets, LDS addresses
  s[60:75]                global base of the wave's A fragments f = 0..7
  s76 step counter, s77 end of segment, s78 segment, s[80:81] return address,
  s82..s84 LDS buffers of B (current, next, being written), s85..s87 scratch,
  s[88:91] W codes / table-offset bases

Run `python gen_gemm_step.py` in this directory to rewrite gemm_step_asm.inc
(the build does it, and the file is committed).
"""
import os

ASET = [40, 72, 104]
BBUF = [136, 152]
CODES = [168, 172, 176]
META = [180, 181, 182]
TAB0, TABADDR = 184, 188
TMP0, OUT0 = 192, 224
EA, EW, VOFF, VCOFF, VMOFF, VLADDR, SB, SBN, SBW, L16W, T0, T1 = range(232, 244)
S_ABASE, S_VC, S_SEGEND, S_SEG, S_RET, S_BCUR, S_BNXT, S_BW, S_T0, S_T1 = 60, 76, 77, 78, 80, 82, 83, 84, 85, 86
S_WC, S_WM = 88, 90
NSLOT = 32
# Timing experiments only (results are wrong, every address stays the same): a comma-separated list in
# DFP4_GEN_EXP drops parts of the step -- noexpand (W expansion), nobarrier, noaload (A loads), nobread (LDS reads of B),
# nomfma (the MFMAs themselves), nowload (loads of W codes and table offsets).
EXP = set(filter(None, os.environ.get('DFP4_GEN_EXP', '').split(',')))
FRAG = 1024                    # bytes per operand fragment
B_BUF_BYTES = 8 * FRAG


def vr(n, cnt=1):
    return f"v{n}" if cnt == 1 else f"v[{n}:{n + cnt - 1}]"


def sr(n, cnt=1):
    return f"s{n}" if cnt == 1 else f"s[{n}:{n + cnt - 1}]"


class Lgkm:
    """In-order queue of outstanding LDS operations, to compute s_waitcnt lgkmcnt(n)."""

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


def expansion_pieces(cset):
    """The 28 two-instruction pieces that expand the four code dwords of code set
    `cset` (see unpack8 in gemm.hip): 16 that need only the codes, then 12 that
    need the dialect table."""
    first, second = [], []
    for d in range(4):
        c = vr(CODES[cset] + d)
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
            [f"v_bfi_b32 {vr(OUT0 + 2 * d)}, {me}, {ne}, {pe}", f"v_bfi_b32 {vr(OUT0 + 2 * d + 1)}, {mo}, {no}, {po}"],
        ]
    return first, second


def a_offset(entry, dst):
    """byte offset of a visit's A fragments: class * class stride + block * 1 KiB + (tile, lane)"""
    return [f"v_bfe_u32 {vr(T0)}, {vr(entry)}, 10, 2",
            f"v_mul_lo_u32 {vr(T0)}, {vr(T0)}, %[cstr]",
            f"v_and_b32 {vr(T1)}, 0x3ff, {vr(entry)}",
            f"v_lshl_add_u32 {vr(T0)}, {vr(T1)}, 10, {vr(T0)}",
            f"v_add3_u32 {vr(dst)}, {vr(T0)}, %[toff], %[alane]"]


def w_offsets(entry, dst_codes, dst_meta):
    """byte offsets of a visit's W codes and of its table offset for the visit's class of W
    (padding visits read the last block)"""
    return [f"v_and_b32 {vr(T1)}, 0x3ff, {vr(entry)}",
            f"v_min_u32 {vr(T1)}, %[kbm], {vr(T1)}",
            f"v_lshl_add_u32 {vr(dst_codes)}, {vr(T1)}, 9, %[wrc]",      # [group][block][row]: 512 bytes of codes
            f"v_lshl_add_u32 {vr(dst_meta)}, {vr(T1)}, 7, %[wrm]",       # and 128 bytes of table dwords per block
            f"v_bfe_u32 {vr(T0)}, {vr(entry)}, 12, 2",
            f"v_mul_lo_u32 {vr(T0)}, {vr(T0)}, %[wcs]",
            f"v_add_u32 {vr(dst_meta)}, {vr(dst_meta)}, {vr(T0)}"]


AFLAGS = os.environ.get('DFP4_GEN_AFLAGS', '')        # timing experiments: cache-policy bits of the A loads


def a_loads(aset, voff):
    return [f"global_load_dwordx4 {vr(ASET[aset] + 4 * f, 4)}, {vr(voff)}, {sr(S_ABASE + 2 * f, 2)}" + (" " + AFLAGS if AFLAGS else "")
            for f in range(8)]


# Slots (MFMA index within the step) after which the vector-memory loads of a step are issued.
# DFP4_GEN_ASLOTS=early (timing experiments) issues the A loads in the first half of the step.
# Slots (MFMA index within the step) after which the eight A loads of a step are issued.  Measured and
# found to make no difference: issuing them in the first half of the step (DFP4_GEN_ASLOTS=early), and
# giving each wave its own copy of the loop with the loads one slot apart from the other waves'.
A_LOAD_SLOT = ({1 + 2 * i: i for i in range(8)} if os.environ.get('DFP4_GEN_ASLOTS') == 'early'
               else {1 + 4 * i: i for i in range(8)})                      # default: slots 1, 5, ..., 29
CODES_SLOT, META_SLOT = ((0, 2) if os.environ.get('DFP4_GEN_WSLOTS') == 'early' else (11, 15))


# LDS operations of a step that its own waits do not cover, in issue order: next step's phase-0 B
# fragments (slots 16, 20, 24, 27) and the writes of the expanded operands (slots 22, 28)
LDS_TAIL = (["w0", "w1"] if "nobread" in EXP else ["b00", "b01", "w0", "b02", "b03", "w1"])


def vm_order():
    """Tags of a step's vector-memory loads in issue order (the memory counter retires them in this
    order): 'A0'..'A7', 'codes', 'meta'."""
    slots = A_LOAD_SLOT
    o = []
    for k in range(NSLOT):
        if k in slots and "noaload" not in EXP:
            o.append(f"A{slots[k]}")
        if k == CODES_SLOT and "nowload" not in EXP:
            o.append("codes")
        if k == META_SLOT and "nowload" not in EXP:
            o.append("meta")
    return o


class Vm:
    """s_waitcnt vmcnt(n) for a load issued two steps ago, given how many loads this step has issued."""

    def __init__(self):
        self.order = vm_order()
        self.issued = 0                 # loads issued so far in the current step
        self.done = -1                  # index (two steps ago) known to have arrived

    def issue(self):
        self.issued += 1

    def need(self, tag):
        i = self.order.index(tag)
        if i <= self.done:
            return None
        self.done = i
        n = len(self.order)
        return f"s_waitcnt vmcnt({(n - 1 - i) + n + self.issued})"


# Timing experiment (DFP4_GEN_ADIST=3): every load three steps ahead instead of two, without a fourth
# register set -- fragment f of the set a step multiplies with is loaded again, for the step three
# later, right after its last MFMA (slot 4 f + 5; fragment 7 at slot 1 of the next step), and the
# W codes and table offset of the set a step expands at slot 16, once the expansion has read them.
# Results are bit-identical to the default schedule; measured, it is no faster (the pipeline fill of
# this variant waits for all its loads once per tile, which costs about what the deeper prefetch gains).
ADIST3 = os.environ.get('DFP4_GEN_ADIST') == '3'
ORDER3 = ["A7", "A0", "A1", "A2", "codes", "meta", "A3", "A4", "A5", "A6"]      # issue order of a step
SLOT3 = {1: 7, 5: 0, 9: 1, 13: 2, 17: 3, 21: 4, 25: 5, 29: 6}


class Vm3:
    def __init__(self):
        self.issued = 0

    def issue(self):
        self.issued += 1

    def need(self, tag):
        ago = 2 if tag == "A7" else 3                 # codes and table offsets too: their set is loaded
                                                      # again at slot 16, once the expansion has read it
        i, n = ORDER3.index(tag), len(ORDER3)
        return f"s_waitcnt vmcnt({(n - 1 - i) + (ago - 1) * n + self.issued})"


def entry_code():
    o = []
    # global bases of the wave's 8 A fragments: a8w + gi * group stride + t * 512
    o.append(f"s_mov_b32 {sr(S_T0)}, 0")
    for gi in range(4):
        lo, hi = S_ABASE + 2 * gi, S_ABASE + 2 * gi + 1
        o += [f"s_add_u32 {sr(lo)}, %[a8lo], {sr(S_T0)}", f"s_addc_u32 {sr(hi)}, %[a8hi], 0"]
        lo1, hi1 = S_ABASE + 2 * (4 + gi), S_ABASE + 2 * (4 + gi) + 1
        o += [f"s_add_u32 {sr(lo1)}, {sr(lo)}, 0x200", f"s_addc_u32 {sr(hi1)}, {sr(hi)}, 0"]
        o.append(f"s_add_u32 {sr(S_T0)}, {sr(S_T0)}, %[gstr]")
    o += [f"s_mov_b32 {sr(S_WC)}, %[wclo]", f"s_mov_b32 {sr(S_WC + 1)}, %[wchi]",
          f"s_mov_b32 {sr(S_WM)}, %[wmlo]", f"s_mov_b32 {sr(S_WM + 1)}, %[wmhi]"]
    o += [f"s_mov_b32 {sr(S_BCUR)}, %[bb]", f"s_add_u32 {sr(S_BNXT)}, %[bb], {B_BUF_BYTES}",
          f"s_add_u32 {sr(S_BW)}, %[bb], {2 * B_BUF_BYTES}"]
    o += [f"s_lshl_b32 {sr(S_T0)}, %[wv], 11", f"v_add_u32 {vr(L16W)}, {sr(S_T0)}, %[l16]",
          f"v_add_u32 {vr(VLADDR)}, %[vlb], %[h2]"]
    o += [f"s_mov_b32 {sr(S_VC)}, 0", f"s_mov_b32 {sr(S_SEG)}, 0", f"s_mov_b32 {sr(S_SEGEND)}, %[e2]"]
    # pipeline fill: A of pairs 0, 1; W codes and table offsets of pairs 2, 3
    for p in range(3 if ADIST3 else 2):
        o += [f"ds_read_u16 {vr(EA)}, {vr(VLADDR)} offset:{4 * p}",
              f"ds_read_u16 {vr(EW)}, {vr(VLADDR)} offset:{4 * (p + 2)}",
              "s_waitcnt lgkmcnt(0)"]
        o += a_offset(EA, VOFF) + w_offsets(EW, VCOFF, VMOFF)
        al = a_loads(p, VOFF)
        if p == 2:
            o += al + [f"global_load_dwordx4 {vr(CODES[p], 4)}, {vr(VCOFF)}, {sr(S_WC, 2)}",
                       f"global_load_dword {vr(META[p])}, {vr(VMOFF)}, {sr(S_WM, 2)}"]
            continue
        for tag in vm_order():                         # same order as inside a step: the waits count on it
            o.append(al[int(tag[1:])] if tag[0] == "A" else
                     f"global_load_dwordx4 {vr(CODES[p], 4)}, {vr(VCOFF)}, {sr(S_WC, 2)}" if tag == "codes" else
                     f"global_load_dword {vr(META[p])}, {vr(VMOFF)}, {sr(S_WM, 2)}")
    if "nowload" in EXP:                             # the registers the loads would have filled: zeros
        o += [f"v_mov_b32 {vr(r)}, 0" for r in list(range(CODES[0], CODES[2] + 4)) + META]
    if ADIST3:
        # everything loaded so far has arrived (the experiment pays one memory latency per tile for it);
        # VOFF stays that of pair 2 (slot 1 of step 0 loads its fragment 7 once more), EA = visit of step 3
        o += ["s_waitcnt vmcnt(0)", f"ds_read_u16 {vr(EA)}, {vr(VLADDR)} offset:12", "s_waitcnt lgkmcnt(0)"]
    else:
        # offsets of the loads of step 0 (A of pair 2, W of pair 4)
        o += [f"ds_read_u16 {vr(EA)}, {vr(VLADDR)} offset:8", f"ds_read_u16 {vr(EW)}, {vr(VLADDR)} offset:16",
              "s_waitcnt lgkmcnt(0)"]
        o += a_offset(EA, VOFF) + w_offsets(EW, VCOFF, VMOFF)
    # B fragments of step 0, phase 0
    o.append(f"v_add_u32 {vr(SB)}, {sr(S_BCUR)}, %[l16]")
    for n in range(4):
        o.append(f"ds_read_b128 {vr(BBUF[0] + 4 * n, 4)}, {vr(SB)} offset:{(2 * n) * FRAG}")
    o.append("s_waitcnt lgkmcnt(0)")
    return o


UNROLL = 3                      # steps per loop iteration (a multiple of the 3 register sets)


def step(v, u=None):
    """One step with A set v, code set v (both step % 3); u: its position in the unrolled loop.  Everything that is not an MFMA is
    spread over the MFMA slots, the barrier included, so that the matrix core never waits at
    the step boundary."""
    o = []
    # LDS operations complete in order.  Those the previous step issued after its last wait may still
    # be in flight (next-phase B fragments read from slot 16 on, the two writes of expanded operands):
    # they are waited for where this step first needs them, not at the step boundary.
    lg = Lgkm()
    tail = ["b00", "b01", "w0", "b02", "b03", "ea", "w1"] if ADIST3 else LDS_TAIL
    lg.q = ["p:" + t for t in tail]
    ld = (v + 2) % 3
    u = v if u is None else u
    # the common path falls through; the end of a class segment (three times per tile) is handled out of line
    o.append(f"s_cmp_lt_u32 {sr(S_VC)}, {sr(S_SEGEND)}")
    o.append(f"s_cbranch_scc0 2{u}f")
    o.append(f"1{u}:")
    # Loads issued two steps ago are waited for where they are first used, not all at the step's
    # start: the W codes now, the table offset at slot 3, A fragment f before MFMA slot 4 f.
    a_load_slot = SLOT3 if ADIST3 else A_LOAD_SLOT
    vm = Vm3() if ADIST3 else Vm()
    if "nowload" not in EXP:
        o.append(vm.need("codes"))
    first, second = expansion_pieces(v)
    loads = a_loads(ld, VOFF)
    if ADIST3:                  # this step's own set, except fragment 7: that of the previous step's set
        loads = a_loads(v, VOFF)[:7] + [a_loads(ld, VOFF)[7]]
    b_reads = {2: (1, 0), 6: (1, 1), 10: (1, 2), 14: (1, 3), 16: (0, 0), 20: (0, 1), 24: (0, 2), 27: (0, 3)}
    extra = {
        0: [f"v_add_u32 {vr(SB)}, {sr(S_BCUR)}, %[l16]", f"v_add_u32 {vr(SBN)}, {sr(S_BNXT)}, %[l16]"],
        1: [f"v_add_u32 {vr(SBW)}, {sr(S_BW)}, {vr(L16W)}"],
        3: ([] if ADIST3 else [f"ds_read_u16 {vr(EA)}, {vr(VLADDR)} offset:12"]) + [f"ds_read_u16 {vr(EW)}, {vr(VLADDR)} offset:20",
            f"v_add_u32 {vr(TABADDR)}, %[tabb], {vr(META[v])}", f"ds_read_b128 {vr(TAB0, 4)}, {vr(TABADDR)}"],
        4: [f"s_mov_b32 {sr(S_T0)}, {sr(S_BCUR)}", f"s_mov_b32 {sr(S_BCUR)}, {sr(S_BNXT)}",
            f"s_mov_b32 {sr(S_BNXT)}, {sr(S_BW)}", f"s_mov_b32 {sr(S_BW)}, {sr(S_T0)}"],
        7: [f"s_add_u32 {sr(S_VC)}, {sr(S_VC)}, 1", f"v_add_u32 {vr(VLADDR)}, 4, {vr(VLADDR)}"],
        # every wave has written its share of the W operands of the next step (previous step,
        # waited for at its end) and has finished reading the buffer this step overwrites
        12: [] if "nobarrier" in EXP else ["s_barrier"],
    }
    if ADIST3:
        extra[2] = a_offset(EA, VOFF)                 # after fragment 7 of the previous visit (slot 1)
        extra[28] = [f"ds_read_u16 {vr(EA)}, {vr(VLADDR)} offset:12"]     # the visit three steps after the next
    for k in range(NSLOT):
        t, gi, n = k // 16, (k % 16) // 4, k % 4
        if k >= 16:
            w = lg.need(f"b1{n}")
            if w:
                o.append(w)
        acc = f"a[{16 * (4 * gi + n)}:{16 * (4 * gi + n) + 15}]"
        if k < 4:                                     # phase-0 fragment n, read during the previous step
            w = lg.need(f"p:b0{n}")
            if w:
                o.append(w)
        if k % 4 == 0 and "noaload" not in EXP:
            w = vm.need(f"A{k // 4}")
            if w:
                o.append(w)
        if "nomfma" not in EXP:
            o.append(f"v_mfma_i32_32x32x32_i8 {acc}, {vr(ASET[v] + 4 * (4 * t + gi), 4)}, {vr(BBUF[t] + 4 * n, 4)}, {acc}")
        if k in b_reads and "nobread" not in EXP:
            bt, bn = b_reads[k]
            src = SB if bt == 1 else SBN
            o.append(f"ds_read_b128 {vr(BBUF[bt] + 4 * bn, 4)}, {vr(src)} offset:{(2 * bn + bt) * FRAG}")
            lg.issue(f"b{bt}{bn}")
        piece = first[k] if k < 16 else (second[k - 16] if k - 16 < len(second) else None)
        if k == 16:
            w = lg.need("tab")
            if w:
                o.append(w)
        if piece and "noexpand" in EXP:
            piece = None
        if piece:
            o.append(piece[0])
        if k in a_load_slot and "noaload" not in EXP:
            o.append(loads[a_load_slot[k]])
            vm.issue()
        wset = v if ADIST3 else ld
        if k == (16 if ADIST3 else CODES_SLOT) and "nowload" not in EXP:
            o.append(f"global_load_dwordx4 {vr(CODES[wset], 4)}, {vr(VCOFF)}, {sr(S_WC, 2)}")
            vm.issue()
        if k == (16 if ADIST3 else META_SLOT) and "nowload" not in EXP:
            o.append(f"global_load_dword {vr(META[wset])}, {vr(VMOFF)}, {sr(S_WM, 2)}")
            vm.issue()
        if piece:
            o.append(piece[1])
        if k == 3 and "nowload" not in EXP:           # the table offset of this step's expansion
            w = vm.need("meta")
            if w:
                o.append(w)
        if k == 12:                                   # own writes of the previous step, before the barrier
            w = lg.need("p:w1")
            if w:
                o.append(w)
        if k == 2 and ADIST3:
            w = lg.need("p:ea")
            if w:
                o.append(w)
        for ins in extra.get(k, []):
            o.append(ins)
            if ins.startswith("ds_read_u16") or ins.startswith("ds_read_b128"):
                lg.issue({"ds_read_u16 " + vr(EA): "ea", "ds_read_u16 " + vr(EW): "ew"}.get(ins.split(",")[0], "tab"))
        if k == 22:
            o.append(f"ds_write_b128 {vr(SBW)}, {vr(OUT0, 4)}")
            lg.issue("w0")
        if k == 28:
            o.append(f"ds_write_b128 {vr(SBW)}, {vr(OUT0 + 4, 4)} offset:{FRAG}")
            lg.issue("w1")
        if k == (13 if ADIST3 else 30):               # after the last A load of this step
            w = lg.need("ew")
            if w:
                o.append(w)
            if not ADIST3:
                o += a_offset(EA, VOFF)
        if k == (13 if ADIST3 else 31):
            o += w_offsets(EW, VCOFF, VMOFF)
    # what is still in flight here is what the next step expects
    assert lg.q == tail, (lg.q, tail)
    return o


DRAIN = ["s_nop 15", "s_nop 15", "s_nop 15"]       # all MFMAs have retired before the vector ALU reads accumulators


def shift4():
    o = list(DRAIN)
    for n0 in range(0, 256, 8):
        o += [f"v_accvgpr_read_b32 {vr(TMP0 + i)}, a{n0 + i}" for i in range(8)]
        o += [f"v_lshlrev_b32 {vr(TMP0 + i)}, 4, {vr(TMP0 + i)}" for i in range(8)]
        o += [f"v_accvgpr_write_b32 a{n0 + i}, {vr(TMP0 + i)}" for i in range(8)]
    o.append("s_nop 4")
    return o


def handler():
    """Reached when the step counter equals the end of the segment: shift the accumulators
    and move to the next class, or leave the loop after the last one."""
    o = ["90:", f"s_cmp_eq_u32 {sr(S_SEG)}, 2", "s_cbranch_scc1 99f",
         f"s_cmp_eq_u32 {sr(S_VC)}, 0", "s_cbranch_scc1 91f"]
    o += shift4()
    o += ["91:", f"s_add_u32 {sr(S_SEG)}, {sr(S_SEG)}, 1", f"s_cmp_eq_u32 {sr(S_SEG)}, 1",
          f"s_cselect_b32 {sr(S_SEGEND)}, %[e1], %[e0]", f"s_cmp_lt_u32 {sr(S_VC)}, {sr(S_SEGEND)}",
          "s_cbranch_scc0 90b", f"s_setpc_b64 {sr(S_RET, 2)}"]
    return o


def main_loop():
    o = [f"v_accvgpr_write_b32 a{n}, 0" for n in range(256)]
    o += entry_code()
    o.append("80:")
    for u in range(UNROLL):
        o += step(u % 3, u)
    o.append("s_branch 80b")
    for u in range(UNROLL):                      # out of line: the step counter has reached the segment's end
        o += [f"2{u}:", f"s_call_b64 {sr(S_RET, 2)}, 90f", f"s_branch 1{u}b"]
    o += handler()
    o += ["99:", "s_waitcnt vmcnt(0) lgkmcnt(0)"] + DRAIN
    return o


def c_string(lines):
    return " \\\n".join(f'    "{l}\\n\\t"' for l in lines)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    parts = ["// Generated by gen_gemm_step.py -- do not edit; see that file for the register map.\n"]
    parts.append("#define DFP4_MAINLOOP_ASM \\\n" + c_string(main_loop()) + "\n")
    for g in range(16):
        rd = [f"v_accvgpr_read_b32 %{i}, a{16 * g + i}" for i in range(16)]
        parts.append(f"#define DFP4_ACC_READ_ASM_{g} \\\n" + c_string(rd) + "\n")
    vclob = ", ".join(f'"v{n}"' for n in range(ASET[0], 256))
    aclob = ", ".join(f'"a{n}"' for n in range(256))
    sclob = ", ".join(f'"s{n}"' for n in range(S_ABASE, S_WM + 2))
    parts.append(f"#define DFP4_LOOP_VGPR_CLOBBERS {vclob}\n")
    parts.append(f"#define DFP4_ACC_CLOBBERS {aclob}\n")
    parts.append(f"#define DFP4_LOOP_SGPR_CLOBBERS {sclob}\n")
    path = os.path.join(here, "gemm_step_asm.inc")
    text = "\n".join(parts)
    if not os.path.exists(path) or open(path).read() != text:
        with open(path, "w") as f:
            f.write(text)
    return path


if __name__ == "__main__":
    print(main())
