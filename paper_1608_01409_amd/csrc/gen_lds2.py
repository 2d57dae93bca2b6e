#!/usr/bin/env python3
"""Writes sconv_lds2_asm.inc: the body of the flat-stream LDS kernel, one asm statement per
accumulator shape (T chunks of 64 positions x 4 images per lane, R rows per wave).

Everything between the first and the last multiply-add of a workgroup's tile runs inside this one
statement, because the accumulators live in a contiguous block of fixed VGPRs that is addressed
through the VGPR index mode (s_set_gpr_idx_on): the row an entry of the nonzero stream belongs to is
data, not code, so the rows of a wave share one stream with no per-row padding.

  stream   per (wave slot, channel block): chunks of 8 entries of 8 bytes,
           word0 = fp32 weight, word1 = (LDS byte offset / 16) << 16 | (row * T * 4): the read address
           is one v_mad_u32_u16 (high half x 16 + lane base), the accumulator index is the low byte.
           Three chunk buffers A (in use), B (next, valid), N (loading); the loop body is unrolled
           three times with the names rotated, so no register moves are needed.
  reads    entry p reads T float4 at lane_base + offset + t*step*16 (ds_read_b128); the reads of entry
           p + D are issued while entry p is multiplied (ring of D*T float4).  LDS returns in order,
           so the oldest read is complete once lgkmcnt <= D*T - 1; the scalar load of chunk N only
           makes that wait stricter, and lgkmcnt(0) at the end of a chunk makes N valid.
  fma      v_fmac_f32 acc(t, e), weight (SGPR), ring(t, e) with the destination indexed by M0.
  staging  block b+1 streams from global memory straight into the other LDS buffer
           (buffer_load_dword ... lds, one instruction per 64 floats, no VGPR data) while block b is
           multiplied.  Lanes whose cell is zero padding carry an out-of-range buffer offset and
           receive 0 from the hardware's range check; lanes past the end of a plane are masked off.
  stores   row bases from row_of, per-lane store offsets from a table (-1 = not an output).

Two ways of keeping the waves of a workgroup in step with the block buffers (template parameter FLOW):

  barrier  two buffers, one s_barrier per channel block: past it every wave's loads of block b have landed
           and every wave is done with the buffer that block b+1 is about to overwrite.  Every block then
           costs what its slowest wave costs, plus a collective start-up (all waves issue their staging
           loads and first reads at once) and a tail in which ever fewer waves are left working.
  flow     three buffers and no barrier after the first.  Each wave issues its share of block b+1's loads
           when it starts block b (into the buffer block b-2 used), and a few chunks into block b, once
           those loads have landed, adds 1 to an LDS counter S[b+1].  A wave starts block b when S[b]
           shows every wave's share of block b present.  A wave that signals S[b+1] is inside block b, so
           S[b+1] complete also means every wave has left block b-1: its buffer may be overwritten with
           block b+2.  Only the first few waves of a workgroup have a share (the kernel hands the slabs to
           the waves the SIMDs serve first, which run ahead); a wave without one adds its 1 on entering
           block b, so S[b+1] fills when the early waves' loads are in and the late waves have entered
           block b: waves drift up to a block apart, and nobody waits for the slowest wave to be well into a
           block.  (FLOW_LOOK = 2 is the same with four buffers, loads two blocks ahead and the
           landing reported when the block during which they were issued is finished: measured slower,
           the blocks being a quarter shorter.)
"""
from __future__ import annotations

import os
import sys

# (T, R, D, batch, step): batch = compute the 8 read addresses of a chunk at once (8 address VGPRs) instead of
# one at a time with the index mode toggled off and on around each (D address VGPRs, for shapes short of VGPRs);
# step = LDS cells between the reads of consecutive chunks of one lane: 64 when the lanes of a wave span 64
# consecutive cells of the plane (chunk t = the next 64 cells), w when they span a block of 64/w rows by w
# columns (chunk t = the same rows, the next w columns).  The step is an immediate of the read instruction.
SHAPES = [
    (1, 8, 4, True, 64), (1, 12, 4, True, 64), (1, 16, 4, True, 64), (2, 8, 4, True, 64), (2, 12, 1, True, 64), (3, 4, 2, True, 64), (3, 6, 2, True, 64),
    (3, 8, 1, True, 64), (4, 4, 2, True, 64), (4, 5, 1, True, 64), (5, 3, 2, True, 64), (5, 4, 1, True, 64),
    (6, 3, 1, True, 64), (7, 2, 2, False, 64), (7, 3, 1, False, 64), (13, 1, 1, False, 64),
    (3, 4, 2, True, 9), (3, 6, 2, True, 9), (3, 8, 1, True, 9),            # 27 columns in 3 strips of 9
    (7, 2, 2, False, 8), (7, 3, 1, False, 8),                              # 55 or 56 columns in 7 strips of 8
]
CH = 8                      # entries per chunk
W = 2 * CH                  # dwords per chunk
# SGPRs owned by the asm: s28-s31, s34-s99 (s32, s33, s100 and up are left to the compiler)
SCB, SREM, SSOFF = 28, 29, 30
SEXEC = 34
SA, SB, SN = 36, 52, 68
SPTR, SCNT, STMP = 84, 86, 87
SHALF, SLEFT, SSEG = 88, 89, 90                  # first chunk of the block is a half chunk; blocks left
SBUF, SSTRIDE, SPLANE, SHW4 = 92, 93, 94, 95
SOFF, SS, SNCH, STGT = 96, 97, 98, 99            # stream byte offset; staging temporaries
SNXT = 31                                        # chunks in the next block's segment
SX0, SX1 = SSEG, SSEG + 1                        # store address pair: the segment pointer is done by then
MAX_VGPR = 128
# flow: how many blocks ahead of the one being multiplied a wave issues loads.  1: three buffers, the landing is
# reported from inside the block loop (at the SIGNAL_AFTER-th first-of-three chunk, or at the segment's end);
# 2: four buffers, the landing is reported when the wave finishes the block during which the loads were issued.
FLOW_LOOK = 1
FLOW_BUFS = FLOW_LOOK + 2
SIGNAL_AFTER = 2
# L2 warming of the stream: each lane of one load touches one line of this many bytes, 64 lines from the point the
# scalar loads have reached.  The host pads the stream by WARM_BYTES so that the last wave slot's loads stay inside.
WARM_LINE_SHIFT = 6
WARM_BYTES = 64 << WARM_LINE_SHIFT

# kernel-argument offsets the asm reads (checked by static_asserts next to the struct)
OFF_PAIRS, OFF_TBL, OFF_CONSTS = 16, 40, 48   # consts: cb nblk Cg plane stride HW4 OHW4 img_stride
OFF_PHASE = 264                                # blocks per phase, stride, source row bytes, bytes of one phase's channels: set below

OPS = ["kern", "rsrc", "segp", "rowp", "outp", "soff0", "nimg", "lim", "ldsbase", "slab0", "slabstep", "nslab",
       "lane_byte", "voff0", "voff1", "voff2", "voff3", "tbloff", "outp_hi", "nch", "nblk", "bias", "flags", "nwv"]
# in/out: LDS byte address of the counter of the block the wave is in (flow only); blocks left to stage before the
# channel walk passes into the next phase of a strided layer, and that phase's column (both idle for other layers)
IO_OPS = ["ctr", "wrap", "px"]
FLAG_RELU = 0                  # bits of the flags operand
FLAG_WIDE = 1                  # stage whole cells (16 bytes a lane) instead of dwords
OP = {n: f"%[{n}]" for n in OPS + IO_OPS}


def gen_shape(T: int, R: int, D: int, batch: bool, step: int, flow: bool = False) -> str:
    assert CH % D == 0 and R * T * 4 <= 256
    nacc = R * T * 4
    ring_regs = D * T * 4
    n_va = CH if batch else D
    total = nacc + ring_regs + n_va + 4
    base = (MAX_VGPR - total) & ~3
    assert base >= 8, (T, R, D, base)
    ACC0 = base
    RING0 = ACC0 + nacc
    VA0 = RING0 + ring_regs
    VLB = VA0 + n_va        # lane base for the current buffer
    VS0, VS1 = VLB + 1, VLB + 2     # scratch of the counter operations (flow)
    VWARM = VLB + 3                 # destination of the loads that warm L2 with the stream: never read
    assert VWARM + 1 <= MAX_VGPR

    def q(slot, t, e=None):
        b = RING0 + (slot * T + t) * 4
        return f"v[{b}:{b + 3}]" if e is None else f"v{b + e}"

    def w0(buf, u):
        return f"s{buf + 2 * u}"

    def w1(buf, u):
        return f"s{buf + 2 * u + 1}"

    L = []
    emit = L.append
    uid = [0]

    def label(stem):
        uid[0] += 1
        return f".L{stem}{uid[0]}_%="

    def signal(off):
        """This wave's share of a block has landed: add 1 to the block's counter at ctr + off (one lane)."""
        emit("s_waitcnt vmcnt(0)")
        emit(f"s_add_u32 s{STMP}, {OP['ctr']}, {off}")
        emit(f"v_mov_b32 v{VS0}, s{STMP}")
        emit(f"v_mov_b32 v{VS1}, 1")
        emit("s_mov_b64 exec, 1")
        emit(f"ds_add_u32 v{VS0}, v{VS1}")
        emit(f"s_mov_b64 exec, s[{SEXEC}:{SEXEC + 1}]")

    def poll():
        """Wait until every wave has added its 1 to the counter at ctr.  Every wave of the workgroup reaches
        its signal for this counter without waiting for anything later than the previous counter, so the
        loop ends."""
        again, go = label("poll"), label("go")
        emit(f"v_mov_b32 v{VS0}, {OP['ctr']}")
        emit(f"{again}:")
        emit(f"ds_read_b32 v{VS1}, v{VS0}")
        emit("s_waitcnt lgkmcnt(0)")
        emit(f"v_readfirstlane_b32 s{STMP}, v{VS1}")
        emit(f"s_cmp_ge_u32 s{STMP}, {OP['nwv']}")
        emit(f"s_cbranch_scc1 {go}")
        emit("s_sleep 1")
        emit(f"s_branch {again}")
        emit(f"{go}:")

    def warm():
        """Pull the next WARM_BYTES of this wave's stream into L2: one vector load, a line per lane, result
        unused.  The stream reaches the chunk buffers through scalar loads that are waited for one chunk after
        they are issued; a workgroup whose stream nobody has read before (a layer with a single image tile: every
        fully connected layer) would otherwise pay a trip to HBM per chunk."""
        emit(f"v_mbcnt_lo_u32_b32 v{VS0}, -1, 0")
        emit(f"v_mbcnt_hi_u32_b32 v{VS0}, -1, v{VS0}")
        emit(f"v_lshlrev_b32 v{VS0}, {WARM_LINE_SHIFT}, v{VS0}")
        emit(f"v_add_u32 v{VS0}, s{SOFF}, v{VS0}")
        emit(f"global_load_dword v{VWARM}, v{VS0}, s[{SPTR}:{SPTR + 1}]")

    def stage_loads(tgt, load):
        """The loads of one block for the (at most four) slabs of this wave: per slab one instruction per channel,
        each lane moving a dword (16 cells x 4 images per instruction) or, where the four images of a cell are
        adjacent in memory, a whole cell (64 cells per instruction)."""
        emit(f"s_add_u32 s{STMP}, s{tgt}, {OP['slab0']}")
        end = label("stend")
        for j in range(4):
            emit(f"s_cmp_le_u32 {OP['nslab']}, {j}")
            emit(f"s_cbranch_scc1 {end}")
            emit(f"v_cmp_ne_u32_e32 vcc, -1, {OP['voff%d' % j]}")
            emit("s_mov_b64 exec, vcc")
            # two channels per trip; M0 (the LDS destination) and the scalar source offset advance in place.
            # An instruction always separates a write of M0 from the load that uses it.
            emit(f"s_mov_b32 m0, s{STMP}")
            emit(f"s_mov_b32 s{SS}, s{SSOFF}")
            emit(f"s_lshr_b32 vcc_lo, s{SNCH}, 1")       # vcc is free again: pairs of channels to go
            lp, tail, nxt = label("stj"), label("sttail"), label("stnext")
            emit("s_cmp_eq_u32 vcc_lo, 0")
            emit(f"s_cbranch_scc1 {tail}")
            emit(f"{lp}:")
            for _ in range(2):
                emit(f"{load} {OP['voff%d' % j]}, {OP['rsrc']}, s{SS} offen lds")
                emit(f"s_add_u32 m0, m0, s{SPLANE}")
                emit(f"s_add_u32 s{SS}, s{SS}, s{SHW4}")
            emit("s_sub_u32 vcc_lo, vcc_lo, 1")
            emit("s_cmp_lg_u32 vcc_lo, 0")
            emit(f"s_cbranch_scc1 {lp}")
            emit(f"{tail}:")
            emit(f"s_bitcmp1_b32 s{SNCH}, 0")
            emit(f"s_cbranch_scc0 {nxt}")
            emit(f"{load} {OP['voff%d' % j]}, {OP['rsrc']}, s{SS} offen lds")
            emit(f"{nxt}:")
            emit(f"s_add_u32 s{STMP}, s{STMP}, {OP['slabstep']}")
        emit(f"{end}:")

    def stage(tgt):
        """Issue the DMA loads of the next block (channels SSOFF.. , min(SCB, SREM) of them) into LDS at tgt."""
        emit(f"s_min_u32 s{SNCH}, s{SCB}, s{SREM}")
        wide, staged = label("stwide"), label("staged")
        emit(f"s_bitcmp1_b32 {OP['flags']}, {FLAG_WIDE}")
        emit(f"s_cbranch_scc1 {wide}")
        stage_loads(tgt, "buffer_load_dword")
        emit(f"s_branch {staged}")
        emit(f"{wide}:")
        stage_loads(tgt, "buffer_load_dwordx4")
        emit(f"{staged}:")
        emit(f"s_mov_b64 exec, s[{SEXEC}:{SEXEC + 1}]")
        emit(f"s_mul_i32 s{STMP}, s{SNCH}, s{SHW4}")
        emit(f"s_add_u32 s{SSOFF}, s{SSOFF}, s{STMP}")
        emit(f"s_sub_u32 s{SREM}, s{SREM}, s{SNCH}")
        # Strided layers staged straight from the caller's input: the virtual channels run phase by phase, and the
        # blocks of a phase are that phase's real channels, a regular walk.  Past a phase's last block the walk
        # returns to the group's first channel, one element further along the row (next column phase) or, past
        # the last column phase, one row further and back to column phase 0.  Other layers never get here.
        nowrap, nextrow, wrapped = label("nowrap"), label("nextrow"), label("wrapped")
        emit(f"s_sub_u32 {OP['wrap']}, {OP['wrap']}, 1")
        emit(f"s_cmp_lg_u32 {OP['wrap']}, 0")
        emit(f"s_cbranch_scc1 {nowrap}")
        emit(f"s_load_dwordx2 vcc, {OP['kern']}, {hex(OFF_PHASE)}")               # blocks per phase, stride
        emit(f"s_load_dwordx2 s[{SNCH}:{STGT}], {OP['kern']}, {hex(OFF_PHASE + 8)}")   # row bytes, bytes of a phase's channels
        emit("s_waitcnt lgkmcnt(0)")
        emit(f"s_mov_b32 {OP['wrap']}, vcc_lo")
        emit(f"s_sub_u32 s{SSOFF}, s{SSOFF}, s{STGT}")
        emit(f"s_add_u32 {OP['px']}, {OP['px']}, 1")
        emit(f"s_cmp_eq_u32 {OP['px']}, vcc_hi")
        emit(f"s_cbranch_scc1 {nextrow}")
        emit(f"s_add_u32 s{SSOFF}, s{SSOFF}, 4")
        emit(f"s_branch {wrapped}")
        emit(f"{nextrow}:")
        emit(f"s_mov_b32 {OP['px']}, 0")
        emit(f"s_add_u32 s{SSOFF}, s{SSOFF}, s{SNCH}")
        emit("s_lshl_b32 vcc_hi, vcc_hi, 2")
        emit(f"s_sub_u32 s{SSOFF}, s{SSOFF}, vcc_hi")
        emit(f"s_add_u32 s{SSOFF}, s{SSOFF}, 4")
        emit(f"{wrapped}:")
        emit(f"{nowrap}:")

    def body(A, B, N, n=CH, check=False):
        """One chunk: multiply the first n entries of A (8, or 4 for the half chunk that may open a segment);
        reads of the entries D ahead (A's tail, B's head) are issued.  check (flow): this body counts down
        vcc_lo, the chunks to go before the landing of the staged block is reported."""
        if check:
            nosig = label("nosig")
            emit("s_cmp_eq_u32 vcc_lo, 0")
            emit(f"s_cbranch_scc1 {nosig}")
            emit("s_sub_u32 vcc_lo, vcc_lo, 1")
            emit("s_cmp_lg_u32 vcc_lo, 0")
            emit(f"s_cbranch_scc1 {nosig}")
            signal(4)
            emit(f"{nosig}:")
        def entry_w1(p):
            return w1(A, p) if p < n else w1(B, p - n)
        def fetch_next():
            # B was requested one chunk ago.  The wait for it (lgkmcnt(0), which also drains the LDS reads in
            # flight) comes as late as B's first use allows, behind address computations that give those reads
            # time to land; the request for N follows it.  (At the end of the previous chunk the same wait
            # costs 1.4 % more.)
            emit("s_waitcnt lgkmcnt(0)")
            emit(f"s_load_dwordx16 s[{N}:{N + W - 1}], s[{SPTR}:{SPTR + 1}], s{SOFF}")
            emit(f"s_add_u32 s{SOFF}, s{SOFF}, {hex(4 * W)}")
        if batch:
            for j in range(n):
                if j == max(n - D, 0):
                    fetch_next()
                emit(f"v_mad_u32_u16 v{VA0 + j}, {entry_w1(j + D)}, 16, v{VLB} op_sel:[1,0,0,0]")
        emit("s_setprio 2")                       # a wave multiplying goes before one that is between chunks or staging
        for u in range(n):
            slot = u % D
            va = VA0 + (u if batch else slot)
            if not batch:
                if u == max(n - D, 0):
                    fetch_next()
                emit(f"v_mad_u32_u16 v{va}, {entry_w1(u + D)}, 16, v{VLB} op_sel:[1,0,0,0]")
            emit(f"s_set_gpr_idx_on {w1(A, u)}, gpr_idx(DST)")
            for t in range(T):
                emit(f"s_waitcnt lgkmcnt({D * T - 1})")
                for e in range(4):
                    emit(f"v_fmac_f32 v{ACC0 + t * 4 + e}, {w0(A, u)}, {q(slot, t, e)}")
                emit(f"ds_read_b128 {q(slot, t)}, v{va} offset:{t * step * 16}")
            if not batch:
                emit("s_set_gpr_idx_off")
        if batch:
            emit("s_set_gpr_idx_off")
        emit("s_setprio 0")
        emit(f"s_cmp_lg_u32 s{SOFF}, s{SCNT}")          # SCNT: the offset at which this segment's loads end

    # ------------------------------------------------------------------ set-up
    emit(f"s_mov_b64 s[{SEXEC}:{SEXEC + 1}], exec")
    for n in range(nacc):
        emit(f"v_mov_b32 v{ACC0 + n}, 0")
    emit(f"s_load_dwordx8 s[{SN}:{SN + 7}], {OP['kern']}, {hex(OFF_CONSTS)}")
    emit("s_waitcnt lgkmcnt(0)")
    emit(f"s_mov_b32 s{SCB}, s{SN}")
    emit(f"s_mov_b32 s{SLEFT}, {OP['nblk']}")      # blocks and channels of this workgroup's channel range
    emit(f"s_mov_b32 s{SREM}, {OP['nch']}")
    emit(f"s_mov_b32 s{SPLANE}, s{SN + 3}")
    emit(f"s_mov_b32 s{SSTRIDE}, s{SN + 4}")
    emit(f"s_mov_b32 s{SHW4}, s{SN + 5}")
    emit(f"s_mov_b32 s{SSOFF}, {OP['soff0']}")
    emit(f"s_mov_b64 s[{SSEG}:{SSEG + 1}], {OP['segp']}")
    emit(f"s_mov_b32 s{SBUF}, 0")
    emit(f"s_load_dwordx2 s[{SN}:{SN + 1}], s[{SSEG}:{SSEG + 1}], 0x0")          # segment of block 0
    emit(f"s_load_dwordx2 s[{SN + 2}:{SN + 3}], {OP['kern']}, {hex(OFF_PAIRS)}")
    emit(f"s_add_u32 s{SSEG}, s{SSEG}, 8")
    emit(f"s_addc_u32 s{SSEG + 1}, s{SSEG + 1}, 0")
    emit(f"s_mov_b32 s{STGT}, {OP['ldsbase']}")
    stage(STGT)
    # The segments of one wave slot follow each other in memory, block after block, so the two chunks the
    # loop has read ahead when a segment ends are the first two of the next one: only block 0 loads them here.
    emit("s_waitcnt lgkmcnt(0)")
    emit(f"s_mov_b64 s[{SPTR}:{SPTR + 1}], s[{SN + 2}:{SN + 3}]")      # base of the streams; SOFF runs over them
    emit(f"s_mov_b32 s{SOFF}, s{SN}")
    emit(f"s_mov_b32 s{SNXT}, s{SN + 1}")
    emit(f"s_load_dwordx16 s[{SA}:{SA + W - 1}], s[{SPTR}:{SPTR + 1}], s{SOFF}")
    emit(f"s_add_u32 s{SOFF}, s{SOFF}, {hex(4 * W)}")
    emit(f"s_load_dwordx16 s[{SB}:{SB + W - 1}], s[{SPTR}:{SPTR + 1}], s{SOFF}")
    emit(f"s_add_u32 s{SOFF}, s{SOFF}, {hex(4 * W)}")
    warm()
    if flow:
        if FLOW_LOOK == 2:
            one = label("oneblock")
            emit(f"s_cmp_le_u32 s{SLEFT}, 1")
            emit(f"s_cbranch_scc1 {one}")
            emit(f"s_add_u32 s{STGT}, s{SSTRIDE}, {OP['ldsbase']}")
            stage(STGT)                                    # the second block, into the second buffer
            signal(4)
            emit(f"{one}:")
        signal(0)                                          # my share of the first block (and the second) is in LDS
        emit("s_mov_b32 vcc_lo, 0")                        # no landing left to report

    # ------------------------------------------------------------------ channel blocks
    blk, nostage, segdone, noreads = label("blk"), label("nostage"), label("segdone"), label("noreads")
    emit(f"{blk}:")
    if flow:
        emit("s_waitcnt lgkmcnt(0)")
        poll()                                             # every wave's share of this block is in LDS
    else:
        emit("s_waitcnt vmcnt(0) lgkmcnt(0)")
        emit("s_barrier")
    emit(f"s_lshr_b32 s{SHALF}, s{SNXT}, 31")              # bit 31: the segment opens with a half chunk
    emit(f"s_lshl_b32 s{SCNT}, s{SNXT}, 6")                # this block's chunks -> where its loads end
    emit(f"s_add_u32 s{SCNT}, s{SCNT}, s{SOFF}")
    emit(f"s_load_dword s{SNXT}, s[{SSEG}:{SSEG + 1}], 0x4")   # chunks of the next block (one spare entry ends the table)
    emit(f"s_add_u32 s{SSEG}, s{SSEG}, 8")
    emit(f"s_addc_u32 s{SSEG + 1}, s{SSEG + 1}, 0")
    # first reads of this block's stream go out before the loads of the next block are issued
    emit(f"s_cmp_eq_u32 s{SCNT}, s{SOFF}")                 # no chunks in this block
    emit(f"s_cbranch_scc1 {noreads}")
    emit(f"s_add_u32 s{STMP}, s{SBUF}, {OP['ldsbase']}")
    emit(f"v_add_u32 v{VLB}, s{STMP}, {OP['lane_byte']}")
    for d in range(D):
        emit(f"v_mad_u32_u16 v{VA0 + d}, {w1(SA, d)}, 16, v{VLB} op_sel:[1,0,0,0]")
        for t in range(T):
            emit(f"ds_read_b128 {q(d, t)}, v{VA0 + d} offset:{t * step * 16}")
    emit(f"{noreads}:")
    emit(f"s_cmp_le_u32 s{SLEFT}, {FLOW_LOOK if flow else 1}")   # the last block(s) stage nothing
    emit(f"s_cbranch_scc1 {nostage}")
    if flow:
        # FLOW_LOOK buffers on from the current one, round the ring: block b-2's buffer, which every wave has left
        emit(f"s_mul_i32 s{SNCH}, s{SSTRIDE}, {FLOW_LOOK}")
        emit(f"s_add_u32 s{STGT}, s{SBUF}, s{SNCH}")
        emit(f"s_mul_i32 s{SNCH}, s{SSTRIDE}, {FLOW_BUFS}")
        emit(f"s_cmp_ge_u32 s{STGT}, s{SNCH}")
        emit(f"s_cselect_b32 s{SNCH}, s{SNCH}, 0")
        emit(f"s_sub_u32 s{STGT}, s{STGT}, s{SNCH}")
        emit(f"s_add_u32 s{STGT}, s{STGT}, {OP['ldsbase']}")
        stage(STGT)
        if FLOW_LOOK == 1:
            # A wave with a share of the block reports its landing that many first-of-three chunks on.  A wave without
            # one (the later waves of a workgroup, which the SIMD's oldest-first arbitration makes the slow ones) has
            # nothing to wait for and reports at once: the counter then fills when the early waves' loads have
            # landed and the late waves have merely entered this block, not when they are three chunks into it.
            mine, told = label("mine"), label("told")
            emit(f"s_cmp_lg_u32 {OP['nslab']}, 0")
            emit(f"s_cbranch_scc1 {mine}")
            signal(4)
            emit("s_mov_b32 vcc_lo, 0")
            emit(f"s_branch {told}")
            emit(f"{mine}:")
            emit(f"s_mov_b32 vcc_lo, {SIGNAL_AFTER}")
            emit(f"{told}:")
    else:
        emit(f"s_sub_u32 s{STGT}, s{SSTRIDE}, s{SBUF}")
        emit(f"s_add_u32 s{STGT}, s{STGT}, {OP['ldsbase']}")
        stage(STGT)
    warm()                                                 # youngest load of the block: the staging loads are not held up
    emit(f"{nostage}:")
    emit(f"s_cmp_eq_u32 s{SCNT}, s{SOFF}")
    emit(f"s_cbranch_scc1 {segdone}")
    loop, exit1, exit2, second, half = label("chunk"), label("exita"), label("exitb"), label("second"), label("half")
    # A segment whose length is an odd number of half chunks opens with 4 entries in a chunk of their own
    # (the other 4 are never executed): padding to whole chunks of 8 would cost twice as many idle entries.
    # Its code sits behind the loop, out of the way.
    emit(f"s_cmp_lg_u32 s{SHALF}, 0")
    emit(f"s_cbranch_scc1 {half}")
    emit(f"{loop}:")
    body(SA, SB, SN, check=flow and FLOW_LOOK == 1)
    emit(f"s_cbranch_scc0 {exit1}")
    emit(f"{second}:")
    body(SB, SN, SA)
    emit(f"s_cbranch_scc0 {exit2}")
    body(SN, SA, SB)
    emit(f"s_cbranch_scc1 {loop}")
    emit(f"s_branch {segdone}")                 # the chunks read ahead sit in A and B already
    emit(f"{exit1}:")                           # ... in B and N
    emit("s_waitcnt lgkmcnt(0)")                # N may still be on its way
    for w in range(0, W, 2):
        emit(f"s_mov_b64 s[{SA + w}:{SA + w + 1}], s[{SB + w}:{SB + w + 1}]")
    for w in range(0, W, 2):
        emit(f"s_mov_b64 s[{SB + w}:{SB + w + 1}], s[{SN + w}:{SN + w + 1}]")
    emit(f"s_branch {segdone}")
    emit(f"{exit2}:")                           # ... in N and A
    emit("s_waitcnt lgkmcnt(0)")
    for w in range(0, W, 2):
        emit(f"s_mov_b64 s[{SB + w}:{SB + w + 1}], s[{SA + w}:{SA + w + 1}]")
    for w in range(0, W, 2):
        emit(f"s_mov_b64 s[{SA + w}:{SA + w + 1}], s[{SN + w}:{SN + w + 1}]")
    emit(f"s_branch {segdone}")
    emit(f"{half}:")
    body(SA, SB, SN, 4)
    emit(f"s_cbranch_scc0 {exit1}")
    emit(f"s_branch {second}")
    emit(f"{segdone}:")
    emit("s_waitcnt lgkmcnt(0)")                # the last request lands before its registers are reused
    if flow:
        reported = label("reported")
        if FLOW_LOOK == 1:
            emit("s_cmp_eq_u32 vcc_lo, 0")      # a short segment ends before the landing was reported
            emit(f"s_cbranch_scc1 {reported}")
            signal(4)
            emit("s_mov_b32 vcc_lo, 0")
        else:
            emit(f"s_cmp_le_u32 s{SLEFT}, 2")   # loads were issued at this block's start: they have had the whole block
            emit(f"s_cbranch_scc1 {reported}")
            signal(8)
        emit(f"{reported}:")
        emit(f"s_add_u32 {OP['ctr']}, {OP['ctr']}, 4")
        emit(f"s_mul_i32 s{STMP}, s{SSTRIDE}, {FLOW_BUFS}")
        emit(f"s_add_u32 s{SBUF}, s{SBUF}, s{SSTRIDE}")
        emit(f"s_cmp_eq_u32 s{SBUF}, s{STMP}")
        emit(f"s_cselect_b32 s{SBUF}, 0, s{SBUF}")
    else:
        emit(f"s_sub_u32 s{SBUF}, s{SSTRIDE}, s{SBUF}")
    emit(f"s_sub_u32 s{SLEFT}, s{SLEFT}, 1")
    emit(f"s_cmp_lg_u32 s{SLEFT}, 0")
    emit(f"s_cbranch_scc1 {blk}")

    # ------------------------------------------------------------------ epilogue and stores
    KROW = SA                    # k of row i in s[KROW + i], R <= 16
    BASE = SB                    # 64-bit output base of row i in s[BASE + 2i : +1]; before that, the row's bias
    emit(f"s_load_dwordx2 s[{SX0}:{SX1}], {OP['kern']}, {hex(OFF_TBL)}")
    emit(f"s_load_dwordx2 s[{SPTR}:{SPTR + 1}], {OP['kern']}, {hex(OFF_CONSTS + 24)}")   # row stride, image stride of out
    for i in range(R):
        emit(f"s_load_dword s{KROW + i}, {OP['rowp']}, {hex(4 * i)}")
    emit("s_waitcnt lgkmcnt(0)")
    for t in range(T):
        emit(f"global_load_dword v{RING0 + t}, {OP['tbloff']}, s[{SX0}:{SX1}] offset:{t * 256}")
    # bias (a null pointer = none) and ReLU on the accumulators, before anything is stored
    nobias, norelu = label("nobias"), label("norelu")
    emit(f"s_cmp_eq_u64 {OP['bias']}, 0")
    emit(f"s_cbranch_scc1 {nobias}")
    for i in range(R):
        emit(f"s_max_i32 s{STMP}, s{KROW + i}, 0")          # rows that do not exist (-1) read bias[0], unused
        emit(f"s_lshl_b32 s{STMP}, s{STMP}, 2")
        emit(f"s_load_dword s{BASE + i}, {OP['bias']}, s{STMP}")
    emit("s_waitcnt lgkmcnt(0)")
    for i in range(R):
        for n in range(T * 4):
            emit(f"v_add_f32 v{ACC0 + i * T * 4 + n}, s{BASE + i}, v{ACC0 + i * T * 4 + n}")
    emit(f"{nobias}:")
    emit(f"s_bitcmp1_b32 {OP['flags']}, {FLAG_RELU}")
    emit(f"s_cbranch_scc0 {norelu}")
    for n in range(nacc):
        emit(f"v_max_f32 v{ACC0 + n}, 0, v{ACC0 + n}")
    emit(f"{norelu}:")
    for i in range(R):
        emit(f"s_mul_hi_u32 s{STMP}, s{KROW + i}, s{SPTR}")
        emit(f"s_mul_i32 s{SCNT}, s{KROW + i}, s{SPTR}")
        emit(f"s_add_u32 s{BASE + 2 * i}, {OP['outp']}, s{SCNT}")
        emit(f"s_addc_u32 s{BASE + 2 * i + 1}, {OP['outp_hi']}, s{STMP}")
    emit("s_waitcnt vmcnt(0)")

    MASKS = [28, 30, 92, 94, 96, 98]   # SGPR pairs that are free once the block loop is over

    def store_all(instr):
        if T <= len(MASKS):
            # The chunks of a lane are neighbours in the output (flat lanes: 64 positions apart; strips: the next
            # few columns of the same row), so they are stored one after the other: pieces of one cache line
            # written together leave L2 as whole lines.  Which lanes hold an output is decided once per chunk.
            for t in range(T):
                emit(f"s_mov_b64 exec, s[{SEXEC}:{SEXEC + 1}]")   # the compare writes vcc for active lanes only
                emit(f"v_cmp_gt_u32_e32 vcc, {OP['lim']}, v{RING0 + t}")
                emit(f"s_mov_b64 s[{MASKS[t]}:{MASKS[t] + 1}], vcc")
            for i in range(R):
                rowend = label("rowend")
                emit(f"s_cmp_lt_i32 s{KROW + i}, 0")
                emit(f"s_cbranch_scc1 {rowend}")
                emit(f"s_mov_b64 s[{SX0}:{SX1}], s[{BASE + 2 * i}:{BASE + 2 * i + 1}]")
                for e in range(4):
                    if e:
                        emit(f"s_cmp_le_u32 {OP['nimg']}, {e}")
                        emit(f"s_cbranch_scc1 {rowend}")
                        emit(f"s_add_u32 s{SX0}, s{SX0}, s{SPTR + 1}")
                        emit(f"s_addc_u32 s{SX1}, s{SX1}, 0")
                    for t in range(T):
                        emit(f"s_mov_b64 exec, s[{MASKS[t]}:{MASKS[t] + 1}]")
                        emit(f"{instr} v{RING0 + t}, v{ACC0 + (i * T + t) * 4 + e}, s[{SX0}:{SX1}]")
                emit(f"{rowend}:")
            return
        for t in range(T):
            emit(f"s_mov_b64 exec, s[{SEXEC}:{SEXEC + 1}]")   # the compare writes vcc for active lanes only
            emit(f"v_cmp_gt_u32_e32 vcc, {OP['lim']}, v{RING0 + t}")
            emit("s_mov_b64 exec, vcc")
            for i in range(R):
                rowend = label("rowend")
                emit(f"s_cmp_lt_i32 s{KROW + i}, 0")
                emit(f"s_cbranch_scc1 {rowend}")
                emit(f"s_mov_b64 s[{SX0}:{SX1}], s[{BASE + 2 * i}:{BASE + 2 * i + 1}]")
                for e in range(4):
                    if e:
                        emit(f"s_cmp_le_u32 {OP['nimg']}, {e}")
                        emit(f"s_cbranch_scc1 {rowend}")
                        emit(f"s_add_u32 s{SX0}, s{SX0}, s{SPTR + 1}")
                        emit(f"s_addc_u32 s{SX1}, s{SX1}, 0")
                    emit(f"{instr} v{RING0 + t}, v{ACC0 + (i * T + t) * 4 + e}, s[{SX0}:{SX1}]")
                emit(f"{rowend}:")

    if T <= len(MASKS):
        # Where the four images of a position are adjacent in the output (feature-major activations: image stride
        # 4 bytes) and all four exist, a lane stores its four sums of a row with one instruction.
        narrow, stored = label("narrow"), label("stored")
        emit(f"s_cmp_eq_u32 s{SPTR + 1}, 4")
        emit(f"s_cbranch_scc0 {narrow}")
        emit(f"s_cmp_eq_u32 {OP['nimg']}, 4")
        emit(f"s_cbranch_scc0 {narrow}")
        for t in range(T):
            emit(f"s_mov_b64 exec, s[{SEXEC}:{SEXEC + 1}]")
            emit(f"v_cmp_gt_u32_e32 vcc, {OP['lim']}, v{RING0 + t}")
            emit(f"s_mov_b64 s[{MASKS[t]}:{MASKS[t] + 1}], vcc")
        for i in range(R):
            rowend = label("rowend")
            emit(f"s_cmp_lt_i32 s{KROW + i}, 0")
            emit(f"s_cbranch_scc1 {rowend}")
            for t in range(T):
                a0 = ACC0 + (i * T + t) * 4
                emit(f"s_mov_b64 exec, s[{MASKS[t]}:{MASKS[t] + 1}]")
                emit(f"global_store_dwordx4 v{RING0 + t}, v[{a0}:{a0 + 3}], s[{BASE + 2 * i}:{BASE + 2 * i + 1}]")
            emit(f"{rowend}:")
        emit(f"s_branch {stored}")
        emit(f"{narrow}:")
        store_all("global_store_dword")
        emit(f"{stored}:")
    else:
        store_all("global_store_dword")
    emit(f"s_mov_b64 exec, s[{SEXEC}:{SEXEC + 1}]")

    vregs = {"lane_byte", "voff0", "voff1", "voff2", "voff3", "tbloff"}
    cnames = {"outp": "outp_lo"}
    ins = ", ".join(f'[{n}] "{"v" if n in vregs else "s"}"({cnames.get(n, n)})' for n in OPS)
    outs = ", ".join(f'[{n}] "+s"({n})' for n in IO_OPS)
    text = []
    for ins_ in L:
        text.append(f'            "{ins_}\\n\\t"')
    clob = [f'"v{r}"' for r in range(ACC0, MAX_VGPR)]
    clob += [f'"s{r}"' for r in list(range(28, 32)) + list(range(34, 100))]
    clob += ['"vcc"', '"scc"', '"memory"']
    return f"""
template <>
struct Lds2Asm<{T}, {R}, {step}, {"true" if flow else "false"}> {{
    static constexpr int kDepth = {D};
    static __device__ __forceinline__ void run(unsigned long long kern, int4v rsrc, const unsigned *segp, const int *rowp,
                                               unsigned outp_lo, unsigned outp_hi, unsigned soff0, unsigned nimg,
                                               unsigned lim, unsigned ldsbase, unsigned slab0, unsigned slabstep,
                                               unsigned nslab, unsigned lane_byte, unsigned voff0, unsigned voff1,
                                               unsigned voff2, unsigned voff3, unsigned tbloff, unsigned nch, unsigned nblk,
                                               unsigned long long bias, unsigned flags, unsigned nwv, unsigned ctr, unsigned wrap, unsigned px)
    {{
        asm volatile(
{chr(10).join(text)}
            : {outs}
            : {ins}
            : {", ".join(clob)});
    }}
}};
"""


def generate() -> str:
    parts = ["// GENERATED by gen_lds2.py -- do not edit; edit the generator and rebuild.\n",
             "template <int T, int R, int STEP, bool FLOW>\nstruct Lds2Asm;\n"]
    for s in SHAPES:
        parts.append(gen_shape(*s))
        parts.append(gen_shape(*s, flow=True))
    parts.append("\n#define SCONV_LDS2_SHAPES(X) " + " ".join(f"X({t}, {r}, {st})" for t, r, _, _, st in SHAPES) + "\n")
    parts.append(f"#define SCONV_LDS2_FLOW_BUFS {FLOW_BUFS}\n#define SCONV_LDS2_OFF_PHASE {OFF_PHASE}\n"
                 f"#define SCONV_LDS2_WARM_BYTES {WARM_BYTES}\n")
    parts.append(f"#define SCONV_LDS2_OFF_PAIRS {OFF_PAIRS}\n#define SCONV_LDS2_OFF_TBL {OFF_TBL}\n"
                 f"#define SCONV_LDS2_OFF_CONSTS {OFF_CONSTS}\n")
    return "".join(parts)


def main() -> int:
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "sconv_lds2_asm.inc")
    text = generate()
    if not os.path.exists(out) or open(out).read() != text:
        with open(out, "w") as fh:
            fh.write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
