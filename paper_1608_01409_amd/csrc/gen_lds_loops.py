#!/usr/bin/env python3
"""Writes sconv_lds_loops.inc: the hand-scheduled inner loops of the LDS-tiled kernel.

One `SegLoop<T, ROWS_W>::run` per accumulator shape.  Each is a single asm
statement that walks the nonzero stream of one wave inside one channel block:

  stream  = chunks of 4 (value, LDS byte offset) pairs, 32 bytes each; the
            chunks of row 0 come first, then row 1, ...; cnt[i] = chunks of row i.
  SGPRs   = three chunk buffers A (in use), B (next, valid), N (being loaded by
            s_load_dwordx8), rotated after every chunk.
  VGPRs   = a ring of D x T float4 read buffers.  Entry p of the stream reads
            T float4 (ds_read_b128, 64 lanes x 16 B each) at lane_byte + off[p]
            + t*1024; they are issued while entry p-D is being multiplied, so D
            entries are in flight.  The ring runs across row boundaries: only the
            accumulators that the v_fmac instructions name change from row to row.
  waits   = LDS reads return in order, so the oldest of the D*T outstanding ones
            is complete once lgkmcnt <= D*T-1.  A pending s_load (which may return
            out of order) only makes that wait stricter.  Once per chunk
            lgkmcnt(0) makes buffer N valid before the rotation.

The C++ side passes the accumulators as "+v" operands; ring, address and chunk
buffers are fixed registers named in the clobber list.
"""
from __future__ import annotations

import os
import sys

# (T, ROWS_W, D): T float4 chunks per lane, rows per wave, read-ahead depth in stream entries.
SHAPES = [
    (1, 8, 4), (2, 4, 4), (2, 8, 2), (3, 4, 4), (3, 6, 2), (3, 8, 1), (4, 4, 2), (4, 6, 1), (5, 4, 1),
    (6, 2, 2), (6, 3, 1), (7, 2, 2), (7, 3, 1), (13, 1, 1), (14, 1, 1),
]

SA, SB, SN = 68, 76, 84        # first SGPR of chunk buffers A, B, N (8 each)
SPTR, SCNT = 92, 94            # stream pointer pair, chunk counter
MAX_VGPR = 128


def gen_shape(T: int, ROWS_W: int, D: int) -> str:
    assert 4 % D == 0 and D * T <= 16
    nacc = ROWS_W * T * 4
    ring_regs = D * T * 4
    ring_base = (MAX_VGPR - D - ring_regs) & ~3
    addr_base = MAX_VGPR - D
    # operand numbers
    op_ptr, op_lane, op_cnt0 = nacc, nacc + 1, nacc + 2

    def q(slot, t, e=None):
        b = ring_base + (slot * T + t) * 4
        return f"v[{b}:{b + 3}]" if e is None else f"v{b + e}"

    def acc(i, t, e):
        return f"%{(i * T + t) * 4 + e}"

    def off_sgpr(p):  # offset word of stream entry p counted from the start of chunk A
        return f"s{(SA if p < 4 else SB) + 2 * (p % 4) + 1}"

    L = []
    emit = L.append
    emit(f"s_mov_b64 s[{SPTR}:{SPTR + 1}], %{op_ptr}")
    emit(f"s_load_dwordx8 s[{SA}:{SA + 7}], s[{SPTR}:{SPTR + 1}], 0x0")
    emit(f"s_load_dwordx8 s[{SB}:{SB + 7}], s[{SPTR}:{SPTR + 1}], 0x20")
    emit(f"s_add_u32 s{SPTR}, s{SPTR}, 0x40")
    emit(f"s_addc_u32 s{SPTR + 1}, s{SPTR + 1}, 0")
    emit("s_waitcnt lgkmcnt(0)")
    for d in range(D):
        emit(f"v_add_u32 v{addr_base + d}, {off_sgpr(d)}, %{op_lane}")
        for t in range(T):
            emit(f"ds_read_b128 {q(d, t)}, v{addr_base + d} offset:{t * 1024}")
    for i in range(ROWS_W):
        emit(f"s_cmp_eq_u32 %{op_cnt0 + i}, 0")
        emit(f"s_cbranch_scc1 .Lsconv_end{i}_%=")
        emit(f"s_mov_b32 s{SCNT}, %{op_cnt0 + i}")
        emit(f".Lsconv_loop{i}_%=:")
        emit(f"s_load_dwordx8 s[{SN}:{SN + 7}], s[{SPTR}:{SPTR + 1}], 0x0")
        emit(f"s_add_u32 s{SPTR}, s{SPTR}, 0x20")
        emit(f"s_addc_u32 s{SPTR + 1}, s{SPTR + 1}, 0")
        for u in range(4):
            slot = u % D
            emit(f"v_add_u32 v{addr_base + slot}, {off_sgpr(u + D)}, %{op_lane}")
            for t in range(T):
                emit(f"s_waitcnt lgkmcnt({D * T - 1})")
                for e in range(4):
                    emit(f"v_fmac_f32 {acc(i, t, e)}, s{SA + 2 * u}, {q(slot, t, e)}")
                emit(f"ds_read_b128 {q(slot, t)}, v{addr_base + slot} offset:{t * 1024}")
        emit("s_waitcnt lgkmcnt(0)")
        for w in range(8):
            emit(f"s_mov_b32 s{SA + w}, s{SB + w}")
        for w in range(8):
            emit(f"s_mov_b32 s{SB + w}, s{SN + w}")
        emit(f"s_sub_u32 s{SCNT}, s{SCNT}, 1")
        emit(f"s_cmp_lg_u32 s{SCNT}, 0")
        emit(f"s_cbranch_scc1 .Lsconv_loop{i}_%=")
        emit(f".Lsconv_end{i}_%=:")
    emit("s_waitcnt lgkmcnt(0)")

    outs = ", ".join(f'"+v"(acc[{n}])' for n in range(nacc))
    ins = '"s"(stream), "v"(lane_byte), ' + ", ".join(f'"s"(cnt[{i}])' for i in range(ROWS_W))
    clob = [f'"v{r}"' for r in range(ring_base, MAX_VGPR)]
    clob += [f'"s{r}"' for r in range(SA, SCNT + 1)]
    clob += ['"scc"', '"memory"']
    body = "\n".join(f'            "{ins_}\\n\\t"' for ins_ in L)
    return f"""
template <>
struct SegLoop<{T}, {ROWS_W}> {{
    static constexpr int kDepth = {D};
    static __device__ __forceinline__ void run(float (&acc)[{nacc}], const unsigned *stream, const int (&cnt)[{ROWS_W}],
                                               unsigned lane_byte)
    {{
        asm volatile(
{body}
            : {outs}
            : {ins}
            : {", ".join(clob)});
    }}
}};
"""


def generate() -> str:
    parts = ["// GENERATED by gen_lds_loops.py -- do not edit; edit the generator and rebuild.\n",
             "// Hand-scheduled inner loops of sconv_lds_kernel (see the generator for the scheme).\n",
             "template <int T, int ROWS_W>\nstruct SegLoop;\n"]
    for s in SHAPES:
        parts.append(gen_shape(*s))
    shapes = " ".join(f"X({t}, {r})" for t, r, _ in SHAPES)
    parts.append(f"\n#define SCONV_ASM_SHAPES(X) {shapes}\n")
    return "".join(parts)


def main() -> int:
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "sconv_lds_loops.inc")
    text = generate()
    if not os.path.exists(out) or open(out).read() != text:
        with open(out, "w") as fh:
            fh.write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
