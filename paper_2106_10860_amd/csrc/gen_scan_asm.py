#!/usr/bin/env python3
"""Writes scan_asm.inc: the instruction text of the per-row table scan of
rows_kernel for C = 16 and C = 32 codebooks.

Why hand-scheduled text: with the tables laid out as [code][codebook][256 B] in
LDS, the address of the 256-byte table row (c, code) is code * (256 C) + 256 c.
`ds_read_addtid_b32` adds M0, a 16-bit immediate and 4 * lane, so the lookup
needs no vector address arithmetic at all: two scalar instructions move
code * (256 C) from the packed code word into M0, the immediate carries 256 c.
That takes one VALU instruction out of four per lookup word.  The compiler has
no intrinsic for this instruction, hence the text.

Schedule: 8 lookups per batch; while batch b is being issued (scalar pair, LDS
read), the words of batch b-1 are consumed (wait, 2 byte extractions, and for
every second word two v_add3 into the even/odd accumulators).  Between a write
of M0 and the LDS instruction that reads it there is always at least one other
instruction (the hazard needs one wait state).  LDS data returns in order, so
while issuing, `s_waitcnt lgkmcnt(7)` is exactly "the word consumed next has
arrived"; the block starts with lgkmcnt(0) so that nothing older is counted and
ends with everything it issued consumed.

Run:  python gen_scan_asm.py   (rewrites scan_asm.inc next to this file)
"""
import os


def block(C: int) -> str:
    kshift = {32: 13, 16: 12}[C]          # log2 of 256 * C: byte stride between codes
    kmask = 0xF << kshift
    lines = []
    emit = lines.append
    emit("s_waitcnt lgkmcnt(0)")

    def stage_a(c):
        q, i = divmod(c, 8)
        sh = kshift - 4 * i
        if sh >= 0:
            emit(f"s_lshl_b32 %[st], %[c{q}], {sh}")
        else:
            emit(f"s_lshr_b32 %[st], %[c{q}], {-sh}")
        emit(f"s_and_b32 m0, %[st], 0x{kmask:x}")

    def stage_b(c):
        emit(f"ds_read_addtid_b32 %[x{c % 8}] offset:{256 * c}")

    def stage_c(j, wait):
        emit(f"s_waitcnt lgkmcnt({wait})")
        if j % 2 == 0:
            emit(f"v_and_b32 %[te], %[mask], %[x{j}]")
            emit(f"v_perm_b32 %[to], %[x{j}], %[x{j}], %[sel]")
        else:
            emit(f"v_and_b32 %[e], %[mask], %[x{j}]")
            emit(f"v_perm_b32 %[o], %[x{j}], %[x{j}], %[sel]")
            emit("v_add3_u32 %[ae], %[te], %[e], %[ae]")
            emit("v_add3_u32 %[ao], %[to], %[o], %[ao]")

    n_batches = C // 8
    for b in range(n_batches):
        for j in range(8):
            c = 8 * b + j
            stage_a(c)
            if b == 0:
                emit("s_nop 0")
            else:
                stage_c(j, 7)
            stage_b(c)
    for j in range(8):
        stage_c(j, 7 - j)
    return "\n".join('    "%s\\n"' % l for l in lines)


def block_averaged(C: int) -> str:
    """The same lookups, reduced by pairwise averages in blocks of 16 codebooks
    (Appendix D of the paper): v_lerp_u8 with a rounding bit in every byte is
    floor((a + b + 1) / 2) on four bytes at once.  Words are combined as they
    arrive: after an odd word a level-1 average, after every 4th a level-2
    average, ... after the 16th the block average, whose four bytes are split
    into the even/odd 16-bit accumulators."""
    kshift = {32: 13, 16: 12}[C]
    kmask = 0xF << kshift
    lines = []
    emit = lines.append
    emit("s_waitcnt lgkmcnt(0)")

    def stage_a(c):
        q, i = divmod(c, 8)
        sh = kshift - 4 * i
        emit(f"s_lshl_b32 %[st], %[c{q}], {sh}" if sh >= 0 else f"s_lshr_b32 %[st], %[c{q}], {-sh}")
        emit(f"s_and_b32 m0, %[st], 0x{kmask:x}")

    def stage_b(c):
        emit(f"ds_read_addtid_b32 %[x{c % 8}] offset:{256 * c}")

    def stage_c(g, wait):
        """consume the pair of words (g - 1, g), g odd (index over all codebooks)"""
        j = g % 16
        emit(f"s_waitcnt lgkmcnt({wait})")
        a, b = (g - 1) % 8, g % 8
        if j % 4 == 1:
            emit(f"v_lerp_u8 %[l1], %[x{a}], %[x{b}], %[ones]")
            return
        emit(f"v_lerp_u8 %[te], %[x{a}], %[x{b}], %[ones]")
        if j % 8 == 3:
            emit("v_lerp_u8 %[l2], %[l1], %[te], %[ones]")
            return
        emit("v_lerp_u8 %[to], %[l1], %[te], %[ones]")
        if j == 7:
            emit("v_lerp_u8 %[l3], %[l2], %[to], %[ones]")
            return
        emit("v_lerp_u8 %[e], %[l2], %[to], %[ones]")
        emit("v_lerp_u8 %[o], %[l3], %[e], %[ones]")        # block average
        emit("v_and_b32 %[te], %[mask], %[o]")
        emit("v_perm_b32 %[to], %[o], %[o], %[sel]")
        emit("v_add_u32 %[ae], %[ae], %[te]")
        emit("v_add_u32 %[ao], %[ao], %[to]")

    # Words are consumed in pairs, and a pair of the previous batch is consumed
    # BEFORE the first load of the current batch that reuses one of its registers
    # is issued: A(j) C(pair j, j+1 of the previous batch) B(j) A(j+1) nop B(j+1).
    # When that pair is consumed, 6 younger loads are outstanding.
    n_batches = C // 8
    for b in range(n_batches):
        for j in range(0, 8, 2):
            c = 8 * b + j
            stage_a(c)
            if b == 0:
                emit("s_nop 0")
            else:
                stage_c(8 * (b - 1) + j + 1, 6)
            stage_b(c)
            stage_a(c + 1)
            emit("s_nop 0")
            stage_b(c + 1)
    for j in range(0, 8, 2):
        stage_c(8 * (n_batches - 1) + j + 1, 6 - j)
    return "\n".join('    "%s\\n"' % l for l in lines)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    out = ["// Generated by gen_scan_asm.py - do not edit.  See that file for the schedule.",
           "// Operands: [ae] [ao] accumulators (in/out VGPR); [x0]..[x7] [te] [to] [e] [o] VGPR scratch;",
           "// [st] SGPR scratch; [c0].. packed code words (SGPR); [mask] = 0x00ff00ff, [sel] = 0x0c030c01 (SGPR).",
           "// The _AVG_ variants also use [l1] [l2] [l3] (VGPR scratch) and [ones] = 0x01010101 (SGPR).",
           "// Clobbers M0 and SCC."]
    for name, fn in (("MADDNESS_SCAN_ASM", block), ("MADDNESS_SCAN_AVG_ASM", block_averaged)):
        for C in (16, 32):
            out.append(f"#define {name}_C{C} \\")
            body = fn(C).split("\n")
            out.extend(l + " \\" for l in body[:-1])
            out.append(body[-1])
            out.append("")
    with open(os.path.join(here, "scan_asm.inc"), "w") as f:
        f.write("\n".join(out))


if __name__ == "__main__":
    main()
