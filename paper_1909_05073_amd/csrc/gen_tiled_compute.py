#!/usr/bin/env python3
"""Generates the record loop of the register-tiled PCONV kernel as gfx950 assembly text.

Why assembly: the loop executes one short straight-line body per record (16 FMAs per kept tap on
fixed accumulator registers), selected by the record's (slot, code).  Expressed as a C++ switch
the compiler emits a compare-and-branch tree per record, and taken branches are what the scalar
front end is slowest at; here every body ends with the fetch of the next record and ONE computed
jump (s_setpc_b64) into a table of fixed-stride bodies.  The weights are read from LDS into
vector registers (an FMA with a scalar-register operand issues at half the rate on this chip).

Output: a C string-literal include (one inline-asm template).  Register map (fixed; the C++ side
pins / clobbers the same registers):
    v[64 + 16*slot + 4*row + col]   accumulators of the 4x4 output patch of a slot (4 slots)
    v[28 + 6*r + m]                 6x6 input neighbourhood of the lane's patch, row r in 0..5; within a
                                    row m = 0..3 are columns x0..x0+3, m = 4 is x0-1, m = 5 is x0+4
    v[24:27]                        the record's four weights (same value in every lane)
    v22, v23                        LDS addresses
    s84 record index, s85 record word, s90 scratch, s[92:93] address of body 0, s[94:95] target
Operands: %[recm] per-lane record words (lane j = record j), %[va] %[vb] per-lane LDS byte
addresses of the lane's patch in the staged buffer (the four centre columns of a row / the two
halo columns, which sit 256 bytes apart), %[wa] LDS byte address
of this wave's weight block (SGPR; 16 bytes per record), %[cnt] number of records (SGPR, 1..32).
"""
import os
import sys

EXP = os.environ.get('PCONV_GEN_EXP', '')   # timing experiments only

ACC, INP, WREG = 64, 28, 24
STRIDE_LOG2 = 9
CODE_MASKS = [0x03A, 0x09A, 0x0B8, 0x0B2, 0x01B, 0x036, 0x0D8, 0x1B0, 0x113, 0x074, 0x191, 0x05C,
              0x007, 0x038, 0x1C0, 0x001, 0x002, 0x004, 0x008, 0x010, 0x020, 0x040, 0x080, 0x100]
SLOTS = 4
CHAN_BYTES = 6 * 64 * 6 * 4      # one staged channel: 6 rows x 64 patches x 6 floats
ROW_BYTES = 64 * 6 * 4


def fetch(lines):
    """Start fetching record s84: weights from LDS, record word from lane s84."""
    lines += [
        "s_lshl_b32 s90, s84, 4",
        "s_add_u32 s90, s90, %[wa]",
        "v_mov_b32 v23, s90",
        "ds_read_b128 v[%d:%d], v23" % (WREG, WREG + 3),
        "v_readlane_b32 s85, %[recm], s84",
        "s_nop 0",
        "s_bitcmp1_b32 s85, 11",
    ]
    if 'nopatch' not in EXP:
        lines.append("s_cbranch_scc1 PATCH_%=")
    if 'noweights' in EXP:
        lines.remove("ds_read_b128 v[%d:%d], v23" % (WREG, WREG + 3))
    jump(lines)


def jump(lines):
    if 'nojump' in EXP:
        lines += ["s_and_b32 s90, s85, 0", "s_min_u32 s90, s90, 95", "s_lshl_b32 s90, s90, 9",
                  "s_add_u32 s94, s92, s90", "s_addc_u32 s95, s93, 0", "s_branch TABLE_%="]
        return
    lines += [
        "s_and_b32 s90, s85, 0xff",
        "s_min_u32 s90, s90, %d" % (SLOTS * len(CODE_MASKS) - 1),
        "s_lshl_b32 s90, s90, %d" % STRIDE_LOG2,
        "s_add_u32 s94, s92, s90",
        "s_addc_u32 s95, s93, 0",
        "s_setpc_b64 s[94:95]",
    ]


def in_reg(row, col):
    """Register of input (row, col) of the 6x6 neighbourhood; col 0 is x0-1, col 5 is x0+4."""
    m = 4 if col == 0 else (5 if col == 5 else col - 1)
    return INP + 6 * row + m


def generate():
    L = []
    L += [
        "s_cmp_eq_u32 %[cnt], 0",
        "s_cbranch_scc1 DONE_%=",
        "s_getpc_b64 s[92:93]",
        "BASE_%=:",
        "s_add_u32 s92, s92, TABLE_%=-BASE_%=",
        "s_addc_u32 s93, s93, 0",
        "s_mov_b32 s84, 0",
    ]
    fetch(L)
    # out of line: a new channel starts, reload the lane's 6x6 neighbourhood from LDS
    L += [
        "PATCH_%=:",
        "s_bfe_u32 s90, s85, 0x30008",
        "s_mul_i32 s90, s90, %d" % CHAN_BYTES,
        "v_add_u32 v22, s90, %[va]",
        "v_add_u32 v23, s90, %[vb]",
    ]
    for r in range(6):
        b = INP + 6 * r
        L.append("ds_read_b128 v[%d:%d], v22 offset:%d" % (b, b + 3, r * ROW_BYTES))
        L.append("ds_read2st64_b32 v[%d:%d], v23 offset0:%d offset1:%d" % (b + 4, b + 5, 6 * r, 6 * r + 1))
    jump(L)
    L.append(".p2align %d" % STRIDE_LOG2)
    L.append("TABLE_%=:")
    for slot in range(SLOTS):
        for mask in CODE_MASKS:
            L.append("s_waitcnt lgkmcnt(0)")
            j = 0
            for t in range(9):
                if not (mask >> t) & 1:
                    continue
                r, c = divmod(t, 3)
                for i in range(4):
                    for k in range(4):
                        L.append("v_fmac_f32 v%d, v%d, v%d" % (ACC + 16 * slot + 4 * i + k, WREG + j,
                                                               in_reg(i + r, k + c)))
                j += 1
            L += [
                "s_add_u32 s84, s84, 1",
                "s_cmp_ge_u32 s84, %[cnt]",
                "s_cbranch_scc1 DONE_%=",
            ]
            fetch(L)
            L.append(".p2align %d" % STRIDE_LOG2)
    L.append("DONE_%=:")
    return L


def main():
    out = sys.argv[1]
    with open(out, "w") as f:
        f.write("// generated by gen_tiled_compute.py - do not edit\n")
        for line in generate():
            f.write('"%s\\n"\n' % line)


if __name__ == "__main__":
    main()
