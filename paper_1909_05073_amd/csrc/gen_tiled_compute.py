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
    v[28 + 4*r + m]                 input rows r = 0..5 of the lane's patch, columns x0..x0+3 (m = 0..3)
    v[52 + r], v[58 + r]            the halo columns x0-1 and x0+4 of row r
    v[24:27]                        the record's four weights (same value in every lane)
    v22 LDS address of the patch, v23 LDS address of the next record's weights
    s84 record index, s85 record word, s86 the word after it, s90 scratch, s91 byte offset of the
    word being loaded, s[92:93] address of body 0, s[94:95] target
Operands: %[recm] per-lane record words (lane j = record j; only lanes 0 and 1 are read), %[mp]
address of the record stream in global memory (SGPR pair) and %[koff] byte offset of record 0 in
it (SGPR; words 2.. are read from there with scalar
loads, because moving a lane of a vector register to a scalar register costs about a tenth of the
loop's rate on this chip; up to two words behind the list are read and not used), %[nb] number
of records (SGPR), %[va] per-lane LDS byte address of
the lane's patch in the staged buffer (a staged channel is nine 1 KiB blocks of one 16-byte
quad per lane: the six rows, then the twelve halo values), %[wa] LDS byte address
of this wave's weight block (SGPR; 16 bytes per record),
%[chmask] channels per chunk - 1 (immediate; 7 or 3).

Record word: bits 0-2 the channel within its chunk, bit 3 set on the first record of a channel (the
lane's 6x6 neighbourhood is then reloaded from LDS before the record runs), bits 9 and up the case
(slot * codes + code) times the body stride, i.e. the byte offset of the record's body in the
table.  Record number %[nb] is replaced by a word whose case is one past the last body: its "body"
is the end of the loop.
"""
import sys

ACC, INP, WREG = 64, 28, 24
STRIDE_LOG2 = 9


def code_masks():
    """The sub-masks ("codes") that get an inner loop of their own; bit 3 * r + s = tap (r, s).  This
    list is the one source of the code table: the packer's copy is generated from it.

    Every 4-tap mask that contains the centre tap (the shape of a PCONV pattern: 56 masks) is one
    code, so a kernel of any such pattern table is one record.  Other masks are split at pack time
    into the largest codes they contain: the three kernel rows (a dense kernel is three records),
    the 36 pairs of taps and the nine single taps make that possible for every mask."""
    taps = range(9)
    four = [m for m in range(512) if bin(m).count("1") == 4 and (m >> 4) & 1]
    rows = [0x007, 0x038, 0x1C0]
    pairs = [(1 << a) | (1 << b) for a in taps for b in taps if a < b]
    singles = [1 << a for a in taps]
    return four + rows + pairs + singles


CODE_MASKS = code_masks()

SLOTS = 4
QUAD_BYTES = 64 * 16             # one 16-byte quad of every lane
CHAN_BYTES = 9 * QUAD_BYTES      # one staged channel: 64 patches x 36 floats


def fetch(lines, uid):
    """Fetch record s84 and go to its body: weights from LDS, record word from lane s84, the patch
    reload in line when the record starts a new channel, then one computed jump."""
    lines += [
        "ds_read_b128 v[%d:%d], v23" % (WREG, WREG + 3),
        "v_add_u32 v23, 16, v23",
    ]
    if uid != "first":
        # s86 holds the word of record s84, asked for one body ago; the word after it is asked
        # for now and lands while this record's body runs
        lines += [
            "s_cmp_lt_u32 s84, %[nb]",
            "s_cselect_b32 s85, s86, %d" % ((SLOTS * len(CODE_MASKS)) << STRIDE_LOG2),
            "s_add_u32 s91, s91, 4",
            "s_load_dword s86, %[mp], s91",
        ]
    lines += [
        "s_bitcmp1_b32 s85, 3",
        "s_cbranch_scc0 GO_%s_%%=" % uid,
        "s_and_b32 s90, s85, %[chmask]",
        "s_mul_i32 s90, s90, %d" % CHAN_BYTES,
        "v_add_u32 v22, s90, %[va]",
    ]
    for k in range(9):
        b = INP + 4 * k
        lines.append("ds_read_b128 v[%d:%d], v22 offset:%d" % (b, b + 3, k * QUAD_BYTES))
    lines += [
        "GO_%s_%%=:" % uid,
        "s_and_b32 s90, s85, 0x%x" % (((1 << 20) - 1) << STRIDE_LOG2),
        "s_min_u32 s90, s90, %d" % ((SLOTS * len(CODE_MASKS)) << STRIDE_LOG2),
        "s_add_u32 s94, s92, s90",
        "s_addc_u32 s95, s93, 0",
        "s_setpc_b64 s[94:95]",
    ]


def in_reg(row, col):
    """Register of input (row, col) of the 6x6 neighbourhood; col 0 is x0-1, col 5 is x0+4."""
    if col == 0:
        return INP + 24 + row
    if col == 5:
        return INP + 30 + row
    return INP + 4 * row + col - 1


def generate():
    L = []
    L += [
        "s_getpc_b64 s[92:93]",
        "BASE_%=:",
        "s_add_u32 s92, s92, TABLE_%=-BASE_%=",
        "s_addc_u32 s93, s93, 0",
        "s_mov_b32 s84, 0",
        "v_mov_b32 v23, %[wa]",
        # the first two record words come from the lanes of a register that was loaded a chunk
        # ahead; every later word comes through the scalar cache, one body ahead of its use
        "v_readlane_b32 s85, %[recm], 0",
        "v_readlane_b32 s86, %[recm], 1",
        "s_add_u32 s91, %[koff], 4",
        # The records run at the lowest issue priority, everything around them (staging the next
        # chunk, the counters that other waves wait for) at the highest: see the end.
        "s_setprio 0",
    ]
    fetch(L, "first")
    L.append(".p2align %d" % STRIDE_LOG2)
    L.append("TABLE_%=:")
    for slot in range(SLOTS):
        for ci, mask in enumerate(CODE_MASKS):
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
            L.append("s_add_u32 s84, s84, 1")
            fetch(L, "%d_%d" % (slot, ci))
            L.append(".p2align %d" % STRIDE_LOG2)
    # the body of the end-of-list record: the loop is over (the weights fetched for it are not used)
    L.append("s_waitcnt lgkmcnt(0)")
    L.append("s_setprio 3")
    return L


def generate_takeover():
    """Adds the partial sums that a predecessor workgroup left in the output tensor to the
    accumulators: acc[slot][row][0..3] += y[so_slot + voff_row .. + 16 bytes].

    Buffer loads (an offset beyond the tensor reads nothing and returns zero), the eight rows of
    two slots at a time into the input registers, which are free after the record loop: two round
    trips to memory in all.  Operands: %[voff0]..%[voff3] per-lane byte offset of row 0..3 of the
    lane's patch in filter plane 0 (out of range for a row below the image or a lane without a
    patch), %[rsrc] buffer resource of the output tensor, %[so0]..%[so3] byte offset of each
    slot's filter plane (SGPRs)."""
    L = []
    for pair in range(2):
        for u in range(2):
            slot = 2 * pair + u
            for i in range(4):
                b = INP - 4 + 16 * u + 4 * i          # v24..v55
                L.append("buffer_load_dwordx4 v[%d:%d], %%[voff%d], %%[rsrc], %%[so%d] offen" % (b, b + 3, i, slot))
        L.append("s_waitcnt vmcnt(0)")
        for u in range(2):
            slot = 2 * pair + u
            for e in range(16):
                a = ACC + 16 * slot + e
                L.append("v_add_f32 v%d, v%d, v%d" % (a, a, INP - 4 + 16 * u + e))
    return L


def write_code_header(path):
    assert all(bin(m).count("1") <= 4 for m in CODE_MASKS)
    with open(path, "w") as f:
        f.write("// generated by gen_tiled_compute.py - do not edit\n")
        f.write("constexpr int kNumCodes = %d;\n" % len(CODE_MASKS))
        f.write("constexpr int kBodyStrideLog2 = %d;\n" % STRIDE_LOG2)
        f.write("constexpr uint16_t kCodeMask[kNumCodes] = {\n")
        for i in range(0, len(CODE_MASKS), 12):
            f.write("    " + ", ".join("0x%03X" % m for m in CODE_MASKS[i:i + 12]) + ",\n")
        f.write("};\n")


def write_inc(path, lines):
    with open(path, "w") as f:
        f.write("// generated by gen_tiled_compute.py - do not edit\n")
        for line in lines:
            f.write('"%s\\n"\n' % line)


def main():
    import os
    out = sys.argv[1]
    write_inc(out, generate())
    write_inc(os.path.join(os.path.dirname(out), "pconv_tiled_takeover.inc"), generate_takeover())
    write_code_header(os.path.join(os.path.dirname(out), "pconv_tiled_code_masks.inc"))


if __name__ == "__main__":
    main()
