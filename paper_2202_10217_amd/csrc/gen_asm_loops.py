#!/usr/bin/env python3
"""Writes syrk_asm_loops.inc: the main loops of the SYRK kernels as gfx950 assembly.

Why assembly: the loop keeps k(k-1)/2 * 16 MFMA accumulators (192 registers in fp64) live across
its back edge.  Compiled from C++ the register allocator moves part of them between the two
register banks on every iteration and the scheduler undoes the software pipelining; written out,
the loop is exactly the schedule documented in syrk_kernels.hip (block_body).

One function is generated per (element type, block shape, slot set).  Its C++ side passes
  acc          the accumulators, bound to accumulation registers ("+a")
  rd0/rd1      LDS byte address of the lane's row-side operand piece in buffer 0 / 1
  rb0/rb1      same for the column side (includes the wavefront's 16-row group)
  wr0/wr1      LDS byte address the thread stores its first staged piece to, buffer 0 / 1
  go[...]      byte offset of each staged 16-byte piece from the matrix base (32-bit)
  gR, gQ       base pointers of the row-side and column-side matrices (scalar registers)
  nch          number of chunks (>= 1), step = bytes per chunk
and the text below does: prologue (stage chunk 0, request chunk 1, read the first operands), then
per chunk KS k-steps of MFMAs with the next k-step's operands read from LDS in between, the next
chunk written to the other LDS buffer during k-step KS-2, one barrier, and the chunk after that
requested from global memory during k-step KS-1.  The last iteration stages the final chunk once
more into the idle buffer (nothing reads it): every iteration is the same code.

Hazards kept by construction: two MFMAs on one accumulator are separated by the MFMAs of all
other accumulators (>= 3 instructions of 16 passes (fp64) / 8 passes (fp32) each, more than the
required issue distance); operand registers are double buffered, so an LDS read never overwrites
what an MFMA in flight still reads; the block ends with 2 x 16 idle cycles before the
accumulators may be read (a 16-pass MFMA needs 18).
"""
import os

TILE = 64
PANEL_BYTES = 64 * 144          # one staged panel: 64 rows of 144 bytes (128 data + 16 pad)
HALF_BYTES = 32 * 144           # rows 32..63 of a panel
RB_BYTES = 16 * 144             # one 16-row group

SHAPES = {
    # name: (number of LDS panels, row-side panels a_i, column-side panels b_j, slots (i, j) in slot order,
    #        column-side predicate for panels)
    "Tri": dict(np=4, a=[1, 2, 3], b=[0, 1, 2],
                slots=[(0, 0), (1, 0), (1, 1), (2, 0), (2, 1), (2, 2)], col_side=lambda p: False),
    "Rect": dict(np=5, a=[3, 4], b=[0, 1, 2],
                 slots=[(0, 0), (0, 1), (0, 2), (1, 0), (1, 1), (1, 2)], col_side=lambda p: p < 3),
}
FAST_SETS = {"Tri": [0x3F, 0x07, 0x01], "Rect": [0x3F, 0x1B, 0x09, 0x07, 0x03, 0x01]}

TYPES = {
    "double": dict(kc=16, kstep_bytes=32, rd="ds_read_b64", mfma="v_mfma_f64_16x16x4_f64", opregs=2,
                   chunk_bytes=128),
    "float": dict(kc=32, kstep_bytes=16, rd="ds_read_b32", mfma="v_mfma_f32_16x16x4_f32", opregs=1,
                  chunk_bytes=128),
}

TMP_BASE = 128                   # first vector register the loop uses as scratch (declared clobbered)


def vreg(first, n):
    return f"v{first}" if n == 1 else f"v[{first}:{first + n - 1}]"


def gen(ty, shape_name, slots_mask):
    T, S = TYPES[ty], SHAPES[shape_name]
    ks_count = T["kc"] // 4
    slots = [(n, ij) for n, ij in enumerate(S["slots"]) if (slots_mask >> n) & 1]
    a_used = sorted({ij[0] for _, ij in slots})
    b_used = sorted({ij[1] for _, ij in slots})
    panels = sorted({S["a"][i] for i in a_used} | {S["b"][j] for j in b_used})
    # operand pieces of one k-step: ("a", i, rb) and ("b", j)
    pieces = [("a", i, rb) for i in a_used for rb in range(4)] + [("b", j) for j in b_used]
    n_op = len(pieces)
    opr = T["opregs"]
    set_base = [TMP_BASE, TMP_BASE + n_op * opr]
    g_base = TMP_BASE + 2 * n_op * opr
    g_base += g_base % 2                                    # 64-bit alignment for 128-bit tuples
    n_g = 2 * len(panels)
    last_tmp = g_base + 4 * n_g - 1

    def op_reg(setno, piece):
        return vreg(set_base[setno] + pieces.index(piece) * opr, opr)

    def rd_instr(setno, piece, buf, ks):
        if piece[0] == "a":
            off = S["a"][piece[1]] * PANEL_BYTES + piece[2] * RB_BYTES + ks * T["kstep_bytes"]
            addr = f"%[rd{buf}]"
        else:
            off = S["b"][piece[1]] * PANEL_BYTES + ks * T["kstep_bytes"]
            addr = f"%[rb{buf}]"
        return f"{T['rd']} {op_reg(setno, piece)}, {addr} offset:{off}"

    # MFMAs of one k-step, in slot order, 4 row groups each
    def mfmas(setno):
        out = []
        for n, (i, j) in slots:
            for rb in range(4):
                acc = f"%[c{n}_{rb}]"
                out.append(f"{T['mfma']} {acc}, {op_reg(setno, ('a', i, rb))}, {op_reg(setno, ('b', j))}, {acc}")
        return out

    g_regs = [vreg(g_base + 4 * q, 4) for q in range(n_g)]
    g_slots = [(p, h) for p in panels for h in range(2)]

    def gload(q):
        p, h = g_slots[q]
        base = "%[gQ]" if S["col_side"](p) else "%[gR]"
        return f"global_load_dwordx4 {g_regs[q]}, %[go{q}], {base}"

    def gstore(q, buf):
        p, h = g_slots[q]
        return f"ds_write_b128 %[wr{buf}], {g_regs[q]} offset:{p * PANEL_BYTES + h * HALF_BYTES}"

    def interleave(main, extras):
        """main[0], extras[0], main[1], extras[1], ...: one extra instruction after each MFMA."""
        out = []
        for n, m in enumerate(main):
            out.append(m)
            if n < len(extras):
                out.append(extras[n])
        out.extend(extras[len(main):])
        return out

    L = []
    # ---- prologue -----------------------------------------------------------------------------
    L += [gload(q) for q in range(n_g)]
    L += ["s_waitcnt vmcnt(0)"]
    L += [gstore(q, 0) for q in range(n_g)]
    L += ["s_waitcnt lgkmcnt(0)", "s_barrier"]
    # request chunk min(1, last): advance the offsets by one chunk if there is a second chunk
    L += ["s_cmp_gt_u32 %[nch], 1", "s_cselect_b32 %[tmp], %[step], 0"]
    L += [f"v_add_u32 %[go{q}], %[tmp], %[go{q}]" for q in range(n_g)]
    L += [gload(q) for q in range(n_g)]
    L += [rd_instr(0, pc, 0, 0) for pc in pieces]
    L += ["s_mov_b32 %[cnt], 0"]
    # ---- the loop: two chunks per trip would avoid the swaps; one chunk per trip keeps it short
    L += ["1:"]
    for ks in range(ks_count):
        cur_set = ks & 1
        nxt_set = cur_set ^ 1
        m = mfmas(cur_set)
        L += ["s_waitcnt lgkmcnt(0)"] if ks > 0 else ["s_waitcnt lgkmcnt(0)"]
        if ks < ks_count - 2:
            extras = [rd_instr(nxt_set, pc, 0, ks + 1) for pc in pieces]
            L += interleave(m, extras)
        elif ks == ks_count - 2:
            extras = [rd_instr(nxt_set, pc, 0, ks + 1) for pc in pieces]
            extras += ["s_waitcnt vmcnt(0)"] + [gstore(q, 1) for q in range(n_g)]
            L += interleave(m, extras)
            L += ["s_waitcnt lgkmcnt(0)", "s_barrier"]
        else:
            # last k-step: first operands of the next chunk from the other buffer, then request the
            # chunk after the next (offsets advance only while such a chunk exists)
            extras = [rd_instr(nxt_set, pc, 1, 0) for pc in pieces]
            extras += ["s_add_u32 %[tmp], %[cnt], 3", "s_cmp_le_u32 %[tmp], %[nch]",
                       "s_cselect_b32 %[tmp], %[step], 0"]
            for q in range(n_g):
                extras += [f"v_add_u32 %[go{q}], %[tmp], %[go{q}]", gload(q)]
            # the wait at the top of this k-step covered the reads of set `cur_set`; the reads
            # issued here are waited for at the top of the next trip
            L += interleave(m, extras)
    # swap buffers, count, loop
    L += ["v_swap_b32 %[rd0], %[rd1]", "v_swap_b32 %[rb0], %[rb1]", "v_swap_b32 %[wr0], %[wr1]",
          "s_add_u32 %[cnt], %[cnt], 1", "s_cmp_lt_u32 %[cnt], %[nch]", "s_cbranch_scc1 1b"]
    # ---- drain ----------------------------------------------------------------------------------
    L += ["s_waitcnt vmcnt(0) lgkmcnt(0)", "s_nop 15", "s_nop 15"]

    text = "\n".join(f'        "{line}\\n\\t"' for line in L)
    accs = ", ".join(f'[c{n}_{rb}] "+a"(acc[{n}][{rb}])' for n, _ in slots for rb in range(4))
    gos = ", ".join(f'[go{q}] "+v"(go[{q}])' for q in range(n_g))
    clob = ", ".join(f'"v{r}"' for r in range(TMP_BASE, last_tmp + 1))
    name = f"asm_loop_{ty}_{shape_name}_{slots_mask:02x}"
    fn = f"""
// {ty}, {shape_name} block, slots 0x{slots_mask:02x}: panels {panels}, {len(slots) * 4} MFMAs and {n_op} operand reads per k-step
__device__ __forceinline__ void {name}(Cfg<{ty}>::acc_t (&acc)[6][4], AsmLoopArgs& g, uint32_t (&go)[10])
{{
    uint32_t cnt, tmp;
    asm volatile(
{text}
        : {accs},
          {gos},
          [rd0] "+v"(g.rd0), [rd1] "+v"(g.rd1), [rb0] "+v"(g.rb0), [rb1] "+v"(g.rb1),
          [wr0] "+v"(g.wr0), [wr1] "+v"(g.wr1), [cnt] "=&s"(cnt), [tmp] "=&s"(tmp)
        : [gR] "s"(g.gR), [gQ] "s"(g.gQ), [nch] "s"(g.nch), [step] "s"(g.step)
        : "memory", "scc", {clob});
}}
"""
    return name, panels, fn


def main():
    out = ["// GENERATED by gen_asm_loops.py -- do not edit; see that file for the schedule.\n"]
    table = []
    for ty in TYPES:
        for shape_name in SHAPES:
            for mask in FAST_SETS[shape_name]:
                name, panels, fn = gen(ty, shape_name, mask)
                out.append(fn)
                table.append((ty, shape_name, mask, name, panels))
    # dispatcher templates
    out.append("\ntemplate <typename T, class Shape, uint32_t SLOTS> struct AsmLoop;\n")
    for ty, shape_name, mask, name, panels in table:
        out.append(f"template <> struct AsmLoop<{ty}, {shape_name}Shape, 0x{mask:02x}u> {{\n"
                   f"    static __device__ __forceinline__ void run(Cfg<{ty}>::acc_t (&acc)[6][4], AsmLoopArgs& g, "
                   f"uint32_t (&go)[10]) {{ {name}(acc, g, go); }}\n}};\n")
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "syrk_asm_loops.inc")
    with open(path, "w") as f:
        f.write("".join(out))
    return path


if __name__ == "__main__":
    print(main())
