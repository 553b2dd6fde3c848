#!/usr/bin/env python3
"""Writes syrk_asm_loops.inc: the main loops of the SYRK kernels as gfx950 assembly.

Why assembly: the loop keeps k(k-1)/2 * 16 MFMA accumulators (192 registers in fp64) live across
its back edge.  Compiled from C++ the register allocator moves part of them between the two
register banks on every iteration and the scheduler undoes the software pipelining; written out,
the loop is exactly the schedule below.

One function is generated per (element type, block shape, slot set).

Data path.  A chunk is KC columns (128 bytes) of every panel the block uses.  Chunks travel from
global memory straight into LDS (`global_load_lds_dwordx4`: lane i of a wavefront deposits its 16
bytes at M0 + 16 i), into a ring of NBUF chunk buffers, so NBUF chunks are in flight or resident and
no vector register or LDS store instruction is spent on staging.  One such instruction fills 8 rows
of 128 bytes; rows are stored unpadded and the 16-byte pieces of row r are permuted by XOR with
(r mod 8) -- the lane picks the global piece that belongs at its LDS position -- so that the 16 rows
an MFMA operand read touches fall into different banks.  A wavefront issues 2 loads per panel and
chunk (rows 8w..8w+7 and 32+8w..), the 4 wavefronts together one chunk.

Schedule per chunk (KS = KC/4 k-steps, one MFMA per accumulator and k-step):
  k-steps 0 .. KS-2: MFMAs of k-step s, with the LDS reads of the operands of k-step s+1 between them
  then: wait until this wavefront's part of the next chunk has landed, barrier (after it, every
        part has landed and nobody reads the current buffer any more: the operands of the last k-step
        are already in registers)
  k-step KS-1: its MFMAs, with between them the reads of the next chunk's first operands and the
        request of chunk (current + NBUF) into the buffer just freed
The prologue requests the first NBUF chunks, waits for chunk 0 and reads its first operands.

No vector ALU instruction between the MFMAs.  A `v_add_u32` issued while the MFMA pipeline is busy
costs about 13 cycles of MFMA time (measured: a loop that recomputed 8 LDS addresses and 8 global
offsets per chunk ran a k-step of 4 / 24 fp64 MFMAs in 322 / 1591 cycles instead of 256 / 1536; LDS
reads, waits, scalar instructions and the barrier are free).  Hence:
  - one iteration of the loop is one pass over the whole ring, so the position of a buffer is a
    constant: operand reads carry it in their offset field (16 bits; one set of address registers
    per 64 KB of the ring, set up once), the LDS target of a load is a constant added to M0;
  - the lanes' global offsets never change (they address a row inside a panel, so 32 bits suffice for
    matrices of any size); the scalar unit moves one pointer per panel one chunk on after each request
    (fixed scalar registers, declared clobbered, as is M0);
  - rarely executed code (the waits near the end, the last k-step without a request) sits after the
    loop, so the steady state takes no branch except the back edge once per pass.

Hazards kept by construction: two MFMAs on one accumulator are separated by the MFMAs of all other
accumulators (>= 3 instructions of 16 (fp64) / 8 (fp32) passes, more than the required distance);
operand registers are double buffered, so an LDS read never overwrites what an MFMA in flight still
reads; the loop ends with 2 x 16 idle cycles before the accumulators may be read (a 16-pass MFMA
needs 18).
"""
import os

PANEL_BYTES = 64 * 128          # one staged panel of one chunk: 64 rows of 128 bytes
HALF_BYTES = 32 * 128
RB_BYTES = 16 * 128             # one 16-row group
LDS_RING_BYTES = 144 * 1024     # ring of chunk buffers (the kernel's LDS allocation)
MAX_BUFS = 8

SHAPES = {
    "Tri": dict(np=4, a=[1, 2, 3], b=[0, 1, 2],
                slots=[(0, 0), (1, 0), (1, 1), (2, 0), (2, 1), (2, 2)], col_side=lambda p: False),
    "Rect": dict(np=5, a=[3, 4], b=[0, 1, 2],
                 slots=[(0, 0), (0, 1), (0, 2), (1, 0), (1, 1), (1, 2)], col_side=lambda p: p < 3),
    # a triangle block on panels 0..3 plus two tiles of the diagonal zones, each between a panel of the
    # block and one further panel (4, 5): slots 6, 7 = panel 4 x panel 0 / 1; slots 8..11 = panel 5 x
    # panel 2, panel 2 x panel 5, panel 5 x panel 3, panel 3 x panel 5 (one of each group per block)
    "Aug": dict(np=6, a=[1, 2, 3, 4, 5], b=[0, 1, 2, 3, 5],
                slots=[(0, 0), (1, 0), (1, 1), (2, 0), (2, 1), (2, 2),
                       (3, 0), (3, 1), (4, 2), (1, 4), (4, 3), (2, 4)], col_side=lambda p: False),
}
# Rect: the full 2 x 3 block and its sub-rectangles, then the three sets a two-row block can be left with
# when it straddles the diagonal (0x3B, 0x19, 0x08: the first row loses its last one or two tiles / is empty)
FAST_SETS = {"Tri": [0x3F, 0x07, 0x01], "Rect": [0x3F, 0x1B, 0x09, 0x07, 0x03, 0x01, 0x3B, 0x19, 0x08],
             "Aug": [0x3F | (1 << e1) | (1 << e2) for e1 in (6, 7) for e2 in (8, 9, 10, 11)]}

TYPES = {
    "double": dict(ks=4, rd="ds_read_b64", mfma="v_mfma_f64_16x16x4_f64", opregs=2),
    "float": dict(ks=8, rd="ds_read_b32", mfma="v_mfma_f32_16x16x4_f32", opregs=1),
}

TMP_BASE = 128                   # first vector register the loop uses as scratch (declared clobbered)
PB = 86                          # scalar registers s[86:97]: the moving pointers of up to six panels


def vreg(first, n):
    return f"v{first}" if n == 1 else f"v[{first}:{first + n - 1}]"


def spread(main, extras):
    """main instructions with the extras distributed evenly after them."""
    out = []
    if not main:
        return list(extras)
    per = -(-len(extras) // len(main))
    e = 0
    for m in main:
        out.append(m)
        out.extend(extras[e:e + per])
        e += per
    out.extend(extras[e:])
    return out


def gen(ty, shape_name, slots_mask):
    T, S = TYPES[ty], SHAPES[shape_name]
    KS = T["ks"]
    slots = [(n, ij) for n, ij in enumerate(S["slots"]) if (slots_mask >> n) & 1]
    a_used = sorted({ij[0] for _, ij in slots})
    b_used = sorted({ij[1] for _, ij in slots})
    panels = sorted({S["a"][i] for i in a_used} | {S["b"][j] for j in b_used})
    sp = {p: n for n, p in enumerate(panels)}              # LDS slot of a panel inside a chunk buffer
    npu = len(panels)
    CB = npu * PANEL_BYTES
    NBUF = min(MAX_BUFS, LDS_RING_BYTES // CB)
    RING = NBUF * CB
    NSEG = (RING + 65535) // 65536                          # 64 KB segments an offset field can span
    LPC = 2 * npu                                           # loads per wavefront and chunk
    pair = {p: f"s[{PB + 2 * n}:{PB + 2 * n + 1}]" for n, p in enumerate(panels)}   # pointer of panel p
    pieces = [("a", i, rb) for i in a_used for rb in range(4)] + [("b", j) for j in b_used]
    n_op, opr = len(pieces), T["opregs"]
    set_base = [TMP_BASE, TMP_BASE + n_op * opr]
    ad_base = TMP_BASE + 2 * n_op * opr                     # per segment: KS row-side + KS column-side addresses
    last_tmp = ad_base + NSEG * 2 * KS - 1
    assert last_tmp < 256

    def op_reg(setno, piece):
        return vreg(set_base[setno] + pieces.index(piece) * opr, opr)

    def rd_instr(setno, piece, buf, ks):
        """Read of an operand piece of k-step ks from ring buffer buf: the address register of the
        64 KB segment the byte lies in, the rest in the offset field."""
        if piece[0] == "a":
            off = buf * CB + sp[S["a"][piece[1]]] * PANEL_BYTES + piece[2] * RB_BYTES
            reg = ad_base + (off >> 16) * 2 * KS + ks
        else:
            off = buf * CB + sp[S["b"][piece[1]]] * PANEL_BYTES
            reg = ad_base + (off >> 16) * 2 * KS + KS + ks
        return f"{T['rd']} {op_reg(setno, piece)}, v{reg} offset:{off & 0xFFFF}"

    def reads(setno, buf, ks):
        return [rd_instr(setno, pc, buf, ks) for pc in pieces]

    def mfmas(setno):
        out = []
        for n, (i, j) in slots:
            for rb in range(4):
                acc = f"%[c{n}_{rb}]"
                out.append(f"{T['mfma']} {acc}, {op_reg(setno, ('a', i, rb))}, {op_reg(setno, ('b', j))}, {acc}")
        return out

    def issue(buf):
        """Request the next chunk into ring buffer buf and move the panel pointers one chunk on."""
        out = []
        for q in range(LPC):
            p, h = panels[q // 2], q % 2
            out += [f"s_add_u32 m0, %[m0b], {buf * CB + sp[p] * PANEL_BYTES + h * HALF_BYTES}", "s_nop 0",
                    f"global_load_lds_dwordx4 %[go{q}], {pair[p]}"]
        for n in range(npu):
            out += [f"s_add_u32 s{PB + 2 * n}, s{PB + 2 * n}, %[step]", f"s_addc_u32 s{PB + 2 * n + 1}, s{PB + 2 * n + 1}, 0"]
        return out

    L = []
    # ---- prologue: request the first min(NBUF, nch) chunks, wait for chunk 0 --------------------
    L += [f"s_mov_b64 {pair[p]}, %[gp{n}]" for n, p in enumerate(panels)] + ["s_mov_b32 %[cnt], 0"]
    for n in range(NBUF):
        # (a scalar register written by the scalar unit may be read by a memory instruction 5 wait
        # states later at the earliest: the moved pointers, also after the s_mov_b64 above)
        L += [f"s_cmp_lt_u32 %[cnt], %[nch]", "s_cbranch_scc0 10f", "s_nop 4"] + issue(n) + ["s_add_u32 %[cnt], %[cnt], 1"]
    L += ["10:", "s_mov_b32 %[cnt], 0"]
    # all NBUF requested: chunk 0 has landed when at most (NBUF-1)*LPC loads are outstanding;
    # fewer chunks than buffers: wait for everything
    L += [f"s_cmp_ge_u32 %[nch], {NBUF}", "s_cbranch_scc1 11f", "s_waitcnt vmcnt(0)", "11:",
          f"s_waitcnt vmcnt({(NBUF - 1) * LPC})", "s_barrier"]
    for seg in range(1, NSEG):                              # address registers of the upper segments
        for j in range(KS):
            L += [f"v_add_u32 v{ad_base + seg * 2 * KS + j}, {seg * 65536}, %[ada{j}]",
                  f"v_add_u32 v{ad_base + seg * 2 * KS + KS + j}, {seg * 65536}, %[adb{j}]"]
    for j in range(KS):
        L += [f"v_mov_b32 v{ad_base + j}, %[ada{j}]", f"v_mov_b32 v{ad_base + KS + j}, %[adb{j}]"]
    L += reads(0, 0, 0)
    # ---- the loop: one pass over the ring per iteration ------------------------------------------
    L += ["1:"]
    tails = []                                              # rarely executed pieces, placed after the loop
    for buf in range(NBUF):
        nxt = (buf + 1) % NBUF
        for ks in range(KS - 1):
            L += ["s_waitcnt lgkmcnt(0)"]
            L += spread(mfmas(ks & 1), reads((ks + 1) & 1, buf, ks + 1))
        # The next chunk has landed (this wavefront's part) when, of the NBUF - 1 chunks requested
        # after it, all but the oldest... are still outstanding; near the end fewer are: wait for all.
        L += [f"s_add_u32 %[tmp], %[cnt], {NBUF}", "s_cmp_le_u32 %[tmp], %[nch]", f"s_cbranch_scc0 {20 + buf}f",
              f"s_waitcnt vmcnt({(NBUF - 2) * LPC}) lgkmcnt(0)", f"{40 + buf}:", "s_barrier"]
        tails += [f"{20 + buf}:", "s_waitcnt vmcnt(0) lgkmcnt(0)", f"s_branch {40 + buf}b"]
        last = mfmas((KS - 1) & 1)
        first_reads = reads(0, nxt, 0)
        # chunk cnt + NBUF goes into the buffer just freed, if it exists
        L += ["s_cmp_lt_u32 %[tmp], %[nch]", f"s_cbranch_scc0 {60 + buf}f"]
        L += spread(last, first_reads + issue(buf))
        L += [f"{80 + buf}:", "s_add_u32 %[cnt], %[cnt], 1", "s_cmp_lt_u32 %[cnt], %[nch]", "s_cbranch_scc0 4f"]
        tails += [f"{60 + buf}:"] + spread(last, first_reads) + [f"s_branch {80 + buf}b"]
    L += ["s_branch 1b"]
    L += tails
    # ---- drain ----------------------------------------------------------------------------------
    L += ["4:", "s_waitcnt vmcnt(0) lgkmcnt(0)", "s_nop 15", "s_nop 15"]

    text = "\n".join(f'        "{line}\\n\\t"' for line in L)
    accs = ", ".join(f'[c{n}_{rb}] "+a"(acc[{n}][{rb}])' for n, _ in slots for rb in range(4))
    gos = ", ".join(f'[go{q}] "v"(go[{q}])' for q in range(LPC))
    ads = ", ".join(f'[ada{j}] "v"(g.ada[{j}]), [adb{j}] "v"(g.adb[{j}])' for j in range(KS))
    gps = ", ".join(f'[gp{n}] "s"(g.gP[{n}])' for n in range(npu))
    clob = ", ".join([f'"v{r}"' for r in range(TMP_BASE, last_tmp + 1)] + [f'"s{r}"' for r in range(PB, PB + 2 * npu)])
    name = f"asm_loop_{ty}_{shape_name}_{slots_mask:02x}"
    fn = f"""
// {ty}, {shape_name} block, slots 0x{slots_mask:02x}: panels {panels}, ring of {NBUF} chunk buffers of {CB} bytes,
// {len(slots) * 4} MFMAs and {n_op} operand reads per k-step, {LPC} loads per wavefront and chunk
__device__ __forceinline__ void {name}(Cfg<{ty}>::acc_t (&acc)[{len(S["slots"])}][4], const AsmLoopArgs& g, const uint32_t (&go)[{2 * S["np"]}])
{{
    uint32_t cnt, tmp;
    asm volatile(
{text}
        : {accs},
          [cnt] "=&s"(cnt), [tmp] "=&s"(tmp)
        : {gos},
          {ads},
          {gps},
          [nch] "s"(g.nch), [step] "s"(g.step), [m0b] "s"(g.m0base)
        : "memory", "scc", "m0", {clob});
}}
"""
    return name, fn


def main():
    out = ["// GENERATED by gen_asm_loops.py -- do not edit; see that file for the schedule.\n"]
    table = []
    for ty in TYPES:
        for shape_name in SHAPES:
            for mask in FAST_SETS[shape_name]:
                name, fn = gen(ty, shape_name, mask)
                out.append(fn)
                table.append((ty, shape_name, mask, name))
    out.append("\ntemplate <typename T, class Shape, uint32_t SLOTS> struct AsmLoop;\n")
    for ty, shape_name, mask, name in table:
        out.append(f"template <> struct AsmLoop<{ty}, {shape_name}Shape, 0x{mask:02x}u> {{\n"
                   f"    static __device__ __forceinline__ void run(Cfg<{ty}>::acc_t (&acc)[{len(SHAPES[shape_name]['slots'])}][4], "
                   f"const AsmLoopArgs& g, const uint32_t (&go)[{2 * SHAPES[shape_name]['np']}]) {{ {name}(acc, g, go); }}\n}};\n")
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "syrk_asm_loops.inc")
    text = "".join(out)
    if not (os.path.exists(path) and open(path).read() == text):   # untouched when nothing changed
        with open(path, "w") as f:
            f.write(text)
    return path


if __name__ == "__main__":
    print(main())
