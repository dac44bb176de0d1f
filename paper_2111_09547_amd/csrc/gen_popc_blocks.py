#!/usr/bin/env python3
"""Writes popc_blocks.inc: the AND + popcount inner blocks of the aggregation
kernel as inline-assembly device functions, one per plane count S = 1..8.

One call handles one 32-bit word column of a 16-row adjacency tile.  The word
of row j sits in lane j of every 16-lane DPP row of `a`; `row_newbcast:j`
broadcasts it to the 16 lanes of the row inside the v_and itself, so a
(row, plane) pair costs exactly one v_and_b32_dpp and one v_bcnt_u32_b32 (which
adds the popcount to its accumulator operand).  Rows are grouped into asm
statements as large as the 30-operand limit allows.  For the kernels that jump
over zero words the same pairs also come one row per function (popc_row), and
for two rows per accumulator register a form that adds the count of rows 8..15
to the upper 16 bits (popc_row_hi: v_bcnt with a zero addend, then
v_lshl_add_u32 by 16).

Run from this directory:  python3 gen_popc_blocks.py > popc_blocks.inc
"""

ROWS = 16
# rows per asm statement for each S (operands: R*S accumulators + S planes + a + 2 temps <= 30)
ROWS_PER_BLOCK = {1: 16, 2: 8, 3: 4, 4: 4, 5: 4, 6: 2, 7: 2, 8: 2}


def block(S, r0, R, first):
    items = [(r, i) for r in range(r0, r0 + R) for i in range(S)]
    lines = []
    if first:
        # two wait states between a VALU write of `a` and its first DPP read
        lines.append("s_nop 1")
    for k in range(0, len(items), 2):
        pair = items[k:k + 2]
        for n, (r, i) in enumerate(pair):
            lines.append(f"v_and_b32_dpp %[t{n}], %[a], %[x{i}] row_newbcast:{r} "
                         "row_mask:0xf bank_mask:0xf bound_ctrl:1")
        for n, (r, i) in enumerate(pair):
            lines.append(f"v_bcnt_u32_b32 %[c{r}_{i}], %[t{n}], %[c{r}_{i}]")
    text = "\n".join(f'      "{l}\\n\\t"' for l in lines)
    outs = ['[t0] "=&v"(t0)', '[t1] "=&v"(t1)'] + \
           [f'[c{r}_{i}] "+v"(acc[{r}][{i}])' for r, i in items]
    ins = ['[a] "v"(a)'] + [f'[x{i}] "v"(x[{i}])' for i in range(S)]
    return ("  asm volatile(\n" + text + "\n      : " + ", ".join(outs) +
            "\n      : " + ", ".join(ins) + ");\n")


def row_block(S, r):
    """One row of a tile by itself (all S planes): the unit the zero-word test skips."""
    items = [(r, i) for i in range(S)]
    lines = []
    for k in range(0, len(items), 2):
        pair = items[k:k + 2]
        for n, (_, i) in enumerate(pair):
            lines.append(f"v_and_b32_dpp %[t{n}], %[a], %[x{i}] row_newbcast:{r} "
                         "row_mask:0xf bank_mask:0xf bound_ctrl:1")
        for n, (_, i) in enumerate(pair):
            lines.append(f"v_bcnt_u32_b32 %[c{i}], %[t{n}], %[c{i}]")
    text = "\n".join(f'      "{l}\\n\\t"' for l in lines)
    outs = ['[t0] "=&v"(t0)', '[t1] "=&v"(t1)'] + [f'[c{i}] "+v"(acc[{i}])' for i in range(S)]
    ins = ['[a] "v"(a)'] + [f'[x{i}] "v"(x[{i}])' for i in range(S)]
    return ("    asm volatile(\n" + text + "\n      : " + ", ".join(outs) +
            "\n      : " + ", ".join(ins) + ");\n")


def row_block_hi(S, r):
    """Row r (8..15) of a tile into the upper 16 bits of the accumulators of row r - 8
    (two rows share a register where counts stay below 65536): popcount into a temporary,
    then one shift-and-add."""
    lines = []
    for k in range(0, S, 2):
        pair = list(range(k, min(S, k + 2)))
        for n, i in enumerate(pair):
            lines.append(f"v_and_b32_dpp %[t{n}], %[a], %[x{i}] row_newbcast:{r} "
                         "row_mask:0xf bank_mask:0xf bound_ctrl:1")
        for n, i in enumerate(pair):
            lines.append(f"v_bcnt_u32_b32 %[t{n}], %[t{n}], 0")
        for n, i in enumerate(pair):
            lines.append(f"v_lshl_add_u32 %[c{i}], %[t{n}], 16, %[c{i}]")
    text = "\n".join(f'      "{l}\\n\\t"' for l in lines)
    outs = ['[t0] "=&v"(t0)', '[t1] "=&v"(t1)'] + [f'[c{i}] "+v"(acc[{i}])' for i in range(S)]
    ins = ['[a] "v"(a)'] + [f'[x{i}] "v"(x[{i}])' for i in range(S)]
    return ("    asm volatile(\n" + text + "\n      : " + ", ".join(outs) +
            "\n      : " + ", ".join(ins) + ");\n")


def lane_pack(S, wpp):
    """Gathers the ballot words of one output row into lanes: plane i's word k
    goes to lane L0 + k of ow[i].  v_writelane_b32 reads its data operand on the
    scalar path; right after the compare that produced it the old SGPR content
    would still be seen, so every statement starts with four wait states."""
    out = []
    out.append(f"template <> struct lane_pack<{S}, {wpp}> {{")
    out.append("  template <int L0>")
    out.append(f"  static __device__ __forceinline__ void run(const uint32_t (&w)[{S}][4], "
               f"uint32_t (&ow)[{S}]) {{")
    group = 4 if wpp == 4 else 8
    for g0 in range(0, S, group):
        planes = list(range(g0, min(S, g0 + group)))
        lines = ["s_nop 3"]
        for i in planes:
            for k in range(wpp):
                lines.append(f"v_writelane_b32 %[o{i}], %[w{i}_{k}], %[l{k}]")
        text = "\n".join(f'      "{l}\\n\\t"' for l in lines)
        outs = [f'[o{i}] "+v"(ow[{i}])' for i in planes]
        ins = [f'[w{i}_{k}] "s"(w[{i}][{k}])' for i in planes for k in range(wpp)] + \
              [f'[l{k}] "n"(L0 + {k})' for k in range(wpp)]
        out.append("    asm volatile(\n" + text + "\n      : " + ", ".join(outs) +
                   "\n      : " + ", ".join(ins) + "\n      : \"vcc\");")
    out.append("  }\n};")
    return "\n".join(out)


def lane_pack_m0(S):
    """Same gather with a run-time lane (in M0): the two ballot halves of plane i
    go to lane `lane` of olo[i] / ohi[i]."""
    out = [f"template <> struct lane_pack_m0<{S}> {{",
           f"  static __device__ __forceinline__ void run(const uint32_t (&lo)[{S}], "
           f"const uint32_t (&hi)[{S}], uint32_t (&olo)[{S}], uint32_t (&ohi)[{S}], int lane) {{"]
    for g0 in range(0, S, 4):
        planes = list(range(g0, min(S, g0 + 4)))
        lines = ["s_mov_b32 m0, %[lane]", "s_nop 3"]
        for i in planes:
            lines.append(f"v_writelane_b32 %[ol{i}], %[l{i}], m0")
            lines.append(f"v_writelane_b32 %[oh{i}], %[h{i}], m0")
        text = "\n".join(f'      "{l}\\n\\t"' for l in lines)
        outs = [f'[ol{i}] "+v"(olo[{i}])' for i in planes] + [f'[oh{i}] "+v"(ohi[{i}])' for i in planes]
        ins = [f'[l{i}] "s"(lo[{i}])' for i in planes] + [f'[h{i}] "s"(hi[{i}])' for i in planes] + \
              ['[lane] "s"(lane)']
        out.append("    asm volatile(\n" + text + "\n      : " + ", ".join(outs) +
                   "\n      : " + ", ".join(ins) + "\n      : \"vcc\", \"m0\");")
    out.append("  }\n};")
    return "\n".join(out)


def main():
    print("// Generated by gen_popc_blocks.py - do not edit by hand.")
    print("// popc_rows<S>::run(a, x, acc): acc[j][i] += popcount(A_word(row j) & x[i])")
    print("// for the 16 rows of a tile and S feature planes; all 64 lanes must be active.")
    print("template <int S> struct popc_rows;")
    for S in range(1, 9):
        R = ROWS_PER_BLOCK[S]
        print(f"template <> struct popc_rows<{S}> {{")
        print("  static __device__ __forceinline__ void run(uint32_t a, "
              f"const uint32_t (&x)[{S}], uint32_t (&acc)[16][{S}]) {{")
        print("  uint32_t t0, t1;")
        for r0 in range(0, ROWS, R):
            print(block(S, r0, R, r0 == 0), end="")
        print("  }\n};")
    print("// popc_row<S, R>::run(a, x, acc): the same for row R alone, acc[i] += popcount(A_word(row R) & x[i]).")
    print("template <int S, int R> struct popc_row;")
    for S in range(1, 9):
        for r in range(ROWS):
            print(f"template <> struct popc_row<{S}, {r}> {{")
            print("  static __device__ __forceinline__ void run(uint32_t a, "
                  f"const uint32_t (&x)[{S}], uint32_t (&acc)[{S}]) {{")
            print("    uint32_t t0, t1;")
            print(row_block(S, r), end="")
            print("  }\n};")
    print("// popc_row_hi<S, R>::run(a, x, acc): row R (8..15) into the upper halves: acc[i] += popcount(A_word(row R) & x[i]) << 16.")
    print("template <int S, int R> struct popc_row_hi;")
    for S in range(5, 9):
        for r in range(8, ROWS):
            print(f"template <> struct popc_row_hi<{S}, {r}> {{")
            print("  static __device__ __forceinline__ void run(uint32_t a, "
                  f"const uint32_t (&x)[{S}], uint32_t (&acc)[{S}]) {{")
            print("    uint32_t t0, t1;")
            print(row_block_hi(S, r), end="")
            print("  }\n};")
    print("// lane_pack<S, WPP>::run<L0>(w, ow): ow[i] lane L0+k = w[i][k] for k < WPP.")
    print("template <int S, int WPP> struct lane_pack;")
    for S in range(1, 9):
        for wpp in (2, 4):
            print(lane_pack(S, wpp))
    print("// lane_pack_m0<S>::run(lo, hi, olo, ohi, lane): olo[i] lane `lane` = lo[i], same for hi.")
    print("template <int S> struct lane_pack_m0;")
    for S in range(1, 9):
        print(lane_pack_m0(S))


if __name__ == "__main__":
    main()
