#!/usr/bin/env python3
"""Writes rtopk_search_loops.inc: the hand-scheduled binary-search loops (inline gfx950 assembly) for
rows held as 2, 4 or 8 values per lane.

Why generated: the loops differ only in how many compare / popcount lines they repeat, and inline
assembly text cannot be produced by C++ templates.  Run by paper_2409_00822_amd/build.py; the output
is committed so that a plain `hipcc` build needs no Python.

Each loop is Algorithm 1 (epsilon = 0) or Algorithm 2 of the RTop-K paper (Section 3.1) for one row:
    thres = (lo + hi) * 0.5f;  cnt = #{x >= thres};  cnt < k ? hi = thres : lo = thres
A step costs E compares that write 64-lane masks to scalar registers, E scalar popcounts, and one
v_mov under a scalar branch for the bound (the bounds are wave-uniform values in vector registers:
gfx950 has no scalar float add).  The masks of the last threshold are returned for the selection.
"""
import os
import sys

ELEMS = (2, 4, 8)


def count_lines(E, t, neg):
    """asm lines: masks m0..m{E-1} = (key_e >= t), c0 = total popcount (c1.. are temporaries).
    key = x, or -x (a free source modifier) for the smallest-k variant."""
    sign = "-" if neg else ""
    out = [f'"v_cmp_ge_f32 %[m{e}], {sign}%[x{e}], %[{t}]\\n\\t"' for e in range(E)]
    if E == 4:  # balanced tree: shorter dependent chain
        out += [f'"s_bcnt1_i32_b64 %[c{e}], %[m{e}]\\n\\t"' for e in range(4)]
        out += ['"s_add_i32 %[c0], %[c0], %[c1]\\n\\t"', '"s_add_i32 %[c2], %[c2], %[c3]\\n\\t"',
                '"s_add_i32 %[c0], %[c0], %[c2]\\n\\t"']
    else:       # two running sums
        out += ['"s_bcnt1_i32_b64 %[c0], %[m0]\\n\\t"', '"s_bcnt1_i32_b64 %[c1], %[m1]\\n\\t"']
        for e in range(2, E):
            tmp = "c2" if e % 2 == 0 else "c3"
            acc = "c0" if e % 2 == 0 else "c1"
            out += [f'"s_bcnt1_i32_b64 %[{tmp}], %[m{e}]\\n\\t"', f'"s_add_i32 %[{acc}], %[{acc}], %[{tmp}]\\n\\t"']
        out += ['"s_add_i32 %[c0], %[c0], %[c1]\\n\\t"']
    return out


def operands(E, extra_out, extra_in):
    outs = ['[lo] "+v"(lo)', '[hi] "+v"(hi)'] + extra_out
    outs += [f'[m{e}] "=&s"(m[{e}])' for e in range(E)]
    outs += [f'[c{i}] "=&s"(c{i})' for i in range(4)]
    ins = [f'[x{e}] "v"(x[{e}])' for e in range(E)] + ['[k] "s"(k)'] + extra_in
    return outs, ins


def emit(lines, outs, ins, indent="      "):
    body = "\n".join(indent + l for l in lines)
    return (f"  asm volatile(\n{body}\n{indent}: " + ", ".join(outs) + f"\n{indent}: " + ", ".join(ins) +
            f'\n{indent}: "vcc", "scc");\n')


# Exact mode on rows stored in 16 bits: each midpoint is truncated to the row type's precision (its low
# 16 fp32 bits cleared for bfloat16, its low 13 for half).  Every element value has those bits clear,
# so once lo and hi are neighbours on that coarser grid all elements in [lo, hi) are one value, the
# midpoint repeats and the search ends -- after ~10-14 steps instead of the ~26 it takes to reach fp32
# resolution, on the many rows whose k-th and (k+1)-th values tie after rounding to 16 bits.
TRUNC = {0: None, 1: "0xffffe000", 2: "0xffff0000"}  # keyed by rtopk::DType


def gen_exact(E, neg, dt=0):
    tr = TRUNC[dt]
    L = []
    L += ['// ---- copy B (entry): midpoint in u, no convergence test', '".Lrtopk_b_%=:\\n\\t"',
          '"v_add_f32 %[u], %[lo], %[hi]\\n\\t"', '"v_mul_f32 %[u], 0.5, %[u]\\n\\t"']
    if tr:
        L += [f'"v_and_b32 %[u], {tr}, %[u]\\n\\t"']
    L += count_lines(E, "u", neg)
    L += ['"s_cmp_lt_i32 %[c0], %[k]\\n\\t"', '"s_cbranch_scc1 .Lrtopk_bless_%=\\n\\t"',
          '"s_cmp_gt_i32 %[c0], %[k]\\n\\t"', '"v_mov_b32 %[lo], %[u]\\n\\t"',
          '"s_cbranch_scc1 .Lrtopk_a_%=\\n\\t"', '"s_branch .Lrtopk_hit_%=\\n\\t"',
          '".Lrtopk_bless_%=:\\n\\t"', '"v_mov_b32 %[hi], %[u]\\n\\t"']
    L += ['// ---- copy A: midpoint in t, compared with copy B\'s (equal or unordered: converged)',
          '".Lrtopk_a_%=:\\n\\t"', '"v_add_f32 %[t], %[lo], %[hi]\\n\\t"', '"v_mul_f32 %[t], 0.5, %[t]\\n\\t"']
    if tr:
        L += [f'"v_and_b32 %[t], {tr}, %[t]\\n\\t"']
    L += ['"v_cmp_lg_f32 vcc, %[t], %[u]\\n\\t"', '"s_cbranch_vccz .Lrtopk_conv_%=\\n\\t"']
    L += count_lines(E, "t", neg)
    L += ['"s_cmp_lt_i32 %[c0], %[k]\\n\\t"', '"s_cbranch_scc1 .Lrtopk_aless_%=\\n\\t"',
          '"s_cmp_gt_i32 %[c0], %[k]\\n\\t"', '"v_mov_b32 %[lo], %[t]\\n\\t"',
          '"s_cbranch_scc1 .Lrtopk_b_%=\\n\\t"', '"s_branch .Lrtopk_hit_%=\\n\\t"',
          '".Lrtopk_aless_%=:\\n\\t"', '"v_mov_b32 %[hi], %[t]\\n\\t"', '"s_branch .Lrtopk_b_%=\\n\\t"',
          '".Lrtopk_conv_%=:\\n\\t"', '"s_mov_b32 %[hit], 0\\n\\t"', '"s_branch .Lrtopk_end_%=\\n\\t"',
          '".Lrtopk_hit_%=:\\n\\t"', '"s_mov_b32 %[hit], 1\\n\\t"', '".Lrtopk_end_%=:"']
    outs, ins = operands(E, ['[t] "=&v"(t)', '[u] "=&v"(u)', '[hit] "=&s"(hit)'], [])
    what = {0: "", 1: ", half rows (midpoints truncated to 11 bits)", 2: ", bfloat16 rows (midpoints truncated to 8 bits)"}[dt]
    return (f"""// Algorithm 1 at epsilon = 0, {E} values per lane{', keys = negated values' if neg else ''}{what}.  Returns true when a step counted exactly k (m[] then
// selects the answer); false when the search converged first (lo, hi hold the final bounds).  Steps
// alternate between two code copies that keep their midpoints in different registers, so that copy A
// can compare its midpoint with the previous one.
__device__ __forceinline__ bool search_exact_asm(const float (&x)[{E}], float& lo, float& hi, int k,
                                                 uint64_t (&m)[{E}], std::{"true" if neg else "false"}_type /*keys negated*/,
                                                 std::integral_constant<int, {dt}> /*row element type*/) {{
  float t, u;
  int c0, c1, c2, c3, hit;
""" + emit(L, outs, ins) + "  return hit != 0;\n}\n")


def gen_early(E, neg):
    L = ['"s_mov_b32 %[c0], -1\\n\\t"', '"s_sub_u32 %[it], %[n], 1\\n\\t"', '"s_cbranch_scc1 .Lrtopk_end_%=\\n\\t"',
         '".Lrtopk_top_%=:\\n\\t"', '"v_add_f32 %[t], %[lo], %[hi]\\n\\t"', '"v_mul_f32 %[t], 0.5, %[t]\\n\\t"']
    L += count_lines(E, "t", neg)
    L += ['"s_cmp_lt_i32 %[c0], %[k]\\n\\t"', '"s_cbranch_scc1 .Lrtopk_less_%=\\n\\t"',
          '"s_cmp_gt_i32 %[c0], %[k]\\n\\t"', '"v_mov_b32 %[lo], %[t]\\n\\t"',
          '"s_cbranch_scc0 .Lrtopk_end_%=\\n\\t"', '"s_sub_u32 %[it], %[it], 1\\n\\t"',
          '"s_cbranch_scc0 .Lrtopk_top_%=\\n\\t"', '"s_branch .Lrtopk_end_%=\\n\\t"',
          '".Lrtopk_less_%=:\\n\\t"', '"v_mov_b32 %[hi], %[t]\\n\\t"', '"s_sub_u32 %[it], %[it], 1\\n\\t"',
          '"s_cbranch_scc0 .Lrtopk_top_%=\\n\\t"', '".Lrtopk_end_%=:"']
    outs, ins = operands(E, ['[t] "=&v"(t)', '[it] "=&s"(it)'], ['[n] "s"(max_iter)'])
    return (f"""// Algorithm 2, {E} values per lane{', keys = negated values' if neg else ''}: max_iter steps (fewer when a step counts exactly k, after which the
// selection cannot change).  Returns the count of the last step, or -1 when no step ran; when it is
// >= k, m[] holds the masks of x >= lo.
__device__ __forceinline__ int search_early_asm(const float (&x)[{E}], float& lo, float& hi, int k, int max_iter,
                                                uint64_t (&m)[{E}], std::{"true" if neg else "false"}_type /*keys negated*/) {{
  float t;
  int c0, c1, c2, c3, it;
""" + emit(L, outs, ins) + "  return c0;\n}\n")


# ---------------------------------------------------------------------------------------------------
# Row minima and maxima of R rows in one transposed reduction.
#
# On entry lane l holds, for each row r, mx[r] = max of its elements and nm[r] = max of its negated
# elements.  Reducing each of the 2R values on its own costs six cross-lane steps per value.  Here every
# step combines the upper and lower halves of TWO registers at once and keeps both results in one
# register (one result in one half of the lanes, the other in the other half), so the number of live
# registers halves with the lane distance: 2R -> R (distance 32, v_permlane32_swap), R -> R/2 (16,
# v_permlane16_swap), -> R/4 (8, row_ror:8 written to the upper banks only for the second register),
# -> R/8 (4, row_half_mirror likewise), then two quad steps on what is left.  4 vector instructions per
# row instead of 9, and no idle slots: the independent pairs fill the two wait states that a cross-lane
# read needs after a write.
# Result: for row r (r < 8; sixteen rows are reduced as two batches of eight) the maximum is in lane
# 16*(r&1) + 8*((r>>1)&1) + 4*((r>>2)&1) and the negated minimum 32 lanes above it.
# ---------------------------------------------------------------------------------------------------
def gen_minmax(R):
    ins = []  # (text, dst regs, src regs)
    mx = [f"mx{r}" for r in range(R)]
    nm = [f"nm{r}" for r in range(R)]

    def op(text, writes, reads):
        ins.append((text, writes, reads))

    for r in range(R):
        op(f"v_permlane32_swap_b32 %[{mx[r]}], %[{nm[r]}]", [mx[r], nm[r]], [mx[r], nm[r]])
    for r in range(R):
        op(f"v_max_f32 %[{mx[r]}], %[{mx[r]}], %[{nm[r]}]", [mx[r]], [mx[r], nm[r]])
    live = list(range(R))  # indices into mx
    # distance 16
    if len(live) > 1:
        for i in range(0, len(live), 2):
            a, b = mx[live[i]], mx[live[i + 1]]
            op(f"v_permlane16_swap_b32 %[{a}], %[{b}]", [a, b], [a, b])
        for i in range(0, len(live), 2):
            a, b = mx[live[i]], mx[live[i + 1]]
            op(f"v_max_f32 %[{a}], %[{a}], %[{b}]", [a], [a, b])
        live = live[0::2]
    cur = [mx[i] for i in live]           # registers holding the partial results
    spare = [nm[i] for i in live]         # free registers of the same count
    for ctrl, banks in (("row_ror:8", "0xc"), ("row_half_mirror", "0xa")):
        if len(cur) > 1:
            nxt, nsp = [], []
            for i in range(0, len(cur), 2):
                d = spare[i]
                op(f"v_max_f32_dpp %[{d}], %[{cur[i]}], %[{cur[i]}] {ctrl} row_mask:0xf bank_mask:0xf", [d], [cur[i]])
                nxt.append(d)
                nsp.append(cur[i])
            for i in range(0, len(cur), 2):
                d = spare[i]
                op(f"v_max_f32_dpp %[{d}], %[{cur[i + 1]}], %[{cur[i + 1]}] {ctrl} row_mask:0xf bank_mask:{banks}",
                   [d], [cur[i + 1], d])
            cur, spare = nxt, nsp
        else:
            d = spare[0]
            op(f"v_max_f32_dpp %[{d}], %[{cur[0]}], %[{cur[0]}] {ctrl} row_mask:0xf bank_mask:0xf", [d], [cur[0]])
            cur, spare = [d], [cur[0]]
    for ctrl in ("quad_perm:[1,0,3,2]", "quad_perm:[2,3,0,1]"):
        nxt, nsp = [], []
        for i in range(len(cur)):
            d = spare[i]
            op(f"v_max_f32_dpp %[{d}], %[{cur[i]}], %[{cur[i]}] {ctrl} row_mask:0xf bank_mask:0xf", [d], [cur[i]])
            nxt.append(d)
            nsp.append(cur[i])
        cur, spare = nxt, nsp
    # two wait states between a write and any later read of the same register inside the block
    lines = ['"s_nop 1\\n\\t"']  # the inputs were written by the instructions just before the block
    last_write = {}
    pos = 0
    for text, writes, reads in ins:
        need = 0
        for rname in set(reads) | set(writes):
            if rname in last_write:
                need = max(need, 3 - (pos - last_write[rname]))
        if need > 0:
            lines.append(f'"s_nop {need - 1}\\n\\t"')
            pos += need
        lines.append(f'"{text}\\n\\t"')
        for w in writes:
            last_write[w] = pos
        pos += 1
    lines[-1] = lines[-1].replace("\\n\\t", "")
    outs = [f'[mx{r}] "+v"(mx[{r}])' for r in range(R)] + [f'[nm{r}] "+v"(nm[{r}])' for r in range(R)]
    body = "\n".join("      " + l for l in lines)
    res = ", ".join(f"{c[:2]}[{c[2:]}]" for c in cur)
    n_valu = len(ins)
    getters = []
    for r in range(R):
        reg = cur[r // 8]
        reg_c = f"{reg[:2]}[{reg[2:]}]"
        lane = 16 * (r & 1) + 8 * ((r >> 1) & 1) + 4 * ((r >> 2) & 1)
        getters.append(f"  hi[{r}] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int({reg_c}), {lane}));\n"
                       f"  lo[{r}] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int({reg_c}), {lane + 32}) ^ (int)0x80000000);")
    return (f"""// Row maxima and minima of {R} rows in one transposed reduction ({n_valu} vector instructions; see
// gen_search_loops.py for the scheme).  mx[r] / nm[r]: per-lane maximum of row r's elements / of their
// negations; both arrays are overwritten.
__device__ __forceinline__ void wave_max_and_negmin_rows(float (&mx)[{R}], float (&nm)[{R}], float (&hi)[{R}],
                                                         float (&lo)[{R}]) {{
  asm volatile(
{body}
      : {", ".join(outs)});
""" + "\n".join(getters) + "\n}\n")


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    text = ("// GENERATED by gen_search_loops.py -- do not edit by hand.\n"
            "// Hand-scheduled search loops (gfx950 inline assembly); included inside namespace rtopk.\n\n")
    for E in ELEMS:
        for neg in (False, True):
            text += gen_exact(E, neg) + "\n" + gen_early(E, neg) + "\n"
        for dt in (1, 2):
            text += gen_exact(E, False, dt) + "\n"
    for R in (2, 4, 8):
        text += gen_minmax(R) + "\n"
    path = os.path.join(here, "rtopk_search_loops.inc")
    old = open(path).read() if os.path.exists(path) else None
    if old != text:
        with open(path, "w") as f:
            f.write(text)
    return path


if __name__ == "__main__":
    print(main())
    sys.exit(0)
