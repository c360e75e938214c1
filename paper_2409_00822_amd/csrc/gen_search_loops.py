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


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    text = ("// GENERATED by gen_search_loops.py -- do not edit by hand.\n"
            "// Hand-scheduled search loops (gfx950 inline assembly); included inside namespace rtopk.\n\n")
    for E in ELEMS:
        for neg in (False, True):
            text += gen_exact(E, neg) + "\n" + gen_early(E, neg) + "\n"
        for dt in (1, 2):
            text += gen_exact(E, False, dt) + "\n"
    path = os.path.join(here, "rtopk_search_loops.inc")
    old = open(path).read() if os.path.exists(path) else None
    if old != text:
        with open(path, "w") as f:
            f.write(text)
    return path


if __name__ == "__main__":
    print(main())
    sys.exit(0)
