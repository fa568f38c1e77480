#!/usr/bin/env python3
"""Writes tile_blocks_gfx950.h: the hand-scheduled gfx950 inner blocks of the tiled forward kernel.

A block advances ONE running extremum (per branch) over TWO consecutive input channels
(2 x 9 taps of a 3x3 kernel) entirely in registers:

    channel A:  tmp  = max(best, s0 .. s8)      4 x v_max3_f32 + 1 x v_max_f32, result in a temporary
                mA   = tmp  > best               "channel A holds a new extremum"
    channel B:  best = max(tmp, s0' .. s8')     written back in place
                mB   = best > tmp
                idx  = mA ? cA : idx ;  idx = mB ? cB : idx

with s = x + w one v_add_f32 per tap (the kernel value is the SGPR operand).  Going
through the temporary and back keeps every accumulator in its own register with no
copy, and the winning CHANNEL is recorded with 2 compares + 2 selects per 18 taps; the
exact tap inside that channel is recovered after the K loop.  Strict compares in
ascending channel order keep the lowest winning channel.

Instruction order is fixed by hand because gfx950 needs two independent instructions
between a VALU write of a lane mask (v_cmp -> VCC / SGPR pair) and the VALU read of it
(v_cndmask); the compiler neither sees nor pads inside an asm block.  Four masks
(three SGPR pairs and VCC) are live at the end of a block so that every select has at
least three other instructions between it and its compare.

Run:  python3 gen_tile_blocks.py > tile_blocks_gfx950.h
      python3 gen_tile_blocks.py f16 > tile_blocks_f16_gfx950.h   (the binary16 blocks, described at F16_HEADER)
"""

PAIRS = [(0, 1), (2, 3), (4, 5), (6, 7)]


def chain(lines, ch, dst_of, src_first, both):
    """One channel (9 taps) for one accumulator.  dst_of/src_first: dict branch -> operand name."""
    first = True
    for a, b in PAIRS:
        lines.append(f"v_add_f32 %[sa], %[w{ch}{a}], %[x{ch}{a}]")
        lines.append(f"v_add_f32 %[sb], %[w{ch}{b}], %[x{ch}{b}]")
        for br, op in both:
            src = src_first[br] if first else dst_of[br]
            lines.append(f"v_{op}3_f32 %[{dst_of[br]}], %[{src}], %[sa], %[sb]")
        first = False
    lines.append(f"v_add_f32 %[sa], %[w{ch}8], %[x{ch}8]")
    for br, op in both:
        lines.append(f"v_{op}_f32 %[{dst_of[br]}], %[{dst_of[br]}], %[sa]")


def emit_asm(lines):
    return "\n".join(f'      "{l}\\n\\t"' for l in lines)


def gen_both():
    both = [("mx", "max"), ("mn", "min")]
    L = []
    chain(L, "A", {"mx": "tmx", "mn": "tmn"}, {"mx": "bmax", "mn": "bmin"}, both)
    L.append("v_cmp_gt_f32 %[m1], %[tmx], %[bmax]")
    L.append("v_cmp_lt_f32 %[m2], %[tmn], %[bmin]")
    chain(L, "B", {"mx": "bmax", "mn": "bmin"}, {"mx": "tmx", "mn": "tmn"}, both)
    L.append("v_cmp_gt_f32 vcc, %[bmax], %[tmx]")
    L.append("v_cmp_lt_f32 %[m3], %[bmin], %[tmn]")
    L.append("v_cndmask_b32 %[imax], %[imax], %[tA], %[m1]")
    L.append("v_cndmask_b32 %[imin], %[imin], %[tA], %[m2]")
    L.append("v_cndmask_b32 %[imax], %[imax], %[tB], vcc")
    L.append("v_cndmask_b32 %[imin], %[imin], %[tB], %[m3]")
    ins = []
    for ch in "AB":
        ins += [f'[x{ch}{i}] "v"(x{ch}[{i}])' for i in range(9)]
        ins += [f'[w{ch}{i}] "s"(w{ch}[{i}])' for i in range(9)]
    ins += ['[tA] "v"(tA)', '[tB] "v"(tB)']
    return f"""
// Compound mode: one shared add per tap feeds both reductions (paper Sec. 3.5, closing remark).
// 46 VALU instructions for 18 candidates x 2 branches.
__device__ __forceinline__ void blk_both(float& bmax, float& bmin, int& imax, int& imin,
                                         const float (&xA)[9], const float (&xB)[9],
                                         const float (&wA)[9], const float (&wB)[9], int tA, int tB) {{
  float tmx, tmn, sa, sb;
  unsigned long long m1, m2, m3;
  asm(
{emit_asm(L)}
      : [tmx] "=&v"(tmx), [tmn] "=&v"(tmn), [sa] "=&v"(sa), [sb] "=&v"(sb),
        [m1] "=&s"(m1), [m2] "=&s"(m2), [m3] "=&s"(m3),
        [bmax] "+v"(bmax), [bmin] "+v"(bmin), [imax] "+v"(imax), [imin] "+v"(imin)
      : {", ".join(ins)}
      : "vcc");
}}
"""


def gen_one2(name, op, cmp):
    """Single branch, two accumulators (two pixels of one output channel) per block."""
    L = []
    # channel A of both accumulators, then their compares
    for p in "01":
        first = True
        for a, b in PAIRS:
            L.append(f"v_add_f32 %[sa], %[wA{a}], %[xA{p}_{a}]")
            L.append(f"v_add_f32 %[sb], %[wA{b}], %[xA{p}_{b}]")
            src = f"b{p}" if first else f"t{p}"
            L.append(f"v_{op}3_f32 %[t{p}], %[{src}], %[sa], %[sb]")
            first = False
        L.append(f"v_add_f32 %[sa], %[wA8], %[xA{p}_8]")
        L.append(f"v_{op}_f32 %[t{p}], %[t{p}], %[sa]")
    L.append(f"v_cmp_{cmp}_f32 %[m1], %[t0], %[b0]")
    L.append(f"v_cmp_{cmp}_f32 %[m2], %[t1], %[b1]")
    for p in "01":
        first = True
        for a, b in PAIRS:
            L.append(f"v_add_f32 %[sa], %[wB{a}], %[xB{p}_{a}]")
            L.append(f"v_add_f32 %[sb], %[wB{b}], %[xB{p}_{b}]")
            src = f"t{p}" if first else f"b{p}"
            L.append(f"v_{op}3_f32 %[b{p}], %[{src}], %[sa], %[sb]")
            first = False
        L.append(f"v_add_f32 %[sa], %[wB8], %[xB{p}_8]")
        L.append(f"v_{op}_f32 %[b{p}], %[b{p}], %[sa]")
    L.append(f"v_cmp_{cmp}_f32 vcc, %[b0], %[t0]")
    L.append(f"v_cmp_{cmp}_f32 %[m3], %[b1], %[t1]")
    L.append("v_cndmask_b32 %[i0], %[i0], %[tA], %[m1]")
    L.append("v_cndmask_b32 %[i1], %[i1], %[tA], %[m2]")
    L.append("v_cndmask_b32 %[i0], %[i0], %[tB], vcc")
    L.append("v_cndmask_b32 %[i1], %[i1], %[tB], %[m3]")
    ins = []
    for ch in "AB":
        for p in "01":
            ins += [f'[x{ch}{p}_{i}] "v"(x{ch}{p}[{i}])' for i in range(9)]
        ins += [f'[w{ch}{i}] "s"(w{ch}[{i}])' for i in range(9)]
    ins += ['[tA] "v"(tA)', '[tB] "v"(tB)']
    return f"""
// One branch ({op}-plus), two pixels of one output channel.  64 VALU instructions for 2 x 18 candidates.
__device__ __forceinline__ void {name}(float& b0, int& i0, float& b1, int& i1,
                                       const float (&xA0)[9], const float (&xB0)[9],
                                       const float (&xA1)[9], const float (&xB1)[9],
                                       const float (&wA)[9], const float (&wB)[9], int tA, int tB) {{
  float t0, t1, sa, sb;
  unsigned long long m1, m2, m3;
  asm(
{emit_asm(L)}
      : [t0] "=&v"(t0), [t1] "=&v"(t1), [sa] "=&v"(sa), [sb] "=&v"(sb),
        [m1] "=&s"(m1), [m2] "=&s"(m2), [m3] "=&s"(m3),
        [b0] "+v"(b0), [i0] "+v"(i0), [b1] "+v"(b1), [i1] "+v"(i1)
      : {", ".join(ins)}
      : "vcc");
}}
"""


def gen_mixed2(name, inner, outer, cmp):
    """Mixed layers (paper Sec. 3.1 (iii) / (vi)): the inner operator reduces the 9 taps of ONE channel on
    its own (v_{inner}3 over three fresh sums, then three more with two sums each), the outer operator
    folds that channel result into the running extremum.  Same instruction count as the single-branch
    blocks: per channel 9 adds, 4 three-operand reductions, 1 compare, 1 outer fold, 1 select."""
    L = []
    masks = {("0", "A"): "%[m1]", ("1", "A"): "%[m2]", ("0", "B"): "%[m3]", ("1", "B"): "vcc"}
    for ch in "AB":
        for p in "01":
            L.append(f"v_add_f32 %[sa], %[w{ch}0], %[x{ch}{p}_0]")
            L.append(f"v_add_f32 %[sb], %[w{ch}1], %[x{ch}{p}_1]")
            L.append(f"v_add_f32 %[sc], %[w{ch}2], %[x{ch}{p}_2]")
            L.append(f"v_{inner}3_f32 %[t{p}], %[sa], %[sb], %[sc]")
            for a, b in [(3, 4), (5, 6), (7, 8)]:
                L.append(f"v_add_f32 %[sa], %[w{ch}{a}], %[x{ch}{p}_{a}]")
                L.append(f"v_add_f32 %[sb], %[w{ch}{b}], %[x{ch}{p}_{b}]")
                L.append(f"v_{inner}3_f32 %[t{p}], %[t{p}], %[sa], %[sb]")
        # the folds of both pixels after both chains: no instruction reads its predecessor's result
        for p in "01":
            L.append(f"v_cmp_{cmp}_f32 {masks[(p, ch)]}, %[t{p}], %[b{p}]")
        for p in "01":
            L.append(f"v_{outer}_f32 %[b{p}], %[b{p}], %[t{p}]")
    L.append("v_cndmask_b32 %[i0], %[i0], %[tA], %[m1]")
    L.append("v_cndmask_b32 %[i1], %[i1], %[tA], %[m2]")
    L.append("v_cndmask_b32 %[i0], %[i0], %[tB], %[m3]")
    L.append("v_cndmask_b32 %[i1], %[i1], %[tB], vcc")
    ins = []
    for ch in "AB":
        for p in "01":
            ins += [f'[x{ch}{p}_{i}] "v"(x{ch}{p}[{i}])' for i in range(9)]
        ins += [f'[w{ch}{i}] "s"(w{ch}[{i}])' for i in range(9)]
    ins += ['[tA] "v"(tA)', '[tB] "v"(tB)']
    return f"""
// Mixed layer: {inner}-plus inside a channel, {outer} across channels; two pixels of one output channel.
// 64 VALU instructions for 2 x 18 candidates.
__device__ __forceinline__ void {name}(float& b0, int& i0, float& b1, int& i1,
                                       const float (&xA0)[9], const float (&xB0)[9],
                                       const float (&xA1)[9], const float (&xB1)[9],
                                       const float (&wA)[9], const float (&wB)[9], int tA, int tB) {{
  float t0, t1, sa, sb, sc;
  unsigned long long m1, m2, m3;
  asm(
{emit_asm(L)}
      : [t0] "=&v"(t0), [t1] "=&v"(t1), [sa] "=&v"(sa), [sb] "=&v"(sb), [sc] "=&v"(sc),
        [m1] "=&s"(m1), [m2] "=&s"(m2), [m3] "=&s"(m3),
        [b0] "+v"(b0), [i0] "+v"(i0), [b1] "+v"(b1), [i1] "+v"(i1)
      : {", ".join(ins)}
      : "vcc");
}}
"""


HEADER = """// GENERATED by gen_tile_blocks.py - do not edit by hand.
//
// Hand-scheduled gfx950 inner blocks of the tiled 3x3 tropical-convolution forward kernel
// (paper Sec. 3.1 layers (iv)/(v): one max / min over all taps of x + w; Sec. 3.3 compound;
// Sec. 3.1 mixed layers (iii)/(vi): min-plus per channel under a max over channels, and the dual).
// See the generator for the scheme and for why the instruction order is fixed.
#pragma once

namespace tconv {

// Makes the compiler forget the value of a wave-uniform integer (it stays in an SGPR), so that
// loads addressed through it are re-issued instead of being kept live across the whole loop body.
__device__ __forceinline__ int launder_uniform(int v) {
  asm volatile("" : "+s"(v));
  return v;
}

// Between a wave's LDS writes and its reads of what other lanes of the SAME wave wrote: the lanes of a
// wave run in lockstep and LDS executes a wave's operations in order, so only the compiler has to
// be kept from moving memory operations across this point.
__device__ __forceinline__ void wave_lds_fence() { asm volatile("" ::: "memory"); }
"""


# ------------------------------------------------------------------ binary16 blocks (packed VALU)

F16_HEADER = """// GENERATED by gen_tile_blocks.py f16 - do not edit by hand.
//
// Inner blocks of the tiled 3x3 forward kernel for binary16 arithmetic on gfx950 (packed 16-bit VALU).
// Numeric contract: every candidate x + w is ONE add rounded to binary16 (v_pk_add_f16), the reductions compare
// those binary16 sums (v_pk_max_f16 / v_pk_min_f16 return the non-NaN operand, so the NaN that stands for padding
// never wins in either branch).
//
// The two halves of a register are two OUTPUT CHANNELS of one pixel.  The kernel values of a channel pair sit in
// SGPRs as (w[co][k], w[co + 1][k]); an x value is broadcast to both halves by the operand-select bits of the
// packed instruction (op_sel / op_sel_hi pick the half of the x register that holds the tap), so x stays packed as
// it was loaded: two neighbouring columns per register.
//
// A block advances the running extrema of one pixel and one output-channel pair over TWO consecutive input
// channels (18 taps): 18 packed adds, 18 packed max (and 18 packed min in compound mode, on the same sums:
// paper Sec. 3.5, closing remark), and per branch 4 instructions that record the input-channel PAIR whenever a
// half of the extremum changed (xor with the old value, 0/1 per half, 0/0xffff per half, bit-select of the pair
// number).  The block reads the old extrema from one register and writes the new ones to another, so the caller
// alternates two register sets and no copy is made.  The exact tap is recovered after the K loop among the 18
// taps of the recorded pair, in ascending k.
#pragma once

namespace tconv {
namespace f16blk {

// x row registers of a lane: D halo columns (one value each, low half), 4 registers with the 8 core columns
// (two per register), D halo columns.  Element e of the row (0 .. 8 + 2D - 1) -> register and half:
constexpr int xreg(int D, int e) { return e < D ? e : (e < D + 8 ? D + (e - D) / 2 : D + 4 + (e - D - 8)); }
constexpr int xhalf(int D, int e) { return (e >= D && e < D + 8) ? ((e - D) & 1) : 0; }
"""


def f16_block(name, branches):
    """branches: list of (tag, op)"""
    L = []
    for t in range(18):
        s = "sa" if t % 2 == 0 else "sb"
        L.append(f"v_pk_add_f16 %[{s}], %[x{t}], %[w{t}] op_sel:[%[h{t}],0] op_sel_hi:[%[h{t}],1]")
        for tag, op in branches:
            src = f"s{tag}" if t == 0 else f"d{tag}"
            L.append(f"v_pk_{op}_f16 %[d{tag}], %[{src}], %[{s}]")
    for tag, _ in branches:
        L.append(f"v_xor_b32 %[c{tag}], %[d{tag}], %[s{tag}]")
    for tag, _ in branches:
        L.append(f"v_pk_min_u16 %[c{tag}], %[c{tag}], %[one2]")
    for tag, _ in branches:
        L.append(f"v_pk_sub_u16 %[c{tag}], 0, %[c{tag}]")
    for tag, _ in branches:
        L.append(f"v_bfi_b32 %[i{tag}], %[c{tag}], %[tid], %[i{tag}]")
    outs = ['[sa] "=&v"(sa)', '[sb] "=&v"(sb)']
    outs += [f'[d{tag}] "=&v"(d{tag})' for tag, _ in branches]
    outs += [f'[c{tag}] "=&v"(c{tag})' for tag, _ in branches]
    outs += [f'[i{tag}] "+v"(i{tag})' for tag, _ in branches]
    ins = [f'[s{tag}] "v"(s{tag})' for tag, _ in branches]
    ins += [f'[x{t}] "v"(xs[{t // 3}][xreg(D, Q + {t % 3} * D)])' for t in range(18)]
    ins += [f'[h{t}] "n"(xhalf(D, Q + {t % 3} * D))' for t in range(18)]
    ins += [f'[w{t}] "s"(w[{t}])' for t in range(18)]
    ins += ['[tid] "s"(tid)', '[one2] "v"(one2)']
    params = ", ".join([f"unsigned& d{tag}" for tag, _ in branches] + [f"unsigned s{tag}" for tag, _ in branches] +
                       [f"unsigned& i{tag}" for tag, _ in branches])
    decl = ", ".join([f"c{tag}" for tag, _ in branches])
    n = 18 + 18 * len(branches) + 4 * len(branches)
    return f"""
// {n} VALU instructions for 18 taps x 2 output channels x {len(branches)} branch(es).
// xs: the six x rows of the two input channels; Q: the pixel; w: 18 kernel-value pairs; tid: the pair number in
// both halves; one2: 0x00010001.
template <int D, int Q>
__device__ __forceinline__ void {name}({params}, const unsigned (&xs)[6][4 + 2 * D],
                                       const unsigned (&w)[18], unsigned tid, unsigned one2) {{
  unsigned sa, sb, {decl};
  asm(
{emit_asm(L)}
      : {", ".join(outs)}
      : {", ".join(ins)});
}}
"""


def gen_f16():
    out = F16_HEADER
    out += f16_block("blk_both", [("mx", "max"), ("mn", "min")])
    out += f16_block("blk_max", [("mx", "max")])
    out += f16_block("blk_min", [("mn", "min")])
    out += "\n}  // namespace f16blk\n}  // namespace tconv\n"
    return out


if __name__ == "__main__":
    import sys
    if len(sys.argv) > 1 and sys.argv[1] == "f16":
        print(gen_f16(), end="")
        sys.exit(0)
    out = HEADER + gen_both() + gen_one2("blk_max2", "max", "gt") + gen_one2("blk_min2", "min", "lt")
    out += gen_mixed2("blk_minmax2", "min", "max", "gt") + gen_mixed2("blk_maxmin2", "max", "min", "lt")
    out += "\n}  // namespace tconv\n"
    print(out, end="")
