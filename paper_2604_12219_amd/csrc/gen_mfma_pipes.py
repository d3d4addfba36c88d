#!/usr/bin/env python3
"""Writes pasa_mfma_pipes.hpp: the software-pipelined LDS-read + MFMA sequences of the attention kernel.

Why generated assembly: the operand fetches of an MFMA chain have to be requested several MFMAs ahead of
their use (an LDS read takes longer than an MFMA), which needs a fixed set of operand buffers and counted
waits.  Each sequence is ONE asm statement, so nothing can be scheduled into it and no register of it can
be copied or reused while a read is in flight.  The operand buffers are fixed registers (v226..v255,
declared as clobbered): a transposing read fills half of an MFMA operand, and inline-asm operands cannot
name half of a register tuple.

Run `python gen_mfma_pipes.py` in this directory after changing it; the header is committed.

LDS addressing (see the tile layout in pasa_device.hpp): within a tile, the address of a lane's row
fragment for contraction step s is a0 ^ (s << 5), 32 rows further down is +64*D bytes; the address of a
column fragment of value-column tile t is a0 ^ (t << 6) (and the same for the rows 8 further down, from a
second lane address), 16 rows further down is +32*D bytes.  XOR by a constant and immediate offsets replace
every per-fetch address computation.
"""
import os

FBASE = 232            # operand buffers: 6 x 4 registers v[232:255]
TBASE = 226            # address temporaries v226..v231
CLOBBER_LO, CLOBBER_HI = 226, 255
MFMA = "v_mfma_f32_32x32x16_bf16"
NOP_AFTER = "s_nop 13"  # an 8-pass MFMA result may be read by a VALU instruction 12 wait states later


def F(i):
    return f"v[{FBASE + 4 * i}:{FBASE + 4 * i + 3}]"


def Flo(i):
    return f"v[{FBASE + 4 * i}:{FBASE + 4 * i + 1}]"


def Fhi(i):
    return f"v[{FBASE + 4 * i + 2}:{FBASE + 4 * i + 3}]"


def T(i):
    return f"v{TBASE + i}"


def off(n):
    return f" offset:{n}" if n else ""


def rows_x_q(D, two_halves, dma):
    """acc(s) += rowfrag(rows 0..31 [and 32..63], step s) x q[s].
    two_halves: c0 <- rows 0..31, c1 <- rows 32..63.  Otherwise rows 0..31 only, even steps -> c0, odd -> c1.
    dma: number of tile-load instructions per tile of this wave (0 = none); requests a K-like and a V-like
    tile into the slots whose LDS addresses are %[lk], %[lv]."""
    ns = D // 16
    half_off = 64 * D
    frags = []  # (step s, immediate offset, accumulator)
    for s in range(ns):
        if two_halves:
            frags.append((s, 0, "c0"))
            frags.append((s, half_off, "c1"))
        else:
            frags.append((s, 0, "c0" if s % 2 == 0 else "c1"))
    nbuf = 6
    lines = []
    last = {"s": 0, "reg": "%[a]", "n": 0}

    def addr(s):  # LDS instructions read their address when they issue, so a temporary can be reused at once
        if s != last["s"]:
            last["s"], last["reg"] = s, T(last["n"] % 2)
            last["n"] += 1
            lines.append(f"v_xor_b32 {last['reg']}, {hex(s << 5)}, %[a]")
        return last["reg"] if s else "%[a]"

    def issue(i):
        s, o, _ = frags[i]
        lines.append(f"ds_read_b128 {F(i % nbuf)}, {addr(s)}{off(o)}")

    dmas = [("k", j) for j in range(dma)] + [("v", j) for j in range(dma)]
    n = len(frags)
    for i in range(min(nbuf, n)):
        issue(i)
    seen = set()
    for i in range(n):
        outstanding = min(nbuf - 1, n - 1 - i)
        s, _, acc = frags[i]
        lines.append(f"s_waitcnt lgkmcnt({outstanding})")
        src_c = f"%[{acc}]" if acc in seen else "0"
        seen.add(acc)
        lines.append(f"{MFMA} %[{acc}], {F(i % nbuf)}, %[q{s}], {src_c}")
        if dmas:  # in the shadow of the MFMA: one tile-load instruction (M0 = its LDS destination)
            lines.append(f"s_add_u32 m0, %[l{dmas[0][0]}], {hex(dmas[0][1] * 4096)}")
        if i + nbuf < n:
            issue(i + nbuf)
        elif dmas:
            lines.append("s_nop 0")  # one wait state between the write of M0 and its use
        if dmas:
            which, jj = dmas.pop(0)
            lines.append(f"global_load_lds_dwordx4 %[x{jj}], %[{which}b]")
    assert not dmas, "more tile-load instructions than MFMAs"
    lines.append(NOP_AFTER)
    return lines


def cols_x_p(D, nks, row0, dma=0):
    """o[t] += colfrag(rows row0 + 16 ks .., value columns 32 t ..) x p[ks], ks < nks, t < D/32.
    dma: as in rows_x_q (two tiles, from %[kb] into the slot at %[lk] and from %[vb] into the slot at %[lv])."""
    nt = D // 32
    step_off = 32 * D
    base_off = row0 * 2 * D
    frags = [(ks, t) for ks in range(nks) for t in range(nt)]
    nbuf = 6
    lines = []
    for t in range(1, nt):  # addresses for t >= 1
        lines.append(f"v_xor_b32 {T(2 * t - 2)}, {hex(t << 6)}, %[a0]")
        lines.append(f"v_xor_b32 {T(2 * t - 1)}, {hex(t << 6)}, %[a1]")

    def a(t, j):
        return (f"%[a{j}]") if t == 0 else T(2 * t - 2 + j)

    def issue(i):
        ks, t = frags[i]
        o = base_off + ks * step_off
        lines.append(f"ds_read_b64_tr_b16 {Flo(i % nbuf)}, {a(t, 0)}{off(o)}")
        lines.append(f"ds_read_b64_tr_b16 {Fhi(i % nbuf)}, {a(t, 1)}{off(o)}")

    dmas = [("k", j) for j in range(dma)] + [("v", j) for j in range(dma)]
    n = len(frags)
    for i in range(min(nbuf, n)):
        issue(i)
    for i in range(n):
        outstanding = 2 * min(nbuf - 1, n - 1 - i)
        ks, t = frags[i]
        lines.append(f"s_waitcnt lgkmcnt({outstanding})")
        lines.append(f"{MFMA} %[o{t}], {F(i % nbuf)}, %[p{ks}], %[o{t}]")
        if dmas:
            lines.append(f"s_add_u32 m0, %[l{dmas[0][0]}], {hex(dmas[0][1] * 4096)}")
        if i + nbuf < n:
            issue(i + nbuf)
        elif dmas:
            lines.append("s_nop 0")
        if dmas:
            which, jj = dmas.pop(0)
            lines.append(f"global_load_lds_dwordx4 %[x{jj}], %[{which}b]")
    assert not dmas, "more tile-load instructions than MFMAs"
    lines.append(NOP_AFTER)
    return lines


def asm_block(lines, outs, ins, extra_clobbers=()):
    text = "\n".join(f'      "{l}\\n\\t"' for l in lines)
    clob = ", ".join([f'"v{r}"' for r in range(CLOBBER_LO, CLOBBER_HI + 1)] + [f'"{c}"' for c in extra_clobbers])
    return f"  asm volatile(\n{text}\n      : {', '.join(outs)}\n      : {', '.join(ins)}\n      : {clob});\n"


def q_inputs(D):
    return [f'[q{s}] "v"(q[{s}])' for s in range(D // 16)]


def gen():
    out = []
    out.append("// GENERATED by gen_mfma_pipes.py -- do not edit.  Software-pipelined LDS-read + MFMA sequences of the\n"
               "// attention kernel (gfx950).  Every function is one asm statement; v226..v255 are its operand buffers.\n"
               "#pragma once\n#include \"pasa_device.hpp\"\n\nnamespace pipes {\n")
    for D in (128, 64):
        ni = (64 // (1024 // (2 * D))) // 4
        # rows_x_q
        out.append(f"// c0 = (tile rows 0..31) x Q^T, c1 = (tile rows 32..63) x Q^T;  a = tile address + lane's row-fragment offset\n"
                   f"PASA_DEVICE void rows_x_q(uint32_t a, const bf16x8 (&q)[{D // 16}], f32x16& c0, f32x16& c1) {{\n")
        out.append(asm_block(rows_x_q(D, True, 0), ['[c0] "=&v"(c0)', '[c1] "=&v"(c1)'], ['[a] "v"(a)'] + q_inputs(D), ("memory",)))
        out.append("}\n\n")
        out.append(f"// the same, and in the shadow of the first MFMAs this wave's share of the next K tile (from kb into the slot\n"
                   f"// at LDS address lk) and V tile (vb, lv) is requested; x = the lane's byte offsets of its {ni} loads per tile\n"
                   f"PASA_DEVICE void rows_x_q_dma(uint32_t a, const bf16x8 (&q)[{D // 16}], f32x16& c0, f32x16& c1, const void* kb,\n"
                   f"                             const void* vb, const uint32_t (&x)[{ni}], uint32_t lk, uint32_t lv) {{\n")
        ins = ['[a] "v"(a)'] + q_inputs(D) + ['[kb] "s"(kb)', '[vb] "s"(vb)', '[lk] "s"(lk)', '[lv] "s"(lv)'] + \
              [f'[x{j}] "v"(x[{j}])' for j in range(ni)]
        out.append(asm_block(rows_x_q(D, True, ni), ['[c0] "=&v"(c0)', '[c1] "=&v"(c1)'], ins, ("memory", "scc", "m0")))
        out.append("}\n\n")
        out.append(f"// rows 0..31 only: c0 + c1 = (tile rows 0..31) x Q^T (even contraction steps in c0, odd ones in c1)\n"
                   f"PASA_DEVICE void rows32_x_q(uint32_t a, const bf16x8 (&q)[{D // 16}], f32x16& c0, f32x16& c1) {{\n")
        out.append(asm_block(rows_x_q(D, False, 0), ['[c0] "=&v"(c0)', '[c1] "=&v"(c1)'], ['[a] "v"(a)'] + q_inputs(D), ("memory",)))
        out.append("}\n\n")
        for name, nks, row0 in (("cols_x_p64", 4, 0), ("cols_x_p32_hi", 2, 32)):
            nt = D // 32
            out.append(f"// o[t] += (tile rows {row0}..{row0 + 16 * nks - 1}, value columns 32t..32t+31)^T x p;  a0, a1 = tile address + the lane's\n"
                       f"// column-fragment offsets (rows 0.. and rows 8..)\n"
                       f"PASA_DEVICE void {name}(uint32_t a0, uint32_t a1, const bf16x8 (&p)[{nks}], f32x16 (&o)[{nt}]) {{\n")
            outs = [f'[o{t}] "+v"(o[{t}])' for t in range(nt)]
            ins = ['[a0] "v"(a0)', '[a1] "v"(a1)'] + [f'[p{k}] "v"(p[{k}])' for k in range(nks)]
            out.append(asm_block(cols_x_p(D, nks, row0), outs, ins, ("memory",)))
            out.append("}\n\n")
        nt = D // 32
        out.append(f"// cols_x_p64, and in the shadow of the first MFMAs this wave's share of two more tiles is requested (see rows_x_q_dma)\n"
                   f"PASA_DEVICE void cols_x_p64_dma(uint32_t a0, uint32_t a1, const bf16x8 (&p)[4], f32x16 (&o)[{nt}], const void* kb,\n"
                   f"                               const void* vb, const uint32_t (&x)[{ni}], uint32_t lk, uint32_t lv) {{\n")
        outs = [f'[o{t}] "+v"(o[{t}])' for t in range(nt)]
        ins = ['[a0] "v"(a0)', '[a1] "v"(a1)'] + [f'[p{k}] "v"(p[{k}])' for k in range(4)] + \
              ['[kb] "s"(kb)', '[vb] "s"(vb)', '[lk] "s"(lk)', '[lv] "s"(lv)'] + [f'[x{j}] "v"(x[{j}])' for j in range(ni)]
        out.append(asm_block(cols_x_p(D, 4, 0, ni), outs, ins, ("memory", "scc", "m0")))
        out.append("}\n\n")
    out.append("}  // namespace pipes\n")
    return "".join(out)


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    with open(os.path.join(here, "pasa_mfma_pipes.hpp"), "w") as f:
        f.write(gen())
