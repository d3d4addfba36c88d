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


# ---- the fused step: logits, online softmax and P V of one 64-key tile whose keys are all valid ----
# The tile is handled as two halves of 32 keys, each with its own online-softmax update, so that the
# VALU work of one half runs in the shadow of the other half's MFMAs (a wave issues a VALU instruction
# only every other issue slot, so a softmax on its own leaves the SIMD mostly idle):
#   S0 = K[0:32] Q^T                      (the next tile pair is requested in the shadow of these MFMAs)
#   S1 = K[32:64] Q^T                     with the softmax of S0 -> P0 in its shadow (accumulators rescaled if needed)
#   O += V[0:32]^T P0                     with the softmax of S1 -> P1 in its shadow
#   (accumulators rescaled if the second half raised the maximum: only now, when no MFMA adds to them)
#   O += V[32:64]^T P1
# Registers.  The accumulators are operands bound to fixed registers (their elements have to be named
# for the rescaling): O v[0:63].  Internal, declared clobbered: S0 v[168:183], S1 v[184:199],
# P0 v[200:207], P1 v[208:215], addresses v[216:223], temporaries v[224:231], operand buffers v[232:255].
FS_O, FS_S0, FS_S1, FS_P0, FS_P1, FS_A, FS_T = 0, 168, 184, 200, 208, 216, 224
FUSED_CLOBBER_LO = 168


def vr(base, n=1):
    return f"v{base}" if n == 1 else f"v[{base}:{base + n - 1}]"


def max_stream(S):
    """T0 = c * max over the lane's 16 logits v[S:S+15] and those of lane ^ 32"""
    s = lambda i: vr(S + i)
    t0, t1 = vr(FS_T), vr(FS_T + 1)
    return [f"v_max3_f32 {t0}, {s(0)}, {s(1)}, {s(2)}", f"v_max3_f32 {t1}, {s(8)}, {s(9)}, {s(10)}",
            f"v_max3_f32 {t0}, {t0}, {s(3)}, {s(4)}", f"v_max3_f32 {t1}, {t1}, {s(11)}, {s(12)}",
            f"v_max3_f32 {t0}, {t0}, {s(5)}, {s(6)}", f"v_max3_f32 {t1}, {t1}, {s(13)}, {s(14)}",
            f"v_max3_f32 {t0}, {t0}, {s(7)}, {s(15)}", f"v_max_f32 {t0}, {t0}, {t1}",
            f"v_mov_b32 {t1}, {t0}", "s_nop 1", f"v_permlane32_swap_b32 {t0}, {t1}", "s_nop 0",
            f"v_max_f32 {t0}, {t0}, {t1}", f"v_mul_f32 {t0}, %[c], {t0}"]


def exp_stream(S, P, convert=True):
    """p = exp2(s c - m) in place, the two P^T fragments into v[P:P+7] (if convert), l += sum.  Three-stage
    pipeline so that no instruction uses the result of the transcendental issued right before it."""
    s = lambda i: vr(S + i)
    t4 = vr(FS_T + 4)
    out = []
    for i in range(19):
        if i < 16:
            out.append(f"v_fma_f32 {s(i)}, {s(i)}, %[c], -%[m]")
        if 1 <= i <= 16:
            out.append(f"v_exp_f32 {s(i - 1)}, {s(i - 1)}")
        e = i - 3
        if 0 <= e < 16:
            if e % 2 == 0:
                out.append(f"v_add_f32 %[l], %[l], {s(e)}")
            elif e == 3:
                out.append(f"v_add_f32 {t4}, {s(1)}, {s(3)}")
            elif e > 3:
                out.append(f"v_add_f32 {t4}, {t4}, {s(e)}")
            if e % 2 == 1 and convert:
                out.append(f"v_cvt_pk_bf16_f32 {vr(P + e // 2)}, {s(e - 1)}, {s(e)}")
    out.append(f"v_add_f32 %[l], %[l], {t4}")
    return out


def convert_stream(S, P):
    return [f"v_cvt_pk_bf16_f32 {vr(P + j)}, {vr(S + 2 * j)}, {vr(S + 2 * j + 1)}" for j in range(8)]


def raise_max(n_o, now, also=()):
    """after max_stream: if the maximum grew for some lane, m <- max(m, T0), T3 = exp2(m_old - m), l *= T3, and
    either the accumulators too (now) or the wave-uniform decision is left in %[flag] for later.
    The conditional part is one item: it must not be split up (nothing else may sit between branch and label)."""
    t0, t1, t2, t3 = (vr(FS_T + i) for i in range(4))
    tag = "a" if now else "b"
    out = [f"v_cmp_gt_f32 vcc, {t0}, %[m]"]
    if not now:
        out.append("s_mov_b64 %[flag], vcc")
    cond = [f"s_cbranch_vccz .Lfs_keep{tag}_%=",
            f"v_max_f32 {t1}, %[m], {t0}", f"v_sub_f32 {t2}, %[m], {t1}", f"v_exp_f32 {t3}, {t2}",
            f"v_mov_b32 %[m], {t1}", "s_nop 0", f"v_mul_f32 %[l], %[l], {t3}"]
    if now:
        cond += [f"v_mul_f32 {vr(FS_O + i)}, {vr(FS_O + i)}, {t3}" for i in range(n_o)]
    cond += [f"v_mul_f32 {r}, {r}, {t3}" for r in also]  # e.g. weights computed against the old maximum, not yet used
    cond.append(f".Lfs_keep{tag}_%=:")
    out.append(tuple(cond))
    return out


class LdsPipe:
    """fragment loads into the ring of operand buffers, with the bookkeeping for counted waits"""
    def __init__(self, lines, D, nbuf=6):
        self.lines, self.D, self.nbuf, self.issued, self.v_ready = lines, D, nbuf, [], False

    def k_addresses(self):
        for st in range(1, self.D // 16):
            self.lines.append(f"v_xor_b32 {vr(FS_A + st - 1)}, {hex(st << 5)}, %[ak]")

    def v_addresses(self):
        for t in range(1, self.D // 32):
            self.lines.append(f"v_xor_b32 {vr(FS_A + 2 * t - 2)}, {hex(t << 6)}, %[av0]")
            self.lines.append(f"v_xor_b32 {vr(FS_A + 2 * t - 1)}, {hex(t << 6)}, %[av1]")
        self.v_ready = True

    def issue(self, k, load):
        f = k % self.nbuf
        kind, a, b = load
        if kind == "k":
            st, half = a, b
            addr = "%[ak]" if st == 0 else vr(FS_A + st - 1)
            self.lines.append(f"ds_read_b128 {F(f)}, {addr}{off(half * 64 * self.D)}")
            self.issued.append(1)
        else:
            if not self.v_ready:  # all K reads have been issued by now: their address registers are free
                self.v_addresses()
            ks, t = a, b
            a0 = "%[av0]" if t == 0 else vr(FS_A + 2 * t - 2)
            a1 = "%[av1]" if t == 0 else vr(FS_A + 2 * t - 1)
            self.lines.append(f"ds_read_b64_tr_b16 {Flo(f)}, {a0}{off(ks * 32 * self.D)}")
            self.lines.append(f"ds_read_b64_tr_b16 {Fhi(f)}, {a1}{off(ks * 32 * self.D)}")
            self.issued.append(2)

    def wait_for(self, k):
        outstanding = sum(self.issued[k + 1:])
        assert outstanding <= 15
        self.lines.append(f"s_waitcnt lgkmcnt({outstanding})")


def spread(after, k0, k1, stream):
    """distributes the items of `stream` over the slots k0..k1 (instructions that follow MFMA k); an item that
    is a tuple of instructions stays together"""
    nslots = k1 - k0 + 1
    per = -(-len(stream) // nslots)
    for i in range(nslots):
        for item in stream[i * per:(i + 1) * per]:
            after.setdefault(k0 + i, []).extend(list(item) if isinstance(item, tuple) else [item])


def fused_step(D):
    ns, nt = D // 16, D // 32
    ni = (64 // (1024 // (2 * D))) // 4
    n_o = 16 * nt
    mf = []
    for half in range(2):
        for st in range(ns):
            mf.append(dict(acc=vr(FS_S0 if half == 0 else FS_S1, 16), first=(st == 0), b=f"%[q{st}]", load=("k", st, half)))
    for half in range(2):
        for ks2 in range(2):
            for t in range(nt):
                mf.append(dict(acc=vr(FS_O + 16 * t, 16), first=False, b=vr((FS_P0 if half == 0 else FS_P1) + 4 * ks2, 4),
                               load=("v", 2 * half + ks2, t)))
    n = len(mf)
    after = {}
    qk1_end, pv0_end = 2 * ns - 1, 2 * ns + 2 * nt - 1
    spread(after, ns + 1, qk1_end, max_stream(FS_S0) + raise_max(n_o, True) + exp_stream(FS_S0, FS_P0))
    spread(after, 2 * ns + 1, pv0_end, max_stream(FS_S1) + raise_max(n_o, False) + exp_stream(FS_S1, FS_P1))
    # the accumulators are rescaled for the second half once the MFMAs that add to them are done
    after[pv0_end] += ["s_cmp_eq_u64 %[flag], 0", "s_cbranch_scc1 .Lfs_nors_%=", "s_nop 13"] + \
        [f"v_mul_f32 {vr(FS_O + i)}, {vr(FS_O + i)}, {vr(FS_T + 3)}" for i in range(n_o)] + [".Lfs_nors_%=:"]
    before = {2 * ns: ["s_nop 1"], 2 * ns + 2 * nt: ["s_nop 1"]}  # P^T / accumulators were written by VALU just before

    lines = []
    pipe = LdsPipe(lines, D)
    pipe.k_addresses()
    for k in range(pipe.nbuf):
        pipe.issue(k, mf[k]["load"])
    dmas = [("k", j) for j in range(ni)] + [("v", j) for j in range(ni)]
    for k in range(n):
        pipe.wait_for(k)
        lines += before.get(k, [])
        m = mf[k]
        lines.append(f"{MFMA} {m['acc']}, {F(k % pipe.nbuf)}, {m['b']}, {'0' if m['first'] else m['acc']}")
        if dmas:
            lines.append(f"s_add_u32 m0, %[l{dmas[0][0]}], {hex(dmas[0][1] * 4096)}")
        if k + pipe.nbuf < n:
            pipe.issue(k + pipe.nbuf, mf[k + pipe.nbuf]["load"])
        elif dmas:
            lines.append("s_nop 0")
        if dmas:
            which, jj = dmas.pop(0)
            lines.append(f"global_load_lds_dwordx4 %[x{jj}], %[{which}b]")
        lines += after.get(k, [])
    assert not dmas
    lines.append(NOP_AFTER)
    return lines


def run_pipe(D, mf, before, after, dmas):
    """MFMA k of `mf` with its operand fetch issued six MFMAs ahead; `before[k]` / `after[k]` are instruction
    lists placed right before / after MFMA k; `dmas`: tile-load instructions (slot tag, index), one per MFMA
    shadow from the first MFMA on."""
    lines = []
    pipe = LdsPipe(lines, D)
    pipe.k_addresses()
    n = len(mf)
    for k in range(min(pipe.nbuf, n)):
        pipe.issue(k, mf[k]["load"])
    dmas = list(dmas)
    for k in range(n):
        pipe.wait_for(k)
        lines += before.get(k, [])
        m = mf[k]
        lines.append(f"{MFMA} {m['acc']}, {F(k % pipe.nbuf)}, {m['b']}, {'0' if m['first'] else m['acc']}")
        if dmas:
            lines.append(f"s_add_u32 m0, %[l{dmas[0][0]}], {hex(dmas[0][1] * 4096)}")
        if k + pipe.nbuf < n:
            pipe.issue(k + pipe.nbuf, mf[k + pipe.nbuf]["load"])
        elif dmas:
            lines.append("s_nop 0")
        if dmas:
            which, jj = dmas.pop(0)
            lines.append(f"global_load_lds_dwordx4 %[x{jj}], %[{which}b]")
        lines += after.get(k, [])
    assert not dmas
    return lines


def flat(stream):
    out = []
    for item in stream:
        out += list(item) if isinstance(item, tuple) else [item]
    return out


# ---- zeroth-order step of the approximation: one chunk of 32 key blocks, all of them existing and of full size ----
#   Z = Kbar Q^T  (rows 0..31 of the statistics tile; the next tile of the stream is requested in the shadow)
#   a_j = exp2(c z_j - m) for the unselected blocks, 0 for the selected ones; l += b sum a_j; A = sum a_j
#   O += VS^T a   (rows 32..63), the first half of it while the second half of the a_j is still being computed
# A selected block takes part in the running maximum: its mean-key logit cannot exceed the largest logit of
# its keys, which the exact pass has already seen, so it never raises it.  Lane (x, h) holds block 8g + 4h + r
# in register 4g + r, so with the bitmap word shifted right by 4h the block's bit is bit 8g + r for every lane.
# Registers: Z v[168:183], per-element masks v[184:199], P^T v[200:207], the rest as in fused_step.
def stats_step(D):
    ns, nt = D // 16, D // 32
    ni = (64 // (1024 // (2 * D))) // 4
    n_o = 16 * nt
    S, U, P = FS_S0, FS_S1, FS_P0
    s = lambda i: vr(S + i)
    u = lambda i: vr(U + i)
    t4, t5, t7 = vr(FS_T + 4), vr(FS_T + 5), vr(FS_T + 7)
    mf = [dict(acc=vr(S, 16), first=(st == 0), b=f"%[q{st}]", load=("k", st, 0)) for st in range(ns)]
    for ks2 in range(2):
        for t in range(nt):
            mf.append(dict(acc=vr(FS_O + 16 * t, 16), first=False, b=vr(P + 4 * ks2, 4), load=("v", 2 + ks2, t)))
    pre = [f"v_lshrrev_b32 {t5}, %[sh], %[unsel]"] + max_stream(S) + raise_max(n_o, True)
    first_half, second_half = [], []
    for i in range(21):  # software pipeline over the 16 elements
        cur = first_half if i - 4 < 8 and i < 12 else second_half
        if i < 16:
            cur.append(f"v_fma_f32 {s(i)}, {s(i)}, %[c], -%[m]")
            cur.append(f"v_bfe_i32 {u(i)}, {t5}, {8 * (i // 4) + i % 4}, 1")
        if 1 <= i <= 16:
            cur.append(f"v_exp_f32 {s(i - 1)}, {s(i - 1)}")
        e = i - 3
        if 0 <= e < 16:
            cur.append(f"v_and_b32 {s(e)}, {s(e)}, {u(e)}")
        e = i - 4
        if 0 <= e < 16:
            if e == 1:
                cur.append(f"v_add_f32 {t4}, {s(0)}, {s(1)}")
            elif e == 3:
                cur.append(f"v_add_f32 {t7}, {s(2)}, {s(3)}")
            elif e > 3:
                cur.append(f"v_add_f32 {t4 if e % 2 == 0 else t7}, {t4 if e % 2 == 0 else t7}, {s(e)}")
            if e % 2 == 1:
                cur.append(f"v_cvt_pk_bf16_f32 {vr(P + e // 2)}, {s(e - 1)}, {s(e)}")
    t1 = vr(FS_T + 1)
    fin = [f"v_add_f32 {t4}, {t4}, {t7}", "s_nop 0", f"v_fmac_f32 %[l], %[bf], {t4}", f"v_mov_b32 {t1}, {t4}", "s_nop 1",
           f"v_permlane32_swap_b32 {t4}, {t1}", "s_nop 0", f"v_add_f32 %[A], {t4}, {t1}"]
    before = {ns: [NOP_AFTER] + flat(pre) + first_half + ["s_nop 1"], ns + nt: ["s_nop 1"]}
    after = {}
    spread(after, ns, ns + nt - 1, second_half)
    spread(after, ns + nt, ns + 2 * nt - 1, fin)
    lines = run_pipe(D, mf, before, after, [("s", j) for j in range(ni)])
    lines.append(NOP_AFTER)
    return lines


# ---- first-order step: 64 value columns of one group,  O^T[part] += A ((scale Hg)^T[part] Q^T) ----
# Rows 0..31 of the tile first, then rows 32..63 with the update from the first product in the shadow of
# their MFMAs.  The next tile of the stream is requested in the shadow of the first MFMAs.
def first_order_step(D, part):
    ns = D // 16
    ni = (64 // (1024 // (2 * D))) // 4
    mf = []
    for half in range(2):
        for st in range(ns):
            mf.append(dict(acc=vr(FS_S0 if half == 0 else FS_S1, 16), first=(st == 0), b=f"%[q{st}]", load=("k", st, half)))
    o0, o1 = FS_O + 32 * part, FS_O + 32 * part + 16
    after = {}
    spread(after, ns + 1, 2 * ns - 1, [f"v_fmac_f32 {vr(o0 + r)}, %[A], {vr(FS_S0 + r)}" for r in range(16)])
    lines = run_pipe(D, mf, {}, after, [("s", j) for j in range(ni)])
    lines.append(NOP_AFTER)
    lines += [f"v_fmac_f32 {vr(o1 + r)}, %[A], {vr(FS_S1 + r)}" for r in range(16)]
    return lines


def asm_block(lines, outs, ins, extra_clobbers=()):
    text = "\n".join(f'      "{l}\\n\\t"' for l in lines)
    clob = ", ".join([f'"v{r}"' for r in range(CLOBBER_LO, CLOBBER_HI + 1)] + [f'"{c}"' for c in extra_clobbers])
    return f"  asm volatile(\n{text}\n      : {', '.join(outs)}\n      : {', '.join(ins)}\n      : {clob});\n"


def logits_softmax(D):
    """The first half of fused_step for loops that must meet a barrier before P V (the V tile lands later):
    S0, S1 = K Q^T with the softmax of S0 in the shadow of the MFMAs of S1, then the softmax of S1; leaves
    P0, P1.  No MFMA adds to the accumulators meanwhile, so both halves rescale them at once; the weights of the
    first half stay fp32 until the second half has settled the maximum."""
    ns, nt = D // 16, D // 32
    ni = (64 // (1024 // (2 * D))) // 4
    n_o = 16 * nt
    mf = []
    for half in range(2):
        for st in range(ns):
            mf.append(dict(acc=vr(FS_S0 if half == 0 else FS_S1, 16), first=(st == 0), b=f"%[q{st}]", load=("k", st, half)))
    n = len(mf)
    after = {}
    spread(after, ns + 1, n - 1, max_stream(FS_S0) + raise_max(n_o, True) + exp_stream(FS_S0, FS_P0, convert=False))
    lines = []
    pipe = LdsPipe(lines, D)
    pipe.k_addresses()
    for k in range(pipe.nbuf):
        pipe.issue(k, mf[k]["load"])
    dmas = [("k", j) for j in range(ni)] + [("v", j) for j in range(ni)]
    for k in range(n):
        pipe.wait_for(k)
        m = mf[k]
        lines.append(f"{MFMA} {m['acc']}, {F(k % pipe.nbuf)}, {m['b']}, {'0' if m['first'] else m['acc']}")
        if dmas:
            lines.append(f"s_add_u32 m0, %[l{dmas[0][0]}], {hex(dmas[0][1] * 4096)}")
        if k + pipe.nbuf < n:
            pipe.issue(k + pipe.nbuf, mf[k + pipe.nbuf]["load"])
        elif dmas:
            lines.append("s_nop 0")
        if dmas:
            which, jj = dmas.pop(0)
            lines.append(f"global_load_lds_dwordx4 %[x{jj}], %[{which}b]")
        lines += after.get(k, [])
    assert not dmas
    lines.append(NOP_AFTER)  # the last MFMA of S1 has to deliver before its maximum is taken
    # the weights of the first half are still fp32: if the second half raises the maximum they follow it
    for item in max_stream(FS_S1) + raise_max(n_o, True, also=[vr(FS_S0 + i) for i in range(16)]) + \
            convert_stream(FS_S0, FS_P0) + exp_stream(FS_S1, FS_P1):
        lines += list(item) if isinstance(item, tuple) else [item]
    # raise_max(.., True) is used twice in this sequence: make its labels distinct
    seen, out = 0, []
    for l in lines:
        if "Lfs_keepa" in l:
            l = l.replace("Lfs_keepa", "Lfs_keepa" if seen < 2 else "Lfs_keepc")
            seen += 1
        out.append(l)
    return out


# Operands that are MFMA results or inputs of several sequences are bound to the same registers everywhere,
# which leaves the register allocator nothing to get wrong: accumulators O v[0:63], logits v[168:199],
# P^T fragments v[200:215].
def o_ops(nt):
    return [f'[o{t}] "+{{v[{FS_O + 16 * t}:{FS_O + 16 * t + 15}]}}"(o[{t}])' for t in range(nt)]


def c_ops():
    return ['[c0] "=&{v[168:183]}"(c0)', '[c1] "=&{v[184:199]}"(c1)']


def p_ops(nks):
    return [f'[p{k}] "{{v[{200 + 4 * k}:{200 + 4 * k + 3}]}}"(p[{k}])' for k in range(nks)]


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
        out.append(asm_block(rows_x_q(D, True, 0), c_ops(), ['[a] "v"(a)'] + q_inputs(D), ("memory",)))
        out.append("}\n\n")
        out.append(f"// the same, and in the shadow of the first MFMAs this wave's share of the next K tile (from kb into the slot\n"
                   f"// at LDS address lk) and V tile (vb, lv) is requested; x = the lane's byte offsets of its {ni} loads per tile\n"
                   f"PASA_DEVICE void rows_x_q_dma(uint32_t a, const bf16x8 (&q)[{D // 16}], f32x16& c0, f32x16& c1, const void* kb,\n"
                   f"                             const void* vb, const uint32_t (&x)[{ni}], uint32_t lk, uint32_t lv) {{\n")
        ins = ['[a] "v"(a)'] + q_inputs(D) + ['[kb] "s"(kb)', '[vb] "s"(vb)', '[lk] "s"(lk)', '[lv] "s"(lv)'] + \
              [f'[x{j}] "v"(x[{j}])' for j in range(ni)]
        out.append(asm_block(rows_x_q(D, True, ni), c_ops(), ins, ("memory", "scc", "m0")))
        out.append("}\n\n")
        out.append(f"// rows 0..31 only: c0 + c1 = (tile rows 0..31) x Q^T (even contraction steps in c0, odd ones in c1)\n"
                   f"PASA_DEVICE void rows32_x_q(uint32_t a, const bf16x8 (&q)[{D // 16}], f32x16& c0, f32x16& c1) {{\n")
        out.append(asm_block(rows_x_q(D, False, 0), c_ops(), ['[a] "v"(a)'] + q_inputs(D), ("memory",)))
        out.append("}\n\n")
        for name, nks, row0 in (("cols_x_p64", 4, 0), ("cols_x_p32_hi", 2, 32)):
            nt = D // 32
            out.append(f"// o[t] += (tile rows {row0}..{row0 + 16 * nks - 1}, value columns 32t..32t+31)^T x p;  a0, a1 = tile address + the lane's\n"
                       f"// column-fragment offsets (rows 0.. and rows 8..)\n"
                       f"PASA_DEVICE void {name}(uint32_t a0, uint32_t a1, const bf16x8 (&p)[{nks}], f32x16 (&o)[{nt}]) {{\n")
            outs = o_ops(nt)
            ins = ['[a0] "v"(a0)', '[a1] "v"(a1)'] + p_ops(nks)
            out.append(asm_block(cols_x_p(D, nks, row0), outs, ins, ("memory",)))
            out.append("}\n\n")
        nt = D // 32
        out.append(f"// cols_x_p64, and in the shadow of the first MFMAs this wave's share of two more tiles is requested (see rows_x_q_dma)\n"
                   f"PASA_DEVICE void cols_x_p64_dma(uint32_t a0, uint32_t a1, const bf16x8 (&p)[4], f32x16 (&o)[{nt}], const void* kb,\n"
                   f"                               const void* vb, const uint32_t (&x)[{ni}], uint32_t lk, uint32_t lv) {{\n")
        outs = o_ops(nt)
        ins = ['[a0] "v"(a0)', '[a1] "v"(a1)'] + p_ops(4) + \
              ['[kb] "s"(kb)', '[vb] "s"(vb)', '[lk] "s"(lk)', '[lv] "s"(lv)'] + [f'[x{j}] "v"(x[{j}])' for j in range(ni)]
        out.append(asm_block(cols_x_p(D, 4, 0, ni), outs, ins, ("memory", "scc", "m0")))
        out.append("}\n\n")
    for D in (128, 64):
        ns, nt = D // 16, D // 32
        ni = (64 // (1024 // (2 * D))) // 4
        out.append(f"// One whole 64-key tile (all keys valid) against the wave's 32 queries: logits, online softmax, P V.\n"
                   f"// ak, av0, av1: K tile address + row-fragment offset, V tile address + the two column-fragment offsets;\n"
                   f"// m, l: running maximum (log2 units) and normaliser share; c = scale * log2(e); kb/vb/x/lk/lv: the next pair\n"
                   f"// of tiles to request (see rows_x_q_dma).\n"
                   f"PASA_DEVICE void fused_step(uint32_t ak, uint32_t av0, uint32_t av1, const bf16x8 (&q)[{ns}], f32x16 (&o)[{nt}],\n"
                   f"                           float& m, float& l, float c, const void* kb, const void* vb,\n"
                   f"                           const uint32_t (&x)[{ni}], uint32_t lk, uint32_t lv) {{\n"
                   f"  uint64_t flag;\n")
        outs = o_ops(nt) + \
               ['[m] "+v"(m)', '[l] "+v"(l)', '[flag] "=&s"(flag)']
        ins = ['[ak] "v"(ak)', '[av0] "v"(av0)', '[av1] "v"(av1)', '[c] "s"(c)'] + q_inputs(D) + \
              ['[kb] "s"(kb)', '[vb] "s"(vb)', '[lk] "s"(lk)', '[lv] "s"(lv)'] + [f'[x{j}] "v"(x[{j}])' for j in range(ni)]
        text = "\n".join(f'      "{l}\\n\\t"' for l in fused_step(D))
        clob = ", ".join([f'"v{r}"' for r in range(FUSED_CLOBBER_LO, 256)] + ['"memory"', '"scc"', '"vcc"', '"m0"'])
        out.append(f"  asm volatile(\n{text}\n      : {', '.join(outs)}\n      : {', '.join(ins)}\n      : {clob});\n}}\n\n")
    for D in (128, 64):
        ns, nt = D // 16, D // 32
        ni = (64 // (1024 // (2 * D))) // 4
        out.append(f"// Logits and online softmax of one whole 64-key tile (all keys valid); leaves the P^T fragments p.  Two more\n"
                   f"// tiles are requested meanwhile (see rows_x_q_dma).  Arguments as in fused_step.\n"
                   f"PASA_DEVICE void logits_softmax(uint32_t ak, const bf16x8 (&q)[{ns}], f32x16 (&o)[{nt}], float& m, float& l, float c,\n"
                   f"                               bf16x8 (&p)[4], const void* kb, const void* vb, const uint32_t (&x)[{ni}],\n"
                   f"                               uint32_t lk, uint32_t lv) {{\n")
        outs = o_ops(nt) + ['[m] "+v"(m)', '[l] "+v"(l)'] + \
               [f'[p{k}] "=&{{v[{200 + 4 * k}:{200 + 4 * k + 3}]}}"(p[{k}])' for k in range(4)]
        ins = ['[ak] "v"(ak)', '[c] "s"(c)'] + q_inputs(D) + \
              ['[kb] "s"(kb)', '[vb] "s"(vb)', '[lk] "s"(lk)', '[lv] "s"(lv)'] + [f'[x{j}] "v"(x[{j}])' for j in range(ni)]
        text = "\n".join(f'      "{l}\\n\\t"' for l in logits_softmax(D))
        clob = ", ".join([f'"v{r}"' for r in range(168, 200)] + [f'"v{r}"' for r in range(216, 256)] +
                         ['"memory"', '"scc"', '"vcc"', '"m0"'])
        out.append(f"  asm volatile(\n{text}\n      : {', '.join(outs)}\n      : {', '.join(ins)}\n      : {clob});\n}}\n\n")
    for D in (128, 64):
        ns, nt = D // 16, D // 32
        ni = (64 // (1024 // (2 * D))) // 4
        dma_ins = ['[sb] "s"(sb)', '[ls] "s"(ls)'] + [f'[x{j}] "v"(x[{j}])' for j in range(ni)]
        out.append(f"// Zeroth-order step of the approximation for a chunk of 32 existing, full key blocks.  ak, av0, av1: the\n"
                   f"// statistics tile's address + row-fragment / column-fragment offsets; unsel: bit x set iff block x of the\n"
                   f"// chunk is NOT selected; sh = 4 * (lane >> 5); bf = tokens per block; A <- sum of the chunk's weights a_j.\n"
                   f"// One more tile (from sb into the slot at LDS address ls) is requested meanwhile.\n"
                   f"PASA_DEVICE void stats_step(uint32_t ak, uint32_t av0, uint32_t av1, const bf16x8 (&q)[{ns}], f32x16 (&o)[{nt}],\n"
                   f"                           float& m, float& l, float c, uint32_t unsel, uint32_t sh, float bf, float& A,\n"
                   f"                           const void* sb, const uint32_t (&x)[{ni}], uint32_t ls) {{\n")
        outs = o_ops(nt) + ['[m] "+v"(m)', '[l] "+v"(l)', '[A] "=&v"(A)']
        ins = ['[ak] "v"(ak)', '[av0] "v"(av0)', '[av1] "v"(av1)', '[c] "s"(c)', '[unsel] "s"(unsel)', '[sh] "v"(sh)',
               '[bf] "s"(bf)'] + q_inputs(D) + dma_ins
        text = "\n".join(f'      "{l}\\n\\t"' for l in stats_step(D))
        clob = ", ".join([f'"v{r}"' for r in range(FUSED_CLOBBER_LO, 256)] + ['"memory"', '"scc"', '"vcc"', '"m0"'])
        out.append(f"  asm volatile(\n{text}\n      : {', '.join(outs)}\n      : {', '.join(ins)}\n      : {clob});\n}}\n\n")
        for part in range(D // 64):
            out.append(f"// First-order step: o[{2 * part}], o[{2 * part + 1}] += A * (tile x Q^T), the tile being rows {64 * part}..{64 * part + 63} of the\n"
                       f"// group's (scale Hg)^T; a = tile address + row-fragment offset; one more tile is requested (see stats_step).\n"
                       f"PASA_DEVICE void first_order_step{part}(uint32_t ak, const bf16x8 (&q)[{ns}], f32x16 (&o)[{nt}], float A,\n"
                       f"                                 const void* sb, const uint32_t (&x)[{ni}], uint32_t ls) {{\n")
            outs = [o_ops(nt)[2 * part], o_ops(nt)[2 * part + 1]]
            ins = ['[ak] "v"(ak)', '[A] "v"(A)'] + q_inputs(D) + dma_ins
            text = "\n".join(f'      "{l}\\n\\t"' for l in first_order_step(D, part))
            out.append(f"  asm volatile(\n{text}\n      : {', '.join(outs)}\n      : {', '.join(ins)}\n      : {clob});\n}}\n\n")
    out.append("}  // namespace pipes\n")
    return "".join(out)


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    with open(os.path.join(here, "pasa_mfma_pipes.hpp"), "w") as f:
        f.write(gen())
