#!/usr/bin/env python3
"""Generates mosaic_w4_tile.inc (greedy) and mosaic_w4_tile_sample.inc (sampling): one vocabulary tile of the 4-wave
fused kernel as one inline-asm statement, the hand-scheduled K-loop followed by the tile's vocabulary reduction.

The K-loop covers the nk K-tiles of the vocabulary tile.  Per K-tile (step g) a wave issues 128
v_mfma_f32_16x16x32_bf16 in two groups of 64 (k 0..31 and k 32..63 of the tile); after every second MFMA
of a group's first half sits one of the 16 ds_read_b128 that fetch the next group's fragments, and after every
fourth one of the group's 8 direct-to-LDS copies, so that nothing but MFMAs is ever waited on in steady state.  The steady-state body (1 <= g, g + 2 < total)
contains no branch at all -- a taken branch costs more than one 16-cycle MFMA -- and all slot / pointer
book-keeping is s_cselect arithmetic; the first step and the last two run a guarded copy of the same schedule.
"""
import os
import re
import sys

# fragment double buffer (2 x 16 tuples of 4 VGPRs) and two address temporaries: early-clobber outputs, so the
# register allocator places them (a fixed clobbered range made it spill everything that lives across the loop)
FA = [[f"%[fa{b}{i}]" for i in range(8)] for b in range(2)]
FB = [[f"%[fb{b}{j}]" for j in range(8)] for b in range(2)]
VT0, VT1 = "%[vt0]", "%[vt1]"
WSRC, HSRC = "s[96:97]", "s[98:99]"
KT = "s95"
NK128 = "s94"

lines = []
uid = [0]


def e(s):
    lines.append(s)


def label(name):
    uid[0] += 1
    return f"L{name}{uid[0]}_%="


# Accumulators: operands of the statement ("+a", for the kernel whose epilogue is C++), or, when the statement
# reduces the tile itself, the AGPR file by number: block (bi, bj) = a[(bi*8 + bj)*4 .. +3].
LITERAL_ACC = [False]


def acc_block(bi, bj):
    if LITERAL_ACC[0]:
        base = (bi * 8 + bj) * 4
        return f"a[{base}:{base + 3}]"
    return f"%[a{bi}{bj}]"


def acc_reg(bi, bj, r):
    return f"a{(bi * 8 + bj) * 4 + r}"


def mfma(bi, bj, buf, zero_c=False):
    """acc += A * B, or acc = A * B (the first product of a tile: no clearing of the accumulator beforehand)"""
    c = "0" if zero_c else acc_block(bi, bj)
    e(f"v_mfma_f32_16x16x32_bf16 {acc_block(bi, bj)}, {FA[buf][bi]}, {FB[buf][bj]}, {c}")


def read_addr(ks):
    e(f"v_add_u32 {VT0}, %[wrd], %[rdw{ks}]")
    e(f"v_add_u32 {VT1}, %[hrd], %[rdh{ks}]")


def reads(buf):
    out = []
    for i in range(8):
        off = f" offset:{2048 * i}" if i else ""
        out.append(f"ds_read_b128 {FA[buf][i]}, {VT0}{off}")
    for j in range(8):
        off = f" offset:{2048 * j}" if j else ""
        out.append(f"ds_read_b128 {FB[buf][j]}, {VT1}{off}")
    return out


def dma_w(i):
    return [f"s_add_u32 m0, %[wdst], {1024 * i}", "s_nop 0", f"global_load_lds_dwordx4 %[woff{i}], {WSRC}"]


def dma_h(i):
    return [f"s_add_u32 m0, %[hdst], {98304 + 1024 * i}", "s_nop 0", f"global_load_lds_dwordx4 %[hoff{i}], {HSRC}"]


def dma_split(i, hidden):
    """the same copy as (m0 setup, the load): in the steady state the setup sits one MFMA ahead of the load, which
    supplies the wait state an M0 write needs before a direct-to-LDS load"""
    seq = dma_h(i) if hidden else dma_w(i)
    return seq[0], seq[2]


def advance_h_ops():
    """next hidden copy: k index, source pointer (forward 128 bytes, back nk*128 after the last K-tile), slot"""
    return ["s_add_u32 %[hk], %[hk], 1",
            "s_add_u32 s98, s98, 128",
            "s_addc_u32 s99, s99, 0",
            "s_cmp_eq_u32 %[hk], %[nk]",
            f"s_cselect_b32 vcc_lo, {NK128}, 0",
            "s_cselect_b32 %[hk], 0, %[hk]",
            "s_sub_u32 s98, s98, vcc_lo",
            "s_subb_u32 s99, s99, 0",
            "s_xor_b32 %[hdst], %[hdst], 0x8000"]


def advance_w_ops():
    """next LM-head copy: k index, source pointer (forward 128 bytes or on to the next 256 rows), slot"""
    return ["s_add_u32 %[wk], %[wk], 1",
            "s_cmp_eq_u32 %[wk], %[nk]",
            "s_cselect_b32 vcc_lo, %[wwrap], 128",
            "s_cselect_b32 %[wk], 0, %[wk]",
            "s_add_u32 s96, s96, vcc_lo",
            "s_addc_u32 s97, s97, 0",
            "s_add_u32 %[wdst], %[wdst], 0x8000",
            "s_cmp_ge_u32 %[wdst], 0x18000",
            "s_cselect_b32 vcc_lo, 0x18000, 0",
            "s_sub_u32 %[wdst], %[wdst], vcc_lo"]


def rotate_read_slots_ops():
    return ["s_add_u32 %[wrd], %[wrd], 0x8000",
            "s_cmp_ge_u32 %[wrd], 0x18000",
            "s_cselect_b32 %[wrd], 0, %[wrd]",
            "s_xor_b32 %[hrd], %[hrd], 0x8000"]


def read_addr_ops(ks):
    return [f"v_add_u32 {VT0}, %[wrd], %[rdw{ks}]", f"v_add_u32 {VT1}, %[hrd], %[rdh{ks}]"]


def advance_h():
    for x in advance_h_ops():
        e(x)


def advance_w():
    for x in advance_w_ops():
        e(x)


def rotate_read_slots():
    for x in rotate_read_slots_ops():
        e(x)


def cond_g_ge1_and(plus):
    """scc = (g >= 1) && (g + plus < total)"""
    e(f"s_add_u32 vcc_lo, %[g], {plus}")
    e("s_cmp_lt_u32 vcc_lo, %[total]")
    e("s_cselect_b32 vcc_lo, 1, 0")
    e("s_cmp_ge_u32 %[g], 1")
    e("s_cselect_b32 vcc_hi, 1, 0")
    e("s_and_b32 vcc_lo, vcc_lo, vcc_hi")


def cond_plus(plus):
    """scc = (g + plus < total)"""
    e(f"s_add_u32 vcc_lo, %[g], {plus}")
    e("s_cmp_lt_u32 vcc_lo, %[total]")


# Copy i of a tile goes out after MFMA COPY_POS[i] of its group: early in the group, so a copy has the longest
# possible time to land before the sync that publishes it, and four MFMAs apart, so the 16 KiB a workgroup
# requests per position never queue up behind the texture addresser (denser or later placement measured slower).
COPY_POS = [1, 5, 9, 13, 17, 21, 25, 29]


def spread(fill, first, ops, per_gap=2):
    """book-keeping instructions `ops`, `per_gap` at a time, into the gaps after MFMA first, first + 1, ..."""
    k = first
    for i in range(0, len(ops), per_gap):
        fill.setdefault(k, []).extend(ops[i:i + per_gap])
        k += 1
    return k


def scheduled_group(buf, fill, zero_c=False):
    """64 MFMAs on fragment buffer `buf`; fill[k] = the instructions that follow MFMA k.  A wave is alone on its
    SIMD and issues one instruction every few cycles, so whatever sits between two MFMAs beyond ~3 instructions
    delays the second one: the steady state keeps every gap that short."""
    order = [(bi, bj) for bi in range(8) for bj in range(8)]
    for k in range(64):
        mfma(*order[k], buf, zero_c)
        for x in fill.get(k, []):
            e(x)


def group(buf, rd=None, dma=None, cond=None, after=None, pos=None):
    """64 MFMAs on fragment buffer `buf` for the guarded (first / last steps) path.  rd = 16 ds_reads, one after
    each even MFMA 0..30.  dma = 8 copy sequences, copy i after MFMA pos[i]; guarded by `cond` when given (then
    the guarded span is pos[0]..pos[7]); `after` runs once the copies are out."""
    e("s_waitcnt lgkmcnt(0)")
    order = [(bi, bj) for bi in range(8) for bj in range(8)]
    if not dma:
        for k in range(64):
            mfma(*order[k], buf)
            if rd and k % 2 == 0 and k < 32:
                e(rd[k // 2])
        return
    lo, hi = pos[0], pos[-1]
    for k in range(lo):
        mfma(*order[k], buf)
        if rd and k % 2 == 0 and k < 32:
            e(rd[k // 2])
    def span(with_dma):
        for k in range(lo, hi + 1):
            mfma(*order[k], buf)
            if rd and k % 2 == 0 and k < 32:
                e(rd[k // 2])
            if with_dma and k in pos:
                for x in dma[pos.index(k)]:
                    e(x)
        if with_dma and after:
            after()
    if cond is None:
        span(True)
    else:
        skip, join = label("nodma"), label("join")
        cond()
        e(f"s_cbranch_scc0 {skip}")
        span(True)
        e(f"s_branch {join}")
        e(f"{skip}:")
        span(False)
        e(f"{join}:")
    for k in range(hi + 1, 64):
        mfma(*order[k], buf)
        if rd and k % 2 == 0 and k < 32:
            e(rd[k // 2])


def steady_fill(buf):
    """Gap contents of one steady-state group: the 16 fragment reads of the other buffer after the even MFMAs of
    the first half, the 8 copies after every fourth MFMA of that half, and the scalar book-keeping spread over the
    second half two instructions at a time."""
    fill = {}
    rd = reads(1 - buf)
    for k in range(0, 32, 2):
        fill.setdefault(k, []).append(rd[k // 2])
    for i, k in enumerate(COPY_POS):
        setup, load = dma_split(i, hidden=(buf == 1))
        fill.setdefault(k - 1, []).append(setup)
        fill.setdefault(k, []).append(load)
    if buf == 0:
        k = spread(fill, 33, advance_w_ops())
        k = spread(fill, k + 1, rotate_read_slots_ops())     # the read slots of the NEXT tile, ahead of the sync
        spread(fill, k + 1, read_addr_ops(0))                # addresses of its first-half fragments
    else:
        k = spread(fill, 33, advance_h_ops())
        k = spread(fill, k + 1, ["s_add_u32 %[g], %[g], 1", f"s_add_u32 {KT}, {KT}, 1"])
        spread(fill, k + 1, read_addr_ops(1))                # next step's second-half fragment addresses
        # scc = (k-tile index < nk) && (g + 2 < total): the next step belongs to this statement and is steady
        spread(fill, 60, ["s_add_u32 vcc_lo, %[g], 2", "s_cmp_lt_u32 vcc_lo, %[total]",
                          "s_cselect_b32 vcc_lo, %[nk], 0", f"s_cmp_lt_u32 {KT}, vcc_lo"])
    return fill


def step_end(top):
    e("s_add_u32 %[g], %[g], 1")
    e(f"s_add_u32 {KT}, {KT}, 1")
    e(f"s_cmp_lt_u32 {KT}, %[nk]")
    e(f"s_cbranch_scc1 {top}")


LOG2E = 0x3FB8AA3B        # fp32 1.4426950408889634
NEG_LOG2E = 0xBFB8AA3B
X = [f"%[x{i}]" for i in range(32)]
ET, EMN, ENML, ESEL, EY = "%[et]", "%[emn]", "%[enml]", "%[esel]", "%[ey]"
MASK = ["s[88:89]", "s[90:91]", "s[92:93]"]


def reduce_column(tb):
    """The vocabulary reduction of one token column of the finished tile (this lane: 8 blocks x 4 ids, element
    e = 4*bi + r is vocabulary id vb + 16*bi + r) into the running (max, sum-exp, arg-max) of the column:
        t = max_e x[e];  sel = lowest e with x[e] == t;  if t > m: i = vb + code(sel)
        mn = max(m, t);  s = s * 2^((m - mn) log2 e) + sum_e 2^(x[e] log2 e - mn log2 e);  m = mn
    Written so that no instruction needs a wait state: a comparison result is consumed three instructions later
    (three SGPR pairs in rotation), an exponential at the earliest two instructions later."""
    M, S, I = f"%[m{tb}]", f"%[s{tb}]", f"%[i{tb}]"
    for el in range(32):
        e(f"v_accvgpr_read_b32 {X[el]}, {acc_reg(el // 4, tb, el % 4)}")
    e(f"v_max3_f32 {ET}, {X[0]}, {X[1]}, {X[2]}")
    for j in range(14):
        e(f"v_max3_f32 {ET}, {ET}, {X[3 + 2 * j]}, {X[4 + 2 * j]}")
    e(f"v_max_f32 {ET}, {ET}, {X[31]}")
    # lowest element attaining the maximum: descending scan, a lower match overwrites a higher one
    e(f"v_mov_b32 {ESEL}, 0")
    order = list(range(31, -1, -1))
    pending = []
    for n, el in enumerate(order):
        mask = MASK[n % 3]
        e(f"v_cmp_eq_f32_e64 {mask}, {X[el]}, {ET}")
        pending.append((mask, el))
        if len(pending) == 3:
            mk, pe = pending.pop(0)
            e(f"v_cndmask_b32_e64 {ESEL}, {ESEL}, {pe}, {mk}")
    # two selects are still pending; the new-maximum test and the running maximum fill the wait states
    e(f"v_cmp_gt_f32 vcc, {ET}, {M}")                 # strict: an equal maximum in a later tile has a higher id
    e(f"v_max_f32 {EMN}, {M}, {ET}")
    for mk, pe in pending:
        e(f"v_cndmask_b32_e64 {ESEL}, {ESEL}, {pe}, {mk}")
    e(f"v_lshrrev_b32 {EY}, 2, {ESEL}")               # code = 16 * (sel / 4) + sel % 4
    e(f"v_and_b32 {ESEL}, 3, {ESEL}")
    e(f"v_lshl_add_u32 {ESEL}, {EY}, 4, {ESEL}")
    e(f"v_add_u32 {ESEL}, %[vb], {ESEL}")
    e(f"v_cndmask_b32 {I}, {I}, {ESEL}, vcc")
    # rescale of the running sum, the common exponent offset
    e(f"v_sub_f32 {EY}, {M}, {EMN}")
    e(f"v_mul_f32 {EY}, {hex(LOG2E)}, {EY}")
    e(f"v_exp_f32 {EY}, {EY}")
    e(f"v_mul_f32 {ENML}, {hex(NEG_LOG2E)}, {EMN}")
    e(f"v_mov_b32 {M}, {EMN}")
    for el in range(32):
        e(f"v_fmamk_f32 {X[el]}, {X[el]}, {hex(LOG2E)}, {ENML}")
    for el in range(32):
        e(f"v_exp_f32 {X[el]}, {X[el]}")
    for step in range(1, 8):                          # four running sums, elements r, r + 4, r + 8, ...
        for r in range(4):
            e(f"v_add_f32 {X[r]}, {X[r]}, {X[4 * step + r]}")
    e(f"v_add_f32 {X[0]}, {X[0]}, {X[1]}")
    e(f"v_add_f32 {X[2]}, {X[2]}, {X[3]}")
    e(f"v_add_f32 {X[0]}, {X[0]}, {X[2]}")
    e(f"v_fma_f32 {S}, {S}, {EY}, {X[0]}")


# ---- the sampling statement (Gumbel-max at temperature tau; noise from Philox4x32-10 keyed by seed, counter =
# (vocabulary id / 4, position, 0, 0), word id % 4).  Its big register blocks are named by number so that the
# reduction can reuse the fragment registers: v[112:239] fragments (the reduction's 32 logits alias the first 32),
# v[240:247] two generations of the generator's two 64-bit products, v[248:249] the per-column product, v[250:255]
# temporaries of the rare exact path.
FRAG_BASE = 112
PHILOX_M0, PHILOX_M1 = "%[pm0]", "%[pm1]"
KNEG = 0xF149F2CA          # -1.0e30f
TWO23_101 = 0x4B0147AE     # 2^23 * 1.01
TWO23 = 0x4B000000
NEG_LN2 = 0xBF317218
TWO_M23 = 0x34000000
TWO_M8 = 0x3B800000
THIRD = 0x3EAAAAAB
slow_blocks = []
# The reduction's temporaries live in fragment registers that are dead by then, the generator's round keys in scalar
# registers the statement fills itself from the seed: neither costs the register allocator anything.
SAMPLE_TEMPS = {name: f"v{FRAG_BASE + 32 + k}" for k, name in enumerate(
    ("et", "emn", "enml", "ey", "yt", "xsel", "sels", "wlo", "wm", "v4b", "v4q", "a0", "sw16", "sw32", "sw48", "pw", "px", "pe", "cnt", "nq"))}
KEY0_BASE, KEY1_BASE = 68, 78
SAMPLE_TEMPS.update({f"k0_{r}": f"s{KEY0_BASE + r}" for r in range(10)})
SAMPLE_TEMPS.update({f"k1_{r}": f"s{KEY1_BASE + r}" for r in range(10)})


def frag_names_literal():
    fa = [[f"v[{FRAG_BASE + (b * 16 + i) * 4}:{FRAG_BASE + (b * 16 + i) * 4 + 3}]" for i in range(8)] for b in range(2)]
    fb = [[f"v[{FRAG_BASE + (b * 16 + 8 + j) * 4}:{FRAG_BASE + (b * 16 + 8 + j) * 4 + 3}]" for j in range(8)]
          for b in range(2)]
    return fa, fb


def philox_quad(tb, bi, XS):
    """Words of the four ids vb + 16*bi .. +3 of column tb's position, and the jump to the exact path when one of
    them could still win.  Rounds 0 and 1 use what is known of the counter: (v4, position, 0, 0) makes the second
    product of round 0 vanish, and the first product of round 1 depends on the position alone (per column, in
    v[248:249], its high half already xored with the round key)."""
    A, B, C, D = ("v240", "v241"), ("v242", "v243"), ("v244", "v245"), ("v246", "v247")
    pair = lambda r: f"v[{r[0][1:]}:{r[1][1:]}]"
    e(f"v_add_u32 %[v4q], {4 * bi}, %[v4b]")
    e(f"v_mad_u64_u32 {pair(A)}, vcc, {PHILOX_M0}, %[v4q], 0")       # round 0: lo -> a3, hi
    e(f"v_xor_b32 {A[1]}, %[k1_0], {A[1]}")                          # a2 = hi ^ k1
    e(f"v_mad_u64_u32 {pair(B)}, vcc, {PHILOX_M1}, {A[1]}, 0")       # round 1, second product: lo -> b1, hi
    e(f"v_xor_b32 {B[1]}, %[k0_1], {B[1]}")                          # b0 = hi ^ k0   (a1 = 0)
    e(f"v_xor_b32 {A[1]}, v249, {A[0]}")                             # b2 = (hi(M0 a0) ^ k1) ^ a3
    c0, c1, c2, c3 = B[1], B[0], A[1], "v248"                        # b3 = lo(M0 a0)
    cur, nxt = (A, B), (C, D)
    for r in range(2, 10):
        PA, PB = nxt
        e(f"v_mad_u64_u32 {pair(PA)}, vcc, {PHILOX_M0}, {c0}, 0")
        e(f"v_mad_u64_u32 {pair(PB)}, vcc, {PHILOX_M1}, {c2}, 0")
        e(f"v_bitop3_b32 {PB[1]}, {PB[1]}, {c1}, %[k0_{r}] bitop3:0x96")     # truth table 0x96: a ^ b ^ c
        e(f"v_bitop3_b32 {PA[1]}, {PA[1]}, {c3}, %[k1_{r}] bitop3:0x96")
        c0, c1, c2, c3 = PB[1], PB[0], PA[1], PA[0]
        cur, nxt = nxt, cur
    words = [c0, c1, c2, c3]
    # a word below the column's bound cannot win: only 2^-23-sized tails of the uniform reach the running best
    e(f"v_max3_u32 %[wm], {words[0]}, {words[1]}, {words[2]}")
    e(f"v_max_u32 %[wm], %[wm], {words[3]}")
    e(f"v_cmp_ge_u32 vcc, %[wm], %[wlo]")
    slow, flush, back = label(f"slow{tb}{bi}"), label(f"flush{tb}{bi}"), label(f"back{tb}{bi}")
    e(f"s_cbranch_vccnz {slow}")
    e(f"{back}:")
    # Out of line: some lane holds a candidate.  Its word, logit and element go into the lane's one-deep queue, to be
    # scored once at the end of the column.  When a lane would queue a second one, the queues are scored and emptied
    # first; when that lane's two candidates are both of this quad, the quad's four ids are scored directly.
    M3, M2, M1, SINK = MASK[0], MASK[1], MASK[2], "s[66:67]"
    els = [bi * 4 + r for r in range(4)]
    queue, full = label(f"queue{tb}{bi}"), label(f"full{tb}{bi}")
    passes = [f"v_cmp_ge_u32_e64 {M3}, {words[3]}, %[wlo]",
              f"v_cmp_ge_u32_e64 {M2}, {words[2]}, %[wlo]",
              f"v_cmp_ge_u32_e64 {M1}, {words[1]}, %[wlo]"]
    blk = [f"{slow}:"] + passes + [
           f"v_cmp_ge_u32 vcc, {words[0]}, %[wlo]",
           f"v_addc_co_u32_e64 %[nq], {SINK}, 0, 0, {M3}",               # candidates of this quad, per lane
           f"v_addc_co_u32_e64 %[nq], {SINK}, 0, %[nq], {M2}",
           f"v_addc_co_u32_e64 %[nq], {SINK}, 0, %[nq], {M1}",
           f"v_addc_co_u32_e64 %[nq], {SINK}, 0, %[nq], vcc",
           f"v_add_u32 %[cnt], %[cnt], %[nq]",
           f"v_cmp_lt_u32 vcc, 1, %[cnt]",
           f"s_cbranch_vccnz {flush}",
           f"{queue}:",
           f"v_cmp_ge_u32 vcc, {words[0]}, %[wlo]"]
    for mk, r in ((M3, 3), (M2, 2), (M1, 1)):
        blk += [f"v_cndmask_b32_e64 %[pw], %[pw], {words[r]}, {mk}",
                f"v_cndmask_b32_e64 %[px], %[px], {XS[els[r]]}, {mk}",
                f"v_cndmask_b32_e64 %[pe], %[pe], {els[r]}, {mk}"]
    blk += [f"v_cndmask_b32 %[pw], %[pw], {words[0]}, vcc",
            f"v_cndmask_b32 %[px], %[px], {XS[els[0]]}, vcc",
            f"v_cndmask_b32_e64 %[pe], %[pe], {els[0]}, vcc",
            f"s_branch {back}",
            f"{flush}:"]
    blk += score_candidate("%[pw]", "%[px]", "%[pe]") + empty_queue()
    blk += [f"v_cmp_lt_u32 vcc, 1, %[nq]",
            f"s_cbranch_vccnz {full}"]
    blk += passes + ["v_mov_b32 %[cnt], %[nq]", f"s_branch {queue}", f"{full}:"]
    for r in range(3, -1, -1):
        blk += score_candidate(words[r], XS[els[r]], str(els[r]))
    blk.append(f"s_branch {back}")
    slow_blocks.append(blk)


def empty_queue():
    return ["v_mov_b32 %[cnt], 0", "v_mov_b32 %[pw], 0", f"v_mov_b32 %[px], {hex(KNEG)}", "v_mov_b32 %[pe], 0"]


def score_candidate(word, x, el):
    """y = x + tau * g(u) of one id per lane (u from the id's word, g = -ln(-ln u), next to u = 1 by the series of
    -ln(1 - e)), and the tile's best (score, element, logit) updated by it: a higher score wins, the lower element
    on equal scores."""
    M3, M2, M1 = MASK
    return [f"v_lshrrev_b32 v250, 9, {word}",                            # k
            f"v_sub_u32 v251, {hex(0x7FFFFF)}, v250",                    # 2^23 - 1 - k
            "v_cvt_f32_u32 v250, v250",
            "v_cvt_f32_u32 v251, v251",
            "v_add_f32 v250, 0.5, v250",
            "v_add_f32 v251, 0.5, v251",
            f"v_mul_f32 v250, {hex(TWO_M23)}, v250",                     # u
            f"v_mul_f32 v251, {hex(TWO_M23)}, v251",                     # e = 1 - u
            "v_log_f32 v252, v250",
            f"v_mul_f32 v253, {hex(THIRD)}, v251",                       # e (1 + e (1/2 + e/3)) = -ln(1 - e) near u = 1
            "v_add_f32 v253, 0.5, v253",
            f"v_mul_f32 v252, {hex(NEG_LN2)}, v252",                     # -ln u
            "v_mul_f32 v253, v251, v253",
            "v_add_f32 v253, 1.0, v253",
            f"v_cmp_gt_f32 vcc, {hex(TWO_M8)}, v251",
            "v_mul_f32 v253, v251, v253",
            "s_nop 0",
            "v_cndmask_b32 v252, v252, v253, vcc",                       # inner = e < 2^-8 ? series : by the logarithm
            "v_log_f32 v252, v252",
            "s_nop 0",
            f"v_mul_f32 v252, {hex(NEG_LN2)}, v252",                     # g = -ln(inner)
            "v_mul_f32 v252, %[tau], v252",
            f"v_add_f32 v252, {x}, v252",                                # y = x + tau g
            f"v_cmp_eq_f32_e64 {M2}, v252, %[yt]",
            f"v_cmp_gt_u32_e64 {M1}, %[sels], {el}",
            "v_cmp_gt_f32 vcc, v252, %[yt]",
            "s_nop 1",
            f"s_and_b64 {M2}, {M2}, {M1}",
            f"s_or_b64 vcc, vcc, {M2}",
            "s_nop 1",
            f"v_cndmask_b32_e64 %[sels], %[sels], {el}, vcc",
            f"v_cndmask_b32 %[xsel], %[xsel], {x}, vcc",
            "v_cndmask_b32 %[yt], %[yt], v252, vcc"]


def reduce_column_sample(tb):
    """Column tb of the finished tile under sampling: running (max, sum-exp) as in the greedy reduction, and the
    arg-max of x + tau*g with the plain logit there.  Exact: an id is skipped only when its uniform lies below what
    the best score seen so far minus the column's largest logit of this tile demands (1 - u < exp((t - ym) / tau),
    taken with a 1% margin), which no winner can."""
    M, S, I, YM, XA, POS = (f"%[m{tb}]", f"%[s{tb}]", f"%[i{tb}]", f"%[ym{tb}]", f"%[xa{tb}]", f"%[pos{tb}]")
    XS = [f"v{FRAG_BASE + i}" for i in range(32)]
    # the best score so far of the three other lanes that hold the same token (lane ^ 16, ^ 32, ^ 48): any score
    # already reached for the row bounds what can still win it
    e(f"ds_bpermute_b32 v253, %[sw16], {YM}")
    e(f"ds_bpermute_b32 v254, %[sw32], {YM}")
    e(f"ds_bpermute_b32 v255, %[sw48], {YM}")
    for el in range(32):
        e(f"v_accvgpr_read_b32 {XS[el]}, {acc_reg(el // 4, tb, el % 4)}")
    e(f"v_max3_f32 {ET}, {XS[0]}, {XS[1]}, {XS[2]}")
    for j in range(14):
        e(f"v_max3_f32 {ET}, {ET}, {XS[3 + 2 * j]}, {XS[4 + 2 * j]}")
    e(f"v_max_f32 {ET}, {ET}, {XS[31]}")
    # the bound on the words: candidates have (w >> 9) >= 2^23 - Z, Z = min(2^23, 1.01 * 2^23 * exp((t - ym)/tau) + 2)
    e("s_waitcnt lgkmcnt(0)")
    e(f"v_max3_f32 v253, v253, v254, v255")
    e(f"v_max_f32 v253, v253, {YM}")
    e(f"v_sub_f32 {EY}, {ET}, v253")
    e(f"v_mul_f32 {EY}, %[itl], {EY}")                               # log2(e) / tau
    e(f"v_exp_f32 {EY}, {EY}")
    e(f"v_xor_b32 %[a0], %[k0_0], {POS}")                            # round 0: a0 = position ^ k0
    e(f"v_mul_f32 {EY}, {hex(TWO23_101)}, {EY}")
    e(f"v_mad_u64_u32 v[248:249], vcc, {PHILOX_M0}, %[a0], 0")       # round 1, first product: position only
    e(f"v_add_f32 {EY}, 2.0, {EY}")
    e(f"v_min_f32 {EY}, {hex(TWO23)}, {EY}")
    e(f"v_cvt_u32_f32 %[wlo], {EY}")
    e(f"v_xor_b32 v249, %[k1_1], v249")
    e(f"v_sub_u32 %[wlo], {hex(0x800000)}, %[wlo]")
    e(f"v_lshlrev_b32 %[wlo], 9, %[wlo]")
    e(f"v_mov_b32 %[yt], {hex(KNEG)}")
    e("v_mov_b32 %[sels], 0")
    e(f"v_mov_b32 %[xsel], 0")
    for ln in empty_queue():
        e(ln)
    for bi in range(7, -1, -1):
        philox_quad(tb, bi, XS)
    empty = label(f"empty{tb}")
    e("v_cmp_ne_u32 vcc, 0, %[cnt]")                                 # what is left in the queues, if anything
    e(f"s_cbranch_vccz {empty}")
    for ln in score_candidate("%[pw]", "%[px]", "%[pe]"):
        e(ln)
    e(f"{empty}:")
    # the tile's best against the running best (strict: an equal score in a later tile has a higher id)
    e(f"v_cmp_gt_f32 vcc, %[yt], {YM}")
    e(f"v_lshrrev_b32 {EY}, 2, %[sels]")
    e(f"v_and_b32 %[sels], 3, %[sels]")
    e(f"v_lshl_add_u32 %[sels], {EY}, 4, %[sels]")
    e(f"v_add_u32 %[sels], %[vb], %[sels]")
    e(f"v_cndmask_b32 {I}, {I}, %[sels], vcc")
    e(f"v_cndmask_b32 {XA}, {XA}, %[xsel], vcc")
    e(f"v_cndmask_b32 {YM}, {YM}, %[yt], vcc")
    # running maximum and sum of exponentials of the unperturbed logits
    e(f"v_max_f32 {EMN}, {M}, {ET}")
    e(f"v_sub_f32 {EY}, {M}, {EMN}")
    e(f"v_mul_f32 {EY}, {hex(LOG2E)}, {EY}")
    e(f"v_exp_f32 {EY}, {EY}")
    e(f"v_mul_f32 {ENML}, {hex(NEG_LOG2E)}, {EMN}")
    e(f"v_mov_b32 {M}, {EMN}")
    for el in range(32):
        e(f"v_fmamk_f32 {XS[el]}, {XS[el]}, {hex(LOG2E)}, {ENML}")
    for el in range(32):
        e(f"v_exp_f32 {XS[el]}, {XS[el]}")
    for step in range(1, 8):
        for r in range(4):
            e(f"v_add_f32 {XS[r]}, {XS[r]}, {XS[4 * step + r]}")
    e(f"v_add_f32 {XS[0]}, {XS[0]}, {XS[1]}")
    e(f"v_add_f32 {XS[2]}, {XS[2]}, {XS[3]}")
    e(f"v_add_f32 {XS[0]}, {XS[0]}, {XS[2]}")
    e(f"v_fma_f32 {S}, {S}, {EY}, {XS[0]}")


def build_tile_sample():
    """The statement of the sampling kernel: K-loop on fragments and accumulators named by number, then the
    reduction with the noise; the rare exact paths sit behind the end of the statement."""
    saved = ([row[:] for row in FA], [row[:] for row in FB])
    fa, fb = frag_names_literal()
    for b in range(2):
        FA[b][:], FB[b][:] = fa[b], fb[b]
    LITERAL_ACC[0] = True
    slow_blocks.clear()
    build()
    e(f"s_mov_b32 %[k0_0], %[seed_lo]")                              # key of round r = seed + r * (golden-ratio words)
    e(f"s_mov_b32 %[k1_0], %[seed_hi]")
    for r in range(1, 10):
        e(f"s_add_u32 %[k0_{r}], %[k0_{r - 1}], 0x9e3779b9")
        e(f"s_add_u32 %[k1_{r}], %[k1_{r - 1}], 0xbb67ae85")
    e("v_lshrrev_b32 %[v4b], 2, %[vb]")
    e("v_mbcnt_lo_u32_b32 %[sw16], -1, 0")                           # lane id, then the byte addresses of the lanes
    e("v_mbcnt_hi_u32_b32 %[sw16], -1, %[sw16]")                     # ^ 16, ^ 32, ^ 48 for the cross-lane reads
    e("v_xor_b32 %[sw32], 32, %[sw16]")
    e("v_xor_b32 %[sw48], 48, %[sw16]")
    e("v_xor_b32 %[sw16], 16, %[sw16]")
    e("v_lshlrev_b32 %[sw32], 2, %[sw32]")
    e("v_lshlrev_b32 %[sw48], 2, %[sw48]")
    e("v_lshlrev_b32 %[sw16], 2, %[sw16]")
    for tb in range(8):
        reduce_column_sample(tb)
    done = label("done")
    e(f"s_branch {done}")
    for blk in slow_blocks:
        for ln in blk:
            e(ln)
    e(f"{done}:")
    LITERAL_ACC[0] = False
    for b in range(2):
        FA[b][:], FB[b][:] = saved[0][b], saved[1][b]
    named = re.compile(r"%\[(\w+)\]")
    lines[:] = [named.sub(lambda m: SAMPLE_TEMPS.get(m.group(1), m.group(0)), ln) for ln in lines]


def build_tile():
    """The statement of the greedy kernel: the K-loop on accumulators it starts itself, then the reduction of the
    tile."""
    LITERAL_ACC[0] = True
    build()
    for tb in range(8):
        reduce_column(tb)
    LITERAL_ACC[0] = False


def build():
    # entry: pointers into fixed SGPR pairs, first fragments of the current step
    e("s_mov_b32 s96, %[wsrc_lo]")
    e("s_mov_b32 s97, %[wsrc_hi]")
    e("s_mov_b32 s98, %[hsrc_lo]")
    e("s_mov_b32 s99, %[hsrc_hi]")
    e(f"s_add_u32 {NK128}, %[hwrap], 128")      # nk * 128
    e(f"s_mov_b32 {KT}, 0")
    read_addr(0)
    for r in reads(0):
        e(r)
    if LITERAL_ACC[0]:
        # the statement owns the accumulators: clear them while the first fragments are on their way (measured:
        # writing a tile's first products without an addend instead saves nothing)
        for i in range(256):
            e(f"v_accvgpr_write_b32 a{i}, 0")
    e("s_nop 7")
    top, steady, generic, out = label("top"), label("steady"), label("generic"), label("out")
    e(f"{top}:")
    # Steady state (1 <= g and g + 2 < total): every copy and the sync happen, no branch inside the body, one taken
    # branch per step (the back edge, issued right behind the last MFMA).
    cond_g_ge1_and(2)
    e(f"s_cbranch_scc0 {generic}")
    read_addr(1)
    e(f"{steady}:")
    leave = label("leave")
    e("s_waitcnt lgkmcnt(0)")
    scheduled_group(0, steady_fill(0))                       # LM-head tile g+2 goes out
    e("s_waitcnt vmcnt(8) lgkmcnt(0)")                       # all copies but the LM-head tile just issued; fragments
    e("s_barrier")
    scheduled_group(1, steady_fill(1))                       # hidden tile g+2 goes out
    e(f"s_cbranch_scc1 {steady}")
    e(f"{leave}:")
    e(f"s_cmp_lt_u32 {KT}, %[nk]")
    e(f"s_cbranch_scc0 {out}")
    # First step and the last two: same schedule with every part guarded.
    e(f"{generic}:")
    read_addr(1)
    group(0, rd=reads(1), dma=[dma_w(i) for i in range(8)], cond=lambda: cond_g_ge1_and(2), after=advance_w, pos=COPY_POS)
    nosync, stepend = label("nosync"), label("stepend")
    cond_plus(1)
    e(f"s_cbranch_scc0 {nosync}")
    e("s_waitcnt lgkmcnt(0)")
    e("s_waitcnt vmcnt(0)")       # outside the steady state no copy younger than step g+1 needs to stay in flight
    e("s_barrier")
    rotate_read_slots()
    read_addr(0)
    group(1, rd=reads(0), dma=[dma_h(i) for i in range(8)], cond=lambda: cond_plus(2), after=advance_h, pos=COPY_POS)
    e(f"s_branch {stepend}")
    e(f"{nosync}:")
    group(1)
    e(f"{stepend}:")
    step_end(top)
    e(f"{out}:")
    # exit: no fragment read may still be in flight, results visible to the VALU, pointers back to the operands
    e("s_waitcnt lgkmcnt(0)")
    e("s_nop 15")
    e("s_nop 15")
    e("s_mov_b32 %[wsrc_lo], s96")
    e("s_mov_b32 %[wsrc_hi], s97")
    e("s_mov_b32 %[hsrc_lo], s98")
    e("s_mov_b32 %[hsrc_hi], s99")


def write_statement(path, sample=False):
    lines.clear()
    uid[0] = 2000 if sample else 1000
    if sample:
        build_tile_sample()
        outs = []
        for tb in range(8):
            outs += [f'[m{tb}] "+v"(run_m[{tb}])', f'[s{tb}] "+v"(run_s[{tb}])', f'[i{tb}] "+v"(run_i[{tb}])',
                     f'[ym{tb}] "+v"(run_ym[{tb}])', f'[xa{tb}] "+v"(run_xa[{tb}])']
    else:
        build_tile()
        outs = []
        for tb in range(8):
            outs += [f'[m{tb}] "+v"(run_m[{tb}])', f'[s{tb}] "+v"(run_s[{tb}])', f'[i{tb}] "+v"(run_i[{tb}])']
        outs += [f'[x{i}] "=&v"(red_x[{i}])' for i in range(32)]
        outs += ['[et] "=&v"(red_t)', '[emn] "=&v"(red_mn)', '[enml] "=&v"(red_nml)', '[esel] "=&v"(red_sel)',
                 '[ey] "=&v"(red_y)']
    for name in ("wsrc_lo", "wsrc_hi", "hsrc_lo", "hsrc_hi", "wrd", "hrd", "wdst", "hdst", "wk", "hk", "g"):
        outs.append(f'[{name}] "+s"(st_{name})')
    if not sample:
        for b in range(2):
            for i in range(8):
                outs.append(f'[fa{b}{i}] "=&v"(frag_a[{b}][{i}])')
            for j in range(8):
                outs.append(f'[fb{b}{j}] "=&v"(frag_b[{b}][{j}])')
    outs.append('[vt0] "=&v"(addr_tmp0)')
    outs.append('[vt1] "=&v"(addr_tmp1)')
    ins = []
    for k in range(2):
        ins.append(f'[rdw{k}] "v"(rdw[{k}])')
    for k in range(2):
        ins.append(f'[rdh{k}] "v"(rdh[{k}])')
    for i in range(8):
        ins.append(f'[woff{i}] "v"(woff[{i}])')
    for i in range(8):
        ins.append(f'[hoff{i}] "v"(hoff[{i}])')
    for name in ("total", "nk", "wwrap", "hwrap"):
        ins.append(f'[{name}] "s"(st_{name})')
    clob = ['"s94"', '"s95"', '"s96"', '"s97"', '"s98"', '"s99"', '"vcc"', '"scc"', '"m0"', '"memory"']
    ins.append('[vb] "v"(vb)')
    clob = [f'"a{i}"' for i in range(256)] + [f'"s{i}"' for i in range(88, 94)] + clob
    if sample:
        ins += [f'[pos{tb}] "v"(pos[{tb}])' for tb in range(8)]
        ins += ['[seed_lo] "s"(seed_lo)', '[seed_hi] "s"(seed_hi)']
        clob = [f'"s{i}"' for i in range(66, KEY1_BASE + 10)] + clob
        ins += ['[pm0] "s"(philox_m0)', '[pm1] "s"(philox_m1)', '[itl] "s"(inv_tau_log2e)', '[tau] "s"(tau_s)']
        clob = [f'"v{i}"' for i in range(FRAG_BASE, 256)] + clob
    with open(path, "w") as f:
        f.write("// GENERATED by gen_w4_loop.py -- do not edit.  " +
                ("One vocabulary tile of the sampling 4-wave kernel: K-loop and vocabulary reduction.\n" if sample else
                 "One vocabulary tile of the greedy 4-wave kernel: K-loop and vocabulary reduction.\n"))
        f.write("asm volatile(\n")
        for ln in lines:
            f.write(f'    "{ln}\\n"\n')
        f.write("    : " + ",\n      ".join(outs) + "\n")
        f.write("    : " + ",\n      ".join(ins) + "\n")
        f.write("    : " + ", ".join(clob) + ");\n")
    print(f"{path}: {len(lines)} asm lines, {len(outs) + len(ins)} operands")


def main(folder):
    write_statement(os.path.join(folder, "mosaic_w4_tile.inc"))
    write_statement(os.path.join(folder, "mosaic_w4_tile_sample.inc"), sample=True)
    lines.clear()
    build()          # leave the bare K-loop listing (accumulators as operands) in `lines` for importers


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else os.path.dirname(os.path.abspath(__file__)))
