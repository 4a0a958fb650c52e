"""The vocabulary reductions inside the 4-wave kernel's statements (generated assembly), interpreted on the CPU with
numpy -- vector registers as arrays over lanes, scalar compares and branches taken per wave -- and compared with the
plain definition of what they stand for: the running (max, sum-exp, arg-max) update of the greedy kernel, and, for
the sampling kernel, the Gumbel-max draw on Philox noise (the uniforms come from the CPU oracle's generator, itself
pinned by the published known-answer vectors).  Also checked, because the assembler inserts no wait states: a
comparison result (SGPR pair or VCC) is read as a select mask no sooner than three instructions later, by a scalar
instruction no sooner than two later, and the result of a transcendental by an ordinary vector instruction no sooner
than two later; and that skipping ids whose uniform cannot win never changes the outcome.  No GPU."""
import importlib.util
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GEN = os.path.join(ROOT, "paper_2601_06562_amd", "csrc", "gen_w4_loop.py")
M32 = np.uint64(0xFFFFFFFF)


def tile_listing(sample=False):
    spec = importlib.util.spec_from_file_location("gen_w4_loop", GEN)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.lines.clear()
    mod.build_tile_sample() if sample else mod.build_tile()
    out = [ln.strip() for ln in mod.lines]
    mod.lines.clear()
    TEMPS.update(mod.SAMPLE_TEMPS)
    return out


TEMPS = {}       # the sampling statement's numbered registers by role (filled when its listing is generated)


def f32(bits):
    return np.array([bits], dtype=np.uint32).view(np.float32)[0]


class Wave:
    """Registers as raw 32-bit patterns, one numpy array of `n` lanes per vector register (scalar operands are
    broadcast arrays); SGPR pairs and VCC written by vector compares are per-lane masks."""
    TRANS = ("v_exp_f32", "v_log_f32")

    def __init__(self, n, agpr):
        self.n = n
        self.reg = {}
        self.mask = {}
        self.agpr = agpr                   # float32[256, n]
        self.mask_written = {}             # mask name -> issue index of the compare
        self.trans_written = {}            # register -> issue index of the transcendental
        self.accvgpr_reads = []
        self.issued = 0
        self.scc = 0
        self.slow_taken = self.quads = self.flushes = self.fulls = 0
        self.pending_lds = set()           # results of cross-lane reads not yet waited for

    # ---- operands
    def fget(self, tok):
        tok = tok.strip()
        if tok.startswith("0x"):
            return np.full(self.n, f32(int(tok, 16)), np.float32)
        if re.fullmatch(r"-?\d+\.\d+", tok):
            return np.full(self.n, np.float32(float(tok)), np.float32)
        return self.reg[tok].view(np.float32)

    def iget(self, tok):
        tok = tok.strip()
        if re.fullmatch(r"-?\d+", tok):
            return np.full(self.n, int(tok) & 0xFFFFFFFF, np.uint32)
        if tok.startswith("0x"):
            return np.full(self.n, int(tok, 16), np.uint32)
        return self.reg[tok]

    def fset(self, tok, v):
        self.reg[tok.strip()] = np.asarray(v, np.float32).view(np.uint32).copy()

    def iset(self, tok, v):
        self.reg[tok.strip()] = (np.asarray(v).astype(np.uint64) & M32).astype(np.uint32)

    # ---- one instruction
    def step(self, ins):
        op, _, rest = ins.partition(" ")
        a = [x.strip() for x in rest.split(",")]
        now = self.issued
        self.issued += 1
        trans = op in self.TRANS
        if op.startswith("v_"):
            for src in a[2:] if op in ("v_addc_co_u32_e64", "v_mad_u64_u32") else a[1:]:   # a[1]: the carry-out
                assert src not in self.pending_lds, f"{ins}: {src} read before the wait for the cross-lane read"
                if src in self.mask_written and op.startswith(("v_cndmask", "v_addc")):
                    assert now - self.mask_written[src] >= 3, f"{ins}: mask {src} read too soon after its comparison"
                if src in self.trans_written and not trans:
                    assert now - self.trans_written[src] >= 2, f"{ins}: {src} read too soon after the transcendental"
        if op == "v_cndmask_b32":                         # VOP2 form reads vcc implicitly
            assert now - self.mask_written.get("vcc", -9) >= 3, f"{ins}: vcc read too soon"
        f64 = lambda t: self.fget(t).astype(np.float64)
        if op == "v_accvgpr_read_b32":
            idx = int(a[1][1:])
            self.fset(a[0], self.agpr[idx])
            self.accvgpr_reads.append(idx)
        elif op == "v_max3_f32":
            self.fset(a[0], np.maximum(np.maximum(self.fget(a[1]), self.fget(a[2])), self.fget(a[3])))
        elif op == "v_max_f32":
            self.fset(a[0], np.maximum(self.fget(a[1]), self.fget(a[2])))
        elif op == "v_min_f32":
            self.fset(a[0], np.minimum(self.fget(a[1]), self.fget(a[2])))
        elif op == "v_mov_b32":
            self.iset(a[0], self.iget(a[1]))
        elif op in ("v_cmp_eq_f32_e64", "v_cmp_gt_f32", "v_cmp_ge_f32"):
            x, y = self.fget(a[1]), self.fget(a[2])
            self.mask[a[0]] = {"eq": x == y, "gt": x > y, "ge": x >= y}[op[6:8]]
            self.mask_written[a[0]] = now
        elif op in ("v_cmp_ge_u32", "v_cmp_ge_u32_e64", "v_cmp_lt_u32", "v_cmp_gt_u32_e64", "v_cmp_ne_u32"):
            x, y = self.iget(a[1]), self.iget(a[2])
            self.mask[a[0]] = {"ge": x >= y, "lt": x < y, "gt": x > y, "ne": x != y}[op[6:8]]
            self.mask_written[a[0]] = now
        elif op == "v_addc_co_u32_e64":                       # d = s0 + s1 + carry-in; the carry-out goes to a[1]
            total = self.iget(a[2]).astype(np.uint64) + self.iget(a[3]) + self.mask[a[4]]
            self.iset(a[0], total)
            self.mask[a[1]] = total >> np.uint64(32) != 0
            self.mask_written[a[1]] = now
        elif op in ("s_and_b64", "s_or_b64"):
            for src in a[1:]:
                assert now - self.mask_written.get(src, -9) >= 2, f"{ins}: scalar read right behind the vector compare"
            x, y = self.mask[a[1]], self.mask[a[2]]
            self.mask[a[0]] = (x & y) if op == "s_and_b64" else (x | y)
            self.mask_written.pop(a[0], None)                 # written by the scalar unit: no wait states owed
        elif op == "v_cndmask_b32_e64":
            self.iset(a[0], np.where(self.mask[a[3]], self.iget(a[2]), self.iget(a[1])))
        elif op == "v_cndmask_b32":
            assert a[3] == "vcc"
            self.iset(a[0], np.where(self.mask["vcc"], self.iget(a[2]), self.iget(a[1])))
        elif op == "v_lshrrev_b32":
            self.iset(a[0], self.iget(a[2]) >> self.iget(a[1]))
        elif op == "v_lshlrev_b32":
            self.iset(a[0], self.iget(a[2]).astype(np.uint64) << self.iget(a[1]).astype(np.uint64))
        elif op == "v_and_b32":
            self.iset(a[0], self.iget(a[1]) & self.iget(a[2]))
        elif op == "v_xor_b32":
            self.iset(a[0], self.iget(a[1]) ^ self.iget(a[2]))
        elif op == "v_bitop3_b32":                            # bit k of the table: k = 4*a + 2*b + c
            last, _, table = a[3].partition(" bitop3:")
            x, y, z = self.iget(a[1]), self.iget(a[2]), self.iget(last)
            out = np.zeros(self.n, np.uint32)
            for k in range(8):
                if int(table, 16) >> k & 1:
                    out |= (x if k & 4 else ~x) & (y if k & 2 else ~y) & (z if k & 1 else ~z)
            self.iset(a[0], out)
        elif op == "v_lshl_add_u32":
            self.iset(a[0], (self.iget(a[1]).astype(np.uint64) << self.iget(a[2]).astype(np.uint64)) + self.iget(a[3]))
        elif op == "v_add_u32":
            self.iset(a[0], self.iget(a[1]).astype(np.uint64) + self.iget(a[2]))
        elif op == "v_sub_u32":
            self.iset(a[0], self.iget(a[1]).astype(np.int64) - self.iget(a[2]).astype(np.int64))
        elif op == "v_max3_u32":
            self.iset(a[0], np.maximum(np.maximum(self.iget(a[1]), self.iget(a[2])), self.iget(a[3])))
        elif op == "v_max_u32":
            self.iset(a[0], np.maximum(self.iget(a[1]), self.iget(a[2])))
        elif op == "v_mad_u64_u32":
            lo, hi = re.fullmatch(r"v\[(\d+):(\d+)\]", a[0]).groups()
            assert int(hi) == int(lo) + 1 and a[1] == "vcc" and a[4] == "0"
            prod = self.iget(a[2]).astype(np.uint64) * self.iget(a[3]).astype(np.uint64)
            self.iset(f"v{lo}", prod & M32)
            self.iset(f"v{hi}", prod >> np.uint64(32))
            self.mask.pop("vcc", None)                        # the carry-out overwrites vcc
            self.mask_written.pop("vcc", None)
        elif op == "v_cvt_u32_f32":
            x = np.nan_to_num(np.trunc(f64(a[1])), nan=0.0, posinf=2.0 ** 32 - 1, neginf=0.0)
            self.iset(a[0], np.clip(x, 0, 2.0 ** 32 - 1))
        elif op == "v_cvt_f32_u32":
            self.fset(a[0], self.iget(a[1]).astype(np.float32))
        elif op == "v_sub_f32":
            with np.errstate(over="ignore"):
                self.fset(a[0], self.fget(a[1]) - self.fget(a[2]))
        elif op == "v_mul_f32":
            with np.errstate(over="ignore"):
                self.fset(a[0], self.fget(a[1]) * self.fget(a[2]))
        elif op == "v_add_f32":
            with np.errstate(over="ignore"):
                self.fset(a[0], self.fget(a[1]) + self.fget(a[2]))
        elif op == "v_exp_f32":
            with np.errstate(over="ignore"):
                self.fset(a[0], np.exp2(f64(a[1])).astype(np.float32))
        elif op == "v_log_f32":
            with np.errstate(divide="ignore", invalid="ignore"):
                self.fset(a[0], np.log2(f64(a[1])).astype(np.float32))
        elif op in ("v_fmamk_f32", "v_fma_f32"):              # d = s0 * s1 + s2, one rounding
            with np.errstate(over="ignore", invalid="ignore"):
                self.fset(a[0], (f64(a[1]) * f64(a[2]) + f64(a[3])).astype(np.float32))
        elif op == "s_mov_b32":
            self.iset(a[0], self.iget(a[1]))
        elif op == "s_add_u32":
            self.iset(a[0], self.iget(a[1]).astype(np.uint64) + self.iget(a[2]))
        elif op == "s_nop":
            self.issued += int(a[0])                          # s_nop n stands for n + 1 issue slots
        elif op == "s_waitcnt":
            assert rest.strip() == "lgkmcnt(0)"
            self.pending_lds.clear()
        elif op in ("v_mbcnt_lo_u32_b32", "v_mbcnt_hi_u32_b32"):
            assert a[1] == "-1" and self.n == 64
            lane = np.arange(64)
            below = np.minimum(lane, 32) if op.endswith("lo_u32_b32") else np.maximum(lane - 32, 0)
            self.iset(a[0], below + self.iget(a[2]))
        elif op == "ds_bpermute_b32":                         # dst[lane] = src[addr[lane] / 4]
            self.iset(a[0], self.iget(a[2])[(self.iget(a[1]) >> 2) % self.n])
            self.pending_lds.add(a[0])
        else:
            raise AssertionError(f"instruction the interpreter does not know: {ins}")
        if op.startswith("v_") and not op.startswith("v_cmp"):
            if trans:
                self.trans_written[a[0]] = now
            else:
                self.trans_written.pop(a[0], None)

    def run(self, prog):
        labels = {ln[:-1]: i for i, ln in enumerate(prog) if ln.endswith(":")}
        pc, steps = 0, 0
        while pc < len(prog):
            ins = prog[pc]
            pc += 1
            steps += 1
            assert steps < 500000, "the listing does not terminate"
            if ins.endswith(":"):
                continue
            op, _, rest = ins.partition(" ")
            if op == "s_branch":
                pc = labels[rest.strip()]
                self.issued += 1
            elif op == "s_cbranch_vccz":                   # taken when no lane's compare held
                self.issued += 1
                if not self.mask["vcc"].any():
                    pc = labels[rest.strip()]
            elif op == "s_cbranch_vccnz":                  # taken when any lane's compare held (the hardware
                self.issued += 1                           # interlocks this read of vcc: no wait states owed)
                kind = rest.strip()[1:5]                   # slow: some lane has a candidate; flus(h): some lane's
                self.quads += kind == "slow"               # queue is full; full: two candidates of one quad
                if self.mask["vcc"].any():
                    self.slow_taken += kind == "slow"
                    self.flushes += kind == "flus"
                    self.fulls += kind == "full"
                    pc = labels[rest.strip()]
            else:
                self.step(ins)


def split_reduction(prog):
    first = next(i for i, ln in enumerate(prog) if ln.startswith(("v_accvgpr_read_b32", "s_mov_b32 s68, %[seed_lo]")))
    assert all(not ln.startswith("v_mfma") for ln in prog[first:])
    assert prog[first - 4:first] == ["s_mov_b32 %[wsrc_lo], s96", "s_mov_b32 %[wsrc_hi], s97",
                                     "s_mov_b32 %[hsrc_lo], s98", "s_mov_b32 %[hsrc_hi], s99"]
    # the tile is complete and visible before it is read: every fragment read waited for, 32 idle issue slots
    assert prog[first - 7:first - 4] == ["s_waitcnt lgkmcnt(0)", "s_nop 15", "s_nop 15"]
    return prog[first:]


def column_logits(agpr, tb):
    """[32, n]: element e of column tb = block (e / 4, tb), register e % 4, i.e. vocabulary id vb + 16*(e/4) + e%4."""
    return np.stack([agpr[((e // 4) * 8 + tb) * 4 + e % 4] for e in range(32)])


@pytest.fixture(scope="module")
def greedy():
    prog = tile_listing()
    return prog, split_reduction(prog)


@pytest.mark.parametrize("sample", [False, True])
def test_statement_addresses_the_accumulators_by_number_and_clears_them_itself(sample):
    """Every MFMA accumulates into an aligned block of four AGPRs named by number, and the statement clears all 256
    registers before its first MFMA (the K-loop checker proves it for every path through the listing)."""
    prog = tile_listing(sample)
    clears = [i for i, ln in enumerate(prog) if ln.startswith("v_accvgpr_write_b32")]
    assert [prog[i] for i in clears] == [f"v_accvgpr_write_b32 a{i}, 0" for i in range(256)]
    assert clears[-1] < next(i for i, ln in enumerate(prog) if ln.startswith("v_mfma"))
    blocks = set()
    for ln in prog:
        if ln.startswith("v_mfma"):
            dst, _, _, src_c = [x.strip() for x in ln.split(" ", 1)[1].split(",")]
            assert src_c == dst and re.fullmatch(r"a\[\d+:\d+\]", dst)
            lo, hi = map(int, dst[2:-1].split(":"))
            assert lo % 4 == 0 and hi == lo + 3
            blocks.add(lo // 4)
    assert blocks == set(range(64))


def planted_tile(rng, n):
    agpr = (rng.standard_normal((256, n)) * 3).astype(np.float32)
    for lane in range(0, n, 7):                            # exact ties: the lowest element must win
        col, e1, e2 = rng.integers(8), rng.integers(32), rng.integers(32)
        top = np.float32(20 + lane % 5)
        agpr[((e1 // 4) * 8 + col) * 4 + e1 % 4, lane] = top
        agpr[((e2 // 4) * 8 + col) * 4 + e2 % 4, lane] = top
    return agpr


def running_state(rng, agpr, n):
    m0 = (rng.standard_normal((8, n)) * 3).astype(np.float32)
    m0[:, :n // 12] = -1.0e30                              # fresh columns
    m0[3, n // 5:n // 4] = 50.0                            # a running maximum far above the tile
    s0 = (1 + rng.random((8, n)) * 100).astype(np.float32)
    s0[:, :n // 12] = 0.0
    for lane in range(5, n, 11):                           # running maximum equal to the tile's: no update (strict)
        m0[2, lane] = column_logits(agpr, 2)[:, lane].max()
    return m0, s0


def check_max_and_sum(w, agpr, m0, s0):
    for tb in range(8):
        x = column_logits(agpr, tb)
        mn = np.maximum(m0[tb], x.max(axis=0))
        x64, mn64 = x.astype(np.float64), mn.astype(np.float64)
        with np.errstate(over="ignore"):
            want_s = s0[tb].astype(np.float64) * np.exp(m0[tb].astype(np.float64) - mn64) + np.exp(x64 - mn64).sum(axis=0)
        got_s = w.fget(f"%[s{tb}]").astype(np.float64)
        assert np.array_equal(w.fget(f"%[m{tb}]"), mn), tb
        assert np.all(np.abs(got_s - want_s) <= 2e-6 * want_s + 1e-30), (tb, np.abs(got_s / want_s - 1).max())


@pytest.mark.parametrize("seed", range(4))
def test_greedy_reduction_equals_the_running_update_it_stands_for(greedy, seed):
    _, red = greedy
    rng = np.random.default_rng(seed)
    n = 512
    agpr = planted_tile(rng, n)
    m0, s0 = running_state(rng, agpr, n)
    i0 = rng.integers(0, 100000, (8, n)).astype(np.uint32)
    vb = (rng.integers(0, 400, n) * 256 + rng.integers(0, 2, n) * 128 + 4 * rng.integers(0, 4, n)).astype(np.uint32)
    w = Wave(n, agpr)
    for tb in range(8):
        w.fset(f"%[m{tb}]", m0[tb])
        w.fset(f"%[s{tb}]", s0[tb])
        w.iset(f"%[i{tb}]", i0[tb])
    w.iset("%[vb]", vb)
    w.run(red)
    assert sorted(w.accvgpr_reads) == list(range(256))        # every accumulator is read exactly once
    check_max_and_sum(w, agpr, m0, s0)
    for tb in range(8):
        x = column_logits(agpr, tb)
        t = x.max(axis=0)
        sel = np.argmax(x == t, axis=0)                        # lowest element at the maximum
        want_i = np.where(t > m0[tb], vb + 16 * (sel // 4) + sel % 4, i0[tb])
        assert np.array_equal(w.iget(f"%[i{tb}]"), want_i.astype(np.uint32)), tb


def test_the_interpreter_catches_a_mask_read_too_soon(greedy):
    """Plant a mistake in a copy of the listing: a select moved right behind its comparison must trip the rule."""
    _, red = greedy
    broken = list(red)
    i = next(k for k, ln in enumerate(broken) if ln.startswith("v_cndmask_b32_e64"))
    mask = broken[i].split(",")[-1].strip()
    j = max(k for k in range(i) if broken[k].startswith("v_cmp_eq_f32_e64 " + mask))
    broken.insert(j + 1, broken.pop(i))
    w = Wave(4, np.zeros((256, 4), np.float32))
    for tb in range(8):
        w.fset(f"%[m{tb}]", np.zeros(4))
        w.fset(f"%[s{tb}]", np.zeros(4))
        w.iset(f"%[i{tb}]", np.zeros(4))
    w.iset("%[vb]", np.zeros(4))
    with pytest.raises(AssertionError):
        w.run(broken)


# ---------------------------------------------------------------- the sampling statement
@pytest.fixture(scope="module")
def sampling():
    return split_reduction(tile_listing(sample=True))


def sampling_wave(red, agpr, m0, s0, ym0, xa0, i0, pos, vb, seed, tau, force_exact=False, mutate=None):
    n = agpr.shape[1]
    prog = list(red) if mutate is None else mutate(list(red))
    if force_exact:      # every id takes the exact path: the bound on the words is dropped
        wlo = TEMPS["wlo"]
        hits = [k for k, ln in enumerate(prog) if ln == f"v_lshlrev_b32 {wlo}, 9, {wlo}"]
        assert len(hits) == 8
        for k in hits:
            prog[k] = f"v_mov_b32 {wlo}, 0"
    w = Wave(n, agpr)
    for tb in range(8):
        w.fset(f"%[m{tb}]", m0[tb])
        w.fset(f"%[s{tb}]", s0[tb])
        w.iset(f"%[i{tb}]", i0[tb])
        w.fset(f"%[ym{tb}]", ym0[tb])
        w.fset(f"%[xa{tb}]", xa0[tb])
        w.iset(f"%[pos{tb}]", pos[tb])
    w.iset("%[vb]", vb)
    w.iset("%[seed_lo]", np.full(n, seed & 0xFFFFFFFF, np.uint64))
    w.iset("%[seed_hi]", np.full(n, seed >> 32, np.uint64))
    w.iset("%[pm0]", np.full(n, 0xD2511F53, np.uint64))
    w.iset("%[pm1]", np.full(n, 0xCD9E8D57, np.uint64))
    w.fset("%[itl]", np.full(n, np.float32(1.4426950408889634) / np.float32(tau), np.float32))
    w.fset("%[tau]", np.full(n, tau, np.float32))
    w.run(prog)
    return w


def token_level(w, tb, i0=None):
    """The four lanes l, l ^ 16, l ^ 32, l ^ 48 hold ids of the same token: its best is the highest score among
    them, the lowest id on equal scores (what the kernel's merge does next).  Returns (score, id, logit) per token."""
    ym, xa, ii = w.fget(f"%[ym{tb}]"), w.fget(f"%[xa{tb}]"), w.iget(f"%[i{tb}]").astype(np.int64)
    out = []
    for t in range(16):
        lanes = [t, t + 16, t + 32, t + 48]
        best = max(lanes, key=lambda l: (ym[l], -ii[l]))
        out.append((ym[best], int(ii[best]), xa[best]))
    return out


@pytest.mark.parametrize("tau", [1.0, 0.4])
def test_sampling_reduction_draws_what_the_oracle_draws_and_skips_only_losers(sampling, tau):
    import oracle
    rng = np.random.default_rng(int(tau * 10))
    n, seed = 64, 0x1234_5678_9ABC_DEF0
    agpr = planted_tile(rng, n)
    lane = np.arange(n, dtype=np.uint32)
    vb = np.full(n, 37 * 256 + 128, np.uint32) + 4 * (lane >> 4)          # as the kernel's lanes: 4 ids per quarter
    pos = [rng.integers(0, 131072, 16).astype(np.uint32)[lane % 16] for _ in range(8)]   # one token per lane % 16
    m0, s0 = running_state(rng, agpr, n)
    i0 = (200000 + rng.permutation(8 * n).reshape(8, n)).astype(np.uint32)             # distinct ids, above the tile's
    xa0 = rng.standard_normal((8, n)).astype(np.float32)
    # the best score so far: fresh on some tokens (everything is a candidate), typical on most (ln V + a few), and
    # unbeatable on others
    ym0 = (11.0 * tau + rng.random((8, n)) * 3).astype(np.float32)
    ym0[:, lane % 16 < 3] = -1.0e30
    ym0[:, 60:] = 1.0e4                                                  # tokens 12..15: one of their lanes holds it
    fast = sampling_wave(sampling, agpr, m0, s0, ym0, xa0, i0, pos, vb, seed, tau)
    exact = sampling_wave(sampling, agpr, m0, s0, ym0, xa0, i0, pos, vb, seed, tau, force_exact=True)
    assert fast.quads == exact.quads == 64 and exact.slow_taken == exact.flushes == exact.fulls == 64
    assert sorted(fast.accvgpr_reads) == list(range(256))
    check_max_and_sum(fast, agpr, m0, s0)
    for tb in range(8):
        for name in ("m", "s"):
            assert np.array_equal(fast.reg[f"%[{name}{tb}]"], exact.reg[f"%[{name}{tb}]"]), (name, tb)
    clear = total = 0
    for tb in range(8):
        # skipping never changes what the token draws
        assert token_level(fast, tb) == token_level(exact, tb), tb
        # ... and the draw is the oracle's: arg-max of x + tau * g over the token's 128 ids, against the best so far
        x = column_logits(agpr, tb).astype(np.float64)
        got = token_level(fast, tb)
        for t in range(16):
            lanes = [t, t + 16, t + 32, t + 48]
            cands = [(float(ym0[tb, l]), int(i0[tb, l]), float(xa0[tb, l])) for l in lanes]
            for l in lanes:
                for el in range(32):
                    v = int(vb[l]) + 16 * (el // 4) + el % 4
                    cands.append((x[el, l] + tau * oracle.gumbel(seed, int(pos[tb][l]), v), v, x[el, l]))
            cands.sort(key=lambda c: (-c[0], c[1]))
            total += 1
            if cands[0][0] - cands[1][0] < 1e-4:
                continue                                   # fp32 against fp64 may legitimately order these differently
            clear += 1
            assert got[t][1] == cands[0][1], (tb, t, got[t], cands[0])
            assert got[t][2] == np.float32(cands[0][2])
            assert abs(float(got[t][0]) - cands[0][0]) <= 1e-4 * (1 + abs(cands[0][0]))
    assert clear >= 0.95 * total
    # with benchmark-like logits (N(0,1): the best score so far sits near ln V while a tile's largest logit is ~3)
    # only a few of the 64 quads need the exact path
    flat = rng.standard_normal((256, n)).astype(np.float32)
    warm = sampling_wave(sampling, flat, m0, s0, np.full((8, n), 3.0 + 9.0 * tau, np.float32), xa0, i0, pos, vb, seed, tau)
    assert warm.slow_taken <= 8 and warm.flushes == 0, (warm.slow_taken, warm.flushes)
    # early in a split (best so far only a few above the tile's largest logit) most quads hold a candidate in some
    # lane, but a lane seldom holds two: the candidates wait in the queues and are scored once per column
    early = sampling_wave(sampling, flat, m0, s0, np.full((8, n), 3.0 + 5.0 * tau, np.float32), xa0, i0, pos, vb, seed, tau)
    assert early.slow_taken >= 24 and early.flushes <= early.slow_taken // 4 and early.fulls <= early.flushes // 2, \
        (early.slow_taken, early.flushes, early.fulls)


def test_a_queue_that_forgets_to_score_before_refilling_is_caught(sampling):
    """Planted mistake: the jump that scores a lane's queue before a second candidate is filed is dropped, so the second
    candidate overwrites the first.  With nothing bounding the scores (a fresh row: every id is a candidate) the
    draw must then differ from the exact one, which is what the comparison above relies on."""
    rng = np.random.default_rng(5)
    n, seed, tau = 64, 0xDEADBEEF12345678, 1.0
    agpr = planted_tile(rng, n)
    lane = np.arange(n, dtype=np.uint32)
    vb = np.full(n, 9 * 256, np.uint32) + 4 * (lane >> 4)
    pos = [rng.integers(0, 4096, 16).astype(np.uint32)[lane % 16] for _ in range(8)]
    m0, s0 = running_state(rng, agpr, n)
    i0 = (300000 + rng.permutation(8 * n).reshape(8, n)).astype(np.uint32)
    xa0 = rng.standard_normal((8, n)).astype(np.float32)
    ym0 = np.full((8, n), -1.0e30, np.float32)

    def drop_flush(prog):
        hits = [k for k, ln in enumerate(prog) if ln.startswith("s_cbranch_vccnz Lflush")]
        assert len(hits) == 64
        for k in hits:
            prog[k] = "s_nop 0"
        return prog
    good = sampling_wave(sampling, agpr, m0, s0, ym0, xa0, i0, pos, vb, seed, tau)
    exact = sampling_wave(sampling, agpr, m0, s0, ym0, xa0, i0, pos, vb, seed, tau, force_exact=True)
    bad = sampling_wave(sampling, agpr, m0, s0, ym0, xa0, i0, pos, vb, seed, tau, mutate=drop_flush)
    assert good.fulls == 64 and bad.fulls == 0
    assert all(token_level(good, tb) == token_level(exact, tb) for tb in range(8))
    assert sum(token_level(bad, tb) != token_level(exact, tb) for tb in range(8)) >= 6
