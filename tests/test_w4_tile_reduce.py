"""The vocabulary reduction inside the greedy 4-wave kernel's statement (generated assembly), interpreted on the CPU
with numpy, many lanes at once, and compared with the plain definition of the running (max, sum-exp, arg-max)
update; plus the two issue rules the listing must respect because the assembler does not insert wait states:
a comparison result (SGPR pair or VCC) is read as a select mask no sooner than three instructions later, and the
result of an exponential is read by an ordinary vector instruction no sooner than two instructions later.  No GPU."""
import importlib.util
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GEN = os.path.join(ROOT, "paper_2601_06562_amd", "csrc", "gen_w4_loop.py")
LOG2E = np.float32(1.4426950408889634)


def tile_listing():
    spec = importlib.util.spec_from_file_location("gen_w4_loop", GEN)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.lines.clear()
    mod.build_tile()
    out = [ln.strip() for ln in mod.lines]
    mod.lines.clear()
    return out


def f32(bits):
    return np.array([bits], dtype=np.uint32).view(np.float32)[0]


class Lanes:
    """Vector registers as numpy arrays over `n` independent lanes; values are kept as raw 32-bit patterns."""

    def __init__(self, n, agpr):
        self.n = n
        self.reg = {}                      # name -> uint32[n]
        self.mask = {}                     # SGPR pair / vcc -> bool[n]
        self.agpr = agpr                   # float32[256, n]
        self.last_mask_write = {}
        self.last_trans_write = {}
        self.accvgpr_reads = []

    def fget(self, tok):
        tok = tok.strip()
        if tok.startswith("0x"):
            return np.full(self.n, f32(int(tok, 16)), np.float32)
        return self.reg[tok].view(np.float32)

    def iget(self, tok):
        tok = tok.strip()
        if re.fullmatch(r"-?\d+", tok):
            return np.full(self.n, int(tok), np.uint32)
        if tok.startswith("0x"):
            return np.full(self.n, int(tok, 16), np.uint32)
        return self.reg[tok]

    def fset(self, tok, v):
        self.reg[tok.strip()] = np.asarray(v, np.float32).view(np.uint32).copy()

    def iset(self, tok, v):
        self.reg[tok.strip()] = np.asarray(v).astype(np.uint32)

    def run(self, prog):
        for pc, ins in enumerate(prog):
            op, _, rest = ins.partition(" ")
            a = [x.strip() for x in rest.split(",")]
            srcs = a[1:]
            trans = op == "v_exp_f32"
            for s_ in srcs:                                   # issue rules
                if s_ in self.last_mask_write and op.startswith("v_cndmask"):
                    assert pc - self.last_mask_write[s_] >= 3, f"{ins}: mask {s_} read too soon after its comparison"
                if s_ in self.last_trans_write and not trans:
                    assert pc - self.last_trans_write[s_] >= 2, f"{ins}: {s_} read too soon after the exponential"
            if op == "v_cndmask_b32":                         # VOP2 form reads vcc implicitly
                assert pc - self.last_mask_write["vcc"] >= 3
            if op == "v_accvgpr_read_b32":
                idx = int(a[1][1:])
                self.fset(a[0], self.agpr[idx])
                self.accvgpr_reads.append((a[0], idx))
            elif op == "v_max3_f32":
                self.fset(a[0], np.maximum(np.maximum(self.fget(a[1]), self.fget(a[2])), self.fget(a[3])))
            elif op == "v_max_f32":
                self.fset(a[0], np.maximum(self.fget(a[1]), self.fget(a[2])))
            elif op == "v_mov_b32":
                self.iset(a[0], self.iget(a[1]))
            elif op in ("v_cmp_eq_f32_e64", "v_cmp_gt_f32"):
                x, y = self.fget(a[1]), self.fget(a[2])
                self.mask[a[0]] = (x == y) if op.startswith("v_cmp_eq") else (x > y)
                self.last_mask_write[a[0]] = pc
            elif op == "v_cndmask_b32_e64":
                self.iset(a[0], np.where(self.mask[a[3]], self.iget(a[2]), self.iget(a[1])))
            elif op == "v_cndmask_b32":
                assert a[3] == "vcc"
                self.iset(a[0], np.where(self.mask["vcc"], self.iget(a[2]), self.iget(a[1])))
            elif op == "v_lshrrev_b32":
                self.iset(a[0], self.iget(a[2]) >> self.iget(a[1]))
            elif op == "v_and_b32":
                self.iset(a[0], self.iget(a[1]) & self.iget(a[2]))
            elif op == "v_lshl_add_u32":
                self.iset(a[0], (self.iget(a[1]) << self.iget(a[2])) + self.iget(a[3]))
            elif op == "v_add_u32":
                self.iset(a[0], self.iget(a[1]) + self.iget(a[2]))
            elif op == "v_sub_f32":
                self.fset(a[0], self.fget(a[1]) - self.fget(a[2]))
            elif op == "v_mul_f32":
                self.fset(a[0], self.fget(a[1]) * self.fget(a[2]))
            elif op == "v_add_f32":
                self.fset(a[0], self.fget(a[1]) + self.fget(a[2]))
            elif op == "v_exp_f32":
                self.fset(a[0], np.exp2(self.fget(a[1]).astype(np.float64)).astype(np.float32))
                self.last_trans_write[a[0]] = pc
            elif op == "v_fmamk_f32":          # d = s0 * K + s1, one rounding
                self.fset(a[0], (self.fget(a[1]).astype(np.float64) * self.fget(a[2]).astype(np.float64)
                                 + self.fget(a[3]).astype(np.float64)).astype(np.float32))
            elif op == "v_fma_f32":
                self.fset(a[0], (self.fget(a[1]).astype(np.float64) * self.fget(a[2]).astype(np.float64)
                                 + self.fget(a[3]).astype(np.float64)).astype(np.float32))
            else:
                raise AssertionError(f"instruction the interpreter does not know: {ins}")
            if not trans:
                self.last_trans_write.pop(a[0], None)


@pytest.fixture(scope="module")
def reduction():
    prog = tile_listing()
    first = next(i for i, ln in enumerate(prog) if ln.startswith("v_accvgpr_read_b32"))
    assert all(not ln.startswith("v_mfma") for ln in prog[first:])
    assert prog[first - 4:first] == ["s_mov_b32 %[wsrc_lo], s96", "s_mov_b32 %[wsrc_hi], s97",
                                     "s_mov_b32 %[hsrc_lo], s98", "s_mov_b32 %[hsrc_hi], s99"]
    # the tile is complete and visible before it is read: every fragment read waited for, 32 idle issue slots
    assert prog[first - 7:first - 4] == ["s_waitcnt lgkmcnt(0)", "s_nop 15", "s_nop 15"]
    return prog, prog[first:]


def test_statement_addresses_the_accumulators_by_number_and_clears_them_itself(reduction):
    """Every MFMA accumulates into an aligned block of four AGPRs named by number, and the statement clears all 256
    registers before its first MFMA (the K-loop checker proves it for every path through the listing)."""
    prog, _ = reduction
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


@pytest.mark.parametrize("seed", range(4))
def test_reduction_equals_the_running_update_it_stands_for(reduction, seed):
    _, red = reduction
    rng = np.random.default_rng(seed)
    n = 512
    agpr = (rng.standard_normal((256, n)) * 3).astype(np.float32)
    # plant exact ties (the lowest element must win), maxima equal to the running maximum (no update: strict), and
    # a column whose running maximum is far above everything in the tile
    for lane in range(0, n, 7):
        col, e1, e2 = rng.integers(8), rng.integers(32), rng.integers(32)
        top = np.float32(20 + lane % 5)
        agpr[((e1 // 4) * 8 + col) * 4 + e1 % 4, lane] = top
        agpr[((e2 // 4) * 8 + col) * 4 + e2 % 4, lane] = top
    L = Lanes(n, agpr)
    m0 = (rng.standard_normal((8, n)) * 3).astype(np.float32)
    m0[:, :40] = -1.0e30                                   # fresh columns
    m0[3, 100:130] = 50.0
    s0 = (1 + rng.random((8, n)) * 100).astype(np.float32)
    s0[:, :40] = 0.0
    i0 = rng.integers(0, 100000, (8, n)).astype(np.uint32)
    for lane in range(5, n, 11):                           # running maximum equal to the tile maximum of column 2
        x = np.array([agpr[((e // 4) * 8 + 2) * 4 + e % 4, lane] for e in range(32)])
        m0[2, lane] = x.max()
    vb = (rng.integers(0, 400, n) * 256 + rng.integers(0, 2, n) * 128 + 4 * rng.integers(0, 4, n)).astype(np.uint32)
    for tb in range(8):
        L.fset(f"%[m{tb}]", m0[tb])
        L.fset(f"%[s{tb}]", s0[tb])
        L.iset(f"%[i{tb}]", i0[tb])
    L.iset("%[vb]", vb)
    L.run(red)
    # every accumulator is read exactly once, element e of column tb from block (e / 4, tb), register e % 4
    assert sorted(idx for _, idx in L.accvgpr_reads) == list(range(256))
    for tb in range(8):
        x = np.stack([agpr[((e // 4) * 8 + tb) * 4 + e % 4] for e in range(32)])          # [32, n]
        t = x.max(axis=0)
        sel = np.argmax(x == t, axis=0)                                                    # lowest element at the maximum
        code = 16 * (sel // 4) + sel % 4
        want_i = np.where(t > m0[tb], vb + code, i0[tb])
        mn = np.maximum(m0[tb], t)
        x64, mn64 = x.astype(np.float64), mn.astype(np.float64)
        want_s = s0[tb].astype(np.float64) * np.exp(m0[tb].astype(np.float64) - mn64) + np.exp(x64 - mn64).sum(axis=0)
        got_m, got_s = L.fget(f"%[m{tb}]"), L.fget(f"%[s{tb}]").astype(np.float64)
        assert np.array_equal(got_m, mn), tb
        assert np.array_equal(L.iget(f"%[i{tb}]"), want_i.astype(np.uint32)), tb
        assert np.all(np.abs(got_s - want_s) <= 2e-6 * want_s + 1e-30), (tb, np.abs(got_s / want_s - 1).max())


def test_the_interpreter_catches_a_mask_read_too_soon(reduction):
    """Plant a mistake in a copy of the listing: a select moved right behind its comparison must trip the rule."""
    _, red = reduction
    broken = list(red)
    i = next(k for k, ln in enumerate(broken) if ln.startswith("v_cndmask_b32_e64"))
    mask = broken[i].split(",")[-1].strip()
    j = max(k for k in range(i) if broken[k].startswith("v_cmp_eq_f32_e64 " + mask))
    ins = broken.pop(i)
    broken.insert(j + 1, ins)
    L = Lanes(4, np.zeros((256, 4), np.float32))
    for tb in range(8):
        L.fset(f"%[m{tb}]", np.zeros(4))
        L.fset(f"%[s{tb}]", np.zeros(4))
        L.iset(f"%[i{tb}]", np.zeros(4))
    L.iset("%[vb]", np.zeros(4))
    with pytest.raises(AssertionError):
        L.run(broken)
