"""The generated K-loop of the 4-wave kernel, interpreted on the CPU (no GPU): the scalar book-keeping is executed
instruction by instruction and every copy, LDS read, wait, barrier and MFMA is checked against the ring protocol.

What is proved for each (K-tiles per vocabulary tile, vocabulary tiles per unit) tried:
  * every direct-to-LDS copy reads a tile that exists (its source pointer decodes to a step below the total: no
    out-of-bounds global read) and each tile is copied exactly once, in order;
  * a copy never targets a slot that any wave may still read (no LDS read of that slot between the two barriers
    around the copy), and a slot is never read while a copy into it is not yet published;
  * a copy is "published" only by a vmcnt wait that covers it followed by a barrier; every LDS read finds the tile
    and K-half it expects;
  * every MFMA group multiplies fragments that were read, waited for (lgkmcnt) and belong to its step and K-half;
  * fragment registers are not overwritten while the group that uses them is still issuing.
Waves run the same instruction stream and meet at every barrier, so one wave's stream plus "anything between two
barriers may overlap across waves" covers the workgroup.
"""
import importlib.util
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GEN = os.path.join(ROOT, "paper_2601_06562_amd", "csrc", "gen_w4_loop.py")

SLOT = 0x8000
NW, NH = 3, 2
W_BASE, H_BASE = 0x10_0000_0000, 0x20_0000_0000       # synthetic device addresses
MASK32 = 0xFFFFFFFF


def generated_lines(fused=False, sample=False):
    """The K-loop listing: of the statement whose accumulators are operands (the tile is reduced in C++), or, with
    fused=True, the K-loop part of a statement that owns the accumulators and reduces the tile itself (the greedy
    one, or with sample=True the sampling one, whose fragment registers are named by number too)."""
    spec = importlib.util.spec_from_file_location("gen_w4_loop", GEN)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.lines.clear()
    if fused:
        mod.build_tile_sample() if sample else mod.build_tile()
        out = list(mod.lines)
        out = out[:next(i for i, ln in enumerate(out) if ln.strip().startswith(("v_accvgpr_read_b32", "s_mov_b32 s68, %[seed_lo]")))]
    else:
        mod.build()
        out = list(mod.lines)
    mod.lines.clear()
    return out


class Sim:
    def __init__(self, lines, nk, ntile):
        self.nk, self.ntile, self.total = nk, ntile, nk * ntile
        self.tile_stride = 256 * nk * 128                  # bytes from one vocabulary tile to the next (d = 64 nk)
        self.prog = []
        self.labels = {}
        for ln in lines:
            ln = ln.strip()
            if ln.endswith(":"):
                self.labels[ln[:-1]] = len(self.prog)
            elif ln:
                self.prog.append(ln)
        self.reg = {}
        self.scc = 0
        # ring state: what each slot holds (published), what is in flight, who read it since the last barrier
        self.published = {}            # slot -> tile id (W: step g, H: k index)
        self.unpublished = {}          # slot -> tile id, copy issued but not yet covered by wait + barrier
        self.landed = set()            # slots whose in-flight copy a vmcnt wait has covered (await the barrier)
        self.vm_queue = []             # destination slots of the outstanding copy instructions, in issue order
        self.reads_this_interval = set()
        self.copies_this_interval = set()
        self.next_w_copy, self.next_h_copy = 0, 0
        self.frag = {}                 # fragment register name -> (operand, tile id, khalf, complete?)
        self.mfma_count = 0
        self.frag_last_group = {}      # fragment register -> last MFMA group that used it
        self.copy_parts = {}           # (slot) -> pieces issued for the current copy (8 instructions per tile per wave)
        self.started = set()           # accumulator registers (by number) started in the current statement
        self.literal_acc = False

    # ---- operand access
    def val(self, tok):
        tok = tok.strip()
        if re.fullmatch(r"-?\d+", tok):
            return int(tok) & MASK32
        if tok.startswith("0x"):
            return int(tok, 16) & MASK32
        return self.reg[tok]

    def set(self, tok, v):
        self.reg[tok.strip()] = v & MASK32

    # ---- events
    def slot_of(self, addr):
        return addr // SLOT

    def copy(self, operand):
        m0 = self.reg["m0"]
        slot = self.slot_of(m0)
        if operand == "W":
            ptr = self.reg["s96"] | (self.reg["s97"] << 32)
            off = ptr - W_BASE
            tile, rest = divmod(off, self.tile_stride)
            assert rest % 128 == 0 and rest // 128 < self.nk, f"W pointer {off} is not a tile start"
            g = tile * self.nk + rest // 128
            assert 0 <= g < self.total, f"W copy of step {g} beyond the {self.total} steps (out-of-bounds read)"
            assert 0 <= slot < NW
            ident = g
            assert g == self.next_w_copy or self.copy_parts.get(slot, 0) > 0, (g, self.next_w_copy)
        else:
            ptr = self.reg["s98"] | (self.reg["s99"] << 32)
            off = ptr - H_BASE
            assert off % 128 == 0 and 0 <= off // 128 < self.nk, f"H pointer {off} outside the row"
            ident = off // 128
            assert NW <= slot < NW + NH
            assert ident == self.next_h_copy % self.nk or self.copy_parts.get(slot, 0) > 0
            assert self.next_h_copy < self.total or self.copy_parts.get(slot, 0) > 0, "hidden copy past the last step"
        assert slot not in self.reads_this_interval, f"copy into slot {slot} that a wave may still be reading"
        parts = self.copy_parts.get(slot, 0)
        if parts == 0:
            assert slot not in self.unpublished, f"second copy into slot {slot} before the first was published"
            self.unpublished[slot] = ident
            self.copies_this_interval.add(slot)
        else:
            assert self.unpublished[slot] == ident
        assert (m0 % SLOT) == 1024 * parts, "the 8 pieces of a tile go to consecutive KiB of the slot"
        self.copy_parts[slot] = parts + 1
        self.vm_queue.append(slot)
        if parts + 1 == 8:
            self.copy_parts[slot] = 0
            if operand == "W":
                self.next_w_copy += 1
            else:
                self.next_h_copy += 1

    def wait_vm(self, n):
        while len(self.vm_queue) > n:
            slot = self.vm_queue.pop(0)
            if slot not in self.vm_queue and self.copy_parts.get(slot, 0) == 0:
                self.landed.add(slot)

    def barrier(self):
        for slot in list(self.landed):
            self.published[slot] = self.unpublished.pop(slot)
        self.landed.clear()
        self.reads_this_interval.clear()
        self.copies_this_interval.clear()

    def ds_read(self, dst, addr_reg, offset):
        addr = self.reg[addr_reg] + offset
        slot = self.slot_of(addr)
        khalf = 1 if (addr % SLOT) % 128 == 64 else 0
        operand = "W" if slot < NW else "H"
        assert (operand == "W") == (addr_reg == "%[vt0]"), "LM-head fragments come from the LM-head ring"
        if dst.startswith("%["):
            assert (operand == "W") == dst.startswith("%[fa")
        else:                             # fragments by number: LM-head tuples first in each buffer of 16
            first = int(re.fullmatch(r"v\[(\d+):\d+\]", dst).group(1))
            assert (operand == "W") == (((first - 112) // 4) % 16 < 8)
        assert slot not in self.unpublished, f"read of slot {slot} while a copy into it is not published"
        assert slot in self.published, f"read of slot {slot} that holds nothing"
        assert slot not in self.copies_this_interval
        self.reads_this_interval.add(slot)
        group = self.mfma_count // 64
        assert self.frag_last_group.get(dst, -1) < group or self.mfma_count % 64 == 0, \
            f"{dst} overwritten while its group is still issuing"
        self.frag[dst] = (operand, self.published[slot], khalf, False)

    def wait_lgkm(self):
        for k, f in self.frag.items():
            self.frag[k] = (f[0], f[1], f[2], True)

    def mfma(self, a, b, dst=None, src_c=None):
        m = re.fullmatch(r"a\[(\d+):(\d+)\]", dst or "")
        if m:                           # accumulators by number: the statement itself must have started them
            self.literal_acc = True
            regs = set(range(int(m.group(1)), int(m.group(2)) + 1))
            if src_c == "0":
                assert self.mfma_count % 128 < 64 and not (regs & self.started), "a product without addend mid-tile"
                self.started |= regs
            else:
                assert src_c == dst and regs <= self.started, f"accumulation into {dst}, which was never started"
        group, g, h = self.mfma_count // 64, (self.mfma_count // 64) // 2, (self.mfma_count // 64) % 2
        for name, operand in ((a, "W"), (b, "H")):
            assert name in self.frag, f"{name} used before it was read"
            f = self.frag[name]
            assert f[3], f"{name} used before the lgkmcnt wait"
            want = g if operand == "W" else g % self.nk
            assert f[0] == operand and f[1] == want and f[2] == h, \
                f"step {g} half {h}: {name} holds {f}, wanted {operand} {want}"
            self.frag_last_group[name] = group
        self.mfma_count += 1

    # ---- the glue around the statement, as the kernel's C++ does it
    def prologue(self):
        def wptr(g):
            return W_BASE + (g // self.nk) * self.tile_stride + (g % self.nk) * 128
        # the kernel issues W0, H0, W1, W2, H1, waits for the first two only, then meets at a barrier
        self.published[0] = 0
        self.published[NW + 0] = 0
        if self.total > 1:
            self.unpublished[1] = 1
            self.vm_queue += [1] * 8
        if self.total > 2:
            self.unpublished[2] = 2
            self.vm_queue += [2] * 8
        if self.total > 1:
            self.unpublished[NW + 1] = 1 % self.nk
            self.vm_queue += [NW + 1] * 8
        self.next_w_copy, self.next_h_copy = 3, 2
        gw, gh = 3, 2
        w0, h0 = wptr(gw), H_BASE + (gh % self.nk) * 128
        self.reg.update({
            "%[wsrc_lo]": w0 & MASK32, "%[wsrc_hi]": w0 >> 32, "%[hsrc_lo]": h0 & MASK32, "%[hsrc_hi]": h0 >> 32,
            "%[wrd]": 0, "%[hrd]": 0, "%[wdst]": (gw % NW) * SLOT, "%[hdst]": (gh % NH) * SLOT,
            "%[wk]": gw % self.nk, "%[hk]": gh % self.nk, "%[g]": 0,
            "%[total]": self.total, "%[nk]": self.nk,
            "%[wwrap]": (self.tile_stride - (self.nk - 1) * 128) & MASK32, "%[hwrap]": (self.nk - 1) * 128,
            "%[rdw0]": 0, "%[rdw1]": 64, "%[rdh0]": NW * SLOT, "%[rdh1]": NW * SLOT + 64,
        })

    def run_statement(self):
        self.frag.clear()                 # fragment registers do not survive between statements
        self.frag_last_group.clear()
        self.started.clear()              # nor do accumulators the statement addresses by number
        pc, steps = 0, 0
        while pc < len(self.prog):
            steps += 1
            assert steps < 200000, "the loop does not terminate"
            ins = self.prog[pc]
            pc += 1
            op, _, rest = ins.partition(" ")
            args = [a.strip() for a in rest.split(",")] if rest else []
            if op == "v_mfma_f32_16x16x32_bf16":
                self.mfma(args[1], args[2], args[0], args[3])
            elif op == "v_accvgpr_write_b32":
                assert args[1] == "0" and self.mfma_count % 128 == 0
                self.started.add(int(args[0][1:]))
            elif op == "ds_read_b128":
                m = re.fullmatch(r"(\S+)(?: offset:(\d+))?", args[1])
                self.ds_read(args[0], m.group(1), int(m.group(2) or 0))
            elif op == "global_load_lds_dwordx4":
                self.copy("W" if args[1] == "s[96:97]" else "H")
            elif op == "v_add_u32":
                self.set(args[0], self.val(args[1]) + self.val(args[2]))
            elif op == "s_waitcnt":
                counters = re.findall(r"(vmcnt|lgkmcnt)\((\d+)\)", rest)
                assert counters and " ".join(f"{c}({n})" for c, n in counters) == rest.strip()
                for counter, n in counters:          # one instruction may wait on both counters
                    if counter == "vmcnt":
                        self.wait_vm(int(n))
                    else:
                        assert n == "0"
                        self.wait_lgkm()
            elif op == "s_barrier":
                assert all(f[3] for f in self.frag.values()), "barrier with LDS reads still in flight"
                self.barrier()
            elif op == "s_nop":
                pass
            elif op == "s_mov_b32":
                self.set(args[0], self.val(args[1]))
            elif op in ("s_add_u32", "s_addc_u32"):
                r = self.val(args[1]) + self.val(args[2]) + (self.scc if op == "s_addc_u32" else 0)
                self.set(args[0], r)
                self.scc = 1 if r > MASK32 else 0
            elif op in ("s_sub_u32", "s_subb_u32"):
                r = self.val(args[1]) - self.val(args[2]) - (self.scc if op == "s_subb_u32" else 0)
                self.set(args[0], r)
                self.scc = 1 if r < 0 else 0
            elif op in ("s_xor_b32", "s_and_b32"):
                r = self.val(args[1]) ^ self.val(args[2]) if op == "s_xor_b32" else self.val(args[1]) & self.val(args[2])
                self.set(args[0], r)
                self.scc = 1 if r != 0 else 0
            elif op == "s_cselect_b32":
                self.set(args[0], self.val(args[1]) if self.scc else self.val(args[2]))
            elif op.startswith("s_cmp_"):
                a, b = self.val(args[0]), self.val(args[1])
                self.scc = int({"s_cmp_lt_u32": a < b, "s_cmp_ge_u32": a >= b, "s_cmp_eq_u32": a == b}[op])
            elif op == "s_branch":
                pc = self.labels[args[0]]
            elif op == "s_cbranch_scc0":
                if not self.scc:
                    pc = self.labels[args[0]]
            elif op == "s_cbranch_scc1":
                if self.scc:
                    pc = self.labels[args[0]]
            else:
                raise AssertionError(f"instruction the checker does not know: {ins}")


@pytest.fixture(scope="module", params=["accumulators as operands", "fused with the reduction",
                                        "fused with the sampling reduction"])
def lines(request):
    return generated_lines(fused=request.param.startswith("fused"), sample="sampling" in request.param)


@pytest.mark.parametrize("nk", [1, 2, 3, 4, 5, 8, 56, 64])
@pytest.mark.parametrize("ntile", [1, 2, 3, 5, 31])
def test_ring_protocol(lines, nk, ntile):
    if nk >= 56 and ntile > 3:
        pytest.skip("long shapes once is enough")
    sim = Sim(lines, nk, ntile)
    sim.prologue()
    for _ in range(ntile):
        sim.run_statement()
    total = nk * ntile
    assert sim.mfma_count == 128 * total                            # every step ran both of its groups
    assert not sim.literal_acc or sim.started == set(range(256))    # the last statement started all 256 registers
    assert sim.reg["%[g]"] == total
    assert sim.next_w_copy == max(total, 3) and sim.next_h_copy == max(total, 2)   # every tile copied exactly once
    assert not sim.unpublished, "copies still unpublished at the end: a later statement would race with them"


def test_the_checker_catches_a_missing_wait(lines):
    """Plant a mistake in a copy of the listing (never in the product): without the vmcnt wait a tile is read
    before it is published, and the checker must say so."""
    broken = [ln for ln in lines if not ln.strip().startswith("s_waitcnt vmcnt")]
    sim = Sim(broken, 4, 3)
    sim.prologue()
    with pytest.raises(AssertionError):
        for _ in range(3):
            sim.run_statement()


def test_the_checker_catches_a_copy_into_a_slot_in_use(lines):
    """Swap the LM-head copy to target the slot being read: the write-after-read rule must fire."""
    broken = [ln.replace("s_add_u32 %[wdst], %[wdst], 0x8000", "s_add_u32 %[wdst], %[wdst], 0x10000") for ln in lines]
    sim = Sim(broken, 4, 3)
    sim.prologue()
    with pytest.raises(AssertionError):
        for _ in range(3):
            sim.run_statement()


def test_steady_state_keeps_every_gap_between_mfmas_short(lines):
    """A wave is alone on its SIMD and issues an instruction every few cycles, so more than three instructions
    between two MFMAs (16 cycles apart) delay the second one; a run of 16 no-ops in one gap measured +1.2% on the
    whole kernel, the same 16 spread one per gap nothing.  In the steady-state body every gap holds at most two
    instructions, the sync between the two groups of a step two (wait + barrier), and the only branch taken is the
    back edge right behind the last MFMA."""
    prog = [ln.strip() for ln in lines if ln.strip() and not ln.strip().endswith(":") or ln.strip().startswith(("Lsteady", "Lleave"))]
    start = next(i for i, ln in enumerate(prog) if ln.startswith("Lsteady"))
    end = next(i for i, ln in enumerate(prog) if ln.startswith("Lleave"))
    body = prog[start + 1:end]
    assert sum(ln.startswith("v_mfma") for ln in body) == 128
    gap, longest = 0, 0
    for ln in body:
        if ln.startswith("v_mfma"):
            longest, gap = max(longest, gap), 0
        else:
            gap += 1
    assert longest <= 2, longest
    branches = [ln for ln in body if ln.startswith(("s_branch", "s_cbranch"))]
    assert len(branches) == 1 and body[-1] == branches[0] and body[-2].startswith("v_mfma")
    assert sum(ln == "s_barrier" for ln in body) == 1
