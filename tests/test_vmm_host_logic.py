"""The VMM workspace's book-keeping on the CPU: csrc/mosaic_vmm.hip linked against a fake of the driver's virtual-memory
calls (tests/fake_vmm_driver.cpp), built with AddressSanitizer and UndefinedBehaviorSanitizer where the image has them.
Growth in place, both ways of opening the new pages, the fall-back when the driver refuses, out of memory during a
growth, shrinking, many growths in a row and clean-up -- with the fake checking every call as a driver would."""
import ctypes
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2601_06562_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
G = 2 << 20
OK, INVALID, TOO_SMALL, HIP = 0, -1, -3, -4

CHILD = r"""
import ctypes, sys
L = ctypes.CDLL(sys.argv[1])
vp, i64 = ctypes.c_void_p, ctypes.c_int64
L.mosaic_vmm_create.argtypes = [ctypes.c_int, i64, ctypes.POINTER(vp)]
L.mosaic_vmm_resize.argtypes = [vp, i64]
L.mosaic_vmm_destroy.argtypes = [vp]
for name in ("mosaic_vmm_committed_bytes", "mosaic_vmm_reserved_bytes"):
    getattr(L, name).restype = i64
    getattr(L, name).argtypes = [vp]
L.mosaic_vmm_kept_contents.argtypes = [vp]
L.mosaic_vmm_last_error.restype = ctypes.c_char_p
L.mosaic_vmm_last_error.argtypes = [vp, ctypes.POINTER(ctypes.c_int)]
L.fake_mapped_bytes.restype = ctypes.c_longlong
L.fake_open_prefix.argtypes = [ctypes.c_longlong]
G, OK, HIP, TOO_SMALL = 2 << 20, 0, -4, -3

def log():
    buf = ctypes.create_string_buffer(1 << 16)
    L.fake_log(buf, len(buf))
    return buf.value.decode()

def fresh(refuse=(0, 0, -1)):
    L.fake_reset()
    L.fake_refuse(*refuse)
    h = vp()
    assert L.mosaic_vmm_create(0, 64 * G, ctypes.byref(h)) == OK
    return h

def consistent(h, want):
    assert L.mosaic_vmm_committed_bytes(h) == want, (L.mosaic_vmm_committed_bytes(h), want)
    assert L.fake_mapped_bytes() == want and L.fake_violations() == 0, log()
    assert L.fake_open_prefix(want) == 1, log()

# growth in place: the driver opens the whole prefix
h = fresh()
assert L.mosaic_vmm_resize(h, G + 5) == OK
consistent(h, 2 * G); assert L.mosaic_vmm_kept_contents(h) == 0 and L.fake_mappings() == 1
assert L.mosaic_vmm_resize(h, 5 * G) == OK
consistent(h, 5 * G); assert L.mosaic_vmm_kept_contents(h) == 1 and L.fake_mappings() == 2 and L.fake_syncs() == 0
assert L.mosaic_vmm_resize(h, 5 * G - 7) == OK and L.fake_mappings() == 2          # same rounded size: nothing happens
assert L.mosaic_vmm_resize(h, 9 * G) == OK
consistent(h, 9 * G); assert L.mosaic_vmm_kept_contents(h) == 1 and L.fake_mappings() == 3
# shrink: wait, drop every piece, one new mapping
assert L.mosaic_vmm_resize(h, 3 * G) == OK
consistent(h, 3 * G); assert L.mosaic_vmm_kept_contents(h) == 0 and L.fake_mappings() == 1 and L.fake_syncs() == 1
assert L.fake_live_handles() == 1
# beyond the reservation: refused, nothing changes
assert L.mosaic_vmm_resize(h, 65 * G) == TOO_SMALL
consistent(h, 3 * G)
assert L.mosaic_vmm_resize(h, 0) == OK
consistent(h, 0); assert L.fake_live_handles() == 0
assert L.mosaic_vmm_destroy(h) == OK and L.fake_violations() == 0, log()

# the driver refuses the whole prefix and accepts the new pages alone
h = fresh((1, 0, -1))
assert L.mosaic_vmm_resize(h, 2 * G) == OK and L.mosaic_vmm_resize(h, 6 * G) == OK
consistent(h, 6 * G); assert L.mosaic_vmm_kept_contents(h) == 2 and L.fake_mappings() == 2 and L.fake_syncs() == 0
assert L.mosaic_vmm_destroy(h) == OK and L.fake_violations() == 0 and L.fake_live_handles() == 0, log()

# the driver refuses both: the new piece is taken back and the range is mapped afresh as one piece
h = fresh((1, 1, -1))
assert L.mosaic_vmm_resize(h, 2 * G) == OK and L.mosaic_vmm_resize(h, 6 * G) == OK
consistent(h, 6 * G); assert L.mosaic_vmm_kept_contents(h) == 0 and L.fake_mappings() == 1 and L.fake_syncs() == 1
assert L.fake_live_handles() == 1
assert L.mosaic_vmm_destroy(h) == OK and L.fake_violations() == 0 and L.fake_live_handles() == 0, log()

# no memory for a growth: the call fails, what was mapped stays, the error names the call
h = fresh((0, 0, 1))
assert L.mosaic_vmm_resize(h, 2 * G) == OK
assert L.mosaic_vmm_resize(h, 6 * G) == HIP
consistent(h, 2 * G)
code = ctypes.c_int(0)
assert L.mosaic_vmm_last_error(h, ctypes.byref(code)) == b"hipMemCreate" and code.value != 0
assert L.mosaic_vmm_destroy(h) == OK and L.fake_violations() == 0 and L.fake_live_handles() == 0, log()

# many growths in a row: pieces are bounded, the range stays whole
h = fresh()
for k in range(1, 50):
    assert L.mosaic_vmm_resize(h, k * G) == OK
    consistent(h, k * G)
    assert L.fake_mappings() <= 32
assert L.mosaic_vmm_destroy(h) == OK and L.fake_violations() == 0 and L.fake_live_handles() == 0, log()
print("vmm host logic ok")
"""


def test_vmm_book_keeping_against_a_fake_driver(tmp_path):
    lib = str(tmp_path / "libmosaic_vmm_fake.so")
    asan = glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    san = ["-Xarch_host", "-fsanitize=address,undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xarch_host", "-shared-libsan"] if asan else []
    cmd = [HIPCC, "--offload-arch=gfx950", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", *san,
           "-Wno-unused-command-line-argument", "-Wno-option-ignored", "-Wl,-Bsymbolic",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-o", lib,
           os.path.join(CSRC, "mosaic_vmm.hip"), os.path.join(ROOT, "tests", "fake_vmm_driver.cpp")]
    built = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert built.returncode == 0, built.stdout[-3000:]
    env = dict(os.environ)
    if asan:
        preload = [asan[0]] + [p for p in env.get("LD_PRELOAD", "").split(":") if p]
        env.update(LD_PRELOAD=":".join(preload), ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0",
                   UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    res = subprocess.run([sys.executable, "-c", CHILD, lib], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=300)
    assert res.returncode == 0 and "vmm host logic ok" in res.stdout, res.stdout[-4000:]
    assert "AddressSanitizer" not in res.stdout and "runtime error:" not in res.stdout, res.stdout[-4000:]
