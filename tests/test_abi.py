"""The C-ABI library loads without a GPU and exports every function that
include/ckpt.h declares; argument errors that need no device are reported."""
import ctypes
import os
import re

import pytest

from paper_2202_07848_amd import binding as ck

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ckpt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ckpt_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    lib = ctypes.CDLL(ck.LIB_PATH)
    names = declared_functions()
    assert {"ckpt_fingerprint", "ckpt_diff", "ckpt_compact", "ckpt_restore",
            "ckpt_plan_create", "ckpt_plan_destroy"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert set(ck.EXPORTS) == set(names)


def test_version_and_strerror():
    assert ck.version() >= 1
    lib = ck._lib()
    for status in range(0, -8, -1):
        assert lib.ckpt_strerror(status).decode() not in ("", "unknown status")
    assert lib.ckpt_strerror(-99).decode() == "unknown status"


def test_host_side_argument_checks_need_no_device():
    lib = ck._lib()
    out = ctypes.c_void_p()
    one = (ck._Buf * 1)()
    one[0].ptr, one[0].nbytes = 0x1000, 4096
    assert lib.ckpt_plan_create(one, 1, 1000, ctypes.byref(out)) == -3        # not a power of two
    assert lib.ckpt_plan_create(one, 1, 128, ctypes.byref(out)) == -3         # too small
    assert lib.ckpt_plan_create(one, 1, 1 << 31, ctypes.byref(out)) == -3     # too large
    assert lib.ckpt_plan_create(None, 1, 4096, ctypes.byref(out)) == -1
    assert lib.ckpt_plan_create(one, 1, 4096, None) == -1
    one[0].ptr = 0x1008
    assert lib.ckpt_plan_create(one, 1, 4096, ctypes.byref(out)) == -2        # misaligned buffer
    one[0].ptr = None
    assert lib.ckpt_plan_create(one, 1, 4096, ctypes.byref(out)) == -1        # NULL with bytes
    assert out.value is None
    # two buffers of one list that share a byte (checked before anything touches a device)
    two = (ck._Buf * 3)()
    two[0].ptr, two[0].nbytes = 0x20000, 8192
    two[1].ptr, two[1].nbytes = 0x10000, 4096
    two[2].ptr, two[2].nbytes = 0x21FF0, 64            # starts 16 bytes before buffer 0 ends
    assert lib.ckpt_plan_create(two, 3, 4096, ctypes.byref(out)) == -1
    two[2].ptr = 0x20000                                # the same buffer twice
    assert lib.ckpt_plan_create(two, 3, 4096, ctypes.byref(out)) == -1
    assert out.value is None
    assert lib.ckpt_plan_set_split_threshold(None, 0) == -1
    assert lib.ckpt_plan_split_threshold(None) == 0
    assert lib.ckpt_fingerprint(None, None, None) == -1
    assert lib.ckpt_diff(None, None, None, 0, None, None, None) == -1
    assert lib.ckpt_compact(None, None, None, None, 0, None, 0, None, None) == -1
    assert lib.ckpt_restore(None, None, 0, None, 0, None, None) == -1
    assert lib.ckpt_manifest(None, None, None, 0, None, 0, None, None) == -1
    assert lib.ckpt_buffer_verdicts(None, None, None, None, None) == -1
    assert lib.ckpt_mask_andnot(None, None, None, None, None) == -1
    assert lib.ckpt_marks_from_buffers(None, None, None, None) == -1
    assert lib.ckpt_restore_chain(None, None, 0, None, None, 0, None, None) == -1
    assert lib.ckpt_restore_chain_workspace_bytes(1000) == 16016
    assert lib.ckpt_merge_chain(None, None, 0, None, 0, None, 0, None, None, 0, None, None) == -1
    assert lib.ckpt_merge_chain_workspace_bytes(1000) == 16016 + 1008
    assert lib.ckpt_exchange(None, None, None, None, 0, None, None, None, 0, 0, None, None, None) == -1
    assert lib.ckpt_snapshot(None, None, 0, None, None, None, None, 0, None, 0, None, None, None, 0,
                             None) == -1
    assert lib.ckpt_snapshot_static(None, None, 0, None, None, None, None, 0, None, 0, None, None,
                                    None) == -1
    assert lib.ckpt_snapshot_static_max_chunks() == 1 << 18
    assert lib.ckpt_snapshot_stats_offset(1000) == 8000
    assert lib.ckpt_bw_streams(None, None, 16, 512, 256, None, None) == -1
    assert lib.ckpt_bw_streams(None, None, 16, 4096, 512, None, None) == -1     # no such tile
    assert lib.ckpt_plan_destroy(None) == 0
    assert lib.ckpt_plan_nchunks(None) == 0


def test_static_scratch_symbol_is_visible_to_the_runtime():
    """hipGetSymbolAddress finds a device variable by name among the code object's global
    symbols.  The static scratch array of ckpt_snapshot_static is made global by the compiler
    because host code names it; an attribute that pins its internal linkage (such as `used`)
    would leave it a local symbol, which the runtime cannot look up."""
    import subprocess
    import tempfile
    from paper_2202_07848_amd import build as hip_build
    readelf = "/opt/rocm/llvm/bin/llvm-readelf"
    if not (os.path.exists(hip_build.HIPCC) and os.path.exists(readelf)):
        pytest.skip("no ROCm toolchain")
    with tempfile.TemporaryDirectory() as tmp:
        obj = os.path.join(tmp, "api_device.o")
        flags = [f for f in hip_build.FLAGS if f != "-shared"]
        subprocess.run([hip_build.HIPCC] + flags + ["--offload-device-only", "--no-gpu-bundle-output",
                        "-c", os.path.join(hip_build.CSRC, "api.hip"), "-o", obj],
                       check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        table = subprocess.run([readelf, "-s", obj], check=True, stdout=subprocess.PIPE,
                               text=True).stdout
    rows = [ln.split() for ln in table.splitlines() if ln.rstrip().endswith("scratch")
            and "OBJECT" in ln]
    assert rows, "the scratch array is not in the device code object"
    assert all(r[4] == "GLOBAL" for r in rows), rows
    assert all(int(r[2]) >= 2_400_000 for r in rows), rows


def test_binding_fails_loudly_without_library(monkeypatch):
    monkeypatch.setattr(ck, "_handle", None)
    monkeypatch.setattr(ck, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libckpt.so"))
    with pytest.raises(ImportError):
        ck.version()


C_PROGRAM = r"""
#include <stddef.h>
#include <stdio.h>
#include "ckpt.h"
int main(void) {
  /* host-only calls: no device is touched */
  ckpt_plan_t *plan = (ckpt_plan_t *)0;
  ckpt_buf_t one = {(void *)0x1000, 4096};
  if (ckpt_plan_create(&one, 1, 1000, &plan) != CKPT_ERR_CHUNK || plan) return 1;
  if (ckpt_restore_chain(0, 0, 0, 0, 0, 0, 0, 0) != CKPT_ERR_INVALID_ARG) return 2;
  if (ckpt_version() < 1 || !ckpt_strerror(CKPT_ERR_CAPACITY)[0]) return 3;
  printf("%zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %d\n", sizeof(ckpt_buf_t), sizeof(ckpt_entry_t),
         offsetof(ckpt_entry_t, buf_off), offsetof(ckpt_entry_t, stage_off),
         offsetof(ckpt_entry_t, digest), sizeof(ckpt_counts_t), sizeof(ckpt_link_t),
         offsetof(ckpt_link_t, d_manifest), offsetof(ckpt_link_t, d_counts),
         sizeof(ckpt_chain_stats_t), CKPT_CHAIN_MAX);
  return 0;
}
"""


def test_header_is_plain_c_and_a_c_program_links_against_the_library(tmp_path):
    """include/ckpt.h under gcc -std=c11 -pedantic, a C caller linked against libckpt.so, and the
    struct layouts the ctypes binding assumes against what the C compiler lays out."""
    import subprocess
    src, exe = tmp_path / "caller.c", tmp_path / "caller"
    src.write_text(C_PROGRAM)
    libdir = os.path.dirname(ck.LIB_PATH)
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I",
                    os.path.join(ROOT, "include"), str(src), "-o", str(exe), "-L", libdir, "-lckpt",
                    "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], stdout=subprocess.PIPE, text=True, check=True).stdout.split()
    got = [int(x) for x in out]
    entry = ck.ENTRY_DTYPE if hasattr(ck, "ENTRY_DTYPE") else None
    assert got == [ctypes.sizeof(ck._Buf), 32, 8, 16, 24, 24, ctypes.sizeof(ck._Link),
                   ck._Link.d_manifest.offset, ck._Link.d_counts.offset, 24, ck.CHAIN_MAX]
    assert ck.ENTRY_BYTES == 32
    if entry is not None:
        assert entry.itemsize == 32 and entry.fields["stage_off"][1] == 16
