"""The gfx950 code object inside libiso.so: every kernel must run without private (scratch) memory.

A kernel that reads its argument struct in very many places can have the whole struct copied into
private memory per lane by the compiler (seen once on the block kernel: 840 bytes of scratch, 18 times
slower, same results), so no parity test notices.  The code object's own metadata does."""
import os
import re
import struct
import subprocess

import pytest

import paper_1606_07676_amd as iso

READELF = "/opt/rocm/llvm/bin/llvm-readelf"
MAGIC = b"__CLANG_OFFLOAD_BUNDLE__"


def _device_code_object(lib_path):
    """The gfx950 ELF of the offload bundle that hipcc embeds in the shared library."""
    data = open(lib_path, "rb").read()
    at = data.find(MAGIC)
    assert at >= 0, "no offload bundle in the library"
    (n,) = struct.unpack_from("<Q", data, at + len(MAGIC))
    pos = at + len(MAGIC) + 8
    for _ in range(n):
        off, size, tlen = struct.unpack_from("<QQQ", data, pos)
        triple = data[pos + 24:pos + 24 + tlen].decode()
        pos += 24 + tlen
        if "gfx950" in triple:
            return data[at + off:at + off + size]
    raise AssertionError("no gfx950 entry in the offload bundle")


@pytest.mark.skipif(not os.path.exists(READELF), reason="llvm-readelf of the ROCm toolchain not found")
def test_no_kernel_uses_private_memory_or_spills(tmp_path):
    lib = os.path.join(os.path.dirname(iso.__file__), "libiso.so")
    elf = tmp_path / "libiso_gfx950.co"
    elf.write_bytes(_device_code_object(lib))
    notes = subprocess.run([READELF, "--notes", str(elf)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                           text=True, check=True).stdout
    kernels = {}
    name = None
    for block in re.split(r"\n\s+- ", notes):
        m = re.search(r"\.name:\s+(\S+)", block)
        p = re.search(r"\.private_segment_fixed_size:\s+(\d+)", block)
        if m and p:
            name = m.group(1)
            spill = re.search(r"\.vgpr_spill_count:\s+(\d+)", block)
            kernels[name] = (int(p.group(1)), int(spill.group(1)) if spill else 0)
    assert len(kernels) > 20, notes[:2000]
    for want in ("shift_round_kernel", "shift_round_uniform_kernel", "vector_round_kernel", "block_round_kernel",
                 "mesh_shift_round_kernel", "staged_round_kernel", "deliver_kernel", "copy_kernel", "table_store_kernel"):
        assert any(want in k for k in kernels), want
    bad = {k: v for k, v in kernels.items() if v != (0, 0)}
    assert not bad, f"kernels with private memory or register spills: {bad}"
