"""Properties of the built kernels, read from the metadata notes of the library's own gfx950 code
objects: none may use scratch memory or spill registers.  (A table build that indexed a small
array by a lane-dependent value and a loader that kept 16-byte values in an array both ended up
in scratch memory once, silently, and cost 25 - 35 % of the run time of their kernels.)"""
import os
import re
import shutil
import struct
import subprocess
import tempfile

import pytest

from paper_2507_04610_amd import binding

READELF = "/opt/rocm/llvm/bin/llvm-readelf"
MAGIC = b"__CLANG_OFFLOAD_BUNDLE__"


def device_code_objects(path):
    """the gfx950 ELF images inside a host library: every translation unit contributes one bundle
    (magic, entry count, then per entry offset / size / triple)"""
    blob = open(path, "rb").read()
    out = []
    pos = blob.find(MAGIC)
    while pos >= 0:
        (count,) = struct.unpack_from("<Q", blob, pos + len(MAGIC))
        cur = pos + len(MAGIC) + 8
        for _ in range(count):
            off, size, tlen = struct.unpack_from("<QQQ", blob, cur)
            triple = blob[cur + 24:cur + 24 + tlen].decode()
            cur += 24 + tlen
            if "gfx950" in triple and size > 0:
                out.append(blob[pos + off:pos + off + size])
        pos = blob.find(MAGIC, pos + len(MAGIC))
    return out


@pytest.mark.skipif(not os.path.exists(READELF), reason="llvm-readelf of the ROCm toolchain is needed")
def test_no_kernel_uses_scratch_memory_or_spills():
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libany4.so has not been built")
    images = device_code_objects(binding.LIB_PATH)
    assert len(images) >= 7, "one code object per kernel source file"
    kernels = {}
    tmp = tempfile.mkdtemp()
    try:
        for i, image in enumerate(images):
            p = os.path.join(tmp, f"co{i}.elf")
            with open(p, "wb") as f:
                f.write(image)
            notes = subprocess.run([READELF, "--notes", p], capture_output=True, text=True, check=True).stdout
            name = None
            for line in notes.splitlines():
                m = re.match(r"\s*\.name:\s+(\S+)", line)
                if m:
                    name = m.group(1)
                    kernels[name] = {}
                m = re.match(r"\s*\.(private_segment_fixed_size|vgpr_spill_count):\s+(\d+)", line)
                if m and name:
                    kernels[name][m.group(1)] = int(m.group(2))
    finally:
        shutil.rmtree(tmp)
    assert len(kernels) > 100, "the streaming kernel alone has more than a hundred variants"
    # (scalar registers parked in lanes of a vector register - sgpr_spill_count - touch no memory and
    # are tolerated: the wavefront-per-row kernel for very long K has a few)
    bad = {k: v for k, v in kernels.items() if any(v.get(f, 0) != 0 for f in
                                                  ("private_segment_fixed_size", "vgpr_spill_count"))}
    assert not bad, bad
