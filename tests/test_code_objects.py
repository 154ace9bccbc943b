"""CPU-only check of the built GPU code: no kernel of libsprnn.so or libsprnn_probe.so uses scratch memory or spills
vector registers.

The persistent kernels keep every packed weight in a register for the whole sequence, addressed with compile-time
indices; a spill or a stack array would silently turn that into memory traffic in the hot loop.  The check reads the
metadata notes of the gfx950 code objects embedded in the libraries (sizes and counts only; no instruction is
decoded): .private_segment_fixed_size and .vgpr_spill_count must be zero for every kernel.  Scalar-register spills go
to lanes of a vector register, not to memory, and are reported for information.
"""
import os
import re
import shutil
import struct
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_1804_10223_amd")
MAGIC = b"__CLANG_OFFLOAD_BUNDLE__"


def _tool(name):
    for cand in (os.path.join("/opt/rocm/llvm/bin", name), shutil.which(name)):
        if cand and os.path.exists(cand):
            return cand
    pytest.skip("%s not found" % name)


def _device_code_objects(lib_path, tmp_path):
    """The gfx950 code objects of every offload bundle in the library's .hip_fatbin section, as files."""
    fat = tmp_path / "fatbin"
    subprocess.run([_tool("llvm-objcopy"), "--dump-section", ".hip_fatbin=%s" % fat, lib_path, str(tmp_path / "unused.so")], check=True)
    blob = fat.read_bytes()
    out, at = [], blob.find(MAGIC)
    while at >= 0:
        (count,) = struct.unpack_from("<Q", blob, at + len(MAGIC))
        pos = at + len(MAGIC) + 8
        for _ in range(count):
            offset, size, idlen = struct.unpack_from("<QQQ", blob, pos)
            ident = blob[pos + 24:pos + 24 + idlen].decode()
            pos += 24 + idlen
            if "gfx950" in ident and size:
                path = tmp_path / ("code_%d.co" % len(out))
                path.write_bytes(blob[at + offset:at + offset + size])
                out.append(str(path))
        at = blob.find(MAGIC, at + len(MAGIC))
    return out


def _kernel_notes(code_object):
    """[{name, private_segment_fixed_size, vgpr_spill_count, sgpr_spill_count, vgpr_count}] from the metadata notes."""
    text = subprocess.run([_tool("llvm-readelf"), "--notes", code_object], check=True, capture_output=True, text=True).stdout
    kernels, cur = [], None
    for line in text.splitlines():
        m = re.match(r"\s*-?\s*\.(\w+):\s*(.*)$", line)
        if not m:
            continue
        key, val = m.group(1), m.group(2).strip()
        if key == "agpr_count" or (key == "args" and cur is None):
            pass
        if re.match(r"\s*- \.", line) and key in ("agpr_count", "args"):   # first key of a kernel's map (keys are sorted)
            cur = {}
            kernels.append(cur)
        if cur is not None and key in ("name", "private_segment_fixed_size", "vgpr_spill_count", "sgpr_spill_count", "vgpr_count"):
            cur[key] = val if key == "name" else int(val)
    return [k for k in kernels if "name" in k]


@pytest.mark.parametrize("lib", ["libsprnn.so", "libsprnn_probe.so"])
def test_no_kernel_uses_scratch_or_spills_vector_registers(lib, tmp_path):
    path = os.path.join(PKG, lib)
    if not os.path.exists(path):
        pytest.skip("%s has not been built" % lib)
    kernels = []
    for co in _device_code_objects(path, tmp_path):
        kernels += _kernel_notes(co)
    assert len(kernels) >= (100 if lib == "libsprnn.so" else 5), "metadata of only %d kernels found" % len(kernels)
    bad = [(k["name"], k.get("private_segment_fixed_size"), k.get("vgpr_spill_count")) for k in kernels
           if k.get("private_segment_fixed_size", -1) != 0 or k.get("vgpr_spill_count", -1) != 0]
    assert not bad, "kernels with scratch or vector-register spills: %s" % bad[:5]
    worst = max(kernels, key=lambda k: k.get("sgpr_spill_count", 0))
    print("%s: %d kernels, no scratch, no VGPR spills; most scalar-register spills (to vector lanes): %d in %s" % (
        lib, len(kernels), worst.get("sgpr_spill_count", 0), worst["name"][:80]))
