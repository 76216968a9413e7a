"""CPU-side check of what the compiler made of the scoring kernels: registers and scratch.

The scoring sweeps are laid out for two wavefronts per SIMD (a SIMD has 512 registers per lane):
a kernel of four-wavefront workgroups that needs more than 256 registers still runs, one
wavefront per SIMD, at a little over half the speed, and a spill inside the tile loop puts
scratch loads between the K loads.  Neither shows in a parity test, and both have happened
after changes that looked harmless, so the build's own metadata is read back here (from the
code objects inside the built library, with the ROCm LLVM tools; nothing is launched)."""
import os
import re
import subprocess
import tempfile

import pytest

import paper_2407_11550_amd.binding as B

LLVM = "/opt/rocm/llvm/bin"
TOOLS = [os.path.join(LLVM, t) for t in ("llvm-objcopy", "clang-offload-bundler", "llvm-readelf")]
MAGIC = b"__CLANG_OFFLOAD_BUNDLE__"


def _kernel_metadata(lib_path):
    """{kernel symbol: {vgpr, agpr, scratch, lds}} over every gfx950 code object in the library."""
    out = {}
    with tempfile.TemporaryDirectory() as tmp:
        fat = os.path.join(tmp, "fat.bin")
        subprocess.run([TOOLS[0], "-O", "binary", "--only-section=.hip_fatbin", lib_path, fat], check=True)
        data = open(fat, "rb").read()
        starts = [m.start() for m in re.finditer(re.escape(MAGIC), data)] + [len(data)]
        for i in range(len(starts) - 1):
            piece, obj = os.path.join(tmp, f"b{i}.bin"), os.path.join(tmp, f"co{i}.o")
            open(piece, "wb").write(data[starts[i]:starts[i + 1]])
            r = subprocess.run([TOOLS[1], "--unbundle", "--type=o", "--targets=hipv4-amdgcn-amd-amdhsa--gfx950",
                                f"--input={piece}", f"--output={obj}"], capture_output=True, text=True)
            if r.returncode != 0 or not os.path.exists(obj) or os.path.getsize(obj) == 0:
                continue
            notes = subprocess.run([TOOLS[2], "--notes", obj], capture_output=True, text=True, check=True).stdout
            for block in notes.split("  - .agpr_count:")[1:]:
                def field(name, block=block):
                    m = re.search(r"\." + name + r":\s+(\S+)", block)
                    return m.group(1) if m else None
                out[field("name")] = dict(agpr=int(block.split()[0]), vgpr=int(field("vgpr_count")),
                                          scratch=int(field("private_segment_fixed_size")),
                                          lds=int(field("group_segment_fixed_size")))
    return out


def _score_kernels(meta):
    """(d, mb, rs, kg, chunk, pass, f16, pool_rows) -> metadata, from the mangled template arguments."""
    pat = re.compile(r"score_mfma_kernelILi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELb(\d)ELb(\d)")
    out = {}
    for name, md in meta.items():
        m = pat.search(name or "")
        if m:
            out[tuple(int(x) for x in m.groups())] = md
    return out


@pytest.fixture(scope="module")
def score_kernels(lib):
    if not all(os.path.exists(t) for t in TOOLS):
        pytest.skip("ROCm LLVM tools not installed")
    ks = _score_kernels(_kernel_metadata(B._LIB_PATH))
    assert len(ks) >= 80, f"only {len(ks)} scoring kernels found in the library's metadata"
    return ks


def test_two_wavefronts_per_simd_where_the_layout_counts_on_them(score_kernels):
    """The 128-row kernels (four wavefronts, two workgroups per compute unit) and the 256- and
    512-row kernels, in both sweeps and both 16-bit types: at most 256 registers (vector plus
    accumulation registers).  The row-pooling form of the weights sweep is known to need more on
    d = 128 and is left out; so are the 32- and 64-row forms with four key groups, which are bound
    by memory with one wavefront per SIMD as well."""
    checked = 0
    for (d, mb, rs, kg, chunk, sweep, f16, pool_rows), md in score_kernels.items():
        if pool_rows or (mb, rs, kg) not in ((2, 2, 2), (2, 4, 1), (2, 8, 1)):
            continue
        assert md["vgpr"] + md["agpr"] <= 256, ((d, mb, rs, kg, chunk, sweep, f16), md)
        checked += 1
    # types x sweeps x (d = 128: four chunk lengths, 256 rows and 512 rows with two each;
    # d = 64: the first six)
    assert checked == 2 * 2 * (8 + 6)


def test_no_scoring_kernel_spills(score_kernels):
    """No scratch memory in any matrix-core scoring kernel."""
    for key, md in score_kernels.items():
        assert md["scratch"] == 0, (key, md)
