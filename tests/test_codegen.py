"""What the hand-scheduled kernels assume of the compiler, checked on the generated gfx950 assembly (no GPU needed).

The tile loops of the prefill kernels (forward and backward) wait for their global -> LDS tile loads with counted
`s_waitcnt vmcnt(N)`: N is the number of loads the source issued after the tile that is needed.  That count is right only
while the compiler puts no vector-memory instruction of its own into those loops (a register spill, a re-read of a
kernel argument structure through global memory): such an instruction would be counted too, and the wait would let a tile
through that has not arrived.  The same loops are scheduled by hand as one stream of MFMAs with the other work dealt
between them, which a spill would also break.  So: in every basic block that holds a stretch of the MFMA stream there is
no vector-memory instruction but the LDS-direct loads and no scratch access.

Second check: no packed fp32 VALU instruction in any kernel of the library (the build switches the feature off).
"""
import os
import re
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2604_24432_amd import build as B

DEVICE_SOURCES = ["ksa_prefill.hip", "ksa_prefill_bwd.hip", "ksa_decode.hip", "ksa_cache.hip"]
MFMA_STREAM = 16          # a block with at least this many MFMAs is a stretch of a tile loop


def _assembly(source: str, out_dir: str) -> str:
    out = os.path.join(out_dir, source + ".s")
    cmd = [B.HIPCC, *B.FLAGS, *B.PER_SOURCE.get(source, []), "-x", "hip", "--cuda-device-only", "-S",
           os.path.join(B.CSRC, source), "-o", out]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    with open(out) as f:
        return f.read()


@pytest.fixture(scope="module")
def assembly():
    if not os.path.exists(B.HIPCC):
        pytest.skip("no hipcc")
    with tempfile.TemporaryDirectory() as d, ThreadPoolExecutor(4) as pool:
        texts = list(pool.map(lambda s: _assembly(s, d), DEVICE_SOURCES))
    return dict(zip(DEVICE_SOURCES, texts))


def _kernels(text: str):
    """{kernel symbol: {block label: [instructions]}} of one assembly file."""
    kernels, name, block = {}, None, None
    for line in text.splitlines():
        m = re.match(r"^(_Z\w+):", line)
        if m:
            name, block = m.group(1), "entry"
            kernels[name] = {block: []}
            continue
        if name is None:
            continue
        if ".end_amdhsa_kernel" in line:
            name = None
            continue
        m = re.match(r"^(\.LBB\d+_\d+):", line)
        if m:
            block = m.group(1)
            kernels[name][block] = []
        elif line.startswith("\t") and not line.strip().startswith((".", ";")):
            kernels[name][block].append(line.strip())
    return kernels


def _is_plain_vector_memory(ins: str) -> bool:
    op = ins.split()[0]
    if op.startswith("scratch_"):
        return True
    if op.startswith(("global_", "flat_", "buffer_")):
        return "lds" not in op        # global_load_lds_*: the tile loads the source issues itself
    return False


@pytest.mark.parametrize("source,kernel_names", [
    ("ksa_prefill.hip", ["ksa_prefill_kernel"]),
    ("ksa_prefill_bwd.hip", ["ksa_bwd_dq_kernel", "ksa_bwd_dkv_kernel"]),
])
def test_tile_loops_hold_only_their_own_tile_loads(assembly, source, kernel_names):
    kernels = _kernels(assembly[source])
    seen = 0
    for name, blocks in kernels.items():
        if not any(k in name for k in kernel_names):
            continue
        hot = {lab: ins for lab, ins in blocks.items() if sum("v_mfma" in i for i in ins) >= MFMA_STREAM}
        assert hot, f"{name}: no MFMA stream found"
        seen += 1
        for lab, ins in hot.items():
            foreign = [i for i in ins if _is_plain_vector_memory(i)]
            assert not foreign, f"{name} {lab}: {foreign[:4]}"
    # head dims 64 and 128, two instantiations each
    assert seen == 4 * len(kernel_names)


def test_tile_loops_load_their_tiles_through_lds_direct_loads(assembly):
    """The check above would pass vacuously if the tile loads were not where it looks."""
    for source in ("ksa_prefill.hip", "ksa_prefill_bwd.hip"):
        for name, blocks in _kernels(assembly[source]).items():
            if "delta" in name or "vt_kernel" in name or "knorm" in name:
                continue
            n = sum(i.startswith("global_load_lds_dwordx4") for lab, ins in blocks.items()
                    if sum("v_mfma" in j for j in ins) >= MFMA_STREAM for i in ins)
            assert n > 0, name


def test_no_packed_fp32_instructions(assembly):
    for source, text in assembly.items():
        found = sorted(set(re.findall(r"\bv_pk_(?:add|mul|fma)_f32\b", text)))
        assert not found, f"{source}: {found}"
