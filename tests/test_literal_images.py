"""CPU checks of the build step behind the weights-as-literals kernels: the placeholder constants are distinct and never
an inline constant of the instruction set, every code object lists every weight, and writing a weight set over the
listed places leaves no placeholder behind and touches nothing else."""
import os
import struct

import numpy as np
import pytest

from paper_1508_01292_amd import build as B


def test_placeholders_are_distinct_ordinary_floats():
    bits = [B.placeholder_bits(i) for i in range(4096)]
    assert len(set(bits)) == len(bits)
    vals = np.array(bits, np.uint32).view(np.float32)
    assert np.all(vals > 0.5) and np.all(vals < 0.75)          # no inline constant (0.5, 1, 2, 4, 1/(2 pi), integers) in there


@pytest.mark.parametrize("spec", B.LITERAL_IMAGES, ids=[s[0] for s in B.LITERAL_IMAGES])
def test_code_object_lists_every_weight_and_patches_cleanly(spec):
    src, _inc, _image, _patch, n = spec
    path = B.literal_code_object(src)
    if not os.path.exists(path):
        pytest.skip("library not built here")
    blob = open(path, "rb").read()
    patches = B.literal_patch_table(blob, n, src)
    assert {i for _, i in patches} == set(range(n))
    assert all(o % 4 == 0 and 0 <= o <= len(blob) - 4 for o, _ in patches) and len({o for o, _ in patches}) == len(patches)
    # write a weight set over the placeholders, as the library does when a context is created
    rng = np.random.default_rng(3)
    w = rng.normal(size=n).astype(np.float32)
    out = bytearray(blob)
    for o, i in patches:
        out[o:o + 4] = struct.pack("<f", float(w[i]))
    keys = {B.placeholder_bits(i) for i in range(n)}
    left = [o for o in range(0, len(out) - 3, 4) if struct.unpack_from("<I", out, o)[0] in keys]
    assert not left
    changed = [o for o in range(0, len(out) - 3, 4) if out[o:o + 4] != blob[o:o + 4]]
    assert set(changed) <= {o for o, _ in patches}
    for o, i in patches[:: max(1, len(patches) // 50)]:
        assert struct.unpack_from("<f", out, o)[0] == w[i]
