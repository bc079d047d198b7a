"""Static checks on what the last build produced (no GPU needed): the kernels that hold MFMA accumulator tiles
must not spill -- the MFMAs are inline asm, invisible to the compiler's hazard handling, so a spill store
placed right after one would save a stale register -- and the dominant kernel must keep two wavefronts per
SIMD at f = 100."""
import pytest

from paper_1808_03843_amd import build as B


@pytest.fixture(scope="module")
def res():
    r = B.kernel_resources()
    if not r:
        pytest.skip("no resource reports: run paper_1808_03843_amd/build.py first")
    return r


def test_build_refuses_a_kernel_that_spills(tmp_path):
    # build() itself raises on such a report; fed a made-up report with one spilled register
    import os
    text = ("remark: Function Name: _ZN3als6k_fakeEv\nremark:     VGPRs: 10\nremark:     AGPRs: 0\n"
            "remark:     ScratchSize [bytes/lane]: 0\nremark:     Occupancy [waves/SIMD]: 8\nremark:     VGPRs Spill: 1\n")
    for src in B.SOURCES[:1]:
        with open(os.path.join(tmp_path, src.replace(".hip", ".o") + ".resources"), "w") as fh:
            fh.write(text)
    with pytest.raises(RuntimeError, match="k_fake"):
        B.check_resources(str(tmp_path))


def test_no_kernel_spills_or_uses_scratch(res):
    # every kernel of the library lives in namespace als
    bad = {k: v for k, v in res.items() if k.startswith("_ZN3als") and (v["spill"] or v["scratch"])}
    assert not bad, bad


def test_dominant_kernel_occupancy(res):
    import re
    # fp32 slot storage (the bf16-slot variants need 9 more registers and run one wavefront per SIMD)
    # (element types 0..2: fp32 and the 16-bit inputs; the three-part route, type 3, runs one wavefront per SIMD;
    # last template argument 0: explicit feedback)
    slots = [v for k, v in res.items() if re.search(r"11k_hermitianILi100E[il]Lb[01]ELi[012]ELb0ELi0E", k)]
    fused = [v for k, v in res.items() if re.search(r"14k_hermitian_cgILi100E[il]Lb[01]ELi[012]ELi[01]ELi0E", k)]
    assert slots and fused
    assert all(v["occupancy"] >= 2 for v in slots), slots
    assert all(v["occupancy"] >= 2 for v in fused), fused
