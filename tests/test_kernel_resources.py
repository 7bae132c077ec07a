"""What the compiler made of the kernels (registers, scratch, LDS), from the resource-usage remarks
the build collects.  A register spill inside the block loop of the fused kernel is not a
correctness problem but a performance cliff (its reload waits on the same counter as the
asynchronous copies of the next key block), and nothing else would notice it: so it is pinned here."""
import re

import pytest

from paper_2603_09582_amd import build

# fused_kernel<DK, MODE, NB, WIDE> variants that are known to spill a few registers: head dimension
# above 96 with the per-block relative-position table, and the single-launch form with a bias that
# is read straight into registers.  Neither is on a benchmarked path.
KNOWN_SPILLS = {(4, 13, 1, 0), (4, 1, 2, 1)}


def fused_variants():
    res = build.kernel_resources()
    if not res:
        pytest.skip("no build in this tree yet (python -m paper_2603_09582_amd.build)")
    out = {}
    for name, r in res.items():
        m = re.match(r"_ZN7binattn12fused_kernelILi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)EEEv", name)
        if m:
            out[tuple(int(x) for x in m.groups())] = r
    return out


def test_fused_kernels_do_not_spill_and_keep_two_waves_per_simd():
    fv = fused_variants()
    assert len(fv) >= 40
    for key, r in sorted(fv.items()):
        assert r["waves_per_simd"] >= 2, (key, r)
        assert r["lds_bytes"] <= 160 * 1024, (key, r)
        if key in KNOWN_SPILLS:
            assert r["scratch_bytes"] <= 160, (key, r)
        else:
            assert r["scratch_bytes"] == 0, (key, r)


def test_headline_kernels_have_the_expected_shape():
    fv = fused_variants()
    pair = fv[(2, 5, 2, 0)]          # d = 64, LDS bias tiles shared by two batch entries (long sequences)
    assert pair["vgprs"] <= 256 and pair["scratch_bytes"] == 0 and 100 * 1024 <= pair["lds_bytes"] <= 128 * 1024
    dit = fv[(3, 5, 1, 0)]           # d = 72, private bias tiles, two workgroups per compute unit
    assert dit["scratch_bytes"] == 0 and dit["lds_bytes"] <= 80 * 1024


def test_four_wave_single_launch_kernels_fit_two_per_compute_unit():
    fv = fused_variants()
    four = {k: r for k, r in fv.items() if k[3] == 3}   # WIDE_ONEHEAD4
    assert len(four) >= 18
    for key, r in sorted(four.items()):
        assert key[2] == 1 and key[0] <= 3, key
        assert r["scratch_bytes"] == 0 and r["lds_bytes"] <= 80 * 1024, (key, r)
