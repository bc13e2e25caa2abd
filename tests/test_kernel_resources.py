"""The compiler's resource usage of the hot kernels stays where it was measured: a change that makes one of
them spill (a few more live registers under a launch bound) costs a multiple of its run time and no parity
test notices.  CPU only: hipcc cross-compiles the sources with -Rpass-analysis=kernel-resource-usage."""
import shutil

import pytest

from paper_2410_09397_amd import pmc_summary

# scratch bytes per lane that each kernel is allowed: the d = 64 forward and dQ kernels keep their
# 4-workgroups-per-CU launch bound and spill 7 and 3 registers (measured faster than the build without scratch)
ALLOWED_SCRATCH = {"fwd_kernel<64>": 28, "bwd_dq_kernel<64, 1>": 12}
MIN_OCCUPANCY = {"fwd_kernel<64>": 4, "bwd_dq_kernel<64, 1>": 4, "bwd_dkdv_kernel<64>": 3, "fwd_kernel<128>": 2,
                 "bwd_dq_kernel<128, 1>": 2, "bwd_dkdv_kernel<128>": 2}


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_hot_kernels_keep_their_registers_and_do_not_spill():
    seen = {r["kernel"]: r for r in pmc_summary.kernel_resources()}  # every kernel of the library
    assert set(MIN_OCCUPANCY) <= set(seen), sorted(seen)
    for name, r in seen.items():
        assert int(r["ScratchSize [bytes/lane]"]) <= ALLOWED_SCRATCH.get(name, 0), (name, r)
        if name in MIN_OCCUPANCY:
            assert int(r["Occupancy [waves/SIMD]"]) >= MIN_OCCUPANCY[name], (name, r)
