"""What the compiler cannot check about the GEMM kernels' inline assembly (matrix instructions, LDS copies) is
checked on the generated gfx950 assembly instead: wait states after accumulator initialisation, scalar base
addresses of the copies, no accumulator copies around MFMAs, no scratch on the throughput path.  CPU only
(cross-compilation); takes about a minute and a half."""
import os

import pytest

from paper_2408_02897_amd import build


@pytest.mark.skipif(not os.path.exists(build.HIPCC), reason="hipcc not installed")
def test_gemm_assembly_is_clean():
    kernels, findings = build.check_asm()
    assert len(kernels) >= 40                 # every instantiation of gemm_kernel and gemm_shortk_kernel was seen
    assert findings == []
