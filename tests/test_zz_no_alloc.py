"""ecc_hard_static (the entry point that allocates nothing: its scratch is a static device array
inside the library) against ecc_hard on the same inputs, bit-exact, on two calls in a row, the
second on a smaller input; and its size limit."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2510_20271_amd import api, synth
from tests.gpu_util import dev, host

pytestmark = pytest.mark.gpu


def test_static_scratch_two_calls_in_a_row():
    bins = 200
    big = dev(np.stack([synth.grf((600, 1000), 2.0, 11 + i) for i in range(3)]))      # single-pass list sweep
    small = dev(synth.grf((40, 50, 70), 1.5, 5)[None])                               # 3D, smaller
    tiny = dev(np.random.default_rng(1).integers(0, 200, (2, 30, 40), dtype=np.uint8))  # levels, the flow for small inputs
    curve = torch.empty((3, bins), dtype=torch.int64, device="cuda")
    for _ in range(2):  # the scratch keeps the last call's contents: a second round must not see them
        a = api.ecc_hard_static(big, 2, bins, curve=curve)
        assert a.data_ptr() == curve.data_ptr()
        np.testing.assert_array_equal(host(a), host(api.ecc_hard(big, 2, bins)))
        np.testing.assert_array_equal(host(api.ecc_hard_static(small, 3, bins)), host(api.ecc_hard(small, 3, bins)))
        np.testing.assert_array_equal(host(api.ecc_hard_static(tiny, 2, bins)), host(api.ecc_hard(tiny, 2, bins)))
        np.testing.assert_array_equal(host(api.ecc_hard_static(small, 3, bins, range=(-0.2, 0.3))),
                                      host(api.ecc_hard(small, 3, bins, range=(-0.2, 0.3))))
    # rough field: most vertices are critical (long lists), all inside the scratch
    rough = dev(np.random.default_rng(2).standard_normal((2, 300, 1000)).astype(np.float32))
    np.testing.assert_array_equal(host(api.ecc_hard_static(rough, 2, bins)), host(api.ecc_hard(rough, 2, bins)))
    # a converted element type (float16 -> float32 copy inside the scratch)
    half = big[:1].half()
    np.testing.assert_array_equal(host(api.ecc_hard_static(half, 2, bins)), host(api.ecc_hard(half, 2, bins)))


def test_static_scratch_rejects_what_does_not_fit():
    n = 6144  # 6144^2 float32 vertices need more than 32 MiB of lists
    g = torch.zeros((1, n, n), dtype=torch.float32, device="cuda")
    assert api.ecc_workspace_bytes((n, n), 1, 64) > 32 << 20
    with pytest.raises(api.EccError) as e:
        api.ecc_hard_static(g, 2, 64)
    assert e.value.status == -2 and "scratch" in str(e.value)
