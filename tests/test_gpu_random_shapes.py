"""GPU parity on seeded random layer geometries: kernel sizes, strides, paddings, dilations,
channel counts on and off the tile sizes, every storage type, both output types, all mask
kinds, list given or built inside the call; where the layer can store 8-bit outputs, those
too.  Each case is a pure function of its number, so a failure names the geometry.
FC_RANDOM_CASES=N in the environment runs the first N cases instead of the default 72
(cases 72..3999 were run once that way: all passed, 1216 of them with 8-bit outputs)."""
import os

import numpy as np
import pytest

from oracle import fc_oracle as O
from paper_2207_10741_amd import binding as B, synth
from tests import gpu_util as G
from tests.test_gpu_fp8 import TOL_FP8
from tests.test_gpu_parity import TOL_F32_OUT, _run_layer

pytestmark = pytest.mark.gpu

N_CASES = int(os.environ.get("FC_RANDOM_CASES", "72"))


def _case(i: int):
    g = synth.rng(77, i)
    dtype = [synth.BF16, synth.F16, synth.F32, synth.FP8][i % 4]
    k = int(g.choice([1, 1, 2, 3, 3, 3, 5, 7]))
    s = int(g.choice([1, 1, 1, 2, 2, 3]))
    d = int(g.choice([1, 1, 1, 2])) if k > 1 else 1
    p = int(g.integers(0, d * (k - 1) // 2 + 2))
    if dtype == synth.FP8:
        ci = 16 * int(g.integers(1, 20))
        co = 8 * int(g.integers(1, 40))
        k = min(k, 5)
    else:
        ci = int(g.choice([3, 5, 8, 16, 24, 40, 64, 72, 128, 200, 256]))
        co = int(g.choice([4, 8, 16, 24, 56, 64, 72, 128, 136, 256, 320]))
    # sizes: keep the oracle's work below about 0.15 GMAC
    budget = 1.5e8 / (k * k * ci * co)
    side = int(np.clip(np.sqrt(budget) * s, d * (k - 1) + 1, 96))
    h = int(g.integers(max(d * (k - 1) + 1 - 2 * p, 1, side // 2), side + 1))
    w = int(g.integers(max(d * (k - 1) + 1 - 2 * p, 1, side // 2), side + 1))
    n = int(g.integers(1, 4))
    mask_kind = ["objects", "bernoulli", "band", "mixed", None][int(g.integers(0, 5))]
    irr = float(g.choice([0.1, 0.48, 0.48, 0.8]))
    return dict(layer=(n, h, w, ci, co, k, s, p, d), dtype=dtype, mask_kind=mask_kind, irr=irr,
                relu=bool(g.integers(0, 2)), use_bias=bool(g.integers(0, 2)),
                precomputed=bool(g.integers(0, 2)), seed=300 + i)


@pytest.mark.parametrize("i", range(N_CASES))
def test_random_layer_matches_oracle(i):
    c = _case(i)
    print("case", i, c, flush=True)
    out, want, keep = _run_layer(*c["layer"], c["dtype"], irr=c["irr"], relu=c["relu"], use_bias=c["use_bias"],
                                 mask_kind=c["mask_kind"], seed=c["seed"], precomputed=c["precomputed"])
    tol = TOL_FP8 if c["dtype"] == synth.FP8 else TOL_F32_OUT
    assert G.rel_err(G.to_f64(out), want, keep) <= tol
    f32 = out.cpu().numpy()
    assert not f32[~keep].view(np.uint32).any()
    # 8-bit output, where the matrix-core or stem kernel takes the layer: the codes are the
    # oracle's narrowing of the fp32 output above
    n, h, w, ci, co, k, s, p, d = c["layer"]
    es = 1 if c["dtype"] == synth.FP8 else 2
    if c["dtype"] != synth.F32 and co % 16 == 0 and k * k <= 32 and \
            ((ci * es) % 16 == 0 or (ci <= 4 and c["dtype"] != synth.FP8)):
        out8, _, _ = _run_layer(*c["layer"], c["dtype"], irr=c["irr"], relu=c["relu"], use_bias=c["use_bias"],
                                mask_kind=c["mask_kind"], seed=c["seed"], precomputed=c["precomputed"],
                                out_dtype=B.FP8)
        expect = O.narrow_fp8(f32.astype(np.float64))
        if c["relu"]:
            expect[f32 == 0] = 0        # the sign-bit rule stores +0 for -0
        got = out8.view(G.torch_mod().uint8).cpu().numpy()
        np.testing.assert_array_equal(got[keep], expect[keep])
        assert not got[~keep].any()
