"""Randomised parity: many seeded layouts (odd and aligned sizes, empty tensors, misaligned
tensor addresses), colour counts, contribution counts, sequences and launch options, through
both forms of the step, against the oracle.  MC_RANDOM_CASES raises the number of cases."""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_1711_00705_amd import mc  # noqa: E402
from paper_1711_00705_amd import workloads as wl  # noqa: E402
import gpu_harness as gh  # noqa: E402

N_CASES = int(os.environ.get("MC_RANDOM_CASES", "24"))
OPTS = (mc.OPT_RU_SHAPE, mc.OPT_STATE_POLICY, mc.OPT_PACK_NONTEMPORAL, mc.OPT_STATE_STORE_SC1, mc.OPT_XCD_RUN,
        mc.OPT_XCD_RUN_PACK, mc.OPT_XCD_RUN_UNPACK, mc.OPT_DIRECT_TILES, mc.OPT_LDS_CAP_UPDATE, mc.OPT_LDS_CAP_PACK)


@pytest.fixture(autouse=True)
def _restore_options():
    keep = {o: mc.get_option(o) for o in OPTS}
    yield
    for o, v in keep.items():
        mc.set_option(o, v)
    torch.cuda.synchronize()


def _case(seed):
    rng = np.random.Generator(np.random.PCG64(1000 + seed))
    n = int(rng.integers(1, 40))
    kind = rng.integers(0, 3)
    if kind == 0:      # CNN-like: multiples of four, a few big ones
        sizes = [int(4 * rng.integers(1, 30000)) for _ in range(n)]
    elif kind == 1:    # arbitrary
        sizes = [int(rng.integers(0, 60000)) for _ in range(n)]
    else:              # many small and empty tensors around a large one
        sizes = [int(rng.choice([0, 1, 2, 3, 5, 64, 255, 257])) for _ in range(n)] + [int(rng.integers(1, 400000))]
        rng.shuffle(sizes)
    if sum(sizes) == 0:
        sizes.append(7)
    k = int(rng.choice([1, 2, 3, 4, 8, 33, 100]))
    P = int(rng.choice([1, 2, 3, 4, 5, 8, 11, 32]))
    order = [None, wl.rotation_order(k, P), wl.random_order(k, P, seed=seed)][int(rng.integers(0, 3))]
    misalign = [None, [0], [int(x) for x in rng.integers(0, 4, size=5)]][int(rng.integers(0, 3))]
    opts = {mc.OPT_RU_SHAPE: int(rng.choice([0, 1, 2])), mc.OPT_STATE_POLICY: int(rng.integers(1, 3)),
            mc.OPT_PACK_NONTEMPORAL: int(rng.integers(0, 4)), mc.OPT_STATE_STORE_SC1: int(rng.integers(0, 2))}
    opts[mc.OPT_XCD_RUN] = int(rng.choice([0, 0, 2, 3, 8, 64]))
    opts[mc.OPT_XCD_RUN_PACK] = int(rng.choice([-1, 0, 2, 16, 64]))
    opts[mc.OPT_XCD_RUN_UNPACK] = int(rng.choice([-1, 0, 3, 16]))
    opts[mc.OPT_DIRECT_TILES] = int(rng.integers(0, 3))
    opts[mc.OPT_LDS_CAP_UPDATE] = int(rng.choice([-1, 0, 4096, 40960]))
    opts[mc.OPT_LDS_CAP_PACK] = int(rng.choice([-1, 0, 8192]))
    hyper = [float(x) for x in (rng.choice([0.1, 0.01, 0.5]), rng.choice([0.9, 0.0, 0.5]), rng.choice([1e-4, 0.0, 5e-4]))]
    return sizes, k, P, order, misalign, opts, hyper, rng


@pytest.mark.parametrize("seed", range(N_CASES))
def test_random_case(seed):
    sizes, k, P, order, misalign, opts, (lr, mu, wd), rng = _case(seed)
    for o, v in opts.items():
        mc.set_option(o, v)
    print(f"random case {seed}: n={len(sizes)} N={sum(sizes)} k={k} P={P} misalign={misalign} opts={list(opts.values())}",
          flush=True)
    xs = [[rng.standard_normal(int(s), dtype=np.float32) * np.float32(1e-3) for s in sizes] for _ in range(P)]
    w = [rng.standard_normal(int(s), dtype=np.float32) * np.float32(0.05) for s in sizes]
    v = [rng.standard_normal(int(s), dtype=np.float32) * np.float32(0.01) for s in sizes]
    st = gh.Step(sizes, k)
    gpu, ref = st.run(xs, w, v, lr, mu, wd, order=order, misalign=misalign)
    st.check(gpu, ref, lr, mu, wd, f"staged case {seed}")
    fs = gh.FusedStep(sizes, k)
    gpu, ref = fs.run(xs, w, v, lr, mu, wd, order=order, misalign=misalign if misalign is not None else [0])
    fs.check(gpu, ref, f"fused case {seed}")
