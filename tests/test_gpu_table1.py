"""The paper's own kernel-level workloads on the GPU (Section 4.1, Table 1): R tenants of identical shape, each with its
own weights and inputs, for the three problem shapes of Table 1 expressed as convolutions (M=256, N=128, K=1152 as a
3x3 convolution; 256x256x256 and 512x1x512 as 1x1 convolutions), in fp32 (the paper's precision) and bf16, under the
three issue policies, every output element against the fp64 oracle.  The tensors are those bench.py --paper-sweep
times (seeded generator, stream key 41)."""
import numpy as np
import pytest

from paper_1901_00041_amd import st_conv as sc
from paper_1901_00041_amd import synth
from paper_1901_00041_amd.synth import ConvShape

pytestmark = pytest.mark.gpu

TABLE1 = {"conv": (1, 128, 16, 16, 128, 3, 3, 1, 1), "matvec": (1, 512, 1, 1, 512, 1, 1, 1, 0), "square": (1, 256, 16, 16, 256, 1, 1, 1, 0)}
KEY = 41


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name", ["conv", "matvec", "square"])
@pytest.mark.parametrize("R", [2, 10, 120])
def test_table1_shapes_all_policies(name, R, dtype):
    import torch
    from tests import helpers
    assert torch.cuda.is_available()
    N, C, H, W, K, R_, S_, st, pd = TABLE1[name]
    shape = ConvShape(N, C, H, W, K, R_, S_, st, pd, dtype, "f32")
    assert shape.gemm == {"conv": (256, 128, 1152), "matvec": (1, 512, 512), "square": (256, 256, 256)}[name]
    tenants = [helpers.Tenant(shape, synth.gen_input(KEY, t, 0, shape), synth.gen_weight(KEY, t, 0, shape)) for t in range(R)]
    refs = [t.reference() for t in tenants]
    plan = helpers.plan_for(tenants)
    solo = [helpers.plan_for([t]) for t in tenants]
    streams = [torch.cuda.Stream() for _ in range(min(R, 16))]
    runs = {"fused": lambda: sc.st_conv_run(plan),
            "time-only": lambda: sc.st_conv_run_time_only(plan),
            "space-only": lambda: sc.st_conv_run_space_only(plan, streams),
            "time-only, each tenant planned alone": lambda: sc.st_conv_run_plans_time_only(solo),
            "space-only, each tenant planned alone": lambda: sc.st_conv_run_plans_space_only(solo, streams)}
    worst = 0.0
    for label, run in runs.items():
        for t in tenants:
            t.clear()
        run()
        torch.cuda.synchronize()
        for i, t in enumerate(tenants):
            got = t.result()
            assert np.isfinite(got).all(), f"{name} R={R} {dtype} {label}: tenant {i} has unwritten outputs"
            err = np.abs(got - refs[i])
            tol = helpers.tolerance(shape, refs[i])
            assert (err <= tol).all(), f"{name} R={R} {dtype} {label}: tenant {i} max err {err.max():.3e}"
            worst = max(worst, float(err.max()))
    # tenants share a shape, not their numbers
    assert not np.array_equal(tenants[0].result(), tenants[1].result())
    print(f"table 1 {name} R={R} {dtype}: worst |gpu-oracle| = {worst:.3e}")
