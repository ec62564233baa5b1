"""lutq_matmul_static (the entry point that allocates nothing: arrival counters and partial sums live in
a device array of the library's own) against lutq_matmul_plan on a caller's workspace: the same plan
gives the same bits.  Two calls in a row share the built-in array, the second on a smaller problem;
the plans cut output tiles across workgroups, so both the counters and the partial-sum slots are used."""
import numpy as np
import pytest

import lutq_inputs as gen
from oracle import lutq_oracle as orc
from gpu_util import DeviceCase, to_bits

pytestmark = pytest.mark.gpu


def _both(lutq, c, plan):
    import torch
    d = DeviceCase(lutq, c)
    want = to_bits(d.matmul(lutq, plan=plan))
    Y = torch.full((c.M, c.N), float("nan"), dtype=d.X.dtype, device="cuda")
    import gc
    gc.collect()
    before = torch.cuda.memory_allocated()
    lutq.lutq_matmul_static(d.X, d.packed, d.S, d.T, c.bits, c.group_size, Y, plan=plan)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() <= before          # nothing was allocated through torch either
    return to_bits(Y), want


def test_static_scratch_matches_workspace_call(lutq):
    import torch
    # (M, N, K, bits, dtype, plan): a large split problem first, then smaller ones on the same array
    specs = [(3, 2048, 4096, 4, "f16", lutq.Plan(1, 250, 8, 2, 2)),
             (1, 256, 2048, 4, "f16", lutq.Plan(1, 7, 8, 2, 1)),
             (17, 192, 1024, 3, "bf16", lutq.Plan(2, 5, 8, 2, 2)),
             (32, 128, 1024, 2, "f16", lutq.Plan(1, 3, 8, 2, 8)),
             (1, 4096, 4096, 4, "f16", None),
             (40, 208, 2048, 4, "bf16", lutq.Plan(1, 5, 8, 2, 1)),
             # 64-row slices: the operand-order copy of the activations lives in the same array
             (64, 4800, 1024, 4, "f16", None),
             (100, 208, 2048, 4, "bf16", lutq.Plan(scheduling=3)),
             # K slices on the row-streaming kernel: the slices' sums and the arrival counters live there too
             (20, 208, 2048, 4, "f16", lutq.Plan(4, 16, 8, 2, 3, 3, 4)),
             (32, 4096, 14336, 4, "bf16", None)]
    for rnd in range(2):
        for i, (M, N, K, bits, dtype, plan) in enumerate(specs):
            c = gen.make_case(900 + i, M, N, K, bits, 64, dtype, "nf")
            got, want = _both(lutq, c, plan)
            assert np.array_equal(got, want), f"round {rnd} case {i}: {np.count_nonzero(got != want)} of {want.size} differ"
            if rnd == 0:
                What = orc.dequant(c.Q, c.T, c.S, c.group_size, dtype)
                err = orc.rel_fro_err(orc.to_f64(got, dtype), orc.matmul_f64(c.X, What, dtype))
                assert err <= (2e-3 if dtype == "f16" else 2.0 ** -8), (i, err)


def test_static_scratch_rejects_what_does_not_fit(lutq):
    import torch
    # 4096 workgroups x 2 ends x R = 4 x two halves of M x 1 KiB = 64 MiB of partial sums: beyond the 16 MiB
    M, N, K, bits = 32, 4096, 16384, 4
    c = gen.make_case(7, M, 64, K, bits, 128, "f16", "random_index")
    d = DeviceCase(lutq, gen.Case(M, 64, K, bits, 128, "f16", c.X, c.Q, c.S, c.T))
    Q = np.tile(c.Q, (N // 64, 1))
    S = np.tile(c.S, (N // 64, 1))
    big = DeviceCase(lutq, gen.Case(M, N, K, bits, 128, "f16", c.X, Q, S, c.T))
    Y = torch.full((M, N), 7.0, dtype=torch.float16, device="cuda")
    with pytest.raises(lutq.LutqError) as e:
        lutq.lutq_matmul_static(big.X, big.packed, big.S, big.T, bits, 128, Y, plan=lutq.Plan(4, 4095, 4, 2, 1))
    assert e.value.code == 11
    torch.cuda.synchronize()
    assert (Y == 7.0).all().item()
    # the same plan is fine on a caller's workspace, and an unsplit plan is fine on the built-in scratch
    big.matmul(lutq, plan=lutq.Plan(4, 4095, 4, 2, 1))
    lutq.lutq_matmul_static(big.X, big.packed, big.S, big.T, bits, 128, Y, plan=lutq.Plan(4, 64, 4, 2, 1))
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(Y), to_bits(big.matmul(lutq, plan=lutq.Plan(4, 64, 4, 2, 1))))


def test_static_scratch_falls_back_to_a_default_that_fits(lutq):
    """Where the library's own plan would need more partial-sum scratch than the built-in array holds (70B
    gate+up, bf16, M = 32: fourteen teams with every tile cut in two, 28 MiB of slots), the call without a
    plan takes the library's low-scratch choice instead of failing: the same bits as that plan on a
    workspace (seven teams, no cut), while the plan that does not fit is refused when asked for by name."""
    import torch
    M, N, K, bits, group = 32, 57344, 8192, 4, 64
    small = gen.make_case(5, M, 64, K, bits, group, "bf16", "random_index")
    c = gen.Case(M, N, K, bits, group, "bf16", small.X, np.tile(small.Q, (N // 64, 1)), np.tile(small.S, (N // 64, 1)), small.T)
    d = DeviceCase(lutq, c)
    assert lutq.lutq_plan_default(bits, group, M, N, K, 1).row_groups_per_workgroup == 14
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    lutq.lutq_matmul_static(d.X, d.packed, d.S, d.T, bits, group, Y)
    torch.cuda.synchronize()
    want = to_bits(d.matmul(lutq, plan=lutq.Plan(2, 256, 7, 2, 7)))
    assert np.array_equal(to_bits(Y), want)
    with pytest.raises(lutq.LutqError) as e:
        lutq.lutq_matmul_static(d.X, d.packed, d.S, d.T, bits, group, Y, plan=lutq.Plan(2, 256, 14, 2, 14))
    assert e.value.code == 11

