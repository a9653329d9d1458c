"""The entry point that allocates nothing (sk_launch_static) against sk_launch, through the C ABI:
identical bits, on two calls in a row, the second with a smaller input; sizes beyond the static scratch are
refused."""
import numpy as np
import pytest
import torch

import paper_1901_10008_amd as sk
import workloads
from workloads import Problem

import sk_harness as H

pytestmark = pytest.mark.gpu


def _both_ways(b, prm, label):
    with b.plan(**prm) as plan:
        b.reset_outputs()
        sk.sk_launch(plan, H.stream_handle())
        torch.cuda.synchronize()
        want = b.all_output_bits()
    with b.plan(host_only=1, **prm) as plan:
        b.reset_outputs()
        before = torch.cuda.memory_allocated()
        sk.sk_launch_static(plan, H.stream_handle())
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        for i, (x, y) in enumerate(zip(want, b.all_output_bits())):
            assert np.array_equal(x, y), f"{label}: operator {i} differs from sk_launch"
    H.check_against_oracle(b, label)


def test_static_launch_matches_the_allocating_one_twice_in_a_row():
    # split reductions in every class (small tile target): queue, arrival counters and workspace all in use
    big = workloads.config(2, seed=1)[:10] + workloads.config(3, seed=0)[2:7] + workloads.config(4, seed=1)[:6]
    small = workloads.config(2, seed=4)[:5] + workloads.config(3, seed=0)[4:6]
    bb, bs = H.Batch(big, seed=1), H.Batch(small, seed=4)
    _both_ways(bb, {"tile_bytes_min": 8192, "tile_bytes_max": 8192}, "first call, larger input")
    _both_ways(bs, {"tile_bytes_min": 8192, "tile_bytes_max": 8192}, "second call, smaller input")
    _both_ways(bb, {}, "third call, default tiles")
    _both_ways(bs, {"grid_limit": 5}, "fourth call, five workgroups")
    # LDS tiles handed out through the per-die lists: their records and counters live in the scratch as well
    _both_ways(bb, {"xcd_part": 4, "tile_bytes_min": 8192, "tile_bytes_max": 65536}, "fifth call, per-die lists")
    _both_ways(bs, {"xcd_part": 1, "grid_limit": 11}, "sixth call, per-die lists, eleven workgroups")


def test_static_launch_refuses_what_it_cannot_hold_or_serve():
    specs = workloads.config(2, seed=1)[:3]
    b = H.Batch(specs, seed=1)
    with b.plan() as plan:                         # device-resident plan: wrong call
        with pytest.raises(sk.SkError) as e:
            sk.sk_launch_static(plan, H.stream_handle())
        assert e.value.status == sk.SK_ERR_STATE
    with b.plan(host_only=1, stamps=1) as plan:
        with pytest.raises(sk.SkError) as e:
            sk.sk_launch_static(plan, H.stream_handle())
        assert e.value.status == sk.SK_ERR_STATE
    # more workspace than the scratch holds: many split reductions of long rows (host-only plan: the
    # operand addresses are never touched because the call is refused)
    wide = [Problem(op="gemm", dtype="bf16", M=64, N=4096, K=8192) for _ in range(12)]
    fake = []
    addr = 1 << 40
    for s in wide:
        fake.append(sk.make_problem(s, addr, addr + (1 << 30), addr + (2 << 30)))
        addr += 4 << 30
    with sk.sk_plan_create(fake, sk.sk_plan_params_default(host_only=1, tile_bytes_min=4096, tile_bytes_max=4096)) as plan:
        with pytest.raises(sk.SkError) as e:
            sk.sk_launch_static(plan, H.stream_handle())
        assert e.value.status == sk.SK_ERR_UNSUPPORTED and "static scratch" in e.value.detail
    with sk.sk_plan_create([], sk.sk_plan_params_default(host_only=1)) as plan:
        sk.sk_launch_static(plan, H.stream_handle())   # empty plan: nothing to do
    torch.cuda.synchronize()
