"""GPU parity: the HIP executor against the CPU oracle, bit for bit, through the C ABI.

Tolerance: 0 ulp.  Copies and int32 sums are exact by nature; fp32 / fp16 sums are compared
bitwise because the schedule fixes the order of every addition and both sides add in fp32
and (fp16) narrow once per reduce group with round-to-nearest-even.
"""
import numpy as np
import pytest

from gpu_util import NP, assert_same_bits, bits, host_inputs, run_both
from helpers import to_binding
from oracle import collective as col
from oracle import generate as gen
from oracle import topology as tp
from oracle.schedule import COPY, REDUCE, make_schedule
from oracle.validate import validate
from paper_2008_08708_amd import inputs, sccl

pytestmark = pytest.mark.gpu


def allreduce_of(topo, C, kind="greedy"):
    ag = col.allgather(topo.num_nodes, C)
    base = gen.ring_allgather(topo.num_nodes, C) if kind == "ring" else gen.greedy_bfs(topo, ag)
    return gen.compose_allreduce(base, ag)


def test_config1_allgather_ring4_exact():
    topo, ag = tp.ring(4), col.allgather(4, 1)
    s = gen.greedy_bfs(topo, ag)
    bufs = host_inputs("uniform", "f32", 1, 4, 4, 1024, ag.pre)
    want, got = run_both(topo, ag, s, "f32", bufs, 1024, label="cfg1")
    assert_same_bits(want, got)
    for n in range(4):                                    # closed form: out[n][c] = in[c mod P][c]
        assert not inputs.is_poison(got[n]).any()
        for c in range(4):
            assert (bits(got[n][c * 1024:(c + 1) * 1024]) == bits(bufs[c % 4][c * 1024:(c + 1) * 1024])).all()


# sizes: several tiles of 256 lanes x 2 vectors x 16 B plus a ragged tail; element counts that force
# every vector width (16, 8, 4, 2 bytes)
RAGGED = [
    ("cfg2-like", tp.hcm8(), 2, "allgather", "greedy", "i32", "u32", 3 * 2048 + 4 * 37),
    ("cfg2-w8", tp.hcm8(), 2, "allgather", "greedy", "i32", "u32", 2 * 2048 + 2 * 33),
    ("cfg2-w4", tp.hcm8(), 2, "allgather", "greedy", "i32", "u32", 1031),
    ("cfg3-like", tp.hcm8(), 1, "allreduce", "greedy", "f32", "uniform", 5 * 2048 + 4 * 101),
    ("cfg3-w4", tp.hcm8(), 1, "allreduce", "greedy", "f32", "uniform", 2 * 2048 + 13),
    ("cfg4-like", tp.ring(8), 4, "allreduce", "ring", "f16", "normal", 3 * 4096 + 8 * 77),
    ("cfg4-paper-row", tp.ring(8), 2, "allreduce", "ring", "f16", "normal", 4096 + 8 * 5),
    ("cfg4-w8", tp.ring(8), 4, "allreduce", "ring", "f16", "normal", 4096 + 4 * 9),
    ("cfg4-w2", tp.ring(8), 4, "allreduce", "ring", "f16", "normal", 777),
    ("cfg5-ag", tp.torus2d(4, 4), 4, "allgather", "greedy", "f32", "uniform", 2048 + 4 * 3),
    ("cfg5-ar", tp.torus2d(4, 4), 4, "allreduce", "greedy", "f32", "uniform", 2048 + 4 * 3),
    ("cfg5-tiny", tp.torus2d(4, 4), 4, "allreduce", "greedy", "f32", "uniform", 4),
    ("cfg5-one", tp.torus2d(4, 4), 4, "allreduce", "greedy", "f32", "uniform", 1),
    ("dgx1-rs", tp.dgx1(), 2, "reducescatter", "greedy", "f32", "uniform", 2048 + 4),
    ("int-ar", tp.hcm8(), 1, "allreduce", "greedy", "i32", "u32", 2048 + 12),
    ("f16-uniform", tp.hcm8(), 1, "allreduce", "greedy", "f16", "uniform", 4096 + 24),
]


@pytest.mark.parametrize("label,topo,C,what,kind,dtype,dist,epc", RAGGED, ids=[r[0] for r in RAGGED])
def test_small_configs_bitwise(label, topo, C, what, kind, dtype, dist, epc):
    P = topo.num_nodes
    ag = col.allgather(P, C)
    base = gen.ring_allgather(P, C) if kind == "ring" else gen.greedy_bfs(topo, ag)
    if what == "allgather":
        coll, sched = ag, base
    elif what == "allreduce":
        sched, coll = gen.compose_allreduce(base, ag)
    else:
        sched, coll = gen.reducescatter_from(base, ag)
    assert validate(topo, coll, sched).ok
    bufs = host_inputs(dist, dtype, 17, P, coll.num_chunks, epc, ag.pre if what == "allgather" else None)
    want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=label)
    assert_same_bits(want, got)          # whole buffers, partial sums left behind included
    if what == "allreduce":
        for g in got[1:]:
            assert (bits(g) == bits(got[0])).all()
        assert not np.isnan(got[0].astype(np.float64)).any()


@pytest.mark.parametrize("block", [64, 128, 256])
@pytest.mark.parametrize("vpt", [1, 2, 4])
@pytest.mark.parametrize("dtype,dist", [("f32", "uniform"), ("f16", "normal")])
def test_every_launch_shape(block, vpt, dtype, dist):
    topo = tp.hcm8()
    sched, coll = allreduce_of(topo, 1)
    epc = 3 * 1024 * (4 if dtype == "f32" else 8) + 4 * 19
    bufs = host_inputs(dist, dtype, 23, 8, coll.num_chunks, epc)
    want, got = run_both(topo, coll, sched, dtype, bufs, epc,
                         options={"block_threads": block, "vectors_per_thread": vpt}, label="shape")
    assert_same_bits(want, got)


def test_single_workgroup_walks_every_item():
    topo = tp.hcm8()
    sched, coll = allreduce_of(topo, 1)
    epc = 4 * 2048 + 8
    bufs = host_inputs("uniform", "f32", 29, 8, coll.num_chunks, epc)
    want, got = run_both(topo, coll, sched, "f32", bufs, epc, options={"max_workgroups": 1}, label="one-wg")
    assert_same_bits(want, got)
    want, got = run_both(topo, coll, sched, "f32", bufs, epc, options={"max_workgroups": 3}, label="three-wg")
    assert_same_bits(want, got)


@pytest.mark.parametrize("P", [2, 8, 12, 16])
@pytest.mark.parametrize("dtype,dist", [("f32", "uniform"), ("f16", "normal"), ("i32", "u32")])
def test_large_fan_in_and_fan_out(P, dtype, dist):
    # on K_P the greedy Allgather takes one step, so the Allreduce has fan-in P-1 (batches of 4 in the kernel)
    topo = tp.complete(P)
    sched, coll = allreduce_of(topo, 1)
    assert sched.num_steps == 2
    epc = 1024 + 8
    bufs = host_inputs(dist, dtype, 31, P, coll.num_chunks, epc)
    want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=f"K{P}")
    assert_same_bits(want, got)


def test_sixty_four_ranks():
    topo = tp.ring(64)
    ag = col.allgather(64, 1)
    s = gen.greedy_bfs(topo, ag)
    bufs = host_inputs("u32", "i32", 37, 64, 64, 68, ag.pre)
    want, got = run_both(topo, ag, s, "i32", bufs, 68, label="ring64")
    assert_same_bits(want, got)


def test_sixty_four_ranks_fan_in_sixty_three():
    # K64: every reduce group has 63 sources (batches of four in one kernel, an overflow list in the other)
    topo = tp.complete(64)
    sched, coll = allreduce_of(topo, 1)
    assert sched.num_steps == 2
    for dtype, dist, epc in (("f32", "uniform", 4 * 5 + 4), ("f16", "normal", 8 * 3)):
        bufs = host_inputs(dist, dtype, 41, 64, coll.num_chunks, epc)
        want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=f"K64-{dtype}")
        assert_same_bits(want, got)
        for g in got[1:]:
            assert (bits(g) == bits(got[0])).all()


def test_addition_order_inside_a_group_is_the_schedules():
    t = tp.complete(4)
    ar = col.allreduce(4, 1)
    x = [np.float32(1.0), np.float32(2.0 ** -24), np.float32(2.0 ** -24), np.float32(-1.0)]
    outs = []
    for order in ([1, 2, 3], [3, 1, 2]):
        sends = [(0, n, 0, 0, REDUCE) for n in order] + [(0, 0, n, 1, COPY) for n in (1, 2, 3)]
        s = make_schedule([1, 1], sends)
        bufs = [np.full(4, v, dtype=np.float32) for v in x]
        want, got = run_both(t, ar, s, "f32", bufs, 4, label=f"order{order}")
        assert_same_bits(want, got)
        outs.append(got[0][0])
    assert outs[0] == np.float32(0.0) and outs[1] == np.float32(2.0 ** -23)


@pytest.mark.parametrize("dtype,epc", [("f32", 2048 + 4 * 3), ("f16", 4096 + 8 * 5)])
def test_wide_range_inputs_where_every_order_of_additions_has_other_bits(dtype, epc):
    # neighbouring elements differ by up to 24 binades (12 for fp16): almost every partial sum rounds, so any change
    # of the order of additions -- inside a group or across the levels of a chunk's tree -- changes bits somewhere
    for topo, C, kind in ((tp.torus2d(4, 4), 4, "greedy"), (tp.hcm8(), 1, "greedy"), (tp.ring(8), 2, "ring")):
        sched, coll = allreduce_of(topo, C, kind)
        bufs = host_inputs("wide", dtype, 29, topo.num_nodes, coll.num_chunks, epc)
        want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=f"wide-{topo.name}-{dtype}")
        assert_same_bits(want, got)
        for g in got[1:]:
            assert (bits(g) == bits(got[0])).all()


def test_fp16_rounding_points_and_special_values():
    t = tp.complete(3)
    ar = col.allreduce(3, 1)
    one_group = make_schedule([1, 1], [(0, 1, 0, 0, REDUCE), (0, 2, 0, 0, REDUCE), (0, 0, 1, 1, COPY), (0, 0, 2, 1, COPY)])
    two_steps = make_schedule([1, 1, 1], [(0, 1, 0, 0, REDUCE), (0, 2, 0, 1, REDUCE), (0, 0, 1, 2, COPY), (0, 0, 2, 2, COPY)])
    # columns: narrowing once (2050), ties to even (2049 -> 2048, 2051 -> 2052), overflow to inf at 65520,
    # largest finite stays finite, subnormals survive, signed zero, fp16 subnormal sum
    a = np.array([2048, 2048, 2050, 65504, 65504, 2.0 ** -24, -0.0, 2.0 ** -24, 1.0], dtype=np.float16)
    b = np.array([1, 1, 1, 16, 8, 0, 0.0, 2.0 ** -24, 2.0 ** -11], dtype=np.float16)
    c = np.array([1, 0, 0, 0, 0, 0, -0.0, 2.0 ** -24, 0], dtype=np.float16)
    pad = 8 - a.size % 8
    bufs = [np.concatenate([v, np.zeros(pad, np.float16)]) for v in (a, b, c)]
    for s, label in ((one_group, "f16-one-group"), (two_steps, "f16-two-steps")):
        want, got = run_both(t, ar, s, "f16", bufs, bufs[0].size, label=label)
        assert_same_bits(want, got)
        if s is one_group:
            assert got[0][0] == np.float16(2050) and got[0][1] == np.float16(2048) and got[0][2] == np.float16(2052)
            assert np.isinf(got[0][3]) and got[0][4] == np.float16(65504)
            assert got[0][5] == np.float16(2.0 ** -24) and got[0][7] == np.float16(3 * 2.0 ** -24)
            assert got[0][8] == np.float16(1.0)
        else:
            assert got[0][0] == np.float16(2048)          # rounded between the steps


def test_fp32_denormals_are_kept():
    t = tp.complete(2)
    ar = col.allreduce(2, 1)
    s = make_schedule([1, 1], [(0, 1, 0, 0, REDUCE), (0, 0, 1, 1, COPY)])
    a = np.array([1e-45, 1e-40, 2.0 ** -126, -1e-45], dtype=np.float32)
    b = np.array([0.0, 1e-40, -(2.0 ** -127), 1e-45], dtype=np.float32)
    want, got = run_both(t, ar, s, "f32", [a, b], 4, label="denormal")
    assert_same_bits(want, got)
    assert got[0][0] == np.float32(1e-45) and got[0][0] != 0


def test_empty_chunks_and_error_paths():
    import torch
    topo, ag = tp.ring(4), col.allgather(4, 1)
    s = gen.greedy_bfs(topo, ag)
    print("[case] empty chunks", flush=True)
    plan = sccl.sccl_plan_create(*to_binding(topo, ag, s, "f32", 0))
    bufs = [torch.zeros(16, dtype=torch.float32, device="cuda") for _ in range(4)]
    sccl.sccl_execute(plan, bufs)                 # nothing to move: OK without a launch
    sccl.sccl_plan_destroy(plan)
    plan = sccl.sccl_plan_create(*to_binding(topo, ag, s, "f32", 8))
    big = torch.zeros(4 * 32 + 8, dtype=torch.float32, device="cuda")
    good = [big[i * 32:(i + 1) * 32] for i in range(4)]
    sccl.sccl_execute(plan, good)
    with pytest.raises(sccl.ScclError) as e:      # 4-byte offset: not 16-byte aligned
        sccl.sccl_execute(plan, [big[1:33]] + good[1:])
    assert e.value.name == "SCCL_ERR_ALIGNMENT"
    with pytest.raises(sccl.ScclError) as e:      # ranks 0 and 1 overlap by half a buffer
        sccl.sccl_execute(plan, [big[0:32], big[16:48], big[64:96], big[96:128]])
    assert e.value.name == "SCCL_ERR_OVERLAP"
    with pytest.raises(sccl.ScclError) as e:
        sccl.sccl_execute(plan, [good[0], good[0], good[2], good[3]])
    assert e.value.name == "SCCL_ERR_OVERLAP"
    with pytest.raises(sccl.ScclError) as e:
        sccl.sccl_execute(plan, [0] + good[1:])
    assert e.value.name == "SCCL_ERR_INVALID_ARG"
    torch.cuda.synchronize()
    sccl.sccl_plan_destroy(plan)


def test_device_generator_matches_host_generator():
    import torch
    for dist, dtype in (("u32", "i32"), ("uniform", "f32"), ("smallint", "f16"), ("uniform", "f16")):
        a = inputs.generate(dist, dtype, 5, 3, 1000, 5000)
        b = inputs.torch_generate(dist, dtype, 5, 3, 1000, 5000, "cuda").cpu().numpy()
        assert (bits(a) == bits(b)).all()


def test_streaming_kernels_of_the_benchmark_move_what_they_say():
    # bench.py's measurement aids (not part of the library): a copy is a copy, a fan-out writes k copies, a fan-in sums
    import torch
    import bench
    n = 3 * 32768                                           # bytes per region: three tiles
    src = torch.randint(0, 1 << 30, (8 * n // 4,), dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    bench.bench_stream("copy", dst, src, 8 * n, grid=2)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    dst.zero_()
    bench.bench_stream("fanout", dst, src, n, k=7, grid=5)
    torch.cuda.synchronize()
    assert torch.equal(dst.view(8, -1)[:7], src.view(8, -1)[:1].expand(7, -1)) and not dst.view(8, -1)[7].any()
    bench.bench_stream("fanin", dst, src, n, k=8, grid=3)
    torch.cuda.synchronize()
    assert torch.equal(dst.view(8, -1)[0], src.view(8, -1).sum(0, dtype=torch.int32))


def test_synthesized_schedules_with_several_rounds_per_step():
    # k > 0 schedules from the exact search: (2,2,3) on the DGX-1 graph -> Allreduce (16,4,6); (2,4,7) on the 8-ring
    from oracle import synthesize as syn
    for topo, (C, S, R), dtype, dist in ((tp.dgx1(), (2, 2, 3), "f32", "uniform"), (tp.ring(8), (2, 4, 7), "f16", "normal")):
        ag = col.allgather(8, C)
        base = syn.solve_instance(topo, ag, S, R)
        sched, coll = gen.compose_allreduce(base, ag)
        assert validate(topo, coll, sched).ok and max(sched.rounds) > 1
        epc = 2048 + 8 * 7
        bufs = host_inputs(dist, dtype, 61, 8, coll.num_chunks, epc)
        want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=f"synth-{topo.name}-{C}-{S}-{R}")
        assert_same_bits(want, got)
        for g in got[1:]:
            assert (bits(g) == bits(got[0])).all()


# ---- small chunks: a chunk is at most one workgroup row; element counts that force every vector width
SMALL = []
for epc in (1, 3, 4, 100, 1000):
    SMALL += [
        (f"hcm8-ar-f32-{epc}", tp.hcm8(), 1, "allreduce", "greedy", "f32", "uniform", epc),
        (f"hcm8-ar-f16-{epc}", tp.hcm8(), 2, "allreduce", "greedy", "f16", "normal", epc),
        (f"ring8-ar-i32-{epc}", tp.ring(8), 4, "allreduce", "ring", "i32", "u32", epc),
        (f"torus-ag-f32-{epc}", tp.torus2d(4, 4), 4, "allgather", "greedy", "f32", "uniform", epc),
        (f"torus-ar-f16-{epc}", tp.torus2d(4, 4), 2, "allreduce", "greedy", "f16", "normal", epc),
        (f"K8-ar-f32-{epc}", tp.complete(8), 1, "allreduce", "greedy", "f32", "uniform", epc),      # fan-in 7
        (f"K12-ar-f16-{epc}", tp.complete(12), 1, "allreduce", "greedy", "f16", "normal", epc),     # fan-in 11
        (f"dgx1-rs-f32-{epc}", tp.dgx1(), 2, "reducescatter", "greedy", "f32", "uniform", epc),
    ]


@pytest.mark.parametrize("label,topo,C,what,kind,dtype,dist,epc", SMALL, ids=[r[0] for r in SMALL])
def test_small_chunks(label, topo, C, what, kind, dtype, dist, epc):
    P = topo.num_nodes
    ag = col.allgather(P, C)
    base = gen.ring_allgather(P, C) if kind == "ring" else gen.greedy_bfs(topo, ag)
    if what == "allgather":
        coll, sched = ag, base
    elif what == "allreduce":
        sched, coll = gen.compose_allreduce(base, ag)
    else:
        sched, coll = gen.reducescatter_from(base, ag)
    bufs = host_inputs(dist, dtype, 71, P, coll.num_chunks, epc, ag.pre if what == "allgather" else None)
    want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=label)
    assert_same_bits(want, got)
