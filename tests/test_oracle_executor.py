"""Pins for oracle/exec.c (through oracle/executor.py): closed forms, exact cases, brute force, conversion tables."""
import numpy as np
import pytest

from oracle import collective as col
from oracle import executor as ex
from oracle import generate as gen
from oracle import topology as tp
from oracle.schedule import COPY, REDUCE, Schedule, make_schedule
from oracle.validate import validate
from paper_2008_08708_amd import inputs

NP = {"i32": np.int32, "f32": np.float32, "f16": np.float16}


def make_bufs(dist, dtype, seed, P, G, epc, pre=None):
    bufs = [inputs.generate(dist, dtype, seed, n, 0, G * epc) for n in range(P)]
    if pre is not None:                       # regions outside pre are undefined inputs: poison them
        for n in range(P):
            for c in range(G):
                if not pre[c, n]:
                    inputs.poison(bufs[n], c * epc, (c + 1) * epc)
    return bufs


def bits(a):
    return a.view(np.uint32 if a.dtype.itemsize == 4 else np.uint16)


# ---------------------------------------------------------------- copies: closed form out[n][c] = in[c mod P][c]

@pytest.mark.parametrize("topo,C,dtype,dist,epc", [
    (tp.ring(4), 1, "f32", "uniform", 1024),
    (tp.hcm8(), 2, "i32", "u32", 257),
    (tp.torus2d(4, 4), 4, "f32", "uniform", 5),
    (tp.ring(8), 4, "f16", "normal", 33),
])
def test_allgather_closed_form_and_no_poison_leak(topo, C, dtype, dist, epc):
    P = topo.num_nodes
    ag = col.allgather(P, C)
    s = gen.ring_allgather(P, C) if topo.name == "ring8" else gen.greedy_bfs(topo, ag)
    assert validate(topo, ag, s).ok
    G = ag.num_chunks
    bufs = make_bufs(dist, dtype, 11, P, G, epc, ag.pre)
    pristine = [b.copy() for b in bufs]
    ex.execute(dtype, G, epc, s, bufs)
    for n in range(P):
        assert not inputs.is_poison(bufs[n]).any()
        for c in range(G):
            want = pristine[c % P][c * epc:(c + 1) * epc]
            assert (bits(bufs[n][c * epc:(c + 1) * epc]) == bits(want)).all()


# ---------------------------------------------------------------- int32: the sum is order free

def test_allreduce_int32_equals_direct_wrapping_sum():
    topo = tp.hcm8()
    ag = col.allgather(8, 1)
    ar, arc = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    G, epc = arc.num_chunks, 101
    bufs = make_bufs("u32", "i32", 2, 8, G, epc)
    want = np.zeros(G * epc, dtype=np.uint32)
    for b in bufs:
        want = want + b.view(np.uint32)        # numpy wraps modulo 2^32
    ex.execute("i32", G, epc, ar, bufs)
    for b in bufs:
        assert (b.view(np.uint32) == want).all()


# ---------------------------------------------------------------- fp: exact inputs make every order equal the direct sum

@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("topo,C", [(tp.hcm8(), 1), (tp.torus2d(4, 4), 1), (tp.ring(8), 2)])
def test_allreduce_small_integers_is_exact(dtype, topo, C):
    P = topo.num_nodes
    ag = col.allgather(P, C)
    base = gen.ring_allgather(P, C) if topo.name == "ring8" else gen.greedy_bfs(topo, ag)
    ar, arc = gen.compose_allreduce(base, ag)
    G, epc = arc.num_chunks, 37
    bufs = make_bufs("smallint", dtype, 5, P, G, epc)
    want = sum(b.astype(np.float64) for b in bufs)
    assert np.abs(want).max() <= 8 * P
    ex.execute(dtype, G, epc, ar, bufs)
    for b in bufs:
        assert (b.astype(np.float64) == want).all()


def test_reducescatter_leaves_the_sum_at_the_owner():
    topo = tp.hcm8()
    ag = col.allgather(8, 2)
    rs, rsc = gen.reducescatter_from(gen.greedy_bfs(topo, ag), ag)
    G, epc = rsc.num_chunks, 19
    bufs = make_bufs("smallint", "f32", 6, 8, G, epc)
    want = sum(b.astype(np.float64) for b in bufs)
    ex.execute("f32", G, epc, rs, bufs)
    for c in range(G):
        assert (bufs[c % 8][c * epc:(c + 1) * epc] == want[c * epc:(c + 1) * epc]).all()


# ---------------------------------------------------------------- fp: rank agreement and the error bound

@pytest.mark.parametrize("dtype,dist", [("f32", "uniform"), ("f16", "normal")])
def test_allreduce_ranks_agree_and_error_is_bounded(dtype, dist):
    topo = tp.hcm8()
    ag = col.allgather(8, 1)
    ar, arc = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    G, epc, P = arc.num_chunks, 211, 8
    bufs = make_bufs(dist, dtype, 3, P, G, epc)
    exact = sum(b.astype(np.float64) for b in bufs)
    sum_abs = sum(np.abs(b.astype(np.float64)) for b in bufs)
    ex.execute(dtype, G, epc, ar, bufs)
    for b in bufs[1:]:
        assert (bits(b) == bits(bufs[0])).all()
    err = np.abs(bufs[0].astype(np.float64) - exact)
    if dtype == "f32":
        assert (err <= (P - 1) * 2.0 ** -24 * sum_abs * 1.01).all()
    else:
        # fp32 accumulation error plus one fp16 rounding per tree level (two levels) of a partial bounded by sum_abs
        assert (err <= (P - 1) * 2.0 ** -24 * sum_abs + 2 * 2.0 ** -11 * sum_abs * 1.01).all()
    assert not np.isnan(bufs[0].astype(np.float32)).any()


# ---------------------------------------------------------------- brute force: an independent expression-tree evaluator

def symbolic_eval(dtype, P, G, sched, inputs_at):
    """Build, from the send list alone, the value of every (c, n) as nested numpy-scalar arithmetic."""
    f32 = np.float32
    val = {(c, n): inputs_at(n, c) for c in range(G) for n in range(P)}
    for s in range(sched.num_steps):
        snap = dict(val)
        groups = {}
        for (c, n, m, st, op) in sched.sends.tolist():
            if st != s:
                continue
            if op == COPY:
                val[(c, m)] = snap[(c, n)]
            else:
                groups.setdefault((c, m), []).append(n)
        for (c, m), srcs in groups.items():
            if dtype == "i32":
                acc = int(snap[(c, m)])
                for n in srcs:
                    acc = (acc + int(snap[(c, n)])) & 0xFFFFFFFF
                val[(c, m)] = acc
            else:
                acc = f32(snap[(c, m)])
                for n in srcs:
                    acc = f32(acc + f32(snap[(c, n)]))
                val[(c, m)] = NP[dtype](acc)          # numpy rounds float32 -> float16 to nearest even
    return val


@pytest.mark.parametrize("dtype,dist", [("f32", "uniform"), ("f16", "normal"), ("f16", "uniform"), ("i32", "u32")])
def test_allreduce_against_symbolic_evaluator(dtype, dist):
    topo = tp.hcm8()
    ag = col.allgather(8, 1)
    ar, arc = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    P, G, epc = 8, arc.num_chunks, 7
    bufs = make_bufs(dist, dtype, 9, P, G, epc)
    pristine = [b.copy() for b in bufs]
    ex.execute(dtype, G, epc, ar, bufs)
    for e in range(epc):
        if dtype == "i32":
            at = lambda n, c: int(pristine[n].view(np.uint32)[c * epc + e])
        else:
            at = lambda n, c: pristine[n][c * epc + e]
        val = symbolic_eval(dtype, P, G, ar, at)
        for c in range(G):
            for n in range(P):
                got = bufs[n][c * epc + e]
                if dtype == "i32":
                    assert int(np.uint32(got.view(np.uint32))) == val[(c, n)]
                else:
                    assert bits(np.array([got]))[0] == bits(np.array([val[(c, n)]], dtype=NP[dtype]))[0]


def test_order_inside_a_group_is_array_order():
    # three sources into node 0 on K4; chosen so that fp32 addition is visibly non-associative
    t = tp.complete(4)
    ar = col.allreduce(4, 1)
    x = [np.float32(1.0), np.float32(2.0 ** -24), np.float32(2.0 ** -24), np.float32(-1.0)]
    def run(order):
        sends = [(0, n, 0, 0, REDUCE) for n in order] + [(0, 0, n, 1, COPY) for n in (1, 2, 3)]
        s = make_schedule([1, 1], sends)
        assert validate(t, ar, s).ok
        bufs = [np.array([v], dtype=np.float32) for v in x]
        ex.execute("f32", 1, 1, s, bufs)
        return bufs[0][0]
    # ((1 + e) + e) - 1 = 0 in fp32 (each e is absorbed, ties to even), while ((1 - 1) + e) + e = 2e
    assert run([1, 2, 3]) == np.float32(0.0)
    assert run([3, 1, 2]) == np.float32(2.0 ** -23)


def test_fp16_group_narrows_once():
    # 2048 + 1 + 1: rounding after each add gives 2048 (2049 ties to even twice); one rounding of 2050 gives 2050
    t = tp.complete(3)
    ar = col.allreduce(3, 1)
    s = make_schedule([1, 1], [(0, 1, 0, 0, REDUCE), (0, 2, 0, 0, REDUCE), (0, 0, 1, 1, COPY), (0, 0, 2, 1, COPY)])
    assert validate(t, ar, s).ok
    bufs = [np.array([v], dtype=np.float16) for v in (2048.0, 1.0, 1.0)]
    ex.execute("f16", 1, 1, s, bufs)
    assert all(b[0] == np.float16(2050.0) for b in bufs)
    # the same three values through a chain 2 -> 1 -> 0 are rounded between steps: (1 + 1) = 2, 2048 + 2 = 2050;
    # and 1 -> 0, then 2 -> 0 in separate steps: 2048 + 1 -> 2048 (tie to even), + 1 -> 2048
    s2 = make_schedule([1, 1, 1], [(0, 1, 0, 0, REDUCE), (0, 2, 0, 1, REDUCE), (0, 0, 1, 2, COPY), (0, 0, 2, 2, COPY)])
    assert validate(t, ar, s2).ok
    bufs = [np.array([v], dtype=np.float16) for v in (2048.0, 1.0, 1.0)]
    ex.execute("f16", 1, 1, s2, bufs)
    assert all(b[0] == np.float16(2048.0) for b in bufs)


# ---------------------------------------------------------------- fp16 <-> fp32 conversions against numpy's

def test_half_to_float_all_65536_values():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = ex.f16_to_f32(h)
    want = h.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert (np.isnan(got) == nan).all()
    assert (got.view(np.uint32)[~nan] == want.view(np.uint32)[~nan]).all()


def test_float_to_half_rne_exhaustive_neighbourhoods_and_random():
    # every half value, the exact midpoints between neighbours, and the floats adjacent to those midpoints
    h = np.arange(0x7c00, dtype=np.uint32).astype(np.uint16)            # non-negative finite halves
    lo = h.view(np.float16).astype(np.float64)
    hi = np.append(lo[1:], 65536.0)
    mid = ((lo + hi) / 2).astype(np.float32)                            # exact in fp32
    cand = np.concatenate([lo.astype(np.float32), mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9))])
    cand = np.concatenate([cand, -cand])
    rng = np.random.default_rng(0)
    rnd = rng.integers(0, 2 ** 32, size=1 << 22, dtype=np.uint64).astype(np.uint32).view(np.float32)
    rnd = rnd[~np.isnan(rnd)]
    tiny = np.array([0.0, 2.0 ** -25, 2.0 ** -24, 1.5 * 2.0 ** -24, 2.0 ** -26, 1e-45, 2.0 ** -126, 65519.996, 65520.0, 1e38, np.inf],
                    dtype=np.float32)
    allv = np.concatenate([cand, rnd, tiny, -tiny])
    got = ex.f32_to_f16(allv)
    with np.errstate(over="ignore"):
        want = allv.astype(np.float16).view(np.uint16)
    assert (got == want).all()


def test_rne_spot_values():
    f = lambda v: ex.f32_to_f16(np.array([v], dtype=np.float32)).view(np.float16)[0]
    assert f(2049.0) == 2048.0 and f(2051.0) == 2052.0
    assert f(1.0 + 2.0 ** -11) == 1.0                       # tie to even
    assert f(1.0 + 3 * 2.0 ** -11) == np.float16(1.0 + 2.0 ** -9)
    assert np.isinf(f(65520.0)) and f(65519.0) == np.float16(65504.0)
    assert f(2.0 ** -24) == np.float16(2.0 ** -24)         # smallest subnormal survives
    assert f(2.0 ** -25) == 0.0                             # tie to even -> 0


def test_denormals_survive_copy_and_add_zero():
    t = tp.complete(2)
    ar = col.allreduce(2, 1)
    s = make_schedule([1, 1], [(0, 1, 0, 0, REDUCE), (0, 0, 1, 1, COPY)])
    assert validate(t, ar, s).ok
    for dtype, tiny in (("f16", np.float16(2.0 ** -24)), ("f32", np.float32(1e-45))):
        bufs = [np.array([tiny], dtype=NP[dtype]), np.array([0], dtype=NP[dtype])]
        ex.execute(dtype, 1, 1, s, bufs)
        assert bufs[0][0] == tiny and bufs[1][0] == tiny and tiny != 0


# ---------------------------------------------------------------- element sub-ranges and threads

def test_subrange_and_threads_do_not_change_bits():
    topo = tp.hcm8()
    ag = col.allgather(8, 1)
    ar, arc = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    G, epc, P = arc.num_chunks, 1000, 8
    ref = make_bufs("uniform", "f32", 21, P, G, epc)
    pristine = [b.copy() for b in ref]
    ex.execute("f32", G, epc, ar, ref)
    par = [b.copy() for b in pristine]
    ex.execute("f32", G, epc, ar, par, threads=4)
    sub = [b.copy() for b in pristine]
    ex.execute("f32", G, epc, ar, sub, first_elem=100, num_elems=50)
    for n in range(P):
        assert (bits(par[n]) == bits(ref[n])).all()
        r = ref[n].reshape(G, epc)
        q = sub[n].reshape(G, epc)
        p0 = pristine[n].reshape(G, epc)
        assert (bits(q[:, 100:150]) == bits(r[:, 100:150])).all()
        assert (bits(q[:, :100]) == bits(p0[:, :100])).all() and (bits(q[:, 150:]) == bits(p0[:, 150:])).all()


def test_algorithmic_bytes():
    # one copy group to 3 destinations: 4 chunks; one reduce group of 2 sources: 4 chunks
    s = make_schedule([1], [(0, 0, 1, 0, COPY), (0, 0, 2, 0, COPY), (0, 0, 3, 0, COPY), (1, 1, 0, 0, REDUCE), (1, 2, 0, 0, REDUCE)])
    fused, unfused = ex.algorithmic_bytes(s, 10)
    assert fused == (4 + 4) * 10 and unfused == (3 * 2 + 2 * 3) * 10
    # headline configuration: 112 sends, unfused 8.75 GiB at 32 MiB chunks
    ag = col.allgather(8, 1)
    ar, _ = gen.compose_allreduce(gen.greedy_bfs(tp.hcm8(), ag), ag)
    fused, unfused = ex.algorithmic_bytes(ar, 32 << 20)
    assert ar.sends.shape[0] == 112 and unfused == int(8.75 * 2 ** 30) and fused < unfused


def test_bad_arguments_are_rejected():
    s = make_schedule([1], [(0, 0, 1, 0, COPY)])
    with pytest.raises(ValueError):
        ex.execute("f32", 1, 4, s, [np.zeros(4, np.float32), np.zeros(5, np.float32)])
    with pytest.raises(ValueError):
        ex.execute("f32", 1, 4, make_schedule([1], [(0, 0, 2, 0, COPY)]), [np.zeros(4, np.float32)] * 2)
