"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Integer outputs (sampled ids, offsets, local ids, gathered bytes, placement order) must be
bit-exact.  PSGS / FAP are fp32 on the GPU against fp64 in the oracle: relative error <= 1e-4
(the tolerance the benchmark spec states), and exactly zero where the oracle is zero.
"""
import numpy as np
import pytest

import oracle
import qvgen

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

REL_TOL = 1e-4


@pytest.fixture(scope="module")
def qv():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2305_10863_amd as m
    m.lib()
    return m


DEDUP_FORMS = {
    # name: (form, partitions_log2, table budget)
    "direct": (1, -1, None),         # table addressed by node id
    "hashed": (1, -1, 0),            # open-addressing hash table
    "part": (2, -1, None),           # partitioned (LDS) dedup, partitions chosen per call
    "part1": (2, 0, None),           # one partition: larger cases overflow its LDS table and split into sub-rounds
    "part64": (2, 6, None),          # as many partitions as a wave has lanes
    "part256": (2, 8, None),         # the most partitions
}


def apply_form(c, name):
    form, p_log2, budget = DEDUP_FORMS[name]
    c.set_dedup(form, p_log2)
    if budget is not None:
        c.set_table_budget(budget)
    c._form = name


@pytest.fixture(scope="module", params=list(DEDUP_FORMS))
def ctx(qv, request):
    """Every test runs with every dedup form: the two table forms and the partitioned form at four partition counts."""
    c = qv.Context(0)
    apply_form(c, request.param)
    yield c
    c.close()


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def make_graph(qv, ctx, rowptr, col):
    return qv.Graph(ctx, dev(rowptr), dev(col))


def assert_sample_equal(got, want):
    for k in ("node_off", "edge_off", "frontier_off", "n_id", "row_local", "col_local", "nbr_global", "frontier"):
        assert np.array_equal(got[k], want[k]), k


def rel_err(g, o):
    g = g.astype(np.float64)
    nz = o != 0
    assert np.all(g[~nz] == 0)
    return np.max(np.abs(g[nz] - o[nz]) / np.abs(o[nz])) if nz.any() else 0.0


# ------------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def tiny(qv, ctx):
    w = qvgen.workload("tiny")
    rowptr, col = w.graph()
    return w, rowptr, col, make_graph(qv, ctx, rowptr, col)


@pytest.mark.parametrize("fanout", [1, 3, 8, 9, 16, 17, 32, 33, 64, 65, 128, 200, 1024])
def test_sample_hop_matches_oracle(qv, ctx, tiny, fanout):
    w, rowptr, col, g = tiny
    rng = np.random.default_rng(fanout)
    deg = np.diff(rowptr)
    hubs = np.argsort(-deg)[:40]                                   # long rows: the drawing path
    frontier = np.concatenate([rng.integers(0, w.n, 3000), hubs, hubs[:5]]).astype(np.int32)
    rng.shuffle(frontier)
    for hop in (1, 3):
        nbr, off = qv.qv_sample_hop(ctx, g, dev(frontier), fanout, 0xC0FFEE1234567 + fanout, hop)
        ctx.sync()
        o_nbr, o_off = oracle.sample_hop(rowptr, col, frontier, fanout, 0xC0FFEE1234567 + fanout, hop)
        off = off.cpu().numpy()
        assert np.array_equal(off, o_off)
        assert np.array_equal(nbr[:off[-1]].cpu().numpy(), o_nbr)


def test_sample_hop_tight_rows_exercise_collisions(qv, ctx):
    # rows only slightly longer than the fanout: nearly every draw collides
    rng = np.random.default_rng(5)
    n = 3000
    deg = rng.integers(0, 90, n)
    rowptr = np.zeros(n + 1, np.int64)
    rowptr[1:] = np.cumsum(deg)
    col = rng.integers(0, n, rowptr[-1]).astype(np.int32)
    g = make_graph(qv, ctx, rowptr, col)
    frontier = np.arange(n, dtype=np.int32)
    for fanout in (2, 7, 15, 31, 50, 64, 70, 88):
        for seed in (1, 2 ** 63 + 12345):
            nbr, off = qv.qv_sample_hop(ctx, g, dev(frontier), fanout, seed, 2)
            ctx.sync()
            o_nbr, o_off = oracle.sample_hop(rowptr, col, frontier, fanout, seed, 2)
            off = off.cpu().numpy()
            assert np.array_equal(off, o_off)
            assert np.array_equal(nbr[:off[-1]].cpu().numpy(), o_nbr), (fanout, seed)


@pytest.mark.parametrize("n_known,n_nbr,universe", [(0, 0, 10), (0, 1, 10), (5, 0, 100), (64, 3000, 500),
                                                     (1000, 100000, 30000), (3, 300000, 50), (70000, 200000, 10 ** 8)])
def test_reindex_matches_oracle(qv, ctx, n_known, n_nbr, universe):
    rng = np.random.default_rng(n_known + n_nbr)
    known = rng.choice(universe, size=n_known, replace=False).astype(np.int32) if n_known else np.zeros(0, np.int32)
    nbr = rng.integers(0, universe, n_nbr).astype(np.int32)
    n_id, n_len, local, front, f_len = qv.qv_reindex(ctx, dev(known), dev(nbr), n_nodes=universe)
    ctx.sync()
    o_n_id, o_local, o_front = oracle.reindex(known, nbr)
    assert int(n_len.item()) == len(o_n_id) and int(f_len.item()) == len(o_front)
    assert np.array_equal(n_id[:len(o_n_id)].cpu().numpy(), o_n_id)
    assert np.array_equal(local[:n_nbr].cpu().numpy(), o_local)
    assert np.array_equal(front[:len(o_front)].cpu().numpy(), o_front)


def test_sample_tiny_workload_all_batches(qv, ctx, tiny):
    w, rowptr, col, g = tiny
    for b in range(8):
        seeds = w.seeds(b)
        out = qv.qv_sample(ctx, g, dev(seeds), w.fanouts, w.rng_seed(b))
        ctx.sync()
        assert_sample_equal(out.to_host(), oracle.sample(rowptr, col, seeds, w.fanouts, w.rng_seed(b)))


@pytest.mark.parametrize("fanouts,n_seeds", [([10, 5], 1), ([15, 10, 5], 512), ([25, 10], 1000), ([3], 4096),
                                             ([70, 2], 200), ([2, 2, 2, 2, 2, 2, 2, 2], 50), ([40, 33], 300),
                                             # seed counts around tile boundaries of the dedup scan
                                             ([4, 3], 4095), ([4, 3], 4097), ([5], 9000), ([6, 2], 255), ([6, 2], 257)])
def test_sample_shapes(qv, ctx, tiny, fanouts, n_seeds):
    w, rowptr, col, g = tiny
    seeds = w.seeds(100 + n_seeds, n_seeds)
    out = qv.qv_sample(ctx, g, dev(seeds), fanouts, 77)
    ctx.sync()
    assert_sample_equal(out.to_host(), oracle.sample(rowptr, col, seeds, fanouts, 77))


def test_sample_large_hop_with_a_hub(qv, ctx):
    """A hop of more than half a million edges over 300 k nodes in which 15 % of all edges end at
    one hub: long runs of repeats next to mostly distinct neighbours."""
    rng = np.random.default_rng(5)
    n = 300_000
    deg = rng.integers(8, 25, n)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=rowptr[1:])
    col = rng.integers(0, n, int(rowptr[-1])).astype(np.int32)
    col[rng.random(len(col)) < 0.15] = 12345
    g = make_graph(qv, ctx, rowptr, col)
    seeds = rng.integers(0, n, 6000).astype(np.int32)
    for cumulative in (False, True):
        out = qv.qv_sample(ctx, g, dev(seeds), [12, 9], 31337, cumulative=cumulative)
        ctx.sync()
        want = oracle.sample(rowptr, col, seeds, [12, 9], 31337, cumulative=cumulative)
        assert want["edge_off"][-1] > 500_000 and len(want["n_id"]) > 200_000
        assert_sample_equal(out.to_host(), want)


def test_sample_int64_rowptr_and_in_degree_skew(qv, ctx):
    w = qvgen.workload("citation", scale=0.003)
    rowptr, col = w.graph()
    assert rowptr.dtype == np.int64
    g = make_graph(qv, ctx, rowptr, col)
    for b in range(3):
        seeds = w.seeds(b)
        out = qv.qv_sample(ctx, g, dev(seeds), w.fanouts, w.rng_seed(b))
        ctx.sync()
        assert_sample_equal(out.to_host(), oracle.sample(rowptr, col, seeds, w.fanouts, w.rng_seed(b)))


@pytest.mark.parametrize("n_batches", [1, 3, 8, 9, 20, 32])      # up to 8: arguments inline; above: uploaded
def test_sample_many_and_gather_many(qv, ctx, tiny, n_batches):
    w, rowptr, col, g = tiny
    sizes = ([64, 1, 500, 0, 2000, 64, 7, 300] * 4)[:n_batches]
    fanouts = [15, 10, 5]
    seeds = [w.seeds(200 + i, n) if n else np.zeros(0, np.int32) for i, n in enumerate(sizes)]
    rngs = [w.rng_seed(200 + i) for i in range(n_batches)]
    d_seeds = [dev(s) if len(s) else torch.zeros(0, dtype=torch.int32, device="cuda") for s in seeds]
    outs = qv.qv_sample_many(ctx, g, d_seeds, fanouts, rngs)
    table = qvgen.features_host(w.seed, w.n, w.dim, w.feat_dtype)
    feat = qv.Features(ctx, torch.from_numpy(table).cuda())
    rows = qv.qv_gather_many(ctx, feat, [o.n_id for o in outs], [o.node_off[-1:] for o in outs])
    ctx.sync()
    for i in range(n_batches):
        want = oracle.sample(rowptr, col, seeds[i], fanouts, rngs[i])
        assert_sample_equal(outs[i].to_host(), want)
        U = len(want["n_id"])
        assert rows[i][:U].cpu().numpy().tobytes() == oracle.gather(table, want["n_id"]).tobytes()
    feat.close()


def test_call_of_the_most_batches(qv, ctx, tiny):
    # the largest call: QV_MAX_BATCHES batches of unequal sizes through one set of launches
    w, rowptr, col, g = tiny
    n = qv.QV_MAX_BATCHES
    assert n == 256
    seeds = [w.seeds(700 + j, 1 + (37 * j) % 300) for j in range(n)]
    rng = [900 + j for j in range(n)]
    outs = qv.qv_sample_many(ctx, g, [dev(s) for s in seeds], [7, 4, 3], rng)
    ctx.sync()
    wants = [oracle.sample(rowptr, col, seeds[j], [7, 4, 3], rng[j]) for j in range(n)]
    for j in range(n):
        assert_sample_equal(outs[j].to_host(), wants[j])
    # the gather of all of them in one call (more id lists than one launch takes)
    table = qvgen.features_host(w.seed, w.n, w.dim, w.feat_dtype)
    feat = qv.Features(ctx, dev(table))
    rows = qv.qv_gather_many(ctx, feat, [o.n_id for o in outs], [o.node_off[-1:] for o in outs])
    ctx.sync()
    for j in range(n):
        U = len(wants[j]["n_id"])
        assert rows[j][:U].cpu().numpy().tobytes() == oracle.gather(table, wants[j]["n_id"]).tobytes()
    feat.close()


@pytest.mark.parametrize("sizes", [[2048, 2047, 1, 0], [2049, 5], [2048] * 9, [4096, 100]])
def test_seed_stage_at_the_limit_of_its_one_kernel_form(qv, ctx, tiny, sizes):
    # batches of up to 2,048 seeds go through stage 0 in one kernel (partitioned form), larger ones through the
    # three general kernels; seeds drawn from 300 ids, so nearly all of them repeat, plus ids outside the graph
    w, rowptr, col, g = tiny
    rng0 = np.random.default_rng(len(sizes) * 10_000 + sizes[0])
    seeds = [rng0.integers(0, 300, n).astype(np.int32) for n in sizes]
    rngs = [77 + i for i in range(len(sizes))]
    outs = qv.qv_sample_many(ctx, g, [dev(s) if len(s) else torch.zeros(0, dtype=torch.int32, device="cuda") for s in seeds],
                             [5, 3], rngs)
    ctx.sync()
    for i, s_ in enumerate(seeds):
        assert_sample_equal(outs[i].to_host(), oracle.sample(rowptr, col, s_, [5, 3], rngs[i]))
    if sizes[0] >= 2048:                                            # an id outside the graph is reported, the rest of the call is unaffected
        bad = [s_.copy() for s_ in seeds]
        bad[0][7] = w.n
        outs = qv.qv_sample_many(ctx, g, [dev(s_) for s_ in bad], [5, 3], rngs)
        with pytest.raises(qv.QvError) as e:
            ctx.sync()
        assert e.value.status == qv.QV_ERANGE
        assert_sample_equal(outs[1].to_host(), oracle.sample(rowptr, col, seeds[1], [5, 3], rngs[1]))


@pytest.mark.parametrize("n", [5, 257, 600, 1024])
def test_step_many_samples_and_gathers_like_the_two_calls(qv, ctx, tiny, n):
    # one serving step through qv_step_many: 1, 2, 3 and 4 groups (the groups after the first run on streams
    # of the context's own); every batch against the oracle, rows clamped by the device-side count and by
    # rows_cap; twice in a row on the same buffers, and a deferred error of a later group reaches qv_ctx_sync
    w, rowptr, col, g = tiny
    fan = [6, 3]
    seeds = [w.seeds(1700 + j, 1 + (53 * j) % 200) for j in range(n)]
    table = qvgen.features_host(w.seed, w.n, w.dim, w.feat_dtype)
    feat = qv.Features(ctx, dev(table))
    bufs = [qv.SampleBuffers(ctx, len(s), fan, w.n) for s in seeds]
    caps = [b.caps[0] if j % 7 else 3 for j, b in enumerate(bufs)]            # every seventh batch: three rows only
    rows = [feat.empty_rows(max(c, 1), ctx.device) for c in caps]
    plan = qv.ManyPlan(ctx, g, feat, bufs, rows, fan)
    for j in range(n):
        plan.n_ids[j] = caps[j]
    d_seeds = [dev(s) for s in seeds]
    for rnd in range(2):
        rng = [3100 + 1000 * rnd + j for j in range(n)]
        for r in rows:
            r.fill_(0)
        torch.cuda.synchronize()
        plan.step(d_seeds, rng)
        ctx.sync()
        for j in range(0, n, 1 if n <= 257 else 5):
            want = oracle.sample(rowptr, col, seeds[j], fan, rng[j])
            assert_sample_equal(bufs[j].to_host(), want)
            U = min(len(want["n_id"]), caps[j])
            got = rows[j].cpu().numpy()
            assert got[:U].tobytes() == oracle.gather(table, want["n_id"][:U]).tobytes(), j
            assert not got[U:].any(), j
    if n > qv.QV_MAX_BATCHES:
        bad = dev(np.array([w.n + 5], dtype=np.int32))                          # an id outside the graph, in the last group
        plan.step(d_seeds[:-1] + [bad], rng)
        with pytest.raises(qv.QvError) as e:
            ctx.sync()
        assert e.value.status == qv.QV_ERANGE
        plan.step(d_seeds, rng)                                                 # ... and the context is usable afterwards
        ctx.sync()
        assert_sample_equal(bufs[n - 1].to_host(), oracle.sample(rowptr, col, seeds[n - 1], fan, rng[n - 1]))
    with pytest.raises(qv.QvError) as e:                                       # one batch more than the call takes
        ctx.check(qv.lib().qv_step_many(ctx.h, g.h, feat.h, qv.QV_MAX_STEP_BATCHES + 1, plan.seed_ptrs, plan.n_seeds, plan.fan,
                                        plan.k, plan.rng, 0, plan.outs, plan.out_ptrs, plan.n_ids, plan.stride))
    assert e.value.status == qv.QV_EINVAL
    feat.close()


def test_step_many_with_cumulative_frontiers(qv, ctx, tiny):
    # the nested-block variant takes the table forms, here in two groups: the second group's tables belong to
    # the context's own second stream; two calls in a row (the tables are reused, never cleared)
    w, rowptr, col, g = tiny
    fan, n = [4, 3], qv.QV_MAX_BATCHES + 40
    seeds = [w.seeds(2600 + j, 1 + (29 * j) % 90) for j in range(n)]
    table = qvgen.features_host(w.seed, w.n, w.dim, w.feat_dtype)
    feat = qv.Features(ctx, dev(table))
    bufs = [qv.SampleBuffers(ctx, len(s), fan, w.n, cumulative=True) for s in seeds]
    rows = [feat.empty_rows(b.caps[0], ctx.device) for b in bufs]
    plan = qv.ManyPlan(ctx, g, feat, bufs, rows, fan, cumulative=True)
    d_seeds = [dev(s) for s in seeds]
    for rnd in range(2):
        rng = [5200 + 700 * rnd + j for j in range(n)]
        plan.step(d_seeds, rng)
        ctx.sync()
        for j in list(range(0, n, 7)) + [n - 1]:
            want = oracle.sample(rowptr, col, seeds[j], fan, rng[j], cumulative=True)
            assert_sample_equal(bufs[j].to_host(), want)
            U = len(want["n_id"])
            assert rows[j][:U].cpu().numpy().tobytes() == oracle.gather(table, want["n_id"]).tobytes(), j
    feat.close()


def test_table_reuse_across_calls_and_epoch_wrap(qv, tiny):
    # the dedup tables are not cleared between calls; results must not depend on what earlier
    # calls (of other sizes, other batch counts) left behind, nor on the counter wrapping
    w, rowptr, col, g0 = tiny
    c = qv.Context(0)
    apply_form(c, g0.ctx._form)
    g = make_graph(qv, c, rowptr, col)
    plan = [(64, [10, 5]), (2000, [15, 10, 5]), (3, [3]), (700, [25, 10]), (64, [10, 5])]
    for rnd in range(3):
        if rnd == 2:
            c.check(qv.lib().qv_ctx_set_epoch(c.h, 0xFFFFE - 3))       # cross the wrap point
        for i, (n, fan) in enumerate(plan * 2):
            seeds = w.seeds(300 + i, n)
            out = qv.qv_sample(c, g, dev(seeds), fan, 1000 + i)
            c.sync()
            assert_sample_equal(out.to_host(), oracle.sample(rowptr, col, seeds, fan, 1000 + i))
        many = [w.seeds(400 + j, 100 + 50 * j) for j in range(4)]
        outs = qv.qv_sample_many(c, g, [dev(s) for s in many], [10, 5], [7, 8, 9, 10])
        c.sync()
        for j in range(4):
            assert_sample_equal(outs[j].to_host(), oracle.sample(rowptr, col, many[j], [10, 5], 7 + j))
    c.close()


@pytest.mark.parametrize("fanouts,n_seeds", [([10, 5], 64), ([15, 10, 5], 300), ([3, 3, 3, 3], 50), ([70, 4], 20), ([6], 100)])
def test_cumulative_frontiers_match_oracle(qv, ctx, tiny, fanouts, n_seeds):
    # every hop expands all nodes sampled so far (nested blocks)
    w, rowptr, col, g = tiny
    seeds = w.seeds(500 + n_seeds, n_seeds)
    out = qv.qv_sample(ctx, g, dev(seeds), fanouts, 4242, cumulative=True)
    ctx.sync()
    want = oracle.sample(rowptr, col, seeds, fanouts, 4242, cumulative=True)
    assert_sample_equal(out.to_host(), want)
    assert qv.qv_sample_bounds(n_seeds, fanouts, w.n, cumulative=True) == oracle.sample_bounds(n_seeds, fanouts, w.n, True)
    many = [w.seeds(600 + j, 40 + 30 * j) for j in range(3)]
    outs = qv.qv_sample_many(ctx, g, [dev(s) for s in many], fanouts, [1, 2, 3], cumulative=True)
    ctx.sync()
    for j in range(3):
        assert_sample_equal(outs[j].to_host(), oracle.sample(rowptr, col, many[j], fanouts, 1 + j, cumulative=True))
    # and the layer-frontier mode still gives its own result on the same context
    out = qv.qv_sample(ctx, g, dev(seeds), fanouts, 4242)
    ctx.sync()
    assert_sample_equal(out.to_host(), oracle.sample(rowptr, col, seeds, fanouts, 4242))


def test_randomised_graphs_and_parameters(qv, ctx):
    # seeded sweep over small random graphs (self-loops, multi-edges, sinks, hubs), hop counts,
    # fanouts on both sides of the sub-wave group widths, seed counts, both frontier modes
    rng = np.random.default_rng(20261127)
    for case in range(40):
        n = int(rng.integers(1, 400))
        deg = np.minimum(rng.zipf(1.5, n), 300) * (rng.random(n) > 0.15)
        rowptr = np.zeros(n + 1, np.int64)
        rowptr[1:] = np.cumsum(deg)
        col = rng.integers(0, n, rowptr[-1]).astype(np.int32)
        if case % 2:
            rowptr = rowptr.astype(np.int32)
        g = make_graph(qv, ctx, rowptr, col)
        K = int(rng.integers(1, 5))
        fanouts = [int(rng.choice([1, 2, 5, 8, 9, 16, 17, 31, 33, 64, 65, 100])) for _ in range(K)]
        while np.prod([f + 1 for f in fanouts]) * 50 > 3e6:
            fanouts = fanouts[:-1]
        cumulative = bool(rng.integers(0, 2))
        sizes = [int(rng.integers(0, 50)) for _ in range(int(rng.integers(1, 5)))]
        seeds = [rng.integers(0, n, s).astype(np.int32) for s in sizes]
        rngs = [int(rng.integers(0, 2 ** 63)) for _ in sizes]
        d_seeds = [dev(s) if len(s) else torch.zeros(0, dtype=torch.int32, device="cuda") for s in seeds]
        outs = qv.qv_sample_many(ctx, g, d_seeds, fanouts, rngs, cumulative=cumulative)
        ctx.sync()
        for i in range(len(sizes)):
            want = oracle.sample(rowptr, col, seeds[i], fanouts, rngs[i], cumulative=cumulative)
            got = outs[i].to_host()
            for k in ("node_off", "edge_off", "frontier_off", "n_id", "row_local", "col_local", "nbr_global", "frontier"):
                assert np.array_equal(got[k], want[k]), (case, i, k, fanouts, cumulative)


def test_graph_in_pinned_host_memory(qv, ctx, tiny):
    # topology read zero-copy over the host link: same results
    w, rowptr, col, _ = tiny
    g = qv.Graph(ctx, torch.from_numpy(rowptr).pin_memory(), torch.from_numpy(col).pin_memory())
    seeds = w.seeds(5)
    out = qv.qv_sample(ctx, g, dev(seeds), w.fanouts, 99)
    Q = qv.qv_psgs(ctx, g, w.fanouts)
    ctx.sync()
    assert_sample_equal(out.to_host(), oracle.sample(rowptr, col, seeds, w.fanouts, 99))
    assert rel_err(Q.cpu().numpy(), oracle.psgs(rowptr, col, w.fanouts)) <= REL_TOL
    with pytest.raises(TypeError):
        qv.Graph(ctx, torch.from_numpy(rowptr), torch.from_numpy(col))       # pageable host memory


def test_sample_degenerate_inputs(qv, ctx):
    rowptr = np.array([0, 0, 2, 2], dtype=np.int64)
    col = np.array([0, 2], dtype=np.int32)
    g = make_graph(qv, ctx, rowptr, col)
    for seeds, fanouts in (([0, 0, 2], [3, 3]), ([1], [1, 4]), ([], [2]), ([1, 1, 1], [5])):
        s = np.array(seeds, dtype=np.int32)
        out = qv.qv_sample(ctx, g, dev(s) if len(s) else torch.zeros(0, dtype=torch.int32, device="cuda"), fanouts, 5)
        ctx.sync()
        assert_sample_equal(out.to_host(), oracle.sample(rowptr, col, s, fanouts, 5))


def test_errors_are_reported_not_fatal(qv, ctx, tiny):
    w, rowptr, col, g = tiny
    seeds = w.seeds(0)
    # id out of range -> deferred QV_ERANGE, the rest of the batch still sampled
    bad = seeds.copy()
    bad[3] = w.n + 5
    qv.qv_sample(ctx, g, dev(bad), w.fanouts, 1)
    with pytest.raises(qv.QvError) as e:
        ctx.sync()
    assert e.value.status == qv.QV_ERANGE
    ctx.sync()                                           # status was cleared
    # output arrays too small -> deferred QV_ECAPACITY, nothing written past the capacity
    buf = qv.SampleBuffers(ctx, len(seeds), w.fanouts, w.n, caps=(100, 150, 80))
    guard = torch.full((1000,), -7, dtype=torch.int32, device="cuda")
    qv.qv_sample(ctx, g, dev(seeds), w.fanouts, 1, out=buf)
    with pytest.raises(qv.QvError) as e:
        ctx.sync()
    assert e.value.status == qv.QV_ECAPACITY
    assert bool((guard == -7).all())
    # host-side argument checks
    for fan in ([0, 5], [5] * 9, [2000]):
        with pytest.raises(qv.QvError) as e:
            qv.qv_sample(ctx, g, dev(seeds), fan, 1)
        assert e.value.status == qv.QV_EINVAL
    # malformed graphs are refused at creation
    rp = rowptr.copy().astype(np.int64)
    rp[5], rp[6] = rp[6] + 1, rp[5]
    with pytest.raises(qv.QvError) as e:
        make_graph(qv, ctx, rp, col)
    assert e.value.status == qv.QV_EINVAL
    c2 = col.copy()
    c2[17] = w.n
    with pytest.raises(qv.QvError):
        make_graph(qv, ctx, rowptr, c2)
    # repeated known ids in the stand-alone reindex
    qv.qv_reindex(ctx, dev(np.array([4, 4], np.int32)), dev(np.array([1], np.int32)))
    with pytest.raises(qv.QvError) as e:
        ctx.sync()
    assert e.value.status == qv.QV_EINVAL
    ctx.sync()


# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,dim", [(np.float32, 64), (np.float16, 128), (np.float32, 602), (np.float32, 100),
                                       (np.float32, 1024), (np.float16, 7), (np.float32, 1), (np.float16, 1),
                                       (np.float16, 1203), (np.float32, 33), (np.float16, 517)])
def test_gather_matches_oracle(qv, ctx, dtype, dim):
    n = 5000
    table = qvgen.features_host(42, n, dim, dtype)
    rng = np.random.default_rng(dim)
    ids = rng.integers(0, n, 12345).astype(np.int32)
    tdtype = torch.float32 if dtype == np.float32 else torch.float16
    t_dev = qvgen.features_device(42, n, dim, tdtype)
    assert t_dev.cpu().numpy().tobytes() == table.tobytes()          # host and device generators agree
    feat = qv.Features(ctx, t_dev)
    out = qv.qv_gather(ctx, feat, dev(ids))
    ctx.sync()
    want = oracle.gather(table, ids)
    assert out.cpu().numpy().tobytes() == want.tobytes()
    # the library's own copy (rows re-laid on 128-byte boundaries where that is cheap) and an
    # output with the same row stride
    feat_own = qv.Features(ctx, t_dev, own_copy=True)
    assert feat_own.row_stride >= feat_own.row_bytes and feat_own.row_stride % 16 == 0
    out_own = qv.qv_gather(ctx, feat_own, dev(ids))
    ctx.sync()
    assert out_own.stride(0) * out_own.element_size() == feat_own.row_stride
    assert out_own.cpu().numpy().tobytes() == want.tobytes()
    feat_own.close()
    # a host table (copied into HBM by the library) and a device-side row count
    feat_h = qv.Features(ctx, torch.from_numpy(table))
    n_dev = torch.tensor([777], dtype=torch.int64, device="cuda")
    out2 = torch.zeros((len(ids), dim), dtype=tdtype, device="cuda")
    qv.qv_gather(ctx, feat_h, dev(ids), n_ids_dev=n_dev, out=out2)
    ctx.sync()
    got = out2.cpu().numpy()
    assert got[:777].tobytes() == want[:777].tobytes() and not got[777:].any()
    # empty gather, out-of-range id
    qv.qv_gather(ctx, feat, torch.zeros(0, dtype=torch.int32, device="cuda"))
    ctx.sync()
    qv.qv_gather(ctx, feat, dev(np.array([1, n], np.int32)))
    with pytest.raises(qv.QvError) as e:
        ctx.sync()
    assert e.value.status == qv.QV_ERANGE
    feat.close()
    feat_h.close()


@pytest.mark.parametrize("on_device", [True, False])
def test_tiered_gather_and_placement(qv, ctx, on_device):
    n, dim = 20000, 96
    table = qvgen.features_host(9, n, dim, np.float32)
    rng = np.random.default_rng(3)
    prob = rng.random(n).astype(np.float32)
    prob[rng.integers(0, n, 4000)] = np.float32(0.5)                 # ties
    rank = qv.qv_place_rank(ctx, dev(prob))
    ctx.sync()
    budget = 3000 * dim * 4 + 100                                    # floor -> 3000 hot rows
    o_rank, o_loc = oracle.place(prob, 3000)
    assert np.array_equal(rank.cpu().numpy(), o_rank)
    src = qvgen.features_device(9, n, dim, torch.float32) if on_device else torch.from_numpy(table)
    feat = qv.Features(ctx, src, hbm_budget_bytes=budget, rank=rank)
    assert feat.n_hot == 3000
    # the lookup table itself: hot index = position in the ranking, cold index = order of the remaining ids
    assert np.array_equal(feat.loc().cpu().numpy(), o_loc)
    ids = rng.integers(0, n, 50000).astype(np.int32)
    out = qv.qv_gather(ctx, feat, dev(ids))
    ctx.sync()
    assert out.cpu().numpy().tobytes() == oracle.gather(table, ids).tobytes()
    cold_frac = (o_loc[ids] < 0).mean()
    assert 0.7 < cold_frac < 0.95                                    # both tiers were exercised
    feat.close()


# ------------------------------------------------------------------------------------------------
def metric_graphs():
    yield "tiny", qvgen.workload("tiny")
    yield "co_purchase_1pct", qvgen.workload("co_purchase", scale=0.01)
    yield "citation_0.3pct", qvgen.workload("citation", scale=0.003)
    yield "dense_social_2pct", qvgen.workload("dense_social", scale=0.02)


@pytest.mark.parametrize("name,w", list(metric_graphs()), ids=[n for n, _ in metric_graphs()])
def test_psgs_and_access_prob_match_oracle(qv, ctx, name, w):
    rowptr, col = w.graph()
    g = make_graph(qv, ctx, rowptr, col)
    rng = np.random.default_rng(1)
    p0 = (rng.random(w.n) ** 4).astype(np.float32)
    p0 /= p0.sum(dtype=np.float64)
    p0 = p0.astype(np.float32)
    for fanouts in (w.fanouts, [15, 10, 5], [7], [3, 1000]):
        Q = qv.qv_psgs(ctx, g, fanouts)
        P = qv.qv_access_prob(ctx, g, fanouts)
        P2 = qv.qv_access_prob(ctx, g, fanouts, p0=dev(p0))
        ctx.sync()
        oQ = oracle.psgs(rowptr, col, fanouts)
        assert rel_err(Q.cpu().numpy(), oQ) <= REL_TOL
        assert rel_err(P.cpu().numpy(), oracle.access_prob(rowptr, col, fanouts)) <= REL_TOL
        assert rel_err(P2.cpu().numpy(), oracle.access_prob(rowptr, col, fanouts, p0=p0.astype(np.float64))) <= REL_TOL
        # accesses per request == expected sample size, on the GPU's own numbers
        assert abs(P.double().sum().item() - Q.double().mean().item()) <= 1e-4 * oQ.mean()
        # the same through the in-edge CSR (gather sweeps, no atomics)
        if fanouts is w.fanouts or len(fanouts) == 3:
            g_in = transposed_graph(qv, ctx, rowptr, col)
            P3 = qv.qv_access_prob(ctx, g, fanouts, graph_in=g_in)
            P4 = qv.qv_access_prob(ctx, g, fanouts, p0=dev(p0), graph_in=g_in)
            ctx.sync()
            assert rel_err(P3.cpu().numpy(), oracle.access_prob(rowptr, col, fanouts)) <= REL_TOL
            assert rel_err(P4.cpu().numpy(), oracle.access_prob(rowptr, col, fanouts, p0=p0.astype(np.float64))) <= REL_TOL
    seeds = w.seeds(0)
    Q = qv.qv_psgs(ctx, g, w.fanouts)
    s = qv.qv_psgs_batch_sum(ctx, Q, dev(seeds))
    ctx.sync()
    assert abs(s.item() - oracle.psgs(rowptr, col, w.fanouts)[seeds].sum()) <= 1e-4 * s.item()


def transpose_csr(rowptr, col):
    """In-edge CSR built with numpy only (a stable sort of the edges by destination)."""
    n = len(rowptr) - 1
    src = np.repeat(np.arange(n, dtype=np.int32), np.diff(rowptr))
    order = np.argsort(col, kind="stable")
    rowptr_t = np.zeros(n + 1, dtype=rowptr.dtype)
    np.cumsum(np.bincount(col, minlength=n), out=rowptr_t[1:])
    return rowptr_t, src[order]


def transposed_graph(qv, ctx, rowptr, col):
    rt, ct = transpose_csr(rowptr, col)
    return make_graph(qv, ctx, rt, ct)


@pytest.mark.parametrize("rp_dtype", [np.int32, np.int64])
def test_psgs_with_out_rows_beyond_the_per_group_limit(qv, ctx, rp_dtype):
    """A few nodes have tens of thousands of out-edges: their rows are summed a workgroup per row
    (listed by the first edge-reading sweep, reused by the later ones); one row sits just below
    the limit, one just above it."""
    rng = np.random.default_rng(21)
    n = 50_000
    deg = rng.integers(0, 10, n)
    deg[rng.random(n) < 0.1] = 0
    deg[[5, 777, 49_999]] = [30_001, 8_193, 12_345]
    deg[6] = 8_192
    rowptr = np.zeros(n + 1, dtype=rp_dtype)
    np.cumsum(deg, out=rowptr[1:])
    col = rng.integers(0, n, int(rowptr[-1])).astype(np.int32)
    g = make_graph(qv, ctx, rowptr, col)
    for fanouts in ([15, 10, 5], [3, 1000, 2, 7], [4]):
        Q = qv.qv_psgs(ctx, g, fanouts)
        ctx.sync()
        assert rel_err(Q.cpu().numpy(), oracle.psgs(rowptr, col, fanouts)) <= REL_TOL


@pytest.mark.parametrize("rp_dtype", [np.int32, np.int64])
def test_access_prob_in_edge_form_directed_graph_with_hub_rows(qv, ctx, rp_dtype):
    """A directed graph in which a few nodes receive tens of thousands of edges (in-rows beyond the
    per-group limit, handled a block per row) and some nodes have no out- or no in-edges."""
    rng = np.random.default_rng(20)
    n = 60_000
    deg = rng.integers(0, 12, n)
    deg[rng.random(n) < 0.1] = 0
    rowptr = np.zeros(n + 1, dtype=rp_dtype)
    np.cumsum(deg, out=rowptr[1:])
    col = rng.integers(100, n, int(rowptr[-1])).astype(np.int32)
    hub = rng.random(len(col))
    col[hub < 0.10] = 3                       # ~33k in-edges
    col[(hub >= 0.10) & (hub < 0.14)] = 4     # ~13k in-edges
    col[(hub >= 0.14) & (hub < 0.16)] = 5     # below the limit
    g = make_graph(qv, ctx, rowptr, col)
    rt, ct = transpose_csr(rowptr, col)
    d_in = np.diff(rt)
    assert d_in.max() > 20_000 and 8_192 < d_in[4] < 20_000 and d_in[5] < 8_192 and (d_in == 0).any()
    g_in = make_graph(qv, ctx, rt.astype(np.int64 if rp_dtype is np.int32 else np.int32), ct)
    # the library's own transpose: identical arrays (sources ascending within a row), same width
    g_lib = g.transpose()
    assert g_lib.fap_items() is None and g.fap_items() is None      # one block of source ids: no work items
    lrt, lct = g_lib.arrays()
    assert lrt.cpu().numpy().dtype == rp_dtype
    assert np.array_equal(lrt.cpu().numpy(), rt) and np.array_equal(lct.cpu().numpy(), ct)
    P = qv.qv_access_prob(ctx, g, [5, 4, 3], graph_in=g_lib)
    ctx.sync()
    assert rel_err(P.cpu().numpy(), oracle.access_prob(rowptr, col, [5, 4, 3])) <= REL_TOL
    # transposing twice gives the graph with every row sorted
    brt, bct = g_lib.transpose().arrays()
    assert np.array_equal(brt.cpu().numpy(), rowptr)
    want_sorted = np.concatenate([np.sort(col[rowptr[v]:rowptr[v + 1]]) for v in range(0, n, 997)])
    got_sorted = np.concatenate([bct.cpu().numpy()[rowptr[v]:rowptr[v + 1]] for v in range(0, n, 997)])
    assert np.array_equal(got_sorted, want_sorted)
    sparse_p0 = np.zeros(n, dtype=np.float32)           # mass on a few nodes only: the first sweeps scatter
    sparse_p0[[7, 1234, 40_000, 59_999]] = [0.4, 0.3, 0.2, 0.1]
    for fanouts in ([5, 4, 3], [20], [2, 2, 2, 2]):
        want = oracle.access_prob(rowptr, col, fanouts)
        want_sparse = oracle.access_prob(rowptr, col, fanouts, p0=sparse_p0.astype(np.float64))
        Ppush = qv.qv_access_prob(ctx, g, fanouts)
        ctx.sync()
        assert rel_err(Ppush.cpu().numpy(), want) <= REL_TOL
        for direction in (0, 1, 2):                     # choose per sweep, gather only, scatter only
            ctx.set_fap_direction(direction)
            P = qv.qv_access_prob(ctx, g, fanouts, graph_in=g_in)
            Ps = qv.qv_access_prob(ctx, g, fanouts, p0=dev(sparse_p0), graph_in=g_in)
            ctx.sync()
            assert rel_err(P.cpu().numpy(), want) <= REL_TOL, direction
            assert rel_err(Ps.cpu().numpy(), want_sparse) <= REL_TOL, direction
        ctx.set_fap_direction(0)
    # in-edge CSRs the library built carry the long rows cut into work items (runs of edges whose sources
    # lie in one block of node ids): those rows are then summed block by block.  Blocks of 4,096 and of 64
    # ids here, so that the hubs' rows are cut into 15 and into 938 parts (with the default block this
    # graph fits one block and has no items)
    for block_log2 in (12, 6):
        ctx.set_fap_block(block_log2)
        g_cut = g.transpose()
        ctx.set_fap_block(0)
        crt, cct = g_cut.arrays()
        assert np.array_equal(crt.cpu().numpy(), rt) and np.array_equal(cct.cpu().numpy(), ct)
        long_rows, items, log2 = g_cut.fap_items()
        long_rows, items = long_rows.cpu().numpy(), items.cpu().numpy()
        assert log2 == block_log2 and sorted(long_rows.tolist()) == np.flatnonzero(d_in > 8192).tolist()
        first = items[:, 0].astype(np.uint32).astype(np.int64) | (items[:, 1].astype(np.int64) << 32)
        k, count = items[:, 2], items[:, 3].astype(np.int64)
        assert count.min() >= 1 and count.max() <= 256 and k.min() >= 0 and k.max() < len(long_rows)
        block_lo, block_hi = ct[first] >> log2, ct[first + count - 1] >> log2
        assert np.array_equal(block_lo, block_hi) and (np.diff(block_lo) >= 0).all()     # one block each, block by block
        for kk, i in enumerate(long_rows):                 # the items of a row cover its edges exactly once
            mine = np.flatnonzero(k == kk)
            order = mine[np.argsort(first[mine], kind="stable")]
            assert first[order[0]] == rt[i] and first[order[-1]] + count[order[-1]] == rt[i + 1]
            assert np.array_equal(first[order[1:]], first[order[:-1]] + count[order[:-1]])
        for fanouts in ([5, 4, 3], [20]):
            want = oracle.access_prob(rowptr, col, fanouts)
            want_sparse = oracle.access_prob(rowptr, col, fanouts, p0=sparse_p0.astype(np.float64))
            for direction in (0, 1):
                ctx.set_fap_direction(direction)
                P = qv.qv_access_prob(ctx, g, fanouts, graph_in=g_cut)
                Ps = qv.qv_access_prob(ctx, g, fanouts, p0=dev(sparse_p0), graph_in=g_cut)
                P2 = qv.qv_access_prob(ctx, g, fanouts, graph_in=g_cut)      # the sums start from zero again
                ctx.sync()
                assert rel_err(P.cpu().numpy(), want) <= REL_TOL, (block_log2, direction)
                assert rel_err(Ps.cpu().numpy(), want_sparse) <= REL_TOL, (block_log2, direction)
                assert rel_err(P2.cpu().numpy(), want) <= REL_TOL, (block_log2, direction)
            ctx.set_fap_direction(0)
        del g_cut
    with pytest.raises(qv.QvError):
        ctx.set_fap_block(5)
    other_rowptr = np.ones(n, dtype=np.int64)          # n-1 nodes, one edge
    other_rowptr[0] = 0
    other = make_graph(qv, ctx, other_rowptr, np.zeros(1, dtype=np.int32))
    with pytest.raises(qv.QvError):
        qv.qv_access_prob(ctx, g, [3], graph_in=other)


def test_access_prob_rows_at_the_long_row_limit(qv, ctx):
    # in-rows of exactly 8,192 edges (summed by a group of lanes) and of 8,193 (the long-row paths: a workgroup
    # per row, or work items by block of sources when the library built the in-edge CSR with small blocks)
    rng = np.random.default_rng(31)
    n, A, B = 20_000, 19_000, 19_001
    rows = [list(rng.integers(100, 18_000, 2)) for _ in range(n)]
    for j in range(8192):
        rows[j].append(A)
    for j in range(8193):
        rows[j].append(B)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum([len(r) for r in rows], out=rowptr[1:])
    col = np.concatenate([np.array(r, dtype=np.int32) for r in rows])
    g = make_graph(qv, ctx, rowptr, col)
    want = oracle.access_prob(rowptr, col, [3, 2])
    rt, ct = transpose_csr(rowptr, col)
    assert rt[A + 1] - rt[A] == 8192 and rt[B + 1] - rt[B] == 8193
    for block_log2 in (0, 6):
        ctx.set_fap_block(block_log2)
        g_in = g.transpose()
        ctx.set_fap_block(0)
        items = g_in.fap_items()
        if block_log2:
            assert items is not None and items[0].cpu().tolist() == [B]
        else:
            assert items is None
        for direction in (0, 1):
            ctx.set_fap_direction(direction)
            P = qv.qv_access_prob(ctx, g, [3, 2], graph_in=g_in)
            ctx.sync()
            assert rel_err(P.cpu().numpy(), want) <= REL_TOL, (block_log2, direction)
        ctx.set_fap_direction(0)
        del g_in


def test_csr_transpose_degenerate_graphs(qv, ctx):
    # no edges at all, a single node with a self loop, and parallel edges
    g0 = make_graph(qv, ctx, np.zeros(6, dtype=np.int64), np.zeros(0, dtype=np.int32))
    rt, ct = g0.transpose().arrays()
    assert np.array_equal(rt.cpu().numpy(), np.zeros(6, dtype=np.int64)) and ct.numel() == 0
    g1 = make_graph(qv, ctx, np.array([0, 1], dtype=np.int32), np.array([0], dtype=np.int32))
    rt, ct = g1.transpose().arrays()
    assert rt.cpu().tolist() == [0, 1] and ct.cpu().tolist() == [0]
    rowptr = np.array([0, 3, 3, 5], dtype=np.int32)
    col = np.array([2, 2, 1, 0, 2], dtype=np.int32)
    rt, ct = make_graph(qv, ctx, rowptr, col).transpose().arrays()
    ert, ect = transpose_csr(rowptr, col)
    assert rt.cpu().tolist() == ert.tolist() == [0, 1, 2, 5] and ct.cpu().tolist() == ect.tolist() == [2, 0, 0, 0, 2]


def test_place_rank_large_with_ties(qv, ctx):
    rng = np.random.default_rng(8)
    prob = rng.random(1_000_003).astype(np.float32)
    prob[rng.integers(0, len(prob), 300000)] = np.float32(0.125)
    prob[rng.integers(0, len(prob), 1000)] = 0.0
    rank = qv.qv_place_rank(ctx, dev(prob))
    ctx.sync()
    assert np.array_equal(rank.cpu().numpy(), oracle.place(prob, 0)[0])
