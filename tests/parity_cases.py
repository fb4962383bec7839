"""Parity cases shared by the GPU tests and by the CPU-emulated kernel checks: each
function runs one operation of the library through its C ABI on buffers supplied by a
backend and compares the result word for word with the CPU oracle on the same seeded
inputs.  Bit-exact is the bar: all ciphertext arithmetic is integer mod q_i."""
import contextlib

import numpy as np

from oracle import oracle as orc
from paper_1911_11377_amd import ckksmi
from paper_1911_11377_amd import workloads as wl
from helpers import Material


class _Tunable:
    """contexts made inside `with be.tuned(n):` aim for n workgroups per transform launch, so that a small batch
    still makes the workgroups loop over items"""
    target_wgs = None

    @contextlib.contextmanager
    def tuned(self, target_wgs):
        old, self.target_wgs = self.target_wgs, target_wgs
        try:
            yield self
        finally:
            self.target_wgs = old

    def _tune(self, ctx):
        if self.target_wgs:
            ctx.tune_target_wgs(self.target_wgs)
        return ctx


class GpuBackend(_Tunable):
    """device buffers are torch tensors on cuda:0"""

    def __init__(self):
        import torch

        self.torch = torch
        assert torch.cuda.is_available(), "GPU tests need a GPU"
        self.lib_path = None

    def context(self, logN, n_q, q_bits, k, special_bits, alpha):
        return self._tune(ckksmi.Context(logN, n_q, q_bits, k, special_bits, alpha, device=0))

    def to_dev(self, arr, dtype=np.uint64):
        a = np.ascontiguousarray(arr, dtype=dtype)
        return self.torch.from_numpy(a.view(np.int64)).to("cuda:0")

    def empty(self, *shape):
        return self.torch.empty(shape, dtype=self.torch.int64, device="cuda:0")

    def ws(self, nbytes):
        return self.torch.empty(max(nbytes // 8, 1), dtype=self.torch.int64, device="cuda:0")

    def to_host(self, buf):
        self.torch.cuda.synchronize()
        return buf.cpu().numpy().view(np.uint64)

    stream = None


class EmuBackend(_Tunable):
    """'device' buffers are guard-paged host memory; kernels run as CPU fibers"""

    def __init__(self):
        import emu_support

        self.es = emu_support
        self.lib_path = emu_support.emu_lib_path()
        self.lib = ckksmi.load(self.lib_path)

    def context(self, logN, n_q, q_bits, k, special_bits, alpha):
        return self._tune(ckksmi.Context(logN, n_q, q_bits, k, special_bits, alpha, device=0, lib=self.lib_path))

    def to_dev(self, arr, dtype=np.uint64):
        return self.es.to_emu(self.lib, arr, dtype)

    def empty(self, *shape):
        b = self.es.EmuBuf(self.lib, shape)
        b.np[...] = 0xDEADBEEFDEADBEEF
        return b

    def ws(self, nbytes):
        return self.es.EmuBuf(self.lib, (max(nbytes // 8, 1),))

    def to_host(self, buf):
        return buf.np.copy()

    stream = 0


def make_material(shape, seed, rotations=()):
    logN, n_q, q_bits, k, special_bits, alpha = shape
    return Material(logN, n_q, q_bits, k, special_bits, alpha, seed=seed, rotations=rotations)


def random_cts(M, level, batch, seed, tag, comps=2):
    """uniform residues: ciphertexts are pseudorandom, and parity does not need them to decrypt"""
    return wl.uniform_limbs(M.O.q[:level], M.N, seed, tag, lead=(batch, comps))


def check_moduli(ctx, M):
    assert ctx.moduli == M.O.moduli and ctx.psis == M.O.psis


def case_ntt(be, shape, seed, batch=2):
    logN, n_q, q_bits, k, special_bits, alpha = shape
    O = orc.Oracle(logN, n_q, q_bits, k, special_bits, alpha)
    ctx = be.context(*shape)
    assert ctx.moduli == O.moduli and ctx.psis == O.psis
    idx = list(range(O.n_q + O.k))
    idx = idx[::-1][: min(len(idx), 5)]  # a few limbs, special primes first
    x = wl.uniform_limbs([O.moduli[t] for t in idx], O.N, seed, "ntt", lead=(batch,))
    d = be.to_dev(x)
    ctx.ntt(d, idx, batch, stream=be.stream)
    got = be.to_host(d).reshape(x.shape)
    for b in range(batch):
        want = O.ntt_limbs(x[b], idx)
        assert np.array_equal(got[b], want), "forward transform differs from the oracle"
    ctx.intt(d, idx, batch, stream=be.stream)
    assert np.array_equal(be.to_host(d).reshape(x.shape), x), "inverse(forward(x)) != x"
    # inverse against the oracle on fresh data
    d2 = be.to_dev(x)
    ctx.intt(d2, idx, batch, stream=be.stream)
    got = be.to_host(d2).reshape(x.shape)
    assert np.array_equal(got[0], O.intt_limbs(x[0], idx))
    ctx.close()


def case_elementwise(be, shape, seed, batch=3):
    M = make_material(shape, seed)
    O = M.O
    ctx = be.context(*shape)
    check_moduli(ctx, M)
    level = O.n_q
    a, b = random_cts(M, level, batch, seed, "a"), random_cts(M, level, batch, seed, "b")
    da, db = be.to_dev(a), be.to_dev(b)
    out = be.empty(batch, 2, level, O.N)
    ctx.add(da, db, out, level, batch, stream=be.stream)
    got = be.to_host(out).reshape(a.shape)
    assert all(np.array_equal(got[i], O.add(a[i], b[i], level)) for i in range(batch))
    ctx.sub(da, db, out, level, batch, stream=be.stream)
    got = be.to_host(out).reshape(a.shape)
    assert all(np.array_equal(got[i], O.sub(a[i], b[i], level)) for i in range(batch))
    for cst in (-123456789012345, 3, -(1 << 62) + 12345):
        ctx.mul_scalar(da, cst, out, level, batch, stream=be.stream)
        got = be.to_host(out).reshape(a.shape)
        assert all(np.array_equal(got[i], O.mul_scalar(a[i], cst, level)) for i in range(batch))
        ctx.add_const(da, cst, out, level, batch, stream=be.stream)
        got = be.to_host(out).reshape(a.shape)
        assert all(np.array_equal(got[i], O.add_const(a[i], cst, level)) for i in range(batch))
    pt = wl.uniform_limbs(O.q[:level], O.N, seed, "pt", lead=(batch,))
    dpt = be.to_dev(pt)
    ctx.mul_plain(da, dpt, level * O.N, out, level, batch, stream=be.stream)
    got = be.to_host(out).reshape(a.shape)
    assert all(np.array_equal(got[i], O.mul_plain(a[i], pt[i], level)) for i in range(batch))
    ctx.mul_plain(da, dpt, 0, out, level, batch, stream=be.stream)
    got = be.to_host(out).reshape(a.shape)
    assert all(np.array_equal(got[i], O.mul_plain(a[i], pt[0], level)) for i in range(batch))
    if level > 1:
        lo = level - 1
        outd = be.empty(batch, 2, lo, O.N)
        ctx.mod_drop(da, level, lo, outd, batch, stream=be.stream)
        got = be.to_host(outd).reshape(batch, 2, lo, O.N)
        assert all(np.array_equal(got[i], O.mod_drop(a[i], level, lo)) for i in range(batch))
    d3 = be.empty(batch, 3, level, O.N)
    ctx.hmul(da, db, d3, level, batch, stream=be.stream)
    got = be.to_host(d3).reshape(batch, 3, level, O.N)
    assert all(np.array_equal(got[i], O.tensor(a[i], b[i], level)) for i in range(batch))
    ctx.close()


def case_plain_mac(be, shape, seed, n_ct=5, level=None):
    """grouped sums of plaintext x ciphertext products against the oracle's products and additions term by term: eleven
    sums (two chunks of groups), one of them empty; a table entry beyond the plaintexts counts as none (documented: no
    access outside the buffers)"""
    M = make_material(shape, seed)
    O = M.O
    ctx = be.context(*shape)
    level = level or O.n_q
    cts = random_cts(M, level, n_ct, seed, "mac.ct")
    n_groups = 11
    r = wl.rng(seed, "mac.table")
    table = np.full((n_groups, n_ct), -1, dtype=np.int32)
    n_pts = 0
    for g in range(n_groups):
        for sct in range(n_ct):
            if g != 3 and r.random() < 0.6:
                table[g, sct] = n_pts
                n_pts += 1
    pts = wl.uniform_limbs(O.q[:level], O.N, seed, "mac.pt", lead=(n_pts,))
    bad = table.copy()
    bad[3, 0] = n_pts + 5  # beyond the plaintexts: none
    def i32(v):
        a = np.zeros((len(v) + 1) // 2 * 2 + 2, dtype=np.int32)
        a[: len(v)] = v
        return be.to_dev(a.view(np.uint64))
    out = be.empty(n_groups, 2, level, O.N)
    dc, dp = be.to_dev(cts), be.to_dev(pts)
    ctx.plain_mac(dc, n_ct, dp, n_pts, i32(bad.reshape(-1)), n_groups, out, level, stream=be.stream)
    got = be.to_host(out).reshape(n_groups, 2, level, O.N)
    for g in range(n_groups):
        want = np.zeros((2, level, O.N), dtype=np.uint64)
        for sct in range(n_ct):
            if table[g, sct] >= 0:
                want = O.add(want, O.mul_plain(cts[sct], pts[table[g, sct]], level), level)
        assert np.array_equal(got[g], want), "grouped plaintext products differ from the oracle (group %d)" % g
    assert not got[3].any()
    # refusals: overlapping output, no ciphertexts
    with_rc = lambda fn, *a: _rc(fn, *a, stream=be.stream)
    assert with_rc(ctx.plain_mac, dc, n_ct, dp, n_pts, i32(table.reshape(-1)), n_groups, dc, level) == ckksmi.EINVAL
    assert with_rc(ctx.plain_mac, dc, 0, dp, n_pts, i32(table.reshape(-1)), n_groups, out, level) == ckksmi.EINVAL
    ctx.close()


def _rc(fn, *args, **kw):
    try:
        fn(*args, **kw)
    except ckksmi.CkksmiError as e:
        return e.code
    return 0


def case_rescale(be, shape, seed, batch=2, levels=None):
    M = make_material(shape, seed)
    O = M.O
    ctx = be.context(*shape)
    for level in levels or [O.n_q, 2]:
        if level < 2 or level > O.n_q:
            continue
        a = random_cts(M, level, batch, seed, ("rs", level))
        da = be.to_dev(a)
        out = be.empty(batch, 2, level - 1, O.N)
        ws = be.ws(ctx.workspace_bytes(ckksmi.OP_RESCALE, level, batch))
        ctx.rescale(da, out, level, batch, ws, stream=be.stream)
        got = be.to_host(out).reshape(batch, 2, level - 1, O.N)
        for i in range(batch):
            assert np.array_equal(got[i], O.rescale(a[i], level)), "rescale differs at level %d" % level
        assert np.array_equal(be.to_host(da).reshape(a.shape), a), "rescale modified its input"
        # the same division of a scalar multiple, in one call: the bits of the two calls
        for cst in (-(1 << 38) + 12345, 7, (1 << 52) + 3):
            out2 = be.empty(batch, 2, level - 1, O.N)
            nb = ctx.workspace_bytes(ckksmi.OP_MUL_SCALAR_RESCALE, level, batch)
            ws2 = be.ws(nb // batch + 8 if (batch > 1 and cst == 7) else nb)  # once with room for one item only
            ctx.mul_scalar_rescale(da, cst, out2, level, batch, ws2, stream=be.stream)
            got2 = be.to_host(out2).reshape(batch, 2, level - 1, O.N)
            for i in range(batch):
                assert np.array_equal(got2[i], O.rescale(O.mul_scalar(a[i], cst, level), level)), "scalar rescale differs at level %d" % level
        assert np.array_equal(be.to_host(da).reshape(a.shape), a), "scalar rescale modified its input"
        if level >= 3:  # input stored one level higher: the drop rides along
            out3 = be.empty(batch, 2, level - 2, O.N)
            ctx.mul_scalar_rescale(da, -99991, out3, level - 1, batch, be.ws(ctx.workspace_bytes(ckksmi.OP_MUL_SCALAR_RESCALE, level - 1, batch)),
                                   stream=be.stream, level_in=level)
            got3 = be.to_host(out3).reshape(batch, 2, level - 2, O.N)
            for i in range(batch):
                want = O.rescale(O.mul_scalar(a[i][:, : level - 1], -99991, level - 1), level - 1)
                assert np.array_equal(got3[i], want), "scalar rescale with a drop differs at level %d" % level
            # ... and added onto a ciphertext already in the output buffer
            base = random_cts(M, level - 2, batch, seed, ("rs.add", level))
            out4 = be.to_dev(base)
            ctx.mul_scalar_rescale(da, -99991, out4, level - 1, batch, be.ws(ctx.workspace_bytes(ckksmi.OP_MUL_SCALAR_RESCALE, level - 1, batch)),
                                   stream=be.stream, level_in=level, addend=out4)
            got4 = be.to_host(out4).reshape(batch, 2, level - 2, O.N)
            for i in range(batch):
                want = O.add(O.rescale(O.mul_scalar(a[i][:, : level - 1], -99991, level - 1), level - 1), base[i], level - 2)
                assert np.array_equal(got4[i], want), "scalar rescale with an addend differs at level %d" % level
    ctx.close()


def case_relin_and_composite(be, shape, seed, batch=2, levels=None, small_ws=False):
    M = make_material(shape, seed)
    O = M.O
    ctx = be.context(*shape)
    check_moduli(ctx, M)
    evk = be.to_dev(M.rlk)
    for level in levels or [O.n_q]:
        a, b = random_cts(M, level, batch, seed, ("a", level)), random_cts(M, level, batch, seed, ("b", level))
        da, db = be.to_dev(a), be.to_dev(b)
        d = be.empty(batch, 3, level, O.N)
        ctx.hmul(da, db, d, level, batch, stream=be.stream)
        r = be.empty(batch, 2, level, O.N)
        nbytes = ctx.workspace_bytes(ckksmi.OP_RELIN, level, batch)
        if small_ws and batch > 1:
            nbytes = nbytes // batch + 8  # forces one item per sweep
        ws = be.ws(nbytes)
        ctx.relin(d, evk, r, level, batch, ws, stream=be.stream)
        got_r = be.to_host(r).reshape(batch, 2, level, O.N)
        hd = be.to_host(d).reshape(batch, 3, level, O.N)
        for i in range(batch):
            assert np.array_equal(got_r[i], O.relin(hd[i], M.rlk, level)), "relin differs at level %d item %d" % (level, i)
        if level >= 2:
            out = be.empty(batch, 2, level - 1, O.N)
            ws2 = be.ws(ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, level, batch))
            ctx.hmul_relin_rescale(da, db, evk, out, level, batch, ws2, stream=be.stream)
            got = be.to_host(out).reshape(batch, 2, level - 1, O.N)
            for i in range(batch):
                assert np.array_equal(got[i], O.hmul_relin_rescale(a[i], b[i], M.rlk, level)), "composite differs"
            # and equals the three-call sequence
            out3 = be.empty(batch, 2, level - 1, O.N)
            ws3 = be.ws(ctx.workspace_bytes(ckksmi.OP_RESCALE, level, batch))
            ctx.rescale(r, out3, level, batch, ws3, stream=be.stream)
            assert np.array_equal(be.to_host(out3), be.to_host(out))
    ctx.close()


def case_merged_product(be, shape, seed, batch=2, levels=None, small_ws=False, expect_kernel=None):
    """the product with one division by P*q_last, word for word against the oracle's definition of it"""
    M = make_material(shape, seed)
    O = M.O
    ctx = be.context(*shape)
    check_moduli(ctx, M)
    evk = be.to_dev(M.rlk)
    for level in levels or [O.n_q]:
        a, b = random_cts(M, level, batch, seed, ("ma", level)), random_cts(M, level, batch, seed, ("mb", level))
        da, db = be.to_dev(a), be.to_dev(b)
        out = be.empty(batch, 2, level - 1, O.N)
        nbytes = ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, level, batch)
        if small_ws and batch > 1:
            nbytes = nbytes // batch + 8
        ws = be.ws(nbytes)
        if expect_kernel:
            ctx.profile_enable(True)
        ctx.hmul_relin_rescale_merged(da, db, evk, out, level, batch, ws, stream=be.stream)
        got = be.to_host(out).reshape(batch, 2, level - 1, O.N)
        if expect_kernel:
            ran = ctx.profile_read()
            ctx.profile_enable(False)
            assert any(expect_kernel in n for n in ran), (expect_kernel, list(ran))
        for i in range(batch):
            assert np.array_equal(got[i], O.hmul_relin_rescale_merged(a[i], b[i], M.rlk, level)), "merged product differs at level %d item %d" % (level, i)
    ctx.close()


def case_rotate(be, shape, seed, rotations, batch=4, level=None):
    M = make_material(shape, seed, rotations=rotations)
    O = M.O
    ctx = be.context(*shape)
    level = level or O.n_q
    keys = {r: be.to_dev(M.gk[r]) for r in rotations}
    for r in rotations:
        ctx.galois_key_register(r, keys[r])
    a = random_cts(M, level, batch, seed, "rot")
    da = be.to_dev(a)
    rots = [rotations[i % len(rotations)] for i in range(batch)]
    out = be.empty(batch, 2, level, O.N)
    ws = be.ws(ctx.workspace_bytes(ckksmi.OP_ROTATE, level, batch))
    ctx.rotate(da, rots, out, level, batch, ws, stream=be.stream)
    got = be.to_host(out).reshape(batch, 2, level, O.N)
    for i in range(batch):
        assert np.array_equal(got[i], O.rotate(a[i], rots[i], M.gk[rots[i]], level)), "rotate item %d by %d differs" % (i, rots[i])
    # a rotation without a key is refused before anything runs
    try:
        ctx.rotate(da, [max(rotations) + 11] * batch, out, level, batch, ws, stream=be.stream)
        raise AssertionError("missing key not reported")
    except ckksmi.CkksmiError as e:
        assert e.code == ckksmi.ENOKEY
    ctx.close()


def case_sum_of_products(be, shape, seed, terms, batch=2, levels=None):
    """one relinearisation and rescale for a sum of products, word for word against the oracle"""
    M = make_material(shape, seed)
    O = M.O
    ctx = be.context(*shape)
    evk = be.to_dev(M.rlk)
    for level in levels or [O.n_q]:
        a = wl.uniform_limbs(O.q[:level], O.N, seed, ("sa", level), lead=(batch, terms, 2))
        b = wl.uniform_limbs(O.q[:level], O.N, seed, ("sb", level), lead=(batch, terms, 2))
        out = be.empty(batch, 2, level - 1, O.N)
        ws = be.ws(ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, level, batch))
        ctx.hmul_sum_relin_rescale(be.to_dev(a), be.to_dev(b), terms, evk, out, level, batch, ws, stream=be.stream)
        got = be.to_host(out).reshape(batch, 2, level - 1, O.N)
        for i in range(batch):
            assert np.array_equal(got[i], O.hmul_sum_relin_rescale(a[i], b[i], M.rlk, level)), "sum of products differs at level %d item %d" % (level, i)
    ctx.close()


def case_rotate_hoisted(be, shape, seed, rotations, batch=3, level=None, small_ws=False):
    """every item through every rotation with one shared ModUp, word for word against the oracle's definition of it"""
    M = make_material(shape, seed, rotations=rotations)
    O = M.O
    ctx = be.context(*shape)
    level = level or O.n_q
    keys = {r: be.to_dev(M.gk[r]) for r in rotations}
    for r in rotations:
        ctx.galois_key_register(r, keys[r])
    a = random_cts(M, level, batch, seed, "hoist")
    da = be.to_dev(a)
    R = len(rotations)
    out = be.empty(batch, R, 2, level, O.N)
    nbytes = ctx.rotate_hoisted_workspace_bytes(level, batch, R)
    if small_ws and batch > 1:
        nbytes = nbytes // batch + 8  # one item per sweep
    ws = be.ws(nbytes)
    ctx.rotate_hoisted(da, list(rotations), out, level, batch, ws, stream=be.stream)
    got = be.to_host(out).reshape(batch, R, 2, level, O.N)
    for i in range(batch):
        want = O.rotate_hoisted(a[i], rotations, [M.gk[r] for r in rotations], level)
        for k, r in enumerate(rotations):
            assert np.array_equal(got[i, k], want[k]), "hoisted rotation of item %d by %d differs" % (i, r)
    half = O.N // 2
    missing = next(r for r in range(1, half) if all((q - r) % half for q in rotations))
    try:
        ctx.rotate_hoisted(da, [missing], out, level, batch, ws, stream=be.stream)
        raise AssertionError("missing key not reported")
    except ckksmi.CkksmiError as e:
        assert e.code == ckksmi.ENOKEY
    ctx.close()


def case_packed_layer(be, shape, seed, M_float, level=None, max_rotations=None):
    """a rotation-packed layer (matrix through hoisted rotations, plaintext diagonals, tree of adds, rescale) against the
    oracle's schedule, word for word; the encoded diagonals are inputs of both sides"""
    from paper_1911_11377_amd import packed
    probe = be.context(*shape)
    level = level or probe.n_q
    n_slots = probe.N // 2
    probe.close()
    Msq = packed.square_pad(M_float)
    diags_lib = packed.matrix_diagonals(Msq, n_slots)
    diags = orc.matrix_diagonals(Msq, n_slots)
    assert sorted(diags) == sorted(diags_lib) and all(np.array_equal(diags[d], diags_lib[d]) for d in diags)
    rots = tuple(d for d in sorted(diags) if d)
    M = make_material(shape, seed, rotations=rots)
    O = M.O
    ctx = be.context(*shape)
    check_moduli(ctx, M)
    keys = {r: be.to_dev(M.gk[r]) for r in rots}
    for r in rots:
        ctx.galois_key_register(r, keys[r])
    n = Msq.shape[0]
    z = np.tile(wl.slots_real(n, seed, "packed").real, n_slots // n).astype(np.complex128)
    scale = 2.0 ** 30
    x = M.encrypt(z, scale, level, "packed")
    pts = {}

    def encode(values, s, l):
        pt = M.encode(values, s, l)
        pts[len(pts)] = pt
        return pt

    plan = packed.plan_linear(ctx, M_float, level, be.to_dev, encode=encode)
    order = ([] if plan.pt0 is None else [0])
    by_d = dict(zip(list(plan.rotations) + order, [pts[i] for i in range(len(pts))]))
    out = be.empty(2, level - 1, O.N)
    mr = max_rotations or packed.MAX_ROTATIONS_PER_CALL
    ws = be.ws(packed.workspace_bytes(ctx, plan, mr))
    packed.linear_transform(ctx, be.to_dev(x), plan, out, ws, stream=be.stream, max_rotations=mr)
    got = be.to_host(out).reshape(2, level - 1, O.N)
    want = O.linear_transform(x, by_d, M.gk, level)
    assert np.array_equal(got, want), "packed layer differs from the oracle"
    dec = M.decrypt(got, scale, level - 1).real[:n]
    assert np.max(np.abs(dec - Msq @ z.real[:n])) < 1e-3
    ctx.close()


def case_packed_network(be, shape, seed, topology, sigma=0.25, max_rotations=None, bsgs=False):
    """one image through a network in the rotation-packed layout (strided convolution and pooling as matrices, vectors that
    may span several ciphertexts, degree-2 activations) against the oracle's schedule: every output ciphertext word for
    word, and decrypted against the float network.  The stage matrices, the activation constants and the encoded diagonals
    are the test's own (from the oracle's definitions) and must equal the library's plan."""
    import helpers
    from paper_1911_11377_amd import packed
    probe = orc.Oracle(*shape)
    n_slots, level, s = probe.N // 2, probe.n_q, 2.0 ** 50
    weights = wl.cnn_weights_float(topology, seed, sigma=sigma)
    stages = helpers.network_stage_matrices(topology, weights)
    lib_stages = packed.stage_matrices(wl.cnn_shapes(topology), weights)
    assert len(stages) == len(lib_stages)
    for a, b in zip(stages, lib_stages):
        assert a[0] == b[0] and (a[0] != "linear" or np.allclose(a[1], b[1], rtol=0, atol=1e-15)), "stage matrices differ"
    n = helpers.network_period(stages, n_slots)
    rots = sorted({d for st in stages if st[0] == "linear" for dd in orc.block_diagonals(st[1], n, n_slots).values() for d in dd if d})
    if bsgs:  # baby steps and giant steps: offset d = g*baby + b needs the keys of b and of g*baby only
        baby = helpers.bsgs_baby(n)
        rots = sorted({d % baby for d in rots if d % baby} | {d - d % baby for d in rots if d >= baby})
    M = make_material(shape, seed, rotations=tuple(rots))
    O = M.O
    # both sides plan from the LIBRARY's stage matrices here (they agree with the test's to rounding, and the encoder must
    # see identical inputs for identical plaintexts)
    ist, rots2, out_level, out_scale = helpers.network_integer_stages(lib_stages, O.q, level, s, n, n_slots, M.encode, bsgs=bsgs)
    assert rots2 == rots
    ctx = be.context(*shape)
    check_moduli(ctx, M)
    keys = {r: be.to_dev(M.gk[r]) for r in rots}
    for r in rots:
        ctx.galois_key_register(r, keys[r])
    plans, n_lib, lvl_lib, scale_lib = packed.plan_network(ctx, wl.cnn_shapes(topology), weights, level, s, be.to_dev, encode=M.encode, bsgs=bsgs)
    assert (n_lib, lvl_lib) == (n, out_level) and scale_lib == out_scale
    for pl, st in zip(plans, ist):
        if st[0] == "poly2":
            assert (pl.k2, pl.k1) == (st[1], st[2]), "activation constants differ"
        elif st[0] == "linear_bsgs":
            assert pl.baby == st[2] == helpers.bsgs_baby(n)
            assert sorted((i, j, g, b) for (i, j), dd in st[1].items() for (g, b) in dd) == sorted(pl.terms), "diagonals differ"
            assert set(pl.rotation_offsets()) <= set(rots)
        else:
            assert {ij: sorted(dd) for ij, dd in st[1].items()} == pl.offsets, "diagonals differ"
    C, H, W = wl.CNN_TOPOLOGIES[topology]["input"]
    img = wl.slots_real(C * H * W, seed, "image", lo=0.0, hi=1.0).real
    blocks = -(-img.size // n)
    zin = np.zeros(blocks * n)
    zin[: img.size] = img
    xs = np.stack([M.encrypt(np.tile(zin[j * n:(j + 1) * n], n_slots // n).astype(complex), s, level, ("img", j)) for j in range(blocks)])
    want, wl_level = O.packed_network(list(xs), ist, M.rlk, M.gk, level)
    mr = max_rotations or packed.MAX_ROTATIONS_PER_CALL
    ws = be.ws(packed.network_workspace_bytes(ctx, plans, level, mr))
    res, n_out, got_level = packed.run_network(ctx, be.to_dev(xs), plans, be.to_dev(M.rlk), level, ws, stream=be.stream, max_rotations=mr)
    assert (n_out, got_level) == (len(want), wl_level)
    got = be.to_host(ws).reshape(-1)
    # the result sits at a known place of the workspace: read it through the same flat view
    off = (res.data_ptr() - ws.data_ptr()) // 8
    got = got[off: off + n_out * 2 * got_level * O.N].reshape(n_out, 2, got_level, O.N)
    for i in range(n_out):
        assert np.array_equal(got[i], want[i]), "output block %d of the packed network differs from the oracle" % i
    dec = np.concatenate([M.decrypt(got[i], out_scale, got_level).real[:n] for i in range(n_out)])
    ref = helpers.network_float(stages, img)
    assert np.max(np.abs(dec[: ref.size] - ref)) < 1e-3
    ctx.close()


def case_encode_encrypt_device(be, shape, seed, batch=3, level=None, log_scale=40, complex_slots=True, small_ws=False):
    """device-side encoding (double-precision complex inverse transform: coefficients within one unit of the oracle's
    encoder, slots back within 1e-9) and device-side encryption (integer work: bit-exact against the oracle)"""
    M = make_material(shape, seed)
    O = M.O
    ctx = be.context(*shape)
    check_moduli(ctx, M)
    level = level or O.n_q
    scale = 2.0 ** log_scale
    half = O.N // 2
    zs = [wl.slots_complex(half, seed, ("enc", i)) if complex_slots else wl.slots_real(half, seed, ("enc", i)) for i in range(batch)]
    re = np.stack([z.real for z in zs]).astype(np.float64)
    im = np.stack([z.imag for z in zs]).astype(np.float64)
    pt = be.empty(batch, level, O.N)
    ws = be.ws(batch * O.N * 16)
    ctx.encode_device(be.to_dev(re, np.float64), be.to_dev(im, np.float64) if complex_slots else None, scale, level, batch, pt, ws, stream=be.stream)
    got = be.to_host(pt).reshape(batch, level, O.N)
    idx = list(range(level))
    worst = 0
    for i in range(batch):
        want = M.encode(zs[i], scale, level)
        cg = orc.crt_reconstruct(O.intt_limbs(got[i], idx), O.q[:level])
        cw = orc.crt_reconstruct(O.intt_limbs(want, idx), O.q[:level])
        worst = max(worst, max(abs(a - b) for a, b in zip(cg, cw)))
        back = orc.decode(cg, scale, O.logN)
        assert np.max(np.abs(back - zs[i])) < max(1e-9, 4.0 * O.N / scale)
    assert worst <= 1, "device encoder is %d units away from the oracle's" % worst
    # encryption of the ORACLE's plaintexts with seeded randomness: every word
    pts = np.stack([M.encode(z, scale, level) for z in zs])
    r = np.stack([wl.ternary(O.N, seed, "dev.r", i) for i in range(batch)]).astype(np.int64)
    e0 = np.stack([wl.gaussian_error(O.N, seed, "dev.e0", i) for i in range(batch)]).astype(np.int64)
    e1 = np.stack([wl.gaussian_error(O.N, seed, "dev.e1", i) for i in range(batch)]).astype(np.int64)
    ct = be.empty(batch, 2, level, O.N)
    nbytes = batch * 3 * level * O.N * 8
    if small_ws and batch > 1:
        nbytes = nbytes // batch + 8
    ws2 = be.ws(nbytes)
    ctx.encrypt_device(be.to_dev(M.pk), be.to_dev(pts), be.to_dev(r, np.int64), be.to_dev(e0, np.int64), be.to_dev(e1, np.int64), level, batch, ct, ws2,
                       stream=be.stream)
    gct = be.to_host(ct).reshape(batch, 2, level, O.N)
    for i in range(batch):
        assert np.array_equal(gct[i], O.encrypt(M.pk, pts[i], r[i], e0[i], e1[i], level)), "device encryption of item %d differs" % i
    ctx.close()


def case_sample_device(be, shape, seed, rows=3, sigma=3.2, first_index=(1 << 33) + 5):
    """the device sampler against the oracle's: integer work on counters, every coefficient"""
    ctx = be.context(*shape)
    logN = shape[0]
    for kind in (0, 1):
        out = be.empty(rows, 1 << logN)
        ctx.sample_device(kind, sigma, seed, first_index, rows, out, stream=be.stream)
        got = be.to_host(out).view(np.int64).reshape(rows, 1 << logN)
        assert np.array_equal(got, orc.sample(kind, sigma, seed, first_index, rows, logN)), "sampler kind %d differs" % kind
    ctx.close()


def case_variant_errors(be, shape=(6, 3, 30, 1, 31, 1)):
    """argument checks of the variant entry points: every refusal happens on the host, before anything is enqueued"""
    ctx = be.context(*shape)
    N, L = 1 << shape[0], shape[1]
    a = be.empty(2, 2, L, N)
    out = be.empty(2, 2, L, N)
    ws = be.ws(1 << 22)
    tiny_ws = be.ws(64)

    def refused(code, fn, *args):
        try:
            fn(*args, stream=be.stream)
        except ckksmi.CkksmiError as e:
            assert e.code == code, (fn.__name__, e.code, code)
            return
        raise AssertionError("%s accepted bad arguments" % fn.__name__)

    # empty batches are fine and enqueue nothing
    ctx.hmul_relin_rescale_merged(a, a, a, out, L, 0, ws, stream=be.stream)
    ctx.hmul_sum_relin_rescale(a, a, 3, a, out, L, 0, ws, stream=be.stream)
    ctx.sample_device(0, 3.2, 1, 0, 0, out, stream=be.stream)
    ctx.encode_device(a, None, 2.0**20, L, 0, out, ws, stream=be.stream)
    ctx.encrypt_device(a, a, a, a, a, L, 0, out, ws, stream=be.stream)
    refused(ckksmi.ELEVEL, ctx.hmul_relin_rescale_merged, a, a, a, out, 1, 1, ws)
    refused(ckksmi.ELEVEL, ctx.hmul_relin_rescale_merged, a, a, a, out, L + 1, 1, ws)
    refused(ckksmi.EWORKSPACE, ctx.hmul_relin_rescale_merged, a, a, a, out, L, 1, tiny_ws)
    refused(ckksmi.EINVAL, ctx.hmul_sum_relin_rescale, a, a, 0, a, out, L, 1, ws)
    refused(ckksmi.EWORKSPACE, ctx.hmul_sum_relin_rescale, a, a, 2, a, out, L, 1, tiny_ws)
    refused(ckksmi.EINVAL, ctx.rotate_hoisted, a, [], out, L, 1, ws)
    refused(ckksmi.EINVAL, ctx.rotate_hoisted, a, list(range(1, 66)), out, L, 1, ws)
    refused(ckksmi.ENOKEY, ctx.rotate_hoisted, a, [1], out, L, 1, ws)
    ctx.galois_key_register(1, be.empty(ctx.beta_top, 2, L + shape[3], N))
    refused(ckksmi.EWORKSPACE, ctx.rotate_hoisted, a, [1], out, L, 1, tiny_ws)
    refused(ckksmi.EINVAL, ctx.rotate_hoisted, a, [1], a, L, 1, ws)  # out must not alias the input
    refused(ckksmi.EINVAL, ctx.sample_device, 2, 3.2, 1, 0, 1, out)
    refused(ckksmi.EINVAL, ctx.sample_device, 1, 0.0, 1, 0, 1, out)
    refused(ckksmi.EINVAL, ctx.sample_device, 1, 100.0, 1, 0, 1, out)
    refused(ckksmi.EINVAL, ctx.encode_device, a, None, -1.0, L, 1, out, ws)
    refused(ckksmi.EWORKSPACE, ctx.encode_device, a, None, 2.0**20, L, 1, out, tiny_ws)
    refused(ckksmi.EWORKSPACE, ctx.encrypt_device, a, a, a, a, a, L, 1, out, tiny_ws)
    refused(ckksmi.ELEVEL, ctx.encrypt_device, a, a, a, a, a, L + 1, 1, out, ws)
    ctx.close()
    # the merged division needs room for q_last beside the special primes: four special primes are too many
    ctx4 = be.context(6, 5, 30, 4, 31, 4)
    refused(ckksmi.EUNSUPPORTED, ctx4.hmul_relin_rescale_merged, a, a, a, out, 2, 1, ws)
    ctx4.close()
    # a value too large to encode is reported, not wrapped
    ctx = be.context(*shape)
    big = be.to_dev(np.full((1, N // 2), 1.0), np.float64)
    refused(ckksmi.EINVAL, ctx.encode_device, big, None, 2.0**70, L, 1, out, ws)
    ctx.close()


def edge_limbs(moduli, N, pattern):
    """[len(moduli)][N] residues at the ends and the middle of [0, q): the values where a lazy range, a canonical form or an
    integer <-> floating-point conversion would first go wrong"""
    out = np.zeros((len(moduli), N), dtype=np.uint64)
    for i, q in enumerate(moduli):
        q = int(q)
        if pattern == "zero":
            pass
        elif pattern == "qm1":
            out[i] = q - 1
        elif pattern == "half_lo":
            out[i] = (q - 1) // 2
        elif pattern == "half_hi":
            out[i] = (q + 1) // 2
        elif pattern == "alt":
            out[i, 1::2] = q - 1
        elif pattern == "alt_halves":
            out[i, 0::2] = (q - 1) // 2
            out[i, 1::2] = (q + 1) // 2
        elif pattern == "onehot":
            out[i, (7 * i + 3) % N] = q - 1
        elif pattern == "one":
            out[i] = 1
        else:
            raise ValueError(pattern)
    return out


EDGE_PATTERNS = ("zero", "qm1", "half_lo", "half_hi", "alt", "alt_halves", "onehot", "one")
# pairs of operands for the products: extreme times extreme, extreme times middle, sparse times dense
EDGE_PAIRS = (("qm1", "qm1"), ("zero", "qm1"), ("half_lo", "half_hi"), ("half_hi", "half_hi"), ("alt", "qm1"), ("onehot", "alt_halves"),
              ("alt_halves", "alt"), ("one", "qm1"))


def edge_ct(M, level, pattern, comps=2):
    return np.stack([edge_limbs(M.O.q[:level], M.N, pattern) for _ in range(comps)])


def case_edge_values(be, shape, seed, level=None, rotation=5, extreme_key=True, seeded_key=True, conv=True, pairs=EDGE_PAIRS):
    """residues at the ends and the middle of [0, q) (all 0, all q-1, (q-1)/2, (q+1)/2, alternating, one-hot) through the
    transforms, the tensor, relinearisation, the composite product, rescale, the scalar rescale, rotation and the
    multiply-accumulate, with the seeded switching key and with a key whose every word is q-1: word for word against the
    oracle.  Uniform inputs almost never reach these values."""
    M = make_material(shape, seed, rotations=(rotation,) if shape[3] else ())
    O = M.O
    ctx = be.context(*shape)
    check_moduli(ctx, M)
    level = level or O.n_q
    N = O.N
    # transforms of every pattern, every modulus of the chain
    idx = list(range(O.n_q + O.k))
    x = np.stack([edge_limbs(O.moduli, N, pat) for pat in EDGE_PATTERNS])
    d = be.to_dev(x)
    ctx.ntt(d, idx, len(EDGE_PATTERNS), stream=be.stream)
    got = be.to_host(d).reshape(x.shape)
    for b, pat in enumerate(EDGE_PATTERNS):
        assert np.array_equal(got[b], O.ntt_limbs(x[b], idx)), "forward transform of pattern %s" % pat
    d = be.to_dev(x)
    ctx.intt(d, idx, len(EDGE_PATTERNS), stream=be.stream)
    got = be.to_host(d).reshape(x.shape)
    for b, pat in enumerate(EDGE_PATTERNS):
        assert np.array_equal(got[b], O.intt_limbs(x[b], idx)), "inverse transform of pattern %s" % pat
    EDGE_PAIRS = pairs
    batch = len(EDGE_PAIRS)
    a = np.stack([edge_ct(M, level, pa) for pa, _ in EDGE_PAIRS])
    b = np.stack([edge_ct(M, level, pb) for _, pb in EDGE_PAIRS])
    da, db = be.to_dev(a), be.to_dev(b)
    # tensor
    d3 = be.empty(batch, 3, level, N)
    ctx.hmul(da, db, d3, level, batch, stream=be.stream)
    hd = be.to_host(d3).reshape(batch, 3, level, N)
    for i in range(batch):
        assert np.array_equal(hd[i], O.tensor(a[i], b[i], level)), "tensor of %r" % (EDGE_PAIRS[i],)
    # rescale and the scalar rescale (scalars that reduce to q-1, to the middle, and far outside (-q/2, q/2))
    if level >= 2:
        ws = be.ws(ctx.workspace_bytes(ckksmi.OP_MUL_SCALAR_RESCALE, level, batch))
        out = be.empty(batch, 2, level - 1, N)
        ctx.rescale(da, out, level, batch, ws, stream=be.stream)
        got = be.to_host(out).reshape(batch, 2, level - 1, N)
        for i in range(batch):
            assert np.array_equal(got[i], O.rescale(a[i], level)), "rescale of %s" % EDGE_PAIRS[i][0]
        for cst in (-1, int(O.q[level - 1]) // 2, (1 << 62) - 1, -(1 << 62) + 1):
            ctx.mul_scalar_rescale(db, cst, out, level, batch, ws, stream=be.stream)
            got = be.to_host(out).reshape(batch, 2, level - 1, N)
            for i in range(batch):
                assert np.array_equal(got[i], O.rescale(O.mul_scalar(b[i], cst, level), level)), "scalar rescale of %s by %d" % (EDGE_PAIRS[i][1], cst)
    if O.k:
        keys = [("seeded", M.rlk, M.gk[rotation])] if seeded_key else []
        if extreme_key:
            kq = np.empty_like(M.rlk)
            for t, q in enumerate(O.moduli):
                kq[:, :, t, :] = np.uint64(int(q) - 1)
            keys.append(("all q-1", kq, kq))
        for name, rlk, gk in keys:
            evk = be.to_dev(rlk)
            # relinearisation of the tensors above, and the composite product
            r = be.empty(batch, 2, level, N)
            ctx.relin(d3, evk, r, level, batch, be.ws(ctx.workspace_bytes(ckksmi.OP_RELIN, level, batch)), stream=be.stream)
            got = be.to_host(r).reshape(batch, 2, level, N)
            for i in range(batch):
                assert np.array_equal(got[i], O.relin(hd[i], rlk, level)), "relin of %r, key %s" % (EDGE_PAIRS[i], name)
            if level >= 2:
                out = be.empty(batch, 2, level - 1, N)
                ctx.hmul_relin_rescale(da, db, evk, out, level, batch, be.ws(ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, level, batch)), stream=be.stream)
                got = be.to_host(out).reshape(batch, 2, level - 1, N)
                for i in range(batch):
                    assert np.array_equal(got[i], O.hmul_relin_rescale(a[i], b[i], rlk, level)), "product of %r, key %s" % (EDGE_PAIRS[i], name)
            # rotation
            dgk = be.to_dev(gk)
            ctx.galois_key_register(rotation, dgk)
            outr = be.empty(batch, 2, level, N)
            ctx.rotate(da, [rotation] * batch, outr, level, batch, be.ws(ctx.workspace_bytes(ckksmi.OP_ROTATE, level, batch)), stream=be.stream)
            got = be.to_host(outr).reshape(batch, 2, level, N)
            for i in range(batch):
                assert np.array_equal(got[i], O.rotate(a[i], rotation, gk, level)), "rotation of %s, key %s" % (EDGE_PAIRS[i][0], name)
    if conv:
        # multiply-accumulate: every input word q-1 (and the other patterns), weights at the ends of int64's usable range
        Cin, H, W, Oc, kh = 2, 3, 4, 9, 3
        pats = [EDGE_PATTERNS[(c * H * W + y * W + xx) % len(EDGE_PATTERNS)] if (c + y + xx) % 3 else "qm1" for c in range(Cin) for y in range(H) for xx in range(W)]
        xin = np.stack([edge_ct(M, level, pat) for pat in pats]).reshape(Cin, H, W, 2, level, N)
        wi = np.rint(wl.weights_float((Oc, Cin, kh, kh), seed, "edge.w") * float(O.q[level - 1])).astype(np.int64)
        wi.flat[0], wi.flat[1], wi.flat[2], wi.flat[3] = (1 << 62) - 1, -(1 << 62) + 1, -1, int(O.q[level - 1]) - 1
        want = O.conv2d_mac(xin, wi, 1, 1, level)
        for nbytes in (ctx.workspace_bytes(ckksmi.OP_CONV2D_MAC, level, wi.size), ctx.conv2d_workspace_bytes(Cin, Oc, kh, kh, level)):
            outc = be.empty(Oc, H, W, 2, level, N)
            ctx.conv2d_mac(be.to_dev(xin), be.to_dev(wi, np.int64), Cin, H, W, Oc, kh, kh, 1, 1, outc, level, be.ws(nbytes), stream=be.stream)
            assert np.array_equal(be.to_host(outc).reshape(want.shape), want), "multiply-accumulate on edge values"
    ctx.close()


def own_poly3_constants(q, level_y, s_y):
    """the three integer constants of 0.5 + 0.25 y - 0.02 y^3 for y at level_y, scale s_y, written out from the schedule:
    t = RS(y * c1) must keep y's scale, so c1 = round(-0.02 * q_dropped); u = RS(y * c2) must reach the scale of y^3
    (s_2 * s_y / q_dropped'), so c2 = round(0.25 * s_2); the constant term enters at the output scale"""
    q_a, q_b = float(q[level_y - 1]), float(q[level_y - 2])
    s_2 = s_y * s_y / q_a
    s_3 = s_2 * s_y / q_b
    return int(round(-0.02 * q_a)), int(round(0.25 * s_2)), int(round(0.5 * s_3)), s_3


def case_activation(be, shape, seed, level, batch, sample, log_scale=50, decrypt=True, workers=1, expect_kernels=()):
    """x^2, then 0.5 + 0.25 y - 0.02 y^3 (three products and two scalar steps, one level each) through the library's call
    sequence, against the oracle's composition: y and the result word for word for the items in `sample`; those items are
    real encryptions and decrypt to the float polynomial, the rest are uniform residues"""
    from concurrent.futures import ThreadPoolExecutor
    from paper_1911_11377_amd import activation

    M = make_material(shape, seed)
    O = M.O
    ctx = be.context(*shape)
    check_moduli(ctx, M)
    N, s = O.N, 2.0 ** log_scale
    x = random_cts(M, level, batch, seed, "act.x")
    zs = {}
    for i in sample:
        zs[i] = wl.slots_real(N // 2, seed, "act.z", i)
        if decrypt:
            x[i] = M.encrypt(zs[i], s, level, ("act", i))
    s_y = s * s / float(O.q[level - 1])
    c1, c2, c3, s_out = own_poly3_constants(O.q, level - 1, s_y)
    consts = activation.poly3_constants(O.q, level - 1, s_y)
    assert (consts.c_m002, consts.c_025, consts.c_05) == (c1, c2, c3), "the call sequence's constants differ from the schedule's"
    assert consts.out_scale == s_out
    dx, evk = be.to_dev(x), be.to_dev(M.rlk)
    y = be.empty(batch, 2, level - 1, N)
    out = be.empty(batch, 2, level - 3, N)
    ws = be.ws(activation.workspace_bytes(ctx, level, batch))
    if expect_kernels:
        ctx.profile_enable(True)
    activation.square(ctx, dx, evk, y, level, batch, ws, stream=be.stream)
    activation.poly3(ctx, y, evk, out, level - 1, batch, consts, ws, stream=be.stream)
    gy = be.to_host(y).reshape(batch, 2, level - 1, N)
    go = be.to_host(out).reshape(batch, 2, level - 3, N)
    if expect_kernels:
        ran = ctx.profile_read()
        ctx.profile_enable(False)
        for k in expect_kernels:
            assert k in ran, (k, sorted(ran))

    def oracle_item(i):
        oy = O.square(x[i], M.rlk, level)
        return oy, O.poly3(oy, M.rlk, level - 1, c1, c2, c3)

    with ThreadPoolExecutor(max(1, min(workers, len(sample)))) as ex:  # the oracle's C calls release the GIL
        wants = list(ex.map(oracle_item, sample))
    for i, (oy, oo) in zip(sample, wants):
        assert np.array_equal(gy[i], oy), "x^2 of item %d differs from the oracle" % i
        assert np.array_equal(go[i], oo), "activation of item %d differs from the oracle" % i
        if decrypt:
            yv = zs[i].real ** 2
            dec = M.decrypt(go[i], s_out, level - 3)
            assert np.max(np.abs(dec.real - (0.5 + 0.25 * yv - 0.02 * yv ** 3))) < 1e-3
    assert np.array_equal(be.to_host(dx).reshape(x.shape), x), "the schedule modified its input"
    ctx.close()


def mfma_kernel_name(Cin, kh, kw, stride):
    """which matrix-core kernel a layer runs on.  At most 128 taps and a window block (2 x 2 or 1 x 4 positions) of at most
    192 lines: four positions share a staged strip; at most 256 taps: weight digits resident in LDS; otherwise they stream"""
    taps = Cin * kh * kw
    if taps <= 128 and min(Cin * (kh + stride) * (kw + stride), Cin * kh * (kw + 3 * stride)) <= 192:
        return "conv_mac_mfma_strip_kernel"
    return "conv_mac_mfma_resident_kernel" if taps <= 256 else "conv_mac_mfma_kernel"


def case_conv(be, shape, seed, Cin, H, W, Oc, kh, stride, pad, level=None, rows_check=True, fc_check=True):
    M = make_material(shape, seed)
    O = M.O
    ctx = be.context(*shape)
    level = level or O.n_q
    x = wl.uniform_limbs(O.q[:level], O.N, seed, "x", lead=(Cin, H, W, 2))
    wf = wl.weights_float((Oc, Cin, kh, kh), seed)
    wi = np.rint(wf * O.q[level - 1]).astype(np.int64)
    wi.flat[0] = -(1 << 62) + 7  # a weight far outside (-q/2, q/2)
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kh) // stride + 1
    dx, dw = be.to_dev(x), be.to_dev(wi, np.int64)
    want = O.conv2d_mac(x, wi, stride, pad, level)
    # both multiply-accumulate kernels: the small workspace only fits the vector one, the layer's own query admits
    # the matrix-core one where the shape allows it
    mfma_shape = O.N >= 64 and Oc >= 8
    for which, nbytes in (("vector", ctx.workspace_bytes(ckksmi.OP_CONV2D_MAC, level, wi.size)),
                          ("auto", ctx.conv2d_workspace_bytes(Cin, Oc, kh, kh, level))):
        out = be.empty(Oc, Ho, Wo, 2, level, O.N)
        ws = be.ws(nbytes)
        ctx.profile_enable(True)
        ctx.conv2d_mac(dx, dw, Cin, H, W, Oc, kh, kh, stride, pad, out, level, ws, stream=be.stream)
        got = be.to_host(out).reshape(Oc, Ho, Wo, 2, level, O.N)
        ran = ctx.profile_read()
        ctx.profile_enable(False)
        mfma_name = mfma_kernel_name(Cin, kh, kh, stride)
        assert (mfma_name in ran) == (which == "auto" and mfma_shape), (which, list(ran))
        assert np.array_equal(got, want), "conv MAC (%s) differs from the oracle" % which
    # the same layer in strips of output rows, each strip handed only the input rows its windows touch
    ws = be.ws(ctx.conv2d_workspace_bytes(Cin, Oc, kh, kh, level))
    cut = max(1, Ho // 2)
    for r0, r1 in ((0, cut), (cut, Ho)):
        if r0 >= r1 or not rows_check:
            continue
        i0 = max(0, r0 * stride - pad)
        i1 = min(H, (r1 - 1) * stride - pad + kh)
        strip = be.to_dev(np.ascontiguousarray(x[:, i0:i1]))
        outs = be.empty(Oc, r1 - r0, Wo, 2, level, O.N)
        ctx.conv2d_mac_rows(strip, dw, Cin, H, W, Oc, kh, kh, stride, pad, i0, i1 - i0, r0, r1 - r0, outs, level, ws, stream=be.stream)
        got = be.to_host(outs).reshape(Oc, r1 - r0, Wo, 2, level, O.N)
        assert np.array_equal(got, want[:, r0:r1]), "conv MAC in strips of rows differs from the oracle (rows %d..%d)" % (r0, r1)
    if not fc_check:
        ctx.close()
        return
    # FC: flat features
    F = Cin * H
    xf = x[:, :, 0].reshape(F, 2, level, O.N)
    wfc = np.rint(wl.weights_float((Oc, F), seed, "fc") * O.q[level - 1]).astype(np.int64)
    dxf, dwf = be.to_dev(xf), be.to_dev(wfc, np.int64)
    outf = be.empty(Oc, 2, level, O.N)
    wsf = be.ws(ctx.conv2d_workspace_bytes(F, Oc, 1, 1, level))
    ctx.fc_mac(dxf, dwf, F, Oc, outf, level, wsf, stream=be.stream)
    assert np.array_equal(be.to_host(outf).reshape(Oc, 2, level, O.N), O.fc_mac(xf, wfc, level)), "FC MAC differs"
    ctx.close()


def case_cnn(be, shape, seed, topology, workers=1):
    """conv - square - conv - square - conv - pool - fc - square - fc on per-pixel ciphertexts, every activation
    resident, against the oracle's layer-by-layer network; plus the first conv layer again in strips of rows"""
    from paper_1911_11377_amd import cnn

    M = make_material(shape, seed)
    O = M.O
    ctx = be.context(*shape)
    check_moduli(ctx, M)
    level = O.n_q
    Cc, H, W = wl.CNN_TOPOLOGIES[topology]["input"]
    x = wl.uniform_limbs(O.q[:level], O.N, seed, "cnn.x", lead=(Cc, H, W, 2))
    shapes = wl.cnn_shapes(topology)
    wf = wl.cnn_weights_float(topology, seed)
    # the test's own integer weights for the oracle: round(w * q_dropped), the pooling's 1/k^2 folded forward
    layers_i, lvl, fold, sc = [], level, 1.0, 2.0**50
    for (layer, _, _), wt in zip(shapes, wf):
        if layer[0] in ("conv", "fc"):
            wi = np.rint(wt * fold * float(O.q[lvl - 1])).astype(np.int64)
            fold = 1.0
            layers_i.append(("conv", wi, layer[3], layer[4]) if layer[0] == "conv" else ("fc", wi))
            lvl -= 1
        elif layer[0] == "square":
            layers_i.append(layer)
            sc = sc * sc / O.q[lvl - 1]
            lvl -= 1
        elif layer[0] == "poly2":
            c2, c1 = 0.000469841857369822, 0.500000000000008  # section 3.1
            s2 = sc * sc / O.q[lvl - 1]
            layers_i.append(("poly2", round(c2 * O.q[lvl - 2]), round(c1 * (s2 / sc) * O.q[lvl - 2])))
            sc = s2
            lvl -= 2
        else:
            layers_i.append(layer)
            fold = 1.0 / (layer[1] * layer[1])
    plans, out_level, _ = cnn.plan(shapes, wf, O.q, level, 2.0**50)
    assert out_level == lvl
    for p, li in zip(plans, layers_i):
        if p.w_int is not None:
            assert np.array_equal(p.w_int, li[1]), "integer weights differ"
        if p.kind == "poly2":
            assert (p.consts.k2, p.consts.k1) == (li[1], li[2]), "activation constants differ"
    want, want_level = O.cnn_forward(x, layers_i, M.rlk, level, workers=workers)
    assert want_level == out_level
    print("[parity] oracle network done, running the library", flush=True)
    ws = be.ws(cnn.workspace_bytes(ctx, plans, max_items=16))
    evk = be.to_dev(M.rlk)
    dx = be.to_dev(x)
    out = cnn.forward(ctx, dx, plans, evk, be.empty, lambda a: be.to_dev(a, np.int64), ws, stream=be.stream, max_items=16)
    got = be.to_host(out).reshape(want.shape)
    assert np.array_equal(got, want), "network output differs from the oracle"

    # first layer in strips: every output row from only the input rows it needs
    p = plans[0]
    assert p.kind == "conv"
    O1, Ho, Wo = p.out_shape
    ref = O.rescale_each(O.conv2d_mac_each(x, layers_i[0][1], p.stride, p.pad, level, workers), level, workers)
    wdev = be.to_dev(p.w_int, np.int64)
    rows_per = 2
    for r0 in range(0, Ho, rows_per):
        rows = min(rows_per, Ho - r0)
        i0 = max(0, r0 * p.stride - p.pad)
        i1 = min(H - 1, (r0 + rows - 1) * p.stride - p.pad + p.kernel - 1)
        strip = be.to_dev(np.ascontiguousarray(x[:, i0:i1 + 1]))
        mac = be.empty(O1, rows, Wo, 2, level, O.N)
        y = be.empty(O1, rows, Wo, 2, level - 1, O.N)
        cnn.conv_rows(ctx, p, strip, wdev, i0, i1 - i0 + 1, r0, rows, mac, y, ws, stream=be.stream)
        assert np.array_equal(be.to_host(y).reshape(O1, rows, Wo, 2, level - 1, O.N), ref[:, r0:r0 + rows]), "strip rows differ"
    # a strip that lacks a needed input row is refused before anything is enqueued
    if Ho >= 2:
        try:
            ctx.conv2d_mac_rows(strip, wdev, Cc, H, W, O1, p.kernel, p.kernel, p.stride, p.pad, 0, 1, 0, 2, mac, level, ws, stream=be.stream)
            raise AssertionError("incomplete strip accepted")
        except ckksmi.CkksmiError as e:
            assert e.code == ckksmi.EINVAL
    ctx.close()


def case_pool(be, shape, seed, Cin, H, W, k, level=None, pad=0):
    M = make_material(shape, seed)
    O = M.O
    ctx = be.context(*shape)
    level = level or O.n_q
    x = wl.uniform_limbs(O.q[:level], O.N, seed, "pool.x", lead=(Cin, H, W, 2))
    Ho, Wo = (H + 2 * pad) // k, (W + 2 * pad) // k
    out = be.empty(Cin, Ho, Wo, 2, level, O.N)
    ctx.sum_pool2d(be.to_dev(x), Cin, H, W, k, out, level, stream=be.stream, pad=pad)
    assert np.array_equal(be.to_host(out).reshape(Cin, Ho, Wo, 2, level, O.N), O.sum_pool2d(x, k, level, pad)), "pooling differs"
    try:
        ctx.sum_pool2d(be.to_dev(x), Cin, H, W, k, out, level, stream=be.stream, pad=k)
        raise AssertionError("padding as wide as the window accepted")
    except ckksmi.CkksmiError as e:
        assert e.code == ckksmi.EINVAL
    ctx.close()

