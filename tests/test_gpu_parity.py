"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs.  Ciphertext words must match bit for bit; decrypted slot values
must match the cleartext computation within 1e-3 at scale 2^40 (1e-2 for the tiny
shape, whose output scale is only about 2^20)."""
import numpy as np
import pytest

import parity_cases as pc
from oracle import oracle as orc
from paper_1911_11377_amd import ckksmi
from paper_1911_11377_amd import workloads as wl

pytestmark = pytest.mark.gpu

TINY = (12, 3, 40, 1, 41, 1)            # N=2^12, 3x40-bit + one 41-bit special prime
C2 = (14, 8, 50, 1, 51, 1)              # N=2^14, 8x50-bit + one special prime
C3 = (15, 16, 50, 0, 51, 1)             # N=2^15, 16x50-bit, no key switching
C4 = (16, 24, 50, 3, 51, 3)             # N=2^16, 24x50-bit + 3 special primes, 8 digits


@pytest.fixture(scope="module")
def be():
    return pc.GpuBackend()


def announce(msg):
    print("[case] " + msg, flush=True)


@pytest.mark.parametrize("shape", [(4, 2, 20, 1, 21, 1), (9, 2, 50, 1, 51, 1), TINY, (13, 2, 50, 1, 51, 1), (14, 2, 50, 1, 51, 1),
                                   (15, 2, 50, 1, 51, 1), (16, 2, 50, 2, 51, 2), (17, 1, 50, 1, 51, 1)])
def test_ntt_matches_oracle(be, shape):
    announce("ntt %r" % (shape,))
    pc.case_ntt(be, shape, seed=300, batch=3)


@pytest.mark.parametrize("shape", [TINY, (14, 3, 50, 1, 51, 1), (5, 7, 50, 3, 51, 3)])
def test_elementwise_matches_oracle(be, shape):
    announce("elementwise %r" % (shape,))
    pc.case_elementwise(be, shape, seed=301, batch=3)


@pytest.mark.parametrize("shape,levels", [(TINY, [3, 2]), ((14, 4, 50, 1, 51, 1), [4]), ((8, 5, 40, 2, 41, 2), [5, 3])])
def test_rescale_matches_oracle(be, shape, levels):
    announce("rescale %r" % (shape,))
    pc.case_rescale(be, shape, seed=302, batch=3, levels=levels)


def test_tiny_shape_full_batch(be):
    """the tiny workload: 16 ciphertext pairs, HMult + relin + rescale, every word compared"""
    announce("tiny shape, batch 16")
    pc.case_relin_and_composite(be, TINY, seed=1, batch=16, levels=[3])


@pytest.mark.parametrize("shape,levels,batch", [
    (TINY, [2, 1], 2),
    ((10, 5, 40, 2, 41, 2), [5, 4, 3, 1], 3),
    ((9, 7, 50, 3, 51, 3), [7, 6, 5, 2], 2),
    ((13, 3, 50, 1, 51, 1), [3], 2),
    ((15, 3, 50, 3, 51, 3), [3, 2], 1),
    ((13, 7, 50, 3, 51, 3), [7, 6, 5, 3], 2),   # register-tiled size, last digit of 1, 3 and 2 limbs
    ((14, 5, 51, 2, 51, 2), [5, 4, 2], 2),      # 51-bit primes throughout: the tighter reduction schedule everywhere
])
def test_relin_and_composite_levels_and_digits(be, shape, levels, batch):
    announce("relin/composite %r levels %r" % (shape, levels))
    pc.case_relin_and_composite(be, shape, seed=303, batch=batch, levels=levels)


def test_largest_ring_uses_generic_kernels(be):
    announce("N=2^17 generic path")
    pc.case_relin_and_composite(be, (17, 2, 50, 1, 51, 1), seed=313, batch=1, levels=[2])


def test_ragged_sweeps_with_small_workspace(be):
    announce("relin with a workspace that holds one item")
    pc.case_relin_and_composite(be, (10, 5, 40, 2, 41, 2), seed=304, batch=5, levels=[5], small_ws=True)


def test_rotate_matches_oracle(be):
    announce("rotate tiny + hybrid")
    pc.case_rotate(be, TINY, seed=305, rotations=[1, 2, 100, 2047], batch=6)
    pc.case_rotate(be, (9, 7, 50, 3, 51, 3), seed=306, rotations=[1, 3, 255], batch=4, level=5)


def test_conv_and_fc_match_oracle(be):
    announce("conv small")
    pc.case_conv(be, (10, 3, 40, 0, 41, 1), seed=307, Cin=3, H=7, W=7, Oc=10, kh=5, stride=2, pad=0)
    pc.case_conv(be, (8, 2, 50, 1, 51, 1), seed=308, Cin=2, H=4, W=5, Oc=3, kh=3, stride=1, pad=1)


def test_conv_matrix_cores_shapes(be):
    """multi-step / multi-group shapes of the matrix-core multiply-accumulate, with zero padding and a ragged channel group"""
    announce("conv matrix cores 51-bit")
    pc.case_conv(be, (7, 2, 51, 0, 52, 1), seed=312, Cin=3, H=4, W=3, Oc=34, kh=5, stride=1, pad=2)
    announce("conv matrix cores N=2^13")
    pc.case_conv(be, (13, 3, 50, 0, 51, 1), seed=313, Cin=8, H=3, W=4, Oc=40, kh=3, stride=1, pad=1)
    announce("conv matrix cores, 100 taps and 27 taps")
    pc.case_conv(be, (8, 2, 50, 0, 51, 1), seed=314, Cin=4, H=6, W=5, Oc=17, kh=5, stride=1, pad=0)
    pc.case_conv(be, (8, 2, 50, 0, 51, 1), seed=315, Cin=3, H=4, W=4, Oc=9, kh=3, stride=1, pad=1)
    announce("conv matrix cores, stride 2 with padding, odd output size, strips of rows that end inside a 2 x 2 block")
    pc.case_conv(be, (7, 2, 50, 0, 51, 1), seed=320, Cin=3, H=9, W=9, Oc=16, kh=3, stride=2, pad=1)
    announce("conv matrix cores, workgroups that walk several tiles / positions")
    with be.tuned(2):
        pc.case_conv(be, (7, 2, 50, 0, 51, 1), seed=316, Cin=3, H=9, W=8, Oc=33, kh=5, stride=1, pad=1)    # 2 x 2 blocks, 35 positions
        pc.case_conv(be, (7, 2, 50, 0, 51, 1), seed=317, Cin=2, H=3, W=13, Oc=8, kh=3, stride=1, pad=0)    # 1 x 4 blocks, three tiles
        pc.case_conv(be, (7, 2, 50, 0, 51, 1), seed=318, Cin=7, H=4, W=16, Oc=9, kh=3, stride=3, pad=1)    # weight digits resident, six positions
        pc.case_conv(be, (7, 2, 50, 0, 51, 1), seed=319, Cin=29, H=3, W=3, Oc=8, kh=3, stride=1, pad=1)    # 261 taps: streaming kernel


def test_conv_at_layer_shape_slice(be):
    """N=2^15, 16x50-bit limbs, 3 input channels, 5x5 stride 2: one output position, three filters"""
    announce("conv N=2^15 level 16 slice")
    pc.case_conv(be, C3, seed=309, Cin=3, H=5, W=5, Oc=3, kh=5, stride=2, pad=0)


def test_pool_and_network_match_oracle(be):
    """the AlexNet-like layer sequence at reduced width, N=2^13 (fused key-switching kernels), 10 levels deep"""
    announce("pool")
    pc.case_pool(be, (10, 3, 40, 0, 41, 1), seed=310, Cin=3, H=6, W=7, k=2)
    pc.case_pool(be, (10, 3, 40, 0, 41, 1), seed=314, Cin=2, H=3, W=3, k=2, pad=1)
    announce("network cnn_reduced N=2^13")
    pc.case_cnn(be, (13, 10, 50, 3, 51, 3), seed=311, topology="cnn_reduced", workers=16)


def test_table1_like_network_matches_oracle(be):
    """the layer sequence of the paper's Table 1 at reduced width with its degree-2 activation, N=2^13, 19 levels deep"""
    announce("network table1_reduced N=2^13")
    pc.case_cnn(be, (13, 20, 50, 3, 51, 3), seed=315, topology="table1_reduced", workers=16)


def _encrypt_batch(M, zs, scale, level, tag):
    return np.stack([M.encrypt(z, scale, level, (tag, i)) for i, z in enumerate(zs)])


def test_tiny_shape_decrypts_to_product(be):
    announce("tiny: decrypt(HMult) vs float product")
    p = wl.PRESETS["tiny"]
    M = pc.make_material(TINY, 1)
    ctx = be.context(*TINY)
    scale = 2.0**p.log_scale
    za = [wl.slots_complex(M.N // 2, 1, "a", i) for i in range(4)]
    zb = [wl.slots_complex(M.N // 2, 1, "b", i) for i in range(4)]
    a, b = _encrypt_batch(M, za, scale, 3, "a"), _encrypt_batch(M, zb, scale, 3, "b")
    out = be.empty(4, 2, 2, M.N)
    ws = be.ws(ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, 3, 4))
    ctx.hmul_relin_rescale(be.to_dev(a), be.to_dev(b), be.to_dev(M.rlk), out, 3, 4, ws)
    got = be.to_host(out).reshape(4, 2, 2, M.N)
    for i in range(4):
        assert np.array_equal(got[i], M.O.hmul_relin_rescale(a[i], b[i], M.rlk, 3))
        dec = ctx.decode(ctx.decrypt(M.s, got[i], 2), 2, scale * scale / M.O.q[2])
        assert np.max(np.abs(dec - za[i] * zb[i])) < 1e-2


def test_2e14_shape_hmul_and_rotations(be):
    """N=2^14, 8x50-bit + special, scale 2^40: the launch shape of the full batch of 256,
    outputs sampled for the oracle; decrypted values within 1e-3"""
    announce("N=2^14 batch 256, sampled parity")
    p = wl.PRESETS["hmul_rot_2e14"]
    rots = wl.rotation_offsets(p.N // 2, 8, 2)
    M = pc.make_material(C2, 2, rotations=rots)
    ctx = be.context(*C2)
    scale = 2.0**p.log_scale
    batch, level = p.batch, p.n_q
    # real encryptions for the sampled items, uniform residues (pseudorandom, like any RLWE ciphertext) elsewhere
    a = pc.random_cts(M, level, batch, 2, "a")
    b = pc.random_cts(M, level, batch, 2, "b")
    sample = [0, 101, batch - 1]
    zs = {}
    for i in sample:
        zs[i] = (wl.slots_real(M.N // 2, 2, "a", i), wl.slots_real(M.N // 2, 2, "b", i))
        a[i] = M.encrypt(zs[i][0], scale, level, ("a", i))
        b[i] = M.encrypt(zs[i][1], scale, level, ("b", i))
    da, db = be.to_dev(a), be.to_dev(b)
    out = be.empty(batch, 2, level - 1, M.N)
    ws = be.ws(ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, level, batch))
    ctx.hmul_relin_rescale(da, db, be.to_dev(M.rlk), out, level, batch, ws)
    got = be.to_host(out).reshape(batch, 2, level - 1, M.N)
    for i in sample:
        assert np.array_equal(got[i], M.O.hmul_relin_rescale(a[i], b[i], M.rlk, level)), "item %d" % i
        dec = ctx.decode(ctx.decrypt(M.s, got[i], level - 1), level - 1, scale * scale / M.O.q[level - 1])
        assert np.max(np.abs(dec - zs[i][0] * zs[i][1])) < 1e-3
    # deterministic: a second run gives the same bits everywhere
    out2 = be.empty(batch, 2, level - 1, M.N)
    ctx.hmul_relin_rescale(da, db, be.to_dev(M.rlk), out2, level, batch, ws)
    assert np.array_equal(be.to_host(out2).reshape(got.shape), got)
    # rotations: every ciphertext by one of the 8 offsets
    announce("N=2^14 rotations")
    for r in rots:
        ctx.galois_key_register(r, be.to_dev(M.gk[r]))
    pick = wl.rng(2, "rot.pick").integers(0, len(rots), size=batch)
    rot = [rots[j] for j in pick]
    outr = be.empty(batch, 2, level, M.N)
    wsr = be.ws(ctx.workspace_bytes(ckksmi.OP_ROTATE, level, batch))
    ctx.rotate(da, rot, outr, level, batch, wsr)
    gotr = be.to_host(outr).reshape(batch, 2, level, M.N)
    for i in sample:
        assert np.array_equal(gotr[i], M.O.rotate(a[i], rot[i], M.gk[rot[i]], level)), "rotation of item %d" % i
        dec = ctx.decode(ctx.decrypt(M.s, gotr[i], level), level, scale)
        assert np.max(np.abs(dec - np.roll(zs[i][0], -rot[i]))) < 1e-3


def test_2e16_hybrid_shape_sampled(be):
    """N=2^16, 24x50-bit + 3 special primes (8 digits of 3): batch 64 in the benchmark's launch
    configuration; the first, a middle and the last item compared word for word with the oracle at
    levels 24, 23 and 22 (the levels the activation schedule multiplies at)"""
    from concurrent.futures import ThreadPoolExecutor
    announce("N=2^16 hybrid batch 64, sampled parity")
    p = wl.PRESETS["act_2e16"]
    M = pc.make_material(C4, 4)
    ctx = be.context(*C4)
    batch = p.batch
    evk = be.to_dev(M.rlk)
    for level, picks in ((24, (0, 17, 63)), (23, (0, 31, 63)), (22, (0, 40, 63))):
        a = pc.random_cts(M, level, batch, 4, ("a", level))
        b = pc.random_cts(M, level, batch, 4, ("b", level))
        out = be.empty(batch, 2, level - 1, M.N)
        ws = be.ws(ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, level, batch))
        ctx.profile_enable(True)
        ctx.hmul_relin_rescale(be.to_dev(a), be.to_dev(b), evk, out, level, batch, ws)
        got = be.to_host(out).reshape(batch, 2, level - 1, M.N)
        ran = ctx.profile_read()
        ctx.profile_enable(False)
        # the launch configuration bench.py times: ModDown and rescale as one conversion
        assert "modup_cols_kernel<4, 4, 3>" in ran and "tensor_rows_kernel" in ran, list(ran)
        announce("oracle for items %r at level %d" % (picks, level))
        with ThreadPoolExecutor(len(picks)) as ex:  # the oracle's C calls release the GIL
            wants = list(ex.map(lambda i: M.O.hmul_relin_rescale(a[i], b[i], M.rlk, level), picks))
        for i, want in zip(picks, wants):
            assert np.array_equal(got[i], want), "item %d at level %d" % (i, level)
        del ws, out


def test_2e16_rotation_sampled(be):
    """ckksmi_rotate at N=2^16, 24 primes, 3-prime digits, batch 64 over two Galois keys: three items word for word"""
    from concurrent.futures import ThreadPoolExecutor
    announce("N=2^16 rotations batch 64, sampled parity")
    rots = (1, 12345)
    M = pc.make_material(C4, 6, rotations=rots)
    ctx = be.context(*C4)
    level, batch = 24, 64
    keys = [be.to_dev(M.gk[r]) for r in rots]
    for r, k in zip(rots, keys):
        ctx.galois_key_register(r, k)
    a = pc.random_cts(M, level, batch, 6, "rot16")
    rot = [rots[(i * 7 // 3) % 2] for i in range(batch)]
    out = be.empty(batch, 2, level, M.N)
    ws = be.ws(ctx.workspace_bytes(ckksmi.OP_ROTATE, level, batch))
    ctx.rotate(be.to_dev(a), rot, out, level, batch, ws)
    got = be.to_host(out).reshape(batch, 2, level, M.N)
    picks = (0, 29, 63)
    assert len({rot[i] for i in picks}) == 2
    announce("oracle for items %r" % (picks,))
    with ThreadPoolExecutor(len(picks)) as ex:
        wants = list(ex.map(lambda i: M.O.rotate(a[i], rot[i], M.gk[rot[i]], level), picks))
    for i, want in zip(picks, wants):
        assert np.array_equal(got[i], want), "rotation of item %d by %d" % (i, rot[i])
    ctx.close()


@pytest.mark.parametrize("seed", [9000, 9001, 9002])
def test_more_seeds_through_the_register_tiled_kernels(be, seed):
    """other random draws (operands, keys, weights) through every fused sequence, word for word"""
    announce("seed %d" % seed)
    pc.case_relin_and_composite(be, (13, 4, 50, 2, 51, 2), seed=seed, batch=3, levels=[4, 3])
    pc.case_relin_and_composite(be, (12, 3, 50, 1, 51, 1), seed=seed, batch=2, levels=[3])
    pc.case_relin_and_composite(be, (14, 5, 40, 3, 41, 3), seed=seed, batch=2, levels=[5, 2])
    pc.case_merged_product(be, (13, 4, 50, 2, 51, 2), seed=seed, batch=2, levels=[4, 2])
    pc.case_rotate(be, (13, 4, 50, 2, 51, 2), seed=seed, rotations=[1, 5, 100], batch=3, level=4)
    pc.case_rotate_hoisted(be, (13, 4, 50, 2, 51, 2), seed=seed, rotations=[1, 2, 9], batch=2, level=3)
    pc.case_sum_of_products(be, (13, 4, 50, 2, 51, 2), seed=seed, terms=3, batch=2, levels=[4])
    pc.case_rescale(be, (15, 3, 50, 0, 51, 1), seed=seed, batch=2, levels=[3, 2])
    pc.case_conv(be, (8, 2, 51, 0, 52, 1), seed=seed, Cin=3, H=7, W=7, Oc=34, kh=5, stride=1, pad=2, rows_check=False)
    pc.case_ntt(be, (16, 2, 50, 1, 51, 1), seed=seed, batch=2)


def test_item_loops_on_gpu(be):
    """few workgroups per launch, so that every register-tiled kernel loops over several items"""
    announce("item loops")
    with be.tuned(64):
        pc.case_relin_and_composite(be, (16, 4, 50, 3, 51, 3), seed=310, batch=3, levels=[4, 2])
        pc.case_relin_and_composite(be, (14, 3, 50, 2, 51, 2), seed=311, batch=5, levels=[3])
        pc.case_rotate(be, (13, 3, 50, 1, 51, 1), seed=312, rotations=[5, 9], batch=3)
        pc.case_ntt(be, (15, 2, 50, 1, 51, 1), seed=313, batch=7)


FEW_PAIRS = (("qm1", "qm1"), ("half_lo", "half_hi"), ("alt", "qm1"), ("onehot", "alt_halves"))


@pytest.mark.parametrize("shape,level,kw", [
    ((5, 5, 40, 2, 41, 2), 5, {}),
    ((9, 9, 51, 2, 51, 2), 9, {}),
    ((12, 6, 51, 2, 51, 2), 6, {"conv": False, "pairs": FEW_PAIRS}),      # smallest register-tiled size (16-point columns)
    ((13, 24, 50, 3, 51, 3), 24, {"conv": False}),                        # 8 digits of 50-bit primes: eight terms per reduction
    ((14, 15, 51, 3, 51, 3), 15, {"conv": False, "pairs": FEW_PAIRS}),    # 51-bit primes: reduced every four terms
    ((15, 4, 50, 1, 51, 1), 4, {"pairs": FEW_PAIRS}),
    ((16, 24, 50, 3, 51, 3), 24, {"conv": False, "pairs": FEW_PAIRS[:3], "seeded_key": False}),  # the benchmark's shape, all-(q-1) key
    ((13, 2, 51, 0, 52, 1), 2, {}),                                       # matrix-core multiply-accumulate, 51-bit prime
])
def test_edge_values_match_oracle(be, shape, level, kw):
    """residues at the ends and the middle of [0, q) (all 0, all q-1, (q-1)/2, (q+1)/2, alternating, one-hot), scalars and
    weights at the ends of their ranges, and a switching key of all q-1, through the transforms, tensor, relinearisation,
    the composite product, rescale, scalar rescale, rotation and the multiply-accumulate: every word against the oracle"""
    announce("edge values %r" % (shape,))
    pc.case_edge_values(be, shape, seed=370, level=level, **kw)


@pytest.mark.parametrize("shape,levels,batch", [
    (TINY, [3, 2], 2),
    ((10, 5, 40, 2, 41, 2), [5, 4, 2], 3),
    ((9, 7, 50, 3, 51, 3), [7, 5, 2], 2),
    ((13, 3, 50, 1, 51, 1), [3], 2),
    ((14, 3, 50, 2, 51, 2), [3, 2], 3),
    ((15, 3, 50, 3, 51, 3), [3, 2], 1),
    ((16, 4, 50, 3, 51, 3), [4, 2], 3),
    ((13, 7, 50, 3, 51, 3), [7, 6, 5, 3], 2),
])
def test_merged_product_matches_oracle(be, shape, levels, batch):
    """the product with one division by P*q_last (exact DivRound): every word against the oracle's definition"""
    announce("merged product %r levels %r" % (shape, levels))
    pc.case_merged_product(be, shape, seed=320, batch=batch, levels=levels)


def test_merged_product_full_size_sampled_and_decrypts(be):
    """N=2^16, 24 limbs, batch 64 in the benchmark's launch configuration: one item word for word against the oracle,
    and an encrypted pair decrypts to the product within 1e-3 at scale 2^40"""
    announce("merged product N=2^16 batch 64, sampled parity")
    p = wl.PRESETS["act_2e16"]
    M = pc.make_material(C4, 4)
    ctx = be.context(*C4)
    batch, level, pick = p.batch, 24, 41
    evk = be.to_dev(M.rlk)
    a = pc.random_cts(M, level, batch, 5, ("a", level))
    b = pc.random_cts(M, level, batch, 5, ("b", level))
    scale = 2.0 ** p.log_scale
    za, zb = wl.slots_real(M.N // 2, 5, "za"), wl.slots_real(M.N // 2, 5, "zb")
    a[0], b[0] = M.encrypt(za, scale, level, "a"), M.encrypt(zb, scale, level, "b")
    out = be.empty(batch, 2, level - 1, M.N)
    ws = be.ws(ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, level, batch))
    ctx.profile_enable(True)
    ctx.hmul_relin_rescale_merged(be.to_dev(a), be.to_dev(b), evk, out, level, batch, ws)
    got = be.to_host(out).reshape(batch, 2, level - 1, M.N)
    ran = ctx.profile_read()
    ctx.profile_enable(False)
    assert "modup_cols_kernel<4, 4, 2>" in ran, list(ran)
    announce("oracle for item %d" % pick)
    assert np.array_equal(got[pick], M.O.hmul_relin_rescale_merged(a[pick], b[pick], M.rlk, level))
    dec = M.decrypt(got[0], scale * scale / M.O.q[level - 1], level - 1)
    assert np.max(np.abs(dec - za * zb)) < 1e-3


@pytest.mark.parametrize("shape,level,rotations,batch", [
    (TINY, 3, (1, 2, 100, 2047), 3),
    ((9, 7, 50, 3, 51, 3), 5, (1, 3, 255), 2),
    ((13, 3, 50, 1, 51, 1), 3, (5, 9), 3),
    ((14, 8, 50, 1, 51, 1), 8, (1, 7, 300, 4000, 8191), 2),
    ((16, 4, 50, 3, 51, 3), 4, (1, 2, 77), 2),
    ((17, 2, 50, 1, 51, 1), 2, (3, 11), 1),
])
def test_hoisted_rotations_match_oracle(be, shape, level, rotations, batch):
    """several rotations of each ciphertext from one shared ModUp: every word against the oracle's definition"""
    announce("hoisted rotations %r level %d offsets %r" % (shape, level, rotations))
    pc.case_rotate_hoisted(be, shape, seed=330, rotations=rotations, batch=batch, level=level)


def test_hoisted_rotations_decrypt_to_rotated_slots(be):
    """N=2^14, 8 limbs: 8 rotations of encrypted vectors decrypt to the rotated vectors within 1e-3 at scale 2^40"""
    announce("hoisted rotations N=2^14 decrypt")
    p = wl.PRESETS["hmul_rot_2e14"]
    rots = wl.rotation_offsets(p.N // 2, 8, 2)
    M = pc.make_material(C2, 2, rotations=rots)
    ctx = be.context(*C2)
    keys = [be.to_dev(M.gk[r]) for r in rots]
    for r, k in zip(rots, keys):
        ctx.galois_key_register(r, k)
    level, scale = 8, 2.0 ** p.log_scale
    z = wl.slots_complex(M.N // 2, 2, "hz")
    ct = M.encrypt(z, scale, level, "hz")
    out = be.empty(1, len(rots), 2, level, M.N)
    ws = be.ws(ctx.rotate_hoisted_workspace_bytes(level, 1, len(rots)))
    ctx.rotate_hoisted(be.to_dev(ct[None]), rots, out, level, 1, ws)
    got = be.to_host(out).reshape(len(rots), 2, level, M.N)
    for k, r in enumerate(rots):
        assert np.max(np.abs(M.decrypt(got[k], scale, level) - np.roll(z, -r))) < 1e-3


@pytest.mark.parametrize("shape,levels,terms,batch", [
    (TINY, [3, 2], 5, 2),
    ((10, 5, 40, 2, 41, 2), [5, 3], 3, 3),
    ((14, 3, 50, 2, 51, 2), [3], 4, 2),
    ((16, 4, 50, 3, 51, 3), [4], 7, 2),
    ((17, 2, 50, 1, 51, 1), [2], 2, 1),
])
def test_sum_of_products_matches_oracle(be, shape, levels, terms, batch):
    """lazy relinearisation: sum of `terms` tensors, one key switch and one rescale"""
    announce("sum of %d products %r levels %r" % (terms, shape, levels))
    pc.case_sum_of_products(be, shape, seed=340, terms=terms, batch=batch, levels=levels)


def test_rotation_packed_layers_match_oracle(be):
    """single-image packing: a dense layer (63 rotations from one ModUp, then again in calls of 16) and a sparse convolution matrix on one
    ciphertext, word for word against the oracle's schedule, and decrypting to the matrix-vector product"""
    from paper_1911_11377_amd import packed
    announce("rotation-packed dense layer 64x48, N=2^13")
    pc.case_packed_layer(be, (13, 3, 40, 2, 41, 2), 350, wl.weights_float((64, 48), 350, "fc"))
    pc.case_packed_layer(be, (13, 3, 40, 2, 41, 2), 350, wl.weights_float((64, 48), 350, "fc"), max_rotations=16)
    announce("rotation-packed convolution 4->4 channels 3x3 on 8x8, N=2^13")
    w = wl.weights_float((4, 4, 3, 3), 351, "conv")
    pc.case_packed_layer(be, (13, 3, 40, 1, 41, 1), 351, packed.conv_matrix(w, 8, 8, 1))
    announce("rotation-packed dense layer 16x16 at a lower level, N=2^12")
    pc.case_packed_layer(be, (12, 4, 40, 2, 41, 2), 352, wl.weights_float((16, 16), 352, "fc"), level=3)


@pytest.mark.parametrize("shape,topology", [
    ((7, 8, 50, 2, 51, 2), "single_image_tiny"),     # 64 slots: the input vector spans two ciphertexts, generic kernels
    ((13, 8, 50, 3, 51, 3), "single_image_tiny"),    # register-tiled kernels, 3-prime digits
])
def test_single_image_network_matches_oracle(be, shape, topology):
    """one image through a network in the rotation-packed layout (strided convolution, degree-2 activations, pooling merged
    into the next layer as a matrix product, vectors that may span several ciphertexts): every output word against the
    oracle's schedule, decrypted output against the float network"""
    announce("single-image network %s %r" % (topology, shape))
    pc.case_packed_network(be, shape, seed=380, topology=topology)
    announce("single-image network %s %r, baby and giant steps" % (topology, shape))
    pc.case_packed_network(be, shape, seed=381, topology=topology, bsgs=True)


def test_grouped_plaintext_products_at_network_size(be):
    """the launch shape of a 3x32x32 image's widest layer (128 rotated copies, 61 sums, 7655 plaintexts at level 8,
    N = 2^14): sampled output words against the sum of products in Python integers"""
    import torch

    announce("grouped plaintext products, 128 x 61 x 7655 at N=2^14")
    shape, level, n_ct, n_groups = (14, 8, 50, 1, 51, 1), 8, 128, 61
    ctx = be.context(*shape)
    N, q = ctx.N, ctx.q
    r = wl.rng(384, "mac.big")
    table = np.full((n_groups, n_ct), -1, dtype=np.int32)
    picks = r.permutation(n_groups * n_ct)[:7655]
    table.reshape(-1)[np.sort(picks)] = np.arange(7655, dtype=np.int32)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(384)
    cts = torch.randint(0, 1 << 49, (n_ct, 2, level, N), dtype=torch.int64, device="cuda:0", generator=gen)  # canonical: every prime exceeds 2^49
    pts = torch.randint(0, 1 << 49, (7655, level, N), dtype=torch.int64, device="cuda:0", generator=gen)
    tab = torch.from_numpy(np.concatenate([table.reshape(-1), np.zeros(2, np.int32)]).view(np.int64)).to("cuda:0")
    out = be.empty(n_groups, 2, level, N)
    ctx.plain_mac(cts, n_ct, pts, 7655, tab, n_groups, out, level)
    torch.cuda.synchronize()
    for _ in range(40):
        g, c, l, w = int(r.integers(n_groups)), int(r.integers(2)), int(r.integers(level)), int(r.integers(N))
        ss = np.nonzero(table[g] >= 0)[0]
        xs = cts[torch.from_numpy(ss).to("cuda:0"), c, l, w].cpu().numpy()
        ys = pts[torch.from_numpy(table[g][ss].astype(np.int64)).to("cuda:0"), l, w].cpu().numpy()
        want = sum(int(a) * int(b) for a, b in zip(xs, ys)) % int(q[l])
        assert int(out[g, c, l, w].item()) == want, (g, c, l, w)
    ctx.close()


def test_grouped_plaintext_products(be):
    announce("grouped plaintext products")
    pc.case_plain_mac(be, TINY, seed=382)
    pc.case_plain_mac(be, (13, 5, 50, 1, 51, 1), seed=383, n_ct=4, level=4)


@pytest.mark.parametrize("shape,log_scale,batch", [
    ((4, 2, 20, 1, 21, 1), 12, 3),
    (TINY, 30, 4),
    ((13, 3, 50, 1, 51, 1), 45, 2),
    (C2, 40, 3),
    ((16, 4, 50, 3, 51, 3), 40, 2),
    ((17, 2, 50, 1, 51, 1), 40, 1),
])
def test_device_encode_and_encrypt(be, shape, log_scale, batch):
    """encoding on the device within one unit per coefficient of the oracle's encoder (and the slots back within 1e-9);
    encryption on the device bit for bit"""
    announce("device encode/encrypt %r scale 2^%d" % (shape, log_scale))
    pc.case_encode_encrypt_device(be, shape, seed=360, batch=batch, log_scale=log_scale)
    if shape == TINY:
        pc.case_encode_encrypt_device(be, shape, seed=361, batch=5, level=2, log_scale=25, complex_slots=False, small_ws=True)


def test_device_sampler_matches_oracle(be):
    """ternary and rounded-Gaussian polynomials drawn on the device: every coefficient equals the oracle's sampler"""
    announce("device sampler")
    pc.case_sample_device(be, TINY, seed=0x1234567890ABCDEF, rows=5)
    pc.case_sample_device(be, (16, 2, 50, 1, 51, 1), seed=362, rows=3, sigma=3.2, first_index=(1 << 40) + 77)
    pc.case_sample_device(be, (13, 2, 50, 1, 51, 1), seed=363, rows=2, sigma=8.0, first_index=0)


def _device_residues(torch, q_list, lead, N, seed):
    """uniform residues below 2^49 (canonical for every 50/51-bit prime) drawn on the device from a seeded generator"""
    g = torch.Generator(device="cuda:0")
    g.manual_seed(wl.BASE_SEED + seed)
    out = torch.empty(tuple(lead) + (len(q_list), N), dtype=torch.int64, device="cuda:0")
    step = 1 << 27
    flat = out.view(-1)
    for o in range(0, flat.numel(), step):
        flat[o:o + step].random_(0, 1 << 49, generator=g)
    return out


def _oracle_window(O, x_dev, wi, Cin, rows_in, W, in_row0, H, kh, stride, pad, level, o, oy, ox):
    """one output ciphertext of a convolution from the oracle: the window's input ciphertexts are copied from the device
    buffer x_dev ([Cin][rows_in][W] holding image rows in_row0..), taps on padding become all-zero ciphertexts"""
    N = O.N
    win = np.zeros((Cin, kh, kh, 2, level, N), dtype=np.uint64)
    for u in range(kh):
        for v in range(kh):
            iy, ix = oy * stride + u - pad, ox * stride + v - pad
            if 0 <= iy < H and 0 <= ix < W:
                win[:, u, v] = x_dev[:, iy - in_row0, ix].cpu().numpy().view(np.uint64)
    return O.conv2d_mac(win, wi[o:o + 1], 1, 0, level)[0, 0, 0]


def test_conv_layer_full_size_sampled(be):
    """the conv layer of the 2^15 workload in the benchmark's launch configuration (3x32x32 pixel ciphertexts, 16 primes,
    3 -> 32 channels, 5x5 stride 2: matrix cores, 128 padded taps) followed by the rescale of all 6272 outputs; four
    output ciphertexts compared word for word with the oracle"""
    import torch
    announce("conv layer N=2^15 full size, sampled parity")
    p3 = wl.PRESETS["conv_2e15"]
    shape = (p3.logN, p3.n_q, p3.q_bits, p3.k, p3.special_bits, p3.alpha)
    O = orc.Oracle(*shape)
    ctx = be.context(*shape)
    assert ctx.moduli == O.moduli
    L, N = p3.n_q, p3.N
    Cin, H, W, Oc, kh, stride = 3, 32, 32, 32, 5, 2
    Ho = (H - kh) // stride + 1
    x = _device_residues(torch, O.q[:L], (Cin, H, W, 2), N, 31)
    wi = np.rint(wl.weights_float((Oc, Cin, kh, kh), 31) * O.q[L - 1]).astype(np.int64)
    dw = be.to_dev(wi, np.int64)
    mac = be.empty(Oc, Ho, Ho, 2, L, N)
    out = be.empty(Oc, Ho, Ho, 2, L - 1, N)
    ws = be.ws(max(ctx.conv2d_workspace_bytes(Cin, Oc, kh, kh, L), ctx.workspace_bytes(ckksmi.OP_RESCALE, L, 256)))
    ctx.profile_enable(True)
    ctx.conv2d_mac(x, dw, Cin, H, W, Oc, kh, kh, stride, 0, mac, L, ws)
    ctx.rescale(mac, out, L, Oc * Ho * Ho, ws)
    torch.cuda.synchronize()
    assert "conv_mac_mfma_strip_kernel" in ctx.profile_read()  # 75 taps: one full step and a quad step, windows shared through LDS
    ctx.profile_enable(False)
    for o, oy, ox in ((0, 0, 0), (31, 13, 13), (17, 6, 9), (8, 13, 0)):
        announce("oracle for output (%d,%d,%d)" % (o, oy, ox))
        want = _oracle_window(O, x, wi, Cin, H, W, 0, H, kh, stride, 0, L, o, oy, ox)
        assert np.array_equal(mac[o, oy, ox].cpu().numpy().view(np.uint64), want), "MAC of output %r" % ((o, oy, ox),)
        assert np.array_equal(out[o, oy, ox].cpu().numpy().view(np.uint64), O.rescale(want, L)), "rescaled output %r" % ((o, oy, ox),)
    ctx.close()


def test_network_layer_shapes_sampled(be):
    """layers of the 2^16 network at their real width (two limbs): the 3136 -> 256 fully connected layer (49 tap steps,
    8 channel groups) at N=2^14 and a strip of the zero-padded 64 -> 64 3x3 convolution at N=2^16, sampled outputs
    against the oracle"""
    import torch
    from concurrent.futures import ThreadPoolExecutor
    announce("FC 3136->256 at N=2^14, sampled parity")
    shape = (14, 2, 50, 0, 51, 1)
    O = orc.Oracle(*shape)
    ctx = be.context(*shape)
    L, N = 2, 1 << 14
    F, Oc = 3136, 256
    x = _device_residues(torch, O.q[:L], (F, 1, 1, 2), N, 32)
    wi = np.rint(wl.weights_float((Oc, F), 32) * O.q[L - 1]).astype(np.int64)
    out = be.empty(Oc, 2, L, N)
    ws = be.ws(ctx.conv2d_workspace_bytes(F, Oc, 1, 1, L))
    ctx.profile_enable(True)
    ctx.fc_mac(x, be.to_dev(wi, np.int64), F, Oc, out, L, ws)
    torch.cuda.synchronize()
    assert "conv_mac_mfma_kernel" in ctx.profile_read()
    ctx.profile_enable(False)
    xh = x.cpu().numpy().view(np.uint64).reshape(F, 2, L, N)
    picks = (0, 255, 100)
    with ThreadPoolExecutor(len(picks)) as ex:  # the oracle's C calls release the GIL
        wants = list(ex.map(lambda o: O.fc_mac(xh, wi[o:o + 1], L)[0], picks))
    for o, want in zip(picks, wants):
        assert np.array_equal(out[o].cpu().numpy().view(np.uint64), want), "FC output %d" % o
    ctx.close()
    del x, xh, out, ws

    announce("padded conv strip 64->64 at N=2^16, sampled parity")
    shape = (16, 2, 50, 0, 51, 1)
    O = orc.Oracle(*shape)
    ctx = be.context(*shape)
    N = 1 << 16
    # rows 12..13 of the 14x14 map from a strip holding image rows 11..13 (the last row touches the bottom padding)
    Cin, H, W, Oc, kh = 64, 14, 14, 64, 3
    in_row0, rows_in, out_row0, out_rows = 11, 3, 12, 2
    xs = _device_residues(torch, O.q[:L], (Cin, rows_in, W, 2), N, 33)
    wc = np.rint(wl.weights_float((Oc, Cin, kh, kh), 33) * O.q[L - 1]).astype(np.int64)
    outs = be.empty(Oc, out_rows, W, 2, L, N)
    ws = be.ws(ctx.conv2d_workspace_bytes(Cin, Oc, kh, kh, L))
    ctx.conv2d_mac_rows(xs, be.to_dev(wc, np.int64), Cin, H, W, Oc, kh, kh, 1, 1, in_row0, rows_in, out_row0, out_rows, outs, L, ws)
    torch.cuda.synchronize()
    picks = ((0, 12, 0), (63, 13, 13), (33, 13, 5), (5, 12, 7))
    with ThreadPoolExecutor(len(picks)) as ex:
        wants = list(ex.map(lambda t: _oracle_window(O, xs, wc, Cin, rows_in, W, in_row0, H, kh, 1, 1, L, *t), picks))
    for (o, oy, ox), want in zip(picks, wants):
        assert np.array_equal(outs[o, oy - out_row0, ox].cpu().numpy().view(np.uint64), want), "strip output %r" % ((o, oy, ox),)
    ctx.close()


@pytest.mark.parametrize("shape,level,batch,sample", [
    ((10, 6, 50, 3, 51, 3), 6, 3, [0, 1, 2]),          # generic kernels
    ((13, 6, 50, 3, 51, 3), 6, 5, [0, 1, 2, 3, 4]),    # register-tiled kernels, every item
    ((14, 8, 51, 3, 51, 3), 7, 4, [0, 3]),             # 51-bit primes, input below the top level
])
def test_activation_schedule_on_gpu(be, shape, level, batch, sample):
    """x^2 then 0.5 + 0.25y - 0.02y^3 with relin + rescale at each level, against the oracle's
    composition (bit-exact, both the square and the result) and the float polynomial; the integer constants are
    the test's own and must equal the call sequence's"""
    announce("activation schedule %r" % (shape,))
    pc.case_activation(be, shape, seed=5, level=level, batch=batch, sample=sample, workers=len(sample))


def test_activation_schedule_full_size_sampled(be):
    """the schedule at the benchmark's shape: N=2^16, 24 primes, level 24 -> 21, batch 64, workspace carved by the call
    sequence; the first, a middle and the last item are real encryptions, compared word for word after x^2 and at the end,
    and decrypt to the float polynomial within 1e-3"""
    announce("activation schedule N=2^16 level 24 batch 64, sampled parity")
    pc.case_activation(be, C4, seed=7, level=24, batch=64, sample=[0, 33, 63], workers=3,
                       expect_kernels=("modup_cols_kernel<4, 4, 3>", "modup_cols_kernel<4, 1, 1>", "tensor_rows_kernel"))


def test_step_replays_from_a_captured_graph(be):
    """HMult + relinearise + rescale enqueues kernels only (no allocation, no memset, no synchronisation): captured into a
    graph on a side stream and replayed with fresh inputs in the same buffers, every replay gives the eager call's words,
    and the first the oracle's"""
    import torch

    announce("graph capture and replay")
    shape, level, batch = (13, 7, 50, 3, 51, 3), 7, 2
    M = pc.make_material(shape, 330)
    O = M.O
    ctx = be.context(*shape)
    evk = be.to_dev(M.rlk)
    xs = [wl.uniform_limbs(O.q[:level], O.N, 330 + r, "graph.x", lead=(batch, 2)) for r in range(3)]
    ys = [wl.uniform_limbs(O.q[:level], O.N, 330 + r, "graph.y", lead=(batch, 2)) for r in range(3)]
    da, db = be.to_dev(xs[0]), be.to_dev(ys[0])
    out, ref = be.empty(batch, 2, level - 1, O.N), be.empty(batch, 2, level - 1, O.N)
    ws = be.ws(ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, level, batch))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ctx.hmul_relin_rescale(da, db, evk, out, level, batch, ws)  # warm-up outside the capture
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        ctx.hmul_relin_rescale(da, db, evk, out, level, batch, ws)
    for r in range(3):
        da.copy_(be.to_dev(xs[r]))
        db.copy_(be.to_dev(ys[r]))
        out.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ctx.hmul_relin_rescale(da, db, evk, ref, level, batch, ws)  # the program's own eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(out, ref), "replay %d differs from the eager call" % r
        if r == 0:
            want = np.stack([O.hmul_relin_rescale(xs[0][i], ys[0][i], M.rlk, level) for i in range(batch)])
            assert np.array_equal(be.to_host(out).reshape(want.shape), want), "replayed step differs from the oracle"
    ctx.close()


def test_edge_cases(be):
    announce("edge cases")
    ctx = be.context(*TINY)
    buf = be.empty(2, 2, 3, 4096)
    ctx.add(buf, buf, buf, 3, 0)  # empty batch: nothing enqueued
    with pytest.raises(ckksmi.CkksmiError) as e:
        ctx.rescale(buf, be.empty(2, 2, 2, 4096), 1, 2, be.ws(1 << 20))
    assert e.value.code == ckksmi.ELEVEL
    with pytest.raises(ckksmi.CkksmiError) as e:
        ctx.relin(be.empty(2, 3, 3, 4096), buf, buf, 3, 2, be.ws(64))
    assert e.value.code == ckksmi.EWORKSPACE
    with pytest.raises(ckksmi.CkksmiError) as e:
        ctx.add(buf, buf, buf, 4, 1)
    assert e.value.code == ckksmi.ELEVEL


def test_variant_entry_points_refuse_bad_arguments(be):
    announce("argument checks of the variant entry points")
    pc.case_variant_errors(be)
