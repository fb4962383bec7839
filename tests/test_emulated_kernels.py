"""The library's kernel sources, compiled against the CPU stand-in under tests/emu
and run fibre by fibre on tiny shapes with guard pages behind every buffer, compared
with the oracle.  This checks indexing and launch shapes on the CPU before a GPU ever
runs them; the parity claims themselves come from the GPU tests."""
import pytest

import parity_cases as pc

# (logN, n_q, q_bits, k, special_bits, alpha)
TINY = (6, 3, 30, 1, 31, 1)
HYBRID = (5, 5, 40, 2, 41, 2)
HYBRID3 = (4, 7, 50, 3, 51, 3)
TWO_PASS = (13, 2, 50, 1, 51, 1)


@pytest.fixture(scope="module")
def be():
    return pc.EmuBackend()


@pytest.mark.parametrize("shape", [TINY, (2, 2, 20, 1, 21, 1), (9, 2, 50, 1, 51, 1), (12, 1, 40, 1, 41, 1), TWO_PASS,
                                   (14, 1, 50, 1, 51, 1), (16, 1, 50, 1, 51, 1), (16, 2, 30, 0, 31, 1)])
def test_emulated_ntt(be, shape):
    pc.case_ntt(be, shape, seed=100)


@pytest.mark.parametrize("shape", [TINY, HYBRID3])
def test_emulated_elementwise(be, shape):
    pc.case_elementwise(be, shape, seed=101)


@pytest.mark.parametrize("shape", [TINY, HYBRID])
def test_emulated_rescale(be, shape):
    pc.case_rescale(be, shape, seed=102)


@pytest.mark.parametrize("shape,levels", [(TINY, [3, 1]), (HYBRID, [5, 4, 3]), (HYBRID3, [7, 5, 2])])
def test_emulated_relin_and_composite(be, shape, levels):
    pc.case_relin_and_composite(be, shape, seed=103, levels=levels)


def test_emulated_relin_small_workspace(be):
    pc.case_relin_and_composite(be, HYBRID, seed=104, batch=3, levels=[5], small_ws=True)


def test_emulated_two_pass_composite(be):
    pc.case_relin_and_composite(be, TWO_PASS, seed=105, batch=1, levels=[2])


@pytest.mark.parametrize("shape,level", [(TINY, 3), (HYBRID3, 5)])
def test_emulated_rotate(be, shape, level):
    pc.case_rotate(be, shape, seed=106, rotations=[1, 3, 7], batch=4, level=level)


def test_emulated_rotate_register_tiled_sizes(be):
    """2^12 <= N: no rotated copy is written; the inverse row pass and the fused inner product read c1 and c0 through the
    automorphism (rows of pairs); several items per workgroup, partial last digit"""
    pc.case_rotate(be, (12, 3, 50, 2, 51, 2), seed=126, rotations=[1, 3, 700], batch=3, level=3)
    with be.tuned(8):
        pc.case_rotate(be, (13, 2, 51, 1, 51, 1), seed=127, rotations=[5, 2047, 4095], batch=4, level=2)


def test_emulated_conv(be):
    pc.case_conv(be, TINY, seed=107, Cin=2, H=5, W=5, Oc=9, kh=3, stride=2, pad=0)
    pc.case_conv(be, TINY, seed=108, Cin=1, H=4, W=4, Oc=2, kh=3, stride=1, pad=1, level=2)


def test_emulated_conv_matrix_cores(be):
    """the three matrix-core kernels: strips shared by 2 x 2 and 1 x 4 positions, weight digits resident, weight digits
    streaming; full and quad steps, two channel groups (the second mostly empty), zero padding, a 51-bit prime, strips of rows"""
    pc.case_conv(be, (6, 2, 51, 0, 52, 1), seed=115, Cin=3, H=3, W=3, Oc=34, kh=5, stride=1, pad=2)     # 75 taps: full + quad step
    pc.case_conv(be, (6, 1, 50, 0, 51, 1), seed=116, Cin=4, H=5, W=5, Oc=8, kh=5, stride=1, pad=0, rows_check=False)    # 100 taps
    # 261 taps: more steps than stay in LDS, the streaming kernel; its FC part has 87 taps (two full steps)
    pc.case_conv(be, (6, 1, 50, 0, 51, 1), seed=117, Cin=29, H=3, W=3, Oc=8, kh=3, stride=1, pad=1, rows_check=False)
    # one output row of five positions: the four waves take 1 x 4 positions (two tiles, three waves without a position)
    pc.case_conv(be, (6, 1, 50, 0, 51, 1), seed=119, Cin=2, H=3, W=7, Oc=8, kh=3, stride=1, pad=0, fc_check=False)
    # stride 2 with padding, 5 x 5 outputs (waves without a position in both directions), strips of rows that end inside a
    # 2 x 2 block: the rows below the strip are neither read nor written
    pc.case_conv(be, (6, 1, 50, 0, 51, 1), seed=123, Cin=3, H=9, W=9, Oc=8, kh=3, stride=2, pad=1, fc_check=False)
    # a workgroup walks several tiles / positions: the double-buffered strip, the request for the next position's words
    with be.tuned(2):
        pc.case_conv(be, (6, 1, 50, 0, 51, 1), seed=120, Cin=3, H=7, W=6, Oc=8, kh=5, stride=1, pad=1, fc_check=False)    # 2 x 2 blocks, 20 positions
        pc.case_conv(be, (6, 1, 50, 0, 51, 1), seed=121, Cin=2, H=3, W=13, Oc=8, kh=3, stride=1, pad=0, rows_check=False, fc_check=False)    # 1 x 4 blocks, three tiles
        # 7 x 3 x 3 = 63 taps at stride 3: the window block (7*3*12 lines) is too wide to stage, weight digits resident, six positions
        pc.case_conv(be, (6, 1, 50, 0, 51, 1), seed=122, Cin=7, H=4, W=16, Oc=9, kh=3, stride=3, pad=1, fc_check=False)


def test_emulated_pooling(be):
    """(whole networks: the Table-1-like one below; the square-activation network runs on the GPU)"""
    pc.case_pool(be, TINY, seed=112, Cin=2, H=5, W=4, k=2)
    pc.case_pool(be, TINY, seed=113, Cin=1, H=3, W=3, k=3, level=2)
    pc.case_pool(be, TINY, seed=120, Cin=2, H=3, W=2, k=2, pad=1)


def test_emulated_table1_like_network(be):
    """the layer kinds of Table 1 with the degree-2 activation and a padded pooling (the full sequence runs on the GPU)"""
    pc.case_cnn(be, (6, 8, 50, 2, 51, 2), seed=121, topology="table1_tiny")


def test_emulated_item_loop_and_composite_at_2e16(be):
    """N = 2^16: both register-tiled passes, with workgroups looping over several items"""
    with be.tuned(16):
        pc.case_ntt(be, (16, 1, 50, 1, 51, 1), seed=109, batch=3)
        pc.case_ntt(be, (13, 2, 50, 1, 51, 1), seed=110, batch=3)
        pc.case_relin_and_composite(be, (16, 2, 50, 1, 51, 1), seed=111, batch=2, levels=[2])


def test_emulated_fused_hybrid_at_2e16(be):
    """N = 2^16 with 3-prime digits: fused ModUp / inner product / ModDown / rescale kernels, partial last digit"""
    with be.tuned(64):
        pc.case_relin_and_composite(be, (16, 4, 50, 3, 51, 3), seed=112, batch=2, levels=[4, 2])
        pc.case_rescale(be, (16, 3, 50, 0, 51, 1), seed=113, batch=2, levels=[3])


@pytest.mark.parametrize("logN", [12, 13, 14, 15])
def test_emulated_fused_path_other_sizes(be, logN):
    """2^12 <= N < 2^16: general column geometry (N1 = 16, 32, 64, 128), 40-, 50- and 51-bit primes"""
    with be.tuned(8):
        pc.case_ntt(be, (logN, 2, 50, 1, 51, 1), seed=116, batch=3)
        pc.case_relin_and_composite(be, (logN, 3, 50, 2, 51, 2), seed=117, batch=2, levels=[3, 2])
        pc.case_relin_and_composite(be, (logN, 2, 40, 1, 41, 1), seed=118, batch=1, levels=[2])


@pytest.mark.parametrize("shape,levels", [(TINY, [3, 2]), (HYBRID, [5, 4, 2]), (HYBRID3, [7, 5, 2])])
def test_emulated_merged_product_small_sizes(be, shape, levels):
    """one division by P*q_last, exact form: elementwise conversion with the double-precision overshoot"""
    pc.case_merged_product(be, shape, seed=121, levels=levels)
    if shape == HYBRID:
        pc.case_merged_product(be, shape, seed=122, batch=3, levels=[5], small_ws=True)


def test_emulated_merged_product_at_2e16(be):
    """the fused form: conversion kernel over {q_last, p_0, p_1, p_2} with the overshoot taken from the source registers"""
    with be.tuned(64):
        pc.case_merged_product(be, (16, 4, 50, 3, 51, 3), seed=123, batch=2, levels=[4, 2], expect_kernel="modup_cols_kernel<4, 4, 2>")


@pytest.mark.parametrize("logN", [13, 14, 15])
def test_emulated_merged_product_other_sizes(be, logN):
    with be.tuned(8):
        pc.case_merged_product(be, (logN, 3, 50, 2, 51, 2), seed=125, batch=2, levels=[3, 2])


@pytest.mark.parametrize("shape,level", [(TINY, 3), (HYBRID, 4), (HYBRID3, 5)])
def test_emulated_hoisted_rotations_small_sizes(be, shape, level):
    pc.case_rotate_hoisted(be, shape, seed=126, rotations=(1, 3, 6), level=level)
    if shape == HYBRID:
        pc.case_rotate_hoisted(be, shape, seed=127, rotations=(2, 5), level=5, small_ws=True)


def test_emulated_hoisted_rotations_at_2e13(be):
    """register-tiled sizes: shared ModUp through the fused conversion kernels, gathered inner product"""
    pc.case_rotate_hoisted(be, (13, 3, 50, 2, 51, 2), seed=128, rotations=(1, 100, 4095), batch=2, level=3)
    # more items than one workgroup stages (64 KiB of LDS: 32 digit rows), ragged last chunk; N = 256: a single run
    pc.case_rotate_hoisted(be, (9, 9, 40, 1, 41, 1), seed=129, rotations=(1, 77), batch=5, level=9)
    pc.case_rotate_hoisted(be, (8, 2, 40, 1, 41, 1), seed=130, rotations=(3,), batch=2, level=2)
    # more digits than the LDS-staged gather takes: the plain gather kernel; and a ring below 256 words
    pc.case_rotate_hoisted(be, (8, 17, 40, 1, 41, 1), seed=138, rotations=(2,), batch=1, level=17)


def test_emulated_sum_of_products(be):
    """lazy relinearisation: the tensor kernels accumulate the terms (elementwise kernel, and the one fused with the row pass)"""
    pc.case_sum_of_products(be, HYBRID, seed=131, terms=3, levels=[5, 2])
    pc.case_sum_of_products(be, (13, 3, 50, 2, 51, 2), seed=132, terms=4, batch=2, levels=[3])


def test_emulated_rotation_packed_layers(be):
    """single-image packing: a dense layer (every diagonal, two chunks of rotations) and a sparse convolution matrix"""
    from paper_1911_11377_amd import packed, workloads as wl
    pc.case_packed_layer(be, (6, 3, 40, 2, 41, 2), 134, wl.weights_float((32, 20), 134, "fc"))
    pc.case_packed_layer(be, (6, 3, 40, 2, 41, 2), 134, wl.weights_float((32, 20), 134, "fc"), max_rotations=7)  # five calls, ragged last
    w = wl.weights_float((2, 2, 3, 3), 135, "conv")
    pc.case_packed_layer(be, (7, 3, 40, 1, 41, 1), 135, packed.conv_matrix(w, 4, 4, 1))


@pytest.mark.parametrize("shape,log_scale", [(TINY, 30), ((2, 2, 20, 1, 21, 1), 12), ((12, 2, 50, 1, 51, 1), 40), ((13, 2, 50, 1, 51, 1), 45)])
def test_emulated_device_encode_and_encrypt(be, shape, log_scale):
    """one-pass and two-pass complex inverse transform, rounding, residues; encryption with supplied randomness"""
    pc.case_encode_encrypt_device(be, shape, seed=136, batch=2, log_scale=log_scale)
    if shape == TINY:
        pc.case_encode_encrypt_device(be, shape, seed=137, batch=3, level=2, log_scale=25, complex_slots=False, small_ws=True)
    if shape[0] == 12:
        # the fused encryption (column pass from the small coefficients, row pass forming the ciphertext): 51-bit primes,
        # workgroups looping over items, a level below the top, the batch swept in chunks
        with be.tuned(2):
            pc.case_encode_encrypt_device(be, (12, 3, 51, 1, 51, 1), seed=138, batch=3, level=2, log_scale=40, small_ws=True)
            pc.case_encode_encrypt_device(be, (12, 3, 51, 1, 51, 1), seed=139, batch=5, log_scale=40)


def test_emulated_device_sampler(be):
    pc.case_sample_device(be, TINY, seed=0x1234567890ABCDEF)
    pc.case_sample_device(be, (9, 2, 50, 1, 51, 1), seed=3, rows=2, sigma=1.5, first_index=0)


def test_emulated_variant_entry_points_refuse_bad_arguments(be):
    pc.case_variant_errors(be)


def test_emulated_misaligned_device_pointer_is_rejected(be):
    """device buffers must be 16-byte aligned (vector accesses of two words): an odd word offset is refused on the host"""
    from paper_1911_11377_amd import ckksmi
    shape = TINY
    ctx = be.context(*shape)
    N, level = 1 << shape[0], shape[1]
    a = be.empty(1 + 2 * level * N)
    out = be.empty(2 * (level - 1) * N)
    ws = be.ws(ctx.workspace_bytes(ckksmi.OP_RESCALE, level, 1))
    with pytest.raises(ckksmi.CkksmiError) as e:
        ctx.rescale(a[1:], out, level, 1, ws, stream=be.stream)
    assert e.value.code == ckksmi.EINVAL
    ctx.close()



FEW_PAIRS = (("qm1", "qm1"), ("half_lo", "half_hi"), ("alt", "qm1"), ("onehot", "alt_halves"))


@pytest.mark.parametrize("shape", [TINY, HYBRID, HYBRID3, (5, 9, 51, 2, 51, 2)])
def test_emulated_edge_values_generic_kernels(be, shape):
    """all-0, all-(q-1), (q-1)/2, (q+1)/2, alternating and one-hot residues, seeded key and all-(q-1) key, through every
    operation (generic kernels)"""
    pc.case_edge_values(be, shape, seed=140)


@pytest.mark.parametrize("shape,level,seeded", [((13, 24, 50, 3, 51, 3), 24, False), ((13, 15, 51, 3, 51, 3), 15, True)])
def test_emulated_edge_values_register_tiled_kernels(be, shape, level, seeded):
    """the same at a register-tiled size with 3-prime digits: 8 digits of 50-bit primes (eight terms meet in the fused inner
    product's accumulators before their one reduction; key of all q-1) and 5 digits of 51-bit primes (reduced every four
    terms; both keys).  Two operand pairs each: the GPU suite runs the full set."""
    pc.case_edge_values(be, shape, seed=142, level=level, conv=False, pairs=FEW_PAIRS[:2], seeded_key=seeded)


def test_emulated_edge_values_matrix_core_mac(be):
    pc.case_edge_values(be, (7, 2, 51, 0, 52, 1), seed=143)
    pc.case_edge_values(be, (7, 3, 50, 1, 51, 1), seed=144)


def test_emulated_activation_schedule_register_tiled(be):
    """x^2 then the degree-3 polynomial at N = 2^13 with 3-prime digits: the scalar rescale reads its input one level up and
    adds onto the output buffer; workspace carved by the call sequence; every item compared"""
    pc.case_activation(be, (13, 6, 50, 3, 51, 3), seed=145, level=6, batch=3, sample=[0, 1, 2])


def test_emulated_grouped_plaintext_products(be):
    pc.case_plain_mac(be, TINY, seed=160)
    pc.case_plain_mac(be, (5, 4, 50, 1, 51, 1), seed=161, n_ct=3, level=3)


def test_emulated_single_image_network_baby_and_giant_steps(be):
    """the same network with baby and giant steps: period 64 with two input ciphertexts (baby 8), period 128 with one"""
    pc.case_packed_network(be, (7, 8, 50, 2, 51, 2), seed=152, topology="single_image_tiny", max_rotations=5, bsgs=True)
    pc.case_packed_network(be, (8, 8, 50, 2, 51, 2), seed=153, topology="single_image_tiny", bsgs=True)


def test_emulated_single_image_network(be):
    """one image in the rotation-packed layout: strided convolution, activation, pooling merged into the next layer; with 64
    slots the input spans two ciphertexts (block matrix), with 128 one; rotations in calls of at most 5 in the first run"""
    pc.case_packed_network(be, (7, 8, 50, 2, 51, 2), seed=150, topology="single_image_tiny", max_rotations=5)
    pc.case_packed_network(be, (8, 8, 50, 2, 51, 2), seed=151, topology="single_image_tiny")
