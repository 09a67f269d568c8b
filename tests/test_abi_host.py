"""Host-side checks of libcct.so that need no GPU: the library loads, exports every symbol the
header declares, validates arguments, and its shape/selector functions obey what the paper fixes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_1504_04343_amd import binding
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cct.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cct_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(B):
    names = declared_functions()
    assert len(names) >= 12
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_strerror(B):
    assert B.strerror(0) == "ok"
    for code in (B.EINVAL, B.EWORKSPACE, B.EUNSUPPORTED, B.EHIP, B.ESCRATCH, -99):
        assert B.strerror(code)


def test_output_dims_and_lowered_shapes_match_golden(B):
    path = os.path.join(ROOT, "tests", "golden", "caffenet_shapes.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        C, H, O, K, s, p, g, hout = map(int, f[1:9])
        want = list(map(int, f[9:15]))
        N = 256
        d = B.make_desc(N, C, H, H, O, K, s, p, g)
        assert B.cct_conv_output_dims(d) == (hout, hout)
        got = []
        for t in (1, 2, 3):
            rows, cols, rcols = B.cct_lowered_shape(d, t)
            assert rows % N == 0                      # Sec. 2.2: b times larger
            got += [rows // N, cols]
            assert rcols == (O // g) * K ** (t - 1)
            assert B.cct_lowered_ld(d, t) >= rows and B.cct_lowered_ld(d, t) % 256 == 0
        assert got == want


BAD = [
    dict(N=0), dict(C=0), dict(H=0), dict(O=0), dict(K=0), dict(stride=0), dict(pad=-1),
    dict(groups=0), dict(groups=4), dict(K=40), dict(lowering=7), dict(precision=5),
]


@pytest.mark.parametrize("bad", BAD)
def test_invalid_descriptors_are_rejected_everywhere(B, bad):
    base = dict(N=2, C=6, H=9, W=9, O=6, K=3, stride=1, pad=1, groups=2, lowering=0, precision=0)
    base.update(bad)
    d = B.make_desc(**base)
    with pytest.raises(B.CctError) as e:
        B.cct_conv_output_dims(d)
    assert e.value.code == B.EINVAL
    with pytest.raises(B.CctError):
        B.cct_conv_workspace_bytes(d, B.PASS_FORWARD)
    with pytest.raises(B.CctError):
        B.cct_pick_lowering(d, B.PASS_FORWARD)
    # device entry points validate before touching anything: null pointers, no launch
    lib = ctypes.CDLL(B.LIB_PATH)
    assert lib.cct_conv_forward(ctypes.byref(d), None, None, None, None, None, ctypes.c_size_t(0),
                                None) == B.EINVAL


def test_null_pointers_and_bad_pass(B):
    lib = ctypes.CDLL(B.LIB_PATH)
    d = B.make_desc(2, 4, 8, 8, 4, 3, 1, 1, 1)
    z = ctypes.c_size_t(1 << 20)
    assert lib.cct_conv_forward(ctypes.byref(d), None, None, None, None, None, z, None) == B.EINVAL
    assert lib.cct_conv_backward_data(ctypes.byref(d), None, None, None, None, z, None) == B.EINVAL
    assert lib.cct_conv_backward_weights(ctypes.byref(d), None, None, None, None, None, z,
                                         None) == B.EINVAL
    assert lib.cct_lower(ctypes.byref(d), 1, None, None, None) == B.EINVAL
    assert lib.cct_conv_output_dims(None, None, None) == B.EINVAL
    out = ctypes.c_size_t()
    assert lib.cct_conv_workspace_bytes(ctypes.byref(d), 9, ctypes.byref(out)) == B.EINVAL
    assert lib.cct_conv_workspace_bytes_for_chunk(ctypes.byref(d), 0, 0, ctypes.byref(out)) == B.EINVAL
    assert lib.cct_conv_workspace_bytes_for_chunk(ctypes.byref(d), 0, 3, ctypes.byref(out)) == B.EINVAL


def test_workspace_too_small_and_misaligned(B):
    lib = ctypes.CDLL(B.LIB_PATH)
    d = B.make_desc(2, 4, 8, 8, 4, 3, 1, 1, 1, lowering=B.LOWER_TYPE1)
    fake = ctypes.c_void_p(0x10000)        # never dereferenced: the call fails before any launch
    assert lib.cct_conv_forward(ctypes.byref(d), fake, fake, None, fake, fake, ctypes.c_size_t(16),
                                None) == B.EWORKSPACE
    odd = ctypes.c_void_p(0x10004)
    assert lib.cct_conv_forward(ctypes.byref(d), fake, fake, None, fake, odd,
                                ctypes.c_size_t(1 << 30), None) == B.EINVAL


def test_workspace_grows_linearly_with_chunk(B):
    # Sec. 2.2: memory footprint of the lowered matrix is proportional to the batch it holds
    d = B.make_desc(256, 96, 27, 27, 256, 5, 1, 2, 2, lowering=B.LOWER_TYPE1)
    b1 = B.cct_conv_workspace_bytes_for_chunk(d, B.PASS_FORWARD, 64)
    b2 = B.cct_conv_workspace_bytes_for_chunk(d, B.PASS_FORWARD, 128)
    b4 = B.cct_conv_workspace_bytes_for_chunk(d, B.PASS_FORWARD, 256)
    assert abs((b4 - b2) - 2 * (b2 - b1)) <= 4096
    assert b4 >= 256 * 729 * 2400 * 4                 # holds the whole Type-1 lowered matrix
    assert B.cct_conv_workspace_bytes(d, B.PASS_FORWARD) <= b4


def test_selector_follows_channel_ratio(B):
    """Appendix A: Type 3 wins as #input/#output channels grows, Type 1 otherwise; the pick is
    always a layout the library accepts."""
    picks = {}
    for C, O in ((16, 512), (64, 256), (256, 256), (256, 64), (512, 16), (1024, 32)):
        d = B.make_desc(128, C, 28, 28, O, 3, 1, 1, 1)
        t = B.cct_pick_lowering(d, B.PASS_FORWARD)
        assert t in (1, 2, 3, 4)
        picks[(C, O)] = t
        costs = {k: B.cct_lowering_cost(d, B.PASS_FORWARD, k) for k in (1, 2, 3, 4)}
        assert costs[t] == min(costs.values())
        # among the three materialised layouts of the paper the ratio rule holds
        best3 = min((1, 2, 3), key=lambda k: costs[k])
        if (C, O) in ((16, 512), (64, 256)):
            assert best3 == 1
        if (C, O) in ((512, 16), (1024, 32)):
            assert best3 == 3
    # the cost ratio type3/type1 falls as C/O grows (shapes with equal C/O form one group)
    groups = {}
    for C, O in picks:
        d = B.make_desc(128, C, 28, 28, O, 3, 1, 1, 1)
        groups.setdefault(C / O, []).append(B.cct_lowering_cost(d, 0, 3) / B.cct_lowering_cost(d, 0, 1))
    keys = sorted(groups)
    for lo, hi in zip(keys, keys[1:]):
        assert min(groups[lo]) >= max(groups[hi])


def test_selector_degenerate_and_strided_cases(B):
    d = B.make_desc(128, 64, 28, 28, 64, 1, 1, 0, 1)
    assert B.cct_pick_lowering(d, B.PASS_FORWARD) == 1          # k = 1: all layouts coincide
    conv1 = B.make_desc(256, 3, 227, 227, 96, 11, 4, 0, 1)
    assert B.cct_pick_lowering(conv1, B.PASS_FORWARD) in (1, 4)  # stride 4: Types 2/3 waste s, s^2 work
    assert B.cct_pick_lowering(conv1, B.PASS_BACKWARD_WEIGHTS) in (1, 4)
    assert B.cct_pick_lowering(conv1, B.PASS_BACKWARD_DATA) in (1, 4)
    for p in (B.PASS_FORWARD, B.PASS_BACKWARD_DATA, B.PASS_BACKWARD_WEIGHTS):
        for L in __import__("paper_1504_04343_amd.synth", fromlist=["x"]).caffenet(256):
            dd = B.make_desc(L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad, L.groups)
            t = B.cct_pick_lowering(dd, p)
            dd.lowering = t
            assert B.cct_conv_workspace_bytes(dd, p) > 0


def test_fused_support_rules(B):
    """Which passes the fused layout accepts (host-side rules only, no device work)."""
    def supported(desc_args, p):
        d = B.make_desc(*desc_args, lowering=B.LOWER_FUSED)
        try:
            B.cct_conv_workspace_bytes(d, p)
            return True
        except B.CctError as e:
            assert e.code == B.EUNSUPPORTED
            return False
    conv1 = (256, 3, 227, 227, 96, 11, 4, 0, 1)
    conv3 = (256, 256, 13, 13, 384, 3, 1, 1, 1)
    assert supported(conv1, B.PASS_FORWARD) and supported(conv3, B.PASS_FORWARD)
    assert supported(conv1, B.PASS_BACKWARD_DATA)          # stride 4: 16 residue classes, 96 kernels = 6 groups of 16
    assert supported(conv3, B.PASS_BACKWARD_DATA)
    few_kernels = (4, 8, 15, 15, 5, 3, 2, 1, 1)             # strided with 5 kernels: a group of 16 would be 2/3 empty
    assert not supported(few_kernels, B.PASS_BACKWARD_DATA)
    assert not supported((4, 8, 15, 15, 32, 3, 1, 3, 1), B.PASS_BACKWARD_DATA)   # stride 1 with pad > K-1
    assert supported(conv1, B.PASS_BACKWARD_WEIGHTS)       # unpadded: rows gathered inside the GEMM
    assert supported(conv3, B.PASS_BACKWARD_WEIGHTS)       # rows staged in LDS
    padded_wide = (2, 6, 14, 400, 9, 4, 3, 1, 3)            # padded, rows too wide for LDS staging
    assert not supported(padded_wide, B.PASS_BACKWARD_WEIGHTS)
    # bf16 operands: only the channel-contiguous kernel exists, so forward and backward-data of
    # layers with enough channels per group; never backward-weights, never conv1's 3 channels
    def supported_bf16(desc_args, p):
        d = B.make_desc(*desc_args, lowering=B.LOWER_FUSED, precision=B.PREC_BF16_IN_F32_ACC)
        try:
            B.cct_conv_workspace_bytes(d, p)
            return True
        except B.CctError as e:
            assert e.code == B.EUNSUPPORTED
            return False
    assert supported_bf16(conv3, B.PASS_FORWARD) and supported_bf16(conv3, B.PASS_BACKWARD_DATA)
    assert not supported_bf16(conv3, B.PASS_BACKWARD_WEIGHTS)
    assert not supported_bf16(conv1, B.PASS_FORWARD)
    assert supported_bf16(conv1, B.PASS_BACKWARD_DATA)     # 96 kernels = 6 groups of 16 on the reduction side


def test_type2_backward_data_needs_no_inverse_lifted_matrix(B):
    """At stride 1 in fp32 the Type-2 backward-data GEMM gathers dy itself: its workspace holds the
    kernel matrix and dD^ only, so it is smaller than Type 3's (which holds dR^ of K*K*O rows)."""
    conv2 = (256, 96, 27, 27, 256, 5, 1, 2, 2)
    t2 = B.cct_conv_workspace_bytes(B.make_desc(*conv2, lowering=2), B.PASS_BACKWARD_DATA)
    ld = 256 * 27 * 27
    ddhat = 96 * 5 * ld * 4                       # C*K rows of the transposed lowered gradient
    assert ddhat <= t2 < ddhat + (64 << 20)
    s2 = B.cct_conv_workspace_bytes(B.make_desc(256, 96, 27, 27, 256, 5, 2, 2, 2, lowering=2),
                                    B.PASS_BACKWARD_DATA)
    assert s2 > 0                                  # stride 2 keeps the materialised route


def test_static_forward_validates_on_the_host_before_touching_the_gpu(B):
    """cct_conv_forward_static checks arguments and sizes first: these calls return without a GPU."""
    lib = ctypes.CDLL(B.LIB_PATH)
    fn = lib.cct_conv_forward_static
    fn.argtypes = [ctypes.c_void_p] * 6
    fn.restype = ctypes.c_int
    d = B.make_desc(1, 64, 128, 128, 8, 5, 1, 2, 1, B.LOWER_TYPE1)
    assert fn(ctypes.byref(d), None, None, None, None, None) == B.EINVAL
    # 64 channels x 25 taps x 16384 positions x 4 bytes = 105 MB for one image: more than the array
    need = B.cct_conv_workspace_bytes_for_chunk(d, B.PASS_FORWARD, 1)
    assert need > B.STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(4096)      # never dereferenced: the size check comes first
    assert fn(ctypes.byref(d), fake, fake, None, fake, None) == B.ESCRATCH
    bad = B.make_desc(0, 64, 128, 128, 8, 5, 1, 2, 1)
    assert fn(ctypes.byref(bad), fake, fake, None, fake, None) == B.EINVAL
    text = open(os.path.join(ROOT, "include", "cct.h")).read()
    assert re.search(r"#define\s+CCT_STATIC_SCRATCH_BYTES\s+\(32u\s*<<\s*20\)", text)


def test_fused_backward_data_chunks_a_batch_whose_pixel_count_exceeds_31_bits(B):
    """N*H*W >= 2^31: the fused backward-data pass cannot cover the batch with one launch (its
    columns are 32-bit), so the whole-batch chunk is refused and the default workspace stands for
    a smaller chunk that the entry point then loops over."""
    d = B.make_desc(40000, 1, 256, 256, 1, 3, 1, 1, 1, B.LOWER_FUSED)
    assert d.N * d.H * d.W >= 2 ** 31
    assert B.cct_conv_workspace_bytes(d, B.PASS_BACKWARD_DATA) > 0
    assert B.cct_conv_workspace_bytes_for_chunk(d, B.PASS_BACKWARD_DATA, 1000) > 0
    with pytest.raises(B.CctError) as e:
        B.cct_conv_workspace_bytes_for_chunk(d, B.PASS_BACKWARD_DATA, d.N)
    assert e.value.code == B.EUNSUPPORTED


def test_group_count_beyond_the_grid_limit_is_unsupported_not_a_late_failure(B):
    d = B.make_desc(1, 70000, 4, 4, 70000, 3, 1, 1, 70000)
    for pass_ in (0, 1, 2):
        with pytest.raises(B.CctError) as e:
            B.cct_pick_lowering(d, pass_)
        assert e.value.code == B.EUNSUPPORTED
    d1 = B.make_desc(1, 70000, 4, 4, 70000, 1, 1, 0, 70000)       # 1x1: the shortcut must check too
    with pytest.raises(B.CctError) as e:
        B.cct_pick_lowering(d1, B.PASS_FORWARD)
    assert e.value.code == B.EUNSUPPORTED


def test_fully_connected_layers_are_planned_as_matrix_products(B):
    """K = H = W, no padding, one group, fp32, lowering AUTO or TYPE1: one output pixel per image,
    every lowering is a reshape (Sec. 2.1 with m = 1).  The optimizer reports TYPE1 and the
    workspace holds no lowered matrix and no kernel pack: the split partial products of the forward
    pass (a multiple of N*O floats), the packed dy of the backward passes (about N*O floats) and the
    split partial products of the backward-data pass (a multiple of N*C*K*K floats)."""
    N, C, K, O = 256, 256, 6, 4096
    F = C * K * K
    d = B.make_desc(N, C, K, K, O, K)
    for p in (B.PASS_FORWARD, B.PASS_BACKWARD_DATA, B.PASS_BACKWARD_WEIGHTS):
        assert B.cct_pick_lowering(d, p) == B.LOWER_TYPE1
    fwd = B.cct_conv_workspace_bytes(d, B.PASS_FORWARD)
    assert fwd % (4 * N * O) == 0 and 1 <= fwd // (4 * N * O) <= 64
    assert fwd < 4 * O * F                                        # smaller than a copy of w
    assert B.cct_conv_workspace_bytes_for_chunk(d, B.PASS_FORWARD, N) == fwd
    assert 4 * N * O <= B.cct_conv_workspace_bytes(d, B.PASS_BACKWARD_WEIGHTS) <= 2 * 4 * N * O
    bwd = B.cct_conv_workspace_bytes(d, B.PASS_BACKWARD_DATA)
    splits = bwd // (4 * N * F)
    assert 2 <= splits <= 64 and O % splits == 0
    assert 4 * N * O <= bwd - splits * 4 * N * F <= 2 * 4 * N * O
    assert bwd < 4 * O * F
    # a forced layout other than TYPE1 keeps the general path and its buffers
    for t in (B.LOWER_TYPE2, B.LOWER_TYPE3):
        dt = B.make_desc(N, C, K, K, O, K, 1, 0, 1, t)
        assert B.cct_conv_workspace_bytes(dt, B.PASS_FORWARD) > 4 * O * F
    # so do groups, the bf16 variant and a feature count that is no multiple of the K tile: their
    # workspace holds (at least) the packed kernel matrix
    for dd in (B.make_desc(N, C, K, K, O, K, 1, 0, 2), B.make_desc(N, C, K, K, O, K, 1, 0, 1, 0, 1),
               B.make_desc(N, 3, 5, 5, O, 5)):
        Fg = (dd.C // dd.groups) * dd.K * dd.K
        assert B.cct_conv_workspace_bytes(dd, B.PASS_FORWARD) >= 2 * dd.O * Fg
