"""GPU parity of the microscaling variant (MXFP4 weights, MXFP8 activations; datatype appendix
and W4A8 rows of the main results) against the oracle: the activation quantiser's codes and
scales bit for bit, and the forward within the tolerance of the W4A16 path (the products of
an E4M3 and an E2M1 element and their power-of-two scales are exact; what differs is fp32
against float64 accumulation and the 16-bit rounding of R)."""
import numpy as np
import pytest
import torch

import paper_2603_25385_amd as G
from glowq_inputs import UnitShape, gen_activations, gen_module_weight
from oracle import glowq_oracle as O
from oracle import mx_oracle as MX
from gpu_util import ACT_CODE, TORCH_ACT, dev_bits, stream
from util import rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-3
ULP = {"f16": 2.0 ** -11, "bf16": 2.0 ** -8}


def gpu_quantize_x(X_bits, act):
    T, d = X_bits.shape
    x = dev_bits(X_bits)
    codes = torch.full((T + 1, d), 0x55, dtype=torch.uint8, device="cuda")
    scales = torch.full((T + 1, d // 32), 0x55, dtype=torch.uint8, device="cuda")
    G.glowq_mx_quantize_activations(x.data_ptr(), T, d, ACT_CODE[act], codes.data_ptr(), scales.data_ptr(), stream())
    torch.cuda.synchronize()
    assert (codes[-1] == 0x55).all() and (scales[-1] == 0x55).all()
    return codes[:-1].cpu().numpy(), scales[:-1].cpu().numpy()


@pytest.mark.parametrize("act", ["f16", "bf16"])
def test_activation_quantiser_bit_exact(act):
    rng = np.random.default_rng(3)
    T, d = 7, 384
    X = rng.standard_normal((T, d)) * np.exp(rng.standard_normal((T, 1)) * 2)
    X[0, 0:32] = 0.0                                              # a block of zeros
    X[1, 32:64] = rng.standard_normal(32) * 3e-7                  # subnormal binary16 values
    X[2, 0:32] = 0.0
    X[2, 5] = 448.0                                               # one element, exactly the largest finite
    X[3, 64:96] = np.linspace(-1, 1, 32) * 60000                  # the top of the binary16 range
    k = np.arange(32)
    X[4, 0:32] = (2 * k + 1) / 16.0                               # ties of the E4M3 grid in several binades
    X[4, 31] = 256.0
    X[5, 0:32] = 1.0
    X[5, 7] = 1.99                                                # the block maximum just under a power of two
    X[6, 0:32] = np.linspace(440, 511, 32) / 256.0                # scaled magnitudes between 448 and 512: clamped
    X[6, 0] = 1.99
    if act == "bf16":
        X[0, 32:96] = rng.standard_normal(64) * 1e-40             # below 2^-126: the scale code clamps at 0
        X[1, 64:96] = rng.standard_normal(32) * 1e-38
        X[3, 96:128] = rng.standard_normal(32) * 1e38             # the top of the bfloat16 range
    Xb = O.f64_to_bits(X, act)
    want_c, want_s = MX.mx_quantize(O.bits_to_f64(Xb, act), "e4m3")
    got_c, got_s = gpu_quantize_x(Xb, act)
    assert np.array_equal(got_s, want_s)
    assert np.array_equal(got_c, want_c)


class MxDeviceUnit:
    def __init__(self, u, out="f32", T=None):
        self.act, self.r, self.d_in = u["act"], u["r"], u["d_in"]
        self.X = dev_bits(u["X"])
        self.T = self.X.shape[0]
        self.B = dev_bits(u["B"]) if self.r else None
        self.out = self.act if out == "act" else "f32"
        self.keep, mods, self.Y = [], [], []
        for m in u["modules"]:
            d_out = m["d_out"]
            codes = torch.from_numpy(MX.pack_fp4(m["codes"]).view(np.int32)).cuda()
            scales = torch.from_numpy(np.ascontiguousarray(m["scales"])).cuda()
            prep = torch.full((G.glowq_mx_prepared_bytes(d_out, self.d_in),), 0xEE, dtype=torch.uint8, device="cuda")
            G.glowq_mx_prepare_weights(codes.data_ptr(), scales.data_ptr(), d_out, self.d_in, prep.data_ptr(), stream())
            A = dev_bits(m["A"]) if self.r else None
            y = torch.full((self.T + 2, d_out + 8), float("nan"), dtype=TORCH_ACT[self.out], device="cuda")
            self.keep += [codes, scales, prep, A]
            self.Y.append(y)
            mods.append(G.make_module(prep.data_ptr(), A.data_ptr() if self.r else 0, y.data_ptr(), d_out, d_out + 8))
        self.desc = G.make_unit(self.X.data_ptr(), self.B.data_ptr() if self.r else 0, mods, self.T, self.d_in,
                                self.r, 0, ACT_CODE[self.act], ACT_CODE[self.out])
        self.ws_bytes = G.glowq_mx_workspace_bytes(self.desc)
        self.ws = torch.full((self.ws_bytes,), 0xFF, dtype=torch.uint8, device="cuda")

    def forward(self, restore=True):
        G.glowq_mx_group_forward(self.desc, 1 if restore else 0, self.ws.data_ptr(), self.ws_bytes, stream())
        torch.cuda.synchronize()
        outs = []
        for y, m in zip(self.Y, self.desc.modules[:len(self.Y)]):
            assert torch.isnan(y[self.T:]).all() and torch.isnan(y[:, m.d_out:]).all(), "canaries overwritten"
            outs.append(y[:self.T, :m.d_out].to(torch.float64).cpu().numpy())
        return outs


def make_unit(shape, T, r, act, seed=11):
    assert r <= min(sum(shape.d_outs), shape.d_in), "the stacked error has fewer singular values than r"
    W = [gen_module_weight(seed, 0, i, o, shape.d_in) for i, o in enumerate(shape.d_outs)]
    X = gen_activations(seed, 0, T, shape.d_in, act, True)
    return MX.build_unit_mx(W, X, r, act)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("T", [1, 3, 7, 16])
def test_forward_small(act, T):
    shape = UnitShape("g", 384, (40, 264, 96))                    # ragged 16-row blocks, three tiles of K
    u = make_unit(shape, T, 24, act)
    du = MxDeviceUnit(u)
    for restore in (True, False):
        got = du.forward(restore)
        ref = MX.mx_group_forward(u, restore)
        for g, y in zip(got, ref):
            assert rel_err(g, y) <= TOL
    # the correction matters at this tolerance (so a dropped or misplaced rank would show)
    assert max(rel_err(a, b) for a, b in zip(MX.mx_group_forward(u, True), MX.mx_group_forward(u, False))) > 10 * TOL


@pytest.mark.parametrize("r", [0, 8, 40, 128])
def test_ranks_and_16_bit_output(r):
    shape = UnitShape("s", 512, (136,))
    u = make_unit(shape, 5, r, "bf16", seed=12)
    du = MxDeviceUnit(u, out="act")
    got = du.forward(True)[0]
    ref = MX.mx_group_forward(u, True)[0]
    assert rel_err(got, ref) <= TOL + ULP["bf16"]


@pytest.mark.parametrize("T", [4, 9, 16])
def test_main_product_is_exact_on_small_integers(T):
    # weights and activations that sit on the grids with small magnitudes: every partial sum
    # is an integer multiple of 2^-10 below 2^14, so fp32 accumulation is exact (one launch at
    # four tokens, two launches with the activations in fragment order beyond)
    rng = np.random.default_rng(13)
    d = 256
    Wg = rng.choice([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], size=(16, d)) * rng.choice([-1, 1], size=(16, d))
    Xg = rng.integers(-8, 9, size=(T, d)).astype(np.float64)
    Xg[:, ::32] = 8.0                                              # every block's maximum: one scale, no clamping
    Wg[:, ::32] = 6.0
    u = MX.build_unit_mx([Wg], O.f64_to_bits(Xg, "f16"), 0, "f16")
    du = MxDeviceUnit(u)
    got = du.forward(False)[0]
    assert np.array_equal(got, Xg @ Wg.T)


def test_full_size_group():
    # the q/k/v group of the 7B shapes: d = 4096, 3 x 4096 rows, r = 64
    shape = UnitShape("qkv", 4096, (4096, 4096, 4096))
    u16 = make_unit(shape, 16, 64, "f16", seed=14)
    for T in (1, 16):
        u = dict(u16, X=u16["X"][:T], T=T)
        du = MxDeviceUnit(u)
        got = du.forward(True)
        ref = MX.mx_group_forward(u, True)
        for g, y in zip(got, ref):
            assert rel_err(g, y) <= TOL


@pytest.mark.parametrize("act,T,d_in,r", [("f16", 4, 4096, 64), ("bf16", 2, 8192, 128), ("f16", 1, 11008, 40),
                                          ("bf16", 3, 5376, 8), ("f16", 1, 12288, 16), ("bf16", 1, 128, 8)])
def test_one_launch_shapes(act, T, d_in, r):
    # up to four tokens in one launch: the most X a workgroup quantises (four pieces per
    # thread), two to four K parts of the in-launch projection, several rounds of register
    # buffers with a ragged last one (86, 42, 96 tiles on four waves), one tile for four waves;
    # and the two-launch path right beside its limit (3 x 5504 and 4 x 4224 values are too many)
    shape = UnitShape("g", d_in, (40, 136))                       # (more rows than the largest rank)
    u = make_unit(shape, T, r, act, seed=21)
    assert u["B"].shape == (r, d_in)
    du = MxDeviceUnit(u)
    for restore in (True, False):
        got = du.forward(restore)
        ref = MX.mx_group_forward(u, restore)
        for g, y in zip(got, ref):
            assert rel_err(g, y) <= TOL


@pytest.mark.parametrize("T,d_in", [(3, 5504), (4, 4224), (2, 12416)])
def test_few_tokens_beyond_the_one_launch_limits(T, d_in):
    shape = UnitShape("g", d_in, (40,))
    u = make_unit(shape, T, 24, "f16", seed=22)
    du = MxDeviceUnit(u)
    got = du.forward(True)[0]
    assert rel_err(got, MX.mx_group_forward(u, True)[0]) <= TOL


def test_one_launch_calls_in_a_row_and_graph_replays():
    # the in-launch hand-off carries a tag of the launch: 300 calls in a row through one
    # workspace, then a captured graph of three calls replayed five times with eager calls in
    # between, every result equal to the first one's bits
    shape = UnitShape("g", 4096, (136, 72))
    u = make_unit(shape, 2, 64, "f16", seed=23)
    du = MxDeviceUnit(u)
    first = du.forward(True)
    for g, y in zip(first, MX.mx_group_forward(u, True)):
        assert rel_err(g, y) <= TOL
    for it in range(300):
        G.glowq_mx_group_forward(du.desc, 1, du.ws.data_ptr(), du.ws_bytes, stream())
    assert all(np.array_equal(a, b) for a, b in zip(first, du.forward(True)))
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for it in range(3):
                G.glowq_mx_group_forward(du.desc, 1, du.ws.data_ptr(), du.ws_bytes, side.cuda_stream)
    for rep in range(5):
        for y, m in zip(du.Y, du.desc.modules[:len(du.Y)]):
            y[:du.T, :m.d_out].fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        outs = [y[:du.T, :m.d_out].to(torch.float64).cpu().numpy() for y, m in zip(du.Y, du.desc.modules[:len(du.Y)])]
        assert all(np.array_equal(a, b) for a, b in zip(first, outs))
        assert all(np.array_equal(a, b) for a, b in zip(first, du.forward(True)))


def test_calls_in_a_row_through_one_workspace():
    # nothing of a call survives in the workspace: 200 calls through one workspace, the
    # output of the last equal to the first one's bits
    shape = UnitShape("g", 512, (136, 72))
    u = make_unit(shape, 16, 40, "f16", seed=15)
    du = MxDeviceUnit(u)
    first = du.forward(True)
    for it in range(200):
        G.glowq_mx_group_forward(du.desc, 1, du.ws.data_ptr(), du.ws_bytes, stream())
    got = du.forward(True)
    assert all(np.array_equal(a, b) for a, b in zip(first, got))


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("T", [17, 48, 130, 300])
def test_tiled_path(act, T):
    # more than 16 tokens: the tiled product (token tiles of 128 with a ragged last one, row
    # tiles of 128 with ragged modules, three K tiles), restored and not
    shape = UnitShape("g", 384, (40, 264, 136))
    u = make_unit(shape, T, 24, act, seed=16)
    du = MxDeviceUnit(u)
    for restore in (True, False):
        got = du.forward(restore)
        ref = MX.mx_group_forward(u, restore)
        for g, y in zip(got, ref):
            assert rel_err(g, y) <= TOL


@pytest.mark.parametrize("r", [0, 8, 128])
def test_tiled_path_ranks_and_16_bit_output(r):
    shape = UnitShape("s", 1024, (200,))
    u = make_unit(shape, 70, r, "bf16", seed=17)
    du = MxDeviceUnit(u, out="act")
    got = du.forward(True)[0]
    ref = MX.mx_group_forward(u, True)[0]
    assert rel_err(got, ref) <= TOL + ULP["bf16"]


def test_tiled_path_exact_on_small_integers():
    rng = np.random.default_rng(18)
    d, T = 256, 150
    Wg = rng.choice([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], size=(144, d)) * rng.choice([-1, 1], size=(144, d))
    Xg = rng.integers(-8, 9, size=(T, d)).astype(np.float64)
    Xg[:, ::32] = 8.0
    Wg[:, ::32] = 6.0
    u = MX.build_unit_mx([Wg], O.f64_to_bits(Xg, "f16"), 0, "f16")
    got = MxDeviceUnit(u).forward(False)[0]
    assert np.array_equal(got, Xg @ Wg.T)


def test_full_size_prefill():
    # 512 tokens on the q/k/v group of the 3B shapes (d = 3072, rows 3072 + 1024 + 1024), r = 64
    shape = UnitShape("qkv", 3072, (3072, 1024, 1024))
    u = make_unit(shape, 512, 64, "bf16", seed=19)
    du = MxDeviceUnit(u)
    got = du.forward(True)
    ref = MX.mx_group_forward(u, True)
    for g, y in zip(got, ref):
        assert rel_err(g, y) <= TOL
