"""Glue for the GPU parity tests: moves an oracle-style unit (numpy bit patterns)
into device memory with torch, prepares the weights, and calls the C ABI through
the Python binding.  Torch is used for memory and streams only."""
from __future__ import annotations

import numpy as np
import torch

import paper_2603_25385_amd as G

ACT_CODE = {"f16": G.GLOWQ_F16, "bf16": G.GLOWQ_BF16, "f32": G.GLOWQ_F32}
TORCH_ACT = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}
GUARD_ROWS = 2


def dev_bits(bits: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> int16 device tensor (same bytes)."""
    return torch.from_numpy(np.ascontiguousarray(bits, np.uint16).view(np.int16)).cuda()


def dev_words(words: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(words, np.uint32).view(np.int32)).cuda()


def stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class DeviceModule:
    def __init__(self, module: dict, d_in: int, Gs: int, r: int = 0):
        self.d_out = int(module["wq"].shape[0])
        self.wq = dev_words(module["wq"]) if not torch.is_tensor(module["wq"]) else module["wq"]
        self.scales = _as_dev16(module["scales"])
        self.zeros = _as_dev16(module["zeros"])
        nbytes = G.glowq_prepared_bytes(self.d_out, d_in, Gs)
        self.prepared = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        G.glowq_prepare_weights(self.wq.data_ptr(), self.scales.data_ptr(), self.zeros.data_ptr(),
                                self.d_out, d_in, Gs, self.prepared.data_ptr(), stream())
        A = module.get("A")
        self.A = None if A is None or A.shape[1] == 0 else _as_dev16(A)
        assert self.A is None or r == 0 or tuple(self.A.shape) == (self.d_out, r), "A_i must be [d_out][r]"


def _as_dev16(x):
    if torch.is_tensor(x):
        return x.cuda().contiguous()
    return dev_bits(x)


class DeviceUnit:
    """Device copy of one unit plus its output buffers."""

    def __init__(self, unit: dict, out: str = "f32", ldy_pad: int = 0):
        self.act, self.Gs, self.r = unit["act"], unit["G"], unit["r"]
        self.d_in = int(unit["d_in"])
        self.X = _as_dev16(unit["X"])
        self.T = int(self.X.shape[0])
        self.B = None if self.r == 0 else _as_dev16(unit["B"])
        assert self.B is None or tuple(self.B.shape) == (self.r, self.d_in), "B must be [r][d_in]"
        self.modules = [DeviceModule(m, self.d_in, self.Gs, self.r) for m in unit["modules"]]
        self.out = self.act if out == "act" else out
        # every output buffer carries canaries: `ldy_pad` columns to the right of the rows
        # and GUARD_ROWS rows below them, all NaN, which no call may touch
        self.Ybuf = [torch.full((self.T + GUARD_ROWS, m.d_out + ldy_pad), float("nan"),
                                dtype=TORCH_ACT[self.out], device="cuda") for m in self.modules]
        self.Y = [b[:self.T] for b in self.Ybuf]
        self.desc = self.describe()

    def describe(self, T=None, r=None, X=None):
        mods = [G.make_module(m.prepared.data_ptr(), 0 if m.A is None else m.A.data_ptr(),
                              y.data_ptr(), m.d_out, y.shape[1])
                for m, y in zip(self.modules, self.Y)]
        return G.make_unit((X if X is not None else self.X).data_ptr(),
                           0 if self.B is None else self.B.data_ptr(), mods,
                           self.T if T is None else T, self.d_in, self.r if r is None else r,
                           self.Gs, ACT_CODE[self.act], ACT_CODE[self.out])

    def outputs(self, T=None):
        """Outputs of the last call (rows of the first T tokens if the call was made for
        fewer tokens than the buffers hold); asserts that the canaries are intact."""
        torch.cuda.synchronize()
        T = self.T if T is None else T
        for b, m in zip(self.Ybuf, self.modules):
            assert torch.isnan(b[:, m.d_out:]).all(), "padding columns of Y were written"
            assert torch.isnan(b[T:]).all(), "rows past T of Y were written"
        return [y[:T, :m.d_out].to(torch.float64).cpu().numpy()
                for y, m in zip(self.Y, self.modules)]

    def clear(self):
        for b in self.Ybuf:
            b.fill_(float("nan"))


class Workspace:
    def __init__(self, descs):
        self.bytes = G.glowq_workspace_bytes(descs)
        self.buf = torch.empty(max(self.bytes, 256), dtype=torch.uint8, device="cuda")
        G.glowq_workspace_init(self.buf.data_ptr(), self.buf.numel(), stream())

        self.offsets, self.tblocks, self.tokens, off = [], [], [], 0
        for d in descs:
            self.offsets.append(off)
            self.tblocks.append((d.T + 15) // 16)
            self.tokens.append(d.T)
            off += G.glowq_workspace_bytes([d])

    @property
    def ptr(self):
        return self.buf.data_ptr()

    def control_words(self):
        """Control words of every unit slice as 32-bit words: launch tag (2 words),
        token blocks done, status, padding to 16 words, then one arrival counter per
        16-token block (decode) or launch-tag word per token tile (prefill)."""
        torch.cuda.synchronize()
        w = self.buf.view(torch.int32).cpu().numpy()
        return [w[o // 4:o // 4 + 16 + nb].tolist() for o, nb in zip(self.offsets, self.tblocks)]

    def assert_idle(self):
        # words 2, 3: the decode handshake's block count (back to zero) and the status word
        # (nonzero: a bounded wait expired); the per-block words behind them hold counters
        # (decode: back to zero) or launch tags (prefill tiles)
        for cw, T in zip(self.control_words(), self.tokens):
            assert cw[2] == 0 and cw[3] == 0, cw
            if T <= 32:
                assert not any(cw[2:]), cw
            else:
                # tiled path: word 1 of each token tile's flag words counts the projection's
                # K parts and is back at zero when the launch has ended
                mb = 4 if T <= 64 else 8
                for i in range(16 + 1, len(cw), mb):
                    assert cw[i] == 0, (i, cw)


def run_group(unit: dict, restore: bool = True, out: str = "f32", ldy_pad: int = 0):
    du = DeviceUnit(unit, out, ldy_pad)
    ws = Workspace([du.desc])
    G.glowq_group_forward(du.desc, restore, ws.ptr, ws.bytes, stream())
    ys = du.outputs()
    ws.assert_idle()
    return ys, du, ws
