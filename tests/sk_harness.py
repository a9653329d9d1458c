"""Shared plumbing for the GPU parity tests: seeded inputs -> device buffers ->
sk_problem list, outputs back as exact values, oracle results beside them.

Inputs are drawn in fp32 (workloads), rounded to the operand type by the
oracle's rounding helper, and the *bit patterns* are shipped to the GPU, so both
sides consume exactly the same operand values.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_1901_10008_amd as sk
import workloads
from oracle import compare, reference as R, rounding as Q

_NAN_BITS = {"f32": 0x7FC00000, "bf16": 0x7FC0, "f16": 0x7E00}
_NP_BITS = {"f32": np.uint32, "bf16": np.uint16, "f16": np.uint16}
_T_BITS = {"f32": torch.int32, "bf16": torch.int16, "f16": torch.int16}
_T_REAL = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
ES = {"f32": 4, "bf16": 2, "f16": 2}


def _to_dev_bits(bits: np.ndarray, dtype: str, device, byte_offset: int = 0, ld: int | None = None):
    """Upload a 2-D bit-pattern array; optionally at a byte offset inside a larger
    buffer (to misalign it) and with a row stride `ld` > row length."""
    bits2 = bits.reshape(bits.shape[0], -1) if bits.ndim > 1 else bits.reshape(1, -1)
    rows, cols = bits2.shape
    ld = cols if ld is None else ld
    es = ES[dtype]
    assert byte_offset % es == 0
    total = rows * ld + byte_offset // es + 64
    host = np.zeros(total, dtype=_NP_BITS[dtype])
    view = host[byte_offset // es: byte_offset // es + rows * ld].reshape(rows, ld)
    view[:, :cols] = bits2
    signed = host.view(np.int16 if es == 2 else np.int32)
    buf = torch.from_numpy(signed.copy()).to(device)
    return buf, buf.data_ptr() + byte_offset


class Batch:
    """Device-resident operands and outputs for a list of operator descriptions."""

    def __init__(self, specs, seed=0, device="cuda", host_draw=True, a_off=0, b_off=0, c_off=0,
                 pad_lda=0, pad_ldb=0, pad_ldc=0, shared_inputs=None):
        self.specs = list(specs)
        self.device = device
        self.bufs = []
        self.problems = []
        self.a_val, self.b_val = [], []       # exact operand values as fp32 numpy (host_draw only)
        self.dA, self.dB = [], []             # device tensors (device draw)
        self.c_bufs, self.c_meta = [], []
        self._ref = {}
        for i, s in enumerate(self.specs):
            es = ES[s.dtype]
            if host_draw:
                A32, B32 = workloads.draw_host(s, seed, i)
                a_bits, a_val = Q.round_to(s.dtype, A32)
                b_bits, b_val = Q.round_to(s.dtype, B32)
                self.a_val.append(a_val)
                self.b_val.append(b_val)
                if s.op == "gemm":
                    lda = s.K + pad_lda
                    ldb = s.K + pad_ldb
                    bufA, pA = _to_dev_bits(a_bits, s.dtype, device, a_off, lda)
                    bufB, pB = _to_dev_bits(b_bits, s.dtype, device, b_off, ldb)
                else:
                    lda = ldb = 0
                    bufA, pA = _to_dev_bits(a_bits.reshape(1, -1), s.dtype, device, a_off)
                    bufB, pB = _to_dev_bits(b_bits.reshape(1, -1), s.dtype, device, b_off)
            else:
                A32, B32 = workloads.draw_device(s, seed, i, device)
                bufA = A32.to(_T_REAL[s.dtype]).contiguous()
                bufB = B32.to(_T_REAL[s.dtype]).contiguous()
                del A32, B32
                pA, pB = bufA.data_ptr(), bufB.data_ptr()
                lda = ldb = 0
                self.dA.append(bufA)
                self.dB.append(bufB)
            cshape = s.c_shape if hasattr(s, "c_shape") else None
            rows = int(np.prod(cshape[:-1]))
            cols = int(cshape[-1])
            ldc = cols + (pad_ldc if s.op == "gemm" else 0)
            nelem = rows * ldc + c_off // es + 64
            cbuf = torch.full((nelem,), 0, dtype=_T_BITS[s.dtype], device=device)
            cbuf.fill_(_NAN_BITS[s.dtype])
            pC = cbuf.data_ptr() + c_off
            self.bufs += [bufA, bufB]
            self.c_bufs.append(cbuf)
            self.c_meta.append((rows, cols, ldc, c_off // es))
            if s.op == "gemm":
                self.problems.append(sk.make_problem(s, pA, pB, pC, lda if (pad_lda or a_off) else 0,
                                                     ldb if (pad_ldb or b_off) else 0, ldc if pad_ldc else 0))
            else:
                self.problems.append(sk.make_problem(s, pA, pB, pC))

    def plan(self, **prm):
        params = sk.sk_plan_params_default(**prm)
        return sk.sk_plan_create(self.problems, params, keepalive=self)

    def reset_outputs(self):
        for s, cbuf in zip(self.specs, self.c_bufs):
            cbuf.fill_(_NAN_BITS[s.dtype])

    def output_bits(self, i) -> np.ndarray:
        """Bit patterns of operator i's output, [rows, cols]; also checks that nothing
        outside the [rows, cols] window of the buffer was touched."""
        s = self.specs[i]
        rows, cols, ldc, off = self.c_meta[i]
        host = self.c_bufs[i].cpu().numpy().view(_NP_BITS[s.dtype])
        win = host[off: off + rows * ldc].reshape(rows, ldc)
        nan = _NAN_BITS[s.dtype]
        assert np.all(host[:off] == nan) and np.all(host[off + rows * ldc:] == nan), "write outside the output"
        if ldc > cols:
            assert np.all(win[:, cols:] == nan), "write into the row padding of the output"
        return win[:, :cols].copy()

    def output(self, i) -> np.ndarray:
        s = self.specs[i]
        return Q.bits_to_f32(s.dtype, self.output_bits(i)).astype(np.float64)

    def all_output_bits(self):
        return [self.output_bits(i) for i in range(len(self.specs))]

    def reference(self, i):
        """(ref, mag) fp64 from the oracle, shaped [rows, cols]."""
        if i not in self._ref:
            s = self.specs[i]
            if s.op == "gemm":
                self._ref[i] = R.gemm(self.a_val[i], self.b_val[i], want_mag=True)
            elif s.op == "conv_nchw":
                Y, S = R.conv2d_nchw(self.a_val[i], self.b_val[i], s.pad_h, s.pad_w, want_mag=True, stride=s.stride)
                self._ref[i] = (Y.reshape(-1, Y.shape[-1]), S.reshape(-1, Y.shape[-1]))
            else:
                Y, S = R.conv2d_nhwc(self.a_val[i], self.b_val[i], s.pad_h, s.pad_w, want_mag=True, stride=s.stride)
                self._ref[i] = (Y.reshape(-1, s.Cout), S.reshape(-1, s.Cout))
        return self._ref[i]


def kg_of(s):
    return s.K if s.op == "gemm" else s.R * s.S * s.Cin


def check_against_oracle(batch: Batch, label="", only=None):
    """Every operator (or those with an index in `only`): no NaN left (everything was written),
    gate error within the dtype tolerance, and the order-free fp32-accumulation bound holds."""
    worst = {}
    for i, s in enumerate(batch.specs):
        if only is not None and i not in only:
            continue
        got = batch.output(i)
        assert not np.isnan(got).any(), f"{label} operator {i} {s}: output not fully written"
        ref, mag = batch.reference(i)
        e = compare.errors(got, ref, mag)
        tol = compare.TOL[s.dtype]
        assert e["gate"] <= tol, f"{label} operator {i} {s}: {e}"
        bound = compare.order_free_bound(ref, mag, kg_of(s), s.dtype)
        viol = np.abs(got - ref) > bound
        assert not viol.any(), f"{label} operator {i} {s}: {int(viol.sum())} outputs beyond the rounding bound; {e}"
        worst[s.dtype] = max(worst.get(s.dtype, 0.0), e["gate"])
    return worst


def stream_handle():
    return torch.cuda.current_stream().cuda_stream
