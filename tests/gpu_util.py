"""Helpers of the GPU parity tests: move a generated case to the device, call the library
through its binding, bring results back as numpy, compare with the oracle's float64."""
from __future__ import annotations

import numpy as np

ATOL, RTOL = 1e-2, 1e-2          # the stated parity bound: |err| <= 1e-2 + 1e-2 |ref|
# What a correct kernel achieves is far tighter, and the tests hold it to that as well:
#   * the output is rounded to bf16 (8 significant bits): half an ulp, at most 2^-8 relative;
#   * the softmax weights enter P.V rounded to bf16 (numerator and denominator alike): each
#     weight carries an independent relative error, uniform in +-2^-9, standard deviation
#     2^-9/sqrt(3); to first order the output moves by sum_t w_t delta_t (v_t - out), whose
#     standard deviation is (2^-9/sqrt 3) * spread with spread = sqrt(sum w_t^2 (v_t-out)^2)
#     (computed by the oracle); 8 standard deviations are allowed;
#   * fp32 accumulation: a small absolute term.
OUT_ULP = 2.0 ** -8
P_SIGMA = 2.0 ** -9 / 3 ** 0.5
TIGHT_ATOL = 5e-5
LSE_ATOL = 1e-3


def torch_mod():
    import torch
    return torch


def to_dev_bf16(bits: np.ndarray):
    torch = torch_mod()
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def to_dev_i32(a):
    torch = torch_mod()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def bf16_to_host_bits(t) -> np.ndarray:
    torch = torch_mod()
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


class DeviceCase:
    """A generated batch resident on the GPU plus a library context over its pool."""

    def __init__(self, case, **ctx_kw):
        import paper_2603_28101_amd as heddle
        torch = torch_mod()
        self.case = case
        self.pool = to_dev_bf16(case["pool"])
        self.row_off = to_dev_i32(case["row_off"])
        self.block_ids = to_dev_i32(case["block_ids"])
        self.q = to_dev_bf16(case["q"])
        self.out = torch.full(case["q"].shape, float("nan"), dtype=torch.bfloat16, device="cuda")
        self.lse = torch.full(case["q"].shape[:2], float("nan"), dtype=torch.float32, device="cuda")
        self.ctx = heddle.Context(case["n_q_heads"], case["n_kv_heads"], case["head_dim"], case["n_blocks"],
                                  kv_pool=self.pool, device=0, **ctx_kw)

    def decode(self, lens=None, k_new=None, v_new=None, want_lse=True):
        torch = torch_mod()
        c = self.case
        self.ctx.attn_decode(c["lens"] if lens is None else lens, c["row_off"], self.row_off, self.block_ids,
                             self.q, self.out, self.lse if want_lse else None, k_new, v_new)
        torch.cuda.synchronize()
        return bits_to_f64(bf16_to_host_bits(self.out)), self.lse.cpu().numpy().astype(np.float64)

    def append(self, want_lse=True):
        torch = torch_mod()
        c = self.case
        self.k_new = to_dev_bf16(c["k_new"])
        self.v_new = to_dev_bf16(c["v_new"])
        self.ctx.attn_append(c["lens"], c["cu_chunk"], c["row_off"], self.row_off, self.block_ids, self.q,
                             self.k_new, self.v_new, self.out, self.lse if want_lse else None)
        torch.cuda.synchronize()
        return bits_to_f64(bf16_to_host_bits(self.out)), self.lse.cpu().numpy().astype(np.float64)

    def pool_bits(self):
        return bf16_to_host_bits(self.pool)


# What the comparisons measured, for the table printed at the end of a GPU run (the stated bound
# is loose next to outputs of magnitude 0.01; the achieved errors are the evidence): per test the
# largest |err|, the largest |err| / rms(ref), the largest |err| as a fraction of the derived bound
# below (output rounding + weight rounding + accumulation) and the largest |lse error| over its
# comparisons.
ERROR_REPORT: dict = {}


def _note(kind, value):
    import os
    test = os.environ.get("PYTEST_CURRENT_TEST", "?").split(" ")[0].split("::", 1)[-1]
    row = ERROR_REPORT.setdefault(test, {"err": 0.0, "rel": 0.0, "tight": 0.0, "lse": 0.0})
    row[kind] = max(row[kind], float(value))


def assert_close(got, ref, what="", spread=None):
    got, ref = np.asarray(got), np.asarray(ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    if err.size:
        _note("err", err.max())
        _note("rel", err.max() / max(float(np.sqrt(np.mean(ref * ref))), 1e-30))
    bound = ATOL + RTOL * np.abs(ref)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert (err <= bound).all(), f"{what}: |err|={err[worst]:.3e} at {worst}, ref={ref[worst]:.4e}"
    if spread is not None:
        tb = TIGHT_ATOL + 1.01 * OUT_ULP * np.abs(ref) + 8 * P_SIGMA * np.asarray(spread)
        if err.size:
            _note("tight", (err / tb).max())
        worst = np.unravel_index(np.argmax(err - tb), err.shape)
        assert (err <= tb).all(), (f"{what} (derived bound): |err|={err[worst]:.3e} > {tb[worst]:.3e} at {worst}, "
                                   f"ref={ref[worst]:.4e}")


def assert_lse_close(got, ref, what=""):
    err = np.abs(np.asarray(got) - np.asarray(ref))
    if err.size and np.isfinite(err).all():
        _note("lse", err.max())
    assert np.isfinite(got).all() and err.max() <= LSE_ATOL, f"{what}: max |lse err| = {err.max():.3e}"
