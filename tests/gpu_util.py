"""Helpers for the GPU parity tests: move a synthetic problem to the device, call the
C-ABI through the binding, and compare with the fp64 oracle under the stated tolerance."""
import numpy as np
import torch

import oracle
from paper_2505_01068_amd import binding as B

# Tolerances of the parity bar: per tensor, max|gpu - oracle| <= tol * max|oracle|.
TOL = {"fp32": 1e-5, "bf16": 2e-2}
W_NAMES = ("wq", "wk", "wv", "wo")
B_NAMES = ("bq", "bk", "bv", "bo")


def tdtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_dev(a, dtype):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype == torch.float32:
        t = t.to(tdtype(dtype))
    return t.cuda()


def rel_err(gpu, ref, scale=None):
    gpu = gpu.detach().float().cpu().numpy().astype(np.float64) if isinstance(gpu, torch.Tensor) else np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), "non-finite values in GPU result"
    scale = np.max(np.abs(ref)) if scale is None else scale
    return float(np.max(np.abs(gpu - ref)) / max(scale, 1e-30))


def assert_close(gpu, ref, tol, what="", scale=None):
    e = rel_err(gpu, ref, scale)
    assert e <= tol, f"{what}: relative error {e:.3e} > {tol:.1e}"
    return e


def grad_scale(name, ref, floor, dk_sum_abs=None):
    """Scale an error of gradient `name` is measured against: max|oracle|, but never below `floor` (one rounding
    unit of the largest gradient of the call: a gradient that is identically zero in exact arithmetic has no
    scale of its own).  The key bias gradient (dbk / dbk of a layer) is identically 0 -- every row of dS sums
    to 0 -- so its max|oracle| is rounding noise; its error is measured against the magnitude of what is summed,
    max over columns of sum |dK| (`dk_sum_abs`)."""
    scale = max(float(np.max(np.abs(ref))), floor)
    if name in ("dbk", "bk") and dk_sum_abs is not None:
        scale = max(float(dk_sum_abs), floor)
    return scale


class Problem:
    """One IM-attention problem resident on the GPU."""

    def __init__(self, g, live_mask):
        self.g, self.lm, self.dtype = g, int(live_mask), g["dtype"]
        x = g["x"]
        self.shape = B.make_shape(x.shape[0], g["seg_len"], x.shape[2], g["n_heads"], live_mask, g["scale"], self.dtype)
        self.t = {n: to_dev(g.get(n), self.dtype) for n in ("x", "dy") + W_NAMES + B_NAMES}
        self.t["valid_len"] = to_dev(g.get("valid_len"), self.dtype)
        self.t["key_pad"] = to_dev(g.get("key_pad"), self.dtype)
        sb, wb = B.im_attention_sizes(self.shape)
        self.saved = torch.empty(sb, dtype=torch.uint8, device="cuda")
        self.ws = torch.empty(max(wb, 1), dtype=torch.uint8, device="cuda")

    def fwd(self, save=True):
        t = self.t
        y = torch.empty_like(t["x"])
        B.im_attention_fwd(self.shape, t["x"], t["wq"], t["wk"], t["wv"], t["wo"], t["bq"], t["bk"], t["bv"], t["bo"],
                           t["valid_len"], t["key_pad"], y=y, saved=self.saved if save else None, workspace=self.ws)
        return y

    def bwd(self):
        t = self.t
        d = t["x"].shape[-1]
        f32 = dict(dtype=torch.float32, device="cuda")
        out = {"dx": torch.empty_like(t["x"])}
        for n in W_NAMES:
            out["d" + n] = torch.empty(d, d, **f32)
        for n in B_NAMES:
            out["d" + n] = torch.empty(d, **f32) if t[n] is not None else None
        B.im_attention_bwd(self.shape, t["x"], t["wq"], t["wk"], t["wv"], t["wo"], self.saved, t["dy"], out["dx"],
                           out["dwq"], out["dwk"], out["dwv"], out["dwo"], out["dbq"], out["dbk"], out["dbv"],
                           out["dbo"], t["valid_len"], t["key_pad"], workspace=self.ws)
        return out

    def oracle_fwd(self, cache=False):
        g = self.g
        return oracle.forward(g["x"], g["wq"], g["wk"], g["wv"], g["wo"], g["seg_len"], self.lm, g["n_heads"],
                              g["scale"], bq=g.get("bq"), bk=g.get("bk"), bv=g.get("bv"), bo=g.get("bo"),
                              valid_len=g.get("valid_len"), key_pad=g.get("key_pad"), return_cache=cache)

    def check(self, backward=True, tol=None, what=""):
        tol = TOL[self.dtype] if tol is None else tol
        y = self.fwd(save=True)
        torch.cuda.synchronize()
        if backward:
            y_ref, cache = self.oracle_fwd(cache=True)
        else:
            y_ref = self.oracle_fwd()
        errs = {"y": assert_close(y, y_ref, tol, what + " y")}
        if backward:
            grads = self.bwd()
            torch.cuda.synchronize()
            ref = oracle.backward(cache, self.g["dy"])
            # A gradient that is identically zero in exact arithmetic (e.g. dQ, dK when a row has a
            # single key, so its softmax is constant) has no scale of its own: errors are then
            # measured against one rounding unit of the largest gradient of the same call.
            ulp = 2.0 ** -8 if self.dtype == "bf16" else 2.0 ** -23
            floor = ulp * max(float(np.max(np.abs(ref[n]))) for n in grads if grads[n] is not None)
            for n, v in grads.items():
                if v is None:
                    continue
                scale = grad_scale(n, ref[n], floor, np.max(np.sum(np.abs(ref["dk"]), axis=(0, 1))))
                errs[n] = assert_close(v, ref[n], tol, what + " " + n, scale)
        return errs


class PackedProblem(Problem):
    """The same problem with packed rows: sample b keeps the first lengths[b, s] rows of segment s and the
    tensors hold no padding rows.  The oracle sees the padded problem with valid_len = lengths and dy = 0
    beyond them, which has the same values on the kept rows and the same weight gradients."""

    def __init__(self, g, live_mask, lengths):
        from paper_2505_01068_amd import synth
        self.g, self.lm, self.dtype = g, int(live_mask), g["dtype"]
        self.lengths = np.asarray(lengths, dtype=np.int32)
        x = g["x"]
        seg = g["seg_len"]
        cu = synth.row_offsets(self.lengths)
        self.cu = torch.from_numpy(cu).cuda()
        self.shape = B.make_shape(x.shape[0], seg, x.shape[2], g["n_heads"], live_mask, g["scale"], self.dtype,
                                  cu_rows=self.cu, total_rows=int(cu[-1]))
        self.t = {n: to_dev(g.get(n), self.dtype) for n in W_NAMES + B_NAMES}
        self.t["x"] = to_dev(synth.pack_rows(x, self.lengths, seg), self.dtype)
        self.t["dy"] = to_dev(synth.pack_rows(g["dy"], self.lengths, seg), self.dtype)
        self.t["valid_len"] = None
        kp = g.get("key_pad")   # [B, T_m] -> [total_rows]
        self.t["key_pad"] = None if kp is None else to_dev(synth.pack_rows(kp, self.lengths, seg), self.dtype)
        sb, wb = B.im_attention_sizes(self.shape)
        self.saved = torch.empty(sb, dtype=torch.uint8, device="cuda")
        self.ws = torch.empty(max(wb, 1), dtype=torch.uint8, device="cuda")

    def check(self, backward=True, tol=None, what=""):
        from paper_2505_01068_amd import synth
        tol = TOL[self.dtype] if tol is None else tol
        g, seg = self.g, self.g["seg_len"]
        pack = lambda a: synth.pack_rows(a, self.lengths, seg)
        y = self.fwd(save=True)
        torch.cuda.synchronize()
        y_ref, cache = oracle.forward(g["x"], g["wq"], g["wk"], g["wv"], g["wo"], seg, self.lm, g["n_heads"], g["scale"],
                                      bq=g.get("bq"), bk=g.get("bk"), bv=g.get("bv"), bo=g.get("bo"),
                                      valid_len=self.lengths, key_pad=g.get("key_pad"), return_cache=True)
        errs = {"y": assert_close(y, pack(y_ref), tol, what + " y")}
        if backward:
            grads = self.bwd()
            torch.cuda.synchronize()
            dy = synth.unpack_rows(pack(g["dy"]), self.lengths, seg)   # zero beyond the lengths
            ref = oracle.backward(cache, dy)
            ulp = 2.0 ** -8 if self.dtype == "bf16" else 2.0 ** -23
            floor = ulp * max(float(np.max(np.abs(ref[n]))) for n in grads if grads[n] is not None)
            for n, v in grads.items():
                if v is None:
                    continue
                r = pack(ref[n]) if n == "dx" else ref[n]
                scale = grad_scale(n, r, floor, np.max(np.sum(np.abs(ref["dk"]), axis=(0, 1))))
                errs[n] = assert_close(v, r, tol, what + " " + n, scale)
        return errs
