"""Helpers for the GPU parity tests: move seeded bf16-grid NumPy data to the device and back."""
import numpy as np
import torch

from oracle import stage_oracle as O

TOL_OUT, TOL_GRAD = 2e-2, 3e-2   # normalised max error: outputs, gradients


def dev_bf16(x: np.ndarray) -> torch.Tensor:
    """fp32 array whose values lie on the bf16 grid -> bf16 device tensor (exact)."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).cuda()


def host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def empty_bf16(*shape) -> torch.Tensor:
    return torch.empty(*shape, dtype=torch.bfloat16, device="cuda")


def scratch(nbytes: int) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def nmax_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref|: the normalised-max error the tolerances are stated in."""
    denom = float(np.max(np.abs(ref))) if ref.size else 0.0
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(got - ref))) / max(denom, 1e-30)


class GpuStage:
    """Allocate buffers with PyTorch, run the library's forward and backward."""

    def __init__(self, B, layers):
        self.B, self.layers = B, layers
        self.h = B.mllm_stage_create(layers)
        self.infos = [B.mllm_stage_param_info(self.h, i) for i in range(B.mllm_stage_param_count(self.h))]

    def close(self):
        self.B.mllm_stage_destroy(self.h)

    def run(self, wl, accumulate=0, dparams=None, want_dx=True):
        B = self.B
        params = [dev_bf16(p) for p in wl.params]
        x_img = dev_bf16(wl.x_img) if wl.x_img is not None else None
        x_seq = dev_bf16(wl.x_seq) if wl.x_seq is not None else None
        dy = dev_bf16(wl.dy)
        sb, wb = B.mllm_stage_sizes(self.h, wl.batch)
        saved, ws = scratch(sb), scratch(wb)
        y = torch.zeros(wl.dy.shape, dtype=torch.bfloat16, device="cuda")
        B.mllm_stage_fwd(self.h, wl.batch, params, x_img, x_seq, y, saved, ws)
        if dparams is None:
            dparams = [torch.full((r, c), float("nan") if not accumulate else 0.0, dtype=torch.float32, device="cuda")
                       for _, _, r, c in self.infos]
        dx_img = torch.zeros_like(x_img) if (x_img is not None and want_dx) else None
        dx_seq = torch.zeros_like(x_seq) if (x_seq is not None and want_dx) else None
        B.mllm_stage_bwd(self.h, wl.batch, params, dy, saved, dx_img, dx_seq, dparams, accumulate, ws)
        torch.cuda.synchronize()
        return y, dx_img, dx_seq, dparams


def oracle_run(wl):
    y, caches = O.stage_fwd(wl.layers, wl.params, wl.batch, wl.x_img, wl.x_seq)
    dx_img, dx_seq, dparams = O.stage_bwd(wl.layers, wl.params, wl.batch, caches, wl.dy.astype(np.float64))
    return y, dx_img, dx_seq, dparams


def compare(stage, wl, got, ref):
    y, dx_img, dx_seq, dparams = got
    y_r, dxi_r, dxs_r, dp_r = ref
    errs = {"y": nmax_err(host_f64(y), y_r)}
    assert errs["y"] <= TOL_OUT, errs
    if dxi_r is not None:
        errs["dx_img"] = nmax_err(host_f64(dx_img), dxi_r)
    if dxs_r is not None:
        errs["dx_seq"] = nmax_err(host_f64(dx_seq), dxs_r)
    for (name, layer, _, _), g, r in zip(stage.infos, dparams, dp_r):
        errs["L%d.%s" % (layer, name)] = nmax_err(host_f64(g), r)
    bad = {k: v for k, v in errs.items() if k != "y" and not v <= TOL_GRAD}
    assert not bad, bad
    return errs
