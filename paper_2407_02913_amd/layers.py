"""One convolution layer set up through the C ABI the way ``bench.py`` runs it.

Argument marshalling and buffer bookkeeping only: the plan (algorithm and path chosen by the
library unless given), the library's own abs-max calibration on the GPU, the filter transform
and the device buffers.  ``bench.py`` and the GPU parity tests both build their layers here,
so what is timed is what is checked.
"""
from __future__ import annotations

import math

import numpy as np

from . import binding


def output_scale(cin: int, kernel: int = 3, x_scale: float = 0.02) -> float:
    """Activation scale of an int8 output tensor for the synthetic distributions of ``synth``:
    four standard deviations of a sum of kernel^2 * Cin products (activations half-normal with
    sigma 30, weights normal with sigma 20, mean filter scale 0.0125) map to 127.  A property
    of the synthetic inputs, not of the method: the scale is an input of library and oracle
    alike."""
    return float(4.0 * x_scale * 0.0125 * 30.0 * 20.0 * math.sqrt(kernel * kernel * cin) / 127.0)


class Layer:
    """A ready-to-run layer: ``run(x_dev, y_dev, workspace)`` queues one convolution.

    ``shape`` is a ``synth.LayerShape``; ``data`` the dict ``synth.make_layer`` returns for it
    (weights, filter scales, calibration activations).  ``out`` is "f32" or "i8".
    """

    def __init__(self, shape, data, out="f32", alg="auto", path="auto", batch=None):
        import torch

        n = shape.N if batch is None else batch
        self.shape, self.N, self.out = shape, n, out
        self.x_scale = float(data["x_scale"])
        self.plan = binding.Plan(n, shape.Cin, shape.Cout, shape.H, shape.W, alg=alg, mode="requant",
                                 out=out, path=path, per_channel_wscale=shape.per_channel_wscale)
        self.alg, self.path, self.P, self.tiles = self.plan.alg, self.plan.path, self.plan.P, self.plan.tiles
        w_dev = torch.from_numpy(data["w"]).cuda()
        xc_dev = torch.from_numpy(data["x_calib"]).cuda()
        # scales from the library's abs-max calibration (a staged plan of the calibration batch)
        calib = binding.Plan(xc_dev.shape[0], shape.Cin, shape.Cout, shape.H, shape.W, alg=self.alg,
                             mode="requant", path="staged", per_channel_wscale=shape.per_channel_wscale)
        scratch = binding.device_buffer(calib.workspace_bytes)
        self.sx = calib.calibrate_act_scales(xc_dev, scratch)
        self.sw = calib.calibrate_filter_scales(w_dev, scratch)
        calib.close()
        self.plan.set_point_scales(self.sx, self.sw)
        self.y_scale = None
        if out == "i8":
            self.y_scale = output_scale(shape.Cin, self.plan.kernel_size, self.x_scale)
            self.plan.set_output_scale(self.y_scale)
        self.filter_buf = binding.device_buffer(self.plan.filter_bytes)
        self.plan.transform_filter(w_dev, data["w_scale"], self.filter_buf)
        self.workspace_bytes = self.plan.workspace_bytes

    def new_output(self):
        import torch

        s = self.shape
        return torch.empty((self.N, s.Cout, s.H, s.W), device="cuda",
                           dtype=torch.int8 if self.out == "i8" else torch.float32)

    def run(self, x_dev, y_dev, workspace, stream=None, stages=binding.STAGE_ALL):
        self.plan.conv2d_stages(x_dev, self.x_scale, y_dev, workspace, stages, stream=stream)

    def kernels(self):
        """The kernels one call launches: name -> (stage mask, algorithmic bytes, int8 MFMA
        operations or 0).  Algorithmic bytes: every tensor a kernel must read or write, once --
        x = N Cin H W, V = P T Cin, U = P Cout Cin, M = P T Cout times the bytes of a sum (three
        while Cin, rounded up to 64, times 127^2 stays below 2^23, as the library stores them; else
        four), y = N Cout H W times the output element size; operations of the products:
        2 P T Cin Cout."""
        s, p, t = self.shape, self.P, self.tiles
        x = self.N * s.Cin * s.H * s.W
        mb = 3 if -(-s.Cin // 64) * 64 * 127 * 127 < 2 ** 23 else 4
        v, u, m = p * t * s.Cin, p * s.Cout * s.Cin, mb * p * t * s.Cout
        y = self.N * s.Cout * s.H * s.W * (1 if self.out == "i8" else 4)
        ops = 2 * p * t * s.Cin * s.Cout
        if self.path == "single":
            return {"single_conv": (binding.STAGE_ALL, x + u + y, ops)}
        if self.path == "fused":
            return {"input_transform": (binding.STAGE_INPUT, x + v, 0),
                    "fused_product_output": (binding.STAGE_PRODUCT | binding.STAGE_OUTPUT, v + u + y, ops)}
        return {"input_transform": (binding.STAGE_INPUT, x + v, 0),
                "product_gemm": (binding.STAGE_PRODUCT, v + u + m, ops),
                "output_transform": (binding.STAGE_OUTPUT, m + y, 0)}

    def close(self):
        self.plan.close()


def np_conv(layer: Layer, x: np.ndarray) -> np.ndarray:
    """One call on host data: numpy in, numpy out (synchronizes)."""
    import torch

    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    y = layer.new_output()
    ws = binding.device_buffer(layer.workspace_bytes)
    layer.run(xd, y, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy()
