"""Soft-PQ training operator (arXiv 2302.03213, Sec. 3): a torch.autograd wrapper around the C ABI.

Forward: the hard operator (arg-min encoding + table lookup, lutnn_build_table + lutnn_linear),
with the table quantised as in inference when `table_dtype` is TABLE_I8 / TABLE_I4 (Sec. 3.3: the
forward pass of training uses the quantised table).  Backward: the gradient of the soft output of
Eq. 5-6 (lutnn_softpq_backward) for the centroids, the temperature and the layer input; the weights
W are fixed, as in the paper, and only the GEMM Z = dL/dY @ W^T is left to torch.
"""
import torch

from . import binding as _b


class _SoftPQLinearFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, X, centroids, temperature, W, bias, table_dtype):
        layer = _b.build_table(centroids.detach(), W, table_dtype, bias=bias)
        Y = _b.linear(layer, X.detach())
        ctx.save_for_backward(X, centroids, temperature, W)
        ctx.has_bias = bias is not None
        ctx.table_dtype = table_dtype
        return Y

    @staticmethod
    def backward(ctx, G):
        X, centroids, temperature, W = ctx.saved_tensors
        G = G.contiguous()
        Z = G @ W.t()  # input gradient of the ordinary linear layer: a plain library GEMM
        C, K, V = centroids.shape
        layer = _b.LutLayer(centroids.detach().contiguous(), None, _b.TABLE_F32, W.shape[1])
        dP, dX, dt = _b.softpq_backward(layer, float(temperature), X.detach(), Z,
                                        need_dx=ctx.needs_input_grad[0])
        dbias = G.sum(dim=0) if ctx.has_bias and ctx.needs_input_grad[4] else None
        return dX, dP, dt.reshape(temperature.shape), None, dbias, None


class SoftPQLinear(torch.nn.Module):
    """A linear layer replaced by table lookup, in training form: learnable centroids [C, K, V] and
    temperature (Sec. 3.2), fixed weights W [D, M] and optional bias."""

    def __init__(self, centroids, W, bias=None, temperature=1.0, table_dtype=_b.TABLE_I8):
        super().__init__()
        self.centroids = torch.nn.Parameter(centroids.clone())
        self.temperature = torch.nn.Parameter(torch.tensor(float(temperature), device=centroids.device))
        self.register_buffer("W", W.clone())
        self.bias = None if bias is None else torch.nn.Parameter(bias.clone())
        self.table_dtype = table_dtype

    def forward(self, X):
        return _SoftPQLinearFn.apply(X, self.centroids, self.temperature, self.W, self.bias, self.table_dtype)
