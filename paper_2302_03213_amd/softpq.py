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


class _SoftPQConv2dFn(torch.autograd.Function):
    """The same operator for a convolution (Sec. 4: a convolution is the linear operator on the rows
    of its im2col matrix).  Forward reads the NCHW batch directly (lutnn_conv2d); backward
    materialises the rows with torch's unfold - training can afford the matrix the inference path
    avoids - and folds the row gradients back onto the image."""

    @staticmethod
    def forward(ctx, inp, centroids, temperature, W, bias, table_dtype, kernel, stride, pad):
        layer = _b.build_table(centroids.detach(), W, table_dtype, bias=bias)
        B, _, H, Wd = inp.shape
        Y = _b.conv2d(layer, inp.detach().contiguous(), kernel, stride, pad)  # [B*Ho*Wo, M]
        geom = _b.conv_geom(inp, kernel, stride, pad)
        Ho = (H + 2 * geom.pad_h - geom.kh) // geom.stride_h + 1
        Wo = (Wd + 2 * geom.pad_w - geom.kw) // geom.stride_w + 1
        ctx.save_for_backward(inp, centroids, temperature, W)
        ctx.has_bias = bias is not None
        ctx.conv = (kernel, stride, pad, Ho, Wo)
        return Y.view(B, Ho, Wo, -1).permute(0, 3, 1, 2)  # NCHW view of the row-major output

    @staticmethod
    def backward(ctx, G):
        inp, centroids, temperature, W = ctx.saved_tensors
        kernel, stride, pad, Ho, Wo = ctx.conv
        B, Cin, H, Wd = inp.shape
        M = W.shape[1]
        G2 = G.permute(0, 2, 3, 1).reshape(-1, M).contiguous()  # rows (b, ho, wo)
        cols = torch.nn.functional.unfold(inp.detach(), kernel, padding=pad, stride=stride)  # [B, D, Ho*Wo]
        X = cols.permute(0, 2, 1).reshape(-1, cols.shape[1]).contiguous()
        Z = G2 @ W.t()
        layer = _b.LutLayer(centroids.detach().contiguous(), None, _b.TABLE_F32, M)
        need_dx = ctx.needs_input_grad[0]
        dP, dX, dt = _b.softpq_backward(layer, float(temperature), X, Z, need_dx=need_dx)
        dinp = None
        if need_dx:
            dcols = dX.view(B, Ho * Wo, -1).permute(0, 2, 1)
            dinp = torch.nn.functional.fold(dcols, (H, Wd), kernel, padding=pad, stride=stride)
        dbias = G2.sum(dim=0) if ctx.has_bias and ctx.needs_input_grad[4] else None
        return dinp, dP, dt.reshape(temperature.shape), None, dbias, None, None, None, None


class SoftPQConv2d(torch.nn.Module):
    """A convolution replaced by table lookup, in training form.  W is the convolution's weight as the
    matrix [Cin*kh*kw, Cout] (rows ordered (ci, r, s)); sub-vector c covers columns [c*V, (c+1)*V)."""

    def __init__(self, centroids, W, kernel, stride=1, pad=0, bias=None, temperature=1.0,
                 table_dtype=_b.TABLE_I8):
        super().__init__()
        self.centroids = torch.nn.Parameter(centroids.clone())
        self.temperature = torch.nn.Parameter(torch.tensor(float(temperature), device=centroids.device))
        self.register_buffer("W", W.clone())
        self.bias = None if bias is None else torch.nn.Parameter(bias.clone())
        self.kernel, self.stride, self.pad = kernel, stride, pad
        self.table_dtype = table_dtype

    def forward(self, inp):
        return _SoftPQConv2dFn.apply(inp, self.centroids, self.temperature, self.W, self.bias,
                                     self.table_dtype, self.kernel, self.stride, self.pad)
