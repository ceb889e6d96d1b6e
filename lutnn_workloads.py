"""Seeded synthetic inputs for the LUT-NN linear operator.

This module only draws random tensors and rearranges them (im2col).  It holds none
of the method's arithmetic: no distances, no tables, no quantisation.  The CPU
oracle, the GPU tests and bench.py all take their inputs from here so that both
sides see identical bytes.

Notation (arXiv 2302.03213, Sec. 2.1 and Table 1): N rows, D = C*V input width,
K centroids per codebook, M outputs; X[N][D], codebooks P[C][K][V], weights
W[D][M] (row-major, as in Table 1), optional bias[M].

The named workloads stand in for activations and trained weights the paper took
from ImageNet / GLUE models (Sec. 6.1), which are not available offline: values
are N(0,1) activations and centroids and N(0, 0.05) weights.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch


@dataclass
class Workload:
    name: str
    N: int
    C: int
    K: int
    V: int
    M: int
    table_dtype: str  # "i8" or "f32"
    X: np.ndarray = field(repr=False)
    P: np.ndarray = field(repr=False)
    W: np.ndarray = field(repr=False)
    bias: Optional[np.ndarray] = field(repr=False, default=None)
    # convolutions given by their image batch: {"inp": [B,Cin,H,W], "kernel", "stride", "pad"};
    # X then holds the unfolded rows of the first image only
    conv: Optional[dict] = field(repr=False, default=None)

    @property
    def D(self):
        return self.C * self.V


def _gen(seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def _normal(g, shape, std=1.0):
    return (torch.randn(shape, generator=g, dtype=torch.float32) * std).numpy()


def make_layer(name, N, C, K, V, M, table_dtype, seed=0, bias=True, outlier_frac=0.0,
               outlier_gain=10.0, x_std=1.0, w_std=0.05):
    """Generic seeded layer: X ~ N(0, x_std), P ~ N(0,1), W ~ N(0, w_std), bias ~ N(0, 0.1)."""
    g = _gen(seed)
    D = C * V
    X = _normal(g, (N, D), x_std)
    if outlier_frac > 0.0:
        mask = torch.rand((N, D), generator=g).numpy() < outlier_frac
        X = np.where(mask, X * np.float32(outlier_gain), X).astype(np.float32)
    P = _normal(g, (C, K, V), 1.0)
    W = _normal(g, (D, M), w_std)
    b = _normal(g, (M,), 0.1) if bias else None
    return Workload(name, N, C, K, V, M, table_dtype, X, P, W, b)


def im2col_3x3(inp):
    """[1, Cin, H, W] -> [H*W, Cin*9]; columns ordered (c_in, kh, kw), zero padding 1, stride 1.

    With V = 9 the c-th sub-vector of a row is channel c's 3x3 patch (Sec. 4: D = input
    channels x filter size^2, N = height x width).
    """
    t = torch.from_numpy(np.ascontiguousarray(inp))
    cols = torch.nn.functional.unfold(t, kernel_size=3, padding=1, stride=1)  # [1, Cin*9, H*W]
    return cols[0].t().contiguous().numpy()


def fc_small(seed=0):
    """Single LUT-FC, fp32 table: N=256, D=512, V=4 (C=128), K=16, M=512."""
    return make_layer("fc_small_f32", 256, 128, 16, 4, 512, "f32", seed=seed)


def conv_resnet18_input(seed=0, batch=1):
    """The NCHW input of conv_resnet18 (image 0 is the one its rows are unfolded from); further
    images of a batch are drawn from the same stream after the layer's parameters."""
    g = _gen(seed)
    inp = _normal(g, (1, 64, 56, 56), 1.0)
    if batch > 1:
        for shape in ((64, 16, 9), (576, 64), (64,)):
            _normal(g, shape)
        inp = np.concatenate([inp, _normal(g, (batch - 1, 64, 56, 56), 1.0)], axis=0)
    return inp


def conv_resnet18(seed=0):
    """3x3 conv 64->64 on 56x56 as a LUT op (the conv of the paper's Sec. 6.4 breakdown):
    im2col rows N=3136, D=576, V=9 (C=64), K=16, M=64, INT8 table."""
    g = _gen(seed)
    inp = _normal(g, (1, 64, 56, 56), 1.0)
    X = im2col_3x3(inp)
    P = _normal(g, (64, 16, 9), 1.0)
    W = _normal(g, (576, 64), 0.05)
    b = _normal(g, (64,), 0.1)
    return Workload("conv3x3_64x64_56x56_i8", 3136, 64, 16, 9, 64, "i8", X, P, W, b)


def conv_resnet18_batch(seed=0, batch=32):
    """conv_resnet18 on a batch of images, handed over as the NCHW batch (N = batch * 3136 rows)."""
    w = conv_resnet18(seed)
    inp = conv_resnet18_input(seed, batch)
    return Workload("conv3x3_64x64_56x56_b%d_nchw_i8" % batch, batch * 3136, 64, 16, 9, 64, "i8", w.X,
                    w.P, w.W, w.bias, conv={"inp": inp, "kernel": 3, "stride": 1, "pad": 1})


def bert_ffn_up(seed=0):
    """BERT-base FFN-up: N=4096 (32 x 128 tokens), D=768, M=3072, V=2 (C=384), K=16, INT8;
    1% of the activations multiplied by 10."""
    return make_layer("bert_ffn_up_i8", 4096, 384, 16, 2, 3072, "i8", seed=seed,
                      outlier_frac=0.01)


def bert_layer(seed=0):
    """The four linears of one BERT-base encoder layer at batch 32 x seq 128, V=2, K=16, INT8."""
    shapes = [("bert_qkv_i8", 768, 2304), ("bert_attn_out_i8", 768, 768),
              ("bert_ffn_up_i8", 768, 3072), ("bert_ffn_down_i8", 3072, 768)]
    return [make_layer(nm, 4096, D // 2, 16, 2, M, "i8", seed=seed + i)
            for i, (nm, D, M) in enumerate(shapes)]


def paper_kv_space(seed=0):
    """Layers in the (K, V) settings the paper itself evaluates (Sec. 6.1, Table 2): (16, 32) and
    (16, 16) for BERT-base linears, (8, 9) for the 3x3 convolution, (16, 4) for a 1x1 convolution
    (ResNet bottleneck 64 -> 256 channels at 56x56).  INT8 tables."""
    g = _gen(seed + 100)
    inp = _normal(g, (1, 64, 56, 56))
    conv = Workload("conv3x3_64x64_56x56_k8_v9_i8", 3136, 64, 8, 9, 64, "i8", im2col_3x3(inp),
                    _normal(g, (64, 8, 9)), _normal(g, (576, 64), 0.05), _normal(g, (64,), 0.1))
    return [
        make_layer("bert_ffn_up_v32_i8", 4096, 24, 16, 32, 3072, "i8", seed=seed + 101),
        make_layer("bert_ffn_up_v16_i8", 4096, 48, 16, 16, 3072, "i8", seed=seed + 102),
        make_layer("bert_ffn_down_v32_i8", 4096, 96, 16, 32, 768, "i8", seed=seed + 103),
        conv,
        make_layer("conv1x1_64x256_56x56_v4_i8", 3136, 16, 16, 4, 256, "i8", seed=seed + 104),
    ]


def bert_ffn_down_tree12(seed=0):
    """BERT-base FFN-down rows (D = 3072) at V = 32 with the hash encoder's deepest setting of Sec. 7:
    12-level trees, K = 4096 buckets per codebook (C = 96, M = 768; a 288 MiB INT8 table).  The
    bucket prototypes are seeded random vectors, the trees come from random_tree."""
    return make_layer("bert_ffn_down_v32_tree12_i8", 4096, 96, 4096, 32, 768, "i8", seed=seed + 200)


def fc_large(seed=0):
    """Large LUT-FC stress: N=16384, D=4096, M=4096, V=4 (C=1024), K=16, INT8 table (64 MiB)."""
    return make_layer("fc_large_i8", 16384, 1024, 16, 4, 4096, "i8", seed=seed)


def rows_from_centroids(P, N, seed=0):
    """X whose every sub-vector is exactly one of the codebook's centroids; returns (X, choice)."""
    C, K, V = P.shape
    g = _gen(seed)
    choice = torch.randint(0, K, (N, C), generator=g).numpy()
    X = P[np.arange(C)[None, :], choice]  # [N, C, V]
    return np.ascontiguousarray(X.reshape(N, C * V), dtype=np.float32), choice.astype(np.uint8)


def centroids_from_rows(X, C, K, V, seed=0):
    """K-means-like codebooks: each centroid is a randomly chosen sub-vector of X."""
    N = X.shape[0]
    g = _gen(seed)
    pick = torch.randint(0, N, (C, K), generator=g).numpy()
    Xs = X.reshape(N, C, V)
    return np.ascontiguousarray(Xs[pick, np.arange(C)[:, None]], dtype=np.float32)  # [C, K, V]


def random_indices(N, C, K, seed=0):
    g = _gen(seed)
    return torch.randint(0, K, (N, C), generator=g).numpy().astype(np.uint8)


def random_table_i8(C, K, M, seed=0):
    """Full-range INT8 table in [-127, 127] (the range Sec. 3.3's scale produces)."""
    g = _gen(seed)
    return torch.randint(-127, 128, (C, K, M), generator=g).numpy().astype(np.int8)


def random_tree(C, V, levels, seed=0, level_dims=False, thr_std=0.5):
    """Threshold trees for the hash encoder (Sec. 2): per codebook 2^levels - 1 nodes in heap order,
    a split index in [0, V) and a threshold ~ N(0, thr_std) each.  level_dims=True gives every node
    of a level the same split index, the form the hashing work cited there uses.  Random stand-ins
    for learned trees; returns (split_dim int32 [C][nodes], threshold fp32 [C][nodes])."""
    g = _gen(seed)
    nodes = (1 << levels) - 1
    if level_dims:
        per_level = torch.randint(0, V, (C, levels), generator=g).numpy()
        level_of = np.floor(np.log2(np.arange(nodes) + 1)).astype(np.int64)
        dims = per_level[:, level_of]
    else:
        dims = torch.randint(0, V, (C, nodes), generator=g).numpy()
    thr = _normal(g, (C, nodes), thr_std)
    return np.ascontiguousarray(dims, dtype=np.int32), thr
