"""Seeded synthetic inputs shaped like the paper's layers.

This module holds shapes and random numbers only -- none of the method's
arithmetic -- so that the CPU oracle and the GPU library can be fed the very
same values without sharing any code.  The tensors stand in for the paper's
datasets (CIFAR-10, ImageNet, WikiText-2, WMT16): the cost of the factorized
layers depends only on shapes, which are taken from the paper's architecture
tables (Appendix D) at the global rank ratio 1/4 (Section 4.1,
"Hyper-parameters").

Every generator returns float32 numpy arrays.  With ``dtype="bf16"`` the
values are first rounded to bfloat16 (round to nearest even) and stored back
in float32, so an exact bf16 copy can be made for the GPU while the oracle
reads the same numbers in double precision.
"""
import numpy as np

SEED_BASE = 0x5EED0000


def round_to_bf16(a):
    """Round float32 values to the nearest bfloat16 (ties to even), keep float32 storage."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a):
    """uint16 bit patterns of float32 values that are exactly bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


class Stream:
    """One counter-based (Philox) stream per (seed, tensor index)."""

    def __init__(self, seed, dtype="f32"):
        self.seed = int(seed)
        self.dtype = dtype
        self.count = 0

    def _gen(self):
        g = np.random.Generator(np.random.Philox(key=[self.seed, self.count]))
        self.count += 1
        return g

    def _finish(self, a):
        a = a.astype(np.float32)
        return round_to_bf16(a) if self.dtype == "bf16" else a

    def normal(self, shape, std=1.0):
        return self._finish(self._gen().standard_normal(shape) * std)

    def uniform(self, shape, lo, hi):
        return self._finish(self._gen().uniform(lo, hi, shape))

    def integers(self, shape, hi):
        return self._gen().integers(0, hi, shape, dtype=np.int64)


# --------------------------------------------------------------- generators

def linear_inputs(M, n_in, n_out, r, dtype="f32", seed=0, bias=False):
    """X ~ N(0,1); V[in x r] ~ N(0, 1/in); U[out x r] ~ N(0, 1/r); dY ~ N(0,1)."""
    s = Stream(SEED_BASE + seed, dtype)
    d = dict(
        X=s.normal((M, n_in)),
        V=s.normal((n_in, r), 1.0 / np.sqrt(max(n_in, 1))),
        U=s.normal((n_out, r), 1.0 / np.sqrt(max(r, 1))),
        dY=s.normal((M, n_out)),
    )
    d["bias"] = s.normal((n_out,)) if bias else None
    return d


def linear_shared_inputs(M, n_in, n_out, r, groups, dtype="f32", seed=0, bias=False):
    """`groups` projections of one input (Q, K, V): X ~ N(0,1); V[G,in,r] ~ N(0, 1/in); U[G,out,r] ~ N(0, 1/r);
    dY[G,M,out] ~ N(0,1)."""
    s = Stream(SEED_BASE + seed, dtype)
    d = dict(
        X=s.normal((M, n_in)),
        V=s.normal((groups, n_in, r), 1.0 / np.sqrt(max(n_in, 1))),
        U=s.normal((groups, n_out, r), 1.0 / np.sqrt(max(r, 1))),
        dY=s.normal((groups, M, n_out)),
    )
    d["bias"] = s.normal((groups, n_out)) if bias else None
    return d


def conv_inputs(N, C, H, W, Cout, r, k, stride=1, pad=0, dtype="f32", seed=0):
    """X ~ N(0,1) NCHW; Uk[r,C,k,k] ~ N(0, 1/(C k^2)); Vp[Cout,r] ~ N(0, 1/r); dY ~ N(0,1)."""
    s = Stream(SEED_BASE + seed, dtype)
    Ho = (H + 2 * pad - k) // stride + 1
    Wo = (W + 2 * pad - k) // stride + 1
    return dict(
        X=s.normal((N, C, H, W)),
        Uk=s.normal((r, C, k, k), 1.0 / np.sqrt(max(C * k * k, 1))),
        Vp=s.normal((Cout, r), 1.0 / np.sqrt(max(r, 1))),
        dY=s.normal((N, Cout, Ho, Wo)),
    )


def lstm_cell_inputs(B, d, h, r, groups=1, dtype="f32", seed=0, bias=True, scale=0.1):
    """One cell step: x, h_prev, c_prev ~ N(0,1)/2; factors and bias ~ U(-scale, scale)."""
    s = Stream(SEED_BASE + seed, dtype)
    gr = groups * r
    out = dict(
        x=s.normal((B, d), 0.5),
        h_prev=s.normal((B, h), 0.5),
        c_prev=s.normal((B, h), 0.5),
        Vx=s.uniform((d, gr), -scale, scale),
        Ux=s.uniform((4 * h, r), -scale, scale),
        Vh=s.uniform((h, gr), -scale, scale),
        Uh=s.uniform((4 * h, r), -scale, scale),
        dh=s.normal((B, h)),
        dc=s.normal((B, h)),
    )
    out["bias"] = s.uniform((4 * h,), -scale, scale) if bias else None
    return out


def lstm_lm_inputs(vocab, d, h, r, layers, T, B, groups=1, seed=0, scale=0.1):
    """Language-model stack: embedding table, token ids, per-layer factors, upstream grads."""
    s = Stream(SEED_BASE + seed, "f32")
    gr = groups * r
    out = dict(
        E=s.uniform((vocab, d), -scale, scale),
        tokens=s.integers((T, B), vocab),
        dH_top=s.normal((T, B, h)),
        layers=[],
    )
    for l in range(layers):
        d_in = d if l == 0 else h
        out["layers"].append(dict(
            Vx=s.uniform((d_in, gr), -scale, scale),
            Ux=s.uniform((4 * h, r), -scale, scale),
            Vh=s.uniform((h, gr), -scale, scale),
            Uh=s.uniform((4 * h, r), -scale, scale),
            bias=s.uniform((4 * h,), -scale, scale),
        ))
    return out


# ------------------------------------------------------------------ configs
# The five benchmark configurations.  Shapes: VGG-19 fc17/fc18 (cfg 0),
# CIFAR ResNet-18 conv4_x (cfg 1), the 2-layer LSTM language model (cfg 2),
# one low-rank Transformer encoder layer (cfg 3), ResNet-50 conv5_x (cfg 4);
# all from Appendix D at rank ratio 1/4.

CONFIGS = {
    "linear_fc_f32": dict(kind="linear", dtype="f32", M=64, n_in=512, n_out=512, r=128, seed=0),
    "resnet18_conv4_bf16": dict(kind="conv", dtype="bf16", N=128, C=256, H=8, W=8, Cout=256, r=64,
                                k=3, stride=1, pad=1, seed=1),
    "lstm_lm_f32": dict(kind="lstm", dtype="f32", vocab=33278, d=1500, h=1500, r=375, layers=2,
                        T=35, B=20, seed=2),
    # the same model through the sequence-level entry points (one call per layer and direction)
    "lstm_lm_seq_f32": dict(kind="lstm", dtype="f32", vocab=33278, d=1500, h=1500, r=375, layers=2,
                            T=35, B=20, seed=2, seq=True),
    # the same model through the stack entry points (one call per direction, layers on the diagonals l + t)
    "lstm_lm_stack_f32": dict(kind="lstm", dtype="f32", vocab=33278, d=1500, h=1500, r=375, layers=2,
                              T=35, B=20, seed=2, stack=True),
    # Algorithm 1's factor initialisation for one layer of each model family (dense weight -> balanced factors)
    "svd_split_f32": dict(kind="svd", dtype="f32", seed=5, layers=dict(
        vgg_fc=(512, 512, 128), resnet18_conv4=(2304, 256, 64), transformer_ffn=(2048, 512, 128),
        lstm_gates=(6000, 1500, 375))),
    "transformer_block_bf16": dict(kind="linear_set", dtype="bf16", M=64 * 128, seed=3, layers=dict(
        wq=(512, 512, 128), wk=(512, 512, 128), wv=(512, 512, 128), wo=(512, 512, 128),
        ffn1=(512, 2048, 128), ffn2=(2048, 512, 128))),
    # the same block with the query, key and value projections (one input) through the shared-input entry points
    "transformer_block_qkv_bf16": dict(kind="linear_set", dtype="bf16", M=64 * 128, seed=3, shared=("wq", "wk", "wv"),
                                       layers=dict(wq=(512, 512, 128), wk=(512, 512, 128), wv=(512, 512, 128),
                                                   wo=(512, 512, 128), ffn1=(512, 2048, 128), ffn2=(2048, 512, 128))),
    # blocks with the layers' epilogues (bias / fixed-statistics batch norm, ReLU, residual) through the *_ep calls:
    # the feed-forward network of a Transformer layer with its residual connection (Section 2.4), and a ResNet-18
    # conv4_x basic block (Appendix D)
    "transformer_ffn_block_bf16": dict(kind="ffn_block", dtype="bf16", M=64 * 128, d=512, dff=2048, r=128, seed=6),
    "resnet18_basic_block_bf16": dict(kind="basic_block", dtype="bf16", N=128, C=256, H=8, W=8, r=64, k=3, seed=7),
    "resnet50_conv5_bf16": dict(kind="conv_set", dtype="bf16", N=256, H=7, W=7, seed=4, layers=dict(
        conv1=(2048, 512, 128, 1, 0), conv2=(512, 512, 128, 3, 1), conv3=(512, 2048, 128, 1, 0))),
}


def linear_flops(M, n_in, n_out, r):
    """Algorithmic fwd+bwd flops of a factorized linear layer: 6 M r (in + out)."""
    return 6.0 * M * r * (n_in + n_out)


def conv_flops(N, C, Ho, Wo, Cout, r, k):
    """Algorithmic fwd+bwd flops of a factorized conv: 6 (N Ho Wo) r (C k^2 + Cout)."""
    return 6.0 * N * Ho * Wo * r * (C * k * k + Cout)
