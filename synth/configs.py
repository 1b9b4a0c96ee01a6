"""Shapes and gradient recipes of the synthetic workloads.

Each workload is a list of parameter tensors grouped into layers (forward
order; the backward pass visits layers in reverse), the gradient storage
format, the number of micro-batches N per mini-batch, the number of mini-batch
steps, the Adam hyper-parameters, and how gradients are drawn.  Only shapes and
input recipes live here: no optimizer arithmetic.

The full-size builders give the five benchmark workloads; every builder also
takes reduced dimensions so that the same structure can be checked against the
CPU oracle in seconds.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

from . import gen

BETA1, BETA2, EPS, LR = 0.9, 0.999, 1e-8, 1e-3


@dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: tuple
    layer: int
    index: int

    @property
    def n(self) -> int:
        return int(math.prod(self.shape))


@dataclass
class Workload:
    name: str
    config_id: int
    gdtype: str                      # "f32" | "bf16" | "f16"
    N: int
    steps: int
    tensors: list = field(default_factory=list)
    layers: list = field(default_factory=list)     # list of lists of tensor indices, forward order
    seed: int = 0
    beta1: float = BETA1
    beta2: float = BETA2
    eps: float = EPS
    lr: float = LR
    sigma_mode: str = "fixed"        # "fixed" | "per_tensor_log_uniform"
    sigma: float = 1e-2
    sigma_lo: float = 1e-4
    sigma_hi: float = 1e-2
    p_zero: float = 0.0
    p_outlier: float = 0.0
    outlier_scale: float = 10.0
    p_sub: float = 0.0
    theta_sigma: float = 0.02

    # ---- construction -------------------------------------------------
    def add_layer(self, named_shapes) -> None:
        li = len(self.layers)
        idx = []
        for name, shape in named_shapes:
            t = TensorSpec(name, tuple(shape), li, len(self.tensors))
            self.tensors.append(t)
            idx.append(t.index)
        self.layers.append(idx)

    # ---- sizes --------------------------------------------------------
    @property
    def P(self) -> int:
        return sum(t.n for t in self.tensors)

    def layer_elems(self, li: int) -> int:
        return sum(self.tensors[i].n for i in self.layers[li])

    @property
    def largest_layer_elems(self) -> int:
        return max(self.layer_elems(li) for li in range(len(self.layers)))

    @property
    def grad_bytes(self) -> int:
        return gen.DTYPE_BYTES[self.gdtype]

    def backward_layers(self):
        """Layer indices in the order the backward pass produces their gradients."""
        return range(len(self.layers) - 1, -1, -1)

    # ---- input streams ------------------------------------------------
    def tensor_sigma(self, ti: int) -> float:
        if self.sigma_mode == "fixed":
            return self.sigma
        return gen.log_uniform(gen.stream_key(self.seed, self.config_id, 0x5167, ti), self.sigma_lo, self.sigma_hi)

    def grad_spec(self, step: int, micro: int, ti: int) -> gen.Spec:
        """Stream of tensor ti's raw gradient in micro-batch `micro` of mini-batch `step` (1-based)."""
        return gen.Spec(key=gen.stream_key(self.seed, self.config_id, 0x6772, step, micro, ti),
                        sigma=self.tensor_sigma(ti), p_zero=self.p_zero, p_outlier=self.p_outlier,
                        outlier_scale=self.outlier_scale, p_sub=self.p_sub)

    def theta_spec(self, ti: int) -> gen.Spec:
        return gen.Spec(key=gen.stream_key(self.seed, self.config_id, 0x7468, ti), sigma=self.theta_sigma)


def mlp_tiny() -> Workload:
    """Config 1: 4 fp32 tensors [256x512],[512],[512x256],[256]; N=4 x 3 steps; N(0, 1e-2), 1% exact zeros."""
    w = Workload("c1_mlp_tiny", 1, "f32", N=4, steps=3, sigma=1e-2, p_zero=0.01)
    w.add_layer([("fc1.weight", (256, 512)), ("fc1.bias", (512,))])
    w.add_layer([("fc2.weight", (512, 256)), ("fc2.bias", (256,))])
    return w


def bert_large(layers: int = 24, hidden: int = 1024, ffn: int = 4096, vocab: int = 30522, positions: int = 512,
               N: int = 8, steps: int = 2) -> Workload:
    """Config 2: BERT-Large-shaped, fp32 gradients, per-tensor sigma log-uniform in [1e-4, 1e-2]."""
    w = Workload("c2_bert_large", 2, "f32", N=N, steps=steps, sigma_mode="per_tensor_log_uniform")
    w.add_layer([("embeddings.word", (vocab, hidden)), ("embeddings.position", (positions, hidden)),
                 ("embeddings.token_type", (2, hidden)), ("embeddings.ln.weight", (hidden,)),
                 ("embeddings.ln.bias", (hidden,))])
    for l in range(layers):
        p = f"layer{l}."
        w.add_layer([(p + "attn.q.weight", (hidden, hidden)), (p + "attn.q.bias", (hidden,)),
                     (p + "attn.k.weight", (hidden, hidden)), (p + "attn.k.bias", (hidden,)),
                     (p + "attn.v.weight", (hidden, hidden)), (p + "attn.v.bias", (hidden,)),
                     (p + "attn.o.weight", (hidden, hidden)), (p + "attn.o.bias", (hidden,)),
                     (p + "attn.ln.weight", (hidden,)), (p + "attn.ln.bias", (hidden,)),
                     (p + "ffn.in.weight", (hidden, ffn)), (p + "ffn.in.bias", (ffn,)),
                     (p + "ffn.out.weight", (ffn, hidden)), (p + "ffn.out.bias", (hidden,)),
                     (p + "ffn.ln.weight", (hidden,)), (p + "ffn.ln.bias", (hidden,))])
    w.add_layer([("pooler.weight", (hidden, hidden)), ("pooler.bias", (hidden,))])
    return w


def gpt2_xl(layers: int = 48, hidden: int = 1600, vocab: int = 50257, positions: int = 1024,
            N: int = 16, steps: int = 2) -> Workload:
    """Config 3: GPT-2-1.5B-shaped, bf16 gradients, N(0, sigma) with 0.1% Student-t(2) x 10 sigma outliers."""
    ffn = 4 * hidden
    w = Workload("c3_gpt2_xl", 3, "bf16", N=N, steps=steps, sigma_mode="per_tensor_log_uniform",
                 p_outlier=1e-3, outlier_scale=10.0)
    w.add_layer([("wte", (vocab, hidden))])
    w.add_layer([("wpe", (positions, hidden))])
    for l in range(layers):
        p = f"h{l}."
        w.add_layer([(p + "ln_1.weight", (hidden,)), (p + "ln_1.bias", (hidden,)),
                     (p + "attn.c_attn.weight", (hidden, 3 * hidden)), (p + "attn.c_attn.bias", (3 * hidden,)),
                     (p + "attn.c_proj.weight", (hidden, hidden)), (p + "attn.c_proj.bias", (hidden,)),
                     (p + "ln_2.weight", (hidden,)), (p + "ln_2.bias", (hidden,)),
                     (p + "mlp.c_fc.weight", (hidden, ffn)), (p + "mlp.c_fc.bias", (ffn,)),
                     (p + "mlp.c_proj.weight", (ffn, hidden)), (p + "mlp.c_proj.bias", (hidden,))])
    w.add_layer([("ln_f.weight", (hidden,)), ("ln_f.bias", (hidden,))])
    return w


def ragged_small(count: int = 2000, group: int = 20, lo: int = 64, hi: int = 262144, N: int = 4,
                 steps: int = 2) -> Workload:
    """Config 4: many small tensors, lengths log-uniform in [lo, hi], fp16 gradients with a sprinkle of
    fp16-subnormal magnitudes, `group` tensors per layer."""
    w = Workload("c4_ragged_small", 4, "f16", N=N, steps=steps, sigma=1e-2, p_sub=0.005)
    names = []
    for i in range(count):
        n = int(round(gen.log_uniform(gen.stream_key(0, 4, 0x6C656E, i), lo, hi)))
        names.append((f"t{i}", (max(lo, min(hi, n)),)))
    for g in range(0, count, group):
        w.add_layer(names[g:g + group])
    return w


def decoder_10b(layers: int = 40, hidden: int = 5120, vocab: int = 32000, N: int = 32, steps: int = 1) -> Workload:
    """Config 5: decoder-shaped single-GPU share, bf16 gradients from one reused per-layer buffer."""
    ffn = 4 * hidden
    w = Workload("c5_decoder_10b", 5, "bf16", N=N, steps=steps, sigma_mode="per_tensor_log_uniform")
    w.add_layer([("embed", (vocab, hidden))])
    for l in range(layers):
        p = f"block{l}."
        shapes = []
        for nm in ("q", "k", "v", "o"):
            shapes += [(p + f"attn.{nm}.weight", (hidden, hidden)), (p + f"attn.{nm}.bias", (hidden,))]
        shapes += [(p + "ln_1.weight", (hidden,)), (p + "ln_1.bias", (hidden,)),
                   (p + "ln_2.weight", (hidden,)), (p + "ln_2.bias", (hidden,)),
                   (p + "mlp.up.weight", (hidden, ffn)), (p + "mlp.up.bias", (ffn,)),
                   (p + "mlp.down.weight", (ffn, hidden)), (p + "mlp.down.bias", (hidden,))]
        w.add_layer(shapes)
    w.add_layer([("ln_f.weight", (hidden,)), ("ln_f.bias", (hidden,))])
    return w


FULL = {"c1": mlp_tiny, "c2": bert_large, "c3": gpt2_xl, "c4": ragged_small, "c5": decoder_10b}


def reduced(name: str) -> Workload:
    """The same structures at sizes the CPU oracle finishes in seconds; dimensions are odd on
    purpose so that tensors end in ragged tails and span several kernel chunks."""
    if name == "c1":
        return mlp_tiny()
    if name == "c2":
        return bert_large(layers=2, hidden=136, ffn=531, vocab=3001, positions=65, N=8, steps=2)
    if name == "c3":
        return gpt2_xl(layers=3, hidden=200, vocab=5003, positions=129, N=16, steps=2)
    if name == "c4":
        return ragged_small(count=120, group=20, lo=64, hi=60000, N=4, steps=2)
    if name == "c5":
        return decoder_10b(layers=2, hidden=168, vocab=2003, N=32, steps=1)
    raise KeyError(name)
