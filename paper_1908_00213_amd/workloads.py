"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws numbers and packs them; it contains none of the method's arithmetic and is the
one piece of code that both the GPU tests/benchmark and the CPU checker are fed from.  All tensors are
NumPy arrays on the host (float32 values, int32 indices) drawn from ``numpy.random.default_rng`` in a
fixed order, so the same seed always gives the same bits.

The paper's own single-GPU workloads are an MNIST classifier (784 inputs, 10 classes; Section
"API Design") and an RNN language model (Section "Conclusion"); neither data set is available here, so
inputs of the same shapes stand in for them.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

BASE_SEED = 190800213


def seed_for(config: int) -> int:
    return BASE_SEED + config


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of ``a`` (float32) rounded to bfloat16, nearest-even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16).reshape(np.shape(a))


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """float32 values of bfloat16 bit patterns."""
    return (bits.astype(np.uint32) << 16).view(np.float32).reshape(bits.shape)


def bf16_exact(a: np.ndarray) -> np.ndarray:
    """float32 array whose every value is exactly representable in bfloat16."""
    return bf16_to_f32(bf16_bits(a))


@dataclass
class MLPWorkload:
    name: str
    sizes: Tuple[int, ...]          # (n_in, hidden..., n_out)
    batch: int
    act: str                        # "relu" | "gelu"
    lr: float
    xs: List[np.ndarray] = field(default_factory=list)      # pool of input batches (B, n_in)
    ts: List[np.ndarray] = field(default_factory=list)      # pool of label vectors (B,) int32
    params: List[Tuple[np.ndarray, np.ndarray]] = field(default_factory=list)  # (W (out,in), b (out,))

    def flops_per_step(self) -> float:
        f = 0.0
        for l in range(len(self.sizes) - 1):
            mnk = 2.0 * self.batch * self.sizes[l] * self.sizes[l + 1]
            f += mnk * (2 if l == 0 else 3)     # forward + dW (+ dx except for the first layer)
        return f

    def n_params(self) -> int:
        return sum(W.size + b.size for W, b in self.params)


def make_mlp(name, sizes, batch, act, seed, n_batches=1, init="he", lr=0.01, classes=None):
    """x ~ N(0,1); labels uniform; W ~ N(0, 2/fan_in) ("he") or N(0, 1/fan_in) ("lecun"); b = 0."""
    rng = np.random.default_rng(seed)
    w = MLPWorkload(name=name, sizes=tuple(sizes), batch=batch, act=act, lr=lr)
    classes = classes or sizes[-1]
    for _ in range(n_batches):
        w.xs.append(rng.standard_normal((batch, sizes[0]), dtype=np.float32))
        w.ts.append(rng.integers(0, classes, size=(batch,), dtype=np.int32))
    for l in range(len(sizes) - 1):
        fan_in = sizes[l]
        std = np.sqrt((2.0 if init == "he" else 1.0) / fan_in)
        W = (rng.standard_normal((sizes[l + 1], fan_in), dtype=np.float32) * np.float32(std))
        w.params.append((W.astype(np.float32), np.zeros((sizes[l + 1],), dtype=np.float32)))
    return w


def config1(seed=None):
    """Tiny MLP 784-100-100-10, ReLU, batch 32, N(0,1/fan_in) weights, one step."""
    return make_mlp("cfg1_tiny_mlp_784-100-100-10_b32", (784, 100, 100, 10), 32, "relu",
                    seed_for(1) if seed is None else seed, 1, init="lecun")


def config3(seed=None, n_batches=4):
    """MLP 784-1000-1000-10, ReLU, batch 1024, He-normal weights."""
    return make_mlp("cfg3_mlp_784-1000-1000-10_b1024", (784, 1000, 1000, 10), 1024, "relu",
                    seed_for(3) if seed is None else seed, n_batches)


def config5(seed=None, n_batches=4, scale=1):
    """Wide MLP 4096-4096-4096-4096-1000, GELU, batch 8192 (``scale`` divides every size but the
    class count, for parity cases the CPU checker can finish)."""
    d, b = 4096 // scale, 8192 // scale
    name = "cfg5_wide_mlp_%d-%d-%d-%d-1000_b%d" % (d, d, d, d, b)
    return make_mlp(name, (d, d, d, d, 1000), b, "gelu",
                    seed_for(5) if seed is None else seed, n_batches)


@dataclass
class ArrayWorkload:
    name: str
    a: np.ndarray
    b: np.ndarray
    c: np.ndarray                   # (1, n) broadcast row


def config2(n=8192, seed=None, m=None):
    """a, b (m,n) ~ U(-1,1); c (1,n) ~ U(-1,1), drawn in that order."""
    rng = np.random.default_rng(seed_for(2) if seed is None else seed)
    m = n if m is None else m
    a = rng.uniform(-1.0, 1.0, size=(m, n)).astype(np.float32)
    b = rng.uniform(-1.0, 1.0, size=(m, n)).astype(np.float32)
    c = rng.uniform(-1.0, 1.0, size=(1, n)).astype(np.float32)
    return ArrayWorkload("cfg2_array_%dx%d" % (m, n), a, b, c)


@dataclass
class LSTMWorkload:
    name: str
    vocab: int
    embed: int
    hidden: int
    batch: int
    bptt: int
    lr: float
    ids: np.ndarray                 # (T, B) int32
    targets: np.ndarray             # (T, B) int32
    params: Dict[str, np.ndarray]   # E (V,E) W (E,4H) U (H,4H) b (4H,) W_out (V,H) b_out (V,)

    def flops_per_step(self) -> float:
        T, B, E, H, V = self.bptt, self.batch, self.embed, self.hidden, self.vocab
        n = T * B
        f = 2.0 * n * E * 4 * H * 3          # x W forward, dW, dX
        f += 2.0 * n * H * 4 * H * 3         # h U forward (T calls), dh (T calls), dU
        f += 2.0 * n * H * V * 3             # output layer forward, dW_out, dH
        return f

    def n_params(self) -> int:
        return sum(v.size for v in self.params.values())


def config4(seed=None, vocab=10000, embed=650, hidden=650, batch=128, bptt=35, lr=0.01):
    """Single-layer LSTM language model step; ids and targets independent uniform tokens;
    E ~ N(0,1); W, U, W_out ~ N(0, 1/fan_in); all biases zero."""
    rng = np.random.default_rng(seed_for(4) if seed is None else seed)
    ids = rng.integers(0, vocab, size=(bptt, batch), dtype=np.int32)
    targets = rng.integers(0, vocab, size=(bptt, batch), dtype=np.int32)
    f32 = np.float32
    P = {
        "E": rng.standard_normal((vocab, embed), dtype=f32),
        "W": rng.standard_normal((embed, 4 * hidden), dtype=f32) * f32(np.sqrt(1.0 / embed)),
        "U": rng.standard_normal((hidden, 4 * hidden), dtype=f32) * f32(np.sqrt(1.0 / hidden)),
        "b": np.zeros((4 * hidden,), dtype=f32),
        "W_out": rng.standard_normal((vocab, hidden), dtype=f32) * f32(np.sqrt(1.0 / hidden)),
        "b_out": np.zeros((vocab,), dtype=f32),
    }
    name = "cfg4_lstm_lm_v%d_e%d_h%d_b%d_t%d" % (vocab, embed, hidden, batch, bptt)
    return LSTMWorkload(name, vocab, embed, hidden, batch, bptt, lr, ids, targets, P)


def pad_lstm_params(P, multiple=32):
    """The language model's parameters embedded in zero arrays whose embedding and hidden widths are
    rounded up to a multiple of `multiple` (gate blocks of W, U and b stay gate blocks, now of the
    rounded width).  The added embedding columns and hidden units are inert: with zero weights and
    biases their cell state and hidden state stay zero and nothing real depends on them, so the loss
    and the gradients of the real entries are those of the unpadded model."""
    V, E = P["E"].shape
    H = P["U"].shape[0]
    up = lambda n: (n + multiple - 1) // multiple * multiple
    Ep, Hp = up(E), up(H)
    out = {"E": np.zeros((V, Ep), np.float32), "W": np.zeros((Ep, 4, Hp), np.float32), "U": np.zeros((Hp, 4, Hp), np.float32),
           "b": np.zeros((4, Hp), np.float32), "W_out": np.zeros((V, Hp), np.float32), "b_out": P["b_out"].astype(np.float32)}
    out["E"][:, :E] = P["E"]
    out["W"][:E, :, :H] = P["W"].reshape(E, 4, H)
    out["U"][:H, :, :H] = P["U"].reshape(H, 4, H)
    out["b"][:, :H] = P["b"].reshape(4, H)
    out["W_out"][:, :H] = P["W_out"]
    out["W"], out["U"], out["b"] = out["W"].reshape(Ep, 4 * Hp), out["U"].reshape(Hp, 4 * Hp), out["b"].reshape(4 * Hp)
    return out
