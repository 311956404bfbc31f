"""Seeded synthetic inputs with the shapes and value structure of the method's workloads.

This module holds no arithmetic of the method itself (no scales, codes, thresholds or tables):
it only draws the activations, hidden states and weights that stand in for real LLM / ViT
tensors, so that both the GPU library's tests and the independent CPU checker can be fed the
same arrays.  Everything is generated on the host with numpy's counter-based seeding
``default_rng([seed, config_id, tensor_id])``, saturated to the fp16 range and cast to fp16.

Recipes (decoder-layer linears written as K -> N, activations as [tokens, K]):

* config 1  tiny: X ~ N(0,1) [16,1024] with feature dimensions 7 and 500 multiplied by 20;
  W ~ N(0, 0.02^2) [1024,1024]; threshold 6; codec on X flattened with 2048-element blocks.
* config 2  Llama-7B-shaped shard, prefill: 2048 tokens, 4 decoder layers of
  4096->12288, 4096->4096, 4096->22016, 11008->4096; X ~ N(0,1) with 0.1 % of the feature
  dimensions multiplied by U(8,60); W ~ N(0, 0.02^2).
* config 3  decode: the same linears with 1, 8, 32 or 64 tokens, X ~ Student-t(3).
* config 4  shard-boundary hidden state [8192,8192] ~ Student-t(3) with 0.05 % of the feature
  dimensions multiplied by 50; codec blocks of 256, 1024 and 4096 elements.
* config 5  70B-shaped shard, prefill: 4096 tokens, 8192->10240, 8192->8192, 8192->57344,
  28672->8192; X as in config 2; W ~ N(0, 0.015^2).
"""
from dataclasses import dataclass

import numpy as np

FP16_MAX = 65504.0
TAU = 6.0


@dataclass(frozen=True)
class LinearShape:
    name: str
    K: int
    N: int


TINY_LINEAR = (LinearShape("tiny", 1024, 1024),)
LLAMA_7B_LINEARS = (
    LinearShape("qkv", 4096, 12288),
    LinearShape("o", 4096, 4096),
    LinearShape("gate_up", 4096, 22016),
    LinearShape("down", 11008, 4096),
)
LLAMA_70B_LINEARS = (
    LinearShape("qkv", 8192, 10240),
    LinearShape("o", 8192, 8192),
    LinearShape("gate_up", 8192, 57344),
    LinearShape("down", 28672, 8192),
)
VIT_L_LINEARS = (            # ViT-L width 1024, with bias; 197 tokens per image
    LinearShape("qkv", 1024, 3072),
    LinearShape("proj", 1024, 1024),
    LinearShape("fc1", 1024, 4096),
    LinearShape("fc2", 4096, 1024),
)

CODEC_BLOCKS_BOUNDARY = (256, 1024, 4096)


def rng_for(config_id: int, tensor_id: int, seed: int = 0) -> np.random.Generator:
    return np.random.default_rng([seed, config_id, tensor_id])


def to_fp16(a: np.ndarray) -> np.ndarray:
    return np.clip(a, -FP16_MAX, FP16_MAX).astype(np.float16)


def gaussian_weight(K: int, N: int, std: float, rng: np.random.Generator) -> np.ndarray:
    """W [K, N] fp16 ~ N(0, std^2)."""
    w = rng.standard_normal((K, N), dtype=np.float32)
    w *= np.float32(std)
    return to_fp16(w)


def gaussian_bias(N: int, std: float, rng: np.random.Generator) -> np.ndarray:
    return to_fp16(rng.standard_normal(N, dtype=np.float32) * np.float32(std))


def gaussian_with_outlier_dims(M: int, K: int, frac: float, lo: float, hi: float,
                               rng: np.random.Generator):
    """X [M, K] fp16 ~ N(0,1) with round(frac*K) feature dimensions each multiplied by its own
    factor ~ U(lo, hi).  Returns (X, sorted indices of the scaled dimensions)."""
    x = rng.standard_normal((M, K), dtype=np.float32)
    n_dims = int(round(frac * K))
    dims = np.sort(rng.choice(K, size=n_dims, replace=False)) if n_dims else np.zeros(0, np.int64)
    factors = rng.uniform(lo, hi, size=n_dims).astype(np.float32)
    x[:, dims] *= factors[None, :]
    return to_fp16(x), dims


def student_t(M: int, K: int, nu: float, rng: np.random.Generator) -> np.ndarray:
    return to_fp16(rng.standard_t(nu, size=(M, K)).astype(np.float32))


def student_t_with_outlier_dims(M: int, K: int, nu: float, frac: float, factor: float,
                                rng: np.random.Generator):
    x = rng.standard_t(nu, size=(M, K)).astype(np.float32)
    n_dims = int(round(frac * K))
    dims = np.sort(rng.choice(K, size=n_dims, replace=False)) if n_dims else np.zeros(0, np.int64)
    x[:, dims] *= np.float32(factor)
    return to_fp16(x), dims


# ------------------------------------------------------------------ the five configurations
def config1():
    """Tiny single linear + codec input."""
    x = rng_for(1, 0).standard_normal((16, 1024), dtype=np.float32)
    x[:, [7, 500]] *= np.float32(20.0)
    W = gaussian_weight(1024, 1024, 0.02, rng_for(1, 1))
    return dict(X=to_fp16(x), W=W, tau=TAU, block=2048, planted=np.array([7, 500]))


def prefill_activation(config_id: int, tensor_id: int, M: int, K: int):
    """Configs 2 and 5: Gaussian bulk, 0.1 % of feature dimensions scaled by U(8,60)."""
    return gaussian_with_outlier_dims(M, K, 0.001, 8.0, 60.0, rng_for(config_id, tensor_id))


def prefill_weight(config_id: int, tensor_id: int, shape: LinearShape, std: float) -> np.ndarray:
    return gaussian_weight(shape.K, shape.N, std, rng_for(config_id, tensor_id))


def decode_activation(tensor_id: int, M: int, K: int) -> np.ndarray:
    """Config 3: heavy-tailed decode activations."""
    return student_t(M, K, 3.0, rng_for(3, tensor_id))


def boundary_hidden_state(rows: int = 8192, cols: int = 8192, tensor_id: int = 0):
    """Config 4: hidden state crossing a shard boundary."""
    return student_t_with_outlier_dims(rows, cols, 3.0, 0.0005, 50.0, rng_for(4, tensor_id))


def adapter_factors(config_id: int, tensor_id: int, K: int, N: int, r: int, std: float = 0.02):
    """Low-rank factors of a trained adapter: A [r, K] and B [N, r], fp16, both ~ N(0, std^2) (after
    fine-tuning neither factor is zero)."""
    rng = rng_for(config_id, tensor_id)
    A = to_fp16(rng.standard_normal((r, K), dtype=np.float32) * np.float32(std))
    B = to_fp16(rng.standard_normal((N, r), dtype=np.float32) * np.float32(std))
    return A, B


def linear_ops(M: int, shapes) -> int:
    """Integer multiply-add operations (2 per MAC) of one pass over the given linears."""
    return sum(2 * M * s.K * s.N for s in shapes)
