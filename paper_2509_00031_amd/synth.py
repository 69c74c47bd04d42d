"""Seeded synthetic inputs shared by the tests and the benchmark.

Only shapes and value distributions live here -- none of the method's arithmetic.
The recipes stand in for the paper's workloads (pre-trained decoder weights and
tokenised text segments), which are dense and whose cost does not depend on the values:
  * linear / embedding / lm_head weights ~ 0.02 * N(0, 1), fp32
  * norm gains = 1 + 0.02 * N(0, 1), biases ~ 0.02 * N(0, 1) (so that a wrong gain or
    bias index changes the result; a pre-trained model has non-trivial values there)
  * token ids uniform over the vocabulary
  * regression inputs / targets ~ N(0, 1)
"""
import numpy as np


def rng(seed, stream=0):
    return np.random.Generator(np.random.PCG64([int(seed), int(stream)]))


def weights(shape, seed, stream=0, scale=0.02):
    return (rng(seed, stream).standard_normal(shape, dtype=np.float32) * np.float32(scale)).astype(np.float32)


def gains(shape, seed, stream=0):
    return (1.0 + 0.02 * rng(seed, stream).standard_normal(shape, dtype=np.float32)).astype(np.float32)


def token_ids(B, S, vocab, seed):
    return rng(seed, 7).integers(0, vocab, size=(B, S), dtype=np.int32)


def activations(shape, seed, stream=11):
    return rng(seed, stream).standard_normal(shape, dtype=np.float32)


def model_params(shapes, seed):
    """`shapes` = ordered (name, shape, quantized) list; returns fp32 arrays in that order."""
    out = []
    for i, (name, shape, _q) in enumerate(shapes):
        last = name.split(".")[-1]
        if last.endswith("norm") or last.endswith("_g"):
            out.append(gains(shape, seed, i))
        else:
            out.append(weights(shape, seed, i))
    return out
