"""Seeded synthetic inputs shaped like the paper's long-video training workloads.

This module only draws random numbers, rounds them to the storage type and lays out
document lengths; it contains none of the attention arithmetic.  It is the one module
that both the tests' oracle side and the HIP side consume, so that both see identical
input bits.

Shapes follow the 7B-class backbone the paper trains (28 query / 4 KV heads, head
dimension 128), about 196 tokens per video frame and hundreds of frames per sample
(Sec. 3.4-3.5 and the model-complexity table in the appendix).
"""
import numpy as np

TENSOR_IDS = {"q": 0, "k": 1, "v": 2, "do": 3}
TOKENS_PER_FRAME = 196


def bf16_round(x):
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x):
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def chunk(name, c, C, H, d, sigma, seed=0, bf16=True):
    """Rows [c*C, (c+1)*C) of tensor `name` ([T,H,d]); addressable per chunk so the long
    configurations never need the whole tensor on the host at once."""
    rng = np.random.default_rng([seed, TENSOR_IDS[name], int(c)])
    x = rng.standard_normal((C, H, d), dtype=np.float32) * np.float32(sigma)
    return bf16_round(x) if bf16 else x


def tensor(name, n_chunks, C, H, d, sigma, seed=0, bf16=True):
    return np.concatenate([chunk(name, c, C, H, d, sigma, seed, bf16) for c in range(n_chunks)], axis=0)


def packed_cu_seqlens(T, seed=0, frames=(32, 512), text=(64, 2048)):
    """Pack multimodal samples (F video frames x 196 tokens + a text span) until the total
    reaches T; the last sample is truncated so the total is exactly T."""
    rng = np.random.default_rng([seed, 99])
    cu = [0]
    while cu[-1] < T:
        f = int(rng.integers(frames[0], frames[1] + 1))
        t = int(rng.integers(text[0], text[1] + 1))
        cu.append(min(T, cu[-1] + f * TOKENS_PER_FRAME + t))
    return np.asarray(cu, dtype=np.int32)


# The five workloads of the benchmark spec, by name.
CONFIGS = {
    "tiny":    dict(dtype="f32",  Hq=2,  Hkv=1, d=64,  N=2,  C=128,  sigma=1.0, seed=0),
    "cfg2":    dict(dtype="bf16", Hq=28, Hkv=4, d=128, N=4,  C=2048, sigma=0.5, seed=0),
    "cfg3":    dict(dtype="bf16", Hq=28, Hkv=4, d=128, N=8,  C=4096, sigma=0.5, seed=0),
    "long":    dict(dtype="bf16", Hq=28, Hkv=4, d=128, N=32, C=4096, sigma=0.5, seed=0),
    "ulysses": dict(dtype="bf16", Hq=7,  Hkv=1, d=128, N=1,  C=131072, sigma=0.5, seed=0),
    # one GPU of a 2D-attention mesh, head degree 4 x ring degree 8 over the 28/4-head, 256K-token workload
    "2d":      dict(dtype="bf16", Hq=7,  Hkv=1, d=128, N=8,  C=16384, sigma=0.5, seed=0),
}
