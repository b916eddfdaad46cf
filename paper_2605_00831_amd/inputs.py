"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the tests of the CPU oracle and the GPU path, and it
contains none of the method's arithmetic: no field operations, no generator
matrices, no encoding -- only random bytes, KV-cache geometry, block tables
and erasure patterns.  It imports neither the oracle nor the HIP binding.

Geometry (Section 6.1 models; GQA with 8 KV heads of dimension 128, 16-bit
values): bytes per token = layers * 2 (K and V) * kv_heads * head_dim * 2.
The paper checkpoints an FP16 KV cache viewed as integers (Section 4.1);
bf16 only changes the byte histogram, not the code.
"""
import itertools

import numpy as np

SEED_BASE = 0x67530000
TABLE_SEED_OFFSET = 0x100
ERASURE_SEED_OFFSET = 0x200

GiB = 1 << 30
MiB = 1 << 20
KiB = 1 << 10


def bytes_per_token(layers, kv_heads=8, head_dim=128, value_bytes=2):
    return layers * 2 * kv_heads * head_dim * value_bytes


# The five workloads the build is measured on.  "S" is bytes per shard.
CONFIGS = {
    "tiny": dict(index=0, layers=2, batch=1, tokens=1024, dtype="fp16", sigma=1.0,
                 k=4, m=2, erased=(1, 3)),
    "llama8b_prefill": dict(index=1, layers=32, batch=8, tokens=32768, dtype="bf16", sigma=0.5,
                            k=4, m=2, chunk_tokens=2048),
    "decode_paged": dict(index=2, layers=32, batch=64, tokens=1, dtype="bf16", sigma=1.0,
                         k=4, m=1, block_tokens=16, steps=1000),
    "llama70b_longctx": dict(index=3, layers=80, batch=1, tokens=131072, dtype="bf16", sigma=1.0,
                             k=8, m=2, chunk_tokens=2048),
    "recovery_stress": dict(index=4, k=8, m=3, shard_bytes=512 * MiB, small_shard_bytes=64 * KiB + 5,
                            patterns_full=20),
}


def config_seed(name):
    return SEED_BASE + CONFIGS[name]["index"]


def config_total_bytes(name):
    c = CONFIGS[name]
    if "shard_bytes" in c:
        return c["shard_bytes"] * c["k"]
    return bytes_per_token(c["layers"]) * c["batch"] * c["tokens"]


def config_shard_bytes(name):
    return config_total_bytes(name) // CONFIGS[name]["k"]


# ---------------------------------------------------------------- numpy side

def _f32_to_bf16_bits(x):
    """float32 -> bf16 bit patterns (round to nearest even), as uint16."""
    u = x.astype(np.float32).view(np.uint32)
    rounded = u + 0x7FFF + ((u >> 16) & 1)
    return (rounded >> 16).astype(np.uint16)


def kv_bytes_np(seed, nbytes, dtype="bf16", sigma=1.0):
    """nbytes raw bytes of an N(0, sigma) KV cache in fp16 or bf16."""
    rng = np.random.default_rng(seed)
    nvals = (nbytes + 1) // 2
    x = (rng.standard_normal(nvals, dtype=np.float32) * np.float32(sigma))
    if dtype == "fp16":
        bits = x.astype(np.float16).view(np.uint16)
    elif dtype == "bf16":
        bits = _f32_to_bf16_bits(x)
    else:
        raise ValueError(dtype)
    return np.ascontiguousarray(bits.view(np.uint8)[:nbytes])


def uniform_bytes_np(seed, nbytes):
    return np.random.default_rng(seed).integers(0, 256, size=nbytes, dtype=np.uint8)


def special_bits(dtype="fp16"):
    """16-bit patterns that a lossy path would damage: NaNs with payloads,
    infinities, signed zeros, denormals, extremes."""
    if dtype == "fp16":
        pats = [0x7E00, 0xFE00, 0x7C01, 0xFDFF, 0x7C00, 0xFC00, 0x0000, 0x8000,
                0x0001, 0x8001, 0x03FF, 0x0400, 0x7BFF, 0xFBFF, 0x3C00, 0xBC00]
    else:
        pats = [0x7FC0, 0xFFC0, 0x7F81, 0xFFFF, 0x7F80, 0xFF80, 0x0000, 0x8000,
                0x0001, 0x8001, 0x007F, 0x0080, 0x7F7F, 0xFF7F, 0x3F80, 0xBF80]
    return np.array(pats, dtype=np.uint16)


def plant_specials(buf, dtype="fp16", seed=0):
    """Overwrite a few 16-bit slots of a byte buffer with special patterns."""
    pats = special_bits(dtype)
    v = buf[: (buf.size // 2) * 2].view(np.uint16)
    if v.size == 0:
        return buf
    pos = np.random.default_rng(seed ^ 0x5BEC).integers(0, v.size, size=4 * len(pats))
    v[pos] = np.tile(pats, 4)
    return buf


def split_shards(buf, k):
    """Contiguous equal split of a byte buffer into k shards (views)."""
    assert buf.size % k == 0
    S = buf.size // k
    return [buf[j * S:(j + 1) * S] for j in range(k)]


def block_table_np(seed, k, pages_per_shard, num_pages):
    """int32 [k][pages_per_shard]: distinct page ids from a seeded permutation."""
    assert k * pages_per_shard <= num_pages
    perm = np.random.default_rng(seed + TABLE_SEED_OFFSET).permutation(num_pages)
    return np.ascontiguousarray(perm[: k * pages_per_shard].reshape(k, pages_per_shard).astype(np.int32))


def all_erasure_patterns(n_shards, max_erased, min_erased=0):
    for e in range(min_erased, max_erased + 1):
        for pat in itertools.combinations(range(n_shards), e):
            yield pat


def random_erasure_patterns(seed, n_shards, e, count):
    rng = np.random.default_rng(seed + ERASURE_SEED_OFFSET)
    return [tuple(sorted(int(x) for x in rng.choice(n_shards, size=e, replace=False)))
            for _ in range(count)]


# ---------------------------------------------------------------- torch side

def kv_bytes_device(seed, nbytes, dtype="bf16", sigma=1.0, device="cuda", piece=GiB, out=None):
    """Same distribution generated on the device, in pieces of at most `piece`
    bytes so the float32 staging stays small.  Returns a uint8 tensor (`out`,
    a uint8 device tensor of nbytes, if one is given)."""
    import torch
    tdt = {"bf16": torch.bfloat16, "fp16": torch.float16}[dtype]
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=device)
    assert out.numel() == nbytes
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    done = 0
    while done < nbytes:
        n = min(piece, nbytes - done)
        nvals = (n + 1) // 2
        x = torch.randn(nvals, generator=gen, device=device, dtype=torch.float32)
        x.mul_(sigma)
        b = x.to(tdt).view(torch.uint8)
        out[done:done + n] = b[:n]
        del x, b
        done += n
    return out


def uniform_bytes_device(seed, nbytes, device="cuda", piece=GiB, out=None):
    import torch
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=device)
    assert out.numel() == nbytes
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    done = 0
    while done < nbytes:
        n = min(piece, nbytes - done)
        out[done:done + n] = torch.randint(0, 256, (n,), generator=gen, device=device,
                                           dtype=torch.uint8)
        done += n
    return out
