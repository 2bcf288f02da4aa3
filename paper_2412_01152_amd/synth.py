"""Seeded synthetic inputs and workload shapes.

This module only makes inputs: tensor shapes of the paper's 10B model (Appendix table "Model
Configuration": 42 layers, hidden 4096, 32 heads, 8 KV heads, vocabulary 128,256; feed-forward
width 14,336 and head size 128 are the Llama-3-8B values the table's caption points to) and random
values with the distributions the benchmark configurations name.  It holds none of the method's
arithmetic, so both the GPU tests and the CPU oracle's tests may draw from it.

Values are produced by torch's seeded generators on whichever device is asked for; CPU and GPU
generators give different (equally distributed) numbers, so a test generates once and hands the
same bits to both sides.
"""
from __future__ import annotations

import math
from typing import List, Sequence

import torch

BASE_SEED = 241201152

HIDDEN = 4096
FFN = 14336
N_HEADS = 32
N_KV_HEADS = 8
HEAD_DIM = 128
N_LAYERS = 42
VOCAB = 128256

STREAM_THETA_OUTER = 0      # random stream ids: 0 = theta_outer, 1 + p = delta of peer p


def layer_tensor_sizes() -> List[int]:
    """Element counts of one decoder layer's tensors, in storage order:
    wq, wk, wv, wo, w_gate, w_up, w_down, attn_norm, ffn_norm."""
    q = N_HEADS * HEAD_DIM * HIDDEN
    kv = N_KV_HEADS * HEAD_DIM * HIDDEN
    ff = FFN * HIDDEN
    return [q, kv, kv, q, ff, ff, ff, HIDDEN, HIDDEN]


def layer_row_sizes() -> List[int]:
    """One decoder layer cut into one quantisation group per matrix row (row = the inner dimension of
    each weight matrix: 4096 everywhere except w_down's 14336; each norm vector is one row): 43,010
    groups over the same 218,112,000 elements."""
    row_len = [HIDDEN, HIDDEN, HIDDEN, HIDDEN, HIDDEN, HIDDEN, FFN, HIDDEN, HIDDEN]
    return [r for n, r in zip(layer_tensor_sizes(), row_len) for _ in range(n // r)]


def model_tensor_sizes(n_layers: int = N_LAYERS) -> List[int]:
    """Element counts of the full untied model: embed, n_layers x layer, final norm, head."""
    sizes = [VOCAB * HIDDEN]
    for _ in range(n_layers):
        sizes += layer_tensor_sizes()
    sizes += [HIDDEN, VOCAB * HIDDEN]
    return sizes


def ring_chunk_sizes(n: int, chunks: int) -> List[int]:
    """Split n elements into `chunks` contiguous pieces of ceil(n / chunks), the last one shorter."""
    c = -(-n // chunks)
    out = []
    left = n
    for _ in range(chunks):
        take = min(c, left)
        out.append(take)
        left -= take
    return out


def offsets_from_sizes(sizes: Sequence[int]) -> List[int]:
    off = [0]
    for s in sizes:
        off.append(off[-1] + int(s))
    return off


def config_segment_sizes(config: int) -> List[int]:
    """Quantisation-group sizes of benchmark configuration 0..4."""
    if config == 0:
        return [1 << 20]
    if config == 1:
        return layer_tensor_sizes()
    if config in (2, 3):
        return model_tensor_sizes()
    if config == 4:
        return ring_chunk_sizes(sum(model_tensor_sizes()), 14)
    raise ValueError(config)


def config_peers(config: int) -> int:
    return {0: 4, 1: 8, 2: 4, 3: 14, 4: 13}[config]


def config_delta_kind(config: int) -> str:
    return "student_t3" if config == 3 else "mixture"


def _gen(device, seed: int, stream: int, chunk: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + stream * 7919 + chunk * 104729 + 12345) % (2 ** 63 - 1))
    return g


def _chunk_elems(device) -> int:
    return (1 << 26) if torch.device(device).type == "cuda" else (1 << 22)


def fill_theta_outer(out: torch.Tensor, seed: int = BASE_SEED, std: float = 0.02) -> torch.Tensor:
    """out[:] ~ N(0, std), fp32, chunk by chunk (no big temporaries)."""
    assert out.dtype == torch.float32 and out.dim() == 1
    step = _chunk_elems(out.device)
    for c, a in enumerate(range(0, out.numel(), step)):
        b = min(a + step, out.numel())
        g = _gen(out.device, seed, STREAM_THETA_OUTER, c)
        out[a:b].normal_(0.0, std, generator=g)
    return out


def _delta_chunk(n: int, kind: str, device, g: torch.Generator) -> torch.Tensor:
    if kind == "mixture":
        # with probability 0.9 a normal of std 1e-3, with probability 0.1 a Laplace of scale 5e-3
        pick = torch.rand(n, device=device, generator=g)
        normal = torch.randn(n, device=device, generator=g) * 1e-3
        v = torch.rand(n, device=device, generator=g) - 0.5
        lap = -5e-3 * torch.sign(v) * torch.log1p(-2.0 * v.abs().clamp_(max=0.5 - 1e-7))
        return torch.where(pick < 0.9, normal, lap)
    if kind == "student_t3":
        # Z / sqrt(chi2_3 / 3) * 1e-3
        z = torch.randn(n, device=device, generator=g)
        chi = torch.randn(n, device=device, generator=g).square_()
        chi += torch.randn(n, device=device, generator=g).square_()
        chi += torch.randn(n, device=device, generator=g).square_()
        return z * torch.rsqrt(chi / 3.0) * 1e-3
    if kind == "normal":
        return torch.randn(n, device=device, generator=g) * 1e-3
    if kind == "zero":
        return torch.zeros(n, device=device)
    raise ValueError(kind)


def fill_theta_local(out: torch.Tensor, theta_outer: torch.Tensor, peer: int,
                     kind: str = "mixture", seed: int = BASE_SEED) -> torch.Tensor:
    """out[:] = fp32(theta_outer + delta_peer), rounded to out's dtype (fp32 or bf16).

    A worker's weights after its inner steps are modelled as the shared starting point plus a
    random displacement; the displacement's distribution is the benchmark configuration's."""
    assert theta_outer.dtype == torch.float32 and out.numel() == theta_outer.numel()
    step = _chunk_elems(out.device)
    for c, a in enumerate(range(0, out.numel(), step)):
        b = min(a + step, out.numel())
        g = _gen(out.device, seed, 1 + peer, c)
        d = _delta_chunk(b - a, kind, out.device, g)
        out[a:b] = (theta_outer[a:b] + d).to(out.dtype)
    return out


def fill_delta(out: torch.Tensor, peer: int, kind: str = "mixture", seed: int = BASE_SEED) -> torch.Tensor:
    """out[:] = a displacement drawn from the configuration's distribution (an fp32 pseudo-gradient
    that is handed over as such: the chunk owner's un-quantised addend)."""
    assert out.dtype == torch.float32 and out.dim() == 1
    step = _chunk_elems(out.device)
    for c, a in enumerate(range(0, out.numel(), step)):
        b = min(a + step, out.numel())
        out[a:b] = _delta_chunk(b - a, kind, out.device, _gen(out.device, seed, 1 + peer, c))
    return out


STREAM_CODES = 1000      # generator streams of the synthetic coded contributions: 1000 + peer


def fill_coded_contribution(codes_out: torch.Tensor, peer: int, seed: int = BASE_SEED) -> torch.Tensor:
    """Synthetic coded contribution for inputs too large to quantise on the host first: bytes with
    the bell-shaped occupancy real codes have (a normal variate fills buckets 128 +- 21.3 per
    standard deviation when the range is +-6 sigma in 256 buckets), clipped to 0..255."""
    assert codes_out.dtype == torch.uint8 and codes_out.dim() == 1
    step = _chunk_elems(codes_out.device)
    for c, a in enumerate(range(0, codes_out.numel(), step)):
        b = min(a + step, codes_out.numel())
        g = _gen(codes_out.device, seed, STREAM_CODES + peer, c)
        z = torch.randn(b - a, device=codes_out.device, generator=g)
        codes_out[a:b] = (z * (256.0 / 12.0) + 128.0).floor_().clamp_(0, 255).to(torch.uint8)
    return codes_out


def synthetic_codebooks(groups: int, peer: int, std: float = 2.43e-3, device="cpu",
                        seed: int = BASE_SEED) -> torch.Tensor:
    """[groups][256] ascending fp32 codebooks to go with fill_coded_contribution: bucket centres of a
    +-6 std range around a small per-group mean, each moved by up to a third of a bucket."""
    g = _gen(device, seed, STREAM_CODES + peer, 1 << 20)
    w = 12.0 * std / 256.0
    k = torch.arange(256, device=device, dtype=torch.float32)
    mean = torch.randn(groups, 1, device=device, generator=g) * (0.01 * std)
    jitter = (torch.rand(groups, 256, device=device, generator=g) - 0.5) * (2.0 / 3.0)
    return (mean + (k - 127.5 + jitter) * w).contiguous()


def make_inputs(sizes: Sequence[int], peers: int, kind: str = "mixture", device="cpu",
                seed: int = BASE_SEED, local_dtype=torch.float32):
    """Small-case helper: (theta_outer, [theta_local_p for p in range(peers)], seg_offsets)."""
    n = int(sum(sizes))
    theta = fill_theta_outer(torch.empty(n, dtype=torch.float32, device=device), seed)
    locals_ = [fill_theta_local(torch.empty(n, dtype=local_dtype, device=device), theta, p, kind, seed)
               for p in range(peers)]
    return theta, locals_, offsets_from_sizes(sizes)


def ragged_sizes(total_hint: int, seed: int = 7) -> List[int]:
    """A ragged mix of segment lengths (tiny, odd, unaligned, large) for parity tests."""
    g = torch.Generator().manual_seed(seed)
    sizes = [1, 3, 4096, 4097, 17, 65536 + 5, 0, 1023]
    left = max(0, total_hint - sum(sizes))
    while left > 0:
        s = int(torch.randint(1, max(2, total_hint // 3), (1,), generator=g))
        s = min(s, left)
        sizes.append(s)
        left -= s
    return sizes


def n_elements(config: int) -> int:
    return int(sum(config_segment_sizes(config)))


assert sum(layer_tensor_sizes()) == 218_112_000
assert len(layer_row_sizes()) == 43_010 and sum(layer_row_sizes()) == 218_112_000
assert sum(model_tensor_sizes()) == 10_211_381_248
assert math.ceil(10_211_381_248 / 14) == 729_384_375
