"""Seeded synthetic inputs shaped like the paper's workloads.

The paper trains GPT-style transformers (Sec. 5.1) and gives no tensors; the
weights and gradients below are stand-ins with the same shapes and plausible
value distributions.  This module only draws random numbers and casts them to
the 16-bit storage types; it contains none of the quantization arithmetic, so
both the GPU library's tests and the CPU oracle's tests may use it.

Every tensor is a pure function of (seed, tensor_id, n, device type): values are
drawn with torch's generator on the requested device in fixed-size chunks.  A
test that needs the same bytes on both sides draws once and copies.
"""
import torch

BASE_SEED = 20230610
_CHUNK = 1 << 26


def _gen(device, seed, tensor_id):
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(tensor_id) * 7919) % (2 ** 63 - 1))
    return g


def gpt_layer_shapes(hidden):
    """The four weight matrices of one transformer layer (QKV, attention output
    projection, the two FFN matrices with 4x expansion): 12*hidden^2 elements."""
    return [("qkv", hidden, 3 * hidden), ("attn_out", hidden, hidden),
            ("ffn_up", hidden, 4 * hidden), ("ffn_down", 4 * hidden, hidden)]


def layer_numel(hidden):
    return sum(r * c for _, r, c in gpt_layer_shapes(hidden))


def weights(n, device="cpu", seed=BASE_SEED, tensor_id=0, dtype=torch.bfloat16,
            std=0.02, outlier_prob=1e-3, outlier_gain=20.0):
    """n weights ~ N(0, std); each one independently, with probability
    outlier_prob, multiplied by outlier_gain (a few large-magnitude weights per
    block, as trained transformer weights have)."""
    g = _gen(device, seed, tensor_id)
    out = torch.empty(n, dtype=dtype, device=device)
    for lo in range(0, n, _CHUNK):
        c = min(_CHUNK, n - lo)
        w = torch.randn(c, generator=g, device=device, dtype=torch.float32) * std
        if outlier_prob > 0:
            u = torch.rand(c, generator=g, device=device, dtype=torch.float32)
            w = torch.where(u < outlier_prob, w * outlier_gain, w)
        out[lo:lo + c] = w.to(dtype)
    return out


def gradients(n, device="cpu", seed=BASE_SEED, tensor_id=0, dtype=torch.float16,
              std=1e-3, tail_std=1e-4, nu=3):
    """n gradients = std * z + tail_std * t, z ~ N(0,1), t ~ Student-t with nu
    degrees of freedom (z0 / sqrt(mean of nu squared normals)).  tail_std = 0
    gives plain N(0, std)."""
    g = _gen(device, seed, tensor_id)
    out = torch.empty(n, dtype=dtype, device=device)
    for lo in range(0, n, _CHUNK):
        c = min(_CHUNK, n - lo)
        x = torch.randn(c, generator=g, device=device, dtype=torch.float32) * std
        if tail_std > 0:
            z0 = torch.randn(c, generator=g, device=device, dtype=torch.float32)
            chi = torch.zeros(c, device=device, dtype=torch.float32)
            for _ in range(nu):
                chi += torch.randn(c, generator=g, device=device, dtype=torch.float32) ** 2
            x = x + tail_std * z0 / torch.sqrt(chi / nu)
        out[lo:lo + c] = x.clamp(-65504.0, 65504.0).to(dtype)
    return out


def as_bits(t):
    """Reinterpret a 16-bit floating tensor as int16/uint16-compatible bit patterns
    (numpy has no bfloat16): returns a host numpy uint16 array."""
    import numpy as np
    if t.dtype in (torch.float16, torch.bfloat16):
        return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
    return t.detach().cpu().contiguous().numpy()
