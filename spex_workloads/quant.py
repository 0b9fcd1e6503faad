"""fp8 (OCP e4m3fn) encoding of synthetic K/V, one fp32 scale per (page, KV head).

This is input preparation: the attention library never quantises, it receives
codes and scales.  The encoder is written with integer tensor operations so the
CPU and the GPU produce the same bytes.
"""

from __future__ import annotations

import torch

E4M3_MAX = 448.0
_MIN_SCALE = 2.0 ** -40


def encode_e4m3(x: torch.Tensor) -> torch.Tensor:
    """Round finite fp32 values to e4m3fn codes (uint8): nearest-even, saturating at +-448."""
    x = x.to(torch.float32).clamp(-E4M3_MAX, E4M3_MAX).contiguous()
    bits = x.view(torch.int32)
    sign = (bits >> 24) & 0x80
    a = bits & 0x7FFFFFFF
    # Normal range (|x| >= 2^-6): round the fp32 mantissa to 3 bits, ties to even.
    r = a + 0x7FFFF + ((a >> 20) & 1)
    code_n = (((r >> 23) - 120) << 3) | ((r >> 20) & 7)
    # Subnormal range: multiples of 2^-9; 8 * 2^-9 is the smallest normal (code 0x08).
    code_s = torch.round(a.view(torch.float32) * 512.0).to(torch.int32)
    code = torch.where(a >= 0x3C800000, code_n, code_s)
    return (code | sign).to(torch.uint8)


def _scale_and_inverse(amax: torch.Tensor):
    """scale = max(amax / 448, tiny) and 1 / scale, both computed on the host: fp32 division
    is not rounded the same way on every device, multiplication is."""
    a = amax.detach().to("cpu", torch.float32)
    s = (a / E4M3_MAX).clamp_min(_MIN_SCALE)
    return s.to(amax.device), (1.0 / s).to(amax.device)


def quantise_pages(x: torch.Tensor, first_slot: int, page_size: int, prev_scale=None):
    """Quantise an append of n tokens, x = [n, H, D] fp32, that starts at slot `first_slot`
    of the node's current last page.

    Tokens that continue a partially filled page reuse that page's scale
    (`prev_scale`, [H]) and saturate; every newly started page gets
    scale = max(amax / 448, tiny) with amax taken over the tokens this append puts
    into that page, separately per KV head.  code = round_to_e4m3(x * (1 / scale)).

    Returns (codes uint8 [n, H, D], new_page_scales fp32 [n_new_pages, H]).
    """
    n, H, D = x.shape
    codes = torch.empty((n, H, D), dtype=torch.uint8, device=x.device)
    head = 0
    if first_slot % page_size != 0:
        head = min(n, page_size - first_slot % page_size)
        if prev_scale is None:
            raise ValueError("continuing a partial page needs that page's scale")
        inv = (1.0 / prev_scale.detach().to("cpu", torch.float32)).to(x.device)
        codes[:head] = encode_e4m3(x[:head] * inv.reshape(1, H, 1))
    rest = n - head
    n_new = (rest + page_size - 1) // page_size
    scales = torch.empty((n_new, H), dtype=torch.float32, device=x.device)
    if rest > 0:
        full = rest // page_size
        if full:
            blk = x[head:head + full * page_size].reshape(full, page_size, H, D)
            s, inv = _scale_and_inverse(blk.abs().amax(dim=(1, 3)))
            scales[:full] = s
            codes[head:head + full * page_size] = encode_e4m3(
                blk * inv.reshape(full, 1, H, 1)).reshape(full * page_size, H, D)
        if rest % page_size:
            tail = x[head + full * page_size:]
            s, inv = _scale_and_inverse(tail.abs().amax(dim=(0, 2)))
            scales[full] = s
            codes[head + full * page_size:] = encode_e4m3(tail * inv.reshape(1, H, 1))
    return codes, scales
