"""CPU checks of the weight packers against the layout the header documents: a [rows, K] output-major
bf16 matrix is stored as [ceil(rows/128)][K/32][128][32] with zero padding, w_gate_up is the tiled
gate matrix followed by the tiled up matrix, fp32 matrices are plain, and unpack inverts pack."""
import numpy as np
import torch

from paper_2602_21140_amd import pack_expert, pack_router, unpack_expert


def _documented_position(r, k, K):
    return ((r // 128 * (K // 32) + k // 32) * 128 + r % 128) * 32 + k % 32


def test_bf16_tiled_layout_matches_the_documented_formula():
    torch.manual_seed(0)
    H, I = 192, 320                      # rows not a multiple of 128 on either matrix
    gate = torch.randn(H, I).to(torch.bfloat16)
    up = torch.randn(H, I).to(torch.bfloat16)
    down = torch.randn(I, H).to(torch.bfloat16)
    gu, dn = pack_expert(gate, up, down)
    gu, dn = gu.flatten(), dn.flatten()
    pad_i, pad_h = 384, 256
    assert gu.numel() == 2 * pad_i * H and dn.numel() == pad_h * I
    rng = np.random.default_rng(1)
    for _ in range(300):
        i, h = int(rng.integers(I)), int(rng.integers(H))
        # output-major: gate row i holds the H weights producing intermediate i
        assert gu[_documented_position(i, h, H)] == gate[h, i]
        assert gu[pad_i * H + _documented_position(i, h, H)] == up[h, i]
        assert dn[_documented_position(h, i, I)] == down[i, h]
    # padding rows are zero
    for r in (I, pad_i - 1):
        for k in (0, H - 1):
            assert gu[_documented_position(r, k, H)] == 0
    assert dn[_documented_position(H, 0, I)] == 0 and dn[_documented_position(pad_h - 1, I - 1, I)] == 0
    g2, u2, d2 = unpack_expert(*pack_expert(gate, up, down), H, I)
    assert torch.equal(g2, gate) and torch.equal(u2, up) and torch.equal(d2, down)


def test_fp32_layout_is_plain_output_major():
    torch.manual_seed(1)
    H, I = 24, 12
    gate, up, down = torch.randn(H, I), torch.randn(H, I), torch.randn(I, H)
    gu, dn = pack_expert(gate, up, down)
    assert gu.shape == (2 * I, H) and dn.shape == (H, I)
    assert torch.equal(gu[:I], gate.t()) and torch.equal(gu[I:], up.t()) and torch.equal(dn, down.t())
    g2, u2, d2 = unpack_expert(gu, dn, H, I)
    assert torch.equal(g2, gate) and torch.equal(u2, up) and torch.equal(d2, down)


def test_router_is_plain_output_major():
    w = torch.randn(16, 5)
    assert torch.equal(pack_router(w), w.t().contiguous())
