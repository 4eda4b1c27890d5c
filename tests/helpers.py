"""Test-side helpers: decode the packed ABI layouts with numpy (independent of
both the oracle and the HIP kernels) and move tensors to/from the GPU."""
import numpy as np


def words_u32(t):
    """int32 torch tensor of packed words -> numpy uint32."""
    return t.detach().cpu().numpy().view(np.uint32)


def unpack_planes(words, rows, K, bits, ldw):
    """uint32 [rows][bits][ldw] -> uint8 codes rows x K; also returns the pad-bit population."""
    w = np.asarray(words, np.uint32)[: rows * bits * ldw].reshape(rows, bits, ldw)
    bitsarr = ((w[..., None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(rows, bits, ldw * 32)
    codes = np.zeros((rows, K), np.uint32)
    for t in range(bits):
        codes |= bitsarr[:, t, :K].astype(np.uint32) << t
    pad = int(bitsarr[:, :, K:].sum())
    return codes.astype(np.uint8), pad


def unpack_matrix(words, rows, K, bits):
    ldw = -(-((K + 31) // 32) // 4) * 4
    return unpack_planes(words, rows, K, bits, ldw)


def unpack_fmap(words, N, H, W, C, bits):
    """-> uint8 codes N x C x H x W (the oracle's logical order)."""
    Cw = (C + 31) // 32
    codes, pad = unpack_planes(words, N * H * W, C, bits, Cw)
    return codes.reshape(N, H, W, C).transpose(0, 3, 1, 2).copy(), pad


def pm1_to_bits(a):
    return (np.asarray(a, np.int8) > 0).astype(np.uint8)
