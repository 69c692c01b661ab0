"""Blocked tensor layouts written out as index identities.  TEST INFRASTRUCTURE ONLY.

The index expressions of the paper's Fig. 4 (Section 5) fix the layouts, with
GEMM_BLOCK = B = 16 (Section 5.1: 16 fp32 values fill one 512-bit vector, so channel widths
are tiled by 16):

    input  [img][ifm_tile][ij][ii][ifm]              = NCHW[img][ifm_tile*B + ifm][ij][ii]
    filter [ofm_tile][ifm_tile][kj][ki][ifm][ofm]    = KCRS[ofm_tile*B + ofm][ifm_tile*B + ifm][kj][ki]
    output [img][ofm_tile][oj][oi][ofm]              = NKPQ[img][ofm_tile*B + ofm][oj][oi]

Reading where the paper is silent: it only evaluates layers whose channel counts are
multiples of 16.  Here an input-channel count that is not a multiple of 16 is padded up with
+0.0 lanes; output-channel counts must be multiples of 16.

bf16 is not in the paper.  For 2-byte elements the 16x16 filter block is stored [c/8][16 k][8 c]
instead of [16 c][16 k]: the same 256 values, permuted so that the 8 input channels a matrix-core
lane multiplies are contiguous (the reduction index must be packed for 16-bit operands, the same
idea as the channel-pair packing CPU libraries use for bf16).  Activations and outputs keep the
order above.

Every function is a pure permutation (plus zero fill) and keeps the dtype, so results can be
compared bit for bit.
"""
from __future__ import annotations

import numpy as np

B = 16


def _blocks(c: int) -> int:
    return -(-c // B)


def act_to_blocked(x: np.ndarray) -> np.ndarray:
    """[N][C][H][W] -> [N][ceil(C/16)][H][W][16]; lanes beyond C hold +0.0."""
    N, C, H, W = x.shape
    blk = np.zeros((N, _blocks(C), H, W, B), dtype=x.dtype)
    for c in range(C):
        blk[:, c // B, :, :, c % B] = x[:, c, :, :]
    return blk


def blocked_to_act(blk: np.ndarray, C: int) -> np.ndarray:
    """Inverse of act_to_blocked; drops the pad lanes."""
    N, Cb, H, W, b = blk.shape
    assert b == B and Cb == _blocks(C)
    x = np.empty((N, C, H, W), dtype=blk.dtype)
    for c in range(C):
        x[:, c, :, :] = blk[:, c // B, :, :, c % B]
    return x


def filt_to_blocked(w: np.ndarray) -> np.ndarray:
    """[K][C][R][S] -> [K/16][ceil(C/16)][R][S][16 c][16 k]; c lanes beyond C hold +0.0."""
    K, C, R, S = w.shape
    if K % B:
        raise ValueError("output channels must be a multiple of 16")
    blk = np.zeros((K // B, _blocks(C), R, S, B, B), dtype=w.dtype)
    for c in range(C):
        for kk in range(B):
            # all output-channel tiles at once: k = ofm_tile*16 + kk
            blk[:, c // B, :, :, c % B, kk] = w[kk::B, c, :, :]
    return blk


def blocked_to_filt(blk: np.ndarray, C: int) -> np.ndarray:
    Kb, Cb, R, S, b1, b2 = blk.shape
    assert b1 == B and b2 == B and Cb == _blocks(C)
    w = np.empty((Kb * B, C, R, S), dtype=blk.dtype)
    for c in range(C):
        for kk in range(B):
            w[kk::B, c, :, :] = blk[:, c // B, :, :, c % B, kk]
    return w


def filt_to_blocked_packed8(w: np.ndarray) -> np.ndarray:
    """[K][C][R][S] -> [K/16][ceil(C/16)][R][S][2 (c/8)][16 k][8 (c%8)]: the 2-byte-element filter layout."""
    std = filt_to_blocked(w)                                   # [Kb][Cb][R][S][16 c][16 k]
    Kb, Cb, R, S = std.shape[:4]
    out = np.zeros((Kb, Cb, R, S, 2, B, 8), dtype=w.dtype)
    for c in range(B):
        for k in range(B):
            out[:, :, :, :, c // 8, k, c % 8] = std[:, :, :, :, c, k]
    return out


def blocked_packed8_to_filt(blk: np.ndarray, C: int) -> np.ndarray:
    Kb, Cb, R, S = blk.shape[:4]
    std = np.zeros((Kb, Cb, R, S, B, B), dtype=blk.dtype)
    for c in range(B):
        for k in range(B):
            std[:, :, :, :, c, k] = blk[:, :, :, :, c // 8, k, c % 8]
    return blocked_to_filt(std, C)


def out_to_blocked(y: np.ndarray) -> np.ndarray:
    """[N][K][P][Q] -> [N][K/16][P][Q][16]."""
    if y.shape[1] % B:
        raise ValueError("output channels must be a multiple of 16")
    return act_to_blocked(y)


def blocked_to_out(blk: np.ndarray) -> np.ndarray:
    """[N][K/16][P][Q][16] -> [N][K][P][Q]."""
    return blocked_to_act(blk, blk.shape[1] * B)
