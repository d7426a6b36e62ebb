"""Test-side decoding of the forward workspace (written from the layout
description in the kernel sources, not shared with them).

Fragment order of a tile with R rows and Kc contraction indices, FE elements
per 16-byte fragment (8 bf16 / 4 fp32), KW = 2*FE indices per slab:
  element (row, kidx) lives in fragment ((row//32)*(Kc//KW) + slab)*64 + lane,
  element e, where within the 32-index block b = kidx//32 the index
  kidx%32 = 8*g + 4*h + r maps to accumulator register j = 4*g + r,
  slab = b*(32//KW) + j//FE, e = j%FE, lane = 32*h + row%32.
Accumulator order of a 32x32 block: (row = 8*g + 4*h + r, col) at
  ((g*64 + 32*h + col)*4 + r).
"""
import numpy as np


def frag_index(R, Kc, FE):
    KW = 2 * FE
    row = np.arange(R)[:, None]
    k = np.arange(Kc)[None, :]
    b, wi = k // 32, k % 32
    g, h, r = wi // 8, (wi // 4) % 2, wi % 4
    j = 4 * g + r
    slab = b * (32 // KW) + j // FE
    lane = 32 * h + row % 32
    return (((row // 32) * (Kc // KW) + slab) * 64 + lane) * FE + j % FE


def unfrag(flat, R, Kc, FE):
    """flat [..., R*Kc] in fragment order -> [..., R, Kc]."""
    return flat[..., frag_index(R, Kc, FE)]


def acc_index():
    row = np.arange(32)[:, None]
    col = np.arange(32)[None, :]
    g, h, r = row // 8, (row // 4) % 2, row % 4
    return (g * 64 + 32 * h + col) * 4 + r


def unacc(flat):
    """flat [..., 1024] in accumulator order -> [..., 32 rows, 32 cols]."""
    return flat[..., acc_index()]
