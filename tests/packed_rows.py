"""Test helper: the packed stream of a sub-matrix made of whole 16-row tiles.

Tiles (16 rows x 256 columns; 512 columns for the 3-bit width) are stored k-tile major: tile (row tile r,
k-tile t) of an M x K matrix is tile number t * (M/16) + r of the stream.  The stream of the sub-matrix that keeps only the listed row tiles, in
the listed order, is therefore, for every k-tile in turn, those row tiles' bytes - what the oracle produces
when it packs the listed rows as a matrix of their own.
"""
import numpy as np
import torch


def row_tiles_of(packed: torch.Tensor, M: int, K: int, tiles, tile_bytes: int, tile_cols: int = 256) -> np.ndarray:
    """packed: uint8 device (or host) tensor of an M x K matrix; tiles: row-tile indices; tile_bytes: bytes of
    one 16 x tile_cols tile at the stream's width (3072 for 6 bits).  Returns the sub-matrix's stream (numpy)."""
    idx = torch.as_tensor(np.asarray(tiles, dtype=np.int64), device=packed.device)
    view = packed.view(-(-K // tile_cols), M // 16, tile_bytes)
    return view[:, idx, :].reshape(-1).cpu().numpy()
