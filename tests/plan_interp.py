"""Host interpreter of the library's copy descriptors and tiles, exactly as the header
documents them (byte (b, r, i) of the source goes to the same (b, r, i) of the
destination).  Test-side only; lets the planner be checked without a GPU."""
import numpy as np


def run_descs(descs, src_u8: np.ndarray, dst_u8: np.ndarray) -> None:
    for d in descs:
        for b in range(d.n_blocks):
            for r in range(d.rows):
                s = d.src_off + b * d.src_block_stride + r * d.src_row_stride
                t = d.dst_off + b * d.dst_block_stride + r * d.dst_row_stride
                dst_u8[t:t + d.row_bytes] = src_u8[s:s + d.row_bytes]


def run_tiles(tiles, src_u8: np.ndarray, dst_u8: np.ndarray) -> None:
    """tiles: [(hf_tile, [destination offsets])] as Plan.tiles() returns them."""
    for tl, dsts in tiles:
        assert len(dsts) == tl.n_dst
        if tl.n_dst == 0:          # a load-only tile: read, written nowhere; the source must exist
            assert tl.src_off + (tl.rows - 1) * tl.src_row_stride + tl.row_bytes <= src_u8.shape[0]
            assert tl.dst_list in (0, tl.rows)                    # plain or chunked form
            continue
        assert dsts[0] == tl.dst_off
        for r in range(tl.rows):
            s = tl.src_off + r * tl.src_row_stride
            for d in dsts:
                t = d + r * tl.dst_row_stride
                dst_u8[t:t + tl.row_bytes] = src_u8[s:s + tl.row_bytes]
