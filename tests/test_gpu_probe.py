"""The streaming-read probe (include/gh_probe.h) reads every tile of every wave exactly once.

The probe is a measurement aid, but the ceiling it reports is only worth something if its loop
really streams the whole buffer: each lane XORs the words it loads, and the kernel writes `sink`
only when the last lane of a wave ends on a magic value.  One magic word planted in that lane's
share of one tile must therefore reach `sink`, wherever the tile lies (first, last, odd, even),
with or without stores and with one or two waves per SIMD; planted twice it cancels out.
"""
import numpy as np
import pytest
import torch

from paper_2501_11779_amd import binding as G

pytestmark = pytest.mark.gpu
DEV = "cuda"
MAGIC = 0x9E3779B9
TILE_WORDS = 4096                      # a 16 KiB tile in 32-bit words


def _word_of(wave, tile, tiles_per_wave, load, lane=63, j=0):
    """Index of word j of the 16 bytes `lane` gets from load instruction `load` of a tile."""
    return ((wave * tiles_per_wave + tile) * TILE_WORDS) + (load * 64 + lane) * 4 + j


def _run(src, n_waves, every, policy):
    rec = torch.zeros(n_waves * 1024, dtype=torch.int32, device=DEV)
    sink = torch.zeros(1, dtype=torch.int32, device=DEV)
    G.check(G.gh_probe_stream_read(src, src.numel() * 4, n_waves, every, policy, rec, sink))
    torch.cuda.synchronize()
    return int(sink.item()) & 0xFFFFFFFF


@pytest.mark.parametrize("n_waves,every,policy", [
    (1024, 0, 0), (2048, 0, 0), (64, 0, 0),
    (1024, 4, G.GH_PROBE_STORE_PLAIN), (1024, 2, G.GH_PROBE_STORE_NT),
    (2048, 4, G.GH_PROBE_STORE_WRITE_THROUGH)])
def test_every_tile_is_read_once(n_waves, every, policy):
    tiles_per_wave = 6
    n_words = n_waves * tiles_per_wave * TILE_WORDS
    rng = np.random.default_rng(n_waves + every)
    places = [(0, 0, 0), (n_waves - 1, tiles_per_wave - 1, 15), (n_waves // 2, 1, 7), (3, 4, 2),
              (int(rng.integers(n_waves)), int(rng.integers(tiles_per_wave)), int(rng.integers(16)))]
    for wave, tile, load in places:
        src = torch.zeros(n_words, dtype=torch.int32, device=DEV)
        at = _word_of(wave, tile, tiles_per_wave, load)
        src[at] = MAGIC - (1 << 32)
        assert _run(src, n_waves, every, policy) == MAGIC, (wave, tile, load)
        # the same word in a second tile of the same wave cancels the first
        other = _word_of(wave, (tile + 1) % tiles_per_wave, tiles_per_wave, load)
        src[other] = MAGIC - (1 << 32)
        assert _run(src, n_waves, every, policy) == 0, (wave, tile, load)


def test_sizes_that_do_not_divide_are_refused():
    src = torch.zeros(1024 * 2 * TILE_WORDS + 4, dtype=torch.int32, device=DEV)
    sink = torch.zeros(1, dtype=torch.int32, device=DEV)
    st = G.gh_probe_stream_read(src, src.numel() * 4, 1024, 0, 0, None, sink)
    assert st == G.GH_ERR_SHAPE
