"""Kernel-choice overrides for the GPU tests: the forced tile / pipeline names the tests use,
as cwac_tuning structs for the ``tuning=`` argument of the binding (the _ex entry points)."""
import paper_2505_20932_amd as P

_B = P.binding
_SHAPES = {"8w": _B.CWAC_SHAPE_256_8W, "128x2": _B.CWAC_SHAPE_256_4W_K128, "64x4": _B.CWAC_SHAPE_256_4W_K64,
           "duo": _B.CWAC_SHAPE_128_PAIR, "q": _B.CWAC_SHAPE_128_128, "persist": _B.CWAC_SHAPE_256_PERSIST}


def tuning_of(tile=None, pipe=None, w4_pipe=None, stats_waves=0, persist_workgroups=0, w4_small_waves=0,
              w4_small_depth=0, persist_loaders=0):
    """tile: None | 64 | 128 | 256 (generic kernel with that tile) | "fast" (direct-to-LDS kernel);
    pipe: None | "8w" | "128x2" | "64x4" | "duo" | "q" | "persist" (its tile shape);
    w4_pipe: None | "tile" | "half" | "wide" (weight-only layer: 256- / 128-token tiles of 256 channels, or the
    128-token tile of 512 channels, at every batch size);
    w4_small_waves: 0 | 4 | 8 (wavefronts per workgroup of its weight-streaming kernel), w4_small_depth: 0 | 2 | 3 | 4
    (its ring depth); persist_loaders: 0 | 4 | 8 (wavefronts of the persistent tile that issue its panel loads).
    Returns None when nothing is forced (the plain entry point is then called)."""
    if (tile is None and pipe is None and w4_pipe is None and not stats_waves and not persist_workgroups
            and not w4_small_waves and not w4_small_depth and not persist_loaders):
        return None
    kernel = 0 if tile is None else (_B.CWAC_KERNEL_DIRECT_LDS if tile == "fast" else int(tile))
    return P.make_tuning(kernel=kernel, shape=_SHAPES[pipe] if pipe else 0, stats_waves=stats_waves,
                         w4_tile={None: 0, "tile": 256, "half": 128, "wide": 512}[w4_pipe], w4_small_waves=w4_small_waves, w4_small_depth=w4_small_depth, persist_loaders=persist_loaders,
                         persist_workgroups=persist_workgroups)


def w4_pipes(n, auto=True):
    """The weight-only layer's kernel choices to walk for n output channels (the 512-channel tile needs n >= 512)."""
    return ((None,) if auto else ()) + ("tile", "half") + (("wide",) if n >= 512 else ())
