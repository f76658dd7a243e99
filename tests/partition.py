"""The sampler's column partition that the HIP library fixes, read from include/e3.h
(E3_TILE_CHUNK, E3_TILE_LANES, E3_TILE_DEPTH).  The oracle takes the partition as an
argument; tests that compare the library with it pass this one."""
import os
import re

_HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "e3.h")


def _read():
    text = open(_HEADER).read()
    return tuple(int(re.search(rf"#define {k} (\d+)", text).group(1))
                 for k in ("E3_TILE_CHUNK", "E3_TILE_LANES", "E3_TILE_DEPTH"))


LIB_PARTITION = _read()
