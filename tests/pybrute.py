"""Brute force on tiny inputs, used to pin the C oracle from outside.

Nothing here is imported by the oracle or by the product.  The region is
materialised as a Python `bytes` object by running the SplitMix64 *generator*
(stateful next(), as published) and packing its outputs little-endian; a read
slices 'line_bytes' bytes out of it and sums the 32-bit little-endian words with
struct.unpack.  Indexing, half-word order, window placement and summation are
therefore exercised through real byte addresses rather than through the
oracle's word-index formula.
"""
import struct

M64 = (1 << 64) - 1


class SplitMix64:
    """The generator as published: state += gamma; output = mix(state)."""

    def __init__(self, seed):
        self.state = seed & M64

    def next(self):
        self.state = (self.state + 0x9E3779B97F4A7C15) & M64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
        return z ^ (z >> 31)


def region_bytes(n_bytes, fill_seed):
    g = SplitMix64(fill_seed)
    return b"".join(struct.pack("<Q", g.next()) for _ in range(n_bytes // 8))


def wave_draws(read_seed, w, n_iters):
    """Draws of logical wave w: a generator split off the read seed's generator."""
    parent = SplitMix64(read_seed)
    for _ in range(w):
        parent.next()
    child = SplitMix64(parent.next())
    return [child.next() for _ in range(n_iters)]


def checksum(region, line_bytes, W, I, read_seed, n_windows=1, window_of_group=None, first_wave=0):
    n_lines = len(region) // line_bytes
    lines_per_window = n_lines // n_windows
    G = len(window_of_group) if window_of_group is not None else 1
    total = 0
    touched = []
    for w in range(first_wave, first_wave + W):
        window = window_of_group[w % G] if window_of_group is not None else 0
        for h in wave_draws(read_seed, w, I):
            line = window * lines_per_window + h % lines_per_window
            touched.append(line)
            chunk = region[line * line_bytes:(line + 1) * line_bytes]
            assert len(chunk) == line_bytes
            total += sum(struct.unpack("<%dI" % (line_bytes // 4), chunk))
    return total & M64, touched
