"""Host logic of the H = 128 scan's schedule (bppsa_scan_h128_schedule): no device work, so these run
without a GPU (the library then assumes 256 compute units)."""
import ctypes
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1907_10134_amd", "libbppsa.so")

S = 64


class Schedule(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in ("segment_steps", "segments", "chain_steps", "slab_segments", "slabs",
                                              "last_slab_steps")] + \
               [("matrix_products", ctypes.c_int64), ("model_us", ctypes.c_double)]


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    lib = ctypes.CDLL(LIB)
    lib.bppsa_scan_h128_schedule.restype = ctypes.c_int
    lib.bppsa_scan_h128_schedule.argtypes = [ctypes.c_int] * 4 + [ctypes.POINTER(Schedule)]
    return lib


def _schedule(lib, T, B, want_g0, generated):
    out = Schedule()
    assert lib.bppsa_scan_h128_schedule(T, B, int(want_g0), int(generated), ctypes.byref(out)) == 0
    return out


def _products_below_chain(segments_below, slab, last, B):
    """Matrix-matrix products of the documented walk: slabs of `slab` segments from the chain
    downwards, segment 0 (no total) riding with the last slab, which may be cut into segments of
    `last` steps."""
    total = 0
    hi = segments_below - 1
    while hi >= 0:
        lo = hi - slab + 1
        if lo <= 1:
            lo = 0
        rlo = max(lo, 1)
        if lo == 0 and last < S:
            total += ((hi + 1) * (S // last) - 1) * (last - 1)
        elif hi >= rlo:
            total += (hi - rlo + 1) * (S - 1)
        hi = lo - 1
    return total * B


@pytest.mark.parametrize("generated", [False, True])
@pytest.mark.parametrize("want_g0", [False, True])
@pytest.mark.parametrize("T,B", [(4096, 16), (2304, 16), (700, 64), (11000, 3), (300, 3), (1000, 2), (129, 33),
                                 (65, 1), (66, 1), (30000, 16), (3000, 64), (513, 127), (4096, 1)])
def test_schedule_accounts_for_every_step(lib, T, B, want_g0, generated):
    s = _schedule(lib, T, B, want_g0, generated)
    n = T - (0 if want_g0 else 1)
    assert s.segment_steps == S
    assert s.segments == -(-n // S)
    top = n - (s.segments - 1) * S                   # the segment nearest the seed may be shorter
    assert top <= s.chain_steps <= n
    assert (s.chain_steps - top) % S == 0
    chain_segments = 1 + (s.chain_steps - top) // S
    below = s.segments - chain_segments
    if below == 0:
        assert s.slabs == 0 and s.matrix_products == 0
        return
    assert s.slab_segments >= 1 and 1 <= s.slabs <= 32
    assert s.slab_segments * B <= 256 - B or s.slabs == 32      # a slab fits beside the serial chains
    assert s.last_slab_steps in (16, 32, 64)
    assert s.matrix_products == _products_below_chain(below, s.slab_segments, s.last_slab_steps, B)
    assert s.model_us > 0


def test_short_chains_are_one_matrix_vector_pass(lib):
    for T, g0 in ((1, False), (1, True), (64, True), (65, False)):
        s = _schedule(lib, T, 4, g0, False)
        assert s.chain_steps == T - (0 if g0 else 1) and s.slabs == 0 and s.matrix_products == 0


def test_a_batch_that_fills_the_device_gets_no_serial_chain(lib):
    """With more than half as many samples as compute units there is no unit left per sample: the
    totals of all interior segments are formed at once and scanned recursively."""
    T, B = 1000, 200
    s = _schedule(lib, T, B, False, False)
    nseg = -(-(T - 1) // S)
    assert s.slabs == 0 and s.chain_steps == (T - 1) - (nseg - 1) * S
    assert s.matrix_products == (nseg - 2) * (S - 1) * B          # one level: nseg - 2 <= 64 totals


def test_generated_jacobians_get_the_longer_chain(lib):
    """A step of the serial chain is cheaper when nothing is read from memory, so more of the chain
    is walked serially and fewer matrix-matrix products are spent."""
    stored = _schedule(lib, 4096, 16, False, False)
    gen = _schedule(lib, 4096, 16, False, True)
    assert gen.chain_steps > stored.chain_steps
    assert gen.matrix_products < stored.matrix_products
    # both spend well under the (nseg - 2)(S - 1) B products of the form without a serial chain
    assert stored.matrix_products < 62 * 63 * 16


def test_schedule_rejects_bad_arguments(lib):
    out = Schedule()
    assert lib.bppsa_scan_h128_schedule(0, 1, 0, 0, ctypes.byref(out)) != 0
    assert lib.bppsa_scan_h128_schedule(10, 0, 0, 0, ctypes.byref(out)) != 0
    assert lib.bppsa_scan_h128_schedule(10, 1, 0, 0, None) != 0
