"""Host model of the LDS index maps of the attention kernels (csrc/attn.hip): for every (head_dim, column slices,
workgroup width) the kernels are built for, enumerate every lane's tile writes and fragment reads and check that the
writes are disjoint and inside the tile, that every element a fragment read touches was written by this tile's writes,
and that the merge states fit the area they reuse.  No GPU, no library call: the formulas are restated here from the
kernel source, so a change there that breaks one of these properties has to be made here too, knowingly."""
import itertools

import pytest

from tests.attn_cases import VARIANT_CASES


def geom(D, DV):
    kstr, vstr = D + 8, DV + 16                 # LDS row strides in elements (Geom::KSTR, VSTR)
    return kstr, vstr, 32 * (kstr + vstr)       # one 32-key K tile followed by its V tile (TILE_ELEMS)


def tile_writes(D, DV, n_threads):
    """(element offset, 8 elements) of every 16-byte chunk the threads that fill one tile write."""
    kstr, vstr, _ = geom(D, DV)
    out = []
    for tensor, width, stride, base in (("k", D, kstr, 0), ("v", DV, vstr, 32 * kstr)):
        lanes_per_row = width // 8
        rows_per_pass = n_threads // lanes_per_row
        assert rows_per_pass >= 1 and 32 % rows_per_pass == 0, (tensor, D, DV, n_threads)
        for tid in range(n_threads):
            row, col = tid // lanes_per_row, tid % lanes_per_row
            for j in range(32 // rows_per_pass):
                out.append((tensor, base + (row + j * rows_per_pass) * stride + col * 8))
    return out


def fragment_reads(D, DV):
    """Element ranges the 64 lanes of a wave read for the MFMA operands of one 32-key tile."""
    kstr, vstr, _ = geom(D, DV)
    reads = []
    for lane in range(64):
        c, g = lane & 15, lane >> 4
        for ks in range(D // 32):                                   # K fragments: ds_read_b128
            for half in range(2):
                reads.append(("k", (half * 16 + c) * kstr + ks * 32 + g * 8, 8))
        v_off = 32 * kstr + (g * 4 + (c >> 2)) * vstr + (c & 3) * 4
        for dt in range(DV // 16):                                  # V fragments: two ds_read_b64_tr_b16 per column tile
            reads.append(("v", v_off + dt * 16, 4))
            reads.append(("v", v_off + dt * 16 + 16 * vstr, 4))
    return reads


def check_tile(D, DV, n_threads):
    kstr, vstr, tile_elems = geom(D, DV)
    writes = tile_writes(D, DV, n_threads)
    written = set()
    for tensor, off in writes:
        cells = set(range(off, off + 8))
        assert not (cells & written), (tensor, off)                 # no two chunks overlap
        assert 0 <= off and off + 8 <= tile_elems
        written |= cells
    # exactly the live part of every row: 32 rows x D (K) and 32 rows x DV (V); the padding is never written
    assert len(written) == 32 * D + 32 * DV
    for tensor, off, n in fragment_reads(D, DV):
        assert set(range(off, off + n)) <= written, (tensor, off)   # reads never touch padding or another tile
        assert off % 4 == 0                                         # 8-byte alignment of the narrowest read


WAVE = sorted({(c.head_dim, int(c.variant.split("<")[1].split(",")[2]), int(c.variant.split("<")[1].split(",")[1]),
                int(c.variant.split("<")[1].split(",")[3].rstrip(">")))
               for c in VARIANT_CASES if c.variant.startswith("attn_wave_kernel")})


@pytest.mark.parametrize("D,DS,NW,QT", WAVE)
def test_wave_kernel_tile_and_merge_areas(D, DS, NW, QT):
    """attn_wave_kernel: a wave fills its private tile (64 lanes), and the merge states reuse the tile areas."""
    DV = D // DS
    check_tile(D, DV, 64)
    _, _, tile_elems = geom(D, DV)
    state_floats = QT * (DV // 16) * 256 + QT * 2 * 64              # StateGeom<DV, QT>::STATE_FLOATS
    assert NW * state_floats * 4 <= NW * tile_elems * 2             # what WaveLds asserts at compile time
    # a wave's state: QT*NDT blocks of 64 lanes x 4 floats, then (reference, sum) of 64 lanes per query tile: disjoint
    cells = set()
    for qt, dt, lane in itertools.product(range(QT), range(DV // 16), range(64)):
        base = ((qt * (DV // 16) + dt) * 64 + lane) * 4
        assert not (set(range(base, base + 4)) & cells)
        cells |= set(range(base, base + 4))
    for qt, which, lane in itertools.product(range(QT), range(2), range(64)):
        off = QT * (DV // 16) * 256 + (qt * 2 + which) * 64 + lane
        assert off not in cells
        cells.add(off)
    assert len(cells) == state_floats


@pytest.mark.parametrize("D,n_threads", [(64, 256), (128, 256), (256, 256), (128, 512), (256, 512), (64, 512)])
def test_shared_tile_kernel_tile_area(D, n_threads):
    """attn_bf16_kernel: all threads of the workgroup (4 or 8 waves) fill one tile; with more threads than a tile has
    16-byte chunks (head_dim 64, 512 threads: the two-key-group form) a pass fills n_threads / chunks tiles, thread t
    working on tile t / chunks as thread t % chunks."""
    chunks = 32 * (D // 8)
    check_tile(D, D, min(n_threads, chunks))
    if n_threads > chunks:
        assert n_threads % chunks == 0
        owners = {}
        for tid in range(n_threads):
            owners.setdefault(tid // chunks, set()).add(tid % chunks)
        assert all(v == set(range(chunks)) for v in owners.values()) and len(owners) == n_threads // chunks
