"""Pins for the packed-format half of the CPU oracle and for the byte accounting (no GPU)."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import sfmp_oracle as O
import sfmp_workloads as W


@pytest.mark.parametrize("b", [2, 3, 4])
def test_tile_size_and_every_bit_written_exactly_once(b):
    pos = O.tile_bit_positions(b)
    assert pos.shape == (128, 128, b)
    flat = np.sort(pos.ravel())
    assert O.tile_bytes(b) == 2048 * b == 128 * 128 * b // 8
    assert np.array_equal(flat, np.arange(O.tile_bytes(b) * 8))  # a bijection: no gap, no overlap


def test_hand_derived_bit_locations(golden):
    for b, r, c, t, bit_index in golden("format_locations.txt")["rows"]:
        assert O.code_bit_position(b, r, c, t) == bit_index, (b, r, c, t)


@pytest.mark.parametrize("b", [2, 3, 4])
def test_single_code_sets_exactly_its_bits(b, golden):
    # one non-zero code in an otherwise zero tile -> exactly popcount(code) bits set, where the fixture says
    rows = [row for row in golden("format_locations.txt")["rows"] if row[0] == b]
    for _, r, c, t, bit_index in rows:
        tile = np.zeros((128, 128), dtype=np.uint8)
        tile[r, c] = 1 << t
        packed = O.pack_tile(tile, b)
        bits = np.unpackbits(packed, bitorder="little")
        assert bits.sum() == 1 and bits[bit_index] == 1
        # little-endian 32-bit word view agrees with the byte/bit view
        words = packed.view("<u4")
        assert words[bit_index // 32] == np.uint32(1) << np.uint32(bit_index % 32)


def test_slab_major_layout():
    # slab sigma = rows {8i + sigma} occupies bytes [sigma*256b, (sigma+1)*256b); inside it lane l owns the
    # 4b contiguous bytes at l*4b, so one load of 4b bytes per lane reads a contiguous 256b-byte segment
    for b in (2, 3, 4):
        pos = O.tile_bit_positions(b)
        byte = pos // 8
        r = np.arange(128)[:, None, None]
        c = np.arange(128)[None, :, None]
        lane_of = 16 * ((c % 32) // 8) + r // 8
        assert np.array_equal(byte // (256 * b), np.broadcast_to(r % 8, byte.shape))
        assert np.array_equal((byte % (256 * b)) // (4 * b), np.broadcast_to(lane_of, byte.shape))


@settings(max_examples=25, deadline=None)
@given(st.integers(0, 2 ** 31 - 1), st.sampled_from([2, 3, 4]))
def test_tile_roundtrip(seed, b):
    rng = np.random.default_rng(seed)
    tile = rng.integers(0, 1 << b, size=(128, 128)).astype(np.uint8)
    packed = O.pack_tile(tile, b)
    assert packed.dtype == np.uint8 and packed.size == 2048 * b
    assert np.array_equal(O.unpack_tile(packed, b), tile)


@settings(max_examples=8, deadline=None)
@given(st.integers(0, 2 ** 31 - 1), st.integers(1, 3), st.integers(1, 3))
def test_matrix_roundtrip_and_stream_sizes(seed, ntr, ntc):
    rng = np.random.default_rng(seed)
    bitmap = rng.integers(2, 5, size=(ntr, ntc)).astype(np.int8)
    bm = np.repeat(np.repeat(bitmap, 128, axis=0), 128, axis=1)
    codes = (rng.integers(0, 16, size=bm.shape) % (1 << bm)).astype(np.uint8)
    pk = O.pack(codes, bitmap)
    for b in (2, 3, 4):
        assert pk[f"s{b}"].size == int((bitmap == b).sum()) * 2048 * b
    assert pk["index"].size == O.index_words(ntr, ntc)
    out = O.unpack(ntr * 128, ntc * 128, pk["s2"], pk["s3"], pk["s4"], pk["index"])
    assert np.array_equal(out, codes)


def test_pack_rejects_out_of_range_code():
    tile = np.zeros((128, 128), dtype=np.uint8)
    tile[5, 5] = 4
    with pytest.raises(ValueError):
        O.pack_tile(tile, 2)


def test_hand_derived_index_table(golden):
    g = golden("index_example.txt")
    bitmap = np.array(g["bitmap"], dtype=np.int8).reshape(2, 2)
    assert O.build_index(bitmap).tolist() == g["index"]


def test_streams_hold_tiles_in_row_major_order_per_width():
    bitmap = np.array([[4, 2, 4], [2, 4, 3]], dtype=np.int8)
    codes = np.zeros((256, 384), dtype=np.uint8)
    # mark each tile with a distinct code at its (0,0) element, which lands in bits [0,b) of the tile
    marks = {(0, 0): 9, (0, 1): 1, (0, 2): 10, (1, 0): 2, (1, 1): 11, (1, 2): 5}
    for (tr, tc), v in marks.items():
        codes[tr * 128, tc * 128] = v
    pk = O.pack(codes, bitmap)
    assert [int(pk["s4"][i * 8192]) for i in range(3)] == [9, 10, 11]
    assert [int(pk["s2"][i * 4096]) for i in range(2)] == [1, 2]
    assert int(pk["s3"][0]) == 5


# ---- byte accounting pinned to the paper's closed forms ------------------------------------
def test_metadata_overhead_matches_paper_value():
    # Section 4.2, paragraph "Extra Metadata": 0.006 BPW on LLaMA-3.1-8B with (512,128) blocks.
    shapes = [W.SHAPES_8B[n] for n in W.LAYER_8B]
    bpw = W.metadata_bits_per_weight(shapes)
    assert round(bpw, 3) == 0.006
    assert sum(k * n for k, n in shapes) == 218_103_808  # weights of one decoder layer


def test_scale_zero_overhead_is_quarter_bit_at_group_128():
    # Appendix G (block-size ablation): 16-bit scale and zero per 128 weights = 0.25 bit/weight.
    bitmap = np.full((8, 8), 3, dtype=np.int8)
    N = K = 1024
    total = W.algorithmic_bytes(N, K, 0, bitmap, col_perm=False, row_perm=False)
    sz = total - bitmap.size - N * K * 3 // 8
    assert 8.0 * sz / (N * K) == 0.25


def test_memory_table_slope_832_mib_per_bit():
    # Table 1: LLaMA-3.1-8B memory 4,085 / 4,501 / 4,917 / 5,333 MB at BPW 2.5 / 3.0 / 3.5 / 4.0,
    # i.e. 832 MiB per extra bit = 32 layers x 218.1 M quantised weights / 8 bits.
    per_layer = sum(k * n for k, n in (W.SHAPES_8B[n] for n in W.LAYER_8B))
    mib_per_bit = 32 * per_layer / 8 / 2 ** 20
    assert mib_per_bit == 832.0
    assert (4501 - 4085) / 0.5 == mib_per_bit and (5333 - 4917) / 0.5 == mib_per_bit


def test_algorithmic_bytes_of_8b_layer():
    # 8B decoder layer at an average of 3.0 code bits, M = 1: about 89.1 MB
    total = 0
    for name in W.LAYER_8B:
        K, N = W.SHAPES_8B[name]
        bitmap = W.make_bitmap(N // 128, K // 128, {2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, np.random.default_rng(0))
        total += W.algorithmic_bytes(N, K, 1, bitmap)
    assert abs(total / 1e6 - 89.1) < 0.5, total
