"""Pins of the oracle's index coder (CPU only).  The paper names its coder and the
rates it reaches but not the algorithm, so what can be pinned is: the round trip is
lossless, the size lies between the information bound and the paper's reached rates
on uniformly random index sets, and the bits of a small record worked out by hand."""
import math
import os

import numpy as np
import pytest

FLAT, TILE = 0, 1
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_numbers.txt")


def paper_numbers():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def make_payload(oracle, descs, k, rng, idx_fn=None):
    """A plain-format payload with random LUTs, index sets and codes."""
    pay = np.zeros(oracle.payload_bytes(descs, k), dtype=np.uint8)
    off = 0
    for d in descs:
        nc = oracle.tensor_chunks(d)
        pay[off:off + 16] = rng.normal(0, 1e-3, 4).astype(np.float32).view(np.uint8)
        for c in range(nc):
            idx = np.sort(rng.choice(4096, k, replace=False)) if idx_fn is None else idx_fn(c)
            code = rng.integers(0, 4, k)
            pay[off + 16 + c * 7 * k // 4: off + 16 + (c + 1) * 7 * k // 4] = oracle.pack_record(idx, code)
        off += oracle.tensor_block_bytes(d, k)
    return pay


def test_rice_parameter_rule(oracle):
    assert [oracle.rice_param(k) for k in (4, 32, 64, 128, 256, 1024, 2048, 2840, 4096)] == \
        [9, 6, 5, 4, 3, 1, 0, 0, 0]


def bits_to_bytes(bits):
    out = bytearray((len(bits) + 7) // 8)
    for i, b in enumerate(bits):
        out[i // 8] |= b << (i % 8)
    return bytes(out)


def test_rice_hand_worked_record(oracle):
    """k = 4 (b = 9), indices 3, 600, 601, 4095 -> gaps 3, 596, 0, 3493, written out by hand:
    quotient in unary (ones, then a zero), remainder 9 bits LSB first; then the 2-bit codes."""
    descs = [(1, 4096, 0, FLAT)]
    pay = np.zeros(oracle.payload_bytes(descs, 4), dtype=np.uint8)
    pay[:16] = np.array([-2.0, -1.0, 1.0, 2.0], dtype=np.float32).view(np.uint8)
    pay[16:23] = oracle.pack_record([3, 600, 601, 4095], [0, 1, 2, 3])
    enc = oracle.rice_encode(descs, 4, pay)
    s = ("0" "110000000"            # gap 3    = 0*512 + 3
         "10" "001010100"           # gap 596  = 1*512 + 84,  84 = 0b001010100 -> LSB first
         "0" "000000000"            # gap 0
         "1111110" "101001011"      # gap 3493 = 6*512 + 421, 421 = 0b110100101 -> LSB first
         "00" "10" "01" "11")       # codes 0, 1, 2, 3, LSB first
    stream = bits_to_bytes([int(ch) for ch in s])
    assert len(s) == 55 and len(stream) == 7
    # header 16 + 8*1 -> 32; block: LUT 16, one group offset (= 20), stream padded to 4 bytes, block to 16
    assert enc[:8].tobytes() == b"SLRICE01"
    assert int(enc[8:16].view(np.uint64)[0]) == enc.size == 32 + 32
    assert int(enc[16:24].view(np.uint64)[0]) == 32
    blk = enc[32:]
    assert np.array_equal(blk[:16], pay[:16])
    assert int(blk[16:20].view(np.uint32)[0]) == 20
    assert blk[20:27].tobytes() == stream and not blk[27:].any()
    assert np.array_equal(oracle.rice_decode(descs, 4, enc), pay)


@pytest.mark.parametrize("k", [4, 8, 32, 64, 100, 128, 256, 1000, 4096])
def test_rice_round_trip(oracle, k):
    rng = np.random.default_rng(900 + k)
    shapes = [(150, 210, TILE), (1, 4096 * 37 + 1100, FLAT), (64, 64, TILE), (1024, 16, TILE)] if k <= 256 \
        else [(160, 224, TILE), (1, 4096 * 3, FLAT)] if k <= 1024 else [(128, 128, TILE), (1, 4096, FLAT)]
    descs, off = [], 0
    for r, c, lay in shapes:
        descs.append((r, c, off, lay))
        off += (r * c + 63) // 64 * 64
    pay = make_payload(oracle, descs, k, rng)
    enc = oracle.rice_encode(descs, k, pay)
    assert enc.size <= oracle.rice_max_bytes(descs, k)
    assert np.array_equal(oracle.rice_decode(descs, k, enc), pay)
    nt = len(descs)
    assert enc[:8].tobytes() == b"SLRICE01" and int(enc[8:16].view(np.uint64)[0]) == enc.size
    toffs = enc[16:16 + 8 * nt].view(np.uint64)
    assert all(int(t) % 16 == 0 for t in toffs) and list(toffs) == sorted(toffs)
    for t, d in zip(toffs, descs):
        ng = (oracle.tensor_chunks(d) + 7) // 8
        goff = enc[int(t) + 16:int(t) + 16 + 4 * ng].view(np.uint32)
        assert goff[0] == 16 + 4 * ng and all(int(g) % 4 == 0 for g in goff) and np.all(np.diff(goff.astype(np.int64)) > 0)


def test_rice_extreme_index_sets(oracle):
    """First k, last k, one cluster, and the largest possible gaps: still lossless and within the bound."""
    k = 32
    descs = [(1, 4096 * 64, 0, FLAT)]
    rng = np.random.default_rng(3)
    sets = [np.arange(k), np.arange(4096 - k, 4096), np.arange(2000, 2000 + k),
            np.concatenate([[0], np.arange(4096 - k + 1, 4096)]), np.arange(k) * 128, np.arange(k) * 128 + 127]

    def idx_fn(c):
        return sets[c % len(sets)]
    pay = make_payload(oracle, descs, k, rng, idx_fn)
    enc = oracle.rice_encode(descs, k, pay)
    assert enc.size <= oracle.rice_max_bytes(descs, k)
    assert np.array_equal(oracle.rice_decode(descs, k, enc), pay)


def test_rice_rate_between_bound_and_paper(oracle):
    """Uniformly random index sets: bits per index above the information bound
    log2 C(4096,k)/k and not above what the paper's own coder reaches (8.9 / 6.6 / 5.6)."""
    p = paper_numbers()
    rng = np.random.default_rng(4)
    for k in (32, 128, 256):
        nc = 1600
        descs = [(1, 4096 * nc, 0, FLAT)]
        pay = make_payload(oracle, descs, k, rng)
        enc = oracle.rice_encode(descs, k, pay)
        bits = enc.size * 8 / (nc * k) - p["value_bits"]
        bound = (math.lgamma(4097) - math.lgamma(k + 1) - math.lgamma(4097 - k)) / math.log(2) / k
        assert abs(bound - p["entropy_bits_k%d" % k]) < 0.1
        assert bound < bits <= p["coder_bits_k%d" % k], (k, bits)
        assert bits < p["naive_index_bits"]
    # Table 1 context: 512M-parameter model at k = 32 would need less than the paper's 5.45 MB
    n_values = int(p["params_512M"]) * 32 / 4096
    assert n_values * (bits_k32(oracle) + 2) / 8 / 1e6 < p["table1_size_MB_density_0p78"]


def bits_k32(oracle):
    rng = np.random.default_rng(5)
    nc = 800
    descs = [(1, 4096 * nc, 0, FLAT)]
    enc = oracle.rice_encode(descs, 32, make_payload(oracle, descs, 32, rng))
    return enc.size * 8 / (nc * 32) - 2


# --------------------------------------------------------------------------- other value widths
def make_payload_b(oracle, descs, k, bits, rng):
    pay = np.zeros(oracle.payload_bytes_b(descs, k, bits), dtype=np.uint8)
    hdr, rec, off = oracle.header_bytes_b(bits), oracle.record_bytes_b(k, bits), 0
    for d in descs:
        if bits != 32:
            pay[off:off + 4 * (1 << bits)] = rng.normal(0, 1e-3, 1 << bits).astype(np.float32).view(np.uint8)
        for c in range(oracle.tensor_chunks(d)):
            idx = np.sort(rng.choice(4096, k, replace=False))
            sent = rng.normal(0, 1e-3, k).astype(np.float32) if bits == 32 else rng.integers(0, 1 << bits, k)
            pay[off + hdr + c * rec: off + hdr + (c + 1) * rec] = oracle.pack_record_b(idx, sent, bits)
        off += oracle.tensor_block_bytes_b(d, k, bits)
    return pay


def test_rice_two_bits_is_the_pinned_coder(oracle):
    rng = np.random.default_rng(950)
    descs = [(150, 210, 0, TILE), (1, 4096 * 9 + 1100, 150 * 210 + 20, FLAT)]
    for k in (4, 32, 64, 100):
        pay = make_payload(oracle, descs, k, rng)
        enc = oracle.rice_encode(descs, k, pay)
        assert np.array_equal(oracle.rice_encode_b(descs, k, 2, pay), enc)
        assert np.array_equal(oracle.rice_decode_b(descs, k, 2, enc), pay)
        assert oracle.rice_max_bytes_b(descs, k, 2) == oracle.rice_max_bytes(descs, k)


@pytest.mark.parametrize("bits", [1, 3, 4, 32])
def test_rice_other_widths_stream_model_and_round_trip(oracle, bits):
    """One tensor of 11 chunks (two groups): the coded block is the table, the group offsets and,
    per group, the chunks' gap codes (the pinned 2-bit coder's, unchanged) each followed by the k
    value fields of `bits` bits - rebuilt here bit by bit from the records."""
    k, nc = 16, 11
    b = oracle.rice_param(k)
    descs = [(1, 4096 * nc, 0, FLAT)]
    rng = np.random.default_rng(960 + bits)
    pay = make_payload_b(oracle, descs, k, bits, rng)
    enc = oracle.rice_encode_b(descs, k, bits, pay)
    assert enc.size <= oracle.rice_max_bytes_b(descs, k, bits)
    assert np.array_equal(oracle.rice_decode_b(descs, k, bits, enc), pay)
    hdr, rec = oracle.header_bytes_b(bits), oracle.record_bytes_b(k, bits)
    assert enc[:8].tobytes() == b"SLRICE01" and int(enc[8:16].view(np.uint64)[0]) == enc.size
    blk = enc[int(enc[16:24].view(np.uint64)[0]):]
    assert np.array_equal(blk[:hdr], pay[:hdr])
    goff = blk[hdr:hdr + 8].view(np.uint32)
    assert goff[0] == hdr + 8
    for g, (lo, hi) in enumerate(((0, 8), (8, 11))):
        stream = []
        for c in range(lo, hi):
            idx, sent = oracle.unpack_record_b(pay[hdr + c * rec: hdr + (c + 1) * rec], k, bits)
            prev = -1
            for v in idx.astype(int):
                gap = v - prev - 1
                prev = v
                stream += [1] * (gap >> b) + [0] + [(gap >> i) & 1 for i in range(b)]
            fields = sent.view(np.uint32) if bits == 32 else sent
            for f in fields.astype(np.uint64):
                stream += [(int(f) >> i) & 1 for i in range(bits)]
        want = bits_to_bytes(stream)
        at = int(goff[g])
        assert blk[at:at + len(want)].tobytes() == want, (bits, g)
        end = int(goff[1]) if g == 0 else blk.size
        if g == 0:
            assert end - at == (len(want) + 3) // 4 * 4          # a group is padded to 4 bytes
        assert not blk[at + len(want):end].any()


@pytest.mark.parametrize("bits", [1, 3, 4, 32])
@pytest.mark.parametrize("k", [8, 64, 104, 1024])
def test_rice_other_widths_round_trip(oracle, bits, k):
    rng = np.random.default_rng(970 + bits + k)
    shapes = [(150, 210, TILE), (1, 4096 * 19 + 1100, FLAT), (1024, 16, TILE)] if k <= 256 else [(160, 224, TILE), (1, 4096 * 3, FLAT)]
    descs, off = [], 0
    for r, c, lay in shapes:
        descs.append((r, c, off, lay))
        off += (r * c + 63) // 64 * 64
    pay = make_payload_b(oracle, descs, k, bits, rng)
    enc = oracle.rice_encode_b(descs, k, bits, pay)
    assert enc.size <= oracle.rice_max_bytes_b(descs, k, bits)
    assert np.array_equal(oracle.rice_decode_b(descs, k, bits, enc), pay)
