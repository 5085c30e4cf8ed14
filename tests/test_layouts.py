"""Host-side checks of the index maps the n = 4096 kernels are built on (no GPU): every layout assigns each of the
4096 points to exactly one (thread, register); the LDS address map sends the 64-bit accesses of any 16 consecutive
lanes to 16 distinct bank pairs in all three layouts; and the chunk placement of the backward kernel's dy ring puts
under every reader what a loader put there.  The formulas are restated here from csrc/bq_k12_kernel.h and
csrc/bq_bwd.hip; a change there that breaks one of these properties fails here."""
import itertools

import numpy as np


def lane_chunk(lane):
    return lane ^ (3 if lane & 4 else 0)


def lds_addr(idx):
    return idx + 2 * (idx >> 5) + 2 * (idx >> 9)


def base_n(wave, lane):            # layout N: 8 consecutive elements per thread
    return (wave * 64 + lane_chunk(lane)) * 8


def base_p(wave, lane):            # layout P of the forward kernels
    c3 = lane_chunk(lane & 15) & 7
    return (c3 << 7) | (((lane >> 3) & 1) << 2) | (((lane >> 4) & 1) << 1) | (((lane >> 5) & 1) << 3) | (wave << 4)


def base_q(wave, lane):            # layout Q of the backward kernel
    c4 = lane_chunk(lane & 15)
    return ((c4 & 7) << 7) | ((c4 >> 3) << 6) | (((lane >> 4) & 1) << 1) | (((lane >> 5) & 1) << 2) | (wave << 3)


def reg_idx_pq(r):                 # register r of layouts P and Q
    return (r & 1) + 1024 * ((r >> 1) & 1) + 2048 * (r >> 2)


LAYOUTS = {"N": (base_n, lambda r: r), "P": (base_p, reg_idx_pq), "Q": (base_q, reg_idx_pq)}


def test_every_layout_is_a_bijection_onto_the_4096_points():
    for name, (base, reg) in LAYOUTS.items():
        seen = sorted(base(w, l) + reg(r) for w in range(8) for l in range(64) for r in range(8))
        assert seen == list(range(4096)), name


def test_layer_partners_sit_where_the_kernels_look_for_them():
    # DPP lane masks 1, 2, 7, 8 flip chunk bits 0, 1, 2, 3 of the 16-lane row
    for l in range(16):
        for mask, bit in ((1, 0), (2, 1), (7, 2), (8, 3)):
            assert lane_chunk(l ^ mask) == lane_chunk(l) ^ (1 << bit)
    # layout N: layers 4..7 are chunk bits 0..3 (index bits 3..6); layout P: layers 8..10 are index bits 7..9;
    # layout Q: layers 8..10 the same and layer 7 (index bit 6) under mask 8
    for w, l in itertools.product(range(8), range(64)):
        for mask, bit in ((1, 3), (2, 4), (7, 5), (8, 6)):
            assert base_n(w, l ^ mask) == base_n(w, l) ^ (1 << bit)
        for mask, bit in ((1, 7), (2, 8), (7, 9)):
            assert base_p(w, l ^ mask) == base_p(w, l) ^ (1 << bit)
            assert base_q(w, l ^ mask) == base_q(w, l) ^ (1 << bit)
        assert base_q(w, l ^ 8) == base_q(w, l) ^ (1 << 6)


def test_64_bit_lds_accesses_of_16_consecutive_lanes_hit_16_distinct_bank_pairs():
    # a 64-bit access of a lane covers two adjacent floats; 16 lanes x 8 bytes = the 128 bytes the LDS moves per
    # cycle, without conflict if the 16 (even) float addresses differ in bits 1..4
    for name, (base, reg) in LAYOUTS.items():
        for w, g, j in itertools.product(range(8), range(4), range(4)):
            addrs = [lds_addr(base(w, 16 * g + l) + reg(2 * j)) for l in range(16)]
            assert all(a % 2 == 0 for a in addrs), name
            assert len({(a >> 1) & 15 for a in addrs}) == 16, (name, w, g, j)
    # the row buffers' size covers the largest address
    assert max(lds_addr(i) for i in range(4096)) < 4368


def test_dy_ring_readers_find_what_the_loaders_put_there():
    # loader: lane l of wave w writes 16 bytes at 16-byte position 64 w + l of a slot and fetches chunk q_load;
    # reader (layout Q): thread (w, l), register pair j reads the 4 bytes of elements (2j, 2j+1) at position `pos`
    where = {}
    for w, l in itertools.product(range(8), range(64)):
        q = ((l >> 3) & 7) | ((w & 1) << 3) | ((l & 7) << 4) | ((w >> 1) << 7)
        where[q] = 64 * w + l
    assert sorted(where) == list(range(512))
    for w, l, j in itertools.product(range(8), range(64), range(4)):
        c4 = lane_chunk(l & 15)
        pos = (c4 & 7) | (w << 3) | ((c4 >> 3) << 6)
        byte = pos * 16 + (((l >> 4) & 1) | (((l >> 5) & 1) << 1)) * 4 + j * 2048
        e = base_q(w, l) + reg_idx_pq(2 * j)          # first of the two adjacent elements
        assert where[e >> 3] * 16 + (e & 7) * 2 == byte
    # one read instruction of a wave (64 lanes x 4 bytes = 256 bytes, two LDS cycles at best): every bank is hit twice
    for w, j in itertools.product(range(8), range(4)):
        banks = []
        for l in range(64):
            c4 = lane_chunk(l & 15)
            pos = (c4 & 7) | (w << 3) | ((c4 >> 3) << 6)
            banks.append(((pos * 16 + (((l >> 4) & 1) | (((l >> 5) & 1) << 1)) * 4 + j * 2048) >> 2) & 31)
        assert sorted(np.bincount(banks, minlength=32)) == [2] * 32


# ---- the two-phase inverse (csrc/bq_k12_inv.h): phase B reads the raw 16-bit row from the input ring in layout P ----
INV_PIECE = 1088


def inv_ring_addr(idx):            # byte offset inside a ring slot of element idx (even)
    j = (idx >> 3) & 63
    pos = (j >> 4) | ((j & 15) << 2)
    return (idx >> 9) * INV_PIECE + pos * 16 + (idx & 7) * 2


def test_inverse_ring_readers_find_what_the_loaders_put_there():
    # wave w, lane l loads the 16 bytes of chunk j(l) of piece w (elements 512 w + 8 j .. + 7) to offset 16 l of the piece
    where = {}
    for w, l in itertools.product(range(8), range(64)):
        j = ((l & 3) << 4) | (l >> 2)
        for b in range(8):
            where[512 * w + 8 * j + b] = w * INV_PIECE + 16 * l + 2 * b
    assert sorted(where) == list(range(4096))
    assert len(set(where.values())) == 4096 and max(where.values()) + 2 <= 8 * INV_PIECE
    # a reader of layout P takes register pair (r1, r2) from inv_ring_addr(base) + (2 r1 + 4 r2) pieces
    for w, l in itertools.product(range(8), range(64)):
        base = base_p(w, l)
        for r1, r2 in itertools.product(range(2), range(2)):
            a = inv_ring_addr(base) + (2 * r1 + 4 * r2) * INV_PIECE
            idx = base + 1024 * r1 + 2048 * r2
            assert a % 4 == 0 and where[idx] == a and where[idx + 1] == a + 2


def test_inverse_ring_reads_are_free_of_bank_conflicts():
    # a 32-bit read of 32 consecutive lanes (half a wave) touches 32 different banks (4 bytes wide, 32 of them)
    for w, half, r in itertools.product(range(8), range(2), range(4)):
        banks = {((inv_ring_addr(base_p(w, 32 * half + l)) + 2 * r * INV_PIECE) >> 2) & 31 for l in range(32)}
        assert len(banks) == 32
