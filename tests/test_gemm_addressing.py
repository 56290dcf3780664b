"""Host model of the addresses the selective-load GEMM's tile loads generate (CPU only).

The kernel reads its operands through range-checked buffer descriptors.  The hardware compares only the per-thread
offset (plus the immediate) with the descriptor's size; the scalar offset is not checked.  This test restates the
kernel's offset formulas for the layout with both operands along the contraction (X[idx] [M,C] against W [N,C]) and
checks, for shapes with ragged tiles (N = 40, C = 1000 among them), that every request whose per-thread offset passes
the range check touches only bytes inside the operand, and that every row or slab that must not be read is refused
(per-thread offset at or past the size, or a descriptor of size zero).
"""
import itertools

import pytest

BM = BN = 256
KB = 128          # bytes of the contraction per slab and row
NLD = 8           # 16-byte loads per thread, operand and slab
THREADS = 256


def requests(M, N, C, S, ldx, ldw, idx, esz=2):
    """Yield (operand, descriptor_base, descriptor_size, voff, soff, wanted) for every load of every tile and slab."""
    cbytes = C * esz
    nk, nfull = -(-cbytes // KB), cbytes // KB
    x_bytes = ((S - 1) * ldx + C) * esz
    for tm, tn in itertools.product(range(-(-M // BM)), range(-(-N // BN))):
        m0, n0 = tm * BM, tn * BN
        b_rows = min(BN, N - n0)
        w_bytes = (b_rows - 1) * ldw * esz + cbytes
        for tid in (0, 7, 8, 63, 100, 255):
            prow, pcc = tid >> 3, tid & 7
            for i in range(NLD):
                m = min(m0 + i * 32 + prow, M - 1)
                a_voff = idx[m] * ldx * esz + pcc * 16
                b_voff = (i * 32 + prow) * ldw * esz + pcc * 16
                for kt in range(nk + 2):                          # the loop also asks for two slabs past the end
                    kbyte = kt * KB
                    full = kt < nfull                              # requested in the loop, through the live descriptor
                    ragged = kt == nfull and nfull < nk            # requested by the predicated fetch
                    in_k = kbyte + pcc * 16 + 16 <= cbytes
                    if full or (ragged and in_k) or (kt < 2 and in_k):   # the prologue fetches slabs 0 and 1 predicated as well
                        yield ("A", 0, x_bytes, a_voff, kbyte, True)
                        yield ("B", n0 * ldw * esz, w_bytes, b_voff, kbyte, i * 32 + prow < b_rows)
                    else:
                        yield ("A", 0, 0, a_voff, kbyte, False)    # descriptor of size zero
                        yield ("B", n0 * ldw * esz, 0, b_voff, kbyte, False)


@pytest.mark.parametrize("M,N,C,S,pad", [(130, 40, 1000, 300, 0), (517, 300, 256, 1000, 8), (513, 257, 1000, 513, 0), (1, 2, 8, 64, 0),
                                         (300, 512, 4096, 700, 0), (256, 256, 64, 256, 24)])
def test_no_request_leaves_its_operand(M, N, C, S, pad):
    ldx, ldw, esz = C + pad, C + pad, 2
    idx = [(7 * m + 3) % S for m in range(M)]
    x_total, w_total = ((S - 1) * ldx + C) * esz, ((N - 1) * ldw + C) * esz
    for op, base, size, voff, soff, wanted in requests(M, N, C, S, ldx, ldw, idx, esz):
        passes = voff + 16 <= size                                  # what the hardware checks (per-thread offset only)
        if passes:
            lo = base + voff + soff
            assert lo + 16 <= (x_total if op == "A" else w_total), (op, base, size, voff, soff)
            assert wanted, (op, base, size, voff, soff)             # nothing is fetched that the tile has no use for
        else:
            assert not wanted or soff + (voff % (ldx * esz if op == "A" else ldw * esz)) + 16 > C * esz, (op, base, size, voff, soff)
