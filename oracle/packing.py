"""2-bit packing of ternary codes (CPU oracle, test infrastructure only).

The paper states only that a ternary weight needs 2 bits (Sec. 2.1, "Model
compression").  The storage format below is this library's own; it is written
here from the format's definition, independently of the GPU code:

* A weight tensor [rows][C][R][S] is viewed as a matrix [rows][K], K = R*S*C,
  with k = (r*S + s)*C + c  (input channel fastest, matching NHWC activations).
* Each row is padded with zero codes to a multiple of 128 weights and occupies
  8*ceil(K/128) little-endian 32-bit words.
* Word j of a row holds the 16 codes k = 16j .. 16j+15.  The code of
  k = 16j + 2i sits in bits [2i, 2i+1]; the code of k = 16j + 2i + 1 sits in
  bits [16+2i, 17+2i]  (i = 0..7): even-k codes in the low half-word, odd-k
  codes in the high half-word.
* A 2-bit field is (bit0 = weight is non-zero, bit1 = weight is negative):
  00 -> 0, 01 -> +1, 11 -> -1; 10 is never written.
* The transposed copy used by the backward-data pass has one row per input
  channel c and K_T = R*S*rows with k_T = (r*S + s)*rows + o.

1-bit format of the sign codes of the binary-weight comparison (this library's own as well):

* Same matrix view and row padding (a multiple of 128 weights: 4*ceil(K/128) words per row).
* Word j of a row holds the 32 codes k = 32j .. 32j+31: the code of k = 32j + 2i sits in bit i, the code of
  k = 32j + 2i + 1 in bit 16+i (i = 0..15): even-k codes in the low half-word, odd-k codes in the high one.
* A bit is 1 for -1 and 0 for +1; padding bits are 0.
"""

import numpy as np


def words_per_row(k):
    return 8 * ((int(k) + 127) // 128)


def packed_bytes(rows, k):
    return int(rows) * words_per_row(k) * 4


def _field(code):
    code = np.asarray(code, dtype=np.int64)
    return (code != 0).astype(np.uint32) | ((code < 0).astype(np.uint32) << np.uint32(1))


def pack_matrix(codes2d):
    """Pack an int8 matrix [rows][K] of codes into uint32 [rows][words_per_row]."""
    codes2d = np.asarray(codes2d, dtype=np.int8)
    rows, k = codes2d.shape
    wpr = words_per_row(k)
    padded = np.zeros((rows, wpr * 16), dtype=np.int8)
    padded[:, :k] = codes2d
    f = _field(padded).reshape(rows, wpr, 8, 2)      # [..., i, parity]
    out = np.zeros((rows, wpr), dtype=np.uint32)
    for i in range(8):
        out |= f[:, :, i, 0] << np.uint32(2 * i)
        out |= f[:, :, i, 1] << np.uint32(16 + 2 * i)
    return out


def unpack_matrix(packed, rows, k):
    """Inverse of pack_matrix; also reports whether the invalid field 10 occurs
    and whether every padding field is zero."""
    wpr = words_per_row(k)
    p = np.asarray(packed, dtype=np.uint32).reshape(rows, wpr)
    fields = np.zeros((rows, wpr, 8, 2), dtype=np.uint32)
    for i in range(8):
        fields[:, :, i, 0] = (p >> np.uint32(2 * i)) & np.uint32(3)
        fields[:, :, i, 1] = (p >> np.uint32(16 + 2 * i)) & np.uint32(3)
    fields = fields.reshape(rows, wpr * 16)
    has_invalid = bool(np.any(fields == 2))
    pad_clean = bool(np.all(fields[:, k:] == 0))
    codes = np.zeros(fields.shape, dtype=np.int8)
    codes[fields == 1] = 1
    codes[fields == 3] = -1
    return codes[:, :k].copy(), has_invalid, pad_clean


def to_matrix(codes_oihw):
    """[rows][C][R][S] codes -> [rows][K] with k = (r*S + s)*C + c."""
    c4 = np.asarray(codes_oihw, dtype=np.int8)
    o, c, r, s = c4.shape
    return np.ascontiguousarray(c4.transpose(0, 2, 3, 1)).reshape(o, r * s * c)


def to_matrix_t(codes_oihw):
    """[rows][C][R][S] codes -> [C][K_T] with k_T = (r*S + s)*rows + o."""
    c4 = np.asarray(codes_oihw, dtype=np.int8)
    o, c, r, s = c4.shape
    return np.ascontiguousarray(c4.transpose(1, 2, 3, 0)).reshape(c, r * s * o)


def pack_weights(codes_oihw):
    return pack_matrix(to_matrix(codes_oihw))


def pack_weights_t(codes_oihw):
    return pack_matrix(to_matrix_t(codes_oihw))


def unpack_weights(packed, rows, c, r, s):
    m, bad, clean = unpack_matrix(packed, rows, r * s * c)
    return m.reshape(rows, r, s, c).transpose(0, 3, 1, 2).copy(), bad, clean


def unpack_weights_t(packed_t, rows, c, r, s):
    m, bad, clean = unpack_matrix(packed_t, c, r * s * rows)
    return m.reshape(c, r, s, rows).transpose(3, 0, 1, 2).copy(), bad, clean


def words_per_row1(k):
    return 4 * ((int(k) + 127) // 128)


def pack_matrix1(codes2d):
    """Pack an int8 matrix [rows][K] of sign codes (-1 / +1) into uint32 [rows][words_per_row1]."""
    codes2d = np.asarray(codes2d, dtype=np.int8)
    rows, k = codes2d.shape
    assert np.all((codes2d == 1) | (codes2d == -1))
    wpr = words_per_row1(k)
    neg = np.zeros((rows, wpr * 32), dtype=np.uint32)
    neg[:, :k] = (codes2d < 0)
    neg = neg.reshape(rows, wpr, 16, 2)                # [..., i, parity]
    out = np.zeros((rows, wpr), dtype=np.uint32)
    for i in range(16):
        out |= neg[:, :, i, 0] << np.uint32(i)
        out |= neg[:, :, i, 1] << np.uint32(16 + i)
    return out


def unpack_matrix1(packed, rows, k):
    """Inverse of pack_matrix1; also reports whether every padding bit is zero."""
    wpr = words_per_row1(k)
    p = np.asarray(packed, dtype=np.uint32).reshape(rows, wpr)
    bits = np.zeros((rows, wpr, 16, 2), dtype=np.uint32)
    for i in range(16):
        bits[:, :, i, 0] = (p >> np.uint32(i)) & np.uint32(1)
        bits[:, :, i, 1] = (p >> np.uint32(16 + i)) & np.uint32(1)
    bits = bits.reshape(rows, wpr * 32)
    pad_clean = bool(np.all(bits[:, k:] == 0))
    return np.where(bits[:, :k] == 1, np.int8(-1), np.int8(1)).astype(np.int8), pad_clean


def pack_weights1(codes_oihw):
    return pack_matrix1(to_matrix(codes_oihw))
