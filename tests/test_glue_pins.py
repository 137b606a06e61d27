"""Pins for the oracle of the copy steps around the attention call (grouping q, k, v into one
row per request, Sec. 3.2.1 step 2; placing returned rows in the decode batch, Sec. 3.2.2):
every expected array below is written out by hand, element by element.  CPU only."""
import numpy as np

from oracle import glue_np


def u16(x):
    return np.asarray(x, dtype=np.uint16)


def test_pack_qkv_two_requests_written_out():
    # B = 2, Hq = 2, Hkv = 1, d = 8; element value = 1000*tensor + 100*request + 10*head + index
    q = u16([[[1000, 1001, 1002, 1003, 1004, 1005, 1006, 1007],
              [1010, 1011, 1012, 1013, 1014, 1015, 1016, 1017]],
             [[1100, 1101, 1102, 1103, 1104, 1105, 1106, 1107],
              [1110, 1111, 1112, 1113, 1114, 1115, 1116, 1117]]])
    k = u16([[[2000, 2001, 2002, 2003, 2004, 2005, 2006, 2007]],
             [[2100, 2101, 2102, 2103, 2104, 2105, 2106, 2107]]])
    v = u16([[[3000, 3001, 3002, 3003, 3004, 3005, 3006, 3007]],
             [[3100, 3101, 3102, 3103, 3104, 3105, 3106, 3107]]])
    want = u16([[1000, 1001, 1002, 1003, 1004, 1005, 1006, 1007,
                 1010, 1011, 1012, 1013, 1014, 1015, 1016, 1017,
                 2000, 2001, 2002, 2003, 2004, 2005, 2006, 2007,
                 3000, 3001, 3002, 3003, 3004, 3005, 3006, 3007],
                [1100, 1101, 1102, 1103, 1104, 1105, 1106, 1107,
                 1110, 1111, 1112, 1113, 1114, 1115, 1116, 1117,
                 2100, 2101, 2102, 2103, 2104, 2105, 2106, 2107,
                 3100, 3101, 3102, 3103, 3104, 3105, 3106, 3107]])
    got = glue_np.pack_qkv(q, k, v)
    assert got.dtype == np.uint16 and got.shape == (2, 32)
    assert np.array_equal(got, want)


def test_pack_qkv_wider_rows_keep_the_fill_behind_the_three_tensors():
    q = u16([[[1, 2]], [[3, 4]]])
    k = u16([[[5, 6]], [[7, 8]]])
    v = u16([[[9, 10]], [[11, 12]]])
    want = u16([[1, 2, 5, 6, 9, 10, 77, 77],
                [3, 4, 7, 8, 11, 12, 77, 77]])
    assert np.array_equal(glue_np.pack_qkv(q, k, v, width=8, fill=77), want)


def test_pack_qkv_order_is_q_then_k_then_v_with_unequal_head_counts():
    # Hq = 3, Hkv = 2, d = 1: the row is q0 q1 q2 | k0 k1 | v0 v1
    q = u16([[[10], [11], [12]]])
    k = u16([[[20], [21]]])
    v = u16([[[30], [31]]])
    assert np.array_equal(glue_np.pack_qkv(q, k, v), u16([[10, 11, 12, 20, 21, 30, 31]]))


def test_scatter_rows_with_a_skipped_and_two_out_of_range_indices():
    dst = u16([[0, 0, 0], [1, 1, 1], [2, 2, 2], [3, 3, 3], [4, 4, 4]])
    src = u16([[10, 11, 12], [20, 21, 22], [30, 31, 32], [40, 41, 42]])
    # row 0 -> 3, row 1 -> -1 (skipped), row 2 -> 5 (one past the end: skipped), row 3 -> 0
    index = np.asarray([3, -1, 5, 0], dtype=np.int32)
    want = u16([[40, 41, 42], [1, 1, 1], [2, 2, 2], [10, 11, 12], [4, 4, 4]])
    before = dst.copy()
    got = glue_np.scatter_rows(dst, src, index)
    assert np.array_equal(got, want)
    assert np.array_equal(dst, before), "the input must not be modified"


def test_scatter_rows_identity_and_reversal():
    dst = u16(np.zeros((3, 2)))
    src = u16([[1, 2], [3, 4], [5, 6]])
    assert np.array_equal(glue_np.scatter_rows(dst, src, np.asarray([0, 1, 2], dtype=np.int32)), src)
    assert np.array_equal(glue_np.scatter_rows(dst, src, np.asarray([2, 1, 0], dtype=np.int32)),
                          u16([[5, 6], [3, 4], [1, 2]]))


def test_scatter_rows_with_no_rows_leaves_the_batch_alone():
    dst = u16([[7, 8], [9, 10]])
    got = glue_np.scatter_rows(dst, u16(np.zeros((0, 2))), np.zeros(0, dtype=np.int32))
    assert np.array_equal(got, dst)
