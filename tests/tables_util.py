"""Table construction for the tests: their own copy of the bin-edge rule (Sec. 5: thresholds halfway between
consecutive levels) and of the table padding, so that no pin leans on the package under test."""
import numpy as np

TABLE_STRIDE = 16


def midpoints(levels) -> np.ndarray:
    """Bin edges halfway between consecutive levels (Sec. 5), in fp64."""
    levels = np.asarray(levels, dtype=np.float64)
    return (levels[:-1] + levels[1:]) / 2.0


def pad_tables(levels_list, thresholds_list=None):
    """([C,16] thresholds padded with +inf, [C,16] mappings padded with 0), fp32.  thresholds_list[c] None (or no
    list): the midpoint rule."""
    C = len(levels_list)
    thr = np.full((C, TABLE_STRIDE), np.inf, dtype=np.float32)
    mp = np.zeros((C, TABLE_STRIDE), dtype=np.float32)
    for c, lv in enumerate(levels_list):
        lv = np.asarray(lv, dtype=np.float64)
        t = None if thresholds_list is None else thresholds_list[c]
        t = midpoints(lv) if t is None else np.asarray(t, dtype=np.float64)
        assert t.size == lv.size - 1
        mp[c, : lv.size] = lv.astype(np.float32)
        thr[c, : lv.size - 1] = t.astype(np.float32)
    return thr, mp


def listing_tables(init_tables):
    """Codebooks 0/1/2 = the 1-/2-/4-bit initial tables the paper prints (App. F listing): the printed mappings, the
    printed thresholds at 1 and 2 bits; the listing prints no 4-bit thresholds, so those follow the midpoint rule."""
    thr, mp = pad_tables([init_tables["mappings_1bit"], init_tables["mappings_2bit"], init_tables["mappings_4bit"]],
                         [init_tables["thresholds_1bit"], init_tables["thresholds_2bit"], None])
    return thr, mp, np.array([1, 2, 4], dtype=np.uint8)
