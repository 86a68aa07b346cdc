"""Brute-force definition of Top_K used to pin the oracle on tiny inputs.

Independent of the oracle: enumerates every K-subset and accepts the one that is
closed under the total order "larger magnitude first, lower index first among
equal magnitudes".  Magnitude is the fp32 bit pattern with the sign cleared.
"""
from itertools import combinations

import numpy as np


def mag_key(x: np.ndarray) -> np.ndarray:
    return x.view(np.uint32) & np.uint32(0x7FFFFFFF)


def brute_topk_set(x: np.ndarray, K: int):
    d = x.shape[0]
    key = [int(k) for k in mag_key(x)]
    good = []
    for S in combinations(range(d), K):
        inS = set(S)
        ok = True
        for i in S:
            for j in range(d):
                if j in inS:
                    continue
                # i must precede j in the total order
                if not (key[i] > key[j] or (key[i] == key[j] and i < j)):
                    ok = False
                    break
            if not ok:
                break
        if ok:
            good.append(S)
    assert len(good) == 1, f"total order must give exactly one subset, got {len(good)}"
    return list(good[0])
