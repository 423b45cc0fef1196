"""Random choices of the test harness for the heterogeneous-device workload.

The paper assigns every device its own number of rows and columns
(alpha_k, beta_k) under the coverage constraint sum alpha*beta = m*q and the
per-device memory constraint alpha*n*b + n*beta*b + alpha*beta*b <= M_k
(Sec. 4.1), with device capabilities sampled from measurement datasets that
are not available here.  As a stand-in, tile edges are drawn from a seeded
categorical over four device classes and packed as guillotine bands (row
bands, each cut into columns), which always tiles the output exactly.  The
draw is done here, once, and handed as plain lists to whichever planner is
under test -- no random generator has to match between implementations.
"""
import math

import numpy as np

# device class -> (preferred tile edge, working-set budget in bytes, weight)
# Phones with 512 MB / 1 GB and laptops with 4 GB / 10 GB of usable memory
# (Sec. 2.1) mapped to tile edges 128 / 256 / 512 / 1024.
DEVICE_CLASSES = (
    (128, 1 << 20, 0.4),
    (256, 3 << 20, 0.3),
    (512, 8 << 20, 0.2),
    (1024, 24 << 20, 0.1),
)
KSPLIT_CHOICES = (1, 2, 4, 8)


def _draw_class(rng):
    w = np.array([c[2] for c in DEVICE_CLASSES])
    return int(rng.choice(len(DEVICE_CLASSES), p=w / w.sum()))


def _cut(total, rng):
    """Cuts [0, total) into pieces whose lengths are class edges; last clipped."""
    pieces, classes = [], []
    pos = 0
    while pos < total:
        c = _draw_class(rng)
        edge = min(DEVICE_CLASSES[c][0], total - pos)
        pieces.append(edge)
        classes.append(c)
        pos += edge
    return pieces, classes


def _pick_ksplit(m_len, n_len, K, budget, in_bytes):
    """Smallest S whose task working set (row block + column block + fp32
    output block; the shape of the paper's memory constraint) fits the budget."""
    for S in KSPLIT_CHOICES:
        k_len = math.ceil(K / S)
        if (S - 1) * k_len >= K:
            break
        if (m_len + n_len) * k_len * in_bytes + m_len * n_len * 4 <= budget:
            return S
    best = 1
    for S in KSPLIT_CHOICES:
        if (S - 1) * math.ceil(K / S) < K:
            best = S
    return best


def draw_explicit_tiling(M, N, K, seed, in_bytes=2):
    """Returns (band_h, col_w, ksplit_per_tile): band heights (sum M), one list
    of column widths per band (each sums to N) and the K-split of every tile in
    band-major order."""
    rng = np.random.default_rng(seed)
    band_h, band_cls = _cut(M, rng)
    col_w, ksplit = [], []
    for h, hc in zip(band_h, band_cls):
        widths, wcls = _cut(N, rng)
        col_w.append(widths)
        for w, wc in zip(widths, wcls):
            budget = DEVICE_CLASSES[max(hc, wc)][1]
            ksplit.append(_pick_ksplit(h, w, K, budget, in_bytes))
    return band_h, col_w, ksplit


def draw_reissue(n_tasks, seed, fraction=0.05):
    """ceil(fraction*n_tasks) distinct task indices in shuffled order: the
    shards whose device left mid-batch and that are issued again."""
    rng = np.random.default_rng(seed)
    count = max(1, math.ceil(fraction * n_tasks))
    return [int(i) for i in rng.permutation(n_tasks)[:count]]


# Device fleet for the cost-model planner: the paper's classes (Sec. 2.1: phones
# with 512 MB - 1 GB, laptops with 4 - 10 GB usable memory; Sec. 5.1 samples
# capabilities from public benchmark and speed-test data that are not
# available here).  Stand-in: log-uniform draws inside per-class ranges.
FLEET_CLASSES = (
    # weight, downlink Mbit/s, uplink Mbit/s, latency ms, TFLOP/s, memory GB
    (0.4, (20, 100), (5, 20), (20, 80), (1, 4), 0.5),
    (0.3, (50, 300), (10, 50), (15, 60), (2, 8), 1.0),
    (0.2, (100, 600), (20, 100), (5, 30), (5, 15), 4.0),
    (0.1, (200, 1000), (50, 300), (2, 20), (10, 30), 10.0),
)


def draw_fleet(n_devices, seed):
    """Returns a list of (down_bw B/s, up_bw B/s, down_lat s, up_lat s, flop/s, mem bytes)."""
    rng = np.random.default_rng(seed)
    weights = [c[0] for c in FLEET_CLASSES]
    out = []
    for _ in range(n_devices):
        c = FLEET_CLASSES[int(rng.choice(len(FLEET_CLASSES), p=weights))]

        def logu(lo_hi):
            return float(np.exp(rng.uniform(np.log(lo_hi[0]), np.log(lo_hi[1]))))
        lat = logu(c[3]) * 1e-3
        out.append((logu(c[1]) * 1e6 / 8, logu(c[2]) * 1e6 / 8, lat, lat, logu(c[4]) * 1e12, c[5] * 1e9))
    return out
