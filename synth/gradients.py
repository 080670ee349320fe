"""Counter-based, bit-reproducible synthetic gradients and attack payloads.

Everything is integer hashing plus one exact int->fp32 conversion and single fp32
multiplies, written with torch element-wise ops, so the same bytes come out on the CPU and
on a GPU and any subset of coordinates can be generated on its own.

honest gradient of file j (Sec. 2: g_{t,j}), coordinate c, step t:
    key_j = mix(mix(seed) ^ mix(t * 2^20 + j + 1))
    z     = key_j + (c + 1) * GOLD                 (mod 2^64)
    h1    = mix(z),  h2 = mix(h1 ^ key_j)          (mix = splitmix64 finaliser)
    S     = sum of the eight 16-bit lanes of h1, h2     (Irwin-Hall, mean 262140, sigma 53510)
    g     = float32(S - 262140) * scale_j,  scale_j = float32(0.01 / 53510) [* file scale]
i.e. N(0, 0.01^2) up to the +-4.9 sigma support of the eight-lane sum.

Attack payloads (Sec. 6.1; the constants are the workloads', the paper leaves them open):
    reversed   x = float32(-c) * g_j                (one fp32 multiply)
    constant   x = value everywhere
    alie       x = float32(mean - z * std) per coordinate, mean and population std over the f
               honest file gradients, accumulated in fp64 in file order; one vector shared by
               every Byzantine copy
    mixed      Byzantine workers of even rank in the ascending Byzantine set send alie,
               odd rank send constant (a worker fabricates all of its l vectors, Algorithm 1)
"""
import numpy as np
import torch

MASK64 = (1 << 64) - 1
M1 = 0xBF58476D1CE4E5B9
M2 = 0x94D049BB133111EB
GOLD = 0x9E3779B97F4A7C15
LANE_MEAN = 262140  # 8 * 65535 / 2
LANE_SIGMA = 53510.0


def _s64(u):
    u &= MASK64
    return u - (1 << 64) if u >= (1 << 63) else u


def mix64_py(u):
    u &= MASK64
    u = ((u ^ (u >> 30)) * M1) & MASK64
    u = ((u ^ (u >> 27)) * M2) & MASK64
    return u ^ (u >> 31)


def _lsr(x, s):
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64_t(x):
    x = (x ^ _lsr(x, 30)) * _s64(M1)
    x = (x ^ _lsr(x, 27)) * _s64(M2)
    return x ^ _lsr(x, 31)


def file_key(seed, step, j):
    return mix64_py(mix64_py(seed) ^ mix64_py((step << 20) + j + 1))


def file_scale(seed, step, j, file_scales):
    base = np.float32(0.01 / LANE_SIGMA)
    if not file_scales:
        return base
    u = (mix64_py(file_key(seed, step, j) ^ MASK64) >> 40)  # 24-bit uniform
    s = np.float32(0.5) + np.float32(1.5) * np.float32(u / float(1 << 24))  # U(0.5, 2)
    return np.float32(base * s)


def honest_gradients(f, d, seed, step=0, device="cpu", file_scales=False, coords=None):
    """[f, n] float32: the honest gradient of every file at coordinates `coords`
    (an int64 tensor; default all of 0..d-1)."""
    if coords is None:
        coords = torch.arange(d, dtype=torch.int64, device=device)
    else:
        coords = coords.to(device=device, dtype=torch.int64)
    G = torch.empty((f, coords.numel()), dtype=torch.float32, device=device)
    cg = (coords + 1) * _s64(GOLD)
    for j in range(f):
        key = _s64(file_key(seed, step, j))
        h1 = _mix64_t(cg + key)
        h2 = _mix64_t(h1 ^ key)
        S = torch.zeros_like(h1)
        for h in (h1, h2):
            for sh in (0, 16, 32, 48):
                S += (h >> sh) & 0xFFFF
        scale = torch.tensor(file_scale(seed, step, j, file_scales), dtype=torch.float32,
                             device=device)
        G[j] = (S - LANE_MEAN).to(torch.float32) * scale
    return G


def alie_vector(G, z):
    """ALIE payload: float32(mean - z*std) over the rows of G, fp64, sequential in file order."""
    f = G.shape[0]
    acc = torch.zeros(G.shape[1], dtype=torch.float64, device=G.device)
    for j in range(f):
        acc = acc + G[j].to(torch.float64)
    mean = acc / f
    acc2 = torch.zeros_like(acc)
    for j in range(f):
        t = G[j].to(torch.float64) - mean
        t = t * t
        acc2 = acc2 + t
    std = torch.sqrt(acc2 / f)
    zs = std * float(z)
    return (mean - zs).to(torch.float32)


def padded_ld(d, multiple=64):
    return (d + multiple - 1) // multiple * multiple


def build_copies(G, file_workers, worker_files, byz_workers, attack, ld=None):
    """Stacked worker returns X[K*l, ld] (Eq. 2): row w*l+t is worker w's t-th file.

    G [f, d] honest gradients; file_workers [f, r], worker_files [K, l] integer arrays (from
    either implementation of the assignment); byz_workers ascending ids of the Byzantine
    set.  Words d..ld-1 of every row are filled with row-dependent garbage that no correct
    implementation may read.
    """
    f, d = G.shape
    worker_files = np.asarray(worker_files)
    K, l = worker_files.shape
    ld = d if ld is None else int(ld)
    assert ld >= d
    X = torch.empty((K * l, ld), dtype=torch.float32, device=G.device)
    if ld > d:
        pad = torch.arange(K * l, dtype=torch.float32, device=G.device).unsqueeze(1) + 0.25
        X[:, d:] = pad
    byz = [int(w) for w in byz_workers]
    kind = attack["kind"]
    alie = None
    if kind in ("alie", "mixed") and byz:
        alie = alie_vector(G, attack["z"])
    for w in range(K):
        for t in range(l):
            j = int(worker_files[w, t])
            row = X[w * l + t]
            if w not in byz:
                row[:d] = G[j]
                continue
            k = kind
            if kind == "mixed":
                k = "alie" if byz.index(w) % 2 == 0 else "constant"
            if k == "reversed":
                row[:d] = G[j] * torch.tensor(-float(attack["c"]), dtype=torch.float32,
                                              device=G.device)
            elif k == "constant":
                row[:d] = float(attack["value"])
            elif k == "alie":
                row[:d] = alie
            else:
                raise ValueError(kind)
    return X
