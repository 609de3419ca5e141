"""Seeded, counter-based synthetic workloads for sparse-DNN inference.

This module only draws inputs: weight sparsity patterns (32 distinct input
columns per output neuron), the constant weight value, the constant bias and
binary input feature maps.  It holds none of the inference arithmetic and is
shared by the CPU oracle's tests and the GPU path's tests so that both see the
same bytes.

Shapes follow the networks of the Sparse DNN Challenge described in the paper's
Section II-A: 60 000 binary inputs of 1024/4096/16384/65536 features, 32
connections per neuron, every weight 1/16, 120/480/1920 layers.  The challenge
files themselves are not available, so patterns and inputs are drawn from a
counter-based hash instead (splitmix64): every (layer, neuron) and every
(row, column) can be regenerated independently, on the host with numpy or on a
GPU with torch, with identical bits.

Backends: all core routines are written against a tiny array shim so that the
same code runs on numpy uint64 arrays (wrap-around arithmetic is defined) and
on torch int64 tensors (two's-complement wrap, logical shifts emulated).
"""
from __future__ import annotations

import numpy as np

try:  # torch is optional for the numpy backend
    import torch
except Exception:  # pragma: no cover
    torch = None

NNZ = 32                    # connections per output neuron (Section II-A)
WEIGHT = 0.0625             # every weight is 1/16 (Section II-A)
CLIP = 32.0                 # ReLU upper clip (Section II-A-1)

_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_STREAM_W = 0x5350444E4E5F5731    # weights
_STREAM_P = 0x5350444E4E5F5031    # window permutation
_STREAM_Y = 0x5350444E4E5F5931    # inputs
_STREAM_D = 0x5350444E4E5F4431    # per-row density

# The five benchmark configurations (neurons, layers, batch, bias, window).
# window=None: columns uniform over [0, N); window=w: the outputs of block
# b=j//w of layer l draw from the contiguous window w*sigma_l(b), sigma_l a
# seeded permutation of the N//w windows ("locality variant").
CONFIGS = {
    0: dict(N=1024, L=120, batch=1000, bias=-0.30, window=None, seed=20200700),
    1: dict(N=1024, L=120, batch=60000, bias=-0.30, window=None, seed=20200700),
    2: dict(N=4096, L=480, batch=60000, bias=-0.35, window=None, seed=20200702),
    3: dict(N=16384, L=1920, batch=60000, bias=-0.40, window=None, seed=20200703),
    4: dict(N=65536, L=1920, batch=60000, bias=-0.45, window=4096, seed=20200704),
}
DENSITY = 0.15              # P(Y0 element == 1)


# --------------------------------------------------------------------------
# backend shim
# --------------------------------------------------------------------------
def _signed(c: int) -> int:
    c &= (1 << 64) - 1
    return c - (1 << 64) if c >= (1 << 63) else c


class _NP:
    name = "numpy"

    @staticmethod
    def const(c):
        return np.uint64(c & ((1 << 64) - 1))

    @staticmethod
    def arange(n, start=0):
        return np.arange(start, start + n, dtype=np.uint64)

    @staticmethod
    def asarray(x):
        return np.asarray(x).astype(np.uint64)

    @staticmethod
    def lsr(x, s):
        return x >> np.uint64(s)

    @staticmethod
    def sort(x):
        return np.sort(x, axis=-1)

    @staticmethod
    def argsort(x):
        return np.argsort(x, axis=-1, kind="stable")

    @staticmethod
    def to_i32(x):
        return x.astype(np.int32)

    @staticmethod
    def to_f32(x):
        return x.astype(np.float32)

    @staticmethod
    def any(x):
        return bool(np.any(x))

    @staticmethod
    def where_rows(mask):
        return np.nonzero(mask)[0]


class _TH:
    name = "torch"

    def __init__(self, device):
        self.device = torch.device(device)

    def const(self, c):
        return _signed(c)

    def arange(self, n, start=0):
        return torch.arange(start, start + n, dtype=torch.int64, device=self.device)

    def asarray(self, x):
        return torch.as_tensor(x, device=self.device).to(torch.int64)

    @staticmethod
    def lsr(x, s):
        return (x >> s) & ((1 << (64 - s)) - 1)

    @staticmethod
    def sort(x):
        return torch.sort(x, dim=-1).values

    @staticmethod
    def argsort(x):
        return torch.argsort(x, dim=-1, stable=True)

    @staticmethod
    def to_i32(x):
        return x.to(torch.int32)

    @staticmethod
    def to_f32(x):
        return x.to(torch.float32)

    @staticmethod
    def any(x):
        return bool(x.any().item())

    @staticmethod
    def where_rows(mask):
        return torch.nonzero(mask, as_tuple=False).flatten()


def _backend(device):
    if device is None or device == "numpy":
        return _NP()
    if torch is None:
        raise RuntimeError("torch backend requested but torch is not importable")
    return _TH(device)


# --------------------------------------------------------------------------
# counter-based hash (splitmix64 finaliser and stream)
# --------------------------------------------------------------------------
def _mix(bk, x):
    """splitmix64 output function of state x + GOLDEN (wrapping 64-bit)."""
    x = x + bk.const(_GOLDEN)
    x = (x ^ bk.lsr(x, 30)) * bk.const(_M1)
    x = (x ^ bk.lsr(x, 27)) * bk.const(_M2)
    return x ^ bk.lsr(x, 31)


def _mix_py(x: int) -> int:
    """Same as _mix on one python integer (used for scalar keys)."""
    m = (1 << 64) - 1
    x = (x + _GOLDEN) & m
    x = ((x ^ (x >> 30)) * _M1) & m
    x = ((x ^ (x >> 27)) * _M2) & m
    return x ^ (x >> 31)


def _stream(bk, key, t):
    """t-th output (t = 0, 1, ...) of the splitmix64 stream seeded by key."""
    return _mix(bk, key + (t * bk.const(_GOLDEN)))


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------
def window_bases(N, l, seed, window, device=None):
    """Start column of the input window of every output neuron of layer l.

    window=None -> zeros (whole row).  Otherwise output block b = j // window
    reads window sigma_l(b), sigma_l = seeded permutation of the N // window
    windows (argsort of one hash per block).
    """
    bk = _backend(device)
    j = bk.arange(N)
    if window is None or window >= N:
        return j * bk.const(0), N
    if N % window:
        raise ValueError("window must divide N")
    nwin = N // window
    k = _mix_py(_mix_py(seed ^ _STREAM_P) ^ l)
    h = bk.lsr(_mix(bk, bk.arange(nwin) ^ bk.const(k)), 1)
    # windows ranked by hash: sigma(b) = rank of block b
    order = bk.argsort(h)
    sigma = bk.argsort(order)
    if bk.name == "numpy":
        sigma = sigma.astype(np.uint64)
        blk = (j // np.uint64(window)).astype(np.int64)
        base = sigma[blk] * np.uint64(window)
    else:
        blk = j // window
        base = sigma[blk] * window
    return base, window


def _draw_small(bk, nkey, base, width):
    """32 distinct columns for narrow windows (width < 1024), where redrawing
    whole rows would rarely succeed: step t draws r in [0, width - t) and takes
    the r-th column not chosen yet (partial shuffle, written as 'skip over the
    ones already taken in ascending order')."""
    akey = _mix(bk, nkey ^ bk.const(0))
    chosen = None                                           # [n, t] ascending
    for t in range(NNZ):
        h = _mix(bk, akey + bk.const(((t + 1) * _GOLDEN) & ((1 << 64) - 1)))   # stream output t+1
        u = bk.lsr(h, 33)
        c = bk.lsr(u * bk.const(width - t), 31)             # in [0, width - t)
        for s in range(t):
            c = c + (c >= chosen[:, s])
        col = c[:, None]
        if chosen is None:
            chosen = col
        elif bk.name == "numpy":
            chosen = np.sort(np.concatenate([chosen, col.astype(np.uint64)], axis=1), axis=1)
        else:
            chosen = torch.sort(torch.cat([chosen, col], dim=1), dim=1).values
    return chosen + base[:, None]


def gen_layer(N, l, seed, window=None, device=None, window_layer=None):
    """Input columns of every output neuron of layer l: int32 [N, 32], each row
    32 distinct columns, ascending.

    Neuron j draws 32 columns base + floor(u * width), u from its own hash
    stream; if two coincide the whole draw is repeated with the next attempt
    number until all 32 are distinct (so the set is uniform over 32-subsets of
    the window).  Windows narrower than 1024 columns use a partial shuffle
    instead (see _draw_small).
    """
    bk = _backend(device)
    # window_layer: take the windows of that layer (gen_layer_general: every draw of a neuron in the neuron's window)
    base, width = window_bases(N, l if window_layer is None else window_layer, seed, window, device)
    if width < NNZ:
        raise ValueError("need at least 32 columns to draw 32 distinct ones")
    kl = _mix_py(_mix_py(seed ^ _STREAM_W) ^ l)
    j = bk.arange(N)
    nkey = _mix(bk, j ^ bk.const(kl))                      # [N]
    if width < 1024:
        return bk.to_i32(_draw_small(bk, nkey, base, width))
    t = bk.arange(NNZ, start=1)                             # [32]
    cols = None
    todo = None                                             # rows still to draw
    attempt = 0
    while True:
        keys = nkey if todo is None else nkey[todo]
        akey = _mix(bk, keys ^ bk.const(attempt))           # [n]
        h = _stream(bk, akey[:, None], t[None, :])          # [n, 32]
        u = bk.lsr(h, 33)                                   # 31 bits
        c = bk.lsr(u * bk.const(width), 31)                 # in [0, width)
        b = base if todo is None else base[todo]
        c = bk.sort(c + b[:, None])
        if todo is None:
            cols = c
        else:
            cols[todo] = c
        dup = (c[:, 1:] == c[:, :-1]).any(-1) if bk.name == "torch" else \
            np.any(c[:, 1:] == c[:, :-1], axis=-1)
        if not bk.any(dup):
            break
        bad = bk.where_rows(dup)
        todo = bad if todo is None else todo[bad]
        attempt += 1
        if attempt > 1000:  # pragma: no cover
            raise RuntimeError("column draw did not converge")
    return bk.to_i32(cols)


_STREAM_S = 0x5350444E4E5F5331    # column scatter


def scatter_columns(cols, N, l, seed, device=None):
    """The "scattered window" variant of a windowed layer: every column c of the
    pattern is replaced by pi_l(c), pi_l a seeded permutation of all N columns (ranks
    of one hash per column), and each neuron's columns are sorted again.  The set of
    columns an output block reads keeps its size but is spread over the whole row."""
    bk = _backend(device)
    k = _mix_py(_mix_py(seed ^ _STREAM_S) ^ l)
    h = bk.lsr(_mix(bk, bk.arange(N) ^ bk.const(k)), 1)
    pi = bk.argsort(bk.argsort(h))                          # rank of column c
    if bk.name == "numpy":
        out = np.sort(pi[np.asarray(cols, dtype=np.int64)], axis=1)
    else:
        out = torch.sort(pi[cols.to(torch.int64)], dim=1).values
    return bk.to_i32(out)


def gen_layer_strided(N, stride, device=None):
    """A strided pattern of the kind the RadiX-Net topologies of the challenge networks are built from
    (Section II-A; ours, the challenge files are not available): neuron j is connected to the 32 columns
    (j + k * stride) mod N, k = 0..31, sorted.  int32 [N, 32]."""
    bk = _backend(device)
    if bk.name == "numpy":
        j = np.arange(N, dtype=np.int64)[:, None]
        k = np.arange(NNZ, dtype=np.int64)[None, :]
        return np.sort((j + k * int(stride)) % N, axis=1).astype(np.int32)
    j = torch.arange(N, dtype=torch.int64, device=device)[:, None]
    k = torch.arange(NNZ, dtype=torch.int64, device=device)[None, :]
    return torch.sort((j + k * int(stride)) % N, dim=1).values.to(torch.int32)


def gen_values(N, device=None):
    """Weight values of one layer: float32 [N, 32], all 1/16."""
    if device is None or device == "numpy":
        return np.full((N, NNZ), WEIGHT, dtype=np.float32)
    return torch.full((N, NNZ), WEIGHT, dtype=torch.float32, device=device)


_STREAM_G = 0x5350444E4E5F4731    # general layers: neuron lengths and weights


def gen_layer_general(N, l, seed, kmin, kmax, window=None, uniform_weight=False):
    """A general sparse layer (Section II-A-1: W_l may be any sparse matrix), as
    numpy arrays (ptr int32 [N+1], idx int32 [nnz], val float32 [nnz]): output
    neuron j owns entries ptr[j] .. ptr[j+1]-1.

    Recipe: neuron j has d_j = kmin + (hash mod (kmax-kmin+1)) connections.  Its
    columns are the first d_j of the concatenation of ceil(kmax/32) independent
    32-column draws of gen_layer, all from the neuron's window in layer l (each
    ascending; a column may repeat across draws -- repeated connections add up).  Weights: m / (d_j * 2**23) with m a
    hashed integer in [2**23, 3 * 2**23), so a neuron's weights sum to about 2, as
    the 32 weights of 1/16 of the challenge networks do; uniform_weight=True gives
    every connection 1/16 instead.
    """
    if not (0 <= kmin <= kmax):
        raise ValueError("need 0 <= kmin <= kmax")
    bk = _NP()
    draws = max(1, -(-kmax // NNZ))
    cols = np.concatenate([gen_layer(N, l + 100003 * t, seed, window, window_layer=l) for t in range(draws)], axis=1)  # [N, 32*draws]
    kg = _mix_py(_mix_py(seed ^ _STREAM_G) ^ l)
    j = bk.arange(N)
    nkey = _mix(bk, j ^ bk.const(kg))
    deg = (np.uint64(kmin) + bk.lsr(nkey, 11) % np.uint64(kmax - kmin + 1)).astype(np.int64)   # [N]
    ptr = np.zeros(N + 1, dtype=np.int64)
    np.cumsum(deg, out=ptr[1:])
    if ptr[N] >= (1 << 31):
        raise ValueError("layer too large for 32-bit offsets")
    k = np.arange(NNZ * draws, dtype=np.int64)[None, :]
    take = k < deg[:, None]
    idx = cols[take].astype(np.int32)
    if uniform_weight:
        val = np.full(idx.shape, WEIGHT, dtype=np.float32)
    else:
        t = bk.arange(NNZ * draws, start=1)
        h = _stream(bk, nkey[:, None], t[None, :])
        m = (np.uint64(1 << 23) + (bk.lsr(h, 20) & np.uint64((1 << 24) - 1))).astype(np.float64)
        w = m / (np.maximum(deg, 1)[:, None].astype(np.float64) * float(1 << 23))
        val = w[take].astype(np.float32)
    return ptr.astype(np.int32), idx, val


def gen_bias(N, value, device=None):
    """Bias vector: float32 [N], one constant (Alg. 1 step 2)."""
    if device is None or device == "numpy":
        return np.full((N,), value, dtype=np.float32)
    return torch.full((N,), value, dtype=torch.float32, device=device)


# --------------------------------------------------------------------------
# inputs
# --------------------------------------------------------------------------
def _row_keys(bk, seed, rows):
    k = _mix_py(seed ^ _STREAM_Y)
    return _mix(bk, rows ^ bk.const(k))


def row_thresholds(seed, rows, density=DENSITY, device=None):
    """24-bit Bernoulli threshold of every row.

    density = float p          -> floor(p * 2**24) for all rows
    density = "mixed"          -> per-row density drawn (integer arithmetic
                                  only) from [0.05, 0.20) or [0.40, 0.60),
                                  each with probability 1/2: rows of the first
                                  kind die within a few layers, rows of the
                                  second kind saturate and survive.
    """
    bk = _backend(device)
    rows = bk.asarray(rows)
    if density == "mixed":
        k = _mix_py(seed ^ _STREAM_D)
        h = _mix(bk, rows ^ bk.const(k))
        kind = bk.lsr(h, 63)                                # 0 or 1
        u = bk.lsr(h, 16) & bk.const((1 << 24) - 1)         # 24 bits
        one = 1 << 24
        lo0, sp0 = int(0.05 * one), int(0.15 * one)
        lo1, sp1 = int(0.40 * one), int(0.20 * one)
        t0 = bk.lsr(u * bk.const(sp0), 24) + bk.const(lo0)
        t1 = bk.lsr(u * bk.const(sp1), 24) + bk.const(lo1)
        return t0 + kind * (t1 - t0)
    thr = int(float(density) * (1 << 24))
    return rows * bk.const(0) + bk.const(thr)


def gen_y0(batch, N, seed, density=DENSITY, rows=None, device=None, chunk_rows=None):
    """Binary input feature map: float32 [len(rows), N], 1.0 where the 24 top
    bits of the element's hash fall below the row's threshold.  rows=None
    means all rows 0..batch-1; a subset regenerates exactly those rows."""
    bk = _backend(device)
    rows_all = bk.arange(batch) if rows is None else bk.asarray(rows)
    n = int(rows_all.shape[0])
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 25) // max(N, 1))
    c = bk.arange(N, start=1)
    out = []
    for s in range(0, n, chunk_rows):
        r = rows_all[s:s + chunk_rows]
        rk = _row_keys(bk, seed, r)
        thr = row_thresholds(seed, r, density, device)
        h = _stream(bk, rk[:, None], c[None, :])
        one = bk.lsr(h, 40) < thr[:, None]
        out.append(bk.to_f32(one))
    if not out:
        if bk.name == "numpy":
            return np.zeros((0, N), dtype=np.float32)
        return torch.zeros((0, N), dtype=torch.float32, device=bk.device)
    if bk.name == "numpy":
        return np.concatenate(out, axis=0)
    return torch.cat(out, dim=0)


def config(k):
    """Copy of benchmark configuration k (0..4)."""
    return dict(CONFIGS[k])


def nominal_edges(N, L, batch):
    """Edge count the throughput metric divides by time: batch * N * 32 * L,
    pruned rows included (Section IV-A)."""
    return int(batch) * int(N) * NNZ * int(L)
