"""A second, independent statement of the step in NumPy library routines.

It exists to pin the C oracle against something other than itself: selection by
`argsort(kind="stable")`, keys by `numpy.sum` over float64, packing by
`numpy.ix_` slicing + `ascontiguousarray`, recovery by zeros + index assignment
(the operations Section 4.4.1 and 4.4.3 of the paper name for its own
implementation).  Used by tests only.
"""
import numpy as np

NONE, FILTER, CHANNEL, BOTH = 0, 1, 2, 3


def _layers(table):
    L = len(table["c_out"])
    gb = 0
    for l in range(L):
        co, ci, s = int(table["c_out"][l]), int(table["c_in"][l]), int(table["khw"][l])
        mode, k = int(table["mode"][l]), int(table["k"][l])
        G = ci if mode == CHANNEL else (co + ci if mode == BOTH else co)
        yield l, int(table["elem_off"][l]), co, ci, s, mode, k, G, gb
        gb += G


def project(table, W, U):
    R = W.shape[0]
    U_new = U.copy()
    Z = np.zeros_like(U)
    Wbar = np.zeros_like(U)
    masks, keys = [], []
    for l, off, co, ci, s, mode, k, G, gb in _layers(table):
        n = co * ci * s
        acc = W[0, off:off + n].astype(np.float32).copy()
        for r in range(1, R):
            acc = (acc + W[r, off:off + n]).astype(np.float32)
        wbar = (acc * (np.float32(1.0) / np.float32(R))).astype(np.float32)
        v = (wbar + U[off:off + n]).astype(np.float32)
        v3 = v.reshape(co, ci, s).astype(np.float64)
        if mode == BOTH:
            # the two projections one after the other: filters of v, then channels of what is left
            x = v.reshape(co, ci, s).copy()
            kf = np.sum(x.astype(np.float64) ** 2, axis=(1, 2))
            mf = np.zeros(co, dtype=np.uint8)
            mf[np.argsort(-kf, kind="stable")[:k]] = 1
            x[mf == 0] = np.float32(0)
            kc = np.sum(x.astype(np.float64) ** 2, axis=(0, 2))
            mc = np.zeros(ci, dtype=np.uint8)
            mc[np.argsort(-kc, kind="stable")[:int(table["k_in"][l])]] = 1
            x[:, mc == 0] = np.float32(0)
            z = x.reshape(-1)
            Z[off:off + n] = z
            U_new[off:off + n] = (U[off:off + n] + (wbar - z).astype(np.float32)).astype(np.float32)
            Wbar[off:off + n] = wbar
            masks.append(np.concatenate([mf, mc]))
            keys.append(np.concatenate([kf, kc]))
            continue
        if mode == CHANNEL:
            key = np.sum(v3 * v3, axis=(0, 2))
        else:
            key = np.sum(v3 * v3, axis=(1, 2))
        if mode == NONE:
            m = np.ones(G, dtype=np.uint8)
        else:
            order = np.argsort(-key, kind="stable")      # descending key, equal keys by index
            m = np.zeros(G, dtype=np.uint8)
            m[order[:k]] = 1
        m3 = m[None, :, None] if mode == CHANNEL else m[:, None, None]
        z = np.where(np.broadcast_to(m3.astype(bool), (co, ci, s)), v.reshape(co, ci, s),
                     np.float32(0)).astype(np.float32).reshape(-1)
        Z[off:off + n] = z
        U_new[off:off + n] = (U[off:off + n] + (wbar - z).astype(np.float32)).astype(np.float32)
        Wbar[off:off + n] = wbar
        masks.append(m)
        keys.append(key)
    return {"U": U_new, "Z": Z, "Wbar": Wbar, "mask": np.concatenate(masks), "key": np.concatenate(keys)}


def index_sets(mode, co, ci, m):
    if mode == BOTH:
        return np.nonzero(m[:co])[0], np.nonzero(m[co:])[0]
    k_out = np.nonzero(m)[0] if mode == FILTER else np.arange(co)
    k_in = np.nonzero(m)[0] if mode == CHANNEL else np.arange(ci)
    return k_out, k_in


def compact(table, src, mask, pack_align=1):
    chunks, offs, kept = [], [0], []
    pos = 0
    for l, off, co, ci, s, mode, k, G, gb in _layers(table):
        m = mask[gb:gb + G]
        k_out, k_in = index_sets(mode, co, ci, m)
        c = src[off:off + co * ci * s].reshape(co, ci, s)
        packed = np.ascontiguousarray(c[np.ix_(k_out, k_in)]).reshape(-1)
        chunks.append((pos, packed))
        pos += packed.size
        pos = -(-pos // pack_align) * pack_align
        offs.append(pos)
        kept.append(np.concatenate([k_out, k_in]) if mode == BOTH else (k_in if mode == CHANNEL else k_out))
    out = np.zeros(pos, dtype=np.float32)
    for p, c in chunks:
        out[p:p + c.size] = c
    return {"packed": out, "layer_off": np.array(offs, dtype=np.int64),
            "kept_idx": np.concatenate(kept).astype(np.int32)}


def expand(table, packed, mask, n_arena, pack_align=1):
    dst = np.zeros(n_arena, dtype=np.float32)
    pos = 0
    for l, off, co, ci, s, mode, k, G, gb in _layers(table):
        m = mask[gb:gb + G]
        k_out, k_in = index_sets(mode, co, ci, m)
        size = len(k_out) * len(k_in) * s
        z = np.zeros((co, ci, s), dtype=np.float32)
        z[np.ix_(k_out, k_in)] = packed[pos:pos + size].reshape(len(k_out), len(k_in), s)
        dst[off:off + co * ci * s] = z.reshape(-1)
        pos += size
        pos = -(-pos // pack_align) * pack_align
    return dst
