"""Marshalling between named logical tensors (filters KCRS) and the library's flat parameter arenas (filters KRSC,
parameter-table order).  No arithmetic: reshapes, transposes and concatenation only."""
import numpy as np

from . import binding as rn


def logical_table():
    """[(name, logical shape, kind name)] in arena order; filters are reported as (K, C, R, S)."""
    out = []
    for name, off, cnt, dims, kind in rn.rn50_param_table():
        if kind == 0:
            k, r, s, c = dims
            shape = (k, c, r, s)
        elif kind == 3:
            shape = (dims[0], dims[1])
        else:
            shape = (dims[0],)
        out.append((name, shape, rn.KIND_NAMES[kind]))
    return out


def flat_from_dict(tensors, dtype=np.float32):
    """{name: logical array} -> flat arena in the library's order and layout."""
    parts = []
    for name, off, cnt, dims, kind in rn.rn50_param_table():
        a = np.asarray(tensors[name])
        if kind == 0:
            a = np.transpose(a, (0, 2, 3, 1))
        parts.append(np.ascontiguousarray(a, dtype=dtype).ravel())
        assert parts[-1].size == cnt, name
    return np.concatenate(parts)


def dict_from_flat(flat):
    """flat arena -> {name: logical float64 array (filters KCRS)}"""
    out = {}
    for name, off, cnt, dims, kind in rn.rn50_param_table():
        a = np.asarray(flat[off:off + cnt], dtype=np.float64)
        if kind == 0:
            k, r, s, c = dims
            a = np.transpose(a.reshape(k, r, s, c), (0, 3, 1, 2))
        elif kind == 3:
            a = a.reshape(dims[0], dims[1])
        out[name] = a
    return out
