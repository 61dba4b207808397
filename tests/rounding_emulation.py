"""The layer with the roundings the bf16 kernels are defined with, in otherwise exact (fp64)
arithmetic, on the CPU: silu(gate) * up is rounded to bf16 once before the down projection,
every expert output row is rounded to bf16 once, the gate-weighted sum once at the end, and
the sum with returned remote rows once more.  The oracle rounds only at the end; the gap
between the two is what the output tolerance has to absorb whatever the kernels do, which
is how tests/test_error_measure.py uses this file.  Test infrastructure: numpy only, no code
shared with the HIP path; routing and the split are taken from the oracle's result."""
import numpy as np

from oracle import prism_oracle as O


def _stored(a, dtype):
    """Values as a buffer of the layer dtype holds them."""
    return O.round_to_dtype(a, dtype).astype(np.float64)


def ffn_rows(xr, weights, dtype):
    wg, wu, wd = (np.asarray(w, dtype=np.float64) for w in weights)
    g = xr @ wg.T
    u = xr @ wu.T
    h = _stored((g / (1.0 + np.exp(-g))) * u, dtype)
    return _stored(h @ wd.T, dtype)


def emulate(inp, route, dispatch):
    """-> dict with y (local rows, then S*T shared rows), out (local partial sum), y_remote
    (rows of the remote list run on a peer hosting every expert) and done (out plus the
    returned rows), each as stored in the layer dtype."""
    c = inp.cfg
    f = inp.f32
    x = f(inp.x).astype(np.float64)
    T, H = x.shape
    k, dtype = c.k, c.dtype

    def grouped(src, offsets):
        y = np.zeros((len(src), H))
        for e in range(c.E):
            b, en = int(offsets[e]), int(offsets[e + 1])
            if en > b:
                y[b:en] = ffn_rows(x[np.asarray(src[b:en]) // k], tuple(f(w) for w in inp.expert(e)), dtype)
        return y

    def weighted(acc, y, src):
        row_of = {int(a): i for i, a in enumerate(src)}
        for t in range(T):
            for j in range(k):
                i = row_of.get(t * k + j)
                if i is not None:
                    acc[t] += float(route.topk_gate[t, j]) * y[i]
        return acc

    y_local = grouped(dispatch.local_src, dispatch.local_offsets)
    y_shared = [ffn_rows(x, tuple(f(w) for w in inp.shared(s)), dtype) for s in range(c.S)]
    acc = weighted(np.zeros((T, H)), y_local, dispatch.local_src)
    for ys in y_shared:
        acc += ys
    out = _stored(acc, dtype)
    y_remote = grouped(dispatch.remote_src, dispatch.remote_offsets)
    done = _stored(weighted(out.copy(), y_remote, dispatch.remote_src), dtype)
    return dict(y=np.concatenate([y_local] + y_shared) if c.S else y_local, out=out,
                y_remote=y_remote, done=done)
