"""Sec. 3 "Linear algebraic primitives for data movement": broadcast,
sum-reduce, all-reduce, scatter / gather, and the generalized halo exchange
H with its adjoint H*, plus the adjoint ("dot-product") test.

A distributed tensor is a Python list with one numpy array per worker; the
space it lives in is the direct sum of the workers' memories with the
Euclidean inner product summed over workers (Sec. 2, Sec. 3 first paragraph).

Sliding-kernel buffers have logical shape [n_b, n_c, buf_0, ..., buf_{D-1}]
(Sec. 4 "Sparse layers" shape convention); along every feature dimension a
buffer is laid out  [ pad_L | halo_L | bulk | halo_R | pad_R ].

Test infrastructure only.
"""
import numpy as np

# --------------------------------------------------------------------------
# inner products and the adjoint test
# --------------------------------------------------------------------------


def inner(a, b):
    """Euclidean inner product on the direct sum of the workers' memories
    (Sec. 2, second displayed equation), accumulated in fp64."""
    if isinstance(a, np.ndarray):
        a, b = [a], [b]
    tot = 0.0
    for u, v in zip(a, b):
        tot += float(np.sum(u.astype(np.float64) * v.astype(np.float64)))
    return tot


def norm(a):
    return float(np.sqrt(inner(a, a)))


def adjoint_test_ratio(Fx, y, x, Fsy):
    """Left-hand side of the adjoint test (Sec. 3 "Implementation"):
    |<Fx,y> - <x,F*y>| / max(|Fx||y|, |x||F*y|)."""
    num = abs(inner(Fx, y) - inner(x, Fsy))
    den = max(norm(Fx) * norm(y), norm(x) * norm(Fsy))
    return num / den if den > 0 else num


# --------------------------------------------------------------------------
# broadcast / sum-reduce / all-reduce
# --------------------------------------------------------------------------


def broadcast(x_a, k):
    """B_{a->{k}} (Sec. 3 "Broadcast"): k out-of-place copies of x_a."""
    return [x_a.copy() for _ in range(k)]


def broadcast_adjoint(y_k, clear_inputs=False):
    """B*_{a->{k}} y = sum_{i=0}^{k-1} K_i S_{i->a} y_i (Sec. 3 "Broadcast"):
    a sum-reduction in index order, accumulated in fp64 and returned in the
    input dtype's fp64 image.  With clear_inputs the K_i are applied."""
    acc = np.zeros(y_k[0].shape, dtype=np.float64)
    for y_i in y_k:                       # i = 0 .. k-1, S_{i->a}
        acc = acc + y_i.astype(np.float64)
    if clear_inputs:
        for y_i in y_k:                   # K_i
            y_i[...] = 0
    return acc


def sum_reduce(x_k, clear_inputs=False):
    """R_{{k}->a} = B*_{a->{k}} (Sec. 3 "Sum-reduce and all-reduce")."""
    return broadcast_adjoint(x_k, clear_inputs)


def sum_reduce_adjoint(y_a, k):
    """R*_{{k}->a} = B_{a->{k}}."""
    return broadcast(y_a, k)


def all_reduce(x_k):
    """A = B R (Sec. 3): every worker ends with the sum.  Self-adjoint."""
    return broadcast(sum_reduce(x_k), len(x_k))


# --------------------------------------------------------------------------
# scatter / gather between a global tensor and per-worker padded buffers
# --------------------------------------------------------------------------


def scatter_bulk(x_global, part, fill=0.0):
    """Sec. 3 "Scatter and Gather": copy each worker's owned block of the
    global tensor [n_b, n_c, m_0..] into the bulk of a fresh padded buffer.
    Non-bulk cells are set to `fill` (use NaN or noise to prove that H does
    not depend on their previous contents)."""
    bufs = []
    for w in range(part.n_workers):
        shape = x_global.shape[:2] + part.buf_shape(w)
        b = np.full(shape, fill, dtype=x_global.dtype)
        b[(slice(None), slice(None)) + part.bulk_slices(w)] = \
            x_global[(slice(None), slice(None)) + part.global_in_slices(w)]
        bufs.append(b)
    return bufs


def gather_bulk(bufs, part):
    """Inverse of scatter_bulk on the bulk cells (a move-type gather)."""
    shape = bufs[0].shape[:2] + part.global_in_shape()
    out = np.zeros(shape, dtype=bufs[0].dtype)
    for w in range(part.n_workers):
        out[(slice(None), slice(None)) + part.global_in_slices(w)] = \
            bufs[w][(slice(None), slice(None)) + part.bulk_slices(w)]
    return out


def gather_out(y_parts, part):
    """Assemble the per-worker output blocks [n_b, n_c, out_0..] into the
    global output tensor."""
    shape = y_parts[0].shape[:2] + part.global_out_shape()
    out = np.zeros(shape, dtype=y_parts[0].dtype)
    for w in range(part.n_workers):
        out[(slice(None), slice(None)) + part.global_out_slices(w)] = y_parts[w]
    return out


def scatter_out(y_global, part):
    return [y_global[(slice(None), slice(None)) + part.global_out_slices(w)].copy()
            for w in range(part.n_workers)]


# --------------------------------------------------------------------------
# halo exchange, nested form: the paper's operator product
# --------------------------------------------------------------------------


def _pad_slabs(part, w):
    """Index tuples (over feature dims) of w's zero-padding cells: every cell
    whose coordinate in at least one dimension lies in pad_L or pad_R."""
    slabs = []
    for d in range(part.D):
        g = part.g(w, d)
        full = [slice(None)] * part.D
        if g["pad"][0]:
            s = list(full)
            s[d] = slice(0, g["pad"][0])
            slabs.append(tuple(s))
        if g["pad"][1]:
            s = list(full)
            s[d] = slice(g["buf"] - g["pad"][1], g["buf"])
            slabs.append(tuple(s))
    return slabs


def clear_pad(bufs, part):
    """K on the zero-padding cells (the "padding shim" of Sec. 4 taken to be
    part of the buffer)."""
    for w in range(part.n_workers):
        for s in _pad_slabs(part, w):
            bufs[w][(slice(None), slice(None)) + s] = 0


def _exchange_slabs(part, w, a, side):
    """For worker w receiving along dimension a on `side` (0 left, 1 right):
    returns (neighbour, slab in the neighbour's buffer that is packed,
    slab in w's buffer that is unpacked), or None when that halo is empty.

    Thickness is the receiver's halo width.  In dimensions before a the slab
    spans the full buffer (those halos are already exchanged, which is how
    corner data travels -- Sec. 3, nested exchange); in dimensions after a it
    spans the bulk only (minimum volume, App. B.2)."""
    g = part.g(w, a)
    h = g["halo"][side]
    if h == 0:
        return None
    nb = part.neighbour(w, a, side)
    gn = part.g(nb, a)
    src, dst = [], []
    for d in range(part.D):
        gd = part.g(w, d)                # same for w and nb when d != a
        if d < a:
            src.append(slice(0, gd["buf"]))
            dst.append(slice(0, gd["buf"]))
        elif d > a:
            sl = slice(gd["bulk_off"], gd["bulk_off"] + gd["in_size"])
            src.append(sl)
            dst.append(sl)
        else:
            if side == 0:   # left halo <- last h bulk cells of the left neighbour
                s0 = gn["bulk_off"] + gn["in_size"] - h
                src.append(slice(s0, s0 + h))
                dst.append(slice(g["bulk_off"] - h, g["bulk_off"]))
            else:           # right halo <- first h bulk cells of the right one
                src.append(slice(gn["bulk_off"], gn["bulk_off"] + h))
                e0 = g["bulk_off"] + g["in_size"]
                dst.append(slice(e0, e0 + h))
    lead = (slice(None), slice(None))
    return nb, lead + tuple(src), lead + tuple(dst)


def halo_exchange(bufs, part):
    """H = (prod over a = D-1..0 of K_T C_U C_E C_P K_S)_a applied after the
    pad clear (Sec. 3 "Halo exchange", second displayed operator product).
    In-place on the list of buffers; dimension 0 is exchanged first."""
    clear_pad(bufs, part)
    for a in range(part.D):
        plans = [(w, side, _exchange_slabs(part, w, a, side))
                 for w in range(part.n_workers) for side in (0, 1)]
        plans = [(w, side, p) for (w, side, p) in plans if p is not None]
        send, recv = {}, {}
        for w, side, (nb, src, dst) in plans:          # K_S: zeroed buffers
            send[(nb, w, side)] = np.zeros_like(bufs[nb][src])
            recv[(w, side)] = np.zeros_like(bufs[w][dst])
        for w, side, (nb, src, dst) in plans:          # C_P: bulk -> send
            send[(nb, w, side)][...] = bufs[nb][src]
        for w, side, (nb, src, dst) in plans:          # C_E: send -> recv
            recv[(w, side)][...] = send[(nb, w, side)]
        for w, side, (nb, src, dst) in plans:          # C_U: recv -> halo
            bufs[w][dst] = recv[(w, side)]
        for key in send:                               # K_T
            send[key][...] = 0
        for key in recv:
            recv[key][...] = 0
    return bufs


def halo_exchange_adjoint(bufs, part):
    """H* (Sec. 3 "Halo exchange", third displayed operator product): the
    factors of H adjointed and applied in reverse order, dimension D-1 first.
    Each in-place copy C_{a->b} = S_{a->b} K_b turns into C* = K_b S_{b->a}:
    add the destination back into the source, then clear the destination --
    which is where the add into the neighbour's bulk comes from."""
    for a in reversed(range(part.D)):
        plans = [(w, side, _exchange_slabs(part, w, a, side))
                 for w in range(part.n_workers) for side in (0, 1)]
        plans = [(w, side, p) for (w, side, p) in plans if p is not None]
        send, recv = {}, {}
        for w, side, (nb, src, dst) in plans:          # K_T* = K_T
            send[(nb, w, side)] = np.zeros_like(bufs[nb][src])
            recv[(w, side)] = np.zeros_like(bufs[w][dst])
        for w, side, (nb, src, dst) in plans:          # C_U*: recv += halo; halo = 0
            recv[(w, side)] += bufs[w][dst]
            bufs[w][dst] = 0
        for w, side, (nb, src, dst) in plans:          # C_E*: send += recv; recv = 0
            send[(nb, w, side)] += recv[(w, side)]
            recv[(w, side)][...] = 0
        for w, side, (nb, src, dst) in plans:          # C_P*: bulk += send; send = 0
            bufs[nb][src] += send[(nb, w, side)]
            send[(nb, w, side)][...] = 0
        # K_S* = K_S: buffers are already zero
    clear_pad(bufs, part)
    return bufs


# --------------------------------------------------------------------------
# halo exchange, direct form: the plain definition of what H and H* compute
# --------------------------------------------------------------------------


def _global_index_of(part, w, d, c):
    g = part.g(w, d)
    return g["in_start"] - g["halo"][0] - g["pad"][0] + c


def halo_exchange_direct(bufs, part):
    """What H leaves behind, stated cell by cell: every in-domain cell of
    every buffer holds the global tensor's value at that cell's global index
    (owned cells keep theirs; non-owned ones get the owner's), every
    out-of-domain cell is zero.  Pure-Python loops: small cases only."""
    x_global = gather_bulk(bufs, part)
    n_glob = part.global_in_shape()
    for w in range(part.n_workers):
        for c in np.ndindex(*part.buf_shape(w)):
            gidx = tuple(_global_index_of(part, w, d, c[d]) for d in range(part.D))
            inside = all(0 <= gidx[d] < n_glob[d] for d in range(part.D))
            sl = (slice(None), slice(None))
            bufs[w][sl + c] = x_global[sl + gidx] if inside else 0
    return bufs


def halo_exchange_adjoint_direct(bufs, part):
    """What H* leaves behind, cell by cell: every bulk cell has gained the sum
    of all non-owned cells (in any worker) that share its global index; all
    halo and pad cells are zero."""
    n_glob = part.global_in_shape()
    acc = np.zeros(bufs[0].shape[:2] + n_glob, dtype=np.float64)
    sl = (slice(None), slice(None))
    for w in range(part.n_workers):            # ascending worker order
        for c in np.ndindex(*part.buf_shape(w)):
            gidx = tuple(_global_index_of(part, w, d, c[d]) for d in range(part.D))
            if all(0 <= gidx[d] < n_glob[d] for d in range(part.D)):
                acc[sl + gidx] += bufs[w][sl + c]
    for w in range(part.n_workers):
        bufs[w][...] = 0
        bufs[w][sl + part.bulk_slices(w)] = acc[sl + part.global_in_slices(w)]
    return bufs


def adjoint_multiplicity(part, w):
    """H* applied to a buffer of ones, in closed form (a pin for H*, Sec. 3
    "Halo exchange"): bulk cell i of worker w ends as the number of buffer
    cells, in all workers, that hold global index i, i.e. the product over
    the dimensions of 1 + (neighbours along d whose halo covers i_d).  Returns
    an integer array over the worker's bulk."""
    out = np.ones([part.g(w, d)["in_size"] for d in range(part.D)], dtype=np.int64)
    for d in range(part.D):
        g = part.g(w, d)
        count = np.ones(g["in_size"], dtype=np.int64)
        left, right = part.neighbour(w, d, 0), part.neighbour(w, d, 1)
        if left is not None:            # the left neighbour's right halo covers my first cells
            count[:part.g(left, d)["halo"][1]] += 1
        if right is not None:           # the right neighbour's left halo covers my last cells
            hl = part.g(right, d)["halo"][0]
            if hl:
                count[-hl:] += 1
        shape = [1] * part.D
        shape[d] = g["in_size"]
        out = out * count.reshape(shape)
    return out


def expected_buffer_after_halo(x_global, part, w):
    """Worker w's buffer after H, by slicing the zero-extended global tensor
    (vectorised statement of halo_exchange_direct for one worker; used for
    sampled parity at sizes where the loops above are too slow)."""
    lo, hi, padw = [], [], []
    n_glob = part.global_in_shape()
    for d in range(part.D):
        g = part.g(w, d)
        start = g["in_start"] - g["halo"][0] - g["pad"][0]
        lo.append(start)
        hi.append(start + g["buf"])
    src = tuple(slice(max(lo[d], 0), min(hi[d], n_glob[d])) for d in range(part.D))
    dst = tuple(slice(max(lo[d], 0) - lo[d], min(hi[d], n_glob[d]) - lo[d])
                for d in range(part.D))
    out = np.zeros(x_global.shape[:2] + part.buf_shape(w), dtype=x_global.dtype)
    sl = (slice(None), slice(None))
    out[sl + dst] = x_global[sl + src]
    return out


# --------------------------------------------------------------------------
# generalized all-to-all: the same tensor under another partition
# --------------------------------------------------------------------------


def partition_blocks(shape, P):
    """Per worker (row-major over the partition vector P) the tuple of slices
    of its block of a tensor of the given shape, every dimension split by the
    balanced rule."""
    import itertools
    from . import geometry as geo
    splits = [geo.balanced_split(int(n), int(p)) for n, p in zip(shape, P)]
    return [tuple(slice(splits[d][c][0], splits[d][c][0] + splits[d][c][1]) for d, c in enumerate(coords))
            for coords in itertools.product(*[range(int(p)) for p in P])]


def repartition(blocks_src, shape, P_src, P_dst):
    """Generalized all-to-all of Sec. 3 ("all-to-all" / repartition): the
    tensor held as blocks of partition P_src, re-cut into the blocks of
    partition P_dst.  Stated through the global tensor: gather, then scatter
    (Sec. 3 "Scatter and Gather").  A permutation of the elements, so its
    adjoint is the inverse: repartition(., shape, P_dst, P_src)."""
    full = np.empty(tuple(int(n) for n in shape), dtype=np.asarray(blocks_src[0]).dtype)
    for blk, sl in zip(blocks_src, partition_blocks(shape, P_src)):
        full[sl] = blk
    return [full[sl].copy() for sl in partition_blocks(shape, P_dst)]
