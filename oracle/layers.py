"""Sec. 4 "Model parallel layers": convolution, affine and pooling, each as
(i) the plain sequential definition and (ii) the paper's distributed forward /
adjoint algorithm composed from the primitives of Sec. 3, plus the point-wise
and loss glue used by the Sec. 5 / App. C network.

Shapes follow Sec. 4: x is [n_b, n_ci, m_0..m_{D-1}], w is
[n_co, n_ci, k_0..k_{D-1}], y is [n_b, n_co, n_0..n_{D-1}]; the affine weight
W is n_fo x n_fi and y = x W^T + b for x of shape [n_b, n_fi].
"Conv" is the cross-correlation of the framework layer the paper wraps
(Sec. 5 says the base layer function is the framework's own).

Everything is fp64.  Test infrastructure only.
"""
import numpy as np

from . import geometry as geo
from . import primitives as prim

_L = (slice(None), slice(None))

# --------------------------------------------------------------------------
# plain definitions (sequential layer functions)
# --------------------------------------------------------------------------


def _tap_view(xp, kappa, out_shape, stride, dilation, origin):
    """View of a padded input holding, for every output index o, the cell
    origin + o*s + kappa*dil read by kernel tap kappa."""
    sl = tuple(slice(origin[d] + kappa[d] * dilation[d],
                     origin[d] + kappa[d] * dilation[d] + stride[d] * (out_shape[d] - 1) + 1,
                     stride[d]) for d in range(len(out_shape)))
    return xp[_L + sl]


def conv_valid(xp, w, bias, out_shape, stride, dilation, origin):
    """y[n,co,o] = b[co] + sum_kappa sum_ci w[co,ci,kappa] xp[n,ci,origin+o*s+kappa*dil]
    on an input that already contains whatever padding it needs."""
    xp = np.asarray(xp, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    y = np.zeros((xp.shape[0], w.shape[0]) + tuple(out_shape))
    for kappa in np.ndindex(*w.shape[2:]):
        xs = _tap_view(xp, kappa, out_shape, stride, dilation, origin)
        y += np.einsum("oc,nc...->no...", w[_L + kappa], xs)
    if bias is not None:
        y += np.asarray(bias, dtype=np.float64).reshape((1, -1) + (1,) * len(out_shape))
    return y


def conv_valid_adjoint(xp, w, dy, stride, dilation, origin, want_bias=True):
    """Adjoint of the Jacobian of conv_valid with respect to xp, w and b:
      dxp[n,ci,origin+o*s+kappa*dil] += sum_co w[co,ci,kappa] dy[n,co,o]
      dw[co,ci,kappa] = sum_{n,o} dy[n,co,o] xp[n,ci,origin+o*s+kappa*dil]
      db[co] = sum_{n,o} dy[n,co,o]."""
    xp = np.asarray(xp, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    out_shape = dy.shape[2:]
    dxp = np.zeros_like(xp)
    dw = np.zeros_like(w)
    for kappa in np.ndindex(*w.shape[2:]):
        xs = _tap_view(xp, kappa, out_shape, stride, dilation, origin)
        dw[_L + kappa] = np.einsum("nos,ncs->oc", dy.reshape(dy.shape[:2] + (-1,)),
                                   xs.reshape(xs.shape[:2] + (-1,)))
        dxs = _tap_view(dxp, kappa, out_shape, stride, dilation, origin)
        dxs += np.einsum("oc,no...->nc...", w[_L + kappa], dy)
    db = dy.sum(axis=(0,) + tuple(range(2, dy.ndim))) if want_bias else None
    return dxp, dw, db


def _zero_pad(x, padding):
    return np.pad(np.asarray(x, dtype=np.float64),
                  [(0, 0), (0, 0)] + [(p, p) for p in padding])


def conv_forward(x, w, bias, stride, padding, dilation):
    """Sequential convolution layer: zero-pad by `padding`, then conv_valid."""
    D = x.ndim - 2
    out = [geo.output_length(x.shape[2 + d], w.shape[2 + d], stride[d], padding[d], dilation[d])
           for d in range(D)]
    return conv_valid(_zero_pad(x, padding), w, bias, out, stride, dilation, [0] * D)


def conv_backward(x, w, dy, stride, padding, dilation):
    """(dx, dw, db) of the sequential layer; dx drops the padding cells."""
    D = x.ndim - 2
    dxp, dw, db = conv_valid_adjoint(_zero_pad(x, padding), w, dy, stride, dilation, [0] * D)
    core = tuple(slice(padding[d], padding[d] + x.shape[2 + d]) for d in range(D))
    return dxp[_L + core], dw, db


def affine_forward(x, W, b):
    """y = x W^T + b (Sec. 4 "Dense layers")."""
    y = np.asarray(x, dtype=np.float64) @ np.asarray(W, dtype=np.float64).T
    return y if b is None else y + np.asarray(b, dtype=np.float64)[None, :]


def affine_backward(x, W, dy):
    x, W, dy = (np.asarray(t, dtype=np.float64) for t in (x, W, dy))
    return dy @ W, dy.T @ x, dy.sum(axis=0)        # dx, dW, db


def relu(x):
    return np.maximum(x, 0.0)


def relu_backward(x, dy):
    """Derivative taken as 0 at x == 0."""
    return np.where(x > 0, dy, 0.0)


def maxpool_valid(xp, ksize, stride, out_shape, origin):
    """Max over each window of an already-trimmed / padded input; also returns,
    per output, the row-major index of the first maximal tap."""
    best = None
    arg = None
    for t, kappa in enumerate(np.ndindex(*ksize)):
        xs = _tap_view(xp, kappa, out_shape, stride, [1] * len(ksize), origin)
        if best is None:
            best, arg = xs.copy(), np.zeros(xs.shape, dtype=np.int64)
        else:
            better = xs > best                      # strict: first maximum wins
            best = np.where(better, xs, best)
            arg = np.where(better, t, arg)
    return best, arg


def maxpool_valid_adjoint(dy, arg, xp_shape, ksize, stride, origin):
    dxp = np.zeros(xp_shape)
    out_shape = dy.shape[2:]
    for t, kappa in enumerate(np.ndindex(*ksize)):
        dxs = _tap_view(dxp, kappa, out_shape, stride, [1] * len(ksize), origin)
        dxs += np.where(arg == t, dy, 0.0)
    return dxp


def avgpool_valid(xp, ksize, stride, out_shape, origin):
    """Mean over each window of an already-trimmed / padded input: the sum of
    the window's taps divided by the window size (padding cells count as the
    zeros they hold)."""
    xp = np.asarray(xp, dtype=np.float64)
    y = None
    for kappa in np.ndindex(*ksize):
        xs = _tap_view(xp, kappa, out_shape, stride, [1] * len(ksize), origin)
        y = xs.copy() if y is None else y + xs
    return y / float(np.prod(ksize))


def avgpool_valid_adjoint(dy, xp_shape, ksize, stride, origin):
    """Adjoint of avgpool_valid (it is linear): every tap of window o receives
    dy[o] / window size."""
    dxp = np.zeros(xp_shape)
    out_shape = dy.shape[2:]
    share = np.asarray(dy, dtype=np.float64) / float(np.prod(ksize))
    for kappa in np.ndindex(*ksize):
        dxs = _tap_view(dxp, kappa, out_shape, stride, [1] * len(ksize), origin)
        dxs += share
    return dxp


def mse_loss(y, target):
    """mean((y - t)^2) over every element, and its gradient."""
    diff = np.asarray(y, dtype=np.float64) - target
    return float(np.mean(diff * diff)), 2.0 * diff / diff.size


# --------------------------------------------------------------------------
# distributed convolution, feature-space partition only (P_co = P_ci = 1)
# --------------------------------------------------------------------------


def dist_conv_forward(x_bufs, w, bias, part, stride, dilation):
    """Forward Convolution Algorithm of Sec. 4 with P_co = P_ci = 1.
    x_bufs: per-worker padded buffers with the bulk filled.  Steps, in the
    paper's order: x <- H x; w^ <- B w; b^ <- B b; x^ <- B x (identity here);
    y^ <- Conv(w^, b^; x^) on each worker's own buffer with no further
    padding, starting at that worker's origin; y <- R y^ (identity here).
    Returns the list of per-worker outputs; x_bufs holds H x afterwards."""
    P = part.n_workers
    prim.halo_exchange(x_bufs, part)
    w_hat = prim.broadcast(np.asarray(w, dtype=np.float64), P)
    b_hat = prim.broadcast(np.asarray(bias, dtype=np.float64), P) if bias is not None else [None] * P
    y_hat = []
    for wk in range(P):
        origin = [part.g(wk, d)["origin"] for d in range(part.D)]
        y_hat.append(conv_valid(x_bufs[wk], w_hat[wk], b_hat[wk], part.out_shape(wk),
                                stride, dilation, origin))
    return y_hat


def dist_conv_adjoint(x_bufs, w, dy_parts, part, stride, dilation, want_bias=True):
    """Adjoint Convolution Algorithm of Sec. 4 with P_co = P_ci = 1:
    dy^ <- B dy (identity); (dw^, db^, dx^) <- [dConv]*(dy^) per worker, dx^
    covering the whole padded buffer; dx <- R dx^ (identity); db <- R db^ and
    dw <- R dw^ over all workers (adjoint of the forward broadcasts);
    dx <- H* dx.  x_bufs must hold H x (saved by the forward pass).
    Returns (dx_bufs, dw, db)."""
    P = part.n_workers
    w_hat = prim.broadcast(np.asarray(w, dtype=np.float64), P)
    dx_hat, dw_hat, db_hat = [], [], []
    for wk in range(P):
        origin = [part.g(wk, d)["origin"] for d in range(part.D)]
        dxp, dw_k, db_k = conv_valid_adjoint(x_bufs[wk], w_hat[wk], dy_parts[wk],
                                             stride, dilation, origin, want_bias)
        dx_hat.append(dxp)
        dw_hat.append(dw_k)
        db_hat.append(db_k)
    dw = prim.sum_reduce(dw_hat)
    db = prim.sum_reduce(db_hat) if want_bias else None
    prim.halo_exchange_adjoint(dx_hat, part)
    return dx_hat, dw, db


# --------------------------------------------------------------------------
# distributed convolution with the channels partitioned too (P_co, P_ci >= 1)
# --------------------------------------------------------------------------


def dist_conv_cp_forward(x_bufs, w_blocks, b_blocks, part, P_co, P_ci, stride, dilation):
    """Forward Convolution Algorithm of Sec. 4 on a P_co x P_ci x (feature
    space) partition.  x_bufs[j][s]: padded buffer of input-channel block j on
    spatial worker s; w_blocks[i][j]: [co_i, ci_j, k..]; b_blocks[i] (or None)
    lives on the ci = 0 sub-partition only.  Steps in the paper's order:
    x <- H x (per channel block); x^ <- B x along P_co; y^_ij <- Conv(w_ij,
    b_i if j == 0; x^_j) per worker; y_i <- R over j of y^_ij.
    Returns y[i][s]; x_bufs holds H x afterwards."""
    S = part.n_workers
    for j in range(P_ci):
        prim.halo_exchange(x_bufs[j], part)
    x_hat = [[prim.broadcast(np.asarray(x_bufs[j][s], dtype=np.float64), P_co) for s in range(S)] for j in range(P_ci)]
    y = []
    for i in range(P_co):
        y_i = []
        for s in range(S):
            origin = [part.g(s, d)["origin"] for d in range(part.D)]
            y_hat = [conv_valid(x_hat[j][s][i], w_blocks[i][j], b_blocks[i] if (b_blocks is not None and j == 0) else None,
                                part.out_shape(s), stride, dilation, origin) for j in range(P_ci)]
            y_i.append(prim.sum_reduce(y_hat))
        y.append(y_i)
    return y


def dist_conv_cp_adjoint(x_bufs, w_blocks, dy, part, P_co, P_ci, stride, dilation, want_bias=True):
    """Adjoint Convolution Algorithm of Sec. 4 on the same partition:
    dy^_ij <- B dy_i along P_ci (adjoint of the forward sum-reduce);
    (dw^_ijs, db^_is, dx^_ijs) <- [dConv]*(dy^_ij) per worker; dx_j <- R over i
    of dx^_ij (adjoint of the forward broadcast of x); dw_ij, db_i <- R over
    the spatial workers; dx_j <- H* dx_j.  x_bufs must hold H x.
    Returns (dx[j][s], dw[i][j], db[i])."""
    S = part.n_workers
    dy_hat = [[prim.broadcast(np.asarray(dy[i][s], dtype=np.float64), P_ci) for s in range(S)] for i in range(P_co)]
    dw = [[None] * P_ci for _ in range(P_co)]
    db = [None] * P_co
    dx_hat = [[[None] * S for _ in range(P_co)] for _ in range(P_ci)]
    for i in range(P_co):
        for j in range(P_ci):
            dw_s, db_s = [], []
            for s in range(S):
                origin = [part.g(s, d)["origin"] for d in range(part.D)]
                dxp, dw_k, db_k = conv_valid_adjoint(x_bufs[j][s], w_blocks[i][j], dy_hat[i][s][j], stride, dilation,
                                                     origin, want_bias and j == 0)
                dx_hat[j][i][s] = dxp
                dw_s.append(dw_k)
                db_s.append(db_k)
            dw[i][j] = prim.sum_reduce(dw_s)
            if want_bias and j == 0:
                db[i] = prim.sum_reduce(db_s)
    dx = []
    for j in range(P_ci):
        dx_j = [prim.sum_reduce([dx_hat[j][i][s] for i in range(P_co)]) for s in range(S)]
        prim.halo_exchange_adjoint(dx_j, part)
        dx.append(dx_j)
    return dx, dw, (db if want_bias else None)


# --------------------------------------------------------------------------
# distributed pooling
# --------------------------------------------------------------------------


def padding_mask(part, wk):
    """Boolean array over worker wk's buffer (feature dims): True on the cells
    that lie outside the global domain (the zero padding)."""
    mask = np.zeros(part.buf_shape(wk), dtype=bool)
    for d in range(part.D):
        g = part.g(wk, d)
        idx = [slice(None)] * part.D
        idx[d] = slice(0, g["pad"][0])
        mask[tuple(idx)] = True
        idx[d] = slice(g["buf"] - g["pad"][1], g["buf"])
        mask[tuple(idx)] = True
    return mask


def dist_maxpool_forward(x_bufs, part, ksize, stride):
    """Forward Pooling Algorithm of Sec. 4: x <- H x; y <- Pool(x), the local
    pool starting at each worker's origin (which skips "extra" input).
    Sec. 4 only says that pooling needs padding shims and takes the layer
    function from the framework it wraps; that framework's max-pool pads with
    -inf, i.e. the maximum runs over the cells of the tensor itself.  So the
    padding cells (zeros in the buffer, as every sliding-kernel layer shares
    one H) are masked to -inf for the local max: they never win and never
    receive gradient."""
    prim.halo_exchange(x_bufs, part)
    ys, args = [], []
    for wk in range(part.n_workers):
        origin = [part.g(wk, d)["origin"] for d in range(part.D)]
        xb = np.array(x_bufs[wk], dtype=np.float64)
        xb[:, :, padding_mask(part, wk)] = -np.inf
        y, a = maxpool_valid(xb, ksize, stride, part.out_shape(wk), origin)
        ys.append(y)
        args.append(a)
    return ys, args


def dist_maxpool_adjoint(dy_parts, args, part, buf_shapes, ksize, stride):
    """Adjoint Pooling Algorithm of Sec. 4: dx <- [dPool]*(dy); dx <- H* dx."""
    dx = []
    for wk in range(part.n_workers):
        origin = [part.g(wk, d)["origin"] for d in range(part.D)]
        dx.append(maxpool_valid_adjoint(dy_parts[wk], args[wk], buf_shapes[wk], ksize, stride, origin))
    prim.halo_exchange_adjoint(dx, part)
    return dx


def dist_avgpool_forward(x_bufs, part, ksize, stride):
    """Forward Pooling Algorithm of Sec. 4 with the mean as the local pool."""
    prim.halo_exchange(x_bufs, part)
    return [avgpool_valid(x_bufs[wk], ksize, stride, part.out_shape(wk),
                          [part.g(wk, d)["origin"] for d in range(part.D)]) for wk in range(part.n_workers)]


def dist_avgpool_adjoint(dy_parts, part, buf_shapes, ksize, stride):
    """Adjoint Pooling Algorithm of Sec. 4 with the mean: dx <- [dPool]*(dy); dx <- H* dx."""
    dx = [avgpool_valid_adjoint(dy_parts[wk], buf_shapes[wk], ksize, stride,
                                [part.g(wk, d)["origin"] for d in range(part.D)]) for wk in range(part.n_workers)]
    prim.halo_exchange_adjoint(dx, part)
    return dx


# --------------------------------------------------------------------------
# distributed affine on a P_fo x P_fi weight partition
# --------------------------------------------------------------------------


def feature_blocks(n, parts):
    return [slice(s, s + z) for (s, z) in geo.balanced_split(n, parts)]


def dist_affine_forward(x_parts, W_parts, b_parts, P_fo, P_fi):
    """Forward Affine Algorithm of Sec. 4.  x_parts[j] is [n_b, fi_j];
    W_parts[i][j] is [fo_i, fi_j]; b_parts[i] (or None) lives on column j = 0
    only.  x^_ij <- B x_j along P_fo; y^_ij <- Affine(W_ij, b_ij; x^_ij);
    y_i <- R over j of y^_ij."""
    x_hat = [prim.broadcast(np.asarray(x_parts[j], dtype=np.float64), P_fo) for j in range(P_fi)]
    y = []
    for i in range(P_fo):
        y_hat_i = []
        for j in range(P_fi):
            b_ij = b_parts[i] if (j == 0 and b_parts is not None) else None
            y_hat_i.append(affine_forward(x_hat[j][i], W_parts[i][j], b_ij))
        y.append(prim.sum_reduce(y_hat_i))
    return y


def dist_affine_adjoint(x_parts, W_parts, dy_parts, P_fo, P_fi):
    """Adjoint Affine Algorithm of Sec. 4: dy^_ij <- B dy_i along P_fi;
    (dW_ij, db_i [j = 0], dx^_ij) <- [dAffine]*(dy^_ij); dx_j <- R over i.
    Returns (dx_parts, dW_parts, db_parts)."""
    dy_hat = [prim.broadcast(np.asarray(dy_parts[i], dtype=np.float64), P_fi) for i in range(P_fo)]
    dW = [[None] * P_fi for _ in range(P_fo)]
    db = [None] * P_fo
    dx_hat = [[None] * P_fo for _ in range(P_fi)]
    for i in range(P_fo):
        for j in range(P_fi):
            dx_ij, dW_ij, db_ij = affine_backward(x_parts[j], W_parts[i][j], dy_hat[i][j])
            dW[i][j] = dW_ij
            dx_hat[j][i] = dx_ij
            if j == 0:
                db[i] = db_ij
    dx = [prim.sum_reduce(dx_hat[j]) for j in range(P_fi)]
    return dx, dW, db


# --------------------------------------------------------------------------
# repartition ("transpose" / generalized all-to-all glue, Sec. 3)
# --------------------------------------------------------------------------


def repartition_spatial_to_features(y_parts, part, P_fi):
    """Block permutation (Sec. 3 "Generalized all-to-all"): gather the
    spatially partitioned [n_b, c, h, w] blocks, flatten to [n_b, c*h*w]
    (row-major, the framework's flatten) and split the features over P_fi."""
    full = prim.gather_out(y_parts, part)
    flat = full.reshape(full.shape[0], -1)
    return [flat[:, s].copy() for s in feature_blocks(flat.shape[1], P_fi)]


def repartition_features_to_spatial(dx_parts, part, n_c):
    """Adjoint (= inverse) of the permutation above."""
    flat = np.concatenate(dx_parts, axis=1)
    full = flat.reshape((flat.shape[0], n_c) + part.global_out_shape())
    return prim.scatter_out(full, part)
