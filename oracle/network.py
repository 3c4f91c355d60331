"""The Sec. 5 / App. C example network, shaped as in the benchmark's small-CNN
configuration: conv5x5(6, padding 2) - ReLU - maxpool2 - conv5x5(16) - ReLU -
maxpool2 - affine 400-120 - ReLU - affine 120-84 - ReLU - affine 84-10, MSE
loss on one-hot targets.  Sequential definition and the distributed version
(conv / pool layers on a 2x2 feature-space partition, affine layers on 2x2
weight partitions, a repartition as glue) with full forward + adjoint passes.

Test infrastructure only.
"""
import numpy as np

from . import geometry as geo
from . import layers
from . import primitives as prim

ONE2 = (1, 1)


def sequential_step(images, target, p):
    """Forward and backward through the plain network.  Returns (loss, grads)
    with grads keyed like the parameter dict plus 'images'."""
    a1 = layers.conv_forward(images, p["c1_w"], p["c1_b"], ONE2, (2, 2), ONE2)
    r1 = layers.relu(a1)
    s2, arg2 = layers.maxpool_valid(r1, (2, 2), (2, 2), (14, 14), (0, 0))
    a3 = layers.conv_forward(s2, p["c3_w"], p["c3_b"], ONE2, (0, 0), ONE2)
    r3 = layers.relu(a3)
    s4, arg4 = layers.maxpool_valid(r3, (2, 2), (2, 2), (5, 5), (0, 0))
    f = s4.reshape(s4.shape[0], -1)
    a5 = layers.affine_forward(f, p["c5_w"], p["c5_b"])
    r5 = layers.relu(a5)
    a6 = layers.affine_forward(r5, p["f6_w"], p["f6_b"])
    r6 = layers.relu(a6)
    out = layers.affine_forward(r6, p["out_w"], p["out_b"])
    loss, d_out = layers.mse_loss(out, target)

    g = {}
    d_r6, g["out_w"], g["out_b"] = layers.affine_backward(r6, p["out_w"], d_out)
    d_a6 = layers.relu_backward(a6, d_r6)
    d_r5, g["f6_w"], g["f6_b"] = layers.affine_backward(r5, p["f6_w"], d_a6)
    d_a5 = layers.relu_backward(a5, d_r5)
    d_f, g["c5_w"], g["c5_b"] = layers.affine_backward(f, p["c5_w"], d_a5)
    d_s4 = d_f.reshape(s4.shape)
    d_r3 = layers.maxpool_valid_adjoint(d_s4, arg4, r3.shape, (2, 2), (2, 2), (0, 0))
    d_a3 = layers.relu_backward(a3, d_r3)
    d_s2, g["c3_w"], g["c3_b"] = layers.conv_backward(s2, p["c3_w"], d_a3, ONE2, (0, 0), ONE2)
    d_r1 = layers.maxpool_valid_adjoint(d_s2, arg2, r1.shape, (2, 2), (2, 2), (0, 0))
    d_a1 = layers.relu_backward(a1, d_r1)
    g["images"], g["c1_w"], g["c1_b"] = layers.conv_backward(images, p["c1_w"], d_a1, ONE2, (2, 2), ONE2)
    return loss, out, g


def _into_bufs(parts_out, part):
    """Place a previous layer's per-worker outputs into the bulk of the next
    layer's padded buffers (both use the balanced split of the same length)."""
    bufs = []
    for w, y in enumerate(parts_out):
        b = np.zeros(y.shape[:2] + part.buf_shape(w))
        b[(slice(None), slice(None)) + part.bulk_slices(w)] = y
        bufs.append(b)
    return bufs


def _bulk_of(bufs, part):
    return [b[(slice(None), slice(None)) + part.bulk_slices(w)].copy() for w, b in enumerate(bufs)]


def distributed_step(images, target, p, P=(2, 2), P_fo=2, P_fi=2):
    """The same step through the distributed layers of Sec. 4."""
    pc1 = geo.Partition.for_kernel((28, 28), P, (5, 5), ONE2, (2, 2), ONE2)
    pp2 = geo.Partition.for_kernel((28, 28), P, (2, 2), (2, 2), (0, 0), ONE2)
    pc3 = geo.Partition.for_kernel((14, 14), P, (5, 5), ONE2, (0, 0), ONE2)
    pp4 = geo.Partition.for_kernel((10, 10), P, (2, 2), (2, 2), (0, 0), ONE2)

    x1 = prim.scatter_bulk(np.asarray(images, dtype=np.float64), pc1)
    a1 = layers.dist_conv_forward(x1, p["c1_w"], p["c1_b"], pc1, ONE2, ONE2)
    r1 = [layers.relu(t) for t in a1]
    x2 = _into_bufs(r1, pp2)
    s2, arg2 = layers.dist_maxpool_forward(x2, pp2, (2, 2), (2, 2))
    x3 = _into_bufs(s2, pc3)
    a3 = layers.dist_conv_forward(x3, p["c3_w"], p["c3_b"], pc3, ONE2, ONE2)
    r3 = [layers.relu(t) for t in a3]
    x4 = _into_bufs(r3, pp4)
    s4, arg4 = layers.dist_maxpool_forward(x4, pp4, (2, 2), (2, 2))
    f = layers.repartition_spatial_to_features(s4, pp4, P_fi)

    def split_w(name):
        W, b = p[name + "_w"], p[name + "_b"]
        rows = layers.feature_blocks(W.shape[0], P_fo)
        cols = layers.feature_blocks(W.shape[1], P_fi)
        return [[W[r][:, c] for c in cols] for r in rows], [b[r] for r in rows], rows, cols

    W5, b5, rows5, cols5 = split_w("c5")
    W6, b6, rows6, cols6 = split_w("f6")
    Wo, bo, rowso, colso = split_w("out")
    a5 = layers.dist_affine_forward(f, W5, b5, P_fo, P_fi)
    r5 = [layers.relu(t) for t in a5]
    a6 = layers.dist_affine_forward(r5, W6, b6, P_fo, P_fi)
    r6 = [layers.relu(t) for t in a6]
    out = layers.dist_affine_forward(r6, Wo, bo, P_fo, P_fi)
    out_full = np.concatenate(out, axis=1)
    loss, d_out_full = layers.mse_loss(out_full, target)
    d_out = [d_out_full[:, r] for r in rowso]

    g = {}

    def join(dW, db):
        return np.block(dW), np.concatenate(db)

    d_r6, dW, db = layers.dist_affine_adjoint(r6, Wo, d_out, P_fo, P_fi)
    g["out_w"], g["out_b"] = join(dW, db)
    d_a6 = [layers.relu_backward(a, d) for a, d in zip(a6, d_r6)]
    d_r5, dW, db = layers.dist_affine_adjoint(r5, W6, d_a6, P_fo, P_fi)
    g["f6_w"], g["f6_b"] = join(dW, db)
    d_a5 = [layers.relu_backward(a, d) for a, d in zip(a5, d_r5)]
    d_f, dW, db = layers.dist_affine_adjoint(f, W5, d_a5, P_fo, P_fi)
    g["c5_w"], g["c5_b"] = join(dW, db)

    d_s4 = layers.repartition_features_to_spatial(d_f, pp4, 16)
    d_x4 = layers.dist_maxpool_adjoint(d_s4, arg4, pp4, [b.shape for b in x4], (2, 2), (2, 2))
    d_r3 = _bulk_of(d_x4, pp4)
    d_a3 = [layers.relu_backward(a, d) for a, d in zip(a3, d_r3)]
    d_x3, g["c3_w"], g["c3_b"] = layers.dist_conv_adjoint(x3, p["c3_w"], d_a3, pc3, ONE2, ONE2)
    d_s2 = _bulk_of(d_x3, pc3)
    d_x2 = layers.dist_maxpool_adjoint(d_s2, arg2, pp2, [b.shape for b in x2], (2, 2), (2, 2))
    d_r1 = _bulk_of(d_x2, pp2)
    d_a1 = [layers.relu_backward(a, d) for a, d in zip(a1, d_r1)]
    d_x1, g["c1_w"], g["c1_b"] = layers.dist_conv_adjoint(x1, p["c1_w"], d_a1, pc1, ONE2, ONE2)
    g["images"] = prim.gather_bulk(d_x1, pc1)
    return loss, out_full, g
