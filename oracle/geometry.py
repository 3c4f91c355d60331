"""Partition geometry for sliding-kernel layers (Sec. 3 "Halo exchange",
App. B.1 "Irregularly structured halo regions").

The paper says what fixes a worker's halo thicknesses -- the first and last
global index of its (load-balanced) output sub-tensor and the kernel's size,
stride, dilation and padding -- but prints no formula.  The reading used here,
per dimension:

  output length   m = floor((n + 2p - dil*(k-1) - 1) / s) + 1
  balanced split  a length L over P workers gives worker r
                  floor(L/P) + (1 if r < L mod P else 0) cells, contiguous,
                  ascending; applied to the input (n) and to the output (m)
                  independently (App. B.1: output drives the load balance and
                  the input "is also balanced").
  needed input    outputs [j0, j1] read inputs [j0*s - p, j1*s - p + dil*(k-1)]
  pad             the part of that range outside [0, n-1]      (zero padding)
  halo            the in-domain part outside the owned range   (neighbour data)
  extra           owned cells outside the needed range         ("extra input"
                  that must be removed before the local kernel, App. B.1)

This reading reproduces all four worked 1-D examples of App. B.1 (see
tests/golden/halo_examples.txt).  The third example's text gives n = 11 but
its figure draws inputs 0..9 and its prose only fits n = 10; n = 10 is used.

All quantities are Python ints.  Test infrastructure only.
"""
from itertools import product


class EmptyPartition(ValueError):
    """Some worker would own no input cell or no output cell."""


class HaloTooWide(ValueError):
    """A halo would need data from beyond the directly adjacent worker
    (Sec. 3 assumes adjacent neighbours only)."""


def output_length(n, k, s, p, dil):
    return (n + 2 * p - dil * (k - 1) - 1) // s + 1


def balanced_split(length, parts):
    """List of (start, size) per worker for the balanced rule above."""
    out, start = [], 0
    for r in range(parts):
        size = length // parts + (1 if r < length % parts else 0)
        out.append((start, size))
        start += size
    return out


def dim_geometry(n, k, s, p, dil, parts):
    """Per-worker geometry along one dimension.  Returns a list of dicts with

      in_start, in_size    owned (bulk) input range [b0, b0+size)
      out_start, out_size  owned output range
      pad, halo, extra     (left, right) widths
      buf                  buffer extent = padL + haloL + bulk + haloR + padR
      bulk_off             buffer coordinate of the first bulk cell
      origin               buffer coordinate of the first tap of the first
                           owned output (= padL+haloL+extraL - what was added
                           on the left, i.e. simply extraL counted from the
                           start of the needed range)
    """
    m = output_length(n, k, s, p, dil)
    ins = balanced_split(n, parts)
    outs = balanced_split(m, parts) if m > 0 else [(0, 0)] * parts
    workers = []
    for r in range(parts):
        b0, nsz = ins[r]
        j0, msz = outs[r]
        if nsz <= 0 or msz <= 0:
            raise EmptyPartition(f"worker {r}: in {nsz} out {msz}")
        b1, j1 = b0 + nsz - 1, j0 + msz - 1
        i0 = j0 * s - p
        i1 = j1 * s - p + dil * (k - 1)
        pad_l, pad_r = max(0, -i0), max(0, i1 - (n - 1))
        c0, c1 = max(i0, 0), min(i1, n - 1)
        halo_l, halo_r = max(0, b0 - c0), max(0, c1 - b1)
        extra_l, extra_r = max(0, c0 - b0), max(0, b1 - c1)
        workers.append(dict(
            in_start=b0, in_size=nsz, out_start=j0, out_size=msz,
            pad=(pad_l, pad_r), halo=(halo_l, halo_r), extra=(extra_l, extra_r),
            buf=pad_l + halo_l + nsz + halo_r + pad_r,
            bulk_off=pad_l + halo_l,
            # buffer coordinate 0 is global index b0 - halo_l - pad_l; the first
            # tap of output j0 sits at global i0.
            origin=i0 - (b0 - halo_l - pad_l)))
    for r in range(parts):
        hl, hr = workers[r]["halo"]
        if hl and (r == 0 or hl > workers[r - 1]["in_size"]):
            raise HaloTooWide(f"worker {r} left halo {hl}")
        if hr and (r == parts - 1 or hr > workers[r + 1]["in_size"]):
            raise HaloTooWide(f"worker {r} right halo {hr}")
    return workers


def explicit_dim_geometry(bulk_sizes, halo_lr):
    """One dimension with user-given bulk sizes and (left, right) halo widths
    per worker and no padding -- the form of the rank-2 example of App. B.2."""
    parts = len(bulk_sizes)
    workers, start = [], 0
    for r in range(parts):
        hl, hr = halo_lr[r]
        if bulk_sizes[r] <= 0:
            raise EmptyPartition(f"worker {r}")
        if hl and (r == 0 or hl > bulk_sizes[r - 1]):
            raise HaloTooWide(f"worker {r} left halo {hl}")
        if hr and (r == parts - 1 or hr > bulk_sizes[r + 1]):
            raise HaloTooWide(f"worker {r} right halo {hr}")
        workers.append(dict(
            in_start=start, in_size=bulk_sizes[r], out_start=start,
            out_size=bulk_sizes[r], pad=(0, 0), halo=(hl, hr), extra=(0, 0),
            buf=hl + bulk_sizes[r] + hr, bulk_off=hl, origin=0))
        start += bulk_sizes[r]
    return workers


class Partition:
    """Tensor-product geometry of a rank-D feature space split over the
    partition vector P (Sec. 4: a d-length vector of workers per dimension).
    Workers are numbered row-major over P (App. C table and App. B.2 text fix
    this: in a 2x2 grid worker 0's vertical neighbour is 2, horizontal is 1)."""

    def __init__(self, dims):
        self.dims = dims                      # list over D of per-worker lists
        self.D = len(dims)
        self.P = [len(d) for d in dims]
        self.n_workers = 1
        for p in self.P:
            self.n_workers *= p

    @classmethod
    def for_kernel(cls, in_shape, P, ksize, stride, padding, dilation):
        return cls([dim_geometry(in_shape[d], ksize[d], stride[d], padding[d],
                                 dilation[d], P[d]) for d in range(len(P))])

    @classmethod
    def explicit(cls, bulk_sizes, halo_lr):
        return cls([explicit_dim_geometry(bulk_sizes[d], halo_lr[d])
                    for d in range(len(bulk_sizes))])

    def coords(self, w):
        """Row-major worker id -> index vector."""
        out = []
        for p in reversed(self.P):
            out.append(w % p)
            w //= p
        return tuple(reversed(out))

    def worker_id(self, coords):
        w = 0
        for c, p in zip(coords, self.P):
            w = w * p + c
        return w

    def workers(self):
        return [self.coords(w) for w in range(self.n_workers)]

    def g(self, w, d):
        """Geometry dict of worker w along dimension d."""
        return self.dims[d][self.coords(w)[d]]

    def buf_shape(self, w):
        return tuple(self.g(w, d)["buf"] for d in range(self.D))

    def out_shape(self, w):
        return tuple(self.g(w, d)["out_size"] for d in range(self.D))

    def bulk_slices(self, w):
        """Slices (over the feature dims of w's buffer) selecting the bulk."""
        return tuple(slice(self.g(w, d)["bulk_off"],
                           self.g(w, d)["bulk_off"] + self.g(w, d)["in_size"])
                     for d in range(self.D))

    def global_in_slices(self, w):
        return tuple(slice(self.g(w, d)["in_start"],
                           self.g(w, d)["in_start"] + self.g(w, d)["in_size"])
                     for d in range(self.D))

    def global_out_slices(self, w):
        return tuple(slice(self.g(w, d)["out_start"],
                           self.g(w, d)["out_start"] + self.g(w, d)["out_size"])
                     for d in range(self.D))

    def global_in_shape(self):
        return tuple(self.dims[d][-1]["in_start"] + self.dims[d][-1]["in_size"]
                     for d in range(self.D))

    def global_out_shape(self):
        return tuple(self.dims[d][-1]["out_start"] + self.dims[d][-1]["out_size"]
                     for d in range(self.D))

    def neighbour(self, w, d, side):
        """Worker adjacent to w along d on side 0 (left) / 1 (right), or None."""
        c = list(self.coords(w))
        c[d] += -1 if side == 0 else 1
        if c[d] < 0 or c[d] >= self.P[d]:
            return None
        return self.worker_id(c)


def all_index_vectors(shape):
    return product(*[range(s) for s in shape])
