"""Independent textbook geometry used to pin the oracle: none of it is the SF weight model.

* analytic chord of a ray through an ellipsoid (closed form of a quadratic),
* chord of a ray through an axis-aligned box (slab method),
* exact area of a convex polygon clipped by a strip (Sutherland-Hodgman),
* world coordinates of rays for the three geometries, written from the coordinate
  conventions stated in oracle/sf_oracle.h.
"""
from __future__ import annotations

import numpy as np


def ray_endpoints(cfg, view, u, v):
    """(point p, unit direction d) of the ray that hits detector coordinates (u, v) mm in `view`."""
    if cfg.geom == 4:       # modular: source S, detector centre C, column axis, row axis of this view
        pose = np.asarray(cfg.poses[view], dtype=np.float64)
        S, C_, eu, ev = pose[0:3], pose[3:6], pose[6:9], pose[9:12]
        uu = np.asarray(u, dtype=np.float64)[..., None]
        vv = np.asarray(v, dtype=np.float64)[..., None]
        d = C_ + uu * eu + vv * ev - S
        d = d / np.linalg.norm(d, axis=-1, keepdims=True)
        return np.broadcast_to(S, d.shape), d
    phi = cfg.angles()[view]
    es = np.array([np.cos(phi), np.sin(phi), 0.0])
    eu = np.array([-np.sin(phi), np.cos(phi), 0.0])
    ev = np.array([0.0, 0.0, 1.0])
    u = np.asarray(u, dtype=np.float64)[..., None]
    v = np.asarray(v, dtype=np.float64)[..., None]
    if cfg.geom == 0:
        p = u * eu + v * ev
        d = np.broadcast_to(-es, p.shape)
        return p, d
    src = cfg.sod * es
    if cfg.geom == 1:
        v = 0.0 * v
    if cfg.geom == 3:       # cylindrical detector of radius sdd around the source axis, u is arc length
        gam = u / cfg.sdd
        pix = src + cfg.sdd * (-np.cos(gam) * es + np.sin(gam) * eu) + v * ev
    else:
        pix = (cfg.sod - cfg.sdd) * es + u * eu + v * ev
    d = pix - src
    d = d / np.linalg.norm(d, axis=-1, keepdims=True)
    return np.broadcast_to(src, d.shape), d


def pixel_centres(cfg):
    u = (np.arange(cfg.ncols) - (cfg.ncols - 1) / 2.0 + cfg.shift_u) * cfg.pixel_u
    v = (np.arange(cfg.nrows) - (cfg.nrows - 1) / 2.0 + cfg.shift_v) * cfg.pixel_v
    return u, v


def ellipsoid_chord(p, d, centre, quadric):
    """Length of {p + s d} inside (X-c)^T Q (X-c) <= 1, |d| = 1; arrays broadcast over leading dims."""
    q = np.asarray(quadric)
    o = p - np.asarray(centre)
    a = np.einsum("...i,ij,...j->...", d, q, d)
    b = np.einsum("...i,ij,...j->...", d, q, o)
    c = np.einsum("...i,ij,...j->...", o, q, o) - 1.0
    disc = b * b - a * c
    return np.where(disc > 0.0, 2.0 * np.sqrt(np.maximum(disc, 0.0)) / a, 0.0)


def analytic_sinogram(cfg, ellipsoids):
    """Line integrals through a sum of uniform ellipsoids along the rays of every pixel CENTRE."""
    u, v = pixel_centres(cfg)
    uu, vv = np.meshgrid(u, v)          # [nrows][ncols]
    out = np.zeros(cfg.sino_shape)
    for a in range(cfg.nviews):
        p, d = ray_endpoints(cfg, a, uu, vv)
        for e in ellipsoids:
            out[a] += e.rho * ellipsoid_chord(p, d, e.center, e.quadric())
    return out


def box_chord(p, d, lo, hi):
    """Length of the ray {p + s d} (|d| = 1) inside the box [lo, hi] (slab method); broadcasts."""
    lo = np.asarray(lo, dtype=np.float64)
    hi = np.asarray(hi, dtype=np.float64)
    with np.errstate(divide="ignore", invalid="ignore"):
        t1 = (lo - p) / d
        t2 = (hi - p) / d
    tmin = np.minimum(t1, t2)
    tmax = np.maximum(t1, t2)
    # a ray parallel to a slab: inside -> (-inf, inf), outside -> empty
    par = d == 0.0
    inside = (p >= lo) & (p <= hi)
    tmin = np.where(par, np.where(inside, -np.inf, np.inf), tmin)
    tmax = np.where(par, np.where(inside, np.inf, -np.inf), tmax)
    enter = tmin.max(axis=-1)
    leave = tmax.min(axis=-1)
    return np.maximum(0.0, leave - enter)


def clip_polygon_halfplane(poly, n, off):
    """Sutherland-Hodgman: keep the part of convex polygon `poly` (list of 2-vectors) with n.x <= off."""
    out = []
    m = len(poly)
    for q in range(m):
        a, b = poly[q], poly[(q + 1) % m]
        da, db = np.dot(n, a) - off, np.dot(n, b) - off
        if da <= 0:
            out.append(a)
        if (da < 0 < db) or (db < 0 < da):
            s = da / (da - db)
            out.append(a + s * (b - a))
    return out


def polygon_area(poly):
    if len(poly) < 3:
        return 0.0
    p = np.asarray(poly)
    x, y = p[:, 0], p[:, 1]
    return 0.5 * abs(np.dot(x, np.roll(y, -1)) - np.dot(y, np.roll(x, -1)))


def strip_square_area(centre_xy, side, phi, u_lo, u_hi):
    """Exact area of {square of `side` centred at centre_xy} with u_lo <= t <= u_hi, t = -x sin + y cos."""
    cx, cy = centre_xy
    h = side / 2.0
    poly = [np.array([cx - h, cy - h]), np.array([cx + h, cy - h]),
            np.array([cx + h, cy + h]), np.array([cx - h, cy + h])]
    eu = np.array([-np.sin(phi), np.cos(phi)])
    poly = clip_polygon_halfplane(poly, eu, u_hi)
    poly = clip_polygon_halfplane(poly, -eu, -u_lo)
    return polygon_area(poly)
