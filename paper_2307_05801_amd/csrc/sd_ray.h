// Siddon projector pair: exact length of each pixel-centre ray inside each voxel (Method section, "CT Projection
// Models and Geometries": the Siddon model, line integrals along thin rays, matched transpose).
//
// Formulation used by every Siddon kernel of this library (forward and back, general and fast), so that the pair is
// matched: a ray is marched along the in-plane axis it advances fastest on (the "major" axis), one slab of voxels at
// a time.  In index coordinates (voxel i covers [i, i+1) on every axis) the ray of detector column c in one view is
//     minor(X) = m X + b,   |m| <= 1                      X: major coordinate
//     Z(X)     = zk0 + v_r h(X),   h(X) = h0 + X dh        v_r: the row's v in mm (cone); h = 1/Tz, dh = 0 (parallel)
// and one unit of X is L = sqrt(lxy^2 + (vscale v_r)^2) mm of ray.  Inside slab n (X in [n, n+1], tau = X - n) the
// ray lies in in-plane cell qa for tau < f and in cell qb afterwards (qa == qb, f = 1 when it does not cross a
// minor-axis face), and its Z moves linearly from Z(n) to Z(n+1).  The weight of a voxel is L times the measure of
// the tau-set where the ray is in its in-plane cell and floor(Z) equals its k.  Faces belong to the cell above them
// (floor), which is the half-open box rule.
//
// The per-(view, column) constants m, b, h0, dh, ... are derived once, in double, on the host (SdRayCol table); the
// kernels only evaluate them.  Absolute positions (minor(n), Z(n)) are formed in double, fractions in float.
#pragma once

#include "sf_footprint.h"

struct SdRayCol {
    double m, b;        // minor index coordinate = m * major index coordinate + b
    double h0, dh;      // h(X) = h0 + X dh
    float inv_m;        // 1/m, magnitude capped at 1e30 (m == 0: 1e30)
    float lxy;          // mm of in-plane path per unit of X: T |d_xy| / |d_major|
    float vscale;       // cone: T / |d_major| (so that the axial rise per unit X is vscale * v_r mm); otherwise 0
    int32_t xmajor;     // 1: the major axis is x
};

// In-plane part of slab n.
struct SdSplit {
    int qa, qb;         // minor index of the cell the ray is in at the slab's entry / exit face
    float f;            // tau at which it changes from qa to qb (1 when qa == qb)
};

SF_HD SdSplit sd_slab_split(const SdRayCol &R, int n)
{
    SdSplit s;
    const double yin = fma(R.m, (double)n, R.b);
    const double yout = yin + R.m;
#if defined(__HIP_DEVICE_COMPILE__)
    // (the device's conversion saturates: rays that miss the volume by far get an index far outside it either way)
    const double fa = floor(yin), fb = floor(yout);
#else
    // rays that miss the volume by far: keep the conversion to int defined
    const double fa = fmin(fmax(floor(yin), -1.0e9), 1.0e9), fb = fmin(fmax(floor(yout), -1.0e9), 1.0e9);
#endif
    s.qa = (int)fa;
    s.qb = (int)fb;
    if (s.qa == s.qb) {
        s.f = 1.0f;
    } else {
        const float t = (float)(fmax(fa, fb) - yin) * R.inv_m;      // distance to the face between them over the slope
        s.f = fminf(fmaxf(t, 0.0f), 1.0f);
    }
    return s;
}

SF_HD double sd_row_v(const SfGeom &g, int r) { return fma((double)r, g.pvd, g.v0d); }

SF_HD float sd_ray_length(const SdRayCol &R, double vr)
{
    const float a = R.vscale * (float)vr;
    return sf_sqrt(fmaf(a, a, R.lxy * R.lxy));
}

// Measure of { t in [0,1] : floor(za + t (zb - za)) == k }: share of a piece of ray whose Z runs linearly from za to zb
// that lies in axial cell k.
SF_HD float sd_axial_share(double za, double zb, int k)
{
    const double lo = fmin(za, zb), hi = fmax(za, zb);
    if (!(hi > lo)) return floor(lo) == (double)k ? 1.0f : 0.0f;
    const double a = fmax(lo, (double)k), b = fmin(hi, (double)k + 1.0);
    return b > a ? (float)((b - a) / (hi - lo)) : 0.0f;
}

// ---- general bodies: any geometry the library validates, one output per call, global memory only ---------------

// Forward: line integral of ray (view table entry R, row r) through vol [nz][ny][nx].
SF_HD float sd_project_ray(const SfGeom &g, const SdRayCol &R, const float *__restrict__ vol, int r)
{
    const int n_major = R.xmajor ? g.nx : g.ny, n_minor = R.xmajor ? g.ny : g.nx;
    const double vr = sd_row_v(g, r);
    const double mz = vr * R.dh;
    const size_t kstride = (size_t)g.nx * g.ny;
    float sum = 0.0f;
    for (int n = 0; n < n_major; ++n) {
        const SdSplit s = sd_slab_split(R, n);
        const double zin = fma(vr, fma((double)n, R.dh, R.h0), g.zk0d);
        for (int piece = 0; piece < 2; ++piece) {
            const int q = piece ? s.qb : s.qa;
            const float t0 = piece ? s.f : 0.0f, t1 = piece ? 1.0f : s.f;
            if (piece && s.qa == s.qb) break;
            if (q < 0 || q >= n_minor || !(t1 > t0)) continue;
            const double za = fma((double)t0, mz, zin), zb = fma((double)t1, mz, zin);
            const double klo = floor(fmin(za, zb)), khi = floor(fmax(za, zb));
            if (khi < 0.0 || klo > (double)(g.nz - 1)) continue;
            const int k0 = klo < 0.0 ? 0 : (int)klo, k1 = khi > (double)(g.nz - 1) ? g.nz - 1 : (int)khi;
            const int i = R.xmajor ? n : q, j = R.xmajor ? q : n;
            const float *__restrict__ col = vol + ((size_t)j * g.nx + i);
            for (int k = k0; k <= k1; ++k) sum = fmaf((t1 - t0) * sd_axial_share(za, zb, k), col[(size_t)k * kstride], sum);
        }
    }
    return sum * sd_ray_length(R, vr);
}

// Back: sum over all rays of weight * sino for voxel (i, j, k).  rays: SdRayCol table [nviews][ncols].
SF_HD float sd_backproject_voxel(const SfGeom &g, const SfView *__restrict__ views, const SdRayCol *__restrict__ rays,
                                 const float *__restrict__ sino, int i, int j, int k)
{
    float acc = 0.0f;
    for (int a = 0; a < g.nviews; ++a) {
        // detector columns whose centre can lie inside the projection of the voxel's in-plane square
        const SfColumn f = sf_column(g, views[a], i, j);
        int c0 = (int)ceil(f.xi + (double)f.o0 - 1e-3), c1 = (int)floor(f.xi + (double)f.o3 + 1e-3);
        c0 = c0 < 0 ? 0 : c0;
        c1 = c1 > g.ncols - 1 ? g.ncols - 1 : c1;
        const float *__restrict__ ya = sino + (size_t)a * g.nrows * g.ncols;
        for (int c = c0; c <= c1; ++c) {
            const SdRayCol R = rays[(size_t)a * g.ncols + c];
            const int n = R.xmajor ? i : j, q = R.xmajor ? j : i;
            const SdSplit s = sd_slab_split(R, n);
            float t0, t1;
            if (q == s.qa) { t0 = 0.0f; t1 = s.f; }
            else if (q == s.qb) { t0 = s.f; t1 = 1.0f; }
            else continue;
            if (!(t1 > t0)) continue;
            if (g.type == SF_FAN) {
                acc = fmaf((t1 - t0) * R.lxy, ya[c], acc);
                continue;
            }
            const double ha = fma((double)n + (double)t0, R.dh, R.h0), hb = fma((double)n + (double)t1, R.dh, R.h0);
            // rows whose Z can reach [k, k+1) somewhere on the piece: v between (k - zk0)/h and (k + 1 - zk0)/h (h > 0)
            const double e0 = (double)k - g.zk0d, e1 = e0 + 1.0;
            const double vlo = fmin(e0 / ha, e0 / hb), vhi = fmax(e1 / ha, e1 / hb);
            double rlo = ceil((vlo - g.v0d) / g.pvd - 1e-6), rhi = floor((vhi - g.v0d) / g.pvd + 1e-6);
            if (rhi < 0.0 || rlo > (double)(g.nrows - 1)) continue;
            const int r0 = rlo < 0.0 ? 0 : (int)rlo, r1 = rhi > (double)(g.nrows - 1) ? g.nrows - 1 : (int)rhi;
            for (int r = r0; r <= r1; ++r) {
                const double vr = sd_row_v(g, r);
                const float share = sd_axial_share(fma(vr, ha, g.zk0d), fma(vr, hb, g.zk0d), k);
                if (share > 0.0f) acc = fmaf((t1 - t0) * share * sd_ray_length(R, vr), ya[(size_t)r * g.ncols + c], acc);
            }
        }
    }
    return acc;
}
