// Footprint projector pair on tilted modules of the modular geometry ("CT Projection Models and Geometries": a
// flexible cone-beam geometry with detectors at any position and orientation; the separable footprint itself is the
// one of "Separable footprint weights").  The paper gives no construction for a detector whose axes are not
// (horizontal, z); the one used here keeps the footprint separable on the module's own axes:
//   columns: trapezoid whose knots are the column coordinates of the central projections (from the source onto the
//            module's plane) of the voxel's four in-plane corners, taken at the height of the voxel's centre;
//   rows   : rectangle between the row coordinates of the central projections of the centres of the voxel's lower
//            and upper face;
//   amplitude: T |D| / max(|Dx|, |Dy|) with D = pixel - source.
// For an upright module these are the circular cone-beam expressions in the module's frame.
//
// General bodies, double precision throughout (every voxel has its own knots in every view, so none of the per-column
// sharing of the circular kernels applies): one voxel per call in the back projection, a few consecutive rows of one
// detector column per call in the forward projection (they share their candidate voxels' footprints).  Both directions
// evaluate the same functions (mf_footprint, mf_fu, mf_fv, mf_amp) on the same arguments, so the pair is matched up to
// summation order.
#pragma once

#include "sf_footprint.h"

// One entry per view, built in double on the host.
struct MfView {
    double S[3], C[3], eu[3], ev[3], n[3];   // source, detector centre, column axis, row axis, n = eu x ev
    double gap;                              // (C - S).n, signed distance of the module's plane from the source
    double su, sv;                           // (S - C).eu, (S - C).ev: the source's foot point in detector coordinates
    double ipu, ipv;                         // 1 / pixel pitch along the column / row axis, 1/mm
    double pad_u, pad_v;                     // mm: how far the column coordinate of a voxel's corner / the row coordinate
                                             // of a face centre can lie from those of the voxel's centre (upper bounds)
};

// Host: fills the derived members of V (S, C, eu, ev set) for the volume of g.  Returns false if the view has no
// footprints: part of the volume is not in front of the source, or a pixel's ray would run along z.
inline bool mf_prepare_view(const SfGeom &g, MfView &V)
{
    V.n[0] = V.eu[1] * V.ev[2] - V.eu[2] * V.ev[1];
    V.n[1] = V.eu[2] * V.ev[0] - V.eu[0] * V.ev[2];
    V.n[2] = V.eu[0] * V.ev[1] - V.eu[1] * V.ev[0];
    V.gap = 0.0; V.su = 0.0; V.sv = 0.0;
    V.ipu = 1.0 / g.pu_d; V.ipv = 1.0 / g.pvd;
    for (int q = 0; q < 3; ++q) {
        V.gap += (V.C[q] - V.S[q]) * V.n[q];
        V.su += (V.S[q] - V.C[q]) * V.eu[q];
        V.sv += (V.S[q] - V.C[q]) * V.ev[q];
    }
    if (!(V.gap > 0.0) && !(V.gap < 0.0)) return false;
    // over the volume's box: the smallest distance from the source along n and the largest tangents of the angle
    // between a point's ray and n (ratios of linear functions: extremes at the corners)
    const double lo[3] = {g.x0d - 0.5 * g.Td, g.y0d - 0.5 * g.Td, g.zlo0d};
    const double hi[3] = {lo[0] + g.nx * g.Td, lo[1] + g.ny * g.Td, lo[2] + g.nz * g.Tzd};
    double along_min = 1e300, tu = 0.0, tv = 0.0;
    for (int corner = 0; corner < 8; ++corner) {
        double along = 0.0, du = 0.0, dv = 0.0;
        for (int q = 0; q < 3; ++q) {
            const double d = ((corner >> q) & 1 ? hi[q] : lo[q]) - V.S[q];
            along += d * V.n[q]; du += d * V.eu[q]; dv += d * V.ev[q];
        }
        if (!(along * V.gap > 0.0)) return false;
        along = along < 0.0 ? -along : along;
        along_min = along < along_min ? along : along_min;
        const double a = (du < 0.0 ? -du : du) / along, b = (dv < 0.0 ? -dv : dv) / along;
        tu = a > tu ? a : tu;
        tv = b > tv ? b : tv;
    }
    // |grad u| = (|gap| / along) sqrt(1 + tan_u^2); a corner lies T / sqrt(2) from the centre, a face centre Tz / 2
    const double mag = (V.gap < 0.0 ? -V.gap : V.gap) / along_min;
    V.pad_u = 1.0001 * mag * sqrt(1.0 + tu * tu) * g.Td * 0.70710678118654757;
    V.pad_v = 1.0001 * mag * sqrt(1.0 + tv * tv) * g.Tzd * 0.5;
    if (V.n[2] > 1e-12 || V.n[2] < -1e-12) {       // where the vertical line through the source meets the plane
        const double lam = V.gap / V.n[2];
        const double u = V.su + lam * V.eu[2], v = V.sv + lam * V.ev[2];
        const double ulo = (-0.5 - g.col_offd) * g.pu_d, uhi = ((double)g.ncols - 0.5 - g.col_offd) * g.pu_d;
        const double vlo = g.v0d - 0.5 * g.pvd, vhi = g.v0d + ((double)g.nrows - 0.5) * g.pvd;
        if (u >= ulo && u <= uhi && v >= vlo && v <= vhi) return false;
    }
    return true;
}

// 1 / x to double precision without the division sequence: the float reciprocal and two Newton steps (relative error
// 1e-7 -> 1e-14 -> rounding).  x must be finite, non-zero and within float range, which distances and knot gaps in mm
// or pixels are.
SF_HD double mf_rcp(double x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    double r = (double)__builtin_amdgcn_rcpf((float)x);
    r = r * fma(-x, r, 2.0);
    return r * fma(-x, r, 2.0);
#else
    return 1.0 / x;
#endif
}

// sqrt(x), x > 0 within float range, the same way: the float reciprocal square root and two Newton steps.
SF_HD double mf_sqrt(double x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    double r = (double)__builtin_amdgcn_rsqf((float)x);
    r = r * fma(-0.5 * x, r * r, 1.5);
    r = r * fma(-0.5 * x, r * r, 1.5);
    return x * r;
#else
    return sqrt(x);
#endif
}

// Detector coordinates (mm from the detector centre) of the central projection of the point S + d.
SF_HD void mf_project_point(const MfView &V, double dx, double dy, double dz, double &u, double &v)
{
    const double lam = V.gap * mf_rcp(fma(dx, V.n[0], fma(dy, V.n[1], dz * V.n[2])));
    u = fma(lam, fma(dx, V.eu[0], fma(dy, V.eu[1], dz * V.eu[2])), V.su);
    v = fma(lam, fma(dx, V.ev[0], fma(dy, V.ev[1], dz * V.ev[2])), V.sv);
}

struct MfFootprint {
    double xi[4];        // sorted knots, column index coordinates (pixel c covers [c - 1/2, c + 1/2])
    double eta0, eta1;   // axial interval, row index coordinates (pixel r covers [r, r + 1))
};

SF_HD MfFootprint mf_footprint(const SfGeom &g, const MfView &V, int i, int j, int k)
{
    const double dx = fma((double)i, g.Td, g.x0d) - V.S[0], dy = fma((double)j, g.Td, g.y0d) - V.S[1];
    const double dz = fma((double)k + 0.5, g.Tzd, g.zlo0d) - V.S[2];
    const double h = 0.5 * g.Td, hz = 0.5 * g.Tzd, ipu = V.ipu, ipv = V.ipv;
    MfFootprint f;
    double u, v, va, vb;
    mf_project_point(V, dx - h, dy - h, dz, u, v); f.xi[0] = fma(u, ipu, g.col_offd);
    mf_project_point(V, dx + h, dy - h, dz, u, v); f.xi[1] = fma(u, ipu, g.col_offd);
    mf_project_point(V, dx - h, dy + h, dz, u, v); f.xi[2] = fma(u, ipu, g.col_offd);
    mf_project_point(V, dx + h, dy + h, dz, u, v); f.xi[3] = fma(u, ipu, g.col_offd);
    mf_project_point(V, dx, dy, dz - hz, u, va);
    mf_project_point(V, dx, dy, dz + hz, u, vb);
#define MF_ORDER(a, b) { const double lo_ = fmin(f.xi[a], f.xi[b]), hi_ = fmax(f.xi[a], f.xi[b]); f.xi[a] = lo_; f.xi[b] = hi_; }
    MF_ORDER(0, 1) MF_ORDER(2, 3) MF_ORDER(0, 2) MF_ORDER(1, 3) MF_ORDER(1, 2)
#undef MF_ORDER
    f.eta0 = (fmin(va, vb) - g.v0d) * ipv + 0.5;
    f.eta1 = (fmax(va, vb) - g.v0d) * ipv + 0.5;
    return f;
}

// Integral of the unit-height trapezoid with knots xi from -infinity to x.
SF_HD double mf_trapezoid_integral(const double xi[4], double x)
{
    const double total = 0.5 * ((xi[3] - xi[0]) + (xi[2] - xi[1]));
    if (x <= xi[0]) return 0.0;
    if (x < xi[1]) return (x - xi[0]) * (x - xi[0]) * (0.5 * mf_rcp(xi[1] - xi[0]));
    if (x <= xi[2]) return fma(0.5, xi[1] - xi[0], x - xi[1]);
    if (x < xi[3]) return total - (xi[3] - x) * (xi[3] - x) * (0.5 * mf_rcp(xi[3] - xi[2]));
    return total;
}

SF_HD double mf_fu(const MfFootprint &f, int c)
{
    return mf_trapezoid_integral(f.xi, (double)c + 0.5) - mf_trapezoid_integral(f.xi, (double)c - 0.5);
}

SF_HD double mf_fv(const MfFootprint &f, int r)
{
    const double w = fmin((double)r + 1.0, f.eta1) - fmax((double)r, f.eta0);
    return w > 0.0 ? w : 0.0;
}

SF_HD double mf_amp(const SfGeom &g, const MfView &V, int r, int c)
{
    const double u = ((double)c - g.col_offd) * g.pu_d, v = fma((double)r, g.pvd, g.v0d);
    const double dx = fma(u, V.eu[0], fma(v, V.ev[0], V.C[0] - V.S[0]));
    const double dy = fma(u, V.eu[1], fma(v, V.ev[1], V.C[1] - V.S[1]));
    const double dz = fma(u, V.eu[2], fma(v, V.ev[2], V.C[2] - V.S[2]));
    return g.Td * mf_sqrt(fma(dx, dx, fma(dy, dy, dz * dz))) * mf_rcp(fmax(fabs(dx), fabs(dy)));
}

// Back projection of one voxel: sum over views and over the pixels its footprint touches.
SF_HD float mf_backproject_voxel(const SfGeom &g, const MfView *__restrict__ views, const float *__restrict__ sino, int i,
                                 int j, int k)
{
    double acc = 0.0;
    for (int a = 0; a < g.nviews; ++a) {
        const MfView &V = views[a];
        const MfFootprint f = mf_footprint(g, V, i, j, k);
        // pixel c touches [xi0, xi3] if c + 1/2 > xi0 and c - 1/2 < xi3; pixel r touches [eta0, eta1] if r + 1 > eta0, r < eta1
        const double fc0 = floor(f.xi[0] + 0.5), fc1 = ceil(f.xi[3] - 0.5), fr0 = floor(f.eta0), fr1 = floor(f.eta1);
        if (fc1 < 0.0 || fr1 < 0.0 || fc0 > (double)(g.ncols - 1) || fr0 > (double)(g.nrows - 1)) continue;
        const int c0 = fc0 < 0.0 ? 0 : (int)fc0, c1 = fc1 > (double)(g.ncols - 1) ? g.ncols - 1 : (int)fc1;
        const int r0 = fr0 < 0.0 ? 0 : (int)fr0, r1 = fr1 > (double)(g.nrows - 1) ? g.nrows - 1 : (int)fr1;
        const float *__restrict__ ya = sino + (size_t)a * g.nrows * g.ncols;
        for (int c = c0; c <= c1; ++c) {
            const double fu = mf_fu(f, c);
            if (!(fu > 0.0)) continue;
            double s = 0.0;
            for (int r = r0; r <= r1; ++r) {
                const double fv = mf_fv(f, r);
                if (fv > 0.0) s = fma(fv * mf_amp(g, V, r, c), (double)ya[(size_t)r * g.ncols + c], s);
            }
            acc = fma(fu, s, acc);
        }
    }
    return (float)acc;
}

// Forward projection of RC consecutive rows of one detector column (one thread's share).  The voxels whose footprints can
// touch those pixels have centres that project into the pixels' rectangle widened by (pad_u, pad_v): a pyramid from the
// source.  The volume is walked layer by layer along the axis the central ray advances fastest on; in each layer the
// pyramid's section (a quadrilateral) bounds the candidate centres, and every candidate's exact footprint decides.  A
// candidate's footprint is formed once and serves all RC rows.
template <int m, int RC>
SF_HD void mf_project_rows_along(const SfGeom &g, const MfView &V, const float *__restrict__ vol, int r0, int c, double (&acc)[RC])
{
    const double uc = ((double)c - g.col_offd) * g.pu_d, vc = fma((double)r0 + 0.5 * (RC - 1), g.pvd, g.v0d);
    const double du = 0.5 * g.pu_d + V.pad_u, dv = 0.5 * RC * g.pvd + V.pad_v;
    double D[3], Dq[4][3];
    for (int q = 0; q < 3; ++q) {
        const double base = V.C[q] - V.S[q];
        D[q] = fma(uc, V.eu[q], fma(vc, V.ev[q], base));
        for (int e = 0; e < 4; ++e)
            Dq[e][q] = fma(uc + ((e & 1) ? du : -du), V.eu[q], fma(vc + ((e & 2) ? dv : -dv), V.ev[q], base));
    }
    constexpr int a1 = m == 0 ? 1 : 0, a2 = m == 2 ? 1 : 2;      // the other two axes, a1 < a2
    const int n[3] = {g.nx, g.ny, g.nz};
    const double pitch[3] = {g.Td, g.Td, g.Tzd}, ipitch[3] = {1.0 / g.Td, 1.0 / g.Td, 1.0 / g.Tzd};
    const double first[3] = {g.x0d, g.y0d, g.zlo0d + 0.5 * g.Tzd};      // centre of voxel 0 along each axis
    // the widened corners' rays must cross the layers the same way as the central ray; otherwise (a very oblique
    // module) every voxel of a layer is a candidate
    bool narrow = true;
    double inv[4];
    for (int e = 0; e < 4; ++e) {
        narrow = narrow && Dq[e][m] * D[m] > 0.0625 * D[m] * D[m];
        inv[e] = 1.0 / Dq[e][m];
    }
    for (int layer = 0; layer < n[m]; ++layer) {
        int lo1 = 0, hi1 = n[a1] - 1, lo2 = 0, hi2 = n[a2] - 1;
        if (narrow) {
            const double s = fma((double)layer, pitch[m], first[m]) - V.S[m];
            double p1min = 1e300, p1max = -1e300, p2min = 1e300, p2max = -1e300;
            bool front = true;
            for (int e = 0; e < 4; ++e) {
                const double lam = s * inv[e];
                front = front && lam > 0.0;
                const double p1 = fma(lam, Dq[e][a1], V.S[a1]), p2 = fma(lam, Dq[e][a2], V.S[a2]);
                p1min = fmin(p1min, p1); p1max = fmax(p1max, p1);
                p2min = fmin(p2min, p2); p2max = fmax(p2max, p2);
            }
            if (!front) continue;                  // the layer lies behind the source as seen along these rays
            const double f1lo = ceil((p1min - first[a1]) * ipitch[a1] - 1e-6), f1hi = floor((p1max - first[a1]) * ipitch[a1] + 1e-6);
            const double f2lo = ceil((p2min - first[a2]) * ipitch[a2] - 1e-6), f2hi = floor((p2max - first[a2]) * ipitch[a2] + 1e-6);
            if (f1hi < 0.0 || f2hi < 0.0 || f1lo > (double)hi1 || f2lo > (double)hi2) continue;
            lo1 = f1lo < 0.0 ? 0 : (int)f1lo; hi1 = f1hi > (double)hi1 ? hi1 : (int)f1hi;
            lo2 = f2lo < 0.0 ? 0 : (int)f2lo; hi2 = f2hi > (double)hi2 ? hi2 : (int)f2hi;
        }
        for (int q2 = lo2; q2 <= hi2; ++q2)
            for (int q1 = lo1; q1 <= hi1; ++q1) {
                const int idx[3] = {m == 0 ? layer : q1, m == 1 ? layer : (m == 0 ? q1 : q2), m == 2 ? layer : q2};
                const MfFootprint f = mf_footprint(g, V, idx[0], idx[1], idx[2]);
                if (!(f.eta1 > (double)r0 && f.eta0 < (double)(r0 + RC))) continue;
                const double fu = mf_fu(f, c);
                if (!(fu > 0.0)) continue;
                const double fx = fu * (double)vol[((size_t)idx[2] * g.ny + idx[1]) * g.nx + idx[0]];
#pragma unroll
                for (int rr = 0; rr < RC; ++rr) acc[rr] = fma(mf_fv(f, r0 + rr), fx, acc[rr]);
            }
    }
}

// out[rr] = line integral of pixel (r0 + rr, c), rr < RC (rows past the detector's last come out as whatever the model
// gives them; the caller does not store them).
template <int RC>
SF_HD void mf_project_rows(const SfGeom &g, const MfView &V, const float *__restrict__ vol, int r0, int c, float (&out)[RC])
{
    const double uc = ((double)c - g.col_offd) * g.pu_d, vc = fma((double)r0 + 0.5 * (RC - 1), g.pvd, g.v0d);
    double D[3], acc[RC];
    for (int q = 0; q < 3; ++q) D[q] = fma(uc, V.eu[q], fma(vc, V.ev[q], V.C[q] - V.S[q]));
#pragma unroll
    for (int rr = 0; rr < RC; ++rr) acc[rr] = 0.0;
    if (fabs(D[0]) >= fabs(D[1]) && fabs(D[0]) >= fabs(D[2])) mf_project_rows_along<0, RC>(g, V, vol, r0, c, acc);
    else if (fabs(D[1]) >= fabs(D[2])) mf_project_rows_along<1, RC>(g, V, vol, r0, c, acc);
    else mf_project_rows_along<2, RC>(g, V, vol, r0, c, acc);
#pragma unroll
    for (int rr = 0; rr < RC; ++rr) out[rr] = (float)(acc[rr] * mf_amp(g, V, r0 + rr, c));
}
