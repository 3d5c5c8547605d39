// Separable-footprint weight factors, shared by the forward (ray-driven) and the back (voxel-driven)
// kernels so that the pair is matched: both obtain F_u and the amplitude from the same functions of
// (view, voxel column, pixel), and F_v from the same axial map.
//
// Weight of voxel (i,j,k) for ray (view,r,c):  w = amp(view,r,c) * F_u(view,c;i,j) * F_v(view,r;i,j,k)
//   F_u: area under a unit-height trapezoid over the pixel's u-interval, divided by the pixel width.  The
//        trapezoid's knots are the detector coordinates of the voxel's four in-plane corners.
//   F_v: overlap of the pixel's v-interval with the voxel's axial extent magnified at the voxel centre,
//        divided by the pixel height (fan-beam: 1).
//   amp: in-plane voxel size times |D| / max(|D_x|,|D_y|) for the ray direction D.
// (Method section, "CT Projection Models and Geometries": separable-footprint model, exact transpose,
// millimetre units.)
#pragma once

#include "sf_types.h"

#if defined(__HIPCC__) || defined(__HIP__)
#define SF_HD __host__ __device__ __forceinline__
#else
#define SF_HD inline
#endif

#include <math.h>

SF_HD float sf_rcp_fast(float x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_rcpf(x);
#else
    return 1.0f / x;
#endif
}

SF_HD float sf_rcp(float x)
{
    float r = sf_rcp_fast(x);
    return fmaf(r, fmaf(-x, r, 1.0f), r);   // one Newton step
}

// double reciprocal from the float estimate: one Newton step squares the 1e-7 error
SF_HD double sf_rcp_d(double x)
{
    double r = (double)sf_rcp_fast((float)x);
    r = fma(r, fma(-x, r, 1.0), r);
    return fma(r, fma(-x, r, 1.0), r);
}

SF_HD float sf_sqrt(float x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_sqrtf(x);
#else
    return sqrtf(x);
#endif
}

SF_HD float sf_clamp(float x, float lo, float hi)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_fmed3f(x, lo, hi);
#else
    return fminf(fmaxf(x, lo), hi);
#endif
}

// float -> int for window bounds: clamped first, so that an infinite or absurd bound (a ragged edge tile whose padding
// voxels reach past the source) converts to a defined value; the host then sees an oversized window and picks
// another kernel.  NaN becomes the lower bound.
SF_HD int sf_f2i(float x) { return (int)fminf(fmaxf(x, -1.0e9f), 1.0e9f); }

// Transaxial footprint of one voxel column in one view.
struct SfColumn {
    double xi;            // detector column coordinate of the voxel centre
    double den;           // sod - l at the voxel centre (1 for parallel-beam)
    double inv;           // 1 / den
    float o0, o1, o2, o3; // sorted knot offsets from xi, in pixels
    float h01, h23;       // 1 / (2 (o1-o0)),  1 / (2 (o3-o2))   (guarded against zero-width ramps)
};

SF_HD void sf_sort4(float a, float b, float c, float d, float &o0, float &o1, float &o2, float &o3)
{
    float lo1 = fminf(a, b), hi1 = fmaxf(a, b), lo2 = fminf(c, d), hi2 = fmaxf(c, d);
    o0 = fminf(lo1, lo2);
    o3 = fmaxf(hi1, hi2);
    float m1 = fmaxf(lo1, lo2), m2 = fminf(hi1, hi2);
    o1 = fminf(m1, m2);
    o2 = fmaxf(m1, m2);
}

// GT: what the caller knows about the detector at compile time (-1: nothing, look at g.type; 0: not curved; 1: curved).
// The fast kernels pass it so that the flat-detector instances carry no code for the cylinder.
template <int GT>
SF_HD bool sf_is_curved(const SfGeom &g)
{
    return GT < 0 ? g.type == SF_CONE_CURVED : GT == 1;
}

template <int GT = -1>
SF_HD SfColumn sf_column(const SfGeom &g, const SfView &v, int i, int j)
{
    SfColumn f;
    const double x = fma((double)i, g.Td, g.x0d);
    const double y = fma((double)j, g.Td, g.y0d);
    const double t = fma(y, v.cd, -x * v.sd);
    if (g.type == SF_PARALLEL) {
        f.xi = fma(t, g.kud, g.col_offd);
        f.den = 1.0;
        f.inv = 1.0;
        f.o0 = -v.par_out; f.o1 = -v.par_in; f.o2 = v.par_in; f.o3 = v.par_out;
    } else if (sf_is_curved<GT>(g)) {
        // Cylindrical detector: the column coordinate is the fan angle (arc length over the pixel width), and the axial
        // magnification goes with the in-plane distance from the source.
        const double dn = g.sodd - fma(x, v.cd, y * v.sd);
        const double r2 = fma(dn, dn, t * t);
        f.den = sqrt(r2);
        f.inv = sf_rcp_d(f.den);
        f.xi = fma(g.kud, atan2(t, dn), g.col_offd);
        // Knot offsets in float: the angle between the centre and a corner displaced by (dt, dl) is
        //   atan2(dt dn + t dl, r2 - dn dl + t dt).
        const float tf = (float)t, dnf = (float)dn, r2f = (float)r2;
        const float dtA = v.p - v.q, dlA = v.p + v.q;
        const float dtB = -dlA, dlB = dtA;
        const float nA = fmaf(dtA, dnf, tf * dlA), nB = fmaf(dtB, dnf, tf * dlB);
        const float eA = fmaf(tf, dtA, -dnf * dlA), eB = fmaf(tf, dtB, -dnf * dlB);
        sf_sort4(g.ku * atanf(nA * sf_rcp(r2f + eA)), -g.ku * atanf(nA * sf_rcp(r2f - eA)),
                 g.ku * atanf(nB * sf_rcp(r2f + eB)), -g.ku * atanf(nB * sf_rcp(r2f - eB)), f.o0, f.o1, f.o2, f.o3);
    } else {
        const double l = fma(x, v.cd, y * v.sd);
        f.den = g.sodd - l;
        f.inv = sf_rcp_d(f.den);
        f.xi = fma(g.kud * t, f.inv, g.col_offd);
        // Knot offsets in float.  Corner (dx,dy) = (+h,+h) has (dt,dl) = (p-q, p+q); (+h,-h) has (-(p+q), p-q); the
        // other two corners are their negatives.  Offset of a corner from the centre on the detector:
        //   ku [ (t+dt)/(den-dl) - t/den ] = (ku/den) (dt den + t dl) / (den - dl)
        const float tf = (float)t, den = (float)f.den;
        const float kin = g.ku * (float)f.inv;
        const float dtA = v.p - v.q, dlA = v.p + v.q;
        const float dtB = -dlA, dlB = dtA;
        const float d2 = den * den;
        const float rA = sf_rcp(fmaf(-dlA, dlA, d2));      // 1/((den-dlA)(den+dlA))
        const float rB = sf_rcp(fmaf(-dlB, dlB, d2));
        const float nA = kin * fmaf(dtA, den, tf * dlA) * rA;
        const float nB = kin * fmaf(dtB, den, tf * dlB) * rB;
        sf_sort4(nA * (den + dlA), -nA * (den - dlA), nB * (den + dlB), -nB * (den - dlB), f.o0, f.o1, f.o2, f.o3);
    }
    f.h01 = 0.5f * sf_rcp(fmaxf(f.o1 - f.o0, 1e-20f));
    f.h23 = 0.5f * sf_rcp(fmaxf(f.o3 - f.o2, 1e-20f));
    return f;
}

// atan for the small angles between a voxel's centre and its corners as seen from the source: three terms of the
// series, error below x^7 / 7 (3e-9 rad at |x| = 0.08; the fast kernels are only chosen below that).
SF_HD float sf_atan_small(float x)
{
    const float x2 = x * x;
    return x * fmaf(x2, fmaf(x2, 0.2f, -0.33333334f), 1.0f);
}

// Cylindrical detector, for kernels whose threads sit close to a reference point (the centre of the workgroup's
// tile): tref, dnref are the reference point's coordinate across the central ray and its distance from the source
// along it, gref its fan angle, all in double.  The voxel's fan angle is gref plus the small angle between the two
// directions from the source, whose tangent is the cross product over the dot product of the two (formed in double,
// divided and fed to atanf in float).  Same results as sf_column to a few 1e-7 pixels at a fraction of the
// instructions of a double-precision atan2.
SF_HD SfColumn sf_column_curved_ref(const SfGeom &g, const SfView &v, int i, int j, double tref, double dnref, double gref)
{
    SfColumn f;
    const double x = fma((double)i, g.Td, g.x0d);
    const double y = fma((double)j, g.Td, g.y0d);
    const double t = fma(y, v.cd, -x * v.sd);
    const double dn = g.sodd - fma(x, v.cd, y * v.sd);
    const double r2 = fma(dn, dn, t * t);
    f.den = sqrt(r2);
    f.inv = sf_rcp_d(f.den);
    const double cross = fma(dnref, t, -tref * dn), dot = fma(dnref, dn, tref * t);
    const float delta = atanf((float)cross * sf_rcp((float)dot));
    f.xi = fma(g.kud, gref + (double)delta, g.col_offd);
    const float tf = (float)t, dnf = (float)dn, r2f = (float)r2;
    const float dtA = v.p - v.q, dlA = v.p + v.q;
    const float dtB = -dlA, dlB = dtA;
    const float nA = fmaf(dtA, dnf, tf * dlA), nB = fmaf(dtB, dnf, tf * dlB);
    const float eA = fmaf(tf, dtA, -dnf * dlA), eB = fmaf(tf, dtB, -dnf * dlB);
    sf_sort4(g.ku * sf_atan_small(nA * sf_rcp(r2f + eA)), -g.ku * sf_atan_small(nA * sf_rcp(r2f - eA)),
             g.ku * sf_atan_small(nB * sf_rcp(r2f + eB)), -g.ku * sf_atan_small(nB * sf_rcp(r2f - eB)), f.o0, f.o1, f.o2, f.o3);
    f.h01 = 0.5f * sf_rcp(fmaxf(f.o1 - f.o0, 1e-20f));
    f.h23 = 0.5f * sf_rcp(fmaxf(f.o3 - f.o2, 1e-20f));
    return f;
}

// Running integral of the unit trapezoid up to u (pixels, measured from the voxel centre's xi), up to an
// additive constant that cancels in differences.
SF_HD float sf_trap_integral(const SfColumn &f, float u)
{
    const float a = sf_clamp(u, f.o0, f.o1) - f.o0;
    const float b = sf_clamp(u, f.o1, f.o2);
    const float c = f.o3 - sf_clamp(u, f.o2, f.o3);
    return fmaf(a * a, f.h01, b) - c * c * f.h23;
}

// First and last detector column the footprint can touch (not yet clipped to the detector).
SF_HD void sf_col_range(const SfColumn &f, int &c_first, int &c_last)
{
    c_first = (int)floor(f.xi + (double)f.o0 + 0.5);
    c_last = (int)floor(f.xi + (double)f.o3 + 0.5);
}

// Lower edge of pixel c measured from the voxel centre, pixels.
SF_HD float sf_pixel_edge(const SfColumn &f, int c) { return (float)(((double)c - 0.5) - f.xi); }

// F_u of the pixel whose lower edge (from sf_pixel_edge) is ulo.
SF_HD float sf_fu_at(const SfColumn &f, float ulo)
{
    return fmaxf(sf_trap_integral(f, ulo + 1.0f) - sf_trap_integral(f, ulo), 0.0f);
}

SF_HD float sf_fu(const SfColumn &f, int c) { return sf_fu_at(f, sf_pixel_edge(f, c)); }

// ---- axial part -----------------------------------------------------------------------------------

// Voxel-driven view: the chunk of voxels starting at k0 (lower face zlo_k0, mm) seen on the detector.
// Relative to row rb, voxel k0+kk covers eta in [phi0 + kk av, phi0 + (kk+1) av).
struct SfRowsOfVoxels {
    int rb;
    float phi0, av;
};

SF_HD SfRowsOfVoxels sf_rows_of_voxels(const SfGeom &g, const SfColumn &f, double zlo_k0)
{
    SfRowsOfVoxels a;
    const double m = g.kvd * f.inv;                    // rows per mm at this voxel column
    const double eta0 = fma(m, zlo_k0, g.row_offd);
    const double fl = floor(eta0);
    a.rb = (int)fl;
    a.phi0 = (float)(eta0 - fl);
    a.av = (float)(m * g.Tzd);
    return a;
}

// F_v of (row rb+rr, voxel k0+kk).
SF_HD float sf_fv_rows(const SfRowsOfVoxels &a, int rr, int kk)
{
    const float lo = fmaf(a.av, (float)kk, a.phi0);
    const float hi = fmaf(a.av, (float)(kk + 1), a.phi0);
    return fmaxf(fminf((float)(rr + 1), hi) - fmaxf((float)rr, lo), 0.0f);
}

// Ray-driven view: the chunk of rows starting at r0 seen in the voxel column.  Relative to voxel kb,
// row r0+rr covers kappa in [psi0 + rr step, psi0 + (rr+1) step); F_v = av * overlap in kappa.
struct SfVoxelsOfRows {
    int kb;
    float psi0, step, av;
};

SF_HD SfVoxelsOfRows sf_voxels_of_rows(const SfGeom &g, const SfColumn &f, int r0)
{
    SfVoxelsOfRows a;
    const double mm_per_row = f.den * g.ikvd;
    const double kap0 = (((double)r0 - g.row_offd) * mm_per_row - g.zlo0d) * g.iTzd;
    const double fl = floor(kap0);
    a.kb = (int)fl;
    a.psi0 = (float)(kap0 - fl);
    a.step = (float)(mm_per_row * g.iTzd);
    a.av = (float)(g.kvd * f.inv * g.Tzd);
    return a;
}

SF_HD float sf_fv_voxels(const SfVoxelsOfRows &a, int rr, int kk)
{
    const float lo = fmaf(a.step, (float)rr, a.psi0);
    const float hi = fmaf(a.step, (float)(rr + 1), a.psi0);
    return a.av * fmaxf(fminf((float)(kk + 1), hi) - fmaxf((float)kk, lo), 0.0f);
}

// ---- ray amplitude --------------------------------------------------------------------------------
// Column part: gcol = T / max(|D_x|,|D_y|) and wcol = sdd^2 + u^2;  amp = gcol * sqrt(wcol + v^2).
struct SfAmpCol {
    float gcol, wcol;
};

template <int GT = -1>
SF_HD SfAmpCol sf_amp_col(const SfGeom &g, const SfView &v, int c)
{
    SfAmpCol a;
    const float u = ((float)c - g.col_off) * g.pu;
    if (sf_is_curved<GT>(g)) {       // pixel at fan angle u / sdd on the cylinder: |D_xy| = sdd
        float sg, cg;
        sincosf(u / g.sdd, &sg, &cg);
        const float dx = -g.sdd * fmaf(cg, v.c, sg * v.s);
        const float dy = g.sdd * fmaf(sg, v.c, -cg * v.s);
        a.gcol = g.T * sf_rcp(fmaxf(fabsf(dx), fabsf(dy)));
        a.wcol = g.sdd * g.sdd;
        return a;
    }
    const float dx = fmaf(-g.sdd, v.c, -u * v.s);
    const float dy = fmaf(-g.sdd, v.s, u * v.c);
    a.gcol = g.T * sf_rcp(fmaxf(fabsf(dx), fabsf(dy)));
    a.wcol = fmaf(g.sdd, g.sdd, u * u);
    return a;
}

// Cylindrical detector, with the cosine and sine of the pixel's fan angle taken from a per-column table (they do not
// depend on the view).
SF_HD SfAmpCol sf_amp_col_curved(const SfGeom &g, const SfView &v, float cg, float sg)
{
    SfAmpCol a;
    const float dx = -g.sdd * fmaf(cg, v.c, sg * v.s);
    const float dy = g.sdd * fmaf(sg, v.c, -cg * v.s);
    a.gcol = g.T * sf_rcp(fmaxf(fabsf(dx), fabsf(dy)));
    a.wcol = g.sdd * g.sdd;
    return a;
}

SF_HD float sf_amp(const SfGeom &g, const SfView &v, const SfAmpCol &a, int r)
{
    if (g.type == SF_PARALLEL) return v.par_amp;
    const float vv = (g.type == SF_FAN) ? 0.0f : fmaf((float)r, g.pv, g.v0);
    return a.gcol * sf_sqrt(fmaf(vv, vv, a.wcol));
}

// The same with the row's detector coordinate v given (callers that walk rows in equal steps add the step).
SF_HD float sf_amp_at(const SfGeom &g, const SfView &v, const SfAmpCol &a, float vv)
{
    if (g.type == SF_PARALLEL) return v.par_amp;
    if (g.type == SF_FAN) vv = 0.0f;
    return a.gcol * sf_sqrt(fmaf(vv, vv, a.wcol));
}
