// Separable-footprint weight factors, evaluated identically by the forward (ray-driven) and the
// back (voxel-driven) kernels so that the pair is matched: both call these functions with the same
// (view, voxel column, pixel) arguments and obtain bit-identical F_u, F_v and amplitude.
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

SF_HD float sf_rcp(float x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    float r = __builtin_amdgcn_rcpf(x);
#else
    float r = 1.0f / x;
#endif
    return fmaf(r, fmaf(-x, r, 1.0f), r);   // one Newton step: below half an ulp of error in practice
}

SF_HD float sf_clamp(float x, float lo, float hi)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_fmed3f(x, lo, hi);
#else
    return fminf(fmaxf(x, lo), hi);
#endif
}

// Transaxial footprint of one voxel column in one view.
struct SfColumn {
    float xi;            // detector column coordinate of the voxel centre
    float o0, o1, o2, o3; // sorted knot offsets from xi, in pixels
    float h01, h23;      // 1 / (2 (o1-o0)),  1 / (2 (o3-o2))   (guarded against zero-width ramps)
    float inv;           // 1 / (sod - l) at the voxel centre (1 for parallel-beam)
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

// x, y: voxel centre in mm.
SF_HD SfColumn sf_column(const SfGeom &g, const SfView &v, float x, float y)
{
    SfColumn f;
    float t = fmaf(y, v.c, -x * v.s);
    if (g.type == SF_PARALLEL) {
        f.xi = fmaf(t, g.ku, g.col_off);
        f.o0 = -v.par_out; f.o1 = -v.par_in; f.o2 = v.par_in; f.o3 = v.par_out;
        f.inv = 1.0f;
    } else {
        float l = fmaf(x, v.c, y * v.s);
        float den = g.sod - l;
        f.inv = sf_rcp(den);
        float kin = g.ku * f.inv;
        f.xi = fmaf(kin, t, g.col_off);
        // corner offsets (dx,dy) = (+h,+h) -> (dt,dl) = (p-q, p+q);  (+h,-h) -> (-(p+q), p-q); the other two are
        // their negatives.  Offset of a corner from the centre on the detector:
        //   ku [ (t+dt)/(den-dl) - t/den ] = kin (dt den + t dl) / (den - dl)
        float dtA = v.p - v.q, dlA = v.p + v.q;
        float dtB = -dlA, dlB = dtA;
        float d2 = den * den;
        float rA = sf_rcp(fmaf(-dlA, dlA, d2));      // 1/((den-dlA)(den+dlA))
        float rB = sf_rcp(fmaf(-dlB, dlB, d2));
        float nA = kin * fmaf(dtA, den, t * dlA) * rA;
        float nB = kin * fmaf(dtB, den, t * dlB) * rB;
        float a0 = nA * (den + dlA);     // corner +A : 1/(den-dlA) = (den+dlA) rA
        float a1 = -nA * (den - dlA);    // corner -A
        float b0 = nB * (den + dlB);
        float b1 = -nB * (den - dlB);
        sf_sort4(a0, a1, b0, b1, f.o0, f.o1, f.o2, f.o3);
    }
    f.h01 = 0.5f / fmaxf(f.o1 - f.o0, 1e-20f);
    f.h23 = 0.5f / fmaxf(f.o3 - f.o2, 1e-20f);
    return f;
}

// Running integral of the unit trapezoid up to u (pixels, measured from the voxel centre's xi), up to an
// additive constant that cancels in differences.
SF_HD float sf_trap_integral(const SfColumn &f, float u)
{
    float a = sf_clamp(u, f.o0, f.o1) - f.o0;
    float b = sf_clamp(u, f.o1, f.o2);
    float c = f.o3 - sf_clamp(u, f.o2, f.o3);
    return fmaf(a * a, f.h01, b) - c * c * f.h23;
}

// First and last detector column the footprint can touch (not yet clipped to the detector).
SF_HD void sf_col_range(const SfColumn &f, int &c_first, int &c_last)
{
    c_first = (int)floorf(f.xi + f.o0 + 0.5f);
    c_last = (int)floorf(f.xi + f.o3 + 0.5f);
}

// F_u of pixel c.
SF_HD float sf_fu(const SfColumn &f, int c)
{
    float ulo = ((float)c - 0.5f) - f.xi;
    return fmaxf(sf_trap_integral(f, ulo + 1.0f) - sf_trap_integral(f, ulo), 0.0f);
}

// Axial map of one voxel column: eta(lower face of voxel k) = av * k + bv.
struct SfAxial {
    float av, bv;
};

SF_HD SfAxial sf_axial(const SfGeom &g, float inv)
{
    SfAxial a;
    float m = g.kv * inv;                 // rows per mm at this voxel column
    a.av = m * g.Tz;
    a.bv = fmaf(m, g.zlo0, g.row_off);
    return a;
}

// F_v of (row r, voxel k): overlap of [r, r+1) with [eta_k, eta_{k+1}).
SF_HD float sf_fv(const SfAxial &a, int r, int k)
{
    float lo = fmaf(a.av, (float)k, a.bv);
    float hi = fmaf(a.av, (float)(k + 1), a.bv);
    return fmaxf(fminf((float)(r + 1), hi) - fmaxf((float)r, lo), 0.0f);
}

// Ray amplitude.  Column part: gcol = T / max(|D_x|,|D_y|) and wcol = sdd^2 + u^2; amp = gcol * sqrt(wcol + v^2).
struct SfAmpCol {
    float gcol, wcol;
};

SF_HD SfAmpCol sf_amp_col(const SfGeom &g, const SfView &v, int c)
{
    SfAmpCol a;
    float u = ((float)c - g.col_off) * g.pu;
    float dx = fmaf(-g.sdd, v.c, -u * v.s);
    float dy = fmaf(-g.sdd, v.s, u * v.c);
    a.gcol = g.T * sf_rcp(fmaxf(fabsf(dx), fabsf(dy)));
    a.wcol = fmaf(g.sdd, g.sdd, u * u);
    return a;
}

SF_HD float sf_amp(const SfGeom &g, const SfView &v, const SfAmpCol &a, int r)
{
    if (g.type == SF_PARALLEL) return v.par_amp;
    float vv = (g.type == SF_FAN) ? 0.0f : fmaf((float)r, g.pv, g.v0);
    return a.gcol * sqrtf(fmaf(vv, vv, a.wcol));
}
