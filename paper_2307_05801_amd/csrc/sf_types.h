// Plain-data parameter blocks shared by the host geometry module and the HIP kernels.
//
// Index coordinates used throughout the kernels:
//   xi  (detector column coordinate): pixel c covers [c - 1/2, c + 1/2];  xi(u) = u / pixel_u + col_off
//   eta (detector row coordinate)   : pixel r covers [r, r + 1);          eta(v) = v / pixel_v + row_off
//   kappa (axial voxel coordinate)  : voxel k covers [k, k + 1);          kappa(z) = (z - zlo0) / Tz
//   z is measured from the source plane z = 0.
//
// Precision plan: absolute positions on the detector (xi of a voxel centre, eta / kappa of the first
// face of a thread's chunk) are formed in double, because a float carries only ~3e-5 pixels at index
// 512 and a back projection of few noisy views shows that error directly.  Everything measured
// relative to such a base (knot offsets, fractions, overlaps, weights) is float.
#pragma once

#include <stdint.h>

enum { SF_PARALLEL = 0, SF_FAN = 1, SF_CONE = 2, SF_CONE_CURVED = 3, SF_MODULAR = 4 };   // CURVED: cylindrical detector, columns equally spaced in arc length; MODULAR: per-view poses
enum { SF_MODEL_FOOTPRINT = 0, SF_MODEL_SIDDON = 1 };

struct SfGeom {
    int32_t type;
    int32_t nviews, nrows, ncols;
    int32_t nx, ny, nz;
    int32_t model;        // SF_MODEL_FOOTPRINT / SF_MODEL_SIDDON
    // double: bases
    double Td, Tzd;       // voxel sizes, mm
    double x0d, y0d;      // centre of voxel (i,j) = (0,0), mm
    double zlo0d;         // lower face of voxel k = 0, mm
    double sodd;          // source to rotation axis, mm
    double kud;           // parallel: 1/pu ; cone/fan: sdd/pu   (xi  = kud * t / den + col_offd; curved: kud * fan angle + col_offd)
    double kvd;           // parallel: 1/pv ; cone    : sdd/pv   (eta = kvd * z / den + row_offd; curved: den = in-plane distance from the source)
    double ikvd;          // 1 / kvd
    double iTzd;          // 1 / Tz
    double col_offd;      // (ncols-1)/2 - shift_u
    double row_offd;      // (nrows-1)/2 - shift_v + 1/2
    double v0d, pvd;      // v (mm) of row 0's centre and the row pitch: v_r = v0d + r pvd
    double pu_d;          // column pitch, mm
    double zk0d;          // kappa of the plane z = 0: -zlo0 / Tz  (fan-beam: 1/2, the middle of the only slice)
    // float: relative quantities
    float T, Tz;
    float sod, sdd;
    float pu, pv;
    float ku;             // (float)kud
    float col_off;        // (float)col_offd, used by the ray amplitude only
    float v0;             // v (mm) of row 0's centre: (-(nrows-1)/2 + shift_v) * pv
};

// One entry per view, built in double on the host.
struct SfView {
    double cd, sd;        // cos(phi), sin(phi)
    float c, s;
    float p, q;           // (T/2) cos(phi), (T/2) sin(phi)
    float par_out;        // parallel: outer half-width of the trapezoid in pixels, (T/2)(|c|+|s|)/pu
    float par_in;         // parallel: inner half-width, (T/2)||c|-|s||/pu
    float par_amp;        // parallel: T / max(|c|,|s|)  (mm)
    int32_t xmajor;       // 1: rays of this view run mostly along x (|cos phi| >= |sin phi|)
};
