// Plain-data parameter blocks shared by the host geometry module and the HIP kernels.
//
// Index coordinates used throughout the kernels:
//   xi  (detector column coordinate): pixel c covers [c - 1/2, c + 1/2];  xi(u) = u / pixel_u + col_off
//   eta (detector row coordinate)   : pixel r covers [r, r + 1);          eta(v) = v / pixel_v + row_off
//   voxel k has its lower face at z = zlo0 + k * Tz (z measured from the source plane z = 0).
#pragma once

#include <stdint.h>

enum { SF_PARALLEL = 0, SF_FAN = 1, SF_CONE = 2 };

struct SfGeom {
    int32_t type;
    int32_t nviews, nrows, ncols;
    int32_t nx, ny, nz;
    float T, Tz;          // voxel sizes, mm
    float x0, y0;         // centre of voxel (i,j) = (0,0), mm
    float zlo0;           // lower face of voxel k = 0, mm
    float sod, sdd;       // mm (cone / fan)
    float pu, pv;         // pixel sizes, mm
    float ku;             // parallel: 1/pu ; cone/fan: sdd/pu   (xi  = ku * t * inv_den + col_off)
    float kv;             // parallel: 1/pv ; cone    : sdd/pv   (eta = kv * z * inv_den + row_off)
    float col_off;        // (ncols-1)/2 - shift_u
    float row_off;        // (nrows-1)/2 - shift_v + 1/2
    float v0;             // v (mm) of row 0's centre: (-(nrows-1)/2 + shift_v) * pv
};

// One entry per view, built in double on the host.
struct SfView {
    float c, s;           // cos(phi), sin(phi)
    float p, q;           // (T/2) cos(phi), (T/2) sin(phi)
    float par_out;        // parallel: outer half-width of the trapezoid in pixels, (T/2)(|c|+|s|)/pu
    float par_in;         // parallel: inner half-width, (T/2)||c|-|s||/pu
    float par_amp;        // parallel: T / max(|c|,|s|)  (mm)
    int32_t xmajor;       // 1: rays of this view run mostly along x (|cos phi| >= |sin phi|)
};
