// Tiled back projection (A^T) of the Siddon model on tilted modules of the modular geometry ("CT Projection Models and
// Geometries": sources and detectors at any position and orientation; matched transpose): voxel-driven, no atomics,
// bitwise reproducible.
//
// Same plan as the circular kernel (sd_backproject_tiled.h): a workgroup of 256 threads owns a 16 x 16 tile of voxel
// columns and ZC voxels along z, a thread one column; per view the workgroup stages into LDS the window of the
// detector that its tile's box projects into; a thread walks rows of the window and adds each row's (at most) two
// shares to its per-thread sums in LDS (slot-major, one writer per slot, plain read-add-write).
//
// What a tilted module changes: the rays of a detector column no longer share their in-plane line, so the in-plane
// piece [t0, t1] of the slab is worked out per (voxel column, pixel), from the slopes the staging step stores with every
// sample.  A pixel's ray is minor(X) = m X + b, Z(X) = mz X + bz along the tile's fastest in-plane axis X; a thread
// needs minor and Z at its own slab X = n relative to its own cell, with a lever arm of a thousand voxels back to the
// source, and it needs the distances to the cell's faces to a RELATIVE accuracy (they are divided by m and mz, which may
// be tiny): positions are formed in double from slopes kept in double, the distance to a face is taken in double and
// only then rounded to float.
//
// A rolled module also turns a voxel column's projection into a slanted strip, so a thread may meet many detector
// columns, each over a short run of rows: the four vertical edges of the column's box project to lines, and the rows a
// detector column can be hit from lie between those lines.
//
// Chosen on the host only if every ray rises by at most 0.8 axial cells per slab along its own fastest in-plane axis and
// every source is at least 102 voxels away from the volume in the plane (then the rise along the TILE's axis stays below
// one cell for every ray through the tile, and a row's piece lies in at most two axial cells), the whole volume lies in
// front of every source, and the windows fit the instance.
#pragma once

#include "md_siddon.h"
#include "sf_backproject_tiled.h"

// Shapes this kernel is instantiated for (voxels along z per thread, staged window columns x rows), in the order they
// are tried.  LDS per workgroup: 28 bytes per staged sample (row stride pw + 1) plus (zc + 4) KiB of sums; the first shape
// leaves room for four workgroups per compute unit, the second for three, the next two for two.
constexpr SfBpShape MD_BP_SHAPES[] = {{16, 32, 21}, {16, 32, 35}, {32, 32, 44}, {16, 32, 44}, {32, 32, 56}, {16, 64, 48}};
constexpr int MD_BP_NSHAPES = 6;
constexpr double MD_BP_ZBIAS = 1048576.0;      // added to axial positions so that truncation is floor for every row of a window

// One entry per view, built in double on the host.
struct MdBpView {
    double A0[3], Au[3], Av[3];      // pixel (r, c) minus source = A0 + c Au + r Av, mm
    double sidx[3];                  // the source in index coordinates (voxel i covers [i, i + 1) on every axis)
    float dlo[3];                    // position of index (0, 0, 0) minus the source, mm
    float euP[3], evP[3], nrm[3];    // a point S + d projects to column coordinate (d.euP)/(d.nrm) + xi0 (pixel c has its
    float xi0, eta0;                 //   centre at c) and row coordinate (d.evP)/(d.nrm) + eta0 (row r at r)
};

inline MdBpView md_bp_view(const SfGeom &g, const MdPose &P)
{
    MdBpView V;
    const double u0 = (0.0 - g.col_offd) * g.pu_d;
    const double lo[3] = {g.x0d - 0.5 * g.Td, g.y0d - 0.5 * g.Td, g.zlo0d}, pitch[3] = {g.Td, g.Td, g.Tzd};
    double n[3] = {P.ucol[1] * P.vrow[2] - P.ucol[2] * P.vrow[1], P.ucol[2] * P.vrow[0] - P.ucol[0] * P.vrow[2],
                   P.ucol[0] * P.vrow[1] - P.ucol[1] * P.vrow[0]};
    double gap = 0.0, su = 0.0, sv = 0.0;
    for (int q = 0; q < 3; ++q) {
        V.A0[q] = P.C[q] - P.S[q] + u0 * P.ucol[q] + g.v0d * P.vrow[q];
        V.Au[q] = g.pu_d * P.ucol[q];
        V.Av[q] = g.pvd * P.vrow[q];
        V.sidx[q] = (P.S[q] - lo[q]) / pitch[q];
        V.dlo[q] = (float)(lo[q] - P.S[q]);
        gap += (P.C[q] - P.S[q]) * n[q];
        su += (P.S[q] - P.C[q]) * P.ucol[q];
        sv += (P.S[q] - P.C[q]) * P.vrow[q];
    }
    for (int q = 0; q < 3; ++q) {
        V.euP[q] = (float)(P.ucol[q] * gap / g.pu_d);
        V.evP[q] = (float)(P.vrow[q] * gap / g.pvd);
        V.nrm[q] = (float)n[q];
    }
    V.xi0 = (float)(su / g.pu_d + g.col_offd);
    V.eta0 = (float)((sv - g.v0d) / g.pvd);
    return V;
}

// The axis-aligned box of index coordinates [x0, x1] x [y0, y1] x [z0, z1], projected onto the detector (index
// coordinates: pixel c has its centre at column coordinate c, row r at row coordinate r): its eight corners.
struct MdBoxShadow {
    float xi[8], eta[8];             // corner q: x1 if q & 1, y1 if q & 2, z1 if q & 4
    float xi_lo, xi_hi, eta_lo, eta_hi;
};

SF_HD MdBoxShadow md_bp_shadow(const SfGeom &g, const MdBpView &V, float x0, float x1, float y0, float y1, float z0, float z1)
{
    // numerators and denominator of the projection are linear in the point: corner 0 in full, the others by increments
    const float dx = fmaf(x0, g.T, V.dlo[0]), dy = fmaf(y0, g.T, V.dlo[1]), dz = fmaf(z0, g.Tz, V.dlo[2]);
    const float ex = (x1 - x0) * g.T, ey = (y1 - y0) * g.T, ez = (z1 - z0) * g.Tz;
    float nu[8], nv[8], dn[8];
    nu[0] = fmaf(dx, V.euP[0], fmaf(dy, V.euP[1], dz * V.euP[2]));
    nv[0] = fmaf(dx, V.evP[0], fmaf(dy, V.evP[1], dz * V.evP[2]));
    dn[0] = fmaf(dx, V.nrm[0], fmaf(dy, V.nrm[1], dz * V.nrm[2]));
    const float sx[3] = {ex * V.euP[0], ex * V.evP[0], ex * V.nrm[0]}, sy[3] = {ey * V.euP[1], ey * V.evP[1], ey * V.nrm[1]},
                sz[3] = {ez * V.euP[2], ez * V.evP[2], ez * V.nrm[2]};
    nu[1] = nu[0] + sx[0]; nv[1] = nv[0] + sx[1]; dn[1] = dn[0] + sx[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) { nu[q + 2] = nu[q] + sy[0]; nv[q + 2] = nv[q] + sy[1]; dn[q + 2] = dn[q] + sy[2]; }
#pragma unroll
    for (int q = 0; q < 4; ++q) { nu[q + 4] = nu[q] + sz[0]; nv[q + 4] = nv[q] + sz[1]; dn[q + 4] = dn[q] + sz[2]; }
    MdBoxShadow B;
    B.xi_lo = B.eta_lo = 3.0e38f;
    B.xi_hi = B.eta_hi = -3.0e38f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const float inv = sf_rcp(dn[q]);
        B.xi[q] = fmaf(nu[q], inv, V.xi0);
        B.eta[q] = fmaf(nv[q], inv, V.eta0);
        B.xi_lo = fminf(B.xi_lo, B.xi[q]); B.xi_hi = fmaxf(B.xi_hi, B.xi[q]);
        B.eta_lo = fminf(B.eta_lo, B.eta[q]); B.eta_hi = fmaxf(B.eta_hi, B.eta[q]);
    }
    return B;
}

// Window of the detector that the voxels of a tile's box can be hit from: pixel centres inside the box's shadow.
SF_HD SfWindow md_bp_window(const SfGeom &g, const MdBpView &V, int i0, int j0, int k0, int zc)
{
    const MdBoxShadow B = md_bp_shadow(g, V, (float)i0, (float)(i0 + BP_T), (float)j0, (float)(j0 + BP_T), (float)k0, (float)(k0 + zc));
    SfWindow w;
    w.c0 = sf_f2i(ceilf(B.xi_lo - 0.02f));
    w.r0 = sf_f2i(ceilf(B.eta_lo - 0.02f));
    w.need_w = sf_f2i(floorf(B.xi_hi + 0.02f)) - w.c0 + 1;
    w.need_h = sf_f2i(floorf(B.eta_hi + 0.02f)) - w.r0 + 1;
    return w;
}

// The in-plane axis the rays through a tile advance fastest on, judged by the ray to the tile's centre.
SF_HD bool md_bp_tile_xmajor(const SfGeom &g, const MdBpView &V, int i0, int j0)
{
    const float dx = fmaf((float)i0 + 0.5f * BP_T, g.T, V.dlo[0]), dy = fmaf((float)j0 + 0.5f * BP_T, g.T, V.dlo[1]);
    return fabsf(dx) >= fabsf(dy);
}

// Slopes of pixel (r, c)'s ray along the tile's axis: minor per unit X, Z per unit X (index units), and mm per unit X.
struct MdBpSlopes {
    double m, mz;
    float len;
};

SF_HD MdBpSlopes md_bp_slopes(const SfGeom &g, const MdBpView &V, bool xmajor, int r, int c)
{
    const double dx = fma((double)r, V.Av[0], fma((double)c, V.Au[0], V.A0[0]));
    const double dy = fma((double)r, V.Av[1], fma((double)c, V.Au[1], V.A0[1]));
    const double dz = fma((double)r, V.Av[2], fma((double)c, V.Au[2], V.A0[2]));
    const double dmaj = xmajor ? dx : dy, dmin = xmajor ? dy : dx;
    double inv = (double)sf_rcp((float)dmaj);
    inv = inv * fma(-dmaj, inv, 2.0);                  // one Newton step: relative error of the float reciprocal, squared
    MdBpSlopes s;
    s.m = dmin * inv;
    s.mz = dz * inv * (g.Td / g.Tzd);
    s.len = g.T * sf_sqrt((float)fma(dx, dx, fma(dy, dy, dz * dz))) * fabsf((float)inv);
    return s;
}

// What the staging step stores per sample of the window.
struct MdBpPixel {
    double m, mz;        // slopes along the tile's axis
    float wy;            // sample times mm of ray per unit of X
    float inv_m;         // 1 / m (1e30 where m vanishes)
    float inv_mz;        // 1 / mz (1e30 where mz vanishes)
};

SF_HD MdBpPixel md_bp_pixel(const MdBpSlopes &s, float y)
{
    MdBpPixel p;
    p.m = s.m;
    p.mz = s.mz;
    p.wy = y * s.len;
    const float mf = (float)s.m, mzf = (float)s.mz;
    p.inv_m = fabsf(mf) > 1e-30f ? 1.0f / mf : 1e30f;
    p.inv_mz = fabsf(mzf) > 1e-30f ? 1.0f / mzf : 1e30f;
    return p;
}

// A thread's voxel column in one view: which detector columns can hit it, and the lines that bound the rows.
struct MdBpColumn {
    int cfirst, clast;
    float ub[4], vb[4], slope[4];    // the four vertical edges of the column's box: shadow of the lower end, rows per column
    bool slanted;                    // false: the edges' shadows are too close to vertical to bound the rows
    float eta_lo, eta_hi;
    double ln, bq, bz;               // n - xs; minor of the source minus the cell's minor index; Z of the source in slots + MD_BP_ZBIAS
};

template <int ZC>
SF_HD MdBpColumn md_bp_column(const SfGeom &g, const MdBpView &V, bool xmajor, int ic, int jc, int k0)
{
    MdBpColumn C;
    const MdBoxShadow B = md_bp_shadow(g, V, (float)ic, (float)(ic + 1), (float)jc, (float)(jc + 1), (float)k0, (float)(k0 + ZC));
    C.cfirst = sf_f2i(ceilf(B.xi_lo - 0.01f));
    C.clast = sf_f2i(floorf(B.xi_hi + 0.01f));
    C.eta_lo = B.eta_lo; C.eta_hi = B.eta_hi;
    // The shadows of the four vertical edges bound the rows only if they all lean the same way by a clear margin (a
    // quarter of a column over the chunk); perspective alone makes near-vertical shadows lean apart by a few hundredths.
    bool right = true, left = true;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float du = B.xi[e + 4] - B.xi[e];
        right = right && du > 0.25f;
        left = left && du < -0.25f;
        C.ub[e] = B.xi[e]; C.vb[e] = B.eta[e];
        C.slope[e] = (B.eta[e + 4] - B.eta[e]) * sf_rcp(fabsf(du) > 0.25f ? du : 1.0f);
    }
    C.slanted = right || left;
    const int n = xmajor ? ic : jc, q = xmajor ? jc : ic;
    C.ln = (double)n - V.sidx[xmajor ? 0 : 1];
    C.bq = V.sidx[xmajor ? 1 : 0] - (double)q;
    C.bz = V.sidx[2] - (double)k0 + 2.0 + MD_BP_ZBIAS;
    return C;
}

// Rows [rs, re) of the window (r0, H rows) that detector column c can hit the voxel column from.
SF_HD void md_bp_rows(const MdBpColumn &C, int c, int r0, int H, int &rs, int &re)
{
    float lo = C.eta_lo, hi = C.eta_hi;
    if (C.slanted) {
        float a = 3.0e38f, b = -3.0e38f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float v = fmaf((float)c - C.ub[e], C.slope[e], C.vb[e]);
            a = fminf(a, v); b = fmaxf(b, v);
        }
        lo = fmaxf(lo, a); hi = fminf(hi, b);
    }
    rs = sf_f2i(ceilf(lo - 0.02f)) - r0;
    re = sf_f2i(floorf(hi + 0.02f)) - r0 + 1;
    rs = rs < 0 ? 0 : rs;
    re = re > H ? H : re;
}

// One row of one detector column against one voxel column: the two shares and the slot of the lower one.
// Returns false when the ray misses the column's in-plane cell.  Positions are formed in double and reduced to the
// distance from the cell's faces before they become floats, so that those distances carry an absolute error of 1e-7 of a
// voxel whatever the lever arm; that keeps the shares good to 1e-6 on average although they are divided by m and mz.
template <int ZC>
SF_HD bool md_bp_row(const MdBpColumn &C, const MdBpPixel &p, int &slot, float &w_low, float &w_high)
{
    const float y0 = (float)fma(C.ln, p.m, C.bq);                // minor position at X = n, relative to the cell
    // (clamping is monotone: the clamped crossing times of the cell's two faces, then their order; the clamp rides on
    // the multiplication)
    const float ta = sf_clamp(-y0 * p.inv_m, 0.0f, 1.0f), tb = sf_clamp((1.0f - y0) * p.inv_m, 0.0f, 1.0f);
    const float t0 = fminf(ta, tb), t1 = fmaxf(ta, tb);
    const float dt = t1 - t0;
    if (!(dt > 0.0f)) return false;
    const double zin = fma(C.ln, p.mz, C.bz);                    // Z at X = n in slots, plus MD_BP_ZBIAS (positive)
#if defined(__HIP_DEVICE_COMPILE__)
    const float fz = (float)__builtin_amdgcn_fract(zin);
    const int kz = (int)zin - (int)MD_BP_ZBIAS;                  // (the device's conversion saturates; the slot is clamped below)
#else
    const float fz = (float)(zin - floor(zin));
    const int kz = (int)fmin(fmax(zin, 0.0), 2.0 * MD_BP_ZBIAS) - (int)MD_BP_ZBIAS;
#endif
    const float lo = fmaf(p.inv_mz >= 0.0f ? t0 : t1, (float)p.mz, fz);      // lower end of the piece, relative to cell kz
    const float kl = floorf(lo);
    const int s = kz + (int)kl;
    slot = s < 0 ? 0 : (s > ZC + 2 ? ZC + 2 : s);
    const float wl = fminf((1.0f - (lo - kl)) * fabsf(p.inv_mz), dt);
    w_low = wl * p.wy;
    w_high = (dt - wl) * p.wy;
    return true;
}

#if defined(__HIPCC__) && !defined(SF_NO_KERNELS)

template <int ZC, int PW, int PH>
__global__ __launch_bounds__(256) void md_backproject_tiled(SfGeom g, const MdBpView *__restrict__ views,
                                                            const float *__restrict__ sino, float *__restrict__ vol, int tiles_x)
{
    constexpr int PS = PW + 1;                     // odd row stride: the lanes of a wave sit in a few adjacent rows and columns
    constexpr int NSLOT = ZC + 4;                  // slot s holds voxel k0 + s - 2; slots 0, 1, ZC+2, ZC+3 are dumps
    constexpr int RSTEP = 256 / PW, NSTAGE = (PH * PW + 255) / 256;
    __shared__ double l_m[PH * PS], l_mz[PH * PS];
    __shared__ float l_wy[PH * PS], l_inv_m[PH * PS], l_inv_mz[PH * PS];
    __shared__ float sums[NSLOT * 256];

    sino += (size_t)blockIdx.z * g.nviews * g.nrows * g.ncols;
    vol += (size_t)blockIdx.z * g.nx * g.ny * g.nz;
    const int tid = threadIdx.x;
    const int ti = tid & (BP_T - 1), tj = tid >> 4;
    const int tx = blockIdx.x % tiles_x, ty = blockIdx.x / tiles_x;
    const int i0 = tx * BP_T, j0 = ty * BP_T;
    const int k0 = blockIdx.y * ZC;
    const int i = i0 + ti, j = j0 + tj;
    const int ic = i < g.nx ? i : g.nx - 1, jc = j < g.ny ? j : g.ny - 1;   // out-of-volume threads shadow the edge
    const int sc = tid & (PW - 1), sr = tid / PW;
    const size_t view_stride = (size_t)g.nrows * g.ncols;

#pragma unroll
    for (int s = 0; s < NSLOT; ++s) sums[s * 256 + tid] = 0.0f;

    float stage[NSTAGE];
    SfWindow win;
    auto load_view = [&](int a) {           // this thread's share of the raw samples of view a's window, into registers
        win = md_bp_window(g, views[a], i0, j0, k0, ZC);
        const int c = win.c0 + sc;
        const bool cin = (unsigned)c < (unsigned)g.ncols;
        const char *__restrict__ yb = reinterpret_cast<const char *>(sino + (size_t)a * view_stride);
        unsigned off = ((unsigned)(win.r0 + sr) * (unsigned)g.ncols + (unsigned)(cin ? c : 0)) * 4u;
        const unsigned step = (unsigned)RSTEP * (unsigned)g.ncols * 4u;
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s) {
            const int r = win.r0 + sr + RSTEP * s;
            const bool in = cin && (unsigned)r < (unsigned)g.nrows && (sr + RSTEP * s) < win.need_h;
            stage[s] = in ? *reinterpret_cast<const float *>(yb + off) : 0.0f;
            off += step;
        }
    };
    auto store_view = [&](int a) {          // the slopes of every sample's ray
        const MdBpView &V = views[a];
        const bool xmajor = md_bp_tile_xmajor(g, V, i0, j0);
        const int c = win.c0 + sc;
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s) {
            const int row = sr + RSTEP * s;
            if (row < PH && row < win.need_h) {           // rows past the window's need are never read
                const MdBpPixel p = md_bp_pixel(md_bp_slopes(g, V, xmajor, win.r0 + row, c), stage[s]);
                const int o = row * PS + sc;
                l_m[o] = p.m; l_mz[o] = p.mz; l_wy[o] = p.wy; l_inv_m[o] = p.inv_m; l_inv_mz[o] = p.inv_mz;
            }
        }
    };

    load_view(0);
    store_view(0);
    SfWindow cur = win;
    __syncthreads();

    for (int a = 0; a < g.nviews; ++a) {
        if (a + 1 < g.nviews) load_view(a + 1);        // global loads in flight during the gather

        const MdBpView &V = views[a];
        const bool xmajor = md_bp_tile_xmajor(g, V, i0, j0);
        const MdBpColumn C = md_bp_column<ZC>(g, V, xmajor, ic, jc, k0);
        const int H = cur.need_h < PH ? cur.need_h : PH;
        // (the loop runs over the window's columns at most, whatever the shadow's extent came out as)
        const int cbeg = C.cfirst > cur.c0 ? C.cfirst : cur.c0, cend = C.clast < cur.c0 + PW - 1 ? C.clast : cur.c0 + PW - 1;
        for (int c = cbeg; c <= cend; ++c) {
            const int wc = c - cur.c0;
            if (c < 0 || c >= g.ncols) continue;
            int rs, re;
            md_bp_rows(C, c, cur.r0, H, rs, re);
            for (int row = rs; row < re; ++row) {
                const int o = row * PS + wc;
                const MdBpPixel p = {l_m[o], l_mz[o], l_wy[o], l_inv_m[o], l_inv_mz[o]};
                int slot;
                float w_low, w_high;
                if (!md_bp_row<ZC>(C, p, slot, w_low, w_high)) continue;
                float *__restrict__ cell = sums + (slot * 256 + tid);
                // plain read-add-write: the slot has no other writer, and a wave's LDS accesses retire in order
                cell[0] += w_low;
                cell[256] += w_high;
            }
        }

        __syncthreads();                               // every thread is done with this view's window
        if (a + 1 < g.nviews) {
            store_view(a + 1);
            cur = win;
        }
        __syncthreads();
    }

    if (i < g.nx && j < g.ny) {
#pragma unroll
        for (int kk = 0; kk < ZC; ++kk)
            if (k0 + kk < g.nz) vol[((size_t)(k0 + kk) * g.ny + j) * g.nx + i] = sums[(kk + 2) * 256 + tid];
    }
}

#endif
