// General-purpose (any footprint size, any fan angle) per-thread bodies of the projector pair.
//
// These are the plain loop nests: one thread owns a few outputs and walks every contribution to them,
// reading the other array straight from global memory.  They accept every geometry the library
// validates and serve as the fallback when a geometry exceeds the static limits of the tiled kernels.
// The bodies are host/device functions so that the same source can be stepped on a CPU when a kernel
// has to be debugged.
#pragma once

#include "sf_footprint.h"

// Back projection: voxels (i, j, k0 .. k0+ZC-1) of one batch item; acc must be zero-initialised.
// geoms: null, or one parameter block per view (modular geometry: every view is a cone-beam view of its own); the
// sizes in `g0` hold for all views.
template <int ZC>
SF_HD void sf_backproject_column_chunk(const SfGeom &g0, const SfView *__restrict__ views,
                                       const float *__restrict__ sino, int i, int j, int k0, float acc[ZC],
                                       const SfGeom *__restrict__ geoms = nullptr)
{
    const size_t view_stride = (size_t)g0.nrows * g0.ncols;
    for (int a = 0; a < g0.nviews; ++a) {
        const SfGeom &g = geoms ? geoms[a] : g0;
        const double zlo_k0 = fma((double)k0, g.Tzd, g.zlo0d);
        const SfView v = views[a];
        const SfColumn f = sf_column(g, v, i, j);
        int c0, c1;
        sf_col_range(f, c0, c1);
        c0 = c0 < 0 ? 0 : c0;
        c1 = c1 > g.ncols - 1 ? g.ncols - 1 : c1;
        if (c0 > c1) continue;
        const SfRowsOfVoxels ax = sf_rows_of_voxels(g, f, zlo_k0);
        const float *__restrict__ ya = sino + (size_t)a * view_stride;
        float ulo = sf_pixel_edge(f, c0);
        for (int c = c0; c <= c1; ++c, ulo += 1.0f) {
            const float fu = sf_fu_at(f, ulo);
            if (!(fu > 0.0f)) continue;
            const SfAmpCol ac = sf_amp_col(g, v, c);
            if (g.type == SF_FAN) {
                acc[0] = fmaf(fu, sf_amp(g, v, ac, 0) * ya[c], acc[0]);
                continue;
            }
#pragma unroll
            for (int kk = 0; kk < ZC; ++kk) {
                if (k0 + kk >= g.nz) break;
                int rr0 = (int)floorf(fmaf(ax.av, (float)kk, ax.phi0));
                int rr1 = (int)floorf(fmaf(ax.av, (float)(kk + 1), ax.phi0));
                rr0 = ax.rb + rr0 < 0 ? -ax.rb : rr0;
                rr1 = ax.rb + rr1 > g.nrows - 1 ? g.nrows - 1 - ax.rb : rr1;
                float s = 0.0f;
                for (int rr = rr0; rr <= rr1; ++rr) {
                    const int r = ax.rb + rr;
                    s = fmaf(sf_fv_rows(ax, rr, kk), sf_amp(g, v, ac, r) * ya[(size_t)r * g.ncols + c], s);
                }
                acc[kk] = fmaf(fu, s, acc[kk]);
            }
        }
    }
}

// Forward projection: rays (view, rows r0 .. r0+RC-1, column c) of one batch item; returns the finished
// line integrals (amplitude applied) in out[].
template <int RC>
SF_HD void sf_project_ray_chunk(const SfGeom &g, const SfView &v, const float *__restrict__ vol, int c, int r0,
                                float out[RC])
{
    float acc[RC];
#pragma unroll
    for (int rr = 0; rr < RC; ++rr) acc[rr] = 0.0f;

    // In-plane lines through the two u-edges of the pixel, as "minor index = m * major index + b".  These only
    // bound the candidate voxels (a superset with a safety margin); the weights come from sf_column.
    const float ue[2] = {((float)c - 0.5f - g.col_off) * g.pu, ((float)c + 0.5f - g.col_off) * g.pu};
    const float uc = ((float)c - g.col_off) * g.pu;
    const float x0 = (float)g.x0d, y0 = (float)g.y0d;
    bool xmajor;
    float m[2], b[2];
    if (g.type == SF_PARALLEL) {
        xmajor = fabsf(v.c) >= fabsf(v.s);
        for (int e = 0; e < 2; ++e) {
            if (xmajor) {   // -x s + y c = u  ->  y = (u + x s)/c
                m[e] = v.s / v.c;
                b[e] = (ue[e] / v.c + x0 * m[e] - y0) / g.T;
            } else {        // x = (y c - u)/s
                m[e] = v.c / v.s;
                b[e] = (-ue[e] / v.s + y0 * m[e] - x0) / g.T;
            }
        }
    } else {
        const float sx = g.sod * v.c, sy = g.sod * v.s;
        float dxc = fmaf(-g.sdd, v.c, -uc * v.s), dyc = fmaf(-g.sdd, v.s, uc * v.c);
        if (g.type == SF_CONE_CURVED) {      // u is arc length on the cylinder: direction at the fan angle u / sdd
            float sg, cg;
            sincosf(uc / g.sdd, &sg, &cg);
            dxc = -fmaf(cg, v.c, sg * v.s); dyc = fmaf(sg, v.c, -cg * v.s);
        }
        xmajor = fabsf(dxc) >= fabsf(dyc);
        for (int e = 0; e < 2; ++e) {
            float dx = fmaf(-g.sdd, v.c, -ue[e] * v.s), dy = fmaf(-g.sdd, v.s, ue[e] * v.c);
            if (g.type == SF_CONE_CURVED) {
                float sg, cg;
                sincosf(ue[e] / g.sdd, &sg, &cg);
                dx = -fmaf(cg, v.c, sg * v.s); dy = fmaf(sg, v.c, -cg * v.s);
            }
            if (xmajor) {
                m[e] = dy / dx;
                b[e] = (sy - y0 + (x0 - sx) * m[e]) / g.T;
            } else {
                m[e] = dx / dy;
                b[e] = (sx - x0 + (y0 - sy) * m[e]) / g.T;
            }
        }
    }
    const float spread = 0.5f * fmaxf(fabsf(m[0]), fabsf(m[1])) + 2e-3f;
    const int n_major = xmajor ? g.nx : g.ny;
    const int n_minor = xmajor ? g.ny : g.nx;
    const size_t kstride = (size_t)g.nx * g.ny;

    for (int n = 0; n < n_major; ++n) {
        const float qa = fmaf(m[0], (float)n, b[0]), qb = fmaf(m[1], (float)n, b[1]);
        int q0 = (int)floorf(fminf(qa, qb) - spread + 0.5f);
        int q1 = (int)floorf(fmaxf(qa, qb) + spread + 0.5f);
        q0 = q0 < 0 ? 0 : q0;
        q1 = q1 > n_minor - 1 ? n_minor - 1 : q1;
        for (int q = q0; q <= q1; ++q) {
            const int i = xmajor ? n : q, j = xmajor ? q : n;
            const SfColumn f = sf_column(g, v, i, j);
            const float fu = sf_fu(f, c);
            if (!(fu > 0.0f)) continue;
            const float *__restrict__ col = vol + ((size_t)j * g.nx + i);
            if (g.type == SF_FAN) {
                acc[0] = fmaf(fu, col[0], acc[0]);
                continue;
            }
            const SfVoxelsOfRows ax = sf_voxels_of_rows(g, f, r0);
#pragma unroll
            for (int rr = 0; rr < RC; ++rr) {
                if (r0 + rr >= g.nrows) break;
                int kk0 = (int)floorf(fmaf(ax.step, (float)rr, ax.psi0));
                int kk1 = (int)floorf(fmaf(ax.step, (float)(rr + 1), ax.psi0));
                kk0 = ax.kb + kk0 < 0 ? -ax.kb : kk0;
                kk1 = ax.kb + kk1 > g.nz - 1 ? g.nz - 1 - ax.kb : kk1;
                float s = 0.0f;
                for (int kk = kk0; kk <= kk1; ++kk)
                    s = fmaf(sf_fv_voxels(ax, rr, kk), col[(size_t)(ax.kb + kk) * kstride], s);
                acc[rr] = fmaf(fu, s, acc[rr]);
            }
        }
    }
    const SfAmpCol ac = sf_amp_col(g, v, c);
#pragma unroll
    for (int rr = 0; rr < RC; ++rr) out[rr] = (r0 + rr < g.nrows) ? sf_amp(g, v, ac, r0 + rr) * acc[rr] : 0.0f;
}
