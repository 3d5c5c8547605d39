// Forward projection (A) of the Siddon model on tilted modules of the modular geometry ("CT Projection Models and
// Geometries": sources and detectors at any position and orientation): ray-driven gather, one ray per lane.
//
// Same slab formulation, same z-fastest scratch copy of one slab of the volume and same launch order as the circular
// kernel (sd_project_columns.h), but nothing is shared between the rays of a detector column any more: a tilted
// module's column does not lie in a vertical plane, so every ray has its own in-plane line.  A wavefront still owns one
// detector column of one view and RG * 64 of its rows, because those rays run side by side through the volume: at any
// slab they sit in the same or in neighbouring voxel columns and their axial cells are consecutive, which is what
// the z-fastest copy is laid out for.  Each lane derives its ray's constants from the view's pose once, in double
// (minor(X) = m X + b with |m| <= 1 along the in-plane axis the ray advances fastest on, Z(X) = mz X + bz), and then
// walks the slabs of the launch's kind: the in-plane split of the slab (sd_slab_split), the lower axial cell and the
// share of the slab spent in it, four gathers.  Rays whose fastest in-plane axis is the other one sit the launch out.
//
// Chosen on the host only if no ray crosses more than one z-face per slab (|mz| <= 1) and every source keeps more than
// a voxel's distance from the volume's box (then a slab that holds the source contributes nothing and is skipped).
#pragma once

#include "md_siddon.h"
#include "sd_project_columns.h"

// A ray of a tilted module in the slab formulation of sd_ray.h.
struct MdSlabRay {
    SdRayCol R;          // m, b, inv_m, xmajor as for the circular scanners; h0 = Z at X = 0, dh = mz (so v_r = 1, zk0 = 0)
    double xs;           // major index coordinate of the source
    float len;           // mm of ray per unit of X
    int n_lo, n_hi;      // slabs that lie wholly in front of the source: n_lo <= n <= n_hi
};

SF_HD MdSlabRay md_slab_ray(const SfGeom &g, const MdPose &P, int r, int c)
{
    MdSlabRay M;
    const double u = ((double)c - g.col_offd) * g.pu_d, v = fma((double)r, g.pvd, g.v0d);
    double D[3];
    for (int a = 0; a < 3; ++a) D[a] = P.C[a] + u * P.ucol[a] + v * P.vrow[a] - P.S[a];
    const bool xmajor = fabs(D[0]) >= fabs(D[1]);
    const double dmaj = xmajor ? D[0] : D[1], dmin = xmajor ? D[1] : D[0];
    const double lo_maj = (xmajor ? g.x0d : g.y0d) - 0.5 * g.Td, lo_min = (xmajor ? g.y0d : g.x0d) - 0.5 * g.Td;
    const double smaj = xmajor ? P.S[0] : P.S[1], smin = xmajor ? P.S[1] : P.S[0];
    const double iT = 1.0 / g.Td, inv = 1.0 / dmaj;
    M.xs = (smaj - lo_maj) * iT;
    M.R.m = dmin * inv;
    M.R.b = (smin - lo_min) * iT - M.R.m * M.xs;
    M.R.dh = D[2] * inv * g.Td / g.Tzd;
    M.R.h0 = (P.S[2] - g.zlo0d) / g.Tzd - M.R.dh * M.xs;
    const double am = fabs(M.R.m);
    M.R.inv_m = am > 1e-30 ? (float)(1.0 / M.R.m) : 1e30f;
    M.R.lxy = 0.0f; M.R.vscale = 0.0f;
    M.R.xmajor = xmajor ? 1 : 0;
    M.len = (float)(g.Td * sqrt(D[0] * D[0] + D[1] * D[1] + D[2] * D[2]) * fabs(inv));
    // towards larger X the slabs from ceil(xs) on, towards smaller X those up to floor(xs) - 1 (bounds kept within int)
    const double far = 1073741824.0;
    const double xc = fmin(fmax(M.xs, -far), far);
    const bool forward = dmaj > 0.0;
    M.n_lo = forward ? (int)ceil(xc) : -1073741824;
    M.n_hi = forward ? 1073741824 : (int)floor(xc) - 1;
    return M;
}

// Slab n lies wholly in front of the source.
SF_HD bool md_slab_in_front(const MdSlabRay &M, int n) { return n >= M.n_lo && n <= M.n_hi; }

// Per-ray constants of the axial split.
struct MdAxial {
    double zadj;         // Z at X = 0 of the lower end of a slab's piece, plus the pad of the scratch copy's z-columns
    float inv_amz;       // 1 / |dZ per slab|
    bool inc;            // Z rises with X
};

SF_HD MdAxial md_axial(const MdSlabRay &M)
{
    MdAxial A;
    const double mz = M.R.dh;
    A.zadj = M.R.h0 + (double)FP_PAD + fmin(mz, 0.0);
    const float amz = fabsf((float)mz);
    A.inv_amz = amz > 1e-30f ? 1.0f / amz : 1e30f;
    A.inc = mz >= 0.0;
    return A;
}

// One slab's contribution to a ray's sum.  volz: the z-fastest copy of the slab (columns of nzp floats; column
// zero_col / nzp is all zero); live: the ray reads this kind of slab.  Returns acc plus the slab's share, in units of X.
SF_HD float md_slab_step(const SfGeom &g, const MdSlabRay &M, const MdAxial &A, int n, const SfSlab &slab,
                         const float *__restrict__ volz, int nzp, unsigned zero_col, bool live, float acc)
{
    const int n_minor = slab.xmajor ? g.ny : g.nx;
    const SdSplit s = sd_slab_split(M.R, n);
    live = live && md_slab_in_front(M, n);
    const bool a_ok = live && s.qa >= 0 && s.qa < n_minor;
    const bool b_ok = live && s.qa != s.qb && s.qb >= 0 && s.qb < n_minor;
    const unsigned base_a = a_ok ? sf_slab_column(slab, g.nx, slab.xmajor ? n : s.qa, slab.xmajor ? s.qa : n) * (unsigned)nzp : zero_col;
    const unsigned base_b = b_ok ? sf_slab_column(slab, g.nx, slab.xmajor ? n : s.qb, slab.xmajor ? s.qb : n) * (unsigned)nzp : zero_col;
    int kf;
    float tlow;
    sd_axial_cell(fma((double)n, M.R.dh, A.zadj), A.inv_amz, nzp - 2, kf, tlow);
    // (a slab without a crossing has f = 1 and reads the zero column for cell b: the same four terms serve both)
    return sd_gather_two(volz + base_a + (unsigned)kf, volz + base_b + (unsigned)kf, A.inc, s.f, 1.0f - s.f, tlow, acc);
}

#if defined(__HIPCC__) && !defined(SF_NO_KERNELS)

template <int RG, int SD_WAVES>
__global__ __launch_bounds__(SD_WAVES * 64) void md_project_columns(SfGeom g, const MdPose *__restrict__ poses,
                                                                    const float *__restrict__ volz, float *__restrict__ sino,
                                                                    int nzp, size_t item_stride, unsigned zero_col, int col_tiles,
                                                                    int bands, int vb, int tb, int views_pad,
                                                                    int tiles_per_xcd_pad, SfSlab slab)
{
    volz += (size_t)blockIdx.y * item_stride;
    sino += (size_t)blockIdx.y * g.nviews * g.nrows * g.ncols;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int ct, band, a;
    {   // block -> (view, band, column tile) in the XCD-aware order of sd_project_columns
        const int xcd = blockIdx.x & 7, sq = blockIdx.x >> 3;
        const int per_chunk = tb * views_pad;
        const int chunk = sq / per_chunk, r = sq - chunk * per_chunk;
        const int vblk = r / (tb * vb), r2 = r - vblk * (tb * vb);
        const int tloc = r2 / vb, v_in = r2 - tloc * vb;
        const int tchunks = tiles_per_xcd_pad / tb;
        band = chunk / tchunks;
        ct = ((chunk - band * tchunks) * tb + tloc) * 8 + xcd;
        a = vblk * vb + v_in;
        if (ct >= col_tiles || a >= g.nviews || band >= bands) return;
    }
    const int c = ct * SD_WAVES + wave;
    if (c >= g.ncols) return;
    const int band0 = band * (RG * 64);
    const MdPose P = poses[a];

    MdSlabRay M[RG];
    MdAxial A[RG];
    float acc[RG];
    bool mine[RG];
    bool any = false;
#pragma unroll
    for (int gq = 0; gq < RG; ++gq) {
        const int r = band0 + 64 * gq + lane;
        M[gq] = md_slab_ray(g, P, r < g.nrows ? r : g.nrows - 1, c);
        A[gq] = md_axial(M[gq]);
        mine[gq] = r < g.nrows && M[gq].R.xmajor == slab.xmajor;
        acc[gq] = 0.0f;
        any = any || mine[gq];
    }
    if (__ballot(any) == 0ull) return;               // no ray of this wave reads this kind of slab

    for (int n = slab.n0; n < slab.n1; ++n) {
#pragma unroll
        for (int gq = 0; gq < RG; ++gq) acc[gq] = md_slab_step(g, M[gq], A[gq], n, slab, volz, nzp, zero_col, mine[gq], acc[gq]);
    }

    float *__restrict__ ya = sino + (size_t)a * g.nrows * g.ncols + c;
#pragma unroll
    for (int gq = 0; gq < RG; ++gq) {
        const int r = band0 + 64 * gq + lane;
        if (mine[gq]) {
            const float part = M[gq].len * acc[gq];
            ya[(size_t)r * g.ncols] = slab.first ? part : ya[(size_t)r * g.ncols] + part;
        }
    }
}

#endif
