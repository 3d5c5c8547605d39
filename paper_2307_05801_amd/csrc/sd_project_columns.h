// Forward projection (A) of the Siddon model: ray-driven gather, one wavefront per detector column.
//
// Uses the z-fastest padded scratch copy of one slab of the volume, as the footprint kernel does (sf_project_columns.h:
// slabs across x serve the rays that advance fastest along x, slabs across y the others; every ray adds the slab's share
// to its sample, the first slab of its kind overwrites), plus one all-zero column at the copy's end that stands in for
// every in-plane cell outside the volume.
//
// Work split.  One 64-lane wavefront owns one detector column of one view and a band of RG * 64 detector rows: lane l
// owns rows band0 + 64 g + l, g < RG.  All those rays share their in-plane line, so which voxel columns they cross in
// a slab, and where inside the slab they change from one to the next, is wave-uniform: 64 slabs at a time, lane n
// works that out for slab n, and the wave then walks the slabs, broadcasting the few numbers through v_readlane.
// What differs between the lanes is the axial position: each lane follows its own Z through the slab and splits the
// slab's piece(s) between the two axial cells it can touch (the kernel is only chosen when no ray crosses more than
// one z-face per slab).  A workgroup is SD_WAVES adjacent columns of one view, which share voxel columns in L1.
#pragma once

#include "sd_ray.h"
#include "sf_project_columns.h"

// ---- the axial part of a slab, shared by the kernel and by the host-side re-enactment of its arithmetic ---------------

// Per ray (lane and row group): the row's v, the constant of its lower-Z map, 1 / |dZ per slab|, and the sign of dZ.
struct SdAxial {
    double vr, zadj;
    float inv_amz;
    bool inc;
};

SF_HD SdAxial sd_axial(const SfGeom &g, const SdRayCol &R, int r)
{
    SdAxial A;
    A.vr = sd_row_v(g, r);
    const double mz = A.vr * R.dh;
    A.zadj = g.zk0d + (double)FP_PAD + fmin(mz, 0.0);     // Z of the lower end of the slab's piece, plus the copy's pad
    const float amz = fabsf((float)mz);
    A.inv_amz = amz > 1e-30f ? 1.0f / amz : 1e30f;
    A.inc = mz >= 0.0;
    return A;
}

// Lower axial cell of the slab's piece as an index into the padded z-column (clamped: far outside the column the ray
// reads the zero pads), and the share of the slab spent in that cell.  zlo: Z of the piece's lower end, plus the pad.
SF_HD void sd_axial_cell(double zlo, float inv_amz, int kmax, int &kf, float &tlow)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const float fr = (float)__builtin_amdgcn_fract(zlo);
    kf = (int)zlo;                                       // the conversion saturates
    asm("v_med3_i32 %0, %1, 0, %2" : "=v"(kf) : "v"(kf), "s"(kmax));
#else
    const float fr = (float)(zlo - floor(zlo));
    kf = (int)fmin(fmax(zlo, 0.0), (double)kmax);
#endif
    tlow = fminf((1.0f - fr) * inv_amz, 1.0f);
}

// The same for a ray of the circular scanners.  h: h(X) at the slab's entry face.
SF_HD void sd_axial_place(const SdAxial &A, double h, int kmax, int &kf, float &tlow)
{
    sd_axial_cell(fma(A.vr, h, A.zadj), A.inv_amz, kmax, kf, tlow);
}

// A slab whose piece stays in one in-plane cell: xa points at the lower axial cell of that cell's z-column.
SF_HD float sd_gather_one(const float *__restrict__ xa, float tlow, float acc)
{
    return fmaf(tlow, xa[0], fmaf(1.0f - tlow, xa[1], acc));
}

// A slab whose piece changes from in-plane cell a to b at tau = f (omf = 1 - f): rising rays are in the lower axial cell
// first (while still in cell a), falling rays last.
SF_HD float sd_gather_two(const float *__restrict__ xa, const float *__restrict__ xb, bool inc, float f, float omf, float tlow, float acc)
{
    const float p = fminf(inc ? f : omf, tlow), q = tlow - p;
    const float a_low = inc ? p : q, b_low = inc ? q : p;
    float t = acc;
    t = fmaf(a_low, xa[0], t);
    t = fmaf(f - a_low, xa[1], t);
    t = fmaf(b_low, xb[0], t);
    return fmaf(omf - b_low, xb[1], t);
}

#if defined(__HIPCC__) && !defined(SF_NO_KERNELS)

// MOD: modular geometry with upright modules: the wave's view brings its own parameter block geoms[a] (the scene
// translated so that the view is a circular cone-beam view; gk holds the sizes, which all views share).
template <int RG, int SD_WAVES, bool MOD>
__global__ __launch_bounds__(SD_WAVES * 64) void sd_project_columns(SfGeom gk, const SdRayCol *__restrict__ rays,
                                                                    const float *__restrict__ volz, float *__restrict__ sino,
                                                                    int nzp, size_t item_stride, unsigned zero_col, int col_tiles,
                                                                    int bands, int vb, int tb, int views_pad,
                                                                    int tiles_per_xcd_pad, SfSlab slab,
                                                                    const SfGeom *__restrict__ geoms)
{
    // blockIdx.y: item of a batch (its scratch copy and its sinogram)
    volz += (size_t)blockIdx.y * item_stride;
    sino += (size_t)blockIdx.y * gk.nviews * gk.nrows * gk.ncols;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Block -> (view, band, column tile), in the XCD-aware order of the footprint kernel: index = 8 s + xcd, and
    // within an XCD's sequence s the view runs fastest inside a block of VB views, then TB tiles, then blocks of views.
    int ct, band, a;
    {
        const int xcd = blockIdx.x & 7, sq = blockIdx.x >> 3;
        const int per_chunk = tb * views_pad;
        const int chunk = sq / per_chunk, r = sq - chunk * per_chunk;
        const int vblk = r / (tb * vb), r2 = r - vblk * (tb * vb);
        const int tloc = r2 / vb, v_in = r2 - tloc * vb;
        const int tchunks = tiles_per_xcd_pad / tb;
        band = chunk / tchunks;
        ct = ((chunk - band * tchunks) * tb + tloc) * 8 + xcd;
        a = vblk * vb + v_in;
        if (ct >= col_tiles || a >= gk.nviews || band >= bands) return;   // padding blocks (no barrier follows)
    }
    const int c = ct * SD_WAVES + wave;
    if (c >= gk.ncols) return;
    const SfGeom &g = MOD ? geoms[a] : gk;
    const int band0 = band * (RG * 64);

    const SdRayCol R = rays[(size_t)a * g.ncols + c];
    if (R.xmajor != slab.xmajor) return;             // this column's rays read the other kind of slab
    const int n_major = slab.n1;
    const int n_minor = R.xmajor ? g.ny : g.nx;
    const int kmax = nzp - 2;

    SdAxial A[RG];
    float acc[RG];
#pragma unroll
    for (int gq = 0; gq < RG; ++gq) {
        A[gq] = sd_axial(g, R, band0 + 64 * gq + lane);
        acc[gq] = 0.0f;
    }

    for (int nb = slab.n0; nb < n_major; nb += 64) {
        // ---- lane-parallel: the in-plane part of slab nb + lane
        const int n = nb + lane;
        const SdSplit s = sd_slab_split(R, n);
        const bool in_n = n < n_major;
        const bool a_ok = in_n && s.qa >= 0 && s.qa < n_minor;
        const bool b_ok = in_n && s.qa != s.qb && s.qb >= 0 && s.qb < n_minor;
        const unsigned base_a = a_ok ? sf_slab_column(slab, g.nx, R.xmajor ? n : s.qa, R.xmajor ? s.qa : n) * (unsigned)nzp : zero_col;
        const unsigned base_b = b_ok ? sf_slab_column(slab, g.nx, R.xmajor ? n : s.qb, R.xmajor ? s.qb : n) * (unsigned)nzp : zero_col;
        const double h = fma((double)n, R.dh, R.h0);
        const int h_lo = __double2loint(h), h_hi = __double2hiint(h);
        const float f = s.f, omf = 1.0f - s.f;
        const unsigned long long cross = __ballot(in_n && s.qa != s.qb);
        const int count = n_major - nb < 64 ? n_major - nb : 64;

        // ---- wave-uniform walk over the slabs
        for (int e = 0; e < count; ++e) {
            const double s_h = __hiloint2double(__builtin_amdgcn_readlane(h_hi, e), __builtin_amdgcn_readlane(h_lo, e));
            const float s_f = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, f), e));
            const float *__restrict__ col_a = volz + (unsigned)__builtin_amdgcn_readlane((int)base_a, e);
            if ((cross >> e) & 1ull) {
                const float s_omf = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, omf), e));
                const float *__restrict__ col_b = volz + (unsigned)__builtin_amdgcn_readlane((int)base_b, e);
#pragma unroll
                for (int gq = 0; gq < RG; ++gq) {
                    int kf;
                    float tlow;
                    sd_axial_place(A[gq], s_h, kmax, kf, tlow);
                    acc[gq] = sd_gather_two(col_a + kf, col_b + kf, A[gq].inc, s_f, s_omf, tlow, acc[gq]);
                }
            } else {
#pragma unroll
                for (int gq = 0; gq < RG; ++gq) {
                    int kf;
                    float tlow;
                    sd_axial_place(A[gq], s_h, kmax, kf, tlow);
                    acc[gq] = sd_gather_one(col_a + kf, tlow, acc[gq]);
                }
            }
        }
    }

    float *__restrict__ ya = sino + (size_t)a * g.nrows * g.ncols + c;
#pragma unroll
    for (int gq = 0; gq < RG; ++gq) {
        const int r = band0 + 64 * gq + lane;
        if (r < g.nrows) {
            const float part = sd_ray_length(R, A[gq].vr) * acc[gq];
            ya[(size_t)r * g.ncols] = slab.first ? part : ya[(size_t)r * g.ncols] + part;
        }
    }
}

#endif
