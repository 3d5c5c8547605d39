// Tiled back projection (A^T) of the Siddon model: voxel-driven in the plane, row-driven along z, no global atomics,
// bitwise reproducible.
//
// A workgroup of 256 threads owns a 16 x 16 tile of voxel columns and ZC voxels along z; a thread owns one column of
// ZC voxels.  Per view the workgroup stages the detector window its tile can be hit from into LDS, every sample
// already multiplied by its ray's length per slab, double-buffered as in the footprint kernel.  A thread then finds
// the (few) detector columns whose centre ray crosses its in-plane square, and for each the piece [t0, t1] of the
// ray's slab parameter that lies inside the square (the same split function the forward kernel uses).  Along z the
// roles are turned round: instead of asking, for each voxel, which rows hit it, the thread walks the rows of the
// window; each row's piece lies in at most two axial cells (the kernel is only chosen when
// no ray crosses more than one z-face per slab) and adds its two shares to those cells.  The ZC sums of a thread live
// in LDS (slot-major, so the 64 lanes of a wave never collide on a bank whatever cells they address), which makes the
// data-dependent cell index cheap; each slot has exactly one writer and is updated by a plain read-add-write, so the
// result does not depend on scheduling.  Two dump slots below and above the chunk take the shares that belong to
// voxels of neighbouring chunks.
#pragma once

#include "sd_ray.h"
#include "sf_backproject_tiled.h"

// Window of the detector that the voxels of one (view, tile, z-chunk) can be hit from: pixel centres inside the
// projection of the tile's box.  hx: half extent of the tile INCLUDING the outer half voxels (mm).
SF_HD SfWindow sd_bp_window(const SfGeom &g, const SfView &v, float xc, float yc, float hx, float z0, float z1)
{
    SfWindow w;
    const float tc = fmaf(yc, v.c, -xc * v.s);
    const float rho = hx * (fabsf(v.c) + fabsf(v.s));
    const float tlo = tc - rho, thi = tc + rho;
    float ilo = 1.0f, ihi = 1.0f;       // smallest / largest 1/den over the tile
    float xi_lo, xi_hi;
    if (g.type == SF_CONE_CURVED) {
        sf_curved_tile_bounds(g, v, xc, yc, hx, xi_lo, xi_hi, ilo, ihi);
    } else {
        if (g.type != SF_PARALLEL) {
            const float lc = fmaf(xc, v.c, yc * v.s);
            ilo = sf_rcp(g.sod - lc + rho);
            ihi = sf_rcp(fmaxf(g.sod - lc - rho, 1e-6f * g.sod));   // padding voxels of an edge tile may reach the source plane
        }
        xi_lo = fmaf(g.ku * tlo, tlo >= 0.0f ? ilo : ihi, g.col_off);
        xi_hi = fmaf(g.ku * thi, thi >= 0.0f ? ihi : ilo, g.col_off);
    }
    const float kv = (float)g.kvd, row_off = (float)g.row_offd;
    const float eta_lo = fmaf(kv * z0, z0 >= 0.0f ? ilo : ihi, row_off);
    const float eta_hi = fmaf(kv * z1, z1 >= 0.0f ? ihi : ilo, row_off);
    // pixel c has its centre at xi = c; row r at eta = r + 1/2.  A margin of 0.02 pixels for float rounding.
    w.c0 = sf_f2i(ceilf(xi_lo - 0.02f));
    w.r0 = sf_f2i(ceilf(eta_lo - 0.52f));
    w.need_w = sf_f2i(floorf(xi_hi + 0.02f)) - w.c0 + 1;
    w.need_h = sf_f2i(floorf(eta_hi - 0.48f)) - w.r0 + 1;
    return w;
}

#if defined(__HIPCC__) && !defined(SF_NO_KERNELS)

// Staging, first half: fetch this thread's share of the window of one view into registers.
template <int PW, int PH, int NSTAGE>
__device__ __forceinline__ void sd_load_view(const SfGeom &g, const SfView v, const float *__restrict__ ya, float xc, float yc,
                                             float hx, float z0, float z1, int sc, int sr, SfWindow &w, float (&stage)[NSTAGE])
{
    constexpr int RSTEP = 256 / PW;
    w = sd_bp_window(g, v, xc, yc, hx, z0, z1);
    const int c = w.c0 + sc;
    const bool cin = (unsigned)c < (unsigned)g.ncols;
    // 32-bit byte offsets from the view's first element (a view has fewer than 2^30 pixels where this kernel is chosen)
    const char *__restrict__ yb = reinterpret_cast<const char *>(ya);
    unsigned off = ((unsigned)(w.r0 + sr) * (unsigned)g.ncols + (unsigned)(cin ? c : 0)) * 4u;
    const unsigned step = (unsigned)RSTEP * (unsigned)g.ncols * 4u;
#pragma unroll
    for (int s = 0; s < NSTAGE; ++s) {
        const int r = w.r0 + sr + RSTEP * s;
        // (the walk stops at row need_h: whole steps beyond it are left out, here and in sd_store_view)
        const bool in = cin && (unsigned)r < (unsigned)g.nrows && (sr + RSTEP * s) < PH && RSTEP * s < w.need_h;
        stage[s] = in ? *reinterpret_cast<const float *>(yb + off) : 0.0f;
        off += step;
    }
}

// Staging, second half: scale by the ray's length per slab and write to LDS; the first window column also writes
// 1/|v| of every window row.
template <int PW, int PH, int NSTAGE>
__device__ __forceinline__ void sd_store_view(const SfGeom &g, const SdRayCol *__restrict__ rays_a, int sc, int sr,
                                              const SfWindow &w, const float (&stage)[NSTAGE], float *__restrict__ buf,
                                              float *__restrict__ rinv)
{
    constexpr int RSTEP = 256 / PW, PS = PW + BP_ROW_PAD;
    int c = w.c0 + sc;
    c = c < 0 ? 0 : (c > g.ncols - 1 ? g.ncols - 1 : c);
    const float lxy = rays_a[c].lxy, vscale = rays_a[c].vscale;
#pragma unroll
    for (int s = 0; s < NSTAGE; ++s) {
        const int row = sr + RSTEP * s;
        if (row < PH && RSTEP * s < w.need_h) {        // the second test is uniform over the workgroup
            const float vr = (float)sd_row_v(g, w.r0 + row);
            const float t = vscale * vr;
            buf[row * PS + sc] = stage[s] * sf_sqrt(fmaf(t, t, lxy * lxy));
            if (sc == 0) {
                const float av = fabsf(vr);
                rinv[row] = av > 1e-30f ? 1.0f / av : 1e30f;
            }
        }
    }
}

// Where a workgroup's tile and z-chunk lie in the scene a view sees.
struct SdBpScene {
    float xc, yc, z0, z1;
    double zrel0;          // Z of the plane z = 0 measured in slots of this chunk
};

template <int ZC>
SF_HD SdBpScene sd_bp_scene(const SfGeom &g, int i0, int j0, int k0)
{
    SdBpScene s;
    s.z0 = (float)fma((double)k0, g.Tzd, g.zlo0d);
    s.z1 = s.z0 + (float)ZC * g.Tz;
    s.xc = (float)(g.x0d + ((double)i0 + 0.5 * (BP_T - 1)) * g.Td);
    s.yc = (float)(g.y0d + ((double)j0 + 0.5 * (BP_T - 1)) * g.Td);
    s.zrel0 = g.zk0d - (double)k0 + 2.0;
    return s;
}

// NCS: detector columns whose centre can fall inside one voxel's in-plane footprint.  MOD: modular geometry with
// upright modules, one parameter block geoms[a] per view (g holds the sizes).
constexpr double SD_BP_MAGIC = 1572864.0;        // 1.5 * 2^20
constexpr unsigned SD_BP_HI = 0x41380000u;       // its high word

template <int NCS, int ZC, int PW, int PH, bool MOD>
__global__ __launch_bounds__(256) void sd_backproject_tiled(SfGeom g, const SfView *__restrict__ views,
                                                            const SdRayCol *__restrict__ rays, const float *__restrict__ sino,
                                                            float *__restrict__ vol, int tiles_x,
                                                            const SfGeom *__restrict__ geoms)
{
    constexpr int PS = PW + BP_ROW_PAD;
    constexpr int NSLOT = ZC + 4;                  // slot s holds voxel k0 + s - 2; slots 0, 1, ZC+2, ZC+3 are dumps
    __shared__ float patch[2][PH * PS];
    __shared__ float rinv[2][PH];
    __shared__ float sums[NSLOT * 256];

    // blockIdx.z: item of a batch
    sino += (size_t)blockIdx.z * g.nviews * g.nrows * g.ncols;
    vol += (size_t)blockIdx.z * g.nx * g.ny * g.nz;
    const int tid = threadIdx.x;
    const int ti = tid & (BP_T - 1), tj = tid >> 4;
    const int tx = blockIdx.x % tiles_x, ty = blockIdx.x / tiles_x;
    const int i0 = tx * BP_T, j0 = ty * BP_T;
    const int k0 = blockIdx.y * ZC;
    const int i = i0 + ti, j = j0 + tj;
    const int ic = i < g.nx ? i : g.nx - 1, jc = j < g.ny ? j : g.ny - 1;   // out-of-volume threads shadow the edge

    const float hx = 0.5f * (float)BP_T * g.T;
    auto geom_of = [&](int a) -> const SfGeom & {
        if constexpr (MOD) return geoms[a];
        else return g;
    };
    const SdBpScene scene0 = sd_bp_scene<ZC>(geom_of(0), i0, j0, k0);

    const int sc = tid & (PW - 1), sr = tid / PW;
    constexpr int NSTAGE = (PH * PW + 255) / 256;
    const size_t view_stride = (size_t)g.nrows * g.ncols;

#pragma unroll
    for (int s = 0; s < NSLOT; ++s) sums[s * 256 + tid] = 0.0f;

    float stage[NSTAGE];
    SfWindow win, win_next;
    sd_load_view<PW, PH, NSTAGE>(geom_of(0), views[0], sino, scene0.xc, scene0.yc, hx, scene0.z0, scene0.z1, sc, sr, win, stage);
    win_next = win;
    sd_store_view<PW, PH, NSTAGE>(geom_of(0), rays, sc, sr, win, stage, patch[0], rinv[0]);
    __syncthreads();

    for (int a = 0; a < g.nviews; ++a) {
        const float *__restrict__ buf = patch[a & 1];
        const float *__restrict__ ri = rinv[a & 1];
        if (a + 1 < g.nviews) {    // global loads in flight during the gather
            const SdBpScene sn = MOD ? sd_bp_scene<ZC>(geom_of(a + 1), i0, j0, k0) : scene0;
            sd_load_view<PW, PH, NSTAGE>(geom_of(a + 1), views[a + 1], sino + (size_t)(a + 1) * view_stride, sn.xc, sn.yc, hx, sn.z0,
                                         sn.z1, sc, sr, win_next, stage);
        }
        const SfGeom &gv = geom_of(a);
        const double zrel0 = MOD ? gv.zk0d - (double)k0 + 2.0 : scene0.zrel0;

        const SfColumn f = sf_column(gv, views[a], ic, jc);
        const int cfirst = (int)ceil(f.xi + (double)f.o0 - 1e-3), clast = (int)floor(f.xi + (double)f.o3 + 1e-3);
        const SdRayCol *__restrict__ rays_a = rays + (size_t)a * g.ncols;
#pragma unroll
        for (int m = 0; m < NCS; ++m) {
            const int c = cfirst + m;
            const int wc = c - win.c0;
            if (c > clast || c < 0 || c >= g.ncols || wc < 0 || wc >= PW) continue;
            const SdRayCol R = rays_a[c];
            const int n = R.xmajor ? ic : jc, q = R.xmajor ? jc : ic;
            const SdSplit s = sd_slab_split(R, n);
            float t0, t1;
            if (q == s.qa) { t0 = 0.0f; t1 = s.f; }
            else if (q == s.qb) { t0 = s.f; t1 = 1.0f; }
            else continue;
            const float dt = t1 - t0;
            if (!(dt > 0.0f)) continue;
            const double ha = fma((double)n + (double)t0, R.dh, R.h0), hb = fma((double)n + (double)t1, R.dh, R.h0);
            // Every row of the window is walked (rows that cannot reach the chunk fall into the dump slots), in two
            // wave-uniform runs: rows below the source plane (v < 0), whose lower end in Z is where h is larger, and
            // rows at or above it.  Within a run the lower end advances by pv * h per row; it is carried as a 32.32
            // fixed-point number whose upper word is the slot and whose lower word the fraction.
            const double hmin = fmin(ha, hb), hmax = fmax(ha, hb);
            const float dh = (float)(hmax - hmin);
            // dt over the piece's rise in Z is scale / |v_r| / 2^32 times the fixed-point distance to the next z-face
            const float scale = dt * (dh > 1e-30f ? 1.0f / dh : 1e30f) * 2.3283064365386963e-10f;
            const int H = win.need_h < PH ? win.need_h : PH;
            int rz = (int)ceil(-gv.v0d / gv.pvd) - win.r0;       // first window row with v >= 0
            rz = rz < 0 ? 0 : (rz > H ? H : rz);
#pragma unroll
            for (int run = 0; run < 2; ++run) {
                const int rs = run ? rz : 0, re = run ? H : rz;
                if (rs >= re) continue;
                const double h = run ? hmin : hmax;
                // The fixed-point number lives in a double: with 1.5 * 2^20 added, a double's unit in the last place is
                // 2^-32, so its low word is the fraction and its high word SD_BP_HI plus the slot, and advancing it is one
                // double addition (exact: both terms are multiples of 2^-32) instead of a 64-bit integer add in two halves.
                double q = floor(fma(sd_row_v(gv, win.r0 + rs), h, zrel0) * 4294967296.0) * 2.3283064365386963e-10 + SD_BP_MAGIC;
                const double dq = rint(gv.pvd * h * 4294967296.0) * 2.3283064365386963e-10;
                unsigned ofs = (unsigned)(rs * PS + wc);
                for (int row = rs; row < re; ++row) {
                    const unsigned long long qbits = __builtin_bit_cast(unsigned long long, q);
                    int slot = (int)((unsigned)(qbits >> 32) - SD_BP_HI);
                    slot = slot < 0 ? 0 : (slot > ZC + 2 ? ZC + 2 : slot);
                    const float up = (float)(~(unsigned)qbits) + 1.0f;  // (1 - fraction) * 2^32, at least 1
                    const float wl = fminf(up * (scale * ri[row]), dt);
                    const float y = buf[ofs];
                    float *__restrict__ cell = sums + (slot * 256 + tid);
                    // plain read-add-write: the slot has no other writer, and a wave's LDS accesses retire in order
                    // (the LDS float atomic measured 7x slower than this on the 512^3 case)
                    cell[0] += wl * y;
                    cell[256] += (dt - wl) * y;
                    q += dq;
                    ofs += PS;
                }
            }
        }

        if (a + 1 < g.nviews)
            sd_store_view<PW, PH, NSTAGE>(geom_of(a + 1), rays + (size_t)(a + 1) * g.ncols, sc, sr, win_next, stage,
                                          patch[(a + 1) & 1], rinv[(a + 1) & 1]);
        win = win_next;
        __syncthreads();
    }

    if (i < g.nx && j < g.ny) {
#pragma unroll
        for (int kk = 0; kk < ZC; ++kk)
            if (k0 + kk < g.nz) vol[((size_t)(k0 + kk) * g.ny + j) * g.nx + i] = sums[(kk + 2) * 256 + tid];
    }
}

#endif
