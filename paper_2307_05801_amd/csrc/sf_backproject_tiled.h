// Tiled back projection (A^T): voxel-driven gather, no atomics, bitwise reproducible.
//
// A workgroup of 256 threads owns a 16 x 16 tile of voxel columns and BP_ZC voxels along z; a thread
// owns one column of BP_ZC voxels and keeps their sums in registers while the workgroup walks all views.
// Per view the workgroup stages the detector window its tile can touch into LDS, already multiplied by
// the ray amplitude (so the weight left per sample is F_u * F_v), double-buffered: the loads of view
// a+1 are in flight while view a is gathered.  Everything outside the detector is staged as zero, which
// is the truncation rule for footprints that leave the detector.
//
// Static limits (checked on the host before this kernel is chosen): a voxel touches at most NC detector
// columns and NV detector rows; the window of any (view, tile, chunk) fits BP_PW x BP_PH.
#pragma once

#include "sf_footprint.h"

constexpr int BP_T = 16;        // tile edge in voxels (x and y)

// LDS row stride = window width + BP_ROW_PAD floats.  Lanes of a wave read windows that differ by a row or two
// and a few columns; a stride of 12 mod 32 banks measured fewest conflicts (1: 52.5 ms, 12: 48.3 ms on 512^3).
#ifndef BP_ROW_PAD
#define BP_ROW_PAD 12
#endif

// Shapes the kernel is instantiated for: voxels along z per thread, staged window columns x rows.
struct SfBpShape {
    int zc, pw, ph;
};
// The last one keeps 64 voxels per thread for footprints up to two rows tall (its 96 rows hold what 64 voxels of up to
// about 1.3 rows each project to); it is instantiated for NV <= 3 only, shape 0 for NV == 2 only (the general gather of
// taller footprints would spill registers).
constexpr SfBpShape BP_SHAPES[] = {{64, 32, 76}, {32, 32, 44}, {32, 32, 56}, {16, 32, 44}, {16, 64, 48}, {64, 32, 96}};
constexpr int BP_NSHAPES = 6;
constexpr int BP_FIRST_SHORT_SHAPE = 1;      // first shape with fewer than 64 voxels per thread
constexpr int BP_LAST_SHORT_SHAPE = 4;       // last one
constexpr int BP_TALL_SHAPE = 5;

// Window of the detector that one (view, tile, z-chunk) can touch.  Evaluated identically on the host
// (limit check) and in the kernel; everything here is uniform over the workgroup.
struct SfWindow {
    int c0, r0;       // first staged column / row
    int need_w, need_h;
};

// Cylindrical detector: column-coordinate range [xi_lo, xi_hi] and the range [ilo, ihi] of 1 / (in-plane distance from
// the source) over the square of half extent hx around (xc, yc).  The fan angle of a convex set is extreme at a
// corner; the distance is bounded by the centre's distance -+ the half diagonal.
SF_HD void sf_curved_tile_bounds(const SfGeom &g, const SfView &v, float xc, float yc, float hx, float &xi_lo, float &xi_hi,
                                 float &ilo, float &ihi)
{
    const float tc = fmaf(yc, v.c, -xc * v.s), dc = g.sod - fmaf(xc, v.c, yc * v.s);
    const float a = hx * (v.c - v.s), b = hx * (v.c + v.s);      // corner (+hx, +hx): (dt, dl) = (a, b); (+hx, -hx): (-b, a)
    const float g0 = atan2f(tc + a, dc - b), g1 = atan2f(tc - a, dc + b);
    const float g2 = atan2f(tc - b, dc - a), g3 = atan2f(tc + b, dc + a);
    xi_lo = fmaf(g.ku, fminf(fminf(g0, g1), fminf(g2, g3)), g.col_off);
    xi_hi = fmaf(g.ku, fmaxf(fmaxf(g0, g1), fmaxf(g2, g3)), g.col_off);
    const float dist = sf_sqrt(fmaf(tc, tc, dc * dc)), rad = 1.4143f * hx;
    ilo = sf_rcp(dist + rad);
    ihi = sf_rcp(fmaxf(dist - rad, 1e-3f * dist));
}

// xc, yc: tile centre (mm); hx: half extent of the voxel centres in x and y (mm); z0, z1: lower / upper face
// of the chunk (mm); wh: half of the widest transaxial footprint (pixels); nc, nv: columns / rows a thread reads
// per voxel (starting at the first one its footprint touches).
// Cylinder: what depends on (tile, view) only, worked out once per geometry on the host: the fan angle of the tile's
// centre in double and sf_curved_tile_bounds of the tile.  Stored [tile][view].
struct SfCurvedBounds {
    double gref;
    float xi_lo, xi_hi, ilo, ihi;
};

template <int GT = -1>
SF_HD SfWindow sf_bp_window(const SfGeom &g, const SfView &v, float xc, float yc, float hx, float z0, float z1, float wh,
                            int nc, int nv, const SfCurvedBounds *pre = nullptr)
{
    SfWindow w;
    const float tc = fmaf(yc, v.c, -xc * v.s);
    const float rho = hx * (fabsf(v.c) + fabsf(v.s));
    const float tlo = tc - rho, thi = tc + rho;
    float ilo = 1.0f, ihi = 1.0f;       // smallest / largest 1/den over the tile
    float xi_lo, xi_hi;
    if (sf_is_curved<GT>(g)) {
        if (pre) {
            xi_lo = pre->xi_lo; xi_hi = pre->xi_hi; ilo = pre->ilo; ihi = pre->ihi;
        } else {
            sf_curved_tile_bounds(g, v, xc, yc, hx, xi_lo, xi_hi, ilo, ihi);
        }
    } else {
        if (g.type != SF_PARALLEL) {
            const float lc = fmaf(xc, v.c, yc * v.s);
            // a ragged edge tile's padding voxels may reach the source plane: keep the distance positive (the window then
            // comes out huge and the host rejects the kernel)
            ilo = sf_rcp(g.sod - lc + rho);
            ihi = sf_rcp(fmaxf(g.sod - lc - rho, 1e-6f * g.sod));
        }
        xi_lo = fmaf(g.ku * tlo, tlo >= 0.0f ? ilo : ihi, g.col_off);
        xi_hi = fmaf(g.ku * thi, thi >= 0.0f ? ihi : ilo, g.col_off);
    }
    const float kv = (float)g.kvd, row_off = (float)g.row_offd;
    const float eta_lo = fmaf(kv * z0, z0 >= 0.0f ? ilo : ihi, row_off);
    const float eta_hi = fmaf(kv * z1, z1 >= 0.0f ? ihi : ilo, row_off);
    w.c0 = sf_f2i(floorf(xi_lo - wh + 0.48f));
    w.r0 = sf_f2i(floorf(eta_lo - 0.02f));
    w.need_w = sf_f2i(floorf(xi_hi + 0.52f)) + nc - w.c0;    // a thread reads nc columns from its first one
    w.need_h = sf_f2i(floorf(eta_hi + 0.02f)) + nv - w.r0;   // and nv rows from the first row of each voxel
    return w;
}

#if defined(__HIPCC__) && !defined(SF_NO_KERNELS)

// Staging, first half: fetch this thread's share of the window of one view into registers.  ya points at the view.
template <int NC, int NV, int PW, int PH, int NSTAGE, int GT>
__device__ __forceinline__ void bp_load_view(const SfGeom &g, const SfView v, const float *__restrict__ ya, float xc, float yc,
                                             float hx, float z0, float z1, float wh, int sc, int sr, SfWindow &w,
                                             float (&stage)[NSTAGE], const SfCurvedBounds *pre = nullptr)
{
    constexpr int RSTEP = 256 / PW;
    w = sf_bp_window<GT>(g, v, xc, yc, hx, z0, z1, wh, NC, NV, pre);
    const int c = w.c0 + sc;
    const bool cin = (unsigned)c < (unsigned)g.ncols;
    // 32-bit byte offsets from the view's first element (a view has fewer than 2^30 pixels where this kernel is
    // chosen): one add per row instead of a 64-bit multiply; offsets of rows off the detector are never used
    const char *__restrict__ yb = reinterpret_cast<const char *>(ya);
    // (unsigned arithmetic: offsets of rows off the detector wrap around harmlessly)
    unsigned off = ((unsigned)(w.r0 + sr) * (unsigned)g.ncols + (unsigned)(cin ? c : 0)) * 4u;
    const unsigned step = (unsigned)RSTEP * (unsigned)g.ncols * 4u;
#pragma unroll
    for (int s = 0; s < NSTAGE; ++s) {
        const int r = w.r0 + sr + RSTEP * s;
        // (rows from need_h on are never read: whole steps beyond it are left out, here and in bp_store_view)
        const bool in = cin && (unsigned)r < (unsigned)g.nrows && (sr + RSTEP * s) < PH && RSTEP * s < w.need_h;
        stage[s] = in ? *reinterpret_cast<const float *>(yb + off) : 0.0f;
        off += step;
    }
}

// Staging, second half: scale by the ray amplitude and write to LDS.
template <int PW, int PH, int NSTAGE, int GT>
__device__ __forceinline__ void bp_store_view(const SfGeom &g, const SfView v, int sc, int sr, const SfWindow &w,
                                              const float (&stage)[NSTAGE], float *__restrict__ buf,
                                              const float2 *__restrict__ colcs = nullptr)
{
    constexpr int RSTEP = 256 / PW, PS = PW + BP_ROW_PAD;
    SfAmpCol ac;
    if (GT == 1 && colcs) {      // cylinder: cosine and sine of the column's fan angle from the per-column table
        int c = w.c0 + sc;
        c = c < 0 ? 0 : (c > g.ncols - 1 ? g.ncols - 1 : c);    // columns off the detector were staged as zeros
        const float2 cs = colcs[c];
        ac = sf_amp_col_curved(g, v, cs.x, cs.y);
    } else {
        ac = sf_amp_col<GT>(g, v, w.c0 + sc);
    }
    float vv = fmaf((float)(w.r0 + sr), g.pv, g.v0);      // this thread's first row; RSTEP rows further per element
    const float dv = (float)RSTEP * g.pv;
#pragma unroll
    for (int s = 0; s < NSTAGE; ++s) {
        const int row = sr + RSTEP * s;
        if (RSTEP * s < w.need_h) {        // uniform over the workgroup
            if (row < PH) buf[row * PS + sc] = stage[s] * sf_amp_at(g, v, ac, vv);
        }
        vv += dv;
    }
}

// Where a workgroup's tile and z-chunk lie in the scene a view sees (mm): tile centre, chunk faces.
struct SfBpScene {
    float xc, yc, z0, z1;
    double zlo_k0;
};

template <int BP_ZC>
SF_HD SfBpScene sf_bp_scene(const SfGeom &g, int i0, int j0, int k0)
{
    SfBpScene s;
    s.zlo_k0 = fma((double)k0, g.Tzd, g.zlo0d);
    s.z0 = (float)s.zlo_k0;
    s.z1 = s.z0 + (float)BP_ZC * g.Tz;
    s.xc = (float)(g.x0d + ((double)i0 + 0.5 * (BP_T - 1)) * g.Td);
    s.yc = (float)(g.y0d + ((double)j0 + 0.5 * (BP_T - 1)) * g.Td);
    return s;
}

// GT: 0 flat or parallel, 1 cylindrical detector, 2 modular geometry with upright modules (every view brings its own
// parameter block geoms[a]: the scene translated so that the view is a circular cone-beam view; g holds the sizes).
template <int NC, int NV, int BP_ZC, int BP_PW, int BP_PH, int GT>
__global__ __launch_bounds__(256, (GT == 1 && NV > 2 && BP_ZC > 32) ? 3 : 4) void sf_backproject_tiled(SfGeom g, const SfView *__restrict__ views,
                                                            const float *__restrict__ sino, float *__restrict__ vol,
                                                            int tiles_x, float wh, const void *__restrict__ aux)
{
    // aux: GT == 2: the per-view parameter blocks; GT == 1: cosine and sine of every detector column's fan angle
    // (ncols pairs of floats), followed by the per-(tile, view) table
    const SfGeom *__restrict__ geoms = GT == 2 ? static_cast<const SfGeom *>(aux) : nullptr;
    const float2 *__restrict__ colcs = GT == 1 ? static_cast<const float2 *>(aux) : nullptr;
    const SfCurvedBounds *__restrict__ cvt =
        GT == 1 ? reinterpret_cast<const SfCurvedBounds *>(static_cast<const float2 *>(aux) + g.ncols) + (size_t)blockIdx.x * g.nviews
                : nullptr;
    constexpr int BP_PS = BP_PW + BP_ROW_PAD;      // LDS row stride (floats)
    __shared__ float patch[2][BP_PH * BP_PS];
    // blockIdx.z: item of a batch
    sino += (size_t)blockIdx.z * g.nviews * g.nrows * g.ncols;
    vol += (size_t)blockIdx.z * g.nx * g.ny * g.nz;

    const int tid = threadIdx.x;
    const int ti = tid & (BP_T - 1), tj = tid >> 4;
    const int tx = blockIdx.x % tiles_x, ty = blockIdx.x / tiles_x;
    const int i0 = tx * BP_T, j0 = ty * BP_T;
    const int k0 = blockIdx.y * BP_ZC;
    const int i = i0 + ti, j = j0 + tj;
    const int ic = i < g.nx ? i : g.nx - 1, jc = j < g.ny ? j : g.ny - 1;   // out-of-volume threads shadow the edge

    const float hx = 0.5f * (float)(BP_T - 1) * g.T;
    auto geom_of = [&](int a) -> const SfGeom & {
        if constexpr (GT == 2) return geoms[a];
        else return g;
    };
    const SfBpScene scene0 = sf_bp_scene<BP_ZC>(geom_of(0), i0, j0, k0);

    // staging role: element e = tid + 256 s  ->  window column tid % PW, window row tid / PW + RSTEP s
    const int sc = tid & (BP_PW - 1), sr = tid / BP_PW;
    constexpr int NSTAGE = (BP_PH * BP_PW + 255) / 256;
    const size_t view_stride = (size_t)g.nrows * g.ncols;

    float acc[BP_ZC];
#pragma unroll
    for (int kk = 0; kk < BP_ZC; ++kk) acc[kk] = 0.0f;

    float stage[NSTAGE];
    SfWindow win_next;

    // tile centre in double (cylinder only)
    const double xcd = g.x0d + ((double)i0 + 0.5 * (BP_T - 1)) * g.Td, ycd = g.y0d + ((double)j0 + 0.5 * (BP_T - 1)) * g.Td;
    auto cv_pre = [&](int a) -> const SfCurvedBounds * {
        if constexpr (GT == 1) return cvt + a;
        else return nullptr;
    };

    SfWindow win;
    bp_load_view<NC, NV, BP_PW, BP_PH, NSTAGE, GT>(geom_of(0), views[0], sino, scene0.xc, scene0.yc, hx, scene0.z0, scene0.z1, wh,
                                                   sc, sr, win, stage, cv_pre(0));
    win_next = win;
    bp_store_view<BP_PW, BP_PH, NSTAGE, GT>(geom_of(0), views[0], sc, sr, win, stage, patch[0], colcs);
    __syncthreads();

    for (int a = 0; a < g.nviews; ++a) {
        const float *buf = patch[a & 1];
        double gref = 0.0;
        if constexpr (GT == 1) gref = cvt[a].gref;
        if (a + 1 < g.nviews) {    // global loads in flight during the gather
            const SfBpScene sn = GT == 2 ? sf_bp_scene<BP_ZC>(geom_of(a + 1), i0, j0, k0) : scene0;
            bp_load_view<NC, NV, BP_PW, BP_PH, NSTAGE, GT>(geom_of(a + 1), views[a + 1], sino + (size_t)(a + 1) * view_stride, sn.xc,
                                                           sn.yc, hx, sn.z0, sn.z1, wh, sc, sr, win_next, stage, cv_pre(a + 1));
        }
        const SfGeom &gv = geom_of(a);
        const double zlo_k0 = GT == 2 ? fma((double)k0, gv.Tzd, gv.zlo0d) : scene0.zlo_k0;

        const SfView v = views[a];
        SfColumn f;
        if constexpr (GT == 1)
            f = sf_column_curved_ref(gv, v, ic, jc, fma(ycd, v.cd, -xcd * v.sd), gv.sodd - fma(xcd, v.cd, ycd * v.sd), gref);
        else
            f = sf_column<GT>(gv, v, ic, jc);
        int cf, cl;
        sf_col_range(f, cf, cl);
        float fu[NC];
        {
            float e = sf_pixel_edge(f, cf);
            float g0 = sf_trap_integral(f, e);
#pragma unroll
            for (int m = 0; m < NC; ++m) {
                e += 1.0f;
                const float g1 = sf_trap_integral(f, e);
                fu[m] = fmaxf(g1 - g0, 0.0f);
                g0 = g1;
            }
        }
        const SfRowsOfVoxels ax = sf_rows_of_voxels(gv, f, zlo_k0);
        unsigned ofs = (unsigned)((ax.rb - win.r0) * BP_PS + (cf - win.c0));

        // Where no voxel of the wave is taller than a detector row in this view, consecutive voxels share rows and the
        // cheaper running scheme applies; tiles far from the source qualify even when the nearest voxels of the volume do
        // not (the instance is built for the tallest footprint).  The choice is uniform over the wave, so it costs one
        // ballot per view.
        // NV == 3 is chosen on the host only when no voxel is taller than two rows (with a margin): every lane takes one
        // of the two running schemes below, whichever fits its voxel column in this view.  Tiles far from the source hold
        // short voxels even when the nearest voxels of the volume are tall; a wave that holds both kinds (rare: the line
        // where a voxel is exactly one row tall crosses its 16 x 4 columns) runs the two schemes one after the other.
        const bool shared_rows = NV == 2 || (NV == 3 ? ax.av <= 1.0f : __builtin_amdgcn_ballot_w64(ax.av > 1.0f) == 0);
        auto row_sum = [&](const float *q) {
            float s = fu[0] * q[0];
#pragma unroll
            for (int m = 1; m < NC; ++m) s = fmaf(fu[m], q[m], s);
            return s;
        };
        // The voxel's first row is carried as a byte offset into the patch array (both buffers), so that every LDS read is
        // that register plus an immediate and a row crossing costs one select and one add.
        const char *const lds0 = reinterpret_cast<const char *>(&patch[0][0]);
        unsigned pb = (unsigned)((a & 1) * (BP_PH * BP_PS) + (int)ofs) * 4u;
        auto at = [&](unsigned byte_ofs) { return reinterpret_cast<const float *>(lds0 + byte_ofs); };
        if (shared_rows) {
            // A voxel is at most one row tall, so consecutive voxels share a row: keep the u-combined samples of the
            // current and the next row in registers and fetch one new row per voxel (half the LDS traffic).
            // f: where the voxel's lower face lies inside its first row, in [0,1); the face moves up by av per voxel.
            float f = ax.phi0;
            float s_cur = row_sum(at(pb)), s_next = row_sum(at(pb + 4u * BP_PS));
#pragma unroll
            for (int kk = 0; kk < BP_ZC; ++kk) {
                const float t = f + ax.av;                        // upper face, still measured from the first row
                const float w1 = sf_clamp(t - 1.0f, 0.0f, 1.0f);  // part of the voxel in the next row
                const float w0 = ax.av - w1;
                acc[kk] = fmaf(w1, s_next, fmaf(w0, s_cur, acc[kk]));
                if (kk + 1 < BP_ZC) {
                    const bool cross = t >= 1.0f;                 // the next voxel starts in the next row
                    pb += cross ? 4u * BP_PS : 0u;
                    const float s_new = row_sum(at(pb + 4u * BP_PS));   // equals s_next when no row was crossed
                    s_cur = cross ? s_next : s_cur;
                    s_next = s_new;
                    f = cross ? w1 : t;                           // t - 1 where a row was crossed
                }
                if ((kk & 3) == 3)
                    asm volatile("" : "+v"(pb), "+v"(acc[kk - 3]), "+v"(acc[kk - 2]), "+v"(acc[kk - 1]), "+v"(acc[kk]));
            }
        } else if constexpr (NV == 3) {
            // Between one and two rows tall: a voxel covers the rest of its first row, then up to one whole row, then
            // part of a third, and the next voxel starts one or two rows further: the u-combined sum of that row is
            // carried over (one select), the two rows after it are fetched fresh.
            float f = ax.phi0;
            float s0 = row_sum(at(pb)), s1 = row_sum(at(pb + 4u * BP_PS)), s2 = row_sum(at(pb + 8u * BP_PS));
#pragma unroll
            for (int kk = 0; kk < BP_ZC; ++kk) {
                const float t = f + ax.av;                        // upper face from the first row's lower edge: in (1, 3)
                const float w2 = sf_clamp(t - 2.0f, 0.0f, 1.0f);  // part in the third row
                const float w0 = 1.0f - f;                        // the rest of the first row
                const float w1 = (ax.av - w0) - w2;
                acc[kk] = fmaf(w2, s2, fmaf(w1, s1, fmaf(w0, s0, acc[kk])));
                if (kk + 1 < BP_ZC) {
                    const bool two = t >= 2.0f;                   // the next voxel starts two rows further
                    pb += two ? 8u * BP_PS : 4u * BP_PS;
                    s0 = two ? s2 : s1;
                    s1 = row_sum(at(pb + 4u * BP_PS));
                    s2 = row_sum(at(pb + 8u * BP_PS));
                    f = two ? w2 : t - 1.0f;                      // t - 2 where two rows were crossed
                }
                if ((kk & 3) == 3)
                    asm volatile("" : "+v"(pb), "+v"(acc[kk - 3]), "+v"(acc[kk - 2]), "+v"(acc[kk - 1]), "+v"(acc[kk]));
            }
        } else if constexpr (NV > 3) {
        float lo = ax.phi0;
#pragma unroll
        for (int kk = 0; kk < BP_ZC; ++kk) {
            const float hi = fmaf(ax.av, (float)(kk + 1), ax.phi0);
            const float fl = floorf(lo);
            const float *q = buf + (ofs + __umul24((unsigned)(int)fl, (unsigned)BP_PS));   // 24-bit multiply: one full-rate op
            float edge = fl + 1.0f;                                   // upper edge of the first row the voxel touches
            float w = fminf(edge, hi) - lo;
            float sum = acc[kk];
#pragma unroll
            for (int jj = 0; jj < NV; ++jj) {
                float s = fu[0] * q[jj * BP_PS];
#pragma unroll
                for (int m = 1; m < NC; ++m) s = fmaf(fu[m], q[jj * BP_PS + m], s);
                sum = fmaf(w, s, sum);
                w = sf_clamp(hi - edge, 0.0f, 1.0f);                  // overlap with the next row
                edge += 1.0f;
            }
            acc[kk] = sum;
            lo = hi;
            // An opaque dependency every few voxels: the LDS reads of the next group need `ofs`, which is only
            // available once this group's sums exist.  Without it the compiler issues all reads of the unrolled
            // loop first and spills them.
            if ((kk & 3) == 3)
                asm volatile("" : "+v"(ofs), "+v"(acc[kk - 3]), "+v"(acc[kk - 2]), "+v"(acc[kk - 1]), "+v"(acc[kk]));
        }
        }

        if (a + 1 < g.nviews)
            bp_store_view<BP_PW, BP_PH, NSTAGE, GT>(geom_of(a + 1), views[a + 1], sc, sr, win_next, stage, patch[(a + 1) & 1], colcs);
        win = win_next;
        __syncthreads();
    }

    if (i < g.nx && j < g.ny) {
#pragma unroll
        for (int kk = 0; kk < BP_ZC; ++kk)
            if (k0 + kk < g.nz) vol[((size_t)(k0 + kk) * g.ny + j) * g.nx + i] = acc[kk];
    }
}

#endif
