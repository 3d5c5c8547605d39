// Host geometry module: validates the CT parameter set ("PyTorch Interfaces and CT Parameters") and turns
// it into the constant tables the kernels read.  All derivations run in double; the tables are rounded to
// float once, here.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <cstring>
#include <new>

#include "leap_internal.h"
#define SF_NO_KERNELS   // this file needs the kernels' host-side limit functions only
#include "sf_backproject_tiled.h"
#include "sf_project_columns.h"
#include "md_backproject_tiled.h"
#include <thread>
#include "sd_backproject_tiled.h"

static thread_local std::string g_last_error;

void leap_set_error(const std::string &msg) { g_last_error = msg; }

int leap_hip_fail(hipError_t e, const char *what)
{
    g_last_error = std::string(what) + ": " + hipGetErrorString(e);
    return LEAP_HIP_ERROR;
}

extern "C" const char *leap_last_error(void) { return g_last_error.c_str(); }

extern "C" const char *leap_status_string(int status)
{
    switch (status) {
    case LEAP_OK: return "ok";
    case LEAP_INVALID_ARG: return "invalid argument";
    case LEAP_BAD_GEOMETRY: return "geometry not supported: source must lie strictly outside the volume";
    case LEAP_HIP_ERROR: return "HIP runtime error";
    case LEAP_UNSUPPORTED: return "size not supported";
    default: return "unknown status";
    }
}

static int invalid(const char *why)
{
    leap_set_error(why);
    return LEAP_INVALID_ARG;
}

static bool finite_pos(double v) { return std::isfinite(v) && v > 0.0; }

// Siddon model: constants of the line of every (view, detector column), in double ("sd_ray.h" states the formulation).
static void build_ray_table(leap_geometry *G)
{
    const leap_geometry_desc &d = G->desc;
    const double T = d.voxel_xy, Tz = d.voxel_z;
    G->raycols.resize((size_t)d.nviews * d.ncols);
    double max_slope = 0.0;
    for (int a = 0; a < d.nviews; ++a) {
        // modular scans with upright modules bring one parameter block per view: a circular cone-beam view of the
        // translated scene, with its own source distance, detector distance and column offset
        const bool per_view = !G->geoms.empty();
        const SfGeom &g = per_view ? G->geoms[a] : G->g;
        const int type = per_view ? (int)LEAP_CONE : d.type;
        const double sod = per_view ? g.sodd : d.sod, sdd = per_view ? g.kud * d.pixel_u : d.sdd;
        const double xlo = g.x0d - 0.5 * T, ylo = g.y0d - 0.5 * T;      // lower faces of voxel (0, 0)
        const double c = G->views[a].cd, s = G->views[a].sd;
        double max_dh = 0.0;
        for (int col = 0; col < d.ncols; ++col) {
            const double u = ((double)col - g.col_offd) * d.pixel_u;
            double ox, oy, dx, dy;
            if (type == LEAP_PARALLEL) {
                ox = -u * s; oy = u * c; dx = c; dy = s;
            } else if (type == LEAP_CONE_CURVED) {    // pixel at fan angle u / sdd on the cylinder
                const double cg = std::cos(u / sdd), sg = std::sin(u / sdd);
                ox = sod * c; oy = sod * s;
                dx = -sdd * (cg * c + sg * s); dy = sdd * (sg * c - cg * s);
            } else {
                ox = sod * c; oy = sod * s;
                dx = -sdd * c - u * s; dy = -sdd * s + u * c;
            }
            SdRayCol R;
            R.xmajor = std::fabs(dx) >= std::fabs(dy) ? 1 : 0;
            const double dmaj = R.xmajor ? dx : dy, dmin = R.xmajor ? dy : dx;
            const double omaj = R.xmajor ? ox : oy, omin = R.xmajor ? oy : ox;
            const double lomaj = R.xmajor ? xlo : ylo, lomin = R.xmajor ? ylo : xlo;
            R.m = dmin / dmaj;
            R.b = (omin - lomin) / T - R.m * (omaj - lomaj) / T;
            const double inv_m = R.m != 0.0 ? 1.0 / R.m : 1e30;
            R.inv_m = (float)std::fmin(std::fmax(inv_m, -1e30), 1e30);
            R.lxy = (float)(T * std::sqrt(dx * dx + dy * dy) / std::fabs(dmaj));
            if (type == LEAP_CONE || type == LEAP_CONE_CURVED) {
                R.h0 = (lomaj - omaj) / (dmaj * Tz);
                R.dh = T / (dmaj * Tz);
                R.vscale = (float)(T / std::fabs(dmaj));
            } else if (type == LEAP_PARALLEL) {
                R.h0 = 1.0 / Tz; R.dh = 0.0; R.vscale = 0.0f;
            } else {
                R.h0 = 0.0; R.dh = 0.0; R.vscale = 0.0f;
            }
            max_dh = std::fmax(max_dh, std::fabs(R.dh));
            G->raycols[(size_t)a * d.ncols + col] = R;
        }
        const double vmax = std::fmax(std::fabs(g.v0d), std::fabs(g.v0d + (d.nrows - 1) * g.pvd));
        max_slope = std::fmax(max_slope, max_dh * vmax);
    }
    G->sd_max_axial_slope = max_slope;
}

// ---- debugging aid ---------------------------------------------------------------------------------------------------
// One environment variable, LEAP_DEBUG, read when a handle is created: comma-separated key=value pairs that override
// what the selection below would pick (include/leap.h lists the keys).  Unknown keys are ignored.
static bool debug_option(const char *key, long &value)
{
    const char *env = std::getenv("LEAP_DEBUG");
    if (!env) return false;
    const size_t klen = std::strlen(key);
    for (const char *p = env; *p;) {
        const char *end = std::strchr(p, ',');
        const size_t len = end ? (size_t)(end - p) : std::strlen(p);
        if (len > klen + 1 && std::strncmp(p, key, klen) == 0 && p[klen] == '=') {
            value = std::atol(p + klen + 1);
            return true;
        }
        if (!end) break;
        p = end + 1;
    }
    return false;
}

// The parameter block view a is projected with: its own (modular scans with upright modules) or the shared one.
static const SfGeom &view_geom(const leap_geometry *G, int a) { return G->geoms.empty() ? G->g : G->geoms[a]; }

// Footprint bounds over the whole volume and all views, in double.  Magnification is extreme at the corner of the
// volume's bounding circle; a flat detector stretches a footprint seen at fan angle gamma by 1 / cos(gamma).
// Returns false when some view's source does not clear the bounding circle (then no fast kernel applies).
static bool footprint_bounds(leap_geometry *G)
{
    const leap_geometry_desc *d = &G->desc;
    const double T = d->voxel_xy, half_x = 0.5 * d->nx * T, half_y = 0.5 * d->ny * T;
    const int blocks = G->geoms.empty() ? 1 : d->nviews;
    double cols = 0.0, rows = 0.0, vpr = 0.0, slope = 1.0;
    for (int a = 0; a < blocks; ++a) {
        const SfGeom &ga = view_geom(G, a);
        const double cx = ga.x0d + 0.5 * (d->nx - 1) * T, cy = ga.y0d + 0.5 * (d->ny - 1) * T;
        const double rx = std::fabs(cx) + half_x, ry = std::fabs(cy) + half_y;
        const double reach = std::sqrt(rx * rx + ry * ry) + T;
        double mag_max = 1.0, mag_min = 1.0, stretch = 1.0;
        if (ga.type != SF_PARALLEL) {
            const double sdd = ga.kud * d->pixel_u, sod = ga.sodd;
            if (!(sod > reach) && !G->geoms.empty()) return false;
            mag_max = sdd / std::fmax(sod - reach, 1e-9 * sod);
            mag_min = sdd / (sod + reach);
            const double umax = std::fmax(std::fabs(-2.0 - ga.col_offd), std::fabs(d->ncols + 1.0 - ga.col_offd)) * d->pixel_u;
            const bool curved = ga.type == SF_CONE_CURVED;
            const double gam = curved ? std::fmin(umax / sdd, 1.57) : std::atan(umax / sdd);
            stretch = curved ? 1.02 : 1.02 / std::cos(gam);       // no stretch on the cylinder
            slope = std::fmax(slope, gam < 0.78 ? std::tan(0.7853981633974483 + gam) : 1e30);
        }
        const bool fan = ga.type == SF_FAN;
        cols = std::fmax(cols, mag_max * T * std::sqrt(2.0) / d->pixel_u * stretch);
        rows = std::fmax(rows, fan ? 1.0 : mag_max * d->voxel_z / d->pixel_v);
        vpr = std::fmax(vpr, fan ? 1.0 : d->pixel_v / (mag_min * d->voxel_z));
    }
    G->max_cols_per_voxel = cols; G->max_rows_per_voxel = rows; G->max_voxels_per_row = vpr; G->max_minor_slope = slope;
    return true;
}

// Largest staged window any (view, tile, first or last z-chunk) of a tiled back projection asks for, evaluated with the
// kernel's own window function on the view's own parameter block.
template <class WindowFn>
static void staged_window_need(const leap_geometry *G, int zc, WindowFn window, int &need_w, int &need_h)
{
    const leap_geometry_desc *d = &G->desc;
    const int tiles_x = (d->nx + BP_T - 1) / BP_T, tiles_y = (d->ny + BP_T - 1) / BP_T;
    const int chunks = (d->nz + zc - 1) / zc;
    // the views are shared out among a few threads (a thousand views of a few thousand tiles each)
    const int workers = (int)std::max(1, std::min(8, d->nviews / 32));
    std::vector<int> w(workers, 0), h(workers, 0);
    auto scan = [&](int t) {
        int wt = 0, ht = 0;                   // kept local: the workers' slots of w and h share a cache line
        for (int a = t; a < d->nviews; a += workers) {
            const SfGeom &ga = view_geom(G, a);
            for (int ty = 0; ty < tiles_y; ++ty)
                for (int tx = 0; tx < tiles_x; ++tx) {
                    const float xc = (float)(ga.x0d + ((double)(tx * BP_T) + 0.5 * (BP_T - 1)) * ga.Td);
                    const float yc = (float)(ga.y0d + ((double)(ty * BP_T) + 0.5 * (BP_T - 1)) * ga.Td);
                    for (int ch = 0; ch < chunks; ch += (chunks > 1 ? chunks - 1 : 1)) {   // extremes: first and last chunk
                        const float z0 = (float)(ga.zlo0d + (double)(ch * zc) * ga.Tzd), z1 = z0 + (float)zc * ga.Tz;
                        const SfWindow win = window(ga, G->views[a], xc, yc, z0, z1);
                        wt = win.need_w > wt ? win.need_w : wt;
                        ht = win.need_h > ht ? win.need_h : ht;
                    }
                }
        }
        w[t] = wt;
        h[t] = ht;
    };
    std::vector<std::thread> pool;
    for (int t = 1; t < workers; ++t) pool.emplace_back(scan, t);
    scan(0);
    for (auto &th : pool) th.join();
    need_w = *std::max_element(w.begin(), w.end());
    need_h = *std::max_element(h.begin(), h.end());
}

// Footprint model, tiled back projection: pick the template instance and verify its staged window.
static void select_footprint_tiled(leap_geometry *G)
{
    const leap_geometry_desc *d = &G->desc;
    if (d->type == LEAP_FAN || d->nz < 8 || !std::isfinite(G->max_cols_per_voxel) || G->max_cols_per_voxel > 4.0 ||
        G->max_rows_per_voxel > 3.0 || !((double)d->nrows * d->ncols < 1073741824.0))     // 32-bit byte offsets within a view
        return;
    G->bp_nc = std::max(2, (int)std::ceil(G->max_cols_per_voxel) + 1);
    // rows a voxel can touch; the three-row instance runs schemes that need every voxel at most two rows tall, so a
    // bound that close to two rows takes the four-row instance
    const double mr = G->max_rows_per_voxel;
    G->bp_nv = mr <= 1.0 + 1e-6 ? 2 : (mr <= 1.999 ? 3 : std::max(4, (int)std::ceil(mr - 1e-6) + 1));
    G->bp_wh = (float)(0.5 * G->max_cols_per_voxel);
    const float hx = 0.5f * (float)(BP_T - 1) * G->g.T;
    // 64-voxel chunks only pay off on tall volumes; the two-row instances keep 64 sums in registers in either 64-voxel
    // shape, the three-row instances in the tall one only
    int order[BP_NSHAPES], norder = 0;
    if (d->nz >= 128 && G->bp_nv == 2) order[norder++] = 0;
    if (d->nz >= 128 && G->bp_nv <= 3) order[norder++] = BP_TALL_SHAPE;
    for (int sh = BP_FIRST_SHORT_SHAPE; sh <= BP_LAST_SHORT_SHAPE; ++sh) order[norder++] = sh;
    long forced;
    if (debug_option("bp_shape", forced)) {        // start at a given shape, then the short ones after it
        forced = ((forced % BP_NSHAPES) + BP_NSHAPES) % BP_NSHAPES;
        norder = 0;
        order[norder++] = (int)forced;
        for (int sh = std::max((int)forced + 1, BP_FIRST_SHORT_SHAPE); sh <= BP_LAST_SHORT_SHAPE; ++sh) order[norder++] = sh;
    }
    for (int n = 0; n < norder && !G->bp_tiled; ++n) {
        const int sh = order[n];
        staged_window_need(G, BP_SHAPES[sh].zc,
                           [&](const SfGeom &ga, const SfView &v, float xc, float yc, float z0, float z1) {
                               return sf_bp_window(ga, v, xc, yc, hx, z0, z1, G->bp_wh, G->bp_nc, G->bp_nv);
                           },
                           G->bp_need_w, G->bp_need_h);
        G->bp_shape = sh;
        // one spare row and column: host and device floats may round apart
        G->bp_tiled = G->bp_need_w <= BP_SHAPES[sh].pw - 1 && G->bp_need_h <= BP_SHAPES[sh].ph - 1;
    }
    // Cylinder: the tiled kernel takes the angle between a voxel's centre and its corners from a short series,
    // good to 3e-9 rad below 0.08 rad.
    if (d->type == LEAP_CONE_CURVED) {
        const double rx = std::fabs(d->center_x) + 0.5 * d->nx * d->voxel_xy, ry = std::fabs(d->center_y) + 0.5 * d->ny * d->voxel_xy;
        const double nearest = d->sod - std::sqrt(rx * rx + ry * ry);
        if (!(0.7072 * d->voxel_xy <= 0.08 * nearest)) G->bp_tiled = false;
    }
}

// Row groups per wave of the column-wise forward kernels.  A wave pays a fixed share per candidate voxel column (its
// parameters, the transaxial record) worth about a group and a half, then one share per group whether or not the group
// holds rows of the detector; the detector needs ceil(groups / rg) bands of waves.
static int row_groups(int nrows, int rows_per_group, const int *choices, int nchoices)
{
    const int groups = (nrows + rows_per_group - 1) / rows_per_group;
    int best = choices[0];
    double best_cost = 1e300;
    for (int n = 0; n < nchoices; ++n) {
        const int rg = choices[n], bands = (groups + rg - 1) / rg;
        const double cost = bands * (1.6 + rg);
        if (cost < best_cost - 1e-9) { best_cost = cost; best = rg; }
    }
    long v;
    if (debug_option("rg", v))
        for (int n = 0; n < nchoices; ++n)
            if (choices[n] == v) best = (int)v;
    return best;
}

static void block_order_options(leap_geometry *G)
{
    long v;
    if (debug_option("vb", v) && v >= 1 && v <= 1024) G->fp_vb = (int)v;
    if (debug_option("tb", v) && v >= 1 && v <= 1024) G->fp_tb = (int)v;
}

// Footprint model, column-wise forward projection: static limits and the marching axis of every bundle.
static void select_footprint_columns(leap_geometry *G)
{
    const leap_geometry_desc *d = &G->desc;
    const double vpr = G->max_voxels_per_row;
    if (d->type == LEAP_FAN || d->nrows < 32 || !std::isfinite(vpr) || vpr > 3.0) return;
    // kappa (the axial voxel coordinate of a row's edge) must stay within +-2^19 for the kernel's placement arithmetic
    if (!((d->nrows + 1024.0) * vpr + d->nz + 64.0 < 500000.0)) return;
    long v;
    G->fp_cw = 4;
    // Short detectors (fewer than about 200 rows) have too few bundles of four to fill the chip: two columns measured
    // 5 to 12 % faster there.  The cylinder's record phase is heavier: four columns only pay off from about 450 rows on.
    if (d->nrows <= 192 || (d->type == LEAP_CONE_CURVED && d->nrows <= 448)) G->fp_cw = 2;
    const bool forced_cw = debug_option("cw", v) && (v == 1 || v == 2 || v == 4);
    if (forced_cw) G->fp_cw = (int)v;
    if (d->type != LEAP_CONE && d->type != LEAP_PARALLEL && G->fp_cw == 1) G->fp_cw = 2;   // instances of 4 and 2 columns only
    // candidate slots per slab: widest range of voxel columns any bundle of cw detector columns can see
    auto slots_needed = [&](int cw) {
        int need = 0;
        for (int a = 0; a < d->nviews && need <= 16; ++a)
            for (int c = 0; c < d->ncols; c += cw) {
                const SfRayLines L = sf_ray_lines(view_geom(G, a), G->views[a], c, cw);
                const int n_major = L.xmajor ? d->nx : d->ny;
                const float d0 = std::fabs(L.b0 - L.b1);
                const float d1 = std::fabs(fmaf(L.m0 - L.m1, (float)(n_major - 1), L.b0 - L.b1));
                const float dm = d0 > d1 ? d0 : d1;
                if (!(dm < 1e6f)) return 1 << 20;
                need = std::max(need, (int)std::floor(dm + 2.0f * L.spread + 1e-3f) + 2);
            }
        return need;
    };
    int need = slots_needed(G->fp_cw);
    const int cw_min = (d->type == LEAP_CONE || d->type == LEAP_PARALLEL) ? 1 : 2;
    while (need > 16 && G->fp_cw > cw_min) {
        G->fp_cw /= 2;
        need = slots_needed(G->fp_cw);
    }
    G->fp_need_q = need;
    G->fp_nq = need <= 4 ? 4 : (need <= 8 ? 8 : 16);
    G->fp_nkp = std::min(FP_MAX_P, std::max(2, (int)std::ceil(2.0 * vpr - 1e-6) + 1));
    static const int pair_groups[] = {1, 2, 3, 4};
    G->fp_rg = row_groups(d->nrows, 128, pair_groups, 4);
    G->fp_columns = need <= 16;
    block_order_options(G);
    if (!G->fp_columns) return;
    const int nbundles = (d->ncols + G->fp_cw - 1) / G->fp_cw;
    G->major.resize((size_t)d->nviews * nbundles);
    for (int a = 0; a < d->nviews; ++a)
        for (int b = 0; b < nbundles; ++b)
            G->major[(size_t)a * nbundles + b] = (unsigned char)sf_ray_lines(view_geom(G, a), G->views[a], b * G->fp_cw, G->fp_cw).xmajor;
}

// Siddon model: static limits of the two fast kernels.
static void select_siddon_fast_kernels(leap_geometry *G)
{
    const leap_geometry_desc *d = &G->desc;
    if (d->type == LEAP_FAN || !(G->sd_max_axial_slope <= 0.999)) return;

    // wave-per-column forward projection: no ray may cross more than one z-face per slab
    if (d->nrows >= 32) {
        G->sd_columns = true;
        static const int single_groups[] = {1, 2, 4, 8};
        G->fp_rg = row_groups(d->nrows, 64, single_groups, 4);
        block_order_options(G);
    }

    // tiled back projection: at most 4 pixel centres inside a voxel's footprint, and the staged window of every
    // (view, tile, z-chunk) must fit the instance (checked with the kernel's own function)
    if (d->nz >= 8 && std::isfinite(G->max_cols_per_voxel) && G->max_cols_per_voxel > 0.0 && G->max_cols_per_voxel < 3.9 &&
        (double)d->nrows * d->ncols < 1073741824.0) {      // the staging loads use 32-bit byte offsets within a view
        G->bp_nc = std::max(2, (int)std::floor(G->max_cols_per_voxel + 0.01) + 1);
        const float hx = 0.5f * (float)BP_T * G->g.T;
        long first_shape = BP_FIRST_SHORT_SHAPE;       // the 64-voxel shapes do not fit: the sums live in LDS
        if (debug_option("bp_shape", first_shape))
            first_shape = std::min((long)BP_LAST_SHORT_SHAPE, std::max((long)BP_FIRST_SHORT_SHAPE, first_shape % BP_NSHAPES));
        for (int sh = (int)first_shape; sh <= BP_LAST_SHORT_SHAPE && !G->bp_tiled; ++sh) {
            staged_window_need(G, BP_SHAPES[sh].zc,
                               [&](const SfGeom &ga, const SfView &v, float xc, float yc, float z0, float z1) {
                                   return sd_bp_window(ga, v, xc, yc, hx, z0, z1);
                               },
                               G->bp_need_w, G->bp_need_h);
            G->bp_shape = sh;
            G->bp_tiled = G->bp_need_w <= BP_SHAPES[sh].pw - 1 && G->bp_need_h <= BP_SHAPES[sh].ph - 1;
        }
    }
}

// Is the convex polygon {rect} cut by the half-planes a u + b v + c >= 0 non-empty?  (Sutherland-Hodgman; a polygon
// that shrinks to a point or a segment still counts.)
static bool rectangle_meets(double u0, double u1, double v0, double v1, const double (*planes)[3], int nplanes)
{
    std::vector<std::pair<double, double>> poly = {{u0, v0}, {u1, v0}, {u1, v1}, {u0, v1}}, next;
    for (int p = 0; p < nplanes && !poly.empty(); ++p) {
        next.clear();
        const double a = planes[p][0], b = planes[p][1], c = planes[p][2];
        for (size_t q = 0; q < poly.size(); ++q) {
            const auto &A = poly[q], &B = poly[(q + 1) % poly.size()];
            const double fa = a * A.first + b * A.second + c, fb = a * B.first + b * B.second + c;
            if (fa >= 0.0) next.push_back(A);
            if ((fa >= 0.0) != (fb >= 0.0)) {
                const double t = fa / (fa - fb);
                next.push_back({A.first + t * (B.first - A.first), A.second + t * (B.second - A.second)});
            }
        }
        poly.swap(next);
    }
    return !poly.empty();
}

// Siddon model on tilted modules: can the per-lane slab kernels serve the scan?  They need every ray to rise by less
// than one axial cell per slab along its faster in-plane axis (kappa |Dz| <= limit * max(|Dx|, |Dy|), kappa = T / Tz;
// D is affine in the detector coordinates, so the rays that break it fill a convex polygon of the detector per sign of
// Dz), and every source more than a voxel away from the volume's box.
static bool tilted_rays_stay_flat(const leap_geometry *G, double limit)
{
    const leap_geometry_desc *d = &G->desc;
    const SfGeom &g = G->g;
    const double kappa = d->voxel_xy / d->voxel_z;
    const double u0 = (0.0 - g.col_offd) * g.pu_d, u1 = ((double)(d->ncols - 1) - g.col_offd) * g.pu_d;
    const double v0 = g.v0d, v1 = g.v0d + (double)(d->nrows - 1) * g.pvd;
    const double half[3] = {0.5 * d->nx * d->voxel_xy + d->voxel_xy, 0.5 * d->ny * d->voxel_xy + d->voxel_xy,
                            0.5 * d->nz * d->voxel_z + d->voxel_z};
    const double ctr[3] = {d->center_x, d->center_y, d->center_z};
    for (const MdPose &P : G->poses) {
        bool clear = false;
        for (int q = 0; q < 3; ++q) clear = clear || std::fabs(P.S[q] - ctr[q]) > half[q];
        if (!clear) return false;
        for (int sign = -1; sign <= 1; sign += 2) {
            double planes[4][3];
            for (int h = 0; h < 4; ++h) {
                const int axis = h >> 1;                       // 0: x, 1: y
                const double w = (h & 1) ? limit : -limit;     // sign kappa Dz -+ limit D_axis >= 0
                planes[h][0] = sign * kappa * P.ucol[2] + w * P.ucol[axis];
                planes[h][1] = sign * kappa * P.vrow[2] + w * P.vrow[axis];
                planes[h][2] = sign * kappa * (P.C[2] - P.S[2]) + w * (P.C[axis] - P.S[axis]);
            }
            if (rectangle_meets(u0, u1, v0, v1, planes, 4)) return false;
        }
    }
    return true;
}

// Siddon model on tilted modules, tiled back projection: largest window any (view, tile, z-chunk) asks for (every chunk
// counts: a tilted module's windows are not extreme at the ends of the volume only).  The corners of all those boxes are
// the points of one lattice, so each view projects the lattice once and every window takes the extremes of its eight
// corners; the kernel's own function forms the same corners by increments and may round apart in the last place, which
// the spare row and column of the fit test absorb.  The views are shared out among a few threads.
static void tilted_window_need(const leap_geometry *G, const std::vector<MdBpView> &views, int zc, int &need_w, int &need_h)
{
    const leap_geometry_desc *d = &G->desc;
    const SfGeom &g = G->g;
    const int tiles_x = (d->nx + BP_T - 1) / BP_T, tiles_y = (d->ny + BP_T - 1) / BP_T, chunks = (d->nz + zc - 1) / zc;
    const int lx = tiles_x + 1, ly = tiles_y + 1, lz = chunks + 1;
    const int workers = (int)std::max<size_t>(1, std::min<size_t>(8, views.size() / 8));
    std::vector<int> w(workers, 0), h(workers, 0);
    auto scan = [&](int t) {
        std::vector<float> xi((size_t)lx * ly * lz), eta(xi.size());
        float ew = 0.0f, eh = 0.0f;             // widest and tallest shadow; a window holds at most that many pixel centres + 1.04
        for (size_t a = t; a < views.size(); a += workers) {
            const MdBpView &V = views[a];
            for (int iz = 0; iz < lz; ++iz)
                for (int iy = 0; iy < ly; ++iy)
                    for (int ix = 0; ix < lx; ++ix) {
                        const float dx = fmaf((float)(ix * BP_T), g.T, V.dlo[0]), dy = fmaf((float)(iy * BP_T), g.T, V.dlo[1]);
                        const float dz = fmaf((float)(iz * zc), g.Tz, V.dlo[2]);
                        const float inv = 1.0f / fmaf(dx, V.nrm[0], fmaf(dy, V.nrm[1], dz * V.nrm[2]));
                        const size_t o = ((size_t)iz * ly + iy) * lx + ix;
                        xi[o] = fmaf(fmaf(dx, V.euP[0], fmaf(dy, V.euP[1], dz * V.euP[2])), inv, V.xi0);
                        eta[o] = fmaf(fmaf(dx, V.evP[0], fmaf(dy, V.evP[1], dz * V.evP[2])), inv, V.eta0);
                    }
            for (int iz = 0; iz < chunks; ++iz)
                for (int iy = 0; iy < tiles_y; ++iy)
                    for (int ix = 0; ix < tiles_x; ++ix) {
                        float a0 = 3.0e38f, a1 = -3.0e38f, b0 = 3.0e38f, b1 = -3.0e38f;
                        for (int q = 0; q < 8; ++q) {
                            const size_t o = ((size_t)(iz + (q >> 2)) * ly + iy + ((q >> 1) & 1)) * lx + ix + (q & 1);
                            const float u = xi[o], v = eta[o];
                            a0 = u < a0 ? u : a0; a1 = u > a1 ? u : a1;
                            b0 = v < b0 ? v : b0; b1 = v > b1 ? v : b1;
                        }
                        ew = a1 - a0 > ew ? a1 - a0 : ew;
                        eh = b1 - b0 > eh ? b1 - b0 : eh;
                        if (!(a1 - a0 < 1.0e6f && b1 - b0 < 1.0e6f)) ew = eh = 1.0e6f;      // NaN or absurd: no instance fits
                    }
        }
        w[t] = sf_f2i(floorf(ew + 1.04f));
        h[t] = sf_f2i(floorf(eh + 1.04f));
    };
    std::vector<std::thread> pool;
    for (int t = 1; t < workers; ++t) pool.emplace_back(scan, t);
    scan(0);
    for (auto &th : pool) th.join();
    need_w = *std::max_element(w.begin(), w.end());
    need_h = *std::max_element(h.begin(), h.end());
}

// Siddon model, scans with tilted modules: the per-lane variants of the two fast kernels.
static void select_tilted_siddon_kernels(leap_geometry *G)
{
    const leap_geometry_desc *d = &G->desc;
    long v;
    if (debug_option("general", v) && v == 1) return;
    if (d->nrows >= 32 && tilted_rays_stay_flat(G, 0.999)) {        // forward projection on the slab scratch
        G->md_tilted = true;
        G->sd_columns = true;
        static const int single_groups[] = {1, 2, 4};
        G->fp_rg = row_groups(d->nrows, 64, single_groups, 3);
        block_order_options(G);
    }
    // Tiled back projection.  Its rays are marched along the TILE's faster in-plane axis: a ray through a tile whose
    // centre lies c_maj from the source along that axis has |d_maj| >= c_maj - 8 T and max(|dx|, |dy|) <= c_maj + 8 T, so
    // a rise of at most 0.8 cells per slab along the ray's own axis stays below one cell along the tile's if
    // c_maj >= 72 T, which an in-plane distance of 102 T between source and volume guarantees.
    if (d->nz < 8 || !((double)d->nrows * d->ncols < 1073741824.0) || !tilted_rays_stay_flat(G, 0.8)) return;
    const double half[3] = {0.5 * d->nx * d->voxel_xy, 0.5 * d->ny * d->voxel_xy, 0.5 * d->nz * d->voxel_z};
    const double ctr[3] = {d->center_x, d->center_y, d->center_z};
    for (const MdPose &P : G->poses) {
        const double ox = std::fmax(std::fabs(P.S[0] - ctr[0]) - half[0], 0.0), oy = std::fmax(std::fabs(P.S[1] - ctr[1]) - half[1], 0.0);
        if (!(std::hypot(ox, oy) >= 102.0 * d->voxel_xy)) return;
        const double n[3] = {P.ucol[1] * P.vrow[2] - P.ucol[2] * P.vrow[1], P.ucol[2] * P.vrow[0] - P.ucol[0] * P.vrow[2],
                             P.ucol[0] * P.vrow[1] - P.ucol[1] * P.vrow[0]};
        const double gap = (P.C[0] - P.S[0]) * n[0] + (P.C[1] - P.S[1]) * n[1] + (P.C[2] - P.S[2]) * n[2];
        for (int corner = 0; corner < 8; ++corner) {                // the whole volume in front of the source
            double along = 0.0;
            for (int q = 0; q < 3; ++q) along += (ctr[q] + ((corner >> q) & 1 ? half[q] : -half[q]) - P.S[q]) * n[q];
            if (!(along * gap > 0.0) || !(std::fabs(along) > 1e-3 * std::fabs(gap))) return;
        }
    }
    std::vector<MdBpView> views;
    views.reserve(G->poses.size());
    for (const MdPose &P : G->poses) views.push_back(md_bp_view(G->g, P));
    long first_shape = 0;
    if (debug_option("bp_shape", first_shape)) first_shape = ((first_shape % MD_BP_NSHAPES) + MD_BP_NSHAPES) % MD_BP_NSHAPES;
    bool fits = false;
    for (int sh = (int)first_shape; sh < MD_BP_NSHAPES && !fits; ++sh) {
        tilted_window_need(G, views, MD_BP_SHAPES[sh].zc, G->bp_need_w, G->bp_need_h);
        G->bp_shape = sh;
        fits = G->bp_need_w <= MD_BP_SHAPES[sh].pw - 1 && G->bp_need_h <= MD_BP_SHAPES[sh].ph - 1;
    }
    if (!fits) return;
    hipError_t e = hipMalloc((void **)&G->d_mdbp, sizeof(MdBpView) * views.size());
    if (e == hipSuccess) e = hipMemcpy(G->d_mdbp, views.data(), sizeof(MdBpView) * views.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (G->d_mdbp) (void)hipFree(G->d_mdbp);
        G->d_mdbp = nullptr;
        (void)hipGetLastError();
        G->note = "table allocation failed: back projection runs on the general kernel";
        return;
    }
    G->bp_tiled = true;
}

// Picks the kernels of a validated scan (circular scanners, or modular scans made of upright modules).
static void select_fast_kernels(leap_geometry *G)
{
    if (!footprint_bounds(G)) return;
    long v;
    if (debug_option("general", v) && v == 1) return;       // testing aid: every call on the general kernels
    if (G->desc.model == LEAP_MODEL_SF) {
        select_footprint_tiled(G);
        select_footprint_columns(G);
    } else {
        select_siddon_fast_kernels(G);
    }
}

// Slab width and items per launch that a scratch of `floats` floats affords for a batch of `batch` volumes: as many
// items at once as the batch has (16 at most) while a slab stays at least 32 voxel layers wide, the whole volume per
// copy if it fits.  Returns false if not even four layers fit.
bool leap_plan_scratch(const leap_geometry *G, size_t floats, int batch, int &width, int &items)
{
    const leap_geometry_desc *d = &G->desc;
    const int n_side = std::max(d->nx, d->ny);                  // a slab holds up to width * n_side voxel columns
    const double nzp = d->nz + 2.0 * FP_PAD;
    auto width_for = [&](int it) {
        const double w = std::floor(((double)floats / it - nzp) / (nzp * n_side));
        return w >= n_side ? n_side : (w < 4 ? 0 : ((int)w & ~3));
    };
    items = std::max(1, std::min(batch, 16));
    while (items > 1 && width_for(items) < std::min(32, n_side)) items = (items + 1) / 2;
    width = width_for(items);
    if (G->dbg_items > 0) items = std::min(G->dbg_items, std::max(1, batch));
    if (G->dbg_slab > 0) width = std::min(G->dbg_slab, n_side);
    if (G->dbg_items > 0 || G->dbg_slab > 0) {                  // overrides must still fit
        while (items > 1 && ((double)width * n_side + 1.0) * nzp * items > (double)floats) --items;
        if (((double)width * n_side + 1.0) * nzp * items > (double)floats) width = width_for(items);
    }
    // the copy kernel puts (voxel rows of a slab) x (items) into one grid dimension
    items = std::max(1, std::min(items, 65535 / std::max(std::max(d->ny, width), 1)));
    return width >= 4 && ((double)width * n_side + 1.0) * nzp < 4294967296.0;     // slab columns are indexed with 32 bits
}

// The scratch of the column-wise forward kernels: z-fastest copies of one slab of the volume (plus a spare zero column
// each).  Large volumes: an eighth of one volume (a quarter for the Siddon kernel, whose waves own a single detector
// column and lose more to narrow slabs); volumes under 512 MiB: 128 MiB, which lets a batch of small training volumes
// go through together.  On failure the handle falls back to the general kernel and says so (leap_last_error, and the
// note shown by leap_geometry_describe).
static void allocate_forward_scratch(leap_geometry *G)
{
    const leap_geometry_desc *d = &G->desc;
    if (!G->fp_columns && !G->sd_columns) return;
    G->nzp = d->nz + 2 * FP_PAD;
    const double volume_bytes = 4.0 * d->nx * d->ny * (double)d->nz;
    const double share = volume_bytes / (d->model == LEAP_MODEL_SIDDON ? 4.0 : 8.0);
    double budget = volume_bytes / 8.0 >= 64.0 * 1048576.0 ? share : 128.0 * 1048576.0;
    long v;
    if (debug_option("scratch_mib", v) && v >= 1) budget = 1048576.0 * (double)v;
    if (debug_option("slab", v) && v >= 4) G->dbg_slab = (int)(v & ~3L);
    if (debug_option("items", v) && v >= 1 && v <= 16) G->dbg_items = (int)v;
    // no more than 16 whole copies
    const double whole = 4.0 * ((double)d->nx * d->ny + 1.0) * G->nzp;
    budget = std::fmin(budget, 16.0 * whole);
    hipError_t e = hipErrorOutOfMemory;
    int width = 0, items = 0;
    for (int attempt = 0; attempt < 6; ++attempt, budget *= 0.5) {
        G->scratch_bytes = (size_t)budget & ~(size_t)255;
        if (!leap_plan_scratch(G, G->scratch_bytes / sizeof(float), 1, width, items)) break;
        e = hipMalloc((void **)&G->d_volz, G->scratch_bytes);
        if (e == hipSuccess) e = hipMemset(G->d_volz, 0, G->scratch_bytes);   // the pads stay zero for the handle's life
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e == hipSuccess) break;
        if (G->d_volz) (void)hipFree(G->d_volz);
        G->d_volz = nullptr;
        (void)hipGetLastError();
    }
    if (e == hipSuccess && !G->major.empty()) {
        e = hipMalloc((void **)&G->d_major, G->major.size());
        if (e == hipSuccess) e = hipMemcpy(G->d_major, G->major.data(), G->major.size(), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipEventCreateWithFlags(&G->scratch_event, hipEventDisableTiming);
    if (e != hipSuccess) {
        if (G->d_volz) (void)hipFree(G->d_volz);
        if (G->d_major) (void)hipFree(G->d_major);
        G->d_volz = nullptr; G->d_major = nullptr;
        G->fp_columns = G->sd_columns = false;
        G->scratch_bytes = 0;
        G->note = "scratch allocation failed: forward projection runs on the general kernel";
        leap_set_error(std::string("leap_geometry_create: ") + G->note + " (" + hipGetErrorString(e) + ")");
        (void)hipGetLastError();
        return;
    }
    G->slab_width = width;
}

static void free_handle(leap_geometry *G)
{
    if (!G) return;
    leap_host_stage_free(G);
    if (G->d_views) (void)hipFree(G->d_views);
    if (G->d_volz) (void)hipFree(G->d_volz);
    if (G->d_major) (void)hipFree(G->d_major);
    if (G->d_raycols) (void)hipFree(G->d_raycols);
    if (G->d_poses) (void)hipFree(G->d_poses);
    if (G->d_geoms) (void)hipFree(G->d_geoms);
    if (G->d_mfviews) (void)hipFree(G->d_mfviews);
    if (G->d_mdbp) (void)hipFree(G->d_mdbp);
    if (G->d_colcs) (void)hipFree(G->d_colcs);
    if (G->scratch_event) (void)hipEventDestroy(G->scratch_event);
    delete G;
}

// Cylindrical detector, tiled back projection: cosine and sine of every detector column's fan angle (ray amplitudes),
// then per (tile, view) the tile centre's fan angle and the tile's window bounds.  No room for the tables: the general
// kernel needs none.
static void upload_curved_tables(leap_geometry *G)
{
    const leap_geometry_desc *d = &G->desc;
    const SfGeom &g = G->g;
    const int tiles_x = (d->nx + BP_T - 1) / BP_T, tiles_y = (d->ny + BP_T - 1) / BP_T;
    const size_t head = 2 * sizeof(float) * (size_t)d->ncols;
    const size_t bytes = head + sizeof(SfCurvedBounds) * (size_t)tiles_x * tiles_y * d->nviews;
    std::vector<unsigned char> blob(bytes);
    float *cs = reinterpret_cast<float *>(blob.data());
    for (int c = 0; c < d->ncols; ++c) {
        const double gam = ((double)c - g.col_offd) * d->pixel_u / d->sdd;
        cs[2 * (size_t)c] = (float)std::cos(gam);
        cs[2 * (size_t)c + 1] = (float)std::sin(gam);
    }
    SfCurvedBounds *tab = reinterpret_cast<SfCurvedBounds *>(blob.data() + head);
    const float hx = 0.5f * (float)(BP_T - 1) * g.T;
    for (int ty = 0; ty < tiles_y; ++ty)
        for (int tx = 0; tx < tiles_x; ++tx) {
            const double xcd = g.x0d + ((double)(tx * BP_T) + 0.5 * (BP_T - 1)) * g.Td;
            const double ycd = g.y0d + ((double)(ty * BP_T) + 0.5 * (BP_T - 1)) * g.Td;
            SfCurvedBounds *row = tab + ((size_t)ty * tiles_x + tx) * d->nviews;
            for (int a = 0; a < d->nviews; ++a) {
                const SfView &v = G->views[a];
                row[a].gref = std::atan2(std::fma(ycd, v.cd, -xcd * v.sd), g.sodd - std::fma(xcd, v.cd, ycd * v.sd));
                sf_curved_tile_bounds(g, v, (float)xcd, (float)ycd, hx, row[a].xi_lo, row[a].xi_hi, row[a].ilo, row[a].ihi);
            }
        }
    hipError_t et = hipMalloc((void **)&G->d_colcs, bytes);
    if (et == hipSuccess) et = hipMemcpy(G->d_colcs, blob.data(), bytes, hipMemcpyHostToDevice);
    if (et != hipSuccess) {
        if (G->d_colcs) (void)hipFree(G->d_colcs);
        G->d_colcs = nullptr;
        G->bp_tiled = false;
        G->note = "no room for the cylinder's tile tables: back projection runs on the general kernel";
        (void)hipGetLastError();
    }
}

// Uploads every table the chosen kernels read to the current device and allocates the forward scratch; on failure
// frees the handle.
static int finish_handle(leap_geometry *G, leap_geometry **out)
{
    const leap_geometry_desc *d = &G->desc;
    auto upload = [](void **dst, const void *src, size_t bytes) {
        hipError_t e = hipMalloc(dst, bytes);
        if (e == hipSuccess) e = hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice);
        return e;
    };
    long kib;
    if (debug_option("stage_kib", kib) && kib >= 4) G->stage_chunk = (size_t)kib << 10;
    hipError_t e = hipGetDevice(&G->device);
    if (e == hipSuccess) (void)leap_static_scratch_init(G->device);   // set-up for leap_project_static_scratch; it reports a failure itself
    if (e == hipSuccess && !G->views.empty()) e = upload((void **)&G->d_views, G->views.data(), sizeof(SfView) * G->views.size());
    if (e == hipSuccess) allocate_forward_scratch(G);
    if (e == hipSuccess && !G->raycols.empty()) e = upload((void **)&G->d_raycols, G->raycols.data(), sizeof(SdRayCol) * G->raycols.size());
    if (e == hipSuccess && !G->geoms.empty()) e = upload((void **)&G->d_geoms, G->geoms.data(), sizeof(SfGeom) * G->geoms.size());
    if (e == hipSuccess && !G->poses.empty()) e = upload((void **)&G->d_poses, G->poses.data(), sizeof(MdPose) * G->poses.size());
    if (e == hipSuccess && !G->mfviews.empty())
        e = upload((void **)&G->d_mfviews, G->mfviews.data(), sizeof(MfView) * G->mfviews.size());
    if (e == hipSuccess && d->type == LEAP_CONE_CURVED && d->model == LEAP_MODEL_SF && G->bp_tiled) upload_curved_tables(G);
    if (e != hipSuccess) {
        free_handle(G);
        return leap_hip_fail(e, "uploading the geometry tables");
    }
    *out = G;
    return LEAP_OK;
}

// Modular geometry: per-view poses instead of the angle list; only the fields the modular kernels read are filled.
static int create_modular(const leap_geometry_desc *d, leap_geometry **out)
{
    if (!d->poses) return invalid("poses is null");
    if (d->nviews > 65535 || (double)d->nx * d->ny * d->nz >= 4294967296.0 ||
        (double)d->nviews * d->nrows * d->ncols >= 4294967296.0 || d->ny > 262140 || d->nz > 65535 || d->nrows > 262140) {
        leap_set_error("sizes beyond what one launch covers");
        return LEAP_UNSUPPORTED;
    }
    const double half[3] = {0.5 * d->nx * d->voxel_xy, 0.5 * d->ny * d->voxel_xy, 0.5 * d->nz * d->voxel_z};
    const double ctr[3] = {d->center_x, d->center_y, d->center_z};
    for (int a = 0; a < d->nviews; ++a) {
        const double *p = d->poses + 12 * (size_t)a;
        for (int q = 0; q < 12; ++q)
            if (!std::isfinite(p[q])) return invalid("poses must be finite");
        const double uu = p[6] * p[6] + p[7] * p[7] + p[8] * p[8], vv = p[9] * p[9] + p[10] * p[10] + p[11] * p[11];
        const double uv = p[6] * p[9] + p[7] * p[10] + p[8] * p[11];
        if (std::fabs(uu - 1.0) > 1e-9 || std::fabs(vv - 1.0) > 1e-9 || std::fabs(uv) > 1e-9)
            return invalid("detector axes must be orthonormal");
        bool inside = true;
        for (int q = 0; q < 3; ++q) inside = inside && std::fabs(p[q] - ctr[q]) <= half[q];
        if (inside) {
            leap_set_error("a source lies inside the volume");
            return LEAP_BAD_GEOMETRY;
        }
    }
    // Upright modules (column axis horizontal, row axis +z, detector behind the volume as seen from the source, source
    // clear of the volume's bounding circle in the module's frame) are circular cone-beam views of a translated scene:
    // both models have fast kernels for scans made of them.  A scan with any other module goes through the general
    // kernels of its model.
    bool tilted = false, upright = true;
    for (int a = 0; a < d->nviews; ++a) {
        const double *p = d->poses + 12 * (size_t)a;
        if (std::fabs(p[8]) > 1e-9 || std::fabs(p[9]) > 1e-9 || std::fabs(p[10]) > 1e-9 || std::fabs(p[11] - 1.0) > 1e-9) {
            tilted = true;
            upright = false;
        }
    }
    for (int a = 0; a < d->nviews && !tilted && upright; ++a) {
        const double *p = d->poses + 12 * (size_t)a;
        const double c = p[7], s = -p[6];
        const double lS = p[0] * c + p[1] * s, lD = p[3] * c + p[4] * s, tS = -p[0] * s + p[1] * c;
        // the volume as this view sees it: moved by -tS along the column axis
        const double mx = std::fabs(d->center_x - tS * p[6]) + half[0], my = std::fabs(d->center_y - tS * p[7]) + half[1];
        const double reach_a = std::sqrt(mx * mx + my * my);
        if (!(lS - lD > 0.0) || !(lS > reach_a) || !(d->pixel_u < 0.25 * (lS - lD))) upright = false;
    }
    if (d->model == LEAP_MODEL_SF && !upright && !tilted) {
        leap_set_error("module does not face its source across the volume");
        return LEAP_BAD_GEOMETRY;
    }
    leap_geometry *G = new (std::nothrow) leap_geometry;
    if (!G) return invalid("out of host memory");
    G->desc = *d;
    G->desc.angles_rad = nullptr;
    SfGeom &g = G->g;
    std::memset(&g, 0, sizeof(g));
    g.type = d->type; g.model = d->model;
    g.nviews = d->nviews; g.nrows = d->nrows; g.ncols = d->ncols;
    g.nx = d->nx; g.ny = d->ny; g.nz = d->nz;
    g.Td = d->voxel_xy; g.Tzd = d->voxel_z;
    g.x0d = d->center_x - 0.5 * (d->nx - 1) * d->voxel_xy;
    g.y0d = d->center_y - 0.5 * (d->ny - 1) * d->voxel_xy;
    g.zlo0d = d->center_z - 0.5 * d->nz * d->voxel_z;
    g.col_offd = 0.5 * (d->ncols - 1) - d->shift_u;
    g.row_offd = 0.5 * (d->nrows - 1) - d->shift_v + 0.5;
    g.v0d = (-0.5 * (d->nrows - 1) + d->shift_v) * d->pixel_v;
    g.pvd = d->pixel_v;
    g.pu_d = d->pixel_u;
    g.T = (float)d->voxel_xy; g.Tz = (float)d->voxel_z; g.pu = (float)d->pixel_u; g.pv = (float)d->pixel_v;
    G->poses.resize(d->nviews);
    std::memcpy(G->poses.data(), d->poses, sizeof(MdPose) * (size_t)d->nviews);
    G->desc.poses = reinterpret_cast<const double *>(G->poses.data());
    if (upright) {
        // per view: the same scene translated so that the source sits on the frame's axis at height 0
        g.iTzd = 1.0 / d->voxel_z;
        G->views.resize(d->nviews);
        G->geoms.resize(d->nviews);
        const double h = 0.5 * d->voxel_xy;
        for (int a = 0; a < d->nviews; ++a) {
            const MdPose &P = G->poses[a];
            const double c = P.ucol[1], s = -P.ucol[0];
            const double lS = P.S[0] * c + P.S[1] * s, tS = -P.S[0] * s + P.S[1] * c, zS = P.S[2];
            const double sdd = lS - (P.C[0] * c + P.C[1] * s), tC = -P.C[0] * s + P.C[1] * c, zC = P.C[2];
            SfView &v = G->views[a];
            std::memset(&v, 0, sizeof(v));
            v.cd = c; v.sd = s; v.c = (float)c; v.s = (float)s;
            v.p = (float)(h * c); v.q = (float)(h * s);
            v.xmajor = std::fabs(c) >= std::fabs(s) ? 1 : 0;
            SfGeom &ga = G->geoms[a];
            ga = g;
            ga.type = SF_CONE;
            ga.x0d = g.x0d - tS * P.ucol[0];
            ga.y0d = g.y0d - tS * P.ucol[1];
            ga.zlo0d = g.zlo0d - zS;
            ga.sodd = lS;
            ga.kud = sdd / d->pixel_u; ga.kvd = sdd / d->pixel_v; ga.ikvd = 1.0 / ga.kvd;
            ga.col_offd = g.col_offd - (tC - tS) / d->pixel_u;
            ga.row_offd = g.row_offd - (zC - zS) / d->pixel_v;
            ga.v0d = g.v0d + (zC - zS);
            ga.zk0d = -ga.zlo0d / d->voxel_z;
            ga.sod = (float)lS; ga.sdd = (float)sdd; ga.ku = (float)ga.kud;
            ga.col_off = (float)ga.col_offd; ga.v0 = (float)ga.v0d;
        }
    }
    if (upright) {
        if (d->model == LEAP_MODEL_SIDDON) build_ray_table(G);
        select_fast_kernels(G);
    } else if (d->model == LEAP_MODEL_SIDDON) {
        select_tilted_siddon_kernels(G);
        // The general back projection bounds a voxel's pixel search by its projected corners; a voxel that reaches behind
        // a source's plane (the plane through the source parallel to its module) has no such bound and tests every pixel
        // of that view.  On large scans that is not a slow call but one that never ends: refuse it.
        if (!G->bp_tiled) {
            double behind = 0.0;
            for (const MdPose &P : G->poses) {
                const double n[3] = {P.ucol[1] * P.vrow[2] - P.ucol[2] * P.vrow[1], P.ucol[2] * P.vrow[0] - P.ucol[0] * P.vrow[2],
                                     P.ucol[0] * P.vrow[1] - P.ucol[1] * P.vrow[0]};
                const double gap = (P.C[0] - P.S[0]) * n[0] + (P.C[1] - P.S[1]) * n[1] + (P.C[2] - P.S[2]) * n[2];
                bool all_in_front = true;
                for (int corner = 0; corner < 8; ++corner) {
                    double along = 0.0;
                    for (int q = 0; q < 3; ++q) along += (ctr[q] + ((corner >> q) & 1 ? half[q] : -half[q]) - P.S[q]) * n[q];
                    all_in_front = all_in_front && along * gap > 0.0;
                }
                behind += all_in_front ? 0.0 : 1.0;
            }
            if (behind * d->nrows * d->ncols * ((double)d->nx * d->ny * d->nz) > 5.0e11) {
                leap_set_error("in " + std::to_string((long)behind) + " views the volume reaches behind the source's plane (the plane "
                               "through the source parallel to its module); on a scan of this size the back projection of such "
                               "views is not supported");
                free_handle(G);
                return LEAP_UNSUPPORTED;
            }
        }
    }
    if (!upright && d->model == LEAP_MODEL_SF) {
        G->mfviews.resize(d->nviews);
        for (int a = 0; a < d->nviews; ++a) {
            const MdPose &P = G->poses[a];
            MfView &V = G->mfviews[a];
            for (int q = 0; q < 3; ++q) { V.S[q] = P.S[q]; V.C[q] = P.C[q]; V.eu[q] = P.ucol[q]; V.ev[q] = P.vrow[q]; }
            if (!mf_prepare_view(g, V)) {
                leap_set_error("view " + std::to_string(a) + " has no footprints: the whole volume must lie in front of the "
                               "source (on the module's side) and no pixel's ray may run along z");
                free_handle(G);
                return LEAP_BAD_GEOMETRY;
            }
            // the forward kernel looks for a pixel's voxels within the footprint's reach around its ray: a source so close
            // to the volume that the nearest voxel's footprint spans dozens of pixels makes that search the whole volume
            if (V.pad_u * V.ipu > 32.0 || V.pad_v * V.ipv > 32.0) {
                leap_set_error("view " + std::to_string(a) + ": the source is so close to the volume that a voxel's footprint on "
                               "this tilted module spans more than 64 pixels; not supported by the footprint kernels for "
                               "tilted modules");
                free_handle(G);
                return LEAP_UNSUPPORTED;
            }
        }
    }
    return finish_handle(G, out);
}

extern "C" int leap_geometry_create(const leap_geometry_desc *d, leap_geometry **out)
{
    if (out) *out = nullptr;
    if (!d || !out) return invalid("null descriptor or output pointer");
    if (d->type != LEAP_PARALLEL && d->type != LEAP_FAN && d->type != LEAP_CONE && d->type != LEAP_CONE_CURVED &&
        d->type != LEAP_MODULAR)
        return invalid("unknown geometry type");
    if (d->model != LEAP_MODEL_SF && d->model != LEAP_MODEL_SIDDON) return invalid("unknown projector model");
    if (d->nviews <= 0 || d->nrows <= 0 || d->ncols <= 0) return invalid("nviews, nrows and ncols must be positive");
    if (d->nx <= 0 || d->ny <= 0 || d->nz <= 0) return invalid("nx, ny and nz must be positive");
    if (!finite_pos(d->pixel_u) || !finite_pos(d->pixel_v)) return invalid("pixel sizes must be positive");
    if (!finite_pos(d->voxel_xy) || !finite_pos(d->voxel_z)) return invalid("voxel sizes must be positive");
    if (!std::isfinite(d->shift_u) || !std::isfinite(d->shift_v)) return invalid("detector shifts must be finite");
    if (!std::isfinite(d->center_x) || !std::isfinite(d->center_y) || !std::isfinite(d->center_z))
        return invalid("volume centre must be finite");
    if (d->type == LEAP_MODULAR) return create_modular(d, out);
    if (!d->angles_rad) return invalid("angles_rad is null");
    for (int a = 0; a < d->nviews; ++a)
        if (!std::isfinite(d->angles_rad[a])) return invalid("view angles must be finite");
    if (d->type == LEAP_FAN && (d->nrows != 1 || d->nz != 1)) return invalid("fan-beam needs nrows == 1 and nz == 1");
    if (d->nviews > 65535) {
        leap_set_error("more than 65535 views in one geometry");
        return LEAP_UNSUPPORTED;
    }
    if ((double)d->nx * d->ny * d->nz >= 2147483648.0 * 2.0 || (double)d->nviews * d->nrows * d->ncols >= 2147483648.0 * 2.0) {
        leap_set_error("array of more than 2^32 elements");
        return LEAP_UNSUPPORTED;
    }

    const double T = d->voxel_xy, h = 0.5 * T;
    const double half_x = 0.5 * d->nx * T, half_y = 0.5 * d->ny * T;
    if (d->type != LEAP_PARALLEL) {
        if (!finite_pos(d->sdd) || !finite_pos(d->sod)) {
            leap_set_error("sod and sdd must be positive");
            return LEAP_BAD_GEOMETRY;
        }
        // farthest in-plane corner of the volume from the rotation axis
        const double rx = std::fabs(d->center_x) + half_x, ry = std::fabs(d->center_y) + half_y;
        const double reach = std::sqrt(rx * rx + ry * ry);
        if (!(d->sod > reach)) {
            leap_set_error("source orbit radius (sod) does not clear the volume's bounding circle");
            return LEAP_BAD_GEOMETRY;
        }
        if (!(d->pixel_u < 0.25 * d->sdd)) {
            leap_set_error("detector pixel wider than a quarter of sdd");
            return LEAP_BAD_GEOMETRY;
        }
        if (d->type == LEAP_CONE_CURVED && !((0.5 * d->ncols + std::fabs(d->shift_u) + 1.0) * d->pixel_u < 1.5 * d->sdd)) {
            leap_set_error("curved detector spans a fan of more than +-1.5 rad");
            return LEAP_BAD_GEOMETRY;
        }
    }

    leap_geometry *G = new (std::nothrow) leap_geometry;
    if (!G) return invalid("out of host memory");
    G->desc = *d;
    G->angles.assign(d->angles_rad, d->angles_rad + d->nviews);
    G->desc.angles_rad = G->angles.data();

    SfGeom &g = G->g;
    std::memset(&g, 0, sizeof(g));
    const bool par = d->type == LEAP_PARALLEL;
    g.type = d->type;
    g.nviews = d->nviews; g.nrows = d->nrows; g.ncols = d->ncols;
    g.nx = d->nx; g.ny = d->ny; g.nz = d->nz;
    g.Td = T; g.Tzd = d->voxel_z;
    g.x0d = d->center_x - 0.5 * (d->nx - 1) * T;
    g.y0d = d->center_y - 0.5 * (d->ny - 1) * T;
    g.zlo0d = d->center_z - 0.5 * d->nz * d->voxel_z;
    g.sodd = par ? 0.0 : d->sod;
    g.kud = par ? 1.0 / d->pixel_u : d->sdd / d->pixel_u;
    g.kvd = par ? 1.0 / d->pixel_v : d->sdd / d->pixel_v;
    g.ikvd = 1.0 / g.kvd;
    g.iTzd = 1.0 / d->voxel_z;
    g.col_offd = 0.5 * (d->ncols - 1) - d->shift_u;
    g.row_offd = 0.5 * (d->nrows - 1) - d->shift_v + 0.5;
    g.T = (float)T; g.Tz = (float)d->voxel_z;
    g.sod = (float)g.sodd; g.sdd = par ? 0.0f : (float)d->sdd;
    g.pu = (float)d->pixel_u; g.pv = (float)d->pixel_v;
    g.ku = (float)g.kud;
    g.col_off = (float)g.col_offd;
    g.v0 = (float)((-0.5 * (d->nrows - 1) + d->shift_v) * d->pixel_v);
    g.model = d->model;
    g.v0d = (-0.5 * (d->nrows - 1) + d->shift_v) * d->pixel_v;
    g.pvd = d->pixel_v;
    g.pu_d = d->pixel_u;
    g.zk0d = d->type == LEAP_FAN ? 0.5 : -g.zlo0d / d->voxel_z;

    G->views.resize(d->nviews);
    for (int a = 0; a < d->nviews; ++a) {
        const double c = std::cos(G->angles[a]), s = std::sin(G->angles[a]);
        SfView &v = G->views[a];
        v.cd = c; v.sd = s;
        v.c = (float)c; v.s = (float)s;
        v.p = (float)(h * c); v.q = (float)(h * s);
        v.par_out = (float)(h * (std::fabs(c) + std::fabs(s)) / d->pixel_u);
        v.par_in = (float)(h * std::fabs(std::fabs(c) - std::fabs(s)) / d->pixel_u);
        v.par_amp = (float)(T / std::fmax(std::fabs(c), std::fabs(s)));
        v.xmajor = std::fabs(c) >= std::fabs(s) ? 1 : 0;
    }

    if (d->model == LEAP_MODEL_SIDDON) build_ray_table(G);
    select_fast_kernels(G);
    return finish_handle(G, out);
}

extern "C" void leap_geometry_destroy(leap_geometry *G) { free_handle(G); }

extern "C" int leap_geometry_describe(const leap_geometry *G, char *buf, int32_t cap)
{
    if (!G || !buf || cap <= 0) return invalid("null handle or buffer");
    char fwd[160], back[96];
    const bool siddon = G->g.model == SF_MODEL_SIDDON;
    if (siddon && G->sd_columns)
        std::snprintf(fwd, sizeof fwd, "columns(rg=%d,slab=%d)", G->fp_rg, G->slab_width);
    else if (!siddon && G->fp_columns)
        std::snprintf(fwd, sizeof fwd, "columns(nq=%d/%d,nkp=%d,rg=%d,cw=%d,slab=%d)", G->fp_need_q, G->fp_nq, G->fp_nkp,
                      G->fp_rg, G->fp_cw, G->slab_width);
    else
        std::snprintf(fwd, sizeof fwd, "general");
    if (G->bp_tiled && G->d_mdbp)
        std::snprintf(back, sizeof back, "tiled(zc=%d,window=%dx%d)", MD_BP_SHAPES[G->bp_shape].zc, G->bp_need_w, G->bp_need_h);
    else if (G->bp_tiled && siddon)
        std::snprintf(back, sizeof back, "tiled(nc=%d,zc=%d,window=%dx%d)", G->bp_nc, BP_SHAPES[G->bp_shape].zc, G->bp_need_w, G->bp_need_h);
    else if (G->bp_tiled)
        std::snprintf(back, sizeof back, "tiled(nc=%d,nv=%d,zc=%d,window=%dx%d)", G->bp_nc, G->bp_nv, BP_SHAPES[G->bp_shape].zc,
                      G->bp_need_w, G->bp_need_h);
    else
        std::snprintf(back, sizeof back, "general");
    const char *modules = G->g.type != SF_MODULAR ? "" : (G->geoms.empty() ? " (tilted modules)" : " (upright modules)");
    std::snprintf(buf, (size_t)cap, "type=%d model=%s A=%s AT=%s scratch=%zu%s cols/voxel<=%.2f rows/voxel<=%.2f voxels/row<=%.2f%s%s",
                  G->g.type, siddon ? "siddon" : "sf", fwd, back, G->scratch_bytes, modules, G->max_cols_per_voxel,
                  G->max_rows_per_voxel, G->max_voxels_per_row, G->note.empty() ? "" : " note=", G->note.c_str());
    return LEAP_OK;
}

static int check_call(const leap_geometry *G, const void *in, const void *out, int32_t batch)
{
    if (!G || !in || !out) return invalid("null handle or data pointer");
    if (batch <= 0) return invalid("batch must be positive");
    if (in == out) return invalid("input and output must not alias");
    return LEAP_OK;
}

extern "C" int leap_project(const leap_geometry *G, const float *d_vol, float *d_sino, int32_t batch, void *hip_stream)
{
    const int rc = check_call(G, d_vol, d_sino, batch);
    if (rc != LEAP_OK) return rc;
    return leap_launch_project_batch(G, d_vol, d_sino, batch, (hipStream_t)hip_stream);
}

extern "C" int leap_backproject(const leap_geometry *G, const float *d_sino, float *d_vol, int32_t batch, void *hip_stream)
{
    const int rc = check_call(G, d_sino, d_vol, batch);
    if (rc != LEAP_OK) return rc;
    return leap_launch_backproject_batch(G, d_sino, d_vol, batch, (hipStream_t)hip_stream);
}
