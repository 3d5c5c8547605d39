// Forward projection (A), ray-driven gather with wave-uniform footprints.
//
// Data layout.  The volume [z][y][x] is first copied into a z-fastest, zero-padded scratch array
//   volz[(j * nx + i) * nzp + FP_PAD + k],   nzp = nz + 2 FP_PAD,
// so that the voxels one ray bundle needs from a voxel column (i,j) are contiguous whatever the view
// angle.  This copy is the only scratch of the library that grows with the volume.
//
// Work split.  One 64-lane wavefront owns CW adjacent detector columns of one view and a band of RG * 64
// detector rows: lane l owns rows band0 + 64 g + l, g < RG, of each of its columns.  Because all lanes
// share (view, columns), the whole transaxial part of the weight (which voxel columns the pixels see, F_u,
// magnification) is the same for the 64 lanes, and the axial part (a row's overlaps with the voxels of a
// voxel column) is the same for the CW pixel columns: it is computed once and applied CW times.  The wave therefore computes it lane-parallel: per block of 64 / NQ slabs along
// the marching axis, lane (slab, slot) evaluates one candidate voxel column; a ballot picks the candidates
// with F_u > 0 and the wave then walks them one by one, broadcasting their few parameters through
// v_readlane, while each lane accumulates its own rows' axial overlaps from coalesced loads of volz.
// The waves of a workgroup are the same column bundle(s) in WV consecutive views: their beams overlap almost
// entirely, they start together and do equal work, so they share the volume through the CU's L1.
#pragma once

#include "sf_footprint.h"

constexpr int FP_PAD = 4;        // zero voxels before and after every z-column of the scratch copy

// Candidate voxel columns of pixel columns c .. c+cw-1 in slab n: in-plane lines through the two outer u-edges of
// the bundle, written as "minor index = m * major index + b".  Wave-uniform.
struct SfRayLines {
    float m0, b0, m1, b1, spread;
    int xmajor;
};

template <int GT = -1>
SF_HD SfRayLines sf_ray_lines(const SfGeom &g, const SfView &v, int c, int cw)
{
    SfRayLines L;
    const float ue0 = ((float)c - 0.5f - g.col_off) * g.pu, ue1 = ((float)(c + cw) - 0.5f - g.col_off) * g.pu;
    const float x0 = (float)g.x0d, y0 = (float)g.y0d;
    const float iT = 1.0f / g.T;
    if (g.type == SF_PARALLEL) {
        L.xmajor = fabsf(v.c) >= fabsf(v.s);
        if (L.xmajor) {            // -x s + y c = u  ->  y = (u + x s)/c
            L.m0 = L.m1 = v.s / v.c;
            L.b0 = (ue0 / v.c + x0 * L.m0 - y0) * iT;
            L.b1 = (ue1 / v.c + x0 * L.m1 - y0) * iT;
        } else {                   // x = (y c - u)/s
            L.m0 = L.m1 = v.c / v.s;
            L.b0 = (-ue0 / v.s + y0 * L.m0 - x0) * iT;
            L.b1 = (-ue1 / v.s + y0 * L.m1 - x0) * iT;
        }
    } else {
        const float uc = 0.5f * (ue0 + ue1);
        const float sx = g.sod * v.c, sy = g.sod * v.s;
        float dxc, dyc, dx0, dy0, dx1, dy1;
        if (sf_is_curved<GT>(g)) {      // u is arc length: directions at the fan angles u / sdd
            float sg, cg;
            sincosf(uc / g.sdd, &sg, &cg);
            dxc = -fmaf(cg, v.c, sg * v.s); dyc = fmaf(sg, v.c, -cg * v.s);
            sincosf(ue0 / g.sdd, &sg, &cg);
            dx0 = -fmaf(cg, v.c, sg * v.s); dy0 = fmaf(sg, v.c, -cg * v.s);
            sincosf(ue1 / g.sdd, &sg, &cg);
            dx1 = -fmaf(cg, v.c, sg * v.s); dy1 = fmaf(sg, v.c, -cg * v.s);
        } else {
            dxc = fmaf(-g.sdd, v.c, -uc * v.s); dyc = fmaf(-g.sdd, v.s, uc * v.c);
            dx0 = fmaf(-g.sdd, v.c, -ue0 * v.s); dy0 = fmaf(-g.sdd, v.s, ue0 * v.c);
            dx1 = fmaf(-g.sdd, v.c, -ue1 * v.s); dy1 = fmaf(-g.sdd, v.s, ue1 * v.c);
        }
        L.xmajor = fabsf(dxc) >= fabsf(dyc);
        if (L.xmajor) {
            L.m0 = dy0 / dx0;
            L.m1 = dy1 / dx1;
            L.b0 = (sy - y0 + (x0 - sx) * L.m0) * iT;
            L.b1 = (sy - y0 + (x0 - sx) * L.m1) * iT;
        } else {
            L.m0 = dx0 / dy0;
            L.m1 = dx1 / dy1;
            L.b0 = (sx - x0 + (y0 - sy) * L.m0) * iT;
            L.b1 = (sx - x0 + (y0 - sy) * L.m1) * iT;
        }
    }
    L.spread = 0.5f * fmaxf(fabsf(L.m0), fabsf(L.m1)) + 2e-3f;
    return L;
}

// First and last candidate (minor index, unclipped) in slab n.
SF_HD void sf_candidates(const SfRayLines &L, int n, int &q_first, int &q_last)
{
    const float qa = fmaf(L.m0, (float)n, L.b0), qb = fmaf(L.m1, (float)n, L.b1);
    q_first = (int)floorf(fminf(qa, qb) - L.spread + 0.5f);
    q_last = (int)floorf(fmaxf(qa, qb) + L.spread + 0.5f);
}

#if defined(__HIPCC__) && !defined(SF_NO_KERNELS)

// vol [nz][ny][nx]  ->  volz [(j nx + i) nzp + FP_PAD + k].  Block 32 x 8 threads, tile 32 (i) x 32 (k) of one j.
__global__ __launch_bounds__(256) void sf_volume_to_columns(const float *__restrict__ vol, float *__restrict__ volz, int nx,
                                                            int ny, int nz, int nzp)
{
    __shared__ float tile[32][33];
    // blockIdx.z = j + ny * item: several volumes of a batch go into consecutive scratch copies in one launch
    const int item = blockIdx.z / ny, j = blockIdx.z - item * ny;
    vol += (size_t)item * nx * ny * nz;
    volz += (size_t)item * ((size_t)nx * ny + 1) * nzp;
    const int i0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
    const int tx = threadIdx.x, ty = threadIdx.y;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int k = k0 + ty + 8 * s, i = i0 + tx;
        tile[ty + 8 * s][tx] = (k < nz && i < nx) ? vol[((size_t)k * ny + j) * nx + i] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int i = i0 + ty + 8 * s, k = k0 + tx;
        if (i < nx && k < nz) volz[((size_t)j * nx + i) * nzp + FP_PAD + k] = tile[tx][ty + 8 * s];
    }
}

// NQ: candidate slots per slab (power of two <= 64); NK: voxels a detector row can overlap; RG: row groups per wave;
// FP_WAVES: waves per workgroup; CW: adjacent detector columns per wave; WV: consecutive views per workgroup
// (the workgroup's waves are WV views x FP_WAVES/WV column bundles); GT: 0 flat or parallel, 1 cylindrical detector.
template <int NQ, int NK, int RG, int FP_WAVES, int CW, int WV, int GT>
__global__ __launch_bounds__(FP_WAVES * 64) void sf_project_columns(SfGeom gk, const SfView *__restrict__ views,
                                                                    const float *__restrict__ volz, float *__restrict__ sino,
                                                                    int nzp, int col_tiles, int bands, int vb, int tb,
                                                                    int vgroups_pad, int tiles_per_xcd_pad,
                                                                    const SfGeom *__restrict__ geoms)
{
    // GT == 2 (modular geometry, upright modules): the wave's view brings its own parameter block, the scene
    // translated so that the view is a circular cone-beam view; gk holds the sizes, which all views share.
    const SfGeom &gsz = gk;
    // blockIdx.y: item of a batch (its scratch copy and its sinogram)
    volz += (size_t)blockIdx.y * ((size_t)gk.nx * gk.ny + 1) * nzp;
    sino += (size_t)blockIdx.y * gk.nviews * gk.nrows * gk.ncols;
    constexpr int SB = 64 / NQ;                       // slabs per record block
    constexpr int WC = FP_WAVES / WV;                 // column bundles per workgroup
    static_assert(WC * WV == FP_WAVES, "waves = column bundles x views");

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wv = wave % WV, wc = wave / WV;
    // Block -> (group of WV consecutive views, band, column tile).  The WV x WC waves of a workgroup start together and
    // do the same amount of work, so they march through the volume in step: the beams of one column tile in WV
    // neighbouring views overlap almost entirely and are shared in the CU's L1.  Workgroups are handed to the 8 XCDs
    // round-robin by index, and each XCD has its own L2, so the blocks one XCD runs at the same time are arranged as
    // (a few column tiles) x (a run of consecutive view groups): index = 8 s + xcd, and within an XCD's sequence s the
    // view group runs fastest inside a block of VB groups, then TB tiles, then blocks of view groups.
    int ct, band, a;
    {
        const int xcd = blockIdx.x & 7, sq = blockIdx.x >> 3;
        const int per_chunk = tb * vgroups_pad;                 // TB tiles x all (padded) view groups
        const int chunk = sq / per_chunk, r = sq - chunk * per_chunk;
        const int vblk = r / (tb * vb), r2 = r - vblk * (tb * vb);
        const int tloc = r2 / vb, v_in = r2 - tloc * vb;
        const int tchunks = tiles_per_xcd_pad / tb;
        band = chunk / tchunks;
        ct = ((chunk - band * tchunks) * tb + tloc) * 8 + xcd;
        a = (vblk * vb + v_in) * WV + wv;
        if (ct >= col_tiles || a >= gsz.nviews || band >= bands) return;   // padding blocks and padding views (no barrier follows)
    }
    const int c0 = (ct * WC + wc) * CW;                  // first detector column of this wave
    const int band0 = band * (RG * 64);

    const SfGeom &g = GT == 2 ? geoms[a] : gk;
    const SfView v = views[a];
    const SfRayLines L = sf_ray_lines<GT>(g, v, c0, CW);
    const int n_major = L.xmajor ? g.nx : g.ny;
    const int n_minor = L.xmajor ? g.ny : g.nx;

    // this lane's rows as doubles relative to the detector's eta origin, and the constant of the kappa map
    double rd[RG];
#pragma unroll
    for (int gq = 0; gq < RG; ++gq) rd[gq] = (double)(band0 + 64 * gq + lane) - g.row_offd;
    const double zkp = -g.zlo0d * g.iTzd + (double)FP_PAD;   // kappa + pad offset
    const int kmax = g.nz + FP_PAD;
    const double mu_scale = g.ikvd * g.iTzd;          // kappa(r) = (r - row_off) * den * mu_scale - zlo0 / Tz

    float acc[CW][RG];
#pragma unroll
    for (int cw = 0; cw < CW; ++cw)
#pragma unroll
        for (int gq = 0; gq < RG; ++gq) acc[cw][gq] = 0.0f;

    const int slot = lane & (NQ - 1), nrel = lane / NQ;

    for (int nb = 0; nb < n_major; nb += SB) {
        // ---- lane-parallel: one candidate voxel column per lane
        const int n = nb + nrel;
        int qf, ql;
        sf_candidates(L, n, qf, ql);
        const int q = qf + slot;
        const bool valid = n < n_major && q >= 0 && q < n_minor && q <= ql;
        const int i = L.xmajor ? n : q, j = L.xmajor ? q : n;
        const int ic = valid ? i : 0, jc = valid ? j : 0;
        const SfColumn f = sf_column<GT>(g, v, ic, jc);
        const double mu = f.den * mu_scale;                       // voxels per detector row at this column
        const float rows_per_voxel = (float)(g.kvd * f.inv * g.Tzd);
        float fa[CW];                                              // F_u times rows per voxel, per detector column
        bool any = false;
        {
            float e = sf_pixel_edge(f, c0);
            float g0 = sf_trap_integral(f, e);
#pragma unroll
            for (int cw = 0; cw < CW; ++cw) {
                e += 1.0f;
                const float g1 = sf_trap_integral(f, e);
                const float fu = (valid && c0 + cw < g.ncols) ? fmaxf(g1 - g0, 0.0f) : 0.0f;
                fa[cw] = fu * rows_per_voxel;
                any = any || fu > 0.0f;
                g0 = g1;
            }
        }
        const unsigned colbase = (unsigned)(jc * g.nx + ic) * (unsigned)nzp;   // start of the padded column
        const int mu_lo = __double2loint(mu), mu_hi = __double2hiint(mu);

        unsigned long long mask = __ballot(any);
        // ---- wave-uniform walk over the candidates that matter
        while (mask) {
            const int e = __builtin_ctzll(mask);
            mask &= mask - 1;
            float s_fa[CW];
#pragma unroll
            for (int cw = 0; cw < CW; ++cw)
                s_fa[cw] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, fa[cw]), e));
            const unsigned s_base = (unsigned)__builtin_amdgcn_readlane((int)colbase, e);
            const double s_mu = __hiloint2double(__builtin_amdgcn_readlane(mu_hi, e), __builtin_amdgcn_readlane(mu_lo, e));
            const float step = (float)s_mu;
            float step_minus[NK];
#pragma unroll
            for (int t = 1; t < NK; ++t) step_minus[t] = step - (float)t;
            const char *__restrict__ col = reinterpret_cast<const char *>(volz + s_base);   // wave-uniform base address
            // Addresses, loads, arithmetic.  Left alone, the compiler schedules a few instances as load - wait - use,
            // load - wait - use (its register-pressure heuristics give up on keeping RG loads in flight), and they run
            // at a third of the speed: those get scheduling barriers between the three phases.  The others are faster
            // without (1 to 2 % at 512^3), so they keep the compiler's own schedule.
            constexpr bool PIN = (GT == 1 && CW == 4) || (NK == 4 && RG == 8 && CW == 4);
            float fr[RG];
            const float *xp[RG];
#pragma unroll
            for (int gq = 0; gq < RG; ++gq) {
                // kappa measured from the start of the padded column; negative values only occur inside the pad
                const double kap = fma(rd[gq], s_mu, zkp);
                fr[gq] = (float)__builtin_amdgcn_fract(kap);
                int kf = (int)kap;                                 // truncation = floor wherever the clamp leaves it alone
                asm("v_med3_i32 %0, %1, 0, %2" : "=v"(kf) : "v"(kf), "s"(kmax));   // clamp to [0, kmax] in one op
                xp[gq] = reinterpret_cast<const float *>(col + ((unsigned)kf << 2));
            }
            if constexpr (PIN) __builtin_amdgcn_sched_barrier(0);
            float xv[RG][NK];
#pragma unroll
            for (int gq = 0; gq < RG; ++gq)
#pragma unroll
                for (int t = 0; t < NK; ++t) xv[gq][t] = xp[gq][t];
            if constexpr (PIN) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int gq = 0; gq < RG; ++gq) {
                // Overlaps of [kap, kap + step) with voxels kf, kf+1, ...: voxel kf+t, t >= 1, gets clamp(fr + step - t)
                // and voxel kf the rest of step, so the sum is step * x[0] plus the differences to x[0] times those
                // overlaps (additions with the clamp modifier issue at twice the rate of min / max).
                float s = step * xv[gq][0];
#pragma unroll
                for (int t = 1; t < NK; ++t) s = fmaf(sf_clamp(fr[gq] + step_minus[t], 0.0f, 1.0f), xv[gq][t] - xv[gq][0], s);
#pragma unroll
                for (int cw = 0; cw < CW; ++cw) acc[cw][gq] = fmaf(s_fa[cw], s, acc[cw][gq]);
            }
        }
    }

    // ---- amplitude and store: CW consecutive floats per lane and row, written together (storing the columns of a
    // bundle one after the other, hundreds of instructions apart, cost 3.7 times the sinogram in partial-line writes)
    float *__restrict__ ya = sino + (size_t)a * g.nrows * g.ncols;
    SfAmpCol ac[CW];
#pragma unroll
    for (int cw = 0; cw < CW; ++cw) ac[cw] = sf_amp_col<GT>(g, v, c0 + cw < g.ncols ? c0 + cw : g.ncols - 1);
    struct __attribute__((packed, aligned(4))) Pair { float lo, hi; };
    struct __attribute__((packed, aligned(4))) Quad { float a, b, c, d; };
#pragma unroll
    for (int gq = 0; gq < RG; ++gq) {
        const int r = band0 + 64 * gq + lane;
        if (r >= g.nrows) continue;
        float out[CW];
#pragma unroll
        for (int cw = 0; cw < CW; ++cw) out[cw] = sf_amp(g, v, ac[cw], r) * acc[cw][gq];
        float *__restrict__ dst = ya + (size_t)r * g.ncols + c0;
        if constexpr (CW == 2) {
            if (c0 + 1 < g.ncols) {
                Pair pr;
                pr.lo = out[0]; pr.hi = out[1];
                *reinterpret_cast<Pair *>(dst) = pr;
                continue;
            }
        }
        if constexpr (CW == 4) {
            if (c0 + 3 < g.ncols) {
                Quad qd;
                qd.a = out[0]; qd.b = out[1]; qd.c = out[2]; qd.d = out[3];
                *reinterpret_cast<Quad *>(dst) = qd;
                continue;
            }
        }
#pragma unroll
        for (int cw = 0; cw < CW; ++cw)
            if (c0 + cw < g.ncols) dst[cw] = out[cw];
    }
}

#endif
