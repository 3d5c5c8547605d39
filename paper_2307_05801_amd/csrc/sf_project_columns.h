// Forward projection (A), ray-driven gather with wave-uniform footprints.
//
// Data layout.  The kernel reads a z-fastest, zero-padded scratch copy of a SLAB of the volume: the voxel columns (i, j)
// whose index along the slab's axis lies in [n0, n0 + width),
//   volz[col * nzp + FP_PAD + k],   nzp = nz + 2 FP_PAD,   col = (j - j0) * ni + (i - i0),
// so that the voxels a ray bundle needs from a voxel column are contiguous whatever the view angle.  A slab across x
// (i0 = n0, ni = width, j0 = 0) serves the ray bundles that advance fastest along x, a slab across y (j0 = n0, ni = nx,
// i0 = 0) those that advance fastest along y; the host walks the volume slab by slab, and every bundle adds the slab's
// share to its sinogram samples (the first slab of its kind overwrites).  The scratch therefore holds a fraction of
// the volume, chosen by the host.
//
// Work split.  One 64-lane wavefront owns CW adjacent detector columns of one view and a band of RG * 128 detector
// rows: lane l owns the row PAIRS band0 + 128 g + 2 l + {0, 1}, g < RG, of each of its columns.  Because all lanes share
// (view, columns), the whole transaxial part of the weight (which voxel columns the pixels see, F_u, magnification) is
// the same for the 64 lanes, and the axial part (a row's overlaps with the voxels of a voxel column) is the same for
// the CW pixel columns: it is computed once and applied CW times.  The wave therefore computes the transaxial part
// lane-parallel: per block of 64 / nq slabs along the marching axis, lane (slab, slot) evaluates one candidate voxel
// column; a ballot picks the candidates with F_u > 0 and the wave then walks them one by one, reading a candidate's
// record back from LDS at a wave-uniform address (and the two numbers that must be scalar through v_readlane), while
// each lane accumulates its own rows' axial overlaps.
//
// Two adjacent rows per lane, one load.  The vector cache serves a wave-wide load at four lanes per clock whether a
// lane asks for 4 or for 16 bytes (measured), and two adjacent rows overlap in the voxels they need.  One load of P
// consecutive voxels starting at the voxel of the lower row's lower edge serves both rows of a pair: half the cache
// time and half the placement arithmetic of one load per row.
//
// Placement without conversions.  kappa, the axial voxel coordinate of a row's lower edge, is formed by one double
// FMA to which 1.5 * 2^20 has been added: the sum's unit in the last place is 2^-32, so its low word is kappa's
// fraction and the low bits of its high word are floor(kappa) -- no floor, no conversion, no clamp.  The loads are
// raw buffer loads on a descriptor of the candidate's own padded z-column: whatever lies outside it reads as zero,
// which is the truncation rule for rows that miss the volume.
#pragma once

#include "sf_footprint.h"

#include <type_traits>

constexpr int FP_PAD = 8;        // zero voxels before and after every z-column of the scratch copy (>= the voxels a row pair spans)
constexpr int FP_MAX_P = 7;      // most voxels a pair of adjacent rows may overlap (rows of up to 3 voxels)

// Candidate voxel columns of pixel columns c .. c+cw-1 in slab n: in-plane lines through the two outer u-edges of
// the bundle, written as "minor index = m * major index + b".  Wave-uniform.
struct SfRayLines {
    float m0, b0, m1, b1, spread;
    int xmajor;
};

// want_major: -1 picks the marching axis from the bundle's central ray, 0 / 1 forces y / x (the kernel takes the host's
// choice, so that both agree on which slabs a bundle reads even where the two directions tie).
template <int GT = -1>
SF_HD SfRayLines sf_ray_lines(const SfGeom &g, const SfView &v, int c, int cw, int want_major = -1)
{
    SfRayLines L;
    const float ue0 = ((float)c - 0.5f - g.col_off) * g.pu, ue1 = ((float)(c + cw) - 0.5f - g.col_off) * g.pu;
    const float x0 = (float)g.x0d, y0 = (float)g.y0d;
    const float iT = 1.0f / g.T;
    if (g.type == SF_PARALLEL) {
        L.xmajor = want_major < 0 ? (int)(fabsf(v.c) >= fabsf(v.s)) : want_major;
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
        L.xmajor = want_major < 0 ? (int)(fabsf(dxc) >= fabsf(dyc)) : want_major;
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

// One slab of the volume as the scratch copy holds it.
struct SfSlab {
    int n0, n1;       // slab indices [n0, n1) along the marching axis
    int xmajor;       // 1: the slab cuts x (serves bundles that advance fastest along x), 0: it cuts y
    int first;        // 1: bundles overwrite their sinogram samples, 0: they add to them
    int width;        // slabs the scratch layout is built for (>= n1 - n0)
};

// Index of voxel column (i, j) among the columns of the slab's scratch copy.
SF_HD unsigned sf_slab_column(const SfSlab &s, int nx, int i, int j)
{
    return s.xmajor ? (unsigned)(j * s.width + (i - s.n0)) : (unsigned)((j - s.n0) * nx + i);
}

// ---- the arithmetic of one lane, shared by the kernel and by the CPU test harness that steps it -----------------------

// Constant of the kappa map: kappa(r) = (r - row_off) mu + zkp is measured from the start of the padded column and
// carries FP_KAP_MAGIC = 1.5 * 2^20 plus half a unit of the 23-bit fraction used below (so that truncating rounds).
constexpr double FP_KAP_MAGIC = 1572864.0;
constexpr unsigned FP_KAP_HI = 0x41380000u;      // high word of FP_KAP_MAGIC: high word of the sum = FP_KAP_HI + floor(kappa)
SF_HD double sf_kappa_const(const SfGeom &g) { return -g.zlo0d * g.iTzd + (double)FP_PAD + FP_KAP_MAGIC + 5.9604644775390625e-08; }

// Lower edge of a row in its candidate column: rd = row - row_off, mu = voxels per row.  fr1 = 1 + the edge's fraction
// inside its voxel (a float in [1, 2) assembled from the sum's bits), hi = FP_KAP_HI + that voxel's index.
SF_HD void sf_place_row(double rd, double mu, double zkp, float &fr1, unsigned &hi)
{
    const double kap = fma(rd, mu, zkp);
    unsigned long long bits;
    __builtin_memcpy(&bits, &kap, 8);
    const unsigned lo = (unsigned)bits;
    hi = (unsigned)(bits >> 32);
#if defined(__HIP_DEVICE_COMPILE__)
    fr1 = __builtin_bit_cast(float, __builtin_amdgcn_alignbit(0x7fu, lo, 9));
#else
    const unsigned f = (0x7fu << 23) | (lo >> 9);
    __builtin_memcpy(&fr1, &f, 4);
#endif
}

// Voxels a row can overlap when a pair of rows overlaps P: rows of up to (P - 1) / 2 voxels.
constexpr int sf_single_of_pair(int P) { return P / 2 + 1; }

// Axial sums of a pair of adjacent rows.  x[0..P-1]: voxels from the one holding the lower row's lower edge; fr1 as
// above; step = voxels per row, fr + 2 step <= P.  The lower row A covers [fr, fr + step) of that run, the upper row B
// [fr + step, fr + 2 step).  With a_t = clamp(fr + step - t), b_t = clamp(fr + 2 step - t) and d_t = x_t - x_0 (t >= 1):
//   S_A = step x_0 + sum a_t d_t,    S_B = 2 step x_0 + sum b_t d_t - S_A
// (voxel 0 gets what the others leave of each row; additions with the clamp modifier are the cheapest way to an overlap).
// What sf_pair_sums needs of a candidate besides the voxels: step and the offsets of the clamps, ka[t-1] = step - (t+1)
// for 1 <= t < NK (NK = sf_single_of_pair(P)) and kb[t-1] = 2 step - (t+1) for 1 <= t < P.  The same for every row
// of the detector, so the forward kernel works them out once per candidate, lane-parallel.
template <int P>
struct SfPairConsts {
    float step;
    float ka[sf_single_of_pair(P) > 1 ? sf_single_of_pair(P) - 1 : 1];
    float kb[P > 1 ? P - 1 : 1];
};

template <int P>
SF_HD SfPairConsts<P> sf_pair_consts(float step)
{
    constexpr int NK = sf_single_of_pair(P);
    SfPairConsts<P> k;
    k.step = step;
    const float step2 = step + step;
#pragma unroll
    for (int t = 1; t < NK && t < P; ++t) k.ka[t - 1] = step - (float)(t + 1);
#pragma unroll
    for (int t = 1; t < P; ++t) k.kb[t - 1] = step2 - (float)(t + 1);
    return k;
}

template <int P>
SF_HD void sf_pair_sums(const float (&x)[P], float fr1, const SfPairConsts<P> &k, float &sa, float &sb)
{
    constexpr int NK = sf_single_of_pair(P);
    float d[P];
#pragma unroll
    for (int t = 1; t < P; ++t) d[t] = x[t] - x[0];
    const float a0 = k.step * x[0];
    float a = a0;
#pragma unroll
    for (int t = 1; t < NK && t < P; ++t) a = fmaf(sf_clamp(fr1 + k.ka[t - 1], 0.0f, 1.0f), d[t], a);
    float b = a0 + a0;                              // 2 step x_0, exactly
#pragma unroll
    for (int t = 1; t < P; ++t) b = fmaf(sf_clamp(fr1 + k.kb[t - 1], 0.0f, 1.0f), d[t], b);
    sa = a;
    sb = b - a;
}

// Transaxial record of one candidate voxel column (i, j) for the bundle of CW detector columns starting at c0:
// fa[cw] = F_u times rows per voxel, mu = voxels per detector row; returns whether any column is touched.
template <int CW, int GT>
SF_HD bool sf_candidate_record(const SfGeom &g, const SfView &v, int i, int j, int c0, bool valid, float (&fa)[CW], double &mu)
{
    const SfColumn f = sf_column<GT>(g, v, i, j);
    mu = f.den * (g.ikvd * g.iTzd);
    const float rows_per_voxel = (float)(g.kvd * f.inv * g.Tzd);
    bool any = false;
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
    return any;
}

#if defined(__HIPCC__) && !defined(SF_NO_KERNELS)

// vol [nz][ny][nx]  ->  the slab's scratch copy: columns (i, j), i0 <= i < i0 + ni, j0 <= j < j0 + nj, at
// volz[((j - j0) ni + (i - i0)) nzp + FP_PAD + k].  Block 32 x 8 threads, tile 32 (i) x 32 (k) of one j.
// blockIdx.z = (j - j0) + nj * item: several volumes of a batch go into consecutive scratch copies in one launch.
__global__ __launch_bounds__(256) void sf_volume_to_columns(const float *__restrict__ vol, float *__restrict__ volz, int nx,
                                                            int ny, int nz, int nzp, int i0, int j0, int ni, int nj,
                                                            size_t item_stride)
{
    __shared__ float tile[32][33];
    const int item = blockIdx.z / nj, jr = blockIdx.z - item * nj, j = j0 + jr;
    vol += (size_t)item * nx * ny * nz;
    volz += (size_t)item * item_stride;
    const int ib = blockIdx.x * 32, k0 = blockIdx.y * 32;
    const int tx = threadIdx.x, ty = threadIdx.y;
    const int ihi = i0 + ni < nx ? i0 + ni : nx;
    if (j >= ny) return;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int k = k0 + ty + 8 * s, i = i0 + ib + tx;
        tile[ty + 8 * s][tx] = (k < nz && i < ihi) ? vol[((size_t)k * ny + j) * nx + i] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int ir = ib + ty + 8 * s, k = k0 + tx;
        if (i0 + ir < ihi && k < nz) volz[((size_t)jr * ni + ir) * nzp + FP_PAD + k] = tile[tx][ty + 8 * s];
    }
}

// Zeroes what the column-wise kernels expect to be zero around the voxels that sf_volume_to_columns writes: FP_PAD
// floats before and after each of the ncolumns z-columns and the whole spare column that follows them (a fill kernel,
// not a memset, so that a caller may capture the call in a graph).
__global__ __launch_bounds__(256) void sf_clear_column_pads(float *__restrict__ volz, unsigned ncolumns, int nz, int nzp)
{
    const unsigned t = blockIdx.x * 256u + threadIdx.x;
    const unsigned col = t / (2u * FP_PAD), e = t % (2u * FP_PAD);
    if (col < ncolumns) volz[(size_t)col * nzp + (e < FP_PAD ? e : nz + e)] = 0.0f;
    if (t < (unsigned)nzp) volz[(size_t)ncolumns * nzp + t] = 0.0f;
}

constexpr int FP_WAVES = 4;      // waves per workgroup: adjacent column bundles of one view (each wave its own LDS, no barrier)

// NKP: voxels a pair of adjacent rows can overlap (2 .. FP_MAX_P); RG: groups of 128 rows per wave; CW: adjacent detector
// columns per wave; GT: 0 flat or parallel, 1 cylindrical detector, 2 modular geometry with upright modules.
// (The cylinder's record phase needs more registers: its instances are held to the waves per SIMD they reach without
// the records' staging, four up to two row groups, three beyond.)
// nq_log2: log2 of the candidate slots per slab (a power of two <= 64).  major[a * nbundles + b]: 1 if bundle b of view
// a advances fastest along x (decided once, on the host, so that both agree on which slabs a bundle reads).
template <int NKP, int RG, int CW, int GT>
__global__ __launch_bounds__(FP_WAVES * 64, GT == 1 ? (RG <= 2 ? 4 : 3) : 1) void sf_project_columns(SfGeom gk, const SfView *__restrict__ views,
                                                                    const float *__restrict__ volz, float *__restrict__ sino,
                                                                    const unsigned char *__restrict__ major, int nzp,
                                                                    size_t item_stride, int nq_log2, int col_tiles, int bands,
                                                                    int vb, int tb, int vgroups_pad, int tiles_per_xcd_pad,
                                                                    SfSlab slab, const SfGeom *__restrict__ geoms)
{
    // GT == 2 (modular geometry, upright modules): the wave's view brings its own parameter block, the scene
    // translated so that the view is a circular cone-beam view; gk holds the sizes, which all views share.
    const SfGeom &gsz = gk;
    // blockIdx.y: item of a batch (its scratch copy and its sinogram)
    volz += (size_t)blockIdx.y * item_stride;
    sino += (size_t)blockIdx.y * gk.nviews * gk.nrows * gk.ncols;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Block -> (view, band, column tile).  Workgroups are handed to the 8 XCDs round-robin by index, and each XCD has
    // its own L2, so the blocks one XCD runs at the same time are arranged as (a few column tiles) x (a run of
    // consecutive views), whose beams overlap almost entirely: index = 8 s + xcd, and within an XCD's sequence s the
    // view runs fastest inside a block of VB views, then TB tiles, then blocks of views.
    int ct, band, a;
    {
        const int xcd = blockIdx.x & 7, sq = blockIdx.x >> 3;
        const int per_chunk = tb * vgroups_pad;                 // TB tiles x all (padded) views
        const int chunk = sq / per_chunk, r = sq - chunk * per_chunk;
        const int vblk = r / (tb * vb), r2 = r - vblk * (tb * vb);
        const int tloc = r2 / vb, v_in = r2 - tloc * vb;
        const int tchunks = tiles_per_xcd_pad / tb;
        band = chunk / tchunks;
        ct = ((chunk - band * tchunks) * tb + tloc) * 8 + xcd;
        a = vblk * vb + v_in;
        if (ct >= col_tiles || a >= gsz.nviews || band >= bands) return;   // padding blocks and padding views (no barrier follows)
    }
    const int bundle = ct * FP_WAVES + wave;
    const int c0 = bundle * CW;                          // first detector column of this wave
    if (c0 >= gsz.ncols) return;
    const int nbundles = (gsz.ncols + CW - 1) / CW;
    if ((int)major[(size_t)a * nbundles + bundle] != slab.xmajor) return;   // this bundle reads the other kind of slab
    const int band0 = band * (RG * 128);

    const SfGeom &g = GT == 2 ? geoms[a] : gk;
    const SfView v = views[a];
    const SfRayLines L = sf_ray_lines<GT>(g, v, c0, CW, slab.xmajor);
    const int n_minor = slab.xmajor ? g.ny : g.nx;

    // the lower row of each of this lane's pairs, as a double relative to the detector's eta origin
    double rd[RG];
#pragma unroll
    for (int gq = 0; gq < RG; ++gq) rd[gq] = (double)(band0 + 128 * gq + 2 * lane) - g.row_offd;
    const double zkp = sf_kappa_const(g);
    // byte offset of voxel floor(kappa) in its column from the high word: (hi << 2) + off_k (mod 2^32); negative
    // kappa wraps to a huge offset, which the buffer load's range check turns into zeros, like kappa beyond the column
    const unsigned off_k = 0u - (FP_KAP_HI << 2);
    const unsigned col_bytes = (unsigned)nzp * 4u;

    float acc[CW][RG][2];
#pragma unroll
    for (int cw = 0; cw < CW; ++cw)
#pragma unroll
        for (int gq = 0; gq < RG; ++gq) acc[cw][gq][0] = acc[cw][gq][1] = 0.0f;

    const int slot = lane & ((1 << nq_log2) - 1), nrel = lane >> nq_log2, sb_slabs = 64 >> nq_log2;

    // What a candidate's visit needs as plain vector operands (the CW column factors, step and the clamp offsets of the
    // four-voxel body) goes through LDS: every lane writes its candidate's record, the wave reads the record of the
    // candidate it visits back at a uniform address, which the LDS serves as a broadcast without touching the vector
    // ALU (a v_readlane costs as much issue time as two and a half FMAs; the kernel is bound by that issue time).
    // Only what must sit in scalar registers still comes by v_readlane: the column's offset (buffer descriptor) and mu
    // (scalar operand of the placement FMAs).
    constexpr int PB = NKP > 4 ? 4 : NKP;           // the body most candidates take
    constexpr int FP_REC = 3;                       // float4s per record
    __shared__ float4 recs[FP_WAVES][64][FP_REC];
    float4 (*rec)[FP_REC] = recs[wave];

    for (int nb = slab.n0; nb < slab.n1; nb += sb_slabs) {
        // ---- lane-parallel: one candidate voxel column per lane
        const int n = nb + nrel;
        int qf, ql;
        sf_candidates(L, n, qf, ql);
        const int q = qf + slot;
        const bool valid = n < slab.n1 && q >= 0 && q < n_minor && q <= ql;
        const int i = slab.xmajor ? n : q, j = slab.xmajor ? q : n;
        const int ic = valid ? i : (slab.xmajor ? slab.n0 : 0), jc = valid ? j : (slab.xmajor ? 0 : slab.n0);
        float fa[CW];                                              // F_u times rows per voxel, per detector column
        double mu;                                                 // voxels per detector row at this column
        const bool any = sf_candidate_record<CW, GT>(g, v, ic, jc, c0, valid, fa, mu);
        const unsigned colbase = sf_slab_column(slab, g.nx, ic, jc) * (unsigned)nzp;   // start of the padded column
        const int mu_lo = __double2loint(mu), mu_hi = __double2hiint(mu);
        const float muf = (float)mu;
        {
            const SfPairConsts<PB> k = sf_pair_consts<PB>(muf);
            float w[4 * FP_REC];
#pragma unroll
            for (int t = 0; t < 4 * FP_REC; ++t) w[t] = 0.0f;
#pragma unroll
            for (int cw = 0; cw < CW; ++cw) w[cw] = fa[cw];
            w[4] = k.step;
#pragma unroll
            for (int t = 0; t < sf_single_of_pair(PB) - 1; ++t) w[5 + t] = k.ka[t];
#pragma unroll
            for (int t = 0; t < PB - 1; ++t) w[8 + t] = k.kb[t];
            // (the wave has consumed every value it read from the previous block's records)
#pragma unroll
            for (int t = 0; t < FP_REC; ++t) rec[lane][t] = make_float4(w[4 * t], w[4 * t + 1], w[4 * t + 2], w[4 * t + 3]);
            // the records are read by the other lanes of this wave only: order the LDS accesses, no barrier
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }

        unsigned long long mask = __ballot(any);
        unsigned long long touch[CW];                              // candidates that touch detector column cw
#pragma unroll
        for (int cw = 0; cw < CW; ++cw) touch[cw] = __ballot(fa[cw] != 0.0f);
        // most candidates of a scan with NKP > 4 still fit four voxels per pair: one 16-byte load per pair
        const unsigned long long wide = NKP > 4 ? __ballot(!(muf <= 1.4999f)) : 0ull;
        // ---- wave-uniform walk over the candidates that matter
        auto pairs = [&](auto pc, int e, const float (&r)[4 * FP_REC], float (&sa)[RG], float (&sb)[RG]) {
            constexpr int P = decltype(pc)::value;
            const unsigned s_base = (unsigned)__builtin_amdgcn_readlane((int)colbase, e);
            const double s_mu = __hiloint2double(__builtin_amdgcn_readlane(mu_hi, e), __builtin_amdgcn_readlane(mu_lo, e));
            SfPairConsts<P> k;
            if constexpr (P == PB) {
                k.step = r[4];
#pragma unroll
                for (int t = 0; t < sf_single_of_pair(P) - 1; ++t) k.ka[t] = r[5 + t];
#pragma unroll
                for (int t = 0; t < P - 1; ++t) k.kb[t] = r[8 + t];
            } else {
                k = sf_pair_consts<P>(r[4]);
            }
            // buffer resource of this candidate's padded z-column: loads beyond it return zero
            const __amdgpu_buffer_rsrc_t col = __builtin_amdgcn_make_buffer_rsrc((void *)(volz + s_base), 0, (int)col_bytes, 0x00020000);
            float fr1[RG];
            unsigned ko[RG];
#pragma unroll
            for (int gq = 0; gq < RG; ++gq) {
                unsigned hi;
                sf_place_row(rd[gq], s_mu, zkp, fr1[gq], hi);
                asm("v_lshl_add_u32 %0, %1, 2, %2" : "=v"(ko[gq]) : "v"(hi), "s"(off_k));
            }
            float xv[RG][P];
#pragma unroll
            for (int gq = 0; gq < RG; ++gq)
#pragma unroll
                for (int t = 0; t < P; ++t)      // the compiler merges these into loads of up to 16 bytes
                    xv[gq][t] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(col, (int)ko[gq] + 4 * t, 0, 0));
#pragma unroll
            for (int gq = 0; gq < RG; ++gq) sf_pair_sums<P>(xv[gq], fr1[gq], k, sa[gq], sb[gq]);
        };
        while (mask) {
            const int e = __builtin_ctzll(mask);
            mask &= mask - 1;
            float r[4 * FP_REC];
#pragma unroll
            for (int t = 0; t < FP_REC; ++t) {
                const float4 q4 = rec[e][t];
                r[4 * t] = q4.x; r[4 * t + 1] = q4.y; r[4 * t + 2] = q4.z; r[4 * t + 3] = q4.w;
            }
            float sa[RG], sb[RG];
            if constexpr (NKP > 4) {
                if (!((wide >> e) & 1ull)) pairs(std::integral_constant<int, 4>{}, e, r, sa, sb);
                else pairs(std::integral_constant<int, NKP>{}, e, r, sa, sb);
            } else {
                pairs(std::integral_constant<int, NKP>{}, e, r, sa, sb);
            }
            // a candidate usually touches only some of the bundle's columns: skip the others (wave-uniform branches)
#pragma unroll
            for (int cw = 0; cw < CW; ++cw) {
                if ((touch[cw] >> e) & 1ull) {
#pragma unroll
                    for (int gq = 0; gq < RG; ++gq) {
                        acc[cw][gq][0] = fmaf(r[cw], sa[gq], acc[cw][gq][0]);
                        acc[cw][gq][1] = fmaf(r[cw], sb[gq], acc[cw][gq][1]);
                    }
                }
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
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int r = band0 + 128 * gq + 2 * lane + h;
            if (r >= g.nrows) continue;
            float out[CW];
#pragma unroll
            for (int cw = 0; cw < CW; ++cw) out[cw] = sf_amp(g, v, ac[cw], r) * acc[cw][gq][h];
            float *__restrict__ dst = ya + (size_t)r * g.ncols + c0;
            if constexpr (CW == 2) {
                if (c0 + 1 < g.ncols) {
                    Pair pr;
                    if (!slab.first) {
                        pr = *reinterpret_cast<const Pair *>(dst);
                        out[0] += pr.lo; out[1] += pr.hi;
                    }
                    pr.lo = out[0]; pr.hi = out[1];
                    *reinterpret_cast<Pair *>(dst) = pr;
                    continue;
                }
            }
            if constexpr (CW == 4) {
                if (c0 + 3 < g.ncols) {
                    Quad qd;
                    if (!slab.first) {
                        qd = *reinterpret_cast<const Quad *>(dst);
                        out[0] += qd.a; out[1] += qd.b; out[2] += qd.c; out[3] += qd.d;
                    }
                    qd.a = out[0]; qd.b = out[1]; qd.c = out[2]; qd.d = out[3];
                    *reinterpret_cast<Quad *>(dst) = qd;
                    continue;
                }
            }
#pragma unroll
            for (int cw = 0; cw < CW; ++cw)
                if (c0 + cw < g.ncols) dst[cw] = slab.first ? out[cw] : dst[cw] + out[cw];
        }
    }
}

#endif
