// Occupancy grid extraction (Sec. 3.4, "Empty Space Skipping"): work decomposition shared by the 16-bit and the
// fp32 density kernels.
//
// Every voxel of the grid being filled is probed at the 27 sub-cell centres of a 3x3x3 subgrid,
// x = bmin + (v + c) * cell per axis with c in {1/6, 1/2, 5/6}, evaluated as fmaf((float)v + c, cell, bmin); the voxel
// is marked iff any probe's density is above tau.  A probe is evaluated by the network of the cell it lies in
// (Eq. 6).  Voxels are dealt out by "home cell", the network cell that holds the voxel's centre: along each
// axis the voxels whose centre lies in cell c form the range first[c] .. first[c+1]-1, so the voxels of a home cell
// form a box, and all probes of a box use the same network unless the grids do not nest (then the probes of a
// voxel that straddles a cell boundary are evaluated in a second pass with the neighbour's weights).
// A box's probe points are numbered voxel by voxel (z fastest), 27 consecutive numbers per voxel, and cut into
// tiles of 64; a workgroup takes one of `parts` equal shares of a box's tiles.  A lane handles the probe numbers
// 64 t + lane of consecutive tiles t: it splits the first into (voxel coordinates inside the box, probe of the voxel)
// once and from then on steps that cursor by 64, without divisions.
#pragma once

#include "kn_common.h"

struct KnProbeJob {
    KnGrid occ;              // the grid being filled
    KnGrid net;              // the network grid
    const int32_t *cell_net; // device, sparse network grids: cell -> network or -1; nullptr on a dense grid
    const int32_t *first[3]; // device, net.res[a] + 1 entries per axis
    int32_t parts;           // workgroups per network cell
    int32_t nested;          // the grid being filled refines the network grid and every probe lies safely inside its
                             // voxel's home cell (the host has checked the rounding margins): Eq. 6 is not evaluated
    float tau;
    uint8_t *occupancy;      // device, occ.res[0]*[1]*[2] bytes, zero before the launch
};

struct KnProbeBox {
    int32_t v0[3], n[3];
    int32_t points, tiles; // 27 * voxels, ceil(points / 64)
};

constexpr int KN_PROBES = 27;
// Largest number of voxels one network cell may own: keeps probe numbers inside int32.
constexpr int64_t KN_PROBE_MAX_BOX = 0x7fffffff / KN_PROBES - 64;

__device__ __forceinline__ KnProbeBox kn_probe_box(const KnProbeJob &j, int32_t cell)
{
    KnProbeBox b;
    int32_t c[3];
    c[2] = cell % j.net.res[2];
    c[1] = (cell / j.net.res[2]) % j.net.res[1];
    c[0] = cell / (j.net.res[2] * j.net.res[1]);
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        b.v0[a] = j.first[a][c[a]];
        b.n[a] = j.first[a][c[a] + 1] - b.v0[a];
    }
    b.points = KN_PROBES * b.n[0] * b.n[1] * b.n[2];
    b.tiles = (b.points + KN_WAVE - 1) / KN_WAVE;
    return b;
}

// A probe of a box: voxel coordinates inside the box (l[0] may run past the box: such a probe does not exist) and
// which of the voxel's 27 probes it is.
struct KnProbeCursor {
    int32_t l[3];
    int32_t probe;
};

__device__ __forceinline__ KnProbeCursor kn_probe_cursor(const KnProbeBox &b, int32_t p)
{
    KnProbeCursor c;
    const uint32_t vl = (uint32_t)p / KN_PROBES;
    c.probe = p - (int32_t)vl * KN_PROBES;
    const uint32_t q = vl / (uint32_t)b.n[2];
    c.l[2] = (int32_t)(vl - q * (uint32_t)b.n[2]);
    c.l[0] = (int32_t)(q / (uint32_t)b.n[1]);
    c.l[1] = (int32_t)(q - (uint32_t)c.l[0] * (uint32_t)b.n[1]);
    return c;
}

// 64 probe numbers further: 64 = 2 * 27 + 10, so two or three voxels on, and at most three carries per axis
__device__ __forceinline__ void kn_probe_cursor_step(const KnProbeBox &b, KnProbeCursor &c)
{
    static_assert(KN_WAVE == 2 * KN_PROBES + 10, "step of one tile");
    c.probe += 10;
    int32_t dv = 2;
    if (c.probe >= KN_PROBES) {
        c.probe -= KN_PROBES;
        dv = 3;
    }
    c.l[2] += dv;
#pragma unroll
    for (int i = 0; i < 3; ++i)
        if (c.l[2] >= b.n[2]) {
            c.l[2] -= b.n[2];
            c.l[1] += 1;
        }
#pragma unroll
    for (int i = 0; i < 3; ++i)
        if (c.l[1] >= b.n[1]) {
            c.l[1] -= b.n[1];
            c.l[0] += 1;
        }
}

// Position of the cursor's probe and the linear index of its voxel.
__device__ __forceinline__ void kn_probe_point(const KnProbeJob &j, const KnProbeBox &b, const KnProbeCursor &c, float &x,
                                               float &y, float &z, int64_t &voxel)
{
    const int32_t vx = b.v0[0] + c.l[0], vy = b.v0[1] + c.l[1], vz = b.v0[2] + c.l[2];
    const int32_t pi = c.probe / 9, pj = (c.probe / 3) % 3, pk = c.probe % 3;
    auto sub = [](int32_t i) { return i == 0 ? 1.0f / 6.0f : (i == 1 ? 0.5f : 5.0f / 6.0f); };
    x = fmaf((float)vx + sub(pi), j.occ.cell[0], j.occ.bmin[0]);
    y = fmaf((float)vy + sub(pj), j.occ.cell[1], j.occ.bmin[1]);
    z = fmaf((float)vz + sub(pk), j.occ.cell[2], j.occ.bmin[2]);
    voxel = ((int64_t)vx * j.occ.res[1] + vy) * j.occ.res[2] + vz;
}

// Marks the voxels of a tile: `above` = this lane's probe is above tau.  The lane that holds the first probe of a
// voxel inside the tile looks at the ballot bits of that voxel's probes; a voxel that continues in the next
// tile is completed by whoever computes that tile (both only ever store 1).
__device__ __forceinline__ void kn_probe_mark(const KnProbeJob &j, bool active, bool above, int64_t voxel, int32_t probe,
                                              int lane)
{
    const unsigned long long mask = __ballot(active && above);
    if (active && (lane == 0 || probe == 0)) {
        const int len = min(KN_PROBES - probe, KN_WAVE - lane);
        const unsigned long long bits = (mask >> lane) & ((1ull << len) - 1ull);
        if (bits) j.occupancy[voxel] = 1;
    }
}
