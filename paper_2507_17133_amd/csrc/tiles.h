// GEMM tile table, built on the device from the unit row counts (shared by the routing kernels, which know
// the counts first, and by the stand-alone table kernel used when the caller brings its own row lists).
//
// int32 header {n_tiles, 0, 0, 0}, then one int4 {unit, first row, rows, 0} per M tile, units in ascending
// order, tiles of a unit consecutive.
#pragma once
#include "internal.h"

namespace bmoe {

struct TileJob {
    int u_lo, u_hi;          // units [u_lo, u_hi)
    TilePlan plan;
    int32_t* table;
};
struct TileJobs {
    int n;                   // 0, 1 or 2 jobs (routed + united units; shared units of another width)
    TileJob job[2];
    int cap;                 // entries a table holds
};

// One wavefront builds the table of one job.  cnt[u], off[u]: rows and first row of unit u (global or LDS).
__device__ __forceinline__ void build_tile_table(const int* cnt, const int* off, const TileJob& j, int cap, int lane)
{
    const int bm = j.plan.bm;
    const int n_units = j.u_hi - j.u_lo;
    const int per = (n_units + 63) / 64;
    int local = 0;
    for (int q = 0; q < per; ++q) {
        const int u = j.u_lo + lane * per + q;
        if (u < j.u_hi) local += (cnt[u] + bm - 1) / bm;
    }
    int incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
    }
    int at = incl - local;
    const int total = __shfl(incl, 63);
    if (lane == 0) {
        j.table[0] = total < cap ? total : cap;
        j.table[1] = 0; j.table[2] = 0; j.table[3] = 0;
    }
    int4* entries = reinterpret_cast<int4*>(j.table + 4);
    for (int q = 0; q < per; ++q) {
        const int u = j.u_lo + lane * per + q;
        if (u >= j.u_hi) break;
        const int c = cnt[u], o = off[u];
        for (int r = 0; r < c; r += bm) {
            if (at < cap) entries[at] = make_int4(u, o + r, min(bm, c - r), 0);
            ++at;
        }
    }
}

}  // namespace bmoe
