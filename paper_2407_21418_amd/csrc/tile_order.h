// Workgroup -> tile descriptor mapping of one launch (host and device).
//
// Workgroups are handed to the XCDs round-robin (workgroup b runs on XCD b % nx).  Each XCD gets
// one contiguous slice of EVERY constituent's block of the descriptor table: tiles that share an
// A row panel or a B column panel meet in the same per-XCD L2, and the large tiles of a
// two-uKernel program are spread over all XCDs instead of filling the first few (the small tiles of
// its tail would otherwise leave the other XCDs nearly idle).  Inside an XCD the first constituent
// (the larger tiles) is started first.
//
// Inside a constituent's tile grid (rows x cols per batch entry, row-major in the table) the slice
// is walked in groups of G tile rows, column by column, so the tiles an XCD runs at once form a
// compact 2-D block that touches few A panels AND few B panels.
#pragma once
#include <stdint.h>

#if defined(__HIP__)      // compiled as HIP source: callable from kernels and from the host
#define FT_HD __attribute__((host)) __attribute__((device)) inline __attribute__((always_inline))
#else
#define FT_HD inline
#endif

namespace ftk {

struct LaunchOrder {
    uint32_t n[2];        // tiles of each constituent (n[1] = 0 for a single-uKernel program)
    uint32_t first[2];    // first descriptor of each constituent's block
    uint32_t rows[2], cols[2], group[2];
    uint32_t nx;          // XCDs
    // what the descriptors of a constituent's block hold, in closed form: descriptor
    // first + (batch * rows + r) * cols + c has m0 = m_base + r * tm, n0 = n_base + c * tn
    uint32_t m_base[2], n_base[2], tm[2], tn[2];
};

// One workgroup's tile as the kernel derives it without reading the table (the table stays the
// plan's definition: the host checks every workgroup's closed form against it when the plan is made).
struct TileOfWorkgroup {
    uint32_t index;       // descriptor index
    uint32_t slot;        // constituent (0 or 1)
    uint32_t batch, m0, n0;
};

// u-th tile of a constituent in launch order -> (batch entry, tile row, tile column) of its grid
FT_HD void grouped_coords(uint32_t u, uint32_t rows, uint32_t cols, uint32_t G, uint32_t *bidx, uint32_t *row, uint32_t *col) {
    // (run-time divisions are costly on the device: a single batch entry and full groups of a
    // power-of-two height, the common cases, get by with one)
    const uint32_t per = rows * cols;
    uint32_t bi = 0, v = u;
    if (u >= per) { bi = u / per; v = u % per; }
    *bidx = bi;
    if (rows < 2 || cols < 2 || G < 2) {
        const uint32_t r = cols > 1 ? v / cols : v;
        *row = r;
        *col = v - r * cols;
        return;
    }
    const uint32_t grp = v / (G * cols), w = v - grp * (G * cols);
    const uint32_t first = grp * G;
    const uint32_t gr = rows - first < G ? rows - first : G;
    uint32_t wq, wr;                                   // w / gr, w % gr
    if (gr == G && (G & (G - 1)) == 0) {
        const uint32_t sh = 31u - (uint32_t)__builtin_clz(G);
        wq = w >> sh;
        wr = w & (G - 1);
    } else {
        wq = w / gr;
        wr = w - wq * gr;
    }
    *row = first + wr;
    *col = wq;
}

// descriptor index of workgroup b; *slot receives the constituent (0 or 1).  NX: the number of XCDs
// when it is known at compile time (divisions by it become shifts), 0 to take it from o.nx.
template <uint32_t NX>
FT_HD TileOfWorkgroup tile_of_workgroup_nx(const LaunchOrder &o, uint32_t b) {
    const uint32_t nx = NX ? NX : o.nx;
    const uint32_t x = b % nx, j = b / nx;
    const uint32_t q0 = o.n[0] / nx, r0 = o.n[0] % nx;
    const uint32_t q1 = o.n[1] / nx, r1 = o.n[1] % nx;
    // constituent 0: XCD x takes q0 tiles, the first r0 XCDs one more
    const uint32_t c0 = q0 + (x < r0 ? 1u : 0u);
    uint32_t s, idx;
    if (j < c0) {
        s = 0;
        idx = x * q0 + (x < r0 ? x : r0) + j;
    } else {
        // constituent 1: the r1 extra tiles go to XCDs r0, r0+1, ... (mod nx), so every XCD ends up
        // with exactly the number of workgroups the round-robin hands it
        s = 1;
        uint32_t before;                       // XCDs below x that hold an extra tile of constituent 1
        if (r0 + r1 <= nx) {
            before = x <= r0 ? 0u : (x - r0 < r1 ? x - r0 : r1);
        } else {
            const uint32_t wrap = r0 + r1 - nx;
            before = (x < wrap ? x : wrap) + (x > r0 ? x - r0 : 0u);
        }
        idx = x * q1 + before + (j - c0);
    }
    // selects, not indexed loads: the fields stay in (scalar) registers on the device
    const uint32_t first = s ? o.first[1] : o.first[0], rows = s ? o.rows[1] : o.rows[0];
    const uint32_t cols = s ? o.cols[1] : o.cols[0], group = s ? o.group[1] : o.group[0];
    uint32_t bidx, row, col;
    grouped_coords(idx, rows, cols, group, &bidx, &row, &col);
    TileOfWorkgroup t;
    t.slot = s;
    t.index = first + (bidx * rows + row) * cols + col;
    t.batch = bidx;
    t.m0 = (s ? o.m_base[1] : o.m_base[0]) + row * (s ? o.tm[1] : o.tm[0]);
    t.n0 = (s ? o.n_base[1] : o.n_base[0]) + col * (s ? o.tn[1] : o.tn[0]);
    return t;
}

FT_HD TileOfWorkgroup tile_of_workgroup(const LaunchOrder &o, uint32_t b) {
    // integer division by a run-time value costs the device some forty instructions each, on the
    // critical path of every workgroup: the usual device (8 XCDs) gets its own instance
    return o.nx == 8 ? tile_of_workgroup_nx<8>(o, b) : tile_of_workgroup_nx<0>(o, b);
}

// Plans with more than two uKernel shapes (second-axis strips) are walked in table order, dealt to
// the XCDs in chunks of kTableChunk consecutive descriptors: neighbouring tiles of a row band stay
// on one XCD (the halves of a cache line of C that two of them share meet in one L2) and every XCD
// gets the same mix of tile shapes.  The grid is rounded up to whole rounds of chunks; a
// workgroup beyond the table (returned index >= n_tiles) has nothing to do.
constexpr uint32_t kTableChunk = 16;

FT_HD uint32_t table_grid(uint32_t n_tiles, uint32_t nx) {
    const uint32_t round = nx * kTableChunk;
    return (n_tiles + round - 1) / round * round;
}

FT_HD uint32_t table_index_of_workgroup(uint32_t b, uint32_t nx) {
    const uint32_t x = b % nx, j = b / nx;
    return ((j / kTableChunk) * nx + x) * kTableChunk + j % kTableChunk;
}

}  // namespace ftk
