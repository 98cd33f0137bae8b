// Work split of the 256 x 256-tile prefill kernels: which workgroup multiplies which blocks of which output
// tile.  One routine for the kernels, their launchers and the host-side diagnostic (plain C++: also compiled
// by the host compiler alone).
#pragma once

#include <stdint.h>
#include <algorithm>

#ifndef __HIPCC__
#ifndef __host__
#define __host__
#endif
#ifndef __device__
#define __device__
#endif
#endif

#define GM_MT 256            // tokens per workgroup tile
#define GM3_NT 256           // outputs per workgroup tile

// Work split of the 256 x 256-tile kernels.  Workgroup ids go round the 8 XCDs (each with its own L2), so
// XCD x runs the workgroups blockIdx.x % 8 == x, gx of them.  Tiles are dealt to the XCDs in units of mu
// token tiles of one output-tile column (mu divides the number of token tiles): unit
// u = tile_n * (m_tiles / mu) + token-tile group belongs to XCD u % 8.
//   mu = 1 (fused kernel: every workgroup streams the same tables, only the activations differ by tile):
//           tile t = tile_n * m_tiles + tile_m belongs to XCD t % 8, so with eight or more token tiles an
//           XCD keeps one token tile's activations in its L2;
//   mu > 1 (staged kernel: both operands come from memory): the workgroups of an XCD that run side by
//           side share weight words as well as activation words; the largest mu that still balances the
//           XCDs is taken (whole columns at best: 8 + 4 distinct operand streams for 32 workgroups at
//           2048 tokens instead of 1 + 32).
// An XCD's tiles are dealt out in rounds of gx whole tiles, and the blocks of the tiles left over after
// the last whole round are cut into equal contiguous shares, one per workgroup, so that every workgroup
// multiplies the same number of blocks (within one).  A share of a leftover tile leaves a float32 partial
// in the workspace; the fix-up kernel adds a tile's partials in workgroup order, which keeps the result
// independent of timing.
struct G3Split {
    uint32_t T, m_tiles, nb, gx;        // tiles, token tiles, blocks per tile, workgroups per XCD
    uint32_t l_max, p_cap;              // workspace slots: [xcd][l_max leftover tiles][p_cap parts]
    uint32_t mu, n_col;                 // token tiles per dealing unit; output tile columns
    uint32_t mt;                        // tokens per tile: GM_MT, or GM_MT / 2 in the single-round mode below
    uint32_t single;                    // every workgroup takes at most one whole tile: no leftovers, no partials
    __host__ __device__ uint32_t tiles_of(uint32_t x) const
    {
        const uint32_t U = n_col * (m_tiles / mu);
        return U > x ? mu * ((U - x + 7) / 8) : 0;
    }
    // the k-th tile of XCD x
    __host__ __device__ void tile_of(uint32_t x, uint32_t k, uint32_t &tile_m, uint32_t &tile_n) const
    {
        const uint32_t n_mg = m_tiles / mu, u = x + 8 * (k / mu);
        tile_n = u / n_mg;
        tile_m = (u % n_mg) * mu + k % mu;
    }
    __host__ __device__ uint32_t rounds(uint32_t x) const { return single ? 1 : tiles_of(x) / gx; }
    __host__ __device__ uint32_t left(uint32_t x) const { return single ? 0 : tiles_of(x) - rounds(x) * gx; }
    __host__ __device__ uint32_t units(uint32_t x) const { return left(x) * nb; }
    // workgroups that take a share of the leftover units: every share holds at least one unit
    __host__ __device__ uint32_t sharers(uint32_t x) const { const uint32_t u = units(x); return u < gx ? u : gx; }
    __host__ __device__ uint32_t share_begin(uint32_t x, uint32_t j) const
    {
        const uint32_t g = sharers(x);
        return j >= g ? units(x) : (uint32_t)(((uint64_t)j * units(x)) / g);
    }
    // the workgroup whose share holds unit v
    __host__ __device__ uint32_t owner(uint32_t x, uint32_t v) const
    {
        return (uint32_t)((((uint64_t)v + 1) * sharers(x) - 1) / units(x));
    }
    __host__ __device__ uint32_t parts(uint32_t x, uint32_t l) const { return owner(x, (l + 1) * nb - 1) - owner(x, l * nb) + 1; }
    __host__ __device__ size_t slot(uint32_t x, uint32_t l, uint32_t part) const { return ((size_t)x * l_max + l) * p_cap + part; }
    // next segment of workgroup wg of XCD x: blocks [k0, k1) of the XCD's k-th tile.  round and u_next
    // carry the position (start: 0 and share_begin(x, wg)); false when the workgroup is done.
    struct Seg { uint32_t k, k0, k1, whole; size_t part_slot; };
    __host__ __device__ bool next(uint32_t x, uint32_t wg, uint32_t &round, uint32_t &u_next, Seg &sg) const
    {
        const uint32_t n_rounds = rounds(x), u_end = share_begin(x, wg + 1);
        sg.part_slot = 0;
        if (round < n_rounds) {
            if (single && wg >= tiles_of(x)) return false;
            sg.k = wg + round * gx; sg.k0 = 0; sg.k1 = nb; sg.whole = 1;
            ++round;
            return true;
        }
        if (u_next >= u_end) return false;
        const uint32_t l = u_next / nb;
        sg.k0 = u_next - l * nb;
        sg.k1 = sg.k0 + (u_end - u_next) < nb ? sg.k0 + (u_end - u_next) : nb;
        sg.k = n_rounds * gx + l;
        // a share of the leftover tiles always leaves a partial, also when it happens to cover a whole
        // tile: the fix-up pass stores every leftover tile from its slots
        sg.whole = 0;
        sg.part_slot = slot(x, l, wg - owner(x, l * nb));
        u_next += sg.k1 - sg.k0;
        return true;
    }
};
#define G3_SLOT_FLOATS 65536u           // one 256 x 256 partial

// The split of a call: nb blocks per tile, 256 CUs = 32 workgroups per XCD (fewer when the busiest XCD's
// share of the work is under four blocks per workgroup).  grouped: deal tiles in units of several token
// tiles of one column -- the largest unit (halving from a whole column) whose busiest XCD is within 3 %
// of the best.
static inline G3Split skl_make_split(uint32_t out, uint32_t nb, uint32_t tokens, bool grouped)
{
    G3Split sp;
    sp.n_col = (out + GM3_NT - 1) / GM3_NT;
    sp.nb = nb;
    auto most = [&]() { uint32_t m = 0; for (uint32_t x = 0; x < 8; ++x) m = std::max(m, sp.tiles_of(x)); return m; };
    auto deal = [&](uint32_t mt) {
        sp.mt = mt;
        sp.m_tiles = (tokens + mt - 1) / mt;
        sp.T = sp.m_tiles * sp.n_col;
        sp.mu = 1;
        if (grouped) {
            const uint32_t best = (sp.T + 7) / 8;               // tiles of the busiest XCD when dealt one by one
            for (uint32_t mu = sp.m_tiles; mu >= 1; mu /= 2) {
                if (sp.m_tiles % mu) continue;
                sp.mu = mu;
                if (most() * 100 <= best * 103) break;
            }
        }
    };
    sp.single = 0;
    sp.gx = 1; sp.l_max = 0; sp.p_cap = 0;
    // Staged kernel, calls whose tiles of half the height (128 tokens: 32 per wavefront instead of 64) fill
    // at least seven eighths of the CUs exactly once: every workgroup multiplies one whole such tile.  With
    // full-height tiles these calls have fewer tiles than CUs, so that every tile would be shared by two
    // workgroups, written as float32 partials and passed through the fix-up.  (A block of a half-height
    // tile takes 0.55 of the time of a full-height one, measured; below 225 tiles sharing is faster.)
    if (grouped) {
        const uint32_t t_half = ((tokens + GM_MT / 2 - 1) / (GM_MT / 2)) * sp.n_col;
        if (t_half > 224 && t_half <= 256) {
            deal(GM_MT / 2);
            if (most() <= 32) {
                sp.single = 1;
                sp.gx = 32;
                return sp;
            }
        }
    }
    deal(GM_MT);
    sp.gx = (uint32_t)std::min<uint64_t>(32, std::max<uint64_t>(1, (uint64_t)most() * nb / 4));
    for (uint32_t x = 0; x < 8; ++x) {
        sp.l_max = std::max(sp.l_max, sp.left(x));
        for (uint32_t l = 0; l < sp.left(x); ++l) sp.p_cap = std::max(sp.p_cap, sp.parts(x, l));
    }
    return sp;
}
