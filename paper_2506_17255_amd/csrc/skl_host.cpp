// Host side of the sketch-linear library: argument validation, the layout
// plan (width metadata -> table offsets, Sec. 3.2 / 3.3 per-group widths),
// re-encoding of the sketch states into order keys, and the C ABI.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <numeric>

#include "skl_internal.h"
#include "skl_split.h"

// ------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

void skl_set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

#define FAIL(code, ...)             \
    do {                            \
        skl_set_error(__VA_ARGS__); \
        return (code);              \
    } while (0)

static inline uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

// ---------------------------------------------------------------- planning
// the caller's struct (first or current version) copied into the current layout
static skl_status_t normalize_desc(const skl_desc_t *user, skl_desc_t *d)
{
    if (!user) FAIL(SKL_ERR_INVALID_ARG, "desc is NULL");
    if (user->struct_size != sizeof(skl_desc_t) && user->struct_size != SKL_DESC_SIZE_V1)
        FAIL(SKL_ERR_INVALID_ARG, "desc.struct_size is %u, expected %zu (or %u, the first version)", user->struct_size,
             sizeof(skl_desc_t), SKL_DESC_SIZE_V1);
    memset(d, 0, sizeof *d);
    memcpy(d, user, user->struct_size);
    return SKL_OK;
}

static int code_at(const skl_desc_t *d, uint64_t i)
{
    if (d->state_bits == 8) return static_cast<const int8_t *>(d->codes)[i];
    const uint8_t b = static_cast<const uint8_t *>(d->codes)[i >> 1];
    const int nib = (i & 1) ? b >> 4 : b & 15;
    return nib >= 8 ? nib - 16 : nib;
}

// geometry_only: the description of a sketch still to be built (no states, codes or scales yet)
static skl_status_t validate_desc(const skl_desc_t *d, uint64_t *n_groups_out, bool geometry_only = false)
{
    if (d->in_features == 0 || d->out_features == 0)
        FAIL(SKL_ERR_INVALID_ARG, "in_features and out_features must be positive");
    if (d->in_features > (1u << 30) || d->out_features > (1u << 30))
        FAIL(SKL_ERR_UNSUPPORTED, "in_features / out_features above 2^30");
    if (d->tile_in == 0 || d->tile_out == 0 || d->in_features % d->tile_in || d->out_features % d->tile_out)
        FAIL(SKL_ERR_INVALID_ARG, "tile %ux%u does not divide the layer %ux%u", d->tile_in, d->tile_out,
             d->in_features, d->out_features);
    if ((uint64_t)d->tile_in * d->tile_out > (1ull << 24))
        FAIL(SKL_ERR_INVALID_ARG, "group of %ux%u weights exceeds 2^24 addresses", d->tile_in, d->tile_out);
    if (d->d < 1 || d->d > SKL_MAX_D) FAIL(SKL_ERR_INVALID_ARG, "d = %u sketch rows, must be 1..8", d->d);
    if (d->query_mode > 1) FAIL(SKL_ERR_INVALID_ARG, "query_mode = %u, must be 0 (Max by magnitude) or 1 (Max of the signed values)", d->query_mode);
    if (d->flags & ~7u) FAIL(SKL_ERR_INVALID_ARG, "unknown bits in flags: 0x%x", d->flags);
    if ((d->flags & 6u) == 6u) FAIL(SKL_ERR_INVALID_ARG, "flags ask for the staged and for the fused prefill at once");
    if (d->state_bits != 0 && d->state_bits != 16 && d->state_bits != 8 && d->state_bits != 4)
        FAIL(SKL_ERR_INVALID_ARG, "state_bits = %u, must be 0, 16, 8 or 4", d->state_bits);
    if (d->reserved != 0) FAIL(SKL_ERR_INVALID_ARG, "desc.reserved must be 0");
    const bool low_bit = d->state_bits == 8 || d->state_bits == 4;
    if (!d->hash_a || !d->hash_c || !d->group_width)
        FAIL(SKL_ERR_INVALID_ARG, "hash_a, hash_c and group_width must not be NULL");
    if (!geometry_only) {
        if (!low_bit && !d->states) FAIL(SKL_ERR_INVALID_ARG, "states must not be NULL");
        if (low_bit && (!d->codes || !d->scales || d->states))
            FAIL(SKL_ERR_INVALID_ARG, "low-bit states need codes and scales, and states must be NULL");
    }
    for (uint32_t r = 0; r < d->d; ++r)
        if (d->hash_a[r] >= (1u << 24) || d->hash_c[r] >= (1u << 24))
            FAIL(SKL_ERR_INVALID_ARG, "hash parameters of row %u are not below 2^24", r);
    const uint64_t n_groups = (uint64_t)(d->in_features / d->tile_in) * (d->out_features / d->tile_out);
    uint64_t sum = 0;
    for (uint64_t g = 0; g < n_groups; ++g) {
        const uint32_t K = d->group_width[g];
        if (K == 0 || K > 65535)
            FAIL(SKL_ERR_INVALID_ARG, "group_width[%llu] = %u, must be 1..65535", (unsigned long long)g, K);
        sum += K;
    }
    if (d->n_states != sum * d->d)
        FAIL(SKL_ERR_INVALID_ARG, "n_states = %llu but d * sum(group_width) = %llu",
             (unsigned long long)d->n_states, (unsigned long long)(sum * d->d));
    if (d->n_states >= (1ull << 32)) FAIL(SKL_ERR_UNSUPPORTED, "more than 2^32 states in one layer");
    if (geometry_only) {
        *n_groups_out = n_groups;
        return SKL_OK;
    }
    if (!low_bit) {
        for (uint64_t i = 0; i < d->n_states; ++i)
            if ((d->states[i] & 0x7C00u) == 0x7C00u)
                FAIL(SKL_ERR_NONFINITE, "states[%llu] = 0x%04x is NaN or infinite", (unsigned long long)i, d->states[i]);
    } else {
        if (n_groups * d->d >= (1ull << 32)) FAIL(SKL_ERR_UNSUPPORTED, "more than 2^32 scales in one layer");
        for (uint64_t i = 0; i < n_groups * d->d; ++i) {
            if ((d->scales[i] & 0x7C00u) == 0x7C00u)
                FAIL(SKL_ERR_NONFINITE, "scales[%llu] = 0x%04x is NaN or infinite", (unsigned long long)i, d->scales[i]);
            if (d->scales[i] & 0x8000u)
                FAIL(SKL_ERR_INVALID_ARG, "scales[%llu] = 0x%04x has its sign bit set", (unsigned long long)i, d->scales[i]);
        }
        const int lowest = d->state_bits == 8 ? -128 : -8;
        for (uint64_t i = 0; i < d->n_states; ++i)
            if (code_at(d, i) == lowest)
                FAIL(SKL_ERR_INVALID_ARG, "codes[%llu] = %d is outside [-qmax, qmax]", (unsigned long long)i, lowest);
    }
    *n_groups_out = n_groups;
    return SKL_OK;
}

// Decode plan for row sketches: cut the layer into n_sseg output segments x
// n_bg block groups, one workgroup each and at most one workgroup per CU.
// Workgroup ids are dealt round-robin to the 8 XCDs of 32 CUs each and a group's
// segments all land on one XCD, so ceil(G/8)*S workgroups compete for 32 CUs.
//
// Cost model of a decode split (microseconds; constants fitted to measurements on MI355X).  A workgroup walks
// the blocks of its group; a block step costs a fixed part (barrier, metadata, issuing the next table's
// copy) plus the larger of its work and the time to stream the next table into LDS -- their sum when the
// group's tables are too large for two buffers.  The work of a step is its vector time on the busiest SIMD
// (ceil(wavefronts / 4) wavefronts x units per wavefront x words per state row) plus its gather time on the
// CU's LDS (all wavefronts; narrow blocks put more unrelated state rows into one clock's 16 lanes and pay
// more bank conflicts), each scaled by a fitted factor.
struct DecodeShape {
    uint32_t seg_units;     // 64-output units of the longest segment
    uint32_t upw;           // units per wavefront
    uint32_t waves;         // wavefronts per workgroup
};

static DecodeShape decode_shape(uint32_t units, uint32_t S)
{
    DecodeShape sh;
    sh.seg_units = (units + S - 1) / S;
    sh.upw = sh.seg_units > 16 ? 2 : 1;
    sh.waves = std::max(2u, (sh.seg_units + sh.upw - 1) / sh.upw);
    return sh;
}

// Fitted by least squares to the batch-1 kernel times of 46 splits of nine layer shapes measured on MI355X
// (root-mean-square error 8 %):
#define SKL_COST_START_US 2.47       // launch, first table, activations, row addresses, fold and store
#define SKL_COST_STEP_US 0.16        // per block step: barrier, metadata, issuing the next table's copy
#define SKL_COST_VEC 1.25            // x the ideal vector issue time of the step on the busiest SIMD
#define SKL_COST_LDS 0.63            // x the gather time of the step at the conflict rate of its words per state row
#define SKL_COST_MIN_WAVES 6u        // fewer wavefronts do not hide each other's LDS latency: priced as this many
#define SKL_COST_FILL_US_PER_KB 0.0154
#define SKL_COST_WORST_SHARE 0.70    // the kernel's time follows the dearest group this much and the mean load per CU for the rest
#define SKL_COST_GROUP_US 0.0289     // per block group, in the kernel
#define SKL_COST_CLASS_US 0.78        // a change of sketch width inside a group: new state-row addresses, per unit of a wavefront
#define SKL_COST_REDUCE_US_PER_MB 1.7   // the reduction pass reads one float per (group, output)
#define SKL_COST_CLOCK_MHZ 2170.0

static double block_step_cost(const skl_block_meta &bm, uint32_t d, const DecodeShape &sh, bool two_bufs)
{
    const uint32_t waves = std::max(sh.waves, SKL_COST_MIN_WAVES);
    // 6 d vector instructions per (lane, output): d - 1 packed maxima x 4, 8 decode, 4 dot products for d = 4
    const double vec = (double)((waves + 3) / 4) * sh.upw * bm.nb * 6 * d * 4 / SKL_COST_CLOCK_MHZ;
    // the 16 lanes served in one clock read 16 / nb different state rows: expected passes per gather
    const double conflicts = bm.nb >= 8 ? 1.5 : bm.nb == 4 ? 2.1 : bm.nb == 2 ? 2.8 : 3.1;
    const double lds = (double)waves * sh.upw * bm.nb * d * 4 * conflicts / SKL_COST_CLOCK_MHZ;
    const double fill = SKL_COST_FILL_US_PER_KB * (((uint64_t)d * bm.K * bm.nb + 63) / 64);
    const double work = SKL_COST_VEC * vec + SKL_COST_LDS * lds;
    return SKL_COST_STEP_US + (two_bufs ? std::max(work, fill) : work + fill + SKL_COST_STEP_US);
}

// P->want_s, P->want_g: 0, or a split to plan instead of the cheapest one (diagnostic; false if the kernels cannot run it)
static bool plan_decode(const skl_desc_t *d, skl_plan *P)
{
    skl_layer &L = P->L;
    const uint32_t want_s = P->want_s, want_g = P->want_g;
    const uint32_t units = (d->out_features + 63) / 64;
    const uint32_t nblk = L.n_blocks;
    auto ptable_bytes = [&](const skl_block_meta &bm) { return (d->d * bm.K * bm.nb + 63) / 64 * 1024u; };
    auto table_bytes = [&](const skl_block_meta &bm) { return d->d * bm.K * bm.rs * 16u; };
    // Group boundaries for G groups: equal shares of the blocks' relative costs, every group at least one block.
    std::vector<double> cum(nblk + 1, 0.0);
    // The shares of the groups are cut by relative block costs measured directly (decode time of six layer
    // shapes against these weights), which the step model above does not resolve: a block costs about the same
    // whatever its word count -- its table is about as large, it takes the same barriers, a new sketch width
    // means new state-row addresses -- so a word of a narrow block is dearer: 8 words 32, 4 words 40, 2 words
    // 20, 1 word 28.  With plain word counts the group that received the outlier channels' narrow blocks ran
    // 2.5 us longer than the others on the 4096 x 11008 layer.  A table too large for double buffering is
    // copied after, not during, the block before it: half as much again.
    auto price_blocks = [&](const DecodeShape &) {
        for (uint32_t b = 0; b < nblk; ++b) {
            const skl_block_meta &bm = P->bmeta[b];
            const double w = bm.nb >= 8 ? 32.0 : bm.nb == 4 ? 40.0 : bm.nb == 2 ? 20.0 : 28.0;
            cum[b + 1] = cum[b] + (ptable_bytes(bm) <= SKL_PBUF_DIST ? w : 1.5 * w);
        }
    };
    auto cut_groups = [&](uint32_t G, std::vector<uint32_t> &start) -> uint32_t {
        start.assign(G + 1, 0);
        uint32_t b = 0, most = 0;
        for (uint32_t g = 0; g < G; ++g) {
            start[g] = b;
            const double target = cum[nblk] * (g + 1) / G;
            while (b < nblk && (cum[b + 1] <= target * (1 + 1e-12) || b == start[g])) ++b;
            if (nblk - b < G - 1 - g) b = nblk - (G - 1 - g);    // leave a block for every later group
            if (g + 1 == G) b = nblk;
            most = std::max(most, b - start[g]);
        }
        start[G] = nblk;
        return most;
    };
    // LDS plan of a cut: which groups run double-buffered, the table areas of the two kernels, the longest
    // channel range; false if some kernel's LDS need exceeds the CU's.
    struct Lds { uint32_t ptab, tab, max_chan; std::vector<uint32_t> flags; };
    auto lds_plan = [&](const std::vector<uint32_t> &start, uint32_t G, uint32_t upw, Lds &o) -> bool {
        o.flags.assign(G, 0);
        o.max_chan = 0;
        bool any1 = false, anyN = false;
        for (uint32_t g = 0; g < G; ++g) {
            uint32_t mp = 0, mt = 0;
            for (uint32_t b = start[g]; b < start[g + 1]; ++b) {
                mp = std::max(mp, ptable_bytes(P->bmeta[b]));
                mt = std::max(mt, table_bytes(P->bmeta[b]));
            }
            if (mp <= SKL_PBUF_DIST) { o.flags[g] |= 1u; any1 = true; }
            if (mt <= SKL_PBUF_DIST) { o.flags[g] |= 2u; anyN = true; }
            const uint32_t c_lo = P->bmeta[start[g]].chan_off;
            const uint32_t c_hi = start[g + 1] < nblk ? P->bmeta[start[g + 1]].chan_off : (uint32_t)P->chan.size();
            o.max_chan = std::max(o.max_chan, c_hi - c_lo);
        }
        // batch-1 kernel: sums of upw x 1024 outputs, block metadata, state-row addresses, the group's activations
        const uint64_t g1_rest = 4096ull * upw + SKL_MAX_GROUP_BLOCKS * 32 + 4096ull * d->d + 2ull * (o.max_chan + 64);
        // batched kernel: block metadata, 16 activation rows of the group
        const uint64_t gn_rest = 16ull * (o.max_chan + 16) * 2 + 2048;
        o.ptab = std::max<uint32_t>(any1 ? 2 * SKL_PBUF_DIST : 0, L.max_ptable_bytes);
        o.tab = std::max<uint32_t>(anyN ? 2 * SKL_PBUF_DIST : 0, L.max_table_bytes);
        if (o.ptab + g1_rest > SKL_LDS_HARD_BYTES) {             // no room for two buffers: one for every group
            o.ptab = L.max_ptable_bytes;
            for (uint32_t &f : o.flags) f &= ~1u;
        }
        if (o.tab + gn_rest > SKL_LDS_HARD_BYTES) {
            o.tab = L.max_table_bytes;
            for (uint32_t &f : o.flags) f &= ~2u;
        }
        return o.ptab + g1_rest <= SKL_LDS_HARD_BYTES && o.tab + gn_rest <= SKL_LDS_HARD_BYTES;
    };
    // Cost of a split: rounds x (start-up + a blend of the dearest group's time and the mean load of a CU)
    // + what the number of groups costs in the kernel and in the reduction pass.  The step model gives the
    // time of all blocks together; a group's part of it is its share of the relative block costs the cut
    // was made with (the model does not resolve the cost of one narrow block against one wide block).
    auto split_cost = [&](const std::vector<uint32_t> &start, uint32_t G, uint32_t S, const DecodeShape &sh, const Lds &lds) {
        double total = 0, heaviest = 0;
        for (uint32_t g = 0; g < G; ++g) {
            for (uint32_t b = start[g]; b < start[g + 1]; ++b) {
                total += block_step_cost(P->bmeta[b], d->d, sh, lds.flags[g] & 1u);
                if (b > start[g] && P->bmeta[b].K != P->bmeta[b - 1].K) total += SKL_COST_CLASS_US * sh.upw;
            }
            heaviest = std::max(heaviest, cum[start[g + 1]] - cum[start[g]]);
        }
        const double worst = total * heaviest / cum[nblk];
        const uint32_t per_xcd = ((G + 7) / 8) * S;
        const uint32_t rounds = (per_xcd + 31) / 32;
        const double mean = total * S / ((double)SKL_N_CU * rounds);
        return rounds * (SKL_COST_START_US + SKL_COST_WORST_SHARE * worst + (1 - SKL_COST_WORST_SHARE) * mean) +
               SKL_COST_GROUP_US * G + SKL_COST_REDUCE_US_PER_MB * G * d->out_features * 4e-6;
    };
    // Candidates: S output segments of at most 32 wave units (one or two 64-output units per wavefront of a
    // workgroup of at most 1024 threads), G block groups of at most SKL_MAX_GROUP_BLOCKS blocks; for layers of
    // 16 blocks or more G is a multiple of 8, so that every XCD runs the same number of groups.  The model
    // cannot rank splits that it prices within 3 % of each other (its own error is larger): among those the
    // one that occupies the most CUs wins, then the one with fewer segments (fewer copies of every table).
    double best = 1e300;
    uint32_t best_s = 0, best_g = 0;
    std::vector<uint32_t> start;
    Lds lds;
    auto try_split = [&](uint32_t S, uint32_t G) -> double {
        const DecodeShape sh = decode_shape(units, S);
        if (sh.upw > 1 && (L.block_classes & ~3u)) return -1.0;              // two units per wavefront: one- and two-word blocks only
        price_blocks(sh);
        if (cut_groups(G, start) > SKL_MAX_GROUP_BLOCKS) return -1.0;       // block metadata of a group sits in LDS
        if (!lds_plan(start, G, sh.upw, lds)) return -1.0;
        return split_cost(start, G, S, sh, lds);
    };
    if (want_s && want_g) {                     // the model's figure for a split the caller names
        if (want_g > nblk || want_s < (units + 31) / 32 || want_s > units) return false;
        best = try_split(want_s, want_g);
        if (best < 0) return false;
        best_s = want_s; best_g = want_g;
    } else {
        struct Cand { double t; uint32_t S, G, cus; };
        std::vector<Cand> cands;
        const uint32_t g_step = nblk >= 16 ? 8 : 1;
        const uint32_t g_lo = (nblk + SKL_MAX_GROUP_BLOCKS - 1) / SKL_MAX_GROUP_BLOCKS;
        for (uint32_t S = (units + 31) / 32; S <= units; ++S)
            for (uint32_t G = (g_lo + g_step - 1) / g_step * g_step; G <= nblk; G += g_step) {
                // a split cannot cost less than its rounds' start-ups: most of the plane is skipped on this bound
                const uint32_t rounds = (((G + 7) / 8) * S + 31) / 32;
                if (rounds * SKL_COST_START_US + SKL_COST_GROUP_US * G >= best * 1.03) continue;
                const double t = try_split(S, G);
                if (t < 0) continue;
                cands.push_back(Cand{t, S, G, std::min<uint32_t>(S * G, SKL_N_CU)});
                best = std::min(best, t);
            }
        if (cands.empty()) return false;
        const Cand *pick = nullptr;
        for (const Cand &c : cands) {
            if (c.t > best * 1.03) continue;
            if (!pick || c.cus > pick->cus || (c.cus == pick->cus && (c.S < pick->S || (c.S == pick->S && c.t < pick->t)))) pick = &c;
        }
        best = pick->t; best_s = pick->S; best_g = pick->G;
    }
    const DecodeShape sh = decode_shape(units, best_s);
    price_blocks(sh);
    cut_groups(best_g, P->bg_start);
    if (!lds_plan(P->bg_start, best_g, sh.upw, lds)) return false;
    L.decode_cost_us = best;
    L.n_sseg = best_s;
    L.n_bg = best_g;
    L.n_wunits = units;
    L.decode_upw = sh.upw;
    L.opl = 1;
    L.tab_bytes = lds.tab;
    L.ptab_bytes = lds.ptab;
    L.max_group_chan = lds.max_chan;
    P->ginfo.assign(best_g, skl_group_info{});
    for (uint32_t g = 0; g < best_g; ++g) {
        const uint32_t lo = P->bg_start[g], hi = P->bg_start[g + 1];
        const uint32_t c_lo = P->bmeta[lo].chan_off;
        const uint32_t c_hi = hi < nblk ? P->bmeta[hi].chan_off : (uint32_t)P->chan.size();
        P->ginfo[g] = skl_group_info{lo, hi, c_lo, c_hi, P->bmeta[lo].K, P->bmeta[lo].rs,
                                     P->bmeta[lo].table_off16, P->bmeta[lo].chan_off, P->bmeta[lo].ptable_off16,
                                     lds.flags[g], 0u, 0u};
    }
    L.n_units = L.n_bg;
    return true;
}

// Prefill plan for row sketches: the 16-channel step lists of the two kernels and which one a call takes.
static void plan_prefill(const skl_desc_t *d, skl_plan *P)
{
    skl_layer &L = P->L;
    // fused kernel: ceil(nb / 2) steps of 16 channels per block, in block order
    P->gsteps.clear();
    for (skl_block_meta &bm : P->bmeta) {
        bm.step_off = (uint32_t)P->gsteps.size();
        for (uint32_t c = 0; c < bm.nb; c += 2)
            P->gsteps.push_back(skl_gemm_step{bm.chan_off + 8 * c, std::min(bm.nb - c, 2u)});
    }
    L.n_gsteps = (uint32_t)P->gsteps.size();
    // the fused kernel keeps two block tables (at most 48 chunks of 1 KiB each), two operand slots of 8 column
    // blocks (34816 B each), a 1 KiB dummy row and the block metadata in LDS
    L.gemm_v3 = L.max_ptable_bytes <= 48 * 1024 &&
                2ull * L.max_ptable_bytes + 2ull * 34816 + 1024 + 32ull * P->bmeta.size() + 256 <= SKL_LDS_HARD_BYTES ? 1 : 0;
    // staged kernel: dense 16-entry steps along the channel list, four per 64-channel block; entries past
    // the end of the list are empty steps (zero activation words)
    L.gemm_kb = (L.n_packed + 63) / 64;
    P->ssteps.clear();
    for (uint32_t st = 0; st < 4 * L.gemm_kb; ++st) {
        const uint32_t c0 = 16 * st;
        P->ssteps.push_back(skl_gemm_step{std::min(c0, L.n_packed), c0 >= L.n_packed ? 0u : std::min(2u, (L.n_packed - c0) / 8)});
    }
    // Which kernel a call takes.  Layers whose tables the fused kernel cannot keep in LDS always rebuild
    // their weights once per call.  The others do so from 513 tokens on: measured on MI355X
    // (4096 x 4096 and 4096 x 11008, 0.5 bit/weight) the two kernels tie up to 512 tokens, where a call
    // is a single round of tiles either way, and the staged one is 10 % faster at 1024 tokens and 25 % at
    // 2048.  flags bit 1: always staged; bit 2: fused whenever the tables allow.
    L.gemm_staged_from = !L.gemm_v3 || (d->flags & 2u) ? 0u : (d->flags & 4u) ? 0xFFFFFFFFu : 513u;
}

// Row-sketch plan.  Returns false when some width is too large for any block
// layout (then the per-weight path is tried).
static bool plan_rows(const skl_desc_t *d, skl_plan *P)
{
    skl_layer &L = P->L;
    const uint32_t in = d->in_features;
    std::vector<uint32_t> order(in);
    std::iota(order.begin(), order.end(), 0u);
    std::stable_sort(order.begin(), order.end(),
                     [&](uint32_t a, uint32_t b) { return d->group_width[a] < d->group_width[b]; });
    P->bmeta.clear();
    P->chan.clear();
    uint64_t off16 = 0, poff16 = 0;
    uint32_t max_table = 0, soff16 = 0;
    static const uint32_t rs_options[4] = {9, 5, 3, 1};
    uint32_t i = 0;
    while (i < in) {
        const uint32_t K = d->group_width[order[i]];
        uint32_t e = i;
        while (e < in && d->group_width[order[e]] == K) ++e;
        uint32_t rs = 0;
        for (uint32_t opt : rs_options) {
            if (opt == 9 && d->d > 6) continue;   // 8 words x 7 or 8 rows: too many row addresses per lane for the batch-1 kernel's registers
            if ((uint64_t)d->d * K * opt * 16u <= SKL_LDS_SOFT_TABLE_BYTES) { rs = opt; break; }
        }
        if (!rs) {
            if ((uint64_t)d->d * K * 16u + 33792u > SKL_LDS_HARD_BYTES) return false;   // table + two activation tiles of the prefill kernel
            rs = 1;
        }
        const uint32_t nb = rs == 1 ? 1 : rs - 1;
        for (uint32_t s = i; s < e; s += 8 * nb) {
            skl_block_meta bm{};
            bm.table_off16 = (uint32_t)off16;
            bm.K = K;
            bm.rs = rs;
            bm.nb = nb;
            bm.chan_off = (uint32_t)P->chan.size();
            bm.ptable_off16 = (uint32_t)poff16;
            bm.scale_off16 = soff16;
            soff16 += d->d * nb;
            poff16 += ((uint64_t)d->d * K * nb + 63) / 64 * 64;    // whole 64-word chunks: copied without bounds checks
            for (uint32_t c = 0; c < 8 * nb; ++c)
                P->chan.push_back(s + c < e ? order[s + c] : SKL_NO_CHANNEL);
            const uint64_t words = (uint64_t)d->d * K * rs;
            off16 += words;
            if (off16 >= (1ull << 32) || poff16 >= (1ull << 32)) return false;   // both copies are addressed with 32-bit word offsets
            max_table = std::max<uint32_t>(max_table, (uint32_t)(words * 16));
            P->bmeta.push_back(bm);
        }
        i = e;
    }
    L.path = 1;
    L.n_blocks = (uint32_t)P->bmeta.size();
    L.n_packed = (uint32_t)P->chan.size();
    L.n_units = L.n_blocks;
    L.max_table_bytes = max_table;
    L.table_bytes = off16 * 16;
    L.ptable_bytes = poff16 * 16;
    L.scale_words = soff16;
    L.max_ptable_bytes = 0;
    L.block_classes = 0;
    L.n_small_blocks = 0;
    L.small_table_bytes = 0;
    for (const skl_block_meta &bm : P->bmeta) {             // three workgroups with tables of 49.5 KiB share a CU
        const uint32_t bytes = d->d * bm.K * bm.rs * 16u;
        if (bytes > 50688u) break;
        ++L.n_small_blocks;
        L.small_table_bytes = std::max(L.small_table_bytes, bytes);
    }
    for (const skl_block_meta &bm : P->bmeta) {
        L.max_ptable_bytes = std::max<uint32_t>(L.max_ptable_bytes, (d->d * bm.K * bm.nb + 63) / 64 * 1024u);
        L.block_classes |= bm.nb == 8 ? 8u : bm.nb == 4 ? 4u : bm.nb == 2 ? 2u : 1u;
    }
    L.n_otiles = (d->out_features + SKL_WG - 1) / SKL_WG;
    // about three workgroups per CU on 256 CUs, split over blocks x output segments
    uint32_t seg = (768 + L.n_blocks / 2) / L.n_blocks;
    L.n_seg = std::min(std::max(seg, 1u), L.n_otiles);
    if (!plan_decode(d, P)) return false;
    plan_prefill(d, P);
    return true;
}

static skl_status_t plan_tiles(const skl_desc_t *d, uint64_t n_groups, skl_plan *P)
{
    skl_layer &L = P->L;
    P->gmeta.resize(n_groups);
    uint64_t off = 0;
    uint32_t max_K = 0;
    for (uint64_t g = 0; g < n_groups; ++g) {
        P->gmeta[g].key_off = (uint32_t)off;
        P->gmeta[g].K = d->group_width[g];
        off += (uint64_t)d->d * d->group_width[g];
        max_K = std::max(max_K, d->group_width[g]);
    }
    if ((uint64_t)d->d * max_K * 2u + 16384u > SKL_LDS_HARD_BYTES)
        FAIL(SKL_ERR_UNSUPPORTED, "a group table of %u rows x %u states does not fit in LDS", d->d, max_K);
    L.path = 0;
    L.n_jb = d->in_features / d->tile_in;
    L.n_ob = d->out_features / d->tile_out;
    L.max_K = max_K;
    L.max_table_bytes = d->d * max_K * 2u;
    L.table_bytes = off * 2;
    const uint64_t noc = (d->tile_out + SKL_WG - 1) / SKL_WG;
    uint64_t want = (1024 + n_groups * noc - 1) / (n_groups * noc);       // chunks per group
    want = std::max<uint64_t>(1, std::min<uint64_t>(want, (d->tile_in + 7) / 8));
    uint32_t rows = (uint32_t)((d->tile_in + want - 1) / want);
    rows = std::min(std::max(rows, 1u), 512u);
    L.jc_rows = rows;
    L.n_jc = (d->tile_in + rows - 1) / rows;
    if ((uint64_t)L.n_jb * L.n_jc > (1u << 20))
        FAIL(SKL_ERR_UNSUPPORTED, "more than 2^20 partial sums per output");
    L.n_units = L.n_jb * L.n_jc;
    return SKL_OK;
}

static skl_status_t make_plan(const skl_desc_t *user, skl_plan *P);

// nothing may leave the C ABI as an exception: the planner's containers can run out of host memory
skl_status_t skl_make_plan(const skl_desc_t *user, skl_plan *P)
{
    try {
        return make_plan(user, P);
    } catch (const std::bad_alloc &) {
        FAIL(SKL_ERR_NO_MEMORY, "out of host memory while planning the layer");
    }
}

static skl_status_t make_plan(const skl_desc_t *user, skl_plan *P)
{
    uint64_t n_groups = 0;
    skl_status_t st = normalize_desc(user, &P->desc);
    if (st != SKL_OK) return st;
    const skl_desc_t *d = &P->desc;
    st = validate_desc(d, &n_groups);
    if (st != SKL_OK) return st;
    skl_layer &L = P->L;
    L.qbits = d->state_bits == 8 || d->state_bits == 4 ? d->state_bits : 0;
    L.n_groups = (uint32_t)n_groups;
    L.code_bytes = L.qbits == 8 ? d->n_states : L.qbits == 4 ? (d->n_states + 1) / 2 : 0;
    L.in = d->in_features; L.out = d->out_features; L.tj = d->tile_in; L.to = d->tile_out; L.d = d->d;
    L.query_mode = d->query_mode;
    for (uint32_t r = 0; r < d->d; ++r) { L.A[r] = d->hash_a[r]; L.C[r] = d->hash_c[r]; }
    L.n_states = d->n_states;
    const bool rows_ok = d->tile_in == 1 && d->tile_out == d->out_features && !(d->flags & 1u);
    if (!(rows_ok && plan_rows(d, P))) {
        st = plan_tiles(d, n_groups, P);
        if (st != SKL_OK) return st;
    }
    // device layout: [scratch 4 KiB][metadata][channel list][tables], 256-byte aligned parts
    uint64_t off = 4096;
    if (L.path == 1) {
        L.off_bmeta = off;  off = align_up(off + P->bmeta.size() * sizeof(skl_block_meta), 256);
        L.off_chan = off;   off = align_up(off + P->chan.size() * sizeof(uint32_t), 256);
        L.off_ginfo = off;  off = align_up(off + P->ginfo.size() * sizeof(skl_group_info), 256);
        L.off_gsteps = off; off = align_up(off + P->gsteps.size() * sizeof(skl_gemm_step), 256);
        L.off_ssteps = off; off = align_up(off + P->ssteps.size() * sizeof(skl_gemm_step), 256);
        if (!L.qbits) {
            L.off_tables = off; off = align_up(off + L.table_bytes, 256);
            L.off_ptables = off; off = align_up(off + L.ptable_bytes, 256);
        }
    } else {
        L.off_gmeta = off;  off = align_up(off + P->gmeta.size() * sizeof(skl_group_meta), 256);
        if (!L.qbits) { L.off_keys = off;   off = align_up(off + L.table_bytes + 16, 256); }
    }
    if (L.qbits) {
        if (n_groups >= (1ull << 32) / SKL_MAX_D) FAIL(SKL_ERR_UNSUPPORTED, "too many groups for low-bit states");
        if (L.path == 1) {
            // re-ordered: eight codes per word of the unpadded tables, eight scales per (block, row, word)
            L.code_bytes = L.ptable_bytes / 16 * (L.qbits == 8 ? 8 : 4);
            L.scale_bytes = (uint64_t)L.scale_words * 16;
        } else {
            L.scale_bytes = n_groups * d->d * sizeof(uint16_t);
        }
        L.off_codes = off;  off = align_up(off + L.code_bytes + 16, 256);
        L.off_scales = off; off = align_up(off + L.scale_bytes, 256);
        if (L.path == 1) {      // channel block of every 64-word chunk of the unpadded tables (the expansion kernel's index)
            L.off_chunk_block = off; off = align_up(off + L.ptable_bytes / 1024 * sizeof(uint32_t), 256);
        }
    }
    P->dev_bytes = off;
    return SKL_OK;
}

// ---------------------------------------------------------- prefill split
// every segment of the split, eight words each: xcd, workgroup, token tile, output tile, first block,
// end block, whole-tile flag, partial slot; returns the number of segments (writes at most cap of them)
uint64_t skl_gemm3_segments(uint32_t out, uint32_t n_blocks, uint32_t tokens, bool grouped, uint32_t *segs, uint64_t cap,
                            uint32_t *shape)
{
    const G3Split sp = skl_make_split(out, n_blocks, tokens, grouped);
    if (shape) { shape[0] = sp.gx; shape[1] = sp.l_max; shape[2] = sp.p_cap; shape[3] = sp.T; shape[4] = sp.mu; shape[5] = sp.mt; }
    uint64_t n = 0;
    for (uint32_t x = 0; x < 8; ++x)
        for (uint32_t wg = 0; wg < sp.gx; ++wg) {
            uint32_t round = 0, u_next = sp.share_begin(x, wg);
            G3Split::Seg sg;
            while (sp.next(x, wg, round, u_next, sg)) {
                if (n < cap) {
                    uint32_t *o = segs + 8 * n;
                    o[0] = x; o[1] = wg;
                    sp.tile_of(x, sg.k, o[2], o[3]);
                    o[4] = sg.k0; o[5] = sg.k1; o[6] = sg.whole; o[7] = (uint32_t)sg.part_slot;
                }
                ++n;
            }
        }
    return n;
}

// ---------------------------------------------------------- debug build
static std::vector<skl_debug_reader> &debug_readers()
{
    static std::vector<skl_debug_reader> readers;      // filled by static initialisers of the kernel files
    return readers;
}

void skl_debug_register(skl_debug_reader fn) { debug_readers().push_back(fn); }

// -------------------------------------------------------------------- ABI
extern "C" {

skl_status_t sketch_linear_debug_selftest(uint32_t value, uint32_t limit, void *hip_stream)
{
    return skl_launch_debug_selftest(value, limit, hip_stream);
}

skl_status_t sketch_linear_debug_violations(uint64_t *count, uint32_t first[5])
{
    if (!count) FAIL(SKL_ERR_INVALID_ARG, "count is NULL");
    if (debug_readers().empty()) FAIL(SKL_ERR_UNSUPPORTED, "this build of the library carries no range asserts");
    *count = 0;
    for (skl_debug_reader fn : debug_readers()) {
        uint32_t rec[8];
        skl_status_t st = fn(rec);
        if (st != SKL_OK) return st;
        if (rec[0] && !*count && first) memcpy(first, rec + 1, 5 * sizeof(uint32_t));
        *count += rec[0];
    }
    return SKL_OK;
}

const char *sketch_linear_last_error(void) { return g_err; }

skl_status_t sketch_linear_device_bytes(const skl_desc_t *desc, uint64_t *bytes)
{
    if (!bytes) FAIL(SKL_ERR_INVALID_ARG, "bytes is NULL");
    skl_plan P;
    skl_status_t st = skl_make_plan(desc, &P);
    if (st != SKL_OK) return st;
    *bytes = P.dev_bytes;
    return SKL_OK;
}

skl_status_t sketch_linear_create(const skl_desc_t *desc, void *dev_buf, uint64_t dev_bytes,
                                  void *hip_stream, skl_layer_t **out_layer)
{
    if (!out_layer) FAIL(SKL_ERR_INVALID_ARG, "out_layer is NULL");
    *out_layer = nullptr;
    skl_plan P;
    skl_status_t st = skl_make_plan(desc, &P);
    if (st != SKL_OK) return st;
    if (!dev_buf) FAIL(SKL_ERR_INVALID_ARG, "dev_buf is NULL");
    if ((uintptr_t)dev_buf % 256) FAIL(SKL_ERR_INVALID_ARG, "dev_buf is not 256-byte aligned");
    if (dev_bytes < P.dev_bytes)
        FAIL(SKL_ERR_BUFFER_TOO_SMALL, "dev_buf holds %llu bytes, %llu needed", (unsigned long long)dev_bytes,
             (unsigned long long)P.dev_bytes);

    std::vector<uint8_t> img;
    std::vector<uint64_t> base;
    try {
        img.assign(P.dev_bytes, 0);
        base.assign((size_t)P.L.in + 1, 0);
    } catch (const std::bad_alloc &) {
        FAIL(SKL_ERR_NO_MEMORY, "out of host memory for a %llu-byte staging image", (unsigned long long)P.dev_bytes);
    }
    skl_layer &L = P.L;
    desc = &P.desc;                 // from here on: the description in the current struct layout
    if (L.qbits && L.path == 0) {
        memcpy(img.data() + L.off_codes, desc->codes, L.code_bytes);
        memcpy(img.data() + L.off_scales, desc->scales, L.scale_bytes);
    }
    if (L.path == 1) {
        memcpy(img.data() + L.off_bmeta, P.bmeta.data(), P.bmeta.size() * sizeof(skl_block_meta));
        memcpy(img.data() + L.off_chan, P.chan.data(), P.chan.size() * sizeof(uint32_t));
        memcpy(img.data() + L.off_ginfo, P.ginfo.data(), P.ginfo.size() * sizeof(skl_group_info));
        memcpy(img.data() + L.off_gsteps, P.gsteps.data(), P.gsteps.size() * sizeof(skl_gemm_step));
        memcpy(img.data() + L.off_ssteps, P.ssteps.data(), P.ssteps.size() * sizeof(skl_gemm_step));
        // state offset of every input channel (one group per channel)
        for (uint32_t j = 0; j < L.in; ++j) base[j + 1] = base[j] + (uint64_t)L.d * desc->group_width[j];
        if (L.qbits) {
            uint32_t *cb = reinterpret_cast<uint32_t *>(img.data() + L.off_chunk_block);
            for (uint32_t b = 0; b < L.n_blocks; ++b) {
                const uint64_t first = P.bmeta[b].ptable_off16 / 64;
                const uint64_t end = b + 1 < L.n_blocks ? P.bmeta[b + 1].ptable_off16 / 64 : L.ptable_bytes / 1024;
                for (uint64_t ch = first; ch < end; ++ch) cb[ch] = b;
            }
            // codes and scales in the word order of the block tables (expanded on the device, per call)
            uint8_t *tc = img.data() + L.off_codes;
            uint16_t *ts = reinterpret_cast<uint16_t *>(img.data() + L.off_scales);
            const uint32_t wb = L.qbits == 8 ? 8 : 4;           // bytes of codes per table word
            for (const skl_block_meta &bm : P.bmeta)
                for (uint32_t c8 = 0; c8 < 8 * bm.nb; ++c8) {
                    const uint32_t ch = P.chan[bm.chan_off + c8], c = c8 / 8, i = c8 % 8;
                    if (ch == SKL_NO_CHANNEL) continue;         // code 0 and scale 0: +0.0
                    for (uint32_t r = 0; r < L.d; ++r) {
                        ts[((uint64_t)bm.scale_off16 + r * bm.nb + c) * 8 + i] = desc->scales[(uint64_t)ch * L.d + r];
                        for (uint32_t k = 0; k < bm.K; ++k) {
                            const int q = code_at(desc, base[ch] + (uint64_t)r * bm.K + k);
                            uint8_t *w = tc + ((uint64_t)bm.ptable_off16 + ((uint64_t)r * bm.K + k) * bm.nb + c) * wb;
                            if (L.qbits == 8) w[i] = (uint8_t)q;
                            else w[i >> 1] |= (uint8_t)((q & 15) << ((i & 1) * 4));
                        }
                    }
                }
        }
        uint16_t *tab = reinterpret_cast<uint16_t *>(img.data() + L.off_tables);
        uint16_t *ptab = reinterpret_cast<uint16_t *>(img.data() + L.off_ptables);
        for (const skl_block_meta &bm : P.bmeta) {
            if (L.qbits) break;     // tables are expanded on the device, per call
            uint16_t *t = tab + (uint64_t)bm.table_off16 * 8;
            uint16_t *pt = ptab + (uint64_t)bm.ptable_off16 * 8;
            for (uint32_t c8 = 0; c8 < 8 * bm.nb; ++c8) {
                const uint32_t ch = P.chan[bm.chan_off + c8];
                const uint16_t *s = ch == SKL_NO_CHANNEL ? nullptr : desc->states + base[ch];
                const uint32_t c = c8 / 8, i = c8 % 8;
                for (uint32_t r = 0; r < L.d; ++r)
                    for (uint32_t k = 0; k < bm.K; ++k) {
                        const uint16_t key = skl_key_of_half(s ? s[(uint64_t)r * bm.K + k] : (uint16_t)0, L.query_mode);    // a slot without a channel: +0.0
                        t[(((uint64_t)r * bm.K + k) * bm.rs + c) * 8 + i] = key;
                        pt[(((uint64_t)r * bm.K + k) * bm.nb + c) * 8 + i] = key;
                    }
            }
        }
    } else {
        memcpy(img.data() + L.off_gmeta, P.gmeta.data(), P.gmeta.size() * sizeof(skl_group_meta));
        if (!L.qbits) {
            uint16_t *keys = reinterpret_cast<uint16_t *>(img.data() + L.off_keys);
            for (uint64_t i = 0; i < desc->n_states; ++i) keys[i] = skl_key_of_half(desc->states[i], L.query_mode);
        }
    }

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipMemcpyAsync(dev_buf, img.data(), P.dev_bytes, hipMemcpyHostToDevice, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) FAIL(SKL_ERR_HIP, "copy of the layer image failed: %s", hipGetErrorString(e));

    skl_layer *out = new (std::nothrow) skl_layer(L);
    if (!out) FAIL(SKL_ERR_NO_MEMORY, "out of host memory");
    out->dev = static_cast<uint8_t *>(dev_buf);
    out->dev_bytes = P.dev_bytes;
    *out_layer = out;
    return SKL_OK;
}

void sketch_linear_destroy(skl_layer_t *layer) { delete layer; }

static skl_status_t fill_info(const skl_layer *L, skl_info_t *info)
{
    if (info->struct_size != sizeof(skl_info_t) && info->struct_size != SKL_INFO_SIZE_V1)
        FAIL(SKL_ERR_INVALID_ARG, "info.struct_size is %u, expected %zu (or %u, the first version)", info->struct_size,
             sizeof(skl_info_t), SKL_INFO_SIZE_V1);
    info->path = L->path;
    info->n_units = L->n_units;
    info->max_table_bytes = L->max_table_bytes;
    info->table_bytes = L->qbits ? L->code_bytes + L->scale_bytes : L->table_bytes;
    info->n_weights = (uint64_t)L->in * L->out;
    info->n_states = L->n_states;
    if (info->struct_size == SKL_INFO_SIZE_V1) return SKL_OK;
    info->decode_segments = L->path == 1 ? L->n_sseg : 0;
    info->decode_groups = L->path == 1 ? L->n_bg : 0;
    info->block_classes = L->block_classes;
    info->prefill_kernel = L->path == 1 ? (L->gemm_staged_from == 0 ? SKL_PREFILL_STAGED : SKL_PREFILL_FUSED) : SKL_PREFILL_PER_WEIGHT;
    info->n_blocks = L->path == 1 ? L->n_blocks : 0;
    info->prefill_staged_from = L->path == 1 ? L->gemm_staged_from : 0xFFFFFFFFu;
    return SKL_OK;
}

skl_status_t sketch_linear_info(const skl_layer_t *L, skl_info_t *info)
{
    if (!L || !info) FAIL(SKL_ERR_INVALID_ARG, "layer or info is NULL");
    return fill_info(L, info);
}

skl_status_t sketch_linear_plan(const skl_desc_t *desc, uint32_t segments, uint32_t groups, skl_info_t *info, double *decode_cost_us)
{
    if (!info) FAIL(SKL_ERR_INVALID_ARG, "info is NULL");
    if ((segments == 0) != (groups == 0)) FAIL(SKL_ERR_INVALID_ARG, "segments and groups must both be 0 or both be given");
    skl_plan P;
    P.want_s = segments; P.want_g = groups;
    skl_status_t st = skl_make_plan(desc, &P);
    if (st != SKL_OK) return st;
    if (segments && (P.L.path != 1 || P.L.n_sseg != segments || P.L.n_bg != groups))
        FAIL(SKL_ERR_UNSUPPORTED, "the decode kernels cannot run %u output segments x %u block groups on this layer", segments, groups);
    if (decode_cost_us) *decode_cost_us = P.L.path == 1 ? P.L.decode_cost_us : 0.0;
    return fill_info(&P.L, info);
}

skl_status_t sketch_linear_workspace_bytes(const skl_layer_t *L, uint32_t op, uint32_t n, uint64_t *bytes)
{
    if (!L || !bytes) FAIL(SKL_ERR_INVALID_ARG, "layer or bytes is NULL");
    if (op == 0) {
        if (n < 1 || n > 16) FAIL(SKL_ERR_INVALID_ARG, "batch = %u, must be 1..16", n);
        *bytes = skl_gemv_workspace_bytes(L, n);
    } else if (op == 1) {
        if (n < 1) FAIL(SKL_ERR_INVALID_ARG, "tokens must be positive");
        *bytes = skl_gemm_workspace_bytes(L, n);
    } else if (op == 2) {
        *bytes = skl_reconstruct_workspace_bytes(L);
    } else {
        FAIL(SKL_ERR_INVALID_ARG, "op = %u, must be 0 (gemv), 1 (gemm) or 2 (reconstruct)", op);
    }
    return SKL_OK;
}

static bool overlap(const void *a, uint64_t na, const void *b, uint64_t nb)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

static uint32_t dtype_size(skl_dtype_t t) { return t == SKL_F32 ? 4 : 2; }

static skl_status_t check_io(const skl_layer_t *L, const void *x, uint32_t ldx, uint32_t x_size, const void *y,
                             uint32_t ldy, uint32_t y_size, uint32_t rows, const void *ws, uint64_t ws_bytes,
                             uint64_t ws_need)
{
    if (!x || !y) FAIL(SKL_ERR_INVALID_ARG, "activation or output pointer is NULL");
    if ((uintptr_t)x % 16 || (uintptr_t)y % 16) FAIL(SKL_ERR_INVALID_ARG, "activation/output pointer not 16-byte aligned");
    if (ldx < L->in) FAIL(SKL_ERR_INVALID_ARG, "ldx = %u is smaller than in_features = %u", ldx, L->in);
    if (ldy < L->out) FAIL(SKL_ERR_INVALID_ARG, "ldy = %u is smaller than out_features = %u", ldy, L->out);
    const uint64_t xb = ((uint64_t)(rows - 1) * ldx + L->in) * x_size;
    const uint64_t yb = ((uint64_t)(rows - 1) * ldy + L->out) * y_size;
    if (overlap(x, xb, y, yb)) FAIL(SKL_ERR_INVALID_ARG, "input and output overlap");
    if (ws_need) {
        if (!ws) FAIL(SKL_ERR_INVALID_ARG, "workspace is NULL (%llu bytes needed)", (unsigned long long)ws_need);
        if ((uintptr_t)ws % 16) FAIL(SKL_ERR_INVALID_ARG, "workspace not 16-byte aligned");
        if (ws_bytes < ws_need)
            FAIL(SKL_ERR_BUFFER_TOO_SMALL, "workspace holds %llu bytes, %llu needed", (unsigned long long)ws_bytes,
                 (unsigned long long)ws_need);
        if (overlap(ws, ws_need, y, yb) || overlap(ws, ws_need, x, xb))
            FAIL(SKL_ERR_INVALID_ARG, "workspace overlaps input or output");
    }
    return SKL_OK;
}

skl_status_t sketch_linear_gemv(const skl_layer_t *L, const void *x, skl_dtype_t x_dt, uint32_t ldx, void *y,
                                skl_dtype_t y_dt, uint32_t ldy, uint32_t batch, void *ws, uint64_t ws_bytes,
                                void *stream)
{
    if (!L) FAIL(SKL_ERR_INVALID_ARG, "layer is NULL");
    if (batch < 1 || batch > 16) FAIL(SKL_ERR_INVALID_ARG, "batch = %u, must be 1..16", batch);
    if (x_dt != SKL_F16) FAIL(SKL_ERR_UNSUPPORTED, "gemv activations must be binary16");
    if (y_dt != SKL_F16 && y_dt != SKL_F32) FAIL(SKL_ERR_UNSUPPORTED, "gemv output must be binary16 or float32");
    skl_status_t st = check_io(L, x, ldx, 2, y, ldy, dtype_size(y_dt), batch, ws, ws_bytes,
                               skl_gemv_workspace_bytes(L, batch));
    if (st != SKL_OK) return st;
    return skl_launch_gemv(L, x, ldx, y, y_dt, ldy, batch, ws, stream, true);
}

skl_status_t sketch_linear_gemv_static(const skl_layer_t *L, const void *x, skl_dtype_t x_dt, uint32_t ldx, void *y,
                                       skl_dtype_t y_dt, uint32_t ldy, uint32_t batch, void *stream)
{
    if (!L) FAIL(SKL_ERR_INVALID_ARG, "layer is NULL");
    if (batch < 1 || batch > 16) FAIL(SKL_ERR_INVALID_ARG, "batch = %u, must be 1..16", batch);
    if (x_dt != SKL_F16) FAIL(SKL_ERR_UNSUPPORTED, "gemv activations must be binary16");
    if (y_dt != SKL_F16 && y_dt != SKL_F32) FAIL(SKL_ERR_UNSUPPORTED, "gemv output must be binary16 or float32");
    const uint64_t need = skl_gemv_workspace_bytes(L, batch);
    if (need > skl_static_scratch_bytes())
        FAIL(SKL_ERR_UNSUPPORTED, "this call needs %llu bytes of scratch, the static array holds %llu; use sketch_linear_gemv",
             (unsigned long long)need, (unsigned long long)skl_static_scratch_bytes());
    skl_status_t st = check_io(L, x, ldx, 2, y, ldy, dtype_size(y_dt), batch, nullptr, 0, 0);
    if (st != SKL_OK) return st;
    return skl_launch_gemv_static(L, x, ldx, y, y_dt, ldy, batch, stream);
}

skl_status_t sketch_linear_gemv_partials(const skl_layer_t *L, const void *x, skl_dtype_t x_dt, uint32_t ldx,
                                         uint32_t batch, void *ws, uint64_t ws_bytes, void *stream)
{
    if (!L) FAIL(SKL_ERR_INVALID_ARG, "layer is NULL");
    if (batch < 1 || batch > 16) FAIL(SKL_ERR_INVALID_ARG, "batch = %u, must be 1..16", batch);
    if (x_dt != SKL_F16) FAIL(SKL_ERR_UNSUPPORTED, "gemv activations must be binary16");
    const uint64_t need = skl_gemv_workspace_bytes(L, batch);
    if (!x || !ws) FAIL(SKL_ERR_INVALID_ARG, "activation or workspace pointer is NULL");
    if ((uintptr_t)x % 16 || (uintptr_t)ws % 16) FAIL(SKL_ERR_INVALID_ARG, "activation/workspace pointer not 16-byte aligned");
    if (ldx < L->in) FAIL(SKL_ERR_INVALID_ARG, "ldx = %u is smaller than in_features = %u", ldx, L->in);
    if (ws_bytes < need)
        FAIL(SKL_ERR_BUFFER_TOO_SMALL, "workspace holds %llu bytes, %llu needed", (unsigned long long)ws_bytes,
             (unsigned long long)need);
    if (overlap(ws, need, x, ((uint64_t)(batch - 1) * ldx + L->in) * 2))
        FAIL(SKL_ERR_INVALID_ARG, "workspace overlaps the activations");
    return skl_launch_gemv(L, x, ldx, nullptr, SKL_F32, 0, batch, ws, stream, false);
}

skl_status_t sketch_linear_gemm(const skl_layer_t *L, const void *X, skl_dtype_t x_dt, uint32_t ldx, void *Y,
                                skl_dtype_t y_dt, uint32_t ldy, uint32_t tokens, void *ws, uint64_t ws_bytes,
                                void *stream)
{
    if (!L) FAIL(SKL_ERR_INVALID_ARG, "layer is NULL");
    if (tokens < 1) FAIL(SKL_ERR_INVALID_ARG, "tokens must be positive");
    if (tokens > (1u << 24)) FAIL(SKL_ERR_UNSUPPORTED, "more than 2^24 tokens in one call");
    if (x_dt != SKL_F16 && x_dt != SKL_BF16) FAIL(SKL_ERR_UNSUPPORTED, "gemm activations must be bfloat16 or binary16");
    if (y_dt != SKL_F16 && y_dt != SKL_BF16 && y_dt != SKL_F32) FAIL(SKL_ERR_INVALID_ARG, "bad output dtype");
    // grid limits of the kernels behind this call, checked before anything is enqueued
    if (L->path == 1 && tokens > 8191u * 256u) FAIL(SKL_ERR_UNSUPPORTED, "more than %u tokens in one call through a row-sketch layer", 8191u * 256u);
    if (L->path == 0 && tokens > 65535u * 64u) FAIL(SKL_ERR_UNSUPPORTED, "more than %u tokens in one call through the per-weight path", 65535u * 64u);
    skl_status_t st = check_io(L, X, ldx, 2, Y, ldy, dtype_size(y_dt), tokens, ws, ws_bytes,
                               skl_gemm_workspace_bytes(L, tokens));
    if (st != SKL_OK) return st;
    return skl_launch_gemm(L, X, x_dt, ldx, Y, y_dt, ldy, tokens, ws, stream);
}

// ---- several layers on the same activations, one launch --------------------
static skl_status_t check_group(const skl_layer_t *const *layers, uint32_t n_layers, uint32_t batch)
{
    if (!layers) FAIL(SKL_ERR_INVALID_ARG, "layers is NULL");
    if (n_layers < 1 || n_layers > 4) FAIL(SKL_ERR_INVALID_ARG, "n_layers = %u, must be 1..4", n_layers);
    if (batch < 1 || batch > 16) FAIL(SKL_ERR_INVALID_ARG, "batch = %u, must be 1..16", batch);
    for (uint32_t i = 0; i < n_layers; ++i)
        if (!layers[i]) FAIL(SKL_ERR_INVALID_ARG, "layers[%u] is NULL", i);
    return SKL_OK;
}

skl_status_t sketch_linear_gemv_group_workspace_bytes(const skl_layer_t *const *layers, uint32_t n_layers, uint32_t batch,
                                                      uint64_t *bytes)
{
    if (!bytes) FAIL(SKL_ERR_INVALID_ARG, "bytes is NULL");
    skl_status_t st = check_group(layers, n_layers, batch);
    if (st != SKL_OK) return st;
    *bytes = skl_gemv_group_workspace_bytes(layers, n_layers, batch);
    return SKL_OK;
}

skl_status_t sketch_linear_gemv_group(const skl_layer_t *const *layers, uint32_t n_layers, const void *x, skl_dtype_t x_dt,
                                      uint32_t ldx, void *const *ys, skl_dtype_t y_dt, uint32_t ldy, uint32_t batch, void *ws,
                                      uint64_t ws_bytes, void *stream)
{
    skl_status_t st = check_group(layers, n_layers, batch);
    if (st != SKL_OK) return st;
    if (!ys) FAIL(SKL_ERR_INVALID_ARG, "ys is NULL");
    if (x_dt != SKL_F16) FAIL(SKL_ERR_UNSUPPORTED, "gemv activations must be binary16");
    if (y_dt != SKL_F16 && y_dt != SKL_F32) FAIL(SKL_ERR_UNSUPPORTED, "gemv output must be binary16 or float32");
    const uint64_t need = skl_gemv_group_workspace_bytes(layers, n_layers, batch);
    for (uint32_t i = 0; i < n_layers; ++i) {
        if (!ys[i]) FAIL(SKL_ERR_INVALID_ARG, "ys[%u] is NULL", i);
        st = check_io(layers[i], x, ldx, 2, ys[i], ldy, dtype_size(y_dt), batch, ws, ws_bytes, need);
        if (st != SKL_OK) return st;
        const uint64_t yb = ((uint64_t)(batch - 1) * ldy + layers[i]->out) * dtype_size(y_dt);
        for (uint32_t k = 0; k < i; ++k)
            if (overlap(ys[i], yb, ys[k], ((uint64_t)(batch - 1) * ldy + layers[k]->out) * dtype_size(y_dt)))
                FAIL(SKL_ERR_INVALID_ARG, "outputs %u and %u overlap", k, i);
    }
    return skl_launch_gemv_group(layers, n_layers, x, ldx, ys, y_dt, ldy, batch, ws, stream, false);
}

skl_status_t sketch_linear_gemv_gate_up(const skl_layer_t *gate, const skl_layer_t *up, const void *x, skl_dtype_t x_dt,
                                        uint32_t ldx, void *h, skl_dtype_t h_dt, uint32_t ldh, uint32_t batch, void *ws,
                                        uint64_t ws_bytes, void *stream)
{
    if (!gate || !up) FAIL(SKL_ERR_INVALID_ARG, "gate or up layer is NULL");
    if (batch < 1 || batch > 16) FAIL(SKL_ERR_INVALID_ARG, "batch = %u, must be 1..16", batch);
    if (x_dt != SKL_F16) FAIL(SKL_ERR_UNSUPPORTED, "gemv activations must be binary16");
    if (h_dt != SKL_F16 && h_dt != SKL_F32) FAIL(SKL_ERR_UNSUPPORTED, "gemv output must be binary16 or float32");
    const skl_layer_t *layers[2] = {gate, up};
    const uint64_t need = skl_gemv_group_workspace_bytes(layers, 2, batch);
    skl_status_t st = check_io(gate, x, ldx, 2, h, ldh, dtype_size(h_dt), batch, ws, ws_bytes, need);
    if (st != SKL_OK) return st;
    void *ys[2] = {h, h};
    return skl_launch_gemv_group(layers, 2, x, ldx, ys, h_dt, ldh, batch, ws, stream, true);
}

// ---- sketch construction on the device ------------------------------------
static uint64_t build_workspace_bytes(const skl_desc_t *d, uint64_t n_groups)
{
    // 64-bit keys of all states, then the state offset and the width of every group
    return align_up(d->n_states * 8, 256) + align_up((n_groups + 1) * 8, 256) + align_up(n_groups * 4, 256);
}

skl_status_t sketch_linear_build_workspace_bytes(const skl_desc_t *user, uint64_t *bytes)
{
    if (!bytes) FAIL(SKL_ERR_INVALID_ARG, "bytes is NULL");
    skl_desc_t d;
    skl_status_t st = normalize_desc(user, &d);
    if (st != SKL_OK) return st;
    uint64_t n_groups = 0;
    st = validate_desc(&d, &n_groups, true);
    if (st != SKL_OK) return st;
    *bytes = build_workspace_bytes(&d, n_groups);
    return SKL_OK;
}

skl_status_t sketch_linear_build_states(const skl_desc_t *user, const uint16_t *W_dev, uint16_t *states_dev, void *ws,
                                        uint64_t ws_bytes, void *stream_)
{
    skl_desc_t d;
    skl_status_t st = normalize_desc(user, &d);
    if (st != SKL_OK) return st;
    uint64_t n_groups = 0;
    st = validate_desc(&d, &n_groups, true);
    if (st != SKL_OK) return st;
    if (!W_dev || !states_dev || !ws) FAIL(SKL_ERR_INVALID_ARG, "W_dev, states_dev or workspace is NULL");
    if ((uintptr_t)W_dev % 16 || (uintptr_t)states_dev % 2 || (uintptr_t)ws % 256)
        FAIL(SKL_ERR_INVALID_ARG, "W_dev must be 16-byte, states_dev 2-byte, workspace 256-byte aligned");
    const uint64_t need = build_workspace_bytes(&d, n_groups);
    if (ws_bytes < need)
        FAIL(SKL_ERR_BUFFER_TOO_SMALL, "workspace holds %llu bytes, %llu needed", (unsigned long long)ws_bytes,
             (unsigned long long)need);
    const uint64_t w_bytes = (uint64_t)d.in_features * d.out_features * 2;
    if (overlap(ws, need, W_dev, w_bytes) || overlap(ws, need, states_dev, d.n_states * 2) ||
        overlap(W_dev, w_bytes, states_dev, d.n_states * 2))
        FAIL(SKL_ERR_INVALID_ARG, "W_dev, states_dev and workspace overlap");
    std::vector<uint64_t> base;
    try {
        base.assign(n_groups + 1, 0);
    } catch (const std::bad_alloc &) {
        FAIL(SKL_ERR_NO_MEMORY, "out of host memory for the offsets of %llu groups", (unsigned long long)n_groups);
    }
    for (uint64_t g = 0; g < n_groups; ++g) base[g + 1] = base[g] + (uint64_t)d.d * d.group_width[g];
    return skl_launch_build(&d, n_groups, base.data(), W_dev, states_dev, ws, stream_);
}

skl_status_t sketch_linear_prefill_split(uint32_t kernel, uint32_t out_features, uint32_t n_blocks, uint32_t tokens,
                                         uint32_t *segments, uint64_t capacity, uint64_t *n_segments, uint32_t *shape)
{
    if (kernel != SKL_PREFILL_FUSED && kernel != SKL_PREFILL_STAGED)
        FAIL(SKL_ERR_INVALID_ARG, "kernel = %u, must be SKL_PREFILL_FUSED or SKL_PREFILL_STAGED", kernel);
    if (!n_segments) FAIL(SKL_ERR_INVALID_ARG, "n_segments is NULL");
    if (!segments && capacity) FAIL(SKL_ERR_INVALID_ARG, "segments is NULL with a non-zero capacity");
    if (out_features < 1 || n_blocks < 1 || tokens < 1) FAIL(SKL_ERR_INVALID_ARG, "out_features, n_blocks and tokens must be positive");
    if (tokens > (1u << 24)) FAIL(SKL_ERR_UNSUPPORTED, "more than 2^24 tokens in one call");
    *n_segments = skl_gemm3_segments(out_features, n_blocks, tokens, kernel == SKL_PREFILL_STAGED, segments, capacity, shape);
    return SKL_OK;
}

static skl_status_t reconstruct_with(const skl_layer_t *L, uint16_t *W_hat_dev, void *ws, uint64_t ws_bytes, void *stream, bool naive)
{
    if (!L || !W_hat_dev) FAIL(SKL_ERR_INVALID_ARG, "layer or W_hat_dev is NULL");
    if ((uintptr_t)W_hat_dev % 16) FAIL(SKL_ERR_INVALID_ARG, "W_hat_dev not 16-byte aligned");
    const uint64_t need = skl_reconstruct_workspace_bytes(L);
    if (need) {
        if (!ws) FAIL(SKL_ERR_INVALID_ARG, "workspace is NULL (%llu bytes needed)", (unsigned long long)need);
        if ((uintptr_t)ws % 16) FAIL(SKL_ERR_INVALID_ARG, "workspace not 16-byte aligned");
        if (ws_bytes < need)
            FAIL(SKL_ERR_BUFFER_TOO_SMALL, "workspace holds %llu bytes, %llu needed", (unsigned long long)ws_bytes,
                 (unsigned long long)need);
        if (overlap(ws, need, W_hat_dev, (uint64_t)L->in * L->out * 2))
            FAIL(SKL_ERR_INVALID_ARG, "workspace overlaps W_hat_dev");
    }
    return naive ? skl_launch_reconstruct_naive(L, W_hat_dev, ws, stream) : skl_launch_reconstruct(L, W_hat_dev, ws, stream);
}

skl_status_t sketch_linear_reconstruct(const skl_layer_t *L, uint16_t *W_hat_dev, void *ws, uint64_t ws_bytes, void *stream)
{
    return reconstruct_with(L, W_hat_dev, ws, ws_bytes, stream, false);
}

skl_status_t sketch_linear_reconstruct_hash_op(const skl_layer_t *L, uint16_t *W_hat_dev, void *ws, uint64_t ws_bytes,
                                               void *stream)
{
    return reconstruct_with(L, W_hat_dev, ws, ws_bytes, stream, true);
}

skl_status_t sketch_linear_microbench(uint32_t kind, uint32_t iters, void *ws, uint64_t ws_bytes, void *stream, uint64_t *work)
{
    if (kind > 4)
        FAIL(SKL_ERR_INVALID_ARG, "kind = %u, must be 0 (vector ALU), 1 (LDS), 2 (matrix cores), 3 (HBM read) or 4 (matrix cores, random operand bits)", kind);
    if (!ws || (uintptr_t)ws % 256) FAIL(SKL_ERR_INVALID_ARG, "workspace is NULL or not 256-byte aligned");
    if (kind != 3 && (iters < 1 || iters > (1u << 20))) FAIL(SKL_ERR_INVALID_ARG, "iters = %u, must be 1..2^20", iters);
    if (!work) FAIL(SKL_ERR_INVALID_ARG, "work is NULL");
    const skl_status_t st = skl_launch_microbench(kind, iters, ws, ws_bytes, stream);
    if (st == SKL_OK) *work = skl_microbench_work(kind, iters, ws_bytes);
    return st;
}

}  // extern "C"
