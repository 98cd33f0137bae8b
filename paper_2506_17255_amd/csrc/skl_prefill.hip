// Fused prefill GEMM over row sketches on the matrix cores (Sec. 3.1 Eq. 5
// fused with Y = X W, Sec. 2.1): the 256 x 256-tile kernel, its work split,
// the fix-up pass, and the launcher that picks a kernel.
#include "skl_prefill_common.h"

namespace SKL_NS {


// ---- activation re-ordering pre-pass ----------------------------------------
// Converts X to negated binary16 and lays it out as the matrix-core A words of the product kernels:
// word (token tile, step, row block of 32 tokens, half q, token n) holds the eight channels 8q .. 8q + 7 of
// the step for one token.  A workgroup takes one row block x PK_STEPS steps and builds its words in LDS rows.
// Phase 1: a thread owns one of the 2 * PK_STEPS words for 32 / PK_PARTS of the 32 tokens.  Where the word's
// eight channels are neighbours in X (the width order moves few channels, so nearly every word) it is cut
// out of the one or two aligned 16-byte pieces of the row that hold it, all loads in flight at once; a
// wavefront then reads about one contiguous KiB of a token's row.  The other words (they span a moved
// channel, or end the channel list) are noted and fetched channel by channel by the whole workgroup, so that
// no wavefront walks the slow path for a few of its lanes.  Phase 2: a wavefront writes one step's 64 words
// -- one contiguous KiB -- from 16-byte LDS reads that spread over all banks (row stride 1040 bytes).
// grid (ceil(tokens / 32), ceil(steps / PK_STEPS)); LDS PK_LDS_BYTES
#define PK_STEPS 32u
#define PK_STRIDE (PK_STEPS * 16u + 8u)          // halfs per LDS row
#define PK_LDS_BYTES (32u * PK_STRIDE * 2u + 4u * (1u + 9u * 2u * PK_STEPS) + 12u)
#define PK_PARTS (SKL_WG / (2u * PK_STEPS))     // threads per word: each takes 32 / PK_PARTS tokens
static_assert(2 * PK_STEPS * PK_PARTS == SKL_WG && 32 % PK_PARTS == 0, "one thread per (word, part of the row block)");

__device__ __forceinline__ uint32_t neg_half_pair(uint32_t e, uint32_t x_dt)
{
    if (x_dt == SKL_BF16) {
        const uint32_t lo = float_to_half_bits(__builtin_bit_cast(float, e << 16));
        const uint32_t hi = float_to_half_bits(__builtin_bit_cast(float, e & 0xFFFF0000u));
        e = lo | (hi << 16);
    }
    return e ^ 0x80008000u;
}

__global__ __launch_bounds__(SKL_WG) void k_pack_activations3(const uint16_t *__restrict__ X, uint32_t x_dt, uint32_t ldx,
                                                               uint32_t tokens, uint32_t in, const uint32_t *__restrict__ chan,
                                                               const skl_gemm_step *__restrict__ steps, uint32_t n_steps,
                                                               uint4 *__restrict__ Xp)
{
    uint16_t *rows = reinterpret_cast<uint16_t *>(smem);
    uint32_t *slow = reinterpret_cast<uint32_t *>(rows + 32 * PK_STRIDE);     // count, then (word, eight channels) per noted word
    const uint32_t t0 = blockIdx.x * 32, s0 = blockIdx.y * PK_STEPS;
    const uint32_t ns = min(PK_STEPS, n_steps - s0);
    if (threadIdx.x == 0) slow[0] = 0;
    __syncthreads();
    {
        const uint32_t word = threadIdx.x & (2 * PK_STEPS - 1), part = threadIdx.x / (2 * PK_STEPS);   // word = 2 * step + q
        const uint32_t step = word >> 1, q = word & 1;
        uint32_t ch[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) ch[i] = SKL_NO_CHANNEL;
        if (step < ns) {
            const skl_gemm_step st = steps[s0 + step];
            if (q < st.n_words) {
                const uint4 c0 = *reinterpret_cast<const uint4 *>(chan + st.chan0 + 8 * q);       // chan0 is a multiple of 8
                const uint4 c1 = *reinterpret_cast<const uint4 *>(chan + st.chan0 + 8 * q + 4);
                ch[0] = c0.x; ch[1] = c0.y; ch[2] = c0.z; ch[3] = c0.w; ch[4] = c1.x; ch[5] = c1.y; ch[6] = c1.z; ch[7] = c1.w;
            }
        }
        // a word whose eight channels are neighbours in X is cut out of the one or two aligned 16-byte pieces
        // of the row that hold it (rows must be 16-byte aligned and long enough for the second piece)
        bool run = ch[0] != SKL_NO_CHANNEL && (ldx & 7u) == 0 && (reinterpret_cast<uintptr_t>(X) & 15u) == 0;
#pragma unroll
        for (int i = 1; i < 8; ++i) run = run && ch[i] == ch[0] + i;
        const uint32_t sh = ch[0] & 7u, base = ch[0] - sh;                 // the word starts sh halfs into the piece at column base
        run = run && (sh == 0 || base + 16 <= in);                          // the second piece lies inside the row
        constexpr uint32_t TPT = 32 / PK_PARTS;                     // tokens per thread
        if (run) {
            uint4 e[TPT], f[TPT];
#pragma unroll
            for (uint32_t j = 0; j < TPT; ++j) {
                const uint32_t t = min(t0 + part * TPT + j, tokens - 1);           // rows past the end re-read the last one
                const uint4 *src = reinterpret_cast<const uint4 *>(X + (size_t)t * ldx + base);
                e[j] = src[0];
                f[j] = sh ? src[1] : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (uint32_t j = 0; j < TPT; ++j) {
                const uint32_t t = part * TPT + j;
                // halfs sh .. sh + 7 of the sixteen: drop four, two, one half in turn
                uint32_t d[8] = {e[j].x, e[j].y, e[j].z, e[j].w, f[j].x, f[j].y, f[j].z, f[j].w};
                if (sh & 4u) { d[0] = d[2]; d[1] = d[3]; d[2] = d[4]; d[3] = d[5]; d[4] = d[6]; d[5] = d[7]; }
                if (sh & 2u) { d[0] = d[1]; d[1] = d[2]; d[2] = d[3]; d[3] = d[4]; d[4] = d[5]; }
                if (sh & 1u) {
                    d[0] = __builtin_amdgcn_alignbit(d[1], d[0], 16); d[1] = __builtin_amdgcn_alignbit(d[2], d[1], 16);
                    d[2] = __builtin_amdgcn_alignbit(d[3], d[2], 16); d[3] = __builtin_amdgcn_alignbit(d[4], d[3], 16);
                }
                uint4 w = make_uint4(neg_half_pair(d[0], x_dt), neg_half_pair(d[1], x_dt), neg_half_pair(d[2], x_dt), neg_half_pair(d[3], x_dt));
                if (t0 + t >= tokens) w = make_uint4(0, 0, 0, 0);
                *reinterpret_cast<uint4 *>(rows + t * PK_STRIDE + word * 8) = w;
            }
        } else if (part == 0) {
            // a word that spans a moved channel (or ends the channel list): noted for the pass below, where the
            // whole workgroup fetches such words channel by channel
            const uint32_t e = atomicAdd(&slow[0], 1u);
            slow[1 + 9 * e] = word;
#pragma unroll
            for (int i = 0; i < 8; ++i) slow[2 + 9 * e + i] = ch[i];
        }
    }
    __syncthreads();
    {
        const uint32_t n_slow = slow[0];
        for (uint32_t idx = threadIdx.x; idx < n_slow * 256; idx += SKL_WG) {      // (word, token, channel slot)
            const uint32_t e = idx >> 8, t = (idx >> 3) & 31, i = idx & 7;
            const uint32_t word = slow[1 + 9 * e], c = slow[2 + 9 * e + i];
            rows[t * PK_STRIDE + word * 8 + i] =
                c != SKL_NO_CHANNEL && t0 + t < tokens ? load_neg_half(X + (size_t)(t0 + t) * ldx, x_dt, c) : (uint16_t)0;
        }
    }
    __syncthreads();
    const uint32_t n = threadIdx.x & 31, q = (threadIdx.x >> 5) & 1;
    const uint32_t tile_m = t0 / GM_MT, rb = (t0 % GM_MT) / 32;
    for (uint32_t step = threadIdx.x >> 6; step < ns; step += SKL_WG / 64) {
        const uint4 w = *reinterpret_cast<const uint4 *>(rows + n * PK_STRIDE + step * 16 + q * 8);
        Xp[(((size_t)tile_m * n_steps + s0 + step) * 8 + rb) * 64 + q * 32 + n] = w;
    }
}


// ---- prefill, third kernel: 256 tokens x 256 outputs per workgroup ---------
// The table stream of a workgroup does not depend on the width of its tile, so
// a tile twice as wide halves the traffic between L2 and the CUs, which is what
// bounds the second kernel.  65536 accumulators need all 512 registers of four
// wavefronts (one per SIMD), so there are no separate producer wavefronts:
// every wavefront owns 64 tokens x 256 outputs (16 accumulator blocks), and
// while its 64 MFMAs of block k run it rebuilds the operand words of block k+1
// for two of the eight column blocks (gather/query/decode between the MFMAs),
// fetches the table of block k+2 through registers and requests its
// activation words two blocks ahead.  Blocks with fewer than eight words per
// state row are rebuilt before the MFMAs instead (rare classes).

template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_row_gemm3(Gemm2Args p)
{
    const uint32_t xcd = blockIdx.x & 7, wg = blockIdx.x >> 3;
    G3Split sp;
    sp.T = p.T; sp.m_tiles = p.m_tiles; sp.nb = p.n_blocks; sp.gx = p.gx; sp.l_max = p.l_max; sp.p_cap = p.p_cap;
    sp.mu = 1; sp.n_col = p.n_col; sp.mt = GM_MT; sp.single = 0;
    uint32_t round = 0, u_next = sp.share_begin(xcd, wg);
    if (sp.rounds(xcd) == 0 && u_next >= sp.share_begin(xcd, wg + 1)) return;
    const uint32_t lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void *)smem;
    const uint32_t tab_bytes = p.tab_words * 16;
    const uint32_t slot_base = lds0 + 2 * tab_bytes;                               // two operand slots
    const uint32_t dummy_addr = slot_base + 2 * G3_SLOT_BYTES + lane * 16;         // 1 KiB nobody reads
    const uint32_t meta_word = (2 * tab_bytes + 2 * G3_SLOT_BYTES + 1024) / 16;
    const uint4 *sm_meta = smem + meta_word;                                       // block metadata, two words per block
    {
        uint4 *meta_w = smem + meta_word;
        const uint4 *gm = reinterpret_cast<const uint4 *>(p.bmeta);
        for (uint32_t i = threadIdx.x; i < 2 * p.n_blocks; i += 256) meta_w[i] = gm[i];
    }
    __syncthreads();

    const uint32_t n = lane & 31, q = lane >> 5;
    uint32_t t0 = 0, o_first = 0;                               // of the current tile: first token of the wavefront; first
                                                                // output of the two column blocks it rebuilds (2*wave, 2*wave + 1)
    float16v acc[16];                                           // [row block][column block]

    // ---- table of a block: global -> registers -> LDS, this wavefront's quarter of the 1 KiB chunks
    // (12 at most), three per MFMA step so that only three registers' worth is in flight at a time
    auto table_step_load = [&](const uint4 *src, uint32_t last, int s, uint4 (&tr)[3]) {
#pragma unroll
        for (int i = 0; i < 3; ++i) tr[i] = src[(size_t)min(wave + 4 * (3 * s + i), last) * 64];   // past the end: the last chunk again
    };
    auto table_step_store = [&](uint4 *dst, uint32_t last, int s, const uint4 (&tr)[3]) {
#pragma unroll
        for (int i = 0; i < 3; ++i) dst[min(wave + 4 * (3 * s + i), last) * 64] = tr[i];
    };
    // source, destination and last chunk of block b's table (b clamped to the last block)
    auto table_of = [&](uint32_t b, const uint4 *&src, uint4 *&dst, uint32_t &last) {
        b = min(b, p.n_blocks - 1);
        const uint4 m0 = sm_meta[2 * b], m1 = sm_meta[2 * b + 1];
        last = ((D * m0.y * m0.w + 63) >> 6) - 1;
        src = p.ptables + m1.y + lane;
        dst = smem + (b & 1) * p.tab_words + lane;
    };
    auto table_whole = [&](uint32_t b) {                        // start-up only
        const uint4 *src; uint4 *dst; uint32_t last;
        table_of(b, src, dst, last);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint4 tr[3];
            table_step_load(src, last, s, tr);
            table_step_store(dst, last, s, tr);
        }
    };
    // ---- activation words
    const uint4 *xa = p.Xp;
    uint4 a[4][2];                                              // [step][row block] of the block being multiplied
    // request the activation words of step s of block b (a page of zeros for steps the block does not
    // have, the last block again past the end: every path issues the same loads)
    auto load_a_step = [&](uint32_t ns, uint32_t s0, int s) {      // ns steps from step s0 on
        const uint4 *src = (uint32_t)s < ns ? xa + (size_t)(s0 + s) * 512 : p.zeros + lane;
        const uint4 *src1 = (uint32_t)s < ns ? src + 64 : src;
        a[s][0] = src[0];
        a[s][1] = src1[0];
    };
    // ---- rebuild state for blocks of NB = 8 or 4 words per state row: a gather instruction of the wavefront
    // covers 64 / NB outputs times NB words (a "set"); a column block has NB / 2 sets, the wavefront's two
    // column blocks have NB, numbered column block first.  LDS byte offsets inside a table, [set][row]
    uint32_t off[8][D];
#pragma unroll
    for (int st = 0; st < 8; ++st)
#pragma unroll
        for (int r = 0; r < D; ++r) off[st][r] = (lane & 3) * 16;
    uint32_t K_prev = 0, nb_prev = 0;
    auto fast_offsets = [&](bool nb4, uint32_t K) {
        const uint32_t NB = nb4 ? 4 : 8;
        if (K == K_prev && nb_prev == NB) return;
        K_prev = K;
        nb_prev = NB;
        const uint32_t Kq = K << 8, sub = nb4 ? lane >> 2 : lane >> 3, cw = nb4 ? lane & 3 : lane & 7;
        const uint32_t sh = nb4 ? 1 : 2, ops = nb4 ? 16 : 8;   // sets per column block (as a shift), outputs per set
        uint32_t of = o_first;
        asm volatile("" : "+v"(of));
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            const uint32_t se = nb4 ? st & 3 : st;             // four words per state row: sets 4..7 repeat sets 0..3
            const uint32_t o = min(of + (se >> sh) * 32 + (se & ((1u << sh) - 1)) * ops + sub, p.out - 1);
#pragma unroll
            for (int r = 0; r < D; ++r) {
                const uint32_t t = __umul24(p.h.A[r], o) + p.h.C[r];
                off[st][r] = ((r * K + select_index(t, Kq)) * NB + cw) * 16;
            }
        }
    };
    // rebuild before the MFMAs (first block, and blocks of the narrow classes)
    auto build_plain = [&](uint32_t b) {
        const uint4 m0 = sm_meta[2 * b];
        const uint32_t K = m0.y, nb = m0.w;
        const uint32_t tab_addr = lds0 + (b & 1) * tab_bytes, slot_addr = slot_base + (b & 1) * G3_SLOT_BYTES;
        uint32_t o2[4][D];
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2) {
            const uint32_t of = o_first + c2 * 32, cb = wave * 2 + c2;
            if (nb == 8) {
                if constexpr (D <= 6) { g2_offsets<D, 8>(p.h, of, p.out, K, lane, o2); g2_build<D, 8>(o2, tab_addr, slot_addr, cb, lane); }
            } else if (nb == 4) { g2_offsets<D, 4>(p.h, of, p.out, K, lane, o2); g2_build<D, 4>(o2, tab_addr, slot_addr, cb, lane);
            } else if (nb == 2) { g2_offsets<D, 2>(p.h, of, p.out, K, lane, o2); g2_build<D, 2>(o2, tab_addr, slot_addr, cb, lane);
            } else { g2_offsets<D, 1>(p.h, of, p.out, K, lane, o2); g2_build<D, 1>(o2, tab_addr, slot_addr, cb, lane); }
        }
    };
    const uint32_t b_lane = slot_base + (q * G2_ROW + n) * 16;
    // Table chunks travel global -> registers -> LDS one group of three per MFMA step; a group is
    // requested at the start of one step and written at the end of the next, so that about two
    // steps of MFMAs cover its latency.  Group 0 of table b + 2 is requested in the last step of
    // block b - 1, groups 1..3 in the first three steps of block b; all four are written during block b.
    uint4 tc0, tc1, tc2;
    auto chunk_at = [&](uint32_t grp, uint32_t i, uint32_t last) { return min(wave + 4 * (3 * grp + i), last) * 64; };
    uint4 *const dummy_w = smem + (dummy_addr - lds0) / 16;
    // ---- the MFMAs of block b with everything else of the pipeline between them: operand words of
    // the next step, the rebuild of the next block's operand words for this wavefront's two column
    // blocks (when that block has eight or four words per state row; with four, two steps complete
    // the rebuild and the other two repeat it), table chunks, activation words
    auto block_mma = [&](uint32_t b) {
        const uint32_t P = b & 1;
        const uint32_t bn = min(b + 1, p.n_blocks - 1);
        const uint32_t nb_next = __builtin_amdgcn_readfirstlane(sm_meta[2 * bn].w);
        const bool nb4 = nb_next == 4;
        const bool fast = b + 1 < p.n_blocks && (nb_next == 8 || nb4) && D <= 6;
        if (b + 1 < p.n_blocks && !fast) build_plain(b + 1);
        if (fast) fast_offsets(nb4, sm_meta[2 * bn].y);
        const uint32_t sub = nb4 ? lane >> 2 : lane >> 3, cw = nb4 ? lane & 3 : lane & 7;
        const uint32_t baddr = b_lane + P * G3_SLOT_BYTES;
        const uint32_t tab_next = lds0 + (bn & 1) * tab_bytes;
        const uint32_t slot_next = slot_base + (bn & 1) * G3_SLOT_BYTES;
        // where this lane's rebuilt words go: word cw of output sub of a set; without a rebuild a place nobody reads
        const uint32_t w_lane = fast ? slot_next + ((wave * 16 + cw) * G2_ROW + sub) * 16 : dummy_addr;
        const uint32_t w_sets = __builtin_amdgcn_readfirstlane(fast ? ~0u : 0u);
        const uint32_t a_ns = (sm_meta[2 * bn].w + 1) >> 1, a_s0 = sm_meta[2 * bn + 1].z;     // next block's activation steps
        const uint4 *src2, *src3; uint4 *dst2, *dst3; uint32_t last2, last3;
        table_of(b + 2, src2, dst2, last2);
        table_of(b + 3, src3, dst3, last3);
        const bool t_store = b + 2 < p.n_blocks;
        uint4 bw[8];
        uint4 g[2][D];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            __builtin_amdgcn_sched_barrier(0);
            // -- requests of the step: a table group, (first step) the operand words, the gathers of two rebuild sets
            const uint4 *ls = s < 3 ? src2 : src3;
            const uint32_t ll = s < 3 ? last2 : last3;
            const uint4 tn0 = ls[chunk_at((s + 1) & 3, 0, ll)], tn1 = ls[chunk_at((s + 1) & 3, 1, ll)],
                        tn2 = ls[chunk_at((s + 1) & 3, 2, ll)];
            if (s == 0) {
#pragma unroll
                for (int cb = 0; cb < 8; ++cb) bw[cb] = lds_word_at(baddr + (cb * G3_CB_WORDS) * 16);
            }
            // rebuild: step s does sets 2 s and 2 s + 1.  Its gathers went
            // out late in the step before (the wavefront has nobody to hide an LDS round trip behind); those
            // of the first step cannot: the table is complete only after the block's barrier
            if (s == 0) {
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int r = 0; r < D; ++r) g[h][r] = lds_word_at(tab_next + off[h][r]);
            }
            __builtin_amdgcn_sched_barrier(0);
            uint4 m[2];
            u32x4v w[2];
#pragma unroll
            for (int cb = 0; cb < 8; ++cb) {
                acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                    __builtin_bit_cast(half8v, a[s][0]), __builtin_bit_cast(half8v, bw[cb]), acc[cb], 0, 0, 0);
                acc[8 + cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                    __builtin_bit_cast(half8v, a[s][1]), __builtin_bit_cast(half8v, bw[cb]), acc[8 + cb], 0, 0, 0);
                if (s < 3) bw[cb] = lds_word_at(baddr + (cb * G3_CB_WORDS + 2 * (s + 1) * G2_ROW) * 16);
                if (cb == 3 || cb == 5) {           // query of one set
                    const int h = (cb - 3) >> 1;
                    m[h] = g[h][0];
#pragma unroll
                    for (int r = 1; r < D; ++r) m[h] = pk_max_u16x8(m[h], g[h][r]);
                }
                if (cb == 4 || cb == 6) {           // its decode and its operand word
                    const int h = (cb - 4) >> 1;
                    w[h].x = keys_to_neg_half2_mad(m[h].x); w[h].y = keys_to_neg_half2_mad(m[h].y);
                    w[h].z = keys_to_neg_half2_mad(m[h].z); w[h].w = keys_to_neg_half2_mad(m[h].w);
                    // set 2 s + h; with four words per state row the sets of steps 2 and 3 are those of steps
                    // 0 and 1 again (same gathers, same words, same place: no branch in the MFMA stream)
                    const uint32_t set8 = 2 * s + h, set4 = set8 & 3;
                    const uint32_t term8 = ((set8 >> 2) * 8 * G2_ROW + (set8 & 3) * 8) * 16;
                    const uint32_t term4 = ((set4 >> 1) * 8 * G2_ROW + (set4 & 1) * 16) * 16;
                    const uint32_t dst = w_lane + ((nb4 ? term4 : term8) & w_sets);
                    *(__attribute__((address_space(3))) u32x4v *)(uintptr_t)dst = w[h];
                }
                if (cb == 6 && s < 3) {             // the next step's gathers
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int r = 0; r < D; ++r) g[h][r] = lds_word_at(tab_next + off[2 * (s + 1) + h][r]);
                }
                if (cb == 7) {                      // the table group requested a step ago
                    uint4 *d0 = t_store ? dst2 + chunk_at(s, 0, last2) : dummy_w;
                    uint4 *d1 = t_store ? dst2 + chunk_at(s, 1, last2) : dummy_w;
                    uint4 *d2 = t_store ? dst2 + chunk_at(s, 2, last2) : dummy_w;
                    *d0 = tc0; *d1 = tc1; *d2 = tc2;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // -- next block's activation words into the registers just used
            load_a_step(a_ns, a_s0, s);
            tc0 = tn0; tc1 = tn1; tc2 = tn2;
        }
    };
    // ---- the segments of this workgroup: whole tiles first, then its share of the leftover blocks
    for (;;) {
        G3Split::Seg sg;
        if (!sp.next(xcd, wg, round, u_next, sg)) break;
        const uint32_t k = sg.k, k0 = sg.k0, k1 = sg.k1;
        const bool whole = sg.whole != 0;
        const size_t part_slot = sg.part_slot;
        uint32_t tile_m, tile_n;
        sp.tile_of(xcd, k, tile_m, tile_n);
        t0 = tile_m * GM_MT + wave * 64;
        o_first = tile_n * GM3_NT + wave * 64;
        xa = p.Xp + ((size_t)tile_m * p.n_steps * 8 + wave * 2) * 64 + lane;
        K_prev = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = (float16v){0.f};
        {
            uint4 *slots = smem + 2 * tab_bytes / 16;           // words no rebuild writes meet zero activations: they must not be NaN
            for (uint32_t i = threadIdx.x; i < (2 * G3_SLOT_BYTES + 1024) / 16; i += 256) slots[i] = make_uint4(0, 0, 0, 0);
        }
        table_whole(k0);
#pragma unroll
        for (int s = 0; s < 4; ++s) load_a_step((sm_meta[2 * k0].w + 1) >> 1, sm_meta[2 * k0 + 1].z, s);
        __syncthreads();                                        // table k0 in LDS
        build_plain(k0);
        if (k0 + 1 < p.n_blocks) table_whole(k0 + 1);
        {
            const uint4 *src; uint4 *dst; uint32_t last;
            table_of(k0 + 2, src, dst, last);
            tc0 = src[chunk_at(0, 0, last)]; tc1 = src[chunk_at(0, 1, last)]; tc2 = src[chunk_at(0, 2, last)];
        }
        __syncthreads();                                        // operands of block k0, table k0 + 1
        for (uint32_t kb = k0; kb < k1; ++kb) {
            block_mma(kb);
            __syncthreads();
        }
        // the addresses of the epilogue are formed here, from a lane number the compiler cannot trace back:
        // hoisted out of the segment loop they would sit in scratch memory while the MFMA loop holds every register
        uint32_t ln = lane;
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" : "+v"(ln));       // also: the last MFMA has left the pipeline
        if (whole && p.rows_aligned) {
            const uint32_t lw = lds0 + wave * G3_EPI_BYTES;
            if (p.y_dt == SKL_F32) gemm3_store_rows<SKL_F32>(acc, lw, p.Y, p.ldy, t0, p.tokens, tile_n * GM3_NT, p.out, ln);
            else if (p.y_dt == SKL_F16) gemm3_store_rows<SKL_F16>(acc, lw, p.Y, p.ldy, t0, p.tokens, tile_n * GM3_NT, p.out, ln);
            else gemm3_store_rows<SKL_BF16>(acc, lw, p.Y, p.ldy, t0, p.tokens, tile_n * GM3_NT, p.out, ln);
        } else if (whole) {
            const uint32_t ne = ln & 31, qe = ln >> 5;
            if (p.y_dt == SKL_F32) gemm3_store<SKL_F32>(acc, p.Y, p.ldy, t0, p.tokens, tile_n * GM3_NT + ne, p.out, qe);
            else if (p.y_dt == SKL_F16) gemm3_store<SKL_F16>(acc, p.Y, p.ldy, t0, p.tokens, tile_n * GM3_NT + ne, p.out, qe);
            else gemm3_store<SKL_BF16>(acc, p.Y, p.ldy, t0, p.tokens, tile_n * GM3_NT + ne, p.out, qe);
        } else {
            // partial tile: [wavefront][accumulator block][4 elements][lane], whole 1 KiB rows per store
            float4 *dst = reinterpret_cast<float4 *>(p.parts + part_slot * G3_SLOT_FLOATS) + (size_t)wave * 4096 + ln;
#pragma unroll
            for (int ab = 0; ab < 16; ++ab)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4)
                    dst[(ab * 4 + i4) * 64] = make_float4(acc_elem(acc[ab][4 * i4]), acc_elem(acc[ab][4 * i4 + 1]),
                                                          acc_elem(acc[ab][4 * i4 + 2]), acc_elem(acc[ab][4 * i4 + 3]));
        }
        __syncthreads();                                        // the epilogue's LDS areas are free again
    }
}

// adds the partials of one accumulator block of a leftover tile in workgroup order and stores it;
// grid (8 * l_max, 16), 256 threads laid out as in the third kernel
__global__ __launch_bounds__(256) void k_gemm3_fixup(G3Split sp, const float *__restrict__ parts, void *Y, uint32_t y_dt,
                                                     uint32_t ldy, uint32_t tokens, uint32_t out, uint32_t tile0)
{
    const uint32_t xcd = blockIdx.x / sp.l_max, l = blockIdx.x % sp.l_max, ab = blockIdx.y;
    if (l >= sp.left(xcd)) return;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 31, q = lane >> 5;
    uint32_t tile_m, tile_n;
    sp.tile_of(xcd, sp.rounds(xcd) * sp.gx + l, tile_m, tile_n);
    const uint32_t n_parts = sp.parts(xcd, l);
    float4 v[4];
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) v[i4] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (uint32_t part = 0; part < n_parts; ++part) {
        const float4 *src = reinterpret_cast<const float4 *>(parts + sp.slot(xcd, l, part) * G3_SLOT_FLOATS) +
                            (size_t)wave * 4096 + ab * 256 + lane;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const float4 w = src[i4 * 64];
            v[i4].x += w.x; v[i4].y += w.y; v[i4].z += w.z; v[i4].w += w.w;
        }
    }
    const uint32_t rb = ab >> 3, cb = ab & 7;
    const uint32_t o = (tile0 + tile_n) * GM3_NT + cb * 32 + n;    // tile0: first output tile of the slab the split covers
    if (o >= out) return;
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
        const float e[4] = {v[i4].x, v[i4].y, v[i4].z, v[i4].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t tk = tile_m * GM_MT + wave * 64 + rb * 32 + i4 * 8 + q * 4 + c;
            if (tk < tokens) store_out(Y, y_dt, (size_t)tk * ldy + o, e[c]);
        }
    }
}


// ========================================================================
// Launchers
// ========================================================================
static G3Split gemm3_split(const skl_layer *L, uint32_t tokens) { return skl_make_split(L->out, L->n_blocks, tokens, false); }

static uint64_t gemm_pack_bytes(const skl_layer *L, uint32_t tokens)
{
    const uint64_t m_tiles = (tokens + GM_MT - 1) / GM_MT;
    return m_tiles * L->n_gsteps * 8192ull;      // 8 row blocks of 64 lanes x 16 bytes per (token tile, step)
}

static uint64_t gemm_own_bytes(const skl_layer *L, uint32_t tokens)
{
    if (L->path != 1) return 0;
    if (skl_gemm_is_staged(L, tokens)) return skl_gemm_staged_bytes(L, tokens);
    const G3Split sp = gemm3_split(L, tokens);
    return gemm_pack_bytes(L, tokens) + 8ull * sp.l_max * sp.p_cap * G3_SLOT_FLOATS * sizeof(float);      // + partial tiles
}

uint64_t skl_gemm_workspace_bytes(const skl_layer *L, uint32_t tokens)
{
    const uint64_t own = gemm_own_bytes(L, tokens);
    return L->qbits ? round256(own) + skl_dequant_bytes(L) : own;
}

// activation re-ordering for the prefill kernels
skl_status_t skl_launch_pack(const skl_layer *L, const uint16_t *X, skl_dtype_t x_dt, uint32_t ldx, uint32_t tokens,
                             const uint32_t *chan, const skl_gemm_step *steps, uint32_t n_steps, uint4 *Xp, hipStream_t stream)
{
    skl_status_t st = allow_lds(k_pack_activations3, PK_LDS_BYTES);
    if (st != SKL_OK) return st;
    hipLaunchKernelGGL(k_pack_activations3, dim3((tokens + 31) / 32, (n_steps + PK_STEPS - 1) / PK_STEPS), dim3(SKL_WG), PK_LDS_BYTES,
                       stream, X, (uint32_t)x_dt, ldx, tokens, L->in, chan, steps, n_steps, Xp);
    return check_launch("activation packing");
}

skl_status_t skl_launch_gemm3_fixup(const G3Split &sp, const float *parts, void *Y, skl_dtype_t y_dt, uint32_t ldy,
                                    uint32_t tokens, uint32_t out, uint32_t tile0, hipStream_t stream)
{
    hipLaunchKernelGGL(k_gemm3_fixup, dim3(8 * sp.l_max, 16), dim3(256), 0, stream, sp, parts, Y, (uint32_t)y_dt, ldy, tokens, out, tile0);
    return check_launch("gemm fix-up");
}

skl_status_t skl_launch_gemm(const skl_layer *L, const void *X_, skl_dtype_t x_dt, uint32_t ldx, void *Y,
                             skl_dtype_t y_dt, uint32_t ldy, uint32_t tokens, void *ws, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const uint16_t *X = static_cast<const uint16_t *>(X_);
    const bool staged = L->path == 1 && skl_gemm_is_staged(L, tokens);      // the rebuild kernel reads the padded tables, the fused kernel the unpadded ones
    TableSrc src;
    skl_status_t st = skl_table_source(L, static_cast<char *>(ws) + round256(gemm_own_bytes(L, tokens)),
                                   L->path == 1 && staged, L->path == 1 && !staged, stream, &src);
    if (st != SKL_OK) return st;
    if (L->path == 1) {
        const RowArgs a = make_row_args(L, src);
        const uint32_t m_tiles = (tokens + GM_MT - 1) / GM_MT;
        if (m_tiles > 8191) {
            skl_set_error("more than 8191 token tiles in one call");
            return SKL_ERR_UNSUPPORTED;
        }
        if (staged) return skl_launch_gemm_staged(L, src, X, x_dt, ldx, Y, y_dt, ldy, tokens, ws, stream);
        {
            const skl_gemm_step *steps = reinterpret_cast<const skl_gemm_step *>(L->dev + L->off_gsteps);
            st = skl_launch_pack(L, X, x_dt, ldx, tokens, a.chan, steps, L->n_gsteps, static_cast<uint4 *>(ws), stream);
            if (st != SKL_OK) return st;
            Gemm2Args g;
            g.h = a.h; g.ptables = src.ptables; g.bmeta = a.bmeta;
            g.Xp = static_cast<const uint4 *>(ws); g.Y = Y;
            g.zeros = reinterpret_cast<const uint4 *>(L->dev);       // the reserved head of the layer buffer stays zero
            g.n_blocks = L->n_blocks; g.n_steps = L->n_gsteps; g.tokens = tokens; g.out = L->out; g.y_dt = (uint32_t)y_dt;
            g.ldy = ldy; g.tab_words = L->max_ptable_bytes / 16; g.n_col = (L->out + GM3_NT - 1) / GM3_NT; g.m_tiles = m_tiles;
            const G3Split sp = gemm3_split(L, tokens);
            g.parts = reinterpret_cast<float *>(static_cast<char *>(ws) + gemm_pack_bytes(L, tokens));
            g.T = sp.T; g.gx = sp.gx; g.l_max = sp.l_max; g.p_cap = sp.p_cap;
            g.rows_aligned = ((size_t)ldy * (y_dt == SKL_F32 ? 4 : 2)) % 16 == 0;
            const size_t lds = 2 * (size_t)L->max_ptable_bytes + 2 * (size_t)G3_SLOT_BYTES + 1024 + 32 * (size_t)L->n_blocks;
            const dim3 grid(8 * sp.gx);
            DISPATCH_D(L->d, {
                st = allow_lds(k_row_gemm3<D>, lds);
                if (st == SKL_OK) hipLaunchKernelGGL((k_row_gemm3<D>), grid, dim3(256), lds, stream, g);
            })
            if (st == SKL_OK) st = check_launch("gemm");
            if (st != SKL_OK || sp.l_max == 0) return st;
            return skl_launch_gemm3_fixup(sp, g.parts, Y, y_dt, ldy, tokens, L->out, 0, stream);
        }
    }
    return skl_tile_launch_gemm(L, src, X, x_dt, ldx, Y, y_dt, ldy, tokens, stream);
}

}  // namespace SKL_NS
