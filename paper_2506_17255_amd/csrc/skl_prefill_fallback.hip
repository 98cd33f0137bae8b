// Prefill GEMM over row sketches, first and second kernel (fallbacks of the
// third one in skl_prefill.hip).
#include "skl_prefill_common.h"

// ---- prefill GEMM ----------------------------------------------------------
// A workgroup of eight wavefronts owns 256 tokens x 128 outputs.  Wavefronts
// 0..3 compute: wavefront w owns all 256 tokens of its own 32 outputs, so every
// reconstructed weight fragment is built exactly once per workgroup and feeds
// eight 32x32x16 MFMAs straight from registers.  Wavefronts 4..7 only move
// data: all operand traffic is asynchronous global -> LDS copies, and a
// wavefront that issues them stalls while the copy queue is full, so the
// compute wavefronts never touch global memory inside the loop.
//
// The channel blocks are walked in units of up to UW 16-byte words (8*UW
// channels, listed by the host in skl_gemm_unit); a unit is UW/2 MFMA steps
// of 16 channels.  LDS holds two table buffers (the next block's table is
// requested when a block starts) and a ring of `ring` activation tiles,
// requested ring-1 units ahead.  One barrier per unit: the copy wavefronts
// arrive once their part of this unit's data has landed, the compute
// wavefronts once they are done with the previous unit.  A copy wavefront
// counts the copy instructions it has issued; they complete in order, so
// "this unit has landed" is a bound on the number still outstanding
// (s_waitcnt vmcnt(n)) and younger copies stay in flight across the barrier.
// Inside a unit the operands of step s+1 (gathers, query, decode, activation
// fragments) are fetched while the MFMAs of step s run.
//
// Activations are prepared by a pre-pass: binary16, negated, one contiguous
// tile of 256 rows x UW words per (token tile, unit), word c of row r at
// position c ^ ((r >> sh) & (UW-1)), sh = log2(16/UW): the 16 rows a
// quarter-wavefront reads then fall into 16 different LDS bank groups, and a
// tile is a flat copy.
template <int UW>
__device__ __forceinline__ uint32_t a_tile_word(uint32_t m, uint32_t c)
{
    constexpr int SH = UW == 8 ? 1 : UW == 4 ? 2 : 3;
    return m * UW + (c ^ ((m >> SH) & (UW - 1)));
}

// grid (unit, token tile); thread -> channel tid % (8*UW) of rows tid / (8*UW) + k * (256 / (8*UW))
template <int UW>
__global__ __launch_bounds__(SKL_WG) void k_pack_activations(const uint16_t *__restrict__ X, uint32_t x_dt, uint32_t ldx,
                                                              uint32_t tokens, const uint32_t *__restrict__ chan,
                                                              const skl_gemm_unit *__restrict__ units, uint32_t n_units,
                                                              uint16_t *__restrict__ Xp)
{
    constexpr int CPU = 8 * UW;                  // channels per unit
    constexpr int RSTEP = SKL_WG / CPU;
    const skl_gemm_unit un = units[blockIdx.x];
    const uint32_t c8 = threadIdx.x % CPU, c = c8 >> 3, e = c8 & 7;
    const uint32_t ch = c < un.w ? chan[un.chan0 + c8] : SKL_NO_CHANNEL;
    uint16_t *tile = Xp + ((size_t)blockIdx.y * n_units + blockIdx.x) * (GM_MT * UW * 8);
    for (uint32_t r = threadIdx.x / CPU; r < GM_MT; r += RSTEP) {
        const uint32_t t = blockIdx.y * GM_MT + r;
        uint16_t v = 0;
        if (ch != SKL_NO_CHANNEL && t < tokens) v = load_neg_half(X, x_dt, (size_t)t * ldx + ch);
        tile[a_tile_word<UW>(r, c) * 8 + e] = v;
    }
}

template <int D>
struct GemmOperands {
    uint4 a[8];          // activation fragments: rows mf*32 + n, 8 channels
    uint4 g[D];          // gathered keys of the d sketch rows (before the query)
    uint4 b;             // reconstructed weights (after query + decode)
};

// Issue the LDS reads of one step: word cw of the unit for this lane (even
// words for lanes 0..31, odd words for lanes 32..63).  Words past the unit's
// last one (w_last) are zero in the activation tile; the gather is clamped to
// a valid word so that the product is a clean zero.
template <int D, int UW>
__device__ __forceinline__ void gemm_issue(GemmOperands<D> &f, const uint4 *tab, const uint32_t (&off)[D], const uint4 *As,
                                           uint32_t c_base, uint32_t cw, uint32_t w_last)
{
    const uint32_t n = threadIdx.x & 31;
    const uint32_t cb = c_base + min(cw, w_last);
#pragma unroll
    for (int r = 0; r < D; ++r) f.g[r] = tab[off[r] + cb];
#pragma unroll
    for (int mf = 0; mf < 8; ++mf) f.a[mf] = As[a_tile_word<UW>(mf * 32 + n, cw)];
}

// query (Eq. 5) and decode of the gathered keys
template <int D>
__device__ __forceinline__ void gemm_finish(GemmOperands<D> &f)
{
    uint4 m = f.g[0];
#pragma unroll
    for (int r = 1; r < D; ++r) m = pk_max_u16x8(m, f.g[r]);
    f.b = keys_to_neg_half8(m);
}

// asynchronous flat copy by the four copy wavefronts (pw = 0..3); returns the
// number of copy instructions this wavefront issued
__device__ __forceinline__ uint32_t copy_counted(uint4 *dst, const uint4 *src, uint32_t n16, uint32_t pw)
{
    const uint32_t lane = threadIdx.x & 63;
    uint32_t issued = 0;
    for (uint32_t base = pw * 64; base < n16; base += 256) {
        if (base + lane < n16) lds_dma_16(src + base + lane, dst + base);
        ++issued;
    }
    return issued;
}

// wait until at most n of this wavefront's vector-memory operations are outstanding
__device__ __forceinline__ void wait_vmcnt_le(uint32_t n)
{
#define SKL_VMCNT_CASE(k) case k: __builtin_amdgcn_s_waitcnt(0x0F70 | ((k) & 15) | (((k) >> 4) << 14)); break;
    switch (n) {
        SKL_VMCNT_CASE(0) SKL_VMCNT_CASE(1) SKL_VMCNT_CASE(2) SKL_VMCNT_CASE(3) SKL_VMCNT_CASE(4) SKL_VMCNT_CASE(5)
        SKL_VMCNT_CASE(6) SKL_VMCNT_CASE(7) SKL_VMCNT_CASE(8) SKL_VMCNT_CASE(9) SKL_VMCNT_CASE(10) SKL_VMCNT_CASE(11)
        SKL_VMCNT_CASE(12) SKL_VMCNT_CASE(13) SKL_VMCNT_CASE(14) SKL_VMCNT_CASE(15) SKL_VMCNT_CASE(16) SKL_VMCNT_CASE(17)
        SKL_VMCNT_CASE(18) SKL_VMCNT_CASE(19) SKL_VMCNT_CASE(20) SKL_VMCNT_CASE(21) SKL_VMCNT_CASE(22) SKL_VMCNT_CASE(23)
        SKL_VMCNT_CASE(24) SKL_VMCNT_CASE(25) SKL_VMCNT_CASE(26) SKL_VMCNT_CASE(27) SKL_VMCNT_CASE(28) SKL_VMCNT_CASE(29)
        SKL_VMCNT_CASE(30) SKL_VMCNT_CASE(31) SKL_VMCNT_CASE(32) SKL_VMCNT_CASE(33) SKL_VMCNT_CASE(34) SKL_VMCNT_CASE(35)
        SKL_VMCNT_CASE(36) SKL_VMCNT_CASE(37) SKL_VMCNT_CASE(38) SKL_VMCNT_CASE(39) SKL_VMCNT_CASE(40)
    default: __builtin_amdgcn_s_waitcnt(0x0F70 | (40 & 15) | ((40 >> 4) << 14)); break;   // fewer outstanding than allowed is always safe
    }
#undef SKL_VMCNT_CASE
}

// epilogue: acc[mf][i] is the output of token t0 + mf*32 + (i/4)*8 + q*4 + i%4
// and output channel o; one rounding to the output type
template <int DT>
__device__ __forceinline__ void gemm_store(const float16v (&acc)[8], void *Y, uint32_t ldy, uint32_t t0, uint32_t tokens,
                                           uint32_t o, uint32_t out, uint32_t q)
{
    if (o >= out) return;
#pragma unroll
    for (int mf = 0; mf < 8; ++mf) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t t = t0 + mf * 32 + (i >> 2) * 8 + q * 4 + (i & 3);
            if (t < tokens) {
                const size_t idx = (size_t)t * ldy + o;
                const float v = acc[mf][i];
                if (DT == SKL_F32) static_cast<float *>(Y)[idx] = v;
                else if (DT == SKL_F16) static_cast<uint16_t *>(Y)[idx] = float_to_half_bits(v);
                else static_cast<uint16_t *>(Y)[idx] = float_to_bf16_bits(v);
            }
        }
    }
}

struct GemmArgs {
    HashArgs h;
    const uint4 *tables;
    const skl_gemm_unit *units;
    const uint4 *Xp;
    void *Y;
    uint32_t n_units, tokens, out, y_dt, ldy, table_words, two_tabs, ring, n_col, m_tiles;
};

// the copy wavefronts' side of the unit loop
template <int D, int UW>
__device__ __forceinline__ void gemm_copy_loop(const GemmArgs &p, uint4 *tab_buf, uint4 *a_buf, const uint4 *Xt, uint32_t pw)
{
    constexpr uint32_t TILE = GM_MT * UW;
    const uint32_t la = p.ring - 1;
    // instructions issued so far (mod 256), and the count right after the last instruction
    // of each activation tile (one byte per ring slot) and of the most recent table
    uint32_t issued = 0, mark_a = 0, mark_t = 0;
    auto set_mark_a = [&](uint32_t slot) { mark_a = (mark_a & ~(0xFFu << (8 * slot))) | ((issued & 0xFFu) << (8 * slot)); };
    {
        const skl_gemm_unit u0 = p.units[0];
        issued += copy_counted(tab_buf, p.tables + u0.table_off16, D * u0.K * u0.rs, pw);
        mark_t = issued;
        for (uint32_t v = 0; v < la && v < p.n_units; ++v) {
            issued += copy_counted(a_buf + v * TILE, Xt + (size_t)v * TILE, TILE, pw);
            set_mark_a(v);
        }
    }
    uint32_t tpar = 0;
    skl_gemm_unit un = p.units[0], un_next = un;
    for (uint32_t u = 0; u < p.n_units; ++u, un = un_next) {
        un_next = p.units[min(u + 1, p.n_units - 1)];      // requested a whole unit before it is needed
        const uint32_t slot = u % p.ring;
        if (un.first && u != 0) tpar ^= 1;
        {
            uint32_t need = (mark_a >> (8 * slot)) & 0xFFu;
            if (un.first && p.two_tabs && ((issued - mark_t) & 0xFFu) < ((issued - need) & 0xFFu)) need = mark_t;
            wait_vmcnt_le((issued - need) & 0xFFu);
        }
        __syncthreads();                                   // unit u is in LDS; the buffers of unit u-1 are free
        if (un.first && !p.two_tabs && u != 0) {           // single table buffer: fetch this block's table now
            issued += copy_counted(tab_buf, p.tables + un.table_off16, D * un.K * un.rs, pw);
            wait_vmcnt_le(0);
            __syncthreads();
        }
        if (un.first && p.two_tabs && un.next_table_words) {
            issued += copy_counted(tab_buf + (tpar ^ 1) * p.table_words, p.tables + un.next_table_off16, un.next_table_words, pw);
            mark_t = issued;
        }
        if (u + la < p.n_units) {
            const uint32_t s2 = (u + la) % p.ring;
            issued += copy_counted(a_buf + s2 * TILE, Xt + (size_t)(u + la) * TILE, TILE, pw);
            set_mark_a(s2);
        }
    }
}

template <int D, int UW>
__global__ __launch_bounds__(GM_THREADS) void k_row_gemm(GemmArgs p)
{
    // Workgroup id -> (token tile, output tile).  Consecutive ids go to different XCDs; all
    // workgroups of one token tile get ids that are equal modulo 8, so a token tile's
    // activations are fetched into one L2 only (and walked in step by its workgroups).
    const uint32_t xcd = blockIdx.x & 7, slot0 = blockIdx.x >> 3;
    const uint32_t tile_m = (slot0 / p.n_col) * 8 + xcd, tile_n = slot0 % p.n_col;
    if (tile_m >= p.m_tiles) return;
    constexpr uint32_t TILE = GM_MT * UW;                  // words per activation tile
    uint4 *tab_buf = smem;
    uint4 *a_buf = smem + (p.two_tabs ? 2 : 1) * p.table_words;
    const uint32_t lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint4 *Xt = p.Xp + (size_t)tile_m * p.n_units * TILE;      // this token tile's activation tiles
    if (wave >= 4) {
        gemm_copy_loop<D, UW>(p, tab_buf, a_buf, Xt, wave - 4);
        return;
    }

    const uint32_t n = lane & 31, q = lane >> 5;
    const uint32_t t0 = tile_m * GM_MT;
    const uint32_t o = tile_n * GM_NT + wave * 32 + n;
    float16v acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = (float16v){0.f};
    uint32_t off[D];
    uint32_t K_prev = 0, rs_prev = 0, tpar = 0;
    skl_gemm_unit un = p.units[0], un_next = un;
    for (uint32_t u = 0; u < p.n_units; ++u, un = un_next) {
        un_next = p.units[min(u + 1, p.n_units - 1)];      // requested a whole unit before it is needed
        if (un.first && u != 0) tpar ^= 1;
        __syncthreads();                                   // unit u is in LDS (see gemm_copy_loop)
        if (un.first && !p.two_tabs && u != 0) __syncthreads();
        if (un.K != K_prev || un.rs != rs_prev) {
            row_offsets<D>(p.h, min(o, p.out - 1), un.K, un.rs, off);
            K_prev = un.K;
            rs_prev = un.rs;
        }
        const uint4 *tab = tab_buf + (p.two_tabs ? tpar * p.table_words : 0);
        const uint4 *As = a_buf + (u % p.ring) * TILE;
        // max(UW/2, 1) steps, straight-line.  A unit with fewer than UW words runs the same
        // steps: its missing words are zero in the activation tile and the gathers are clamped
        // to its last word.  Step s+1's LDS reads are issued before step s's MFMAs and may not
        // sink below them; its query/decode VALU work is spread between the later MFMAs.
        constexpr int NS = UW >= 2 ? UW / 2 : 1;
        constexpr int NV = 4 * (D - 1) + 12;               // VALU instructions of gemm_finish
        const uint32_t w_last = un.w - 1;
        GemmOperands<D> f[2];
        gemm_issue<D, UW>(f[0], tab, off, As, un.c_base, q, w_last);
        gemm_finish<D>(f[0]);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            if (s + 1 < NS) {
                gemm_issue<D, UW>(f[(s + 1) & 1], tab, off, As, un.c_base, 2 * (s + 1) + q, w_last);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int mf = 0; mf < 8; ++mf)
                acc[mf] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8v, f[s & 1].a[mf]),
                                                                  __builtin_bit_cast(half8v, f[s & 1].b), acc[mf], 0, 0, 0);
            if (s + 1 < NS) {
                gemm_finish<D>(f[(s + 1) & 1]);
                __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);      // three MFMAs cover the gather latency
#pragma unroll
                for (int i = 0; i < 5; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x002, (NV + 4) / 5, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    if (p.y_dt == SKL_F32) gemm_store<SKL_F32>(acc, p.Y, p.ldy, t0, p.tokens, o, p.out, q);
    else if (p.y_dt == SKL_F16) gemm_store<SKL_F16>(acc, p.Y, p.ldy, t0, p.tokens, o, p.out, q);
    else gemm_store<SKL_BF16>(acc, p.Y, p.ldy, t0, p.tokens, o, p.out, q);
}

// ---- prefill, second kernel ------------------------------------------------
// Used when two unpadded block tables fit in LDS next to two operand slots.
// A workgroup of 8 wavefronts owns 256 tokens x 128 outputs.
//   * Wavefronts 4..7 (producers) rebuild the weights: producer p owns the 32
//     outputs of column block p; per channel block it gathers whole state rows
//     from the unpadded table (lanes = (output, word) pairs, as in the batch-1
//     decode kernel), takes the query maximum (Eq. 5), decodes, and writes the
//     16-byte MFMA operand words into an LDS slot -- every weight of the tile
//     is rebuilt once per workgroup.  They also issue the asynchronous
//     global -> LDS copy of the table two blocks ahead.
//   * Wavefronts 0..3 (consumers) own 64 tokens each: per 16-channel step they
//     read the four operand words of the step from the slot, take their two
//     activation words straight from global memory (re-ordered by the pre-pass
//     so that a wavefront's load is one contiguous KiB, requested two blocks
//     ahead into a register ring) and issue eight 32x32x16 MFMAs.
// One workgroup barrier per channel block hands the slots and tables over.
//
// epilogue of the second kernel: acc[rb*4+cb][i] is token t0 + rb*32 + (i/4)*8 + q*4 + i%4,
// output o0 + cb*32; one rounding to the output type
template <int DT>
__device__ __forceinline__ void gemm2_store(const float16v (&acc)[8], void *Y, uint32_t ldy, uint32_t t0, uint32_t tokens,
                                            uint32_t o0, uint32_t out, uint32_t q)
{
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        const uint32_t o = o0 + cb * 32;
        if (o >= out) continue;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t t = t0 + rb * 32 + (i >> 2) * 8 + q * 4 + (i & 3);
                if (t < tokens) {
                    const size_t idx = (size_t)t * ldy + o;
                    const float v = acc[rb * 4 + cb][i];
                    if (DT == SKL_F32) static_cast<float *>(Y)[idx] = v;
                    else if (DT == SKL_F16) static_cast<uint16_t *>(Y)[idx] = float_to_half_bits(v);
                    else static_cast<uint16_t *>(Y)[idx] = float_to_bf16_bits(v);
                }
            }
        }
    }
}

// NS: 16-channel steps per block of the layer's widest class (4, 2 or 1)
template <int D, int NS>
__global__ __launch_bounds__(GM_THREADS) void k_row_gemm2(Gemm2Args p)
{
    const uint32_t xcd = blockIdx.x & 7, slot0 = blockIdx.x >> 3;
    const uint32_t tile_m = (slot0 / p.n_col) * 8 + xcd, tile_n = slot0 % p.n_col;
    if (tile_m >= p.m_tiles) return;
    const uint32_t lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void *)smem;
    const uint32_t tab_bytes = p.tab_words * 16;
    const uint32_t slot_base = lds0 + 2 * tab_bytes;                       // two operand slots
    const uint4 *sm_meta = smem + (2 * tab_bytes + 2 * SKL_G2_SLOT_BYTES) / 16;   // block metadata, two words per block
    {
        uint4 *meta_w = smem + (2 * tab_bytes + 2 * SKL_G2_SLOT_BYTES) / 16;
        const uint4 *gm = reinterpret_cast<const uint4 *>(p.bmeta);
        for (uint32_t i = threadIdx.x; i < 2 * p.n_blocks; i += GM_THREADS) meta_w[i] = gm[i];
        uint4 *slots = smem + 2 * tab_bytes / 16;                          // stale bits must not reach the MFMAs as NaN
        for (uint32_t i = threadIdx.x; i < 2 * SKL_G2_SLOT_BYTES / 16; i += GM_THREADS) slots[i] = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();

    if (wave >= 4) {
        // ------------------------------------------------------------ producers
        const uint32_t pw = wave - 4;                      // column block of this wavefront
        const uint32_t o_first = tile_n * GM_NT + pw * 32;
        auto table_copy = [&](uint32_t b) {               // asynchronous copy of block b's table into buffer b % 2
            const uint4 m0 = sm_meta[2 * b], m1 = sm_meta[2 * b + 1];
            const uint32_t n_chunks = (D * m0.y * m0.w + 63) >> 6;
            uint4 *dst = smem + (b & 1) * p.tab_words;
            const uint4 *src = p.ptables + m1.y;
            for (uint32_t ch = pw; ch < n_chunks; ch += 4) lds_dma_16(src + ch * 64 + lane, dst + ch * 64);
        };
        uint32_t off[4][D];
        uint32_t K_prev = 0, nb_prev = 0;
        auto build = [&](uint32_t b) {                     // operand words of block b into slot b % 2
            const uint4 m0 = sm_meta[2 * b];               // {table_off16, K, rs, nb}
            const uint32_t K = m0.y, nb = m0.w;
            const bool fresh = K != K_prev || nb != nb_prev;
            K_prev = K; nb_prev = nb;
            const uint32_t tab_addr = lds0 + (b & 1) * tab_bytes, slot_addr = slot_base + (b & 1) * SKL_G2_SLOT_BYTES;
            switch (nb) {
            case 8:
                if constexpr (D <= 6) {
                    if (fresh) g2_offsets<D, 8>(p.h, o_first, p.out, K, lane, off);
                    g2_build<D, 8>(off, tab_addr, slot_addr, pw, lane);
                    break;
                }
            case 4:
                if (fresh) g2_offsets<D, 4>(p.h, o_first, p.out, K, lane, off);
                g2_build<D, 4>(off, tab_addr, slot_addr, pw, lane);
                break;
            case 2:
                if (fresh) g2_offsets<D, 2>(p.h, o_first, p.out, K, lane, off);
                g2_build<D, 2>(off, tab_addr, slot_addr, pw, lane);
                break;
            default:
                if (fresh) g2_offsets<D, 1>(p.h, o_first, p.out, K, lane, off);
                g2_build<D, 1>(off, tab_addr, slot_addr, pw, lane);
                break;
            }
        };
        table_copy(0);
        wait_async_copies();
        __syncthreads();                                   // table 0 is in LDS
        if (p.n_blocks > 1) table_copy(1);
        build(0);
        wait_async_copies();
        __syncthreads();                                   // operands of block 0 and table 1 are in LDS
        for (uint32_t k = 0; k < p.n_blocks; ++k) {
            if (k + 2 < p.n_blocks) table_copy(k + 2);     // into the buffer of table k, not read any more
            if (k + 1 < p.n_blocks) build(k + 1);
            wait_async_copies();
            __syncthreads();                               // block k consumed; operands k+1 and table k+2 in place
        }
        return;
    }

    // ---------------------------------------------------------------- consumers
    const uint32_t n = lane & 31, q = lane >> 5;
    const uint32_t t0 = tile_m * GM_MT + wave * 64;        // first token of this wavefront
    float16v acc[8];                                       // [row block][column block]
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = (float16v){0.f};
    // activation words: Xp[((tile_m * n_steps + step) * 8 + row block) * 64 + lane]
    const uint4 *xa = p.Xp + ((size_t)tile_m * p.n_steps * 8 + wave * 2) * 64 + lane;
    uint4 a[2][NS][2];                                     // [block parity][step][row block]
    // Request the activation words of block b.  Always 2*NS loads, so that the
    // number of loads in flight is the same on every path and the waits can be
    // counted: steps a block does not have (fewer words per state row than the
    // widest class of the layer) read a page of zeros and contribute nothing;
    // past the last block the last block is read again and never used.
    auto load_a = [&](uint32_t b, auto par) {
        constexpr int P = decltype(par)::value;
        b = min(b, p.n_blocks - 1);
        const uint4 m0 = sm_meta[2 * b], m1 = sm_meta[2 * b + 1];
        const uint32_t ns = (m0.w + 1) >> 1, s0 = m1.z;    // steps of the block, first step
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const uint4 *src = (uint32_t)s < ns ? xa + (size_t)(s0 + s) * 512 : p.zeros + lane;
            const uint4 *src1 = (uint32_t)s < ns ? src + 64 : src;
            a[P][s][0] = src[0];
            a[P][s][1] = src1[0];
        }
    };
    const uint32_t b_lane = slot_base + (q * G2_ROW + n) * 16;
    // NS steps of one block, straight-line: the operand words of step s+1 are
    // read from LDS before the MFMAs of step s are issued
    auto block_mma = [&](auto par) {
        constexpr int P = decltype(par)::value;
        const uint32_t baddr = b_lane + P * SKL_G2_SLOT_BYTES;
        uint4 bw[2][4];
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) bw[0][cb] = lds_word_at(baddr + cb * G2_CB_WORDS * 16);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            if (s + 1 < NS) {
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
                    bw[(s + 1) & 1][cb] = lds_word_at(baddr + (cb * G2_CB_WORDS + 2 * (s + 1) * G2_ROW) * 16);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
                    acc[rb * 4 + cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                        __builtin_bit_cast(half8v, a[P][s][rb]), __builtin_bit_cast(half8v, bw[s & 1][cb]), acc[rb * 4 + cb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    const std::integral_constant<int, 0> even;
    const std::integral_constant<int, 1> odd;
    load_a(0, even);
    load_a(1, odd);
    __syncthreads();                                       // (table 0)
    __syncthreads();                                       // operands of block 0
    // blocks in pairs (both register sets in fixed roles, the same number of
    // loads in flight on every path round the loop), an odd last block after it
    uint32_t k = 0;
    for (; k + 1 < p.n_blocks; k += 2) {
        block_mma(even);
        load_a(k + 2, even);
        __syncthreads();
        block_mma(odd);
        load_a(k + 3, odd);
        __syncthreads();
    }
    if (k < p.n_blocks) {
        block_mma(even);
        __syncthreads();
    }
    if (p.y_dt == SKL_F32) gemm2_store<SKL_F32>(acc, p.Y, p.ldy, t0, p.tokens, tile_n * GM_NT + n, p.out, q);
    else if (p.y_dt == SKL_F16) gemm2_store<SKL_F16>(acc, p.Y, p.ldy, t0, p.tokens, tile_n * GM_NT + n, p.out, q);
    else gemm2_store<SKL_BF16>(acc, p.Y, p.ldy, t0, p.tokens, tile_n * GM_NT + n, p.out, q);
}


skl_status_t skl_launch_gemm_fallback(const skl_layer *L, const TableSrc &src, const uint16_t *X, skl_dtype_t x_dt, uint32_t ldx,
                                      void *Y, skl_dtype_t y_dt, uint32_t ldy, uint32_t tokens, void *ws, hipStream_t stream)
{
    skl_status_t st = SKL_OK;
    uint16_t *Xp = static_cast<uint16_t *>(ws);
    const RowArgs a = make_row_args(L, src);
    const skl_gemm_unit *units = reinterpret_cast<const skl_gemm_unit *>(L->dev + L->off_gunits);
    const uint32_t m_tiles = (tokens + GM_MT - 1) / GM_MT;
        if (L->gemm_v2) {
            const skl_gemm_step *steps = reinterpret_cast<const skl_gemm_step *>(L->dev + L->off_gsteps);
            st = skl_launch_pack(L, X, x_dt, ldx, tokens, a.chan, steps, static_cast<uint4 *>(ws), stream);
            if (st != SKL_OK) return st;
            Gemm2Args g;
            g.h = a.h; g.ptables = src.ptables; g.bmeta = a.bmeta;
            g.Xp = static_cast<const uint4 *>(ws); g.Y = Y;
            g.n_blocks = L->n_blocks; g.n_steps = L->n_gsteps; g.tokens = tokens; g.out = L->out; g.y_dt = (uint32_t)y_dt;
            g.ldy = ldy; g.tab_words = L->max_ptable_bytes / 16; g.n_col = (L->out + GM_NT - 1) / GM_NT; g.m_tiles = m_tiles;
            const size_t lds = 2 * (size_t)L->max_ptable_bytes + 2 * (size_t)SKL_G2_SLOT_BYTES + 32 * (size_t)L->n_blocks;
            const dim3 grid(8 * ((m_tiles + 7) / 8) * g.n_col);
            g.zeros = reinterpret_cast<const uint4 *>(L->dev);       // the reserved head of the layer buffer stays zero
#define LAUNCH_GEMM2(NS_)                                                                                            \
    DISPATCH_D(L->d, {                                                                                               \
        st = allow_lds(k_row_gemm2<D, NS_>, lds);                                                                    \
        if (st == SKL_OK) hipLaunchKernelGGL((k_row_gemm2<D, NS_>), grid, dim3(GM_THREADS), lds, stream, g);         \
    })
            if (L->gemm_ns == 4) LAUNCH_GEMM2(4)
            else if (L->gemm_ns == 2) LAUNCH_GEMM2(2)
            else LAUNCH_GEMM2(1)
#undef LAUNCH_GEMM2
            return st == SKL_OK ? check_launch("gemm") : st;
        }
#define LAUNCH_PACK(UW_)                                                                                             \
    hipLaunchKernelGGL(k_pack_activations<UW_>, dim3(L->n_gunits, m_tiles), dim3(SKL_WG), 0, stream, X, (uint32_t)x_dt,  \
                       ldx, tokens, a.chan, units, L->n_gunits, Xp)
        if (L->gemm_uw == 8) LAUNCH_PACK(8);
        else if (L->gemm_uw == 4) LAUNCH_PACK(4);
        else LAUNCH_PACK(2);
#undef LAUNCH_PACK
        st = check_launch("activation packing");
        if (st != SKL_OK) return st;
        const uint32_t tw = L->max_table_bytes / 16;
        const size_t lds = (size_t)(L->gemm_two_tabs ? 2 : 1) * tw * 16 + (size_t)L->gemm_ring * GM_MT * L->gemm_uw * 16;
        GemmArgs g;
        g.h = a.h; g.tables = a.tables; g.units = units; g.Xp = reinterpret_cast<const uint4 *>(Xp); g.Y = Y;
        g.n_units = L->n_gunits; g.tokens = tokens; g.out = L->out; g.y_dt = (uint32_t)y_dt; g.ldy = ldy;
        g.table_words = tw; g.two_tabs = L->gemm_two_tabs; g.ring = L->gemm_ring;
        g.n_col = (L->out + GM_NT - 1) / GM_NT; g.m_tiles = m_tiles;
        const dim3 grid(8 * ((m_tiles + 7) / 8) * g.n_col);
#define LAUNCH_GEMM(UW_)                                                                                            \
    DISPATCH_D(L->d, {                                                                                              \
        st = allow_lds(k_row_gemm<D, UW_>, lds);                                                                    \
        if (st == SKL_OK) hipLaunchKernelGGL((k_row_gemm<D, UW_>), grid, dim3(GM_THREADS), lds, stream, g);         \
    })
        if (L->gemm_uw == 8) LAUNCH_GEMM(8)
        else if (L->gemm_uw == 4) LAUNCH_GEMM(4)
        else LAUNCH_GEMM(2)
#undef LAUNCH_GEMM
    return st == SKL_OK ? check_launch("gemm") : st;
}
