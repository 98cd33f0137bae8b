// Staged prefill over row sketches (Sec. 3 inference flow: decompress the layer, compute, release -- here at
// the granularity of one call, through a cache-sized part of the workspace; W_hat of Sec. 3.1 Eq. 5, the
// product Y = X W_hat of Sec. 2.1).
//
// For layers whose block tables are too large for the fused kernel (wide sketches put few input channels
// behind one table: a 256-output workgroup would have to stream tables that cover all outputs, several
// times the bytes of the dense weights of its tile), every weight is rebuilt exactly once per call:
//   1. k_rebuild_operands: one workgroup per (channel block, range of output tiles) stages the block's table
//      in LDS once, runs select / gather / query / decode for all its outputs and writes the weights as
//      16-byte matrix-core operand words, already in the order the product kernel's LDS slot has;
//   2. k_staged_gemm: 256 tokens x 256 outputs per workgroup, one wavefront per SIMD with the 65536
//      float32 accumulators in its registers (the shape of the fused kernel); per 64 channels a wavefront
//      loads its own activation words straight into registers, copies a quarter of the workgroup's weight
//      words into an LDS slot, and issues 64 MFMAs on words read back from the slot filled one block earlier.
// The work split, partial tiles and fix-up pass are those of the fused kernel, dealt by output-tile column.
#include "skl_prefill_common.h"

namespace SKL_NS {


#define SG_SLOT_WORDS 2048u             // 64 channels x 256 outputs: [column block 8][row 8 = (step, half)][32 outputs] words
#define SG_SLOT_BYTES (SG_SLOT_WORDS * 16u)
static_assert(4 * G3_EPI_BYTES >= 2 * SG_SLOT_BYTES, "the epilogue areas are the larger use of LDS");
#define SG_LDS_BYTES (4 * G3_EPI_BYTES)

struct RebuildArgs {
    HashArgs h;
    const skl_block_meta *bmeta;
    const uint4 *tables;                // padded block tables, [r][k][rs] words
    uint4 *Wp;                          // [output tile of the slab][64-channel block][SG_SLOT_WORDS]
    uint32_t out, n_blocks, KB, n_words;
    uint32_t tile0, n_col, n_oseg;      // the slab: first output tile, output tiles, output segments
};

template <int D, int RS>
__device__ __forceinline__ void rebuild_body(const RebuildArgs &p, uint32_t blk, uint32_t seg, const skl_block_meta &bm, const uint4 *tab)
{
    constexpr int NB = RS == 1 ? 1 : RS - 1;
    const uint32_t lo = (uint32_t)(((uint64_t)seg * p.n_col) / p.n_oseg);
    const uint32_t hi = (uint32_t)(((uint64_t)(seg + 1) * p.n_col) / p.n_oseg);
    const uint32_t w0 = bm.chan_off >> 3;                       // first operand word of the block along the channel list
    const bool pad = blk + 1 == p.n_blocks;                     // the last block also fills the words up to the end of the last 64-channel block
    for (uint32_t tile = lo; tile < hi; ++tile) {
        // outputs past the end of the layer are rebuilt like the last one: their products are never stored
        const uint32_t o = min((p.tile0 + tile) * GM3_NT + threadIdx.x, p.out - 1);
        uint4 *dst = p.Wp + (size_t)tile * p.KB * SG_SLOT_WORDS + (threadIdx.x >> 5) * 256 + (threadIdx.x & 31);
        uint32_t off[D];
        row_offsets<D>(p.h, o, bm.K, RS, off);
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            const uint32_t w = w0 + c;
            dst[(size_t)(w >> 3) * SG_SLOT_WORDS + (w & 7) * 32] = keys_to_neg_half8(row_query8<D>(tab, off, c));
        }
        if (pad)
            for (uint32_t w = p.n_words; w < 8 * p.KB; ++w) dst[(size_t)(w >> 3) * SG_SLOT_WORDS + (w & 7) * 32] = make_uint4(0, 0, 0, 0);
    }
}

// Workgroup `idx` of n_blocks * n_oseg: channel block idx % n_blocks, output segment idx / n_blocks.
// LDS: the block's padded table.
template <int D>
__device__ __forceinline__ void rebuild_block(const RebuildArgs &p, uint32_t idx)
{
    const uint32_t blk = idx % p.n_blocks, seg = idx / p.n_blocks;
    if (!skl_in_range(blk, p.n_blocks, SKL_DBG_BLOCK) || !skl_in_range(seg, p.n_oseg, SKL_DBG_OUTPUT)) return;
    const skl_block_meta bm = p.bmeta[blk];
    // global -> LDS without passing through registers: all of a wavefront's chunks are in flight at once
    copy_words_to_lds_async(smem, p.tables + bm.table_off16, D * bm.K * bm.rs, SKL_WG / 64);
    wait_async_copies();
    __syncthreads();
    switch (bm.rs) {
    case 9: rebuild_body<D, 9>(p, blk, seg, bm, smem); break;
    case 5: rebuild_body<D, 5>(p, blk, seg, bm, smem); break;
    case 3: rebuild_body<D, 3>(p, blk, seg, bm, smem); break;
    default: rebuild_body<D, 1>(p, blk, seg, bm, smem); break;
    }
}

// grid (channel blocks x output segments)
template <int D>
__global__ __launch_bounds__(SKL_WG) void k_rebuild_operands(RebuildArgs r)
{
    rebuild_block<D>(r, blockIdx.x);
}

struct StagedArgs {
    const uint4 *Xp;                    // activation words: [token tile][step][8 row blocks][64 lanes]
    const uint4 *Wp;                    // weight words: [output tile][64-channel block][SG_SLOT_WORDS]
    void *Y;
    float *parts;
    uint32_t KB, tokens, out, y_dt, ldy, rows_aligned;
    uint32_t tile0;                     // first output tile of the slab (Wp and the split are slab-relative)
    G3Split sp;
};

// RB: 32-token row blocks per wavefront: 2 (256 x 256 tiles) or 1 (128 x 256 tiles, the single-round mode of the split)
template <int RB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_staged_gemm(StagedArgs p)
{
    const uint32_t xcd = blockIdx.x & 7, wg = blockIdx.x >> 3;
    const G3Split sp = p.sp;
    uint32_t round = 0, u_next = sp.share_begin(xcd, wg);
    if (sp.rounds(xcd) == 0 && u_next >= sp.share_begin(xcd, wg + 1)) return;
    const uint32_t lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void *)smem;
    const uint32_t n = lane & 31, q = lane >> 5;
    const uint32_t b_lane = lds0 + (q * 32 + n) * 16;           // this lane's operand word of (column block 0, step 0)
    // where this lane's eight copied words go inside a slot (+ 64 i); native vectors, so that the words in flight stay in registers
    u32x4v *const copy_w = reinterpret_cast<u32x4v *>(smem) + wave * 512 + lane;
    const uint32_t last_kb = p.KB - 1;
    float16v acc[8 * RB];                                       // [row block][column block]
    for (;;) {
        G3Split::Seg sg;
        if (!sp.next(xcd, wg, round, u_next, sg)) break;
        const uint32_t k0 = sg.k0, k1 = sg.k1;
        const bool whole = sg.whole != 0;
        const size_t part_slot = sg.part_slot;
        uint32_t tile_m, tile_n;
        sp.tile_of(xcd, sg.k, tile_m, tile_n);
        const uint32_t t0 = tile_m * (128 * RB) + wave * (32 * RB);
        const uint32_t o_tile = (p.tile0 + tile_n) * GM3_NT;        // first output of the tile in the layer
        // activation words of the wavefront's first row block (step st: + 512 st; second row block: + 64); the
        // words are laid out by 256-token tiles of eight row blocks, a half-height tile is four of them
        const uint4 *xa = RB == 2 ? p.Xp + ((size_t)tile_m * p.KB * 32 + wave * 2) * 64 + lane
                                  : p.Xp + ((size_t)(tile_m >> 1) * p.KB * 32 + (tile_m & 1) * 4 + wave) * 64 + lane;
        const u32x4v *wb = reinterpret_cast<const u32x4v *>(p.Wp) + (size_t)tile_n * p.KB * SG_SLOT_WORDS + wave * 512 + lane;    // block kb: + 2048 kb; word i: + 64 i
#pragma unroll
        for (int i = 0; i < 8 * RB; ++i) acc[i] = (float16v){0.f};
        uint4 a[4][RB];
        u32x4v tb[8];
        {
            const u32x4v *w0 = wb + (size_t)k0 * SG_SLOT_WORDS;
#pragma unroll
            for (int i = 0; i < 8; ++i) tb[i] = w0[i * 64];
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int r = 0; r < RB; ++r) a[s][r] = xa[(size_t)(k0 * 4 + s) * 512 + r * 64];
            u32x4v *dst = copy_w + (k0 & 1) * SG_SLOT_WORDS;
#pragma unroll
            for (int i = 0; i < 8; ++i) dst[i * 64] = tb[i];
            const u32x4v *w1 = wb + (size_t)min(k0 + 1, last_kb) * SG_SLOT_WORDS;
#pragma unroll
            for (int i = 0; i < 8; ++i) tb[i] = w1[i * 64];
        }
        __syncthreads();                                        // weight words of block k0 are in their slot
        for (uint32_t kb = k0; kb < k1; ++kb) {
            const uint32_t baddr = b_lane + (kb & 1) * SG_SLOT_BYTES;
            u32x4v *const nxt = copy_w + ((kb & 1) ^ 1) * SG_SLOT_WORDS;
            const uint4 *xn = xa + (size_t)min(kb + 1, last_kb) * 2048;                         // next block's activation words (the last block again past the end)
            const u32x4v *w2 = wb + (size_t)min(kb + 2, last_kb) * SG_SLOT_WORDS;
            uint4 bw[8];
#pragma unroll
            for (int cb = 0; cb < 8; ++cb) bw[cb] = lds_word_at(baddr + cb * 4096);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int cb = 0; cb < 8; ++cb) {
#pragma unroll
                    for (int r = 0; r < RB; ++r)
                        acc[8 * r + cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                            __builtin_bit_cast(half8v, a[s][r]), __builtin_bit_cast(half8v, bw[cb]), acc[8 * r + cb], 0, 0, 0);
                    if (s < 3) bw[cb] = lds_word_at(baddr + cb * 4096 + (s + 1) * 1024);
                    if (cb == 3) {                  // two of the next block's weight words into the other slot, their successors requested
                        nxt[(2 * s) * 64] = tb[2 * s];
                        nxt[(2 * s + 1) * 64] = tb[2 * s + 1];
                    }
                    if (cb == 5) {
                        tb[2 * s] = w2[(2 * s) * 64];
                        tb[2 * s + 1] = w2[(2 * s + 1) * 64];
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                // next block's activation words into the registers just used
#pragma unroll
                for (int r = 0; r < RB; ++r) a[s][r] = xn[s * 512 + r * 64];
            }
            __syncthreads();                                    // everyone is done with this block's slot; the other one is complete
        }
        // the addresses of the epilogue are formed from a lane number the compiler cannot trace back, so that
        // they are not kept in registers (or scratch memory) across the block loop
        uint32_t ln = lane;
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" : "+v"(ln));       // also: the last MFMA has left the pipeline
        if (whole && p.rows_aligned) {
            const uint32_t lw = lds0 + wave * G3_EPI_BYTES;
            if (p.y_dt == SKL_F32) gemm3_store_rows<SKL_F32, RB>(acc, lw, p.Y, p.ldy, t0, p.tokens, o_tile, p.out, ln);
            else if (p.y_dt == SKL_F16) gemm3_store_rows<SKL_F16, RB>(acc, lw, p.Y, p.ldy, t0, p.tokens, o_tile, p.out, ln);
            else gemm3_store_rows<SKL_BF16, RB>(acc, lw, p.Y, p.ldy, t0, p.tokens, o_tile, p.out, ln);
        } else if (whole) {
            const uint32_t ne = ln & 31, qe = ln >> 5;
            if (p.y_dt == SKL_F32) gemm3_store<SKL_F32, RB>(acc, p.Y, p.ldy, t0, p.tokens, o_tile + ne, p.out, qe);
            else if (p.y_dt == SKL_F16) gemm3_store<SKL_F16, RB>(acc, p.Y, p.ldy, t0, p.tokens, o_tile + ne, p.out, qe);
            else gemm3_store<SKL_BF16, RB>(acc, p.Y, p.ldy, t0, p.tokens, o_tile + ne, p.out, qe);
        } else if constexpr (RB == 2) {         // (the single-round mode of the half-height tiles has no partial tiles)
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

// ========================================================================
// Launcher
// ========================================================================
// Output-tile columns per slab.  The weight words of a slab (KB x 32 KiB per column) are rebuilt, multiplied
// and released before the next slab is touched, which bounds the workspace for very large layers; up to
// 1 GiB of weight words the layer is one slab (measured on the 8192 x 28672 layer: four slabs of 134 MB
// cost 8 % -- every slab stages all tables again -- and the product kernel gained nothing from finding its
// words in the memory-side cache).  Slabs are whole rounds of the product kernel (32 columns x 8 token
// tiles = one tile per workgroup at 2048 tokens).
static uint32_t staged_slab_cols(const skl_layer *L, uint32_t tokens)
{
    const uint32_t n_col = (L->out + GM3_NT - 1) / GM3_NT, m_tiles = (tokens + GM_MT - 1) / GM_MT;
    const uint64_t col_bytes = (uint64_t)L->gemm_kb * SG_SLOT_BYTES;
    if (n_col * col_bytes <= (1ull << 30)) return n_col;
    const uint32_t round_cols = std::max(1u, 256 / std::max(1u, m_tiles));      // columns of one tile per workgroup
    const uint32_t cols = round_cols * (uint32_t)std::max<uint64_t>(1, (512ull << 20) / (round_cols * col_bytes));
    return std::min(n_col, cols);
}

static uint64_t staged_pack_bytes(const skl_layer *L, uint32_t tokens)
{
    const uint64_t m_tiles = (tokens + GM_MT - 1) / GM_MT;
    return m_tiles * L->gemm_kb * 4 * 8192ull;                  // 8 row blocks of 64 lanes x 16 bytes per (token tile, step)
}

static uint64_t staged_part_bytes(const skl_layer *L, uint32_t tokens)
{
    // the widest slab has the most leftover tiles
    const G3Split sp = skl_make_split(staged_slab_cols(L, tokens) * GM3_NT, L->gemm_kb, tokens, true);
    uint64_t most = 8ull * sp.l_max * sp.p_cap;
    const uint32_t n_col = (L->out + GM3_NT - 1) / GM3_NT, cols = staged_slab_cols(L, tokens);
    if (n_col % cols) {
        const G3Split last = skl_make_split((n_col % cols) * GM3_NT, L->gemm_kb, tokens, true);
        most = std::max<uint64_t>(most, 8ull * last.l_max * last.p_cap);
    }
    return most * G3_SLOT_FLOATS * sizeof(float);
}

uint64_t skl_gemm_staged_bytes(const skl_layer *L, uint32_t tokens)
{
    return round256(staged_pack_bytes(L, tokens)) + round256(staged_part_bytes(L, tokens)) +
           (uint64_t)staged_slab_cols(L, tokens) * L->gemm_kb * SG_SLOT_BYTES;
}

skl_status_t skl_launch_gemm_staged(const skl_layer *L, const TableSrc &src, const uint16_t *X, skl_dtype_t x_dt, uint32_t ldx,
                                    void *Y, skl_dtype_t y_dt, uint32_t ldy, uint32_t tokens, void *ws, hipStream_t stream)
{
    const RowArgs a = make_row_args(L, src);
    char *area = static_cast<char *>(ws);
    uint4 *Xp = reinterpret_cast<uint4 *>(area);
    area += round256(staged_pack_bytes(L, tokens));
    float *parts = reinterpret_cast<float *>(area);
    area += round256(staged_part_bytes(L, tokens));
    uint4 *Wp = reinterpret_cast<uint4 *>(area);
    const uint32_t KB = L->gemm_kb, n_col = (L->out + GM3_NT - 1) / GM3_NT, slab_cols = staged_slab_cols(L, tokens);

    const skl_gemm_step *steps = reinterpret_cast<const skl_gemm_step *>(L->dev + L->off_ssteps);
    skl_status_t st = skl_launch_pack(L, X, x_dt, ldx, tokens, a.chan, steps, 4 * KB, Xp, stream);
    if (st != SKL_OK) return st;
    for (uint32_t tile0 = 0; tile0 < n_col; tile0 += slab_cols) {
        const uint32_t cols = std::min(slab_cols, n_col - tile0);
        RebuildArgs r;
        r.h = a.h; r.bmeta = a.bmeta; r.tables = src.tables; r.Wp = Wp;
        r.out = L->out; r.n_blocks = L->n_blocks; r.KB = KB; r.n_words = L->n_packed / 8;
        r.tile0 = tile0; r.n_col = cols;
        // Output segments per channel block: a workgroup stages its block's table once (as many bytes as
        // the weight words of one or two tiles), so it should rebuild a dozen tiles; but at least ~1024
        // workgroups, and every segment at least one tile column.
        const uint32_t few = (1024 + L->n_blocks - 1) / L->n_blocks, many = (4096 + L->n_blocks - 1) / L->n_blocks;
        r.n_oseg = std::max(1u, std::min(cols, std::max(few, std::min(cols / 12, many))));
        const size_t lds = L->max_table_bytes;
        DISPATCH_D(L->d, {
            st = allow_lds(k_rebuild_operands<D>, lds);
            if (st == SKL_OK) hipLaunchKernelGGL((k_rebuild_operands<D>), dim3(L->n_blocks * r.n_oseg), dim3(SKL_WG), lds, stream, r);
        })
        if (st == SKL_OK) st = check_launch("operand rebuild");
        if (st != SKL_OK) return st;

        StagedArgs g;
        g.Xp = Xp; g.Wp = Wp; g.Y = Y; g.parts = parts;
        g.KB = KB; g.tokens = tokens; g.out = L->out; g.y_dt = (uint32_t)y_dt; g.ldy = ldy;
        g.rows_aligned = ((size_t)ldy * (y_dt == SKL_F32 ? 4 : 2)) % 16 == 0;
        g.tile0 = tile0;
        g.sp = skl_make_split(cols * GM3_NT, KB, tokens, true);
        if (g.sp.mt == GM_MT) {
            st = allow_lds(k_staged_gemm<2>, SG_LDS_BYTES);
            if (st != SKL_OK) return st;
            hipLaunchKernelGGL(k_staged_gemm<2>, dim3(8 * g.sp.gx), dim3(256), SG_LDS_BYTES, stream, g);
        } else {
            st = allow_lds(k_staged_gemm<1>, SG_LDS_BYTES);
            if (st != SKL_OK) return st;
            hipLaunchKernelGGL(k_staged_gemm<1>, dim3(8 * g.sp.gx), dim3(256), SG_LDS_BYTES, stream, g);
        }
        st = check_launch("staged gemm");
        if (st != SKL_OK) return st;
        if (g.sp.l_max) {
            st = skl_launch_gemm3_fixup(g.sp, parts, Y, y_dt, ldy, tokens, L->out, tile0, stream);
            if (st != SKL_OK) return st;
        }
    }
    return SKL_OK;
}

}  // namespace SKL_NS
