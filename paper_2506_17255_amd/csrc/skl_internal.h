// Internal declarations shared by the host side (skl_host.cpp) and the
// kernels (skl_kernels.hip) of the sketch-linear library.  Not installed.
#pragma once

#include <stdint.h>
#include <vector>

#include "sketch_linear.h"

#define SKL_MAX_D 8
#define SKL_WG 256            // threads per workgroup: 4 wavefronts of 64
#define SKL_SWG 1024          // threads per workgroup of the streaming decode kernels
#define SKL_N_CU 256          // compute units of the target (MI355X)
#define SKL_NO_CHANNEL 0xFFFFFFFFu
#define SKL_MAX_GROUP_BLOCKS 64   // most channel blocks in one block group of the decode plan (metadata kept in LDS)

// LDS budgets.  A CU of gfx950 has 160 KiB of LDS.  A block takes the most words per state row (8, 4, 2, 1)
// whose padded table still fits one of the decode kernels' two table buffers.
#define SKL_LDS_SOFT_TABLE_BYTES 65280u
#define SKL_LDS_HARD_BYTES 163840u
// Distance between the two table buffers of the batch-1 decode kernel: below
// 2^16, so that the buffer is chosen by the offset field of the LDS reads.
#define SKL_PBUF_DIST 65280u
// file-scope device array behind sketch_linear_gemv_static: the workspace of one decode call
#define SKL_STATIC_SCRATCH_BYTES SKL_STATIC_SCRATCH_MAX

// ---- path 0: 2-D groups, one hash evaluation per weight and sketch row ----
struct skl_group_meta {
    uint32_t key_off;   // first key of the group, in 16-bit units from the key base
    uint32_t K;         // states per sketch row (Sec. 3.3: K may differ per group)
};

// ---- path 1: row sketches (tile_in = 1, tile_out = d_out) -------------------
// Input channels are sorted by width and cut into blocks of 8*nb channels that
// share one width K.  A block's table is laid out [r][k][rs] in 16-byte words:
// word (r*K + k)*rs + c holds the keys of channels 8c..8c+7 of the block for
// state (r,k); rs is odd so that consecutive k fall into different LDS bank
// groups, and nb = rs - 1 words per state row are used (nb = 1 when rs = 1).
struct skl_block_meta {
    uint32_t table_off16;  // table start, in 16-byte words from the table base
    uint32_t K;
    uint32_t rs;           // words per state row: 1, 3, 5 or 9
    uint32_t nb;           // used words per state row (8*nb channels per block)
    uint32_t chan_off;     // first entry of the block in the channel list
                           // (= first packed activation column of the block)
    uint32_t ptable_off16; // the block's table in the unpadded copy ([r][k][nb] words)
    uint32_t step_off;     // first 16-channel MFMA step of the block in the prefill walk
    uint32_t scale_off16;  // low-bit states: the block's scale words ([r][c] x eight binary16 scales) from the scale base
};

// One block group of the decode plan: consecutive blocks [b_lo, b_hi), their
// channel-list range [c_lo, c_hi), and the first block's metadata so that a
// workgroup needs one load before it can fetch its first table.
struct skl_group_info {
    uint32_t b_lo, b_hi, c_lo, c_hi;
    uint32_t K0, rs0, table_off16_0, chan_off0;
    uint32_t ptable_off16_0;
    uint32_t flags;        // bit 0: every unpadded table of the group fits one of the two LDS buffers (batch-1 kernel);
                           // bit 1: the same for the padded tables (batched kernel)
    uint32_t pad1, pad2;
};

// One 16-channel step of the prefill walk: two 16-byte words of a block (one
// for blocks with a single word per state row).
struct skl_gemm_step {
    uint32_t chan0;        // first entry of the step in the channel list
    uint32_t n_words;      // 1 or 2
};

struct skl_layer {
    uint32_t in = 0, out = 0, tj = 0, to = 0, d = 0;
    uint32_t A[SKL_MAX_D] = {0}, C[SKL_MAX_D] = {0};
    uint32_t path = 0;
    uint32_t query_mode = 0;        // 0: Max by magnitude, 1: Max of the signed values (Sec. 3.1 Eq. 5 as printed)
    uint8_t *dev = nullptr;
    uint64_t dev_bytes = 0;
    uint64_t n_states = 0;
    uint64_t table_bytes = 0;
    uint32_t max_table_bytes = 0;   // largest per-workgroup table
    uint32_t n_units = 0;           // partial sums per output in gemv

    // path 0
    uint32_t n_jb = 0, n_ob = 0, max_K = 0;
    uint32_t jc_rows = 0, n_jc = 0; // a group's tile_in rows are cut into n_jc chunks
    uint64_t off_gmeta = 0, off_keys = 0;

    // path 1
    uint32_t n_blocks = 0;
    uint32_t n_packed = 0;          // channel-list length = sum of 8*nb over blocks
    uint32_t n_otiles = 0, n_seg = 0;
    uint64_t off_bmeta = 0, off_chan = 0, off_tables = 0;
    // second copy of the tables without the padding word per state row, for
    // the batch-1 decode kernel whose lanes read whole state rows
    uint64_t off_ptables = 0, ptable_bytes = 0;
    uint32_t max_ptable_bytes = 0;
    uint32_t block_classes = 0;     // bit log2(nb) set for every words-per-state-row class present
    uint32_t n_small_blocks = 0;    // blocks before the first one whose padded table exceeds 49.5 KiB,
    uint32_t small_table_bytes = 0; // and the largest padded table among them
    // decode plan: workgroup (s, g) owns output segment s (a range of 64-output
    // wave units) and block group g (consecutive channel blocks bg_start[g] ..
    // bg_start[g+1]); n_sseg * n_bg workgroups of 1024 threads, one per CU
    uint32_t n_sseg = 0, n_bg = 0, n_wunits = 0;
    double decode_cost_us = 0;      // the planner's model for this split
    uint32_t max_group_chan = 0;    // most channel-list entries in one block group
    uint32_t opl = 1;               // outputs per lane: ceil(segment length / 1024)
    uint32_t decode_upw = 1;        // 64-output units per wavefront of the batch-1 kernel (segments of up to 16 x upw units)
    uint32_t tab_bytes = 0;         // LDS table area of the batched kernel (padded tables): two buffers SKL_PBUF_DIST apart
                                    // if any block group is double-buffered, and never less than the largest table
    uint32_t ptab_bytes = 0;        // the same for the batch-1 kernel and the unpadded tables
    uint64_t off_ginfo = 0;
    // fused prefill kernel (256 x 256 tile, weights rebuilt between the matrix instructions): usable when two
    // unpadded block tables (at most 48 KiB each), two operand slots and the block metadata fit in LDS
    uint32_t gemm_v3 = 0, n_gsteps = 0;
    uint64_t off_gsteps = 0;
    // staged prefill (weights rebuilt once per call into the workspace): 64-channel blocks along the channel
    // list, and its dense step list (4 steps of 16 list entries per block)
    uint32_t gemm_staged_from = 0, gemm_kb = 0;     // calls with at least gemm_staged_from tokens are staged
    uint64_t off_ssteps = 0;

    // low-bit states: only codes and scales are resident (row sketches: re-ordered into the word order of the
    // block tables); every call expands them into 16-bit tables at the end of its workspace
    uint32_t qbits = 0;             // 0 (binary16 states), 8 or 4
    uint64_t off_codes = 0, off_scales = 0, code_bytes = 0, scale_bytes = 0;
    uint32_t scale_words = 0;       // row sketches: 16-byte scale words over all blocks
    uint64_t off_chunk_block = 0;   // row sketches: channel block of every 64-word chunk of the unpadded tables
    uint32_t n_groups = 0;
};

// The host-side plan: everything create() copies to the device.
struct skl_plan {
    skl_layer L;
    skl_desc_t desc;                // the caller's description in the current layout of the struct
    uint32_t want_s = 0, want_g = 0;   // diagnostic: plan this decode split (segments, groups) instead of the cheapest
    uint64_t dev_bytes = 0;
    std::vector<skl_group_meta> gmeta;
    std::vector<skl_block_meta> bmeta;
    std::vector<uint32_t> chan;
    std::vector<uint32_t> bg_start;
    std::vector<skl_group_info> ginfo;
    std::vector<skl_gemm_step> gsteps;
    std::vector<skl_gemm_step> ssteps;
};

static inline bool skl_gemm_is_staged(const skl_layer *L, uint32_t tokens) { return tokens >= L->gemm_staged_from; }

// error text of the calling thread
void skl_set_error(const char *fmt, ...);

// Debug build (-DSKL_DEBUG_BOUNDS): every translation unit with kernels registers a reader of its
// range-assert record (count, then code, value, limit, workgroup, thread of the first violation).
typedef skl_status_t (*skl_debug_reader)(uint32_t rec[8]);
void skl_debug_register(skl_debug_reader fn);

// validation + planning (host only); fills `plan` without touching `states`
// beyond the finiteness check
skl_status_t skl_make_plan(const skl_desc_t *desc, skl_plan *plan);

// Order key of a binary16 bit pattern: the query (Eq. 5) becomes an unsigned 16-bit maximum of keys.
//   mode 0: magnitude first, the clear sign bit wins a tie;
//   mode 1: the order of the signed values, +0 above -0.
static inline uint16_t skl_key_of_half(uint16_t b, uint32_t mode)
{
    if (mode == 0) return (uint16_t)(((b & 0x7FFFu) << 1) | (1u - (b >> 15)));
    return (uint16_t)(b & 0x8000u ? ~b : b | 0x8000u);
}

// ---- launchers implemented in skl_kernels.hip (all enqueue only) -----------
skl_status_t skl_launch_reconstruct(const skl_layer *L, uint16_t *W_hat, void *ws, void *stream);
// the hash-based operator as a comparator: per-weight select, states fetched from device memory (skl_naive.hip)
skl_status_t skl_launch_reconstruct_naive(const skl_layer *L, uint16_t *W_hat, void *ws, void *stream);
// bytes of expanded tables at the end of every workspace of a layer with low-bit states (else 0)
uint64_t skl_dequant_bytes(const skl_layer *L);
uint64_t skl_reconstruct_workspace_bytes(const skl_layer *L);
// with_reduction = false: partial sums only (y, y_dt, ldy unused)
skl_status_t skl_launch_gemv(const skl_layer *L, const void *x, uint32_t ldx, void *y,
                             skl_dtype_t y_dt, uint32_t ldy, uint32_t batch, void *ws, void *stream,
                             bool with_reduction);
skl_status_t skl_launch_gemm(const skl_layer *L, const void *X, skl_dtype_t x_dt, uint32_t ldx,
                             void *Y, skl_dtype_t y_dt, uint32_t ldy, uint32_t tokens, void *ws,
                             void *stream);
uint64_t skl_gemv_workspace_bytes(const skl_layer *L, uint32_t batch);
// decode with the library's static device array as workspace (at most skl_static_scratch_bytes())
uint64_t skl_static_scratch_bytes();
skl_status_t skl_launch_gemv_static(const skl_layer *L, const void *x, uint32_t ldx, void *y, skl_dtype_t y_dt, uint32_t ldy,
                                    uint32_t batch, void *stream);
uint64_t skl_gemm_workspace_bytes(const skl_layer *L, uint32_t tokens);
// decode of 1..4 row-sketch layers of one shape that share x; gate_up: n = 2 (gate, up), ys[0] receives SiLU(gate) * up
uint64_t skl_gemv_group_workspace_bytes(const skl_layer *const *layers, uint32_t n, uint32_t batch);
skl_status_t skl_launch_gemv_group(const skl_layer *const *layers, uint32_t n, const void *x, uint32_t ldx, void *const *ys,
                                   skl_dtype_t y_dt, uint32_t ldy, uint32_t batch, void *ws, void *stream, bool gate_up);
// sketch construction: group_base holds n_groups + 1 state offsets (host); synchronises the stream once
skl_status_t skl_launch_build(const skl_desc_t *d, uint64_t n_groups, const uint64_t *group_base, const uint16_t *W,
                              uint16_t *states, void *ws, void *stream);
// ceilings of the machine: four small kernels (skl_microbench.hip)
uint64_t skl_microbench_work(uint32_t kind, uint32_t iters, uint64_t ws_bytes);
skl_status_t skl_launch_microbench(uint32_t kind, uint32_t iters, void *ws, uint64_t ws_bytes, void *stream);
skl_status_t skl_launch_debug_selftest(uint32_t value, uint32_t limit, void *stream);
uint64_t skl_gemm3_segments(uint32_t out, uint32_t n_blocks, uint32_t tokens, bool by_col, uint32_t *segs, uint64_t cap,
                            uint32_t *shape);
