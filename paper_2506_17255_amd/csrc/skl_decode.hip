// Fused decode GEMV over row sketches (Sec. 3.1 Eq. 5 fused with y = x W,
// Sec. 2.1): batch-1 kernel, batched (matrix-core) kernel, the grouped
// variants for layers that share their input, and the split reduction.
#include "skl_device.h"

namespace SKL_NS {


// ---- decode GEMV -----------------------------------------------------------
// One workgroup per CU (one wavefront per 64 outputs, up to 16) owns an output
// segment and a group of consecutive channel blocks.  The block tables are
// streamed through two LDS buffers (the next table is copied in while the
// current one is being gathered from), and the per-output sums stay on chip
// across the blocks, so a workgroup emits one partial sum per output for its
// whole block group.
struct StreamArgs {
    RowArgs r;
    const skl_group_info *ginfo;
    uint32_t n_wunits;      // 64-output wave units of the layer
    uint32_t n_sseg;        // output segments
    uint32_t n_bg;          // block groups
    uint32_t tab_bytes;     // LDS bytes of the table area: two buffers SKL_PBUF_DIST apart, or the largest table
    uint32_t upw;           // 64-output units per wavefront (a segment holds at most upw x 16)
    uint32_t buf_flag;      // which bit of a group's flags says that its tables are double-buffered (1: unpadded, 2: padded)
};


struct StreamCtx {
    uint32_t s, g, b_lo, b_hi, c_lo, c_hi, o_lo, o_hi;
    uint32_t K0, rs0, toff0, chan_off0, ptoff0;
    bool live;
    bool two_bufs;          // every table of the group fits one of the two buffers: the next table streams in during a block
};

// Workgroup id -> (segment, group).  Consecutive workgroup ids go to
// different XCDs (8 of them, each with its own L2), so all segments of one
// block group are given ids that are equal modulo 8: a group's tables are
// then fetched from HBM into one L2 only.
__device__ __forceinline__ StreamCtx stream_ctx(const StreamArgs &p)
{
    StreamCtx c;
    const uint32_t xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const uint32_t s = slot % p.n_sseg;
    c.s = s;
    c.g = (slot / p.n_sseg) * 8 + xcd;
    c.live = c.g < p.n_bg;
    const skl_group_info gi = p.ginfo[min(c.g, p.n_bg - 1)];
    c.b_lo = gi.b_lo; c.b_hi = gi.b_hi; c.c_lo = gi.c_lo; c.c_hi = gi.c_hi;
    c.K0 = gi.K0; c.rs0 = gi.rs0; c.toff0 = gi.table_off16_0; c.chan_off0 = gi.chan_off0;
    c.ptoff0 = gi.ptable_off16_0;
    c.two_bufs = (gi.flags & p.buf_flag) != 0;
    if (!skl_in_range(c.b_hi, p.r.n_blocks + 1, SKL_DBG_BLOCK) || !skl_in_range(c.b_lo, c.b_hi + 1, SKL_DBG_BLOCK)) c.live = false;
    c.o_lo = (uint32_t)(((uint64_t)s * p.n_wunits) / p.n_sseg) * 64;
    c.o_hi = min((uint32_t)(((uint64_t)(s + 1) * p.n_wunits) / p.n_sseg) * 64, p.r.out);
    return c;
}

// ---- decode GEMV, batch 1 ---------------------------------------------------
// This kernel reads the unpadded copy of the tables ([r][k][nb] words) and
// spreads a wavefront over (output, word) pairs: with nb words per state row,
// lane l works on word l % nb of 64/nb outputs at a time, so the lanes that
// share an output read one contiguous state row (128 bytes for nb = 8) instead
// of 64 lanes reading 64 unrelated rows.  Measured on MI355X the gather then
// stops being bound by LDS bank conflicts (35 instead of 46 clocks per
// 512 weights and CU) and runs at the rate of the vector ALU.  A lane keeps nb
// partial sums (one per output it visits) across all blocks of a width class;
// they are folded across the nb lanes of an output and parked in LDS when the
// class changes and at the end.
//
// A wavefront owns U units of 64 outputs, unit u of wavefront w being unit w + u * (wavefronts) of the
// segment: with U = 2 a segment is twice as long, half as many workgroups stage each table and a block step
// carries twice the arithmetic between its barriers -- what layers with wide sketches (large tables behind
// few channels) need.
//
// LDS: [table buffer 0][table buffer 1 at SKL_PBUF_DIST][1024 x U sums][block
// metadata][state-row addresses, 1024 x d][activations].  The kernel has no static LDS, so the dynamic region
// starts at LDS address 0 and the second buffer is reached through the 16-bit
// offset field of the read instruction: no address arithmetic per gather.
#define SKL_G1_FIXED_LDS(d, u) (SKL_SWG * 4 * (u) + SKL_MAX_GROUP_BLOCKS * 32 + SKL_SWG * 4 * (d))

// 16 bytes at an absolute LDS address

template <int D, int NB>
__device__ __forceinline__ void lane_offsets(const HashArgs &h, uint32_t o_base, uint32_t out, uint32_t K, uint32_t lane,
                                             uint32_t *row_addr_w, uint32_t (&off)[NB][D])
{
    constexpr uint32_t OPI = 64 / NB;               // outputs per instruction
    const uint32_t sub = lane / NB, cw = lane % NB;
    const uint32_t Kq = K << 8;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void *)smem;
    // The hash values A*o + C do not depend on K; hide that from the compiler,
    // which would otherwise keep them in registers across the block loop.
    asm volatile("" : "+v"(o_base));
    // every lane hashes one output (Eq. 3 for the D rows) and leaves the LDS
    // addresses of its state rows (first buffer, word cw = 0) in the wavefront's
    // scratch area [64][D] ...
    const uint32_t o = min(o_base + lane, out - 1);
#pragma unroll
    for (int r = 0; r < D; ++r) {
        const uint32_t t = __umul24(h.A[r], o) + h.C[r];
        row_addr_w[lane * D + r] = lds0 + (r * K + select_index(t, Kq)) * (NB * 16);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    // ... and picks up the rows of the NB outputs it works on
#pragma unroll
    for (int i = 0; i < NB; ++i) {
#pragma unroll
        for (int r = 0; r < D; ++r) off[i][r] = row_addr_w[(sub + OPI * i) * D + r] + cw * 16;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
}

// sum over the NB adjacent lanes of an output (data-parallel primitives, no LDS)
template <int NB>
__device__ __forceinline__ float sum_over_words(float v)
{
    if (NB >= 2)    // lane ^ 1
        v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
    if (NB >= 4)    // lane ^ 2
        v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
    if (NB >= 8)    // mirror inside 8 lanes: the other quad
        v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
    return v;
}

// one block: NB outputs per lane, one 16-byte word (8 channels) of each.
// The D gathers of the next output are issued before the arithmetic of the
// current one (the scheduling barriers keep them there); left alone, the
// compiler waits for every single gather right after issuing it.
template <int D, int NB, uint32_t BUF_OFF, int MAXW>
__device__ __forceinline__ void lane_block_dot(const uint32_t (&off)[NB][D], uint4 xv, float (&acc)[NB])
{
    // Outputs whose gathers are in flight ahead of the arithmetic, as far as
    // the registers allow: a workgroup of at most 12 wavefronts may use 168
    // registers per lane, one of 16 wavefronts 128.
    constexpr int AHEAD = MAXW <= 12 ? (D <= 4 ? 2 : 1) : (D <= 4 ? 1 : 0);
    constexpr int RING = AHEAD + 1;
    uint4 q[RING][D];
#pragma unroll
    for (int a = 0; a < AHEAD && a < NB; ++a)
#pragma unroll
        for (int r = 0; r < D; ++r) q[a][r] = lds_word_at(off[a][r] + BUF_OFF);
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        if (i + AHEAD < NB) {
#pragma unroll
            for (int r = 0; r < D; ++r) q[(i + AHEAD) % RING][r] = lds_word_at(off[i + AHEAD][r] + BUF_OFF);
        }
        if (AHEAD) __builtin_amdgcn_sched_barrier(0);
        uint4 m = q[i % RING][0];
#pragma unroll
        for (int r = 1; r < D; ++r) m = pk_max_u16x8(m, q[i % RING][r]);
        acc[i] = dot2_acc(keys_to_neg_half2_mad(m.x), xv.x, acc[i]);
        acc[i] = dot2_acc(keys_to_neg_half2_mad(m.y), xv.y, acc[i]);
        acc[i] = dot2_acc(keys_to_neg_half2_mad(m.z), xv.z, acc[i]);
        acc[i] = dot2_acc(keys_to_neg_half2_mad(m.w), xv.w, acc[i]);
        if (AHEAD) __builtin_amdgcn_sched_barrier(0);
    }
}

// The block loop of one workgroup, shared by all width classes.
struct G1Walk {
    const uint4 *sm_meta;    // metadata of the group's blocks in LDS (two 16-byte words each)
    const uint16_t *xs;      // the group's activations (negated binary16) in LDS
    float *yw;               // the wavefront's 64 output sums in LDS
    uint32_t *row_addr_w;    // the wavefront's scratch for state-row addresses, [64][D]
    uint32_t nblk, bi;       // blocks of the group, current block
    uint32_t K, rs, chan_off;   // current block
    uint32_t lane, o_base;   // o_base: first output of the wavefront's unit 0; unit u starts unit_stride outputs further on
    uint32_t unit_stride, o_hi;
    bool wave_live;
    bool first_wait;         // the first table, the activations and the metadata are still on their way
};

// A run of consecutive blocks of one width class (NB words per state row).
// The partial sums and the table offsets of the run live in registers.
template <int D, int NB, int MAXW, int U>
__device__ __forceinline__ void g1_run(const StreamArgs &p, const StreamCtx &c, G1Walk &w)
{
    const uint32_t nw = blockDim.x >> 6;
    constexpr uint32_t OPI = 64 / NB;
    uint4 *const buf0 = smem, *const buf1 = smem + SKL_PBUF_DIST / 16;
    float acc[U][NB];
    uint32_t off[U][NB][D];
    bool live[U];            // wavefront-uniform: unit u of this wavefront lies inside the segment
#pragma unroll
    for (int u = 0; u < U; ++u) {
        live[u] = w.o_base + u * w.unit_stride < w.o_hi;
#pragma unroll
        for (int i = 0; i < NB; ++i) acc[u][i] = 0.f;
    }
    uint32_t K_prev = 0;
    const uint32_t rs_run = w.rs;
    // One block out of the buffer at byte offset BO (a compile-time constant, so that it ends up in the
    // offset field of the LDS reads); with two buffers the next block's table streams into the other one
    // meanwhile, with one it is copied after the block.
    auto step = [&](auto bo_tag, auto bufs_tag) {
        constexpr uint32_t BO = decltype(bo_tag)::value;
        constexpr int BUFS = decltype(bufs_tag)::value;
        const bool more = w.bi + 1 < w.nblk;
        const uint32_t bn = min(w.bi + 1, w.nblk - 1);
        // the state-row addresses need no table: at the start of the workgroup they are computed while
        // the first table is still arriving
        if (w.wave_live && w.K != K_prev) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (live[u]) lane_offsets<D, NB>(p.r.h, w.o_base + u * w.unit_stride, p.r.out, w.K, w.lane, w.row_addr_w, off[u]);
            K_prev = w.K;
        }
        if (w.first_wait) {
            wait_async_copies();
            __syncthreads();
            w.first_wait = false;
        }
        const uint4 m0 = w.sm_meta[2 * bn];          // {table_off16, K, rs, nb}
        const uint4 m1 = w.sm_meta[2 * bn + 1];      // {chan_off, ptable_off16, ..}
        if (BUFS == 2 && more) copy_chunks_to_lds_async(BO ? buf0 : buf1, p.r.tables + m1.y, D * m0.y * m0.w, nw);
        if (w.wave_live) {
            const uint4 xv = reinterpret_cast<const uint4 *>(w.xs + (w.chan_off - c.c_lo))[w.lane % NB];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (live[u]) lane_block_dot<D, NB, BO, MAXW>(off[u], xv, acc[u]);
        }
        if (BUFS == 1 && more) {
            __syncthreads();                 // everyone is done with the only buffer
            copy_chunks_to_lds_async(buf0, p.r.tables + m1.y, D * m0.y * m0.w, nw);
        }
        wait_async_copies();
        __syncthreads();
        w.K = m0.y; w.rs = m0.z; w.chan_off = m1.x;
        ++w.bi;
    };
    const std::integral_constant<uint32_t, 0> at_0;
    const std::integral_constant<uint32_t, SKL_PBUF_DIST> at_dist;
    const std::integral_constant<int, 1> one_buf;
    const std::integral_constant<int, 2> two_bufs;
    auto in_run = [&]() { return w.bi < w.nblk && w.rs == rs_run; };
    if (c.two_bufs) {
        // even blocks sit in the first buffer, odd blocks in the second
        if (w.bi & 1) step(at_dist, two_bufs);
        while (in_run()) {
            step(at_0, two_bufs);
            if (!in_run()) break;
            step(at_dist, two_bufs);
        }
    } else {
        while (in_run()) step(at_0, one_buf);
    }
    // fold the NB lanes of every output, add the totals to the wavefront's sums
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!live[u]) continue;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            // LDS add without a returned value: nothing to wait for between the NB updates
            const float v = sum_over_words<NB>(acc[u][i]);
            if (w.lane % NB == 0)
                __hip_atomic_fetch_add(&w.yw[u * w.unit_stride + w.lane / NB + OPI * i], v, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
}

template <int D, int MAXW, int U>
__device__ __forceinline__ void gemv1_body(const StreamArgs &p, const uint16_t *__restrict__ x, float *__restrict__ partial)
{
    const StreamCtx c = stream_ctx(p);
    if (!c.live) return;
    char *lds = reinterpret_cast<char *>(smem);
    const uint32_t tab_bytes = p.tab_bytes;
    float *ysum = reinterpret_cast<float *>(lds + tab_bytes);
    uint4 *sm_meta = reinterpret_cast<uint4 *>(lds + tab_bytes + SKL_SWG * 4 * U);
    uint32_t *row_addr = reinterpret_cast<uint32_t *>(lds + tab_bytes + SKL_SWG * 4 * U + SKL_MAX_GROUP_BLOCKS * 32);
    uint16_t *xs = reinterpret_cast<uint16_t *>(lds + tab_bytes + SKL_G1_FIXED_LDS(D, U));
    G1Walk w;
    w.lane = threadIdx.x & 63;
    const uint32_t wave = threadIdx.x >> 6;
    w.o_base = c.o_lo + wave * 64;
    w.unit_stride = blockDim.x;          // 64 outputs x wavefronts
    w.o_hi = c.o_hi;
    w.wave_live = w.o_base < c.o_hi;
    w.yw = ysum + wave * 64;
    w.row_addr_w = row_addr + wave * 64 * D;
    w.xs = xs;
    w.nblk = min(c.b_hi - c.b_lo, (uint32_t)SKL_MAX_GROUP_BLOCKS);
    w.bi = 0;
    w.sm_meta = sm_meta;
    w.K = c.K0; w.rs = c.rs0; w.chan_off = c.chan_off0;
    copy_chunks_to_lds_async(smem, p.r.tables + c.ptoff0, D * w.K * (w.rs == 1 ? 1u : w.rs - 1), blockDim.x >> 6);
    // the plan keeps a group at SKL_MAX_GROUP_BLOCKS blocks or fewer
    for (uint32_t i = threadIdx.x; i < 2 * w.nblk; i += blockDim.x) sm_meta[i] = reinterpret_cast<const uint4 *>(p.r.bmeta + c.b_lo)[i];
#pragma unroll
    for (int u = 0; u < U; ++u) w.yw[u * w.unit_stride + w.lane] = 0.f;
    for (uint32_t i = threadIdx.x; i < c.c_hi - c.c_lo; i += blockDim.x) {
        const uint32_t ch = p.r.chan[c.c_lo + i];
        xs[i] = ch != SKL_NO_CHANNEL && skl_in_range(ch, p.r.in, SKL_DBG_CHANNEL) ? (uint16_t)(x[ch] ^ 0x8000u) : (uint16_t)0;
    }
    w.first_wait = true;                 // waited for in the first step of the first run
    while (w.bi < w.nblk) {
        switch (w.rs) {
        case 9:
            if constexpr (D <= 6 && U == 1) {      // the plan uses 8-word blocks for d <= 6 only,
                g1_run<D, 8, MAXW, U>(p, c, w);    // and two units per wavefront only for layers of one- and two-word blocks
                break;                              // (the row addresses of two units x 4 or 8 words do not fit the registers)
            }
        case 5:
            if constexpr (U == 1) {
                g1_run<D, 4, MAXW, U>(p, c, w);
                break;
            }
        case 3: g1_run<D, 2, MAXW, U>(p, c, w); break;
        default: g1_run<D, 1, MAXW, U>(p, c, w); break;
        }
    }
    if (w.first_wait) {                  // a group without blocks: nothing may stay in flight
        wait_async_copies();
        __syncthreads();
    }
    if (w.wave_live) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t o = w.o_base + u * w.unit_stride + w.lane;
            if (o < c.o_hi) partial[(size_t)c.g * p.r.out + o] = w.yw[u * w.unit_stride + w.lane];     // ordinary store: measured 0.25 us faster per call than a non-temporal one
        }
    }
}

template <int D, int MAXW, int U>
__global__ __launch_bounds__(MAXW * 64) void k_row_gemv1(StreamArgs p, const uint16_t *__restrict__ x,
                                                          float *__restrict__ partial)
{
    gemv1_body<D, MAXW, U>(p, x, partial);
}

// Several layers that read the same activations in one launch (q/k/v, gate/up): grid row y runs layer y.
// The layers' workgroups follow each other on the CUs without a kernel boundary, so the start-up and drain
// of one layer overlap the main loop of another and two or three launches become one.
#define SKL_MAX_GROUP_LAYERS 4
struct GroupArgs {
    StreamArgs a[SKL_MAX_GROUP_LAYERS];
    uint64_t partial_stride;        // floats between the partial sums of consecutive layers
    uint32_t xs_stride[SKL_MAX_GROUP_LAYERS];   // batched kernel: halfs per staged activation row
};

template <int D, int MAXW, int U>
__global__ __launch_bounds__(MAXW * 64) void k_row_gemv1_group(GroupArgs m, const uint16_t *__restrict__ x,
                                                                float *__restrict__ partial)
{
    gemv1_body<D, MAXW, U>(m.a[blockIdx.y], x, partial + blockIdx.y * m.partial_stride);
}

// ---- decode GEMV, batch 2..16: the reconstructed weights feed the matrix
// cores.  Same plan, table streaming and buffer scheme as the batch-1 kernel,
// but on the padded tables with lanes = outputs, which is the layout the MFMA
// operand wants: v_mfma_f32_16x16x32_f16 takes the batch as the 16 rows of A
// and, from lane l, the 8 weights of output l % 16 for the channels of word
// l / 16 as B.  A wavefront owns 64 outputs (four 16-output sub-blocks); per
// 32 channels it gathers/queries/decodes four operand words and issues four
// MFMAs.  The sums stay in registers for the whole block group.
typedef float float4v __attribute__((ext_vector_type(4)));

template <int D, int NB>
__device__ __forceinline__ void gn_offsets(const HashArgs &h, uint32_t o_base, uint32_t out, uint32_t K, uint32_t lane,
                                           uint32_t (&off)[4][D])
{
    constexpr uint32_t RS = NB == 1 ? 1 : NB + 1;
    const uint32_t n = lane & 15, kg = lane >> 4;
    const uint32_t word = min(kg, (uint32_t)NB - 1);       // classes with fewer than 4 words: lanes past the last word re-read it, their activations are zero
    const uint32_t Kq = K << 8;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void *)smem;
    asm volatile("" : "+v"(o_base));                        // keep the hashes out of the loop-invariant registers
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t o = min(o_base + 16 * j + n, out - 1);
#pragma unroll
        for (int r = 0; r < D; ++r) {
            const uint32_t t = __umul24(h.A[r], o) + h.C[r];
            off[j][r] = lds0 + ((r * K + select_index(t, Kq)) * RS + word) * 16;
        }
    }
}

// one block: NB words = NB/4 (at least one) slabs of 32 channels x 4 output sub-blocks
template <int D, int NB, uint32_t BUF_OFF>
__device__ __forceinline__ void gn_block(const uint32_t (&off)[4][D], uint32_t x_addr, bool x_live, float4v (&acc)[4])
{
    constexpr int NH = NB == 8 ? 2 : 1;
    constexpr int NP = 4 * NH;                              // (slab, sub-block) pairs
    uint4 a[NH];
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) a[hh] = keep_if(x_live, lds_word_at(x_addr + hh * 64));
    constexpr bool PIPE = D <= 5;                           // gathers of the next pair in flight during the arithmetic (registers allowing)
    uint4 q[PIPE ? 2 : 1][D];
#pragma unroll
    for (int r = 0; r < D; ++r) q[0][r] = lds_word_at(off[0][r] + BUF_OFF);
#pragma unroll
    for (int pr = 0; pr < NP; ++pr) {
        if (PIPE && pr + 1 < NP) {
#pragma unroll
            for (int r = 0; r < D; ++r) q[(pr + 1) & 1][r] = lds_word_at(off[(pr + 1) & 3][r] + BUF_OFF + ((pr + 1) >> 2) * 64);
            __builtin_amdgcn_sched_barrier(0);
        }
        uint4 m = q[PIPE ? pr & 1 : 0][0];
#pragma unroll
        for (int r = 1; r < D; ++r) m = pk_max_u16x8(m, q[PIPE ? pr & 1 : 0][r]);
        uint4 w;
        w.x = keys_to_neg_half2_mad(m.x); w.y = keys_to_neg_half2_mad(m.y);
        w.z = keys_to_neg_half2_mad(m.z); w.w = keys_to_neg_half2_mad(m.w);
        acc[pr & 3] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a[pr >> 2]), __builtin_bit_cast(half8v, w),
                                                              acc[pr & 3], 0, 0, 0);
        if (PIPE && pr + 1 < NP) __builtin_amdgcn_sched_barrier(0);
        if (!PIPE && pr + 1 < NP) {
#pragma unroll
            for (int r = 0; r < D; ++r) q[0][r] = lds_word_at(off[(pr + 1) & 3][r] + BUF_OFF + ((pr + 1) >> 2) * 64);
        }
    }
}

struct GnWalk {
    const uint4 *sm_meta;    // metadata of the group's blocks in LDS
    uint32_t xs_addr;        // LDS address of this lane's activation row (batch row lane % 16)
    uint32_t nblk, bi;
    uint32_t K, rs, chan_off;
    uint32_t lane, o_base;
    bool wave_live;
};

template <int D, int NB>
__device__ __forceinline__ void gn_run(const StreamArgs &p, const StreamCtx &c, GnWalk &w, float4v (&acc)[4])
{
    const uint32_t nw = blockDim.x >> 6;
    uint4 *const buf0 = smem, *const buf1 = smem + SKL_PBUF_DIST / 16;
    uint32_t off[4][D];
    uint32_t K_prev = 0;
    const uint32_t rs_run = w.rs;
    const bool x_live = NB >= 4 || (w.lane >> 4) < (uint32_t)NB;
    auto copy_next = [&](uint4 *dst, const uint4 *src, uint32_t n16) { copy_words_to_lds_async(dst, src, n16, nw); };
    auto step = [&](auto bo_tag) {
        constexpr uint32_t BO = decltype(bo_tag)::value;
        uint4 *nxt = BO || !c.two_bufs ? buf0 : buf1;
        const bool more = w.bi + 1 < w.nblk;
        const uint32_t bn = min(w.bi + 1, w.nblk - 1);
        const uint4 m0 = w.sm_meta[2 * bn];          // {table_off16, K, rs, nb}
        const uint4 m1 = w.sm_meta[2 * bn + 1];      // {chan_off, ..}
        if (more && c.two_bufs) copy_next(nxt, p.r.tables + m0.x, D * m0.y * m0.z);
        if (w.wave_live) {
            if (w.K != K_prev) {
                gn_offsets<D, NB>(p.r.h, w.o_base, p.r.out, w.K, w.lane, off);
                K_prev = w.K;
            }
            gn_block<D, NB, BO>(off, w.xs_addr + (w.chan_off - c.c_lo) * 2 + (x_live ? (w.lane >> 4) * 16 : 0), x_live, acc);
        }
        if (more && !c.two_bufs) {
            __syncthreads();                 // everyone is done with the only buffer
            copy_next(nxt, p.r.tables + m0.x, D * m0.y * m0.z);
        }
        wait_async_copies();
        __syncthreads();
        w.K = m0.y; w.rs = m0.z; w.chan_off = m1.x;
        ++w.bi;
    };
    const std::integral_constant<uint32_t, 0> first_buf;
    const std::integral_constant<uint32_t, SKL_PBUF_DIST> second_buf;
    auto in_run = [&]() { return w.bi < w.nblk && w.rs == rs_run; };
    if (c.two_bufs) {
        if (w.bi & 1) step(second_buf);
        while (in_run()) {
            step(first_buf);
            if (!in_run()) break;
            step(second_buf);
        }
    } else {
        while (in_run()) step(first_buf);
    }
}

#define SKL_GN_FIXED_LDS (SKL_MAX_GROUP_BLOCKS * 32)

template <int D>
__device__ __forceinline__ void gemvN_body(const StreamArgs &p, const uint16_t *__restrict__ x, uint32_t ldx, uint32_t batch,
                                           uint32_t xs_stride, float *__restrict__ partial)
{
    const StreamCtx c = stream_ctx(p);
    if (!c.live) return;
    char *lds = reinterpret_cast<char *>(smem);
    const uint32_t tab_bytes = p.tab_bytes;
    uint4 *sm_meta = reinterpret_cast<uint4 *>(lds + tab_bytes);
    uint16_t *xs = reinterpret_cast<uint16_t *>(lds + tab_bytes + SKL_GN_FIXED_LDS);   // 16 rows of xs_stride halfs
    GnWalk w;
    w.lane = threadIdx.x & 63;
    const uint32_t wave = threadIdx.x >> 6, nwv = blockDim.x >> 6;
    w.nblk = min(c.b_hi - c.b_lo, (uint32_t)SKL_MAX_GROUP_BLOCKS);
    w.sm_meta = sm_meta;
    w.xs_addr = (uint32_t)(uintptr_t)(lds_void *)xs + (w.lane & 15) * xs_stride * 2;
    auto first_table = [&]() { copy_words_to_lds_async(smem, p.r.tables + c.toff0, D * c.K0 * c.rs0, nwv); };
    first_table();
    for (uint32_t i = threadIdx.x; i < 2 * w.nblk; i += blockDim.x) sm_meta[i] = reinterpret_cast<const uint4 *>(p.r.bmeta + c.b_lo)[i];
    // activations of the group's channels, 16 rows (rows >= batch are zero): one
    // thread per (channel, half of the rows), so that the channel number is
    // fetched once and the eight activation loads that depend on it go out together
    const uint32_t nch = c.c_hi - c.c_lo;
    for (uint32_t i = threadIdx.x; i < 2 * nch; i += blockDim.x) {
        const uint32_t cc = i >> 1, b0 = (i & 1) * 8;
        const uint32_t ch = p.r.chan[c.c_lo + cc];
        uint16_t v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            v[k] = 0;
            if (ch != SKL_NO_CHANNEL && b0 + k < batch && skl_in_range(ch, p.r.in, SKL_DBG_CHANNEL)) v[k] = x[(size_t)(b0 + k) * ldx + ch] ^ 0x8000u;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) xs[(b0 + k) * xs_stride + cc] = v[k];
    }
    // A segment of more than 16 units (plans made for the batch-1 kernel's two units per wavefront) is
    // walked in passes: the wavefronts take units 0 .. nwv - 1, then nwv .. 2 nwv - 1, streaming the group's
    // tables again for each pass.
    for (uint32_t pass = 0; pass < p.upw; ++pass) {
        w.o_base = c.o_lo + (pass * nwv + wave) * 64;
        w.wave_live = w.o_base < c.o_hi;
        w.bi = 0;
        w.K = c.K0; w.rs = c.rs0; w.chan_off = c.chan_off0;
        if (pass) first_table();             // the last step of the previous pass ended with a barrier: the first buffer is free
        wait_async_copies();
        __syncthreads();
        float4v acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = (float4v){0.f, 0.f, 0.f, 0.f};
        while (w.bi < w.nblk) {
            switch (w.rs) {
            case 9: gn_run<D, 8>(p, c, w, acc); break;
            case 5: gn_run<D, 4>(p, c, w, acc); break;
            case 3: gn_run<D, 2>(p, c, w, acc); break;
            default: gn_run<D, 1>(p, c, w, acc); break;
            }
        }
        if (w.wave_live) {
            // acc[j][i]: batch row 4 * (lane / 16) + i, output o_base + 16 * j + lane % 16
            float *pblk = partial + (size_t)c.g * batch * p.r.out;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t o = w.o_base + 16 * j + (w.lane & 15);
                if (o < c.o_hi) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t m = 4 * (w.lane >> 4) + i;
                        if (m < batch) __builtin_nontemporal_store(acc[j][i], &pblk[(size_t)m * p.r.out + o]);
                    }
                }
            }
        }
    }
}

template <int D>
__global__ __launch_bounds__(SKL_SWG) void k_row_gemvN(StreamArgs p, const uint16_t *__restrict__ x, uint32_t ldx,
                                                        uint32_t batch, uint32_t xs_stride, float *__restrict__ partial)
{
    gemvN_body<D>(p, x, ldx, batch, xs_stride, partial);
}

// the batched kernel for a group of layers on the same activations: grid row y runs layer y
template <int D>
__global__ __launch_bounds__(SKL_SWG) void k_row_gemvN_group(GroupArgs m, const uint16_t *__restrict__ x, uint32_t ldx,
                                                              uint32_t batch, float *__restrict__ partial)
{
    gemvN_body<D>(m.a[blockIdx.y], x, ldx, batch, m.xs_stride[blockIdx.y], partial + blockIdx.y * m.partial_stride);
}


// ---- second pass of the split reduction: y[b][o] = sum_u partial[u][b][o] ---
// A workgroup owns 64 outputs (16 lanes x 4 consecutive outputs) of one batch
// row; its 16 lane rows each sum every 16th partial, then the 16 slices are
// added in a fixed order, so the result is the same on every run.
#define RED_O 64
__device__ __forceinline__ void reduce_body(const float *__restrict__ partial, uint32_t n_units, uint32_t batch, uint32_t out,
                                            void *__restrict__ y, uint32_t y_dt, uint32_t ldy)
{
    __shared__ float4 red[16][16];
    const uint32_t oq = threadIdx.x & 15, slice = threadIdx.x >> 4;
    const uint32_t o = blockIdx.x * RED_O + oq * 4;
    const uint32_t b = blockIdx.y;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (o < out) {
        const bool vec = (out & 3u) == 0;   // rows of `partial` are 16-byte aligned
        for (uint32_t u = slice; u < n_units; u += 16) {
            const float *p = partial + ((size_t)u * batch + b) * out + o;
            if (vec) {
                const float4 v = *reinterpret_cast<const float4 *>(p);
                s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
            } else {
                s.x += p[0];
                if (o + 1 < out) s.y += p[1];
                if (o + 2 < out) s.z += p[2];
                if (o + 3 < out) s.w += p[3];
            }
        }
    }
    red[slice][oq] = s;
    __syncthreads();
    if (slice == 0 && o < out) {
        float4 t = red[0][oq];
#pragma unroll
        for (int i = 1; i < 16; ++i) {
            const float4 v = red[i][oq];
            t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
        }
        const size_t base = (size_t)b * ldy + o;
        store_out(y, y_dt, base, t.x);
        if (o + 1 < out) store_out(y, y_dt, base + 1, t.y);
        if (o + 2 < out) store_out(y, y_dt, base + 2, t.z);
        if (o + 3 < out) store_out(y, y_dt, base + 3, t.w);
    }
}

__global__ __launch_bounds__(SKL_WG) void k_reduce_partials(const float *__restrict__ partial, uint32_t n_units,
                                                             uint32_t batch, uint32_t out, void *__restrict__ y,
                                                             uint32_t y_dt, uint32_t ldy)
{
    reduce_body(partial, n_units, batch, out, y, y_dt, ldy);
}

// the reductions of a group of layers: grid (ceil(out / 64), batch, layers)
struct GroupReduceArgs {
    void *y[SKL_MAX_GROUP_LAYERS];
    uint32_t n_units[SKL_MAX_GROUP_LAYERS];
    uint64_t partial_stride;
};

// gate/up pair of a feed-forward block (Sec. 2.1, Eq. 2 with SiLU as the activation): both reductions and
// h[o] = SiLU(gate[o]) * up[o] in one pass; layer 0 of the group is the gate, layer 1 the up projection
// grid (ceil(out / 64), batch)
__global__ __launch_bounds__(SKL_WG) void k_reduce_gate_up(const float *__restrict__ partial, GroupReduceArgs g, uint32_t batch,
                                                            uint32_t out, void *__restrict__ h, uint32_t h_dt, uint32_t ldh)
{
    __shared__ float4 red[2][16][16];
    const uint32_t oq = threadIdx.x & 15, slice = threadIdx.x >> 4;
    const uint32_t o = blockIdx.x * RED_O + oq * 4, b = blockIdx.y;
    const bool vec = (out & 3u) == 0;
#pragma unroll
    for (int l = 0; l < 2; ++l) {
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        if (o < out) {
            for (uint32_t u = slice; u < g.n_units[l]; u += 16) {
                const float *p = partial + l * g.partial_stride + ((size_t)u * batch + b) * out + o;
                if (vec) {
                    const float4 v = *reinterpret_cast<const float4 *>(p);
                    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
                } else {
                    s.x += p[0];
                    if (o + 1 < out) s.y += p[1];
                    if (o + 2 < out) s.z += p[2];
                    if (o + 3 < out) s.w += p[3];
                }
            }
        }
        red[l][slice][oq] = s;
    }
    __syncthreads();
    if (slice == 0 && o < out) {
        float4 t[2];
#pragma unroll
        for (int l = 0; l < 2; ++l) {
            t[l] = red[l][0][oq];
#pragma unroll
            for (int i = 1; i < 16; ++i) {
                const float4 v = red[l][i][oq];
                t[l].x += v.x; t[l].y += v.y; t[l].z += v.z; t[l].w += v.w;
            }
        }
        const float a[4] = {t[0].x, t[0].y, t[0].z, t[0].w}, bb[4] = {t[1].x, t[1].y, t[1].z, t[1].w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (o + i < out) store_out(h, h_dt, (size_t)b * ldh + o + i, a[i] / (1.0f + expf(-a[i])) * bb[i]);
    }
}

__global__ __launch_bounds__(SKL_WG) void k_reduce_partials_group(const float *__restrict__ partial, GroupReduceArgs g,
                                                                   uint32_t batch, uint32_t out, uint32_t y_dt, uint32_t ldy)
{
    reduce_body(partial + blockIdx.z * g.partial_stride, g.n_units[blockIdx.z], batch, out, g.y[blockIdx.z], y_dt, ldy);
}


// ========================================================================
// Launchers
// ========================================================================
// partial sums of the split reduction
static uint64_t gemv_partial_bytes(const skl_layer *L, uint32_t batch)
{
    return (uint64_t)L->n_units * batch * L->out * sizeof(float);
}

// low-bit states: the expanded tables follow the call's own scratch
uint64_t skl_gemv_workspace_bytes(const skl_layer *L, uint32_t batch)
{
    const uint64_t own = gemv_partial_bytes(L, batch);
    return L->qbits ? round256(own) + skl_dequant_bytes(L) : own;
}

uint64_t skl_reconstruct_workspace_bytes(const skl_layer *L) { return skl_dequant_bytes(L); }

// LDS bytes of the batch-1 kernel for a layer
static size_t gemv1_lds_bytes(const skl_layer *L)
{
    return (size_t)L->ptab_bytes + SKL_G1_FIXED_LDS(L->d, L->decode_upw) + (size_t)(L->max_group_chan + 64) * sizeof(uint16_t);
}

// the batch-1 kernel by sketch rows, register budget (workgroups of up to 12 wavefronts may use 168 registers
// per lane, larger ones 128) and units per wavefront
template <int MAXW, int U>
static skl_status_t launch_gemv1_as(uint32_t d, uint32_t waves, dim3 grid, size_t lds, hipStream_t stream, const StreamArgs &a,
                                    const uint16_t *x, float *partial)
{
    skl_status_t st = SKL_OK;
    DISPATCH_D(d, {
        st = allow_lds(k_row_gemv1<D, MAXW, U>, lds);
        if (st == SKL_OK) hipLaunchKernelGGL((k_row_gemv1<D, MAXW, U>), grid, dim3(64 * waves), lds, stream, a, x, partial);
    })
    return st;
}

static skl_status_t launch_gemv1(uint32_t d, uint32_t waves, uint32_t upw, dim3 grid, size_t lds, hipStream_t stream,
                                 const StreamArgs &a, const uint16_t *x, float *partial)
{
    if (upw == 1) return waves <= 12 ? launch_gemv1_as<12, 1>(d, waves, grid, lds, stream, a, x, partial)
                                     : launch_gemv1_as<16, 1>(d, waves, grid, lds, stream, a, x, partial);
    return waves <= 12 ? launch_gemv1_as<12, 2>(d, waves, grid, lds, stream, a, x, partial)
                       : launch_gemv1_as<16, 2>(d, waves, grid, lds, stream, a, x, partial);
}

skl_status_t skl_launch_gemv(const skl_layer *L, const void *x_, uint32_t ldx, void *y, skl_dtype_t y_dt,
                             uint32_t ldy, uint32_t batch, void *ws, void *stream_, bool with_reduction)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const uint16_t *x = static_cast<const uint16_t *>(x_);
    float *partial = static_cast<float *>(ws);
    TableSrc src;
    skl_status_t st = skl_table_source(L, static_cast<char *>(ws) + round256(gemv_partial_bytes(L, batch)),
                                   L->path == 1 && batch > 1, L->path == 1 && batch == 1, stream, &src);
    if (st != SKL_OK) return st;
    if (L->path == 1) {
        StreamArgs a;
        a.r = make_row_args(L, src);
        a.ginfo = reinterpret_cast<const skl_group_info *>(L->dev + L->off_ginfo);
        a.n_wunits = L->n_wunits; a.n_sseg = L->n_sseg; a.n_bg = L->n_bg;
        a.upw = L->decode_upw;
        const dim3 grid(8 * ((L->n_bg + 7) / 8) * L->n_sseg);
        // one wavefront per upw 64-output units of the longest segment (at least two for the start-up loads)
        const uint32_t seg_units = (L->n_wunits + L->n_sseg - 1) / L->n_sseg;
        const uint32_t waves = std::max(2u, (seg_units + L->decode_upw - 1) / L->decode_upw);
        if (batch == 1) {
            // unpadded tables; buffers at fixed LDS addresses
            a.r.tables = src.ptables;
            a.tab_bytes = L->ptab_bytes;
            a.buf_flag = 1;
            const size_t lds = gemv1_lds_bytes(L);
            st = launch_gemv1(L->d, waves, L->decode_upw, grid, lds, stream, a, x, partial);
        } else {
            // padded tables; 16 activation rows of xs_stride halfs, xs_stride / 8 odd (bank spread of the MFMA A reads)
            const uint32_t xs_stride = (L->max_group_chan / 8 | 1u) * 8;
            a.tab_bytes = L->tab_bytes;
            a.buf_flag = 2;
            const size_t lds = (size_t)L->tab_bytes + SKL_GN_FIXED_LDS + (size_t)16 * xs_stride * sizeof(uint16_t);
            DISPATCH_D(L->d, {
                st = allow_lds(k_row_gemvN<D>, lds);
                if (st == SKL_OK)
                    hipLaunchKernelGGL((k_row_gemvN<D>), grid, dim3(64 * waves), lds, stream, a, x, ldx, batch, xs_stride, partial);
            })
        }
    } else {
        st = skl_tile_launch_gemv(L, src, x, ldx, batch, partial, stream);
    }
    if (st != SKL_OK) return st;
    st = check_launch("gemv");
    if (st != SKL_OK || !with_reduction) return st;
    hipLaunchKernelGGL(k_reduce_partials, dim3((L->out + RED_O - 1) / RED_O, batch), dim3(SKL_WG), 0, stream, partial,
                       L->n_units, batch, L->out, y, (uint32_t)y_dt, ldy);
    return check_launch("gemv reduction");
}

// ---- batch-1 decode of up to four layers that share their activations --------
static bool group_layer_ok(const skl_layer *L, const skl_layer *first)
{
    return L->path == 1 && L->in == first->in && L->out == first->out && L->d == first->d && L->decode_upw == first->decode_upw;
}

static uint64_t group_partial_stride(const skl_layer *const *layers, uint32_t n, uint32_t batch)
{
    uint64_t stride = 0;
    for (uint32_t i = 0; i < n; ++i) stride = std::max(stride, round256(gemv_partial_bytes(layers[i], batch)));
    return stride;
}

uint64_t skl_gemv_group_workspace_bytes(const skl_layer *const *layers, uint32_t n, uint32_t batch)
{
    uint64_t expanded = 0;
    for (uint32_t i = 0; i < n; ++i) expanded += skl_dequant_bytes(layers[i]);     // low-bit layers: their tables, after all partial sums
    return group_partial_stride(layers, n, batch) * n + expanded;
}

template <int MAXW, int U>
static skl_status_t launch_gemv1_group_as(uint32_t d, uint32_t waves, dim3 grid, size_t lds, hipStream_t stream, const GroupArgs &m,
                                          const uint16_t *x, float *partial)
{
    skl_status_t st = SKL_OK;
    DISPATCH_D(d, {
        st = allow_lds(k_row_gemv1_group<D, MAXW, U>, lds);
        if (st == SKL_OK) hipLaunchKernelGGL((k_row_gemv1_group<D, MAXW, U>), grid, dim3(64 * waves), lds, stream, m, x, partial);
    })
    return st;
}

static skl_status_t launch_gemv1_group(uint32_t d, uint32_t waves, uint32_t upw, dim3 grid, size_t lds, hipStream_t stream,
                                       const GroupArgs &m, const uint16_t *x, float *partial)
{
    if (upw == 1) return waves <= 12 ? launch_gemv1_group_as<12, 1>(d, waves, grid, lds, stream, m, x, partial)
                                     : launch_gemv1_group_as<16, 1>(d, waves, grid, lds, stream, m, x, partial);
    return waves <= 12 ? launch_gemv1_group_as<12, 2>(d, waves, grid, lds, stream, m, x, partial)
                       : launch_gemv1_group_as<16, 2>(d, waves, grid, lds, stream, m, x, partial);
}

skl_status_t skl_launch_gemv_group(const skl_layer *const *layers, uint32_t n, const void *x_, uint32_t ldx, void *const *ys,
                                   skl_dtype_t y_dt, uint32_t ldy, uint32_t batch, void *ws, void *stream_, bool gate_up)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const skl_layer *F = layers[0];
    for (uint32_t i = 0; i < n; ++i)
        if (!group_layer_ok(layers[i], F)) {
            skl_set_error("layer %u of the group is not a row-sketch layer of the first layer's shape and decode plan (units per wavefront)", i);
            return SKL_ERR_UNSUPPORTED;
        }
    const bool one = batch == 1;                               // the batch-1 kernel reads the unpadded tables
    GroupArgs m;
    GroupReduceArgs gr;
    const uint64_t stride_bytes = group_partial_stride(layers, n, batch);
    m.partial_stride = gr.partial_stride = stride_bytes / sizeof(float);
    uint32_t grid_x = 0, waves = 2;
    size_t lds = 0;
    char *area = static_cast<char *>(ws) + stride_bytes * n;
    TableSrc srcs[SKL_MAX_GROUP_LAYERS];
    for (uint32_t i = 0; i < n; ++i) {                          // low-bit layers: expand their tables first
        skl_status_t st0 = skl_table_source(layers[i], area, !one, one, stream, &srcs[i]);
        if (st0 != SKL_OK) return st0;
        area += skl_dequant_bytes(layers[i]);
    }
    for (uint32_t i = 0; i < SKL_MAX_GROUP_LAYERS; ++i) {
        const skl_layer *L = layers[i < n ? i : 0];            // unused slots repeat the first layer
        const TableSrc &src = srcs[i < n ? i : 0];
        StreamArgs &a = m.a[i];
        a.r = make_row_args(L, src);
        a.ginfo = reinterpret_cast<const skl_group_info *>(L->dev + L->off_ginfo);
        a.n_wunits = L->n_wunits; a.n_sseg = L->n_sseg; a.n_bg = L->n_bg;
        a.upw = L->decode_upw;
        const uint32_t xs_stride = (L->max_group_chan / 8 | 1u) * 8;
        m.xs_stride[i] = xs_stride;
        size_t need;
        if (one) {
            a.r.tables = src.ptables;
            a.tab_bytes = L->ptab_bytes;
            a.buf_flag = 1;
            need = gemv1_lds_bytes(L);
        } else {
            a.tab_bytes = L->tab_bytes;
            a.buf_flag = 2;
            need = (size_t)L->tab_bytes + SKL_GN_FIXED_LDS + (size_t)16 * xs_stride * sizeof(uint16_t);
        }
        gr.y[i] = ys[i < n ? i : 0];
        gr.n_units[i] = L->n_units;
        if (i >= n) continue;
        grid_x = std::max(grid_x, 8 * ((L->n_bg + 7) / 8) * L->n_sseg);
        const uint32_t seg_units = (L->n_wunits + L->n_sseg - 1) / L->n_sseg;
        waves = std::max(waves, (seg_units + L->decode_upw - 1) / L->decode_upw);
        lds = std::max(lds, need);
    }
    const uint16_t *x = static_cast<const uint16_t *>(x_);
    float *partial = static_cast<float *>(ws);
    skl_status_t st = SKL_OK;
    const dim3 grid(grid_x, n);
    if (!one) {
        DISPATCH_D(F->d, {
            st = allow_lds(k_row_gemvN_group<D>, lds);
            if (st == SKL_OK)
                hipLaunchKernelGGL((k_row_gemvN_group<D>), grid, dim3(64 * waves), lds, stream, m, x, ldx, batch, partial);
        })
    } else {
        st = launch_gemv1_group(F->d, waves, F->decode_upw, grid, lds, stream, m, x, partial);
    }
    if (st != SKL_OK) return st;
    st = check_launch("grouped gemv");
    if (st != SKL_OK) return st;
    if (gate_up)
        hipLaunchKernelGGL(k_reduce_gate_up, dim3((F->out + RED_O - 1) / RED_O, batch), dim3(SKL_WG), 0, stream, partial, gr, batch,
                           F->out, ys[0], (uint32_t)y_dt, ldy);
    else
        hipLaunchKernelGGL(k_reduce_partials_group, dim3((F->out + RED_O - 1) / RED_O, batch, n), dim3(SKL_WG), 0, stream, partial, gr,
                           batch, F->out, (uint32_t)y_dt, ldy);
    return check_launch("grouped gemv reduction");
}

}  // namespace SKL_NS

#if SKL_QM == 0
// ---- decode without a caller workspace ----------------------------------------
// For callers that cannot allocate (code under HIP graph capture, serving loops, harnesses that forbid it):
// the partial sums of the split reduction (and, for low-bit layers, the expanded tables) go to a file-scope
// device array instead of a workspace argument.  Every GPU the library runs on holds its own copy of the
// array at its own address until the process ends; the address is looked up once per device, with that
// device current, and only that pointer (never the array's name) is handed on: the decode kernels of either
// query mode take it as their workspace argument.
static __device__ __align__(256) unsigned char scratch[SKL_STATIC_SCRATCH_BYTES];

#define SKL_MAX_DEVICES 64
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[SKL_MAX_DEVICES];

uint64_t skl_static_scratch_bytes() { return SKL_STATIC_SCRATCH_BYTES; }

// device address of the current device's copy of the array
skl_status_t skl_static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= SKL_MAX_DEVICES) {
        skl_set_error("cannot identify the current device: %s", e != hipSuccess ? hipGetErrorString(e) : "device number out of range");
        return SKL_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            skl_set_error("address of the static scratch array on device %d: %s", dev, hipGetErrorString(e));
            return SKL_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return SKL_OK;
}
#endif
