// HIP kernels (gfx950 only) of the sketch-linear library and their launchers.
//
// Common ground of every kernel here (Sec. 3.1 of the paper):
//   select  Eq. 3   t = (A_r * a + C_r) mod 2^24,  k = floor(t * K / 2^24)
//                   -> one 24-bit multiply-add and one 24-bit multiply-high
//   gather          the d candidate states come from an LDS-resident copy of
//                   the group's sketch table
//   query   Eq. 5   the states are stored as 16-bit order keys
//                   key = magnitude << 1 | (sign bit clear), so the AbsMaxMin
//                   query is a plain unsigned 16-bit maximum (two weights per
//                   packed instruction)
//   decode          the winning key is turned back into binary16 with the
//                   sign bit inverted: -w = (key >> 1) | (key << 15 & 0x8000);
//                   the activations are negated once when they are staged, so
//                   every product x * w keeps its sign and value.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>
#include <mutex>
#include <unordered_map>

#include "skl_internal.h"

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));

extern __shared__ uint4 smem[];

// --------------------------------------------------------------- helpers
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b)
{
    ushort2v m = __builtin_elementwise_max(__builtin_bit_cast(ushort2v, a), __builtin_bit_cast(ushort2v, b));
    return __builtin_bit_cast(uint32_t, m);
}

__device__ __forceinline__ uint4 pk_max_u16x8(uint4 a, uint4 b)
{
    return make_uint4(pk_max_u16(a.x, b.x), pk_max_u16(a.y, b.y), pk_max_u16(a.z, b.z), pk_max_u16(a.w, b.w));
}

// two keys -> two binary16 values with inverted sign bits
__device__ __forceinline__ uint32_t keys_to_neg_half2(uint32_t k)
{
    return ((k >> 1) & 0x7FFF7FFFu) | ((k << 15) & 0x80008000u);
}

// The same in two instructions instead of three, for loops bound by the vector
// ALU: per 16-bit half, (k >> 1) + k * 0x8000 (the product keeps bit 0 of k in
// bit 15; the two terms share no bit).  The compiler turns the multiply back
// into a shift and an OR, hence the explicit packed multiply-add.
__device__ __forceinline__ uint32_t keys_to_neg_half2_mad(uint32_t k)
{
    uint32_t t, r;
    asm("v_pk_lshrrev_b16 %0, 1, %1 op_sel_hi:[0,1]" : "=v"(t) : "v"(k));
    asm("v_pk_mad_u16 %0, %1, %2, %3" : "=v"(r) : "v"(k), "s"(0x80008000u), "v"(t));
    return r;
}

__device__ __forceinline__ uint4 keys_to_neg_half8(uint4 k)
{
    return make_uint4(keys_to_neg_half2(k.x), keys_to_neg_half2(k.y), keys_to_neg_half2(k.z), keys_to_neg_half2(k.w));
}

// value or zero, component by component (a select of whole 16-byte objects
// would be turned into a select of addresses and spill the object to memory)
__device__ __forceinline__ uint4 keep_if(bool keep, uint4 v)
{
    return make_uint4(keep ? v.x : 0u, keep ? v.y : 0u, keep ? v.z : 0u, keep ? v.w : 0u);
}

// Asynchronous copy global -> LDS without passing through registers
// (global_load_lds_dwordx4): a wavefront moves 64 consecutive 16-byte words,
// lane i's word landing at dst + i.  The copy is complete after
// wait_async_copies() by the issuing wavefront (and a barrier for everybody
// else).
typedef __attribute__((address_space(3))) void lds_void;

// One global_load_lds_dwordx4: every active lane moves 16 bytes from its own
// global address to lds_dst + lane (lds_dst is the same for the whole
// wavefront).  Written as inline assembly on purpose: the compiler then does
// not know that LDS is being written behind its back and does not force the
// copy to complete before the next LDS read; completion is awaited explicitly
// (wait_async_copies / wait_vmcnt_le) before a barrier publishes the data.
__device__ __forceinline__ void lds_dma_16(const void *gptr, uint4 *lds_dst)
{
    const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void *)lds_dst);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr) : "memory", "m0");
}

// A source padded to whole 64-word chunks (no bounds check per lane), copied
// by a workgroup of nw wavefronts: wavefront w moves chunks w, w + nw, ..
__device__ __forceinline__ void copy_chunks_to_lds_async(uint4 *dst, const uint4 *src, uint32_t n16, uint32_t nw)
{
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint32_t n_chunks = (n16 + 63) >> 6;
    for (uint32_t ch = wave; ch < n_chunks; ch += nw) lds_dma_16(src + ch * 64 + lane, dst + ch * 64);
}

__device__ __forceinline__ void wait_async_copies()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), other counters untouched
}

// Eq. 3: index inside a sketch row of width K; Kq = K << 8 (< 2^24).  Only the
// low 24 bits of t count, so t may be kept as a wrapping 32-bit number.
__device__ __forceinline__ uint32_t select_index(uint32_t t, uint32_t Kq)
{
    return (uint32_t)(((uint64_t)(t & 0xFFFFFFu) * (uint64_t)(Kq & 0xFFFFFFu)) >> 32);
}

__device__ __forceinline__ float dot2_acc(uint32_t w2, uint32_t x2, float acc)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, w2), __builtin_bit_cast(half2v, x2), acc, false);
}

__device__ __forceinline__ float half_bits_to_float(uint16_t h)
{
    return (float)__builtin_bit_cast(_Float16, h);
}

__device__ __forceinline__ uint16_t float_to_half_bits(float f)
{
    return __builtin_bit_cast(uint16_t, (_Float16)f);   // round to nearest even
}

__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)
{
    // the conversion instruction of the hardware: nearest even, denormals kept, NaN stays a quiet NaN
    // (checked against the integer formulation over all 2^32 binary32 patterns)
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}

__device__ __forceinline__ void store_out(void *y, uint32_t dt, size_t idx, float v)
{
    if (dt == SKL_F32) static_cast<float *>(y)[idx] = v;
    else if (dt == SKL_F16) static_cast<uint16_t *>(y)[idx] = float_to_half_bits(v);
    else static_cast<uint16_t *>(y)[idx] = float_to_bf16_bits(v);
}

// activation element -> binary16 bits with the sign inverted
__device__ __forceinline__ uint16_t load_neg_half(const uint16_t *X, uint32_t x_dt, size_t idx)
{
    uint16_t b = X[idx];
    if (x_dt == SKL_BF16) b = float_to_half_bits(__builtin_bit_cast(float, (uint32_t)b << 16));
    return b ^ 0x8000u;
}

static_assert(sizeof(skl_block_meta) == 32, "block metadata is read as two 16-byte words");

struct HashArgs {
    uint32_t A[SKL_MAX_D];
    uint32_t C[SKL_MAX_D];
};

// ========================================================================
// Path 1: row sketches.  One sketch per input channel over all d_out outputs,
// so the state index of (j, o) depends on o and on the channel's width only.
// ========================================================================
struct RowArgs {
    HashArgs h;
    const skl_block_meta *bmeta;
    const uint32_t *chan;
    const uint4 *tables;
    uint32_t in, out, n_blocks, n_otiles, n_seg;
};

__device__ __forceinline__ void stage_table(uint4 *dst, const uint4 *src, uint32_t n16)
{
    for (uint32_t i = threadIdx.x; i < n16; i += SKL_WG) dst[i] = src[i];
}

// word offsets (r*K + k_r(o)) * rs of output channel o in a block table
template <int D>
__device__ __forceinline__ void row_offsets(const HashArgs &h, uint32_t o, uint32_t K, uint32_t rs, uint32_t (&off)[D])
{
    const uint32_t Kq = K << 8;
#pragma unroll
    for (int r = 0; r < D; ++r) {
        const uint32_t t = __umul24(h.A[r], o) + h.C[r];
        off[r] = (r * K + select_index(t, Kq)) * rs;
    }
}

// query for 8 consecutive channels of the block: word c of every row
template <int D>
__device__ __forceinline__ uint4 row_query8(const uint4 *tab, const uint32_t (&off)[D], uint32_t c)
{
    uint4 m = tab[off[0] + c];
#pragma unroll
    for (int r = 1; r < D; ++r) m = pk_max_u16x8(m, tab[off[r] + c]);
    return m;
}

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
    uint32_t buf_words;     // 16-byte words per table buffer
    uint32_t two_bufs;
};


struct StreamCtx {
    uint32_t s, g, b_lo, b_hi, c_lo, c_hi, o_lo, o_hi;
    uint32_t K0, rs0, toff0, chan_off0, ptoff0;
    bool live;
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
// LDS: [table buffer 0][table buffer 1 at SKL_PBUF_DIST][1024 sums][block
// metadata][state-row addresses, 1024 x d][activations].  The kernel has no static LDS, so the dynamic region
// starts at LDS address 0 and the second buffer is reached through the 16-bit
// offset field of the read instruction: no address arithmetic per gather.
#define SKL_G1_FIXED_LDS(d) (SKL_SWG * 4 + SKL_MAX_GROUP_BLOCKS * 32 + SKL_SWG * 4 * (d))

// 16 bytes at an absolute LDS address
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 lds_word_at(uint32_t addr)
{
    const u32x4v v = *(const __attribute__((address_space(3))) u32x4v *)(uintptr_t)addr;
    return make_uint4(v.x, v.y, v.z, v.w);
}

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
    uint32_t lane, o_base;
    bool wave_live;
    bool first_wait;         // the first table, the activations and the metadata are still on their way
};

// A run of consecutive blocks of one width class (NB words per state row).
// The partial sums and the table offsets of the run live in registers.
template <int D, int NB, int MAXW>
__device__ __forceinline__ void g1_run(const StreamArgs &p, const StreamCtx &c, G1Walk &w)
{
    const uint32_t nw = blockDim.x >> 6;
    constexpr uint32_t OPI = 64 / NB;
    uint4 *const buf0 = smem, *const buf1 = smem + SKL_PBUF_DIST / 16;
    float acc[NB];
    uint32_t off[NB][D];
#pragma unroll
    for (int i = 0; i < NB; ++i) acc[i] = 0.f;
    uint32_t K_prev = 0;
    const uint32_t rs_run = w.rs;
    // one block out of the buffer at byte offset BO (a compile-time constant, so
    // that it ends up in the offset field of the LDS reads); meanwhile the
    // next block's table streams into the other buffer
    auto step = [&](auto bo_tag) {
        constexpr uint32_t BO = decltype(bo_tag)::value;
        uint4 *nxt = BO || !p.two_bufs ? buf0 : buf1;
        const bool more = w.bi + 1 < w.nblk;
        const uint32_t bn = min(w.bi + 1, w.nblk - 1);
        // the state-row addresses need no table: at the start of the workgroup they are computed while
        // the first table is still arriving
        if (w.wave_live && w.K != K_prev) {
            lane_offsets<D, NB>(p.r.h, w.o_base, p.r.out, w.K, w.lane, w.row_addr_w, off);
            K_prev = w.K;
        }
        if (w.first_wait) {
            wait_async_copies();
            __syncthreads();
            w.first_wait = false;
        }
        const uint4 m0 = w.sm_meta[2 * bn];          // {table_off16, K, rs, nb}
        const uint4 m1 = w.sm_meta[2 * bn + 1];      // {chan_off, ptable_off16, ..}
        if (more && p.two_bufs) copy_chunks_to_lds_async(nxt, p.r.tables + m1.y, D * m0.y * m0.w, nw);
        if (w.wave_live) {
            const uint4 xv = reinterpret_cast<const uint4 *>(w.xs + (w.chan_off - c.c_lo))[w.lane % NB];
            lane_block_dot<D, NB, BO, MAXW>(off, xv, acc);
        }
        if (more && !p.two_bufs) {
            __syncthreads();                 // everyone is done with the only buffer
            copy_chunks_to_lds_async(nxt, p.r.tables + m1.y, D * m0.y * m0.w, nw);
        }
        wait_async_copies();
        __syncthreads();
        w.K = m0.y; w.rs = m0.z; w.chan_off = m1.x;
        ++w.bi;
    };
    const std::integral_constant<uint32_t, 0> first_buf;
    const std::integral_constant<uint32_t, SKL_PBUF_DIST> second_buf;
    auto in_run = [&]() { return w.bi < w.nblk && w.rs == rs_run; };
    if (p.two_bufs) {
        // even blocks sit in the first buffer, odd blocks in the second
        if (w.bi & 1) step(second_buf);
        while (in_run()) {
            step(first_buf);
            if (!in_run()) break;
            step(second_buf);
        }
    } else {
        while (in_run()) step(first_buf);
    }
    // fold the NB lanes of every output, add the totals to the wavefront's sums
    if (w.wave_live) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            // LDS add without a returned value: nothing to wait for between the NB updates
            const float v = sum_over_words<NB>(acc[i]);
            if (w.lane % NB == 0)
                __hip_atomic_fetch_add(&w.yw[w.lane / NB + OPI * i], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
}

template <int D, int MAXW>
__device__ __forceinline__ void gemv1_body(const StreamArgs &p, const uint16_t *__restrict__ x, float *__restrict__ partial)
{
    const StreamCtx c = stream_ctx(p);
    if (!c.live) return;
    char *lds = reinterpret_cast<char *>(smem);
    const uint32_t tab_bytes = p.two_bufs ? 2 * SKL_PBUF_DIST : p.buf_words * 16;
    float *ysum = reinterpret_cast<float *>(lds + tab_bytes);
    uint4 *sm_meta = reinterpret_cast<uint4 *>(lds + tab_bytes + SKL_SWG * 4);
    uint32_t *row_addr = reinterpret_cast<uint32_t *>(lds + tab_bytes + SKL_SWG * 4 + SKL_MAX_GROUP_BLOCKS * 32);
    uint16_t *xs = reinterpret_cast<uint16_t *>(lds + tab_bytes + SKL_G1_FIXED_LDS(D));
    G1Walk w;
    w.lane = threadIdx.x & 63;
    const uint32_t wave = threadIdx.x >> 6;
    w.o_base = c.o_lo + wave * 64;
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
    w.yw[w.lane] = 0.f;
    for (uint32_t i = threadIdx.x; i < c.c_hi - c.c_lo; i += blockDim.x) {
        const uint32_t ch = p.r.chan[c.c_lo + i];
        xs[i] = ch != SKL_NO_CHANNEL ? (uint16_t)(x[ch] ^ 0x8000u) : (uint16_t)0;
    }
    w.first_wait = true;                 // waited for in the first step of the first run
    while (w.bi < w.nblk) {
        switch (w.rs) {
        case 9:
            if constexpr (D <= 6) {      // the plan uses 8-word blocks for d <= 6 only
                g1_run<D, 8, MAXW>(p, c, w);
                break;
            }
        case 5: g1_run<D, 4, MAXW>(p, c, w); break;
        case 3: g1_run<D, 2, MAXW>(p, c, w); break;
        default: g1_run<D, 1, MAXW>(p, c, w); break;
        }
    }
    if (w.first_wait) {                  // a group without blocks: nothing may stay in flight
        wait_async_copies();
        __syncthreads();
    }
    if (w.wave_live) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        const uint32_t o = w.o_base + w.lane;
        if (o < c.o_hi) partial[(size_t)c.g * p.r.out + o] = w.yw[w.lane];     // ordinary store: measured 0.25 us faster per call than a non-temporal one
    }
}

template <int D, int MAXW>
__global__ __launch_bounds__(MAXW * 64) void k_row_gemv1(StreamArgs p, const uint16_t *__restrict__ x,
                                                          float *__restrict__ partial)
{
    gemv1_body<D, MAXW>(p, x, partial);
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

template <int D, int MAXW>
__global__ __launch_bounds__(MAXW * 64) void k_row_gemv1_group(GroupArgs m, const uint16_t *__restrict__ x,
                                                                float *__restrict__ partial)
{
    gemv1_body<D, MAXW>(m.a[blockIdx.y], x, partial + blockIdx.y * m.partial_stride);
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
    auto copy_next = [&](uint4 *dst, const uint4 *src, uint32_t n16) {
        const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        for (uint32_t base = wave * 64; base < n16; base += 64 * nw)
            if (base + lane < n16) lds_dma_16(src + base + lane, dst + base);
    };
    auto step = [&](auto bo_tag) {
        constexpr uint32_t BO = decltype(bo_tag)::value;
        uint4 *nxt = BO || !p.two_bufs ? buf0 : buf1;
        const bool more = w.bi + 1 < w.nblk;
        const uint32_t bn = min(w.bi + 1, w.nblk - 1);
        const uint4 m0 = w.sm_meta[2 * bn];          // {table_off16, K, rs, nb}
        const uint4 m1 = w.sm_meta[2 * bn + 1];      // {chan_off, ..}
        if (more && p.two_bufs) copy_next(nxt, p.r.tables + m0.x, D * m0.y * m0.z);
        if (w.wave_live) {
            if (w.K != K_prev) {
                gn_offsets<D, NB>(p.r.h, w.o_base, p.r.out, w.K, w.lane, off);
                K_prev = w.K;
            }
            gn_block<D, NB, BO>(off, w.xs_addr + (w.chan_off - c.c_lo) * 2 + (x_live ? (w.lane >> 4) * 16 : 0), x_live, acc);
        }
        if (more && !p.two_bufs) {
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
    if (p.two_bufs) {
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
    const uint32_t tab_bytes = p.two_bufs ? 2 * SKL_PBUF_DIST : p.buf_words * 16;
    uint4 *sm_meta = reinterpret_cast<uint4 *>(lds + tab_bytes);
    uint16_t *xs = reinterpret_cast<uint16_t *>(lds + tab_bytes + SKL_GN_FIXED_LDS);   // 16 rows of xs_stride halfs
    GnWalk w;
    w.lane = threadIdx.x & 63;
    const uint32_t wave = threadIdx.x >> 6;
    w.o_base = c.o_lo + wave * 64;
    w.wave_live = w.o_base < c.o_hi;
    w.nblk = min(c.b_hi - c.b_lo, (uint32_t)SKL_MAX_GROUP_BLOCKS);
    w.bi = 0;
    w.sm_meta = sm_meta;
    w.K = c.K0; w.rs = c.rs0; w.chan_off = c.chan_off0;
    w.xs_addr = (uint32_t)(uintptr_t)(lds_void *)xs + (w.lane & 15) * xs_stride * 2;
    {
        const uint32_t nwv = blockDim.x >> 6, n16 = D * w.K * w.rs;
        for (uint32_t base = wave * 64; base < n16; base += 64 * nwv)
            if (base + w.lane < n16) lds_dma_16(p.r.tables + c.toff0 + base + w.lane, smem + base);
    }
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
            if (ch != SKL_NO_CHANNEL && b0 + k < batch) v[k] = x[(size_t)(b0 + k) * ldx + ch] ^ 0x8000u;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) xs[(b0 + k) * xs_stride + cc] = v[k];
    }
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

// ---- reconstruct (diagnostic): the same table, offsets and query ----------
template <int D, int RS>
__device__ __forceinline__ void row_reconstruct_body(const RowArgs &p, const skl_block_meta &bm, const uint4 *tab,
                                                     const uint32_t *chs, uint16_t *W_hat)
{
    constexpr int NB = RS == 1 ? 1 : RS - 1;
    const uint32_t seg = blockIdx.y;
    const uint32_t lo = (uint32_t)(((uint64_t)seg * p.n_otiles) / p.n_seg);
    const uint32_t hi = (uint32_t)(((uint64_t)(seg + 1) * p.n_otiles) / p.n_seg);
    for (uint32_t tile = lo; tile < hi; ++tile) {
        const uint32_t o = tile * SKL_WG + threadIdx.x;
        if (o >= p.out) continue;
        uint32_t off[D];
        row_offsets<D>(p.h, o, bm.K, RS, off);
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            const uint4 w = keys_to_neg_half8(row_query8<D>(tab, off, c));
            const uint32_t v[4] = {w.x ^ 0x80008000u, w.y ^ 0x80008000u, w.z ^ 0x80008000u, w.w ^ 0x80008000u};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t ch = chs[c * 8 + i];
                if (ch != SKL_NO_CHANNEL) W_hat[(size_t)ch * p.out + o] = (uint16_t)(v[i >> 1] >> ((i & 1) * 16));
            }
        }
    }
}

template <int D>
__global__ __launch_bounds__(SKL_WG) void k_row_reconstruct(RowArgs p, uint16_t *__restrict__ W_hat)
{
    const skl_block_meta bm = p.bmeta[blockIdx.x];
    const uint32_t n16 = D * bm.K * bm.rs;
    stage_table(smem, p.tables + bm.table_off16, n16);
    uint32_t *chs = reinterpret_cast<uint32_t *>(smem + n16);
    if (threadIdx.x < 8 * bm.nb) chs[threadIdx.x] = p.chan[bm.chan_off + threadIdx.x];
    __syncthreads();
    switch (bm.rs) {
    case 9: row_reconstruct_body<D, 9>(p, bm, smem, chs, W_hat); break;
    case 5: row_reconstruct_body<D, 5>(p, bm, smem, chs, W_hat); break;
    case 3: row_reconstruct_body<D, 3>(p, bm, smem, chs, W_hat); break;
    default: row_reconstruct_body<D, 1>(p, bm, smem, chs, W_hat); break;
    }
}

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
#define GM_MT 256            // tokens per workgroup
#define GM_NT 128            // outputs per workgroup
#define GM_THREADS 512       // four compute + four copy wavefronts

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
// Operand slot: word (cb, row = 2*step + k-group, n) at ((cb*8 + row)*34 + n);
// 34 instead of 32 words per row keeps the producers' scattered writes (eight
// rows, two neighbouring n per 16 lanes) on distinct banks.
#define G2_ROW 34u
#define G2_CB_WORDS (8u * G2_ROW)

// grid (ceil(steps / 4), 8 * token tiles); a workgroup re-orders 32 tokens x 4 steps
__global__ __launch_bounds__(SKL_WG) void k_pack_activations2(const uint16_t *__restrict__ X, uint32_t x_dt, uint32_t ldx,
                                                               uint32_t tokens, const uint32_t *__restrict__ chan,
                                                               const skl_gemm_step *__restrict__ steps, uint32_t n_steps,
                                                               uint4 *__restrict__ Xp)
{
    const uint32_t g = threadIdx.x & 7, n = threadIdx.x >> 3;      // k-group (step, half) and token of the 32-token row block
    const uint32_t step = blockIdx.x * 4 + (g >> 1), q = g & 1;
    if (step >= n_steps) return;
    const uint32_t rb = blockIdx.y & 7, tile_m = blockIdx.y >> 3;
    const uint32_t t = tile_m * GM_MT + rb * 32 + n;
    const skl_gemm_step st = steps[step];
    uint16_t v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        v[i] = 0;
        if (q < st.n_words && t < tokens) {
            const uint32_t ch = chan[st.chan0 + 8 * q + i];
            if (ch != SKL_NO_CHANNEL) v[i] = load_neg_half(X, x_dt, (size_t)t * ldx + ch);
        }
    }
    uint4 w;
    w.x = v[0] | ((uint32_t)v[1] << 16); w.y = v[2] | ((uint32_t)v[3] << 16);
    w.z = v[4] | ((uint32_t)v[5] << 16); w.w = v[6] | ((uint32_t)v[7] << 16);
    Xp[(((size_t)tile_m * n_steps + step) * 8 + rb) * 64 + q * 32 + n] = w;
}

// The same re-ordering with the rows staged in LDS: a workgroup reads TOK whole token rows with
// coalesced loads (converting them to negated binary16 once), then gathers every step's channels from
// LDS.
// grid (ceil(tokens / TOK)); TOK divides 32; LDS TOK * (in + 4) * 2 bytes.
template <int TOK>
__global__ __launch_bounds__(SKL_WG) void k_pack_activations3(const uint16_t *__restrict__ X, uint32_t x_dt, uint32_t ldx,
                                                               uint32_t tokens, uint32_t in, const uint32_t *__restrict__ chan,
                                                               const skl_gemm_step *__restrict__ steps, uint32_t n_steps,
                                                               uint4 *__restrict__ Xp)
{
    uint16_t *rows = reinterpret_cast<uint16_t *>(smem);
    const uint32_t stride = ((in + 1) & ~1u) + 2;               // elements: even, and off the power-of-two bank pattern
    const uint32_t t_first = blockIdx.x * TOK;
    const bool vec = ldx % 8 == 0;
    for (uint32_t j = 0; j < TOK; ++j) {
        const uint32_t t = t_first + j;
        if (t >= tokens) break;
        const uint16_t *src = X + (size_t)t * ldx;
        uint16_t *dst = rows + j * stride;
        if (vec) {
            for (uint32_t c = threadIdx.x * 8; c < in; c += SKL_WG * 8) {
                if (c + 8 <= in) {
                    const uint4 w = *reinterpret_cast<const uint4 *>(src + c);
                    const uint32_t e[4] = {w.x, w.y, w.z, w.w};
                    uint32_t *d32 = reinterpret_cast<uint32_t *>(dst + c);      // rows and c are even: dword aligned
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        uint32_t lo = e[i] & 0xFFFFu, hi = e[i] >> 16;
                        if (x_dt == SKL_BF16) {
                            lo = float_to_half_bits(__builtin_bit_cast(float, lo << 16));
                            hi = float_to_half_bits(__builtin_bit_cast(float, hi << 16));
                        }
                        d32[i] = (lo | (hi << 16)) ^ 0x80008000u;
                    }
                } else {
                    for (uint32_t i = c; i < in; ++i) dst[i] = load_neg_half(src, x_dt, i);
                }
            }
        } else {
            for (uint32_t c = threadIdx.x; c < in; c += SKL_WG) dst[c] = load_neg_half(src, x_dt, c);
        }
    }
    __syncthreads();
    // a thread takes one 8-channel word position and fills it for all TOK tokens: its channel list is
    // read once, and its TOK words are neighbours in the packed layout
    const uint32_t tile_m = t_first / GM_MT, rb = (t_first % GM_MT) / 32, n0 = t_first % 32;
    for (uint32_t item = threadIdx.x; item < 2 * n_steps; item += SKL_WG) {
        const uint32_t step = item >> 1, q = item & 1;
        const skl_gemm_step st = steps[step];
        uint32_t ch[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) ch[i] = q < st.n_words ? chan[st.chan0 + 8 * q + i] : SKL_NO_CHANNEL;
        uint4 *dst = Xp + (((size_t)tile_m * n_steps + step) * 8 + rb) * 64 + q * 32 + n0;
#pragma unroll
        for (uint32_t j = 0; j < TOK; ++j) {
            const uint16_t *row = rows + j * stride;
            uint16_t v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = ch[i] != SKL_NO_CHANNEL && t_first + j < tokens ? row[ch[i]] : (uint16_t)0;
            uint4 w;
            w.x = v[0] | ((uint32_t)v[1] << 16); w.y = v[2] | ((uint32_t)v[3] << 16);
            w.z = v[4] | ((uint32_t)v[5] << 16); w.w = v[6] | ((uint32_t)v[7] << 16);
            dst[j] = w;
        }
    }
}

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

struct Gemm2Args {
    HashArgs h;
    const uint4 *ptables;
    const skl_block_meta *bmeta;
    const uint4 *Xp;
    const uint4 *zeros;        // at least 1 KiB of zero bytes
    void *Y;
    uint32_t n_blocks, n_steps, tokens, out, y_dt, ldy, tab_words, n_col, m_tiles;
    float *parts;              // third kernel: partial tiles
    uint32_t T, gx, l_max, p_cap;
    uint32_t rows_aligned;     // every row of Y starts on a 16-byte boundary
};

// producers: table offsets (bytes from the table start) of the rows this lane gathers
template <int D, int NB>
__device__ __forceinline__ void g2_offsets(const HashArgs &h, uint32_t o_first, uint32_t out, uint32_t K, uint32_t lane,
                                           uint32_t (&off)[4][D])
{
    constexpr uint32_t OPI = 64 / NB;                       // outputs per gather instruction
    constexpr int SETS = NB >= 2 ? NB / 2 : 1;              // instructions for the 32 outputs of a column block
    const uint32_t sub = lane / NB, cw = lane % NB;
    const uint32_t Kq = K << 8;
    asm volatile("" : "+v"(o_first));                       // keep the hashes out of the loop-invariant registers
#pragma unroll
    for (int s = 0; s < SETS; ++s) {
        const uint32_t o = min(o_first + min(OPI * s + sub, 31u), out - 1);
#pragma unroll
        for (int r = 0; r < D; ++r) {
            const uint32_t t = __umul24(h.A[r], o) + h.C[r];
            off[s][r] = ((r * K + select_index(t, Kq)) * NB + cw) * 16;
        }
    }
}

// producers: rebuild the operand words of one block for column block cb
template <int D, int NB>
__device__ __forceinline__ void g2_build(const uint32_t (&off)[4][D], uint32_t tab_addr, uint32_t slot_addr, uint32_t cb,
                                         uint32_t lane)
{
    constexpr uint32_t OPI = 64 / NB;
    constexpr int SETS = NB >= 2 ? NB / 2 : 1;
    const uint32_t sub = lane / NB, cw = lane % NB;
    uint4 q[2][D];
#pragma unroll
    for (int r = 0; r < D; ++r) q[0][r] = lds_word_at(tab_addr + off[0][r]);
#pragma unroll
    for (int s = 0; s < SETS; ++s) {
        if (s + 1 < SETS) {
#pragma unroll
            for (int r = 0; r < D; ++r) q[(s + 1) & 1][r] = lds_word_at(tab_addr + off[s + 1][r]);
            __builtin_amdgcn_sched_barrier(0);
        }
        uint4 m = q[s & 1][0];
#pragma unroll
        for (int r = 1; r < D; ++r) m = pk_max_u16x8(m, q[s & 1][r]);
        u32x4v w;
        w.x = keys_to_neg_half2_mad(m.x); w.y = keys_to_neg_half2_mad(m.y);
        w.z = keys_to_neg_half2_mad(m.z); w.w = keys_to_neg_half2_mad(m.w);
        const uint32_t n = OPI * s + sub;
        if (NB > 1 || n < 32)
            *(__attribute__((address_space(3))) u32x4v *)(uintptr_t)(slot_addr + ((cb * 8 + cw) * G2_ROW + n) * 16) = w;
        __builtin_amdgcn_sched_barrier(0);
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
#define GM3_NT 256
#define G3_CB_WORDS (8u * G2_ROW)
#define G3_SLOT_BYTES (8u * G3_CB_WORDS * 16u)

// Work split of the third kernel.  Tile t = tile_n * m_tiles + tile_m belongs to XCD t % 8 (workgroup
// ids go round the XCDs, so with eight or more token tiles an XCD keeps one token tile's activations
// in its L2).  An XCD runs gx workgroups; its tiles are dealt out in rounds of gx whole tiles, and the
// blocks of the tiles left over after the last whole round are cut into equal contiguous shares, one
// per workgroup, so that every workgroup multiplies the same number of blocks (within one).  A share
// that covers part of a tile leaves a float32 partial in the workspace; the fix-up kernel adds a
// tile's partials in workgroup order, which keeps the result independent of timing.
struct G3Split {
    uint32_t T, m_tiles, nb, gx;        // tiles, token tiles, blocks per tile, workgroups per XCD
    uint32_t l_max, p_cap;              // workspace slots: [xcd][l_max leftover tiles][p_cap parts]
    __host__ __device__ uint32_t tiles_of(uint32_t x) const { return T > x ? (T - x + 7) / 8 : 0; }
    __host__ __device__ uint32_t rounds(uint32_t x) const { return tiles_of(x) / gx; }
    __host__ __device__ uint32_t left(uint32_t x) const { return tiles_of(x) - rounds(x) * gx; }
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
            sg.k = wg + round * gx; sg.k0 = 0; sg.k1 = nb; sg.whole = 1;
            ++round;
            return true;
        }
        if (u_next >= u_end) return false;
        const uint32_t l = u_next / nb;
        sg.k0 = u_next - l * nb;
        sg.k1 = sg.k0 + (u_end - u_next) < nb ? sg.k0 + (u_end - u_next) : nb;
        sg.k = n_rounds * gx + l;
        sg.whole = sg.k0 == 0 && sg.k1 == nb;
        sg.part_slot = slot(x, l, wg - owner(x, l * nb));
        u_next += sg.k1 - sg.k0;
        return true;
    }
};
#define G3_SLOT_FLOATS 65536u           // one 256 x 256 partial

// One accumulator element, read where it is used.  Left to itself the compiler copies all 256
// elements out of the accumulation registers after the block loop and parks half of them in scratch memory.
__device__ __forceinline__ float acc_elem(float v)
{
    float r;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(v));
    return r;
}

template <int DT>
__device__ __forceinline__ void gemm3_store(const float16v (&acc)[16], void *Y, uint32_t ldy, uint32_t t0, uint32_t tokens,
                                            uint32_t o0, uint32_t out, uint32_t q)
{
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) {
        const uint32_t o = o0 + cb * 32;
        if (o >= out) continue;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t t = t0 + rb * 32 + (i >> 2) * 8 + q * 4 + (i & 3);
                if (t < tokens) {
                    const size_t idx = (size_t)t * ldy + o;
                    const float v = acc_elem(acc[rb * 8 + cb][i]);
                    if (DT == SKL_F32) static_cast<float *>(Y)[idx] = v;
                    else if (DT == SKL_F16) static_cast<uint16_t *>(Y)[idx] = float_to_half_bits(v);
                    else static_cast<uint16_t *>(Y)[idx] = float_to_bf16_bits(v);
                }
            }
        }
    }
}

// Row-major epilogue of the third kernel: a wavefront turns its 64 x 256 results round in a private LDS
// area, one group of rows at a time, and stores 16-byte pieces, so that every store instruction writes
// whole 512-byte (1 KiB for float32) rows of Y instead of 2-byte elements.  Needs 16-byte aligned rows.
#define G3_EPI_BYTES 16896u             // per wavefront: 32 rows x (512 + 16) bytes, or 16 rows x (1024 + 16)
static_assert(4 * G3_EPI_BYTES <= 2 * G3_SLOT_BYTES + 1024, "the epilogue areas must end below the block metadata");
template <int DT>
__device__ __forceinline__ void gemm3_store_rows(const float16v (&acc)[16], uint32_t lds_wave, void *Y, uint32_t ldy,
                                                 uint32_t t0, uint32_t tokens, uint32_t o_tile, uint32_t out, uint32_t lane)
{
    constexpr uint32_t ES = DT == SKL_F32 ? 4 : 2;
    constexpr uint32_t ROWB = 256 * ES + 16;                    // padded: the two token groups of a store land on other banks
    constexpr int GROUPS = DT == SKL_F32 ? 2 : 1;               // row groups per 32-row block
    constexpr uint32_t ROWS = 32 / GROUPS, CH = 256 * ES / 16;  // rows per group, 16-byte pieces per row
    const uint32_t n = lane & 31, q = lane >> 5;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int gr = 0; gr < GROUPS; ++gr) {
#pragma unroll
            for (int cb = 0; cb < 8; ++cb)
#pragma unroll
                for (int ii = 0; ii < 16 / GROUPS; ++ii) {
                    const int i = gr * (16 / GROUPS) + ii;
                    const uint32_t row = (ii >> 2) * 8 + q * 4 + (ii & 3);
                    const uint32_t addr = lds_wave + row * ROWB + (cb * 32 + n) * ES;
                    const float v = acc_elem(acc[rb * 8 + cb][i]);
                    if (DT == SKL_F32) *(__attribute__((address_space(3))) float *)(uintptr_t)addr = v;
                    else *(__attribute__((address_space(3))) uint16_t *)(uintptr_t)addr =
                        DT == SKL_F16 ? float_to_half_bits(v) : float_to_bf16_bits(v);
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (uint32_t it = 0; it < ROWS * CH / 64; ++it) {
                const uint32_t idx = it * 64 + lane, row = idx / CH, c = idx % CH;
                const uint4 w = lds_word_at(lds_wave + row * ROWB + c * 16);
                const uint32_t t = t0 + rb * 32 + gr * ROWS + row, o = o_tile + c * (16 / ES);
                if (t < tokens && o < out) {
                    char *dst = static_cast<char *>(Y) + ((size_t)t * ldy + o) * ES;
                    if (o + 16 / ES <= out) {
                        *reinterpret_cast<uint4 *>(dst) = w;
                    } else {                                    // ragged last piece of the layer
                        const uint32_t e[4] = {w.x, w.y, w.z, w.w};
                        for (uint32_t b = 0; b < (out - o) * ES; b += 2)
                            *reinterpret_cast<uint16_t *>(dst + b) = (uint16_t)(e[b >> 2] >> ((b & 2) * 8));
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
}

template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_row_gemm3(Gemm2Args p)
{
    const uint32_t xcd = blockIdx.x & 7, wg = blockIdx.x >> 3;
    G3Split sp;
    sp.T = p.T; sp.m_tiles = p.m_tiles; sp.nb = p.n_blocks; sp.gx = p.gx; sp.l_max = p.l_max; sp.p_cap = p.p_cap;
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
        const uint32_t t = xcd + 8 * k, tile_m = t % p.m_tiles, tile_n = t / p.m_tiles;
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
                                                     uint32_t ldy, uint32_t tokens, uint32_t out)
{
    const uint32_t xcd = blockIdx.x / sp.l_max, l = blockIdx.x % sp.l_max, ab = blockIdx.y;
    if (l >= sp.left(xcd)) return;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 31, q = lane >> 5;
    const uint32_t k = sp.rounds(xcd) * sp.gx + l, t = xcd + 8 * k, tile_m = t % sp.m_tiles, tile_n = t / sp.m_tiles;
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
    const uint32_t o = tile_n * GM3_NT + cb * 32 + n;
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
// Path 0: 2-D groups, one hash evaluation per weight and sketch row.
// A workgroup owns (group, chunk of the group's input rows, 256 outputs).
// ========================================================================
struct TileArgs {
    HashArgs h;
    const skl_group_meta *gmeta;
    const uint16_t *keys;
    uint32_t in, out, tj, to, n_ob, jc_rows, n_jc;
};

__device__ __forceinline__ void stage_keys(uint16_t *dst, const uint16_t *src, uint32_t n)
{
    for (uint32_t i = threadIdx.x; i < n; i += SKL_WG) dst[i] = src[i];
}

struct TileUnit {
    uint32_t g, jb, ob, jc, j_lo, j_hi, K, key_off;
};

__device__ __forceinline__ TileUnit tile_unit(const TileArgs &p, uint32_t unit)
{
    TileUnit u;
    u.g = unit / p.n_jc;
    u.jc = unit - u.g * p.n_jc;
    u.jb = u.g / p.n_ob;
    u.ob = u.g - u.jb * p.n_ob;
    u.j_lo = u.jc * p.jc_rows;
    u.j_hi = min(u.j_lo + p.jc_rows, p.tj);
    const skl_group_meta gm = p.gmeta[u.g];
    u.K = gm.K;
    u.key_off = gm.key_off;
    return u;
}

// running hash state of one lane: t_r for the current address, advanced by one
// input row (tile_out addresses) per step
template <int D>
struct TileHash {
    uint32_t t[D], step[D];
    __device__ __forceinline__ void init(const HashArgs &h, uint32_t a0, uint32_t to)
    {
#pragma unroll
        for (int r = 0; r < D; ++r) {
            t[r] = __umul24(h.A[r], a0) + h.C[r];
            step[r] = __umul24(h.A[r], to);
        }
    }
    __device__ __forceinline__ uint16_t query(const uint16_t *tab, uint32_t K, uint32_t Kq)
    {
        uint16_t m = 0;
#pragma unroll
        for (int r = 0; r < D; ++r) {
            const uint16_t k = tab[r * K + select_index(t[r], Kq)];
            m = k > m ? k : m;
            t[r] += step[r];
        }
        return m;
    }
};

__device__ __forceinline__ uint16_t key_to_half_bits(uint16_t k)
{
    return (uint16_t)((k >> 1) | ((~k & 1u) << 15));
}

template <int D>
__global__ __launch_bounds__(SKL_WG) void k_tile_reconstruct(TileArgs p, uint16_t *__restrict__ W_hat)
{
    uint16_t *tab = reinterpret_cast<uint16_t *>(smem);
    const TileUnit u = tile_unit(p, blockIdx.x);
    stage_keys(tab, p.keys + u.key_off, D * u.K);
    __syncthreads();
    const uint32_t ol = blockIdx.y * SKL_WG + threadIdx.x;
    if (ol >= p.to) return;
    TileHash<D> th;
    th.init(p.h, u.j_lo * p.to + ol, p.to);
    const uint32_t Kq = u.K << 8;
    for (uint32_t jl = u.j_lo; jl < u.j_hi; ++jl) {
        const uint16_t k = th.query(tab, u.K, Kq);
        W_hat[(size_t)(u.jb * p.tj + jl) * p.out + u.ob * p.to + ol] = key_to_half_bits(k);
    }
}

// decode GEMV for BT batch rows per pass (grid z walks the batch)
template <int D, int BT>
__global__ __launch_bounds__(SKL_WG) void k_tile_gemv(TileArgs p, const uint16_t *__restrict__ x, uint32_t ldx,
                                                      uint32_t batch, float *__restrict__ partial, uint32_t key_words)
{
    uint16_t *tab = reinterpret_cast<uint16_t *>(smem);
    float *xs = reinterpret_cast<float *>(smem + key_words);   // [BT][jc_rows]
    const TileUnit u = tile_unit(p, blockIdx.x);
    stage_keys(tab, p.keys + u.key_off, D * u.K);
    const uint32_t b0 = blockIdx.z * BT;
    const uint32_t rows = u.j_hi - u.j_lo;
    for (uint32_t i = threadIdx.x; i < BT * rows; i += SKL_WG) {
        const uint32_t b = i / rows, jr = i - b * rows;
        xs[b * p.jc_rows + jr] =
            b0 + b < batch ? half_bits_to_float(x[(size_t)(b0 + b) * ldx + u.jb * p.tj + u.j_lo + jr]) : 0.f;
    }
    __syncthreads();
    const uint32_t ol = blockIdx.y * SKL_WG + threadIdx.x;
    if (ol >= p.to) return;
    TileHash<D> th;
    th.init(p.h, u.j_lo * p.to + ol, p.to);
    const uint32_t Kq = u.K << 8;
    float acc[BT];
#pragma unroll
    for (int b = 0; b < BT; ++b) acc[b] = 0.f;
    for (uint32_t jr = 0; jr < rows; ++jr) {
        const float w = half_bits_to_float(key_to_half_bits(th.query(tab, u.K, Kq)));
#pragma unroll
        for (int b = 0; b < BT; ++b) acc[b] = fmaf(w, xs[b * p.jc_rows + jr], acc[b]);
    }
    const uint32_t unit = u.jb * p.n_jc + u.jc;   // partial-sum slot of this chunk
#pragma unroll
    for (int b = 0; b < BT; ++b)
        if (b0 + b < batch)
            partial[((size_t)unit * batch + b0 + b) * p.out + u.ob * p.to + ol] = acc[b];
}

// prefill GEMM on path 0: 64 tokens x 64 outputs per workgroup; per 16 input
// rows the weights are reconstructed once into LDS (transposed, binary16 with
// inverted sign) and fed to 32x32x16 MFMAs.
#define TG_T 64
#define TG_AS 24   // halfs per LDS row of the 16-wide operand tiles (16 + 8)

template <int D>
__global__ __launch_bounds__(SKL_WG) void k_tile_gemm(TileArgs p, const uint16_t *__restrict__ X, uint32_t x_dt,
                                                      uint32_t ldx, uint32_t tokens, void *__restrict__ Y, uint32_t y_dt,
                                                      uint32_t ldy, uint32_t key_words)
{
    uint16_t *tab = reinterpret_cast<uint16_t *>(smem);
    uint16_t *As = reinterpret_cast<uint16_t *>(smem + key_words);   // [64 tokens][TG_AS]
    uint16_t *Bs = As + TG_T * TG_AS;                                // [64 outputs][TG_AS]
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t wm = wave >> 1, wn = wave & 1;
    const uint32_t n = lane & 31, q = lane >> 5;
    const uint32_t n_oc = (p.to + TG_T - 1) / TG_T;       // 64-wide output chunks per group column
    const uint32_t ob = blockIdx.x / n_oc, oc = blockIdx.x - ob * n_oc;
    const uint32_t t0 = blockIdx.y * TG_T;
    const uint32_t ol_b = oc * TG_T + (threadIdx.x & 63);   // output (inside the group) this thread reconstructs
    const uint32_t jsub = threadIdx.x >> 6;                 // ... for input rows jsub*4 .. jsub*4+3 of each 16
    float16v acc = {0.f};
    const uint32_t n_jb = p.in / p.tj;
    for (uint32_t jb = 0; jb < n_jb; ++jb) {
        const skl_group_meta gm = p.gmeta[jb * p.n_ob + ob];
        __syncthreads();
        stage_keys(tab, p.keys + gm.key_off, D * gm.K);
        __syncthreads();
        const uint32_t Kq = gm.K << 8;
        for (uint32_t j0 = 0; j0 < p.tj; j0 += 16) {
            // reconstruct 16 x 64 weights: thread -> (output ol_b, rows j0 + jsub*4 .. +3)
            {
                TileHash<D> th;
                const uint32_t olc = min(ol_b, p.to - 1);
                th.init(p.h, (j0 + jsub * 4) * p.to + olc, p.to);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t jl = j0 + jsub * 4 + i;
                    uint16_t v = 0;
                    const uint16_t k = th.query(tab, gm.K, Kq);   // addresses past the group are never used below
                    if (jl < p.tj && ol_b < p.to) v = key_to_half_bits(k) ^ 0x8000u;
                    Bs[(threadIdx.x & 63) * TG_AS + jsub * 4 + i] = v;
                }
            }
            // activations: 64 tokens x 16 input rows, thread -> (token, 4 rows)
            {
                const uint32_t tr = threadIdx.x >> 2, js = (threadIdx.x & 3) * 4;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t jl = j0 + js + i;
                    uint16_t v = 0;
                    if (t0 + tr < tokens && jl < p.tj) v = load_neg_half(X, x_dt, (size_t)(t0 + tr) * ldx + jb * p.tj + jl);
                    As[tr * TG_AS + js + i] = v;
                }
            }
            __syncthreads();
            const uint4 a = *reinterpret_cast<const uint4 *>(As + (wm * 32 + n) * TG_AS + q * 8);
            const uint4 b = *reinterpret_cast<const uint4 *>(Bs + (wn * 32 + n) * TG_AS + q * 8);
            // both operands carry an inverted sign: the product is x * w
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8v, a), __builtin_bit_cast(half8v, b), acc, 0, 0, 0);
            __syncthreads();
        }
    }
    const uint32_t ol = oc * TG_T + wn * 32 + n;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t t = t0 + wm * 32 + (i >> 2) * 8 + q * 4 + (i & 3);
        if (t < tokens && ol < p.to) store_out(Y, y_dt, (size_t)t * ldy + ob * p.to + ol, acc[i]);
    }
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
// Low-bit states: codes -> order keys.  A layer with 8- or 4-bit states keeps
// only codes and one binary16 scale per (group, sketch row) resident; every
// call first expands them into the 16-bit tables its kernels read (the same
// layouts create() builds on the host for binary16 states).  The state a code
// stands for is q * scale / qmax rounded once to binary16: the product is
// exact in float32 (7 x 11 significant bits), the correctly rounded float32
// quotient is either exact or far from any binary16 rounding boundary (qmax is
// odd), so the second rounding never changes the result.
// ========================================================================
template <int BITS>
__device__ __forceinline__ int code_at(const uint8_t *codes, uint32_t i)
{
    if (BITS == 8) return static_cast<int8_t>(codes[i]);
    const uint32_t b = codes[i >> 1];
    return (int)(((i & 1) ? b >> 4 : b & 15u) ^ 8u) - 8;      // sign-extend the nibble
}

template <int BITS>
__device__ __forceinline__ uint16_t key_of_code(int q, uint16_t scale_bits)
{
    const float v = __fdiv_rn((float)q * half_bits_to_float(scale_bits), BITS == 8 ? 127.0f : 7.0f);
    const uint16_t h = float_to_half_bits(v);
    return (uint16_t)(((h & 0x7FFFu) << 1) | (1u - (h >> 15)));
}

// row sketches: grid (channel blocks, chunks of 256 words), one thread per 16-byte word: word (r, k, c) of a
// block holds the keys of channels 8c .. 8c + 7; writes the padded layout, the unpadded one, or both
template <int BITS>
__global__ __launch_bounds__(SKL_WG) void k_expand_rows(const skl_block_meta *__restrict__ bmeta, const uint32_t *__restrict__ chan,
                                                         const uint32_t *__restrict__ choff, const uint8_t *__restrict__ codes,
                                                         const uint16_t *__restrict__ scales, uint32_t d,
                                                         uint4 *__restrict__ padded, uint4 *__restrict__ unpadded)
{
    const skl_block_meta bm = bmeta[blockIdx.x];
    const uint32_t K = bm.K, nb = bm.nb;
    const uint32_t idx = blockIdx.y * SKL_WG + threadIdx.x;
    if (idx >= d * nb * K) return;
    const uint32_t k = idx % K, c = (idx / K) % nb, r = idx / (K * nb);         // k fastest: neighbouring lanes read neighbouring codes
    uint32_t ch[8], at[8], sc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) ch[i] = chan[bm.chan_off + 8 * c + i];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t cc = ch[i] != SKL_NO_CHANNEL ? ch[i] : 0;                // every lane issues the same loads; unused ones are dropped below
        at[i] = choff[cc] + r * K + k;
        sc[i] = scales[cc * d + r];
    }
    uint32_t key[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t kk = key_of_code<BITS>(code_at<BITS>(codes, at[i]), (uint16_t)sc[i]);
        key[i] = ch[i] != SKL_NO_CHANNEL ? kk : 1u;                              // a channel slot past the end: +0.0
    }
    const uint4 w = make_uint4(key[0] | key[1] << 16, key[2] | key[3] << 16, key[4] | key[5] << 16, key[6] | key[7] << 16);
    if (padded) padded[bm.table_off16 + (size_t)(r * K + k) * bm.rs + c] = w;
    if (unpadded) unpadded[bm.ptable_off16 + (size_t)(r * K + k) * nb + c] = w;
}

// 2-D groups: keys in the caller's state order; grid (groups)
template <int BITS>
__global__ __launch_bounds__(SKL_WG) void k_expand_groups(const skl_group_meta *__restrict__ gmeta, const uint8_t *__restrict__ codes,
                                                           const uint16_t *__restrict__ scales, uint32_t d, uint16_t *__restrict__ keys)
{
    const skl_group_meta gm = gmeta[blockIdx.x];
    for (uint32_t idx = threadIdx.x; idx < d * gm.K; idx += SKL_WG)
        keys[gm.key_off + idx] = key_of_code<BITS>(code_at<BITS>(codes, gm.key_off + idx), scales[blockIdx.x * d + idx / gm.K]);
}

// ========================================================================
// Sketch construction (Eq. 4).  One thread per weight: for every sketch row
// an atomic minimum on a 64-bit key (magnitude, address inside the group,
// sign) in the state's slot.  The smallest key is the weight of smallest
// magnitude and, among equals, of smallest address -- the one the sequential
// update stream keeps -- whatever the order in which threads arrive.
// ========================================================================
struct BuildArgs {
    HashArgs h;
    const uint16_t *W;
    const uint64_t *base;       // state offset of every group
    const uint32_t *width;
    unsigned long long *keys;
    uint32_t in, out, tj, to, n_ob, d;
};

__global__ __launch_bounds__(SKL_WG) void k_build_clear(unsigned long long *keys, uint64_t n)
{
    for (uint64_t i = (uint64_t)blockIdx.x * SKL_WG + threadIdx.x; i < n; i += (uint64_t)gridDim.x * SKL_WG) keys[i] = ~0ull;
}

// grid (ceil(out / 256), min(in, 65535)): a thread owns one output column and walks the input rows of its grid row
__global__ __launch_bounds__(SKL_WG) void k_build_scatter(BuildArgs p)
{
    const uint32_t o = blockIdx.x * SKL_WG + threadIdx.x;
    if (o >= p.out) return;
    for (uint32_t j = blockIdx.y; j < p.in; j += gridDim.y) {
        const uint32_t g = (j / p.tj) * p.n_ob + o / p.to;
        const uint32_t a = (j % p.tj) * p.to + o % p.to;
        const uint32_t K = p.width[g];
        const uint16_t w = p.W[(size_t)j * p.out + o];
        const unsigned long long key = ((unsigned long long)(w & 0x7FFFu) << 25) | ((unsigned long long)a << 1) | (w >> 15);
        unsigned long long *S = p.keys + p.base[g];
        for (uint32_t r = 0; r < p.d; ++r) {
            const uint32_t t = __umul24(p.h.A[r], a) + p.h.C[r];
            atomicMin(S + (size_t)r * K + select_index(t, K << 8), key);
        }
    }
}

// row sketches (one group per input channel) whose d x K keys fit in LDS: a workgroup owns one channel, takes
// the minima with LDS atomics and writes the states itself; grid (in), LDS d * K * 8 bytes
__global__ __launch_bounds__(SKL_WG) void k_build_rows(BuildArgs p, uint16_t *__restrict__ states)
{
    unsigned long long *S = reinterpret_cast<unsigned long long *>(smem);
    const uint32_t j = blockIdx.x, K = p.width[j], n = p.d * K;
    for (uint32_t i = threadIdx.x; i < n; i += SKL_WG) S[i] = ~0ull;
    __syncthreads();
    const uint16_t *row = p.W + (size_t)j * p.out;
    for (uint32_t o = threadIdx.x; o < p.out; o += SKL_WG) {
        const uint16_t w = row[o];
        const unsigned long long key = ((unsigned long long)(w & 0x7FFFu) << 25) | ((unsigned long long)o << 1) | (w >> 15);
        for (uint32_t r = 0; r < p.d; ++r) {
            const uint32_t t = __umul24(p.h.A[r], o) + p.h.C[r];
            atomicMin(S + r * K + select_index(t, K << 8), key);
        }
    }
    __syncthreads();
    uint16_t *dst = states + p.base[j];
    for (uint32_t i = threadIdx.x; i < n; i += SKL_WG) {
        const unsigned long long k = S[i];
        dst[i] = k == ~0ull ? (uint16_t)0 : (uint16_t)(((k & 1) << 15) | (k >> 25));
    }
}

__global__ __launch_bounds__(SKL_WG) void k_build_finish(const unsigned long long *keys, uint64_t n, uint16_t *states)
{
    for (uint64_t i = (uint64_t)blockIdx.x * SKL_WG + threadIdx.x; i < n; i += (uint64_t)gridDim.x * SKL_WG) {
        const unsigned long long k = keys[i];
        states[i] = k == ~0ull ? (uint16_t)0 : (uint16_t)(((k & 1) << 15) | (k >> 25));
    }
}

// ========================================================================
// Launchers
// ========================================================================
static skl_status_t check_launch(const char *what);

// the tables a call's kernels read: the resident ones, or for low-bit states their expansion in `area`
struct TableSrc {
    const uint4 *tables = nullptr, *ptables = nullptr;
    const uint16_t *keys = nullptr;
};

static uint64_t round256(uint64_t v) { return (v + 255) / 256 * 256; }

uint64_t skl_dequant_bytes(const skl_layer *L)
{
    if (!L->qbits) return 0;
    return L->path == 1 ? round256(L->table_bytes) + round256(L->ptable_bytes) : round256(L->table_bytes + 16);
}

static skl_status_t table_source(const skl_layer *L, void *area, bool want_padded, bool want_unpadded, hipStream_t stream,
                                 TableSrc *src)
{
    if (!L->qbits) {
        if (L->path == 1) {
            src->tables = reinterpret_cast<const uint4 *>(L->dev + L->off_tables);
            src->ptables = reinterpret_cast<const uint4 *>(L->dev + L->off_ptables);
        } else {
            src->keys = reinterpret_cast<const uint16_t *>(L->dev + L->off_keys);
        }
        return SKL_OK;
    }
    const uint8_t *codes = L->dev + L->off_codes;
    const uint16_t *scales = reinterpret_cast<const uint16_t *>(L->dev + L->off_scales);
    if (L->path == 1) {
        uint4 *padded = static_cast<uint4 *>(area);
        uint4 *unpadded = reinterpret_cast<uint4 *>(static_cast<char *>(area) + round256(L->table_bytes));
        src->tables = padded; src->ptables = unpadded;
        const skl_block_meta *bmeta = reinterpret_cast<const skl_block_meta *>(L->dev + L->off_bmeta);
        const uint32_t *chan = reinterpret_cast<const uint32_t *>(L->dev + L->off_chan);
        const uint32_t *choff = reinterpret_cast<const uint32_t *>(L->dev + L->off_choff);
        // max_ptable_bytes: the largest block's unpadded table, rounded up to KiB: 16-byte words per block
        const dim3 grid(L->n_blocks, (L->max_ptable_bytes / 16 + SKL_WG - 1) / SKL_WG);
        if (L->qbits == 8)
            hipLaunchKernelGGL(k_expand_rows<8>, grid, dim3(SKL_WG), 0, stream, bmeta, chan, choff, codes, scales,
                               L->d, want_padded ? padded : nullptr, want_unpadded ? unpadded : nullptr);
        else
            hipLaunchKernelGGL(k_expand_rows<4>, grid, dim3(SKL_WG), 0, stream, bmeta, chan, choff, codes, scales,
                               L->d, want_padded ? padded : nullptr, want_unpadded ? unpadded : nullptr);
    } else {
        uint16_t *keys = static_cast<uint16_t *>(area);
        src->keys = keys;
        const skl_group_meta *gmeta = reinterpret_cast<const skl_group_meta *>(L->dev + L->off_gmeta);
        if (L->qbits == 8)
            hipLaunchKernelGGL(k_expand_groups<8>, dim3(L->n_groups), dim3(SKL_WG), 0, stream, gmeta, codes, scales, L->d, keys);
        else
            hipLaunchKernelGGL(k_expand_groups<4>, dim3(L->n_groups), dim3(SKL_WG), 0, stream, gmeta, codes, scales, L->d, keys);
    }
    return check_launch("expansion of low-bit states");
}

static RowArgs make_row_args(const skl_layer *L, const TableSrc &src)
{
    RowArgs a;
    for (int r = 0; r < SKL_MAX_D; ++r) { a.h.A[r] = L->A[r]; a.h.C[r] = L->C[r]; }
    a.bmeta = reinterpret_cast<const skl_block_meta *>(L->dev + L->off_bmeta);
    a.chan = reinterpret_cast<const uint32_t *>(L->dev + L->off_chan);
    a.tables = src.tables;
    a.in = L->in; a.out = L->out; a.n_blocks = L->n_blocks; a.n_otiles = L->n_otiles; a.n_seg = L->n_seg;
    return a;
}

static TileArgs make_tile_args(const skl_layer *L, const TableSrc &src)
{
    TileArgs a;
    for (int r = 0; r < SKL_MAX_D; ++r) { a.h.A[r] = L->A[r]; a.h.C[r] = L->C[r]; }
    a.gmeta = reinterpret_cast<const skl_group_meta *>(L->dev + L->off_gmeta);
    a.keys = src.keys;
    a.in = L->in; a.out = L->out; a.tj = L->tj; a.to = L->to; a.n_ob = L->n_ob;
    a.jc_rows = L->jc_rows; a.n_jc = L->n_jc;
    return a;
}

static skl_status_t check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        skl_set_error("launch of %s failed: %s", what, hipGetErrorString(e));
        return SKL_ERR_HIP;
    }
    return SKL_OK;
}

// Kernels that need more than 64 KiB of dynamic LDS must be told so once.
template <typename K>
static skl_status_t allow_lds(K kernel, size_t bytes)
{
    if (bytes <= 65536) return SKL_OK;
    static std::mutex mu;
    static std::unordered_map<const void *, size_t> granted;
    const void *fn = reinterpret_cast<const void *>(kernel);
    std::lock_guard<std::mutex> lock(mu);
    auto it = granted.find(fn);
    if (it != granted.end() && it->second >= bytes) return SKL_OK;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) {
        skl_set_error("cannot reserve %zu bytes of LDS: %s", bytes, hipGetErrorString(e));
        return SKL_ERR_HIP;
    }
    granted[fn] = bytes;
    return SKL_OK;
}

#ifdef SKL_DEV_D4_ONLY
#define DISPATCH_D(d, CALL) { constexpr int D = 4; CALL; }
#else
#define DISPATCH_D(d, CALL)                                         \
    switch (d) {                                                    \
    case 1: { constexpr int D = 1; CALL; } break;                   \
    case 2: { constexpr int D = 2; CALL; } break;                   \
    case 3: { constexpr int D = 3; CALL; } break;                   \
    case 4: { constexpr int D = 4; CALL; } break;                   \
    case 5: { constexpr int D = 5; CALL; } break;                   \
    case 6: { constexpr int D = 6; CALL; } break;                   \
    case 7: { constexpr int D = 7; CALL; } break;                   \
    default: { constexpr int D = 8; CALL; } break;                  \
    }
#endif

static inline size_t tile_key_words(const skl_layer *L) { return ((size_t)L->d * L->max_K * 2 + 15) / 16; }

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

// split of the third prefill kernel for a call with this many tokens (256 CUs: 32 workgroups per XCD,
// fewer when an XCD's share of the work is under four blocks per workgroup)
static G3Split gemm3_split(const skl_layer *L, uint32_t tokens)
{
    G3Split sp;
    sp.m_tiles = (tokens + GM_MT - 1) / GM_MT;
    sp.T = sp.m_tiles * ((L->out + GM3_NT - 1) / GM3_NT);
    sp.nb = L->n_blocks;
    const uint64_t units0 = (uint64_t)((sp.T + 7) / 8) * sp.nb;
    sp.gx = (uint32_t)std::min<uint64_t>(32, std::max<uint64_t>(1, units0 / 4));
    sp.l_max = 0; sp.p_cap = 0;
    for (uint32_t x = 0; x < 8; ++x) {
        sp.l_max = std::max(sp.l_max, sp.left(x));
        for (uint32_t l = 0; l < sp.left(x); ++l) sp.p_cap = std::max(sp.p_cap, sp.parts(x, l));
    }
    return sp;
}

// every segment of the split, eight words each: xcd, workgroup, token tile, output tile, first block,
// end block, whole-tile flag, partial slot; returns the number of segments (writes at most cap of them)
uint64_t skl_gemm3_segments(uint32_t out, uint32_t n_blocks, uint32_t tokens, uint32_t *segs, uint64_t cap, uint32_t *shape)
{
    skl_layer L;
    L.out = out; L.n_blocks = n_blocks;
    const G3Split sp = gemm3_split(&L, tokens);
    if (shape) { shape[0] = sp.gx; shape[1] = sp.l_max; shape[2] = sp.p_cap; shape[3] = sp.T; }
    uint64_t n = 0;
    for (uint32_t x = 0; x < 8; ++x)
        for (uint32_t wg = 0; wg < sp.gx; ++wg) {
            uint32_t round = 0, u_next = sp.share_begin(x, wg);
            G3Split::Seg sg;
            while (sp.next(x, wg, round, u_next, sg)) {
                if (n < cap) {
                    const uint32_t t = x + 8 * sg.k;
                    uint32_t *o = segs + 8 * n;
                    o[0] = x; o[1] = wg; o[2] = t % sp.m_tiles; o[3] = t / sp.m_tiles; o[4] = sg.k0; o[5] = sg.k1;
                    o[6] = sg.whole; o[7] = (uint32_t)sg.part_slot;
                }
                ++n;
            }
        }
    return n;
}

static uint64_t gemm_pack_bytes(const skl_layer *L, uint32_t tokens)
{
    const uint64_t m_tiles = (tokens + GM_MT - 1) / GM_MT;
    // second and third kernel: 8 row blocks of 64 lanes x 16 bytes per (token tile, step);
    // first kernel: one tile of 256 rows x gemm_uw words per (token tile, unit)
    return L->gemm_v2 || L->gemm_v3 ? m_tiles * L->n_gsteps * 8192ull : m_tiles * L->n_gunits * GM_MT * L->gemm_uw * 16;
}

static uint64_t gemm_own_bytes(const skl_layer *L, uint32_t tokens)
{
    if (L->path != 1) return 0;
    uint64_t bytes = gemm_pack_bytes(L, tokens);
    if (L->gemm_v3) {
        const G3Split sp = gemm3_split(L, tokens);
        bytes += 8ull * sp.l_max * sp.p_cap * G3_SLOT_FLOATS * sizeof(float);      // partial tiles
    }
    return bytes;
}

uint64_t skl_gemm_workspace_bytes(const skl_layer *L, uint32_t tokens)
{
    const uint64_t own = gemm_own_bytes(L, tokens);
    return L->qbits ? round256(own) + skl_dequant_bytes(L) : own;
}

skl_status_t skl_launch_build(const skl_desc_t *d, uint64_t n_groups, const uint64_t *group_base, const uint16_t *W,
                              uint16_t *states, void *ws, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    char *area = static_cast<char *>(ws);
    BuildArgs a;
    for (int r = 0; r < SKL_MAX_D; ++r) { a.h.A[r] = r < (int)d->d ? d->hash_a[r] : 0; a.h.C[r] = r < (int)d->d ? d->hash_c[r] : 0; }
    a.W = W;
    a.keys = reinterpret_cast<unsigned long long *>(area);
    area += round256(d->n_states * 8);
    uint64_t *base_dev = reinterpret_cast<uint64_t *>(area);
    area += round256((n_groups + 1) * 8);
    uint32_t *width_dev = reinterpret_cast<uint32_t *>(area);
    a.base = base_dev; a.width = width_dev;
    a.in = d->in_features; a.out = d->out_features; a.tj = d->tile_in; a.to = d->tile_out;
    a.n_ob = d->out_features / d->tile_out; a.d = d->d;
    hipError_t e = hipMemcpyAsync(base_dev, group_base, (n_groups + 1) * 8, hipMemcpyHostToDevice, stream);
    if (e == hipSuccess) e = hipMemcpyAsync(width_dev, d->group_width, n_groups * 4, hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) {
        skl_set_error("copy of the group offsets failed: %s", hipGetErrorString(e));
        return SKL_ERR_HIP;
    }
    uint32_t max_K = 0;
    for (uint64_t g = 0; g < n_groups; ++g) max_K = std::max(max_K, d->group_width[g]);
    const size_t row_lds = (size_t)d->d * max_K * 8;
    skl_status_t st = SKL_OK;
    if (d->tile_in == 1 && d->tile_out == d->out_features && row_lds <= 64 * 1024) {
        hipLaunchKernelGGL(k_build_rows, dim3(a.in), dim3(SKL_WG), row_lds, stream, a, states);
    } else {
        const uint32_t sweep = (uint32_t)std::min<uint64_t>((d->n_states + SKL_WG - 1) / SKL_WG, 4096);
        hipLaunchKernelGGL(k_build_clear, dim3(sweep), dim3(SKL_WG), 0, stream, a.keys, d->n_states);
        hipLaunchKernelGGL(k_build_scatter, dim3((a.out + SKL_WG - 1) / SKL_WG, std::min(a.in, 65535u)), dim3(SKL_WG), 0, stream, a);
        hipLaunchKernelGGL(k_build_finish, dim3(sweep), dim3(SKL_WG), 0, stream, a.keys, d->n_states, states);
    }
    st = check_launch("sketch construction");
    if (st != SKL_OK) return st;
    e = hipStreamSynchronize(stream);          // the host arrays behind the two copies may go away now
    if (e != hipSuccess) {
        skl_set_error("sketch construction failed: %s", hipGetErrorString(e));
        return SKL_ERR_HIP;
    }
    return SKL_OK;
}

skl_status_t skl_launch_reconstruct(const skl_layer *L, uint16_t *W_hat, void *ws, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    TableSrc src;
    skl_status_t st = table_source(L, ws, true, false, stream, &src);
    if (st != SKL_OK) return st;
    if (L->path == 1) {
        const RowArgs a = make_row_args(L, src);
        const size_t lds = (size_t)L->max_table_bytes + 64 * sizeof(uint32_t);
        const dim3 grid(L->n_blocks, L->n_seg);
        DISPATCH_D(L->d, {
            st = allow_lds(k_row_reconstruct<D>, lds);
            if (st == SKL_OK) hipLaunchKernelGGL(k_row_reconstruct<D>, grid, dim3(SKL_WG), lds, stream, a, W_hat);
        });
    } else {
        const TileArgs a = make_tile_args(L, src);
        const size_t lds = tile_key_words(L) * 16;
        const dim3 grid(L->n_jb * L->n_ob * L->n_jc, (L->to + SKL_WG - 1) / SKL_WG);
        DISPATCH_D(L->d, {
            st = allow_lds(k_tile_reconstruct<D>, lds);
            if (st == SKL_OK) hipLaunchKernelGGL(k_tile_reconstruct<D>, grid, dim3(SKL_WG), lds, stream, a, W_hat);
        });
    }
    return st == SKL_OK ? check_launch("reconstruct") : st;
}

skl_status_t skl_launch_gemv(const skl_layer *L, const void *x_, uint32_t ldx, void *y, skl_dtype_t y_dt,
                             uint32_t ldy, uint32_t batch, void *ws, void *stream_, bool with_reduction)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const uint16_t *x = static_cast<const uint16_t *>(x_);
    float *partial = static_cast<float *>(ws);
    TableSrc src;
    skl_status_t st = table_source(L, static_cast<char *>(ws) + round256(gemv_partial_bytes(L, batch)),
                                   L->path == 1 && batch > 1, L->path == 1 && batch == 1, stream, &src);
    if (st != SKL_OK) return st;
    if (L->path == 1) {
        StreamArgs a;
        a.r = make_row_args(L, src);
        a.ginfo = reinterpret_cast<const skl_group_info *>(L->dev + L->off_ginfo);
        a.n_wunits = L->n_wunits; a.n_sseg = L->n_sseg; a.n_bg = L->n_bg; a.buf_words = L->max_table_bytes / 16;
        a.two_bufs = L->two_bufs;
        const dim3 grid(8 * ((L->n_bg + 7) / 8) * L->n_sseg);
        if (batch == 1) {
            // unpadded tables; buffers at fixed LDS addresses
            a.r.tables = src.ptables;
            a.buf_words = L->max_ptable_bytes / 16;
            a.two_bufs = L->two_pbufs;
            // one wavefront per 64-output unit of the longest segment (at least two for the start-up loads)
            const uint32_t g1_waves = std::max(2u, (L->n_wunits + L->n_sseg - 1) / L->n_sseg);
            const size_t lds = (L->two_pbufs ? 2 * (size_t)SKL_PBUF_DIST : (size_t)L->max_ptable_bytes) + SKL_G1_FIXED_LDS(L->d) +
                               (size_t)(L->max_group_chan + 64) * sizeof(uint16_t);
            if (g1_waves <= 12) {
                DISPATCH_D(L->d, {
                    st = allow_lds(k_row_gemv1<D, 12>, lds);
                    if (st == SKL_OK)
                        hipLaunchKernelGGL((k_row_gemv1<D, 12>), grid, dim3(64 * g1_waves), lds, stream, a, x, partial);
                })
            } else {
                DISPATCH_D(L->d, {
                    st = allow_lds(k_row_gemv1<D, 16>, lds);
                    if (st == SKL_OK)
                        hipLaunchKernelGGL((k_row_gemv1<D, 16>), grid, dim3(64 * g1_waves), lds, stream, a, x, partial);
                })
            }
        } else {
            // padded tables; 16 activation rows of xs_stride halfs, xs_stride / 8 odd (bank spread of the MFMA A reads)
            const uint32_t xs_stride = (L->max_group_chan / 8 | 1u) * 8;
            a.two_bufs = L->two_bufs;
            const uint32_t gn_waves = std::max(2u, (L->n_wunits + L->n_sseg - 1) / L->n_sseg);
            const size_t lds = (L->two_bufs ? 2 * (size_t)SKL_PBUF_DIST : (size_t)L->max_table_bytes) + SKL_GN_FIXED_LDS +
                               (size_t)16 * xs_stride * sizeof(uint16_t);
            DISPATCH_D(L->d, {
                st = allow_lds(k_row_gemvN<D>, lds);
                if (st == SKL_OK)
                    hipLaunchKernelGGL((k_row_gemvN<D>), grid, dim3(64 * gn_waves), lds, stream, a, x, ldx, batch, xs_stride, partial);
            })
        }
    } else {
        const TileArgs a = make_tile_args(L, src);
        const uint32_t kw = (uint32_t)tile_key_words(L);
        const uint32_t units = L->n_jb * L->n_ob * L->n_jc, noc = (L->to + SKL_WG - 1) / SKL_WG;
        if (batch == 1) {
            const size_t lds = (size_t)kw * 16 + (size_t)L->jc_rows * sizeof(float);
            DISPATCH_D(L->d, {
                st = allow_lds(k_tile_gemv<D, 1>, lds);
                if (st == SKL_OK)
                    hipLaunchKernelGGL((k_tile_gemv<D, 1>), dim3(units, noc, 1), dim3(SKL_WG), lds, stream, a, x, ldx,
                                       batch, partial, kw);
            });
        } else {
            const size_t lds = (size_t)kw * 16 + (size_t)4 * L->jc_rows * sizeof(float);
            DISPATCH_D(L->d, {
                st = allow_lds(k_tile_gemv<D, 4>, lds);
                if (st == SKL_OK)
                    hipLaunchKernelGGL((k_tile_gemv<D, 4>), dim3(units, noc, (batch + 3) / 4), dim3(SKL_WG), lds, stream,
                                       a, x, ldx, batch, partial, kw);
            });
        }
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
    return L->path == 1 && L->in == first->in && L->out == first->out && L->d == first->d;
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

skl_status_t skl_launch_gemv_group(const skl_layer *const *layers, uint32_t n, const void *x_, uint32_t ldx, void *const *ys,
                                   skl_dtype_t y_dt, uint32_t ldy, uint32_t batch, void *ws, void *stream_, bool gate_up)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const skl_layer *F = layers[0];
    for (uint32_t i = 0; i < n; ++i)
        if (!group_layer_ok(layers[i], F)) {
            skl_set_error("layer %u of the group is not a row-sketch layer of the first layer's shape", i);
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
        skl_status_t st0 = table_source(layers[i], area, !one, one, stream, &srcs[i]);
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
        const uint32_t xs_stride = (L->max_group_chan / 8 | 1u) * 8;
        m.xs_stride[i] = xs_stride;
        size_t need;
        if (one) {
            a.r.tables = src.ptables;
            a.buf_words = L->max_ptable_bytes / 16;
            a.two_bufs = L->two_pbufs;
            need = (L->two_pbufs ? 2 * (size_t)SKL_PBUF_DIST : (size_t)L->max_ptable_bytes) + SKL_G1_FIXED_LDS(L->d) +
                   (size_t)(L->max_group_chan + 64) * sizeof(uint16_t);
        } else {
            a.buf_words = L->max_table_bytes / 16;
            a.two_bufs = L->two_bufs;
            need = (L->two_bufs ? 2 * (size_t)SKL_PBUF_DIST : (size_t)L->max_table_bytes) + SKL_GN_FIXED_LDS +
                   (size_t)16 * xs_stride * sizeof(uint16_t);
        }
        gr.y[i] = ys[i < n ? i : 0];
        gr.n_units[i] = L->n_units;
        if (i >= n) continue;
        grid_x = std::max(grid_x, 8 * ((L->n_bg + 7) / 8) * L->n_sseg);
        waves = std::max(waves, (L->n_wunits + L->n_sseg - 1) / L->n_sseg);
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
    } else if (waves <= 12) {
        DISPATCH_D(F->d, {
            st = allow_lds(k_row_gemv1_group<D, 12>, lds);
            if (st == SKL_OK) hipLaunchKernelGGL((k_row_gemv1_group<D, 12>), grid, dim3(64 * waves), lds, stream, m, x, partial);
        })
    } else {
        DISPATCH_D(F->d, {
            st = allow_lds(k_row_gemv1_group<D, 16>, lds);
            if (st == SKL_OK) hipLaunchKernelGGL((k_row_gemv1_group<D, 16>), grid, dim3(64 * waves), lds, stream, m, x, partial);
        })
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

// activation re-ordering for the second and third prefill kernels: rows staged in LDS when four
// of them fit, else gathered from global memory
static skl_status_t launch_pack(const skl_layer *L, const uint16_t *X, skl_dtype_t x_dt, uint32_t ldx, uint32_t tokens,
                                const uint32_t *chan, const skl_gemm_step *steps, uint4 *Xp, hipStream_t stream)
{
    const uint32_t m_tiles = (tokens + GM_MT - 1) / GM_MT;
    const size_t row_bytes = ((size_t)L->in + 4) * 2;           // an even number of elements plus one dword of padding
    skl_status_t st = SKL_OK;
    if (4 * row_bytes <= 160 * 1024) {                          // up to 10 KiB rows: four workgroups per CU overlap their phases
        st = allow_lds(k_pack_activations3<4>, 4 * row_bytes);
        if (st != SKL_OK) return st;
        hipLaunchKernelGGL(k_pack_activations3<4>, dim3((tokens + 3) / 4), dim3(SKL_WG), 4 * row_bytes, stream, X, (uint32_t)x_dt,
                           ldx, tokens, L->in, chan, steps, L->n_gsteps, Xp);
    } else {
        hipLaunchKernelGGL(k_pack_activations2, dim3((L->n_gsteps + 3) / 4, 8 * m_tiles), dim3(SKL_WG), 0, stream, X,
                           (uint32_t)x_dt, ldx, tokens, chan, steps, L->n_gsteps, Xp);
    }
    return check_launch("activation packing");
}

skl_status_t skl_launch_gemm(const skl_layer *L, const void *X_, skl_dtype_t x_dt, uint32_t ldx, void *Y,
                             skl_dtype_t y_dt, uint32_t ldy, uint32_t tokens, void *ws, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const uint16_t *X = static_cast<const uint16_t *>(X_);
    const bool rebuilt_once = L->gemm_v3 || L->gemm_v2;      // the kernels that read the unpadded tables
    TableSrc src;
    skl_status_t st = table_source(L, static_cast<char *>(ws) + round256(gemm_own_bytes(L, tokens)),
                                   L->path == 1 && !rebuilt_once, L->path == 1 && rebuilt_once, stream, &src);
    if (st != SKL_OK) return st;
    if (L->path == 1) {
        uint16_t *Xp = static_cast<uint16_t *>(ws);
        const RowArgs a = make_row_args(L, src);
        const skl_gemm_unit *units = reinterpret_cast<const skl_gemm_unit *>(L->dev + L->off_gunits);
        const uint32_t m_tiles = (tokens + GM_MT - 1) / GM_MT;
        if (m_tiles > 8191) {
            skl_set_error("more than 8191 token tiles in one call");
            return SKL_ERR_UNSUPPORTED;
        }
        if (L->gemm_v3) {
            const skl_gemm_step *steps = reinterpret_cast<const skl_gemm_step *>(L->dev + L->off_gsteps);
            st = launch_pack(L, X, x_dt, ldx, tokens, a.chan, steps, static_cast<uint4 *>(ws), stream);
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
            hipLaunchKernelGGL(k_gemm3_fixup, dim3(8 * sp.l_max, 16), dim3(256), 0, stream, sp, g.parts, Y, (uint32_t)y_dt, ldy,
                               tokens, L->out);
            return check_launch("gemm fix-up");
        }
        if (L->gemm_v2) {
            const skl_gemm_step *steps = reinterpret_cast<const skl_gemm_step *>(L->dev + L->off_gsteps);
            st = launch_pack(L, X, x_dt, ldx, tokens, a.chan, steps, static_cast<uint4 *>(ws), stream);
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
    } else {
        const TileArgs a = make_tile_args(L, src);
        const uint32_t kw = (uint32_t)tile_key_words(L);
        const size_t lds = (size_t)kw * 16 + (size_t)2 * TG_T * TG_AS * sizeof(uint16_t);
        const uint32_t n_oc = (L->to + TG_T - 1) / TG_T;
        const dim3 grid(L->n_ob * n_oc, (tokens + TG_T - 1) / TG_T);
        DISPATCH_D(L->d, {
            st = allow_lds(k_tile_gemm<D>, lds);
            if (st == SKL_OK)
                hipLaunchKernelGGL(k_tile_gemm<D>, grid, dim3(SKL_WG), lds, stream, a, X, (uint32_t)x_dt, ldx, tokens, Y,
                                   (uint32_t)y_dt, ldy, kw);
        });
    }
    return st == SKL_OK ? check_launch("gemm") : st;
}
