// Device-side helpers and host-side launch plumbing shared by the kernel
// files of the sketch-linear library (gfx950 only).
//
// Common ground of every kernel (Sec. 3.1 of the paper):
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
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>
#include <mutex>
#include <unordered_map>

#include "skl_internal.h"

// Query mode this translation unit is compiled for (Sec. 3.1 Eq. 5): 0 = Max by magnitude, 1 = Max of the
// signed values.  The kernel files are compiled once per mode, their kernels and launchers in a namespace
// of their own; skl_dispatch.cpp picks the namespace by the layer's mode.  The modes differ only in the
// order-key encoding (host side, at create) and in the decode below; the query is an unsigned 16-bit
// maximum in both.
//   mode 0   key = magnitude << 1 | (sign clear);        -w = rotate-right(key, 1) with the sign inverted
//   mode 1   key = w | 0x8000 for w >= +0, ~w for w < 0;  -w = key ^ (key >= 0x8000 ? 0 : 0x7FFF)
#ifndef SKL_QM
#define SKL_QM 0
#endif
#if SKL_QM == 0
#define SKL_NS skl_qm0
#else
#define SKL_NS skl_qm1
#endif

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));

extern __shared__ uint4 smem[];

// ---------------------------------------------------------- range asserts
// The debug build of the library (-DSKL_DEBUG_BOUNDS, libsketch_linear_debug.so) checks the index ranges the
// kernels rely on: select indices against the sketch width, LDS addresses of gathers and table copies
// against the CU's LDS, channel numbers against d_in, block numbers against the layer's blocks.  A violation
// never traps (a faulting kernel can take the machine down): it is counted in a device array of the
// translation unit, the first one is kept with its code, value, limit, workgroup and thread, and the access
// is redirected to a harmless place.  sketch_linear_debug_violations() adds the arrays of all translation
// units up.  In the normal build the checks compile to nothing.
#define SKL_DBG_SELECT 1u        // select index >= sketch width K
#define SKL_DBG_LDS_READ 2u      // 16-byte LDS read outside the CU's LDS or misaligned
#define SKL_DBG_LDS_COPY 3u      // table copy lands outside the CU's LDS
#define SKL_DBG_CHANNEL 4u       // input channel number >= d_in
#define SKL_DBG_BLOCK 5u         // channel block number >= blocks of the layer
#define SKL_DBG_OUTPUT 6u        // output index >= d_out
#define SKL_DBG_SELFTEST 7u      // sketch_linear_debug_selftest
#ifdef SKL_DEBUG_BOUNDS
namespace {
__device__ uint32_t skl_debug_rec[8];              // count, then the first violation: code, value, limit, workgroup, thread
skl_status_t skl_debug_read_this_unit(uint32_t rec[8])
{
    hipError_t e = hipMemcpyFromSymbol(rec, HIP_SYMBOL(skl_debug_rec), 8 * sizeof(uint32_t));
    if (e != hipSuccess) {
        skl_set_error("reading the range-assert record: %s", hipGetErrorString(e));
        return SKL_ERR_HIP;
    }
    return SKL_OK;
}
struct SklDebugRegistrar { SklDebugRegistrar() { skl_debug_register(&skl_debug_read_this_unit); } } skl_debug_registrar;
}  // namespace
namespace {
__device__ __attribute__((noinline)) void skl_debug_record(uint32_t value, uint32_t limit, uint32_t code)
{
    if (atomicAdd(&skl_debug_rec[0], 1u) == 0) {
        skl_debug_rec[1] = code; skl_debug_rec[2] = value; skl_debug_rec[3] = limit;
        skl_debug_rec[4] = blockIdx.x; skl_debug_rec[5] = threadIdx.x;
    }
}
}  // namespace
__device__ __forceinline__ bool skl_in_range(uint32_t value, uint32_t limit, uint32_t code)
{
    if (__builtin_expect(value < limit, 1)) return true;
    skl_debug_record(value, limit, code);       // out of line: the checks sit at every gather of unrolled loops
    return false;
}
#else
__device__ __forceinline__ bool skl_in_range(uint32_t, uint32_t, uint32_t) { return true; }
#endif

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

typedef short short2v __attribute__((ext_vector_type(2)));

// two keys -> two binary16 values with inverted sign bits
__device__ __forceinline__ uint32_t keys_to_neg_half2(uint32_t k)
{
#if SKL_QM == 0
    return ((k >> 1) & 0x7FFF7FFFu) | ((k << 15) & 0x80008000u);
#else
    const uint32_t top = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2v, k) >> 15);    // 0xFFFF per half with the top bit set
    return k ^ (~top & 0x7FFF7FFFu);
#endif
}

// The same in two instructions instead of three (mode 0), for loops bound by the vector
// ALU: per 16-bit half, (k >> 1) + k * 0x8000 (the product keeps bit 0 of k in
// bit 15; the two terms share no bit).  The compiler turns the multiply back
// into a shift and an OR, hence the explicit packed multiply-add.
__device__ __forceinline__ uint32_t keys_to_neg_half2_mad(uint32_t k)
{
#if SKL_QM == 0
    uint32_t t, r;
    asm("v_pk_lshrrev_b16 %0, 1, %1 op_sel_hi:[0,1]" : "=v"(t) : "v"(k));
    asm("v_pk_mad_u16 %0, %1, %2, %3" : "=v"(r) : "v"(k), "s"(0x80008000u), "v"(t));
    return r;
#else
    return keys_to_neg_half2(k);
#endif
}

__device__ __forceinline__ uint4 keys_to_neg_half8(uint4 k)
{
    return make_uint4(keys_to_neg_half2(k.x), keys_to_neg_half2(k.y), keys_to_neg_half2(k.z), keys_to_neg_half2(k.w));
}

// one key -> the binary16 pattern it stands for
__device__ __forceinline__ uint16_t key_to_half_bits(uint32_t k)
{
#if SKL_QM == 0
    return (uint16_t)((k >> 1) | ((~k & 1u) << 15));
#else
    return (uint16_t)(k & 0x8000u ? k & 0x7FFFu : ~k);
#endif
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

// One global_load_lds_dwordx4: every active lane moves 16 bytes from gbase + lane_bytes to LDS byte address
// lds_addr + 16 * lane.  gbase and lds_addr are the same for the whole wavefront and sit in scalar registers
// (the saddr form of the instruction: scalar base plus the lane's own 32-bit byte offset).  Written as inline
// assembly on purpose: the compiler then does not know that LDS is being written behind its back and does
// not force the copy to complete before the next LDS read; completion is awaited explicitly
// (wait_async_copies) before a barrier publishes the data.
__device__ __forceinline__ void lds_dma_16_uniform(const void *gbase, uint32_t lane_bytes, uint32_t lds_addr)
{
    if (!skl_in_range(lds_addr, SKL_LDS_HARD_BYTES - 1023u, SKL_DBG_LDS_COPY)) return;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_bytes), "s"(gbase), "s"(lds_addr) : "memory", "m0");
}

// A source padded to whole 64-word chunks (no bounds check per lane), copied
// by a workgroup of nw wavefronts: wavefront w moves chunks w, w + nw, ..
// Everything but the lane's offset inside a chunk is the same for the whole wavefront and is kept in scalar
// registers, so that a chunk costs a handful of scalar instructions and the copy instruction (with the
// addresses formed per lane a chunk took 18 instructions, 8 of them vector, and the six chunks a wavefront
// issues per block were a sixth of a block's time).
__device__ __forceinline__ void copy_chunks_to_lds_async(uint4 *dst, const uint4 *src, uint32_t n16, uint32_t nw)
{
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const uint32_t n_chunks = __builtin_amdgcn_readfirstlane((n16 + 63) >> 6);
    const uint32_t step = __builtin_amdgcn_readfirstlane(nw);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void *)dst);
    const uint64_t s = reinterpret_cast<uint64_t>(src);
    // (the builtin returns a signed int: without the casts the low word would be sign-extended over the high one)
    const uint32_t s_lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)s), s_hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(s >> 32));
    const uint64_t base = (uint64_t)s_hi << 32 | (uint64_t)s_lo;
    for (uint32_t ch = wave; ch < n_chunks; ch += step)
        lds_dma_16_uniform(reinterpret_cast<const char *>(base + (uint64_t)ch * 1024), lane * 16, lds0 + ch * 1024);
}

// The same for a source of any length (the padded tables end inside a chunk): the lanes past the end sit out.
__device__ __forceinline__ void copy_words_to_lds_async(uint4 *dst, const uint4 *src, uint32_t n16, uint32_t nw)
{
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const uint32_t n = __builtin_amdgcn_readfirstlane(n16), step = __builtin_amdgcn_readfirstlane(nw);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void *)dst);
    const uint64_t s = reinterpret_cast<uint64_t>(src);
    const uint32_t s_lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)s), s_hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(s >> 32));
    const uint64_t base = (uint64_t)s_hi << 32 | (uint64_t)s_lo;
    for (uint32_t ch = wave; ch * 64 < n; ch += step)
        if (ch * 64 + lane < n)
            lds_dma_16_uniform(reinterpret_cast<const char *>(base + (uint64_t)ch * 1024), lane * 16, lds0 + ch * 1024);
}

__device__ __forceinline__ void wait_async_copies()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), other counters untouched
}

// Eq. 3: index inside a sketch row of width K; Kq = K << 8 (< 2^24).  Only the
// low 24 bits of t count, so t may be kept as a wrapping 32-bit number.
__device__ __forceinline__ uint32_t select_index(uint32_t t, uint32_t Kq)
{
    const uint32_t k = (uint32_t)(((uint64_t)(t & 0xFFFFFFu) * (uint64_t)(Kq & 0xFFFFFFu)) >> 32);
    return skl_in_range(k, Kq >> 8, SKL_DBG_SELECT) ? k : 0u;
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

// 16 bytes at an absolute LDS address
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 lds_word_at(uint32_t addr)
{
    if (!skl_in_range(addr | (addr & 15u ? 0xFFFFFFFFu : 0u), SKL_LDS_HARD_BYTES - 15u, SKL_DBG_LDS_READ)) addr = 0;
    const u32x4v v = *(const __attribute__((address_space(3))) u32x4v *)(uintptr_t)addr;
    return make_uint4(v.x, v.y, v.z, v.w);
}

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


// ========================================================================
// Host side: what every launcher needs
// ========================================================================
// the tables a call's kernels read: the resident ones, or for low-bit states their expansion in `area`
struct TableSrc {
    const uint4 *tables = nullptr, *ptables = nullptr;
    const uint16_t *keys = nullptr;
};

static inline uint64_t round256(uint64_t v) { return (v + 255) / 256 * 256; }


// the tables a call's kernels read (low-bit states: expanded into `area` first); skl_lowbit.hip
skl_status_t skl_table_source(const skl_layer *L, void *area, bool want_padded, bool want_unpadded, hipStream_t stream,
                              TableSrc *src);

// launchers of the per-weight path (skl_tile.hip)
namespace SKL_NS {
skl_status_t skl_tile_launch_reconstruct(const skl_layer *L, const TableSrc &src, uint16_t *W_hat, hipStream_t stream);
skl_status_t skl_tile_launch_gemv(const skl_layer *L, const TableSrc &src, const uint16_t *x, uint32_t ldx, uint32_t batch,
                                  float *partial, hipStream_t stream);
skl_status_t skl_tile_launch_gemm(const skl_layer *L, const TableSrc &src, const uint16_t *X, skl_dtype_t x_dt, uint32_t ldx,
                                  void *Y, skl_dtype_t y_dt, uint32_t ldy, uint32_t tokens, hipStream_t stream);
}  // namespace SKL_NS

static inline skl_status_t check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        skl_set_error("launch of %s failed: %s", what, hipGetErrorString(e));
        return SKL_ERR_HIP;
    }
    return SKL_OK;
}

static inline RowArgs make_row_args(const skl_layer *L, const TableSrc &src)
{
    RowArgs a;
    for (int r = 0; r < SKL_MAX_D; ++r) { a.h.A[r] = L->A[r]; a.h.C[r] = L->C[r]; }
    a.bmeta = reinterpret_cast<const skl_block_meta *>(L->dev + L->off_bmeta);
    a.chan = reinterpret_cast<const uint32_t *>(L->dev + L->off_chan);
    a.tables = src.tables;
    a.in = L->in; a.out = L->out; a.n_blocks = L->n_blocks; a.n_otiles = L->n_otiles; a.n_seg = L->n_seg;
    return a;
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
