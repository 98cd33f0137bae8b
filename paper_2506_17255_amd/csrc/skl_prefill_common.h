// Shared by the prefill kernels: tile shapes, the activation re-ordering
// pre-pass and the operand rebuild used by producers.
#pragma once
#include "skl_device.h"
#include "skl_split.h"

struct skl_gemm_step;
struct G3Split;
namespace SKL_NS {
// activation re-ordering for the second and third prefill kernels (skl_prefill.hip)
skl_status_t skl_launch_pack(const skl_layer *L, const uint16_t *X, skl_dtype_t x_dt, uint32_t ldx, uint32_t tokens,
                             const uint32_t *chan, const skl_gemm_step *steps, uint32_t n_steps, uint4 *Xp, hipStream_t stream);
// staged prefill (skl_prefill_staged.hip): workspace bytes of a call (activation words, partial tiles, weight words)
uint64_t skl_gemm_staged_bytes(const skl_layer *L, uint32_t tokens);
skl_status_t skl_launch_gemm_staged(const skl_layer *L, const TableSrc &src, const uint16_t *X, skl_dtype_t x_dt, uint32_t ldx,
                                    void *Y, skl_dtype_t y_dt, uint32_t ldy, uint32_t tokens, void *ws, hipStream_t stream);
// adds the partials of the leftover tiles in workgroup order and stores them (skl_prefill.hip)
skl_status_t skl_launch_gemm3_fixup(const G3Split &sp, const float *parts, void *Y, skl_dtype_t y_dt, uint32_t ldy,
                                    uint32_t tokens, uint32_t out, uint32_t tile0, hipStream_t stream);
}  // namespace SKL_NS

#define GM_NT 128            // outputs per workgroup
#define GM_THREADS 512       // four compute + four copy wavefronts

// Operand slot: word (cb, row = 2*step + k-group, n) at ((cb*8 + row)*34 + n);
// 34 instead of 32 words per row keeps the producers' scattered writes (eight
// rows, two neighbouring n per 16 lanes) on distinct banks.
#define G2_ROW 34u
#define G2_CB_WORDS (8u * G2_ROW)

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


// ---- 256 x 256 output tiles: shared by the fused and the staged prefill kernel ----
#define G3_CB_WORDS (8u * G2_ROW)
#define G3_SLOT_BYTES (8u * G3_CB_WORDS * 16u)

// One accumulator element, read where it is used.  Left to itself the compiler copies all 256
// elements out of the accumulation registers after the block loop and parks half of them in scratch memory.
__device__ __forceinline__ float acc_elem(float v)
{
    float r;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(v));
    return r;
}

// RB: 32-row blocks per wavefront (2: 64 tokens x 256 outputs; 1: the half-height tiles of the staged kernel)
template <int DT, int RB = 2>
__device__ __forceinline__ void gemm3_store(const float16v (&acc)[8 * RB], void *Y, uint32_t ldy, uint32_t t0, uint32_t tokens,
                                            uint32_t o0, uint32_t out, uint32_t q)
{
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) {
        const uint32_t o = o0 + cb * 32;
        if (o >= out) continue;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
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
template <int DT, int RB = 2>
__device__ __forceinline__ void gemm3_store_rows(const float16v (&acc)[8 * RB], uint32_t lds_wave, void *Y, uint32_t ldy,
                                                 uint32_t t0, uint32_t tokens, uint32_t o_tile, uint32_t out, uint32_t lane)
{
    constexpr uint32_t ES = DT == SKL_F32 ? 4 : 2;
    constexpr uint32_t ROWB = 256 * ES + 16;                    // padded: the two token groups of a store land on other banks
    constexpr int GROUPS = DT == SKL_F32 ? 2 : 1;               // row groups per 32-row block
    constexpr uint32_t ROWS = 32 / GROUPS, CH = 256 * ES / 16;  // rows per group, 16-byte pieces per row
    const uint32_t n = lane & 31, q = lane >> 5;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
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


