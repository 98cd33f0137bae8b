// Shared by the prefill kernels: tile shapes, the activation re-ordering
// pre-pass and the operand rebuild used by producers.
#pragma once
#include "skl_device.h"

struct skl_gemm_step;
// activation re-ordering for the second and third prefill kernels (skl_prefill.hip)
skl_status_t skl_launch_pack(const skl_layer *L, const uint16_t *X, skl_dtype_t x_dt, uint32_t ldx, uint32_t tokens,
                             const uint32_t *chan, const skl_gemm_step *steps, uint4 *Xp, hipStream_t stream);
// first and second prefill kernel (skl_prefill_fallback.hip)
skl_status_t skl_launch_gemm_fallback(const skl_layer *L, const TableSrc &src, const uint16_t *X, skl_dtype_t x_dt, uint32_t ldx,
                                      void *Y, skl_dtype_t y_dt, uint32_t ldy, uint32_t tokens, void *ws, hipStream_t stream);

#define GM_MT 256            // tokens per workgroup
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

