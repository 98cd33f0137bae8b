#include "skl_device.h"

// ========================================================================
// Low-bit states: codes -> order keys.  A layer with 8- or 4-bit states keeps
// only codes and one binary16 scale per (group, sketch row) resident; every
// call first expands them into the 16-bit tables its kernels read (the same
// layouts create() builds on the host for binary16 states).  The state a code
// stands for is q * scale / qmax rounded once to binary16.  It is computed in
// float32 as |q| * (scale * (1 / qmax)): three roundings, 1.5 * 2^-23 relative
// in all.  The exact quotient m / qmax (m an integer of at most 18 bits) is
// never closer to a binary16 rounding boundary than 1 / (2 qmax) of a binary16
// spacing -- 2^-19 relative for qmax = 127, 2^-15 for qmax = 7 -- so rounding
// the approximation to binary16 gives the correctly rounded state.
// ========================================================================
template <int BITS>
__device__ __forceinline__ int code_at(const uint8_t *codes, uint32_t i)
{
    if (BITS == 8) return static_cast<int8_t>(codes[i]);
    const uint32_t b = codes[i >> 1];
    return (int)(((i & 1) ? b >> 4 : b & 15u) ^ 8u) - 8;      // sign-extend the nibble
}

// mode: the layer's query mode (the order-key encoding of skl_key_of_half)
// step: scale / qmax in float32 (one rounding more than the exact product followed by one multiplication:
// 2^-23 relative in all, still far inside the quotient's distance from every binary16 rounding boundary)
__device__ __forceinline__ uint16_t key_of_code_step(int q, float step, uint32_t mode)
{
    // magnitude and sign apart: the sign of a zero state (negative code, zero scale) must survive, and a
    // multiply fused with the conversion (fma with a +0 addend) would lose it
    const float mag = (float)(q < 0 ? -q : q) * step;
    const uint16_t h = (uint16_t)(float_to_half_bits(mag) | (q < 0 ? 0x8000u : 0u));
    if (mode == 0) return (uint16_t)(((h & 0x7FFFu) << 1) | (1u - (h >> 15)));
    return (uint16_t)(h & 0x8000u ? ~h : h | 0x8000u);
}

template <int BITS>
__device__ __forceinline__ uint16_t key_of_code(int q, uint16_t scale_bits, uint32_t mode)
{
    return key_of_code_step(q, half_bits_to_float(scale_bits) * (BITS == 8 ? 1.0f / 127.0f : 1.0f / 7.0f), mode);
}

// Row sketches.  create() keeps the codes in the order of the block tables: word (r, k, c) of a block holds
// the eight codes of channels 8c .. 8c + 7 for state (r, k) -- 4 bytes (nibble i = channel 8c + i) or
// 8 bytes per word, at the word's index in the unpadded table -- and the scales as one 16-byte word of
// eight binary16 values per (r, c) of a block.  One thread per word of the unpadded tables, whole layer in
// one flat grid: the block of a thread's 64-word chunk comes from a map create() wrote (the same for the
// whole wavefront), then one load of codes, one (cached) load of scales, eight conversions, one or two
// 16-byte stores.  The padding words at the end of a block's last chunk are left alone: no kernel reads them.
template <int BITS>
__global__ __launch_bounds__(SKL_WG) void k_expand_rows(const skl_block_meta *__restrict__ bmeta, const uint32_t *__restrict__ chunk_block,
                                                         const uint8_t *__restrict__ tcodes, const uint4 *__restrict__ tscales,
                                                         uint32_t n_words, uint32_t d, uint32_t mode,
                                                         uint4 *__restrict__ padded, uint4 *__restrict__ unpadded)
{
    const uint32_t gid = blockIdx.x * SKL_WG + threadIdx.x;     // word of the unpadded tables
    if (gid >= n_words) return;
    const uint32_t blk = __builtin_amdgcn_readfirstlane(chunk_block[gid >> 6]);
    const skl_block_meta bm = bmeta[blk];
    const uint32_t K = bm.K, nb = bm.nb;
    const uint32_t idx = gid - bm.ptable_off16;                 // (r * K + k) * nb + c
    if (idx >= d * nb * K) return;
    const uint32_t c = idx & (nb - 1), rk = idx >> (31 - __builtin_clz(nb));    // nb is 1, 2, 4 or 8
    uint32_t r = 0;
    for (uint32_t i = 1; i < d; ++i) r += rk >= i * K;
    uint64_t packed;
    if (BITS == 8) packed = reinterpret_cast<const uint64_t *>(tcodes)[gid];
    else packed = reinterpret_cast<const uint32_t *>(tcodes)[gid];
    const uint4 sw = tscales[bm.scale_off16 + r * nb + c];
    const uint32_t sc[4] = {sw.x, sw.y, sw.z, sw.w};
    uint32_t key[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int q = BITS == 8 ? (int)(int8_t)(packed >> (8 * i)) : (int)(((uint32_t)(packed >> (4 * i)) & 15u) ^ 8u) - 8;
        key[i] = key_of_code<BITS>(q, (uint16_t)(sc[i >> 1] >> ((i & 1) * 16)), mode);     // a slot without a channel has code 0: +0.0
    }
    const uint4 w = make_uint4(key[0] | key[1] << 16, key[2] | key[3] << 16, key[4] | key[5] << 16, key[6] | key[7] << 16);
    if (padded) padded[bm.table_off16 + (size_t)rk * bm.rs + c] = w;
    if (unpadded) unpadded[gid] = w;
}

// 2-D groups: keys in the caller's state order; grid (groups)
template <int BITS>
__global__ __launch_bounds__(SKL_WG) void k_expand_groups(const skl_group_meta *__restrict__ gmeta, const uint8_t *__restrict__ codes,
                                                           const uint16_t *__restrict__ scales, uint32_t d, uint32_t mode,
                                                           uint16_t *__restrict__ keys)
{
    const skl_group_meta gm = gmeta[blockIdx.x];
    for (uint32_t idx = threadIdx.x; idx < d * gm.K; idx += SKL_WG)
        keys[gm.key_off + idx] = key_of_code<BITS>(code_at<BITS>(codes, gm.key_off + idx), scales[blockIdx.x * d + idx / gm.K], mode);
}


uint64_t skl_dequant_bytes(const skl_layer *L)
{
    if (!L->qbits) return 0;
    return L->path == 1 ? round256(L->table_bytes) + round256(L->ptable_bytes) : round256(L->table_bytes + 16);
}

skl_status_t skl_table_source(const skl_layer *L, void *area, bool want_padded, bool want_unpadded, hipStream_t stream,
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
        const uint4 *tscales = reinterpret_cast<const uint4 *>(scales);
        const uint32_t *chunk_block = reinterpret_cast<const uint32_t *>(L->dev + L->off_chunk_block);
        const uint32_t n_words = (uint32_t)(L->ptable_bytes / 16);      // below 2^32: the planner checks the word offsets
        const dim3 grid((n_words + SKL_WG - 1) / SKL_WG);
        if (L->qbits == 8)
            hipLaunchKernelGGL(k_expand_rows<8>, grid, dim3(SKL_WG), 0, stream, bmeta, chunk_block, codes, tscales, n_words,
                               L->d, L->query_mode, want_padded ? padded : nullptr, want_unpadded ? unpadded : nullptr);
        else
            hipLaunchKernelGGL(k_expand_rows<4>, grid, dim3(SKL_WG), 0, stream, bmeta, chunk_block, codes, tscales, n_words,
                               L->d, L->query_mode, want_padded ? padded : nullptr, want_unpadded ? unpadded : nullptr);
    } else {
        uint16_t *keys = static_cast<uint16_t *>(area);
        src->keys = keys;
        const skl_group_meta *gmeta = reinterpret_cast<const skl_group_meta *>(L->dev + L->off_gmeta);
        if (L->qbits == 8)
            hipLaunchKernelGGL(k_expand_groups<8>, dim3(L->n_groups), dim3(SKL_WG), 0, stream, gmeta, codes, scales, L->d, L->query_mode, keys);
        else
            hipLaunchKernelGGL(k_expand_groups<4>, dim3(L->n_groups), dim3(SKL_WG), 0, stream, gmeta, codes, scales, L->d, L->query_mode, keys);
    }
    return check_launch("expansion of low-bit states");
}

