// Diagnostic reconstruction of W_hat over row sketches (Sec. 3.1 Eq. 5): the
// same tables, offsets and query as the fused kernels, written to memory.
#include "skl_device.h"

namespace SKL_NS {


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
                if (ch != SKL_NO_CHANNEL && skl_in_range(ch, p.in, SKL_DBG_CHANNEL))
                    W_hat[(size_t)ch * p.out + o] = (uint16_t)(v[i >> 1] >> ((i & 1) * 16));
            }
        }
    }
}

// grid (channel blocks from block0 on, output segments)
template <int D>
__global__ __launch_bounds__(SKL_WG) void k_row_reconstruct(RowArgs p, uint32_t block0, uint16_t *__restrict__ W_hat)
{
    if (!skl_in_range(block0 + blockIdx.x, p.n_blocks, SKL_DBG_BLOCK)) return;
    const skl_block_meta bm = p.bmeta[block0 + blockIdx.x];
    const uint32_t n16 = D * bm.K * bm.rs;
    copy_words_to_lds_async(smem, p.tables + bm.table_off16, n16, SKL_WG / 64);    // global -> LDS, no registers in between
    uint32_t *chs = reinterpret_cast<uint32_t *>(smem + n16);
    if (threadIdx.x < 8 * bm.nb) chs[threadIdx.x] = p.chan[bm.chan_off + threadIdx.x];
    wait_async_copies();
    __syncthreads();
    switch (bm.rs) {
    case 9: row_reconstruct_body<D, 9>(p, bm, smem, chs, W_hat); break;
    case 5: row_reconstruct_body<D, 5>(p, bm, smem, chs, W_hat); break;
    case 3: row_reconstruct_body<D, 3>(p, bm, smem, chs, W_hat); break;
    default: row_reconstruct_body<D, 1>(p, bm, smem, chs, W_hat); break;
    }
}


skl_status_t skl_launch_reconstruct(const skl_layer *L, uint16_t *W_hat, void *ws, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    TableSrc src;
    skl_status_t st = skl_table_source(L, ws, true, false, stream, &src);
    if (st != SKL_OK) return st;
    if (L->path == 1) {
        const RowArgs a = make_row_args(L, src);
        // The blocks are sorted by sketch width.  Those before the first large table are launched with the LDS
        // they need (three workgroups per CU for tables up to 49.5 KiB), the rest with room for the largest table.
        const uint32_t n_small = L->n_small_blocks;
        const size_t lds_small = (size_t)L->small_table_bytes + 64 * sizeof(uint32_t);
        const size_t lds = (size_t)L->max_table_bytes + 64 * sizeof(uint32_t);
        DISPATCH_D(L->d, {
            st = allow_lds(k_row_reconstruct<D>, lds);
            if (st == SKL_OK && n_small)
                hipLaunchKernelGGL(k_row_reconstruct<D>, dim3(n_small, L->n_seg), dim3(SKL_WG), lds_small, stream, a, 0u, W_hat);
            if (st == SKL_OK && n_small < L->n_blocks)
                hipLaunchKernelGGL(k_row_reconstruct<D>, dim3(L->n_blocks - n_small, L->n_seg), dim3(SKL_WG), lds, stream, a, n_small, W_hat);
        });
    } else {
        return skl_tile_launch_reconstruct(L, src, W_hat, stream);
    }
    return st == SKL_OK ? check_launch("reconstruct") : st;
}

}  // namespace SKL_NS
