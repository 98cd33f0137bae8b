// The hash-based decompression operator as a comparator (Sec. 3.3 calls it the original, hash-based
// operation; the decompression speed-up figure of Sec. 4 measures the matrix form against it): one select
// (Eq. 3) per weight and sketch row, every candidate state fetched from device memory where the layer's
// tables live, no staging in LDS, no sharing of hash values between the weights of an output -- deliberately
// none of what the fused kernels do.  It reconstructs the same W_hat (Eq. 5) and exists to be measured
// against sketch_linear_reconstruct and the fused calls.
#include "skl_device.h"

namespace SKL_NS {


struct NaiveRowArgs {
    HashArgs h;
    const skl_block_meta *bmeta;
    const uint32_t *chan;
    const uint16_t *keys;       // the padded block tables, addressed by 16-bit key
    uint32_t out, d;
};

// grid (channel blocks, ceil(out / 256)): a thread owns one output and walks the block's input channels
__global__ __launch_bounds__(SKL_WG) void k_naive_rows(NaiveRowArgs p, uint16_t *__restrict__ W_hat)
{
    const skl_block_meta bm = p.bmeta[blockIdx.x];
    const uint32_t o = blockIdx.y * SKL_WG + threadIdx.x;
    if (o >= p.out) return;
    const uint16_t *tab = p.keys + (size_t)bm.table_off16 * 8;
    for (uint32_t c8 = 0; c8 < 8 * bm.nb; ++c8) {
        const uint32_t ch = p.chan[bm.chan_off + c8];
        if (ch == SKL_NO_CHANNEL) continue;
        uint32_t best = 0;
        for (uint32_t r = 0; r < p.d; ++r) {
            const uint32_t t = __umul24(p.h.A[r], o) + p.h.C[r];                // the weight's address in its group is o
            const uint32_t k = select_index(t, bm.K << 8);
            const uint32_t key = tab[((size_t)(r * bm.K + k) * bm.rs + (c8 >> 3)) * 8 + (c8 & 7)];
            best = key > best ? key : best;
        }
        W_hat[(size_t)ch * p.out + o] = key_to_half_bits(best);
    }
}

struct NaiveTileArgs {
    HashArgs h;
    const skl_group_meta *gmeta;
    const uint16_t *keys;       // keys in the caller's state order
    uint32_t in, out, tj, to, n_ob, d;
};

// grid (ceil(out / 256), min(in, 65535)): one thread per weight of a row, rows strided over grid.y
__global__ __launch_bounds__(SKL_WG) void k_naive_tiles(NaiveTileArgs p, uint16_t *__restrict__ W_hat)
{
    const uint32_t o = blockIdx.x * SKL_WG + threadIdx.x;
    if (o >= p.out) return;
    for (uint32_t j = blockIdx.y; j < p.in; j += gridDim.y) {
        const skl_group_meta gm = p.gmeta[(j / p.tj) * p.n_ob + o / p.to];
        const uint32_t a = (j % p.tj) * p.to + o % p.to;
        uint32_t best = 0;
        for (uint32_t r = 0; r < p.d; ++r) {
            const uint32_t t = __umul24(p.h.A[r], a) + p.h.C[r];
            const uint32_t key = p.keys[(size_t)gm.key_off + (size_t)r * gm.K + select_index(t, gm.K << 8)];
            best = key > best ? key : best;
        }
        W_hat[(size_t)j * p.out + o] = key_to_half_bits(best);
    }
}

skl_status_t skl_launch_reconstruct_naive(const skl_layer *L, uint16_t *W_hat, void *ws, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    TableSrc src;
    skl_status_t st = skl_table_source(L, ws, true, false, stream, &src);
    if (st != SKL_OK) return st;
    if (L->path == 1) {
        NaiveRowArgs a;
        for (int r = 0; r < SKL_MAX_D; ++r) { a.h.A[r] = L->A[r]; a.h.C[r] = L->C[r]; }
        a.bmeta = reinterpret_cast<const skl_block_meta *>(L->dev + L->off_bmeta);
        a.chan = reinterpret_cast<const uint32_t *>(L->dev + L->off_chan);
        a.keys = reinterpret_cast<const uint16_t *>(src.tables);
        a.out = L->out; a.d = L->d;
        const uint32_t oc = (L->out + SKL_WG - 1) / SKL_WG;
        if (oc > 65535) {
            skl_set_error("more than %u outputs", 65535u * SKL_WG);
            return SKL_ERR_UNSUPPORTED;
        }
        hipLaunchKernelGGL(k_naive_rows, dim3(L->n_blocks, oc), dim3(SKL_WG), 0, stream, a, W_hat);
    } else {
        NaiveTileArgs a;
        for (int r = 0; r < SKL_MAX_D; ++r) { a.h.A[r] = L->A[r]; a.h.C[r] = L->C[r]; }
        a.gmeta = reinterpret_cast<const skl_group_meta *>(L->dev + L->off_gmeta);
        a.keys = src.keys;
        a.in = L->in; a.out = L->out; a.tj = L->tj; a.to = L->to; a.n_ob = L->n_ob; a.d = L->d;
        hipLaunchKernelGGL(k_naive_tiles, dim3((L->out + SKL_WG - 1) / SKL_WG, std::min(L->in, 65535u)), dim3(SKL_WG), 0, stream, a, W_hat);
    }
    return check_launch("hash-based reconstruction");
}

}  // namespace SKL_NS
