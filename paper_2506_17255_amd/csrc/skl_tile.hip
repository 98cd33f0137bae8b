// Per-weight path: 2-D groups, one hash evaluation (Sec. 3.1 Eq. 3) per
// weight and sketch row.
#include "skl_device.h"

namespace SKL_NS {


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

static inline size_t tile_key_words(const skl_layer *L) { return ((size_t)L->d * L->max_K * 2 + 15) / 16; }


skl_status_t skl_tile_launch_reconstruct(const skl_layer *L, const TableSrc &src, uint16_t *W_hat, hipStream_t stream)
{
    skl_status_t st = SKL_OK;
    const TileArgs a = make_tile_args(L, src);
    const size_t lds = tile_key_words(L) * 16;
    const dim3 grid(L->n_jb * L->n_ob * L->n_jc, (L->to + SKL_WG - 1) / SKL_WG);
    DISPATCH_D(L->d, {
        st = allow_lds(k_tile_reconstruct<D>, lds);
        if (st == SKL_OK) hipLaunchKernelGGL(k_tile_reconstruct<D>, grid, dim3(SKL_WG), lds, stream, a, W_hat);
    });
    return st == SKL_OK ? check_launch("reconstruct") : st;
}

// first kernel of the decode call: one partial sum per (group chunk, output); the caller adds the reduction
skl_status_t skl_tile_launch_gemv(const skl_layer *L, const TableSrc &src, const uint16_t *x, uint32_t ldx, uint32_t batch,
                                  float *partial, hipStream_t stream)
{
    skl_status_t st = SKL_OK;
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
    return st;
}

skl_status_t skl_tile_launch_gemm(const skl_layer *L, const TableSrc &src, const uint16_t *X, skl_dtype_t x_dt, uint32_t ldx,
                                  void *Y, skl_dtype_t y_dt, uint32_t ldy, uint32_t tokens, hipStream_t stream)
{
    skl_status_t st = SKL_OK;
    const TileArgs a = make_tile_args(L, src);
    const uint32_t kw = (uint32_t)tile_key_words(L);
    const size_t lds = (size_t)kw * 16 + (size_t)2 * TG_T * TG_AS * sizeof(uint16_t);
    const uint32_t n_oc = (L->to + TG_T - 1) / TG_T;
    const uint32_t n_tt = (tokens + TG_T - 1) / TG_T;
    if (n_tt > 65535) {
        skl_set_error("more than %u tokens in one call through the per-weight path", 65535u * TG_T);
        return SKL_ERR_UNSUPPORTED;
    }
    const dim3 grid(L->n_ob * n_oc, n_tt);
    DISPATCH_D(L->d, {
        st = allow_lds(k_tile_gemm<D>, lds);
        if (st == SKL_OK)
            hipLaunchKernelGGL(k_tile_gemm<D>, grid, dim3(SKL_WG), lds, stream, a, X, (uint32_t)x_dt, ldx, tokens, Y,
                               (uint32_t)y_dt, ldy, kw);
    });
    return st == SKL_OK ? check_launch("gemm") : st;
}

}  // namespace SKL_NS
