#include "skl_device.h"

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

