// Ceilings of the machine as this library's kernels can reach them, measured by four small kernels: the
// rooflines of the benchmark are stated against these as well as against the data-sheet figures.
//   0  vector ALU: independent chains of packed 16-bit maximum and packed multiply-add (the instruction
//      classes of the query and decode stages), no memory access;
//   1  LDS gathers: 16-byte reads at lane-dependent addresses without bank conflicts;
//   2  matrix cores: v_mfma_f32_32x32x16_f16 on registers only, one wavefront per SIMD;
//   3  HBM: a streaming read of the workspace (16-byte loads, every byte once);
//   4  matrix cores as in 2, with operands of random sign and mantissa bits that change from one MFMA to
//      the next: the switching activity of real data, at which the chip lowers its clock.
// Each kernel runs `iters` rounds of a fixed amount of work per lane (stated in skl_microbench_work) and
// leaves one value per lane in the workspace so that nothing is optimised away.
#include "skl_device.h"

#define MB_RESULT_BYTES (4u << 20)  // head of the workspace: one word per lane of the largest grid
#define MB_VALU_PER_ROUND 64u       // lane-instructions per round and lane
#define MB_LDS_PER_ROUND 16u        // 16-byte reads per round and lane
#define MB_MFMA_PER_ROUND 16u       // MFMAs per round and wavefront

__global__ __launch_bounds__(1024) void k_mb_valu(uint32_t iters, uint32_t *out)
{
    uint32_t a[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = threadIdx.x * 0x9E3779B1u + i;
    const uint32_t m = 0x00030005u;
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            uint32_t t[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) asm volatile("v_pk_max_u16 %0, %1, %2" : "=v"(t[i]) : "v"(a[i]), "v"(a[(i + 1) & 7]));
#pragma unroll
            for (int i = 0; i < 8; ++i) asm volatile("v_pk_mad_u16 %0, %1, %2, %3" : "=v"(a[i]) : "v"(t[i]), "v"(m), "v"(a[i]));
        }
    }
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) s ^= a[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// 64 KiB of LDS; lane l of a wavefront reads word (base + l) mod 4096: 64 consecutive 16-byte words, no conflicts
__global__ __launch_bounds__(1024) void k_mb_lds(uint32_t iters, uint32_t *out)
{
    for (uint32_t i = threadIdx.x; i < 4096; i += blockDim.x) smem[i] = make_uint4(i, i + 1, i + 2, i + 3);
    __syncthreads();
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void *)smem;
    uint32_t pos = threadIdx.x;
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < (int)MB_LDS_PER_ROUND; ++r) {
            const uint4 v = lds_word_at(lds0 + ((pos + 64u * r) & 4095u) * 16);
            acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
        }
        pos += 1024;
        asm volatile("" : "+v"(pos) : : "memory");      // the reads of a round are issued in that round
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_mb_mfma(uint32_t iters, uint32_t *out)
{
    float16v acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = (float16v){0.f};
    // ordinary binary16 operands (values between 0.25 and 1.5, varying with the lane)
    const uint32_t v = (threadIdx.x & 0xFFu) << 2;
    const uint4 a = make_uint4(0x3C003800u + v, 0x38003C00u ^ v, 0x3A003900u + v, 0x39003A00u ^ v);
    const uint4 b = make_uint4(0x34003600u + v, 0x38003400u ^ v, 0x36003800u + v, 0x35003500u ^ v);
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < (int)MB_MFMA_PER_ROUND; ++r)
            acc[r & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8v, a), __builtin_bit_cast(half8v, b), acc[r & 3], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) t += acc[i][0] + acc[i][7];
    out[blockIdx.x * blockDim.x + threadIdx.x] = __builtin_bit_cast(uint32_t, t);
}

// Kind 2 multiplies the same two operand words over and over.  Here every MFMA gets another pair out of
// eight words of random bits (binary16 values in +-[0.5, 1)), so that the operand buses and the multiplier
// arrays toggle as they do on real activations and weights.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_mb_mfma_random(uint32_t iters, uint32_t *out)
{
    float16v acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = (float16v){0.f};
    uint4 a[8], b[8];
    uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    auto bits = [&]() { h ^= h << 13; h ^= h >> 17; h ^= h << 5; return (h & 0x83FF83FFu) | 0x38003800u; };
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = make_uint4(bits(), bits(), bits(), bits());
        b[i] = make_uint4(bits(), bits(), bits(), bits());
    }
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < (int)MB_MFMA_PER_ROUND; ++r)
            acc[r & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8v, a[r & 7]),
                                                               __builtin_bit_cast(half8v, b[(r + 3) & 7]), acc[r & 3], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) t += acc[i][0] + acc[i][7];
    out[blockIdx.x * blockDim.x + threadIdx.x] = __builtin_bit_cast(uint32_t, t);
}

// grid-stride streaming read of n16 16-byte words
__global__ __launch_bounds__(256) void k_mb_stream(const u32x4v *__restrict__ src, uint64_t n16, uint32_t *out)
{
    u32x4v acc = {0, 0, 0, 0};
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (uint64_t)gridDim.x * blockDim.x) {
        const u32x4v v = __builtin_nontemporal_load(src + i);
        acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) out[0] = 1;      // practically never: keeps the loads alive
}

// work one launch of kernel `kind` does: lane-instructions, LDS bytes, flops or HBM bytes
uint64_t skl_microbench_work(uint32_t kind, uint32_t iters, uint64_t ws_bytes)
{
    switch (kind) {
    case 0: return (uint64_t)SKL_N_CU * 4 * 1024 * iters * MB_VALU_PER_ROUND;                  // 4 workgroups of 1024 lanes per CU
    case 1: return (uint64_t)SKL_N_CU * 2 * 1024 * iters * MB_LDS_PER_ROUND * 16;              // 2 workgroups (64 KiB of LDS each) per CU
    case 2:
    case 4: return (uint64_t)SKL_N_CU * 4 * iters * MB_MFMA_PER_ROUND * (2ull * 32 * 32 * 16); // one wavefront per SIMD
    default: return (ws_bytes - MB_RESULT_BYTES) / 16 * 16;
    }
}

skl_status_t skl_launch_microbench(uint32_t kind, uint32_t iters, void *ws, uint64_t ws_bytes, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (ws_bytes < MB_RESULT_BYTES + 16) {
        skl_set_error("workspace holds %llu bytes, at least %u needed", (unsigned long long)ws_bytes, MB_RESULT_BYTES + 16);
        return SKL_ERR_BUFFER_TOO_SMALL;
    }
    skl_status_t st = SKL_OK;
    switch (kind) {
    case 0:
        hipLaunchKernelGGL(k_mb_valu, dim3(SKL_N_CU * 4), dim3(1024), 0, stream, iters, static_cast<uint32_t *>(ws));
        break;
    case 1:
        st = allow_lds(k_mb_lds, 65536);
        if (st != SKL_OK) return st;
        hipLaunchKernelGGL(k_mb_lds, dim3(SKL_N_CU * 2), dim3(1024), 65536, stream, iters, static_cast<uint32_t *>(ws));
        break;
    case 2:
        hipLaunchKernelGGL(k_mb_mfma, dim3(SKL_N_CU), dim3(256), 0, stream, iters, static_cast<uint32_t *>(ws));
        break;
    case 4:
        hipLaunchKernelGGL(k_mb_mfma_random, dim3(SKL_N_CU), dim3(256), 0, stream, iters, static_cast<uint32_t *>(ws));
        break;
    default:
        hipLaunchKernelGGL(k_mb_stream, dim3(SKL_N_CU * 16), dim3(256), 0, stream,
                           reinterpret_cast<const u32x4v *>(static_cast<char *>(ws) + MB_RESULT_BYTES), (ws_bytes - MB_RESULT_BYTES) / 16,
                           static_cast<uint32_t *>(ws));
        break;
    }
    return check_launch("microbenchmark");
}

// ---- range asserts of the debug build: one thread evaluates `value < limit` and touches no memory, so
// that a test can watch a violation being counted -----------------------------------------------
#ifdef SKL_DEBUG_BOUNDS
__global__ void k_debug_selftest(uint32_t value, uint32_t limit)
{
    if (threadIdx.x == 0) skl_in_range(value, limit, SKL_DBG_SELFTEST);
}
#endif

skl_status_t skl_launch_debug_selftest(uint32_t value, uint32_t limit, void *stream_)
{
#ifdef SKL_DEBUG_BOUNDS
    hipLaunchKernelGGL(k_debug_selftest, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream_), value, limit);
    return check_launch("range-assert self-test");
#else
    (void)value; (void)limit; (void)stream_;
    skl_set_error("this build of the library carries no range asserts");
    return SKL_ERR_UNSUPPORTED;
#endif
}
