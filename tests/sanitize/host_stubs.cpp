// Stand-ins for the kernel launchers, so that the host side of the library (validation, planning, the
// prefill work split, the C ABI) can be built without any device code for the sanitizer run of the CPU test
// suite.  Every launcher reports SKL_ERR_HIP: no test of that suite reaches one.
#include "skl_internal.h"

static skl_status_t no_device(const char *what)
{
    skl_set_error("%s: this build has no device code (host-only sanitizer build)", what);
    return SKL_ERR_HIP;
}

skl_status_t skl_launch_reconstruct(const skl_layer *, uint16_t *, void *, void *) { return no_device("reconstruct"); }
skl_status_t skl_launch_reconstruct_naive(const skl_layer *, uint16_t *, void *, void *) { return no_device("reconstruct"); }
uint64_t skl_dequant_bytes(const skl_layer *) { return 0; }
uint64_t skl_reconstruct_workspace_bytes(const skl_layer *) { return 0; }
skl_status_t skl_launch_gemv(const skl_layer *, const void *, uint32_t, void *, skl_dtype_t, uint32_t, uint32_t, void *, void *, bool)
{
    return no_device("gemv");
}
skl_status_t skl_launch_gemm(const skl_layer *, const void *, skl_dtype_t, uint32_t, void *, skl_dtype_t, uint32_t, uint32_t, void *,
                             void *)
{
    return no_device("gemm");
}
uint64_t skl_gemv_workspace_bytes(const skl_layer *, uint32_t) { return 0; }
uint64_t skl_static_scratch_bytes() { return 0; }
skl_status_t skl_launch_gemv_static(const skl_layer *, const void *, uint32_t, void *, skl_dtype_t, uint32_t, uint32_t, void *)
{
    return no_device("gemv");
}
uint64_t skl_gemm_workspace_bytes(const skl_layer *, uint32_t) { return 0; }
uint64_t skl_gemv_group_workspace_bytes(const skl_layer *const *, uint32_t, uint32_t) { return 0; }
skl_status_t skl_launch_gemv_group(const skl_layer *const *, uint32_t, const void *, uint32_t, void *const *, skl_dtype_t, uint32_t,
                                   uint32_t, void *, void *, bool)
{
    return no_device("grouped gemv");
}
skl_status_t skl_launch_build(const skl_desc_t *, uint64_t, const uint64_t *, const uint16_t *, uint16_t *, void *, void *)
{
    return no_device("sketch construction");
}
uint64_t skl_microbench_work(uint32_t, uint32_t, uint64_t) { return 0; }
skl_status_t skl_launch_microbench(uint32_t, uint32_t, void *, uint64_t, void *) { return no_device("microbenchmark"); }
skl_status_t skl_launch_debug_selftest(uint32_t, uint32_t, void *) { return no_device("range-assert self-test"); }
