// The kernel files are compiled once per query mode (Sec. 3.1 Eq. 5: Max by magnitude, or Max of the signed
// values), each into a namespace of its own.  The functions the host side calls are defined here and hand
// every call to the namespace of the layer's mode; sizes and plans do not depend on the mode.
#include <hip/hip_runtime.h>

#include "skl_internal.h"

#define SKL_DECLARE_MODE(NS)                                                                                                      \
    namespace NS {                                                                                                                \
    skl_status_t skl_launch_reconstruct(const skl_layer *L, uint16_t *W_hat, void *ws, void *stream);                            \
    skl_status_t skl_launch_reconstruct_naive(const skl_layer *L, uint16_t *W_hat, void *ws, void *stream);                      \
    uint64_t skl_reconstruct_workspace_bytes(const skl_layer *L);                                                                \
    skl_status_t skl_launch_gemv(const skl_layer *L, const void *x, uint32_t ldx, void *y, skl_dtype_t y_dt, uint32_t ldy,       \
                                 uint32_t batch, void *ws, void *stream, bool with_reduction);                                   \
    skl_status_t skl_launch_gemm(const skl_layer *L, const void *X, skl_dtype_t x_dt, uint32_t ldx, void *Y, skl_dtype_t y_dt,   \
                                 uint32_t ldy, uint32_t tokens, void *ws, void *stream);                                         \
    uint64_t skl_gemv_workspace_bytes(const skl_layer *L, uint32_t batch);                                                       \
    uint64_t skl_gemm_workspace_bytes(const skl_layer *L, uint32_t tokens);                                                      \
    uint64_t skl_gemv_group_workspace_bytes(const skl_layer *const *layers, uint32_t n, uint32_t batch);                         \
    skl_status_t skl_launch_gemv_group(const skl_layer *const *layers, uint32_t n, const void *x, uint32_t ldx,                  \
                                       void *const *ys, skl_dtype_t y_dt, uint32_t ldy, uint32_t batch, void *ws, void *stream,  \
                                       bool gate_up);                                                                            \
    }
SKL_DECLARE_MODE(skl_qm0)
SKL_DECLARE_MODE(skl_qm1)

skl_status_t skl_static_scratch(void **ptr);        // skl_decode.hip

#define BY_MODE(L, CALL) ((L)->query_mode ? skl_qm1::CALL : skl_qm0::CALL)

skl_status_t skl_launch_reconstruct(const skl_layer *L, uint16_t *W_hat, void *ws, void *stream)
{
    return BY_MODE(L, skl_launch_reconstruct(L, W_hat, ws, stream));
}

skl_status_t skl_launch_reconstruct_naive(const skl_layer *L, uint16_t *W_hat, void *ws, void *stream)
{
    return BY_MODE(L, skl_launch_reconstruct_naive(L, W_hat, ws, stream));
}

skl_status_t skl_launch_gemv(const skl_layer *L, const void *x, uint32_t ldx, void *y, skl_dtype_t y_dt, uint32_t ldy,
                             uint32_t batch, void *ws, void *stream, bool with_reduction)
{
    return BY_MODE(L, skl_launch_gemv(L, x, ldx, y, y_dt, ldy, batch, ws, stream, with_reduction));
}

skl_status_t skl_launch_gemv_static(const skl_layer *L, const void *x, uint32_t ldx, void *y, skl_dtype_t y_dt, uint32_t ldy,
                                    uint32_t batch, void *stream)
{
    void *ptr = nullptr;
    const skl_status_t st = skl_static_scratch(&ptr);
    if (st != SKL_OK) return st;
    return BY_MODE(L, skl_launch_gemv(L, x, ldx, y, y_dt, ldy, batch, ptr, stream, true));
}

skl_status_t skl_launch_gemm(const skl_layer *L, const void *X, skl_dtype_t x_dt, uint32_t ldx, void *Y, skl_dtype_t y_dt,
                             uint32_t ldy, uint32_t tokens, void *ws, void *stream)
{
    return BY_MODE(L, skl_launch_gemm(L, X, x_dt, ldx, Y, y_dt, ldy, tokens, ws, stream));
}

skl_status_t skl_launch_gemv_group(const skl_layer *const *layers, uint32_t n, const void *x, uint32_t ldx, void *const *ys,
                                   skl_dtype_t y_dt, uint32_t ldy, uint32_t batch, void *ws, void *stream, bool gate_up)
{
    for (uint32_t i = 1; i < n; ++i)
        if (layers[i]->query_mode != layers[0]->query_mode) {
            skl_set_error("layer %u of the group has another query mode than the first", i);
            return SKL_ERR_UNSUPPORTED;
        }
    return BY_MODE(layers[0], skl_launch_gemv_group(layers, n, x, ldx, ys, y_dt, ldy, batch, ws, stream, gate_up));
}

uint64_t skl_reconstruct_workspace_bytes(const skl_layer *L) { return skl_qm0::skl_reconstruct_workspace_bytes(L); }
uint64_t skl_gemv_workspace_bytes(const skl_layer *L, uint32_t batch) { return skl_qm0::skl_gemv_workspace_bytes(L, batch); }
uint64_t skl_gemm_workspace_bytes(const skl_layer *L, uint32_t tokens) { return skl_qm0::skl_gemm_workspace_bytes(L, tokens); }
uint64_t skl_gemv_group_workspace_bytes(const skl_layer *const *layers, uint32_t n, uint32_t batch)
{
    return skl_qm0::skl_gemv_group_workspace_bytes(layers, n, batch);
}
