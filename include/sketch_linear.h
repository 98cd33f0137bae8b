/*
 * sketch_linear.h -- C ABI of the fused sketch-query linear layer for
 * AMD MI355X (gfx950).
 *
 * A layer's d_in x d_out weight matrix W exists only as a multi-row AbsMaxMin
 * sketch (UltraSketchLLM, arXiv 2506.17255).  Every call below that touches
 * weights reconstructs them on the fly,
 *
 *     W_hat[j][o] = Max_r  S_g[r][ H_r(Addr(j,o)) ]          (Sec. 3.1, Eq. 5)
 *
 * with the select function of Eq. 3 and per-group sketch widths (importance
 * aware allocation, Sec. 3.2; a width per group, Sec. 3.3), and multiplies
 * them into the activations, y = x W_hat
 * (Sec. 2.1, Eq. 1/2: W is d_in x d_out, activations multiply from the left).
 * W_hat is never written to device memory, except by the diagnostic call
 * sketch_linear_reconstruct().
 *
 * Conventions fixed by this library where the paper is silent:
 *   group     a tile of tile_in x tile_out weights; groups are numbered
 *             g = (j / tile_in) * (d_out / tile_out) + (o / tile_out).
 *   Addr      offset inside the group, a = (j % tile_in) * tile_out + (o % tile_out).
 *   H_r       t = (hash_a[r] * a + hash_c[r]) mod 2^24;  H_r(a) = floor(t * K_g / 2^24),
 *             K_g = group_width[g]; the same d pairs serve every group.
 *   Max       by magnitude; of two candidates with equal magnitude the one
 *             with the clear sign bit.
 *   states    IEEE binary16 bit patterns, group-major, then sketch row r,
 *             then index k:  states[base_g + r * K_g + k].
 *   low-bit   states may instead be given as 8- or 4-bit codes (the paper
 *   states    combines the sketch with 4-/8-bit scalar quantisation, Sec. 3.3
 *             last paragraph and Sec. 4, without fixing a format; this is the
 *             format fixed here): one binary16 scale per sketch row of a
 *             group, scales[g * d + r] >= 0, and signed codes q in
 *             [-qmax, qmax], qmax = 127 (8 bit) or 7 (4 bit), in the order of
 *             `states`.  The state a code stands for is q * scale / qmax
 *             rounded once to binary16 (nearest even).  Such a layer keeps
 *             only codes and scales resident in dev_buf; every call expands
 *             them into the kernels' 16-bit tables inside its workspace.
 *
 * General rules
 *   - Every function returns a status code and never throws, aborts or
 *     prints.  sketch_linear_last_error() returns a thread-local text for
 *     the last non-OK status of the calling thread.
 *   - Pointers are HOST pointers unless the parameter comment says DEVICE.
 *   - The library never allocates device memory: dev_buf, workspace,
 *     activations and outputs are caller-allocated, borrowed, and must stay
 *     valid until the work enqueued on them has completed (dev_buf: until
 *     sketch_linear_destroy).  Device pointers must be 16-byte aligned.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *     gemv / gemm / reconstruct only enqueue work and never synchronise;
 *     create synchronises the stream once so that the host arrays may be
 *     freed when it returns.
 *   - Calls that share a workspace must be ordered on one stream.
 *   - All arguments are validated before anything is enqueued.
 */
#ifndef SKETCH_LINEAR_H
#define SKETCH_LINEAR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SKL_API __attribute__((visibility("default")))

typedef enum {
    SKL_OK = 0,
    SKL_ERR_INVALID_ARG = 1,      /* NULL pointer, bad size, misaligned pointer, bad dtype */
    SKL_ERR_UNSUPPORTED = 2,      /* valid request outside what the kernels cover
                                     (e.g. a group table that does not fit in LDS) */
    SKL_ERR_BUFFER_TOO_SMALL = 3, /* dev_buf or workspace smaller than required */
    SKL_ERR_NONFINITE = 4,        /* a state is NaN or infinite */
    SKL_ERR_HIP = 5,              /* a HIP runtime call failed; see last_error */
    SKL_ERR_NO_MEMORY = 6         /* the host ran out of memory while planning or staging a layer */
} skl_status_t;

typedef enum { SKL_F16 = 0, SKL_BF16 = 1, SKL_F32 = 2 } skl_dtype_t;

/* Description of one sketched layer (all pointers HOST). */
typedef struct {
    uint32_t struct_size;      /* sizeof(skl_desc_t), for ABI checking */
    uint32_t in_features;      /* d_in  >= 1 */
    uint32_t out_features;     /* d_out >= 1 */
    uint32_t tile_in;          /* divides in_features  */
    uint32_t tile_out;         /* divides out_features; tile_in * tile_out <= 2^24 */
    uint32_t d;                /* sketch rows, 1..8 */
    uint32_t query_mode;       /* 0 = Max by magnitude as described above (default reading of Eq. 5);
                                  1 = Max of the signed values, Eq. 5 as printed (+0 wins over -0) */
    uint32_t flags;            /* bit 0: always hash per weight (path 0) even when the geometry
                                  allows the row-sketch path; bit 1: row sketches take the staged
                                  prefill (SKL_PREFILL_STAGED) at every token count; bit 2: they take
                                  the fused prefill whenever their tables allow (bits 1 and 2 exclude
                                  each other; without either the library chooses per call); other bits
                                  must be 0 */
    const uint32_t *hash_a;    /* [d], each < 2^24 */
    const uint32_t *hash_c;    /* [d], each < 2^24 */
    const uint32_t *group_width; /* [(in/tile_in) * (out/tile_out)], each 1..65535 */
    const uint16_t *states;    /* [n_states] binary16 bit patterns, layout above
                                  (NULL when state_bits is 8 or 4) */
    uint64_t n_states;         /* must equal d * sum(group_width) */
    /* -- end of the first version of this struct (72 bytes, still accepted: binary16 states) -- */
    uint32_t state_bits;       /* 0 or 16: binary16 `states`;  8 or 4: `codes` and `scales` */
    uint32_t reserved;         /* must be 0 */
    const void *codes;         /* state_bits 8: int8 [n_states];  4: two's-complement nibbles, state i in
                                  byte i / 2, low nibble for even i, [(n_states + 1) / 2] bytes; the codes
                                  -128 and -8 are invalid */
    const uint16_t *scales;    /* binary16, finite, sign bit clear, [n_groups * d] */
} skl_desc_t;

#define SKL_DESC_SIZE_V1 72u

typedef struct skl_layer skl_layer_t;   /* opaque host object */

/* What create() decided; for diagnostics, tests and benchmarks. */
typedef struct {
    uint32_t struct_size;
    uint32_t path;             /* 0 = per-weight hashing over 2-D groups;
                                  1 = row sketches (tile_in = 1, tile_out = d_out):
                                      index depends on the output channel only */
    uint32_t n_units;          /* channel blocks (path 1) or group chunks (path 0): the
                                  number of partial sums per output in the split reduction */
    uint32_t max_table_bytes;  /* largest LDS-resident table of one workgroup */
    uint64_t table_bytes;      /* bytes of sketch tables (or of codes and scales) resident in dev_buf */
    uint64_t n_weights;        /* in_features * out_features */
    uint64_t n_states;
    /* -- end of the first version of this struct (40 bytes, still accepted) -- */
    uint32_t decode_segments;  /* path 1: output segments of the decode plan */
    uint32_t decode_groups;    /* path 1: block groups of the decode plan (= n_units) */
    uint32_t block_classes;    /* path 1: bit i set when some channel block has 2^i 16-byte words per
                                  state row (8 * 2^i input channels per block) */
    uint32_t prefill_kernel;   /* what sketch_linear_gemm runs on calls with fewer than
                                  prefill_staged_from tokens: SKL_PREFILL_* */
    uint32_t n_blocks;         /* path 1: channel blocks */
    uint32_t prefill_staged_from; /* row sketches: calls with at least this many tokens take
                                  SKL_PREFILL_STAGED (0: every call, 0xFFFFFFFF: none) */
} skl_info_t;

#define SKL_INFO_SIZE_V1 40u

/* skl_info_t.prefill_kernel */
#define SKL_PREFILL_PER_WEIGHT 0u   /* 2-D groups: weights hashed one by one, 64 x 64 tiles */
#define SKL_PREFILL_FUSED 3u        /* row sketches, tables of two blocks resident in LDS: weights rebuilt
                                       between the matrix instructions of a 256 x 256 tile */
#define SKL_PREFILL_STAGED 4u       /* row sketches with larger tables, and long calls: weights rebuilt once per
                                       call into a cache-sized slab of the workspace, then a 256 x 256-tile
                                       product */

/* Bytes of device memory create() needs for this description.
 * Validates the whole description (Sec. 3.1 states must be finite). */
SKL_API skl_status_t sketch_linear_device_bytes(const skl_desc_t *desc, uint64_t *bytes);

/* Build a layer: validate, lay the tables out for the kernels (states are
 * re-encoded as order keys and, for row sketches, transposed so that eight
 * consecutive input channels of one state sit in one 16-byte word) and copy
 * them into dev_buf (DEVICE, 256-byte aligned, >= device_bytes).  This is
 * the sketch state S of Sec. 3.1 that "stays permanently in memory". */
SKL_API skl_status_t sketch_linear_create(const skl_desc_t *desc, void *dev_buf, uint64_t dev_bytes,
                                  void *hip_stream, skl_layer_t **out_layer);

SKL_API skl_status_t sketch_linear_info(const skl_layer_t *layer, skl_info_t *info);

/* Diagnostic, host only (no GPU call, no device memory): what create() would
 * decide for this description, and the decode planner's own cost model (Sec.
 * 3.2 / 3.3 widths -> channel blocks -> output segments x block groups, one
 * workgroup each).  segments = groups = 0: the plan the library picks.
 * Otherwise: the same layer planned with that decode split --
 * SKL_ERR_UNSUPPORTED if the kernels cannot run it (more than 16 wave units
 * of 64 outputs per segment, or more than 64 channel blocks per group).
 * *decode_cost_us (may be NULL) receives the model's microseconds for the
 * split (0 for layers on the per-weight path). */
SKL_API skl_status_t sketch_linear_plan(const skl_desc_t *desc, uint32_t segments, uint32_t groups, skl_info_t *info,
                                double *decode_cost_us);

/* Bytes of DEVICE workspace needed by gemv (op = 0, n = batch), gemm
 * (op = 1, n = tokens) or reconstruct (op = 2, n ignored).  The workspace
 * holds the partial sums of the split reduction (gemv), the re-ordered fp16
 * activations and partial tiles (gemm) and, for layers with low-bit states,
 * the 16-bit tables expanded for the call; its contents are scratch. */
SKL_API skl_status_t sketch_linear_workspace_bytes(const skl_layer_t *layer, uint32_t op, uint32_t n,
                                           uint64_t *bytes);

/* Decode:  y[b][o] = sum_j x[b][j] * W_hat[j][o],  b < batch (1..16).
 *   x  DEVICE, binary16, [batch][ldx], ldx >= in_features  (x_dtype must be SKL_F16)
 *   y  DEVICE, binary16 or float32, [batch][ldy], ldy >= out_features
 * Products are exact, accumulation is float32, the result is rounded to
 * nearest-even once.  The summation order is fixed: results are
 * bit-identical from run to run.  (Sec. 3 inference flow: decompress then
 * compute, here fused; Eq. 5 and Eq. 1/2.) */
SKL_API skl_status_t sketch_linear_gemv(const skl_layer_t *layer, const void *x, skl_dtype_t x_dtype,
                                uint32_t ldx, void *y, skl_dtype_t y_dtype, uint32_t ldy,
                                uint32_t batch, void *workspace, uint64_t workspace_bytes,
                                void *hip_stream);

/* The same decode for callers that cannot allocate device memory or pass a
 * workspace (code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation): the call's scratch lives in a device array inside
 * the library, SKL_STATIC_SCRATCH_MAX bytes per GPU, held until the process
 * ends.  The call allocates nothing and returns SKL_ERR_UNSUPPORTED when
 * sketch_linear_workspace_bytes(layer, 0, batch) exceeds that size.  All such
 * calls on one GPU share the array: calls that may overlap in time (different
 * streams, different host threads without ordering) race; order them on one
 * stream.  Arguments, results and summation order as sketch_linear_gemv. */
#define SKL_STATIC_SCRATCH_MAX (16u << 20)
SKL_API skl_status_t sketch_linear_gemv_static(const skl_layer_t *layer, const void *x, skl_dtype_t x_dtype,
                                       uint32_t ldx, void *y, skl_dtype_t y_dtype, uint32_t ldy,
                                       uint32_t batch, void *hip_stream);

/* Decode through 1..4 layers that read the same activations (the q/k/v or
 * the gate/up projections of a block; Sec. 2.1, Eq. 1/2) in one pair of
 * launches:  ys[i][b][o] = sum_j x[b][j] * W_hat_i[j][o],  b < batch (1..16).
 * The layers must be row-sketch layers with the same in_features,
 * out_features and d (SKL_ERR_UNSUPPORTED otherwise; binary16 and low-bit
 * states may be mixed); x as for sketch_linear_gemv; ys HOST array of
 * n_layers DEVICE pointers, each [batch][ldy] of y_dtype (binary16 or
 * float32), not overlapping.  Results are bit-identical to n_layers calls of
 * sketch_linear_gemv. */
SKL_API skl_status_t sketch_linear_gemv_group_workspace_bytes(const skl_layer_t *const *layers, uint32_t n_layers,
                                                      uint32_t batch, uint64_t *bytes);
SKL_API skl_status_t sketch_linear_gemv_group(const skl_layer_t *const *layers, uint32_t n_layers, const void *x,
                                      skl_dtype_t x_dtype, uint32_t ldx, void *const *ys, skl_dtype_t y_dtype,
                                      uint32_t ldy, uint32_t batch, void *workspace, uint64_t workspace_bytes,
                                      void *hip_stream);

/* The first half of a feed-forward block (Sec. 2.1, Eq. 2, with SiLU as the
 * activation, as in the Llama-shaped configurations):
 *     h[b][o] = SiLU(sum_j x[b][j] W_hat_gate[j][o]) * (sum_j x[b][j] W_hat_up[j][o]),
 * SiLU(a) = a / (1 + exp(-a)) in float32.  Same layer requirements, workspace
 * (sketch_linear_gemv_group_workspace_bytes of {gate, up}) and argument rules
 * as sketch_linear_gemv_group; h DEVICE [batch][ldh], binary16 or float32. */
SKL_API skl_status_t sketch_linear_gemv_gate_up(const skl_layer_t *gate, const skl_layer_t *up, const void *x,
                                        skl_dtype_t x_dtype, uint32_t ldx, void *h, skl_dtype_t h_dtype,
                                        uint32_t ldh, uint32_t batch, void *workspace, uint64_t workspace_bytes,
                                        void *hip_stream);

/* Diagnostic: only the first of the two kernels behind sketch_linear_gemv
 * (query, Eq. 5, fused with the products; one partial sum per output and
 * block group left in workspace), without the reduction that produces y.
 * For timing that kernel by itself; same argument rules as gemv. */
SKL_API skl_status_t sketch_linear_gemv_partials(const skl_layer_t *layer, const void *x, skl_dtype_t x_dtype,
                                         uint32_t ldx, uint32_t batch, void *workspace,
                                         uint64_t workspace_bytes, void *hip_stream);

/* Prefill (Sec. 3 inference flow, decompression and product fused; Eq. 5 for
 * W_hat, Sec. 2.1 Eq. 1/2 for the product):
 *     Y[t][o] = sum_j X[t][j] * W_hat[j][o],  t < tokens (>= 1).
 *   X  DEVICE, bfloat16 or binary16, [tokens][ldx]; |X| must not exceed 65504:
 *      bfloat16 inputs are converted to binary16 (exact inside that range,
 *      down to the binary16 subnormal step) so that W_hat enters the matrix
 *      cores unrounded.
 *   Y  DEVICE, bfloat16, binary16 or float32, [tokens][ldy]
 * float32 accumulation on the matrix cores (MFMA), one final rounding. */
SKL_API skl_status_t sketch_linear_gemm(const skl_layer_t *layer, const void *X, skl_dtype_t x_dtype,
                                uint32_t ldx, void *Y, skl_dtype_t y_dtype, uint32_t ldy,
                                uint32_t tokens, void *workspace, uint64_t workspace_bytes,
                                void *hip_stream);

/* Diagnostic, host only (no GPU call): how sketch_linear_gemm divides a
 * prefill of `tokens` tokens through a row-sketch layer with `out_features`
 * outputs over the workgroups of its main kernel.  `kernel` is
 * SKL_PREFILL_FUSED (a block is one input-channel block of the layer) or
 * SKL_PREFILL_STAGED (a block is 64 entries of the layer's channel list);
 * `n_blocks` is the number of such blocks.  Output tiles are 256 tokens x 256
 * outputs; every (tile, block) product belongs to exactly one segment.  Each
 * segment is eight words in `segments` (HOST, room for `capacity` segments):
 * XCD, workgroup within the XCD, token tile, output tile, first block, end
 * block, 1 if the segment is a whole tile stored by the main kernel else 0,
 * and the float32 partial-tile slot a partial segment leaves for the fix-up
 * pass (partials of one tile occupy consecutive slots in workgroup order,
 * which fixes the summation order).  Tiles are dealt to the 8 XCDs in units
 * of mu token tiles of one output-tile column, unit
 * u = output tile * (token tiles / mu) + token tile / mu to XCD u % 8; the
 * fused kernel has mu = 1, the staged kernel the largest mu that keeps the
 * XCDs balanced.  Tiles are 256 tokens high, except in staged calls whose
 * 128-token tiles number between 225 and 256 (2048 tokens x 4096 outputs):
 * there every workgroup takes one whole tile of 128 tokens and nothing is left
 * over.
 * *n_segments receives the number of segments (also when it exceeds
 * `capacity`; then only the first `capacity` are written).  `shape` (HOST,
 * 6 words, may be NULL) receives workgroups per XCD, partial tiles per XCD,
 * slots per partial tile, the tile count, mu, and the tokens per tile. */
SKL_API skl_status_t sketch_linear_prefill_split(uint32_t kernel, uint32_t out_features, uint32_t n_blocks,
                                         uint32_t tokens, uint32_t *segments, uint64_t capacity,
                                         uint64_t *n_segments, uint32_t *shape);

/* Sketch construction on the device (Sec. 3.1, Eq. 4: a state keeps the
 * weight of smallest magnitude that maps to it, the first one in address order
 * among equals; Sec. 3.3, Eq. 8 and Alg. 1 compute the same states).  Builds
 * the binary16 states of the weights W_dev (DEVICE, [in_features][out_features]
 * binary16, row major, finite) for the geometry, hash parameters and widths
 * of `desc` (its states / codes / scales fields are ignored; n_states must be
 * d * sum(group_width)) and writes them to states_dev (DEVICE, [n_states], the
 * order `states` has in the description); states no weight reaches are +0.0.
 * Offline step: the call synchronises hip_stream once before it returns.
 * The result is independent of timing.  Workspace (DEVICE, 256-byte aligned):
 * sketch_linear_build_workspace_bytes. */
SKL_API skl_status_t sketch_linear_build_workspace_bytes(const skl_desc_t *desc, uint64_t *bytes);
SKL_API skl_status_t sketch_linear_build_states(const skl_desc_t *desc, const uint16_t *W_dev, uint16_t *states_dev,
                                        void *workspace, uint64_t workspace_bytes, void *hip_stream);

/* Diagnostic: write W_hat (Eq. 5) as binary16 bit patterns to
 * W_hat_dev (DEVICE, [in_features][out_features], row major).  The only call
 * that materialises the weights.  The workspace (op = 2) is needed only by
 * layers with low-bit states and may be NULL otherwise. */
SKL_API skl_status_t sketch_linear_reconstruct(const skl_layer_t *layer, uint16_t *W_hat_dev, void *workspace,
                                       uint64_t workspace_bytes, void *hip_stream);

/* Comparator: the same W_hat through the hash-based operator the paper starts
 * from (Sec. 3.3, the operation its matrix form replaces; Sec. 4, the
 * decompression speed-up figure): one select (Eq. 3) per weight and sketch
 * row, every candidate state fetched from device memory, nothing staged or
 * shared.  Same arguments and result as sketch_linear_reconstruct; exists to
 * be timed against it and against the fused calls. */
SKL_API skl_status_t sketch_linear_reconstruct_hash_op(const skl_layer_t *layer, uint16_t *W_hat_dev, void *workspace,
                                               uint64_t workspace_bytes, void *hip_stream);

/* Diagnostic: one launch of a small kernel that measures a ceiling of the
 * machine as this library's kernels can reach it, for stating roofline
 * fractions against measured figures as well as data-sheet ones.
 *   kind 0  vector ALU: packed 16-bit maximum and packed multiply-add on
 *           registers (the instruction classes of the query and decode stages);
 *           *work = lane-instructions issued;
 *   kind 1  LDS: 16-byte reads at lane-dependent addresses without bank
 *           conflicts; *work = bytes read;
 *   kind 2  matrix cores: f16 MFMA 32x32x16 on registers, one wavefront per
 *           SIMD; *work = floating-point operations;
 *   kind 3  HBM: streaming read of the workspace past its first 4 MiB;
 *           *work = bytes read;
 *   kind 4  matrix cores as kind 2, but every MFMA takes other operand words
 *           of random sign and mantissa bits (kind 2 multiplies two constant
 *           words): the rate at the switching activity of real data, where the
 *           chip runs below its top clock; *work = floating-point operations.
 * `iters` scales the work of kinds 0..2 and 4 (1..2^20; ignored for kind 3).
 * workspace: DEVICE, 256-byte aligned, more than 4 MiB (kind 3: as much as
 * should be streamed; use several times the cache sizes).  Only enqueues;
 * time the launch with events on hip_stream. */
SKL_API skl_status_t sketch_linear_microbench(uint32_t kind, uint32_t iters, void *workspace, uint64_t workspace_bytes,
                                      void *hip_stream, uint64_t *work);

/* Layer file: a description (the sketch state S of Sec. 3.1 with its select
 * parameters of Eq. 3 and the per-group widths of Sec. 3.2 / 3.3 -- everything
 * create() takes) as one flat little-endian image: a 128-byte header (magic
 * "SKLAYER1", version, geometry, section offsets, 64-bit FNV-1a checksum),
 * then hash_a, hash_c, group_width, the states (or codes) and the scales,
 * each section 64-byte aligned.  Host only, no GPU call.
 *   file_bytes  size of the image of a (fully validated) description;
 *   file_write  writes the image into `image` (HOST, >= file_bytes);
 *   file_save   the same into a file at `path`;
 *   file_open   checks an image (magic, version, size, checksum, section
 *               offsets against the geometry, then the whole validation of
 *               create()) and fills *desc with pointers INTO the image --
 *               nothing is copied, so a file can be mapped and used in
 *               place; the image must be 8-byte aligned and outlive every
 *               use of *desc.  SKL_ERR_INVALID_ARG for anything that is not
 *               an intact layer file, SKL_ERR_UNSUPPORTED for another
 *               version of the format. */
SKL_API skl_status_t sketch_linear_file_bytes(const skl_desc_t *desc, uint64_t *bytes);
SKL_API skl_status_t sketch_linear_file_write(const skl_desc_t *desc, void *image, uint64_t image_bytes);
SKL_API skl_status_t sketch_linear_file_save(const skl_desc_t *desc, const char *path);
SKL_API skl_status_t sketch_linear_file_open(const void *image, uint64_t image_bytes, skl_desc_t *desc);

/* Debug build only (libsketch_linear_debug.so, compiled with
 * -DSKL_DEBUG_BOUNDS): its kernels check the index ranges they rely on --
 * select indices (Eq. 3) against the sketch width, LDS addresses of gathers
 * and table copies, channel and block numbers -- and count violations
 * instead of faulting (the offending access is redirected).  *count receives
 * the violations since the library was loaded (synchronise the streams
 * first); first[5] (may be NULL) the first one: code, value, limit,
 * workgroup, thread.  SKL_ERR_UNSUPPORTED in the normal build, whose kernels
 * carry no checks. */
SKL_API skl_status_t sketch_linear_debug_violations(uint64_t *count, uint32_t first[5]);
/* Debug build only: enqueues one thread that evaluates the range assert
 * `value < limit` (code 7) and touches no memory -- lets a test watch a
 * violation being counted.  SKL_ERR_UNSUPPORTED in the normal build. */
SKL_API skl_status_t sketch_linear_debug_selftest(uint32_t value, uint32_t limit, void *hip_stream);

/* Frees the host object only; dev_buf stays the caller's. NULL is accepted. */
SKL_API void sketch_linear_destroy(skl_layer_t *layer);

/* Text for the calling thread's last non-OK status ("" if none). */
SKL_API const char *sketch_linear_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SKETCH_LINEAR_H */
