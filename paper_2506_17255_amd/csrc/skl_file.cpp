// Flat layer file: a sketched layer (the description sketch_linear_create() takes: geometry, hash
// parameters of Sec. 3.1 Eq. 3, per-group widths of Sec. 3.2 / 3.3, states or codes and scales) as one
// little-endian image that can be written to disk as it is and used in place after reading or mapping it:
// the description handed back points into the image.  Host only.
//
//   [header, 128 bytes][hash_a][hash_c][group_width][states or codes][scales]   sections 64-byte aligned
#include <stdio.h>
#include <string.h>

#include "skl_internal.h"

namespace {

const char MAGIC[8] = {'S', 'K', 'L', 'A', 'Y', 'E', 'R', '1'};
const uint32_t VERSION = 1;
const uint32_t HEADER_BYTES = 128;

struct FileHeader {
    char magic[8];
    uint32_t version, header_bytes;
    uint32_t in_features, out_features, tile_in, tile_out, d, query_mode, flags, state_bits;
    uint64_t n_groups, n_states;
    uint64_t off_hash_a, off_hash_c, off_widths, off_states, off_scales, file_bytes;
    uint64_t checksum;          // FNV-1a, 64 bit, over the header with this field zero and everything after the header
    uint64_t reserved;
};
static_assert(sizeof(FileHeader) == HEADER_BYTES, "the header is part of the file format");

uint64_t fnv1a(const uint8_t *p, uint64_t n, uint64_t h)
{
    for (uint64_t i = 0; i < n; ++i) { h ^= p[i]; h *= 0x100000001B3ull; }
    return h;
}

uint64_t image_checksum(const uint8_t *image, uint64_t bytes)
{
    FileHeader h;
    memcpy(&h, image, sizeof h);
    h.checksum = 0;
    uint64_t sum = fnv1a(reinterpret_cast<const uint8_t *>(&h), sizeof h, 0xCBF29CE484222325ull);
    return fnv1a(image + HEADER_BYTES, bytes - HEADER_BYTES, sum);
}

uint64_t align64(uint64_t v) { return (v + 63) & ~63ull; }

// groups and payload sizes of a description (geometry checked by the caller through skl_make_plan)
struct Sizes { uint64_t n_groups, state_bytes, scale_bytes; };

Sizes sizes_of(uint32_t in, uint32_t out, uint32_t ti, uint32_t to, uint32_t d, uint32_t state_bits, uint64_t n_states)
{
    Sizes s;
    s.n_groups = (uint64_t)(in / ti) * (out / to);
    const bool low = state_bits == 8 || state_bits == 4;
    s.state_bytes = !low ? n_states * 2 : state_bits == 8 ? n_states : (n_states + 1) / 2;
    s.scale_bytes = low ? s.n_groups * d * 2 : 0;
    return s;
}

void layout(FileHeader &h, const Sizes &s)
{
    uint64_t off = HEADER_BYTES;
    h.off_hash_a = off; off = align64(off + 4ull * h.d);
    h.off_hash_c = off; off = align64(off + 4ull * h.d);
    h.off_widths = off; off = align64(off + 4 * s.n_groups);
    h.off_states = off; off = align64(off + s.state_bytes);
    h.off_scales = off; off = align64(off + s.scale_bytes);
    h.file_bytes = off;
}

#define FAIL(code, ...) do { skl_set_error(__VA_ARGS__); return code; } while (0)

skl_status_t header_of(const skl_desc_t *user, FileHeader *h, Sizes *s, skl_desc_t *d)
{
    skl_plan P;
    skl_status_t st = skl_make_plan(user, &P);       // the whole validation of create()
    if (st != SKL_OK) return st;
    *d = P.desc;
    memset(h, 0, sizeof *h);
    memcpy(h->magic, MAGIC, 8);
    h->version = VERSION; h->header_bytes = HEADER_BYTES;
    h->in_features = d->in_features; h->out_features = d->out_features; h->tile_in = d->tile_in; h->tile_out = d->tile_out;
    h->d = d->d; h->query_mode = d->query_mode; h->flags = d->flags;
    h->state_bits = d->state_bits == 16 ? 0 : d->state_bits;
    *s = sizes_of(d->in_features, d->out_features, d->tile_in, d->tile_out, d->d, d->state_bits, d->n_states);
    h->n_groups = s->n_groups; h->n_states = d->n_states;
    layout(*h, *s);
    return SKL_OK;
}

}  // namespace

extern "C" {

skl_status_t sketch_linear_file_bytes(const skl_desc_t *desc, uint64_t *bytes)
{
    if (!bytes) FAIL(SKL_ERR_INVALID_ARG, "bytes is NULL");
    FileHeader h; Sizes s; skl_desc_t d;
    skl_status_t st = header_of(desc, &h, &s, &d);
    if (st != SKL_OK) return st;
    *bytes = h.file_bytes;
    return SKL_OK;
}

skl_status_t sketch_linear_file_write(const skl_desc_t *desc, void *image_, uint64_t image_bytes)
{
    if (!image_) FAIL(SKL_ERR_INVALID_ARG, "image is NULL");
    FileHeader h; Sizes s; skl_desc_t d;
    skl_status_t st = header_of(desc, &h, &s, &d);
    if (st != SKL_OK) return st;
    if (image_bytes < h.file_bytes)
        FAIL(SKL_ERR_BUFFER_TOO_SMALL, "image of %llu bytes, the layer needs %llu", (unsigned long long)image_bytes,
             (unsigned long long)h.file_bytes);
    uint8_t *image = static_cast<uint8_t *>(image_);
    memset(image, 0, h.file_bytes);
    memcpy(image + h.off_hash_a, d.hash_a, 4ull * d.d);
    memcpy(image + h.off_hash_c, d.hash_c, 4ull * d.d);
    memcpy(image + h.off_widths, d.group_width, 4 * s.n_groups);
    const bool low = d.state_bits == 8 || d.state_bits == 4;
    memcpy(image + h.off_states, low ? d.codes : static_cast<const void *>(d.states), s.state_bytes);
    if (low) memcpy(image + h.off_scales, d.scales, s.scale_bytes);
    memcpy(image, &h, sizeof h);
    h.checksum = image_checksum(image, h.file_bytes);
    memcpy(image, &h, sizeof h);
    return SKL_OK;
}

skl_status_t sketch_linear_file_open(const void *image_, uint64_t image_bytes, skl_desc_t *desc)
{
    if (!image_ || !desc) FAIL(SKL_ERR_INVALID_ARG, "image or desc is NULL");
    if (reinterpret_cast<uintptr_t>(image_) % 8) FAIL(SKL_ERR_INVALID_ARG, "the image must be 8-byte aligned");
    if (image_bytes < HEADER_BYTES) FAIL(SKL_ERR_INVALID_ARG, "%llu bytes are less than a layer file's header", (unsigned long long)image_bytes);
    const uint8_t *image = static_cast<const uint8_t *>(image_);
    FileHeader h;
    memcpy(&h, image, sizeof h);
    if (memcmp(h.magic, MAGIC, 8) != 0) FAIL(SKL_ERR_INVALID_ARG, "not a layer file (magic)");
    if (h.version != VERSION || h.header_bytes != HEADER_BYTES)
        FAIL(SKL_ERR_UNSUPPORTED, "layer file version %u with a %u-byte header; this library reads version %u", h.version,
             h.header_bytes, VERSION);
    if (h.file_bytes > image_bytes || h.file_bytes < HEADER_BYTES)
        FAIL(SKL_ERR_INVALID_ARG, "the file says %llu bytes, %llu are there (truncated?)", (unsigned long long)h.file_bytes,
             (unsigned long long)image_bytes);
    if (image_checksum(image, h.file_bytes) != h.checksum) FAIL(SKL_ERR_INVALID_ARG, "layer file checksum mismatch");
    // the section offsets must be the ones this geometry gives (nothing in the header is trusted before that)
    if (h.d < 1 || h.d > SKL_MAX_D || !h.tile_in || !h.tile_out || !h.in_features || !h.out_features ||
        h.in_features % h.tile_in || h.out_features % h.tile_out || (h.state_bits != 0 && h.state_bits != 8 && h.state_bits != 4))
        FAIL(SKL_ERR_INVALID_ARG, "layer file header: impossible geometry");
    const Sizes s = sizes_of(h.in_features, h.out_features, h.tile_in, h.tile_out, h.d, h.state_bits, h.n_states);
    FileHeader want = h;
    layout(want, s);
    if (s.n_groups != h.n_groups || s.n_groups > (1ull << 40) || h.n_states > (1ull << 40) || want.off_hash_a != h.off_hash_a || want.off_hash_c != h.off_hash_c ||
        want.off_widths != h.off_widths || want.off_states != h.off_states || want.off_scales != h.off_scales ||
        want.file_bytes != h.file_bytes)
        FAIL(SKL_ERR_INVALID_ARG, "layer file header: section offsets do not match the geometry");
    memset(desc, 0, sizeof *desc);
    desc->struct_size = sizeof *desc;
    desc->in_features = h.in_features; desc->out_features = h.out_features; desc->tile_in = h.tile_in; desc->tile_out = h.tile_out;
    desc->d = h.d; desc->query_mode = h.query_mode; desc->flags = h.flags;
    desc->hash_a = reinterpret_cast<const uint32_t *>(image + h.off_hash_a);
    desc->hash_c = reinterpret_cast<const uint32_t *>(image + h.off_hash_c);
    desc->group_width = reinterpret_cast<const uint32_t *>(image + h.off_widths);
    desc->n_states = h.n_states;
    desc->state_bits = h.state_bits;
    if (h.state_bits) {
        desc->codes = image + h.off_states;
        desc->scales = reinterpret_cast<const uint16_t *>(image + h.off_scales);
    } else {
        desc->states = reinterpret_cast<const uint16_t *>(image + h.off_states);
    }
    skl_plan P;                                     // the contents get the same validation as any description
    return skl_make_plan(desc, &P);
}

skl_status_t sketch_linear_file_save(const skl_desc_t *desc, const char *path)
{
    if (!path) FAIL(SKL_ERR_INVALID_ARG, "path is NULL");
    uint64_t bytes = 0;
    skl_status_t st = sketch_linear_file_bytes(desc, &bytes);
    if (st != SKL_OK) return st;
    std::vector<uint8_t> image;
    try {
        image.resize(bytes);
    } catch (const std::bad_alloc &) {
        FAIL(SKL_ERR_NO_MEMORY, "out of host memory for a %llu-byte layer file", (unsigned long long)bytes);
    }
    st = sketch_linear_file_write(desc, image.data(), bytes);
    if (st != SKL_OK) return st;
    FILE *f = fopen(path, "wb");
    if (!f) FAIL(SKL_ERR_INVALID_ARG, "cannot open %s for writing", path);
    const bool ok = fwrite(image.data(), 1, bytes, f) == bytes;
    if (fclose(f) != 0 || !ok) FAIL(SKL_ERR_INVALID_ARG, "writing %s failed", path);
    return SKL_OK;
}

}  // extern "C"
