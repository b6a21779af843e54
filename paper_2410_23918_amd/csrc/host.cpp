// Host side of the BitStack C ABI: argument checks, packing into the private
// device layout, kernel dispatch.  See include/bitstack.h for the contract.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/bitstack.h"
#include "../../include/bitstack_bench.h"
#include "kernels.h"
#include "kparams.h"
#include "layout.h"

using namespace bitstack;

struct bitstack_weight {
    Geometry geo;
    unsigned char* dev;  // caller-owned device buffer
    int resident;        // blocks 0 .. resident-1 are loaded (Section 2.2: blocks come and go in stack order)
};

static thread_local int g_last_hip = 0;

static int hip_fail(hipError_t e) {
    g_last_hip = static_cast<int>(e);
    return BITSTACK_E_HIP;
}
#define BS_HIP(call)                                   \
    do {                                               \
        hipError_t e__ = (call);                       \
        if (e__ != hipSuccess) return hip_fail(e__);   \
    } while (0)

extern "C" {

size_t bitstack_block_bytes(int out, int in, int k) {
    if (!shape_ok(out, in, k)) return 0;
    return (size_t(out) * size_t(in) + size_t(16) * k * (size_t(out) + size_t(in))) / 8;
}

size_t bitstack_packed_bytes(int out, int in, int k, int n, int max_batch) {
    if (!shape_ok(out, in, k) || n < 0 || max_batch < 1) return 0;
    return make_geometry(out, in, n, max_batch).total;
}

int bitstack_pack_signs_from_f32(int out, int in, const float* residual, uint32_t* sign_words) {
    if (!residual || !sign_words) return BITSTACK_E_NULL;
    if (out <= 0 || in <= 0 || in % 32) return BITSTACK_E_SHAPE;
    const int wpr = in / 32;
    for (int o = 0; o < out; ++o) {
        const float* row = residual + size_t(o) * in;
        for (int w = 0; w < wpr; ++w) {
            uint32_t word = 0;
            for (int b = 0; b < 32; ++b)
                if (row[w * 32 + b] >= 0.0f) word |= (uint32_t(1) << b);  // +0, -0 -> +1
            sign_words[size_t(o) * wpr + w] = word;
        }
    }
    return BITSTACK_OK;
}

static int check_pack_args(int out, int in, int k, int n, int max_batch, const uint32_t* sw,
                           const uint16_t* U, const uint16_t* V, const float* s) {
    if (!shape_ok(out, in, k) || n < 0 || max_batch < 1) return BITSTACK_E_SHAPE;
    if (!s || (n > 0 && (!sw || !U || !V))) return BITSTACK_E_NULL;
    for (int j = 0; j < in; ++j)
        if (!(std::isfinite(s[j]) && s[j] > 0.0f)) return BITSTACK_E_SCALE;
    return BITSTACK_OK;
}

// device form of one block: sign tiles, V panels, U rows into blk (block_stride bytes), and the
// derived per-channel maxima of V into vm (in values, panel order)
static void pack_block(const Geometry& g, unsigned char* blk, uint16_t* vm, const uint32_t* csw, const uint16_t* cu,
                       const uint16_t* cv) {
    const int out = g.out, in = g.in, wpr = in / 32;
    uint32_t* dsw = reinterpret_cast<uint32_t*>(blk);
    for (int o = 0; o < out; ++o)
        for (int w = 0; w < wpr; ++w) dsw[sign_word_index(in, o, w)] = csw[size_t(o) * wpr + w];
    uint16_t* dv = reinterpret_cast<uint16_t*>(blk + g.off_v);
    for (int j = 0; j < in; ++j)
        for (int r = 0; r < kRank; ++r) dv[v_index(j, r)] = cv[size_t(j) * kRank + r];
    std::memcpy(blk + g.off_u, cu, size_t(out) * kRank * 2);
    // max_r |V[j][r]| per channel (fp16 magnitudes compare like their bit patterns)
    for (int j = 0; j < in; ++j) {
        uint16_t m = 0;
        for (int r = 0; r < kRank; ++r) {
            uint16_t a = cv[size_t(j) * kRank + r] & 0x7FFFu;
            if (a > 0x7C00u) a = 0x7C00u;  // NaN payloads: treat as infinity
            if (a > m) m = a;
        }
        vm[panel_index(j)] = m;
    }
}

int bitstack_pack_image_host(int out, int in, int k, int n, int max_batch,
                             const uint32_t* sign_words, const uint16_t* U, const uint16_t* V,
                             const float* s, void* image, size_t image_bytes) {
    int rc = check_pack_args(out, in, k, n, max_batch, sign_words, U, V, s);
    if (rc) return rc;
    if (!image) return BITSTACK_E_NULL;
    const Geometry g = make_geometry(out, in, n, max_batch);
    if (image_bytes < g.total) return BITSTACK_E_BUFSIZE;
    unsigned char* img = static_cast<unsigned char*>(image);
    std::memset(img, 0, g.total);
    float* rs = reinterpret_cast<float*>(img + g.off_rs);
    for (int j = 0; j < in; ++j) rs[j] = 1.0f / s[j];
    const int wpr = in / 32;
    for (int i = 0; i < n; ++i)
        pack_block(g, img + g.off_blocks + size_t(i) * g.block_stride,
                   reinterpret_cast<uint16_t*>(img + g.off_vmax) + size_t(i) * in, sign_words + size_t(i) * out * wpr,
                   U + size_t(i) * out * kRank, V + size_t(i) * in * kRank);
    return BITSTACK_OK;
}

static void unpack_block(const Geometry& g, const unsigned char* blk, uint32_t* sign_words,
                         uint16_t* U, uint16_t* V) {
    const int wpr = g.in / 32;
    if (sign_words) {
        const uint32_t* dsw = reinterpret_cast<const uint32_t*>(blk);
        for (int o = 0; o < g.out; ++o)
            for (int w = 0; w < wpr; ++w)
                sign_words[size_t(o) * wpr + w] = dsw[sign_word_index(g.in, o, w)];
    }
    if (V) {
        const uint16_t* dv = reinterpret_cast<const uint16_t*>(blk + g.off_v);
        for (int j = 0; j < g.in; ++j)
            for (int r = 0; r < kRank; ++r) V[size_t(j) * kRank + r] = dv[v_index(j, r)];
    }
    if (U) std::memcpy(U, blk + g.off_u, size_t(g.out) * kRank * 2);
}

int bitstack_unpack_image_host(int out, int in, int k, int n, int max_batch, const void* image,
                               int block, uint32_t* sign_words, uint16_t* U, uint16_t* V) {
    if (!shape_ok(out, in, k) || n < 0 || max_batch < 1) return BITSTACK_E_SHAPE;
    if (!image) return BITSTACK_E_NULL;
    if (block < 0 || block >= n) return BITSTACK_E_RANGE;
    const Geometry g = make_geometry(out, in, n, max_batch);
    unpack_block(g, static_cast<const unsigned char*>(image) + g.off_blocks + size_t(block) * g.block_stride,
                 sign_words, U, V);
    return BITSTACK_OK;
}

int bitstack_pack_blocks(int out, int in, int k, int n, int max_batch, const uint32_t* sign_words,
                         const uint16_t* U, const uint16_t* V, const float* s, void* device_buf,
                         size_t device_buf_bytes, bitstack_stream_t stream,
                         bitstack_weight_t** handle) {
    if (!handle) return BITSTACK_E_NULL;
    *handle = nullptr;
    int rc = check_pack_args(out, in, k, n, max_batch, sign_words, U, V, s);
    if (rc) return rc;
    if (!device_buf) return BITSTACK_E_NULL;
    if (reinterpret_cast<uintptr_t>(device_buf) % 256) return BITSTACK_E_ALIGN;
    const Geometry g = make_geometry(out, in, n, max_batch);
    if (device_buf_bytes < g.total) return BITSTACK_E_BUFSIZE;
    std::vector<unsigned char> img;
    try {
        img.resize(g.total);
    } catch (const std::bad_alloc&) {
        return BITSTACK_E_BUFSIZE;
    }
    rc = bitstack_pack_image_host(out, in, k, n, max_batch, sign_words, U, V, s, img.data(), img.size());
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    BS_HIP(hipMemcpyAsync(device_buf, img.data(), g.total, hipMemcpyHostToDevice, st));
    BS_HIP(hipStreamSynchronize(st));
    bitstack_weight* w = new (std::nothrow) bitstack_weight;
    if (!w) return BITSTACK_E_BUFSIZE;
    w->geo = g;
    w->dev = static_cast<unsigned char*>(device_buf);
    w->resident = n;
    *handle = w;
    return BITSTACK_OK;
}

// ---- dynamic loading: one block at a time (Section 2.2; appendix on minimal transmission units)

size_t bitstack_block_staging_bytes(int out, int in, int k) {
    if (!shape_ok(out, in, k)) return 0;
    return align256(bitstack_block_bytes(out, in, k)) + align256(size_t(in) * 2);
}

int bitstack_stage_block_host(int out, int in, int k, const uint32_t* sign_words, const uint16_t* U,
                              const uint16_t* V, void* staging, size_t staging_bytes) {
    if (!shape_ok(out, in, k)) return BITSTACK_E_SHAPE;
    if (!sign_words || !U || !V || !staging) return BITSTACK_E_NULL;
    if (staging_bytes < bitstack_block_staging_bytes(out, in, k)) return BITSTACK_E_BUFSIZE;
    const Geometry g = make_geometry(out, in, 1, 1);
    unsigned char* st = static_cast<unsigned char*>(staging);
    std::memset(st, 0, bitstack_block_staging_bytes(out, in, k));
    pack_block(g, st, reinterpret_cast<uint16_t*>(st + align256(g.block_stride)), sign_words, U, V);
    return BITSTACK_OK;
}

int bitstack_create_stack(int out, int in, int k, int n_slots, int max_batch, const float* s, void* device_buf,
                          size_t device_buf_bytes, bitstack_stream_t stream, bitstack_weight_t** handle) {
    if (!handle) return BITSTACK_E_NULL;
    *handle = nullptr;
    int rc = check_pack_args(out, in, k, 0, max_batch, nullptr, nullptr, nullptr, s);
    if (rc) return rc;
    if (n_slots < 1) return BITSTACK_E_RANGE;
    if (!device_buf) return BITSTACK_E_NULL;
    if (reinterpret_cast<uintptr_t>(device_buf) % 256) return BITSTACK_E_ALIGN;
    const Geometry g = make_geometry(out, in, n_slots, max_batch);
    if (device_buf_bytes < g.total) return BITSTACK_E_BUFSIZE;
    std::vector<float> rs;
    try {
        rs.resize(in);
    } catch (const std::bad_alloc&) {
        return BITSTACK_E_BUFSIZE;
    }
    for (int j = 0; j < in; ++j) rs[j] = 1.0f / s[j];
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* dev = static_cast<unsigned char*>(device_buf);
    BS_HIP(hipMemcpyAsync(dev + g.off_rs, rs.data(), size_t(in) * 4, hipMemcpyHostToDevice, st));
    // workspace and counters start at zero; block slots and row maxima are written by the pushes
    BS_HIP(hipMemsetAsync(dev + g.off_part, 0, g.total - g.off_part, st));
    BS_HIP(hipStreamSynchronize(st));
    bitstack_weight* w = new (std::nothrow) bitstack_weight;
    if (!w) return BITSTACK_E_BUFSIZE;
    w->geo = g;
    w->dev = dev;
    w->resident = 0;
    *handle = w;
    return BITSTACK_OK;
}

int bitstack_push_block(bitstack_weight_t* w, const void* staging, bitstack_stream_t stream) {
    if (!w || !staging) return BITSTACK_E_NULL;
    const Geometry& g = w->geo;
    if (w->resident >= g.n) return BITSTACK_E_RANGE;
    const unsigned char* st = static_cast<const unsigned char*>(staging);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int i = w->resident;
    BS_HIP(hipMemcpyAsync(w->dev + g.off_blocks + size_t(i) * g.block_stride, st, g.block_stride,
                          hipMemcpyHostToDevice, hs));
    BS_HIP(hipMemcpyAsync(w->dev + g.off_vmax + size_t(i) * g.in * 2, st + align256(g.block_stride), size_t(g.in) * 2,
                          hipMemcpyHostToDevice, hs));
    w->resident = i + 1;
    return BITSTACK_OK;
}

int bitstack_push_block_device(bitstack_weight_t* w, const uint32_t* sign_words, const uint16_t* U, const uint16_t* V,
                               bitstack_stream_t stream) {
    if (!w || !sign_words || !U || !V) return BITSTACK_E_NULL;
    const Geometry& g = w->geo;
    if (w->resident >= g.n) return BITSTACK_E_RANGE;
    if (reinterpret_cast<uintptr_t>(sign_words) % 4 || reinterpret_cast<uintptr_t>(U) % 16 ||
        reinterpret_cast<uintptr_t>(V) % 2)
        return BITSTACK_E_ALIGN;
    hipError_t e = launch_pack_block_device(g, w->dev, w->resident, sign_words, U, V, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    ++w->resident;
    return BITSTACK_OK;
}

int bitstack_pop_block(bitstack_weight_t* w) {
    if (!w) return BITSTACK_E_NULL;
    if (w->resident < 1) return BITSTACK_E_RANGE;
    --w->resident;
    return BITSTACK_OK;
}

int bitstack_resident_blocks(const bitstack_weight_t* w) { return w ? w->resident : BITSTACK_E_NULL; }

size_t bitstack_resident_bytes(const bitstack_weight_t* w) {
    return w ? size_t(w->resident) * w->geo.block_stride : 0;
}

int bitstack_unpack_blocks(const bitstack_weight_t* w, int block, uint32_t* sign_words, uint16_t* U,
                           uint16_t* V, bitstack_stream_t stream) {
    if (!w) return BITSTACK_E_NULL;
    const Geometry& g = w->geo;
    if (block < 0 || block >= w->resident) return BITSTACK_E_RANGE;
    std::vector<unsigned char> buf;
    try {
        buf.resize(g.block_stride);
    } catch (const std::bad_alloc&) {
        return BITSTACK_E_BUFSIZE;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t off = g.off_blocks + size_t(block) * g.block_stride;
    BS_HIP(hipMemcpyAsync(buf.data(), w->dev + off, g.block_stride, hipMemcpyDeviceToHost, st));
    BS_HIP(hipStreamSynchronize(st));
    unpack_block(g, buf.data(), sign_words, U, V);
    return BITSTACK_OK;
}

int bitstack_weight_shape(const bitstack_weight_t* w, int* out, int* in, int* k, int* n, int* max_batch) {
    if (!w) return BITSTACK_E_NULL;
    if (out) *out = w->geo.out;
    if (in) *in = w->geo.in;
    if (k) *k = kRank;
    if (n) *n = w->geo.n;
    if (max_batch) *max_batch = w->geo.max_batch;
    return BITSTACK_OK;
}

// Which kernel serves (batch, n_loaded) fastest, from estimates that live beside the launchers
// (constants fitted to measurements on MI355X): the decode kernel with up to four tokens per
// launch streams the blocks once per token; the batch path rebuilds signed tiles per group of 32
// tokens (up to 64 tokens) or a weight tile once per 512 tokens; with a scratch buffer for the
// dense weight, restoring it once and one dense product wins for prefill-sized batches.
// Rows of the weight a scratch buffer of this size holds at a time on the materialising path
// (multiples of 256, the dense kernel's tile height; the whole matrix if it fits; 0: too small to
// be worth it -- below 1024 rows the dense product no longer fills the chip).
static int slab_rows(const Geometry& g, size_t workspace_bytes) {
    const size_t fit = workspace_bytes / (size_t(g.in) * 2);
    if (fit >= size_t(g.out)) return g.out;
    const int rows = int(fit / 256) * 256;
    return rows >= 1024 ? rows : 0;
}

// The scratch the materialising path works in: the caller's, or -- when none is lent or the image's
// is larger -- the image's own activation scratch, which only the weight-tile kernel uses (the
// dense product reads x in place).  Images packed for at most 64 tokens have none.
static size_t scratch_bytes(const Geometry& g, size_t workspace_bytes) {
    return workspace_bytes >= g.xpack_bytes ? workspace_bytes : g.xpack_bytes;
}

static int choose_kernel(const Geometry& g, int batch, int n_loaded, size_t workspace_bytes) {
    if (batch == 1) return BITSTACK_KERNEL_DECODE;
    workspace_bytes = scratch_bytes(g, workspace_bytes);
    const double t_decode = decode_tokens_time_us(g, batch, n_loaded);   // up to four tokens per launch
    double t_panel;
    if (batch <= kSmallBatch) {
        t_panel = fused_time_us(g.out, g.in, batch, n_loaded, g.part_slots);
        if (batch > 32 && g.xpack_bytes) {   // launch_panel takes the cheaper of the two here
            const double t_tile = tile_time_us(g.out, g.in, batch, n_loaded);
            t_panel = t_tile < t_panel ? t_tile : t_panel;
        }
    } else {
        t_panel = tile_time_us(g.out, g.in, batch, n_loaded);
    }
    int kernel = t_decode <= t_panel ? BITSTACK_KERNEL_DECODE : BITSTACK_KERNEL_PANEL;
    const double t_best = t_decode <= t_panel ? t_decode : t_panel;
    const int slab = slab_rows(g, workspace_bytes);
    // (the dense product addresses x and a slab of the dense weight with 32-bit byte offsets)
    const bool dense_ok = size_t(batch) * g.in * 2 <= 0xffffffffull && size_t(slab) * g.in * 2 <= 0xffffffffull;
    if (restore_fits(g.block_stride, n_loaded) && slab > 0 && dense_ok) {
        // per slab of rows: restore + product, two launches (~4 us each between kernels of one stream)
        double t_mat = 0.0;
        for (int r0 = 0; r0 < g.out; r0 += slab) {
            const int rows = slab < g.out - r0 ? slab : g.out - r0;
            t_mat += 8.0 + restore_time_us(rows, g.in, n_loaded, nullptr) + dense_time_us(rows, g.in, batch);
        }
        if (t_mat < t_best) kernel = BITSTACK_KERNEL_MATERIALISE;
    }
    return kernel;
}

int bitstack_choose_kernel(int out, int in, int n_slots, int max_batch, int batch, int n_loaded,
                           size_t workspace_bytes) {
    if (!shape_ok(out, in, kRank) || n_slots < 0 || max_batch < 1) return BITSTACK_E_SHAPE;
    if (batch < 1 || batch > max_batch || n_loaded < 0 || n_loaded > n_slots) return BITSTACK_E_RANGE;
    if (n_loaded == 0) return BITSTACK_KERNEL_AUTO;   // nothing to choose: y is cleared
    return choose_kernel(make_geometry(out, in, n_slots, max_batch), batch, n_loaded, workspace_bytes);
}

static int linear_impl(const void* x, int batch, const bitstack_weight_t* w, int n_loaded, void* y, int y_dtype,
                       int kernel, void* workspace, size_t workspace_bytes, bitstack_stream_t stream) {
    if (!x || !w || !y) return BITSTACK_E_NULL;
    const Geometry& g = w->geo;
    if (n_loaded < 0 || n_loaded > w->resident || batch < 1 || batch > g.max_batch) return BITSTACK_E_RANGE;
    if (y_dtype != BITSTACK_Y_F16 && y_dtype != BITSTACK_Y_F32) return BITSTACK_E_ARG;
    if (reinterpret_cast<uintptr_t>(x) % 16 || reinterpret_cast<uintptr_t>(y) % 16) return BITSTACK_E_ALIGN;
    if (workspace && reinterpret_cast<uintptr_t>(workspace) % 256) return BITSTACK_E_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    LaunchArgs a;
    a.x = x;
    a.y = y;
    a.image = w->dev;
    a.geo = g;
    a.batch = batch;
    a.n_loaded = n_loaded;
    a.y_f32 = (y_dtype == BITSTACK_Y_F32);
    hipError_t e = hipSuccess;
    if (n_loaded == 0) {
        e = launch_zero(a, st);
    } else {
        if (kernel == BITSTACK_KERNEL_AUTO) kernel = choose_kernel(g, batch, n_loaded, workspace ? workspace_bytes : 0);
        switch (kernel) {
            case BITSTACK_KERNEL_REFERENCE:
                e = launch_reference(a, st);
                break;
            case BITSTACK_KERNEL_DECODE:
                e = launch_decode_tokens(a, st);   // the decode kernel takes single activation vectors
                break;
            case BITSTACK_KERNEL_PANEL:
                e = launch_panel(a, st);
                break;
            case BITSTACK_KERNEL_MATERIALISE:
                if (!workspace || workspace_bytes < g.xpack_bytes) {   // the image's own scratch (see scratch_bytes)
                    if (!g.xpack_bytes) return BITSTACK_E_BUFSIZE;
                    workspace = w->dev + g.off_xpack;
                    workspace_bytes = g.xpack_bytes;
                }
                return bitstack_linear_materialised(x, batch, w, n_loaded, workspace, workspace_bytes, y, y_dtype, stream);
            default:
                return BITSTACK_E_ARG;
        }
    }
    if (e != hipSuccess) return hip_fail(e);
    return BITSTACK_OK;
}

int bitstack_linear_select(const void* x, int batch, const bitstack_weight_t* w, int n_loaded, void* y,
                           int y_dtype, int kernel, bitstack_stream_t stream) {
    return linear_impl(x, batch, w, n_loaded, y, y_dtype, kernel, nullptr, 0, stream);
}

int bitstack_linear_batched_ws(const void* x, int batch, const bitstack_weight_t* w, int n_loaded, void* y,
                               int y_dtype, void* workspace, size_t workspace_bytes, bitstack_stream_t stream) {
    return linear_impl(x, batch, w, n_loaded, y, y_dtype, BITSTACK_KERNEL_AUTO, workspace, workspace_bytes, stream);
}

int bitstack_linear_batched(const void* x, int batch, const bitstack_weight_t* w, int n_loaded, void* y,
                            int y_dtype, bitstack_stream_t stream) {
    return bitstack_linear_select(x, batch, w, n_loaded, y, y_dtype, BITSTACK_KERNEL_AUTO, stream);
}

int bitstack_linear(const void* x, const bitstack_weight_t* blocks, int n_loaded, void* y,
                    bitstack_stream_t stream) {
    return bitstack_linear_select(x, 1, blocks, n_loaded, y, BITSTACK_Y_F16, BITSTACK_KERNEL_AUTO, stream);
}

size_t bitstack_static_workspace_bytes(void) { return kStaticScratchBytes; }

int bitstack_linear_static(const void* x, const bitstack_weight_t* blocks, int n_loaded, void* y,
                           bitstack_stream_t stream) {
    if (!x || !blocks || !y) return BITSTACK_E_NULL;
    const Geometry& g = blocks->geo;
    if (n_loaded < 0 || n_loaded > blocks->resident) return BITSTACK_E_RANGE;
    if (reinterpret_cast<uintptr_t>(x) % 16 || reinterpret_cast<uintptr_t>(y) % 16) return BITSTACK_E_ALIGN;
    // the partial rows of even the coarsest work split must fit the static array
    if (size_t(g.out) * 4 * size_t((g.in / kChunkCols + kDecodeMaxRangeChunks - 1) / kDecodeMaxRangeChunks) > kStaticPartBytes)
        return BITSTACK_E_BUFSIZE;
    LaunchArgs a;
    a.x = x;
    a.y = y;
    a.image = blocks->dev;
    a.geo = g;
    a.batch = 1;
    a.n_loaded = n_loaded;
    a.y_f32 = false;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = n_loaded == 0 ? launch_zero(a, st) : launch_decode_static(a, st);
    if (e == hipErrorOutOfMemory) return BITSTACK_E_BUFSIZE;
    if (e != hipSuccess) return hip_fail(e);
    return BITSTACK_OK;
}

size_t bitstack_dense_bytes(int out, int in) {
    if (!shape_ok(out, in, kRank)) return 0;
    return size_t(out) * size_t(in) * 2;
}

int bitstack_restore_max_blocks(void) { return restore_max_blocks(); }

static int dense_args(const bitstack_weight_t* w, const void* w_dense, size_t w_dense_bytes, bool check_size) {
    if (!w || !w_dense) return BITSTACK_E_NULL;
    if (reinterpret_cast<uintptr_t>(w_dense) % 256) return BITSTACK_E_ALIGN;
    if (check_size && w_dense_bytes < size_t(w->geo.out) * size_t(w->geo.in) * 2) return BITSTACK_E_BUFSIZE;
    return BITSTACK_OK;
}

int bitstack_restore_weight(const bitstack_weight_t* w, int n_loaded, void* w_dense, size_t w_dense_bytes,
                            bitstack_stream_t stream) {
    int rc = dense_args(w, w_dense, w_dense_bytes, true);
    if (rc) return rc;
    if (n_loaded < 0 || n_loaded > w->resident || !restore_fits(w->geo.block_stride, n_loaded)) return BITSTACK_E_RANGE;
    LaunchArgs a;
    a.x = nullptr;
    a.y = nullptr;
    a.image = w->dev;
    a.geo = w->geo;
    a.batch = 1;
    a.n_loaded = n_loaded;
    a.y_f32 = false;
    a.wdense = w_dense;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = n_loaded == 0 ? launch_dense_zero(a, st) : launch_restore(a, st);
    if (e != hipSuccess) return hip_fail(e);
    return BITSTACK_OK;
}

int bitstack_linear_dense(const void* x, int batch, const bitstack_weight_t* w, const void* w_dense, void* y,
                          int y_dtype, bitstack_stream_t stream) {
    if (!x || !y) return BITSTACK_E_NULL;
    int rc = dense_args(w, w_dense, 0, false);
    if (rc) return rc;
    const Geometry& g = w->geo;
    if (batch < 1 || batch > g.max_batch) return BITSTACK_E_RANGE;
    if (y_dtype != BITSTACK_Y_F16 && y_dtype != BITSTACK_Y_F32) return BITSTACK_E_ARG;
    if (reinterpret_cast<uintptr_t>(x) % 16 || reinterpret_cast<uintptr_t>(y) % 16) return BITSTACK_E_ALIGN;
    LaunchArgs a;
    a.x = x;
    a.y = y;
    a.image = w->dev;
    a.geo = g;
    a.batch = batch;
    a.n_loaded = 0;
    a.y_f32 = (y_dtype == BITSTACK_Y_F32);
    a.wdense = const_cast<void*>(w_dense);
    hipError_t e = launch_dense(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return BITSTACK_OK;
}

int bitstack_linear_materialised(const void* x, int batch, const bitstack_weight_t* w, int n_loaded,
                                 void* w_dense, size_t w_dense_bytes, void* y, int y_dtype,
                                 bitstack_stream_t stream) {
    if (!x || !y) return BITSTACK_E_NULL;
    int rc = dense_args(w, w_dense, w_dense_bytes, false);
    if (rc) return rc;
    // every argument is checked before anything is enqueued
    const Geometry& g = w->geo;
    const int slab = slab_rows(g, w_dense_bytes);
    if (slab == 0) return BITSTACK_E_BUFSIZE;
    if (n_loaded < 0 || n_loaded > w->resident || !restore_fits(w->geo.block_stride, n_loaded)) return BITSTACK_E_RANGE;
    if (batch < 1 || batch > g.max_batch) return BITSTACK_E_RANGE;
    if (y_dtype != BITSTACK_Y_F16 && y_dtype != BITSTACK_Y_F32) return BITSTACK_E_ARG;
    if (reinterpret_cast<uintptr_t>(x) % 16 || reinterpret_cast<uintptr_t>(y) % 16) return BITSTACK_E_ALIGN;
    if (slab >= g.out) {
        rc = bitstack_restore_weight(w, n_loaded, w_dense, w_dense_bytes, stream);
        if (rc) return rc;
        return bitstack_linear_dense(x, batch, w, w_dense, y, y_dtype, stream);
    }
    // the scratch holds a slab of rows at a time: restore it, multiply it, next slab (stream order
    // keeps a slab's product ahead of the next restore that overwrites the scratch)
    LaunchArgs a;
    a.x = x;
    a.y = y;
    a.image = w->dev;
    a.geo = g;
    a.batch = batch;
    a.n_loaded = n_loaded;
    a.y_f32 = (y_dtype == BITSTACK_Y_F32);
    a.wdense = w_dense;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_loaded == 0) {
        hipError_t e = launch_zero(a, st);
        return e == hipSuccess ? BITSTACK_OK : hip_fail(e);
    }
    for (int r0 = 0; r0 < g.out; r0 += slab) {
        a.row_begin = r0;
        a.rows = slab;
        hipError_t e = launch_restore(a, st);
        if (e == hipSuccess) e = launch_dense(a, st);
        if (e != hipSuccess) return hip_fail(e);
    }
    return BITSTACK_OK;
}

size_t bitstack_decompose_workspace_bytes(int out, int in, int k) {
    if (!shape_ok(out, in, k)) return 0;
    return align256(size_t(in) * 4) + decompose_workspace_bytes(out, in, decompose_slices(out, in));
}

int bitstack_decompose(const float* W, const float* s, int out, int in, int k, int n, int iterations,
                       uint32_t* sign_words, uint16_t* U, uint16_t* V, void* workspace, size_t workspace_bytes,
                       bitstack_stream_t stream) {
    if (!W || !s || !sign_words || !U || !V || !workspace) return BITSTACK_E_NULL;
    if (!shape_ok(out, in, k)) return BITSTACK_E_SHAPE;
    if (n < 0 || iterations < 0 || iterations > 1000) return BITSTACK_E_RANGE;
    for (int j = 0; j < in; ++j)
        if (!std::isfinite(s[j]) || !(s[j] > 0.0f)) return BITSTACK_E_SCALE;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 || reinterpret_cast<uintptr_t>(W) % 16 ||
        reinterpret_cast<uintptr_t>(sign_words) % 4 || reinterpret_cast<uintptr_t>(U) % 2 ||
        reinterpret_cast<uintptr_t>(V) % 2)
        return BITSTACK_E_ALIGN;
    if (workspace_bytes < bitstack_decompose_workspace_bytes(out, in, k)) return BITSTACK_E_BUFSIZE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    BS_HIP(hipMemcpyAsync(ws, s, size_t(in) * 4, hipMemcpyHostToDevice, st));
    if (n == 0) return BITSTACK_OK;
    hipError_t e = launch_decompose(W, reinterpret_cast<const float*>(ws), out, in, n, iterations ? iterations : 16, sign_words,
                                    reinterpret_cast<__half*>(U), reinterpret_cast<__half*>(V),
                                    ws + align256(size_t(in) * 4), st);
    if (e != hipSuccess) return hip_fail(e);
    return BITSTACK_OK;
}

int bitstack_probe_read(const void* device_buf, size_t bytes, void* device_sink, int workgroups,
                        bitstack_stream_t stream) {
    if (!device_buf || !device_sink) return BITSTACK_E_NULL;
    if (reinterpret_cast<uintptr_t>(device_buf) % 16 || bytes % 16) return BITSTACK_E_ALIGN;
    if (workgroups < 1 || workgroups > (1 << 20)) return BITSTACK_E_RANGE;
    hipError_t e = launch_stream_read(device_buf, bytes, device_sink, workgroups, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return BITSTACK_OK;
}

int bitstack_set_option(int option, int value) {
    if (value < 0) return BITSTACK_E_ARG;
    switch (option) {
        case BITSTACK_OPT_DECODE_BGROUPS: decode_tuning().bgroups = value; return BITSTACK_OK;
        case BITSTACK_OPT_DECODE_TILES: decode_tuning().tiles = value; return BITSTACK_OK;
        case BITSTACK_OPT_DECODE_KS_CHUNKS: decode_tuning().ks_chunks = value; return BITSTACK_OK;
        case BITSTACK_OPT_DECODE_EARLY: decode_tuning().early = value - 1; return BITSTACK_OK;
        case BITSTACK_OPT_DENSE_TILE: dense_force_tile(value); return BITSTACK_OK;
        default: return BITSTACK_E_ARG;
    }
}

// can job j ride in the same decode launch as the jobs [first, j) before it?  Same input
// vector, non-empty stacks, aligned pointers on both sides, and no output of the group
// overlapping the input or another output (jobs of one launch run concurrently).
static bool can_join(const bitstack_job_t* jobs, int first, int j) {
    const bitstack_job_t& a = jobs[first];
    const bitstack_job_t& b = jobs[j];
    if (!a.x || !a.blocks || !a.y || !b.x || !b.blocks || !b.y) return false;
    if (b.x != a.x || b.blocks->geo.in != a.blocks->geo.in) return false;
    if (b.n_loaded < 1 || b.n_loaded > b.blocks->resident || a.n_loaded < 1 || a.n_loaded > a.blocks->resident) return false;
    if (reinterpret_cast<uintptr_t>(a.x) % 16 || reinterpret_cast<uintptr_t>(a.y) % 16 ||
        reinterpret_cast<uintptr_t>(b.y) % 16)
        return false;
    const char* x0 = static_cast<const char*>(a.x);
    const char* x1 = x0 + size_t(a.blocks->geo.in) * 2;
    for (int k = first; k <= j; ++k) {
        const char* y0 = static_cast<const char*>(jobs[k].y);
        const char* y1 = y0 + size_t(jobs[k].blocks->geo.out) * 2;
        if (y0 < x1 && x0 < y1) return false;
        for (int m = first; m < k; ++m) {   // two jobs of a launch must not share a stack (its workspace) or an output
            if (jobs[m].blocks == jobs[k].blocks) return false;
            const char* z0 = static_cast<const char*>(jobs[m].y);
            const char* z1 = z0 + size_t(jobs[m].blocks->geo.out) * 2;
            if (y0 < z1 && z0 < y1) return false;
        }
    }
    return true;
}

static LaunchArgs job_args(const bitstack_job_t& jb) {
    LaunchArgs a;
    a.x = jb.x;
    a.y = jb.y;
    a.image = jb.blocks->dev;
    a.geo = jb.blocks->geo;
    a.batch = 1;
    a.n_loaded = jb.n_loaded;
    a.y_f32 = false;
    return a;
}

// length of the run of jobs starting at i that go out as one decode launch (1: a call of its own)
static int group_length(const bitstack_job_t* jobs, int count, int i) {
    int len = 1;
    while (i + len < count && len < kMaxGroup && can_join(jobs, i, i + len)) ++len;
    if (len > 1) {
        // a joint work split must fit the members' workspaces; else the jobs go out one by one
        LaunchArgs a[kMaxGroup];
        for (int k = 0; k < len; ++k) a[k] = job_args(jobs[i + k]);
        DecodeLaunch d;
        if (prepare_decode_group(a, len, &d) != hipSuccess) len = 1;
    }
    return len;
}

int bitstack_linear_many(const bitstack_job_t* jobs, int count, int repeat, bitstack_stream_t stream) {
    if (!jobs) return BITSTACK_E_NULL;
    if (count < 0 || repeat < 0) return BITSTACK_E_RANGE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (int r = 0; r < repeat; ++r) {
        int i = 0;
        while (i < count) {
            const int len = group_length(jobs, count, i);
            if (len > 1) {
                LaunchArgs a[kMaxGroup];
                for (int k = 0; k < len; ++k) a[k] = job_args(jobs[i + k]);
                hipError_t e = launch_decode_group(a, len, st);
                if (e != hipSuccess) return hip_fail(e);
            } else {
                int rc = bitstack_linear(jobs[i].x, jobs[i].blocks, jobs[i].n_loaded, jobs[i].y, stream);
                if (rc) return rc;
            }
            i += len;
        }
    }
    return BITSTACK_OK;
}

// ---- a token plan: the job list of bitstack_linear_many with grouping, work splits and kernel
// arguments worked out once
struct bitstack_plan {
    struct Step {
        bool zero;        // y = 0 (no block loaded)
        LaunchArgs za;    // for zero
        DecodeLaunch d;   // else
    };
    std::vector<Step> steps;
    std::vector<bitstack_job_t> jobs;   // kept to check at launch that the stacks still hold the blocks
};

int bitstack_plan_create(const bitstack_job_t* jobs, int count, bitstack_plan_t** handle) {
    if (!handle) return BITSTACK_E_NULL;
    *handle = nullptr;
    if (!jobs) return BITSTACK_E_NULL;
    if (count < 0) return BITSTACK_E_RANGE;
    for (int i = 0; i < count; ++i) {   // the checks of bitstack_linear, for every job, before anything is built
        const bitstack_job_t& jb = jobs[i];
        if (!jb.x || !jb.blocks || !jb.y) return BITSTACK_E_NULL;
        if (jb.n_loaded < 0 || jb.n_loaded > jb.blocks->resident) return BITSTACK_E_RANGE;
        if (reinterpret_cast<uintptr_t>(jb.x) % 16 || reinterpret_cast<uintptr_t>(jb.y) % 16) return BITSTACK_E_ALIGN;
    }
    bitstack_plan* pl = new (std::nothrow) bitstack_plan;
    if (!pl) return BITSTACK_E_BUFSIZE;
    try {
        pl->jobs.assign(jobs, jobs + count);
        int i = 0;
        while (i < count) {
            const int len = group_length(jobs, count, i);
            pl->steps.emplace_back();
            bitstack_plan::Step& s = pl->steps.back();
            LaunchArgs a[kMaxGroup];
            for (int k = 0; k < len; ++k) a[k] = job_args(jobs[i + k]);
            s.zero = len == 1 && jobs[i].n_loaded == 0;
            if (s.zero) {
                s.za = a[0];
            } else {
                const hipError_t e = prepare_decode_group(a, len, &s.d);
                if (e != hipSuccess) {
                    delete pl;
                    return hip_fail(e);
                }
            }
            i += len;
        }
    } catch (const std::bad_alloc&) {
        delete pl;
        return BITSTACK_E_BUFSIZE;
    }
    *handle = pl;
    return BITSTACK_OK;
}

int bitstack_plan_launch(const bitstack_plan_t* plan, bitstack_stream_t stream) {
    if (!plan) return BITSTACK_E_NULL;
    for (const bitstack_job_t& jb : plan->jobs)
        if (jb.n_loaded > jb.blocks->resident) return BITSTACK_E_RANGE;   // a block of the plan has been offloaded
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (const bitstack_plan::Step& s : plan->steps) {
        const hipError_t e = s.zero ? launch_zero(s.za, st) : run_decode_launch(s.d, st);
        if (e != hipSuccess) return hip_fail(e);
    }
    return BITSTACK_OK;
}

int bitstack_plan_steps(const bitstack_plan_t* plan) { return plan ? int(plan->steps.size()) : BITSTACK_E_NULL; }

void bitstack_plan_release(bitstack_plan_t* plan) { delete plan; }

void bitstack_release(bitstack_weight_t* w) { delete w; }

const char* bitstack_strerror(int code) {
    switch (code) {
        case BITSTACK_OK: return "ok";
        case BITSTACK_E_NULL: return "null pointer argument";
        case BITSTACK_E_SHAPE: return "unsupported shape (need k == 16, in % 256 == 0, out % 32 == 0)";
        case BITSTACK_E_RANGE: return "n_loaded, batch or block index out of range";
        case BITSTACK_E_ALIGN: return "misaligned device pointer";
        case BITSTACK_E_SCALE: return "scale vector entry not finite or not positive";
        case BITSTACK_E_BUFSIZE: return "buffer too small";
        case BITSTACK_E_HIP: return "HIP runtime error (see bitstack_last_hip_error)";
        case BITSTACK_E_ARG: return "invalid dtype or kernel selector";
        default: return "unknown error code";
    }
}

int bitstack_last_hip_error(void) { return g_last_hip; }

}  // extern "C"
