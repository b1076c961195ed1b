// C ABI of the library (declared in include/nvfp4.h): argument validation on the host,
// workspace layout, and the composition of kernels into the fused linear entries.
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <initializer_list>
#include <mutex>

#include "kernels.h"
#include "nvfp4_math.h"

using namespace nvfp4;

// Scratch of nvfp4_quantize_static (the entry point for callers that cannot allocate): the workspace that
// nvfp4_quantize takes as an argument -- header plus per-workgroup partial maxima -- as one array per GPU in the
// library's own image.  Host code never uses this name as an address: static_scratch() asks the runtime for the
// array's device address once per device and everything else goes through that pointer.
constexpr size_t STATIC_SCRATCH_BYTES = 256 + 4 * 16384;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t WS_ALIGN = 256;
constexpr size_t WS_HEADER = 256;  // tensor scales and maxima live at the front of a workspace
constexpr int64_t MAX_CONTRACTION = (int64_t)1 << 23;  // the GEMM kernels keep 32-bit byte offsets inside a 256-row tile

inline size_t align_up(size_t n) { return (n + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN; }
// Bytes of an internal packed operand of `rows` rows and contraction length K: rows padded to whole slabs, so
// that the buffer can hold either the plain or the slab layout.
inline size_t op_codes(int64_t rows, int64_t K) { return align_up((size_t)slab_rows_padded(rows) * K / 2); }
inline size_t op_scales(int64_t rows, int64_t K, int64_t block) { return align_up((size_t)slab_rows_padded(rows) * (K / block)); }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elem_size(int dt) { return dt == NVFP4_BF16 ? 2 : 4; }
inline bool valid_dtype(int dt) { return dt == NVFP4_F32 || dt == NVFP4_BF16; }
// An enumeration argument of the C ABI as the integer the caller passed (C callers and foreign-function interfaces
// pass plain ints, possibly outside the enumeration: the bytes are read, never an out-of-range enumeration value).
template <class E>
inline int raw(const E &e)
{
    static_assert(sizeof(E) == sizeof(int), "C enumerations of this ABI are int-sized");
    int v;
    memcpy(&v, &e, sizeof(v));
    return v;
}

nvfp4_status check_format(const nvfp4_format *f)
{
    if (!f) return NVFP4_EINVAL;
    if (f->scale != NVFP4_SCALE_E4M3 && f->scale != NVFP4_SCALE_E8M0) return NVFP4_EINVAL;
    if (f->tensor_scale != 0 && f->tensor_scale != 1) return NVFP4_EINVAL;
    if (f->block != 16 && f->block != 32 && f->block != 64 && f->block != 128) return NVFP4_EUNSUPPORTED;
    if (f->scale == NVFP4_SCALE_E8M0 && f->tensor_scale) return NVFP4_EUNSUPPORTED;
    return NVFP4_OK;
}

// Two cross-check switches, neither of which changes a result bit.  They are taken from the environment once,
// at the first call that needs them, and can be replaced by nvfp4_cross_check_switches() (tests flip them inside
// one process).  Bit 0: round elements and block scales with the integer/fp32 formulation (the one the host probes
// evaluate) instead of the gfx950 convert instructions.  Bit 1: keep the packed operands inside the fused linear
// entries row-major instead of in the slab layout (kernels.h).
// Bit 2: GEMMs with E4M3 scales at blocks of 64 / 128 (K a multiple of 128) run on the FP4 matrix instruction with binary32
// rescaling of the block sums instead of expanding their operands to fp16 like NVFP4 (same results to rounding order; the
// measured slower route, kept selectable as the reference for that measurement).
constexpr uint32_t SW_SOFT_CONVERT = 1u, SW_PLAIN_OPERANDS = 2u, SW_FP4_WIDE_BLOCKS = 4u, SW_ALL = 7u, SW_UNREAD = 0x80000000u;
std::atomic<uint32_t> g_switches{SW_UNREAD};

uint32_t switches()
{
    uint32_t v = g_switches.load(std::memory_order_relaxed);
    if (v == SW_UNREAD) {
        const char *a = getenv("NVFP4_SOFT_CONVERT"), *b = getenv("NVFP4_PLAIN_OPERANDS"), *c = getenv("NVFP4_FP4_WIDE_BLOCKS");
        v = ((a && a[0] == '1') ? SW_SOFT_CONVERT : 0u) | ((b && b[0] == '1') ? SW_PLAIN_OPERANDS : 0u) |
            ((c && c[0] == '1') ? SW_FP4_WIDE_BLOCKS : 0u);
        g_switches.store(v, std::memory_order_relaxed);
        set_fp4_rescale_route((v & SW_FP4_WIDE_BLOCKS) != 0);
    }
    return v;
}
bool use_hw_convert() { return (switches() & SW_SOFT_CONVERT) == 0; }
bool use_slabs() { return (switches() & SW_PLAIN_OPERANDS) == 0; }

// A dense [rows, cols] tensor goes through the one-pass dual quantizer (the only writer of slabs) with these
// roundings; its answer does not depend on the element type for shapes the linear entries accept.
bool dual_writes_slabs(const nvfp4_format *f, int dt, int64_t rows, int64_t cols, int rnd_r, int rnd_c)
{
    const bool slab_format = (f->block == 16 && f->scale == NVFP4_SCALE_E4M3) || (f->block == 32 && f->scale == NVFP4_SCALE_E8M0);
    return use_slabs() && slab_format &&
           quantize_dual_fused(dt, rows, cols, cols, f->block, use_hw_convert()) && !(rnd_r == NVFP4_SR && rnd_c == NVFP4_RTN);
}

// An empty tensor (rows or cols 0) may come with a null data pointer.
nvfp4_status check_tensor(const void *x, int dt, int64_t rows, int64_t cols, int64_t ld)
{
    if (!valid_dtype(dt)) return NVFP4_EINVAL;
    if (rows < 0 || cols < 0 || ld < cols) return NVFP4_ESHAPE;
    if (!x && rows > 0 && cols > 0) return NVFP4_EINVAL;
    if (!aligned16(x) || (ld * elem_size(dt)) % 16 != 0) return NVFP4_EALIGN;
    return NVFP4_OK;
}

struct QuantPlan {
    const void *x;
    int dt;
    int64_t rows, cols, ld;
    int axis, rounding;
    uint64_t seed;
    uint8_t *codes, *scales;
    const float *g_src;
    float *g_out;
    int g_mode;
    int n_partials = 0;
};

// Where a quantizer finds the tensor maximum: one folded bit pattern (n == 0) or n partial maxima.
struct GSource {
    const float *src;
    int n;
};
constexpr size_t PARTIAL_SLOT = 4 * (size_t)AMAX_DENSE_PARTIALS;  // bytes of one tensor's partial maxima

// Maximum pass over a dense tensor into slot `slot` of the workspace's partials area; the
// quantizers fold the partials themselves, so no fold kernel runs between the two.
hipError_t amax_dense(const void *x, int dt, int64_t n_elements, uint32_t *partials, int slot, hipStream_t st, GSource *g)
{
    uint32_t *dst = partials + slot * AMAX_DENSE_PARTIALS;
    g->src = reinterpret_cast<const float *>(dst);
    return launch_tensor_amax_dense(x, dt, n_elements, dst, &g->n, st);
}

hipError_t run_quantize(const QuantPlan &q, const nvfp4_format *f, hipStream_t st)
{
    QuantArgs a;
    a.x = q.x;
    a.rows = q.rows;
    a.cols = q.cols;
    a.ld = q.ld;
    a.codes = q.codes;
    a.scales = q.scales;
    a.g_src = q.g_src;
    a.g_out = q.g_out;
    a.g_mode = q.g_mode;
    a.seed = q.seed;
    a.n_partials = q.n_partials;
    return launch_quantize(a, q.dt, q.axis, q.rounding, f->block, f->scale, use_hw_convert(), st);
}

// What nvfp4_linear_fwd leaves for nvfp4_linear_bwd: {gX, gW}, then the transposed operands.
struct SavedLayout {
    float *g;
    uint8_t *xtc, *xts, *wtc, *wts;
};

SavedLayout saved_layout(void *saved, int64_t M, int64_t N, int64_t K, int64_t B)
{
    uint8_t *p = reinterpret_cast<uint8_t *>(saved);
    SavedLayout L;
    L.g = reinterpret_cast<float *>(p);
    p += WS_HEADER;
    L.xtc = p; p += op_codes(K, M);
    L.xts = p; p += op_scales(K, M, B);
    L.wtc = p; p += op_codes(K, N);
    L.wts = p;
    return L;
}

// Identity of a `saved` buffer: shapes, format, seed and the layout each transposed operand was written in.
constexpr size_t SAVED_TAG_OFFSET = 64;  // bytes into the header; {gX, gW} sit at its front
TagArgs saved_tag(int64_t M, int64_t N, int64_t K, const nvfp4_format *f, uint64_t seed, bool xt_slab, bool wt_slab,
                  bool x_only = false)
{
    TagArgs t;
    t.w[0] = 0x4E564634u;  // "NVF4"
    t.w[1] = (xt_slab ? 1u : 0u) | (wt_slab ? 2u : 0u) | (use_hw_convert() ? 4u : 0u) | (x_only ? 8u : 0u);
    t.w[2] = (uint32_t)f->block | ((uint32_t)f->scale << 8) | ((uint32_t)f->tensor_scale << 9);
    t.w[3] = (uint32_t)M;
    t.w[4] = (uint32_t)N;
    t.w[5] = (uint32_t)K;
    t.w[6] = (uint32_t)seed;
    t.w[7] = (uint32_t)(seed >> 32);
    return t;
}

// What nvfp4_quantize_weight leaves for the forward and backward calls of every micro-batch: gW, then W blocked
// along K (operand of Eq. 4) and W^T blocked along N (operand of Eq. 5).
struct WeightLayout {
    float *g;
    uint8_t *wc, *wsc, *wtc, *wts;
};

WeightLayout weight_layout(const void *w_operands, int64_t N, int64_t K, int64_t B)
{
    uint8_t *p = reinterpret_cast<uint8_t *>(const_cast<void *>(w_operands));
    WeightLayout L;
    L.g = reinterpret_cast<float *>(p);
    p += WS_HEADER;
    L.wc = p; p += op_codes(N, K);
    L.wsc = p; p += op_scales(N, K, B);
    L.wtc = p; p += op_codes(K, N);
    L.wts = p;
    return L;
}

// Layout of the two weight operands for micro-batches of M tokens: slabs where the GEMM that consumes them takes them.
void weight_slabs(const nvfp4_format *f, int64_t M, int64_t N, int64_t K, bool *w_slab, bool *wt_slab)
{
    const bool sw = dual_writes_slabs(f, NVFP4_BF16, N, K, NVFP4_RTN, NVFP4_RTN);  // (does not depend on the element type)
    *w_slab = sw && gemm_takes_slabs(M, N, K, f->block, f->scale);
    *wt_slab = sw && gemm_takes_slabs(M, K, N, f->block, f->scale);
}

TagArgs weight_tag(int64_t M, int64_t N, int64_t K, const nvfp4_format *f)
{
    bool w_slab, wt_slab;
    weight_slabs(f, M, N, K, &w_slab, &wt_slab);
    TagArgs t = saved_tag(M, N, K, f, 0, w_slab, wt_slab);
    t.w[0] = 0x4E565734u;  // "NVW4"
    return t;
}

// Host-side record of the last forward calls' `saved` buffers (address -> tag), so that a backward call whose
// shapes, format, seed or operand layouts differ from what the forward call wrote is refused before anything is
// launched.  A buffer the table does not know (written more than SAVED_SLOTS forward calls ago) is trusted; the
// tag in the buffer's own header then still poisons the outputs on a mismatch (TagArgs).
constexpr int SAVED_SLOTS = 256;
struct SavedRecord {
    const void *ptr = nullptr;
    uint32_t w[8];
};
SavedRecord g_saved[SAVED_SLOTS];
int g_saved_next = 0;
std::mutex g_saved_mutex;

void saved_remember(const void *ptr, const TagArgs &t)
{
    std::lock_guard<std::mutex> lock(g_saved_mutex);
    int slot = -1;
    for (int i = 0; i < SAVED_SLOTS; ++i)
        if (g_saved[i].ptr == ptr) slot = i;
    if (slot < 0) {
        slot = g_saved_next;
        g_saved_next = (g_saved_next + 1) % SAVED_SLOTS;
    }
    g_saved[slot].ptr = ptr;
    memcpy(g_saved[slot].w, t.w, sizeof(t.w));
}

// false only if the buffer is known and was written for something else
bool saved_matches(const void *ptr, const TagArgs &t)
{
    std::lock_guard<std::mutex> lock(g_saved_mutex);
    for (int i = 0; i < SAVED_SLOTS; ++i)
        if (g_saved[i].ptr == ptr) return memcmp(g_saved[i].w, t.w, sizeof(t.w)) == 0;
    return true;
}

// Device address of `scratch` on the current device (each GPU holds its own copy at its own address).
constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;

nvfp4_status static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return NVFP4_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return NVFP4_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return NVFP4_OK;
}

// Scratch bytes nvfp4_quantize really touches for this tensor: a dense tensor leaves at most AMAX_DENSE_PARTIALS
// partial maxima, a strided one one per 8192-element span of a row.
size_t quantize_scratch_need(int64_t rows, int64_t cols, int64_t ld)
{
    if (rows <= 0 || cols <= 0 || ld == cols) return WS_HEADER + PARTIAL_SLOT;
    return WS_HEADER + 4 * (size_t)tensor_amax_partials(rows, cols, ld);
}

nvfp4_status quantize_impl(const void *x, int dt, int64_t rows, int64_t cols, int64_t ld, int axis,
                           int rounding, uint64_t seed, const nvfp4_format *f, uint8_t *codes,
                           uint8_t *scales, float *tensor_scale, uint32_t flags, void *workspace,
                           size_t workspace_bytes, size_t workspace_required, void *stream, bool validate_only = false);

}  // namespace

extern "C" {

uint32_t nvfp4_cross_check_switches(int set, uint32_t value)
{
    const uint32_t before = switches();
    if (set) {
        g_switches.store(value & SW_ALL, std::memory_order_relaxed);
        set_fp4_rescale_route((value & SW_FP4_WIDE_BLOCKS) != 0);
    }
    return before;
}

const char *nvfp4_status_string(nvfp4_status s)
{
    // (a C caller may hand over any integer: read the argument's bytes, not an enumeration value)
    int code;
    memcpy(&code, &s, sizeof(code));
    switch (code) {
    case NVFP4_OK: return "ok";
    case NVFP4_EINVAL: return "invalid argument";
    case NVFP4_ESHAPE: return "invalid shape";
    case NVFP4_EALIGN: return "misaligned pointer or leading dimension";
    case NVFP4_EUNSUPPORTED: return "unsupported format";
    case NVFP4_EWORKSPACE: return "workspace missing or too small";
    case NVFP4_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

size_t nvfp4_codes_bytes(int64_t rows, int64_t cols)
{
    if (rows <= 0 || cols <= 0) return 0;
    return (size_t)rows * (size_t)cols / 2;
}

size_t nvfp4_scales_bytes(int64_t rows, int64_t cols, int axis, const nvfp4_format *f)
{
    if (rows <= 0 || cols <= 0 || check_format(f) != NVFP4_OK || (axis != 0 && axis != 1)) return 0;
    return axis == 1 ? (size_t)rows * (size_t)(cols / f->block) : (size_t)cols * (size_t)(rows / f->block);
}

// bytes of per-workgroup partial maxima for one tensor (sized for the strided case, which
// needs at least as many as the dense one)
static size_t partials_bytes(int64_t rows, int64_t cols)
{
    if (rows <= 0 || cols <= 0) return align_up(3 * PARTIAL_SLOT);
    const size_t strided = align_up(4 * (size_t)tensor_amax_partials(rows, cols, cols + 8));
    return strided > 3 * PARTIAL_SLOT ? strided : align_up(3 * PARTIAL_SLOT);  // up to three dense tensors side by side
}

size_t nvfp4_quantize_workspace_bytes(int64_t rows, int64_t cols) { return WS_HEADER + partials_bytes(rows, cols); }

size_t nvfp4_linear_fwd_workspace_bytes(int64_t M, int64_t N, int64_t K, const nvfp4_format *f)
{
    if (M <= 0 || N <= 0 || K <= 0 || check_format(f) != NVFP4_OK) return 0;
    const size_t part = partials_bytes(M, K) > partials_bytes(N, K) ? partials_bytes(M, K) : partials_bytes(N, K);
    return WS_HEADER + part + op_codes(M, K) + op_scales(M, K, f->block) +
           op_codes(N, K) + op_scales(N, K, f->block);
}

size_t nvfp4_linear_saved_bytes(int64_t M, int64_t N, int64_t K, const nvfp4_format *f)
{
    if (M <= 0 || N <= 0 || K <= 0 || check_format(f) != NVFP4_OK) return 0;
    const size_t B = (size_t)f->block;
    return WS_HEADER + op_codes(K, M) + op_scales(K, M, B) +  // X^T blocked along M
           op_codes(K, N) + op_scales(K, N, B);               // W^T blocked along N
}

size_t nvfp4_linear_bwd_workspace_bytes(int64_t M, int64_t N, int64_t K, const nvfp4_format *f)
{
    if (M <= 0 || N <= 0 || K <= 0 || check_format(f) != NVFP4_OK) return 0;
    const size_t B = (size_t)f->block;
    size_t part = partials_bytes(M, N);
    if (partials_bytes(N, K) > part) part = partials_bytes(N, K);
    if (partials_bytes(M, K) > part) part = partials_bytes(M, K);
    return WS_HEADER + part +
           op_codes(M, N) + op_scales(M, N, B) +  // dY blocked along N
           op_codes(K, N) + op_scales(K, N, B) +  // W^T blocked along N
           op_codes(N, M) + op_scales(N, M, B) +  // dY^T blocked along M
           op_codes(K, M) + op_scales(K, M, B);   // X^T blocked along M
}

nvfp4_status nvfp4_tensor_scale(const void *x, nvfp4_dtype dt_, int64_t rows, int64_t cols,
                                int64_t ld, float *tensor_scale, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    const int dt = raw(dt_);
    nvfp4_status s = check_tensor(x, dt, rows, cols, ld);
    if (s != NVFP4_OK) return s;
    if (!tensor_scale) return NVFP4_EINVAL;
    if (!workspace || workspace_bytes < nvfp4_quantize_workspace_bytes(rows, cols)) return NVFP4_EWORKSPACE;
    if (!aligned16(workspace)) return NVFP4_EALIGN;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    uint32_t *bits = reinterpret_cast<uint32_t *>(workspace);
    uint32_t *partials = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(workspace) + WS_HEADER);
    if (launch_tensor_amax(x, dt, rows, cols, ld, bits, partials, tensor_scale, st) != hipSuccess) return NVFP4_EHIP;
    return NVFP4_OK;
}

nvfp4_status nvfp4_quantize(const void *x, nvfp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                            int axis, nvfp4_rounding rounding, uint64_t seed,
                            const nvfp4_format *f, uint8_t *codes, uint8_t *scales,
                            float *tensor_scale, uint32_t flags, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    return quantize_impl(x, raw(dt), rows, cols, ld, axis, raw(rounding), seed, f, codes, scales, tensor_scale, flags, workspace,
                         workspace_bytes, nvfp4_quantize_workspace_bytes(rows, cols), stream);
}

nvfp4_status nvfp4_quantize_static(const void *x, nvfp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                                   int axis, nvfp4_rounding rounding, uint64_t seed,
                                   const nvfp4_format *f, uint8_t *codes, uint8_t *scales,
                                   float *tensor_scale, uint32_t flags, void *stream)
{
    // (a shape whose partial maxima do not fit the array is refused here, before the device is touched)
    if (rows > 0 && cols > 0 && ld >= cols && quantize_scratch_need(rows, cols, ld) > STATIC_SCRATCH_BYTES) return NVFP4_EWORKSPACE;
    // (arguments are checked before the device is asked for the array's address)
    void *ws = reinterpret_cast<void *>(WS_ALIGN);
    nvfp4_status s = quantize_impl(x, raw(dt), rows, cols, ld, axis, raw(rounding), seed, f, codes, scales, tensor_scale, flags, ws,
                                   STATIC_SCRATCH_BYTES, quantize_scratch_need(rows, cols, ld), stream, true);
    if (s != NVFP4_OK) return s;
    s = static_scratch(&ws);
    if (s != NVFP4_OK) return s;
    return quantize_impl(x, raw(dt), rows, cols, ld, axis, raw(rounding), seed, f, codes, scales, tensor_scale, flags, ws,
                         STATIC_SCRATCH_BYTES, quantize_scratch_need(rows, cols, ld), stream);
}

}  // extern "C"

namespace {

nvfp4_status quantize_impl(const void *x, int dt, int64_t rows, int64_t cols, int64_t ld, int axis,
                           int rounding, uint64_t seed, const nvfp4_format *f, uint8_t *codes,
                           uint8_t *scales, float *tensor_scale, uint32_t flags, void *workspace,
                           size_t workspace_bytes, size_t workspace_required, void *stream, bool validate_only)
{
    nvfp4_status s = check_format(f);
    if (s != NVFP4_OK) return s;
    s = check_tensor(x, dt, rows, cols, ld);
    if (s != NVFP4_OK) return s;
    const bool empty = rows == 0 || cols == 0;
    if (!tensor_scale || (!empty && (!codes || !scales))) return NVFP4_EINVAL;
    if (axis != 0 && axis != 1) return NVFP4_EINVAL;
    if (rounding != NVFP4_RTN && rounding != NVFP4_SR) return NVFP4_EINVAL;
    if (flags & ~NVFP4_PRESET_TSCALE) return NVFP4_EINVAL;
    const int64_t inner = axis == 1 ? cols : rows;
    if (inner % f->block != 0) return NVFP4_ESHAPE;
    if (!aligned16(codes) || !aligned16(scales)) return NVFP4_EALIGN;
    const bool preset = (flags & NVFP4_PRESET_TSCALE) != 0;
    const bool need_amax = f->tensor_scale && !preset;
    if (need_amax) {
        if (!workspace || workspace_bytes < workspace_required) return NVFP4_EWORKSPACE;
        if (!aligned16(workspace)) return NVFP4_EALIGN;
    }
    if (validate_only) return NVFP4_OK;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);

    QuantPlan q{x, dt, rows, cols, ld, axis, rounding, seed, codes, scales, tensor_scale, tensor_scale, G_NONE};
    if (f->tensor_scale) {
        if (preset) {
            q.g_mode = G_PRESET;
        } else {
            uint32_t *bits = reinterpret_cast<uint32_t *>(workspace);
            uint32_t *partials = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(workspace) + WS_HEADER);
            q.g_src = reinterpret_cast<const float *>(bits);
            q.g_mode = G_FROM_AMAX;
            if (!empty && ld == cols) {
                GSource g;
                if (amax_dense(x, dt, rows * cols, partials, 0, st, &g) != hipSuccess) return NVFP4_EHIP;
                q.g_src = g.src;
                q.n_partials = g.n;
            } else if (launch_tensor_amax(x, dt, rows, cols, ld, bits, partials, empty ? tensor_scale : nullptr, st) != hipSuccess) {
                // (an empty tensor gets its scale (1) written there, by the fold alone; otherwise the quantizer writes it)
                return NVFP4_EHIP;
            }
        }
    }
    if (empty) return NVFP4_OK;  // nothing to encode
    return run_quantize(q, f, st) == hipSuccess ? NVFP4_OK : NVFP4_EHIP;
}

}  // namespace

extern "C" {

nvfp4_status nvfp4_quantize_dual(const void *x, nvfp4_dtype dt_, int64_t rows, int64_t cols, int64_t ld,
                                 nvfp4_rounding rounding_rows_, uint64_t seed_rows,
                                 nvfp4_rounding rounding_cols_, uint64_t seed_cols,
                                 const nvfp4_format *f, uint8_t *codes_rows, uint8_t *scales_rows,
                                 uint8_t *codes_cols, uint8_t *scales_cols, float *tensor_scale,
                                 uint32_t flags, void *workspace, size_t workspace_bytes, void *stream)
{
    const int dt = raw(dt_);
    const int rounding_rows = raw(rounding_rows_);
    const int rounding_cols = raw(rounding_cols_);
    nvfp4_status s = check_format(f);
    if (s != NVFP4_OK) return s;
    s = check_tensor(x, dt, rows, cols, ld);
    if (s != NVFP4_OK) return s;
    const bool empty = rows == 0 || cols == 0;
    if (!tensor_scale || (!empty && (!codes_rows || !scales_rows || !codes_cols || !scales_cols))) return NVFP4_EINVAL;
    if (rounding_rows != NVFP4_RTN && rounding_rows != NVFP4_SR) return NVFP4_EINVAL;
    if (rounding_cols != NVFP4_RTN && rounding_cols != NVFP4_SR) return NVFP4_EINVAL;
    if (flags & ~(NVFP4_PRESET_TSCALE | NVFP4_SLAB_ROWS | NVFP4_SLAB_COLS)) return NVFP4_EINVAL;
    if (rows % f->block != 0 || cols % f->block != 0) return NVFP4_ESHAPE;
    if (!aligned16(codes_rows) || !aligned16(scales_rows) || !aligned16(codes_cols) || !aligned16(scales_cols))
        return NVFP4_EALIGN;
    const bool slab_r = (flags & NVFP4_SLAB_ROWS) != 0, slab_c = (flags & NVFP4_SLAB_COLS) != 0;
    if (slab_r || slab_c) {
        // only the one-pass kernel writes slabs
        const bool slab_format = (f->block == 16 && f->scale == NVFP4_SCALE_E4M3) || (f->block == 32 && f->scale == NVFP4_SCALE_E8M0);
        if (!slab_format || !use_hw_convert() ||
            !quantize_dual_fused(dt, rows, cols, ld, f->block, true) || (rounding_rows == NVFP4_SR && rounding_cols == NVFP4_RTN))
            return NVFP4_EUNSUPPORTED;
        if ((slab_r && cols % SLAB_K != 0) || (slab_c && rows % SLAB_K != 0)) return NVFP4_ESHAPE;
    }
    const bool preset = (flags & NVFP4_PRESET_TSCALE) != 0;
    const bool need_amax = f->tensor_scale && !preset;
    if (need_amax) {
        if (!workspace || workspace_bytes < nvfp4_quantize_workspace_bytes(rows, cols)) return NVFP4_EWORKSPACE;
        if (!aligned16(workspace)) return NVFP4_EALIGN;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);

    DualArgs d;
    d.c.x = x;
    d.c.rows = rows;
    d.c.cols = cols;
    d.c.ld = ld;
    d.c.codes = codes_cols;
    d.c.scales = scales_cols;
    d.c.g_src = tensor_scale;
    d.c.g_out = tensor_scale;
    d.c.g_mode = G_NONE;
    d.c.seed = seed_cols;
    d.codes_r = codes_rows;
    d.scales_r = scales_rows;
    d.seed_r = seed_rows;
    d.g_out2 = nullptr;
    d.slab_r = slab_r;
    d.slab_c = slab_c;
    if (f->tensor_scale) {
        if (preset) {
            d.c.g_mode = G_PRESET;
        } else {
            uint32_t *bits = reinterpret_cast<uint32_t *>(workspace);
            uint32_t *partials = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(workspace) + WS_HEADER);
            d.c.g_src = reinterpret_cast<const float *>(bits);
            d.c.g_mode = G_FROM_AMAX;
            if (!empty && ld == cols) {
                GSource g;
                if (amax_dense(x, dt, rows * cols, partials, 0, st, &g) != hipSuccess) return NVFP4_EHIP;
                d.c.g_src = g.src;
                d.c.n_partials = g.n;
            } else if (launch_tensor_amax(x, dt, rows, cols, ld, bits, partials, empty ? tensor_scale : nullptr, st) != hipSuccess) {
                return NVFP4_EHIP;
            }
        }
    }
    if (empty) return NVFP4_OK;
    return launch_quantize_dual(d, dt, rounding_rows, rounding_cols, f->block, f->scale, use_hw_convert(), st) == hipSuccess
               ? NVFP4_OK
               : NVFP4_EHIP;
}

static nvfp4_status gemm_impl(int64_t M, int64_t N, int64_t K, const nvfp4_format *f,
                              const uint8_t *A_codes, const uint8_t *A_scales, const uint8_t *B_codes,
                              const uint8_t *B_scales, const float *tensor_scales, void *out,
                              int out_dt, int64_t ldc, int a_slab, int b_slab, void *stream);

nvfp4_status nvfp4_gemm(int64_t M, int64_t N, int64_t K, const nvfp4_format *f,
                        const uint8_t *A_codes, const uint8_t *A_scales, const uint8_t *B_codes,
                        const uint8_t *B_scales, const float *tensor_scales, void *out,
                        nvfp4_dtype out_dt, int64_t ldc, void *stream)
{
    return gemm_impl(M, N, K, f, A_codes, A_scales, B_codes, B_scales, tensor_scales, out, raw(out_dt), ldc, 0, 0, stream);
}

int nvfp4_gemm_takes_slabs(int64_t M, int64_t N, int64_t K, const nvfp4_format *f)
{
    return check_format(f) == NVFP4_OK && M > 0 && N > 0 && K > 0 && gemm_takes_slabs(M, N, K, f->block, f->scale) ? 1 : 0;
}

size_t nvfp4_slab_codes_bytes(int64_t rows, int64_t K)
{
    return rows <= 0 || K <= 0 ? 0 : (size_t)slab_rows_padded(rows) * (size_t)K / 2;
}

size_t nvfp4_slab_scales_bytes(int64_t rows, int64_t K)
{
    return rows <= 0 || K <= 0 ? 0 : (size_t)slab_rows_padded(rows) * (size_t)K / 16;
}

static nvfp4_status gemm_impl(int64_t M, int64_t N, int64_t K, const nvfp4_format *f,
                              const uint8_t *A_codes, const uint8_t *A_scales, const uint8_t *B_codes,
                              const uint8_t *B_scales, const float *tensor_scales, void *out,
                              int out_dt, int64_t ldc, int a_slab, int b_slab, void *stream)
{
    (void)switches();  // (the GEMM route for wide E4M3 blocks follows a switch)
    nvfp4_status s = check_format(f);
    if (s != NVFP4_OK) return s;
    if (!A_codes || !A_scales || !B_codes || !B_scales || !tensor_scales || !out) return NVFP4_EINVAL;
    if (!valid_dtype(out_dt)) return NVFP4_EINVAL;
    if (M < 0 || N < 0 || K <= 0 || K > MAX_CONTRACTION || ldc < N) return NVFP4_ESHAPE;
    if (K % f->block != 0 || K % 32 != 0) return NVFP4_ESHAPE;
    if (!aligned16(A_codes) || !aligned16(A_scales) || !aligned16(B_codes) || !aligned16(B_scales) ||
        !aligned16(out))
        return NVFP4_EALIGN;
    if (f->scale == NVFP4_SCALE_E8M0 && f->block != 32) return NVFP4_EUNSUPPORTED;  // E8M0 GEMM: MXFP4 only
    if ((a_slab || b_slab) && !gemm_takes_slabs(M, N, K, f->block, f->scale)) return NVFP4_EUNSUPPORTED;
    if (M == 0 || N == 0) return NVFP4_OK;
    GemmArgs g{M, N, K, A_codes, A_scales, B_codes, B_scales, tensor_scales, tensor_scales + 1, out, ldc, a_slab != 0, b_slab != 0};
    return launch_gemm(g, f->block, f->scale, out_dt, reinterpret_cast<hipStream_t>(stream)) == hipSuccess
               ? NVFP4_OK
               : NVFP4_EHIP;
}

nvfp4_status nvfp4_gemm_slab(int64_t M, int64_t N, int64_t K, const nvfp4_format *f,
                             const uint8_t *A_codes, const uint8_t *A_scales, const uint8_t *B_codes,
                             const uint8_t *B_scales, const float *tensor_scales, void *out,
                             nvfp4_dtype out_dt, int64_t ldc, int a_slab, int b_slab, void *stream)
{
    return gemm_impl(M, N, K, f, A_codes, A_scales, B_codes, B_scales, tensor_scales, out, raw(out_dt), ldc, a_slab, b_slab, stream);
}

}  // extern "C"

namespace {

// nvfp4_linear_fwd, with W either as a tensor (w_ops == nullptr) or as the operands nvfp4_quantize_weight wrote.
nvfp4_status linear_fwd_impl(const void *X, const void *W, const void *w_ops, void *Y, int64_t M, int64_t N,
                             int64_t K, int in_dt, int out_dt,
                             const nvfp4_format *f, void *workspace, size_t workspace_bytes,
                             void *stream, float *xw_scales_out, void *saved, uint64_t bwd_seed)
{
    (void)switches();
    nvfp4_status s = check_format(f);
    if (s != NVFP4_OK) return s;
    if (!X || (!W && !w_ops) || !Y) return NVFP4_EINVAL;
    if (!valid_dtype(in_dt) || !valid_dtype(out_dt)) return NVFP4_EINVAL;
    if (M <= 0 || N <= 0 || K <= 0 || K > MAX_CONTRACTION) return NVFP4_ESHAPE;
    if (K % f->block != 0 || K % 32 != 0) return NVFP4_ESHAPE;
    if (f->scale == NVFP4_SCALE_E8M0 && f->block != 32) return NVFP4_EUNSUPPORTED;  // E8M0 GEMM: MXFP4 only
    if (!aligned16(X) || !aligned16(W) || !aligned16(Y)) return NVFP4_EALIGN;
    if (!workspace || workspace_bytes < nvfp4_linear_fwd_workspace_bytes(M, N, K, f)) return NVFP4_EWORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & (WS_ALIGN - 1)) != 0) return NVFP4_EALIGN;
    if (saved || w_ops) {
        // X^T is blocked along M and W^T along N, and those are the backward GEMMs' contractions
        if (saved && (M % f->block != 0 || M % 32 != 0)) return NVFP4_ESHAPE;
        if (N % f->block != 0 || N % 32 != 0) return NVFP4_ESHAPE;
        if (M > MAX_CONTRACTION || N > MAX_CONTRACTION) return NVFP4_ESHAPE;
        if ((reinterpret_cast<uintptr_t>(saved) & (WS_ALIGN - 1)) != 0) return NVFP4_EALIGN;
        if ((reinterpret_cast<uintptr_t>(w_ops) & (WS_ALIGN - 1)) != 0) return NVFP4_EALIGN;
    }
    if (w_ops && !saved_matches(w_ops, weight_tag(M, N, K, f))) return NVFP4_EINVAL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);

    uint8_t *ws = reinterpret_cast<uint8_t *>(workspace);
    // {gX, gW}: written by the quantizers (1 for a format without tensor scale), read by the GEMM
    float *ts = xw_scales_out ? xw_scales_out : reinterpret_cast<float *>(ws);
    uint32_t *amax = reinterpret_cast<uint32_t *>(ws + 64);    // two maxima
    uint32_t *partials = reinterpret_cast<uint32_t *>(ws + WS_HEADER);
    uint8_t *p = ws + WS_HEADER + (partials_bytes(M, K) > partials_bytes(N, K) ? partials_bytes(M, K) : partials_bytes(N, K));
    uint8_t *xc = p; p += op_codes(M, K);
    uint8_t *xs = p; p += op_scales(M, K, f->block);
    const uint8_t *wc = p; p += op_codes(N, K);
    const uint8_t *wsc = p;
    const float *g_w = ts + 1;

    const int gm = f->tensor_scale ? G_FROM_AMAX : G_NONE;
    GSource gx{reinterpret_cast<const float *>(amax + 0), 0}, gw{reinterpret_cast<const float *>(amax + 1), 0};
    if (f->tensor_scale) {
        if (amax_dense(X, in_dt, M * K, partials, 0, st, &gx) != hipSuccess) return NVFP4_EHIP;
        if (!w_ops && amax_dense(W, in_dt, N * K, partials, 1, st, &gw) != hipSuccess) return NVFP4_EHIP;
    }
    int a_slab = 0, b_slab = 0;
    const bool t_fwd = gemm_takes_slabs(M, N, K, f->block, f->scale);
    if (w_ops) {
        // W as quantized once for all micro-batches of the optimizer step: no pass over W here
        const WeightLayout WL = weight_layout(w_ops, N, K, f->block);
        bool w_slab, wt_slab;
        weight_slabs(f, M, N, K, &w_slab, &wt_slab);
        wc = WL.wc;
        wsc = WL.wsc;
        g_w = WL.g;
        b_slab = w_slab;
        if (xw_scales_out && hipMemcpyAsync(xw_scales_out + 1, WL.g, sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return NVFP4_EHIP;
    }
    if (saved) {
        // one pass over X and one over W also leave what Eqs. 5-6 need of them: Q_SR(X^T) with
        // the backward call's third stream, and Q_RtN(W^T)
        const SavedLayout L = saved_layout(saved, M, N, K, f->block);
        DualArgs dx{{X, M, K, K, L.xtc, L.xts, gx.src, ts + 0, gm, bwd_seed + 2, gx.n}, xc, xs, 0, L.g + 0};
        DualArgs dw{{W, N, K, K, L.wtc, L.wts, gw.src, ts + 1, gm, 0, gw.n}, const_cast<uint8_t *>(wc), const_cast<uint8_t *>(wsc), 0, L.g + 1};
        // row-blocked sides feed this call's GEMM, Q(X^T) the update GEMM (Eq. 6), Q(W^T) the input-gradient GEMM (Eq. 5)
        const bool sx = dual_writes_slabs(f, in_dt, M, K, NVFP4_RTN, NVFP4_SR), sw = dual_writes_slabs(f, in_dt, N, K, NVFP4_RTN, NVFP4_RTN);
        dx.slab_r = a_slab = sx && t_fwd;
        dx.slab_c = sx && gemm_takes_slabs(N, K, M, f->block, f->scale);
        dw.slab_c = sw && gemm_takes_slabs(M, K, N, f->block, f->scale);
        // the buffer's identity is written by the last quantizer that fills it
        DualArgs &last = w_ops ? dx : dw;
        last.tag = saved_tag(M, N, K, f, bwd_seed, dx.slab_c != 0, w_ops ? false : dw.slab_c != 0, w_ops != nullptr);
        last.tag.dst = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(saved) + SAVED_TAG_OFFSET);
        saved_remember(saved, last.tag);
        if (launch_quantize_dual(dx, in_dt, NVFP4_RTN, NVFP4_SR, f->block, f->scale, use_hw_convert(), st) != hipSuccess) return NVFP4_EHIP;
        if (!w_ops) {
            dw.slab_r = b_slab = sw && t_fwd;
            if (launch_quantize_dual(dw, in_dt, NVFP4_RTN, NVFP4_RTN, f->block, f->scale, use_hw_convert(), st) != hipSuccess) return NVFP4_EHIP;
        }
    } else {
        QuantPlan qx{X, in_dt, M, K, K, 1, NVFP4_RTN, 0, xc, xs, gx.src, ts + 0, gm, gx.n};
        QuantPlan qw{W, in_dt, N, K, K, 1, NVFP4_RTN, 0, const_cast<uint8_t *>(wc), const_cast<uint8_t *>(wsc), gw.src, ts + 1, gm, gw.n};
        if (run_quantize(qx, f, st) != hipSuccess) return NVFP4_EHIP;
        if (!w_ops && run_quantize(qw, f, st) != hipSuccess) return NVFP4_EHIP;
    }
    GemmArgs g{M, N, K, xc, xs, wc, wsc, ts, g_w, Y, N, a_slab, b_slab};
    return launch_gemm(g, f->block, f->scale, out_dt, st) == hipSuccess ? NVFP4_OK : NVFP4_EHIP;
}

nvfp4_status linear_bwd_impl(const void *dY, const nvfp4_dual_operands *dyq, const void *X, const void *W, const void *w_ops, void *dX, void *dW,
                             int64_t M, int64_t N, int64_t K, int in_dt,
                             int out_dt, const nvfp4_format *f, uint64_t seed,
                             void *workspace, size_t workspace_bytes, void *stream, const float *xw_scales,
                             const void *saved)
{
    nvfp4_status s = check_format(f);
    if (s != NVFP4_OK) return s;
    if ((!dY && !dyq) || (dX && !W && !saved && !w_ops) || (dW && !X && !saved)) return NVFP4_EINVAL;
    if (dyq) {
        // the upstream gradient arrives quantized: each side that a requested GEMM consumes must be there
        if (!dyq->g || (dX && (!dyq->codes_rows || !dyq->scales_rows)) || (dW && (!dyq->codes_cols || !dyq->scales_cols))) return NVFP4_EINVAL;
        if (dyq->layout & ~(NVFP4_SLAB_ROWS | NVFP4_SLAB_COLS)) return NVFP4_EINVAL;
        if (!aligned16(dyq->codes_rows) || !aligned16(dyq->scales_rows) || !aligned16(dyq->codes_cols) || !aligned16(dyq->scales_cols)) return NVFP4_EALIGN;
    }
    if (saved && (reinterpret_cast<uintptr_t>(saved) & (WS_ALIGN - 1)) != 0) return NVFP4_EALIGN;
    if (w_ops && (reinterpret_cast<uintptr_t>(w_ops) & (WS_ALIGN - 1)) != 0) return NVFP4_EALIGN;
    if (!valid_dtype(in_dt) || !valid_dtype(out_dt)) return NVFP4_EINVAL;
    if (M <= 0 || N <= 0 || K <= 0) return NVFP4_ESHAPE;
    const int64_t B = f->block;
    // dX contracts over N, dW over M; K is a leading dimension of X and W read down columns
    if (dX && (N % B != 0 || N % 32 != 0 || N > MAX_CONTRACTION)) return NVFP4_ESHAPE;
    if (dW && (M % B != 0 || M % 32 != 0 || M > MAX_CONTRACTION)) return NVFP4_ESHAPE;
    if ((saved || w_ops) && (M % B != 0 || N % B != 0)) return NVFP4_ESHAPE;  // the shapes the forward call accepted
    if ((K * (int64_t)elem_size(in_dt)) % 16 != 0 || (N * (int64_t)elem_size(in_dt)) % 16 != 0) return NVFP4_EALIGN;
    if (f->scale == NVFP4_SCALE_E8M0 && f->block != 32) return NVFP4_EUNSUPPORTED;  // E8M0 GEMM: MXFP4 only
    if (!aligned16(dY) || !aligned16(X) || !aligned16(W) || !aligned16(dX) || !aligned16(dW)) return NVFP4_EALIGN;
    if (!workspace || workspace_bytes < nvfp4_linear_bwd_workspace_bytes(M, N, K, f)) return NVFP4_EWORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & (WS_ALIGN - 1)) != 0) return NVFP4_EALIGN;
    if (w_ops && !saved_matches(w_ops, weight_tag(M, N, K, f))) return NVFP4_EINVAL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);

    uint8_t *ws = reinterpret_cast<uint8_t *>(workspace);
    float *ts = reinterpret_cast<float *>(ws);               // {g_dY, g_W, g_dY, g_X}
    uint32_t *amax = reinterpret_cast<uint32_t *>(ws + 64);  // maxima of dY, W, X
    uint32_t *partials = reinterpret_cast<uint32_t *>(ws + WS_HEADER);
    size_t part = partials_bytes(M, N);
    if (partials_bytes(N, K) > part) part = partials_bytes(N, K);
    if (partials_bytes(M, K) > part) part = partials_bytes(M, K);
    uint8_t *p = ws + WS_HEADER + part;
    uint8_t *dyc = p; p += op_codes(M, N);
    uint8_t *dys = p; p += op_scales(M, N, B);
    uint8_t *wtc = p; p += op_codes(K, N);
    uint8_t *wts = p; p += op_scales(K, N, B);
    uint8_t *dytc = p; p += op_codes(N, M);
    uint8_t *dyts = p; p += op_scales(N, M, B);
    uint8_t *xtc = p; p += op_codes(K, M);
    uint8_t *xts = p;
    const float *g_w = ts + 1, *g_x = ts + 3;  // written by the W^T and X^T quantizers below, or saved by the forward call
    const bool have_xt = saved != nullptr, have_wt = saved != nullptr || w_ops != nullptr;
    if (saved) {
        // Q_RtN(W^T) and Q_SR(X^T) as the forward call left them (its bwd_seed must equal seed)
        const SavedLayout L = saved_layout(const_cast<void *>(saved), M, N, K, B);
        wtc = L.wtc;
        wts = L.wts;
        xtc = L.xtc;
        xts = L.xts;
        g_x = L.g + 0;
        g_w = L.g + 1;
    }
    bool w_slab = false, wq_wt_slab = false;
    if (w_ops) {
        // Q_RtN(W^T) as nvfp4_quantize_weight left it
        const WeightLayout WL = weight_layout(w_ops, N, K, B);
        weight_slabs(f, M, N, K, &w_slab, &wq_wt_slab);
        wtc = WL.wtc;
        wts = WL.wts;
        g_w = WL.g;
    }

    const int gm = f->tensor_scale ? G_FROM_AMAX : G_NONE;
    // X and W: scales handed over from the forward call (used as given), else from their maxima
    const bool known = f->tensor_scale && xw_scales != nullptr;
    const int gm_xw = known ? G_PRESET : gm;
    GSource gdy{reinterpret_cast<const float *>(amax + 0), 0};
    GSource gw{known ? xw_scales + 1 : reinterpret_cast<const float *>(amax + 1), 0};
    GSource gx{known ? xw_scales + 0 : reinterpret_cast<const float *>(amax + 2), 0};
    // with both GEMMs wanted, dY is read once for its two orientations (streams seed, seed+1)
    const bool dual = !dyq && dX && dW && quantize_dual_fused(in_dt, M, N, N, f->block, use_hw_convert());
    // layouts: dY's two sides as this call's dual pass writes them, W^T and X^T as the forward call wrote them
    const bool t_dx = gemm_takes_slabs(M, K, N, f->block, f->scale), t_dw = gemm_takes_slabs(N, K, M, f->block, f->scale);
    const bool sdy = dual && dual_writes_slabs(f, in_dt, M, N, NVFP4_SR, NVFP4_SR);
    int dy_slab_r = sdy && t_dx, dy_slab_c = sdy && t_dw;
    const float *g_dy_r = ts + 0, *g_dy_c = ts + 2;  // written by this call's quantizers of dY
    if (dyq) {
        dy_slab_r = (dyq->layout & NVFP4_SLAB_ROWS) != 0;
        dy_slab_c = (dyq->layout & NVFP4_SLAB_COLS) != 0;
        if ((dX && dy_slab_r && !t_dx) || (dW && dy_slab_c && !t_dw)) return NVFP4_EUNSUPPORTED;
        dyc = dyq->codes_rows;
        dys = dyq->scales_rows;
        dytc = dyq->codes_cols;
        dyts = dyq->scales_cols;
        g_dy_r = g_dy_c = dyq->g;
    } else if (f->tensor_scale) {
        if (amax_dense(dY, in_dt, M * N, partials, 0, st, &gdy) != hipSuccess) return NVFP4_EHIP;
    }
    const int wt_slab = w_ops ? (int)wq_wt_slab : (int)(saved && t_dx && dual_writes_slabs(f, in_dt, N, K, NVFP4_RTN, NVFP4_RTN));
    const int xt_slab = saved && t_dw && dual_writes_slabs(f, in_dt, M, K, NVFP4_RTN, NVFP4_SR);
    TagArgs tag;
    if (saved) {
        tag = saved_tag(M, N, K, f, seed, xt_slab != 0, w_ops ? false : wt_slab != 0, w_ops != nullptr);
        tag.chk = reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint8_t *>(saved) + SAVED_TAG_OFFSET);
        if (!saved_matches(saved, tag)) return NVFP4_EINVAL;
    }
    if (dual) {
        DualArgs d;
        d.tag = tag;
        d.c.x = dY;
        d.c.rows = M;
        d.c.cols = N;
        d.c.ld = N;
        d.c.codes = dytc;
        d.c.scales = dyts;
        d.c.g_src = gdy.src;
        d.c.n_partials = gdy.n;
        d.c.g_out = ts + 0;
        d.c.g_mode = gm;
        d.c.seed = seed + 1;
        d.codes_r = dyc;
        d.scales_r = dys;
        d.seed_r = seed;
        d.g_out2 = ts + 2;
        d.slab_r = dy_slab_r;
        d.slab_c = dy_slab_c;
        if (launch_quantize_dual(d, in_dt, NVFP4_SR, NVFP4_SR, f->block, f->scale, true, st) != hipSuccess) return NVFP4_EHIP;
    }
    if (dX) {
        if (f->tensor_scale && !known && !have_wt && amax_dense(W, in_dt, N * K, partials, 1, st, &gw) != hipSuccess) return NVFP4_EHIP;
        // Eq. 5: dX[M, K] = Q_SR(dY)[M, N] * Q_RtN(W^T)[K, N]^T
        QuantPlan qa{dY, in_dt, M, N, N, 1, NVFP4_SR, seed, dyc, dys, gdy.src, ts + 0, gm, gdy.n};
        QuantPlan qb{W, in_dt, N, K, K, 0, NVFP4_RTN, 0, wtc, wts, gw.src, ts + 1, gm_xw, gw.n};
        if (!dual && !dyq && run_quantize(qa, f, st) != hipSuccess) return NVFP4_EHIP;
        if (!dual && !dyq && launch_saved_tag(tag, ts + 0, nullptr, st) != hipSuccess) return NVFP4_EHIP;
        if (!have_wt && run_quantize(qb, f, st) != hipSuccess) return NVFP4_EHIP;
        GemmArgs g{M, K, N, dyc, dys, wtc, wts, g_dy_r, g_w, dX, K, dy_slab_r, wt_slab};
        if (launch_gemm(g, f->block, f->scale, out_dt, st) != hipSuccess) return NVFP4_EHIP;
    }
    if (dW) {
        if (f->tensor_scale && !known && !have_xt && amax_dense(X, in_dt, M * K, partials, 2, st, &gx) != hipSuccess) return NVFP4_EHIP;
        // Eq. 6: dW[N, K] = Q_SR(dY^T)[N, M] * Q_SR(X^T)[K, M]^T
        QuantPlan qa{dY, in_dt, M, N, N, 0, NVFP4_SR, seed + 1, dytc, dyts, gdy.src, ts + 2, gm, gdy.n};
        QuantPlan qb{X, in_dt, M, K, K, 0, NVFP4_SR, seed + 2, xtc, xts, gx.src, ts + 3, gm_xw, gx.n};
        if (!dual && !dyq && run_quantize(qa, f, st) != hipSuccess) return NVFP4_EHIP;
        if (!dual && !dyq && launch_saved_tag(tag, ts + 2, nullptr, st) != hipSuccess) return NVFP4_EHIP;
        if (!have_xt && run_quantize(qb, f, st) != hipSuccess) return NVFP4_EHIP;
        GemmArgs g{N, K, M, dytc, dyts, xtc, xts, g_dy_c, g_x, dW, K, dy_slab_c, xt_slab};
        if (launch_gemm(g, f->block, f->scale, out_dt, st) != hipSuccess) return NVFP4_EHIP;
    }
    return NVFP4_OK;
}

}  // namespace

extern "C" {

nvfp4_status nvfp4_linear_fwd(const void *X, const void *W, void *Y, int64_t M, int64_t N,
                              int64_t K, nvfp4_dtype in_dt, nvfp4_dtype out_dt,
                              const nvfp4_format *f, void *workspace, size_t workspace_bytes,
                              void *stream, float *xw_scales_out, void *saved, uint64_t bwd_seed)
{
    if (!W) return NVFP4_EINVAL;
    return linear_fwd_impl(X, W, nullptr, Y, M, N, K, raw(in_dt), raw(out_dt), f, workspace, workspace_bytes, stream, xw_scales_out, saved, bwd_seed);
}

nvfp4_status nvfp4_linear_bwd(const void *dY, const void *X, const void *W, void *dX, void *dW,
                              int64_t M, int64_t N, int64_t K, nvfp4_dtype in_dt,
                              nvfp4_dtype out_dt, const nvfp4_format *f, uint64_t seed,
                              void *workspace, size_t workspace_bytes, void *stream, const float *xw_scales,
                              const void *saved)
{
    return linear_bwd_impl(dY, nullptr, X, W, nullptr, dX, dW, M, N, K, raw(in_dt), raw(out_dt), f, seed, workspace, workspace_bytes, stream, xw_scales, saved);
}

nvfp4_status nvfp4_linear_bwd_dyq(const nvfp4_dual_operands *dY, const void *X, const void *W,
                                  const void *w_operands, void *dX, void *dW, int64_t M, int64_t N, int64_t K,
                                  nvfp4_dtype in_dt, nvfp4_dtype out_dt, const nvfp4_format *f, uint64_t seed,
                                  void *workspace, size_t workspace_bytes, void *stream,
                                  const float *xw_scales, const void *saved)
{
    if (!dY) return NVFP4_EINVAL;
    return linear_bwd_impl(nullptr, dY, X, W, w_operands, dX, dW, M, N, K, raw(in_dt), raw(out_dt), f, seed, workspace, workspace_bytes, stream, xw_scales, saved);
}

size_t nvfp4_swiglu_bwd_workspace_bytes(int64_t M, int64_t F)
{
    (void)M;
    (void)F;
    return WS_HEADER + 2 * PARTIAL_SLOT;  // partial maxima of dG and of dU
}

nvfp4_status nvfp4_swiglu_bwd_quantize(const void *dH, const void *G, const void *U, nvfp4_dtype dt_, int64_t M,
                                       int64_t F, uint64_t seed_gate, uint64_t seed_up, const nvfp4_format *f,
                                       const nvfp4_dual_operands *dG, const nvfp4_dual_operands *dU,
                                       void *dG_store, void *dU_store,
                                       void *workspace, size_t workspace_bytes, void *stream)
{
    const int dt = raw(dt_);
    if ((dG_store == nullptr) != (dU_store == nullptr)) return NVFP4_EINVAL;
    if (!aligned16(dG_store) || !aligned16(dU_store)) return NVFP4_EALIGN;
    nvfp4_status s = check_format(f);
    if (s != NVFP4_OK) return s;
    if (!valid_dtype(dt) || !dH || !G || !U || !dG || !dU) return NVFP4_EINVAL;
    if (M <= 0 || F <= 0 || M % f->block != 0 || F % f->block != 0) return NVFP4_ESHAPE;
    const bool fmt_ok = (f->block == 16 && f->scale == NVFP4_SCALE_E4M3 && f->tensor_scale) || (f->block == 32 && f->scale == NVFP4_SCALE_E8M0);
    if (!fmt_ok || !use_hw_convert() || !quantize_dual_fused(dt, M, F, F, f->block, true)) return NVFP4_EUNSUPPORTED;
    if (!aligned16(dH) || !aligned16(G) || !aligned16(U)) return NVFP4_EALIGN;
    for (const nvfp4_dual_operands *o : {dG, dU}) {
        if (!o->codes_rows || !o->scales_rows || !o->codes_cols || !o->scales_cols || !o->g) return NVFP4_EINVAL;
        if (o->layout & ~(NVFP4_SLAB_ROWS | NVFP4_SLAB_COLS)) return NVFP4_EINVAL;
        if (!aligned16(o->codes_rows) || !aligned16(o->scales_rows) || !aligned16(o->codes_cols) || !aligned16(o->scales_cols)) return NVFP4_EALIGN;
        if (((o->layout & NVFP4_SLAB_ROWS) && F % SLAB_K != 0) || ((o->layout & NVFP4_SLAB_COLS) && M % SLAB_K != 0)) return NVFP4_ESHAPE;
    }
    const bool need_ws = f->tensor_scale || dG_store;  // (the first pass leaves its partial maxima there)
    if (need_ws) {
        if (!workspace || workspace_bytes < nvfp4_swiglu_bwd_workspace_bytes(M, F)) return NVFP4_EWORKSPACE;
        if (!aligned16(workspace)) return NVFP4_EALIGN;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    uint32_t *partials = need_ws ? reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(workspace) + WS_HEADER) : nullptr;
    const int gm = f->tensor_scale ? G_FROM_AMAX : G_NONE;
    auto plan = [&](const nvfp4_dual_operands *o, uint64_t seed) {
        DualArgs d;
        d.c.x = dH;
        d.c.rows = M;
        d.c.cols = F;
        d.c.ld = F;
        d.c.codes = o->codes_cols;
        d.c.scales = o->scales_cols;
        d.c.g_src = o->g;
        d.c.g_out = o->g;
        d.c.g_mode = gm;
        d.c.seed = seed + 1;
        d.codes_r = o->codes_rows;
        d.scales_r = o->scales_rows;
        d.seed_r = seed;
        d.g_out2 = nullptr;
        d.slab_r = (o->layout & NVFP4_SLAB_ROWS) != 0;
        d.slab_c = (o->layout & NVFP4_SLAB_COLS) != 0;
        d.src_g = G;
        d.src_u = U;
        return d;
    };
    DualArgs dg = plan(dG, seed_gate), du = plan(dU, seed_up);
    return launch_swiglu_bwd_dual(dg, du, dt, f->block, f->scale, partials, partials ? partials + AMAX_DENSE_PARTIALS : nullptr, dG_store, dU_store, st) == hipSuccess ? NVFP4_OK : NVFP4_EHIP;
}

nvfp4_status nvfp4_swiglu_bwd(const void *dH, const void *G, const void *U, nvfp4_dtype dt_, int64_t n, void *dG,
                              void *dU, void *stream)
{
    const int dt = raw(dt_);
    if (!valid_dtype(dt)) return NVFP4_EINVAL;
    if (n < 0 || n % 8 != 0) return NVFP4_ESHAPE;
    if (n == 0) return NVFP4_OK;
    if (!dH || !G || !U || !dG || !dU) return NVFP4_EINVAL;
    if (!aligned16(dH) || !aligned16(G) || !aligned16(U) || !aligned16(dG) || !aligned16(dU)) return NVFP4_EALIGN;
    return launch_swiglu_bwd(dH, G, U, dt, n, dG, dU, reinterpret_cast<hipStream_t>(stream)) == hipSuccess ? NVFP4_OK : NVFP4_EHIP;
}

void nvfp4_host_swiglu_bwd(const float *dH, const float *G, const float *U, int64_t n, float *dG, float *dU)
{
    for (int64_t t = 0; t < n; ++t) swiglu_bwd_elem(dH[t], G[t], U[t], &dG[t], &dU[t]);
}

size_t nvfp4_weight_operands_bytes(int64_t N, int64_t K, const nvfp4_format *f)
{
    if (N <= 0 || K <= 0 || check_format(f) != NVFP4_OK) return 0;
    return WS_HEADER + op_codes(N, K) + op_scales(N, K, f->block) + op_codes(K, N) + op_scales(K, N, f->block);
}

nvfp4_status nvfp4_quantize_weight(const void *W, nvfp4_dtype dt_, int64_t M, int64_t N, int64_t K,
                                   const nvfp4_format *f, void *w_operands, void *workspace,
                                   size_t workspace_bytes, void *stream)
{
    const int dt = raw(dt_);
    nvfp4_status s = check_format(f);
    if (s != NVFP4_OK) return s;
    if (!W || !w_operands || !valid_dtype(dt)) return NVFP4_EINVAL;
    if (M <= 0 || N <= 0 || K <= 0 || K > MAX_CONTRACTION || N > MAX_CONTRACTION || M > MAX_CONTRACTION) return NVFP4_ESHAPE;
    if (K % f->block != 0 || K % 32 != 0 || N % f->block != 0 || N % 32 != 0) return NVFP4_ESHAPE;
    if (f->scale == NVFP4_SCALE_E8M0 && f->block != 32) return NVFP4_EUNSUPPORTED;  // E8M0 GEMM: MXFP4 only
    if (!aligned16(W) || (reinterpret_cast<uintptr_t>(w_operands) & (WS_ALIGN - 1)) != 0) return NVFP4_EALIGN;
    if (f->tensor_scale) {
        if (!workspace || workspace_bytes < nvfp4_quantize_workspace_bytes(N, K)) return NVFP4_EWORKSPACE;
        if (!aligned16(workspace)) return NVFP4_EALIGN;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const WeightLayout WL = weight_layout(w_operands, N, K, f->block);
    GSource gw{WL.g, 0};
    if (f->tensor_scale) {
        uint32_t *partials = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(workspace) + WS_HEADER);
        if (amax_dense(W, dt, N * K, partials, 0, st, &gw) != hipSuccess) return NVFP4_EHIP;
    }
    bool w_slab, wt_slab;
    weight_slabs(f, M, N, K, &w_slab, &wt_slab);
    DualArgs dw{{W, N, K, K, WL.wtc, WL.wts, gw.src, WL.g, f->tensor_scale ? G_FROM_AMAX : G_NONE, 0, gw.n}, WL.wc, WL.wsc, 0, nullptr};
    dw.slab_r = w_slab;
    dw.slab_c = wt_slab;
    dw.tag = weight_tag(M, N, K, f);
    dw.tag.dst = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(w_operands) + SAVED_TAG_OFFSET);
    saved_remember(w_operands, dw.tag);
    return launch_quantize_dual(dw, dt, NVFP4_RTN, NVFP4_RTN, f->block, f->scale, use_hw_convert(), st) == hipSuccess ? NVFP4_OK : NVFP4_EHIP;
}

nvfp4_status nvfp4_linear_fwd_wq(const void *X, const void *w_operands, void *Y, int64_t M, int64_t N,
                                 int64_t K, nvfp4_dtype in_dt, nvfp4_dtype out_dt,
                                 const nvfp4_format *f, void *workspace, size_t workspace_bytes,
                                 void *stream, float *xw_scales_out, void *saved, uint64_t bwd_seed)
{
    if (!w_operands) return NVFP4_EINVAL;
    return linear_fwd_impl(X, nullptr, w_operands, Y, M, N, K, raw(in_dt), raw(out_dt), f, workspace, workspace_bytes, stream, xw_scales_out, saved, bwd_seed);
}

nvfp4_status nvfp4_linear_bwd_wq(const void *dY, const void *X, const void *w_operands, void *dX, void *dW,
                                 int64_t M, int64_t N, int64_t K, nvfp4_dtype in_dt,
                                 nvfp4_dtype out_dt, const nvfp4_format *f, uint64_t seed,
                                 void *workspace, size_t workspace_bytes, void *stream, const float *xw_scales,
                                 const void *saved)
{
    if (!w_operands) return NVFP4_EINVAL;
    return linear_bwd_impl(dY, nullptr, X, nullptr, w_operands, dX, dW, M, N, K, raw(in_dt), raw(out_dt), f, seed, workspace, workspace_bytes, stream, xw_scales, saved);
}

size_t nvfp4_quant_noise_workspace_bytes(int64_t rows, int64_t cols, int axis)
{
    if (axis != 0 && axis != 1) return 0;
    return align_up(16 * (size_t)quant_noise_partials(rows, cols, axis));
}

nvfp4_status nvfp4_quant_noise(const void *x, nvfp4_dtype dt_, int64_t rows, int64_t cols, int64_t ld, int axis,
                               const nvfp4_format *f, const uint8_t *codes, const uint8_t *scales,
                               const float *tensor_scale, double *sums, void *workspace, size_t workspace_bytes,
                               void *stream)
{
    const int dt = raw(dt_);
    nvfp4_status s = check_format(f);
    if (s != NVFP4_OK) return s;
    s = check_tensor(x, dt, rows, cols, ld);
    if (s != NVFP4_OK) return s;
    if (axis != 0 && axis != 1) return NVFP4_EINVAL;
    const bool empty = rows == 0 || cols == 0;
    if (!sums || (!empty && (!codes || !scales)) || (f->tensor_scale && !tensor_scale)) return NVFP4_EINVAL;
    const int64_t inner = axis == 1 ? cols : rows;
    if (inner % f->block != 0) return NVFP4_ESHAPE;
    if (!aligned16(codes) || !aligned16(scales) || (reinterpret_cast<uintptr_t>(sums) & 7u) != 0) return NVFP4_EALIGN;
    if (!workspace || workspace_bytes < nvfp4_quant_noise_workspace_bytes(rows, cols, axis)) return NVFP4_EWORKSPACE;
    if (!aligned16(workspace)) return NVFP4_EALIGN;
    return launch_quant_noise(x, dt, rows, cols, ld, axis, f->block, f->scale, codes, scales,
                              f->tensor_scale ? tensor_scale : nullptr, reinterpret_cast<double *>(workspace), sums,
                              reinterpret_cast<hipStream_t>(stream)) == hipSuccess
               ? NVFP4_OK
               : NVFP4_EHIP;
}

// ---- host evaluations of the scalar steps (no GPU involved)

uint8_t nvfp4_host_e4m3_encode(float r)
{
    float s;
    return (uint8_t)e4m3_encode(r, &s);
}
float nvfp4_host_e4m3_decode(uint8_t byte) { return e4m3_decode(byte); }
uint8_t nvfp4_host_round_rtn(float m) { return (uint8_t)round_rtn(m); }
uint8_t nvfp4_host_round_sr(float m, uint32_t u16) { return (uint8_t)round_sr(m, u16); }
void nvfp4_host_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    u32x4 d = philox4x32_10(ctr[0], ctr[1], ctr[2], ctr[3], key[0], key[1]);
    out[0] = d.x; out[1] = d.y; out[2] = d.z; out[3] = d.w;
}
uint32_t nvfp4_host_sr_bits(uint64_t seed, uint64_t e) { return sr_bits_of(sr_draw(seed, e >> 3), (uint32_t)e & 7u); }
uint8_t nvfp4_host_e8m0_encode(float a)
{
    float q;
    return (uint8_t)e8m0_encode(a, &q);
}
void nvfp4_host_e4m3_encode_n(const float *r, int64_t n, uint8_t *out)
{
    for (int64_t t = 0; t < n; ++t) out[t] = nvfp4_host_e4m3_encode(r[t]);
}
void nvfp4_host_round_rtn_n(const float *m, int64_t n, uint8_t *out)
{
    for (int64_t t = 0; t < n; ++t) out[t] = nvfp4_host_round_rtn(m[t]);
}
void nvfp4_host_round_sr_n(const float *m, const uint32_t *u16, int64_t n, uint8_t *out)
{
    for (int64_t t = 0; t < n; ++t) out[t] = nvfp4_host_round_sr(m[t], u16[t]);
}

}  // extern "C"
