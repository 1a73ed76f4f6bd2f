// C-ABI boundary of libwino: argument validation on the host, variant choice,
// workspace carving, and the chain of launches for the three Winograd steps
// (Section "Techniques").  Nothing here computes; every step runs in a kernel.
#include "../../include/wino.h"
#include "wino_internal.h"

#include <limits.h>
#include <mutex>

using namespace wino;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool dtype_ok(int d) { return d == WINO_F32 || d == WINO_F16 || d == WINO_BF16; }
inline size_t esize(int d) { return d == WINO_F32 ? 4 : 2; }
inline bool wino_variant_ok(int v) { return v == WINO_F2 || v == WINO_F4 || v == WINO_FUSED_F2 || v == WINO_FUSED_F4; }
inline bool fused_variant(int v) { return v == WINO_FUSED_F2 || v == WINO_FUSED_F4; }
// output tile edge m of a Winograd variant (the fused variants are F(2x2,3x3) / F(4x4,3x3) with steps (ii) and (iii) in one kernel)
inline int tile_edge(int v) { return (v == WINO_F4 || v == WINO_FUSED_F4) ? 4 : 2; }
// the fused F(4x4) kernel exists for the two-byte storage types only
inline bool variant_dtype_ok(int v, int d) { return !(v == WINO_FUSED_F4 && d == WINO_F32); }

// products that must fit: element counts as size_t and tile counts as int
bool dims_ok(int N, int C, int H, int W, int K, int m) {
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1) return false;
    if (C > (1 << 22) || K > (1 << 22)) return false;      // grid.y of the transform kernels carries C/64
    const unsigned long long lim = 1ULL << 40;    // elements; far above 288 GB of fp16 already
    const unsigned long long th = (unsigned long long)(H + m - 1) / m, tw = (unsigned long long)(W + m - 1) / m;
    const unsigned long long T = (unsigned long long)N * th * tw;
    if (T > (unsigned long long)INT_MAX / 2) return false;
    const unsigned long long a2 = (unsigned long long)(m + 2) * (m + 2);
    const unsigned long long Cp = (unsigned long long)(C + 7) / 8 * 8;
    if ((unsigned long long)N * C * H > lim / W) return false;
    if ((unsigned long long)N * K * H > lim / W) return false;
    if (a2 * T > lim / Cp) return false;
    if (a2 * T > lim / (unsigned long long)K) return false;
    if (a2 * (unsigned long long)K > lim / Cp) return false;
    if ((unsigned long long)K * T > (unsigned long long)INT_MAX * 128ULL) return false;
    return true;
}

bool igemm_dims_ok(int N, int C, int H, int W, int K, int R, int st) {
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1) return false;
    if ((R != 1 && R != 3) || (st != 1 && st != 2)) return false;
    if (C > (1 << 22) || K > (1 << 22)) return false;
    const unsigned long long lim = 1ULL << 40;
    const unsigned long long Cp = (unsigned long long)(C + 7) / 8 * 8;
    if ((unsigned long long)N * H * W > (unsigned long long)INT_MAX / 2) return false;    // pixel indices are ints
    if ((unsigned long long)N * H * W > lim / Cp) return false;
    if ((unsigned long long)N * H * W > lim / (unsigned long long)K) return false;
    if ((unsigned long long)R * R * K > lim / Cp) return false;
    return true;
}

// bytes of the re-laid copy of x (0: x is used in place), and of the fp32 partial products
size_t igemm_xh_bytes(int N, int C, int H, int W, int dtype, int layout) {
    if (layout == WINO_NHWC && C % 8 == 0) return 0;
    return align_up((size_t)N * H * W * (size_t)round_up(C, 8) * esize(dtype));
}
size_t igemm_part_bytes(int N, int C, int H, int W, int K, int R, int stride, int dtype) {
    const int pad = (R - 1) / 2;
    const long long T = (long long)N * ((H + 2 * pad - R) / stride + 1) * ((W + 2 * pad - R) / stride + 1);
    const int sp = igemm_split((int)T, K, round_up(C, 8), R, dtype);
    return sp > 1 ? align_up((size_t)sp * (size_t)K * (size_t)T * sizeof(float)) : 0;
}

struct Workspace { size_t v_bytes, m_bytes, total; };
Workspace workspace_layout(const Geom& g, int dtype, int variant) {
    Workspace ws;
    const size_t a2 = (size_t)g.alpha * g.alpha;
    ws.v_bytes = align_up(a2 * (size_t)g.T * g.Cp * esize(dtype));
    if (fused_variant(variant)) { ws.m_bytes = 0; ws.total = ws.v_bytes; return ws; }   // the product never leaves the registers
    // the product, times the number of partial copies the GEMM stage writes for this shape (the
    // policy depends on the operand order only through the block shape; take the larger of the two)
    const int sp_a = gemm_split(g.K, g.T, g.Cp, (int)a2, dtype), sp_b = gemm_split(g.T, g.K, g.Cp, (int)a2, dtype);
    ws.m_bytes = align_up(a2 * (size_t)g.K * g.T * sizeof(float) * (size_t)(sp_a > sp_b ? sp_a : sp_b));
    ws.total = ws.v_bytes + ws.m_bytes;
    return ws;
}

int run_chain(const void* x, const wino_filter* w_t, const float* bias, void* y, const Geom& g,
              void* workspace, bool nhwc, const PreOp* pre, const PostOp* post, hipStream_t s, bool half_product = false) {
    const int dt = w_t->dtype;
    const Workspace ws = workspace_layout(g, w_t->dtype, w_t->variant);
    void* V = workspace;
    float* M = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + ws.v_bytes);
    if (launch_input_transform(x, V, g, dt, nhwc, pre, s) != hipSuccess) return WINO_ERR_HIP;
    if (w_t->variant == WINO_FUSED_F2)
        return launch_fused_gemm_output(w_t->data, V, bias, y, g, dt, nhwc, post, -1, s) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
    if (w_t->variant == WINO_FUSED_F4)
        return launch_fused4_gemm_output(w_t->data, V, bias, y, g, dt, nhwc, post, -1, s) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
    // channel-last: operands swapped, so the product comes out as M[alpha^2][T][K], k contiguous
    const int a2 = g.alpha * g.alpha;
    const int nsplit = nhwc ? gemm_split(g.T, g.K, g.Cp, a2, dt) : gemm_split(g.K, g.T, g.Cp, a2, dt);
    // the half-product mode applies to fp16 storage with an unsplit reduction; elsewhere M stays fp32
    const bool hp = half_product && dt == WINO_F16 && nsplit == 1;
    const hipError_t ge = nhwc ? launch_batched_gemm(V, w_t->data, M, g.T, g.Cp, g.K, a2, nsplit, dt, hp, s)
                               : launch_batched_gemm(w_t->data, V, M, g.K, g.Cp, g.T, a2, nsplit, dt, hp, s);
    if (ge != hipSuccess) return WINO_ERR_HIP;
    if (launch_output_transform(M, bias, y, g, nsplit, dt, nhwc, hp, post, s) != hipSuccess) return WINO_ERR_HIP;
    return WINO_OK;
}

int check_conv_args(const void* x, const wino_filter* w_t, const float* bias, const void* y,
                    int N, int C, int H, int W, int K, int up = 0) {
    if (!x || !w_t || !y || !w_t->data) return WINO_ERR_NULL;
    if (!dtype_ok(w_t->dtype)) return WINO_ERR_DTYPE;
    if (w_t->variant == WINO_DIRECT) {
        if (!igemm_dims_ok(N, C, H, W, K, 3, 1)) return WINO_ERR_DIM;
    } else {
        if (!wino_variant_ok(w_t->variant)) return WINO_ERR_VARIANT;
        if (!variant_dtype_ok(w_t->variant, w_t->dtype)) return WINO_ERR_DTYPE;
        if (!dims_ok(N, C, H, W, K, tile_edge(w_t->variant))) return WINO_ERR_DIM;
    }
    if (w_t->K != K || w_t->C != C) return WINO_ERR_DIM;
    if (!aligned16(x) || !aligned16(y) || !aligned16(w_t->data) || (bias && (reinterpret_cast<uintptr_t>(bias) & 3u)))
        return WINO_ERR_ALIGN;
    const size_t es = esize(w_t->dtype);
    const uintptr_t xb = reinterpret_cast<uintptr_t>(x), xe = xb + (size_t)N * C * (H >> up) * (W >> up) * es;
    const uintptr_t yb = reinterpret_cast<uintptr_t>(y), ye = yb + (size_t)N * K * H * W * es;
    if (xb < ye && yb < xe) return WINO_ERR_ALIAS;
    return WINO_OK;
}

}  // namespace

extern "C" {

int wino_version(void) { return 100; }   // 0.1.0

const char* wino_status_string(int status) {
    switch (status) {
        case WINO_OK: return "ok";
        case WINO_ERR_NULL: return "required pointer is NULL";
        case WINO_ERR_DIM: return "bad dimension (non-positive, mismatching the transformed filter, or too large)";
        case WINO_ERR_DTYPE: return "unsupported dtype";
        case WINO_ERR_VARIANT: return "unsupported variant";
        case WINO_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case WINO_ERR_WORKSPACE: return "workspace missing or too small";
        case WINO_ERR_ALIAS: return "x and y overlap";
        case WINO_ERR_HIP: return "HIP call failed";
        case WINO_ERR_LAYOUT: return "unsupported layout";
        case WINO_ERR_SCRATCH: return "problem needs more scratch than the library's static buffer holds";
        default: return "unknown status";
    }
}

int wino_resolve_variant(int N, int C, int H, int W, int K, int dtype, int variant) {
    if (!dtype_ok(dtype)) return -1;
    if (variant == WINO_DIRECT || wino_variant_ok(variant)) {
        return (dims_ok(N, C, H, W, K, tile_edge(variant)) && variant_dtype_ok(variant, dtype)) ? variant : -1;
    }
    if (variant != WINO_AUTO) return -1;
    if (!dims_ok(N, C, H, W, K, 2) || !dims_ok(N, C, H, W, K, 4)) return -1;
    // Measured over the SD-shaped layers: F(4x4) moves fewer activation bytes and wins whenever
    // there are enough tiles to fill the GEMM's column blocks; with very few tiles (8x8 and 16x16
    // images) the 2.25x larger transformed filter and the empty MFMA columns make F(2x2) faster.
    const Geom g4 = make_geom(N, C, H, W, K, 4);
    int pick = g4.T >= 64 ? WINO_F4 : WINO_F2;
    // fp32 storage promises 1e-5: F(4x4) rounding grows with the reduction length, keep a margin
    if (dtype == WINO_F32 && C > 640) pick = WINO_F2;
    // bfloat16 has 8 significant bits: F(4x4) would sit near 2.5e-2, F(2x2) near 4e-3
    if (dtype == WINO_BF16) pick = WINO_F2;
    // The fused variants (steps (ii) and (iii) in one kernel) where they measured faster with 2-byte storage.  F(2x2): against
    // the F(2x2) chain from 4096 tiles on (128x128 images at batch 2 and everything larger: 0.6-0.9x the time).  F(4x4): against
    // the F(4x4) chain from 4096 tiles on, with at most 512 channels and enough 64x64 blocks for two rounds of workgroups
    // (512 channels at 256x256: 0.96x, 256 at 512x512: 0.85x, 128 at 1024x1024: 0.67x; with fewer tiles 1.2-2.2x slower).
    const Geom g2 = make_geom(N, C, H, W, K, 2);
    if (dtype != WINO_F32 && K >= 32) {
        if (pick == WINO_F2 && g2.T >= 4096) pick = WINO_FUSED_F2;
        const long long blocks4 = (long long)((K + 63) / 64) * ((g4.T + 63) / 64);
        if (pick == WINO_F4 && g4.T >= 4096 && C <= 512 && K <= 512 && blocks4 >= 512) pick = WINO_FUSED_F4;
    }
    return pick;
}

int wino_recommend_variant(int N, int C, int H, int W, int K, int dtype) {
    const int v = wino_resolve_variant(N, C, H, W, K, dtype, WINO_AUTO);
    if (v < 0 || !igemm_dims_ok(N, C, H, W, K, 3, 1)) return v;
    // Measured on the VAE-sized layers: with few channels and many pixels the Winograd path is bound by the
    // traffic of V and M (about 27 bytes per output pixel and channel for F(4x4), 48 for F(2x2)), the direct
    // path by its 18*C*K flops per pixel at 0.6-1.0 PFLOP/s.  256 channels at 512x512: direct 1.25x faster;
    // 512 channels at 256x256: Winograd 1.18x faster.  The crossing is put at sqrt(C*K) = 320 against
    // F(4x4) and 448 against F(2x2).
    // A handful of output channels on a large image (the VAE's 128 -> 3 at 1024 x 1024): the Winograd path would write and
    // re-read a transformed activation tensor far larger than x; the direct path has a one-pass kernel for it (fp16, at
    // least 512 tiles of 8 x 64 pixels; measured 130-160 us against 320-360 us for F(4x4))
    if (dtype == WINO_F16 && K <= 4 && C >= 16 && C % 16 == 0 && W % 8 == 0 &&
        (long long)N * ((H + 7) / 8) * ((W + 63) / 64) >= 512)
        return WINO_DIRECT;
    // where WINO_AUTO takes the fused F(4x4) variant it is also ahead of the direct path (256 channels at 512x512: 342-350 us in
    // either layout against 417 / 356 NCHW / NHWC; 128 at 1024x1024: 530 / 498 against 702 / 541; 512 at 256x256: 254 / 252 against 351 / 326)
    if (v == WINO_FUSED_F4) return v;
    const long long pixels = (long long)N * H * W;
    const long long ck = (long long)C * K;
    const long long cross = v == WINO_F4 ? 320LL * 320LL : 448LL * 448LL;
    if (pixels >= 65536 && ck <= cross && K >= 32) return WINO_DIRECT;
    return v;
}

int wino_transformed_dims(int N, int C, int H, int W, int K, int variant, int* alpha, int* Cp, int* T) {
    if (!wino_variant_ok(variant)) return WINO_ERR_VARIANT;
    if (!dims_ok(N, C, H, W, K, tile_edge(variant))) return WINO_ERR_DIM;
    const Geom g = make_geom(N, C, H, W, K, tile_edge(variant));
    if (alpha) *alpha = g.alpha;
    if (Cp) *Cp = g.Cp;
    if (T) *T = g.T;
    return WINO_OK;
}

size_t wino_filter_bytes(int K, int C, int dtype, int variant) {
    if (variant == WINO_DIRECT) return wino_igemm_filter_bytes(K, C, 3, dtype);
    if (!dtype_ok(dtype) || !wino_variant_ok(variant) || !variant_dtype_ok(variant, dtype) || !dims_ok(1, C, 1, 1, K, tile_edge(variant))) return 0;
    const size_t a = tile_edge(variant) + 2;
    return a * a * (size_t)K * (size_t)round_up(C, 8) * esize(dtype);
}

size_t wino_workspace_bytes(int N, int C, int H, int W, int K, int dtype, int variant) {
    // the direct path: what the NCHW call needs (the channel-last call needs no more than that)
    if (variant == WINO_DIRECT) return wino_igemm_workspace_bytes(N, C, H, W, K, 3, 1, dtype, WINO_NCHW);
    if (!dtype_ok(dtype) || !wino_variant_ok(variant) || !variant_dtype_ok(variant, dtype) || !dims_ok(N, C, H, W, K, tile_edge(variant))) return 0;
    return workspace_layout(make_geom(N, C, H, W, K, tile_edge(variant)), dtype, variant).total;
}

int wino_filter_transform(const void* w, void* w_t_data, int K, int C, int dtype, int variant,
                          wino_filter* out, void* stream) {
    if (!w || !w_t_data || !out) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (variant == WINO_DIRECT) {
        const int rc = wino_igemm_filter_repack(w, w_t_data, K, C, 3, dtype, stream);
        if (rc != WINO_OK) return rc;
        out->data = w_t_data; out->K = K; out->C = C; out->dtype = dtype; out->variant = variant;
        return WINO_OK;
    }
    if (!wino_variant_ok(variant)) return WINO_ERR_VARIANT;
    if (!variant_dtype_ok(variant, dtype)) return WINO_ERR_DTYPE;
    if (!dims_ok(1, C, 1, 1, K, tile_edge(variant)) || K > 65535) return WINO_ERR_DIM;   // grid.y carries k
    if (!aligned16(w) || !aligned16(w_t_data)) return WINO_ERR_ALIGN;
    if (launch_filter_transform(w, w_t_data, K, C, round_up(C, 8), tile_edge(variant), dtype,
                                static_cast<hipStream_t>(stream)) != hipSuccess)
        return WINO_ERR_HIP;
    out->data = w_t_data; out->K = K; out->C = C; out->dtype = dtype; out->variant = variant;
    return WINO_OK;
}

int wino_conv2d_ex(const void* x, const wino_filter* w_t, const float* bias, void* y,
                   int N, int C, int H, int W, int K, int layout,
                   void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_conv_args(x, w_t, bias, y, N, C, H, W, K);
    if (rc != WINO_OK) return rc;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    if (w_t->variant == WINO_DIRECT)
        return wino_igemm_conv2d(x, w_t->data, bias, y, N, C, H, W, K, 3, 1, w_t->dtype, layout, workspace, workspace_bytes, stream);
    const Geom g = make_geom(N, C, H, W, K, tile_edge(w_t->variant));
    const Workspace ws = workspace_layout(g, w_t->dtype, w_t->variant);
    if (!workspace || workspace_bytes < ws.total) return WINO_ERR_WORKSPACE;
    if (!aligned16(workspace)) return WINO_ERR_ALIGN;
    return run_chain(x, w_t, bias, y, g, workspace, layout == WINO_NHWC, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

int wino_conv2d(const void* x, const wino_filter* w_t, const float* bias, void* y,
                int N, int C, int H, int W, int K, void* stream) {
    const int rc = check_conv_args(x, w_t, bias, y, N, C, H, W, K);
    if (rc != WINO_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    void* workspace = nullptr;
    if (w_t->variant == WINO_DIRECT) {
        const size_t need = wino_igemm_workspace_bytes(N, C, H, W, K, 3, 1, w_t->dtype, WINO_NCHW);
        if (hipMallocAsync(&workspace, need, s) != hipSuccess || !workspace) return WINO_ERR_HIP;
        const int rc2 = wino_igemm_conv2d(x, w_t->data, bias, y, N, C, H, W, K, 3, 1, w_t->dtype, WINO_NCHW, workspace, need, stream);
        if (hipFreeAsync(workspace, s) != hipSuccess) return WINO_ERR_HIP;
        return rc2;
    }
    const Geom g = make_geom(N, C, H, W, K, tile_edge(w_t->variant));
    const Workspace ws = workspace_layout(g, w_t->dtype, w_t->variant);
    if (hipMallocAsync(&workspace, ws.total, s) != hipSuccess || !workspace) return WINO_ERR_HIP;
    const int rc2 = run_chain(x, w_t, bias, y, g, workspace, false, nullptr, nullptr, s);
    if (hipFreeAsync(workspace, s) != hipSuccess) return WINO_ERR_HIP;
    return rc2;
}

// ---- the entry point that allocates nothing -----------------------------------------------------------------
// V and M (or the direct path's re-laid x and partial sums) live in a file-scope device array instead of a
// caller's workspace or the stream-ordered allocator.  Each GPU holds its own copy of the array at its own
// address; the address is looked up once per device and kept.
}  // extern "C"

namespace {
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (the array's name itself is only a host-side handle)
int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return WINO_ERR_HIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return WINO_ERR_HIP;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return WINO_OK;
}
}  // namespace

extern "C" {

size_t wino_static_scratch_bytes(void) { return kStaticScratchBytes; }

int wino_conv2d_static(const void* x, const wino_filter* w_t, const float* bias, void* y,
                       int N, int C, int H, int W, int K, int layout, void* stream) {
    const int rc = check_conv_args(x, w_t, bias, y, N, C, H, W, K);
    if (rc != WINO_OK) return rc;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    const size_t need = w_t->variant == WINO_DIRECT
                            ? wino_igemm_workspace_bytes(N, C, H, W, K, 3, 1, w_t->dtype, layout)
                            : workspace_layout(make_geom(N, C, H, W, K, tile_edge(w_t->variant)), w_t->dtype, w_t->variant).total;
    if (need > kStaticScratchBytes) return WINO_ERR_SCRATCH;
    void* ws = nullptr;
    const int rs = static_scratch(&ws);
    if (rs != WINO_OK) return rs;
    // every kernel of the chain writes the part of the scratch it later reads (V with its zero padding, M, partial
    // sums), so nothing a previous call left there is ever read and nothing has to be cleared
    if (w_t->variant == WINO_DIRECT)
        return wino_igemm_conv2d(x, w_t->data, bias, y, N, C, H, W, K, 3, 1, w_t->dtype, layout, need ? ws : nullptr, need, stream);
    const Geom g = make_geom(N, C, H, W, K, tile_edge(w_t->variant));
    return run_chain(x, w_t, bias, y, g, ws, layout == WINO_NHWC, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

size_t wino_groupnorm_stats_bytes(int N, int groups) {
    if (N < 1 || groups < 1 || (long long)N * groups > (1LL << 24)) return 0;
    return groupnorm_stats_bytes(N, groups);
}

int wino_groupnorm_stats(const void* x, float* stats, int N, int C, int H, int W, int groups, float eps,
                         int dtype, int layout, void* stream) {
    if (!x || !stats) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    if (!dims_ok(N, C, H, W, 1, 2) || groups < 1 || C % groups != 0 || (long long)N * groups > (1LL << 24) ||
        (long long)H * W > INT_MAX || !(eps >= 0.f)) return WINO_ERR_DIM;
    if (!aligned16(x) || !aligned16(stats)) return WINO_ERR_ALIGN;
    return launch_groupnorm_stats(x, stats, N, C, H, W, groups, eps, dtype, layout == WINO_NHWC,
                                  static_cast<hipStream_t>(stream)) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
}

int wino_conv2d_fused(const void* x, const wino_filter* w_t, const float* bias, void* y,
                      int N, int C, int H, int W, int K, int layout, const wino_fusion* f,
                      void* workspace, size_t workspace_bytes, void* stream) {
    if (!f) return WINO_ERR_NULL;
    if (f->upsample != 0 && f->upsample != 1) return WINO_ERR_DIM;
    if (f->upsample && ((H | W) & 1)) return WINO_ERR_DIM;
    const int rc = check_conv_args(x, w_t, bias, y, N, C, H, W, K, f->upsample);
    if (rc != WINO_OK) return rc;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    if (w_t->variant == WINO_DIRECT) {
        // the direct path reads x through the upsampling by address arithmetic, adds the vector and the residual
        // in its epilogue, and applies GroupNorm + SiLU while it re-lays x (a channel-last x is then copied once)
        PreOp dpre;
        if (f->gn_stats) {
            if (!f->gn_gamma || !f->gn_beta) return WINO_ERR_NULL;
            if (f->gn_groups < 1 || C % f->gn_groups != 0) return WINO_ERR_DIM;
            if ((reinterpret_cast<uintptr_t>(f->gn_stats) | reinterpret_cast<uintptr_t>(f->gn_gamma) |
                 reinterpret_cast<uintptr_t>(f->gn_beta)) & 3u) return WINO_ERR_ALIGN;
            dpre.stats = f->gn_stats; dpre.gamma = f->gn_gamma; dpre.beta = f->gn_beta;
            dpre.groups = f->gn_groups; dpre.cpg = C / f->gn_groups;
        }
        if (f->addvec && (reinterpret_cast<uintptr_t>(f->addvec) & 3u)) return WINO_ERR_ALIGN;
        const int dt = w_t->dtype;
        const size_t es = esize(dt);
        if (f->residual) {
            if (!aligned16(f->residual)) return WINO_ERR_ALIGN;
            const uintptr_t rb = reinterpret_cast<uintptr_t>(f->residual), re = rb + (size_t)N * K * H * W * es;
            const uintptr_t yb = reinterpret_cast<uintptr_t>(y), ye = yb + (size_t)N * K * H * W * es;
            if (rb != yb && rb < ye && yb < re) return WINO_ERR_ALIAS;
        }
        const int up = f->upsample;
        const size_t xh = f->gn_stats ? igemm_xh_bytes(N, C, H >> up, W >> up, dt, WINO_NCHW)      // always a copy
                                      : igemm_xh_bytes(N, C, H >> up, W >> up, dt, layout);
        const size_t need = xh + igemm_part_bytes(N, C, H, W, K, 3, 1, dt);
        if (need && (!workspace || workspace_bytes < need)) return WINO_ERR_WORKSPACE;
        if (need && !aligned16(workspace)) return WINO_ERR_ALIGN;
        return launch_igemm_conv2d(x, w_t->data, bias, y, N, C, H, W, K, 3, 1, dt, layout == WINO_NHWC, workspace, xh, up,
                                   f->gn_stats ? &dpre : nullptr, f->addvec, f->residual, static_cast<hipStream_t>(stream)) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
    }
    PreOp pre; PostOp post;
    pre.up = f->upsample;
    const bool has_pre = f->gn_stats != nullptr;
    if (has_pre) {
        if (!f->gn_gamma || !f->gn_beta) return WINO_ERR_NULL;
        if (f->gn_groups < 1 || C % f->gn_groups != 0) return WINO_ERR_DIM;
        if ((reinterpret_cast<uintptr_t>(f->gn_stats) | reinterpret_cast<uintptr_t>(f->gn_gamma) |
             reinterpret_cast<uintptr_t>(f->gn_beta)) & 3u) return WINO_ERR_ALIGN;
        pre.stats = f->gn_stats; pre.gamma = f->gn_gamma; pre.beta = f->gn_beta;
        pre.groups = f->gn_groups; pre.cpg = C / f->gn_groups;
    }
    if (f->addvec && (reinterpret_cast<uintptr_t>(f->addvec) & 3u)) return WINO_ERR_ALIGN;
    if (f->residual) {
        if (!aligned16(f->residual)) return WINO_ERR_ALIGN;
        const size_t es = esize(w_t->dtype);
        const uintptr_t rb = reinterpret_cast<uintptr_t>(f->residual), re = rb + (size_t)N * K * H * W * es;
        const uintptr_t yb = reinterpret_cast<uintptr_t>(y), ye = yb + (size_t)N * K * H * W * es;
        if (rb != yb && rb < ye && yb < re) return WINO_ERR_ALIAS;    // identical is fine (each element read, then written, by one lane)
    }
    post.addvec = f->addvec; post.residual = f->residual;
    const Geom g = make_geom(N, C, H, W, K, tile_edge(w_t->variant));
    const Workspace ws = workspace_layout(g, w_t->dtype, w_t->variant);
    if (!workspace || workspace_bytes < ws.total) return WINO_ERR_WORKSPACE;
    if (!aligned16(workspace)) return WINO_ERR_ALIGN;
    if (f->product_fp16 != 0 && f->product_fp16 != 1) return WINO_ERR_DIM;
    return run_chain(x, w_t, bias, y, g, workspace, layout == WINO_NHWC, (has_pre || pre.up) ? &pre : nullptr, &post,
                     static_cast<hipStream_t>(stream), f->product_fp16 != 0);
}

int wino_input_transform(const void* x, void* V, int N, int C, int H, int W,
                         int dtype, int variant, int layout, void* stream) {
    if (!x || !V) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (!wino_variant_ok(variant)) return WINO_ERR_VARIANT;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    if (!dims_ok(N, C, H, W, 1, tile_edge(variant))) return WINO_ERR_DIM;
    if (!aligned16(x) || !aligned16(V)) return WINO_ERR_ALIGN;
    const Geom g = make_geom(N, C, H, W, 1, tile_edge(variant));
    return launch_input_transform(x, V, g, dtype, layout == WINO_NHWC, nullptr, static_cast<hipStream_t>(stream)) == hipSuccess
               ? WINO_OK : WINO_ERR_HIP;
}

int wino_batched_gemm(const void* U, const void* V, float* M, int K, int C, int T,
                      int dtype, int variant, void* stream) {
    if (!U || !V || !M) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (variant != WINO_F2 && variant != WINO_F4) return WINO_ERR_VARIANT;      // the fused variant has no stored product
    if (K < 1 || C < 1 || T < 1 || T > INT_MAX / 2 || !dims_ok(1, C, 1, 1, K, tile_edge(variant))) return WINO_ERR_DIM;
    const unsigned long long a2 = (unsigned long long)(tile_edge(variant) + 2) * (tile_edge(variant) + 2);
    if (a2 * (unsigned long long)T > (1ULL << 40) / (unsigned long long)round_up(C, 8) ||
        a2 * (unsigned long long)T > (1ULL << 40) / (unsigned long long)K) return WINO_ERR_DIM;
    if (!aligned16(U) || !aligned16(V) || !aligned16(M)) return WINO_ERR_ALIGN;
    return launch_batched_gemm(U, V, M, K, round_up(C, 8), T, (int)a2, 1, dtype, false,
                               static_cast<hipStream_t>(stream)) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
}

int wino_batched_gemm_shape(const void* U, const void* V, float* M, int K, int C, int T,
                            int dtype, int variant, int block_shape, void* stream) {
    if (block_shape < 0 || block_shape > 8) return WINO_ERR_VARIANT;
    if (!U || !V || !M) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (variant != WINO_F2 && variant != WINO_F4) return WINO_ERR_VARIANT;
    if (K < 1 || C < 1 || T < 1 || T > INT_MAX / 2 || !dims_ok(1, C, 1, 1, K, tile_edge(variant))) return WINO_ERR_DIM;
    const unsigned long long a2 = (unsigned long long)(variant + 2) * (variant + 2);
    if (a2 * (unsigned long long)T > (1ULL << 40) / (unsigned long long)round_up(C, 8) ||
        a2 * (unsigned long long)T > (1ULL << 40) / (unsigned long long)K) return WINO_ERR_DIM;
    if (!aligned16(U) || !aligned16(V) || !aligned16(M)) return WINO_ERR_ALIGN;
    return launch_batched_gemm(U, V, M, K, round_up(C, 8), T, (int)a2, 1, dtype, false,
                               static_cast<hipStream_t>(stream), block_shape) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
}

int wino_output_transform(const float* M, const float* bias, void* y, int N, int K, int H, int W,
                          int dtype, int variant, int layout, void* stream) {
    if (!M || !y) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (variant != WINO_F2 && variant != WINO_F4) return WINO_ERR_VARIANT;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    if (!dims_ok(N, 1, H, W, K, tile_edge(variant))) return WINO_ERR_DIM;
    if (!aligned16(M) || !aligned16(y)) return WINO_ERR_ALIGN;
    const Geom g = make_geom(N, 1, H, W, K, tile_edge(variant));
    return launch_output_transform(M, bias, y, g, 1, dtype, layout == WINO_NHWC, false, nullptr, static_cast<hipStream_t>(stream)) == hipSuccess
               ? WINO_OK : WINO_ERR_HIP;
}

int wino_fused_gemm_output(const void* U, const void* V, const float* bias, void* y, int N, int C, int H, int W, int K,
                           int dtype, int layout, int block_shape, void* stream) {
    if (!U || !V || !y) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    if (block_shape < -1 || block_shape > 6) return WINO_ERR_VARIANT;
    if (!dims_ok(N, C, H, W, K, 2)) return WINO_ERR_DIM;
    if (!aligned16(U) || !aligned16(V) || !aligned16(y) || (bias && (reinterpret_cast<uintptr_t>(bias) & 3u))) return WINO_ERR_ALIGN;
    const Geom g = make_geom(N, C, H, W, K, 2);
    return launch_fused_gemm_output(U, V, bias, y, g, dtype, layout == WINO_NHWC, nullptr, block_shape,
                                    static_cast<hipStream_t>(stream)) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
}

int wino_fused_f4_gemm_output(const void* U, const void* V, const float* bias, void* y, int N, int C, int H, int W, int K,
                              int dtype, int layout, int block_shape, void* stream) {
    if (!U || !V || !y) return WINO_ERR_NULL;
    if (dtype != WINO_F16 && dtype != WINO_BF16) return WINO_ERR_DTYPE;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    if (block_shape < -1 || block_shape > 1) return WINO_ERR_VARIANT;
    if (!dims_ok(N, C, H, W, K, 4)) return WINO_ERR_DIM;
    if (!aligned16(U) || !aligned16(V) || !aligned16(y) || (bias && (reinterpret_cast<uintptr_t>(bias) & 3u))) return WINO_ERR_ALIGN;
    const Geom g = make_geom(N, C, H, W, K, 4);
    return launch_fused4_gemm_output(U, V, bias, y, g, dtype, layout == WINO_NHWC, nullptr, block_shape,
                                     static_cast<hipStream_t>(stream)) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
}

int wino_direct_conv2d(const void* x, const void* w, const float* bias, void* y,
                       int N, int C, int H, int W, int K, int dtype, void* stream) {
    if (!x || !w || !y) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (!dims_ok(N, C, H, W, K, 2)) return WINO_ERR_DIM;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return WINO_ERR_ALIGN;
    const size_t es = esize(dtype);
    const uintptr_t xb = reinterpret_cast<uintptr_t>(x), xe = xb + (size_t)N * C * H * W * es;
    const uintptr_t yb = reinterpret_cast<uintptr_t>(y), ye = yb + (size_t)N * K * H * W * es;
    if (xb < ye && yb < xe) return WINO_ERR_ALIAS;
    return launch_direct_conv2d(x, w, bias, y, N, C, H, W, K, dtype,
                                static_cast<hipStream_t>(stream)) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
}


size_t wino_igemm_filter_bytes(int K, int C, int R, int dtype) {
    if (!dtype_ok(dtype) || !igemm_dims_ok(1, C, 1, 1, K, R, 1)) return 0;
    const size_t Cp = (size_t)round_up(C, 8);
    return ((size_t)R * R * K * Cp + Cp) * esize(dtype);
}

int wino_igemm_filter_repack(const void* w, void* w_r, int K, int C, int R, int dtype, void* stream) {
    if (!w || !w_r) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (!igemm_dims_ok(1, C, 1, 1, K, R, 1)) return WINO_ERR_DIM;
    if (!aligned16(w) || !aligned16(w_r)) return WINO_ERR_ALIGN;
    return launch_igemm_filter_repack(w, w_r, K, C, R, dtype, static_cast<hipStream_t>(stream)) == hipSuccess
               ? WINO_OK : WINO_ERR_HIP;
}


size_t wino_igemm_workspace_bytes(int N, int C, int H, int W, int K, int R, int stride, int dtype, int layout) {
    if (!dtype_ok(dtype) || !igemm_dims_ok(N, C, H, W, K, R, stride)) return 0;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return 0;
    return igemm_xh_bytes(N, C, H, W, dtype, layout) + igemm_part_bytes(N, C, H, W, K, R, stride, dtype);
}

int wino_igemm_conv2d(const void* x, const void* w_r, const float* bias, void* y,
                      int N, int C, int H, int W, int K, int R, int stride, int dtype, int layout,
                      void* workspace, size_t workspace_bytes, void* stream) {
    if (!x || !w_r || !y) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    if (!igemm_dims_ok(N, C, H, W, K, R, stride)) return WINO_ERR_DIM;
    if (!aligned16(x) || !aligned16(w_r) || !aligned16(y) || (bias && (reinterpret_cast<uintptr_t>(bias) & 3u)))
        return WINO_ERR_ALIGN;
    const int pad = (R - 1) / 2;
    const int Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - R) / stride + 1;
    const size_t es = esize(dtype);
    const uintptr_t xb = reinterpret_cast<uintptr_t>(x), xe = xb + (size_t)N * C * H * W * es;
    const uintptr_t yb = reinterpret_cast<uintptr_t>(y), ye = yb + (size_t)N * K * Ho * Wo * es;
    if (xb < ye && yb < xe) return WINO_ERR_ALIAS;
    const size_t need = wino_igemm_workspace_bytes(N, C, H, W, K, R, stride, dtype, layout);
    if (need && (!workspace || workspace_bytes < need)) return WINO_ERR_WORKSPACE;
    if (need && !aligned16(workspace)) return WINO_ERR_ALIGN;
    return launch_igemm_conv2d(x, w_r, bias, y, N, C, H, W, K, R, stride, dtype, layout == WINO_NHWC,
                               workspace, igemm_xh_bytes(N, C, H, W, dtype, layout), 0, nullptr, nullptr, nullptr,
                               static_cast<hipStream_t>(stream)) == hipSuccess
               ? WINO_OK : WINO_ERR_HIP;
}

namespace {
bool scale_ok(float v) { return v > 0.f && v < 3.0e38f && v == v; }
size_t fp8_xq_bytes(int N, int C, int H, int W) { return align_up((size_t)N * H * W * (size_t)round_up(C, 16)); }
size_t fp8_part_bytes(int N, int C, int H, int W, int K, int R, int stride) {
    const int pad = (R - 1) / 2;
    const long long T = (long long)N * ((H + 2 * pad - R) / stride + 1) * ((W + 2 * pad - R) / stride + 1);
    const int sp = igemm_split((int)T, K, round_up(C, 16), R, -1);
    return sp > 1 ? align_up((size_t)sp * (size_t)K * (size_t)T * sizeof(float)) : 0;
}
}  // namespace

size_t wino_fp8_filter_bytes(int K, int C, int R) {
    if (!igemm_dims_ok(1, C, 1, 1, K, R, 1)) return 0;
    const size_t Cq = (size_t)round_up(C, 16);
    return (size_t)R * R * K * Cq + Cq;
}

int wino_fp8_filter_quantize(const void* w, void* w_q, int K, int C, int R, int dtype, float scale_w, void* stream) {
    if (!w || !w_q) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (!igemm_dims_ok(1, C, 1, 1, K, R, 1) || !scale_ok(scale_w)) return WINO_ERR_DIM;
    if (!aligned16(w) || !aligned16(w_q)) return WINO_ERR_ALIGN;
    return launch_igemm_fp8_filter_quant(w, w_q, K, C, R, dtype, scale_w, static_cast<hipStream_t>(stream)) == hipSuccess
               ? WINO_OK : WINO_ERR_HIP;
}

size_t wino_fp8_workspace_bytes(int N, int C, int H, int W, int K, int R, int stride) {
    if (!igemm_dims_ok(N, C, H, W, K, R, stride)) return 0;
    return fp8_xq_bytes(N, C, H, W) + fp8_part_bytes(N, C, H, W, K, R, stride);
}

int wino_fp8_conv2d(const void* x, const void* w_q, const float* bias, void* y,
                    int N, int C, int H, int W, int K, int R, int stride, int dtype, int layout,
                    float scale_x, float scale_w, const wino_fusion* f,
                    void* workspace, size_t workspace_bytes, void* stream) {
    if (!x || !w_q || !y) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    if (!igemm_dims_ok(N, C, H, W, K, R, stride) || !scale_ok(scale_x) || !scale_ok(scale_w)) return WINO_ERR_DIM;
    const int up = f ? f->upsample : 0;
    if (up != 0 && up != 1) return WINO_ERR_DIM;
    if (up && ((H | W) & 1)) return WINO_ERR_DIM;
    if (!aligned16(x) || !aligned16(w_q) || !aligned16(y) || (bias && (reinterpret_cast<uintptr_t>(bias) & 3u)))
        return WINO_ERR_ALIGN;
    const int pad = (R - 1) / 2;
    const int Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - R) / stride + 1;
    const size_t es = esize(dtype);
    const uintptr_t xb = reinterpret_cast<uintptr_t>(x), xe = xb + (size_t)N * C * (H >> up) * (W >> up) * es;
    const uintptr_t yb = reinterpret_cast<uintptr_t>(y), ye = yb + (size_t)N * K * Ho * Wo * es;
    if (xb < ye && yb < xe) return WINO_ERR_ALIAS;
    PreOp pre;
    const float* addvec = nullptr; const void* residual = nullptr;
    if (f) {
        if (f->gn_stats) {
            if (!f->gn_gamma || !f->gn_beta) return WINO_ERR_NULL;
            if (f->gn_groups < 1 || C % f->gn_groups != 0) return WINO_ERR_DIM;
            if ((reinterpret_cast<uintptr_t>(f->gn_stats) | reinterpret_cast<uintptr_t>(f->gn_gamma) |
                 reinterpret_cast<uintptr_t>(f->gn_beta)) & 3u) return WINO_ERR_ALIGN;
            pre.stats = f->gn_stats; pre.gamma = f->gn_gamma; pre.beta = f->gn_beta;
            pre.groups = f->gn_groups; pre.cpg = C / f->gn_groups;
        }
        if (f->addvec && (reinterpret_cast<uintptr_t>(f->addvec) & 3u)) return WINO_ERR_ALIGN;
        if (f->residual) {
            if (!aligned16(f->residual)) return WINO_ERR_ALIGN;
            const uintptr_t rb = reinterpret_cast<uintptr_t>(f->residual), re = rb + (size_t)N * K * Ho * Wo * es;
            if (rb != yb && rb < ye && yb < re) return WINO_ERR_ALIAS;
        }
        addvec = f->addvec; residual = f->residual;
    }
    const size_t xq = fp8_xq_bytes(N, C, H >> up, W >> up);
    const size_t need = xq + fp8_part_bytes(N, C, H, W, K, R, stride);
    if (!workspace || workspace_bytes < need) return WINO_ERR_WORKSPACE;
    if (!aligned16(workspace)) return WINO_ERR_ALIGN;
    return launch_igemm_fp8_conv2d(x, w_q, bias, y, N, C, H, W, K, R, stride, dtype, layout == WINO_NHWC, workspace, xq, up,
                                   pre.stats ? &pre : nullptr, addvec, residual, scale_x, scale_w,
                                   static_cast<hipStream_t>(stream)) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
}

// ---- Winograd F(2x2,3x3) with 8-bit integer U and V -------------------------------------------------------------
namespace {
constexpr int kI8MaxC = 65536;                    // 65536 * 127^2 < 2^31: the int32 sums cannot overflow
inline int i8_cq(int C) { return round_up(C, 16); }
bool i8_dims_ok(int N, int C, int H, int W, int K) { return dims_ok(N, C, H, W, K, 2) && C <= kI8MaxC; }
size_t i8_codes_bytes(int rows, int Cq) { return align_up((size_t)16 * (size_t)rows * (size_t)Cq); }
size_t i8_steps_bytes(int rows) { return align_up((size_t)16 * (size_t)rows * sizeof(float)); }
int i8_split(const Geom& g, bool nhwc) {
    return nhwc ? gemm_split(g.T, g.K, i8_cq(g.C), 16, DT_I8) : gemm_split(g.K, g.T, i8_cq(g.C), 16, DT_I8);
}
}  // namespace

size_t wino_i8_filter_bytes(int K, int C) {
    if (!i8_dims_ok(1, C, 1, 1, K)) return 0;
    return i8_codes_bytes(K, i8_cq(C)) + i8_steps_bytes(K);
}

int wino_i8_filter_transform(const void* w, void* u_q, int K, int C, int dtype, void* stream) {
    if (!w || !u_q) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (!i8_dims_ok(1, C, 1, 1, K)) return WINO_ERR_DIM;
    if (!aligned16(w) || !aligned16(u_q)) return WINO_ERR_ALIGN;
    float* dU = reinterpret_cast<float*>(static_cast<unsigned char*>(u_q) + i8_codes_bytes(K, i8_cq(C)));
    return launch_filter_quant_i8(w, u_q, dU, K, C, i8_cq(C), dtype, static_cast<hipStream_t>(stream)) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
}

size_t wino_i8_workspace_bytes(int N, int C, int H, int W, int K) {
    if (!i8_dims_ok(N, C, H, W, K)) return 0;
    const Geom g = make_geom(N, C, H, W, K, 2);
    const int sp_a = i8_split(g, false), sp_b = i8_split(g, true);
    return i8_codes_bytes(g.T, i8_cq(C)) + i8_steps_bytes(g.T) +
           align_up((size_t)16 * (size_t)K * (size_t)g.T * sizeof(float) * (size_t)(sp_a > sp_b ? sp_a : sp_b));
}

int wino_i8_input_transform(const void* x, void* Vq, float* dV, int N, int C, int H, int W, int dtype, int layout, void* stream) {
    if (!x || !Vq || !dV) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    if (!i8_dims_ok(N, C, H, W, 1)) return WINO_ERR_DIM;
    if (!aligned16(x) || !aligned16(Vq) || (reinterpret_cast<uintptr_t>(dV) & 3u)) return WINO_ERR_ALIGN;
    const Geom g = make_geom(N, C, H, W, 1, 2);
    return launch_input_transform_i8(x, Vq, dV, g, i8_cq(C), dtype, layout == WINO_NHWC, static_cast<hipStream_t>(stream)) == hipSuccess
               ? WINO_OK : WINO_ERR_HIP;
}

int wino_i8_batched_gemm(const void* Uq, const float* dU, const void* Vq, const float* dV, float* M, int K, int C, int T,
                         int block_shape, void* stream) {
    if (block_shape < -1 || block_shape > 8) return WINO_ERR_VARIANT;
    if (!Uq || !dU || !Vq || !dV || !M) return WINO_ERR_NULL;
    if (K < 1 || C < 1 || T < 1 || T > INT_MAX / 2 || !i8_dims_ok(1, C, 1, 1, K)) return WINO_ERR_DIM;
    if (16ULL * (unsigned long long)T > (1ULL << 40) / (unsigned long long)i8_cq(C) ||
        16ULL * (unsigned long long)T > (1ULL << 40) / (unsigned long long)K) return WINO_ERR_DIM;
    if (!aligned16(Uq) || !aligned16(Vq) || !aligned16(M) ||
        ((reinterpret_cast<uintptr_t>(dU) | reinterpret_cast<uintptr_t>(dV)) & 3u)) return WINO_ERR_ALIGN;
    return launch_batched_gemm_i8(Uq, dU, Vq, dV, M, K, i8_cq(C), T, 16, 1, static_cast<hipStream_t>(stream), block_shape) == hipSuccess
               ? WINO_OK : WINO_ERR_HIP;
}

int wino_i8_conv2d(const void* x, const void* u_q, const float* bias, void* y, int N, int C, int H, int W, int K,
                   int dtype, int layout, void* workspace, size_t workspace_bytes, void* stream) {
    if (!x || !u_q || !y) return WINO_ERR_NULL;
    if (!dtype_ok(dtype)) return WINO_ERR_DTYPE;
    if (layout != WINO_NCHW && layout != WINO_NHWC) return WINO_ERR_LAYOUT;
    if (!i8_dims_ok(N, C, H, W, K)) return WINO_ERR_DIM;
    if (!aligned16(x) || !aligned16(u_q) || !aligned16(y) || (bias && (reinterpret_cast<uintptr_t>(bias) & 3u))) return WINO_ERR_ALIGN;
    const size_t es = esize(dtype);
    const uintptr_t xb = reinterpret_cast<uintptr_t>(x), xe = xb + (size_t)N * C * H * W * es;
    const uintptr_t yb = reinterpret_cast<uintptr_t>(y), ye = yb + (size_t)N * K * H * W * es;
    if (xb < ye && yb < xe) return WINO_ERR_ALIAS;
    if (!workspace || workspace_bytes < wino_i8_workspace_bytes(N, C, H, W, K)) return WINO_ERR_WORKSPACE;
    if (!aligned16(workspace)) return WINO_ERR_ALIGN;
    const bool nhwc = layout == WINO_NHWC;
    const Geom g = make_geom(N, C, H, W, K, 2);
    const int Cq = i8_cq(C);
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    void* Vq = ws;
    float* dV = reinterpret_cast<float*>(ws + i8_codes_bytes(g.T, Cq));
    float* M = reinterpret_cast<float*>(ws + i8_codes_bytes(g.T, Cq) + i8_steps_bytes(g.T));
    const float* dU = reinterpret_cast<const float*>(static_cast<const unsigned char*>(u_q) + i8_codes_bytes(K, Cq));
    if (launch_input_transform_i8(x, Vq, dV, g, Cq, dtype, nhwc, s) != hipSuccess) return WINO_ERR_HIP;
    const int nsplit = i8_split(g, nhwc);
    // channel-last: operands swapped, so the product comes out as M[16][T][K], k contiguous
    const hipError_t ge = nhwc ? launch_batched_gemm_i8(Vq, dV, u_q, dU, M, g.T, Cq, g.K, 16, nsplit, s)
                               : launch_batched_gemm_i8(u_q, dU, Vq, dV, M, g.K, Cq, g.T, 16, nsplit, s);
    if (ge != hipSuccess) return WINO_ERR_HIP;
    return launch_output_transform(M, bias, y, g, nsplit, dtype, nhwc, false, nullptr, s) == hipSuccess ? WINO_OK : WINO_ERR_HIP;
}

}  // extern "C"
