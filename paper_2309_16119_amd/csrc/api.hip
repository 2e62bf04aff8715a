// The C ABI of the library: argument validation (host only, before any HIP call),
// workspace carving, kernel selection, and the benchmark timing hook.
// Declarations and the contract of every entry point are in include/modulora.h.
#include "modulora.h"

#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <string>
#include <cmath>
#include <vector>

#include "launch.h"

namespace {

constexpr int32_t kMaxDim = 1 << 20;
constexpr int32_t kMaxTokens = 1 << 22;
constexpr int32_t kMaxRank = 64;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align256(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

int check_layer_shape(const modulora_qweight *w) {
    if (!w) return MODULORA_ERR_NULL;
    if (w->bits != 2 && w->bits != 3 && w->bits != 4) return MODULORA_ERR_BITS;
    if (w->d_in < 32 || w->d_in > kMaxDim || w->d_out < 8 || w->d_out > kMaxDim) return MODULORA_ERR_SHAPE;
    if (w->d_in % 32 != 0 || w->d_out % 8 != 0) return MODULORA_ERR_SHAPE;
    if (w->group_size <= 0 || w->group_size % 32 != 0 || w->d_in % w->group_size != 0) return MODULORA_ERR_GROUP;
    return MODULORA_OK;
}

int check_layer(const modulora_qweight *w) {
    const int s = check_layer_shape(w);
    if (s != MODULORA_OK) return s;
    if (!w->qweight || !w->scales || !w->zeros) return MODULORA_ERR_NULL;
    if (!aligned16(w->qweight) || !aligned16(w->scales) || !aligned16(w->zeros)) return MODULORA_ERR_ALIGN;
    return MODULORA_OK;
}

int check_rank(int32_t r, const float *A, const float *B, bool allow_zero) {
    if (r < (allow_zero ? 0 : 1) || r > kMaxRank) return MODULORA_ERR_RANK;
    if (r > 0) {
        if (!A || !B) return MODULORA_ERR_RANK;
        if (!aligned16(A) || !aligned16(B)) return MODULORA_ERR_ALIGN;
    }
    return MODULORA_OK;
}

mlr::LayerView view_of(const modulora_qweight *w) {
    mlr::LayerView v;
    v.K = w->d_in;
    v.N = w->d_out;
    v.bits = w->bits;
    v.group = w->group_size;
    v.qweight = w->qweight;
    v.scales = w->scales;
    v.zeros = w->zeros;
    return v;
}

// Workspace carving, shared by the size query and the entry points.
struct WsLayout {
    size_t act_ext, w_ext, p0, p1, gpart, gemm_part, dpart, total;
    size_t gemm_part_bytes;      // size of the region at gemm_part
};

WsLayout ws_layout(int32_t K, int32_t N, int32_t M, int32_t r) {
    WsLayout l{};
    // the streaming kernels for a handful of tokens keep the slices' partial tiles and the
    // adapter partial sums in the workspace (also when r == 0)
    const size_t small = M <= mlr::SMALLM_MAX_M ? mlr::smallm_ws_bytes(K, N, r) : 0;
    // fp32 partial tiles of the split contraction of the 256 x 256 kernel (also when r == 0)
    const size_t part = align256(mlr::gemm_partial_bytes(M, K, N));
    l.gemm_part_bytes = part;
    if (r <= 0) {
        l.gemm_part = 0;
        l.total = small > part ? small : part;
        return l;
    }
    const size_t RE = (size_t)mlr::lora_ext_len(r);
    const size_t maxdim = (size_t)(K > N ? K : N);
    size_t off = 0;
    l.act_ext = off; off += align256((size_t)M * RE * 2);
    l.w_ext = off;   off += align256(maxdim * RE * 2);
    l.p0 = off;      off += align256((size_t)M * r * 4);
    l.p1 = off;      off += align256((size_t)M * r * 4);
    l.gpart = off;   off += align256(mlr::grad_geom(M, K, N, r).partial_floats * 4);
    l.gemm_part = off; off += part;
    l.dpart = off;   off += align256(mlr::lora_down_partial_bytes(M, K, N, r));
    l.total = off > small ? off : small;
    return l;
}

// What modulora_fwd alone touches for this layer (no backward, no adapter-gradient regions), for
// a scratch buffer of `avail` bytes: the M <= 16 stream's exact need, or the adapter operands of
// the tile kernels plus -- only if they still fit -- the partial tiles of a split contraction
// (without them the 256 x 256 kernel runs whole tiles).
WsLayout ws_layout_fwd(const mlr::LayerView &v, int32_t M, int32_t r, size_t avail) {
    WsLayout l{};
    if (mlr::smallm_fwd_supported(v, M)) {
        l.total = mlr::smallm_fwd_ws_bytes(v, r);
        return l;
    }
    size_t off = 0;
    if (r > 0) {
        const size_t RE = (size_t)mlr::lora_ext_len(r);
        l.act_ext = off; off += align256((size_t)M * RE * 2);
        l.w_ext = off;   off += align256((size_t)v.N * RE * 2);
        l.p0 = off;      off += align256((size_t)M * r * 4);
        l.dpart = off;   off += align256(mlr::lora_down_partial_bytes(M, v.K, v.N, r));
    }
    const size_t part = align256(mlr::big_plan(M, v.K, v.N).partial_bytes());
    l.gemm_part = off;
    if (off + part <= avail) {
        l.gemm_part_bytes = part;
        off += part;
    }
    l.total = off;
    return l;
}

int check_workspace(const WsLayout &l, const void *ws, size_t bytes) {
    if (l.total == 0) return MODULORA_OK;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || bytes < l.total) return MODULORA_ERR_WORKSPACE;
    return MODULORA_OK;
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? MODULORA_OK : MODULORA_ERR_HIP; }

// ---- forward: validation and body, shared by modulora_fwd and modulora_fwd_static ----------
int check_fwd_args(const modulora_qweight *w, const uint16_t *X, int32_t M, const float *A, const float *B, int32_t r,
                   const uint16_t *Y, const float *XA) {
    int s = check_layer(w);
    if (s != MODULORA_OK) return s;
    if (!X || !Y) return MODULORA_ERR_NULL;
    if (M < 1 || M > kMaxTokens) return MODULORA_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(Y) || (XA && !aligned16(XA))) return MODULORA_ERR_ALIGN;
    return check_rank(r, A, B, true);
}

int run_fwd(const modulora_qweight *w, const uint16_t *X, int32_t M, const float *A, const float *B, int32_t r,
            float lora_scale, uint16_t *Y, float *XA, char *ws, const WsLayout &l, hipStream_t st) {
    if (mlr::smallm_fwd_supported(view_of(w), M)) {
        mlr::SmallArgs sa{};
        sa.w = view_of(w);
        sa.act = X; sa.M = M; sa.out = Y;
        sa.A = A; sa.B = B; sa.r = r; sa.lora_scale = lora_scale;
        sa.P_out = XA; sa.ws = ws;
        return hip_status(mlr::launch_smallm_fwd(sa, st));
    }
    mlr::GemmArgs g{};
    g.w = view_of(w);
    g.backward = false;
    g.act = X;
    g.M = M;
    g.out = Y;
    g.partials = l.gemm_part_bytes ? reinterpret_cast<float *>(ws + l.gemm_part) : nullptr;
    g.partials_bytes = l.gemm_part_bytes;
    if (r > 0) {
        mlr::DownArgs d{};
        d.act = X; d.M = M; d.C = w->d_in; d.r = r;
        d.Fm = A; d.f_is_A = true;
        d.P = XA ? XA : reinterpret_cast<float *>(ws + l.p0);
        d.lora_scale = lora_scale;
        d.act_ext = reinterpret_cast<uint16_t *>(ws + l.act_ext);
        d.RE = mlr::lora_ext_len(r);
        d.w_ext = reinterpret_cast<uint16_t *>(ws + l.w_ext);
        d.Wsrc = B; d.w_from_A = false; d.Cw = w->d_out;
        d.partials = reinterpret_cast<float *>(ws + l.dpart);
        const int s = hip_status(mlr::launch_lora_down(d, st));
        if (s != MODULORA_OK) return s;
        g.act_ext = d.act_ext;
        g.w_ext = d.w_ext;
        g.RE = d.RE;
    }
    return hip_status(mlr::launch_gemm(g, st));
}

// ---- the library's own scratch for modulora_fwd_static ---------------------------------------
// One array per GPU, in that GPU's memory from the moment the code object is loaded there until
// the process ends.  In host code the array's name is only a handle: the device address comes
// from hipGetSymbolAddress, once per device, and only that pointer is ever given to kernels.
constexpr size_t kStaticScratchBytes = MODULORA_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

}  // namespace

static __device__ __align__(256) unsigned char scratch[MODULORA_STATIC_SCRATCH_BYTES];

namespace {

int static_scratch(char **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MODULORA_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return MODULORA_ERR_HIP;
        if ((reinterpret_cast<uintptr_t>(p) & 255u) != 0) return MODULORA_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<char *>(g_scratch_ptr[dev]);
    return MODULORA_OK;
}

// ---- profiling state ------------------------------------------------------------
struct ProfRecord {
    const char *name;
    hipEvent_t start, stop;
};
bool g_prof_on = false;
std::vector<ProfRecord> g_prof;

}  // namespace

namespace mlr {

bool prof_events(const char *kernel_name, hipEvent_t *start, hipEvent_t *stop) {
    if (!g_prof_on) return false;
    ProfRecord rec{kernel_name, nullptr, nullptr};
    if (hipEventCreate(&rec.start) != hipSuccess) return false;
    if (hipEventCreate(&rec.stop) != hipSuccess) {
        (void)hipEventDestroy(rec.start);
        return false;
    }
    g_prof.push_back(rec);
    *start = rec.start;
    *stop = rec.stop;
    return true;
}

}  // namespace mlr

extern "C" {

const char *modulora_status_string(int status) {
    switch (status) {
        case MODULORA_OK: return "ok";
        case MODULORA_ERR_NULL: return "a required pointer is NULL";
        case MODULORA_ERR_SHAPE: return "d_in, d_out or M out of range or not divisible as required";
        case MODULORA_ERR_BITS: return "bits must be 2, 3 or 4";
        case MODULORA_ERR_GROUP: return "group_size must be a multiple of 32 that divides d_in";
        case MODULORA_ERR_ALIGN: return "a pointer is not 16-byte aligned";
        case MODULORA_ERR_RANK: return "LoRA rank out of range, or A/B missing";
        case MODULORA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case MODULORA_ERR_HIP: return "a HIP call failed";
        case MODULORA_ERR_HYPER: return "optimizer step or hyper-parameter out of range";
        default: return "unknown status";
    }
}

size_t modulora_workspace_bytes(const modulora_qweight *w, int32_t M, int32_t r) {
    if (check_layer_shape(w) != MODULORA_OK) return 0;
    if (M < 1 || M > kMaxTokens || r < 0 || r > kMaxRank) return 0;
    return ws_layout(w->d_in, w->d_out, M, r).total;
}

int modulora_dequant(const modulora_qweight *w, uint16_t *What_bf16, void *stream) {
    const int s = check_layer(w);
    if (s != MODULORA_OK) return s;
    if (!What_bf16) return MODULORA_ERR_NULL;
    if (!aligned16(What_bf16)) return MODULORA_ERR_ALIGN;
    return hip_status(mlr::launch_dequant(view_of(w), What_bf16, static_cast<hipStream_t>(stream)));
}

int modulora_fwd(const modulora_qweight *w, const uint16_t *X, int32_t M, const float *A, const float *B,
                 int32_t r, float lora_scale, uint16_t *Y, float *XA, void *workspace,
                 size_t workspace_bytes, void *stream) {
    int s = check_fwd_args(w, X, M, A, B, r, Y, XA);
    if (s != MODULORA_OK) return s;
    const WsLayout l = ws_layout(w->d_in, w->d_out, M, r);
    if ((s = check_workspace(l, workspace, workspace_bytes)) != MODULORA_OK) return s;
    return run_fwd(w, X, M, A, B, r, lora_scale, Y, XA, static_cast<char *>(workspace), l, static_cast<hipStream_t>(stream));
}

int modulora_fwd_static(const modulora_qweight *w, const uint16_t *X, int32_t M, const float *A, const float *B,
                        int32_t r, float lora_scale, uint16_t *Y, float *XA, void *stream) {
    int s = check_fwd_args(w, X, M, A, B, r, Y, XA);
    if (s != MODULORA_OK) return s;
    const WsLayout l = ws_layout_fwd(view_of(w), M, r, kStaticScratchBytes);
    if (l.total > kStaticScratchBytes) return MODULORA_ERR_WORKSPACE;     // beyond the library's scratch
    char *ws = nullptr;
    if ((s = static_scratch(&ws)) != MODULORA_OK) return s;
    return run_fwd(w, X, M, A, B, r, lora_scale, Y, XA, ws, l, static_cast<hipStream_t>(stream));
}

int modulora_bwd_input(const modulora_qweight *w, const uint16_t *dY, int32_t M, const float *A,
                       const float *B, int32_t r, float lora_scale, uint16_t *dX, float *dYBt,
                       void *workspace, size_t workspace_bytes, void *stream) {
    int s = check_layer(w);
    if (s != MODULORA_OK) return s;
    if (!dY || !dX) return MODULORA_ERR_NULL;
    if (M < 1 || M > kMaxTokens) return MODULORA_ERR_SHAPE;
    if (!aligned16(dY) || !aligned16(dX) || (dYBt && !aligned16(dYBt))) return MODULORA_ERR_ALIGN;
    if ((s = check_rank(r, A, B, true)) != MODULORA_OK) return s;
    const WsLayout l = ws_layout(w->d_in, w->d_out, M, r);
    if ((s = check_workspace(l, workspace, workspace_bytes)) != MODULORA_OK) return s;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    if (mlr::smallm_bwd_supported(view_of(w), M)) {
        mlr::SmallArgs sa{};
        sa.w = view_of(w);
        sa.act = dY; sa.M = M; sa.out = dX;
        sa.A = A; sa.B = B; sa.r = r; sa.lora_scale = lora_scale;
        sa.P_out = dYBt; sa.ws = ws;
        return hip_status(mlr::launch_smallm_bwd(sa, st));
    }
    mlr::GemmArgs g{};
    g.w = view_of(w);
    g.backward = true;
    g.act = dY;
    g.M = M;
    g.out = dX;
    g.partials = reinterpret_cast<float *>(ws + l.gemm_part);
    g.partials_bytes = l.gemm_part_bytes;
    if (r > 0) {
        mlr::DownArgs d{};
        d.act = dY; d.M = M; d.C = w->d_out; d.r = r;
        d.Fm = B; d.f_is_A = false;
        d.P = dYBt ? dYBt : reinterpret_cast<float *>(ws + l.p0);
        d.lora_scale = lora_scale;
        d.act_ext = reinterpret_cast<uint16_t *>(ws + l.act_ext);
        d.RE = mlr::lora_ext_len(r);
        d.w_ext = reinterpret_cast<uint16_t *>(ws + l.w_ext);
        d.Wsrc = A; d.w_from_A = true; d.Cw = w->d_in;
        d.partials = reinterpret_cast<float *>(ws + l.dpart);
        if ((s = hip_status(mlr::launch_lora_down(d, st))) != MODULORA_OK) return s;
        g.act_ext = d.act_ext;
        g.w_ext = d.w_ext;
        g.RE = d.RE;
    }
    return hip_status(mlr::launch_gemm(g, st));
}

int modulora_bwd_lora(int32_t d_in, int32_t d_out, int32_t M, int32_t r, float lora_scale,
                      const uint16_t *X, const uint16_t *dY, const float *A, const float *B,
                      const float *XA, const float *dYBt, float *dA, float *dB, int32_t accumulate,
                      void *workspace, size_t workspace_bytes, void *stream) {
    if (d_in < 32 || d_in > kMaxDim || d_out < 8 || d_out > kMaxDim || d_in % 32 != 0 || d_out % 8 != 0)
        return MODULORA_ERR_SHAPE;
    if (M < 1 || M > kMaxTokens) return MODULORA_ERR_SHAPE;
    if (!X || !dY || !dA || !dB) return MODULORA_ERR_NULL;
    int s = check_rank(r, A, B, false);
    if (s != MODULORA_OK) return s;
    if (!aligned16(X) || !aligned16(dY) || !aligned16(dA) || !aligned16(dB) || (XA && !aligned16(XA)) ||
        (dYBt && !aligned16(dYBt)))
        return MODULORA_ERR_ALIGN;
    const WsLayout l = ws_layout(d_in, d_out, M, r);
    if ((s = check_workspace(l, workspace, workspace_bytes)) != MODULORA_OK) return s;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    if (!XA) {
        mlr::DownArgs d{};
        d.act = X; d.M = M; d.C = d_in; d.r = r; d.Fm = A; d.f_is_A = true;
        d.P = reinterpret_cast<float *>(ws + l.p0);
        d.lora_scale = lora_scale;
        d.partials = reinterpret_cast<float *>(ws + l.dpart);
        if ((s = hip_status(mlr::launch_lora_down(d, st))) != MODULORA_OK) return s;
        XA = d.P;
    }
    if (!dYBt) {
        mlr::DownArgs d{};
        d.act = dY; d.M = M; d.C = d_out; d.r = r; d.Fm = B; d.f_is_A = false;
        d.P = reinterpret_cast<float *>(ws + l.p1);
        d.lora_scale = lora_scale;
        d.partials = reinterpret_cast<float *>(ws + l.dpart);
        if ((s = hip_status(mlr::launch_lora_down(d, st))) != MODULORA_OK) return s;
        dYBt = d.P;
    }
    mlr::GradPairArgs ga{};
    ga.X = X; ga.dY = dY; ga.M = M; ga.K = d_in; ga.N = d_out; ga.r = r;
    ga.XA = XA; ga.dYBt = dYBt; ga.lora_scale = lora_scale;
    ga.dA = dA; ga.dB = dB; ga.accumulate = accumulate ? 1 : 0;
    ga.partials = reinterpret_cast<float *>(ws + l.gpart);
    return hip_status(mlr::launch_lora_grad_pair(ga, st));
}

// ---- the paper-literal variant (float zero point, binary16, bias) ---------------------------
namespace {
int check_layer_f16(const modulora_qweight_f16 *w, bool pointers) {
    if (!w) return MODULORA_ERR_NULL;
    modulora_qweight shape{w->d_in, w->d_out, w->bits, w->group_size, nullptr, nullptr, nullptr};
    const int s = check_layer_shape(&shape);
    if (s != MODULORA_OK || !pointers) return s;
    if (!w->qweight || !w->scales || !w->zeros) return MODULORA_ERR_NULL;
    if (!aligned16(w->qweight) || !aligned16(w->scales) || !aligned16(w->zeros) || (w->bias && !aligned16(w->bias)))
        return MODULORA_ERR_ALIGN;
    return MODULORA_OK;
}
mlr::F16Layer view_of(const modulora_qweight_f16 *w) {
    return mlr::F16Layer{w->d_in, w->d_out, w->bits, w->group_size, w->qweight, w->scales, w->zeros, w->bias};
}
struct F16Ws {
    size_t p0, p1, gpart, dpart, gemm_part, total;
};
F16Ws f16_ws(int32_t K, int32_t N, int32_t M, int32_t r) {
    F16Ws l{};
    size_t off = 0;
    if (r > 0) {
        l.p0 = off;    off += align256((size_t)M * r * 4);
        l.p1 = off;    off += align256((size_t)M * r * 4);
        l.gpart = off; off += align256(mlr::grad_geom(M, K, N, r).partial_floats * 4);
        l.dpart = off; off += align256(mlr::lora_down_partial_bytes(M, K, N, r));   // slices of the rank-r projection
    }
    l.gemm_part = off; off += align256(mlr::gemm_partial_bytes(M, K, N));   // partial tiles of the 256 x 256 kernel
    l.total = off;
    // the streaming kernels for a handful of tokens lay out their own scratch from the start of the workspace
    if (M <= mlr::SMALLM_MAX_M) {
        const size_t small = mlr::smallm_ws_bytes(K, N, r);
        if (small > l.total) l.total = small;
    }
    return l;
}
// P = act F for binary16 activations (X A or dY B^T; fp32-exact products on the matrix cores): the
// projection kernel of the bfloat16 path with each activation split into two bfloat16 operands.  No
// extended-contraction operands here: this path adds the adapter term in the product kernel's epilogue.
int f16_project(const uint16_t *act, int32_t M, int32_t C, const float *F, bool f_is_A, int32_t r, float *P, char *ws,
                const F16Ws &l, hipStream_t st) {
    mlr::DownArgs d{};
    d.act = act; d.act_f16 = true; d.M = M; d.C = C; d.r = r;
    d.Fm = F; d.f_is_A = f_is_A;
    d.P = P; d.lora_scale = 1.0f;
    d.act_ext = nullptr; d.RE = 0; d.w_ext = nullptr; d.Wsrc = nullptr; d.w_from_A = false; d.Cw = 0;
    d.partials = reinterpret_cast<float *>(ws + l.dpart);
    return hip_status(mlr::launch_lora_down(d, st));
}

// the codes and scales of the layer as the streaming kernels take them (zero points travel separately)
mlr::LayerView stream_view_of(const modulora_qweight_f16 *w) {
    mlr::LayerView v;
    v.K = w->d_in; v.N = w->d_out; v.bits = w->bits; v.group = w->group_size;
    v.qweight = w->qweight; v.scales = w->scales; v.zeros = nullptr;
    return v;
}
int check_ws_f16(const F16Ws &l, const void *ws, size_t bytes) {
    if (l.total == 0) return MODULORA_OK;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || bytes < l.total) return MODULORA_ERR_WORKSPACE;
    return MODULORA_OK;
}
}  // namespace

size_t modulora_f16_workspace_bytes(const modulora_qweight_f16 *w, int32_t M, int32_t r) {
    if (check_layer_f16(w, false) != MODULORA_OK) return 0;
    if (M < 1 || M > kMaxTokens || r < 0 || r > kMaxRank) return 0;
    return f16_ws(w->d_in, w->d_out, M, r).total;
}

int modulora_f16_dequant(const modulora_qweight_f16 *w, uint16_t *What_f16, void *stream) {
    const int s = check_layer_f16(w, true);
    if (s != MODULORA_OK) return s;
    if (!What_f16) return MODULORA_ERR_NULL;
    if (!aligned16(What_f16)) return MODULORA_ERR_ALIGN;
    return hip_status(mlr::launch_f16_dequant(view_of(w), What_f16, static_cast<hipStream_t>(stream)));
}

int modulora_f16_fwd(const modulora_qweight_f16 *w, const uint16_t *X, int32_t M, const float *A, const float *B,
                     int32_t r, float lora_scale, uint16_t *Y, float *XA, void *workspace, size_t workspace_bytes,
                     void *stream) {
    int s = check_layer_f16(w, true);
    if (s != MODULORA_OK) return s;
    if (!X || !Y) return MODULORA_ERR_NULL;
    if (M < 1 || M > kMaxTokens) return MODULORA_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(Y) || (XA && !aligned16(XA))) return MODULORA_ERR_ALIGN;
    if ((s = check_rank(r, A, B, true)) != MODULORA_OK) return s;
    const F16Ws l = f16_ws(w->d_in, w->d_out, M, r);
    if ((s = check_ws_f16(l, workspace, workspace_bytes)) != MODULORA_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (mlr::smallm_fwd_supported(stream_view_of(w), M)) {
        // a handful of tokens: the direct product with the quantized matrix (Section 3.1.2)
        mlr::SmallArgs sa{};
        sa.w = stream_view_of(w);
        sa.act = X; sa.M = M; sa.out = Y;
        sa.A = A; sa.B = B; sa.r = r; sa.lora_scale = lora_scale;
        sa.P_out = XA; sa.ws = workspace;
        sa.f16 = true; sa.zeros16 = w->zeros; sa.bias16 = w->bias;
        return hip_status(mlr::launch_smallm_fwd(sa, st));
    }
    float *P = nullptr;
    if (r > 0) {
        P = XA ? XA : reinterpret_cast<float *>(static_cast<char *>(workspace) + l.p0);
        if ((s = f16_project(X, M, w->d_in, A, true, r, P, static_cast<char *>(workspace), l, st)) != MODULORA_OK) return s;
    }
    float *parts = l.total > 0 ? reinterpret_cast<float *>(static_cast<char *>(workspace) + l.gemm_part) : nullptr;
    return hip_status(mlr::launch_f16_gemm(view_of(w), false, X, M, Y, P, B, r, lora_scale, parts, st));
}

int modulora_f16_bwd_input(const modulora_qweight_f16 *w, const uint16_t *dY, int32_t M, const float *A, const float *B,
                           int32_t r, float lora_scale, uint16_t *dX, float *dYBt, void *workspace,
                           size_t workspace_bytes, void *stream) {
    int s = check_layer_f16(w, true);
    if (s != MODULORA_OK) return s;
    if (!dY || !dX) return MODULORA_ERR_NULL;
    if (M < 1 || M > kMaxTokens) return MODULORA_ERR_SHAPE;
    if (!aligned16(dY) || !aligned16(dX) || (dYBt && !aligned16(dYBt))) return MODULORA_ERR_ALIGN;
    if ((s = check_rank(r, A, B, true)) != MODULORA_OK) return s;
    const F16Ws l = f16_ws(w->d_in, w->d_out, M, r);
    if ((s = check_ws_f16(l, workspace, workspace_bytes)) != MODULORA_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (mlr::smallm_bwd_supported(stream_view_of(w), M)) {
        mlr::SmallArgs sa{};
        sa.w = stream_view_of(w);
        sa.act = dY; sa.M = M; sa.out = dX;
        sa.A = A; sa.B = B; sa.r = r; sa.lora_scale = lora_scale;
        sa.P_out = dYBt; sa.ws = workspace;
        sa.f16 = true; sa.zeros16 = w->zeros; sa.bias16 = nullptr;
        return hip_status(mlr::launch_smallm_bwd(sa, st));
    }
    float *P = nullptr;
    if (r > 0) {
        P = dYBt ? dYBt : reinterpret_cast<float *>(static_cast<char *>(workspace) + l.p0);
        if ((s = f16_project(dY, M, w->d_out, B, false, r, P, static_cast<char *>(workspace), l, st)) != MODULORA_OK) return s;
    }
    float *parts = l.total > 0 ? reinterpret_cast<float *>(static_cast<char *>(workspace) + l.gemm_part) : nullptr;
    return hip_status(mlr::launch_f16_gemm(view_of(w), true, dY, M, dX, P, A, r, lora_scale, parts, st));
}

int modulora_f16_bwd_lora(int32_t d_in, int32_t d_out, int32_t M, int32_t r, float lora_scale, const uint16_t *X,
                          const uint16_t *dY, const float *A, const float *B, const float *XA, const float *dYBt,
                          float *dA, float *dB, int32_t accumulate, void *workspace, size_t workspace_bytes,
                          void *stream) {
    if (d_in < 32 || d_in > kMaxDim || d_out < 8 || d_out > kMaxDim || d_in % 32 != 0 || d_out % 8 != 0)
        return MODULORA_ERR_SHAPE;
    if (M < 1 || M > kMaxTokens) return MODULORA_ERR_SHAPE;
    if (!X || !dY || !dA || !dB) return MODULORA_ERR_NULL;
    int s = check_rank(r, A, B, false);
    if (s != MODULORA_OK) return s;
    if (!aligned16(X) || !aligned16(dY) || !aligned16(dA) || !aligned16(dB) || (XA && !aligned16(XA)) ||
        (dYBt && !aligned16(dYBt)))
        return MODULORA_ERR_ALIGN;
    const F16Ws l = f16_ws(d_in, d_out, M, r);
    if ((s = check_ws_f16(l, workspace, workspace_bytes)) != MODULORA_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    if (!XA) {
        float *P = reinterpret_cast<float *>(ws + l.p0);
        if ((s = f16_project(X, M, d_in, A, true, r, P, ws, l, st)) != MODULORA_OK) return s;
        XA = P;
    }
    if (!dYBt) {
        float *P = reinterpret_cast<float *>(ws + l.p1);
        if ((s = f16_project(dY, M, d_out, B, false, r, P, ws, l, st)) != MODULORA_OK) return s;
        dYBt = P;
    }
    mlr::GradPairArgs ga{};
    ga.X = X; ga.dY = dY; ga.M = M; ga.K = d_in; ga.N = d_out; ga.r = r;
    ga.XA = XA; ga.dYBt = dYBt; ga.lora_scale = lora_scale;
    ga.dA = dA; ga.dB = dB; ga.accumulate = accumulate ? 1 : 0;
    ga.partials = reinterpret_cast<float *>(ws + l.gpart);
    ga.f16 = 1;
    return hip_status(mlr::launch_lora_grad_pair(ga, st));
}

int modulora_quantize_rtn(const float *W, int32_t d_in, int32_t d_out, int32_t bits, int32_t group_size,
                          uint32_t *qweight, uint16_t *scales, uint8_t *zeros, void *stream) {
    modulora_qweight shape{d_in, d_out, bits, group_size, qweight, scales, zeros};
    const int s = check_layer(&shape);
    if (s != MODULORA_OK) return s;
    if (!W) return MODULORA_ERR_NULL;
    if (!aligned16(W)) return MODULORA_ERR_ALIGN;
    mlr::QuantArgs q{W, d_in, d_out, bits, group_size, qweight, scales, zeros};
    return hip_status(mlr::launch_quantize_rtn(q, static_cast<hipStream_t>(stream)));
}

int modulora_adamw(float *param, const float *grad, float *exp_avg, float *exp_avg_sq, size_t n,
                   float lr, float beta1, float beta2, float eps, float weight_decay, int32_t step,
                   void *stream) {
    if (!param || !grad || !exp_avg || !exp_avg_sq) return MODULORA_ERR_NULL;
    if (!aligned16(param) || !aligned16(grad) || !aligned16(exp_avg) || !aligned16(exp_avg_sq)) return MODULORA_ERR_ALIGN;
    if (n == 0) return MODULORA_ERR_SHAPE;
    const bool finite = std::isfinite(lr) && std::isfinite(beta1) && std::isfinite(beta2) && std::isfinite(eps) &&
                        std::isfinite(weight_decay);
    if (!finite || step < 1 || lr < 0.f || beta1 < 0.f || beta1 >= 1.f || beta2 < 0.f || beta2 >= 1.f || eps <= 0.f ||
        weight_decay < 0.f)
        return MODULORA_ERR_HYPER;
    mlr::AdamWArgs a{};
    a.p = param; a.g = grad; a.m = exp_avg; a.v = exp_avg_sq; a.n = n;
    a.beta1 = beta1; a.beta2 = beta2;
    a.one_minus_beta1 = (float)(1.0 - (double)beta1);
    a.one_minus_beta2 = (float)(1.0 - (double)beta2);
    a.decay = (float)(1.0 - (double)lr * (double)weight_decay);
    a.step_size = (float)((double)lr / (1.0 - std::pow((double)beta1, (double)step)));
    a.inv_sqrt_bc2 = (float)(1.0 / std::sqrt(1.0 - std::pow((double)beta2, (double)step)));
    a.eps = eps;
    return hip_status(mlr::launch_adamw(a, static_cast<hipStream_t>(stream)));
}

int modulora_profile_begin(void) {
    for (auto &rec : g_prof) {
        (void)hipEventDestroy(rec.start);
        (void)hipEventDestroy(rec.stop);
    }
    g_prof.clear();
    g_prof_on = true;
    return MODULORA_OK;
}

int modulora_profile_end(modulora_kernel_time *out, int32_t capacity, int32_t *count) {
    g_prof_on = false;
    if (!count || (capacity > 0 && !out)) return MODULORA_ERR_NULL;
    int32_t n = 0;
    int status = MODULORA_OK;
    for (auto &rec : g_prof) {
        float ms = 0.f;
        if (hipEventSynchronize(rec.stop) != hipSuccess || hipEventElapsedTime(&ms, rec.start, rec.stop) != hipSuccess)
            status = MODULORA_ERR_HIP;
        (void)hipEventDestroy(rec.start);
        (void)hipEventDestroy(rec.stop);
        int32_t slot = -1;
        for (int32_t i = 0; i < n; ++i)
            if (std::strncmp(out[i].name, rec.name, sizeof(out[i].name)) == 0) { slot = i; break; }
        if (slot < 0) {
            if (n >= capacity) continue;
            slot = n++;
            std::memset(&out[slot], 0, sizeof(out[slot]));
            std::strncpy(out[slot].name, rec.name, sizeof(out[slot].name) - 1);
        }
        out[slot].launches += 1;
        out[slot].total_ms += ms;
    }
    g_prof.clear();
    *count = n;
    return status;
}

}  // extern "C"
