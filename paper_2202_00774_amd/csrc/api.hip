// extern "C" boundary of the SDGP library: argument validation and dispatch.
// Every check happens before the first launch, so a failing call has no effect.
#include <atomic>

#include "common.h"

namespace sdgp {
int prune_launch(const void* dO, int64_t total, int dt, int n, int m, int rk, uint64_t seed, void* pruned, void* vals,
                 uint8_t* idx, hipStream_t stream);
int bwd_simple_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                      int64_t C_out, int R, int S, int stride, int pad, int dt, int n, int m, int rk, uint64_t seed,
                      hipStream_t stream);
int bwd_simple_grouped_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                              int64_t C_out, int R, int S, int stride, int pad, int64_t groups, int dt, int n, int m, int rk,
                              uint64_t seed, hipStream_t stream);
size_t bwd_grouped_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad,
                             int64_t groups, int dt, int n, int m);
int bwd_grouped_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R,
                       int S, int stride, int pad, int64_t groups, int dt, int n, int m, int rk, uint64_t seed, void* workspace,
                       hipStream_t stream);
int bwd_narrow_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                      int64_t C_out, int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed,
                      void* workspace, hipStream_t stream);
size_t bwd_narrow_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride,
                            int pad, int n, int m);
int bwd_pw_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                  int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed, void* workspace, size_t workspace_bytes,
                  hipStream_t stream);
int bwd_gather_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                      int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed, void* workspace, size_t workspace_bytes,
                      hipStream_t stream);
size_t bwd_pw_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int n,
                        int m);
int bwd_row_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                   int64_t C_out, int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed,
                   hipStream_t stream);
int bwd_conv3_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                     int64_t C_out, int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed,
                     hipStream_t stream);
int bwd_tiled_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                     int64_t C_out, int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed,
                     hipStream_t stream);
size_t channel_scales_workspace(int64_t rows, int64_t C, int dt, int m);
int channel_scales_launch(const void* dO, int64_t rows, int64_t C, int dt, int n, int m, float* scale, double* sums,
                          void* partial, hipStream_t stream);
int prune_channel_rescaled_launch(const void* dO, int64_t rows, int64_t C, int dt, int n, int m, const float* scale,
                                  void* pruned, hipStream_t stream);
int scale_rows_launch(const void* W, const float* scale, void* out, int64_t C_out, int64_t inner, int dt, hipStream_t stream);
int kprime_launch(const void* vals, const uint8_t* idx, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                  int64_t C_out, int R, int S, int stride, int pad, int n, int m, hipStream_t stream);
int peak_probe_launch(int kind, const void* a, void* b, size_t bytes, int iters, double* work, hipStream_t stream);
int mirror_transpose_filter_launch(const void* W, void* V, int64_t C_out, int64_t C_in, int R, int S, int dt, hipStream_t stream);
int fwd_narrow_launch(const void* D, const void* W, void* O, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                      int R, int S, int stride, int pad, int dt, hipStream_t stream);
int fwd_simple_launch(const void* D, const void* W, void* O, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                      int R, int S, int stride, int pad, int dt, hipStream_t stream);
size_t wgrad_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int dt);
int wgrad_launch(const void* D, const void* dO, float* dW, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                 int R, int S, int stride, int pad, int dt, void* workspace, hipStream_t stream);
}  // namespace sdgp

// Scratch memory of sdgp_conv_bwd_data_noalloc: lives in the library's device image, one copy per GPU, for the life
// of the process.  Host code never uses this name as an address: it asks the runtime where the array sits on the
// current device (scratch_on_current_device) and hands that pointer to the kernels.
static __device__ __align__(256) unsigned char scratch[SDGP_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int64_t kMaxElements = (int64_t)1 << 40;

// Device address of `scratch` on the current device, looked up once per device; null when the runtime refuses.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

void* scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // every thread finds the same address
    }
    return ptr;
}

bool valid_dtype(int dt) { return dt == SDGP_F32 || dt == SDGP_BF16; }
bool valid_ranker(int rk) { return rk == SDGP_RANDOM || rk == SDGP_GREEDY || rk == SDGP_GREEDY_ADJUSTED; }
bool valid_nm(int n, int m) { return n >= 1 && n <= m && m <= 32; }

// a*b with overflow / range check against kMaxElements; false when out of range.
bool mul_checked(int64_t a, int64_t b, int64_t* out) {
    if (a < 0 || b < 0) return false;
    if (a == 0 || b == 0) {
        *out = 0;
        return true;
    }
    if (a > kMaxElements / b) return false;
    *out = a * b;
    return true;
}


struct ConvGeom {
    int64_t P, Q, n_dO, n_W, n_dD;
};

// Full validation of a convolution backward-data problem; SDGP_OK and the derived sizes, or the error.
int check_conv(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad,
               int dt, int n, int m, ConvGeom* g) {
    if (!valid_dtype(dt)) return SDGP_ERR_DTYPE;
    if (!valid_nm(n, m)) return SDGP_ERR_NM;
    if (B < 0 || H < 0 || Wd < 0 || C_in < 0 || C_out < 0) return SDGP_ERR_SHAPE;
    if (R < 1 || R > 11 || S < 1 || S > 11 || stride < 1 || stride > 4 || pad < 0 || pad >= R || pad >= S)
        return SDGP_ERR_SHAPE;
    if ((C_out % m) != 0) return SDGP_ERR_SHAPE;
    if (H > kMaxElements || Wd > kMaxElements) return SDGP_ERR_SHAPE;
    if (H + 2 * pad < R || Wd + 2 * pad < S) return SDGP_ERR_SHAPE;
    g->P = (H + 2 * pad - R) / stride + 1;
    g->Q = (Wd + 2 * pad - S) / stride + 1;
    int64_t t = 0;
    if (!mul_checked(B, g->P, &t) || !mul_checked(t, g->Q, &t) || !mul_checked(t, C_out, &g->n_dO)) return SDGP_ERR_SHAPE;
    if (!mul_checked(C_out, (int64_t)R * S, &t) || !mul_checked(t, C_in, &g->n_W)) return SDGP_ERR_SHAPE;
    if (!mul_checked(B, H, &t) || !mul_checked(t, Wd, &t) || !mul_checked(t, C_in, &g->n_dD)) return SDGP_ERR_SHAPE;
    return SDGP_OK;
}


// Matrix-core kernel when the problem fits it, the shape-agnostic kernel otherwise.
// workspace: what sdgp_conv_bwd_data_workspace asked for, or null (entry points without one); the first-layer kernel
// needs all of its share, the pointwise kernels use theirs when workspace_bytes covers it and run fused otherwise.
int bwd_dispatch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                 int R, int S, int stride, int pad, int dt, int n, int m, int rk, uint64_t seed, void* workspace,
                 size_t workspace_bytes, hipStream_t stream) {
    // no output channels: every element of dD is an empty sum.  The shape-agnostic kernel writes the zeros; the
    // matrix-core kernels assume at least one reduction chunk.
    if (C_out == 0) return sdgp::bwd_simple_launch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, rk, seed, stream);
    if (dt == SDGP_BF16 && C_in <= 4) {
        const int rc = sdgp::bwd_narrow_launch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, rk, seed, workspace,
                                               stream);
        if (rc <= 0) return rc;
    }
    if (dt == SDGP_BF16 && sdgp::is_aligned16(dD)) {
        int rc = sdgp::bwd_pw_launch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, rk, seed, workspace, workspace_bytes, stream);
        if (rc <= 0) return rc;
        rc = sdgp::bwd_row_launch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, rk, seed, stream);
        if (rc <= 0) return rc;
        rc = sdgp::bwd_gather_launch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, rk, seed, workspace, workspace_bytes, stream);
        if (rc <= 0) return rc;
        rc = sdgp::bwd_conv3_launch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, rk, seed, stream);
        if (rc <= 0) return rc;
        rc = sdgp::bwd_tiled_launch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, rk, seed, stream);
        if (rc <= 0) return rc;
    }
    return sdgp::bwd_simple_launch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, rk, seed, stream);
}

// [rows, C] pruned along C in groups of m: the checks sdgp_prune and the per-channel entry points share.
int check_rows(int64_t rows, int64_t C, int dt, int n, int m, int64_t* total) {
    if (!valid_dtype(dt)) return SDGP_ERR_DTYPE;
    if (!valid_nm(n, m)) return SDGP_ERR_NM;
    if (!mul_checked(rows, C, total) || (C % m) != 0) return SDGP_ERR_SHAPE;
    return SDGP_OK;
}

size_t align256(size_t x) { return (x + 255u) & ~(size_t)255u; }

// Workspace of the fused per-channel call: partial sums | factors | rescaled filter.
struct ChannelWorkspace {
    size_t off_scale, off_filter, total;
};

ChannelWorkspace channel_workspace(int64_t rows, int64_t C_out, int64_t n_W, int dt, int m) {
    ChannelWorkspace w;
    w.off_scale = align256(rows > 0 && C_out > 0 ? sdgp::channel_scales_workspace(rows, C_out, dt, m) : 0);
    w.off_filter = w.off_scale + align256((size_t)C_out * sizeof(float));
    w.total = w.off_filter + align256((size_t)n_W * (dt == SDGP_BF16 ? 2u : 4u));
    return w;
}

// the first-layer kernel builds a re-indexed image of a wide filter (the 7x7 stem) once per call
size_t first_layer_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad,
                             int dt, int n, int m, const ConvGeom& g) {
    if (dt == SDGP_BF16 && C_in <= 4 && g.n_dD > 0) return sdgp::bwd_narrow_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m);
    return 0;
}

}  // namespace

extern "C" {

int sdgp_prune(const void* dO, int64_t rows, int64_t C, int dt, int n, int m, int rk, uint64_t seed, void* pruned,
               void* vals, uint8_t* idx, void* hip_stream) {
    if (!valid_dtype(dt)) return SDGP_ERR_DTYPE;
    if (!valid_ranker(rk)) return SDGP_ERR_RANKER;
    if (!valid_nm(n, m)) return SDGP_ERR_NM;
    int64_t total = 0;
    if (!mul_checked(rows, C, &total) || (C % m) != 0) return SDGP_ERR_SHAPE;
    if (total == 0) return SDGP_OK;  // nothing to read or write; pointers of empty tensors may be NULL
    if ((vals == nullptr) != (idx == nullptr)) return SDGP_ERR_NULL;
    if (pruned == nullptr && vals == nullptr) return SDGP_ERR_NULL;
    if (dO == nullptr) return SDGP_ERR_NULL;
    return sdgp::prune_launch(dO, total, dt, n, m, rk, seed, pruned, vals, idx, static_cast<hipStream_t>(hip_stream));
}

int sdgp_conv_bwd_data(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                       int64_t C_out, int R, int S, int stride, int pad, int dt, int n, int m, int rk, uint64_t seed,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
    ConvGeom g;
    const int rc = check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, &g);
    if (rc != SDGP_OK) return rc;
    if (!valid_ranker(rk)) return SDGP_ERR_RANKER;
    if (g.n_dD == 0) return SDGP_OK;
    if (dD == nullptr || (g.n_dO > 0 && dO == nullptr) || (g.n_W > 0 && W == nullptr)) return SDGP_ERR_NULL;
    const size_t need = sdgp_conv_bwd_data_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15u) != 0))
        return SDGP_ERR_WORKSPACE;
    return bwd_dispatch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, rk, seed, need > 0 ? workspace : nullptr,
                        need > 0 ? workspace_bytes : 0, static_cast<hipStream_t>(hip_stream));
}

int sdgp_conv_bwd_data_noalloc(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                               int64_t C_out, int R, int S, int stride, int pad, int dt, int n, int m, int rk,
                               uint64_t seed, void* hip_stream) {
    ConvGeom g;
    const int rc = check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, &g);
    if (rc != SDGP_OK) return rc;
    if (!valid_ranker(rk)) return SDGP_ERR_RANKER;
    if (g.n_dD == 0) return SDGP_OK;
    if (dD == nullptr || (g.n_dO > 0 && dO == nullptr) || (g.n_W > 0 && W == nullptr)) return SDGP_ERR_NULL;
    // what the call cannot do without (a first layer's filter image); a pass that ranks the gradient ahead of the
    // product is only an option, taken when its arrays fit the scratch
    const size_t must = first_layer_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, g);
    if (must > (size_t)SDGP_NOALLOC_SCRATCH_BYTES) return SDGP_ERR_WORKSPACE;  // more scratch than the library holds
    const size_t need = sdgp_conv_bwd_data_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m);
    void* ws = nullptr;
    if (need > 0 && need <= (size_t)SDGP_NOALLOC_SCRATCH_BYTES) {
        ws = scratch_on_current_device();
        if (ws == nullptr) return SDGP_ERR_HIP;
    }
    return bwd_dispatch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, rk, seed, ws,
                        ws != nullptr ? (size_t)SDGP_NOALLOC_SCRATCH_BYTES : 0, static_cast<hipStream_t>(hip_stream));
}

size_t sdgp_conv_bwd_data_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S,
                                    int stride, int pad, int dt, int n, int m) {
    ConvGeom g;
    if (check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, &g) != SDGP_OK) return (size_t)-1;
    const size_t first = first_layer_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, g);
    if (first > 0) return first;
    // 1x1 layers many column tiles wide and strided filters: room for the gradient ranked and compressed once
    if (dt == SDGP_BF16 && C_in > 4 && g.n_dD > 0 && g.n_dO > 0) return sdgp::bwd_pw_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m);
    return 0;
}

// The checks of a grouped problem beyond check_conv's.
static int check_groups(int64_t C_in, int64_t C_out, int64_t groups, int m) {
    if (groups < 1 || (C_in % groups) != 0 || (C_out % groups) != 0) return SDGP_ERR_SHAPE;
    if (groups > 1 && ((C_out / groups) % m) != 0) return SDGP_ERR_SHAPE;   // an m-group would straddle two convolution groups
    return SDGP_OK;
}

size_t sdgp_conv_bwd_data_grouped_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S,
                                            int stride, int pad, int64_t groups, int dt, int n, int m) {
    ConvGeom g;
    if (check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, &g) != SDGP_OK) return (size_t)-1;
    if (check_groups(C_in, C_out, groups, m) != SDGP_OK) return (size_t)-1;
    if (groups == 1) return sdgp_conv_bwd_data_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m);
    if (g.n_dD == 0) return 0;
    // 16 channels per group, 3x3, stride 1: the matrix-core kernel wants the filter re-indexed
    const size_t image = sdgp::bwd_grouped_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, groups, dt, n, m);
    if (image > 0) return image;
    if (n == m) return 0;
    return (size_t)g.n_dO * (dt == SDGP_BF16 ? 2u : 4u);   // the pruned gradient
}

int sdgp_conv_bwd_data_grouped(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                               int64_t C_out, int R, int S, int stride, int pad, int64_t groups, int dt, int n, int m,
                               int rk, uint64_t seed, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (groups == 1)
        return sdgp_conv_bwd_data(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, rk, seed, workspace,
                                  workspace_bytes, hip_stream);
    ConvGeom g;
    int rc = check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, &g);
    if (rc != SDGP_OK) return rc;
    if (!valid_ranker(rk)) return SDGP_ERR_RANKER;
    rc = check_groups(C_in, C_out, groups, m);
    if (rc != SDGP_OK) return rc;
    if (g.n_dD == 0) return SDGP_OK;
    if (dD == nullptr || (g.n_dO > 0 && dO == nullptr) || (g.n_W > 0 && W == nullptr)) return SDGP_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const size_t image = sdgp::bwd_grouped_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, groups, dt, n, m);
    if (image > 0 && workspace != nullptr && workspace_bytes >= image) {
        rc = sdgp::bwd_grouped_launch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, groups, dt, n, m, rk, seed, workspace, stream);
        if (rc <= 0) return rc;   // (a positive value: pointers not aligned for it -- the plain kernel below)
    }
    const void* grad = dO;
    if (n != m && g.n_dO > 0) {
        // Alg. 1 once over the whole gradient, then the dense sum reads the pruned copy
        const size_t need = (size_t)g.n_dO * (dt == SDGP_BF16 ? 2u : 4u);
        if (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15u) != 0)
            return SDGP_ERR_WORKSPACE;
        rc = sdgp::prune_launch(dO, g.n_dO, dt, n, m, rk, seed, workspace, nullptr, nullptr, stream);
        if (rc != SDGP_OK) return rc;
        grad = workspace;
    }
    return sdgp::bwd_simple_grouped_launch(grad, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, groups, dt, m, m, SDGP_GREEDY, 0,
                                           stream);
}

int sdgp_linear_bwd_data(const void* dO, const void* W, void* dD, int64_t rows, int64_t C_out, int64_t C_in, int dt,
                         int n, int m, int rk, uint64_t seed, void* hip_stream) {
    // A linear layer is a 1x1 convolution over rows "pixels".
    ConvGeom g;
    const int rc = check_conv(rows, 1, 1, C_in, C_out, 1, 1, 1, 0, dt, n, m, &g);
    if (rc != SDGP_OK) return rc;
    if (!valid_ranker(rk)) return SDGP_ERR_RANKER;
    if (g.n_dD == 0) return SDGP_OK;
    if (dD == nullptr || (g.n_dO > 0 && dO == nullptr) || (g.n_W > 0 && W == nullptr)) return SDGP_ERR_NULL;
    return bwd_dispatch(dO, W, dD, rows, 1, 1, C_in, C_out, 1, 1, 1, 0, dt, n, m, rk, seed, nullptr, 0,
                        static_cast<hipStream_t>(hip_stream));
}

size_t sdgp_channel_scales_workspace(int64_t rows, int64_t C, int dt, int n, int m) {
    int64_t total = 0;
    if (check_rows(rows, C, dt, n, m, &total) != SDGP_OK) return (size_t)-1;
    return C == 0 ? 0 : sdgp::channel_scales_workspace(rows, C, dt, m);
}

int sdgp_channel_scales(const void* dO, int64_t rows, int64_t C, int dt, int n, int m, float* scale, double* sums,
                        void* workspace, size_t workspace_bytes, void* hip_stream) {
    int64_t total = 0;
    const int rc = check_rows(rows, C, dt, n, m, &total);
    if (rc != SDGP_OK) return rc;
    if (C == 0) return SDGP_OK;  // no channel, no factor
    if (scale == nullptr || (total > 0 && dO == nullptr)) return SDGP_ERR_NULL;
    // a tensor without rows still defines every factor (1: the kept sum is 0); the kernels handle rows == 0
    const size_t need = sdgp::channel_scales_workspace(rows, C, dt, m);
    if (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 7u) != 0)
        return SDGP_ERR_WORKSPACE;
    return sdgp::channel_scales_launch(dO, rows, C, dt, n, m, scale, sums, workspace, static_cast<hipStream_t>(hip_stream));
}

int sdgp_prune_channel_rescaled(const void* dO, int64_t rows, int64_t C, int dt, int n, int m, const float* scale,
                                void* pruned, void* hip_stream) {
    int64_t total = 0;
    const int rc = check_rows(rows, C, dt, n, m, &total);
    if (rc != SDGP_OK) return rc;
    if (total == 0) return SDGP_OK;
    if (dO == nullptr || scale == nullptr || pruned == nullptr) return SDGP_ERR_NULL;
    return sdgp::prune_channel_rescaled_launch(dO, rows, C, dt, n, m, scale, pruned, static_cast<hipStream_t>(hip_stream));
}

int sdgp_scale_filter(const void* W, const float* scale, void* W_scaled, int64_t C_out, int64_t inner, int dt,
                      void* hip_stream) {
    if (!valid_dtype(dt)) return SDGP_ERR_DTYPE;
    int64_t total = 0;
    if (!mul_checked(C_out, inner, &total)) return SDGP_ERR_SHAPE;
    if (total == 0) return SDGP_OK;
    if (W == nullptr || scale == nullptr || W_scaled == nullptr) return SDGP_ERR_NULL;
    return sdgp::scale_rows_launch(W, scale, W_scaled, C_out, inner, dt, static_cast<hipStream_t>(hip_stream));
}

size_t sdgp_conv_bwd_data_channel_rescaled_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R,
                                                     int S, int stride, int pad, int dt, int n, int m) {
    ConvGeom g;
    if (check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, &g) != SDGP_OK) return (size_t)-1;
    if (g.n_dD == 0) return 0;
    return channel_workspace(B * g.P * g.Q, C_out, g.n_W, dt, m).total;
}

int sdgp_conv_bwd_data_channel_rescaled(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd,
                                        int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int dt, int n,
                                        int m, void* workspace, size_t workspace_bytes, void* hip_stream) {
    ConvGeom g;
    int rc = check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, &g);
    if (rc != SDGP_OK) return rc;
    if (g.n_dD == 0) return SDGP_OK;
    if (dD == nullptr || (g.n_dO > 0 && dO == nullptr) || (g.n_W > 0 && W == nullptr)) return SDGP_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (g.n_dO == 0 || g.n_W == 0)  // nothing to rescale: the product of an empty sum, zeros
        return bwd_dispatch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, SDGP_GREEDY, 0, nullptr, 0, stream);
    const int64_t rows = B * g.P * g.Q;
    const ChannelWorkspace w = channel_workspace(rows, C_out, g.n_W, dt, m);
    if (workspace == nullptr || workspace_bytes < w.total || (reinterpret_cast<uintptr_t>(workspace) & 15u) != 0)
        return SDGP_ERR_WORKSPACE;
    char* base = static_cast<char*>(workspace);
    float* scale = reinterpret_cast<float*>(base + w.off_scale);
    void* filter = base + w.off_filter;
    rc = sdgp::channel_scales_launch(dO, rows, C_out, dt, n, m, scale, nullptr, base, stream);
    if (rc != SDGP_OK) return rc;
    rc = sdgp::scale_rows_launch(W, scale, filter, C_out, (int64_t)R * S * C_in, dt, stream);
    if (rc != SDGP_OK) return rc;
    return bwd_dispatch(dO, filter, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, SDGP_GREEDY, 0, nullptr, 0, stream);
}

size_t sdgp_conv_bwd_data_compact_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S,
                                            int stride, int pad, int dt, int n, int m) {
    ConvGeom g;
    if (check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, &g) != SDGP_OK || dt != SDGP_BF16) return (size_t)-1;
    if (g.n_dD == 0) return 0;
    if (C_in % 8 != 0 || (int64_t)m * R * S * (C_in <= 64 ? 128 : C_in <= 128 ? 256 : C_in <= 256 ? 512 : 1024) > 150 * 1024)
        return (size_t)-1;
    const size_t kept = (size_t)(g.n_dO / m * n);
    return align256(kept * 2) + align256(kept);   // values | positions
}

int sdgp_conv_bwd_data_compact(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                               int64_t C_out, int R, int S, int stride, int pad, int dt, int n, int m, int rk, uint64_t seed,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
    ConvGeom g;
    const int rc = check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, &g);
    if (rc != SDGP_OK) return rc;
    if (dt != SDGP_BF16) return SDGP_ERR_DTYPE;
    if (!valid_ranker(rk)) return SDGP_ERR_RANKER;
    if (g.n_dD == 0) return SDGP_OK;
    if (dD == nullptr || (g.n_dO > 0 && dO == nullptr) || (g.n_W > 0 && W == nullptr)) return SDGP_ERR_NULL;
    const size_t need = sdgp_conv_bwd_data_compact_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m);
    if (need == (size_t)-1 || !sdgp::is_aligned16(dD) || !sdgp::is_aligned16(W)) return SDGP_ERR_SHAPE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (g.n_dO == 0 || g.n_W == 0)  // empty sums: zeros, written by the shape-agnostic kernel
        return bwd_dispatch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, rk, seed, nullptr, 0, stream);
    if (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15u) != 0)
        return SDGP_ERR_WORKSPACE;
    const size_t kept = (size_t)(g.n_dO / m * n);
    void* vals = workspace;
    uint8_t* idx = static_cast<uint8_t*>(workspace) + align256(kept * 2);
    const int rcp = sdgp::prune_launch(dO, g.n_dO, dt, n, m, rk, seed, nullptr, vals, idx, stream);
    if (rcp != SDGP_OK) return rcp;
    const int rck = sdgp::kprime_launch(vals, idx, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, stream);
    return rck > 0 ? SDGP_ERR_SHAPE : rck;
}

// The forward sum is a backward-data sum of the mirrored, transposed filter when stride is 1 and the filter square;
// the matrix-core kernels take it when the transposed problem's channel counts suit them (its reduction runs over C_in).
static bool fwd_as_bwd(int64_t C_in, int64_t C_out, int R, int S, int stride) {
    return stride == 1 && R == S && C_out > 4 && C_in > 0 && C_in % 32 == 0;
}

size_t sdgp_conv_fwd_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride,
                               int pad, int dt) {
    ConvGeom g;
    if (check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, 1, 1, &g) != SDGP_OK) return (size_t)-1;
    if (g.n_dO == 0 || !fwd_as_bwd(C_in, C_out, R, S, stride)) return 0;
    return align256((size_t)g.n_W * (dt == SDGP_BF16 ? 2u : 4u));
}

int sdgp_conv_fwd(const void* D, const void* W, void* O, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                  int R, int S, int stride, int pad, int dt, void* workspace, size_t workspace_bytes, void* hip_stream) {
    ConvGeom g;
    const int rc = check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, 1, 1, &g);
    if (rc != SDGP_OK) return rc;
    if (g.n_dO == 0) return SDGP_OK;  // O has no element
    if (O == nullptr || (g.n_dD > 0 && D == nullptr) || (g.n_W > 0 && W == nullptr)) return SDGP_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const size_t need = sdgp_conv_fwd_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt);
    if (need == 0) {
        const int rcn = sdgp::fwd_narrow_launch(D, W, O, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, stream);
        if (rcn <= 0) return rcn;
        return sdgp::fwd_simple_launch(D, W, O, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, stream);
    }
    if (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15u) != 0)
        return SDGP_ERR_WORKSPACE;
    const int rc2 = sdgp::mirror_transpose_filter_launch(W, workspace, C_out, C_in, R, S, dt, stream);
    if (rc2 != SDGP_OK) return rc2;
    // backward-data problem with the channel axes exchanged: "gradient" D [B,H,Wd,C_in], "input" O [B,P,Q,C_out]
    return bwd_dispatch(D, workspace, O, B, g.P, g.Q, C_out, C_in, R, S, 1, R - 1 - pad, dt, 1, 1, SDGP_GREEDY, 0, nullptr, 0, stream);
}

size_t sdgp_conv_bwd_weight_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S,
                                      int stride, int pad, int dt) {
    ConvGeom g;
    if (check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, 1, 1, &g) != SDGP_OK) return (size_t)-1;
    if (g.n_W == 0) return 0;
    return sdgp::wgrad_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt);
}

int sdgp_conv_bwd_weight(const void* D, const void* dO, float* dW, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                         int64_t C_out, int R, int S, int stride, int pad, int dt, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
    ConvGeom g;
    const int rc = check_conv(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, 1, 1, &g);
    if (rc != SDGP_OK) return rc;
    if (g.n_W == 0) return SDGP_OK;
    if (dW == nullptr || (g.n_dD > 0 && D == nullptr) || (g.n_dO > 0 && dO == nullptr)) return SDGP_ERR_NULL;
    const size_t need = sdgp::wgrad_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt);
    const bool aligned = sdgp::is_aligned16(D) && sdgp::is_aligned16(dO);  // unaligned tensors take the plain kernel
    if (need > 0 && aligned &&
        (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15u) != 0))
        return SDGP_ERR_WORKSPACE;
    return sdgp::wgrad_launch(D, dO, dW, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, (need > 0 && aligned) ? workspace : nullptr,
                              static_cast<hipStream_t>(hip_stream));
}

int sdgp_peak_probe(int kind, const void* a, void* b, size_t bytes, int iters, double* work, void* hip_stream) {
    if (!work || !b) return SDGP_ERR_NULL;
    if (kind < 0 || kind > 3) return SDGP_ERR_SHAPE;
    if (kind <= 1) {
        if (!a) return SDGP_ERR_NULL;
        if (((uintptr_t)a | (uintptr_t)b) & 15u) return SDGP_ERR_SHAPE;
    } else if (iters < 1 || iters > (1 << 20)) {
        return SDGP_ERR_SHAPE;
    }
    return sdgp::peak_probe_launch(kind, a, b, bytes, iters, work, static_cast<hipStream_t>(hip_stream));
}

const char* sdgp_status_string(int status) {
    switch (status) {
        case SDGP_OK: return "ok";
        case SDGP_ERR_NULL: return "a required pointer is NULL";
        case SDGP_ERR_NM: return "n and m must satisfy 1 <= n <= m <= 32";
        case SDGP_ERR_SHAPE: return "invalid shape: channels not a multiple of m, negative or overflowing size, or inconsistent geometry";
        case SDGP_ERR_DTYPE: return "unknown dtype";
        case SDGP_ERR_RANKER: return "unknown ranker";
        case SDGP_ERR_WORKSPACE: return "workspace missing or too small";
        case SDGP_ERR_HIP: return "the HIP runtime reported an error";
        default: return "unknown status";
    }
}

int sdgp_version(void) { return 200; }

}  // extern "C"
