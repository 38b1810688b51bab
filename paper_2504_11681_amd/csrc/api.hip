// C ABI of libtfno.so: argument checking, workspace registry, shape dispatch.  See include/tfno.h.
#include "../../include/tfno.h"
#include "common.h"
#include "fused1d.h"
#include "fused2d.h"
#include "pruned1d.h"
#include "staged.h"

#include <atomic>
#include <cstdlib>
#include <mutex>

using namespace tfno;

// Library-owned scratch of tfno_spectral_conv2d_noalloc: every GPU the library runs on holds its own copy of this
// array until the process ends.  In host code the name is a stand-in, not a device address: host code only ever
// uses the per-device address that scratch_address() looks up once per device.
static __device__ __align__(256) unsigned char scratch[TFNO_NOALLOC_SCRATCH_BYTES];

namespace {

struct Workspace { void *ptr; size_t bytes; };
std::atomic<void *> g_ws_ptr{nullptr};
std::atomic<size_t> g_ws_bytes{0};

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up on the first call there; no allocation).
tfno_status scratch_address(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return TFNO_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TFNO_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return TFNO_OK;
}

bool is_pow2(int n) { return n > 0 && (n & (n - 1)) == 0; }

bool overlaps(const void *a, size_t abytes, const void *b, size_t bbytes)
{
    uintptr_t a0 = (uintptr_t)a, a1 = a0 + abytes, b0 = (uintptr_t)b, b1 = b0 + bbytes;
    return a0 < b1 && b0 < a1;
}

// Transformed axes of a call: N1 x N2 points (N2 contiguous) keeping K1 x K2 modes; 1-D calls have N1 = K1 = 1.
struct Shape {
    int dims, N1, N2, K1, K2;
    size_t pts() const { return (size_t)N1 * N2; }
    size_t kpts() const { return (size_t)K1 * K2; }
    bool image_kernels() const { return dims == 2 && fused2d_supported(N1, N2, K1, K2); }
};
Shape shape1d(int N, int K) { return Shape{1, 1, N, 1, K}; }
Shape shape2d(int N1, int N2, int K1, int K2) { return Shape{2, N1, N2, K1, K2}; }

// any_n: the staged pipeline also takes lengths that are not powers of two
bool axis_ok(int N, int K, bool any_n = false) { return N >= 2 && N <= 4096 && (any_n || is_pow2(N)) && K >= 1 && K <= N; }
bool sizes_ok(const Shape &sh, int B, int C_in, int C_out, bool any_n = false)
{
    return B >= 0 && C_in >= 1 && C_out >= 1 && axis_ok(sh.N2, sh.K2, any_n) &&
           (sh.dims == 1 || axis_ok(sh.N1, sh.K1, any_n));
}

// complex64 elements are read and written as 8-byte words, and the real-valued kernels move pairs of floats
bool aligned8(const void *a, const void *b, const void *c)
{
    return (((uintptr_t)a | (uintptr_t)b | (uintptr_t)c) & 7u) == 0;
}

// Everything that can be decided on the host.  *empty is set for a valid call with nothing to do.
tfno_status validate(const Shape &sh, const void *x, const void *W, const void *y, int B, int C_in, int C_out,
                     bool *empty, bool per_mode = false, bool any_n = false)
{
    *empty = false;
    if (!sizes_ok(sh, B, C_in, C_out, any_n)) return TFNO_ERR_SHAPE;
    if (B == 0) { *empty = true; return TFNO_OK; }
    if (!x || !W || !y) return TFNO_ERR_NULL;
    const size_t pts = sh.pts();
    // element counts must stay below 2^40 (byte offsets then fit comfortably in 64 bits) and the
    // launch grids below 2^31 workgroups
    const long double in_elems = (long double)B * C_in * pts, out_elems = (long double)B * C_out * pts;
    if (in_elems >= 1099511627776.0L || out_elems >= 1099511627776.0L) return TFNO_ERR_SHAPE;
    if ((long double)B * (C_in > C_out ? C_in : C_out) * (sh.dims == 2 ? (sh.N1 > sh.N2 ? sh.N1 : sh.N2) : 1) >=
        2147483647.0L)
        return TFNO_ERR_SHAPE;
    const size_t xb = sizeof(c64) * (size_t)B * C_in * pts, yb = sizeof(c64) * (size_t)B * C_out * pts;
    const size_t wb = sizeof(c64) * (size_t)C_in * C_out * (per_mode ? sh.kpts() : 1);
    if (overlaps(y, yb, x, xb) || overlaps(y, yb, W, wb)) return TFNO_ERR_ALIAS;
    if (!aligned8(x, W, y)) return TFNO_ERR_ALIGN;
    return TFNO_OK;
}

// the strip pipeline keeps two [B, C, K1, N2] intermediates
size_t strip2d_workspace_bytes(long long B, int C_in, int C_out, int N2, int K1)
{
    return sizeof(c64) * (size_t)B * K1 * N2 * ((size_t)C_in + C_out);
}

size_t workspace_for(const Shape &sh, int variant, int B, int C_in, int C_out);


// Mode counts between the built kernel sizes: the request runs on the next power of two K' >= K for which a kernel
// exists and the forward side zeroes bins K .. K'-1 before the contraction (exactly the truncation to K).
template <class Pred>
int round_modes(int N, int K, Pred pred)
{
    for (int k = 1; k <= N; k <<= 1)
        if (k >= K && pred(N, k)) return k;
    return 0;
}
bool image_modes(int, int k) { return k == 16 || k == 32 || k == 64; }
bool permode_1d(int N, int K) { return N <= 1024 && pruned1d_supported(N, K); }

// Shape the kernels of `variant` run for the request `req` (its K1, K2 replaced by built sizes); false: no kernel.
bool kernel_shape(const Shape &req, int variant, Shape *ks)
{
    *ks = req;
    if (variant == 1) return true;                          // the staged pipeline takes every K
    if (req.dims == 1) {
        const int k = variant == 6 ? round_modes(req.N2, req.K2, permode_1d)
                    : variant == 2 ? round_modes(req.N2, req.K2, pruned1d_supported)
                    : (variant == 3 || variant == 4) ? round_modes(req.N2, req.K2, fused1d_partial_supported)
                    : round_modes(req.N2, req.K2, fused1d_supported);
        ks->K2 = k;
        return k != 0;
    }
    if (variant == 7) {                                     // the strip pipeline on request: the first axis takes any K1
        const int k = round_modes(req.N2, req.K2, fused1d_supported);
        ks->K2 = k;
        return k != 0;
    }
    if (variant != 0 && variant != 6) return false;
    const int k1 = round_modes(req.N1, req.K1, image_modes), k2 = round_modes(req.N2, req.K2, image_modes);
    if (k1 && k2 && fused2d_supported(req.N1, req.N2, k1, k2)) {
        ks->K1 = k1;
        ks->K2 = k2;
        return true;
    }
    if (variant == 6) return false;                         // per-mode weights: transform kernels on whole images only
    const int k = round_modes(req.N2, req.K2, fused1d_supported);    // strip pipeline: the first axis takes any K1
    ks->K2 = k;
    return k != 0;
}

tfno_status check_workspace(size_t need, const void *x, size_t xb, const void *W, size_t wb, const void *y, size_t yb,
                            void **ws)
{
    void *p = g_ws_ptr.load();
    size_t have = g_ws_bytes.load();
    if (need == 0) { *ws = nullptr; return TFNO_OK; }
    if (!p || have < need) return TFNO_ERR_WORKSPACE;
    if (overlaps(p, need, x, xb) || overlaps(p, need, W, wb) || overlaps(p, need, y, yb)) return TFNO_ERR_ALIAS;
    *ws = p;
    return TFNO_OK;
}

enum Variant { FUSED = 0, STAGED = 1, PRUNED = 2, FFT_GEMM = 3, GEMM_IFFT = 4, STRIPS = 7 };

// own_scratch: the intermediates go to the library's static scratch array instead of the registered workspace
tfno_status run(const Shape &req, Variant variant, const void *x, const void *W, void *y, int B, int C_in, int C_out,
                void *stream, bool own_scratch = false)
{
    const bool staged = variant == STAGED;
    bool empty;
    tfno_status st = validate(req, x, W, y, B, C_in, C_out, &empty, false, staged);
    if (st != TFNO_OK || empty) return st;
    Shape sh;                                               // the kernels' shape: req with K rounded up to a built size
    if (!kernel_shape(req, (int)variant, &sh)) return TFNO_ERR_UNSUPPORTED;
    const int dims = sh.dims, N = sh.N2, K = sh.K2;         // N, K: the last (contiguous) axis
    const int keep1 = req.K1, keep2 = req.K2;               // modes actually kept

    const size_t pts = sh.pts();
    const size_t xb = sizeof(c64) * (size_t)B * C_in * pts, yb = sizeof(c64) * (size_t)B * C_out * pts;
    const size_t wb = sizeof(c64) * (size_t)C_in * C_out;
    void *ws = nullptr;
    if (own_scratch) {
        if (workspace_for(req, (int)variant, B, C_in, C_out) > (size_t)TFNO_NOALLOC_SCRATCH_BYTES) return TFNO_ERR_WORKSPACE;
        st = scratch_address(&ws);
    } else {
        st = check_workspace(workspace_for(req, (int)variant, B, C_in, C_out), x, xb, W, wb, y, yb, &ws);
    }
    if (st != TFNO_OK) return st;

    hipStream_t s = (hipStream_t)stream;
    const c64 *xc = (const c64 *)x, *Wc = (const c64 *)W;
    c64 *yc = (c64 *)y;
    hipError_t e;

    if (staged) {
        e = staged_conv(dims, xc, Wc, yc, B, C_in, C_out, sh.N1, sh.N2, sh.K1, sh.K2, (c64 *)ws, s);
    } else if (variant == PRUNED) {
        e = pruned1d_launch(xc, Wc, yc, B, C_in, C_out, N, K, keep2, (c64 *)ws, s);
    } else if (variant == FFT_GEMM || variant == GEMM_IFFT) {
        // the workspace holds one truncated spectrum: the output's (FFT + CGEMM kernel, then the pruned inverse
        // kernel) or the input's (pruned forward kernel, then the CGEMM + iFFT kernel)
        Fused1dArgs a{};
        a.x = xc; a.W = Wc; a.y = yc; a.C_in = C_in; a.C_out = C_out;
        a.inner_count = 1;
        a.x_outer_stride = (long long)C_in * N;  a.x_inner_stride = 0; a.x_chan_stride = N;
        a.y_outer_stride = (long long)C_out * N; a.y_inner_stride = 0; a.y_chan_stride = N;
        a.scale = 1.0f / (float)N;
        a.K_keep = keep2;
        a.Xh = (const c64 *)ws; a.Yh = (c64 *)ws;
        if (variant == FFT_GEMM) {
            e = fused1d_partial_launch(1, N, K, a, B, s);
            if (e == hipSuccess) e = pruned1d_stages(PRUNED_INV, xc, Wc, yc, nullptr, (c64 *)ws, B, C_in, C_out, N, K, keep2, s);
        } else {
            e = pruned1d_stages(PRUNED_FWD, xc, Wc, yc, (c64 *)ws, nullptr, B, C_in, C_out, N, K, keep2, s);
            if (e == hipSuccess) e = fused1d_partial_launch(2, N, K, a, B, s);
        }
    } else if (dims == 1) {
        Fused1dArgs a{};
        a.x = xc; a.W = Wc; a.y = yc; a.C_in = C_in; a.C_out = C_out;
        a.inner_count = 1;
        a.x_outer_stride = (long long)C_in * N;  a.x_inner_stride = 0; a.x_chan_stride = N;
        a.y_outer_stride = (long long)C_out * N; a.y_inner_stride = 0; a.y_chan_stride = N;
        a.scale = 1.0f / (float)N;
        a.K_keep = keep2;
        e = fused1d_launch(N, K, a, B, s);
    } else if (variant != STRIPS && sh.image_kernels()) {
        // image kernels: only the truncated K1 x K2 spectra cross global memory
        e = fused2d_launch(xc, Wc, yc, B, C_in, C_out, sh.N1, sh.N2, sh.K1, sh.K2, keep1, keep2, (c64 *)ws, s);
    } else {
        // strip pipeline (Sec. 3.2 / 3.3), for shapes the image kernels do not cover: truncated forward transform
        // along the first axis, fused kernel along the last axis on the K1 retained rows, zero-padded inverse along
        // the first axis.
        const int N1 = sh.N1, K1 = sh.K1;
        c64 *T1 = (c64 *)ws;                                   // [B, C_in,  K1, N]
        c64 *T2 = T1 + (size_t)B * C_in * K1 * N;              // [B, C_out, K1, N]
        const long long NN = (long long)N1 * N, KN = (long long)K1 * N;
        e = launch_axis_fft(-1, xc, T1, N1, (long long)B * C_in * N, N, NN, KN, N, N1, K1, 1.f, s);
        if (e == hipSuccess) {
            Fused1dArgs a{};
            a.x = T1; a.W = Wc; a.y = T2; a.C_in = C_in; a.C_out = C_out;
            a.inner_count = K1;
            a.x_outer_stride = (long long)C_in * KN;  a.x_inner_stride = N; a.x_chan_stride = KN;
            a.y_outer_stride = (long long)C_out * KN; a.y_inner_stride = N; a.y_chan_stride = KN;
            a.scale = 1.0f / ((float)N1 * (float)N);
            a.K_keep = keep2;
            e = fused1d_launch(N, K, a, (long long)B * K1, s);
        }
        if (e == hipSuccess)
            e = launch_axis_fft(+1, T2, yc, N1, (long long)B * C_out * N, N, KN, NN, N, K1, N1, 1.f, s);
    }
    return e == hipSuccess ? TFNO_OK : TFNO_ERR_HIP;
}

// W: [C_in, C_out, K] (1-D) or [C_in, C_out, K1, K2] (2-D), an own matrix per retained mode.
tfno_status run_permode(const Shape &req, const void *x, const void *W, void *y, int B, int C_in, int C_out, void *stream)
{
    bool empty;
    tfno_status st = validate(req, x, W, y, B, C_in, C_out, &empty, true);
    if (st != TFNO_OK || empty) return st;
    Shape sh;                                               // the transform kernels' shape
    if (!kernel_shape(req, 6, &sh)) return TFNO_ERR_UNSUPPORTED;
    const size_t pts = sh.pts(), M = sh.kpts();
    const size_t xb = sizeof(c64) * (size_t)B * C_in * pts, yb = sizeof(c64) * (size_t)B * C_out * pts;
    const size_t wb = sizeof(c64) * (size_t)C_in * C_out * req.kpts();
    void *wsp = nullptr;
    st = check_workspace(workspace_for(req, 6, B, C_in, C_out), x, xb, W, wb, y, yb, &wsp);
    if (st != TFNO_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const c64 *xc = (const c64 *)x, *Wc = (const c64 *)W;
    c64 *yc = (c64 *)y, *Xh = (c64 *)wsp;
    const float scale = 1.0f / ((float)sh.N1 * (float)sh.N2);
    hipError_t e;
    if (sh.dims == 1) {
        const int N = sh.N2, K = sh.K2;
        c64 *Yh = Xh + pruned1d_spectrum_elems(B, C_in, K);
        const long long tiles = ((long long)B * K + 127) / 128;
        e = pruned1d_stages(PRUNED_FWD, xc, nullptr, yc, Xh, Yh, B, C_in, C_out, N, K, req.K2, s);
        if (e == hipSuccess)
            e = cgemm_permode_launch(Xh, Wc, Yh, C_in, C_out, K, tiles, K >= 128 ? K / 128 : 1, scale, K, 1, req.K2, s);
        if (e == hipSuccess) e = pruned1d_stages(PRUNED_INV, xc, nullptr, yc, Xh, Yh, B, C_in, C_out, N, K, K, s);
    } else {
        c64 *Yh = Xh + (size_t)B * C_in * M;
        e = fused2d_images(-1, xc, Xh, (long long)B * C_in, C_in, sh.N1, sh.N2, sh.K1, sh.K2, req.K1, req.K2, false, 0, s);
        if (e == hipSuccess)
            e = cgemm_permode_launch(Xh, Wc, Yh, C_in, C_out, (int)M, (long long)B * (long long)(M / 128), (int)(M / 128), scale,
                                     sh.K2, req.K1, req.K2, s);
        if (e == hipSuccess)
            e = fused2d_images(+1, Yh, yc, (long long)B * C_out, C_out, sh.N1, sh.N2, sh.K1, sh.K2, sh.K1, sh.K2, false, 0, s);
    }
    return e == hipSuccess ? TFNO_OK : TFNO_ERR_HIP;
}

// Real-valued 1-D layer: x [B, C_in, N] and y [B, C_out, N] float32, W [C_in, C_out] c64, K <= N / 2.
tfno_status run_real1d(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N, int K, void *stream)
{
    if (B < 0 || C_in < 1 || C_out < 1 || !axis_ok(N, K) || 2 * K > N) return TFNO_ERR_SHAPE;
    if (B == 0) return TFNO_OK;
    if (!x || !W || !y) return TFNO_ERR_NULL;
    if ((long double)B * C_in * N >= 1099511627776.0L || (long double)B * C_out * N >= 1099511627776.0L ||
        (long double)B * (C_in > C_out ? C_in : C_out) >= 2147483647.0L)
        return TFNO_ERR_SHAPE;
    const size_t xb = sizeof(float) * (size_t)B * C_in * N, yb = sizeof(float) * (size_t)B * C_out * N;
    const size_t wb = sizeof(c64) * (size_t)C_in * C_out;
    if (overlaps(y, yb, x, xb) || overlaps(y, yb, W, wb)) return TFNO_ERR_ALIAS;
    if (!aligned8(x, W, y)) return TFNO_ERR_ALIGN;
    const int Kk = round_modes(N, K, fused1d_real_supported);       // the kernel's K; bins K .. Kk-1 are zeroed
    if (!Kk) return TFNO_ERR_UNSUPPORTED;
    Fused1dArgs a{};
    a.x = (const c64 *)x; a.W = (const c64 *)W; a.y = (c64 *)y; a.C_in = C_in; a.C_out = C_out;   // x, y: float tensors
    a.K_keep = K;
    a.inner_count = 1;
    a.x_outer_stride = (long long)C_in * N;  a.x_inner_stride = 0; a.x_chan_stride = N;            // in floats
    a.y_outer_stride = (long long)C_out * N; a.y_inner_stride = 0; a.y_chan_stride = N;
    a.scale = 2.0f / (float)N;
    return fused1d_real_launch(N, Kk, a, B, (hipStream_t)stream) == hipSuccess ? TFNO_OK : TFNO_ERR_HIP;
}

// The 2-D Fourier layer of FNO models on real fields: x [B, C_in, N1, N2] and y [B, C_out, N1, N2] float32,
// W [C_in, C_out, 2 M1, M2] c64 (first-axis frequencies -M1 .. M1-1 at index k1 + M1, last-axis 0 .. M2-1).
tfno_status run_fno2d(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N1, int N2, int M1, int M2,
                      void *stream, size_t *ws_bytes)
{
    if (ws_bytes) *ws_bytes = 0;
    if (B < 0 || C_in < 1 || C_out < 1 || !axis_ok(N1, 1) || !axis_ok(N2, 1) || M1 < 1 || M2 < 1 || 2 * M1 > N1 ||
        2 * M2 > N2)
        return TFNO_ERR_SHAPE;
    // the transform kernels' block of modes: the next built sizes
    const int K1 = round_modes(N1, 2 * M1, image_modes), K2 = round_modes(N2, M2, image_modes);
    const bool have = K1 && K2 && fused2d_supported(N1, N2, K1, K2);
    if (ws_bytes) {                                         // size query only
        if (have && B > 0) *ws_bytes = fused2d_workspace_bytes(B, C_in, C_out, K1, K2);
        return have ? TFNO_OK : TFNO_ERR_UNSUPPORTED;
    }
    if (B == 0) return TFNO_OK;
    if (!x || !W || !y) return TFNO_ERR_NULL;
    const size_t pts = (size_t)N1 * N2;
    if ((long double)B * C_in * pts >= 1099511627776.0L || (long double)B * C_out * pts >= 1099511627776.0L ||
        (long double)B * (C_in > C_out ? C_in : C_out) >= 2147483647.0L)
        return TFNO_ERR_SHAPE;
    const size_t xb = sizeof(float) * (size_t)B * C_in * pts, yb = sizeof(float) * (size_t)B * C_out * pts;
    const size_t wb = sizeof(c64) * (size_t)C_in * C_out * 2 * M1 * M2;
    if (overlaps(y, yb, x, xb) || overlaps(y, yb, W, wb)) return TFNO_ERR_ALIAS;
    if (!aligned8(x, W, y)) return TFNO_ERR_ALIGN;
    if (!have) return TFNO_ERR_UNSUPPORTED;
    void *wsp = nullptr;
    tfno_status st = check_workspace(fused2d_workspace_bytes(B, C_in, C_out, K1, K2), x, xb, W, wb, y, yb, &wsp);
    if (st != TFNO_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const size_t M = (size_t)K1 * K2;
    c64 *Xh = (c64 *)wsp, *Yh = Xh + (size_t)B * C_in * M;
    const float scale = 2.0f / ((float)N1 * (float)N2);     // C2R along the last axis: twice the real part
    hipError_t e = fused2d_images(-1, (const c64 *)x, Xh, (long long)B * C_in, C_in, N1, N2, K1, K2, 2 * M1, M2, true, M1, s);
    if (e == hipSuccess)
        e = cgemm_permode_launch(Xh, (const c64 *)W, Yh, C_in, C_out, (int)M, (long long)B * (long long)(M / 128),
                                 (int)(M / 128), scale, K2, 2 * M1, M2, s);
    if (e == hipSuccess)
        e = fused2d_images(+1, Yh, (c64 *)y, (long long)B * C_out, C_out, N1, N2, K1, K2, K1, K2, true, M1, s);
    return e == hipSuccess ? TFNO_OK : TFNO_ERR_HIP;
}

// The 1-D Fourier layer of FNO models on real fields: x [B, C_in, N], y [B, C_out, N] float32, W [C_in, C_out, M] c64.
tfno_status run_fno1d(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N, int M, void *stream,
                      size_t *ws_bytes)
{
    if (ws_bytes) *ws_bytes = 0;
    if (B < 0 || C_in < 1 || C_out < 1 || !axis_ok(N, M) || 2 * M > N) return TFNO_ERR_SHAPE;
    const int K = round_modes(N, M, permode_1d);            // the transform kernels' K
    if (ws_bytes) {                                         // size query only
        if (K && B > 0) *ws_bytes = pruned1d_workspace_bytes(B, C_in, C_out, K);
        return K ? TFNO_OK : TFNO_ERR_UNSUPPORTED;
    }
    if (B == 0) return TFNO_OK;
    if (!x || !W || !y) return TFNO_ERR_NULL;
    if ((long double)B * C_in * N >= 1099511627776.0L || (long double)B * C_out * N >= 1099511627776.0L ||
        (long double)B * (C_in > C_out ? C_in : C_out) >= 2147483647.0L)
        return TFNO_ERR_SHAPE;
    const size_t xb = sizeof(float) * (size_t)B * C_in * N, yb = sizeof(float) * (size_t)B * C_out * N;
    const size_t wb = sizeof(c64) * (size_t)C_in * C_out * M;
    if (overlaps(y, yb, x, xb) || overlaps(y, yb, W, wb)) return TFNO_ERR_ALIAS;
    if (!aligned8(x, W, y)) return TFNO_ERR_ALIGN;
    if (!K) return TFNO_ERR_UNSUPPORTED;
    void *wsp = nullptr;
    tfno_status st = check_workspace(pruned1d_workspace_bytes(B, C_in, C_out, K), x, xb, W, wb, y, yb, &wsp);
    if (st != TFNO_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    c64 *Xh = (c64 *)wsp, *Yh = Xh + pruned1d_spectrum_elems(B, C_in, K);
    const long long tiles = ((long long)B * K + 127) / 128;
    hipError_t e = pruned1d_real_stages(PRUNED_FWD, (const float *)x, (float *)y, Xh, Yh, B, C_in, C_out, N, K, M, s);
    if (e == hipSuccess)
        e = cgemm_permode_launch(Xh, (const c64 *)W, Yh, C_in, C_out, K, tiles, K >= 128 ? K / 128 : 1, 2.0f / (float)N, K,
                                 1, M, s);
    if (e == hipSuccess)
        e = pruned1d_real_stages(PRUNED_INV, (const float *)x, (float *)y, Xh, Yh, B, C_in, C_out, N, K, K, s);
    return e == hipSuccess ? TFNO_OK : TFNO_ERR_HIP;
}

// Variant E of the paper (Sec. 5): per-shape choice among the variants.  Measured on MI355X over the hidden-dimension
// sweep (B = 512, N = 256): the fully fused kernel is fastest whenever one workgroup covers all output channels of a
// batch row (up to 256 at N = 256, up to 128 elsewhere); above that every slab repeats the forward transform of its
// batch row, and the CGEMM + iFFT variant, which transforms once and re-reads only the truncated spectrum, wins.
Variant choose_variant(int N, int K, int C_out)
{
    // (N = 256 has fused kernels that cover 256 outputs per workgroup and beat the CGEMM + iFFT variant there; at
    // N = 128 the fused kernel wins from K = 64 on -- C 256: 258 against 296 us, K = 128: 447 against 495 us -- and
    // loses by 3 % at K = 32)
    if (C_out > 128 && N == 128 && round_modes(N, K, fused1d_partial_supported) == 32) return GEMM_IFFT;
    if (round_modes(N, K, fused1d_supported)) return FUSED;
    // long pencils (N = 2048, 4096) have no fused kernel: one workgroup cannot hold the K >= 128 retained modes of
    // all its output channels; the three pruned kernels move only 4 K / N of the tensor bytes extra
    if (round_modes(N, K, pruned1d_supported)) return PRUNED;
    return STAGED;
}

}  // namespace

namespace tfno {

bool fused1d_supported(int N, int K)
{
    if (!is_pow2(K)) return false;
    switch (N) {
    case 64: return K >= 8 && K <= 64;
    case 128: return K >= 16 && K <= 128;
    case 256: return K >= 16 && K <= 256;
    case 512: return K >= 32 && K <= 256;
    case 1024: return K >= 32 && K <= 256;
    default: return false;
    }
}

bool fused1d_real_supported(int N, int K)
{
    if (!is_pow2(K) || 2 * K > N) return false;
    switch (N) {
    case 64: return K >= 8;
    case 128: case 256: return K >= 16;
    case 512: case 1024: return K >= 32 && K <= 256;
    default: return false;
    }
}

static int kernel_choice();

hipError_t fused1d_real_launch(int N, int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    if (!fused1d_real_supported(N, K)) return hipErrorInvalidValue;
    // N = 1024: the symmetric-wave kernel where it exists and no bins are masked (it has no mode mask)
    // (fewer than half a chip of workgroups: the four-wave kernel's narrower slabs, unless TFNO_KERNEL=sym)
    const bool sym_fills = (kernel_choice() == 0 && rows * ((a.C_out + 127) / 128) >= 128 && a.C_out > 64) || kernel_choice() == 3;
    if (fused1d_sym_supported(N, K) && a.K_keep == K && sym_fills && !contraction_forced_f32())
        return fused1d_sym_real_launch(N, K, a, rows, s);
    switch (N) {
    case 64: return fused1d_real_launch_n64(K, a, rows, s);
    case 128: return fused1d_real_launch_n128(K, a, rows, s);
    case 256: return fused1d_real_launch_n256(K, a, rows, s);
    case 512: return fused1d_real_launch_n512(K, a, rows, s);
    default: return fused1d_real_launch_n1024(K, a, rows, s);
    }
}

bool fused1d_partial_supported(int N, int K)
{
    return (N == 128 || N == 256) && (K == 32 || K == 64 || K == 128) && pruned1d_supported(N, K);
}

hipError_t fused1d_partial_launch(int mode, int N, int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    if (!fused1d_partial_supported(N, K) || (mode != 1 && mode != 2)) return hipErrorInvalidValue;
    if (N == 128) return mode == 1 ? fused1d_fftgemm_launch_n128(K, a, rows, s) : fused1d_gemmifft_launch_n128(K, a, rows, s);
    return mode == 1 ? fused1d_fftgemm_launch_n256(K, a, rows, s) : fused1d_gemmifft_launch_n256(K, a, rows, s);
}

// TFNO_CONTRACTION=f32 forces the kernels whose channel contraction uses FP32 MFMA; the default lets
// shapes that have a wave-specialised kernel use the exact-split BF16x3 contraction.
bool contraction_forced_f32()
{
    static const bool forced = [] {
        const char *e = getenv("TFNO_CONTRACTION");
        return e && e[0] == 'f' && e[1] == '3' && e[2] == '2' && e[3] == 0;
    }();
    return forced;
}

// TFNO_KERNEL (read once): 0 default, 1 "ws", 2 "generic", 3 "sym"
static int kernel_choice()
{
    static const int which = [] {
        const char *e = getenv("TFNO_KERNEL");
        if (e && e[0] == 'w' && e[1] == 's' && e[2] == 0) return 1;
        if (e && e[0] == 'g' && e[1] == 'e' && e[2] == 'n') return 2;
        if (e && e[0] == 's' && e[1] == 'y' && e[2] == 'm' && e[3] == 0) return 3;
        return 0;
    }();
    return which;
}

bool generic_kernels_forced() { return kernel_choice() == 2; }

hipError_t fused1d_launch(int N, int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    if (!fused1d_supported(N, K)) return hipErrorInvalidValue;
    if (!contraction_forced_f32()) {
        // N = 1024 has three kernels.  Default: the symmetric-wave kernel where it exists (K in {64, 128}; the
        // fastest at the sustained clock), else the wave-specialised one.  TFNO_KERNEL=ws forces the
        // wave-specialised kernel, TFNO_KERNEL=generic the four-wave kernel.
        const int which = kernel_choice();
        // (they have no mode mask: a request for fewer modes than the kernel's K runs on the four-wave kernel)
        const bool exact = a.K_keep == 0 || a.K_keep == K;
        // (and one workgroup per batch row and 128 outputs: below half a chip of such workgroups the four-wave kernel
        // with its narrower output slabs puts the idle CUs to work -- B = 64, C = 128: 70 against 83 us; B = 64, C = 64:
        // 41 against 62 us; from B = 128 on the symmetric kernel is level or ahead)
        // TFNO_KERNEL=sym keeps the symmetric kernel for every batch size.
        // (and more than 64 outputs: both kernels contract and invert whole 128-output slabs, so for narrower layers
        // the four-wave kernel with a 32- or 64-output slab is ahead -- B = 1024, C = 32: 127 against 180 us at
        // K = 128, 121 against 163 us at K = 64; B = 512, C = 64: 126 against 138 us and 124 against 130 us)
        const bool fills = rows * ((a.C_out + 127) / 128) >= 128 && a.C_out > 64;
        if (exact && ((which == 0 && fills) || which == 3) && fused1d_sym_supported(N, K)) return fused1d_sym_launch(N, K, a, rows, s);
        if (exact && (which == 1 || (which == 0 && fills)) && fused1d_ws_supported(N, K)) return fused1d_ws_launch(N, K, a, rows, s);
    }
    switch (N) {
    case 64: return fused1d_launch_n64(K, a, rows, s);
    case 128: return fused1d_launch_n128(K, a, rows, s);
    case 256: return fused1d_launch_n256(K, a, rows, s);
    case 512: return fused1d_launch_n512(K, a, rows, s);
    case 1024: return fused1d_launch_n1024(K, a, rows, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno

namespace {

size_t workspace_for(const Shape &req, int variant, int B, int C_in, int C_out)
{
    if (variant == 5) {
        if (req.dims != 1) return 0;
        variant = (int)choose_variant(req.N2, req.K2, C_out);
    }
    if (B < 1 || !sizes_ok(req, B, C_in, C_out, variant == 1)) return 0;
    if (variant < 0 || variant > 7 || variant == 5 || (variant >= 2 && variant <= 4 && req.dims != 1)) return 0;
    if (variant == 7 && req.dims != 2) return 0;
    Shape sh;                                               // the kernels' shape (K rounded up to a built size)
    if (!kernel_shape(req, variant, &sh)) return 0;
    if (variant == 6)       // per-mode weights: the truncated spectra of input and output
        return sh.dims == 1 ? pruned1d_workspace_bytes(B, C_in, C_out, sh.K2)
                            : fused2d_workspace_bytes(B, C_in, C_out, sh.K1, sh.K2);
    if (variant == 2) return pruned1d_workspace_bytes(B, C_in, C_out, sh.K2);
    if (variant == 3 || variant == 4) return sizeof(c64) * pruned1d_spectrum_elems(B, variant == 3 ? C_out : C_in, sh.K2);
    if (variant == 1) return staged_workspace_bytes(B, C_in, C_out, req.N1, req.N2, req.K1, req.K2);
    if (sh.dims == 1) return 0;
    return variant != 7 && sh.image_kernels() ? fused2d_workspace_bytes(B, C_in, C_out, sh.K1, sh.K2)
                                              : strip2d_workspace_bytes(B, C_in, C_out, sh.N2, sh.K1);
}

}  // namespace

extern "C" {

tfno_status tfno_spectral_conv1d(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N, int K,
                                 void *stream)
{
    return run(shape1d(N, K), FUSED, x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv2d(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N, int K,
                                 void *stream)
{
    return run(shape2d(N, N, K, K), FUSED, x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv2d_noalloc(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N, int K,
                                         void *stream)
{
    return run(shape2d(N, N, K, K), FUSED, x, W, y, B, C_in, C_out, stream, true);
}

tfno_status tfno_spectral_conv1d_pruned(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N,
                                        int K, void *stream)
{
    return run(shape1d(N, K), PRUNED, x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv1d_fft_gemm(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N,
                                          int K, void *stream)
{
    return run(shape1d(N, K), FFT_GEMM, x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv1d_gemm_ifft(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N,
                                           int K, void *stream)
{
    return run(shape1d(N, K), GEMM_IFFT, x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv1d_auto(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N, int K,
                                      void *stream)
{
    return run(shape1d(N, K), choose_variant(N, K, C_out), x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv1d_staged(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N,
                                        int K, void *stream)
{
    return run(shape1d(N, K), STAGED, x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv2d_staged(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N,
                                        int K, void *stream)
{
    return run(shape2d(N, N, K, K), STAGED, x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv2d_rect(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N1,
                                      int N2, int K1, int K2, void *stream)
{
    return run(shape2d(N1, N2, K1, K2), FUSED, x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv2d_strips(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N1,
                                        int N2, int K1, int K2, void *stream)
{
    return run(shape2d(N1, N2, K1, K2), STRIPS, x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv2d_rect_staged(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N1,
                                             int N2, int K1, int K2, void *stream)
{
    return run(shape2d(N1, N2, K1, K2), STAGED, x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv1d_real(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N, int K,
                                      void *stream)
{
    return run_real1d(x, W, y, B, C_in, C_out, N, K, stream);
}

tfno_status tfno_fno1d_real(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N, int M, void *stream)
{
    return run_fno1d(x, W, y, B, C_in, C_out, N, M, stream, nullptr);
}

size_t tfno_fno1d_real_workspace_bytes(int B, int C_in, int C_out, int N, int M)
{
    size_t bytes = 0;
    run_fno1d(nullptr, nullptr, nullptr, B, C_in, C_out, N, M, nullptr, &bytes);
    return bytes;
}

tfno_status tfno_fno2d_real(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N1, int N2, int M1,
                            int M2, void *stream)
{
    return run_fno2d(x, W, y, B, C_in, C_out, N1, N2, M1, M2, stream, nullptr);
}

size_t tfno_fno2d_real_workspace_bytes(int B, int C_in, int C_out, int N1, int N2, int M1, int M2)
{
    size_t bytes = 0;
    run_fno2d(nullptr, nullptr, nullptr, B, C_in, C_out, N1, N2, M1, M2, nullptr, &bytes);
    return bytes;
}

tfno_status tfno_spectral_conv1d_permode(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N,
                                         int K, void *stream)
{
    return run_permode(shape1d(N, K), x, W, y, B, C_in, C_out, stream);
}

tfno_status tfno_spectral_conv2d_permode(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N1,
                                         int N2, int K1, int K2, void *stream)
{
    return run_permode(shape2d(N1, N2, K1, K2), x, W, y, B, C_in, C_out, stream);
}

size_t tfno_workspace_bytes(int dims, int variant, int B, int C_in, int C_out, int N, int K)
{
    if (dims != 1 && dims != 2) return 0;
    return workspace_for(dims == 1 ? shape1d(N, K) : shape2d(N, N, K, K), variant, B, C_in, C_out);
}

size_t tfno_workspace_bytes_2d(int variant, int B, int C_in, int C_out, int N1, int N2, int K1, int K2)
{
    return workspace_for(shape2d(N1, N2, K1, K2), variant, B, C_in, C_out);
}

tfno_status tfno_set_workspace(void *dev_ptr, size_t bytes)
{
    if (!dev_ptr && bytes != 0) return TFNO_ERR_NULL;
    if (dev_ptr && bytes == 0) return TFNO_ERR_SHAPE;
    if (((uintptr_t)dev_ptr & 255u) != 0) return TFNO_ERR_SHAPE;
    g_ws_bytes.store(0);
    g_ws_ptr.store(dev_ptr);
    g_ws_bytes.store(bytes);
    return TFNO_OK;
}

const char *tfno_status_string(tfno_status s)
{
    switch (s) {
    case TFNO_OK: return "ok";
    case TFNO_ERR_NULL: return "a required pointer is NULL";
    case TFNO_ERR_SHAPE: return "a size argument is out of range";
    case TFNO_ERR_UNSUPPORTED: return "no fused kernel for this shape (use the staged entry point)";
    case TFNO_ERR_ALIAS: return "y or the workspace overlaps another buffer";
    case TFNO_ERR_WORKSPACE: return "workspace missing or too small (see tfno_workspace_bytes), or the shape needs more than the built-in scratch";
    case TFNO_ERR_HIP: return "the HIP runtime reported an error at launch";
    case TFNO_ERR_ALIGN: return "x, W or y is not aligned to 8 bytes";
    default: return "unknown status";
    }
}

int tfno_version(void) { return 100; }

}  // extern "C"
