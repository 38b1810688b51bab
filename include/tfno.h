/*
 * tfno.h -- C ABI of the MI355X (gfx950) spectral-convolution library.
 *
 * The operator is the Fourier layer of a Fourier Neural Operator as TurboFNO
 * (arxiv 2504.11681) defines it: forward FFT along the spatial axis or axes,
 * truncation to the first K frequency bins of every transformed axis, a complex
 * linear layer over the hidden (channel) dimension that uses ONE weight matrix
 * for all retained modes, zero padding back to N bins, inverse FFT
 * (Sec. 2.1 and Fig. 1 for the pipeline and the tensor shapes; Sec. 3.1 for the
 * GEMM shape M = batch x modes, N = OutputDim, K = HiddenDim; Sec. 3.3 for
 * which bins are kept and how padding mirrors truncation).
 *
 * Conventions common to every entry point
 * ---------------------------------------
 *  - All data pointers are DEVICE pointers to contiguous row-major tensors of
 *    interleaved complex64 (float re, float im; 8 bytes per element).
 *      x : [B, C_in,  N]      (1-D)   or   [B, C_in,  N, N]   (2-D)   read only
 *      W : [C_in, C_out]                                              read only
 *      y : [B, C_out, N]      (1-D)   or   [B, C_out, N, N]   (2-D)   written
 *  - Forward transform uses exp(-2 pi i k n / N) and is unscaled; the inverse
 *    uses exp(+2 pi i k n / N) and is scaled by 1/N per transformed axis.  No
 *    conjugation of W.  Retained bins are k = 0..K-1 on each transformed axis
 *    (the low corner [0,K)x[0,K) in 2-D).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls are asynchronous: they enqueue kernels and return; they never
 *    synchronise and never allocate device memory.
 *  - Ownership: the caller owns every buffer (including the workspace) and must
 *    keep it alive and unmodified until the stream has passed the call.
 *  - y must not overlap x or W (checked on address ranges: TFNO_ERR_ALIAS).
 *  - x, W and y must be aligned to 8 bytes (TFNO_ERR_ALIGN), the float32 tensors of the real-valued entry points
 *    included: complex64 elements move as 8-byte words and the real-valued kernels move pairs of floats.
 *  - Argument errors are detected on the host before anything is launched, so a
 *    failed call has no effect on y.  B == 0 is a valid empty call (TFNO_OK,
 *    nothing launched, pointers may be NULL).
 *  - N must be a power of two, 2 <= N <= 4096; 1 <= K <= N; C_in, C_out >= 1.  The staged entry points (and
 *    tfno_spectral_conv1d_auto, which falls back to them) also take any other 2 <= N <= 4096.
 *  - Mode counts: the kernels are built for the power-of-two K that each entry point lists.  Every other K, down
 *    to 1, runs on the next built size K' >= K: the forward transform zeroes bins K .. K'-1 before the contraction,
 *    which is exactly the truncation to K (Sec. 3.3), so e.g. K = 12, 20 or 48 are served by the fused kernels; a
 *    call is TFNO_ERR_UNSUPPORTED only when no built size >= K exists for its N.  Workspace sizes follow K'.
 *  - Thread safety: entry points may be called concurrently from several host
 *    threads; tfno_set_workspace must not race with calls that use the workspace.
 *  - The workspace is ONE buffer per process (not per stream, not per device): every entry point that needs
 *    intermediates uses the buffer registered last, on whatever stream it is given.  Calls that use it must
 *    therefore be ordered against each other by the caller, and a buffer may be replaced or freed only after
 *    every stream has passed the calls that used it (a captured HIP graph keeps the address it was captured with).
 *  - Two environment variables, read once per process, select alternative kernels for A/B measurements and tests:
 *    TFNO_CONTRACTION=f32 (FP32-MFMA contractions instead of the exact-split BF16 ones) and, for N = 1024,
 *    TFNO_KERNEL=ws | generic | sym (the wave-specialised, the four-wave or the symmetric-wave kernel whatever the
 *    batch size, instead of the per-shape default).  Results stay within the same tolerance; production callers
 *    leave both unset.
 */
#ifndef TFNO_H
#define TFNO_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TFNO_OK = 0,
    TFNO_ERR_NULL = 1,        /* a required pointer is NULL                               */
    TFNO_ERR_SHAPE = 2,       /* a size is out of range (non power-of-two N, K > N, ...)  */
    TFNO_ERR_UNSUPPORTED = 3, /* valid shape, but this entry point has no kernel for it   */
    TFNO_ERR_ALIAS = 4,       /* y overlaps x or W                                        */
    TFNO_ERR_WORKSPACE = 5,   /* workspace missing or smaller than tfno_workspace_bytes() */
    TFNO_ERR_HIP = 6,         /* the HIP runtime reported a launch error                  */
    TFNO_ERR_ALIGN = 7        /* x, W or y is not aligned to 8 bytes                      */
} tfno_status;

/*
 * Fused 1-D spectral convolution (the fully fused FFT-CGEMM-iFFT kernel, Sec. 4.3,
 * with the built-in truncation, zero padding and butterfly pruning of Sec. 3.3):
 *
 *   y[b,o,:] = iFFT_N( pad_N( sum_c trunc_K( FFT_N(x[b,c,:]) ) * W[c,o] ) )
 *
 * One kernel launch; the spectra never leave the chip.  Needs no workspace.  Which instantiation runs (workgroups of
 * four or eight waves, 128 or 256 outputs per workgroup, one or two operand tiles) is chosen from the shape and does
 * not change the result beyond the order of floating-point accumulation.
 * Built sizes of the fused kernel: K a power of two, 8..64 for N = 64, 16..128 for N = 128, 16..256 for N = 256,
 * 32..256 for N = 512 and N = 1024 (K = N allowed where listed); every smaller K runs on the next built size (see
 * "Mode counts" above).  Other valid shapes: TFNO_ERR_UNSUPPORTED (use the staged entry point or
 * tfno_spectral_conv1d_auto).
 */
tfno_status tfno_spectral_conv1d(const void *x, const void *W, void *y,
                                 int B, int C_in, int C_out, int N, int K, void *stream);

/*
 * Fused 2-D spectral convolution (Sec. 3.2 / 3.3: separable transform, truncation and zero padding built
 * into both axes, pruned butterflies):
 *
 *   y[b,o] = iFFT2( pad_NxN( sum_c trunc_KxK( FFT2(x[b,c]) ) * W[c,o] ) )
 *
 * N in {64,128,256}, K <= 64 (built sizes 16, 32, 64): three launches -- a per-image truncated forward transform, the
 * CGEMM over the K*K retained modes, a per-image zero-padded inverse -- whose only intermediates are the
 * truncated spectra (tfno_workspace_bytes(2, 0, ...) = 8 B K^2 (C_in + C_out) bytes of workspace).
 * Other shapes that the 1-D fused kernel supports run the paper's 2-D pipeline instead: truncated forward
 * FFT along the first axis, the fused 1-D kernel along the last axis on the K retained rows, zero-padded
 * inverse along the first axis, with two [B, C, K, N] strips in the workspace.  Shapes neither path covers:
 * TFNO_ERR_UNSUPPORTED.
 */
tfno_status tfno_spectral_conv2d(const void *x, const void *W, void *y,
                                 int B, int C_in, int C_out, int N, int K, void *stream);

/*
 * tfno_spectral_conv2d for callers that cannot allocate device memory or register a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result and kernels as
 * tfno_spectral_conv2d, but the intermediates (the truncated spectra, or the strips of the strip pipeline) live in
 * a scratch array of TFNO_NOALLOC_SCRATCH_BYTES that is part of the library image: every GPU the library runs on
 * holds its own copy until the process ends, and the call allocates and frees nothing and ignores
 * tfno_set_workspace.  A shape whose tfno_workspace_bytes(2, 0, ...) exceeds TFNO_NOALLOC_SCRATCH_BYTES returns
 * TFNO_ERR_WORKSPACE before anything is launched.  The first call on a device looks up the array's address there
 * (hipGetSymbolAddress); a failure of that lookup is TFNO_ERR_HIP.  All calls on one GPU share that GPU's array:
 * calls that may overlap in time on one GPU (different streams, or host threads without ordering) race on it and
 * must be serialised by the caller.  Nothing in the array needs clearing between calls: every element a launch
 * reads was written earlier in the same call.
 */
#define TFNO_NOALLOC_SCRATCH_BYTES (32u << 20)
tfno_status tfno_spectral_conv2d_noalloc(const void *x, const void *W, void *y,
                                         int B, int C_in, int C_out, int N, int K, void *stream);

/*
 * Unfused baseline with the structure the paper attributes to the PyTorch Fourier
 * layer (Sec. 1, Sec. 2.1): full FFT, truncate copy, CGEMM, zero-pad copy, full
 * inverse FFT, every intermediate in global memory (five launches in 1-D; the 2-D
 * version transforms both axes with separate launches).  Same contract and same
 * result as the fused entry points; accepts every valid shape.  Needs
 * tfno_workspace_bytes(dims, 1, ...) bytes of workspace.
 */
tfno_status tfno_spectral_conv1d_staged(const void *x, const void *W, void *y,
                                        int B, int C_in, int C_out, int N, int K, void *stream);
tfno_status tfno_spectral_conv2d_staged(const void *x, const void *W, void *y,
                                        int B, int C_in, int C_out, int N, int K, void *stream);

/*
 * 2-D spectral convolution on a non-square grid (the separable pipeline of Sec. 3.2 / 3.3 with each axis keeping
 * its own modes; the paper evaluates the square case):
 *
 *   y[b,o] = iFFT2( pad_N1xN2( sum_c trunc_K1xK2( FFT2(x[b,c]) ) * W[c,o] ) )      (iFFT2 scaled by 1 / (N1 N2))
 *
 * x is [B, C_in, N1, N2] and y [B, C_out, N1, N2], row-major with N2 contiguous; the modes kept are k1 < K1 along
 * the first spatial axis and k2 < K2 along the last.  N1, N2 powers of two in [2, 4096], 1 <= K1 <= N1,
 * 1 <= K2 <= N2.  N1, N2 in {64,128,256} with K1, K2 in {16,32,64} run the image kernels of
 * tfno_spectral_conv2d (workspace 8 B K1 K2 (C_in + C_out) bytes); other shapes whose last axis (N2, K2) the fused
 * 1-D kernel supports run the strip pipeline (workspace 8 B K1 N2 (C_in + C_out) bytes); the rest return
 * TFNO_ERR_UNSUPPORTED from the fused entry point.  The staged twin accepts every valid shape.  Pointer, aliasing,
 * stream and error rules as for tfno_spectral_conv2d; with N1 = N2 and K1 = K2 the calls are identical to
 * tfno_spectral_conv2d / tfno_spectral_conv2d_staged.  Workspace sizes: tfno_workspace_bytes_2d.
 */
tfno_status tfno_spectral_conv2d_rect(const void *x, const void *W, void *y, int B, int C_in, int C_out,
                                      int N1, int N2, int K1, int K2, void *stream);
tfno_status tfno_spectral_conv2d_rect_staged(const void *x, const void *W, void *y, int B, int C_in, int C_out,
                                             int N1, int N2, int K1, int K2, void *stream);

/*
 * The paper's own 2-D pipeline (Sec. 3.2, Sec. 3.3 and the fully fused 2-D variant of Sec. 5.2) on request, for
 * every shape including those that tfno_spectral_conv2d_rect runs on the image kernels: truncated forward FFT along
 * the first axis (writes the K1 retained rows), the fully fused 1-D kernel along the last axis on those rows,
 * zero-padded inverse FFT along the first axis; the two [B, C, K1, N2] strips go through the workspace
 * (tfno_workspace_bytes_2d(7, ...) = 8 B K1 N2 (C_in + C_out) bytes).  Same arguments, contract and result as
 * tfno_spectral_conv2d_rect.  It exists for comparison (the 2-D ablation of the paper): on this machine the image
 * kernels, which keep both axes of an image on chip, are several times faster.  Shapes: N1 a power of two in
 * [2, 4096] with any K1 <= N1, (N2, K2) a shape of the fused 1-D kernel; others TFNO_ERR_UNSUPPORTED.
 */
tfno_status tfno_spectral_conv2d_strips(const void *x, const void *W, void *y, int B, int C_in, int C_out,
                                        int N1, int N2, int K1, int K2, void *stream);

/*
 * Spectral convolution with an own weight matrix per retained mode -- the Fourier layer as the FNO model defines
 * it (Sec. 1, Sec. 2.1 step 3: a learned linear transformation in the frequency domain); the entry points above
 * take the single shared matrix of the paper's GEMM formulation (Sec. 3.1), which is the special case of equal
 * matrices:
 *
 *   1-D  y[b,o,:] = iFFT_N ( pad_N    ( sum_c trunc_K    ( FFT_N (x[b,c,:]) )[k]     * W[c,o,k]     ) )
 *   2-D  y[b,o]   = iFFT2  ( pad_N1xN2( sum_c trunc_K1xK2( FFT2  (x[b,c])   )[k1,k2] * W[c,o,k1,k2] ) )
 *
 * W is a device pointer to a contiguous row-major c64 tensor [C_in, C_out, K] (1-D) or [C_in, C_out, K1, K2]
 * (2-D), modes innermost; x, y, stream, aliasing and error rules as for the other entry points.  Three launches:
 * pruned forward transform with built-in truncation, per-mode contraction on the truncated spectra, pruned inverse
 * with built-in zero padding (the transform kernels of tfno_spectral_conv1d_pruned and tfno_spectral_conv2d_rect).
 * Shapes: 1-D those of tfno_spectral_conv1d_pruned with N <= 1024; 2-D N1, N2 in {64,128,256}, K1, K2 <= 64
 * (W holds exactly the K, or K1 x K2, matrices of the modes kept, whatever built size the transforms run);
 * others TFNO_ERR_UNSUPPORTED.  Workspace: tfno_workspace_bytes(1, 6, ...) and
 * tfno_workspace_bytes_2d(6, ...) bytes.
 */
tfno_status tfno_spectral_conv1d_permode(const void *x, const void *W, void *y,
                                         int B, int C_in, int C_out, int N, int K, void *stream);
tfno_status tfno_spectral_conv2d_permode(const void *x, const void *W, void *y, int B, int C_in, int C_out,
                                         int N1, int N2, int K1, int K2, void *stream);

/*
 * Real-valued 1-D layer (the R2C / C2R transforms FNO layers apply to real fields; the pipeline of Sec. 2.1 with
 * real input and output):
 *
 *   y[b,o,:] = C2R_N( pad( sum_c R2C_N(x[b,c,:])[k] * W[c,o],  k < K ) )
 *
 * x [B, C_in, N] and y [B, C_out, N] are device pointers to contiguous float32 tensors, W [C_in, C_out] to c64;
 * K <= N/2.  One launch of the fully fused kernel: the pencils are read as 4-byte reals, bin 0 enters the
 * contraction with weight 1/2 and the epilogue stores 2/N times the real part of the zero-padded inverse -- the
 * C2R transform of the Hermitian extension -- so the layer moves half the bytes of the complex one.  Shapes: N in
 * {64,128,256,512,1024}, K <= N/2 (built sizes: powers of two from 8 (N = 64), 16 (N = 128, 256), 32 (N = 512,
 * 1024); K <= 256); others TFNO_ERR_UNSUPPORTED.  Needs no workspace.  Pointer, aliasing, stream and error rules as above.
 */
tfno_status tfno_spectral_conv1d_real(const void *x, const void *W, void *y,
                                      int B, int C_in, int C_out, int N, int K, void *stream);

/*
 * The 2-D Fourier layer as FNO models apply it to real fields (Sec. 1 and Sec. 2.1 describe the pipeline; the
 * paper's kernels and the entry points above are its C2C form with one low-frequency corner and a shared W):
 *
 *   y = irfft2( pad( sum_c rfft2(x[b,c])[k1, k2] * W[c, o, k1 + M1, k2] ) ),   -M1 <= k1 < M1,  0 <= k2 < M2
 *
 * x [B, C_in, N1, N2] and y [B, C_out, N1, N2] are device pointers to contiguous float32 tensors; W is
 * [C_in, C_out, 2 M1, M2] c64, an own matrix per retained mode, the first-axis index holding the frequencies
 * -M1 .. M1-1 in this order (the block of negative frequencies first; public FNO implementations keep the two
 * blocks as two weight tensors: concatenate "weights2" then "weights1" along that axis).  2 M1 <= N1, 2 M2 <= N2.
 * Three launches: the forward image kernel (reads float32 rows, R2C along the last axis, both low-frequency blocks
 * of the first), the per-mode contraction, the inverse image kernel (C2R: stores the real part).  Shapes: N1, N2 in
 * {64, 128, 256}, 2 M1 <= 64, M2 <= 64 (any such M1, M2: the kernels run the next built block size); others
 * TFNO_ERR_UNSUPPORTED.  Needs tfno_fno2d_real_workspace_bytes(...) bytes of workspace (0 for unsupported or invalid
 * arguments).  Pointer, aliasing, stream and error rules as above.
 */
tfno_status tfno_fno2d_real(const void *x, const void *W, void *y, int B, int C_in, int C_out,
                            int N1, int N2, int M1, int M2, void *stream);
size_t tfno_fno2d_real_workspace_bytes(int B, int C_in, int C_out, int N1, int N2, int M1, int M2);

/*
 * The 1-D counterpart:  y = irfft( pad( sum_c rfft(x[b,c])[k] * W[c, o, k] ) ),  0 <= k < M,  2 M <= N.
 * x [B, C_in, N], y [B, C_out, N] float32, W [C_in, C_out, M] c64.  Three launches (pruned forward transform of the
 * real pencils, per-mode contraction, pruned inverse storing the real part).  Shapes: N in {64, 128, 256} with
 * M <= N/2, or N = 1024 with M <= 128; others TFNO_ERR_UNSUPPORTED.  Workspace:
 * tfno_fno1d_real_workspace_bytes(...) bytes.
 */
tfno_status tfno_fno1d_real(const void *x, const void *W, void *y, int B, int C_in, int C_out, int N, int M,
                            void *stream);
size_t tfno_fno1d_real_workspace_bytes(int B, int C_in, int C_out, int N, int M);

/*
 * 1-D spectral convolution as three launches with truncation, zero padding and butterfly pruning built into the
 * transforms but no fusion across the contraction (the variant "A" of Table 2, Sec. 5: pruned FFT, CGEMM, pruned
 * iFFT): only the K retained bins of every pencil cross global memory between the launches.  Same contract and
 * same result as tfno_spectral_conv1d.  Shapes: N in {64,128,256} with K a multiple of 16 such that K/16 is a
 * power of two not above N/16, N = 1024 with K in {64,128}, or long pencils N in {2048,4096} with K / (N/256) in
 * {16,32,64,128,256} (the pencil is transformed as N/256 rows of 256 points, every row truncated to K / (N/256)
 * bins); others TFNO_ERR_UNSUPPORTED.  Needs
 * tfno_workspace_bytes(1, 2, ...) bytes of workspace.  It is faster than a fused kernel whose contraction runs
 * on FP32 MFMA at hidden dimension 256 (the crossover Sec. 5.1 describes); against the default fused kernel
 * (BF16 matrix pipe) it is not.
 */
tfno_status tfno_spectral_conv1d_pruned(const void *x, const void *W, void *y,
                                        int B, int C_in, int C_out, int N, int K, void *stream);

/*
 * The two partially fused 1-D variants of the paper (variants "B" and "C" of Table 2, Sec. 5), two launches each:
 *   tfno_spectral_conv1d_fft_gemm   forward transform and CGEMM in one kernel (Sec. 4.1): x is read once, the
 *                                   truncated output spectrum Yh[B, C_out, K] goes through the workspace to the
 *                                   zero-padded, input-pruned inverse kernel;
 *   tfno_spectral_conv1d_gemm_ifft  CGEMM and inverse transform in one kernel (Sec. 4.2): the output-pruned
 *                                   forward kernel writes the truncated input spectrum Xh[B, C_in, K] to the
 *                                   workspace, the second kernel contracts it and writes y once.
 * Same contract and same result as tfno_spectral_conv1d.  Shapes: N in {128, 256}, K in {32, 64, 128} (K <= N);
 * others TFNO_ERR_UNSUPPORTED.  Workspace: tfno_workspace_bytes(1, 3, ...) and (1, 4, ...) bytes.
 */
tfno_status tfno_spectral_conv1d_fft_gemm(const void *x, const void *W, void *y,
                                          int B, int C_in, int C_out, int N, int K, void *stream);
tfno_status tfno_spectral_conv1d_gemm_ifft(const void *x, const void *W, void *y,
                                           int B, int C_in, int C_out, int N, int K, void *stream);

/*
 * Per-shape dispatch (variant "E" of Table 2, Sec. 5: the best of the variants for each shape), with the rule
 * measured on MI355X: the CGEMM + iFFT variant when C_out > 128, N = 128 and K <= 32 (the fully fused kernel
 * repeats the forward transform for every 128-output slab, which only there costs more than the detour of the
 * truncated spectrum; at N = 256 it covers 256 outputs per workgroup), else the fully fused kernel where one exists, else the three pruned kernels of tfno_spectral_conv1d_pruned where they exist (N = 2048, 4096), else the
 * staged path.  Accepts every valid 1-D shape; same contract and same result as
 * tfno_spectral_conv1d.  Workspace: tfno_workspace_bytes(1, 5, ...) bytes (0 when the fused kernel is chosen).
 */
tfno_status tfno_spectral_conv1d_auto(const void *x, const void *W, void *y,
                                      int B, int C_in, int C_out, int N, int K, void *stream);

/*
 * Workspace (device memory for intermediates) that an entry point needs for a
 * shape: dims = 1 or 2, variant = 0 (fused entry point), 1 (staged twin), 2
 * (tfno_spectral_conv1d_pruned), 3 (tfno_spectral_conv1d_fft_gemm), 4 (tfno_spectral_conv1d_gemm_ifft), 5
 * (tfno_spectral_conv1d_auto), 6 (tfno_spectral_conv1d_permode) or 7 (tfno_spectral_conv2d_strips, dims = 2 only).
 * Returns 0 when none is needed or the arguments are invalid.
 */
size_t tfno_workspace_bytes(int dims, int variant, int B, int C_in, int C_out, int N, int K);
/* The same for the 2-D entry points that take N1, N2, K1, K2: variant = 0 (tfno_spectral_conv2d_rect), 1 (its
 * staged twin) or 6 (tfno_spectral_conv2d_permode). */
size_t tfno_workspace_bytes_2d(int variant, int B, int C_in, int C_out, int N1, int N2, int K1, int K2);

/*
 * Registers a caller-owned device buffer as the library's workspace for all
 * later calls (the library never allocates).  dev_ptr = NULL with bytes = 0
 * clears it.  The buffer must be 256-byte aligned.  Calls that share the
 * workspace must be ordered on one stream (or otherwise serialised) by the caller.
 */
tfno_status tfno_set_workspace(void *dev_ptr, size_t bytes);

/* Static, NUL-terminated description of a status code. */
const char *tfno_status_string(tfno_status s);

/* Library version, major * 10000 + minor * 100 + patch. */
int tfno_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TFNO_H */
