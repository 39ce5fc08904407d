/*
 * wino.h -- C ABI of libwino: the forward path of a Winograd-aware 3x3
 * convolution layer, F(m x m, 3 x 3) with m in {2, 4, 6}, on one AMD MI355X
 * (gfx950).  Every step runs in hand-written HIP kernels; there is no CPU
 * fallback.
 *
 * The operation (paper, Sec. 3.1, Eq. 1, applied to every patch of the
 * activations as Sec. 3.2 describes, channels summed in the Winograd domain as
 * in the GEMM formulation of Sec. 5.3):
 *
 *     Y = A^T [ sum_c (G g G^T) (.) (B^T d B) ] A
 *
 * with a per-layer symmetric quantizer after every stage in the int8 mode
 * (Sec. 3.2, Fig. 2; Sec. 5.1).  B^T, G and A^T are arguments of every call, so
 * fixed Cook-Toom matrices and learned ("flex", Sec. 3.2) ones take the same
 * path.
 *
 * Conventions common to all entry points
 *   - Pointers named *_dev are DEVICE pointers, everything else is HOST memory.
 *   - The caller owns all buffers.  The library allocates and frees nothing on
 *     the device and keeps no state between calls (the one exception is the
 *     built-in scratch buffer of wino_conv2d_fwd_noalloc, described there).
 *   - Matrices in a wino_desc are read on the host during the call and passed to
 *     the kernels by value; the caller may change them as soon as the call
 *     returns.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream).  No entry point synchronises.
 *   - Every argument check happens before the first HIP call, so error paths
 *     never touch the GPU.  Errors are returned, never thrown or aborted on.
 *   - Tensors: X[N][C][H][W], g[K][C][3][3], Y[N][K][Ho][Wo] with
 *     Ho = H + 2 pad - 2 (stride is 1 by definition of the Winograd path),
 *     row-major, last index fastest.  dtype WINO_I8: X and Y hold int8 codes
 *     (x = s_x * code); dtype WINO_F32: float, no quantizer anywhere;
 *     WINO_I16 / WINO_I8W16: wider stages, see wino_dtype.
 *   - Tiling: n = m + 2, P = n*n Winograd positions p = i*n + j,
 *     TH = ceil(Ho/m), TW = ceil(Wo/m), T = N*TH*TW tiles,
 *     t = (img*TH + th)*TW + tw.  Tile (th,tw) reads input rows
 *     th*m - pad + j and columns tw*m - pad + l (zero outside the image) and
 *     writes output rows th*m + a, columns tw*m + b (dropped outside).
 */
#ifndef WINO_H_
#define WINO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  WINO_OK = 0,
  WINO_E_NULL = -1,       /* a required pointer is NULL                          */
  WINO_E_BAD_M = -2,      /* m is not 2, 4 or 6                                  */
  WINO_E_BAD_SHAPE = -3,  /* a dimension is < 1, pad not in {0,1}, output empty,
                             or a size overflows the 31-bit index range          */
  WINO_E_BAD_DTYPE = -4,  /* dtype is not one of wino_dtype                      */
  WINO_E_BAD_SCALE = -5,  /* quantized modes: a scale is not finite and > 0, a
                             qmax outside the range of its container, quant
                             missing; or a matrix entry is not finite            */
  WINO_E_WORKSPACE = -6,  /* workspace smaller than wino_workspace_bytes()       */
  WINO_E_HIP = -7,        /* a HIP call or kernel launch failed                  */
  WINO_E_BAD_ARG = -8,    /* other invalid argument (stride, tap selector, ...)  */
  WINO_E_SCRATCH_LIMIT = -9 /* wino_conv2d_fwd_noalloc: the problem needs more scratch
                             than WINO_NOALLOC_SCRATCH_BYTES                      */
} wino_status;

/* WINO_F32   float everywhere, no quantizer.
 * WINO_I8    int8 codes after every stage (X, U, V, Y; M int32), Sec. 5.1's INT8.
 * WINO_I16   up to 16-bit codes after every stage (Sec. 5.1's INT10 and INT16): X and Y are
 *            int16 arrays, U and V hold 16-bit codes, M is the exact int64 sum.
 * WINO_I8W16 8-bit activations with a 16-bit Winograd domain (Sec. 3.2, "quantization
 *            diversity"; Sec. 7, different bit-widths through Eq. 1): X and Y are int8
 *            arrays, U, V and the Hadamard-stage quantizer may use up to 16 bits.
 * The two wide modes accept one code range per stage (wino_quant.qmax_*), need C <= 1024,
 * and run as two kernels (input transform; GEMM fused with the output transform) or, for
 * layers with few tiles and channel counts whose padding is not 64/128/256/512, three.
 * WINO_BF16  the float path with bf16 operands in the Winograd-domain GEMM (the variant
 *            of the method's GEMM stage for speed): X, g and Y are
 *            float, the transforms run in fp32 exactly as for WINO_F32, U and V are rounded
 *            to bf16 (nearest even) where they enter the per-position GEMM, which
 *            accumulates in fp32 on v_mfma_f32_16x16x16_bf16.  Error against WINO_F32 about
 *            2^-9 relative per operand: a speed option, outside the float mode's 1e-4.
 *            Built as a one-kernel forward for m in {2, 4}; other tile sizes, and shapes
 *            whose staging does not fit the kernel, return WINO_E_BAD_SHAPE / WINO_E_BAD_M.
 *            No stage-by-stage calls and no taps. */
typedef enum { WINO_F32 = 0, WINO_I8 = 1, WINO_I16 = 2, WINO_I8W16 = 3, WINO_BF16 = 4 } wino_dtype;

/* One layer problem.  BT is n x n, G is n x 3, AT is m x n, row-major, HOST. */
typedef struct {
  int N, C, K, H, W;
  int pad;          /* 0 or 1 */
  int m;            /* 2, 4 or 6 */
  int dtype;        /* a wino_dtype, held as int so that any value can be passed and refused */
  const float* BT;
  const float* G;
  const float* AT;
} wino_desc;

/* Scales of the quantizers (Sec. 3.2: one after each stage; Sec. 5.1: one
 * symmetric scale per layer and stage).  real value = scale * code.
 *   s_x input, s_v transformed input B^T d B, s_u transformed weights G g G^T,
 *   s_y output, s_m Hadamard/GEMM result (0 = that quantizer is off).
 * Codes saturate to [-qmax, qmax]; rounding is half-to-even. */
typedef struct {
  float s_x, s_v, s_u, s_y, s_m;
  int qmax;         /* 1..127 (1..32767 in the wide modes); see qmax_* below */
  /* Optional finer granularity (Sec. 7 suggests finer-grained quantization than one scale
   * per tensor as the way to recover the accuracy of the larger tiles):
   * one scale per Winograd position p = i*n + j for the transformed input and the
   * transformed weights, HOST arrays of n*n floats, both or neither (NULL).  When given,
   * s_v and s_u are ignored, Vq[p] = sat(rne(V[p] * s_x / s_v_pos[p])),
   * Uq[p] = sat(rne(U[p] / s_u_pos[p])), and every accumulator is brought to real units
   * before the output transform, Mf[p] = (float)M[p] * (s_u_pos[p] * s_v_pos[p]), so that
   * y_q = sat(rne(Yt / s_y)) (with the Hadamard-stage quantizer: Mq = sat(rne(Mf / s_m)),
   * y_q = sat(rne(Yt * s_m / s_y))).  The kernel sequence is that of per-tensor
   * scales, except that F(6x6,3x3) with at most 64 channels takes three kernels. */
  const float* s_v_pos;
  const float* s_u_pos;
  /* One code range per quantizer (Sec. 3.2: each stage may be quantized to its own number
   * of bits), 0 = qmax: transformed weights, transformed input, Hadamard stage, output.
   * Limits: 127 where the codes live in int8 (every stage of WINO_I8, where all ranges
   * must also agree; qmax_y of WINO_I8W16), 32767 otherwise.  The codes of X are the
   * caller's; they only have to fit X's container. */
  int qmax_u, qmax_v, qmax_m, qmax_y;
} wino_quant;

const char* wino_status_string(wino_status s);

/* Bytes of the transformed-weight buffer U / of the workspace (transformed input
 * V followed by the Hadamard/GEMM result M) for this problem; 0 if the
 * descriptor is invalid.  Both layouts are private to the library. */
size_t wino_weights_bytes(const wino_desc* d);
size_t wino_workspace_bytes(const wino_desc* d);

/* Weight stage of Eq. 1: U = G g G^T for every (k, c) (Sec. 3.1; amortised over
 * inferences).  int8 mode: Uq = sat(rne(U / s_u)) with one scale for the whole
 * tensor; `q` may be NULL only for WINO_F32.
 *   g_dev  in   DEVICE float [K][C][3][3] (weights always enter as fp32)
 *   U_dev  out  DEVICE, wino_weights_bytes(d) bytes, 256-byte aligned        */
wino_status wino_transform_weights(const wino_desc* d, const wino_quant* q,
                                   const float* g_dev, void* U_dev, void* stream);

/* Forward of the layer (Sec. 3.2): input transform B^T d B on every
 * overlapping patch (+ quantizer), one GEMM per Winograd position summing over
 * input channels (+ optional quantizer), output transform A^T M A (+ quantizer)
 * and scatter to NCHW.
 *   x_dev          in   DEVICE X, int8 / int16 codes or float (aligned to its element)
 *   U_dev          in   DEVICE, produced by wino_transform_weights for the same d
 *   y_dev          out  DEVICE Y, int8 / int16 codes or float
 *   workspace_dev       DEVICE scratch, >= wino_workspace_bytes(d), 256-byte
 *                       aligned.  What it holds afterwards depends on the kernel
 *                       sequence (wino_fwd_num_kernels): nothing new after the
 *                       one-kernel forward, V after two kernels, V and M after
 *                       three; the parity taps (wino_debug_export) therefore read it
 *                       after wino_conv2d_fwd_stages has run the stages separately */
wino_status wino_conv2d_fwd(const wino_desc* d, const wino_quant* q, const void* x_dev,
                            const void* U_dev, void* y_dev, void* workspace_dev,
                            size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: wino_conv2d_fwd without the workspace
 * argument.  V and M live in a buffer of WINO_NOALLOC_SCRATCH_BYTES that is part of the
 * library's device image (every GPU the library runs on holds one copy until the process
 * ends); the call allocates and frees nothing.  Same kernels, same results and same
 * argument checks as wino_conv2d_fwd.  The buffer only has to hold what the problem's
 * kernel sequence touches (nothing for one kernel, V for two, V and M for three, see
 * wino_fwd_num_kernels); a problem that needs more returns WINO_E_SCRATCH_LIMIT before
 * anything is launched.  All calls on one GPU share that GPU's buffer: calls that overlap
 * in time on one GPU (different streams, or a captured graph replayed next to eager calls)
 * race on it.  The first call on a device looks the buffer's address up
 * (hipGetSymbolAddress) and must therefore happen outside stream capture. */
#define WINO_NOALLOC_SCRATCH_BYTES (32u << 20)
wino_status wino_conv2d_fwd_noalloc(const wino_desc* d, const wino_quant* q, const void* x_dev,
                                    const void* U_dev, void* y_dev, void* stream);

/* How many kernels wino_conv2d_fwd launches for this problem (0 if the descriptor is
 * invalid): 1 = input transform, GEMM and output transform in one
 * kernel (small layers; V and M never reach memory), 2 = input transform, then GEMM fused
 * with the output transform (M never reaches memory), 3 = input transform, tiled GEMM,
 * output transform (F(6x6,3x3) and F(4x4,3x3) with long reductions and few tiles, more
 * than 512 input channels).  The wide modes run as 2 or 3 kernels.  Reads d->BT /
 * d->AT (HOST) if they are not NULL: which variant applies can depend on them. */
int wino_fwd_num_kernels(const wino_desc* d);

/* Kernel sequences of the int8 forward.  wino_conv2d_fwd picks one from a table of times
 * measured on MI355X over a grid of layer shapes (as the paper picks the algorithm per layer
 * from measured latencies, Sec. 5.3); the calls below let a tuner or a test name it. */
#define WINO_SEQ_AUTO 0    /* the table's choice                                          */
#define WINO_SEQ_FUSED 1   /* one kernel                                                   */
#define WINO_SEQ_COL 2     /* input stage; GEMM + column-wise output transform             */
#define WINO_SEQ_COL2 3    /* ... two tile blocks per wavefront                            */
#define WINO_SEQ_LDS 4     /* input stage; GEMM + output transform, 32 x 64 workgroup tiles */
#define WINO_SEQ_REGS 5    /* input stage; GEMM + output transform, accumulators in registers */
#define WINO_SEQ_STAGED 6  /* input stage; GEMM writing M; output transform               */
#define WINO_SEQ_TROW 7    /* input stage; GEMM + output transform on whole rows of tiles
                            * (F(6x6,3x3); a y_dev that is not 16-byte aligned runs
                            * WINO_SEQ_COL instead, named or not)                        */
#define WINO_SEQ_COUNT 8
/* seq = WINO_SEQ_AUTO: the sequence wino_conv2d_fwd takes for this problem; any other seq:
 * seq itself if that sequence can run the problem, else 0.  0 also for an invalid
 * descriptor and for dtypes other than WINO_I8.  HOST only; reads d->BT if not NULL. */
int wino_fwd_sequence(const wino_desc* d, int seq);
/* wino_conv2d_fwd with the kernel sequence named by the caller (same arguments, results
 * and checks; the workspace must hold wino_workspace_bytes(d)).  WINO_E_BAD_ARG if the
 * sequence cannot run the problem (wino_fwd_sequence(d, seq) == 0). */
wino_status wino_conv2d_fwd_seq(const wino_desc* d, const wino_quant* q, const void* x_dev,
                                const void* U_dev, void* y_dev, void* workspace_dev,
                                size_t workspace_bytes, int seq, void* stream);

/* The same forward, restricted to the stages named in `stages` (a mask of
 * WINO_STAGE_*), for per-kernel timing and for tests: a stage reads what the
 * previous one left in the workspace.  WINO_STAGE_ALL is wino_conv2d_fwd.
 * Pointers a selected stage does not touch may be NULL (x_dev without INPUT,
 * U_dev without GEMM, y_dev without OUTPUT). */
enum { WINO_STAGE_INPUT = 1, WINO_STAGE_GEMM = 2, WINO_STAGE_OUTPUT = 4, WINO_STAGE_ALL = 7 };
wino_status wino_conv2d_fwd_stages(const wino_desc* d, const wino_quant* q, const void* x_dev,
                                   const void* U_dev, void* y_dev, void* workspace_dev,
                                   size_t workspace_bytes, int stages, void* stream);

/* Parity taps: copy one intermediate out of the private layout into the
 * canonical dense order.
 *   which = WINO_TAP_U : src_dev = U buffer      -> out [P][K][C] int8 | float | int16
 *   which = WINO_TAP_V : src_dev = workspace     -> out [P][T][C] int8 | float | int16
 *   which = WINO_TAP_M : src_dev = workspace     -> out [P][T][K] int32 | float | int64
 * (third type: the wide modes WINO_I16 and WINO_I8W16) */
enum { WINO_TAP_U = 0, WINO_TAP_V = 1, WINO_TAP_M = 2 };
wino_status wino_debug_export(const wino_desc* d, int which, const void* src_dev,
                              void* out_dev, void* stream);

/* Matrix-core peak probe for the roofline figures (measurement infrastructure, not part
 * of the paper's method): launches `workgroups` x 256 threads, every wavefront issuing
 * 8 * iters independent MFMAs of the path's instruction (v_mfma_i32_16x16x64_i8 for
 * WINO_I8, v_mfma_f32_16x16x4_f32 for WINO_F32) and nothing else.
 *   out_dev         out  DEVICE, workgroups * 256 floats (checksums, ignore)
 *   ops_per_launch  out  HOST, may be NULL: multiply-adds x 2 the launch performs
 * Time it with events on `stream`; ops / time is the achievable matrix rate. */
wino_status wino_debug_mfma_loop(int dtype, int workgroups, int iters, float* out_dev,
                                 double* ops_per_launch, void* stream);

/* Vector-memory-path probe (not the paper's): `workgroups` workgroups of `waves` (4, 8 or 16)
 * wavefronts; every wavefront walks its own slice (workgroup_bytes / waves) of its
 * workgroup's part of buf_dev round and round, eight loads in flight, `iters` rounds of
 * eight loads.  mode 0: 16 bytes per lane into registers, 1: 8 bytes, 2: 4 bytes, 3: 16 bytes
 * per lane straight into LDS.  A slice that fits the L1 measures the L1, a workgroup part
 * that fits its XCD's share of the L2 the L2 -> L1 path, a larger one what lies behind.
 *   buf_dev           in   DEVICE, workgroups * workgroup_bytes bytes (any contents)
 *   out_dev           out  DEVICE, workgroups * waves * 64 floats (checksums, ignore)
 *   bytes_per_launch  out  HOST, may be NULL: bytes one launch loads
 * workgroup_bytes: a multiple of waves * 1024.  Time it with events on `stream`. */
wino_status wino_debug_load_loop(int mode, int waves, int workgroups, size_t workgroup_bytes,
                                 int iters, const void* buf_dev, float* out_dev,
                                 double* bytes_per_launch, void* stream);

/* Cook-Toom matrices for F(m,3) from m+1 distinct finite points (NULL = the
 * usual 0, 1, -1, 1/2, -1/2, 2, -2 prefix) plus the point at infinity
 * (Sec. 3.1).  HOST outputs: BT n*n, G n*3, AT m*n floats. */
wino_status wino_cook_toom(int m, const double* points, float* BT, float* G, float* AT);

/* Baseline the paper compares against: im2row 3x3 convolution (Sec. 5.3, Table 3),
 * stride 1 or 2: every output pixel is a row of 9*C taps, one GEMM with the packed
 * weights, requantize and scatter to NCHW.  Weights are packed once with
 * conv2d_ref_pack_weights.
 * int8 mode: y = sat(rne(acc * (s_x*s_w/s_y))), codes in [-qmax,qmax].
 * conv2d_ref_gpu runs int8 as ONE kernel that gathers the rows of its pixels in LDS
 * and never writes the row matrix (the workspace is then left untouched), fp32 as
 * three kernels (gather to the workspace, GEMM, epilogue); conv2d_ref_gpu_rows always
 * runs the three kernels.  Both give the same y; both take the same arguments and
 * need the same workspace size. */
size_t conv2d_ref_packed_weights_bytes(int C, int K, int dtype);
size_t conv2d_ref_workspace_bytes(int N, int C, int K, int H, int W, int stride, int pad,
                                  int dtype);
/*   w_dev   in  DEVICE [K][C][3][3], int8 codes or float
 *   wp_dev  out DEVICE packed weights, conv2d_ref_packed_weights_bytes bytes, aligned to
 *           256: one row of 9*Cp values per output channel, tap-major, zero padded; for
 *           int8 the same weights follow once more in matrix-core operand order (what
 *           the one-kernel form reads)                                             */
wino_status conv2d_ref_pack_weights(int C, int K, int dtype, const void* w_dev,
                                    void* wp_dev, void* stream);
wino_status conv2d_ref_gpu(int N, int C, int K, int H, int W, int stride, int pad,
                           int dtype, const void* x_dev, const void* wp_dev,
                           void* y_dev, float s_x, float s_w, float s_y, int qmax,
                           void* workspace_dev, size_t workspace_bytes, void* stream);
wino_status conv2d_ref_gpu_rows(int N, int C, int K, int H, int W, int stride, int pad,
                                int dtype, const void* x_dev, const void* wp_dev,
                                void* y_dev, float s_x, float s_w, float s_y, int qmax,
                                void* workspace_dev, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* WINO_H_ */
