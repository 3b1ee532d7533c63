/*
 * rnswino -- exact INT8 2-D convolution by Winograd minimal filtering inside a
 * residue number system, for AMD MI355X (gfx950).  C ABI.
 *
 * Method: "Efficient Residue Number System Based Winograd Convolution"
 * (arXiv 2007.12216).  A quantised layer g (*) x between an (R x R x C x K)
 * signed-int8 weight tensor and a (B x W x H x C) signed-int8 input
 * (section 6, first paragraph) is computed with F(M x M, R x R) over
 * RNS(m_0 .. m_{n-1}) (section 5, eq. "fast_algorithm_rns"; section 6, eqs.
 * "direct_sum_winograd" / "direct_sum_2" / "gemm"), and the result is
 * converted back from the residues (section 3, which names mixed-radix
 * conversion or the Chinese remainder theorem for this step).  The kernels
 * take the CRT sum with a rounded quotient,
 *   y = sum_i (P/m_i) w_i - P rint(sum_i w_i / m_i),  w_i = Y_i (P/m_i)^-1 mod m_i,
 * which is the same representative in [-(P-1)/2, (P-1)/2], P = prod m_i, that
 * mixed-radix conversion with symmetric digits yields; the tests compare the
 * two bit for bit.
 * The result is the exact integer convolution (abstract; section 9).
 *
 * In this header the paper's M, R, N = M+R-1 are spelled m, r, t; N, C, K, H, W
 * are the tensor dimensions.  Tensors are NCHW / KCrr, contiguous, in DEVICE
 * memory unless a parameter says "host".
 *
 * Ownership: the caller owns every device buffer (x, w, U, workspace, y).  A
 * plan owns only its own small constant tables (host and device).  None of
 * rnswino_filter_transform / rnswino_conv2d / rnswino_requant_pool allocates,
 * frees or synchronises: they enqueue kernels on `stream` (a hipStream_t
 * passed as void*, NULL = the default stream) and return.  Calls that share a
 * workspace must be ordered by the caller (same stream or events).
 *
 * Errors: every int-returning function returns RNSWINO_OK (0) or a negative
 * code; nothing throws, aborts or prints.
 */
#ifndef RNSWINO_H
#define RNSWINO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  RNSWINO_OK = 0,
  RNSWINO_E_INVALID = -1,              /* null pointer, non-positive size, t > 16, m < 1, output empty      */
  RNSWINO_E_UNSUPPORTED = -2,          /* stride != 1, r > 7, even modulus, modulus < 3, in 254..256 or > 65521,
                                          8/16-bit mix, 2^14 r^2 C beyond int32, 16-bit moduli with C > 65472,
                                          fused glue on other tile sizes                                     */
  RNSWINO_E_NOT_COPRIME = -3,          /* two moduli share a factor (section 3: pairwise coprime)           */
  RNSWINO_E_POINT_NOT_INVERTIBLE = -4, /* a modulus shares a factor with a difference of two interpolation
                                          points, so a denominator of V^-1 has no inverse (section 5)       */
  RNSWINO_E_RANGE = -5,                /* 2^14 r^2 C (or the caller's output_bound) exceeds (prod m_i - 1)/2: the
                                          dynamic range of the RNS cannot hold the output (sections 3, 5, 8) */
  RNSWINO_E_HIP = -6,                  /* a HIP runtime call or kernel launch failed                        */
  RNSWINO_E_NO_DEVICE = -7,            /* the plan was made host-only, or no GPU is present                 */
  RNSWINO_E_WORKSPACE = -8             /* rnswino_conv2d_static: the layer needs more workspace than
                                          RNSWINO_STATIC_WORKSPACE_BYTES                                    */
};

enum {
  RNSWINO_FLAG_ALLOW_UNCHECKED_RANGE = 1u, /* skip the worst-case range test: the caller vouches that every
                                              output lies in [-(P-1)/2, (P-1)/2], P = prod m_i, as the paper
                                              does with a measured range (section 8); otherwise the output
                                              is the true result reduced to that interval (mod 2^32)       */
  RNSWINO_FLAG_HOST_ONLY = 2u,             /* build the host tables only (no GPU touched): such a plan can
                                              be queried but not executed                                   */
  RNSWINO_FLAG_GEMM_BLOCK_64X16 = 4u       /* measurement only (8-bit moduli): run the residue GEMM on workgroup blocks
                                              of 64 rows x 16 tiles -- the largest block whose GEMM output (n t^2
                                              bytes per (k, tile) pair) one workgroup could keep in LDS if the
                                              inverse transform were fused into the GEMM (section 6: the stages
                                              compose per tile group).  Same result, slower; used to price that fusion */
};

typedef struct rnswino_plan_s rnswino_plan_t;   /* opaque, owned by the library */

typedef struct {
  int32_t  N, C, K, H, W;   /* activations x: int8 [N][C][H][W]                                              */
  int32_t  r;               /* filter r x r, 1 <= r <= 7; weights w: int8 [K][C][r][r]                       */
  int32_t  m;               /* output tile m x m; transform tile t = m + r - 1, 2 <= t <= 16                */
  int32_t  pad;             /* zeros added on each side of H and W (>= 0)                                   */
  int32_t  stride;          /* must be 1 (0 is read as 1)                                                    */
  int32_t  n_moduli;        /* 1 .. 8                                                                        */
  uint32_t moduli[8];       /* odd, pairwise coprime; either all in [3,253] (residues stored in 8 bits) or
                               all in [257,65521] (16 bits)                                                  */
  uint32_t flags;           /* RNSWINO_FLAG_*                                                                */
  uint64_t output_bound;    /* 0: the range test uses the worst case 2^14 r^2 C of int8 operands.  Otherwise an upper
                               bound on |y| that the caller guarantees for this layer, e.g. 128 * max_k sum_{c,i,j}
                               |w[k][c][i][j]| for its actual weights (a proof, where the paper trusts a measured
                               range, section 8): the range test and the choice of the conversion use it (if it is
                               smaller than the worst case), so fewer moduli may pass.  With weights that exceed it
                               the result is the true value reduced to the symmetric range of the moduli set.       */
} rnswino_desc_t;

/* Transform matrices modulo one modulus, entries in [-(p-1)/2, (p-1)/2] (section 5):
 * A^T is m x t, G is t x r, B^T is t x t, row-major. */
enum { RNSWINO_MATRIX_AT = 0, RNSWINO_MATRIX_G = 1, RNSWINO_MATRIX_BT = 2 };

/* Intermediate tensors of the pipeline (section 6), for stage-level checks. */
enum { RNSWINO_STAGE_U = 0, RNSWINO_STAGE_V = 1, RNSWINO_STAGE_O = 2 };

/*
 * Build a plan (sections 4-5): interpolation points 0, +1, -1, +2, -2, ..., infinity; A^T, G, B^T modulo
 * every modulus by exact modular arithmetic; checks (coprimality, invertibility of every point difference,
 * dynamic range); mixed-radix constants; the transform tables the kernels read, uploaded to the current
 * HIP device unless RNSWINO_FLAG_HOST_ONLY.  `desc` is host memory and is copied.  On error *out is NULL.
 * The plan belongs to that device: rnswino_filter_transform and the rnswino_conv2d calls must be made with the same
 * device current (RNSWINO_E_INVALID otherwise), on buffers and a stream of that device.
 */
int rnswino_plan(rnswino_plan_t **out, const rnswino_desc_t *desc);
int rnswino_plan_destroy(rnswino_plan_t *plan);

/* Output plane size Ho = H + 2 pad - r + 1 (and Wo likewise); y is int32 [N][K][Ho][Wo]. */
int rnswino_output_dims(const rnswino_plan_t *plan, int32_t *Ho, int32_t *Wo);

/* Bytes of the transformed filter U (all residues, all t*t transform points) and of the workspace that
 * holds the transformed input V and the GEMM output O.  0 if plan is NULL. */
size_t rnswino_filter_bytes(const rnswino_plan_t *plan);
size_t rnswino_workspace_bytes(const rnswino_plan_t *plan);

/*
 * Offline filter transform (section 6: it depends on the weights only, so it is computed ahead of time):
 *   U[i][xi,nu][k][c] = (G_p g^(c)(k) G_p^T)[xi,nu] mod m_i.
 * w_dev: int8 [K][C][r][r].  U_dev: rnswino_filter_bytes() bytes, 256-byte aligned, written in the library's
 * own tiled layout; it stays valid for any plan with the same C, K, r, m and moduli.
 */
int rnswino_filter_transform(const rnswino_plan_t *plan, const int8_t *w_dev, void *U_dev, void *stream);

/*
 * The layer (section 6): residues of x, input transform B^T d B per tile and residue, one GEMM over C per
 * transform point and residue with the modulo after the sum, inverse transform A^T (.) A after that
 * reduction, conversion out of the RNS to int32 (section 3; the CRT sum described at the top of this file).
 * x_dev: int8 [N][C][H][W].  U_dev: from rnswino_filter_transform.  y_dev: int32 [N][K][Ho][Wo].
 * workspace_dev: rnswino_workspace_bytes() bytes, 256-byte aligned; contents are scratch.  U_dev, workspace_dev
 * and y_dev must be 16-byte aligned (E_INVALID otherwise); x_dev may have any alignment.
 * When the plan passed the range test, y equals the direct convolution
 *   y[n][k][oy][ox] = sum_{c,i,j} xpad[n][c][oy+i-pad][ox+j-pad] * w[k][c][i][j]
 * (correlation orientation of section 3.1) bit for bit.
 */
int rnswino_conv2d(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev,
                   int32_t *y_dev, void *workspace_dev, void *stream);

/*
 * rnswino_conv2d for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation and same kernels; the transformed
 * input V and the GEMM output O live in a buffer of RNSWINO_STATIC_WORKSPACE_BYTES that is part of the library's loaded
 * code object on each GPU (held until the process ends; its per-device address is looked up once, when the first plan is
 * made on that device).  The call allocates and frees nothing and does not synchronise.  Layers whose
 * rnswino_workspace_bytes() exceeds the buffer are refused with RNSWINO_E_WORKSPACE (nothing is launched).
 * Every call on a GPU uses that GPU's one buffer: calls that may overlap in time (different streams without an event
 * between them, or different host threads) race; calls on one stream are ordered and safe.  The buffer keeps the last
 * call's contents; nothing in it needs clearing: the only bytes a call reads before it has written them belong to padding
 * tiles, whose results are never stored.
 * x_dev, U_dev, y_dev: as for rnswino_conv2d.
 */
#define RNSWINO_STATIC_WORKSPACE_BYTES (16u << 20)
int rnswino_conv2d_static(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev, int32_t *y_dev, void *stream);

/*
 * rnswino_conv2d fused with the layer glue of rnswino_requant_pool: the inverse-transform kernel writes
 *   a = clamp(floor(y / 2^shift), -128, 127)   (int8 [N][K][Ho][Wo]), after a 2x2 stride-2 max-pool when pool != 0
 * (int8 [N][K][Ho/2][Wo/2]), and the int32 y is never stored.  Without pooling every tile size is supported (m of 4 or 8
 * with an even Wo stores two or four bytes at a time, anything else single bytes); pooling needs m of 4 or 8, Wo a multiple
 * of 4 and an even Ho, otherwise RNSWINO_E_UNSUPPORTED (use rnswino_conv2d + rnswino_requant_pool).
 * a_dev must be 4-byte aligned.  Not part of the paper's method (the 13-layer stack workload needs it).
 */
int rnswino_conv2d_requant(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev, int8_t *a_dev,
                           int32_t shift, int32_t pool, void *workspace_dev, void *stream);

/*
 * rnswino_conv2d with six caller-created hipEvent_t (passed as void*): events[2j] and events[2j+1] receive the
 * start and stop timestamps of kernel j (0: input transform, 1: residue GEMM, 2: inverse transform + conversion),
 * so hipEventElapsedTime(events[2j], events[2j+1]) is that kernel's own duration.  For per-stage measurement
 * (the paper's time breakdown of section 8); does not synchronise.
 */
int rnswino_conv2d_events(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev, int32_t *y_dev,
                          void *workspace_dev, void *stream, void *const events[6]);

/*
 * Glue for chaining layers (not part of the paper's method; the 13-layer stack workload needs it):
 *   a = clamp(floor(y / 2^shift), -128, 127), optionally followed by a 2x2 stride-2 max-pool.
 * y_dev: int32 [planes][H][W]; a_dev: int8 [planes][H][W], or [planes][H/2][W/2] when pool != 0 (H, W even).
 */
int rnswino_requant_pool(const int32_t *y_dev, int8_t *a_dev, int64_t planes, int32_t H, int32_t W,
                         int32_t shift, int32_t pool, void *stream);

/*
 * Direct int8 convolution as an implicit GEMM on the matrix cores: the baseline the paper measures against (section 8,
 * Tables 4 and 5: Im2col + INT8 GEMM), provided so that the two paths can be timed on the same chip.  Same result as
 * rnswino_conv2d (the exact int32 convolution, correlation orientation of section 3.1, stride 1), no RNS, no transforms.
 *   rnswino_direct_filter_pack: w_dev int8 [K][C][r][r] -> wt_dev, rnswino_direct_filter_bytes(C, K, r) bytes, 16-byte
 *     aligned, in matrix-core fragment order (ahead of time: the weights are constants of the layer);
 *   rnswino_direct_conv2d: x_dev int8 [N][C][H][W], y_dev int32 [N][K][Ho][Wo]; workspace_dev holds
 *     rnswino_direct_workspace_bytes(N, C, H, W, pad) bytes (16-byte aligned): the activations copied once into a
 *     channel-innermost, zero-bordered layout.  No im2col matrix is written: operand fragments are gathered from that copy.
 * Nothing is allocated or synchronised; kernels are enqueued on `stream`.  r <= 16; sizes whose 32-bit offsets would
 * overflow are RNSWINO_E_UNSUPPORTED (the byte counts are then 0).
 */
size_t rnswino_direct_filter_bytes(int32_t C, int32_t K, int32_t r);
size_t rnswino_direct_workspace_bytes(int32_t N, int32_t C, int32_t H, int32_t W, int32_t pad);
int rnswino_direct_filter_pack(const int8_t *w_dev, void *wt_dev, int32_t C, int32_t K, int32_t r, void *stream);
int rnswino_direct_conv2d(const int8_t *x_dev, const void *wt_dev, int32_t *y_dev, int32_t N, int32_t C, int32_t K, int32_t H,
                          int32_t W, int32_t r, int32_t pad, void *workspace_dev, void *stream);

/* ---- query / test surface ---- */

/* Copy one transform matrix (which = RNSWINO_MATRIX_*, modulus_idx < n_moduli) to host_out (row-major int32). */
int rnswino_plan_get_matrix(const rnswino_plan_t *plan, int which, int modulus_idx, int32_t *host_out);

/* Copy the Kronecker table of one modulus, as the kernels read it, to host_out: which = RNSWINO_TABLE_INPUT is
 * (B^T kron B^T) mod p (input transform, section 5: V = B^T d B) as int8 [CB][KS1][planes][64 lanes][16]: fragment (cb, s)
 * holds, for lane l and byte b, the entry of transform point 16 cb + l%16 and contraction slot f = 64 s + 16 (l/16) + b =
 * tile pixel (row f / RP, column f % RP), RP = 4 ceil(t/4), zero outside the t x t tile; which = RNSWINO_TABLE_INVERSE is (A^T kron A^T) (P/p)^-1 mod p (inverse transform folded with
 * the CRT factor, sections 3 and 5) as int8 [RB][KS3][planes][64][16]: fragment (rb, s), lane l, byte b = output
 * 16 rb + l%16 and transform point 64 s + 16 (l/16) + b.  CB = ceil(t^2/16), KS1 = ceil(t RP / 64), RB = ceil(m^2/16),
 * KS3 = ceil(t^2/64); planes = 1 (8-bit moduli: the symmetric residue) or 2 (16-bit moduli: high byte plane, then low
 * byte plane, entry = 256 h + l).  Returns the number of bytes (copied only if capacity suffices), or a negative code. */
#define RNSWINO_TABLE_INPUT 0
#define RNSWINO_TABLE_INVERSE 1
int64_t rnswino_plan_get_table(const rnswino_plan_t *plan, int which, int modulus_idx, int8_t *host_out, size_t capacity);

/* Mixed-radix constant of section 3: inverse of moduli[l] modulo moduli[j] (l < j), in [0, moduli[j]).  A query for
 * tests and for callers that convert residues themselves: no kernel reads these (the kernels use the CRT sum). */
int rnswino_plan_get_mrc_inverse(const rnswino_plan_t *plan, int l, int j, uint32_t *host_out);

/*
 * Which kernel instantiations rnswino_conv2d (output_mode 0), or rnswino_conv2d_requant without (1) or with (2)
 * pooling, launches for this plan, their grids, and which form of the conversion out of the RNS (section 3) the layer
 * takes -- as text in host_out, one line per kernel in launch order, written as a profiler prints kernel names, e.g.
 *   k1_input_transform<2, false, false> grid=200x4
 *   k2_residue_gemm<4, 4, 2, false> grid=6400 xgroup=1
 *   k3_inverse_crt<4, 2, false, true> grid=784x1
 *   conversion=unreduced-binary32
 * conversion: "unreduced-binary32" / "unreduced-binary64" = CRT sum over unreduced accumulators with the quotient rounded
 * in that precision; "reduced-binary32" / "reduced-binary64" = over reduced residues; "reduced-binary64-mul32" = the same
 * with full 32-bit multiplies (a partial product P/m_i of 2^24 or more).  Works on host-only plans (grids of the
 * streaming inverse transform then assume 256 compute units).  Returns the number of bytes including the terminating
 * zero (copied only if capacity suffices), or a negative code.  For tests and measurement scripts.
 */
int64_t rnswino_plan_describe(const rnswino_plan_t *plan, int32_t output_mode, char *host_out, size_t capacity);

/* Launches a kernel that does nothing on grid_x x grid_y workgroups of 256 threads, between two optional caller-created
 * hipEvent_t (passed as void*, may be NULL) that receive its start and stop timestamps.  Chains of such launches measure what a
 * stage's launch costs with no work in it (dispatch, ramp-up, completion).  For measurement (the time breakdown of section 8). */
int rnswino_debug_empty_launch(uint32_t grid_x, uint32_t grid_y, void *stream, void *start_event, void *stop_event);

/* Every kernel instantiation of the three hot stages the library can launch, one name per line in the form of
 * rnswino_plan_describe (host memory; same return convention).  The tests use it to check that each is exercised. */
int64_t rnswino_kernel_variants(char *host_out, size_t capacity);

/* (prod m_i - 1)/2 saturated to 2^63-1: the largest magnitude the plan's RNS represents. */
int64_t rnswino_plan_dynamic_range(const rnswino_plan_t *plan);

/*
 * Copy an intermediate tensor to HOST memory as int32 canonical residues in [-(p-1)/2, (p-1)/2], in the
 * plain index order of section 6 (synchronises the device; test use only):
 *   RNSWINO_STAGE_U: src_dev = U_dev,         host_out [n][t*t][K][C]
 *   RNSWINO_STAGE_V: src_dev = workspace_dev, host_out [n][t*t][T][C],  T = N * ceil(Ho/m) * ceil(Wo/m)
 *   RNSWINO_STAGE_O: src_dev = workspace_dev, host_out [n][t*t][K][T]
 * Tile index tau = (n * th + ty) * tw + tx.
 */
int rnswino_debug_stage(const rnswino_plan_t *plan, int stage, const void *src_dev, int32_t *host_out);

const char *rnswino_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* RNSWINO_H */
