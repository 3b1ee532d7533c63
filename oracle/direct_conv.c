/*
 * CPU oracle: the plain definition of the integer convolution the method
 * reproduces exactly.  TEST INFRASTRUCTURE ONLY -- nothing in the product
 * library links, includes or calls this file, and it shares no code with it.
 *
 * The paper states that its RNS-Winograd scheme yields the precise integer
 * result of the quantised layer (abstract; conclusions), so the reference is
 * the definition itself:
 *   - orientation: correlation, y_k = sum_j d_{k+j} g_j, no filter flip
 *     (section 3.1, the subsection on convolution in the RNS);
 *   - layer shape: K filters of r x r x C applied to a batch of C-channel
 *     planes, summed over the depth C (section 6, first paragraph);
 *   - stride 1 (strided layers are excluded in the paper's Table 5 footnote);
 *   - zero padding of `pad` pixels on every side.
 * Layout: x int8 [N][C][H][W], w int8 [K][C][r][r], y int32 [N][K][Ho][Wo],
 * Ho = H + 2 pad - r + 1, Wo = W + 2 pad - r + 1.  |y| <= 2^14 r^2 C, so a
 * 32-bit accumulator cannot overflow for any shape the library accepts.
 *
 * Deliberately the seven nested loops, nothing blocked or reordered.
 */
#include <stdint.h>
#include <stddef.h>

void oracle_direct_conv2d(const int8_t *x, const int8_t *w, int32_t *y,
                          int N, int C, int K, int H, int W, int r, int pad)
{
    const int Ho = H + 2 * pad - r + 1;
    const int Wo = W + 2 * pad - r + 1;
    if (Ho <= 0 || Wo <= 0) return;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            for (int oy = 0; oy < Ho; ++oy) {
                for (int ox = 0; ox < Wo; ++ox) {
                    int32_t acc = 0;
                    for (int c = 0; c < C; ++c) {
                        for (int i = 0; i < r; ++i) {
                            const int iy = oy + i - pad;
                            if (iy < 0 || iy >= H) continue;
                            for (int j = 0; j < r; ++j) {
                                const int ix = ox + j - pad;
                                if (ix < 0 || ix >= W) continue;
                                const int32_t xv = x[(((size_t)n * C + c) * H + iy) * W + ix];
                                const int32_t wv = w[(((size_t)k * C + c) * r + i) * r + j];
                                acc += xv * wv;
                            }
                        }
                    }
                    y[(((size_t)n * K + k) * Ho + oy) * Wo + ox] = acc;
                }
            }
        }
    }
}

/*
 * Glue between layers of the 13-layer stack workload.  None of it is in the
 * paper (which measures each layer on its own); it is the fixed, integer-only
 * re-quantisation the workload description asks for:
 *   a = clamp(y >> shift, -128, 127)   with an arithmetic (floor) shift,
 * and a 2x2, stride-2 max-pool on the int8 result (H and W even).
 */
void oracle_requant_shift_clamp(const int32_t *y, int8_t *a, size_t count, int shift)
{
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < count; ++e) {
        const int64_t v = y[e];
        const int64_t d = (int64_t)1 << shift;      /* shift 0..31: 64-bit, so that 2^31 is representable */
        /* floor division by 2^shift, written without relying on >> of negatives */
        int64_t q = v >= 0 ? v / d : -((-v + d - 1) / d);
        if (q < -128) q = -128;
        if (q > 127) q = 127;
        a[e] = (int8_t)q;
    }
}

void oracle_maxpool2x2(const int8_t *a, int8_t *b, int planes, int H, int W)
{
    const int Hp = H / 2, Wp = W / 2;
#pragma omp parallel for schedule(static)
    for (int p = 0; p < planes; ++p)
        for (int yy = 0; yy < Hp; ++yy)
            for (int xx = 0; xx < Wp; ++xx) {
                int8_t best = -128;
                for (int dy = 0; dy < 2; ++dy)
                    for (int dx = 0; dx < 2; ++dx) {
                        int8_t v = a[((size_t)p * H + 2 * yy + dy) * W + 2 * xx + dx];
                        if (v > best) best = v;
                    }
                b[((size_t)p * Hp + yy) * Wp + xx] = best;
            }
}
