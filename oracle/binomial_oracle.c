/*
 * CPU oracle for the 3x3 binomial filter -- TEST INFRASTRUCTURE ONLY (never called by the GPU
 * library; shares no code with it).
 *
 * Definition: the two-dimensional binomial filter of the paper's Section 2.1 (the figure with
 * the Halide form) and Section 5 (the RISE form: pad2D(1), slide2D(3)(1), dot with the 3x3
 * weights): every output pixel is the weighted sum of its 3x3 neighbourhood with weights
 *     1 2 1
 *     2 4 2    times 1/16,
 *     1 2 1
 * and the input is extended by repeating its edge pixels (repeat_edge / pad).
 * Arithmetic: fp32 input widened to fp64, nine exact products, fp64 sum in the order the figure
 * lists the taps (row above, row, row below; left to right), one multiplication by 1/16 (exact).
 *
 * Layout: row-major, element (y, x) at in[y*ld_in + x]; out likewise with ld_out; ld >= W.
 * Pinned by tests: constant and linear images, impulse response, separability restated through a
 * library padding routine, exact integer images, transpose symmetry, a hand-computed 3x3 case.
 */
#include <stdint.h>
#include <stddef.h>

static int64_t clampi(int64_t v, int64_t lo, int64_t hi) { return v < lo ? lo : (v > hi ? hi : v); }

int oracle_binomial3x3_f32(int64_t H, int64_t W, const float *in, int64_t ld_in, double *out, int64_t ld_out)
{
    if (H < 0 || W < 0) return -1;
    if (ld_in < (W > 1 ? W : 1) || ld_out < (W > 1 ? W : 1)) return -1;
    if (H > 0 && W > 0 && (in == NULL || out == NULL)) return -1;
    static const double w[3][3] = {{1.0, 2.0, 1.0}, {2.0, 4.0, 2.0}, {1.0, 2.0, 1.0}};
    for (int64_t y = 0; y < H; ++y)
        for (int64_t x = 0; x < W; ++x) {
            double acc = 0.0;
            for (int dy = -1; dy <= 1; ++dy)
                for (int dx = -1; dx <= 1; ++dx) {
                    const int64_t yy = clampi(y + dy, 0, H - 1), xx = clampi(x + dx, 0, W - 1);
                    acc += w[dy + 1][dx + 1] * (double)in[yy * ld_in + xx];
                }
            out[y * ld_out + x] = acc * (1.0 / 16.0);
        }
    return 0;
}
