/*
 * binomial3x3_f32 -- 3x3 binomial filter of an fp32 image on one AMD MI355X (gfx950).
 *
 * The second workload of the paper (Section 2.1, the figure with the two Halide forms; Section 5,
 * the RISE form bf = pad2D(1) |> slide2D(3)(1) |> map2D(dot with the 3x3 weights)):
 *     out(x,y) = ( 1*in(x-1,y-1) + 2*in(x,y-1) + 1*in(x+1,y-1)
 *                + 2*in(x-1,y)   + 4*in(x,y)   + 2*in(x+1,y)
 *                + 1*in(x-1,y+1) + 2*in(x,y+1) + 1*in(x+1,y+1) ) * (1/16),
 * with the input extended by repeating its edge pixels.  The kernel evaluates the separated,
 * scanline form (horizontal 1-2-1 per row, rows combined 1-2-1; Section 5.1/5.2), which is the
 * same value up to fp32 rounding order.
 *
 *   in, out   DEVICE pointers owned by the caller; row-major, pixel (y,x) at p[y*ld + x],
 *             ld_in >= max(W,1), ld_out >= max(W,1).  out must not overlap in
 *             (same pointer: GEMMF32_EALIAS; partial overlap is undefined).
 *   Pixels outside [0,H) x [0,W) of out (the ld padding) are never written.
 *   H == 0 or W == 0: success, nothing launched.
 *   Asynchronous on the stream the calling host thread gave to binomial3x3_f32_set_stream (default: null stream).
 *   Returns 0 or a negative gemmf32_status (see gemm_f32.h); nothing is launched on error.
 */
#ifndef BINOMIAL_F32_H
#define BINOMIAL_F32_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int binomial3x3_f32(int64_t H, int64_t W, const float *in, int64_t ld_in, float *out, int64_t ld_out);

/*
 * The same filter in the three forms the paper contrasts (Section 2.1: the two Halide programs;
 * Section 5.1: the scanline form), kept so that they can be measured side by side:
 *   0 "naive"      one thread per pixel, nine taps from the image;
 *   1 "separated"  horizontal 1-2-1 pass into tmp, vertical 1-2-1 pass from tmp (tmp: DEVICE
 *                  buffer of the caller, H rows of ld_tmp >= W floats, overwritten; must not be
 *                  in or out);
 *   2 "scanline"   binomial3x3_f32 above (tmp unused, may be NULL).
 * All three compute the same value up to fp32 rounding order and are exact for images of small
 * integers.  Variants 0 and 1 are limited to H <= 65535 (separated) / H <= 262140 (naive):
 * larger images return GEMMF32_EINVAL.  Other arguments and errors as binomial3x3_f32.
 */
int binomial3x3_f32_variant(int variant, int64_t H, int64_t W, const float *in, int64_t ld_in, float *out,
                            int64_t ld_out, float *tmp, int64_t ld_tmp);
int binomial3x3_f32_variants(void);
const char *binomial3x3_f32_variant_name(int variant);   /* "?" if out of range */

/* Stream for later launches (hipStream_t as void*; NULL = null stream). */
int binomial3x3_f32_set_stream(void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* BINOMIAL_F32_H */
