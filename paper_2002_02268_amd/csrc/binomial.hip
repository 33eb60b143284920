// 3x3 binomial filter (weights 1-2-1 x 1-2-1, /16, repeat-edge) for gfx950.
//
// Bound by HBM: 4 bytes read and 4 written per pixel, 17 flops.  Each thread owns 4 adjacent
// columns and walks a band of rows downwards (the "scanline" form of Section 5.1 of the paper): per
// input row it forms the horizontal 1-2-1 sums of its 4 columns (one 16-byte load plus the two
// neighbouring pixels, which hit the cache lines its neighbours load), keeps the sums of three
// consecutive rows in registers and combines them 1-2-1.  A band re-reads
// only its two halo rows.
#include "../../include/binomial_f32.h"
#include "../../include/gemm_f32.h"

#include <hip/hip_runtime.h>

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef v4f v4f_g __attribute__((aligned(4)));   // 16-byte access to 4-byte-aligned global memory

thread_local hipStream_t g_stream = nullptr;   // per host thread

struct Args {
    const float *in;
    float *out;
    int H, W;
    int rows;            // output rows per thread (a band re-reads its two halo rows)
    int64_t ld_in, ld_out;
};

// horizontal 1-2-1 sums of columns x0..x0+3 of row y (y already clamped), edges repeated
__device__ __forceinline__ v4f hsum(const Args &p, int y, int x0)
{
    const float *row = p.in + (int64_t)y * p.ld_in;
    const int W = p.W;
    v4f v;
    if (x0 + 3 < W) {
        v = *reinterpret_cast<const v4f_g *>(row + x0);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = row[(x0 + j < W) ? x0 + j : W - 1];
    }
    const float left = row[x0 > 0 ? x0 - 1 : 0];
    const float right = row[(x0 + 4 < W) ? x0 + 4 : W - 1];
    v4f h;
    h[0] = left + 2.f * v[0] + v[1];
    h[1] = v[0] + 2.f * v[1] + v[2];
    h[2] = v[1] + 2.f * v[2] + v[3];
    h[3] = v[2] + 2.f * v[3] + right;
    return h;
}

__global__ void __launch_bounds__(256) binomial3x3_kernel(const Args p)
{
    const int x0 = 4 * (blockIdx.x * 256 + threadIdx.x);
    if (x0 >= p.W) return;
    const int y0 = blockIdx.y * p.rows;
    const int y1 = (y0 + p.rows < p.H) ? y0 + p.rows : p.H;
    v4f prev = hsum(p, y0 > 0 ? y0 - 1 : 0, x0);
    v4f cur = hsum(p, y0, x0);
    // four rows per step: their loads are all issued before the first result is formed
    for (int y = y0; y < y1; y += 4) {
        v4f next[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) next[r] = hsum(p, (y + r + 1 < p.H) ? y + r + 1 : p.H - 1, x0);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (y + r < y1) {
                const v4f o = (prev + 2.f * cur + next[r]) * 0.0625f;
                float *dst = p.out + (int64_t)(y + r) * p.ld_out + x0;
                if (x0 + 3 < p.W) {
                    *reinterpret_cast<v4f_g *>(dst) = o;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (x0 + j < p.W) dst[j] = o[j];
                }
            }
            prev = cur;
            cur = next[r];
        }
    }
}

// ---- the two plainer forms of the same filter, kept to be measured beside the scanline kernel ----

// Direct form: one thread per output pixel, the nine taps read straight from the image
// (the first of the two Halide forms in Section 2.1).
__global__ void __launch_bounds__(256) binomial3x3_naive_kernel(const Args p)
{
    const int x = blockIdx.x * 64 + (threadIdx.x & 63);
    const int y = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (x >= p.W || y >= p.H) return;
    const int xl = x > 0 ? x - 1 : 0, xr = x + 1 < p.W ? x + 1 : p.W - 1;
    const float *r0 = p.in + (int64_t)(y > 0 ? y - 1 : 0) * p.ld_in;
    const float *r1 = p.in + (int64_t)y * p.ld_in;
    const float *r2 = p.in + (int64_t)(y + 1 < p.H ? y + 1 : p.H - 1) * p.ld_in;
    const float s = 1.f * r0[xl] + 2.f * r0[x] + 1.f * r0[xr]
                  + 2.f * r1[xl] + 4.f * r1[x] + 2.f * r1[xr]
                  + 1.f * r2[xl] + 2.f * r2[x] + 1.f * r2[xr];
    p.out[(int64_t)y * p.ld_out + x] = s * 0.0625f;
}

// Separated form with the intermediate image materialised (the second Halide form of Section 2.1
// with its first stage computed in full before the second): a horizontal 1-2-1 pass into tmp,
// then a vertical 1-2-1 pass over tmp.  Twice the memory traffic of the scanline kernel.
__global__ void __launch_bounds__(256) binomial_rows_kernel(const Args p)    // in -> out, horizontal, unscaled
{
    const int x = blockIdx.x * 256 + threadIdx.x;
    const int y = blockIdx.y;
    if (x >= p.W) return;
    const float *row = p.in + (int64_t)y * p.ld_in;
    p.out[(int64_t)y * p.ld_out + x] = row[x > 0 ? x - 1 : 0] + 2.f * row[x] + row[x + 1 < p.W ? x + 1 : p.W - 1];
}
__global__ void __launch_bounds__(256) binomial_cols_kernel(const Args p)    // in -> out, vertical, scaled by 1/16
{
    const int x = blockIdx.x * 256 + threadIdx.x;
    const int y = blockIdx.y;
    if (x >= p.W) return;
    const float a = p.in[(int64_t)(y > 0 ? y - 1 : 0) * p.ld_in + x];
    const float b = p.in[(int64_t)y * p.ld_in + x];
    const float c = p.in[(int64_t)(y + 1 < p.H ? y + 1 : p.H - 1) * p.ld_in + x];
    p.out[(int64_t)y * p.ld_out + x] = (a + 2.f * b + c) * 0.0625f;
}

int check_image_args(int64_t H, int64_t W, const float *in, int64_t ld_in, float *out, int64_t ld_out)
{
    if (H < 0 || W < 0 || H > 2147483647LL || W > 2147483647LL) return GEMMF32_EINVAL;
    if (ld_in < (W > 1 ? W : 1) || ld_out < (W > 1 ? W : 1)) return GEMMF32_EINVAL;
    if (H == 0 || W == 0) return 1;      // nothing to do
    if (in == nullptr || out == nullptr) return GEMMF32_ENULL;
    if (in == out) return GEMMF32_EALIAS;
    return GEMMF32_OK;
}

}  // namespace

extern "C" {

int binomial3x3_f32_variants(void) { return 3; }

const char *binomial3x3_f32_variant_name(int variant)
{
    static const char *names[] = {"naive", "separated", "scanline"};
    return (variant >= 0 && variant < 3) ? names[variant] : "?";
}

int binomial3x3_f32_variant(int variant, int64_t H, int64_t W, const float *in, int64_t ld_in, float *out,
                            int64_t ld_out, float *tmp, int64_t ld_tmp)
{
    if (variant < 0 || variant >= 3) return GEMMF32_EINVAL;
    if (variant == 2) return binomial3x3_f32(H, W, in, ld_in, out, ld_out);
    const int st = check_image_args(H, W, in, ld_in, out, ld_out);
    if (st != GEMMF32_OK) return st > 0 ? GEMMF32_OK : st;
    Args a;
    a.in = in; a.out = out; a.H = (int)H; a.W = (int)W; a.rows = 1; a.ld_in = ld_in; a.ld_out = ld_out;
    if (variant == 0) {
        // grid.y is limited to 65535: taller images would need a loop; they are refused instead
        if ((H + 3) / 4 > 65535) return GEMMF32_EINVAL;
        hipLaunchKernelGGL(binomial3x3_naive_kernel, dim3((unsigned)((W + 63) / 64), (unsigned)((H + 3) / 4)),
                           dim3(256), 0, g_stream, a);
    } else {
        if (tmp == nullptr) return GEMMF32_ENULL;
        if (ld_tmp < W) return GEMMF32_EINVAL;
        if (tmp == in || tmp == out) return GEMMF32_EALIAS;
        if (H > 65535) return GEMMF32_EINVAL;
        Args h = a, v = a;
        h.out = tmp; h.ld_out = ld_tmp;
        v.in = tmp; v.ld_in = ld_tmp;
        const dim3 grid((unsigned)((W + 255) / 256), (unsigned)H);
        hipLaunchKernelGGL(binomial_rows_kernel, grid, dim3(256), 0, g_stream, h);
        hipLaunchKernelGGL(binomial_cols_kernel, grid, dim3(256), 0, g_stream, v);
    }
    return hipGetLastError() == hipSuccess ? GEMMF32_OK : GEMMF32_ELAUNCH;
}

int binomial3x3_f32_set_stream(void *hip_stream)
{
    g_stream = reinterpret_cast<hipStream_t>(hip_stream);
    return GEMMF32_OK;
}

int binomial3x3_f32(int64_t H, int64_t W, const float *in, int64_t ld_in, float *out, int64_t ld_out)
{
    if (H < 0 || W < 0 || H > 2147483647LL || W > 2147483647LL) return GEMMF32_EINVAL;
    if (ld_in < (W > 1 ? W : 1) || ld_out < (W > 1 ? W : 1)) return GEMMF32_EINVAL;
    if (H == 0 || W == 0) return GEMMF32_OK;
    if (in == nullptr || out == nullptr) return GEMMF32_ENULL;
    if (in == out) return GEMMF32_EALIAS;
    // rows per thread: as many as possible (fewer halo re-reads) while the image still gives every
    // compute unit about 16 waves to hide memory latency with
    // Images that do not fit the 256 MB memory-side cache stream from HBM: short bands keep the rows
    // that are in flight at one time close together (measured: 103 instead of 115 us at 8192 x 8192).
    int rows = (8 * H * W > (256LL << 20)) ? 8 : 32;
    while (rows > 8 && (W + 3) / 4 * ((H + rows - 1) / rows) < 256 * 16 * 64) rows /= 2;
    const int64_t gx = (W + 1023) / 1024;
    int64_t gy = (H + rows - 1) / rows;
    while (gy > 65535) { rows *= 2; gy = (H + rows - 1) / rows; }
    Args a;
    a.in = in; a.out = out; a.H = (int)H; a.W = (int)W; a.rows = rows; a.ld_in = ld_in; a.ld_out = ld_out;
    hipLaunchKernelGGL(binomial3x3_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, g_stream, a);
    return hipGetLastError() == hipSuccess ? GEMMF32_OK : GEMMF32_ELAUNCH;
}

}  // extern "C"
