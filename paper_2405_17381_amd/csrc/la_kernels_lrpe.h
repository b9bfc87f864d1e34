// LRPE-d rotation (Sec. 4.1, "Position Encoding"): the relative phase exp(i theta (t - s))
// of the attention score is split between query and key by giving every row the cos / sin
// features
//     Xw[t] = [ x_t cos(t theta) , x_t sin(t theta) ]            (theta: one angle per head and feature)
// so that the plain inner product Qw[t] . Kw[s] = sum_i q_ti k_si cos(theta_i (t - s)); the wide
// attention entry points then run on Qw, Kw.  Backward of the rotation:
//     dX[t] = dXw_c[t] cos(t theta) + dXw_s[t] sin(t theta)
//     dtheta_i = sum_{b,t} t x_ti (dXw_s[t,i] cos(t theta_i) - dXw_c[t,i] sin(t theta_i)).
// Memory-bound elementwise kernels.  The angle t * theta is reduced exactly: theta / 2 pi is
// taken once per thread in fp64, t * (theta / 2 pi) and its fractional part in fp64 per row,
// and the hardware sin / cos (which take revolutions) see a fraction in [0, 1).
// One thread holds 8 features of a row; D/8 lanes cover a row, 2048/D rows per pass of a
// workgroup, LRPE_ROWS rows per workgroup.  The theta gradient is reduced without atomics:
// per-thread sums over the workgroup's rows, a fixed-order LDS reduction over its row groups,
// one partial per (batch, head, row tile) in the caller's scratch, then a second kernel that
// sums the partials of each (head, feature) in a fixed order in fp64.
#pragma once
#include "la_common.h"

constexpr int LRPE_ROWS = 128;      // rows per workgroup

struct LrpeArgs {
    const void *X;        // [B, H, n, D]
    const float *theta;   // [H, D] (device)
    void *Xw;             // forward: output [B, H, n, 2D]; backward: input dXw
    void *dX;             // backward: output [B, H, n, D]
    float *partial;       // backward: [B, H, tiles, D] fp32 partial theta gradients
    int H, n, tiles;
};

template <bool BF16>
__device__ __forceinline__ void lrpe_load8(const void *p, size_t idx, float (&x)[8])
{
    if (BF16) {
        const uint4 r = *(const uint4 *)((const uint16_t *)p + idx);
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    } else {
        const float4 a = *(const float4 *)((const float *)p + idx);
        const float4 b = *(const float4 *)((const float *)p + idx + 4);
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
}

__device__ __forceinline__ uint32_t lrpe_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if (f != f) return 0x7fc0u;                 // NaN stays a (quiet) NaN whatever its payload
    u += 0x7fffu + ((u >> 16) & 1u);            // round to nearest even; overflow gives inf
    return u >> 16;
}

template <bool BF16>
__device__ __forceinline__ void lrpe_store8(void *p, size_t idx, const float (&x)[8])
{
    if (BF16) {
        uint4 r;
        r.x = lrpe_bf16_rne(x[0]) | (lrpe_bf16_rne(x[1]) << 16);
        r.y = lrpe_bf16_rne(x[2]) | (lrpe_bf16_rne(x[3]) << 16);
        r.z = lrpe_bf16_rne(x[4]) | (lrpe_bf16_rne(x[5]) << 16);
        r.w = lrpe_bf16_rne(x[6]) | (lrpe_bf16_rne(x[7]) << 16);
        *(uint4 *)((uint16_t *)p + idx) = r;
    } else {
        *(float4 *)((float *)p + idx) = make_float4(x[0], x[1], x[2], x[3]);
        *(float4 *)((float *)p + idx + 4) = make_float4(x[4], x[5], x[6], x[7]);
    }
}

// cos and sin of t * theta, theta given as revolutions u = theta / 2 pi (fp64)
__device__ __forceinline__ void lrpe_cos_sin(double u, int t, float &c, float &s)
{
    const double rev = (double)t * u;
    const float f = (float)(rev - floor(rev));          // exact range reduction, [0, 1]
    c = __builtin_amdgcn_cosf(f);
    s = __builtin_amdgcn_sinf(f);
}

template <int D, bool BF16, bool BWD>
__global__ __launch_bounds__(256) void la_lrpe_rotate_kernel(LrpeArgs a)
{
    constexpr int CHK = D / 8;                 // lanes per row
    constexpr int RPP = 256 / CHK;             // rows per pass
    __shared__ float red[BWD ? RPP : 1][BWD ? D : 1];

    const int tid = threadIdx.x;
    const int ch = tid % CHK, rl = tid / CHK;
    const int tile = blockIdx.x;
    const int scan = blockIdx.y;               // b * H + h
    const int h = scan % a.H;

    double u[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) u[i] = (double)a.theta[h * D + 8 * ch + i] * 0.15915494309189533577;

    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const int t_end = min(a.n, (tile + 1) * LRPE_ROWS);
    for (int t = tile * LRPE_ROWS + rl; t < t_end; t += RPP) {
        const size_t row = (size_t)scan * a.n + t;
        float x[8], c[8], s[8];
        lrpe_load8<BF16>(a.X, row * D + 8 * ch, x);
#pragma unroll
        for (int i = 0; i < 8; ++i) lrpe_cos_sin(u[i], t, c[i], s[i]);
        if (!BWD) {
            float yc[8], ys[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) { yc[i] = x[i] * c[i]; ys[i] = x[i] * s[i]; }
            lrpe_store8<BF16>(a.Xw, row * (2 * D) + 8 * ch, yc);
            lrpe_store8<BF16>(a.Xw, row * (2 * D) + D + 8 * ch, ys);
        } else {
            float gc[8], gs[8], dx[8];
            lrpe_load8<BF16>(a.Xw, row * (2 * D) + 8 * ch, gc);
            lrpe_load8<BF16>(a.Xw, row * (2 * D) + D + 8 * ch, gs);
            const float tf = (float)t;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                dx[i] = fmaf(gc[i], c[i], gs[i] * s[i]);
                acc[i] = fmaf(tf * x[i], fmaf(gs[i], c[i], -gc[i] * s[i]), acc[i]);
            }
            lrpe_store8<BF16>(a.dX, row * D + 8 * ch, dx);
        }
    }
    if (BWD) {
#pragma unroll
        for (int i = 0; i < 8; ++i) red[rl][8 * ch + i] = acc[i];
        __syncthreads();
        if (tid < D) {
            float sum = 0.f;
            for (int r = 0; r < RPP; ++r) sum += red[r][tid];
            a.partial[((size_t)scan * a.tiles + tile) * D + tid] = sum;
        }
    }
}

// dtheta[h, i] = (accumulate ? dtheta[h, i] : 0) + sum over b and tiles of the partials, in fp64
// and in a fixed order: 8 threads per (head, feature) each add every 8th partial, then one of
// them adds the 8 sums.  A workgroup covers 32 consecutive (head, feature) entries.
__global__ __launch_bounds__(256) void la_lrpe_theta_reduce(const float *partial, float *dtheta, int B, int H,
                                                            int tiles, int D, int accumulate)
{
    __shared__ double red[8][32];
    const int lane = threadIdx.x % 32, slice = threadIdx.x / 32;
    const int e = blockIdx.x * 32 + lane;              // h * D + i  (H * D is a multiple of 32)
    const int h = e / D, i = e % D;
    const int count = B * tiles;
    double sum = 0.0;
    for (int idx0 = slice; idx0 < count; idx0 += 64) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {                  // eight loads in flight
            const int idx = idx0 + 8 * j;
            const int b = idx / tiles, k = idx % tiles;
            v[j] = idx < count ? partial[(((size_t)b * H + h) * tiles + k) * D + i] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) sum += (double)v[j];
    }
    red[slice][lane] = sum;
    __syncthreads();
    if (slice == 0) {
        double total = accumulate ? (double)dtheta[e] : 0.0;
        for (int r = 0; r < 8; ++r) total += red[r][lane];
        dtheta[e] = (float)total;
    }
}
