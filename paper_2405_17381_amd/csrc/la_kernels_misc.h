// Small kernels around the block scan: the scan over segment states and the
// single-token decode step.  Both are plain fp32 and memory-bound.
#pragma once
#include "la_common.h"

// In-place exclusive scan of the segment states of each (batch, head):
// forward  P_0 = 0, P_{s+1} = lambda^L P_s + S_s     (App. C, KV_t at segment granularity)
// reverse  D_{S-1} = 0, D_{s-1} = lambda^L D_s + S_s (App. C, dKV_t likewise)
// One thread carries four adjacent state entries through the segments; the
// loads of a batch of eight segments are issued together (they do not depend
// on the carry), only the stores follow the recurrence.
template <bool REV>
__device__ __forceinline__ void segment_scan_body(const SegScanArgs &a, const LaLambdas &lams)
{
    const int scan = blockIdx.y;
    const int e = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= a.DD) return;
    const float lam = lams.v[scan % a.H];
    float *W = a.states + (size_t)scan * a.S * a.DD + e;
    // chain-free heads (see la_entering_state) read their neighbour's local state directly;
    // only a carried-in state is placed, in the slot no local state uses
    if (a.skip_bits > 0.f && -lams.lg2[scan % a.H] * (float)a.L >= a.skip_bits) {
        if (!REV && a.init)
            *(float4 *)(W + (size_t)(a.S - 1) * a.DD) = *(const float4 *)(a.init + (size_t)scan * a.DD + e);
        return;
    }
    const float lamL = (float)pow((double)lam, (double)a.L);
    float4 carry = make_float4(0.f, 0.f, 0.f, 0.f);
    if (!REV && a.init) carry = *(const float4 *)(a.init + (size_t)scan * a.DD + e);
    for (int i0 = 0; i0 < a.S; i0 += 8) {
        float4 loc[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u;
            const int s = REV ? (a.S - 1 - i) : i;
            // the final segment's own local state was not produced and is not needed
            loc[u] = (i < a.S - 1) ? *(const float4 *)(W + (size_t)s * a.DD) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u;
            if (i < a.S) {
                const int s = REV ? (a.S - 1 - i) : i;
                *(float4 *)(W + (size_t)s * a.DD) = carry;
                carry.x = fmaf(lamL, carry.x, loc[u].x);
                carry.y = fmaf(lamL, carry.y, loc[u].y);
                carry.z = fmaf(lamL, carry.z, loc[u].z);
                carry.w = fmaf(lamL, carry.w, loc[u].w);
            }
        }
    }
}

template <bool REV>
__global__ __launch_bounds__(256) void la_segment_scan(SegScanArgs a, LaLambdas lams)
{
    segment_scan_body<REV>(a, lams);
}

// The backward pass's two segment scans (forward states of one scan, reverse states
// of another) in one launch: blockIdx.z selects.
__global__ __launch_bounds__(256) void la_segment_scan_pair(SegScanArgs fwd, SegScanArgs rev, LaLambdas lams)
{
    if (blockIdx.z == 0) segment_scan_body<false>(fwd, lams);
    else segment_scan_body<true>(rev, lams);
}

// One token of the recurrence for every (batch, head) (App. A, recurrence form):
//     kv <- lambda kv + k v^T ,  o = q^T kv
// kv: [scans, D, D] fp32, updated in place; q, k, v, o: [scans, D] in T (fp32 or
// bf16 stored as uint16).  One workgroup per scan; HBM-bound on the 2 x 4 D^2
// bytes of state it streams.  Thread layout: D/4 threads cover a state row with
// 16-byte accesses, 1024/D row groups stride the rows; per-column partial sums
// of q^T kv are combined through LDS in a fixed order (deterministic).
template <int D, bool BF16>
__global__ __launch_bounds__(256) void la_decode_kernel(const void *q_, const void *k_, const void *v_,
                                                        float *kv, void *o_, int H, LaLambdas lams)
{
    constexpr int TPR = D / 4;            // threads per state row
    constexpr int RG = 256 / TPR;         // row groups
    __shared__ float sq[D], sk[D], sv[D];
    __shared__ float part[RG][D];
    const int scan = blockIdx.x, tid = threadIdx.x;
    const float lam = lams.v[scan % H];
    auto ld = [&](const void *p, int i) -> float {
        if (BF16) return __uint_as_float((uint32_t)((const uint16_t *)p)[(size_t)scan * D + i] << 16);
        return ((const float *)p)[(size_t)scan * D + i];
    };
    if (tid < D) { sq[tid] = ld(q_, tid); sk[tid] = ld(k_, tid); sv[tid] = ld(v_, tid); }
    __syncthreads();
    const int j4 = (tid % TPR) * 4, rg = tid / TPR;
    float *base = kv + (size_t)scan * D * D;
    const float4 vv = make_float4(sv[j4], sv[j4 + 1], sv[j4 + 2], sv[j4 + 3]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int i = rg; i < D; i += RG) {
        float4 x = *(const float4 *)(base + (size_t)i * D + j4);
        const float ki = sk[i], qi = sq[i];
        x.x = fmaf(lam, x.x, ki * vv.x); x.y = fmaf(lam, x.y, ki * vv.y);
        x.z = fmaf(lam, x.z, ki * vv.z); x.w = fmaf(lam, x.w, ki * vv.w);
        *(float4 *)(base + (size_t)i * D + j4) = x;
        acc.x = fmaf(qi, x.x, acc.x); acc.y = fmaf(qi, x.y, acc.y);
        acc.z = fmaf(qi, x.z, acc.z); acc.w = fmaf(qi, x.w, acc.w);
    }
    part[rg][j4] = acc.x; part[rg][j4 + 1] = acc.y; part[rg][j4 + 2] = acc.z; part[rg][j4 + 3] = acc.w;
    __syncthreads();
    if (tid < D) {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < RG; ++r) s += part[r][tid];
        if (BF16) {
            uint32_t u = __float_as_uint(s);
            u += 0x7fffu + ((u >> 16) & 1u);            // round to nearest even
            if (s != s) u = 0x7fc00000u;                // NaN stays a (quiet) NaN whatever its payload
            ((uint16_t *)o_)[(size_t)scan * D + tid] = (uint16_t)(u >> 16);
        } else {
            ((float *)o_)[(size_t)scan * D + tid] = s;
        }
    }
}

// Measurement aid (reached only through la_debug_mfma_rate): what the matrix cores deliver
// on v_mfma_f32_32x32x16_bf16 when nothing else is in the way.  Every wave keeps four
// independent accumulator tiles busy from registers only; the result is stored only if it
// equals a value it cannot take, so that the loop survives and no memory traffic happens.
typedef __bf16 misc_bf16x8_t __attribute__((ext_vector_type(8)));
typedef float misc_f32x16_t __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void la_mfma_rate_kernel(float *sink, int iters)
{
    misc_f32x16_t acc[4];
    misc_bf16x8_t a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(float)((threadIdx.x + e) & 3);
        b[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 1);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float sum = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += acc[j][v];
    if (sum == -1.0f) sink[0] = sum;          // never true: the sums are non-negative
}
