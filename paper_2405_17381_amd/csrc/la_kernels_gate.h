// Gated, normalised output stage of the attention block (Sec. 4.2):
//     Y = SRMSNorm(O) * U ,  SRMSNorm(x) = x / (||x||_2 / sqrt(H d))  per token,
// the norm running over all H*d features of a token (heads concatenated), and
// its backward.  Tensors are [B, H, n, d] like the attention's own.
//
// Memory-bound.  One workgroup takes TT = 8 tokens of one batch element and all
// heads.  Pass 1 streams O (backward: O, U, dY) once and reduces per token;
// pass 2 re-reads the same 8-token tiles, which are still in L2, and writes the
// result, so HBM sees each tensor once; on the bf16 path the first KC = 8 head
// steps (all of them up to H = 16 at d = 128) do not even go back to L2: pass 1
// keeps their 16-byte loads in registers.  Threads: d/8 lanes cover a row with
// 16-byte (bf16) or 32-byte (fp32) accesses, 8 tokens, 256/(d) heads per step.
// The per-token sums are combined through LDS in a fixed order (deterministic).
#pragma once
#include "la_common.h"

struct GateArgs {
    const void *O, *U, *dY;     // dY: backward only
    void *Y, *dO, *dU;          // Y: forward only; dO, dU: backward only
    int H, n;
    float eps;
};

typedef uint32_t gate_u32x4 __attribute__((ext_vector_type(4)));

// one 8-element chunk as loaded: 16 bytes (bf16) or 32 bytes (fp32)
template <bool BF16>
struct GateRaw {
    uint4 lo, hi;       // bf16 uses lo only
};

// NT: the chunk is read once and kept in registers (non-temporal hint)
template <bool BF16, bool NT = false>
__device__ __forceinline__ GateRaw<BF16> gate_fetch(const void *p, size_t idx)
{
    GateRaw<BF16> r;
    if (BF16 && NT) {
        const gate_u32x4 v = __builtin_nontemporal_load((const gate_u32x4 *)((const uint16_t *)p + idx));
        r.lo = make_uint4(v[0], v[1], v[2], v[3]);
    } else if (BF16) {
        r.lo = *(const uint4 *)((const uint16_t *)p + idx);
    } else {
        r.lo = *(const uint4 *)((const float *)p + idx);
        r.hi = *(const uint4 *)((const float *)p + idx + 4);
    }
    return r;
}

template <bool BF16>
__device__ __forceinline__ void gate_unpack(const GateRaw<BF16> &r, float (&x)[8])
{
    if (BF16) {
        const uint32_t w[4] = {r.lo.x, r.lo.y, r.lo.z, r.lo.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    } else {
        x[0] = __uint_as_float(r.lo.x); x[1] = __uint_as_float(r.lo.y);
        x[2] = __uint_as_float(r.lo.z); x[3] = __uint_as_float(r.lo.w);
        x[4] = __uint_as_float(r.hi.x); x[5] = __uint_as_float(r.hi.y);
        x[6] = __uint_as_float(r.hi.z); x[7] = __uint_as_float(r.hi.w);
    }
}

template <bool BF16>
__device__ __forceinline__ void gate_load8(const void *p, size_t idx, float (&x)[8])
{
    gate_unpack<BF16>(gate_fetch<BF16>(p, idx), x);
}

__device__ __forceinline__ uint32_t gate_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if (f != f) return 0x7fc0u;                 // NaN stays a (quiet) NaN whatever its payload
    u += 0x7fffu + ((u >> 16) & 1u);            // round to nearest even; overflow gives inf
    return u >> 16;
}

template <bool BF16>
__device__ __forceinline__ void gate_store8(void *p, size_t idx, const float (&x)[8])
{
    if (BF16) {
        uint4 r;
        r.x = gate_bf16_rne(x[0]) | (gate_bf16_rne(x[1]) << 16);
        r.y = gate_bf16_rne(x[2]) | (gate_bf16_rne(x[3]) << 16);
        r.z = gate_bf16_rne(x[4]) | (gate_bf16_rne(x[5]) << 16);
        r.w = gate_bf16_rne(x[6]) | (gate_bf16_rne(x[7]) << 16);
        const gate_u32x4 v = {r.x, r.y, r.z, r.w};       // results are not read again here
        __builtin_nontemporal_store(v, (gate_u32x4 *)((uint16_t *)p + idx));
    } else {
        *(float4 *)((float *)p + idx) = make_float4(x[0], x[1], x[2], x[3]);
        *(float4 *)((float *)p + idx + 4) = make_float4(x[4], x[5], x[6], x[7]);
    }
}

template <int D, bool BF16, bool BWD>
__global__ __launch_bounds__(256) void la_gate_norm_kernel(GateArgs a)
{
    constexpr int TT = 8;                 // tokens per workgroup
    constexpr int CHK = D / 8;            // 8-element chunks per row
    constexpr int HPS = 256 / (CHK * TT); // heads per step
    constexpr int NPT = CHK * HPS;        // threads that share a token (= 32)
    __shared__ float red[2][TT][NPT];

    const int tid = threadIdx.x;
    const int ch = tid % CHK, tl = (tid / CHK) % TT, hh = tid / (CHK * TT);
    const int b = blockIdx.y;
    const int t = blockIdx.x * TT + tl;
    const bool live = t < a.n;
    const int slot = hh * CHK + ch;

    auto index = [&](int h) -> size_t { return (((size_t)b * a.H + h) * a.n + t) * D + 8 * ch; };

    // ---- pass 1: per-token sums over all heads and features ------------------------
    constexpr int KC = BF16 ? 8 : 0;      // head steps whose loads stay in registers
    GateRaw<BF16> co[KC > 0 ? KC : 1], cu[KC > 0 ? KC : 1], cg[KC > 0 ? KC : 1];
    float s2 = 0.f, s1 = 0.f;             // sum O^2 ; backward: sum dY*U*O
    if (live) {
#pragma unroll
        for (int k = 0; k < KC; ++k) {    // issue every cached load before using any
            const int h = hh + HPS * k;
            if (h < a.H) {
                co[k] = gate_fetch<BF16, true>(a.O, index(h));
                cu[k] = gate_fetch<BF16, true>(a.U, index(h));
                if (BWD) cg[k] = gate_fetch<BF16, true>(a.dY, index(h));
            }
        }
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            const int h = hh + HPS * k;
            if (h < a.H) {
                float x[8];
                gate_unpack<BF16>(co[k], x);
#pragma unroll
                for (int i = 0; i < 8; ++i) s2 = fmaf(x[i], x[i], s2);
                if (BWD) {
                    float u[8], g[8];
                    gate_unpack<BF16>(cu[k], u);
                    gate_unpack<BF16>(cg[k], g);
#pragma unroll
                    for (int i = 0; i < 8; ++i) s1 = fmaf(g[i] * u[i], x[i], s1);
                }
            }
        }
        for (int h = hh + HPS * KC; h < a.H; h += HPS) {
            float x[8];
            gate_load8<BF16>(a.O, index(h), x);
#pragma unroll
            for (int i = 0; i < 8; ++i) s2 = fmaf(x[i], x[i], s2);
            if (BWD) {
                float u[8], g[8];
                gate_load8<BF16>(a.U, index(h), u);
                gate_load8<BF16>(a.dY, index(h), g);
#pragma unroll
                for (int i = 0; i < 8; ++i) s1 = fmaf(g[i] * u[i], x[i], s1);
            }
        }
    }
    red[0][tl][slot] = s2;
    if (BWD) red[1][tl][slot] = s1;
    __syncthreads();
    float t2 = 0.f, t1 = 0.f;
#pragma unroll
    for (int i = 0; i < NPT; ++i) {
        t2 += red[0][tl][i];
        if (BWD) t1 += red[1][tl][i];
    }
    const float inv_n = 1.0f / (float)(a.H * D);
    const float inv_r = rsqrtf(t2 * inv_n + a.eps);         // 1 / sqrt(mean(O^2) + eps)
    const float c3 = BWD ? t1 * inv_n * inv_r * inv_r * inv_r : 0.f;   // mean(dN*O) / r^3

    // ---- pass 2 ------------------------------------------------------------------------
    if (!live) return;
    auto emit = [&](size_t at, const float (&x)[8], const float (&u)[8], const float (&g)[8]) {
        if (!BWD) {
            float y[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) y[i] = x[i] * inv_r * u[i];
            gate_store8<BF16>(a.Y, at, y);
        } else {
            float dx[8], du[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                du[i] = g[i] * x[i] * inv_r;
                dx[i] = g[i] * u[i] * inv_r - x[i] * c3;
            }
            gate_store8<BF16>(a.dO, at, dx);
            gate_store8<BF16>(a.dU, at, du);
        }
    };
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        const int h = hh + HPS * k;
        if (h < a.H) {
            float x[8], u[8], g[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            gate_unpack<BF16>(co[k], x);
            gate_unpack<BF16>(cu[k], u);
            if (BWD) gate_unpack<BF16>(cg[k], g);
            emit(index(h), x, u, g);
        }
    }
    for (int h = hh + HPS * KC; h < a.H; h += HPS) {     // the tiles are still in L2
        const size_t at = index(h);
        float x[8], u[8], g[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        gate_load8<BF16>(a.O, at, x);
        gate_load8<BF16>(a.U, at, u);
        if (BWD) gate_load8<BF16>(a.dY, at, g);
        emit(at, x, u, g);
    }
}
