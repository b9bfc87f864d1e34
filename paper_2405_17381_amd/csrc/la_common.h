// Shared declarations of the HIP kernels (gfx950 only).
//
// Every kernel here evaluates one "decayed causal scan"
//
//     Out[t] = sum_{s <= t} lambda^(t-s) (A[t] . Bm[s]) C[s]        (forward in time)
//     Out[t] = sum_{s >= t} lambda^(s-t) (A[t] . Bm[s]) C[s]        (REV, backward in time)
//
// over one (batch, head) slice of [n, D] tensors, tiled as in Alg. 5 / Alg. 6:
// per block an intra part [(A Bm^T) * M] C and an inter part against a running
// D x D state  St[i][j] = sum_s w_s Bm[s][i] C[s][j].  The four results of the
// method are this scan with different operands:
//
//     O  = scan(Q,  K,  V )            dQ = scan(dO, V,  K )         (Alg. 6, first loop)
//     dK = scan_rev(V, dO, Q)          dV = scan_rev(K, Q, dO)       (Alg. 6, second loop)
//
// State normalisation.  With 0-based row r inside a block of BK rows starting
// at t0, the forward state at a block start weights the immediately preceding
// token by 1:  St = sum_{s < t0} lambda^(t0-1-s) Bm[s] C[s]^T  (the paper's KV_t).
// The reverse state weights the immediately following token by 1:
// St = sum_{s >= t0+BK} lambda^(s-t0-BK) Bm[s] C[s]^T; the paper's dKV_t carries
// one more factor lambda, which it takes back in its row scale lambda^(B-r);
// the products are identical.
//
//   forward : mask lambda^(r-c) (r >= c), inter row scale lambda^(r+1),
//             state update weight of row r: lambda^(BK-1-r)
//   reverse : mask lambda^(c-r) (c >= r), inter row scale lambda^(BK-r),
//             state update weight of row r: lambda^r
//   both    : St <- lambda^BK St + sum_r weight_r Bm[r] C[r]^T
// No negative power of lambda is ever formed (Lambda^-1 of Alg. 5 would
// overflow for small lambda).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/la.h"

struct LaLambdas {
    float v[LA_MAX_HEADS];      // lambda_h
    float lg2[LA_MAX_HEADS];    // log2(lambda_h), evaluated in double on the host
    uint8_t order[LA_MAX_HEADS]; // heads by decreasing lambda: the pre-pass dispatches the
                                // slowly decaying heads (longest chains) first
};

// Where one (batch, head) slab of an operand lives: element offset b * bs + h * hs, rows
// `ld` elements apart.  Contiguous [B, H, n, D]: bs = H n D, hs = n D, ld = D.  A slice of
// D features out of a wider tensor has the wider row as ld.  Only the kernel variants built
// with the extensions (ACT) read these; the plain ones assume the contiguous layout.
struct LaLayout {
    long bs, hs;
    int ld;
};

struct ScanArgs {
    const void *A;       // role of Q   [scans, n, D]
    const void *Bm;      // role of K
    const void *C;       // role of V
    void *Out;           // role of O
    float *states;       // [scans, S, D*D] fp32 segment-boundary states (or nullptr)
    int n;               // sequence length
    int H;               // heads (scan index % H selects lambda)
    int L;               // segment length in tokens (multiple of the tile length)
    int S;               // segments per scan
    int B;               // batch size (scan index = b * H + h)
    float skip_bits;     // segment-state pre-pass only: rows whose decay weight is below
                         // 2^-skip_bits are not read (0 = read everything)
    int transpose_init;  // the stored segment states are those of the scan with Bm and C
                         // exchanged: read them transposed
    int rev;             // segment-state pre-pass only: direction of this role's scan
                         // (block scans take the direction from the kernel's template)
    const float *st_in;  // forward scans only: state carried in from earlier tokens,
                         // [scans, D, D] fp32 (rows = Bm feature), or nullptr for zero
    float *st_out;       // forward scans only: state after the last token, or nullptr
    int act;             // LA_ACT_* bits: operands that are pre-activations (Swish is applied
                         // as they are staged) and whether Out is a pre-activation gradient
    const void *E;       // LA_ACT_OUT: the pre-activation whose gradient Out is, [scans, n, D]
    LaLayout lA, lB, lC, lO, lE;   // layouts of A, Bm, C, Out, E
};

// Swish on the query / key projections (Sec. 4.2: Q = phi(X W_q), K = phi(X W_k)).
// The scans take the pre-activations and apply phi while staging a tile; a scan
// whose result is the gradient of an activated operand multiplies it by phi' of the
// matching pre-activation tile as it is stored (chain rule).
// LA_ACT_ACC: the result is added to what Out already holds (a scan over one slice of a
// wider query / key feature dimension adds to the scans over the other slices).
// LA_ACT_EXT alone only selects the extended kernel variants (strided operands).
enum : int { LA_ACT_A = 1, LA_ACT_BM = 2, LA_ACT_C = 4, LA_ACT_OUT = 8, LA_ACT_ACC = 16, LA_ACT_EXT = 32 };

// phi(x) = x sigmoid(x).  exp2 overflows to +inf for x < -88, giving sigmoid = 0: the limit.
__device__ __forceinline__ float la_sigmoid(float x)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}
__device__ __forceinline__ float la_swish(float x) { return x * la_sigmoid(x); }
// phi'(x) = s (1 + x (1 - s)), s = sigmoid(x)
__device__ __forceinline__ float la_swish_grad(float x)
{
    const float sg = la_sigmoid(x);
    return sg * fmaf(x, 1.0f - sg, 1.0f);
}

// One launch of the block-scan kernel runs one scan, or two scans that read
// mostly the same tensors (the dK and dV scans of Alg. 6's second loop).  In a
// paired launch the two workgroups of one (scan, segment) item are placed on
// the same XCD in consecutive dispatch slots, so that the tiles both of them
// read are fetched from HBM once and served to the second reader from that
// XCD's L2.  Workgroup ids go round-robin over the 8 XCDs:
//   xcd = id % 8, slot = id / 8, role = slot % 2, item = (slot / 2) * 8 + xcd.
struct ScanLaunch {
    ScanArgs r[3];
    int nroles;          // 1, 2, or 3 = the whole backward pass in one launch of the direct-to-LDS block
                         // scan: r[0] forward in time (dQ), r[1] and r[2] reversed (dK, dV), the three
                         // workgroups of an item on one XCD (id % 8), roles in consecutive slots
    int items;           // scans * S
};

// kernel arguments travel in the dispatch packet: 4 KB at most
static_assert(sizeof(ScanLaunch) + sizeof(LaLambdas) <= 4096, "kernel arguments exceed the 4 KB limit");

// Segment scan over local segment states, in place:
//   forward: W[s] <- state entering segment s  (W[0] <- carried-in state or 0)
//   reverse: W[s] <- state entering segment s from the right (W[S-1] <- 0)
// Entering state of segment `seg` of scan `scan` (nullptr = zero).  Normally the
// slot the segment scan wrote.  Heads whose decay over one whole segment is below
// the pre-pass cut-off (lambda^L <= 2^-skip_bits) are "chain free": what entered the
// previous segment no longer matters, the entering state IS the previous segment's
// local state, and the segment scan leaves their local states alone.  A state carried
// in by the caller enters such a head's first segment through the last slot, which no
// local state occupies (the final segment's is never produced): the segment scan copies
// it there, so that no block-scan workgroup reads the caller's buffer while another one
// may already be writing the state handed back into that same buffer.
__device__ __forceinline__ const float *la_entering_state(const ScanArgs &a, int scan, int seg, bool rev,
                                                          float lg2_lambda, int dd)
{
    if (a.S <= 1) return (!rev && a.st_in) ? a.st_in + (size_t)scan * dd : nullptr;
    if (!a.states) return nullptr;
    const float *slot0 = a.states + (size_t)scan * a.S * dd;
    const bool chain_free = a.skip_bits > 0.f && -lg2_lambda * (float)a.L >= a.skip_bits;
    if (!chain_free) return slot0 + (size_t)seg * dd;
    if (!rev) return seg > 0 ? slot0 + (size_t)(seg - 1) * dd : (a.st_in ? slot0 + (size_t)(a.S - 1) * dd : nullptr);
    return seg < a.S - 1 ? slot0 + (size_t)(seg + 1) * dd : nullptr;
}

struct SegScanArgs {
    float *states;       // [scans, S, DD]
    float skip_bits;     // heads with lambda^L <= 2^-skip_bits are not scanned (0 = scan all)
    const float *init;   // state entering the first (forward) segment, [scans, DD], or nullptr
    int H, S, L, DD;
};
