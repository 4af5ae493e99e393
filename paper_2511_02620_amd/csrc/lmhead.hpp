// Shapes, launch plan and workspace layout of the fused LM-head scoring path, shared by the
// kernels (lmhead.hip) and the C ABI layer.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace difr {

constexpr int kLmTileV = 256;  // vocabulary entries per workgroup tile
constexpr int kLmTileT = 256;  // token rows per workgroup tile
constexpr int kLmTileK = 64;   // hidden-dimension slab staged through LDS per step

// Kernel-side image of difr_lmhead.
struct LmHeadBatch {
    const uint16_t *hidden;  // [N, ldh] bf16
    const uint16_t *weight;  // [V, ldw] bf16
    int64_t N, V, d, ldh, ldw;
    float temperature;
    const float *temperatures;
    const uint64_t *seeds;
    int64_t S;
    const int32_t *seq_ids;
    const uint32_t *positions;
    const int32_t *claimed_gumbel;
    const int32_t *claimed_ipt;
};

// How the [N, V] logit matrix is cut into workgroups: n_tb token blocks times `splits` contiguous
// ranges of vocabulary tiles.  Every workgroup walks its range tile by tile and leaves one partial
// result per token; a last kernel merges the `splits` partials of each token in vocabulary order.
struct LmHeadPlan {
    int n_tb;    // token blocks of kLmTileT rows
    int n_vt;    // vocabulary tiles of kLmTileV entries
    int splits;  // vocabulary ranges (1 <= splits <= n_vt)
};

inline LmHeadPlan lmhead_plan(int64_t N, int64_t V)
{
    LmHeadPlan p;
    p.n_tb = (int)((N + kLmTileT - 1) / kLmTileT);
    p.n_vt = (int)((V + kLmTileV - 1) / kLmTileV);
    // one workgroup per compute unit (256 of them) when the token blocks alone do not fill the chip
    int s = p.n_tb > 0 ? 256 / p.n_tb : 1;
    if (s < 1) s = 1;
    if (s > p.n_vt) s = p.n_vt;
    p.splits = s;
    return p;
}

// Device pointers into the caller's workspace.
struct LmHeadWorkspace {
    double *Z, *P;         // [splits][N]  softmax sums relative to m: all entries / entries below the IPT claim
    float *m;              // [splits][N]  largest logit seen
    float *best_y;         // [splits][N]  best perturbed score
    int32_t *best_v;       // [splits][N]  and its token
    int32_t *above;        // [splits][N]  entries whose logit exceeds the Token-DiFR claim's (logit rank; only if asked for)
    float *L0;             // [N] lower bound on the row's best perturbed score (-inf if none)
    float *x_claim_gumbel; // [N] logit of the Token-DiFR claim as the tile that holds it computed it (NaN until then)
    float *x_claim_ipt;    // [N] same for the Token-IPT-DiFR claim
    float *x_claim_ref;    // [N] logit of the Token-DiFR claim as a plain fp32 dot product (NaN without a claim)
    // only when the sampler's own Token-IPT-DiFR token is asked for (null otherwise):
    float2 *half_sum;      // [2 n_vt][N] softmax mass of each half tile (128 vocabulary entries) and its exponent reference
    double *cross_rest;    // [N] mass still to be covered inside the half tile in which the CDF passes u, relative to final_m
    float *final_m;        // [N] the row's final exponent reference
    int32_t *cross_half;   // [N] that half tile, or -1 if the token is already known
};

// want_token: room for the per-half-tile masses that the search for the sampler's own token needs
inline size_t lmhead_workspace_bytes(int64_t N, int splits, int n_vt = 0, bool want_token = false)
{
    size_t bytes = (size_t)N * (size_t)splits * (8 + 8 + 4 + 4 + 4 + 4) + (size_t)N * 16 + 64;
    if (want_token) bytes += (size_t)N * (size_t)n_vt * 16 + (size_t)N * 16;
    return bytes;
}

inline LmHeadWorkspace lmhead_carve(void *base, int64_t N, int splits, int n_vt = 0, bool want_token = false)
{
    LmHeadWorkspace w;
    const size_t n = (size_t)N * (size_t)splits;
    char *p = (char *)base;
    w.Z = (double *)p;
    p += n * 8;
    w.P = (double *)p;
    p += n * 8;
    w.m = (float *)p;
    p += n * 4;
    w.best_y = (float *)p;
    p += n * 4;
    w.best_v = (int32_t *)p;
    p += n * 4;
    w.above = (int32_t *)p;
    p += n * 4;
    w.L0 = (float *)p;
    p += (size_t)N * 4;
    w.x_claim_gumbel = (float *)p;
    p += (size_t)N * 4;
    w.x_claim_ipt = (float *)p;
    p += (size_t)N * 4;
    w.x_claim_ref = (float *)p;
    p += (size_t)N * 4;
    w.half_sum = nullptr;
    w.cross_rest = nullptr;
    w.final_m = nullptr;
    w.cross_half = nullptr;
    if (want_token) {
        p = (char *)(((uintptr_t)p + 7u) & ~(uintptr_t)7u);
        w.half_sum = (float2 *)p;
        p += (size_t)N * (size_t)n_vt * 16;
        w.cross_rest = (double *)p;
        p += (size_t)N * 8;
        w.final_m = (float *)p;
        p += (size_t)N * 4;
        w.cross_half = (int32_t *)p;
    }
    return w;
}

}  // namespace difr
