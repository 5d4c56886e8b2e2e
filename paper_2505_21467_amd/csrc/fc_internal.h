// Internal declarations shared by the host layer and the kernel files of libfreecache.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "freecache.h"

#define FC_VTILE 64  // rows per transposed V tile; Spad is a multiple of it

struct fc_cache {
    fc_config cfg;
    int32_t spad;        // max_seq rounded up to FC_VTILE
    size_t layer_elems;  // elements of one layer's K (== V) storage: B * Hkv * spad * Dh
    size_t esize;        // bytes per element
    void *k;             // device
    void *v;             // device
    bool owned;
    double inv_freq[64]; // rotary frequencies rope_base^(-2i/Dh), i < Dh/2, computed once on the host
    // Device scratch owned by the handle (nullptr when no GPU was present at creation): space for the
    // partial sums that the short-window projection hands from its first kernel to its second.
    void *scratch;
    // Carve-up of the whole-layer workspace for the last (d_ff, A) seen: fc_full_layer_step is called
    // with the same shape step after step, and planning it anew walks every window size up to A.
    int32_t ws_d_ff, ws_A;
    size_t ws_part[10];
};

#define FC_SCRATCH_BYTES (32u * 1024u * 1024u)

// Tuning knobs: defaults (0 / -1 = the planner decides), overridden once from the environment
// variables of the same names at first use and afterwards only through fc_tuning_set.  Planners and
// launchers read this struct; nothing on a launch path calls getenv.
struct FcKnobs {
    int attn_r, attn_w;     // FC_ATTN_TILES=R,W      row tiles and waves per attention workgroup
    int attn_wgs;           // FC_ATTN_WGS=n          workgroups the split heuristic aims for
    int lin_wgs;            // FC_LIN_WGS=n           workgroups of the weight-streaming linear kernels
    int lin_no_rows;        // FC_LIN_NO_ROWS         slice-wise instead of whole-row weight streaming
    int lin_wide_shape;     // FC_LIN_WIDE_SHAPE=0..2 (4: gated layer only) one tile shape for the tiled linear GEMM (-1 = planned)
    int lin_ksplit;         // FC_LIN_KSPLIT=n        parts of the hidden dimension
    int gemm_no_split;      // FC_GEMM_NO_SPLIT       never cut a GEMM into two launches
    int proj_gemm_shape;    // FC_PROJ_GEMM_SHAPE=0..5 one tile shape for the projection GEMM (-1 = planned)
    int proj_no_headsplit;  // FC_PROJ_NO_HEADSPLIT   short-window projection without the head-split kernels
    int accept_wgs;         // FC_ACCEPT_WGS=n        workgroups of the acceptance scan
};
const FcKnobs &fc_knobs();

// Geometry handed to kernels by value.
struct FcGeom {
    int32_t B, d, Hq, Hkv, Dh, max_seq, spad, g;
    float scale;      // softmax scale
    double log_base;  // ln(rope_base)
};

// Element offset of K[b][j][row][i] inside one layer.
__host__ __device__ inline size_t fc_k_index(const FcGeom &G, int b, int j, int row, int i)
{
    return (((size_t)b * G.Hkv + j) * G.spad + row) * G.Dh + i;
}
// Element offset of V[b][j][row][i] inside one layer (64-row tiles, key index fastest).
__host__ __device__ inline size_t fc_v_index(const FcGeom &G, int b, int j, int row, int i)
{
    return ((size_t)b * G.Hkv + j) * G.spad * G.Dh + (size_t)(row / FC_VTILE) * (FC_VTILE * G.Dh) +
           (size_t)i * FC_VTILE + (row % FC_VTILE);
}

// Launch plan of the split-KV attention (host, pure function of the shape).
struct FcAttnPlan {
    int kind;            // 0 = generic kernel (no workspace), 1 = MFMA split-KV
    int splits;          // key ranges per (sequence, kv head); every one is non-empty
    int splits_bound;    // upper bound of `splits` over all kv_len <= the given one (workspace sizing)
    int keys_per_split;  // multiple of 64
    int row_tiles;       // 32-row tiles of the flattened (head-in-group, a) rows per (b, kv head)
    int tiles_per_wg;    // row tiles handled by one workgroup
    int waves;           // waves per workgroup (tiles_per_wg or twice that)
};
FcAttnPlan fc_plan_attention(const fc_config &cfg, int A, int kv_len);
size_t fc_plan_workspace(const fc_config &cfg, const FcAttnPlan &p, int A);

// Kernel launchers (defined in the .hip kernel files).  All return hipGetLastError() after launch.
hipError_t fc_launch_copy_rows(const FcGeom &G, int dtype, void *k_layer, void *v_layer, void *k_rows,
                               void *v_rows, int start, int rows, bool to_cache, hipStream_t s);
hipError_t fc_launch_project_generic(const FcGeom &G, int dtype, const void *x, const void *w,
                                     const void *bias, const int32_t *pos, int win_start, int A,
                                     void *q_out, void *k_layer, void *v_layer, hipStream_t s);
hipError_t fc_launch_attention_generic(const FcGeom &G, int dtype, const void *q, const void *k_layer,
                                       const void *v_layer, const int32_t *pos, int A, int kv_len,
                                       void *out, hipStream_t s);
bool fc_project_mfma_supported(const fc_config &cfg, int A);
hipError_t fc_launch_project_mfma(const FcGeom &G, const double *inv_freq, const void *x, const void *w, const void *bias,
                                  const int32_t *pos, int win_start, int A, void *q_out,
                                  void *k_layer, void *v_layer, void *scratch, hipStream_t s);
bool fc_project_gemm_supported(const fc_config &cfg, int M);
hipError_t fc_launch_project_gemm(const FcGeom &G, const void *x, const void *w, const void *bias,
                                  const int32_t *pos, int win_start, int A, void *q_out, void *k_layer,
                                  void *v_layer, hipStream_t s);
hipError_t fc_launch_attention_mfma(const FcGeom &G, const FcAttnPlan &p, const void *q,
                                    const void *k_layer, const void *v_layer, const int32_t *pos,
                                    int A, int kv_len, void *out, void *workspace, hipStream_t s);

// Rest of the layer on the window rows: RMS normalisation and the linear layers around attention.
enum { FC_LIN_RESIDUAL = 0, FC_LIN_GATE_UP = 1, FC_LIN_VOCAB = 2 };
// Vocabulary mode: per (part of the vocabulary, row) the largest logit, its index and the sum of
// exp(logit - largest) over the part, each array [parts][M].
struct FcArgmaxPart {
    float *mx;
    int32_t *arg;
    float *sm;
};
// (largest, index, sum) of a union of two parts; equal maxima keep the smaller index.
__host__ __device__ inline void fc_argmax_merge(float &mx, int &arg, float &sm, float mx2, int arg2, float sm2)
{
    if (mx2 > mx || (mx2 == mx && arg2 < arg)) {
        const float t = mx;
        mx = mx2;
        mx2 = t;
        const float u = sm;
        sm = sm2;
        sm2 = u;
        arg = arg2;
    }
    // now mx >= mx2; a part that is still empty has mx2 = -inf and sm2 = 0
    if (sm2 != 0.f) sm += sm2 * expf(mx2 - mx);
}
hipError_t fc_launch_rmsnorm(int dtype, const void *x, const void *weight, float eps, int rows, int d,
                             void *out, hipStream_t s);
// Plain-ALU linear layer for any dtype and shape.  FC_LIN_RESIDUAL: out = aux + x w^T (aux = residual
// or nullptr); FC_LIN_GATE_UP: out = silu(x w^T) * (x aux^T) (aux = up matrix).
hipError_t fc_launch_linear_generic(int dtype, int mode, const void *x, const void *w, const void *aux,
                                    int M, int K, int N, void *out, hipStream_t s);
// Launch plan of the weight-streaming linear kernels (host, pure function of the shape).
struct FcSkinnyPlan {
    int kind;    // 0 = plain kernel (no workspace), 1 = streaming kernels, 2 = whole-row kernel (T = half items, G)
    int mt;      // 16-row tiles per pass (1 or 2)
    int chunks;  // passes of up to 32 rows
    int slabs;   // 128-row slabs of the weight matrix (64 gate + 64 up rows in gated mode)
    int S;       // hidden-dimension slices per slab
    int T;       // work items = slabs * S
    int G;       // workgroups
    int maxseg;  // upper bound of the workgroups that meet one slab
};
FcSkinnyPlan fc_plan_skinny(int dtype, int mode, int M, int K, int N);
size_t fc_skinny_workspace(const FcSkinnyPlan &p);
hipError_t fc_launch_linear_skinny(const FcSkinnyPlan &pl, int mode, const void *x, const void *w,
                                   const void *w2, const void *res, int M, int K, int N, void *out,
                                   void *workspace, hipStream_t s, const FcArgmaxPart *am = nullptr);
// Unmasking step: plain vocabulary projection (any dtype / shape), merge of the vocabulary parts, and
// the confidence-ranked fill.
hipError_t fc_launch_lmhead_generic(int dtype, const void *x, const void *w, int M, int K, int V,
                                    const FcArgmaxPart &am, hipStream_t s);
#define FC_LMHEAD_GENERIC_CHUNK 256  // vocabulary entries per part of the plain kernel
hipError_t fc_launch_lmhead_reduce(const FcArgmaxPart &am, int parts, int M, int32_t *tok, float *conf,
                                   hipStream_t s);
#define FC_UNMASK_MAX_ROWS 8192
hipError_t fc_launch_unmask_select(const int32_t *tok, const float *conf, const int32_t *pos, int win_start,
                                   int B, int A, int n_unmask, int mask_id, int32_t *tokens, int L,
                                   int32_t *pos_next, int32_t *count_next, hipStream_t s);
// Tiled-GEMM plan of the same linear layers on more than 32 rows.
struct FcWidePlan {
    int kind;    // 0 = not covered, 1 = tiled GEMM
    int shape;   // 0: 256 rows x slab, 1: 128 rows x slab, 2: 128 rows x half slab
    int ksplit;  // parts of the hidden dimension (1 = epilogue inside the GEMM, no workspace)
};
FcWidePlan fc_plan_wide(int dtype, int mode, int M, int K, int N);
size_t fc_wide_workspace(const FcWidePlan &p, int M, int N);
hipError_t fc_launch_linear_wide(const FcWidePlan &pl, int mode, const void *x, const void *w, const void *w2,
                                 const void *res, int M, int K, int N, void *out, void *workspace, hipStream_t s,
                                 const FcArgmaxPart *am = nullptr);
hipError_t fc_launch_gather_rows(const void *table, int64_t R, int row_bytes, const int32_t *idx, int64_t n, void *out,
                                 hipStream_t s);
#define FC_ACCEPT_MAX_TOPK 8
size_t fc_accept_workspace(int B, int A, int V);
hipError_t fc_launch_guided_accept(const float *dlm, const float *ar, const int32_t *pos, int win_start, int B, int A,
                                   int V, int topk, float tau, int mask_id, int32_t *tokens, int L, int32_t *n_accept,
                                   int32_t *pos_next, int32_t *count_next, void *workspace, hipStream_t s);
hipError_t fc_launch_kv_similarity(const FcGeom &G, int dtype, const void *k_layer, const void *v_layer,
                                   const void *k_prev, const void *v_prev, int start, int rows, float *sim_k,
                                   float *sim_v, hipStream_t s);
