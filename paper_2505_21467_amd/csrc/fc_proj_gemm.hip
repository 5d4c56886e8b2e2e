// QKV projection of a wide window (hundreds to thousands of rows: refreshes, batched blocks) as a
// tiled matrix-core GEMM (bf16, head_dim 128), fused with bias, rotary embedding and the scatter into
// the cache.  Table 1's "W_Q, W_K, W_V projections" row with L replaced by the window length.
//
// Y^T = W X^T: the weight rows are the A operand of v_mfma_f32_32x32x16_bf16 and the window rows the B
// operand, so a lane of the accumulator holds 16 output features of ONE window row.  A wave owns 32
// window rows and all NSUB 32-feature sub-tiles of its workgroup; with NSUB = 4 the workgroup covers a
// whole head (features i and i + 64 of a rotary pair sit in sub-tiles t and t + 2, same lane, same
// register), with NSUB = 2 it covers the rotary-paired half head {32 h .. 32 h + 31} u {64 + 32 h ..}
// (more, smaller workgroups when the window is too short to fill the chip).  The rotation, the bias and
// the stores to q_out / the K rows / the transposed V tiles therefore need no exchange between lanes.
//
// Both operands are contiguous along the hidden dimension.  64 hidden elements of every row of the
// tile (128-byte row pieces) stream HBM/L2 -> LDS with direct-to-LDS 16-byte loads into a ring of
// three stages, two ahead of the multiply; the 16-byte chunks of a row piece are XOR-swizzled with
// bits 1..3 of the row (applied to the global address of the loading lane), which spreads the 16 lanes
// the LDS serves per clock over 16 different bank groups.
#include <stdlib.h>

#include "fc_device.h"
#include "fc_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int KS = 64;          // hidden elements per stage
constexpr int ROWB = KS * 2;    // bytes of one row piece
constexpr int SLOTS = 3;

struct GemmArgs {
    const uint16_t *X;     // [M][K]
    const uint16_t *W;     // [N][K]
    const uint16_t *bias;  // [N] or nullptr
    const int32_t *pos;    // [M] or nullptr
    uint16_t *Q;           // [B][Hq][A][128]
    uint16_t *Kc;          // one layer
    uint16_t *Vc;          // one layer
    FcGeom G;
    int M, A, K, win_start;
    int n_mt;              // row tiles of 32 * NW window rows
    int n_units;           // head slots (NSUB = 4) or half-head slots (NSUB = 2)
    double log2_base_64;   // log2(rope_base) / 64
};

__device__ __forceinline__ void load_lds16g(const void *g, void *l)
{
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)g,
                                     (void __attribute__((address_space(3))) *)l, 16, 0, 0);
}

template <int N>
__device__ __forceinline__ void wait_vmg()
{
    // gfx9 s_waitcnt immediate: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// NW waves (32 window rows each), NSUB feature sub-tiles of 32.
template <int NW, int NSUB>
__global__ __launch_bounds__(NW * 64) void k_proj_gemm(GemmArgs p)
{
    constexpr int WROWS = 32 * NSUB, XROWS = 32 * NW;
    constexpr int WBYTES = WROWS * ROWB, STAGE = (WROWS + XROWS) * ROWB;
    constexpr int NBLK = (WROWS + XROWS) / 8;  // 1 KB blocks (8 row pieces) per stage
    constexpr int LBW = NBLK / NW;             // blocks per wave and stage
    constexpr int WBW = (WROWS / 8) / NW;      // of which weight blocks (the first ones)
    static_assert(NBLK % NW == 0 && (WROWS / 8) % NW == 0, "tile shape");
    extern __shared__ __align__(1024) unsigned char smem[];
    const FcGeom &G = p.G;

    // Workgroup -> (unit, row tile): the n_mt workgroups that stream the same weight rows get ids that
    // are equal modulo 8, i.e. land on the same XCD and share its L2.
    const int id = blockIdx.x;
    const int xcd = id & 7, qd = id >> 3;
    const int mt = qd % p.n_mt;
    const int unit = (qd / p.n_mt) * 8 + xcd;
    if (unit >= p.n_units) return;
    const int hs = NSUB == 4 ? unit : unit >> 1;   // head slot: Hq query heads, Hkv key heads, Hkv value heads
    const int half = NSUB == 4 ? 0 : unit & 1;     // which rotary-paired half of the head
    const int m0 = mt * XROWS;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hi = lane >> 5;

    // ---- loader: per-lane source offsets (bytes from W / X, hidden offset 0) of this wave's blocks
    uint32_t goff[LBW];
#pragma unroll
    for (int i = 0; i < LBW; ++i) {
        const int bid = wave + NW * i;              // block of the stage: weight blocks first
        const int rl = 8 * (i < WBW ? bid : bid - WROWS / 8) + (lane >> 3);  // row of the W / X tile
        const int c = (lane & 7) ^ ((rl >> 1) & 7);  // logical 16-byte chunk that lands at position lane & 7
        if (i < WBW) {
            const int n = hs * 128 + (NSUB == 4 ? rl : ((rl >> 5) * 64 + 32 * half + (rl & 31)));
            goff[i] = (uint32_t)n * (uint32_t)(p.K * 2) + c * 16;
        } else {
            const int m = min(m0 + rl, p.M - 1);    // rows past the end re-read the last row; never stored
            goff[i] = (uint32_t)m * (uint32_t)(p.K * 2) + c * 16;
        }
    }
    auto issue_stage = [&](int st) {
        unsigned char *dst = smem + (st % SLOTS) * STAGE;
#pragma unroll
        for (int i = 0; i < LBW; ++i) {
            const unsigned char *src = (const unsigned char *)(i < WBW ? p.W : p.X) + (size_t)st * ROWB;
            load_lds16g(src + goff[i], dst + (wave + NW * i) * 1024);
        }
    };

    // ---- operand read offsets inside a stage (bytes): row `col` of a 32-row sub-tile, k-step kk
    uint32_t foff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) foff[kk] = (uint32_t)(col * ROWB + (((2 * kk + hi) ^ ((col >> 1) & 7)) << 4));

    f32x16 acc[NSUB];
#pragma unroll
    for (int t = 0; t < NSUB; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    const int n_stages = p.K / KS;
    issue_stage(0);
    if (n_stages > 1) issue_stage(1);
    for (int it = 0; it < n_stages; ++it) {
        if (it + 1 < n_stages) wait_vmg<LBW>();
        else wait_vmg<0>();
        // Behind this barrier stage `it` is complete for every wave and every wave has left stage
        // it-1, whose slot is the one refilled next.
        __builtin_amdgcn_s_barrier();
        if (it + 2 < n_stages) issue_stage(it + 2);
        const unsigned char *st = smem + (it % SLOTS) * STAGE;
        const unsigned char *xs = st + WBYTES + wave * (32 * ROWB);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const bf16x8 xf = *(const bf16x8 *)(xs + foff[kk]);
            bf16x8 wf[NSUB];
#pragma unroll
            for (int t = 0; t < NSUB; ++t) wf[t] = *(const bf16x8 *)(st + t * (32 * ROWB) + foff[kk]);
#pragma unroll
            for (int t = 0; t < NSUB; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[t], xf, acc[t], 0, 0, 0);
        }
    }

    // ---- epilogue, in registers.  Lane (col, hi) holds window row m0 + 32 wave + col; register r of
    // sub-tile t is feature 32 t' + 8 (r >> 2) + 4 hi + (r & 3) of the head, with t' = t for a whole
    // head and {half, half + 2} for a half head.
    const int m = m0 + 32 * wave + col;
    const bool mvalid = m < p.M;
    const int mm = mvalid ? m : 0;
    const int b = mm / p.A, a = mm - b * p.A;
    const int pp = p.pos ? p.pos[mm] : p.win_start + a;
    const bool valid = mvalid && pp >= 0 && pp < G.max_seq;
    const bool rotate = hs < G.Hq + G.Hkv;
    constexpr int NP = NSUB / 2;  // rotary pairs of sub-tiles: (t, t + NP)

    if (p.bias) {
#pragma unroll
        for (int t = 0; t < NSUB; ++t) {
            const int tq = NSUB == 4 ? t : half + 2 * t;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[t][r] += fc_to_float(bf16_t{p.bias[hs * 128 + 32 * tq + 8 * (r >> 2) + 4 * hi + (r & 3)]});
        }
    }
    if (rotate) {
        // base^(-i/64) / (2 pi) in double by powers of r1 = base^(-1/64); the angle is reduced to a
        // fraction of a turn in double, then hardware sine / cosine (argument in turns).
        const double r1 = exp2(-p.log2_base_64);
        const double r2 = r1 * r1, r4 = r2 * r2, r8 = r4 * r4, r16 = r8 * r8, r32 = r16 * r16;
#pragma unroll
        for (int t = 0; t < NP; ++t) {
            const int tq = NSUB == 4 ? t : half;  // i = 32 tq + 8 rq + 4 hi + (r & 3) < 64
            double f = 0.15915494309189533576888;
            if (tq) f *= r32;
            if (hi) f *= r4;
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                double fr = f;
#pragma unroll
                for (int r3 = 0; r3 < 4; ++r3) {
                    const int r = 4 * rq + r3;
                    const double turns = (double)pp * fr;
                    const float ph = (float)(turns - rint(turns));
                    const float c = __builtin_amdgcn_cosf(ph), sn = __builtin_amdgcn_sinf(ph);
                    const float lo = acc[t][r], hi2 = acc[t + NP][r];
                    acc[t][r] = lo * c - hi2 * sn;
                    acc[t + NP][r] = hi2 * c + lo * sn;
                    fr *= r1;
                }
                f *= r8;
            }
        }
    }
    if (!mvalid) return;

#pragma unroll
    for (int t = 0; t < NSUB; ++t) {
        const int tq = NSUB == 4 ? t : half + 2 * t;
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            const int d0 = 32 * tq + 8 * rq + 4 * hi;
            uint2 w;
            w.x = (uint32_t)fc_bf16_bits(acc[t][4 * rq]) | ((uint32_t)fc_bf16_bits(acc[t][4 * rq + 1]) << 16);
            w.y = (uint32_t)fc_bf16_bits(acc[t][4 * rq + 2]) | ((uint32_t)fc_bf16_bits(acc[t][4 * rq + 3]) << 16);
            if (hs < G.Hq) {
                if (!valid) w = make_uint2(0, 0);
                *(uint2 *)(p.Q + (((size_t)b * G.Hq + hs) * p.A + a) * 128 + d0) = w;
            } else if (valid) {
                if (hs < G.Hq + G.Hkv) {
                    *(uint2 *)(p.Kc + fc_k_index(G, b, hs - G.Hq, pp, d0)) = w;
                } else {
                    const int j = hs - G.Hq - G.Hkv;
                    uint16_t *v = p.Vc + fc_v_index(G, b, j, pp, d0);
                    v[0] = (uint16_t)(w.x & 0xffff);
                    v[FC_VTILE] = (uint16_t)(w.x >> 16);
                    v[2 * FC_VTILE] = (uint16_t)(w.y & 0xffff);
                    v[3 * FC_VTILE] = (uint16_t)(w.y >> 16);
                }
            }
        }
    }
}

template <int NW, int NSUB>
hipError_t launch_gemm(GemmArgs a, hipStream_t s)
{
    constexpr int LDS = SLOTS * (32 * NSUB + 32 * NW) * ROWB;
    static hipError_t attr = hipFuncSetAttribute((const void *)k_proj_gemm<NW, NSUB>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (attr != hipSuccess) return attr;
    const int slots = a.G.Hq + 2 * a.G.Hkv;
    a.n_units = NSUB == 4 ? slots : 2 * slots;
    a.n_mt = (a.M + 32 * NW - 1) / (32 * NW);
    const unsigned grid = (unsigned)(((a.n_units + 7) / 8) * 8 * a.n_mt);
    k_proj_gemm<NW, NSUB><<<dim3(grid), dim3(NW * 64), LDS, s>>>(a);
    return hipGetLastError();
}

}  // namespace

bool fc_project_gemm_supported(const fc_config &cfg, int M)
{
    // 32-bit byte offsets inside X and W; the hidden dimension in whole stages
    const int64_t n = (int64_t)(cfg.n_q_heads + 2 * cfg.n_kv_heads) * cfg.head_dim;
    return cfg.dtype == FC_BF16 && cfg.head_dim == 128 && cfg.hidden % KS == 0 && M > 32 &&
           n * cfg.hidden * 2 < ((int64_t)1 << 32) && (int64_t)M * cfg.hidden * 2 < ((int64_t)1 << 32);
}

hipError_t fc_launch_project_gemm(const FcGeom &G, const void *x, const void *w, const void *bias,
                                  const int32_t *pos, int win_start, int A, void *q_out, void *k_layer,
                                  void *v_layer, hipStream_t s)
{
    GemmArgs a;
    a.X = (const uint16_t *)x;
    a.W = (const uint16_t *)w;
    a.bias = (const uint16_t *)bias;
    a.pos = pos;
    a.Q = (uint16_t *)q_out;
    a.Kc = (uint16_t *)k_layer;
    a.Vc = (uint16_t *)v_layer;
    a.G = G;
    a.M = G.B * A;
    a.A = A;
    a.K = G.d;
    a.win_start = win_start;
    a.n_mt = a.n_units = 0;
    a.log2_base_64 = G.log_base * 1.4426950408889634074 / 64.0;
    // Tile choice: the largest tile that still gives the chip about one workgroup per compute unit.
    const int slots = G.Hq + 2 * G.Hkv;
    int shape = 0;  // 0: 256 rows x head, 1: 128 rows x head, 2: 128 rows x half head
    if ((int64_t)slots * ((a.M + 255) / 256) < 192) shape = (int64_t)slots * ((a.M + 127) / 128) >= 144 ? 1 : 2;
    if (const char *e = getenv("FC_PROJ_GEMM_SHAPE")) shape = atoi(e);  // tuning knob
    if (shape == 0) return launch_gemm<8, 4>(a, s);
    if (shape == 1) return launch_gemm<4, 4>(a, s);
    return launch_gemm<4, 2>(a, s);
}
