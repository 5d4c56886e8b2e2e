// QKV projection of the active rows on the matrix cores (bf16, head_dim 128), fused with bias, rotary
// embedding and the scatter into the cache.
//
// The window is short (tens to a few hundred rows), so the product Y^T = W X^T is bound by streaming
// the weight matrix once from HBM.  Both operands are contiguous along the hidden dimension, which is
// exactly the per-lane operand layout of v_mfma_f32_16x16x32_bf16 (8 consecutive k per lane), so W and
// X fragments are loaded straight from global memory into operand registers: no LDS, no transposes.
//
// A workgroup owns 16 rows of W -- 8 rows i0..i0+7 of one head and their rotary partners
// i0+64..i0+71 -- and up to 64 rows of X.  Its four waves split the hidden dimension; every wave
// issues all loads of its quarter of the 16 weight rows up front (about 30 KB in flight per wave, which
// is what keeps HBM busy), multiplies, and the four partial tiles are summed through LDS.  In the
// 16x16 accumulator layout a lane holds 4 consecutive head-dim indices of one window row, and the
// rotary partner of every value sits in the lane 32 away, so the rotation needs one cross-lane swap.
// The rotated q goes to q_out; k and v go directly to their cache rows (v into the transposed tiles).
#include "fc_device.h"
#include "fc_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct ProjArgs {
    const uint16_t *X;     // [M][K]
    const uint16_t *W;     // [N][K]
    const uint16_t *bias;  // [N] or nullptr
    const int32_t *pos;    // [M] or nullptr
    uint16_t *Q;           // [B][Hq][A][128]
    uint16_t *Kc;          // one layer
    uint16_t *Vc;          // one layer
    FcGeom G;
    int M, A, K, win_start, n_tiles;
};

__device__ __forceinline__ bf16x8 ld8(const uint16_t *p)
{
    union { uint4 u; bf16x8 v; } x;
    x.u = *(const uint4 *)p;
    return x.v;
}

__device__ __forceinline__ float swap32f(float v)
{
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    // r[0] = lower half in all lanes, r[1] = upper half in all lanes
    return (threadIdx.x & 32) ? __uint_as_float(r[0]) : __uint_as_float(r[1]);
}

// KS = k-steps (of 32) per wave when known at compile time, 0 = runtime loop.
template <int MT, int KS>
__global__ __launch_bounds__(256) void k_proj_skinny(ProjArgs p)
{
    __shared__ float red[3][MT][4][64];
    const FcGeom &G = p.G;
    // workgroup id -> (m chunk, n tile): chunks of one n tile have ids equal modulo 8 (same XCD)
    const int tiles8 = (p.n_tiles + 7) & ~7;
    const int mc = blockIdx.x / tiles8, tile = blockIdx.x % tiles8;
    if (tile >= p.n_tiles) return;
    const int hs = tile >> 3, i0 = (tile & 7) * 8;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rho = lane & 15, q = lane >> 4;
    const int n = hs * 128 + (rho < 8 ? i0 + rho : 64 + i0 + rho - 8);
    const int kq = p.K >> 2;  // hidden elements per wave
    const int m0 = mc * (16 * MT);

    const uint16_t *wrow = p.W + (size_t)n * p.K + (size_t)wave * kq + 8 * q;
    const uint16_t *xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int m = m0 + 16 * mt + rho;
        if (m >= p.M) m = p.M - 1;  // padding rows of the last chunk read a valid row; never stored
        xrow[mt] = p.X + (size_t)m * p.K + (size_t)wave * kq + 8 * q;
    }

    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (KS > 0) {
        bf16x8 wf[KS > 0 ? KS : 1];
#pragma unroll
        for (int s = 0; s < KS; ++s) wf[s] = ld8(wrow + 32 * s);
        bf16x8 xf[2][MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int s = 0; s < 4; ++s) xf[0][mt][s] = ld8(xrow[mt] + 32 * s);
#pragma unroll
        for (int c = 0; c < KS / 4; ++c) {
            if (c + 1 < KS / 4) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int s = 0; s < 4; ++s) xf[(c + 1) & 1][mt][s] = ld8(xrow[mt] + 32 * (4 * (c + 1) + s));
            }
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[4 * c + s], xf[c & 1][mt][s], acc[mt], 0, 0, 0);
        }
    } else {
        const int ks = kq >> 5;
        for (int s = 0; s < ks; ++s) {
            const bf16x8 wfrag = ld8(wrow + 32 * s);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfrag, ld8(xrow[mt] + 32 * s), acc[mt], 0, 0, 0);
        }
    }

    // sum the four hidden-dimension quarters in wave 0
    if (wave > 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[wave - 1][mt][r][lane] = acc[mt][r];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[mt][r] += red[0][mt][r][lane] + red[1][mt][r][lane] + red[2][mt][r][lane];

    // lane (rho, q) holds W rows 4q..4q+3 of the tile for window row rho of each m tile:
    // q = 0,1 -> head-dim i0 + 4q + r; q = 2,3 -> 64 + i0 + 4(q-2) + r (the rotary partners)
    const bool second = q >= 2;
    const int ib = i0 + 4 * (q & 1);           // rotary index of r = 0
    const int d0 = (second ? 64 : 0) + ib;     // head-dim index of r = 0
    float bs[4] = {0.f, 0.f, 0.f, 0.f};
    if (p.bias) {
#pragma unroll
        for (int r = 0; r < 4; ++r) bs[r] = fc_to_float(bf16_t{p.bias[hs * 128 + d0 + r]});
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = m0 + 16 * mt + rho;
        const bool mvalid = m < p.M;
        const int mm = mvalid ? m : 0;
        const int b = mm / p.A, a = mm - b * p.A;
        const int pp = p.pos ? p.pos[mm] : p.win_start + a;
        const bool valid = mvalid && pp >= 0 && pp < G.max_seq;
        float y[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) y[r] = acc[mt][r] + bs[r];
        if (hs < G.Hq + G.Hkv) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float other = swap32f(y[r]);
                float c, s;
                fc_rope_cs(valid ? pp : 0, ib + r, 128, G.log_base, &c, &s);
                y[r] = second ? y[r] * c + other * s : y[r] * c - other * s;
            }
        }
        uint2 w;
        w.x = (uint32_t)fc_bf16_bits(y[0]) | ((uint32_t)fc_bf16_bits(y[1]) << 16);
        w.y = (uint32_t)fc_bf16_bits(y[2]) | ((uint32_t)fc_bf16_bits(y[3]) << 16);
        if (hs < G.Hq) {
            if (mvalid) {
                if (!valid) w = make_uint2(0, 0);
                *(uint2 *)(p.Q + (((size_t)b * G.Hq + hs) * p.A + a) * 128 + d0) = w;
            }
        } else if (valid) {
            if (hs < G.Hq + G.Hkv) {
                *(uint2 *)(p.Kc + fc_k_index(G, b, hs - G.Hq, pp, d0)) = w;
            } else {
                const int j = hs - G.Hq - G.Hkv;
#pragma unroll
                for (int r = 0; r < 4; ++r) p.Vc[fc_v_index(G, b, j, pp, d0 + r)] = fc_bf16_bits(y[r]);
            }
        }
    }
}

template <int MT>
hipError_t launch_mt(const ProjArgs &a, int m_chunks, hipStream_t s)
{
    const unsigned grid = (unsigned)(((a.n_tiles + 7) & ~7) * m_chunks);
    const int ks = a.K / 128;
    if (ks == 28) k_proj_skinny<MT, 28><<<dim3(grid), dim3(256), 0, s>>>(a);
    else if (ks == 32) k_proj_skinny<MT, 32><<<dim3(grid), dim3(256), 0, s>>>(a);
    else k_proj_skinny<MT, 0><<<dim3(grid), dim3(256), 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace

bool fc_project_mfma_supported(const fc_config &cfg, int A)
{
    (void)A;
    return cfg.dtype == FC_BF16 && cfg.head_dim == 128 && cfg.hidden % 128 == 0;
}

hipError_t fc_launch_project_mfma(const FcGeom &G, const void *x, const void *w, const void *bias,
                                  const int32_t *pos, int win_start, int A, void *q_out, void *k_layer,
                                  void *v_layer, hipStream_t s)
{
    ProjArgs a;
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
    a.n_tiles = (G.Hq + 2 * G.Hkv) * 8;
    if (a.M <= 16) return launch_mt<1>(a, 1, s);
    if (a.M <= 32) return launch_mt<2>(a, 1, s);
    return launch_mt<4>(a, (a.M + 63) / 64, s);
}
