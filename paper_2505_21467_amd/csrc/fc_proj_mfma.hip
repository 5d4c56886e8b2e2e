// QKV projection of the active rows on the matrix cores (bf16, head_dim 128), fused with bias, rotary
// embedding and the scatter into the cache.
//
// The window is short (tens to a few hundred rows), so the product Y^T = W X^T is bound by streaming
// the weight matrix once from HBM.  Both operands are contiguous along the hidden dimension, which is
// exactly the per-lane operand layout of v_mfma_f32_16x16x32_bf16 (8 consecutive k per lane), so W and
// X fragments are loaded straight from global memory into operand registers: no LDS, no transposes.
//
// A workgroup owns 16 rows of W -- 8 rows i0..i0+7 of one head and their rotary partners
// i0+64..i0+71 -- and up to 32 rows of X.  Its eight waves split the hidden dimension; every wave
// issues all loads of its slice (weights from HBM, activations from L2) before the first multiply, so
// there is no dependent chain of memory latencies, and the partial tiles are summed through LDS.  In the
// 16x16 accumulator layout a lane holds 4 consecutive head-dim indices of one window row, and the
// rotary partner of every value sits in the lane 32 away, so the rotation needs one cross-lane swap.
// The rotated q goes to q_out; k and v go directly to their cache rows (v into the transposed tiles).
#include <stdlib.h>

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
    double log2_base_64;   // log2(rope_base) / 64
    float *partials;       // cache scratch: partial tiles of the hidden-dimension slices
};


#ifndef FC_PROJ_VARIANT
#define FC_PROJ_VARIANT 0  // tuning builds: 1 = no activation loads, 2 = no weight loads
#endif
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

// NW = waves per workgroup (they split the hidden dimension), KS = k-steps (of 32) per wave when
// known at compile time (then every load of the wave is issued before the first multiply), 0 = loop.
template <int MT, int NW, int KS>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_proj_skinny(ProjArgs p)
{
    __shared__ float red[NW - 1][MT][4][64];
    __shared__ float2 cs[16 * MT][8];  // (cos, sin) for (window row of this chunk, rotary index i0 + e)
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
    const int kq = p.K / NW;  // hidden elements per wave
    const int m0 = mc * (16 * MT);

    const uint16_t *wrow = p.W + (size_t)n * p.K + (size_t)wave * kq + 8 * q;
    const uint16_t *xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int m = m0 + 16 * mt + rho;
        if (m >= p.M) m = p.M - 1;  // padding rows of the last chunk read a valid row; never stored
        xrow[mt] = p.X + (size_t)m * p.K + (size_t)wave * kq + 8 * q;
    }

    // Rotary factors for this workgroup's rows and its 8 rotary indices, one (or two) per thread.
    // The angle pos * inv_freq is formed and reduced to a fraction of a turn in double; the
    // hardware sine/cosine take their argument in turns.  Called once the loads are in flight: the
    // table does not depend on them and their latency covers it.
    auto rope_table = [&]() {
        if (hs >= G.Hq + G.Hkv) return;
        for (int idx = tid; idx < 16 * MT * 8; idx += NW * 64) {
            const int lr = idx >> 3, e = idx & 7;
            const int m = min(m0 + lr, p.M - 1);
            const int pp = p.pos ? p.pos[m] : p.win_start + (m % p.A);
            // rope_base^(-2i/128) = 2^(-i * log2(base) / 64), evaluated in double
            const double inv_freq = exp2(-(double)(i0 + e) * p.log2_base_64);
            const double turns = (double)pp * inv_freq * 0.15915494309189533576888;
            const float fr = (float)(turns - rint(turns));
            cs[lr][e] = make_float2(__builtin_amdgcn_cosf(fr), __builtin_amdgcn_sinf(fr));
        }
    };

    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (KS > 0) {
        // All weight loads of the wave and the first half of its activation loads are issued before
        // the first multiply; the second half follows once the first has been consumed, which keeps
        // the kernel within 128 registers so that two workgroups share a compute unit.
        constexpr int H = KS / 2;
        bf16x8 wf[KS > 0 ? KS : 1], xf[MT][H > 0 ? H : 1];
#pragma unroll
        for (int s = 0; s < KS; ++s) wf[s] = (FC_PROJ_VARIANT == 2) ? bf16x8{} : ld8(wrow + 32 * s);
#pragma unroll
        for (int s = 0; s < H; ++s)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xf[mt][s] = (FC_PROJ_VARIANT == 1) ? wf[s] : ld8(xrow[mt] + 32 * s);
        __builtin_amdgcn_sched_barrier(0);
        rope_table();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < H; ++s)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[s], xf[mt][s], acc[mt], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < H; ++s)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xf[mt][s] = (FC_PROJ_VARIANT == 1) ? wf[H + s] : ld8(xrow[mt] + 32 * (H + s));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < H; ++s)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[H + s], xf[mt][s], acc[mt], 0, 0, 0);
    } else {
        const int ks = kq >> 5;
        rope_table();
        for (int s = 0; s < ks; ++s) {
            const bf16x8 wfrag = ld8(wrow + 32 * s);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfrag, ld8(xrow[mt] + 32 * s), acc[mt], 0, 0, 0);
        }
    }

    // sum the partial tiles of the NW waves in wave 0
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
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int w2 = 0; w2 < NW - 1; ++w2) acc[mt][r] += red[w2][mt][r][lane];

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
                const float2 f = cs[16 * mt + rho][4 * (q & 1) + r];
                y[r] = second ? y[r] * f.x + other * f.y : y[r] * f.x - other * f.y;
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

// -------------------------------------------------------------------------------------------------
// Head-split kernel for windows of at most 32 rows and hidden sizes that are multiples of 512.
//
// A workgroup owns one whole head slot (128 rows of W: 8 waves x 16 rows) and one 512-wide slice of
// the hidden dimension, so the 32 x 512 slice of X is fetched once per workgroup (direct-to-LDS,
// swizzled) and shared by the 8 waves instead of being re-read by every 16-row tile.  The partial
// tiles of the hidden-dimension slices of a head go to the cache's device scratch and are summed
// by k_proj_finish.
constexpr int HS_K = 512;  // hidden elements per workgroup

__device__ __forceinline__ void load_lds16p(const void *g, void *l)
{
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)g,
                                     (void __attribute__((address_space(3))) *)l, 16, 0, 0);
}

template <int MT>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_proj_headsplit(ProjArgs p)
{
    __shared__ __align__(1024) unsigned char xs[16 * MT * 1024];  // X slice: [row][64 chunks of 16 B]
    const int S = p.K / HS_K;
    const int hs = blockIdx.x / S, ks = blockIdx.x % S;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rho = lane & 15, q = lane >> 4;
    const int i0 = wave * 8;
    const int n = hs * 128 + (rho < 8 ? i0 + rho : 64 + i0 + rho - 8);

    // X slice -> LDS: one 1 KB row per wave-wide load; chunk c of row m is stored at c ^ (m & 15)
#pragma unroll
    for (int i = 0; i < 2 * MT; ++i) {
        const int m = wave * 2 * MT + i;
        const int mg = min(m, p.M - 1);
        const int c = lane ^ (m & 15);
        load_lds16p(p.X + (size_t)mg * p.K + (size_t)ks * HS_K + c * 8, xs + m * 1024);
    }
    // W fragments of this wave's 16 rows: all 16 k-steps in flight
    const uint16_t *wrow = p.W + (size_t)n * p.K + (size_t)ks * HS_K + 8 * q;
    bf16x8 wf[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) wf[s] = ld8(wrow + 32 * s);
    __builtin_amdgcn_sched_barrier(0);

    __syncthreads();  // waits for every load of the workgroup, X slice included

    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 16; ++s)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = 16 * mt + rho;
            const bf16x8 xf = *(const bf16x8 *)(xs + m * 1024 + (((4 * s + q) ^ (m & 15)) << 4));
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[s], xf, acc[mt], 0, 0, 0);
        }

    // hand the partial tile over: [head][slice][wave][mt][r][lane]
    float *part = p.partials + ((((size_t)hs * S + ks) * 8 + wave) * MT) * 256;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[mt * 256 + r * 64 + lane] = acc[mt][r];
}

// Second half of the head-split projection: one wave per (head slot, 16-row tile) sums the partial
// tiles of the hidden-dimension slices (a kernel boundary is the only cross-workgroup ordering used:
// device-scope fences inside a kernel cost an L2 write-back per workgroup on this multi-die part),
// then applies bias and rotary embedding and scatters q, k and v.  Rotary factors are computed per
// lane: base^(-i/64) by binary powering in double, the angle reduced to a fraction of a turn in
// double, hardware sine/cosine (argument in turns).
template <int MT>
__global__ __launch_bounds__(64) void k_proj_finish(ProjArgs p)
{
    const FcGeom &G = p.G;
    const int S = p.K / HS_K;
    const int hs = blockIdx.x >> 3, wave = blockIdx.x & 7;  // the wave index of the first kernel = tile
    const int lane = threadIdx.x;
    const int rho = lane & 15, q = lane >> 4;
    const int i0 = wave * 8;

    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int kb = 0; kb < S; kb += 8) {  // eight slices' worth of loads in flight at a time
        float v[8][MT][4];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k2 = min(kb + u, S - 1);
            const float *pp2 = p.partials + ((((size_t)hs * S + k2) * 8 + wave) * MT) * 256;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) v[u][mt][r] = pp2[mt * 256 + r * 64 + lane];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (kb + u < S) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[mt][r] += v[u][mt][r];
            }
    }

    const bool second = q >= 2;
    const int ib = i0 + 4 * (q & 1);
    const int d0 = (second ? 64 : 0) + ib;
    const bool rotate = hs < G.Hq + G.Hkv;
    double freq[4];  // base^(-(ib + r)/64) / (2 pi): turns per position
    if (rotate) {
        const double r1 = exp2(-p.log2_base_64);
        double f = 0.15915494309189533576888, b2 = r1;
#pragma unroll
        for (int bit = 0; bit < 6; ++bit) {
            if (ib & (1 << bit)) f *= b2;
            b2 *= b2;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            freq[r] = f;
            f *= r1;
        }
    }
    float bs[4] = {0.f, 0.f, 0.f, 0.f};
    if (p.bias) {
#pragma unroll
        for (int r = 0; r < 4; ++r) bs[r] = fc_to_float(bf16_t{p.bias[hs * 128 + d0 + r]});
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + rho;
        const bool mvalid = m < p.M;
        const int mm = mvalid ? m : 0;
        const int b = mm / p.A, a = mm - b * p.A;
        const int pp = p.pos ? p.pos[mm] : p.win_start + a;
        const bool valid = mvalid && pp >= 0 && pp < G.max_seq;
        float y[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) y[r] = acc[mt][r] + bs[r];
        if (rotate) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float other = swap32f(y[r]);
                const double turns = (double)pp * freq[r];
                const float fr = (float)(turns - rint(turns));
                const float c = __builtin_amdgcn_cosf(fr), sn = __builtin_amdgcn_sinf(fr);
                y[r] = second ? y[r] * c + other * sn : y[r] * c - other * sn;
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
    if (a.K % 256 == 0) {  // eight waves split the hidden dimension
        const int ks = a.K / 256;
        if (ks == 14) k_proj_skinny<MT, 8, 14><<<dim3(grid), dim3(512), 0, s>>>(a);
        else if (ks == 16) k_proj_skinny<MT, 8, 16><<<dim3(grid), dim3(512), 0, s>>>(a);
        else k_proj_skinny<MT, 8, 0><<<dim3(grid), dim3(512), 0, s>>>(a);
    } else {
        k_proj_skinny<MT, 4, 0><<<dim3(grid), dim3(256), 0, s>>>(a);
    }
    return hipGetLastError();
}

}  // namespace

bool fc_project_mfma_supported(const fc_config &cfg, int A)
{
    (void)A;
    return cfg.dtype == FC_BF16 && cfg.head_dim == 128 && cfg.hidden % 128 == 0;
}

hipError_t fc_launch_project_mfma(const FcGeom &G, const double *inv_freq, const void *x, const void *w, const void *bias,
                                  const int32_t *pos, int win_start, int A, void *q_out, void *k_layer,
                                  void *v_layer, void *scratch, hipStream_t s)
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
    (void)inv_freq;
    a.log2_base_64 = G.log_base * 1.4426950408889634074 / 64.0;
    a.partials = (float *)scratch;
    const int slots = G.Hq + 2 * G.Hkv;
    const bool no_headsplit = fc_knobs().proj_no_headsplit != 0;  // tuning knob
    if (!no_headsplit && scratch && a.M <= 32 && a.K % HS_K == 0 &&
        (size_t)slots * (a.K / HS_K) * 8 * 2 * 256 * sizeof(float) <= FC_SCRATCH_BYTES) {
        const unsigned grid = (unsigned)(slots * (a.K / HS_K));
        if (a.M <= 16) {
            k_proj_headsplit<1><<<dim3(grid), dim3(512), 0, s>>>(a);
            k_proj_finish<1><<<dim3((unsigned)slots * 8), dim3(64), 0, s>>>(a);
        } else {
            k_proj_headsplit<2><<<dim3(grid), dim3(512), 0, s>>>(a);
            k_proj_finish<2><<<dim3((unsigned)slots * 8), dim3(64), 0, s>>>(a);
        }
        return hipGetLastError();
    }
    if (a.M <= 16) return launch_mt<1>(a, 1, s);
    return launch_mt<2>(a, (a.M + 31) / 32, s);
}
