// Weight-streaming linear layers for short windows (bf16, at most 32 rows per pass): the output
// projection and the two feed-forward matrices of the layer evaluated on the window rows only
// (paper, Table 1, rows "Output projection", "FFN W_1", "FFN W_2" with the row count L replaced by
// the window size A).
//
// With a few dozen rows the product Y^T = W X^T is bound by reading W once from HBM.  Two kernels:
// the slice-wise one described here, for any hidden size that is a multiple of 512, and a whole-row
// one (k_linear_rows, further down) for the hidden sizes whose X block fits in registers.  The weight
// matrix is cut into work items of 128 rows x KSL hidden elements (every row piece is 1 KB, or 512 B,
// of contiguous memory); the items, ordered row slab by row slab, are dealt out in equal contiguous
// runs to one workgroup per compute unit, so the matrix streams once, evenly, whatever its shape.
// Inside an item the eight waves own 16 weight rows each and load them straight into the operand
// registers of v_mfma_f32_16x16x32_bf16 (8 consecutive k per lane); the matching slice of X goes
// through LDS (direct-to-LDS loads, swizzled) and is shared by the waves.  Loads of item i+1 are
// issued before the multiplies of item i.
//
// A run of items may start and end inside a row slab, so every (slab, workgroup) pair that meet
// writes an fp32 partial tile; a second kernel sums a slab's partial tiles (a kernel boundary is
// the only cross-workgroup ordering used) and applies the epilogue: residual add, or the SiLU gate.
// For the gated W_1 a slab holds 64 rows of the gate matrix and the same 64 rows of the up matrix,
// laid out so that g and u of one output sit in lanes 32 apart of the same accumulator register.
#include <stdlib.h>
#include <string.h>

#include "fc_device.h"
#include "fc_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct LinArgs {
    const uint16_t *X;    // [M][K]
    const uint16_t *W;    // [N][K]  (gate matrix in gated mode)
    const uint16_t *W2;   // up matrix [N][K] in gated mode
    const uint16_t *res;  // [M][N] or nullptr
    uint16_t *out;        // [M][N]
    FcArgmaxPart am;      // vocabulary mode: per (slab, row) running maximum, its index, sum of exponentials
    float *partials;      // [m chunk][slab][maxseg][wave][mt][4][64]
    int M, K, N;          // N = output columns
    int S, T, G, maxseg, slabs;
};


__device__ __forceinline__ bf16x8 ld8(const uint16_t *p)
{
    union { uint4 u; bf16x8 v; } x;
    x.u = *(const uint4 *)p;
    return x.v;
}

__device__ __forceinline__ void load_lds16(const void *g, void *l)
{
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)g,
                                     (void __attribute__((address_space(3))) *)l, 16, 0, 0);
}

__device__ __forceinline__ float swap32(float v)
{
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return (threadIdx.x & 32) ? __uint_as_float(r[0]) : __uint_as_float(r[1]);
}

// Workgroup that owns unit u when U units are dealt to G workgroups as runs
// [floor(w U / G), floor((w + 1) U / G)).  A unit is one k-step (32 hidden elements) of one slab.
__host__ __device__ __forceinline__ int owner_of(int64_t u, int64_t U, int G)
{
    return (int)(((u + 1) * G - 1) / U);
}

template <int MT, int KSL, int MODE>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(KSL >= 512 ? 2 : 4, KSL >= 512 ? 2 : 4))) void k_linear_stream(LinArgs p)
{
    constexpr int KS = KSL / 32;        // k-steps of 32 per item
    constexpr int ROWB = KSL * 2;       // bytes of one X row of a slice
    constexpr int RPL = 1024 / ROWB;    // X rows per wave-wide 1 KB load
    constexpr int NLD = 16 * MT / RPL / 8;
    static_assert(NLD >= 1, "slice too narrow for this row count");
    __shared__ __align__(1024) unsigned char xs[2][16 * MT * ROWB];

    const int wg = blockIdx.x, m0 = blockIdx.y * 32;
    // this workgroup's run of k-steps [ulo, uhi): whole items except possibly the first and the last
    const int64_t U = (int64_t)p.T * KS;
    const int64_t ulo = (int64_t)wg * U / p.G, uhi = ((int64_t)wg + 1) * U / p.G;
    const int lo = (int)(ulo / KS), hi = (int)((uhi + KS - 1) / KS);
    const int s_first = (int)(ulo - (int64_t)lo * KS);        // first k-step of item lo
    const int s_last = (int)(uhi - (int64_t)(hi - 1) * KS);   // end of the k-steps of item hi - 1
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rho = lane & 15, q = lane >> 4;

    auto issue = [&](int item, bf16x8(&wf)[KS], unsigned char *xb) {
        const int slab = item / p.S, sl = item - slab * p.S;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int ld = wave * NLD + i;
            const int mrow = ld * RPL + lane / (64 / RPL);
            const int c = (lane % (64 / RPL)) ^ (mrow & 15);  // chunk c of row m is stored at c ^ (m & 15)
            const int mg = min(m0 + mrow, p.M - 1);            // padding rows read a valid row
            load_lds16(p.X + (size_t)mg * p.K + (size_t)sl * KSL + c * 8, xb + ld * 1024);
        }
        const uint16_t *wrow;
        if (MODE == FC_LIN_GATE_UP)
            wrow = (rho < 8 ? p.W : p.W2) + (size_t)(slab * 64 + wave * 8 + (rho & 7)) * p.K;
        else
            wrow = p.W + (size_t)(slab * 128 + wave * 16 + rho) * p.K;
        wrow += (size_t)sl * KSL + 8 * q;
        const int sa = item == lo ? s_first : 0, sb = item == hi - 1 ? s_last : KS;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (s >= sa && s < sb)
                wf[s] = ld8(wrow + 32 * s);
            else
                wf[s] = bf16x8{};  // k-steps of a neighbouring run: contribute nothing
        }
    };

    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](const bf16x8(&wf)[KS], const unsigned char *xb) {
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = 16 * mt + rho;
                const bf16x8 xf = *(const bf16x8 *)(xb + m * ROWB + (((4 * s + q) ^ (m & 15)) << 4));
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[s], xf, acc[mt], 0, 0, 0);
            }
    };

    // hand the partial tile over when the run leaves the slab (or ends)
    auto tail = [&](int item) {
        if (item + 1 < hi && (item + 1) % p.S != 0) return;
        const int slab = item / p.S;
        const int seg = wg - owner_of((int64_t)slab * p.S * KS, U, p.G);
        float *part = p.partials +
                      ((((size_t)blockIdx.y * p.slabs + slab) * p.maxseg + seg) * 8 + wave) * (MT * 256);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                part[mt * 256 + r * 64 + lane] = acc[mt][r];
                acc[mt][r] = 0.f;
            }
    };

    if (ulo >= uhi) return;
    bf16x8 wa[KS], wb[KS];
    issue(lo, wa, xs[0]);
    int item = lo;
    for (;;) {
        __syncthreads();  // the loads of `item` have landed; every wave is done with the other buffers
        if (item + 1 < hi) issue(item + 1, wb, xs[1]);
        compute(wa, xs[0]);
        tail(item);
        if (++item >= hi) break;
        __syncthreads();
        if (item + 1 < hi) issue(item + 1, wa, xs[0]);
        compute(wb, xs[1]);
        tail(item);
        if (++item >= hi) break;
    }
}

// Sum of a slab's partial tiles + epilogue; one wave per (slab, 16-row tile of W), grid.y = m chunk.
template <int MT, int KSL, int MODE>
__global__ __launch_bounds__(64) void k_linear_finish(LinArgs p)
{
    constexpr int KS = KSL / 32;
    const int64_t U = (int64_t)p.T * KS;
    const int slab = blockIdx.x >> 3, wave = blockIdx.x & 7;
    const int m0 = blockIdx.y * 32;
    const int lane = threadIdx.x, rho = lane & 15, q = lane >> 4;
    const int first = owner_of((int64_t)slab * p.S * KS, U, p.G);
    const int nseg = owner_of((int64_t)(slab + 1) * p.S * KS - 1, U, p.G) - first + 1;
    const float *base = p.partials + ((((size_t)blockIdx.y * p.slabs + slab) * p.maxseg) * 8 + wave) * (MT * 256);
    const size_t seg_stride = (size_t)8 * MT * 256;

    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < nseg; s0 += 4) {  // four segments' worth of loads in flight
        float v[4][MT][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float *pp = base + (size_t)min(s0 + u, nseg - 1) * seg_stride;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) v[u][mt][r] = pp[mt * 256 + r * 64 + lane];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (s0 + u < nseg) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[mt][r] += v[u][mt][r];
            }
    }

#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = m0 + 16 * mt + rho;
        const bool mvalid = m < p.M;
        float y[4];
        if (MODE == FC_LIN_GATE_UP) {
            // lanes q = 0, 1 hold the gate products of outputs 4q + r, lanes q = 2, 3 the up products
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float other = swap32(acc[mt][r]);
                const float g = acc[mt][r];
                y[r] = g / (1.0f + expf(-g)) * other;
            }
            if (!mvalid || q >= 2) continue;
            const int f = slab * 64 + wave * 8 + 4 * q;
            uint2 w;
            w.x = (uint32_t)fc_bf16_bits(y[0]) | ((uint32_t)fc_bf16_bits(y[1]) << 16);
            w.y = (uint32_t)fc_bf16_bits(y[2]) | ((uint32_t)fc_bf16_bits(y[3]) << 16);
            *(uint2 *)(p.out + (size_t)m * p.N + f) = w;
        } else {
            if (!mvalid) continue;
            const int n = slab * 128 + wave * 16 + 4 * q;
#pragma unroll
            for (int r = 0; r < 4; ++r) y[r] = acc[mt][r];
            if (p.res) {
                const uint2 rv = *(const uint2 *)(p.res + (size_t)m * p.N + n);
                y[0] += __uint_as_float(rv.x << 16);
                y[1] += __uint_as_float(rv.x & 0xffff0000u);
                y[2] += __uint_as_float(rv.y << 16);
                y[3] += __uint_as_float(rv.y & 0xffff0000u);
            }
            uint2 w;
            w.x = (uint32_t)fc_bf16_bits(y[0]) | ((uint32_t)fc_bf16_bits(y[1]) << 16);
            w.y = (uint32_t)fc_bf16_bits(y[2]) | ((uint32_t)fc_bf16_bits(y[3]) << 16);
            *(uint2 *)(p.out + (size_t)m * p.N + n) = w;
        }
    }
}

// Vocabulary mode (the unmasking step, section 3.1): the outputs of a slab are 128 logits per row, of
// which only the largest, its index and the sum of exp(logit - largest) are kept, per (slab, row); a
// last kernel merges the slabs.  One workgroup per slab: wave wt sums the partial tiles of the slab's
// weight tile wt, the lanes that share a row merge, and one thread per row merges the eight tiles
// (the merge keeps the smaller index on equal maxima, so its order does not matter).
template <int MT, int KSL>
__global__ __launch_bounds__(512) void k_lmhead_finish(LinArgs p)
{
    constexpr int KS = KSL / 32;
    __shared__ float s_mx[8][16 * MT], s_sm[8][16 * MT];
    __shared__ int s_arg[8][16 * MT];
    const int64_t U = (int64_t)p.T * KS;
    const int slab = blockIdx.x, m0 = blockIdx.y * 32;
    const int lane = threadIdx.x & 63, wt = threadIdx.x >> 6;  // wave wt sums the slab's weight tile wt
    const int rho = lane & 15, q = lane >> 4;
    const int first = owner_of((int64_t)slab * p.S * KS, U, p.G);
    const int nseg = owner_of((int64_t)(slab + 1) * p.S * KS - 1, U, p.G) - first + 1;
    const size_t seg_stride = (size_t)8 * MT * 256;
    const float *base = p.partials + ((((size_t)blockIdx.y * p.slabs + slab) * p.maxseg) * 8 + wt) * (MT * 256);
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int sg = 0; sg < nseg; ++sg)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[mt][r] += base[(size_t)sg * seg_stride + mt * 256 + r * 64 + lane];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        // lane (rho, q) holds logits 4q .. 4q + 3 of the tile for row rho, in ascending order
        float mx = -INFINITY, sm = 0.f;
        int arg = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) fc_argmax_merge(mx, arg, sm, acc[mt][r], slab * 128 + wt * 16 + 4 * q + r, 1.0f);
#pragma unroll
        for (int off = 16; off < 64; off <<= 1) {
            const float mx2 = __shfl_xor(mx, off, 64), sm2 = __shfl_xor(sm, off, 64);
            const int arg2 = __shfl_xor(arg, off, 64);
            fc_argmax_merge(mx, arg, sm, mx2, arg2, sm2);
        }
        if (q == 0) {
            s_mx[wt][16 * mt + rho] = mx;
            s_sm[wt][16 * mt + rho] = sm;
            s_arg[wt][16 * mt + rho] = arg;
        }
    }
    __syncthreads();
    const int row = threadIdx.x;  // one thread per row merges the eight tiles
    if (row < 16 * MT && m0 + row < p.M) {
        float mx = s_mx[0][row], sm = s_sm[0][row];
        int arg = s_arg[0][row];
        for (int w2 = 1; w2 < 8; ++w2) fc_argmax_merge(mx, arg, sm, s_mx[w2][row], s_arg[w2][row], s_sm[w2][row]);
        const size_t at = (size_t)slab * p.M + m0 + row;
        p.am.mx[at] = mx;
        p.am.arg[at] = arg;
        p.am.sm[at] = sm;
    }
}


// -------------------------------------------------------------------------------------------------
// Hidden sizes of 512, 3584 and 4096 (the whole activation block fits in registers): whole rows.
//
// A work item is 16 rows of W over the whole hidden dimension (16 x 2K bytes, contiguous in memory);
// the eight waves of a workgroup cut the hidden dimension in eight, and every wave keeps its part of
// the X block (at most 32 rows) in operand registers for the whole kernel, so X is read once per
// workgroup and never again.  The weight fragments of a wave are refilled one by one, right behind
// the multiply that consumed them, with the same fragment of the next item: a full item of loads
// stays in flight and the wave never drains its queue.  The eight partial 16 x 32 tiles of an item
// are summed through LDS (double-buffered: one barrier per item) by the first MT waves, which apply
// the epilogue -- residual add, SiLU gate (an item being 8 gate rows and the same 8 up rows), or the
// running (largest logit, index, sum of exponentials) per row, written once per workgroup at the end.
// No partial sums leave the workgroup and there is no second kernel.  Items are dealt in contiguous
// runs measured in half items (8 rows, or 4 gated features), so runs differ by at most half an item;
// a lane whose half of an item belongs to the neighbouring run re-reads the row of the other half
// (same cache lines: no extra traffic) and its results are dropped.
template <int MT, int NKW, int MODE>
__global__ __launch_bounds__(512) void k_linear_rows(LinArgs p)
{
    __shared__ __align__(16) float red[2][8][MT * 4][64];
    const int wg = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rho = lane & 15, q = lane >> 4;
    const int U = p.T;  // half items
    const int u0 = (int)((int64_t)wg * U / p.G), u1 = (int)(((int64_t)wg + 1) * U / p.G);
    if (u0 >= u1) return;
    const int it0 = u0 >> 1, it1 = (u1 + 1) >> 1;
    const size_t kw0 = (size_t)wave * (NKW * 32) + 8 * q;  // this lane's first hidden element

    bf16x8 xr[NKW][MT];
#pragma unroll
    for (int s = 0; s < NKW; ++s)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = min(16 * mt + rho, p.M - 1);  // padding rows read a valid row
            xr[s][mt] = ld8(p.X + (size_t)m * p.K + kw0 + 32 * s);
        }
    __builtin_amdgcn_sched_barrier(0);

    // this lane's weight row of item `it`
    auto wrow_of = [&](int it) -> const uint16_t * {
        if (MODE == FC_LIN_GATE_UP) {
            int fi = rho & 7;  // feature of the item; half item = 4 features
            const int uu = 2 * it + (fi >> 2);
            if (uu < u0 || uu >= u1) fi ^= 4;
            return (rho < 8 ? p.W : p.W2) + (size_t)(8 * it + fi) * p.K + kw0;
        }
        int r = rho;  // row of the item; half item = 8 rows
        const int uu = 2 * it + (r >> 3);
        if (uu < u0 || uu >= u1) r ^= 8;
        return p.W + (size_t)(16 * it + r) * p.K + kw0;
    };

    bf16x8 wf[NKW];
    {
        const uint16_t *cur = wrow_of(it0);
#pragma unroll
        for (int s = 0; s < NKW; ++s) wf[s] = ld8(cur + 32 * s);
    }
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float run_mx = -INFINITY, run_sm = 0.f;  // vocabulary mode: running state of row 16 mt + rho (lanes q = 0 of wave mt)
    int run_arg = 0x7fffffff;
    int buf = 0;

    // Outputs are collected in LDS and leave as whole row segments (flush): an item gives a row only 16 or
    // 32 bytes, and written item by item those pieces cost the streaming a tenth of its rate (memory
    // switching between reading and writing for every piece); a run's segment of a row is one or two
    // cache lines.  Wave mt stages and flushes its own 16 rows, so no barrier is involved.
    constexpr int HALF_EL = MODE == FC_LIN_GATE_UP ? 4 : 8;  // output columns of a half item
    constexpr int STG_ITEMS = 16;                            // items staged between two flushes
    constexpr int STG_CH = STG_ITEMS * 2 * HALF_EL / 4;      // 8-byte pieces of a staged row (at most 64)
    __shared__ uint2 stage[MODE == FC_LIN_VOCAB ? 1 : MT * 16][STG_CH + 1];
    int stage_it0 = it0;  // item in the first staging slot
    auto flush = [&](int it_end) {  // items stage_it0 .. it_end - 1 are staged
        const int c0 = max(u0 * HALF_EL, stage_it0 * 2 * HALF_EL), c1 = min(u1 * HALF_EL, it_end * 2 * HALF_EL);
        const int nch = (c1 - c0) >> 2, ch0 = (c0 - stage_it0 * 2 * HALF_EL) >> 2;
#pragma unroll 4
        for (int r = 0; r < 16; ++r) {
            const int m = 16 * wave + r;
            if (m < p.M && lane < nch) *(uint2 *)(p.out + (size_t)m * p.N + c0 + 4 * lane) = stage[m][ch0 + lane];
        }
    };

    // Sum of the eight partial tiles of item `it` (in red[rb]) and epilogue, by wave mt < MT for tile mt.
    auto finish_item = [&](int it, int rb) {
        if (MODE != FC_LIN_VOCAB && it - stage_it0 == STG_ITEMS) {
            flush(it);
            stage_it0 = it;
        }
        // wave mt sums tile mt: lane (rho, q) = X row 16 mt + rho, item rows 4 q .. 4 q + 3
        const int mt = wave, m = 16 * mt + rho;
        float sum[4] = {0.f, 0.f, 0.f, 0.f}, sum2[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w2 = 0; w2 < 8; ++w2)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                sum[r] += red[rb][w2][mt * 4 + r][lane];
                if (MODE == FC_LIN_GATE_UP) sum2[r] += red[rb][w2][mt * 4 + r][lane ^ 32];  // up rows: 8 item rows on
            }
        if (MODE == FC_LIN_GATE_UP) {
            const int uu = 2 * it + (q & 1);
            if (q < 2 && m < p.M && uu >= u0 && uu < u1) {
                float y[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) y[r] = sum[r] / (1.0f + expf(-sum[r])) * sum2[r];
                uint2 o;
                o.x = (uint32_t)fc_bf16_bits(y[0]) | ((uint32_t)fc_bf16_bits(y[1]) << 16);
                o.y = (uint32_t)fc_bf16_bits(y[2]) | ((uint32_t)fc_bf16_bits(y[3]) << 16);
                stage[m][(it - stage_it0) * 2 + q] = o;
            }
        } else if (MODE == FC_LIN_RESIDUAL) {
            const int uu = 2 * it + (q >> 1);
            if (m < p.M && uu >= u0 && uu < u1) {
                const size_t at = (size_t)m * p.N + 16 * it + 4 * q;
                if (p.res) {
                    const uint2 rv = *(const uint2 *)(p.res + at);
                    sum[0] += __uint_as_float(rv.x << 16);
                    sum[1] += __uint_as_float(rv.x & 0xffff0000u);
                    sum[2] += __uint_as_float(rv.y << 16);
                    sum[3] += __uint_as_float(rv.y & 0xffff0000u);
                }
                uint2 o;
                o.x = (uint32_t)fc_bf16_bits(sum[0]) | ((uint32_t)fc_bf16_bits(sum[1]) << 16);
                o.y = (uint32_t)fc_bf16_bits(sum[2]) | ((uint32_t)fc_bf16_bits(sum[3]) << 16);
                stage[m][(it - stage_it0) * 4 + q] = o;
            }
        } else {
            // the item's 16 logits of a row: four per lane in ascending order, then the four lanes of the row
            const int uu = 2 * it + (q >> 1);
            float mx = -INFINITY, sm = 0.f;
            int arg = 0x7fffffff;
            if (uu >= u0 && uu < u1) {
#pragma unroll
                for (int r = 0; r < 4; ++r) fc_argmax_merge(mx, arg, sm, sum[r], 16 * it + 4 * q + r, 1.0f);
            }
#pragma unroll
            for (int off = 16; off < 64; off <<= 1) {
                const float mx2 = __shfl_xor(mx, off, 64), sm2 = __shfl_xor(sm, off, 64);
                const int arg2 = __shfl_xor(arg, off, 64);
                fc_argmax_merge(mx, arg, sm, mx2, arg2, sm2);
            }
            fc_argmax_merge(run_mx, run_arg, run_sm, mx, arg, sm);
        }
    };

    for (int it = it0; it < it1; ++it) {
        // The previous item is finished here, one iteration late: what it loads or stores is then issued
        // behind the wait for this item's fragments and never part of it.
        __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8) | (0 << 14));  // vmcnt(0): this item's fragments have landed
        __builtin_amdgcn_sched_barrier(0);
        if (it > it0 && wave < MT) finish_item(it - 1, buf ^ 1);
        __builtin_amdgcn_sched_barrier(0);
        // Fragment s of the next item goes into its register as soon as the multiplies of fragment s are
        // issued.  After the last item every lane re-reads the first 16 bytes of W instead (never used):
        // unconditional loads keep the compiler's wait counts exact.
        const bool has_next = it + 1 < it1;
        const uint16_t *nxt = has_next ? wrow_of(it + 1) : p.W;
        const int nstep = has_next ? 32 : 0;
#pragma unroll
        for (int s = 0; s < NKW; ++s) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[s], xr[s][mt], acc[mt], 0, 0, 0);
            wf[s] = ld8(nxt + nstep * s);
        }
        float *mine = &red[buf][wave][0][lane];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                mine[(mt * 4 + r) * 64] = acc[mt][r];
                acc[mt][r] = 0.f;
            }
        __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14));  // lgkmcnt(0): the tile is in LDS
        __builtin_amdgcn_s_barrier();
        buf ^= 1;
    }
    if (wave < MT) {
        finish_item(it1 - 1, buf ^ 1);
        if (MODE != FC_LIN_VOCAB) flush(it1);
    }
    if (MODE == FC_LIN_VOCAB && wave < MT && q == 0 && 16 * wave + rho < p.M) {
        const size_t at = (size_t)wg * p.M + 16 * wave + rho;
        p.am.mx[at] = run_mx;
        p.am.arg[at] = run_arg;
        p.am.sm[at] = run_sm;
    }
}

#ifndef FC_LIN_KSL
#define FC_LIN_KSL 512
#endif
constexpr int KSL = FC_LIN_KSL;  // hidden elements per work item

template <int MODE>
hipError_t launch_mode(const FcSkinnyPlan &pl, const LinArgs &a, hipStream_t s)
{
    const dim3 g1((unsigned)pl.G, (unsigned)pl.chunks), g2((unsigned)pl.slabs * 8, (unsigned)pl.chunks);
    if (pl.mt == 1) {
        k_linear_stream<1, KSL, MODE><<<g1, dim3(512), 0, s>>>(a);
        k_linear_finish<1, KSL, MODE><<<g2, dim3(64), 0, s>>>(a);
    } else {
        k_linear_stream<2, KSL, MODE><<<g1, dim3(512), 0, s>>>(a);
        k_linear_finish<2, KSL, MODE><<<g2, dim3(64), 0, s>>>(a);
    }
    return hipGetLastError();
}

template <int MT, int NKW>
hipError_t launch_rows(int mode, const FcSkinnyPlan &pl, const LinArgs &a, hipStream_t s)
{
    const dim3 g((unsigned)pl.G), b(512);
    if (mode == FC_LIN_GATE_UP) k_linear_rows<MT, NKW, FC_LIN_GATE_UP><<<g, b, 0, s>>>(a);
    else if (mode == FC_LIN_VOCAB) k_linear_rows<MT, NKW, FC_LIN_VOCAB><<<g, b, 0, s>>>(a);
    else k_linear_rows<MT, NKW, FC_LIN_RESIDUAL><<<g, b, 0, s>>>(a);
    return hipGetLastError();
}

// hidden sizes the whole-row kernel is built for (256 x the fragments per wave)
bool rows_kernel_covers(int K) { return K == 512 || K == 3584 || K == 4096; }

}  // namespace

FcSkinnyPlan fc_plan_skinny(int dtype, int mode, int M, int K, int N)
{
    FcSkinnyPlan p;
    memset(&p, 0, sizeof p);
    int target = 256;  // one workgroup per compute unit
    if (fc_knobs().lin_wgs > 0) target = fc_knobs().lin_wgs;  // tuning and test knob: runs of any length
    {
        // whole-row kernel: at most 32 rows, a hidden size it is built for, whole half items
        const bool off = fc_knobs().lin_no_rows != 0;  // tuning knob
        const int per_half = mode == FC_LIN_GATE_UP ? 4 : 8;
        // With less than one item per compute unit at a long hidden size (W_out of the 7B geometry: 224
        // items) the X block, K x 64 bytes per workgroup, is a third of what a workgroup reads, and the
        // slice-wise kernel below, which reads only the slices it needs, is as fast (12.2 against 12.8 us).
        const int items = N >= per_half && N % per_half == 0 ? (N / per_half + 1) / 2 : 0;
        if (!off && dtype == FC_BF16 && M >= 1 && M <= 32 && rows_kernel_covers(K) && items >= 1 &&
            (items >= 256 || K < 2048)) {
            p.kind = 2;
            p.mt = M <= 16 ? 1 : 2;
            p.chunks = 1;
            p.T = N / per_half;               // half items
            p.G = items < target ? items : target;  // at least one item each
            return p;
        }
    }
    const int rows_per_slab = mode == FC_LIN_GATE_UP ? 64 : 128;  // FC_LIN_VOCAB: slabs of 128 vocabulary rows
    if (dtype != FC_BF16 || M < 1 || K < KSL || K % KSL != 0 || N < rows_per_slab || N % rows_per_slab != 0)
        return p;  // kind 0: plain kernel, no workspace
    p.kind = 1;
    p.mt = M <= 16 ? 1 : 2;
    p.chunks = M <= 16 ? 1 : (M + 31) / 32;
    p.slabs = N / rows_per_slab;
    p.S = K / KSL;
    const int64_t T = (int64_t)p.slabs * p.S;
    if (T > (1 << 26) || p.chunks > 65535) {
        p.kind = 0;
        return p;
    }
    p.T = (int)T;
    p.G = p.T < target ? p.T : target;
    // runs are measured in k-steps of 32 hidden elements, so every workgroup streams the same
    // amount to within one k-step; a slab of S * KS k-steps meets at most this many runs
    const int64_t per_slab = (int64_t)p.S * (KSL / 32), upw = T * (KSL / 32) / p.G;
    const int64_t bound = (per_slab + upw - 1) / upw + 1;
    p.maxseg = (int)(bound < p.G ? bound : p.G);
    return p;
}

size_t fc_skinny_workspace(const FcSkinnyPlan &p)
{
    if (p.kind != 1) return 0;  // the whole-row kernel keeps its partial sums inside the workgroup
    return (size_t)p.chunks * p.slabs * p.maxseg * 8 * p.mt * 256 * sizeof(float);
}

hipError_t fc_launch_linear_skinny(const FcSkinnyPlan &pl, int mode, const void *x, const void *w, const void *w2,
                                   const void *res, int M, int K, int N, void *out, void *workspace,
                                   hipStream_t s, const FcArgmaxPart *am)
{
    if (pl.kind == 2) {
        if (M < 1 || M > 32 || !rows_kernel_covers(K) || pl.G < 1 || pl.T < 1 || pl.G > (pl.T + 1) / 2 ||
            (mode == FC_LIN_VOCAB && !am))
            return hipErrorInvalidValue;
        LinArgs a;
        memset(&a, 0, sizeof a);
        a.X = (const uint16_t *)x;
        a.W = (const uint16_t *)w;
        a.W2 = (const uint16_t *)w2;
        a.res = (const uint16_t *)res;
        a.out = (uint16_t *)out;
        if (am) a.am = *am;
        a.M = M;
        a.K = K;
        a.N = N;
        a.T = pl.T;
        a.G = pl.G;
        const int nkw = K / 256;
        if (pl.mt == 1) {
            if (nkw == 2) return launch_rows<1, 2>(mode, pl, a, s);
            if (nkw == 14) return launch_rows<1, 14>(mode, pl, a, s);
            return launch_rows<1, 16>(mode, pl, a, s);
        }
        if (nkw == 2) return launch_rows<2, 2>(mode, pl, a, s);
        if (nkw == 14) return launch_rows<2, 14>(mode, pl, a, s);
        return launch_rows<2, 16>(mode, pl, a, s);
    }
    // The kernels index the partial tiles by (slab, position of the workgroup among those that meet
    // the slab); make sure on the host that no slab meets more workgroups than the plan reserved.
    for (int slab = 0; slab < pl.slabs; ++slab) {
        const int64_t per_slab = (int64_t)pl.S * (KSL / 32), U = (int64_t)pl.T * (KSL / 32);
        const int first = owner_of(slab * per_slab, U, pl.G), last = owner_of((slab + 1) * per_slab - 1, U, pl.G);
        if (last - first + 1 > pl.maxseg) return hipErrorInvalidValue;
    }
    if (pl.kind != 1 || pl.G < 1 || pl.G > pl.T || M > pl.chunks * 32 || !workspace) return hipErrorInvalidValue;
    LinArgs a;
    memset(&a, 0, sizeof a);
    a.X = (const uint16_t *)x;
    a.W = (const uint16_t *)w;
    a.W2 = (const uint16_t *)w2;
    a.res = (const uint16_t *)res;
    a.out = (uint16_t *)out;
    a.partials = (float *)workspace;
    a.M = M;
    a.K = K;
    a.N = N;
    a.S = pl.S;
    a.T = pl.T;
    a.G = pl.G;
    a.maxseg = pl.maxseg;
    a.slabs = pl.slabs;
    if (mode == FC_LIN_VOCAB) {
        if (!am) return hipErrorInvalidValue;
        a.am = *am;
        const dim3 g1((unsigned)pl.G, (unsigned)pl.chunks), g2((unsigned)pl.slabs, (unsigned)pl.chunks);
        if (pl.mt == 1) {
            k_linear_stream<1, KSL, FC_LIN_RESIDUAL><<<g1, dim3(512), 0, s>>>(a);
            k_lmhead_finish<1, KSL><<<g2, dim3(512), 0, s>>>(a);
        } else {
            k_linear_stream<2, KSL, FC_LIN_RESIDUAL><<<g1, dim3(512), 0, s>>>(a);
            k_lmhead_finish<2, KSL><<<g2, dim3(512), 0, s>>>(a);
        }
        return hipGetLastError();
    }
    return mode == FC_LIN_GATE_UP ? launch_mode<FC_LIN_GATE_UP>(pl, a, s) : launch_mode<FC_LIN_RESIDUAL>(pl, a, s);
}
