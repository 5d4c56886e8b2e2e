// Active-query attention on the matrix cores (bf16, head_dim 128), split over the key axis.
//
// Work decomposition.  For one (sequence, kv head) the g*A query rows (head-in-group major, then
// window row) are cut into 32-row tiles.  A workgroup owns R row tiles and one contiguous key range
// ("split"); its W waves each own one row tile and, when W = 2R, one 32-key half of every 64-key
// stage.  K rows and transposed V tiles stream HBM -> registers -> LDS as 16-byte coalesced chunks,
// double buffered; every wave reads its operands from LDS.
//
// Per 32 keys a wave computes S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (K rows are the A operand,
// so each lane ends up holding 16 scores of ONE query row), does the online-softmax update with a
// single cross-lane exchange (lanes l and l^32 hold the two halves of a row), and feeds the
// probabilities, converted to bf16 in place, straight back as the B operand of O^T += V^T P^T.  The
// key order inside a 32-key group is permuted on the K side (bits 2 and 3 of the row index
// swapped) so that the accumulator layout of S^T is exactly the operand layout P^T needs for
// natural-order V^T rows: no shuffles and no LDS round trip for P.
//
// Each split writes unnormalised partial outputs with their running max and sum; a small second
// kernel merges the splits.  With one split the first kernel writes the final output itself.
#include "fc_device.h"
#include "fc_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int DH = 128;
constexpr int KT = 64;                         // keys per LDS stage (= one transposed V tile)
constexpr int K_STRIDE = 272;                  // bytes per key row in LDS: 256 + 16 of padding
constexpr int V_STRIDE = 144;                  // bytes per head-dim row of V^T in LDS: 128 + 16
constexpr int K_BYTES = KT * K_STRIDE;         // 17408
constexpr int V_BYTES = DH * V_STRIDE;         // 18432
constexpr int STAGE_BYTES = K_BYTES + V_BYTES; // 35840

struct AttnArgs {
    const uint16_t *Q;    // [B][Hq][A][128]
    const uint16_t *Kc;   // one layer, [B][Hkv][spad][128]
    const uint16_t *Vc;   // one layer, [B][Hkv][spad/64][128][64]
    const int32_t *pos;   // [B][A] or nullptr
    uint16_t *out;        // [B][A][Hq*128]
    float *part_o;        // [B*Hq*A][splits][128]
    float *part_ml;       // [B*Hq*A][splits][2]  (max in the log2 domain, sum)
    int B, Hq, Hkv, g, A, kv_len, spad, max_seq;
    int row_tiles, n_rg, splits, keys_per_split, n_units;
    float c;              // softmax scale * log2(e)
};

__device__ __forceinline__ int kappa(int x) { return (x & 0x13) | ((x & 4) << 1) | ((x & 8) >> 1); }

__device__ __forceinline__ float swap32(float v)
{
    // value held by the lane 32 away (the other half of the same query row)
    return __shfl_xor(v, 32, 64);
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v)
{
    union { uint4 u; bf16x8 b; } x;
    x.u = v;
    return x.b;
}

__device__ __forceinline__ bool row_is_padded(const int32_t *pos, int idx, int max_seq)
{
    if (!pos) return false;
    const int p = pos[idx];
    return p < 0 || p >= max_seq;
}

template <int R, int W>
__global__ __launch_bounds__(W * 64) void k_attn_mfma(AttnArgs p)
{
    constexpr int KP = W / R;        // waves per row tile, each on its own 32-key half of a stage
    static_assert(KP == 1 || KP == 2, "W must be R or 2R");
    constexpr int NT = W * 64;
    constexpr int ROUNDS = 1024 / NT;  // 16-byte chunks per thread for one 16 KB tile
    extern __shared__ __align__(16) unsigned char smem[];

    // Workgroup -> (unit, row group): the n_rg workgroups that stream the same keys get ids that are
    // equal modulo 8, i.e. land on the same XCD and share its L2.
    const int id = blockIdx.x;
    const int xcd = id & 7, q = id >> 3;
    const int rg = q % p.n_rg;
    const int unit = (q / p.n_rg) * 8 + xcd;
    if (unit >= p.n_units) return;
    const int split = unit % p.splits, bj = unit / p.splits;
    const int b = bj / p.Hkv, j = bj % p.Hkv;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col = lane & 31, hi = lane >> 5;
    const int rt = rg * R + (wave % R);
    const int kh = wave / R;
    const bool tile_valid = rt < p.row_tiles;
    const int rho = rt * 32 + col;
    const bool row_valid = tile_valid && rho < p.g * p.A;
    const int hg = row_valid ? rho / p.A : 0;
    const int a = row_valid ? rho - hg * p.A : 0;
    const int hq = j * p.g + hg;
    const size_t grow = ((size_t)b * p.Hq + hq) * p.A + a;  // global row id

    bf16x8 qf[8];
    {
        const uint4 *qrow = (const uint4 *)(p.Q + grow * DH);
#pragma unroll
        for (int s = 0; s < 8; ++s) qf[s] = as_bf16x8(row_valid ? qrow[2 * s + hi] : make_uint4(0, 0, 0, 0));
    }

    const int k0 = split * p.keys_per_split;
    const int k1 = min(p.kv_len, k0 + p.keys_per_split);
    const int n_stages = (k1 - k0 + KT - 1) / KT;
    const uint16_t *Kbase = p.Kc + ((size_t)bj * p.spad) * DH;
    const uint16_t *Vbase = p.Vc + ((size_t)bj * p.spad) * DH;

    uint4 kreg[ROUNDS], vreg[ROUNDS];
    auto load_stage = [&](int ks) {
        const uint4 *kg = (const uint4 *)(Kbase + (size_t)ks * DH);
        const uint4 *vg = (const uint4 *)(Vbase + (size_t)ks * DH);  // tile ks/64 starts at ks*128
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            kreg[r] = kg[r * NT + tid];
            vreg[r] = vg[r * NT + tid];
        }
    };
    auto store_stage = [&](unsigned char *st, int ks) {
        const bool tail = ks + KT > p.kv_len;  // rows past kv_len may hold anything: zero their V
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const int c = r * NT + tid;
            *(uint4 *)(st + (c >> 4) * K_STRIDE + (c & 15) * 16) = kreg[r];
            uint4 v = vreg[r];
            if (tail) {
                const int key = ks + (c & 7) * 8;  // first of the 8 keys in this chunk
                uint32_t *w = (uint32_t *)&v;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (key + 2 * e >= p.kv_len) w[e] = 0;
                    else if (key + 2 * e + 1 >= p.kv_len) w[e] &= 0xffffu;
                }
            }
            *(uint4 *)(st + K_BYTES + (c >> 3) * V_STRIDE + (c & 7) * 16) = v;
        }
    };

    f32x16 O[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[dt][r] = 0.f;
    float m = -INFINITY, l = 0.f;

    load_stage(k0);
    store_stage(smem, k0);
    __syncthreads();

    for (int it = 0; it < n_stages; ++it) {
        const int ks = k0 + it * KT;
        const bool more = it + 1 < n_stages;
        if (more) load_stage(ks + KT);
        const unsigned char *st = smem + (it & 1) * STAGE_BYTES;

        if (tile_valid) {
#pragma unroll
            for (int hh = 0; hh < 2 / KP; ++hh) {
                const int sub = (KP == 2) ? kh : hh;
                const int kbase = ks + 32 * sub;
                if (kbase >= k1) continue;  // wave-uniform
                f32x16 s;
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = 0.f;
                const unsigned char *krow = st + (32 * sub + kappa(col)) * K_STRIDE + hi * 16;
#pragma unroll
                for (int ss = 0; ss < 8; ++ss) {
                    const bf16x8 kf = *(const bf16x8 *)(krow + ss * 32);
                    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ss], s, 0, 0, 0);
                }
                float mx = -INFINITY;
                if (kbase + 32 > k1) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = kbase + kappa(8 * (r >> 2) + 4 * hi + (r & 3));
                        if (key >= k1) s[r] = -INFINITY;
                    }
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[r]);
                mx = fmaxf(mx, swap32(mx));
                const float m_new = fmaxf(m, mx);
                const float alpha = __builtin_amdgcn_exp2f((m - m_new) * p.c);
                if (__any(alpha != 1.0f)) {
                    l *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
                }
                m = m_new;
                const float mc = m_new * p.c;
                bf16x8 pf[2];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pr = __builtin_amdgcn_exp2f(s[r] * p.c - mc);
                    l += pr;
                    pf[r >> 3][r & 7] = (__bf16)pr;
                }
                const unsigned char *vrow = st + K_BYTES + col * V_STRIDE + (32 * sub + 8 * hi) * 2;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) {
                        const bf16x8 vf = *(const bf16x8 *)(vrow + dt * 32 * V_STRIDE + jj * 32);
                        O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[jj], O[dt], 0, 0, 0);
                    }
                }
            }
        }
        if (more) store_stage(smem + ((it + 1) & 1) * STAGE_BYTES, ks + KT);
        __syncthreads();
    }

    l += swap32(l);

    if (KP == 2) {
        // merge the two key halves of each row tile: the kh = 1 wave hands over through LDS
        float *xo = (float *)smem + (size_t)(wave % R) * (66 * 64);
        if (kh == 1) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) xo[(dt * 16 + r) * 64 + lane] = O[dt][r];
            xo[64 * 64 + lane] = m;
            xo[65 * 64 + lane] = l;
        }
        __syncthreads();
        if (kh == 0) {
            const float m1 = xo[64 * 64 + lane], l1 = xo[65 * 64 + lane];
            const float mf = fmaxf(m, m1);
            const float a0 = __builtin_amdgcn_exp2f((m - mf) * p.c);
            const float a1 = __builtin_amdgcn_exp2f((m1 - mf) * p.c);
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) O[dt][r] = a0 * O[dt][r] + a1 * xo[(dt * 16 + r) * 64 + lane];
            l = a0 * l + a1 * l1;
            m = mf;
        }
    }
    if (kh != 0 || !row_valid) return;

    // lane holds, for its row, head-dim indices 32 dt + 8 (r / 4) + 4 hi + (r % 4)
    if (p.splits == 1) {
        const bool padded = row_is_padded(p.pos, b * p.A + a, p.max_seq);
        const float inv = padded ? 0.f : 1.0f / l;
        uint16_t *o = p.out + ((size_t)b * p.A + a) * ((size_t)p.Hq * DH) + (size_t)hq * DH;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                uint2 w;
                w.x = (uint32_t)fc_bf16_bits(O[dt][4 * rq] * inv) | ((uint32_t)fc_bf16_bits(O[dt][4 * rq + 1] * inv) << 16);
                w.y = (uint32_t)fc_bf16_bits(O[dt][4 * rq + 2] * inv) | ((uint32_t)fc_bf16_bits(O[dt][4 * rq + 3] * inv) << 16);
                *(uint2 *)(o + 32 * dt + 8 * rq + 4 * hi) = w;
            }
    } else {
        float *po = p.part_o + (grow * p.splits + split) * DH;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq)
                *(float4 *)(po + 32 * dt + 8 * rq + 4 * hi) =
                    make_float4(O[dt][4 * rq], O[dt][4 * rq + 1], O[dt][4 * rq + 2], O[dt][4 * rq + 3]);
        if (hi == 0) {
            float *ml = p.part_ml + (grow * p.splits + split) * 2;
            *(float2 *)ml = make_float2(m * p.c, l);
        }
    }
}

// Merge the per-split partials of one query row: one block per (sequence, head, row), one thread
// per head-dim lane.
__global__ __launch_bounds__(DH) void k_attn_combine(AttnArgs p)
{
    const size_t grow = blockIdx.x;
    const int a = (int)(grow % p.A);
    const int hq = (int)((grow / p.A) % p.Hq);
    const int b = (int)(grow / ((size_t)p.A * p.Hq));
    const int i = threadIdx.x;
    uint16_t *o = p.out + ((size_t)b * p.A + a) * ((size_t)p.Hq * DH) + (size_t)hq * DH;
    if (row_is_padded(p.pos, b * p.A + a, p.max_seq)) {
        o[i] = 0;
        return;
    }
    const float *ml = p.part_ml + grow * p.splits * 2;
    const float *po = p.part_o + grow * p.splits * DH;
    float mx = -INFINITY;
    for (int s = 0; s < p.splits; ++s) mx = fmaxf(mx, ml[2 * s]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < p.splits; ++s) {
        const float w = __builtin_amdgcn_exp2f(ml[2 * s] - mx);
        num += w * po[s * DH + i];
        den += w * ml[2 * s + 1];
    }
    o[i] = fc_bf16_bits(num / den);
}

template <int R, int W>
hipError_t launch(const AttnArgs &args, hipStream_t s)
{
    static hipError_t attr = hipFuncSetAttribute((const void *)k_attn_mfma<R, W>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STAGE_BYTES);
    if (attr != hipSuccess) return attr;
    const int groups8 = (args.n_units + 7) / 8;
    const unsigned grid = (unsigned)(groups8 * 8 * args.n_rg);
    k_attn_mfma<R, W><<<dim3(grid), dim3(W * 64), 2 * STAGE_BYTES, s>>>(args);
    return hipGetLastError();
}

}  // namespace

hipError_t fc_launch_attention_mfma(const FcGeom &G, const FcAttnPlan &pl, const void *q, const void *k_layer,
                                    const void *v_layer, const int32_t *pos, int A, int kv_len, void *out,
                                    void *workspace, hipStream_t s)
{
    AttnArgs a;
    a.Q = (const uint16_t *)q;
    a.Kc = (const uint16_t *)k_layer;
    a.Vc = (const uint16_t *)v_layer;
    a.pos = pos;
    a.out = (uint16_t *)out;
    const size_t rows = (size_t)G.B * G.Hq * A;
    a.part_o = (float *)workspace;
    a.part_ml = workspace ? (float *)workspace + rows * pl.splits * DH : nullptr;
    a.B = G.B;
    a.Hq = G.Hq;
    a.Hkv = G.Hkv;
    a.g = G.g;
    a.A = A;
    a.kv_len = kv_len;
    a.spad = G.spad;
    a.max_seq = G.max_seq;
    a.row_tiles = pl.row_tiles;
    a.n_rg = (pl.row_tiles + pl.tiles_per_wg - 1) / pl.tiles_per_wg;
    a.splits = pl.splits;
    a.keys_per_split = pl.keys_per_split;
    a.n_units = G.B * G.Hkv * pl.splits;
    a.c = G.scale * 1.4426950408889634f;
    hipError_t e;
    if (pl.tiles_per_wg == 2 && pl.waves == 4) e = launch<2, 4>(a, s);
    else if (pl.tiles_per_wg == 4 && pl.waves == 4) e = launch<4, 4>(a, s);
    else if (pl.tiles_per_wg == 4 && pl.waves == 8) e = launch<4, 8>(a, s);
    else if (pl.tiles_per_wg == 8 && pl.waves == 8) e = launch<8, 8>(a, s);
    else return hipErrorInvalidValue;
    if (e != hipSuccess || pl.splits == 1) return e;
    k_attn_combine<<<dim3((unsigned)rows), dim3(DH), 0, s>>>(a);
    return hipGetLastError();
}
