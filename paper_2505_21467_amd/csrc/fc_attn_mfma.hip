// Active-query attention on the matrix cores (bf16, head_dim 128), split over the key axis.
//
// Work decomposition.  For one (sequence, kv head) the g*A query rows (head-in-group major, then
// window row) are cut into 32-row tiles.  A workgroup of W waves owns R row tiles and one contiguous
// key range ("split").  A wave owns T row tiles; KW waves share the same tiles and divide the keys
// among themselves (KW = 2: one 32-key half of every 64-key stage each; KW = 4: additionally
// alternate stages), so R = T * W / KW.
//
// Data movement.  K rows and transposed V tiles stream HBM -> LDS with 16-byte direct-to-LDS loads
// (no registers in between) into a ring of four 32 KB stages, two stages ahead of the compute.  The
// LDS image is XOR-swizzled at 16-byte granularity (the swizzle is applied to the global address of
// each lane, since direct loads land in lane order) so that the 16 lanes the LDS serves per clock
// hit 16 different 16-byte bank groups: K rows (256 B) by the low four bits of the row, V^T rows
// (128 B, two per 256 B of banks) by bits 1..3 of the row.
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
#include <stdlib.h>

#include "fc_device.h"
#include "fc_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int DH = 128;
constexpr int KT = 64;                 // keys per stage (= one transposed V tile)
constexpr int K_BYTES = KT * DH * 2;   // 16384
constexpr int STAGE_BYTES = 2 * K_BYTES;
// Eight-wave workgroups (one per compute unit) keep a ring of four stages, two in flight ahead of the
// one being consumed; four-wave workgroups (two per compute unit, drifting independently so that one
// computes while the other waits) keep two stages, one in flight.  The ring is reused as exchange /
// output staging area (17152 B per wave group).
__host__ __device__ constexpr int ring_slots(int W) { return W == 8 ? 4 : 2; }
__host__ __device__ constexpr int lds_bytes(int W) { return W == 8 ? 136 * 1024 : 68 * 1024; }
constexpr int XCHG_FLOATS = 66 * 64;   // one tile state handed between waves: 64 O regs + m + l per lane
constexpr int OROW = 132;              // floats per row of the output staging tile (128 + 4 padding)

struct AttnArgs {
    const uint16_t *Q;    // [B][Hq][A][128]
    const uint16_t *Kc;   // one layer, [B][Hkv][spad][128]
    const uint16_t *Vc;   // one layer, [B][Hkv][spad/64][128][64]
    const int32_t *pos;   // [B][A] or nullptr
    uint16_t *out;        // [B][A][Hq*128]
    float *part_o;        // [B*Hkv*row_tiles][splits][8 slot pairs][64 lanes][8 halves]: accumulators as the lanes hold them
    float *part_ml;       // [B*Hkv*row_tiles][splits][32 rows][4]  (max in the log2 domain, sum, scaling exponent, -)
    int B, Hq, Hkv, g, A, kv_len, spad, max_seq;
    int row_tiles, n_rg, splits, keys_per_split, n_units;
    float c;              // softmax scale * log2(e)
};


__device__ __forceinline__ int kappa(int x) { return (x & 0x13) | ((x & 4) << 1) | ((x & 8) >> 1); }

// Lanes l and l^32 hold the two halves of a query row.  v_permlane32_swap exchanges the upper 32
// lanes of its first operand with the lower 32 lanes of its second; fed the same value twice it
// returns (lower half in all lanes, upper half in all lanes), so one instruction pairs the halves.
__device__ __forceinline__ float row_max2(float v)
{
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float row_sum2(float v)
{
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ bool row_is_padded(const int32_t *pos, int idx, int max_seq)
{
    if (!pos) return false;
    const int p = pos[idx];
    return p < 0 || p >= max_seq;
}

__device__ __forceinline__ void load_lds16(const void *g, void *l)
{
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)g,
                                     (void __attribute__((address_space(3))) *)l, 16, 0, 0);
}

// wait until at most N of this wave's vector-memory operations are outstanding
template <int N>
__device__ __forceinline__ void wait_vm()
{
    // gfx9 s_waitcnt immediate: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// State of one 32-row tile inside a wave.
struct Tile {
    bf16x8 q[8];
    f32x16 o[4];
    float m, l;
};

// One 32-key group against one row tile: online softmax on the scores s, bf16 probabilities out.
__device__ __forceinline__ void softmax_tile(Tile &t, f32x16 &s, bf16x8 (&pf)[2], float c, int kbase, int k1,
                                             int hi)
{
    if (kbase + 32 > k1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = kbase + kappa(8 * (r >> 2) + 4 * hi + (r & 3));
            s[r] = key < k1 ? s[r] : -INFINITY;
        }
    }
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    mx = row_max2(mx);
    // t.m is a reference maximum, not the exact running one: it only moves (and the accumulators are
    // only rescaled) when some row's scores exceed it by more than 8 in the log2 domain, so the
    // probabilities stay below 2^8 and the common case costs no rescaling work at all.
    if (__any((mx - t.m) * c > 8.0f)) {
        const float m_new = fmaxf(t.m, mx);
        const float alpha = __builtin_amdgcn_exp2f((t.m - m_new) * c);
        t.l *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) t.o[dt][r] *= alpha;
        t.m = m_new;
    }
    const float mc = t.m * c;
    float lsum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float pr = __builtin_amdgcn_exp2f(s[r] * c - mc);
        lsum += pr;
        pf[r >> 3][r & 7] = (__bf16)pr;
    }
    t.l += lsum;
}

template <int T, int W, int KW>
__global__ __launch_bounds__(W * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_attn_mfma(AttnArgs p)
{
    constexpr int NT = W * 64;
    constexpr int SLOTS = ring_slots(W);
    constexpr int AHEAD = SLOTS / 2;  // stages in flight ahead of the one being consumed
    constexpr int G = W / KW;      // wave groups: each owns T row tiles, its KW waves split the keys
    constexpr int R = G * T;       // row tiles per workgroup
    constexpr int LB = 32 / W;     // 1 KB load blocks per wave and stage
    static_assert(W % KW == 0 && (KW == 1 || KW == 2 || KW == 4) && (W == 4 || W == 8), "shape");
    extern __shared__ __align__(1024) unsigned char smem[];

    // Workgroup -> (unit, row group).  Workgroup ids that are equal modulo 8 land on the same XCD; the
    // (unit, row group) pairs, ordered unit by unit, are dealt to the eight XCDs in equal contiguous
    // runs, so the workgroups that stream the same keys share an L2 and every XCD gets the same number
    // of workgroups whatever the number of units.
    const int id = blockIdx.x;
    const int xcd = id & 7, qd = id >> 3;
    const int64_t n_tiles = (int64_t)p.n_units * p.n_rg;
    const int tile = (int)(xcd * n_tiles / 8) + qd;
    if (tile >= (int)((xcd + 1) * n_tiles / 8)) return;
    const int unit = tile / p.n_rg, rg = tile - unit * p.n_rg;
    const int split = unit % p.splits, bj = unit / p.splits;
    const int b = bj / p.Hkv, j = bj % p.Hkv;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: keeps per-wave branches uniform
    const int col = lane & 31, hi = lane >> 5;
    const int gi = wave % G, kw = wave / G;
    const int rt0 = rg * R + gi * T;  // first row tile of this wave
    const int nrows = p.g * p.A;

    bool tile_valid[T], row_valid[T];
    int hq[T], a[T];
    size_t grow[T];
    Tile t[T];
#pragma unroll
    for (int u = 0; u < T; ++u) {
        tile_valid[u] = rt0 + u < p.row_tiles;
        const int rho = (rt0 + u) * 32 + col;
        row_valid[u] = tile_valid[u] && rho < nrows;
        const int hg = row_valid[u] ? rho / p.A : 0;
        a[u] = row_valid[u] ? rho - hg * p.A : 0;
        hq[u] = j * p.g + hg;
        grow[u] = ((size_t)b * p.Hq + hq[u]) * p.A + a[u];
        const uint4 *qrow = (const uint4 *)(p.Q + grow[u] * DH);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            union { uint4 u4; bf16x8 v; } x;
            x.u4 = row_valid[u] ? qrow[2 * s + hi] : make_uint4(0, 0, 0, 0);
            t[u].q[s] = x.v;
        }
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) t[u].o[dt][r] = 0.f;
        t[u].m = -INFINITY;
        t[u].l = 0.f;
    }

    const int k0 = split * p.keys_per_split;
    const int k1 = min(p.kv_len, k0 + p.keys_per_split);
    const int n_stages = (k1 - k0 + KT - 1) / KT;

    // ---- loader: the first half of the waves brings the 16 K blocks of a stage, the second half the
    // 16 V^T blocks; a block is one wave-wide direct-to-LDS load of 1 KB.  Per-lane source offsets (in
    // bytes, relative to the stage's first K row / V tile) are fixed for the whole kernel.
    const unsigned char *gsrc;  // this wave's source for stage k0
    uint32_t goff[LB];
    uint32_t lds_dst;           // byte offset inside a stage of this wave's first block
    if (wave < W / 2) {
        gsrc = (const unsigned char *)(p.Kc + ((size_t)bj * p.spad + k0) * DH);
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int bi = wave * LB + i;
            const int rf = 4 * bi + (lane >> 4);  // LDS row 0..63: half * 32 + rho
            const int rho = rf & 31;
            const int key = (rf & 32) + kappa(rho);
            const int c = (lane & 15) ^ (rho & 15);
            goff[i] = (uint32_t)(key * 256 + c * 16);
        }
        lds_dst = (uint32_t)(wave * LB * 1024);
    } else {
        gsrc = (const unsigned char *)(p.Vc + ((size_t)bj * p.spad + k0) * DH);
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int bi = (wave - W / 2) * LB + i;
            const int dh = 8 * bi + (lane >> 3);
            const int c = (lane & 7) ^ ((dh >> 1) & 7);
            goff[i] = (uint32_t)(dh * 128 + c * 16);
        }
        lds_dst = (uint32_t)(K_BYTES + (wave - W / 2) * LB * 1024);
    }
    auto issue_stage = [&](int st) {
        const unsigned char *src = gsrc + (size_t)st * (STAGE_BYTES / 2);  // 64 keys * 256 B for K and for V
        unsigned char *dst = smem + (st % SLOTS) * STAGE_BYTES + lds_dst;
#pragma unroll
        for (int i = 0; i < LB; ++i) load_lds16(src + goff[i], dst + i * 1024);
    };

    // ---- operand read offsets inside a stage (bytes)
    uint32_t koff[8];  // K fragment ss of LDS row `col` (add half * 8192)
#pragma unroll
    for (int ss = 0; ss < 8; ++ss) koff[ss] = (uint32_t)(col * 256 + (((2 * ss + hi) ^ (col & 15)) << 4));
    uint32_t voff[2][2];  // V^T fragment (half, jj) of row `col` (add dt * 4096)
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
            voff[sub][jj] = (uint32_t)(K_BYTES + col * 128 + (((4 * sub + 2 * jj + hi) ^ ((col >> 1) & 7)) << 4));

    if (n_stages > 0) issue_stage(0);
    if (AHEAD > 1 && n_stages > 1) issue_stage(1);

    for (int it = 0; it < n_stages; ++it) {
        const int ks = k0 + it * KT;
        if (SLOTS == 4) {
            // The slot of stage it+2 last held stage it-2, which every wave left before the barrier of
            // stage it-1: the load can go out ahead of this stage's barrier.
            if (it + AHEAD < n_stages) {
                issue_stage(it + AHEAD);
                wait_vm<2 * LB>();
            } else if (it + 1 < n_stages) {
                wait_vm<LB>();
            } else {
                wait_vm<0>();
            }
            __builtin_amdgcn_s_barrier();
        } else {
            // Two slots: the next stage overwrites stage it-1, which other waves may still be reading
            // until they arrive at this barrier, so its load goes out behind the barrier.
            wait_vm<0>();
            __builtin_amdgcn_s_barrier();
            if (it + 1 < n_stages) issue_stage(it + 1);
        }
        unsigned char *st = smem + (it % SLOTS) * STAGE_BYTES;

        if (ks + KT > p.kv_len) {
            // Rows past kv_len may hold anything (also NaN): zero their V so that 0 * V stays 0.
            for (int e = tid; e < DH * KT; e += NT) {
                const int dh = e >> 6, kl = e & 63;
                if (ks + kl >= p.kv_len)
                    *(uint16_t *)(st + K_BYTES + dh * 128 + (((kl >> 3) ^ ((dh >> 1) & 7)) << 4) + (kl & 7) * 2) = 0;
            }
            __syncthreads();
        }
        if (KW == 4 && (it & 1) != (kw >> 1)) continue;
#pragma unroll
        for (int hh = 0; hh < (KW == 1 ? 2 : 1); ++hh) {
            const int sub = (KW == 1) ? hh : (kw & 1);
            const int kbase = ks + 32 * sub;
            if (kbase >= k1 || !tile_valid[0]) continue;  // wave-uniform
            const unsigned char *kb = st + sub * 8192;
            bf16x8 kf[8];
#pragma unroll
            for (int ss = 0; ss < 8; ++ss) kf[ss] = *(const bf16x8 *)(kb + koff[ss]);
            f32x16 s[T];
#pragma unroll
            for (int u = 0; u < T; ++u) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[u][r] = 0.f;
                if (u == 0 || tile_valid[u]) {
#pragma unroll
                    for (int ss = 0; ss < 8; ++ss)
                        s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ss], t[u].q[ss], s[u], 0, 0, 0);
                }
            }
            bf16x8 vf[8];
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
                    vf[dt * 2 + jj] = *(const bf16x8 *)(st + voff[sub][jj] + dt * 4096);
#pragma unroll
            for (int u = 0; u < T; ++u) {
                if (u == 0 || tile_valid[u]) {
                    bf16x8 pf[2];
                    softmax_tile(t[u], s[u], pf, p.c, kbase, k1, hi);
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj)
                            t[u].o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt * 2 + jj], pf[jj], t[u].o[dt], 0, 0, 0);
                }
            }
        }
    }
    __syncthreads();  // every wave is done with the ring; LDS is reused below

    float *xch = (float *)smem;
#pragma unroll
    for (int u = 0; u < T; ++u) t[u].l = row_sum2(t[u].l);

    if (KW > 1) {
        // merge the KW partial states of each tile into the kw == 0 wave
        if (kw > 0) {
#pragma unroll
            for (int u = 0; u < T; ++u) {
                float *x = xch + (size_t)(((kw - 1) * G + gi) * T + u) * XCHG_FLOATS;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq)  // 16-byte LDS accesses, lane-contiguous
                        *(float4 *)(x + ((dt * 4 + rq) * 64 + lane) * 4) =
                            make_float4(t[u].o[dt][4 * rq], t[u].o[dt][4 * rq + 1], t[u].o[dt][4 * rq + 2],
                                        t[u].o[dt][4 * rq + 3]);
                x[64 * 64 + lane] = t[u].m;
                x[65 * 64 + lane] = t[u].l;
            }
        }
        __syncthreads();
        if (kw == 0) {
#pragma unroll
            for (int u = 0; u < T; ++u) {
                for (int w2 = 1; w2 < KW; ++w2) {
                    const float *x = xch + (size_t)(((w2 - 1) * G + gi) * T + u) * XCHG_FLOATS;
                    const float m1 = x[64 * 64 + lane], l1 = x[65 * 64 + lane];
                    const float mf = fmaxf(t[u].m, m1);
                    const float a0 = (t[u].m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((t[u].m - mf) * p.c);
                    const float a1 = (m1 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m1 - mf) * p.c);
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                        for (int rq = 0; rq < 4; ++rq) {
                            const float4 v = *(const float4 *)(x + ((dt * 4 + rq) * 64 + lane) * 4);
                            t[u].o[dt][4 * rq] = a0 * t[u].o[dt][4 * rq] + a1 * v.x;
                            t[u].o[dt][4 * rq + 1] = a0 * t[u].o[dt][4 * rq + 1] + a1 * v.y;
                            t[u].o[dt][4 * rq + 2] = a0 * t[u].o[dt][4 * rq + 2] + a1 * v.z;
                            t[u].o[dt][4 * rq + 3] = a0 * t[u].o[dt][4 * rq + 3] + a1 * v.w;
                        }
                    t[u].l = a0 * t[u].l + a1 * l1;
                    t[u].m = mf;
                }
            }
        }
        __syncthreads();  // the exchange area is reused as output staging
    }
    if (kw != 0) return;

    if (p.splits > 1) {
        // ---- partial output, in accumulator order, as scaled half floats: the partial of a row is
        // normalised by its own sum (a convex combination of V rows, so it is no larger than the
        // largest |V|) and by a power of two that brings the row's largest magnitude into
        // [2^14, 2^15); eleven significant bits per value, with the row's max, sum and exponent in
        // fp32.  That halves the one traffic this kernel adds on top of the key/value stream.
        // Lane (col, hi) holds for query row `col` the head-dim elements 32 dt + 8 rq + 4 hi .. + 3 in
        // registers o[dt][4 rq .. 4 rq + 3]; a 16-byte store takes the two rq of a pair.
#pragma unroll
        for (int u = 0; u < T; ++u) {
            if (!tile_valid[u]) continue;
            const size_t ts = ((size_t)bj * p.row_tiles + rt0 + u) * p.splits + split;
            uint4 *po = (uint4 *)p.part_o + ts * (8 * 64) + lane;
            float amax = 0.f;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) amax = fmaxf(amax, fabsf(t[u].o[dt][r]));
            amax = row_max2(amax);
            const float inv_l = 1.0f / t[u].l;
            const int k = 15 - __builtin_amdgcn_frexp_expf(amax * inv_l);  // 15 for an all-zero row
#pragma unroll
            for (int q2 = 0; q2 < 8; ++q2) {
                union { _Float16 h[8]; uint4 u4; } x;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    x.h[e] = (_Float16)__builtin_amdgcn_ldexpf(t[u].o[q2 >> 1][8 * (q2 & 1) + e] * inv_l, k);
                po[q2 * 64] = x.u4;
            }
            if (hi == 0) ((float4 *)p.part_ml)[ts * 32 + col] = make_float4(t[u].m * p.c, t[u].l, (float)k, 0.f);
        }
        return;
    }

    // ---- final output (single split).  Each owner wave stages its tile as [row][128] floats in its
    // own LDS area, then writes whole rows of 256 bytes.
    float *stg = xch + (size_t)gi * (32 * OROW + 64);
    size_t *rowid = (size_t *)(stg + 32 * OROW);  // 32 entries
#pragma unroll
    for (int u = 0; u < T; ++u) {
        if (!tile_valid[u]) continue;
        const float inv = 1.0f / t[u].l;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq)
                *(float4 *)(stg + col * OROW + 32 * dt + 8 * rq + 4 * hi) =
                    make_float4(t[u].o[dt][4 * rq] * inv, t[u].o[dt][4 * rq + 1] * inv,
                                t[u].o[dt][4 * rq + 2] * inv, t[u].o[dt][4 * rq + 3] * inv);
        if (hi == 0) {
            // destination row (or an all-ones marker for rows that do not exist)
            size_t dst = ((size_t)b * p.A + a[u]) * ((size_t)p.Hq * DH) + (size_t)hq[u] * DH;
            if (row_is_padded(p.pos, b * p.A + a[u], p.max_seq)) dst |= (size_t)1 << 62;
            rowid[col] = row_valid[u] ? dst : ~(size_t)0;
        }
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the staged tile is visible to the whole wave
#pragma unroll 2
        for (int i = 0; i < 16; ++i) {
            const int idx = i * 64 + lane;
            const int row = idx >> 5, c4 = idx & 31;
            const size_t dst = rowid[row];
            if (dst == ~(size_t)0) continue;
            const float4 v = *(const float4 *)(stg + row * OROW + c4 * 4);
            const bool padded = (dst >> 62) & 1;
            uint16_t *o = p.out + (dst & (((size_t)1 << 62) - 1)) + c4 * 4;
            uint2 w;
            w.x = padded ? 0u : ((uint32_t)fc_bf16_bits(v.x) | ((uint32_t)fc_bf16_bits(v.y) << 16));
            w.y = padded ? 0u : ((uint32_t)fc_bf16_bits(v.z) | ((uint32_t)fc_bf16_bits(v.w) << 16));
            *(uint2 *)o = w;
        }
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_s_waitcnt(0xc07f);  // reads of the staging area are done before the next tile reuses it
    }
}

// Merge the per-split partials: one workgroup of NWV waves per (row tile, pair of 16-byte accumulator
// slots).  Lane (col, hi) owns row `col` of the tile and two groups of four consecutive head-dim
// elements, exactly as in the first kernel's accumulators, so every load is a wave-wide contiguous
// 1 KB.  Each wave merges an equal share of the splits, CB of them per batch with all their loads in
// flight together (the launch picks NWV and CB so that one batch per wave covers every split up to
// 128: the merge is one memory round trip); the waves' states are then merged through LDS.
template <int CB, int NWV>
__global__ __launch_bounds__(64 * NWV) void k_attn_combine(AttnArgs p)
{
    __shared__ float xw[NWV > 1 ? NWV : 1][10][64];
    const int lane = threadIdx.x & 63, col = lane & 31, hi = lane >> 5;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int per = (p.splits + NWV - 1) / NWV;
    const int s_lo = min(wv * per, p.splits), s_hi = min(s_lo + per, p.splits);
    const int q2 = blockIdx.x & 7;           // accumulator slots 2 q2 and 2 q2 + 1: dt = q2 >> 1, rq = 2 (q2 & 1) + {0, 1}
    const size_t tg = blockIdx.x >> 3;       // (b * Hkv + j) * row_tiles + rt
    const int rt = (int)(tg % p.row_tiles);
    const int bj = (int)(tg / p.row_tiles);
    const int b = bj / p.Hkv, j = bj % p.Hkv;
    const uint4 *po = (const uint4 *)p.part_o + tg * p.splits * (8 * 64) + q2 * 64 + lane;
    const float4 *ml = (const float4 *)p.part_ml + tg * p.splits * 32 + col;

    float m_run = -INFINITY, den = 0.f;
    float num[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) num[e] = 0.f;
    for (int sb = s_lo; sb < s_hi; sb += CB) {
        uint4 v[CB];
        float4 mlv[CB];  // (max in the log2 domain, sum, exponent of the half-float scaling, -)
#pragma unroll
        for (int u = 0; u < CB; ++u) {
            const int s = min(sb + u, s_hi - 1);
            v[u] = po[(size_t)s * (8 * 64)];
            mlv[u] = ml[(size_t)s * 32];
        }
        float mb = mlv[0].x;
#pragma unroll
        for (int u = 1; u < CB; ++u) mb = fmaxf(mb, mlv[u].x);
        const float m_new = fmaxf(m_run, mb);
        const float keep = __builtin_amdgcn_exp2f(m_run - m_new);  // 0 on the first batch
#pragma unroll
        for (int e = 0; e < 8; ++e) num[e] *= keep;
        den *= keep;
#pragma unroll
        for (int u = 0; u < CB; ++u) {
            // weight of the split's sum; its stored values are (partial / sum) * 2^k
            const float w = (sb + u < s_hi) ? __builtin_amdgcn_exp2f(mlv[u].x - m_new) * mlv[u].y : 0.f;
            const float wn = __builtin_amdgcn_ldexpf(w, -(int)mlv[u].z);
            union { uint4 u4; _Float16 h[8]; } x;
            x.u4 = v[u];
#pragma unroll
            for (int e = 0; e < 8; ++e) num[e] += wn * (float)x.h[e];
            den += w;
        }
        m_run = m_new;
    }
    if (NWV > 1) {
        // wave 0 (which always has a split) merges the states; a wave without splits holds (-inf, 0, 0)
        xw[wv][0][lane] = m_run;
        xw[wv][1][lane] = den;
#pragma unroll
        for (int e = 0; e < 8; ++e) xw[wv][2 + e][lane] = num[e];
        __syncthreads();
        if (wv != 0) return;
        float m_all = m_run;
#pragma unroll
        for (int w2 = 1; w2 < NWV; ++w2) m_all = fmaxf(m_all, xw[w2][0][lane]);
        const float k0 = __builtin_amdgcn_exp2f(m_run - m_all);
        den *= k0;
#pragma unroll
        for (int e = 0; e < 8; ++e) num[e] *= k0;
#pragma unroll
        for (int w2 = 1; w2 < NWV; ++w2) {
            const float kw2 = __builtin_amdgcn_exp2f(xw[w2][0][lane] - m_all);
            den += kw2 * xw[w2][1][lane];
#pragma unroll
            for (int e = 0; e < 8; ++e) num[e] += kw2 * xw[w2][2 + e][lane];
        }
    }

    const int rho = rt * 32 + col;
    if (rho >= p.g * p.A) return;  // row past the end of the last tile
    const int hg = rho / p.A, a = rho - hg * p.A;
    const int hq = j * p.g + hg;
    const bool padded = row_is_padded(p.pos, b * p.A + a, p.max_seq);
    uint16_t *orow = p.out + ((size_t)b * p.A + a) * ((size_t)p.Hq * DH) + (size_t)hq * DH;
#pragma unroll
    for (int g2 = 0; g2 < 2; ++g2) {
        uint2 w;
        w.x = padded ? 0u : ((uint32_t)fc_bf16_bits(num[4 * g2] / den) | ((uint32_t)fc_bf16_bits(num[4 * g2 + 1] / den) << 16));
        w.y = padded ? 0u : ((uint32_t)fc_bf16_bits(num[4 * g2 + 2] / den) | ((uint32_t)fc_bf16_bits(num[4 * g2 + 3] / den) << 16));
        const int dh = 32 * (q2 >> 1) + 8 * (2 * (q2 & 1) + g2) + 4 * hi;
        *(uint2 *)(orow + dh) = w;
    }
}

template <int T, int W, int KW>
hipError_t launch(const AttnArgs &args, hipStream_t s)
{
    constexpr int LDS_BYTES = lds_bytes(W);
    static hipError_t attr = hipFuncSetAttribute((const void *)k_attn_mfma<T, W, KW>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (attr != hipSuccess) return attr;
    const unsigned grid = (unsigned)(((int64_t)args.n_units * args.n_rg + 7) / 8 * 8);
    k_attn_mfma<T, W, KW><<<dim3(grid), dim3(W * 64), LDS_BYTES, s>>>(args);
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
    // workspace: per (row tile, split) 32 x 128 scaled half floats, then 32 x (max, sum, exponent, -)
    const size_t tiles = (size_t)G.B * G.Hkv * pl.row_tiles;
    a.part_o = (float *)workspace;
    a.part_ml = workspace ? (float *)workspace + tiles * pl.splits * (32 * DH / 2) : nullptr;
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
    const int R = pl.tiles_per_wg;
    if (pl.waves == 8) {  // one tile per wave
        if (R == 8) e = launch<1, 8, 1>(a, s);
        else if (R == 4) e = launch<1, 8, 2>(a, s);
        else if (R == 2) e = launch<1, 8, 4>(a, s);
        else return hipErrorInvalidValue;
    } else {              // four-wave workgroups, two per compute unit
        if (R == 4) e = launch<1, 4, 1>(a, s);
        else if (R == 2) e = launch<1, 4, 2>(a, s);
        else return hipErrorInvalidValue;
    }
    if (e != hipSuccess || pl.splits == 1) return e;
    const dim3 cgrid((unsigned)(tiles * 8));
    if (pl.splits <= 2) k_attn_combine<2, 1><<<cgrid, dim3(64), 0, s>>>(a);
    else if (pl.splits <= 8) k_attn_combine<8, 1><<<cgrid, dim3(64), 0, s>>>(a);
    else if (pl.splits <= 16) k_attn_combine<8, 2><<<cgrid, dim3(128), 0, s>>>(a);
    else if (pl.splits <= 32) k_attn_combine<8, 4><<<cgrid, dim3(256), 0, s>>>(a);
    else if (pl.splits <= 64) k_attn_combine<16, 4><<<cgrid, dim3(256), 0, s>>>(a);
    else k_attn_combine<32, 4><<<cgrid, dim3(256), 0, s>>>(a);
    return hipGetLastError();
}
