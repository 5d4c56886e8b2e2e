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
// Two more shapes (NSUB = 5, 3) deal the rotary pairs of all head slots, laid end to end, 80 or 48 to a
// workgroup (16 per sub-tile, low rows then high rows: the partner of register r is register r + 8): a
// quarter more work per workgroup than a head for grids that would otherwise be a little more than one
// round, a quarter less for grids well short of one.
//
// Both operands are contiguous along the hidden dimension.  64 (or 128) hidden elements of every row
// of the tile (128- or 256-byte row pieces) stream HBM/L2 -> LDS with direct-to-LDS 16-byte loads into
// a ring of two to four stages; the 16-byte chunks of a row piece are XOR-swizzled with bits 1..3 (or
// 0..3) of the row (applied to the global address of the loading lane), which spreads the 16 lanes the
// LDS serves per clock over 16 different bank groups.
//
// A wave that issues a direct-to-LDS load waits until the memory pipeline has taken it (about 46
// cycles per load measured), and that wait is not hidden when the wave is alone on its SIMD.  The
// 128-row shapes (four multiplying waves) therefore carry four more waves that do nothing but issue
// the loads; in the 256-row shapes (two multiplying waves per SIMD) every wave issues its share, a
// quarter at a time between its multiplies.
#include <stdlib.h>
#include <string.h>

#include "fc_device.h"
#include "fc_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int KS_MIN = 64;      // hidden elements per stage: 64 or 128 (template parameter KS)

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
    int n_slots;           // 128-row slabs of W: head slots (EPI 0), N / 128 (EPI 1, 3), d_ff / 64 (EPI 2)
    // The part of the problem this launch covers (a problem may be cut into two launches with different
    // tile shapes, see launch_pieces): slabs [slot_base, slot_base + slots_here), rows [m_base, m_end).
    int slot_base, slots_here, m_base, m_end;
    double log2_base_64;   // log2(rope_base) / 64
    // plain linear layers of the rest of the layer (EPI != 0)
    const uint16_t *W2;    // EPI 2: the up matrix [N][K] (W is the gate matrix)
    const uint16_t *res;   // EPI 1: residual [M][N] or nullptr
    uint16_t *out;         // EPI 1, 2: [M][N]
    float *part;           // EPI 3: partial sums [ksplit][M][N]
    int N;                 // output columns
    int ksplit;            // EPI 3: parts the hidden dimension is cut into
    FcArgmaxPart am;       // EPI 4: per (slab, row) largest logit, its index, sum of exponentials
};


__device__ __forceinline__ void load_lds16g(const void *g, void *l)
{
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)g,
                                     (void __attribute__((address_space(3))) *)l, 16, 0, 0);
}

// wait until at most N vector-memory operations of this wave are outstanding; LGKM0: and no LDS one
template <int N, bool LGKM0 = false>
__device__ __forceinline__ void wait_vmg()
{
    // gfx9 s_waitcnt immediate: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | ((LGKM0 ? 0 : 15) << 8) | ((N >> 4) << 14));
}
// the same with N = k * PER for a run-time k in 0..3
template <int PER, bool LGKM0>
__device__ __forceinline__ void wait_stages(int k)
{
    if (k >= 3) wait_vmg<3 * PER, LGKM0>();
    else if (k == 2) wait_vmg<2 * PER, LGKM0>();
    else if (k == 1) wait_vmg<PER, LGKM0>();
    else wait_vmg<0, LGKM0>();
}

// Workgroup tile: NG head groups x WM row groups of waves (NW = NG * WM waves).  A wave owns MW
// 32-row sub-tiles of window rows and the NSUB 32-feature sub-tiles of one head (NSUB = 4) or of one
// rotary-paired half head (NSUB = 2).  SLOTS = stages in the LDS ring.
// NL = 0: every wave also issues its share of the loads; NL > 0: NL extra waves do nothing but issue
// the loads, so that the multiplying waves never wait for the memory pipeline to take a load.
// EPI selects the epilogue: 0 = QKV (bias, rotary embedding, scatter into the cache); the others are
// the plain linear layers of the rest of the layer, whose 128-row slabs of W take the place of the
// head slots: 1 = out = residual + x w^T; 2 = out = silu(x w_gate^T) * (x w_up^T), a slab being 64
// gate rows (sub-tiles 0, 1) and the same 64 up rows (sub-tiles 2, 3), so that both products of an
// output sit in one lane like a rotary pair; 3 = fp32 partial sums of one part of the hidden dimension
// (the parts are tiles of their own), for matrices with too few slabs to fill the chip; 4 = vocabulary projection of the
// unmasking step: of the 128 logits of a slab only the largest, its index and the sum of
// exp(logit - largest) are kept per row (NSUB = 4 only).
template <int KS, int NW, int NSUB, int MW, int NG, int SLOTS, int NL, int EPI>
__global__ __launch_bounds__((NW + NL) * 64) void k_proj_gemm(GemmArgs p)
{
    constexpr int ROWB = KS * 2;               // bytes of one row piece: 128 or 256
    constexpr int CPR = ROWB / 16;             // 16-byte chunks per row piece
    constexpr int RPB = 1024 / ROWB;           // row pieces per 1 KB block (= one wave-wide load)
    constexpr int NKK = KS / 16;               // k-steps per stage
    constexpr int WM = NW / NG;
    constexpr int NLW = NL > 0 ? NL : NW;      // waves that issue loads
    constexpr bool DEALT = NSUB == 5 || NSUB == 3;
    constexpr int PPU = 16 * NSUB;             // DEALT: pairs per workgroup
    constexpr int WROWS = DEALT ? 32 * NSUB : 32 * NSUB * NG, XROWS = 32 * MW * WM;
    constexpr int WBYTES = WROWS * ROWB, STAGE = (WROWS + XROWS) * ROWB;
    constexpr int NBLK = (WROWS + XROWS) / RPB;  // 1 KB blocks per stage
    // NSUB = 5 or 3 ("dealt pairs", EPI 0 and 2 only): the workgroup takes 16 NSUB consecutive PAIRS of weight rows
    // -- rotary pairs (i, i + 64) of the head slots laid end to end, or (gate row, up row) pairs -- 16
    // pairs per sub-tile: the low rows in rows 0..15 of the sub-tile, the high rows in rows 16..31, so
    // that the two members of a pair sit in one lane, registers r and r + 8.  The 52 blocks of a stage
    // of the 80-pair shape do not divide by its eight waves: waves 0..3 issue seven loads per stage, waves
    // 4..7 six (the 48-pair shape has four loading waves of seven blocks each).
    // With NG = 2 the five sub-tiles are split between the two waves of a SIMD (sub-tiles 0..2 and 3..4),
    // each wave taking MW = 2 row sub-tiles: the pair of waves reads 5 + 4 fragments for its 6 + 4
    // multiplies of a k-step instead of 2 x 6 for 2 x 5 with 32-row waves (same time measured, less LDS
    // traffic).
    constexpr int NT = DEALT && NG == 2 ? (NSUB + 1) / 2 : NSUB;  // sub-tiles a wave owns (at most)
    constexpr int WBLK = WROWS / RPB;          // weight blocks of a stage (the first ones)
    constexpr int LBW = (NBLK + NLW - 1) / NLW;  // blocks per loading wave and stage (DEALT: at most)
    constexpr int WBW = WBLK / NLW;            // of which weight blocks (not DEALT)
    static_assert(KS == 64 || KS == 128, "stage depth");
    static_assert(NW % NG == 0 && (DEALT || (NBLK % NLW == 0 && WBLK % NLW == 0)) && (NSUB >= 4 || NG == 1), "tile shape");
    static_assert(!DEALT || ((EPI == 0 || EPI == 2) && (NG == 1 || NG == 2) &&
                             (NL == 0 ? NBLK - (LBW - 1) * NLW == NLW / 2 : (NBLK % NLW == 0 && WBLK % NLW == 0))),
                  "dealt pairs: QKV or gated epilogue");
    static_assert((SLOTS - 1) * LBW < 64 && SLOTS >= 2 && SLOTS <= 4, "vmcnt range");
    static_assert(EPI == 0 || NG == 1 || DEALT, "the plain linear layers use one slab per workgroup");
    extern __shared__ __align__(1024) unsigned char smem[];
    const FcGeom &G = p.G;

    // Workgroup -> (unit, row tile).  Workgroup ids that are equal modulo 8 land on the same XCD; the
    // tiles, ordered unit by unit, are dealt to the eight XCDs in equal contiguous runs, so the
    // workgroups that stream the same weight rows share an L2 and every XCD gets the same number of
    // tiles (dealing whole units instead left 35 tiles on four XCDs and 28 on the others for 36 head
    // slots x 7 row tiles: two rounds of 32 compute units instead of one, 100 us instead of 62).
    const int id = blockIdx.x;
    const int xcd = id & 7, qd = id >> 3;
    // (EPI 3: the parts of the hidden dimension count as tiles too, so that they are dealt evenly as well)
    const int n_kp = EPI == 3 ? p.ksplit : 1;
    const int64_t n_tiles = (int64_t)p.n_units * p.n_mt * n_kp;
    const int tile_k = (int)(xcd * n_tiles / 8) + qd;
    if (tile_k >= (int)((xcd + 1) * n_tiles / 8)) return;
    const int tile = tile_k / n_kp, kpart = tile_k - tile * n_kp;
    const int unit = tile / p.n_mt, mt = tile - unit * p.n_mt;
    const int m0 = p.m_base + mt * XROWS;
    const int n_slots = p.n_slots;             // EPI 0: Hq query heads, Hkv key heads, Hkv value heads

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hi = lane >> 5;
    const bool is_loader = NL > 0 && wave >= NW;  // wave-uniform
    const int lw = NL > 0 ? wave - NW : wave;     // index among the loading waves
    const int wn = (wave % NW) / WM, wm = wave % WM;  // this wave's head group and row group
    const int hs = p.slot_base + (NSUB >= 4 ? unit * NG + wn : unit >> 1);  // (DEALT: not used)
    const int half = NSUB >= 4 ? 0 : unit & 1;  // which rotary-paired half of the head
    const bool head_valid = DEALT || hs < n_slots;  // an odd number of heads leaves the last pair half empty
    const int n_pairs = n_slots * 64;           // DEALT: pairs of the whole problem
    const int my_blocks = DEALT && NL == 0 && lw >= NLW / 2 ? LBW - 1 : LBW;  // wave-uniform
    const int t0 = DEALT && NG == 2 && wn ? NT : 0;              // DEALT: first sub-tile of this wave
    const int nt_mine = DEALT && NG == 2 && wn ? NSUB - NT : NT;  // and how many it owns (wave-uniform)

    // ---- loader: per-lane source offsets (bytes from W / X, hidden offset 0) of this wave's blocks
    uint32_t goff[LBW];
#pragma unroll
    for (int i = 0; i < LBW; ++i) {
        const int bid = lw + NLW * i;               // block of the stage: weight blocks first (junk for lw < 0)
        const bool is_w = DEALT ? bid < WBLK : i < WBW;
        const int rl = RPB * (is_w ? bid : bid - WBLK) + lane / CPR;  // row of the W / X tile
        // logical 16-byte chunk that lands at position lane % CPR of the row piece: 128-byte pieces are
        // swizzled with bits 1..3 of the row, 256-byte pieces with bits 0..3
        const int c = (lane % CPR) ^ (KS == 64 ? (rl >> 1) & 7 : rl & 15);
        if (is_w) {
            int n;
            if (DEALT) {
                const int pr = min(PPU * unit + 16 * (rl >> 5) + (rl & 15), n_pairs - 1);  // pairs past the end are never stored
                if (EPI == 2) n = pr;  // row pr of the gate matrix (low) or of the up matrix (high)
                else n = (pr >> 6) * 128 + (pr & 63) + ((rl & 16) ? 64 : 0);
            } else if (EPI == 2) {  // row of the gate or of the up matrix (which of the two: see issue_stage)
                const int u = min(hs, n_slots - 1);  // NG = 1 here: hs is the slab of the whole workgroup
                n = u * 64 + (NSUB == 4 ? rl & 63 : 32 * half + (rl & 31));
            } else if (NSUB == 4) {
                n = min(p.slot_base + unit * NG + rl / 128, n_slots - 1) * 128 + (rl & 127);
            } else {
                n = min(hs, n_slots - 1) * 128 + (rl >> 5) * 64 + 32 * half + (rl & 31);
            }
            goff[i] = (uint32_t)n * (uint32_t)(p.K * 2) + c * 16;
        } else {
            const int m = min(m0 + rl, p.m_end - 1);  // rows past the end re-read the last row; never stored
            goff[i] = (uint32_t)m * (uint32_t)(p.K * 2) + c * 16;
        }
    }
    // The loads of a stage are issued in four parts spread over the multiplies of the stage before,
    // because a wave that issues many of them back to back waits for the memory pipeline to take
    // them before it can issue anything else.  part < 0: all of them.
    // part of the hidden dimension this workgroup covers (EPI 3 only: part kpart of p.ksplit)
    const int all_stages = p.K / KS;
    const int st0 = EPI == 3 ? (int)((int64_t)kpart * all_stages / p.ksplit) : 0;
    const int n_stages = EPI == 3 ? (int)(((int64_t)kpart + 1) * all_stages / p.ksplit) - st0 : all_stages;
    auto issue_stage = [&](int st, int part) {
        unsigned char *dst = smem + (st % SLOTS) * STAGE;
#pragma unroll
        for (int i = 0; i < LBW; ++i) {
            if (part >= 0 && (i & 3) != part) continue;
            if (DEALT && i >= my_blocks) continue;
            const uint16_t *mat = p.X;
            if (DEALT) {
                // rows 16..31 of a sub-tile are the high rows: EPI 2 takes them from the up matrix
                const int bid = lw + NLW * i;
                if (bid < WBLK) mat = (EPI == 2 && ((RPB * bid) & 16)) ? p.W2 : p.W;
            } else if (i < WBW) {
                // EPI 2: the second half of the tile rows (a whole number of 1 KB blocks) is the up matrix
                const bool up = EPI == 2 && RPB * (lw + NLW * i) >= (NSUB == 4 ? 64 : 32);
                mat = up ? p.W2 : p.W;
            }
            const unsigned char *src = (const unsigned char *)mat + (size_t)(st0 + st) * ROWB;
            load_lds16g(src + goff[i], dst + (lw + NLW * i) * 1024);
        }
    };

    // ---- operand read offsets inside a stage (bytes): row `col` of a 32-row sub-tile, k-step kk
    uint32_t foff[NKK];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
        foff[kk] = (uint32_t)(col * ROWB + (((2 * kk + hi) ^ (KS == 64 ? (col >> 1) & 7 : col & 15)) << 4));
    const uint32_t w_base = (uint32_t)((DEALT ? t0 : wn * NSUB) * 32 * ROWB);
    const uint32_t x_base = (uint32_t)(WBYTES + wm * MW * 32 * ROWB);

    f32x16 acc[MW][NT];
#pragma unroll
    for (int i = 0; i < MW; ++i)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][t][r] = 0.f;

    // Fragments are double-buffered in registers: the LDS reads of k-step kk+1 are issued before the
    // multiplies of k-step kk, and the first reads of the next stage go out (behind that stage's
    // barrier) before the last multiplies of this one, so the matrix core never waits for LDS.
    bf16x8 xf[2][MW], wf[2][NT];
    auto read_frags = [&](int slot, int kk, int buf) {
        const unsigned char *st = smem + slot * STAGE;
#pragma unroll
        for (int i = 0; i < MW; ++i) xf[buf][i] = *(const bf16x8 *)(st + x_base + i * (32 * ROWB) + foff[kk]);
#pragma unroll
        for (int t = 0; t < NT; ++t)
            if (t < nt_mine) wf[buf][t] = *(const bf16x8 *)(st + w_base + t * (32 * ROWB) + foff[kk]);
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int i = 0; i < MW; ++i)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                if (t < nt_mine)
                    acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][t], xf[buf][i], acc[i][t], 0, 0, 0);
    };

    const int n_pro = min(SLOTS, n_stages);
    if (NL > 0) {
        // ---- loading waves: one barrier per stage, shared with the multiplying waves.  Barrier `it`
        // (it = 0 .. n_stages - 2) means: stage it+1 is complete and every multiplying wave has left
        // stage it, whose slot takes stage it + SLOTS.
        if (is_loader) {
            for (int st = 0; st < n_pro; ++st) issue_stage(st, -1);
            wait_stages<LBW, false>(n_pro - 1);
            __builtin_amdgcn_s_barrier();  // stage 0 is complete
            for (int it = 0; it + 1 < n_stages; ++it) {
                // stages requested so far: min(n_stages, it + SLOTS); those after it+1 may stay in flight
                wait_stages<LBW, false>(min(n_stages, it + SLOTS) - (it + 2));
                __builtin_amdgcn_s_barrier();
                if (it + SLOTS < n_stages) issue_stage(it + SLOTS, -1);
            }
            return;
        }
        __builtin_amdgcn_s_barrier();  // stage 0 is complete
        read_frags(0, 0, 0);
        int slot = 0;
        for (int it = 0; it < n_stages; ++it) {
#pragma unroll
            for (int kk = 0; kk < NKK - 1; ++kk) {
                read_frags(slot, kk + 1, (kk + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
                multiply(kk & 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            const int nslot = slot == SLOTS - 1 ? 0 : slot + 1;
            if (it + 1 < n_stages) {
                wait_vmg<63, true>();  // lgkmcnt(0): the reads of stage `it` have returned
                __builtin_amdgcn_s_barrier();
                read_frags(nslot, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            multiply(1);
            __builtin_amdgcn_sched_barrier(0);
            slot = nslot;
        }
    } else {
    for (int st = 0; st < n_pro; ++st) issue_stage(st, -1);
    if (my_blocks == LBW) wait_stages<LBW, false>(n_pro - 1);
    else wait_stages<LBW - 1, false>(n_pro - 1);
    __builtin_amdgcn_s_barrier();  // stage 0 is complete for every wave
    read_frags(0, 0, 0);
    int slot = 0;
    for (int it = 0; it < n_stages; ++it) {
        // The slot of stage it-1 was released by the barrier in the middle of the previous iteration;
        // stage it-1+SLOTS goes there: its first quarter was issued behind that barrier, the rest now.
        const int refill = it - 1 + SLOTS;
        const bool do_refill = it > 0 && refill < n_stages;
#pragma unroll
        for (int kk = 0; kk < NKK - 1; ++kk) {
            read_frags(slot, kk + 1, (kk + 1) & 1);
            if (do_refill && kk < 3) issue_stage(refill, kk + 1);
            __builtin_amdgcn_sched_barrier(0);
            multiply(kk & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        const int nslot = slot == SLOTS - 1 ? 0 : slot + 1;
        if (it + 1 < n_stages) {
            // This wave's reads of stage `it` have all returned (lgkmcnt 0); behind the barrier that
            // holds for every wave, and stage it+1 is complete (later stages may still be in flight).
            if (my_blocks == LBW) wait_stages<LBW, true>(min(n_stages, it + SLOTS) - (it + 2));
            else wait_stages<LBW - 1, true>(min(n_stages, it + SLOTS) - (it + 2));
            __builtin_amdgcn_s_barrier();
            if (it + SLOTS < n_stages) issue_stage(it + SLOTS, 0);
            read_frags(nslot, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        multiply(1);
        __builtin_amdgcn_sched_barrier(0);
        slot = nslot;
    }
    }

    // ---- epilogue, in registers.  Lane (col, hi) of sub-tile i holds window row m0 + 32 (wm MW + i) + col;
    // register r of sub-tile t is feature 32 t' + 8 (r >> 2) + 4 hi + (r & 3) of the head, with t' = t
    // for a whole head and {half, half + 2} for a half head.
    if (!head_valid) return;
    if constexpr (EPI == 4) {
        // Lane (col, hi) holds, for window row col, the logits 32 t + 8 (r >> 2) + 4 hi + (r & 3) of the
        // slab: ascending in (t, r), so ties keep the smaller index; the other half is in lane ^ 32.
        static_assert(EPI != 4 || NSUB == 4, "vocabulary mode uses whole slabs");
#pragma unroll
        for (int i = 0; i < MW; ++i) {
            const int m = m0 + 32 * (wm * MW + i) + col;
            float mx = -INFINITY, sm = 0.f;
            int arg = 0;
#pragma unroll
            for (int t = 0; t < NSUB; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float z = acc[i][t][r];
                    const int v = hs * 128 + 32 * t + 8 * (r >> 2) + 4 * hi + (r & 3);
                    if (z > mx) {
                        sm = sm * expf(mx - z) + 1.0f;
                        mx = z;
                        arg = v;
                    } else {
                        sm += expf(z - mx);
                    }
                }
            const float mx2 = __shfl_xor(mx, 32, 64), sm2 = __shfl_xor(sm, 32, 64);
            const int arg2 = __shfl_xor(arg, 32, 64);
            fc_argmax_merge(mx, arg, sm, mx2, arg2, sm2);
            if (hi == 0 && m < p.m_end) {
                const size_t at = (size_t)hs * p.M + m;
                p.am.mx[at] = mx;
                p.am.arg[at] = arg;
                p.am.sm[at] = sm;
            }
        }
        return;
    }
    if (DEALT && EPI == 2) {
        // Gated layer, dealt pairs: registers 4 rq + e (gate) and 8 + 4 rq + e (up), rq < 2, of sub-tile t
        // are output column 80 unit + 16 t + 8 rq + 4 hi + e.
#pragma unroll
        for (int i = 0; i < MW; ++i) {
            const int m = m0 + 32 * (wm * MW + i) + col;
            if (m >= p.m_end) continue;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int base = PPU * unit + 16 * (t0 + t);
                if (t >= nt_mine || base >= n_pairs) continue;
#pragma unroll
                for (int rq = 0; rq < 2; ++rq) {
                    float y[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float g = acc[i][t][4 * rq + e];
                        y[e] = g / (1.0f + expf(-g)) * acc[i][t][8 + 4 * rq + e];
                    }
                    uint2 w;
                    w.x = (uint32_t)fc_bf16_bits(y[0]) | ((uint32_t)fc_bf16_bits(y[1]) << 16);
                    w.y = (uint32_t)fc_bf16_bits(y[2]) | ((uint32_t)fc_bf16_bits(y[3]) << 16);
                    *(uint2 *)(p.out + (size_t)m * p.N + base + 8 * rq + 4 * hi) = w;
                }
            }
        }
        return;
    }
    if constexpr (EPI != 0 && !DEALT) {
        // Plain linear layers.  Register r of sub-tile t of lane (col, hi) is output column
        // 32 t' + 8 (r >> 2) + 4 hi + (r & 3) of the slab (of its 64 outputs for EPI 2, t' < 2).
#pragma unroll
        for (int i = 0; i < MW; ++i) {
            const int m = m0 + 32 * (wm * MW + i) + col;
            if (m >= p.m_end) continue;
#pragma unroll
            for (int t = 0; t < (EPI == 2 ? NSUB / 2 : NSUB); ++t) {
                const int tq = NSUB == 4 ? t : (EPI == 2 ? half : half + 2 * t);
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const size_t at = (size_t)m * p.N + (size_t)hs * (EPI == 2 ? 64 : 128) + 32 * tq + 8 * rq + 4 * hi;
                    float y[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        y[e] = acc[i][t][4 * rq + e];
                        if (EPI == 2) y[e] = y[e] / (1.0f + expf(-y[e])) * acc[i][t + NSUB / 2][4 * rq + e];
                    }
                    if (EPI == 3) {
                        *(float4 *)(p.part + (size_t)kpart * p.M * p.N + at) = make_float4(y[0], y[1], y[2], y[3]);
                        continue;
                    }
                    if (EPI == 1 && p.res) {
                        const uint2 rv = *(const uint2 *)(p.res + at);
                        y[0] += __uint_as_float(rv.x << 16);
                        y[1] += __uint_as_float(rv.x & 0xffff0000u);
                        y[2] += __uint_as_float(rv.y << 16);
                        y[3] += __uint_as_float(rv.y & 0xffff0000u);
                    }
                    uint2 w;
                    w.x = (uint32_t)fc_bf16_bits(y[0]) | ((uint32_t)fc_bf16_bits(y[1]) << 16);
                    w.y = (uint32_t)fc_bf16_bits(y[2]) | ((uint32_t)fc_bf16_bits(y[3]) << 16);
                    *(uint2 *)(p.out + at) = w;
                }
            }
        }
        return;
    }
    // base^(-1/64) and its powers; base^(-i/64) / (2 pi) = turns per position of pair i
    const double r1 = exp2(-p.log2_base_64);
    const double r2 = r1 * r1, r4 = r2 * r2, r8 = r4 * r4, r16 = r8 * r8, r32 = r16 * r16;
    if constexpr (DEALT) {
        // Dealt pairs: sub-tile t holds the 16 rotary pairs ib .. ib + 15 of head slot hs_t; registers
        // 4 rq + e (feature ib + 8 rq + 4 hi + e) and 8 + 4 rq + e (the same + 64), rq < 2.
#pragma unroll
        for (int i = 0; i < MW; ++i) {
            const int m = m0 + 32 * (wm * MW + i) + col;
            const bool mvalid = m < p.m_end;
            const int mm = mvalid ? m : 0;
            const int b = mm / p.A, a = mm - b * p.A;
            const int pp = p.pos ? p.pos[mm] : p.win_start + a;
            const bool valid = mvalid && pp >= 0 && pp < G.max_seq;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int base = PPU * unit + 16 * (t0 + t);
                if (t >= nt_mine || base >= n_pairs) continue;  // wave-uniform
                const int hs_t = base >> 6, ib = base & 63;
                if (p.bias) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        acc[i][t][r] += fc_to_float(
                            bf16_t{p.bias[hs_t * 128 + ib + 8 * ((r >> 2) & 1) + 4 * hi + (r & 3) + 64 * (r >> 3)]});
                }
                if (hs_t < G.Hq + G.Hkv) {
                    double f = 0.15915494309189533576888;
                    if (ib & 16) f *= r16;
                    if (ib & 32) f *= r32;
                    if (hi) f *= r4;
#pragma unroll
                    for (int rq = 0; rq < 2; ++rq) {
                        double fr = f;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int r = 4 * rq + e;
                            const double turns = (double)pp * fr;
                            const float ph = (float)(turns - rint(turns));
                            const float c = __builtin_amdgcn_cosf(ph), sn = __builtin_amdgcn_sinf(ph);
                            const float lo = acc[i][t][r], hi2 = acc[i][t][r + 8];
                            acc[i][t][r] = lo * c - hi2 * sn;
                            acc[i][t][r + 8] = hi2 * c + lo * sn;
                            fr *= r1;
                        }
                        f *= r8;
                    }
                }
                if (!mvalid) continue;
#pragma unroll
                for (int rq4 = 0; rq4 < 4; ++rq4) {
                    const int d0 = ib + 8 * (rq4 & 1) + 4 * hi + 64 * (rq4 >> 1);
                    uint2 w;
                    w.x = (uint32_t)fc_bf16_bits(acc[i][t][4 * rq4]) | ((uint32_t)fc_bf16_bits(acc[i][t][4 * rq4 + 1]) << 16);
                    w.y = (uint32_t)fc_bf16_bits(acc[i][t][4 * rq4 + 2]) | ((uint32_t)fc_bf16_bits(acc[i][t][4 * rq4 + 3]) << 16);
                    if (hs_t < G.Hq) {
                        if (!valid) w = make_uint2(0, 0);
                        *(uint2 *)(p.Q + (((size_t)b * G.Hq + hs_t) * p.A + a) * 128 + d0) = w;
                    } else if (valid) {
                        if (hs_t < G.Hq + G.Hkv) {
                            *(uint2 *)(p.Kc + fc_k_index(G, b, hs_t - G.Hq, pp, d0)) = w;
                        } else {
                            uint16_t *v = p.Vc + fc_v_index(G, b, hs_t - G.Hq - G.Hkv, pp, d0);
                            v[0] = (uint16_t)(w.x & 0xffff);
                            v[FC_VTILE] = (uint16_t)(w.x >> 16);
                            v[2 * FC_VTILE] = (uint16_t)(w.y & 0xffff);
                            v[3 * FC_VTILE] = (uint16_t)(w.y >> 16);
                        }
                    }
                }
            }
        }
        return;
    }
    if constexpr (!DEALT) {
    const bool rotate = hs < G.Hq + G.Hkv;
    constexpr int NP = NSUB / 2;  // rotary pairs of sub-tiles: (t, t + NP)

#pragma unroll
    for (int i = 0; i < MW; ++i) {
        const int m = m0 + 32 * (wm * MW + i) + col;
        const bool mvalid = m < p.m_end;
        const int mm = mvalid ? m : 0;
        const int b = mm / p.A, a = mm - b * p.A;
        const int pp = p.pos ? p.pos[mm] : p.win_start + a;
        const bool valid = mvalid && pp >= 0 && pp < G.max_seq;

        if (p.bias) {
#pragma unroll
            for (int t = 0; t < NSUB; ++t) {
                const int tq = NSUB == 4 ? t : half + 2 * t;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[i][t][r] += fc_to_float(bf16_t{p.bias[hs * 128 + 32 * tq + 8 * (r >> 2) + 4 * hi + (r & 3)]});
            }
        }
        if (rotate) {
            // the angle is reduced to a fraction of a turn in double, then hardware sine / cosine
            // (argument in turns)
#pragma unroll
            for (int t = 0; t < NP; ++t) {
                const int tq = NSUB == 4 ? t : half;  // pair index 32 tq + 8 rq + 4 hi + (r & 3) < 64
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
                        const float lo = acc[i][t][r], hi2 = acc[i][t + NP][r];
                        acc[i][t][r] = lo * c - hi2 * sn;
                        acc[i][t + NP][r] = hi2 * c + lo * sn;
                        fr *= r1;
                    }
                    f *= r8;
                }
            }
        }
        if (!mvalid) continue;

#pragma unroll
        for (int t = 0; t < NSUB; ++t) {
            const int tq = NSUB == 4 ? t : half + 2 * t;
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int d0 = 32 * tq + 8 * rq + 4 * hi;
                uint2 w;
                w.x = (uint32_t)fc_bf16_bits(acc[i][t][4 * rq]) | ((uint32_t)fc_bf16_bits(acc[i][t][4 * rq + 1]) << 16);
                w.y = (uint32_t)fc_bf16_bits(acc[i][t][4 * rq + 2]) | ((uint32_t)fc_bf16_bits(acc[i][t][4 * rq + 3]) << 16);
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
    }
}

template <int KS, int NW, int NSUB, int MW, int NG, int SLOTS, int NL, int EPI = 0>
hipError_t launch_gemm(GemmArgs a, hipStream_t s)
{
    constexpr int XROWS = 32 * MW * (NW / NG);
    constexpr bool DEALT = NSUB == 5 || NSUB == 3;
    constexpr int LDS = SLOTS * ((DEALT ? 32 * NSUB : 32 * NSUB * NG) + XROWS) * KS * 2;
    static_assert(LDS <= 160 * 1024, "LDS ring too large");
    static hipError_t attr = hipFuncSetAttribute((const void *)k_proj_gemm<KS, NW, NSUB, MW, NG, SLOTS, NL, EPI>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (attr != hipSuccess) return attr;
    const int slots = a.slots_here;
    a.n_units = DEALT ? (a.n_slots * 64 + 16 * NSUB - 1) / (16 * NSUB) : NSUB == 4 ? (slots + NG - 1) / NG : 2 * slots;
    if (DEALT && (a.slot_base != 0 || slots != a.n_slots)) return hipErrorInvalidValue;  // dealt pairs cover every slab
    a.n_mt = (a.m_end - a.m_base + XROWS - 1) / XROWS;
    if (slots < 1 || a.n_mt < 1 || a.slot_base < 0 || a.slot_base + slots > a.n_slots || a.m_base < 0 || a.m_end > a.M)
        return hipErrorInvalidValue;
    const int64_t n_tiles = (int64_t)a.n_units * a.n_mt * (EPI == 3 ? a.ksplit : 1);
    if (n_tiles > (1 << 30) || (EPI == 3 && a.ksplit < 1)) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)((n_tiles + 7) / 8 * 8);
    k_proj_gemm<KS, NW, NSUB, MW, NG, SLOTS, NL, EPI><<<dim3(grid), dim3((NW + NL) * 64), LDS, s>>>(a);
    return hipGetLastError();
}

// Sum of the hidden-dimension parts of an EPI 3 launch + residual, four outputs per thread.
__global__ __launch_bounds__(256) void k_splitk_finish(const float *__restrict__ part, const uint16_t *res,
                                                       uint16_t *out, size_t quads, size_t plane, int ksplit)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= quads) return;
    float4 a = *(const float4 *)(part + 4 * i);
    for (int k = 1; k < ksplit; ++k) {
        const float4 b = *(const float4 *)(part + (size_t)k * plane + 4 * i);
        a.x += b.x;
        a.y += b.y;
        a.z += b.z;
        a.w += b.w;
    }
    if (res) {
        const uint2 rv = *(const uint2 *)(res + 4 * i);
        a.x += __uint_as_float(rv.x << 16);
        a.y += __uint_as_float(rv.x & 0xffff0000u);
        a.z += __uint_as_float(rv.y << 16);
        a.w += __uint_as_float(rv.y & 0xffff0000u);
    }
    uint2 w;
    w.x = (uint32_t)fc_bf16_bits(a.x) | ((uint32_t)fc_bf16_bits(a.y) << 16);
    w.y = (uint32_t)fc_bf16_bits(a.z) | ((uint32_t)fc_bf16_bits(a.w) << 16);
    *(uint2 *)(out + 4 * i) = w;
}

template <int EPI>
hipError_t launch_wide_shape(int shape, const GemmArgs &a, hipStream_t s)
{
    if (shape == 4) {  // 256 rows x 80 dealt pairs (gated layer only)
        if constexpr (EPI == 2) return launch_gemm<64, 8, 5, 2, 2, 3, 0, EPI>(a, s);
        else return hipErrorInvalidValue;
    }
    if (shape == 0) return launch_gemm<64, 8, 4, 1, 1, 3, 0, EPI>(a, s);  // 256 rows x slab
    if (shape == 1) return launch_gemm<64, 4, 4, 1, 1, 4, 4, EPI>(a, s);  // 128 rows x slab
    return launch_gemm<64, 4, 2, 1, 1, 4, 4, EPI>(a, s);                  // 128 rows x half slab
}

// Tile choice: the largest tile that still gives the chip about one workgroup per compute unit.
// 0: 256 rows x slab, 1: 128 rows x slab, 2: 128 rows x half slab.
int pick_shape(int64_t slots, int64_t rows, bool allow_half)
{
    // Up to 128 rows the 256-row tile is mostly padding; with that many slabs the half slab is the
    // fastest (gated W_1 of the 7B widths, 296 slabs, 48 / 64 / 128 rows: 67.6 / 71.7 / 83.8 us against
    // 72.9 / 74.4 / 85.1 with whole slabs and 81.8 / 80.7 / 88.7 with the 256-row tile).
    if (rows <= 128 && slots >= 192) return allow_half ? 2 : 1;
    if (slots * ((rows + 255) / 256) >= 192) return 0;
    if (slots * ((rows + 127) / 128) >= 144 || !allow_half) return 1;
    return 2;
}

// One workgroup of the 256-row shape fills a compute unit, so a grid of a little more than 256 such
// workgroups ends with a nearly empty second round.  Such a problem is cut in two: one round in the
// 256-row shape and the rest -- the other slabs when there is one row tile (256 rows x 296 slabs:
// 115 -> 96 us), else the last rows (36 slabs x 8 row tiles: 7 row tiles, then the last 256 rows) -- as
// a second launch with the (smaller) tile that suits it.  Grids of several rounds are left alone
// (cutting them was measured slower).
struct GemmPiece {
    int shape, slot_base, slots, m_base, m_end;
};
int plan_pieces(int slots, int M, bool allow_half, bool allow_dealt, GemmPiece out[2])
{
    out[0] = GemmPiece{pick_shape(slots, M, allow_half), 0, slots, 0, M};
    const bool no_split = fc_knobs().gemm_no_split != 0;  // tuning knob
    if (out[0].shape != 0 || no_split) return 1;
    const int64_t mt = (M + 255) / 256, tiles = (int64_t)slots * mt, rounds = tiles / 256, rem = tiles % 256;
    if (rounds != 1 || rem == 0 || rem > 160) return 1;
    // Layers whose weight rows come in pairs (rotary pairs, gate and up rows) have a fifth shape, 256
    // rows x 80 dealt pairs: a quarter more work per workgroup, so up to 320 tiles of the 256-row shape
    // still make one round, in one launch (36 head slots x 8 row tiles: 89.5 -> 82.5 us; 296 gated slabs
    // x 256 rows: 98.5 -> 88.5 us).
    if (allow_dealt && (((int64_t)slots * 64 + 79) / 80) * mt <= 256) {
        out[0].shape = 4;
        return 1;
    }
    if (mt == 1) {
        out[0].slots = 256;
        out[1] = GemmPiece{pick_shape(slots - 256, M, allow_half), 256, slots - 256, 0, M};
    } else {
        const int mt1 = 256 / slots;  // row tiles of the first round
        if (mt1 * slots < 224) return 1;
        out[0].m_end = mt1 * 256;
        out[1] = GemmPiece{pick_shape(slots, M - mt1 * 256, allow_half), 0, slots, mt1 * 256, M};
    }
    return 2;
}

template <int EPI>
hipError_t launch_pieces(GemmArgs a, bool allow_half, hipStream_t s)
{
    GemmPiece pc[2];
    const int n = plan_pieces(a.n_slots, a.M, allow_half, EPI == 2, pc);
    for (int i = 0; i < n; ++i) {
        a.slot_base = pc[i].slot_base;
        a.slots_here = pc[i].slots;
        a.m_base = pc[i].m_base;
        a.m_end = pc[i].m_end;
        const hipError_t e = launch_wide_shape<EPI>(pc[i].shape, a, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

// Tiled-GEMM plan of a plain linear layer on more than 32 rows (host, pure function of the shape).
FcWidePlan fc_plan_wide(int dtype, int mode, int M, int K, int N)
{
    FcWidePlan p;
    p.kind = 0;
    p.shape = 0;
    p.ksplit = 1;
    const int per_slab = mode == FC_LIN_GATE_UP ? 64 : 128;  // FC_LIN_VOCAB: slabs of 128 vocabulary rows
    if (dtype != FC_BF16 || M <= 32 || K < 4 * KS_MIN || K % KS_MIN != 0 || N < per_slab || N % per_slab != 0) return p;
    // 32-bit byte offsets inside X and each weight matrix
    if ((int64_t)N * K * 2 >= ((int64_t)1 << 32) || (int64_t)M * K * 2 >= ((int64_t)1 << 32)) return p;
    p.kind = 1;
    const int64_t units = N / per_slab, t256 = (M + 255) / 256, t128 = (M + 127) / 128;
    // the largest tile that still gives the chip about one workgroup per compute unit; up to 128 rows
    // the 256-row tile is mostly padding (vocabulary projection of the 7B widths at 48 / 64 / 128 rows:
    // 263 / 253 / 271 us with the 128-row tile against 345 / 329 / 323)
    if (M <= 128 && units >= 192) p.shape = mode == FC_LIN_VOCAB ? 1 : 2;
    else if (units * t256 >= 192) p.shape = 0;
    else if (units * t128 >= 144 || mode == FC_LIN_VOCAB) p.shape = 1;
    else p.shape = 2;
    // Too few slabs even for the smallest tile: also cut the hidden dimension (partial sums in fp32).
    // Tile and number of parts are chosen together by a two-term estimate that reproduces the measured
    // order (256 rows, 28 slabs, hidden 18944: 53 us for the 256-row tile in 8 parts, 58 for the 128-row
    // tile in 4, 68 for the half slab in 2; hidden 3584: 24, 20, 18): a workgroup pulls the rows of
    // both its operands at about 50 GB/s, and the partial sums are written and read at about 3 TB/s.
    const int64_t wgs = 2 * units * t128;
    if (mode == FC_LIN_RESIDUAL && p.shape == 2 && wgs < 192) {
        const int64_t stages = K / KS_MIN;
        double best = 1e30;
        for (int sh = 0; sh < 3; ++sh) {
            const int64_t rows = sh == 0 ? 256 : 128, wrows = sh == 2 ? 64 : 128;
            const int64_t tiles = units * (sh == 2 ? 2 : 1) * ((M + rows - 1) / rows);
            for (int64_t ks = 1; ks <= 16; ++ks) {
                if (ks > 1 && ks > stages / 8) break;
                const int64_t wg = tiles * ks;
                if (wg > 288) break;
                const double fill_us = (double)((wg + 255) / 256) * (double)(rows + wrows) * (double)(K / ks) * 2.0 / 50e3;
                const double part_us = ks > 1 ? (double)ks * M * N * 8.0 / 3e6 : 0.0;
                if (fill_us + part_us < best) {
                    best = fill_us + part_us;
                    p.shape = sh;
                    p.ksplit = (int)ks;
                }
            }
        }
    }
    {  // tuning knobs
        const int v = fc_knobs().lin_wide_shape;
        if ((v >= 0 && v <= (mode == FC_LIN_VOCAB ? 1 : 2)) || (v == 4 && mode == FC_LIN_GATE_UP)) p.shape = v;
        const int ks = fc_knobs().lin_ksplit;
        if (ks >= 1 && ks <= 16 && ks <= K / KS_MIN / 4 && mode == FC_LIN_RESIDUAL) p.ksplit = ks;
    }
    return p;
}

size_t fc_wide_workspace(const FcWidePlan &p, int M, int N)
{
    return p.kind == 1 && p.ksplit > 1 ? (size_t)p.ksplit * M * N * sizeof(float) : 0;
}

hipError_t fc_launch_linear_wide(const FcWidePlan &pl, int mode, const void *x, const void *w, const void *w2,
                                 const void *res, int M, int K, int N, void *out, void *workspace, hipStream_t s,
                                 const FcArgmaxPart *am)
{
    if (pl.kind != 1 || (pl.ksplit > 1 && !workspace)) return hipErrorInvalidValue;
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.X = (const uint16_t *)x;
    a.W = (const uint16_t *)w;
    a.W2 = (const uint16_t *)w2;
    a.res = (const uint16_t *)res;
    a.out = (uint16_t *)out;
    a.part = (float *)workspace;
    a.M = M;
    a.A = M;
    a.K = K;
    a.N = N;
    a.n_slots = mode == FC_LIN_GATE_UP ? N / 64 : N / 128;
    a.ksplit = pl.ksplit;
    a.slot_base = 0;
    a.slots_here = a.n_slots;
    a.m_base = 0;
    a.m_end = M;
    const bool forced = fc_knobs().lin_wide_shape >= 0;  // a forced shape is used for the whole problem
    if (mode == FC_LIN_VOCAB) {
        if (!am || pl.shape > 1) return hipErrorInvalidValue;
        a.am = *am;
        return pl.shape == 0 ? launch_gemm<64, 8, 4, 1, 1, 3, 0, 4>(a, s) : launch_gemm<64, 4, 4, 1, 1, 4, 4, 4>(a, s);
    }
    if (mode == FC_LIN_GATE_UP) return forced ? launch_wide_shape<2>(pl.shape, a, s) : launch_pieces<2>(a, true, s);
    if (pl.ksplit <= 1) return forced ? launch_wide_shape<1>(pl.shape, a, s) : launch_pieces<1>(a, true, s);
    hipError_t e = launch_wide_shape<3>(pl.shape, a, s);
    if (e != hipSuccess) return e;
    const size_t quads = (size_t)M * N / 4;
    k_splitk_finish<<<dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s>>>((const float *)workspace, a.res, a.out,
                                                                                  quads, (size_t)M * N, pl.ksplit);
    return hipGetLastError();
}

bool fc_project_gemm_supported(const fc_config &cfg, int M)
{
    // 32-bit byte offsets inside X and W; the hidden dimension in whole stages
    const int64_t n = (int64_t)(cfg.n_q_heads + 2 * cfg.n_kv_heads) * cfg.head_dim;
    return cfg.dtype == FC_BF16 && cfg.head_dim == 128 && cfg.hidden % KS_MIN == 0 && M > 32 &&
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
    a.n_slots = G.Hq + 2 * G.Hkv;
    a.W2 = a.res = nullptr;
    a.out = nullptr;
    a.part = nullptr;
    a.N = 0;
    a.ksplit = 1;
    a.log2_base_64 = G.log_base * 1.4426950408889634074 / 64.0;
    // The two 128-row shapes get four extra waves that only issue the loads (their four multiplying
    // waves are alone on their SIMDs); the half-head shape also takes 128 hidden elements per stage.
    auto launch_shape = [&](int shape, const GemmArgs &g) -> hipError_t {
        if (shape == 4) return launch_gemm<64, 8, 5, 2, 2, 3, 0>(g, s);   // 256 rows x 80 dealt rotary pairs
        if (shape == 5) return launch_gemm<64, 4, 3, 1, 1, 4, 4>(g, s);   // 128 rows x 48 dealt rotary pairs, 4 + 4 waves
        if (shape == 3) return launch_gemm<64, 8, 4, 2, 2, 2, 0>(g, s);   // 256 rows x two heads
        if (shape == 0) return launch_gemm<64, 8, 4, 1, 1, 3, 0>(g, s);   // 256 rows x head
        if (shape == 1) return launch_gemm<64, 4, 4, 1, 1, 4, 4>(g, s);   // 128 rows x head
        if (g.K % 128 == 0) return launch_gemm<128, 4, 2, 1, 1, 3, 4>(g, s);  // 128 rows x half head
        return launch_gemm<64, 4, 2, 1, 1, 4, 4>(g, s);
    };
    a.slot_base = 0;
    a.slots_here = a.n_slots;
    a.m_base = 0;
    a.m_end = a.M;
    if (fc_knobs().proj_gemm_shape >= 0) return launch_shape(fc_knobs().proj_gemm_shape, a);  // tuning knob: one shape for all
    GemmPiece pc[2];
    const int n = plan_pieces(a.n_slots, a.M, true, true, pc);
    if (n == 1 && pc[0].shape == 1) {
        // 128 rows x head leaves compute units idle when the grid is well short of a round (96 head slots
        // x 2 row tiles = 192 workgroups); dealt in units of 48 rotary pairs the same rows make more,
        // smaller workgroups (256 there).  A workgroup's time goes with the rows of both operands it
        // pulls (128 + 128 against 128 + 96): 44.3 -> 40.8 us at 256 rows, 96 slots, hidden 4096.  (64
        // rows x 48 pairs for the 36-slot geometry measured the same as the half-head shape: not used.)
        const int64_t t128 = (a.M + 127) / 128;
        const int64_t wg1 = (int64_t)a.n_slots * t128, wg5 = (((int64_t)a.n_slots * 64 + 47) / 48) * t128;
        if (((wg5 + 255) / 256) * 224 < ((wg1 + 255) / 256) * 256) pc[0].shape = 5;
    }
    for (int i = 0; i < n; ++i) {
        a.slot_base = pc[i].slot_base;
        a.slots_here = pc[i].slots;
        a.m_base = pc[i].m_base;
        a.m_end = pc[i].m_end;
        const hipError_t e = launch_shape(pc[i].shape, a);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}
