// Unmasking step of a diffusion language model on the window rows (paper, section 3.1: the masked set
// M_t, the logits z_t of the masked positions, the arg-max fill of the selected subset U_t; with
// FreeCache, section 3.2.1, only the rows of the active window are evaluated).
//
// The vocabulary projection never writes its logits: every kernel that produces a part of a row's
// logits keeps (largest, its index, sum of exp(logit - largest)) of that part; k_lmhead_reduce merges
// the parts into the arg-max token and its softmax probability 1 / sum.  k_unmask_select then fills,
// per sequence, the n most confident still-masked window positions and lists the positions that stay
// masked (the next step's active rows).
#include <stdlib.h>

#include "fc_device.h"
#include "fc_internal.h"

namespace {

__device__ __forceinline__ float wave_sum_f(float v)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Plain vocabulary projection, block = (row, FC_LMHEAD_GENERIC_CHUNK vocabulary entries); wave w owns
// entries w, w + 4, ... of the chunk (ascending), lanes run along the hidden dimension.
template <typename T>
__global__ __launch_bounds__(256) void k_lmhead_generic(const T *__restrict__ X, const T *__restrict__ W, int M,
                                                        int K, int V, FcArgmaxPart am)
{
    __shared__ float s_mx[4], s_sm[4];
    __shared__ int s_arg[4];
    const int m = blockIdx.x, part = blockIdx.y;
    const int v0 = part * FC_LMHEAD_GENERIC_CHUNK;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const T *x = X + (size_t)m * K;
    float mx = -INFINITY, sm = 0.f;
    int arg = 0;
    for (int c = wave; c < FC_LMHEAD_GENERIC_CHUNK; c += 4) {
        const int v = v0 + c;
        if (v >= V) break;
        const T *w = W + (size_t)v * K;
        float acc = 0.f;
        for (int k = lane; k < K; k += 64) acc += fc_to_float(w[k]) * fc_to_float(x[k]);
        const float z = wave_sum_f(acc);
        fc_argmax_merge(mx, arg, sm, z, v, 1.0f);
    }
    if (lane == 0) {
        s_mx[wave] = mx;
        s_sm[wave] = sm;
        s_arg[wave] = arg;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w2 = 1; w2 < 4; ++w2) fc_argmax_merge(mx, arg, sm, s_mx[w2], s_arg[w2], s_sm[w2]);
        const size_t at = (size_t)part * M + m;
        am.mx[at] = mx;
        am.arg[at] = arg;
        am.sm[at] = sm;
    }
}

// Merge of the vocabulary parts of one row: one workgroup per row.
__global__ __launch_bounds__(256) void k_lmhead_reduce(FcArgmaxPart am, int parts, int M, int32_t *tok, float *conf)
{
    __shared__ float s_mx[4], s_sm[4];
    __shared__ int s_arg[4];
    const int m = blockIdx.x, tid = threadIdx.x;
    float mx = -INFINITY, sm = 0.f;
    int arg = 0x7fffffff;
    for (int base = 0; base < parts; base += 256 * 8) {  // eight parts per thread in flight at a time
        float vmx[8], vsm[8];
        int varg[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int pt = base + 256 * u + tid;
            const size_t at = (size_t)min(pt, parts - 1) * M + m;
            vmx[u] = am.mx[at];
            varg[u] = am.arg[at];
            vsm[u] = am.sm[at];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (base + 256 * u + tid < parts) fc_argmax_merge(mx, arg, sm, vmx[u], varg[u], vsm[u]);
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float mx2 = __shfl_xor(mx, off, 64), sm2 = __shfl_xor(sm, off, 64);
        const int arg2 = __shfl_xor(arg, off, 64);
        fc_argmax_merge(mx, arg, sm, mx2, arg2, sm2);
    }
    if ((tid & 63) == 0) {
        s_mx[tid >> 6] = mx;
        s_sm[tid >> 6] = sm;
        s_arg[tid >> 6] = arg;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w2 = 1; w2 < 4; ++w2) fc_argmax_merge(mx, arg, sm, s_mx[w2], s_arg[w2], s_sm[w2]);
        tok[m] = arg;
        conf[m] = 1.0f / sm;
    }
}

// Confidence-ranked fill, one block per sequence.  A candidate is a window row whose position is valid
// and whose token is still the mask.  Its rank is the number of candidates that come before it in the
// order (larger confidence first, then smaller row); ranks below n_unmask are filled.  The remaining
// candidates are listed in row order (block-wide prefix sum over chunks of 256 rows).
__global__ __launch_bounds__(256) void k_unmask_select(const int32_t *__restrict__ tok, const float *__restrict__ conf,
                                                       const int32_t *__restrict__ pos, int win_start, int A,
                                                       int n_unmask, int mask_id, int32_t *tokens, int L,
                                                       int32_t *pos_next, int32_t *count_next)
{
    extern __shared__ unsigned char sm_raw[];
    float *s_conf = (float *)sm_raw;            // [A]; -1 marks "not a candidate" (confidences are > 0)
    int *s_scan = (int *)(s_conf + A);          // [256]
    __shared__ int s_base;
    const int b = blockIdx.x, tid = threadIdx.x;
    int32_t *seq = tokens + (size_t)b * L;
    auto position = [&](int a) { return pos ? pos[(size_t)b * A + a] : win_start + a; };

    for (int a = tid; a < A; a += 256) {
        const int p = position(a);
        const bool cand = p >= 0 && p < L && seq[p] == mask_id;
        s_conf[a] = cand ? conf[(size_t)b * A + a] : -1.0f;
    }
    if (tid == 0) s_base = 0;
    __syncthreads();

    for (int a0 = 0; a0 < A; a0 += 256) {
        const int a = a0 + tid;
        bool keep = false;  // candidate that stays masked
        if (a < A && s_conf[a] >= 0.f) {
            const float c = s_conf[a];
            int rank = 0;
            for (int o = 0; o < A; ++o) {
                const float co = s_conf[o];
                rank += (co > c || (co == c && o < a)) ? 1 : 0;  // non-candidates hold -1 and never count
            }
            if (rank < n_unmask)
                seq[position(a)] = tok[(size_t)b * A + a];
            else
                keep = true;
        }
        // inclusive scan of `keep` over the 256 rows of this chunk
        s_scan[tid] = keep ? 1 : 0;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const int v = tid >= off ? s_scan[tid - off] : 0;
            __syncthreads();
            s_scan[tid] += v;
            __syncthreads();
        }
        const int base = s_base;
        if (keep) pos_next[(size_t)b * A + base + s_scan[tid] - 1] = position(a);
        __syncthreads();
        if (tid == 255) s_base = base + s_scan[255];
        __syncthreads();
    }
    const int n = s_base;
    for (int a = n + tid; a < A; a += 256) pos_next[(size_t)b * A + a] = -1;
    if (tid == 0) count_next[b] = n;
}

// -------------------------------------------------------------------------------------------------
// Guided Diffusion acceptance (paper, section 3.2.2, Algorithm 1; Top-K match and threshold tau from the
// implementation details).  k_accept_scan: several workgroups per still masked window row, each scans a
// part of the row's two logit vectors (DLM and AR guide): largest DLM logit, the topk best entries of
// the AR row (every thread keeps its own best list; the lists are merged by topk rounds of a block-wide
// arg-max).  k_accept_rowmerge: one wave per row merges the parts the same way and decides whether the
// row matches.  k_accept_seq: one workgroup per sequence finds the longest matching prefix of the masked
// rows, fills it (or the first masked row) and lists the rest.
constexpr int ACC_MAXK = 8;

// (value, id) order: larger value first, then smaller id
__device__ __forceinline__ bool acc_before(float v1, int i1, float v2, int i2) { return v1 > v2 || (v1 == v2 && i1 < i2); }

// Partial results of one part of a row's vocabulary: DLM (largest, id) and the AR's topk best, best first.
struct AccPart {
    float dv;
    int di;
    float tv[ACC_MAXK];
    int ti[ACC_MAXK];
};

// grid (parts, A, B): workgroup (part, a, b) scans entries [part * chunk, (part + 1) * chunk) of row (b, a).
__global__ __launch_bounds__(256) void k_accept_scan(const float *__restrict__ dlm, const float *__restrict__ ar,
                                                     const int32_t *__restrict__ pos, int win_start, int A, int V,
                                                     int chunk, int topk, int mask_id, const int32_t *tokens, int L,
                                                     AccPart *parts)
{
    __shared__ float s_v[256];
    __shared__ int s_i[256];
    __shared__ int s_who;
    const int part = blockIdx.x, a = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int p = pos ? pos[(size_t)b * A + a] : win_start + a;
    const size_t at = (size_t)b * A + a;
    if (!(p >= 0 && p < L && tokens[(size_t)b * L + p] == mask_id)) return;  // not a candidate: nothing to scan
    const float *zd = dlm + at * V, *za = ar + at * V;
    const int v0 = part * chunk, v1 = min(V, v0 + chunk);
    // DLM arg-max and this thread's topk best AR entries (sorted best first)
    float dv = -INFINITY;
    int di = 0x7fffffff;
    float tv[ACC_MAXK];
    int ti[ACC_MAXK];
#pragma unroll
    for (int r = 0; r < ACC_MAXK; ++r) {
        tv[r] = -INFINITY;
        ti[r] = 0x7fffffff;
    }
    float worst_v = -INFINITY;  // the list's last kept entry: most elements fail against it and cost two compares
    int worst_i = 0x7fffffff;
    auto visit = [&](float d, float x, int v) {
        if (acc_before(d, v, dv, di)) {
            dv = d;
            di = v;
        }
        if (!acc_before(x, v, worst_v, worst_i)) return;
        int xi = v;
#pragma unroll
        for (int r = 0; r < ACC_MAXK; ++r) {  // insertion into the sorted list
            if (r < topk && acc_before(x, xi, tv[r], ti[r])) {
                const float t0 = tv[r];
                const int t1 = ti[r];
                tv[r] = x;
                ti[r] = xi;
                x = t0;
                xi = t1;
            }
        }
#pragma unroll
        for (int r = 0; r < ACC_MAXK; ++r)
            if (r == topk - 1) {
                worst_v = tv[r];
                worst_i = ti[r];
            }
    };
    // rows of V floats are 16-byte aligned when V is a multiple of 4 (chunk always is): four entries per load
    if ((V & 3) == 0) {
        for (int v = v0 + 4 * tid; v < v1; v += 1024) {
            const float4 d4 = *(const float4 *)(zd + v), x4 = *(const float4 *)(za + v);
            visit(d4.x, x4.x, v);
            visit(d4.y, x4.y, v + 1);
            visit(d4.z, x4.z, v + 2);
            visit(d4.w, x4.w, v + 3);
        }
    } else {
        for (int v = v0 + tid; v < v1; v += 256) visit(zd[v], za[v], v);
    }
    // block arg-max of the DLM part
    s_v[tid] = dv;
    s_i[tid] = di;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (tid < off && acc_before(s_v[tid + off], s_i[tid + off], s_v[tid], s_i[tid])) {
            s_v[tid] = s_v[tid + off];
            s_i[tid] = s_i[tid + off];
        }
        __syncthreads();
    }
    AccPart *out = parts + at * gridDim.x + part;
    if (tid == 0) {
        out->dv = s_v[0];
        out->di = s_i[0];
    }
    __syncthreads();
    // topk rounds: the best head among the threads' lists is the next entry of the part's list
    for (int r = 0; r < topk; ++r) {
        s_v[tid] = tv[0];
        s_i[tid] = ti[0];
        __syncthreads();
        for (int off = 128; off > 0; off >>= 1) {
            if (tid < off && acc_before(s_v[tid + off], s_i[tid + off], s_v[tid], s_i[tid])) {
                s_v[tid] = s_v[tid + off];
                s_i[tid] = s_i[tid + off];
            }
            __syncthreads();
        }
        const float bv = s_v[0];
        const int bi = s_i[0];
        if (tid == 0) {
            out->tv[r] = bv;  // (-inf, int max) once the part is exhausted
            out->ti[r] = bi;
            s_who = -1;
        }
        __syncthreads();
        if (ti[0] == bi && bi != 0x7fffffff) s_who = tid;  // ids are unique: one thread owns the winner
        __syncthreads();
        if (s_who == tid) {  // pop the head
#pragma unroll
            for (int q = 0; q + 1 < ACC_MAXK; ++q) {
                tv[q] = tv[q + 1];
                ti[q] = ti[q + 1];
            }
            tv[ACC_MAXK - 1] = -INFINITY;
            ti[ACC_MAXK - 1] = 0x7fffffff;
        }
        __syncthreads();
    }
}

// One wave per row merges the parts (at most 64, one per lane) and decides whether the row matches.
__global__ __launch_bounds__(64) void k_accept_rowmerge(const AccPart *__restrict__ parts, int n_parts,
                                                        const int32_t *__restrict__ pos, int win_start, int A, int topk,
                                                        float tau, int mask_id, const int32_t *tokens, int L,
                                                        int32_t *row_tok, int32_t *row_match)
{
    const int a = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const int p = pos ? pos[(size_t)b * A + a] : win_start + a;
    const size_t at = (size_t)b * A + a;
    if (!(p >= 0 && p < L && tokens[(size_t)b * L + p] == mask_id)) {
        if (lane == 0) {
            row_tok[at] = -1;
            row_match[at] = -1;
        }
        return;
    }
    float dv = -INFINITY;
    int di = 0x7fffffff;
    float tv[ACC_MAXK];
    int ti[ACC_MAXK];
#pragma unroll
    for (int r = 0; r < ACC_MAXK; ++r) {
        tv[r] = -INFINITY;
        ti[r] = 0x7fffffff;
    }
    if (lane < n_parts) {
        const AccPart *pt = parts + at * n_parts + lane;
        dv = pt->dv;
        di = pt->di;
#pragma unroll
        for (int r = 0; r < ACC_MAXK; ++r)
            if (r < topk) {
                tv[r] = pt->tv[r];
                ti[r] = pt->ti[r];
            }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float v2 = __shfl_xor(dv, off, 64);
        const int i2 = __shfl_xor(di, off, 64);
        if (acc_before(v2, i2, dv, di)) {
            dv = v2;
            di = i2;
        }
    }
    bool in_top = false;
    float za_max = 0.f;
    for (int r = 0; r < topk; ++r) {
        float bv = tv[0];
        int bi = ti[0];
        for (int off = 32; off > 0; off >>= 1) {
            const float v2 = __shfl_xor(bv, off, 64);
            const int i2 = __shfl_xor(bi, off, 64);
            if (acc_before(v2, i2, bv, bi)) {
                bv = v2;
                bi = i2;
            }
        }
        if (r == 0) za_max = bv;
        if (bi == di) in_top = true;
        if (ti[0] == bi && bi != 0x7fffffff) {  // this lane owns the winner: pop
#pragma unroll
            for (int q = 0; q + 1 < ACC_MAXK; ++q) {
                tv[q] = tv[q + 1];
                ti[q] = ti[q + 1];
            }
            tv[ACC_MAXK - 1] = -INFINITY;
            ti[ACC_MAXK - 1] = 0x7fffffff;
        }
    }
    if (lane == 0) {
        const float thr = tau * za_max;
        row_tok[at] = di;
        row_match[at] = (in_top && (!(tau > 0.0f) || dv > thr)) ? 1 : 0;
    }
}

__global__ __launch_bounds__(256) void k_accept_seq(const int32_t *__restrict__ row_tok, const int32_t *__restrict__ row_match,
                                                    const int32_t *__restrict__ pos, int win_start, int A,
                                                    int32_t *tokens, int L, int32_t *n_accept, int32_t *pos_next,
                                                    int32_t *count_next)
{
    __shared__ int s_scan[256];
    __shared__ int s_base, s_first_miss;
    const int b = blockIdx.x, tid = threadIdx.x;
    int32_t *seq = tokens + (size_t)b * L;
    auto position = [&](int a) { return pos ? pos[(size_t)b * A + a] : win_start + a; };
    if (tid == 0) {
        s_base = 0;
        s_first_miss = 0x7fffffff;
    }
    __syncthreads();
    // pass 1: index j of every masked row among the masked rows; the first j that does not match
    for (int a0 = 0; a0 < A; a0 += 256) {
        const int a = a0 + tid;
        const int mt = a < A ? row_match[(size_t)b * A + a] : -1;
        s_scan[tid] = mt >= 0 ? 1 : 0;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const int v = tid >= off ? s_scan[tid - off] : 0;
            __syncthreads();
            s_scan[tid] += v;
            __syncthreads();
        }
        if (mt == 0) atomicMin(&s_first_miss, s_base + s_scan[tid] - 1);
        __syncthreads();
        if (tid == 255) s_base += s_scan[255];
        __syncthreads();
    }
    const int m = s_base;                                  // masked rows
    const int k = min(s_first_miss, m);                    // longest matching prefix
    const int n = m == 0 ? 0 : (k > 0 ? k : 1);
    __syncthreads();
    if (tid == 0) s_base = 0;
    __syncthreads();
    // pass 2: fill the first n masked rows, list the others
    for (int a0 = 0; a0 < A; a0 += 256) {
        const int a = a0 + tid;
        const int mt = a < A ? row_match[(size_t)b * A + a] : -1;
        s_scan[tid] = mt >= 0 ? 1 : 0;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const int v = tid >= off ? s_scan[tid - off] : 0;
            __syncthreads();
            s_scan[tid] += v;
            __syncthreads();
        }
        if (mt >= 0) {
            const int j = s_base + s_scan[tid] - 1;
            if (j < n)
                seq[position(a)] = row_tok[(size_t)b * A + a];
            else
                pos_next[(size_t)b * A + (j - n)] = position(a);
        }
        __syncthreads();
        if (tid == 255) s_base += s_scan[255];
        __syncthreads();
    }
    for (int a = m - n + tid; a < A; a += 256) pos_next[(size_t)b * A + a] = -1;
    if (tid == 0) {
        n_accept[b] = n;
        count_next[b] = m - n;
    }
}

// Row gather in 16-byte pieces: out[i] = table[idx[i]], zeros for a negative or too large index.
__global__ __launch_bounds__(256) void k_gather_rows(const uint4 *__restrict__ table, int64_t R, int pieces,
                                                     const int32_t *__restrict__ idx, uint4 *__restrict__ out)
{
    const int64_t i = blockIdx.x;
    const int32_t r = idx[i];
    const bool ok = r >= 0 && r < R;
    for (int c = threadIdx.x; c < pieces; c += 256)
        out[i * pieces + c] = ok ? table[(int64_t)r * pieces + c] : make_uint4(0, 0, 0, 0);
}

}  // namespace

// Parts a row's vocabulary is cut into: several workgroups per compute unit (measured: 20.7 us with 2048
// workgroups, 26.6 with 512, 37.5 with 256 for a 32-row block at vocabulary 152064), chunks of whole float4s.
int fc_accept_parts(int B, int A, int V)
{
    const int target = fc_knobs().accept_wgs > 0 ? fc_knobs().accept_wgs : 2048;  // tuning knob
    int64_t parts = (target > 0 ? target : 2048) / ((int64_t)B * A);
    if (parts > 64) parts = 64;
    if (parts > (V + 2047) / 2048) parts = (V + 2047) / 2048;  // at least 2048 entries per part
    if (parts < 1) parts = 1;
    return (int)parts;
}

size_t fc_accept_workspace(int B, int A, int V)
{
    return (size_t)2 * B * A * sizeof(int32_t) + (size_t)B * A * fc_accept_parts(B, A, V) * sizeof(AccPart);
}

hipError_t fc_launch_guided_accept(const float *dlm, const float *ar, const int32_t *pos, int win_start, int B, int A,
                                   int V, int topk, float tau, int mask_id, int32_t *tokens, int L, int32_t *n_accept,
                                   int32_t *pos_next, int32_t *count_next, void *workspace, hipStream_t s)
{
    if (topk < 1 || topk > ACC_MAXK || !workspace) return hipErrorInvalidValue;
    const int n_parts = fc_accept_parts(B, A, V);
    const int chunk = (((V + n_parts - 1) / n_parts) + 3) & ~3;
    int32_t *row_tok = (int32_t *)workspace, *row_match = row_tok + (size_t)B * A;
    AccPart *parts = (AccPart *)(row_match + (size_t)B * A);
    k_accept_scan<<<dim3((unsigned)n_parts, (unsigned)A, (unsigned)B), dim3(256), 0, s>>>(dlm, ar, pos, win_start, A, V,
                                                                                          chunk, topk, mask_id, tokens, L,
                                                                                          parts);
    k_accept_rowmerge<<<dim3((unsigned)A, (unsigned)B), dim3(64), 0, s>>>(parts, n_parts, pos, win_start, A, topk, tau,
                                                                          mask_id, tokens, L, row_tok, row_match);
    k_accept_seq<<<dim3((unsigned)B), dim3(256), 0, s>>>(row_tok, row_match, pos, win_start, A, tokens, L, n_accept,
                                                         pos_next, count_next);
    return hipGetLastError();
}

hipError_t fc_launch_gather_rows(const void *table, int64_t R, int row_bytes, const int32_t *idx, int64_t n, void *out,
                                 hipStream_t s)
{
    k_gather_rows<<<dim3((unsigned)n), dim3(256), 0, s>>>((const uint4 *)table, R, row_bytes / 16, idx, (uint4 *)out);
    return hipGetLastError();
}

hipError_t fc_launch_lmhead_generic(int dtype, const void *x, const void *w, int M, int K, int V,
                                    const FcArgmaxPart &am, hipStream_t s)
{
    const dim3 grid((unsigned)M, (unsigned)((V + FC_LMHEAD_GENERIC_CHUNK - 1) / FC_LMHEAD_GENERIC_CHUNK));
    if (dtype == FC_F32)
        k_lmhead_generic<float><<<grid, dim3(256), 0, s>>>((const float *)x, (const float *)w, M, K, V, am);
    else
        k_lmhead_generic<bf16_t><<<grid, dim3(256), 0, s>>>((const bf16_t *)x, (const bf16_t *)w, M, K, V, am);
    return hipGetLastError();
}

hipError_t fc_launch_lmhead_reduce(const FcArgmaxPart &am, int parts, int M, int32_t *tok, float *conf,
                                   hipStream_t s)
{
    k_lmhead_reduce<<<dim3((unsigned)M), dim3(256), 0, s>>>(am, parts, M, tok, conf);
    return hipGetLastError();
}

hipError_t fc_launch_unmask_select(const int32_t *tok, const float *conf, const int32_t *pos, int win_start,
                                   int B, int A, int n_unmask, int mask_id, int32_t *tokens, int L,
                                   int32_t *pos_next, int32_t *count_next, hipStream_t s)
{
    if (A > FC_UNMASK_MAX_ROWS) return hipErrorInvalidValue;
    const size_t lds = (size_t)A * sizeof(float) + 256 * sizeof(int);
    k_unmask_select<<<dim3((unsigned)B), dim3(256), lds, s>>>(tok, conf, pos, win_start, A, n_unmask, mask_id, tokens, L,
                                                               pos_next, count_next);
    return hipGetLastError();
}
