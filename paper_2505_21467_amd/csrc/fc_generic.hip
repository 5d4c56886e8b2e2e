// Plain-ALU kernels of the cached layer-step for any supported dtype / head_dim.
//
// They are the whole path for fp32 caches (the small full-precision configuration) and for bf16
// shapes the matrix-core kernels do not cover.  Arithmetic: fp32 accumulation everywhere, rotary
// angles reduced in double, results rounded once to the storage dtype.
#include "fc_device.h"
#include "fc_internal.h"

namespace {

__device__ __forceinline__ float wave_sum(float v)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// ---------------------------------------------------------------------------------------------
// Row copies between the plain [B][Hkv][rows][Dh] layout and the cache layout.
template <typename T>
__global__ __launch_bounds__(256) void k_copy_rows(FcGeom G, T *__restrict__ kc, T *__restrict__ vc,
                                                   T *__restrict__ kr, T *__restrict__ vr, int start,
                                                   int rows, bool to_cache)
{
    const size_t total = (size_t)G.B * G.Hkv * rows * G.Dh;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (size_t)gridDim.x * blockDim.x) {
        const int i = (int)(e % G.Dh);
        size_t r = e / G.Dh;
        const int row = (int)(r % rows);
        r /= rows;
        const int j = (int)(r % G.Hkv);
        const int b = (int)(r / G.Hkv);
        const size_t ki = fc_k_index(G, b, j, start + row, i);
        const size_t vi = fc_v_index(G, b, j, start + row, i);
        if (to_cache) {
            kc[ki] = kr[e];
            vc[vi] = vr[e];
        } else {
            kr[e] = kc[ki];
            vr[e] = vc[vi];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Projection + RoPE + scatter.  Block = (4 rows, one head slot); each wave owns every 4th output
// column of the head and runs the dot product with lanes along the hidden dimension.
constexpr int PG_ROWS = 4;

template <typename T>
__global__ __launch_bounds__(256) void k_project_generic(FcGeom G, const T *__restrict__ X,
                                                         const T *__restrict__ W,
                                                         const T *__restrict__ bias,
                                                         const int32_t *__restrict__ pos, int win_start,
                                                         int A, T *__restrict__ Q, T *__restrict__ Kc,
                                                         T *__restrict__ Vc)
{
    __shared__ float y[PG_ROWS][128];
    const int hs = blockIdx.y;  // head slot: q heads, then k heads, then v heads
    const int m0 = blockIdx.x * PG_ROWS;
    const int M = G.B * A;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;

    for (int i = wave; i < G.Dh; i += 4) {
        const int n = hs * G.Dh + i;
        const T *w = W + (size_t)n * G.d;
        float acc[PG_ROWS];
#pragma unroll
        for (int r = 0; r < PG_ROWS; ++r) acc[r] = 0.f;
        for (int k = lane; k < G.d; k += 64) {
            const float wv = fc_to_float(w[k]);
#pragma unroll
            for (int r = 0; r < PG_ROWS; ++r)
                if (m0 + r < M) acc[r] += wv * fc_to_float(X[(size_t)(m0 + r) * G.d + k]);
        }
#pragma unroll
        for (int r = 0; r < PG_ROWS; ++r) {
            const float s = wave_sum(acc[r]);
            if (lane == 0) y[r][i] = s + (bias ? fc_to_float(bias[n]) : 0.f);
        }
    }
    __syncthreads();

    const int half = G.Dh / 2;
    for (int idx = threadIdx.x; idx < PG_ROWS * half; idx += 256) {
        const int r = idx / half, i = idx % half;
        const int m = m0 + r;
        if (m >= M) continue;
        const int b = m / A, a = m % A;
        const int p = pos ? pos[m] : win_start + a;
        const bool valid = p >= 0 && p < G.max_seq;
        float y0 = y[r][i], y1 = y[r][i + half];
        if (hs < G.Hq + G.Hkv && valid) {
            float c, s;
            fc_rope_cs(p, i, G.Dh, G.log_base, &c, &s);
            const float r0 = y0 * c - y1 * s;
            const float r1 = y1 * c + y0 * s;
            y0 = r0;
            y1 = r1;
        }
        if (hs < G.Hq) {
            T *q = Q + (((size_t)b * G.Hq + hs) * A + a) * G.Dh;
            q[i] = fc_from_float<T>(valid ? y0 : 0.f);
            q[i + half] = fc_from_float<T>(valid ? y1 : 0.f);
        } else if (valid) {
            if (hs < G.Hq + G.Hkv) {
                const int j = hs - G.Hq;
                Kc[fc_k_index(G, b, j, p, i)] = fc_from_float<T>(y0);
                Kc[fc_k_index(G, b, j, p, i + half)] = fc_from_float<T>(y1);
            } else {
                const int j = hs - G.Hq - G.Hkv;
                Vc[fc_v_index(G, b, j, p, i)] = fc_from_float<T>(y0);
                Vc[fc_v_index(G, b, j, p, i + half)] = fc_from_float<T>(y1);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Attention, one block per (query row, head, sequence); keys in chunks of 256 with an online
// softmax (running max m, running sum l, rescaled accumulator).
template <typename T>
__global__ __launch_bounds__(256) void k_attention_generic(FcGeom G, const T *__restrict__ Q,
                                                           const T *__restrict__ Kc,
                                                           const T *__restrict__ Vc,
                                                           const int32_t *__restrict__ pos, int A,
                                                           int kv_len, T *__restrict__ O)
{
    __shared__ float qs[128];
    __shared__ float ps[256];
    __shared__ float red[4];
    const int a = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    T *o = O + ((size_t)b * A + a) * ((size_t)G.Hq * G.Dh) + (size_t)h * G.Dh;
    if (pos) {  // padded row: same rule as the projection (negative or beyond the cache)
        const int p = pos[b * A + a];
        if (p < 0 || p >= G.max_seq) {
            if (tid < G.Dh) o[tid] = fc_from_float<T>(0.f);
            return;
        }
    }
    const int j = h / G.g;
    if (tid < G.Dh) qs[tid] = fc_to_float(Q[(((size_t)b * G.Hq + h) * A + a) * G.Dh + tid]);
    __syncthreads();

    float m = -INFINITY, l = 0.f, acc = 0.f;
    for (int c0 = 0; c0 < kv_len; c0 += 256) {
        const int t = c0 + tid;
        float s = -INFINITY;
        if (t < kv_len) {
            const T *k = Kc + fc_k_index(G, b, j, t, 0);
            float dot = 0.f;
            for (int i = 0; i < G.Dh; ++i) dot += qs[i] * fc_to_float(k[i]);
            s = dot * G.scale;
        }
        float mx = wave_max(s);
        if (lane == 0) red[wave] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        const float m_new = fmaxf(m, mx);
        const float p = (t < kv_len) ? expf(s - m_new) : 0.f;
        ps[tid] = p;
        float sum = wave_sum(p);
        __syncthreads();  // everyone has read red[] for the max; ps[] is complete after this
        if (lane == 0) red[wave] = sum;
        __syncthreads();
        sum = red[0] + red[1] + red[2] + red[3];
        const float alpha = (m == -INFINITY) ? 0.f : expf(m - m_new);
        l = l * alpha + sum;
        m = m_new;
        if (tid < G.Dh) {
            const int n = min(256, kv_len - c0);
            float part = 0.f;
            for (int u = 0; u < n; ++u) part += ps[u] * fc_to_float(Vc[fc_v_index(G, b, j, c0 + u, tid)]);
            acc = acc * alpha + part;
        }
        __syncthreads();  // ps[] and red[] are rewritten by the next chunk
    }
    if (tid < G.Dh) o[tid] = fc_from_float<T>(acc / l);
}

// ---------------------------------------------------------------------------------------------
// RMS normalisation, one block per row: out = x / sqrt(mean(x^2) + eps) * weight.
template <typename T>
__global__ __launch_bounds__(256) void k_rmsnorm(const T *X, const T *__restrict__ w, float eps, int d, T *out)
{
    __shared__ float red[4];
    const size_t row = blockIdx.x;
    const T *x = X + row * d;
    const int tid = threadIdx.x;
    float ss = 0.f;
    for (int k = tid; k < d; k += 256) {
        const float v = fc_to_float(x[k]);
        ss += v * v;
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float tot = (red[0] + red[1]) + (red[2] + red[3]);
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    // out may be x: element k is read and written by the same thread only
    for (int k = tid; k < d; k += 256) out[row * d + k] = fc_from_float<T>(fc_to_float(x[k]) * inv * fc_to_float(w[k]));
}

// bf16 rows whose length is a multiple of 8 and at most 2048 * NJ: every thread keeps its NJ 16-byte
// pieces of the row in registers, so the row is read once.
template <int NJ>
__global__ __launch_bounds__(256) void k_rmsnorm_bf16_row(const uint16_t *X, const uint16_t *__restrict__ w, float eps,
                                                          int d, uint16_t *out)
{
    __shared__ float red[4];
    const size_t row = blockIdx.x;
    const int tid = threadIdx.x, chunks = d >> 3;
    uint4 v[NJ], g[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int c = tid + 256 * j;
        v[j] = c < chunks ? *(const uint4 *)(X + row * d + 8 * c) : make_uint4(0, 0, 0, 0);
        g[j] = c < chunks ? *(const uint4 *)(w + 8 * c) : make_uint4(0, 0, 0, 0);
    }
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const uint32_t u[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float a = __uint_as_float(u[e] << 16), b = __uint_as_float(u[e] & 0xffff0000u);
            ss += a * a;
            ss += b * b;
        }
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float tot = (red[0] + red[1]) + (red[2] + red[3]);
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int c = tid + 256 * j;
        if (c >= chunks) continue;
        const uint32_t u[4] = {v[j].x, v[j].y, v[j].z, v[j].w}, gw[4] = {g[j].x, g[j].y, g[j].z, g[j].w};
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float a = __uint_as_float(u[e] << 16) * inv * __uint_as_float(gw[e] << 16);
            const float b = __uint_as_float(u[e] & 0xffff0000u) * inv * __uint_as_float(gw[e] & 0xffff0000u);
            o[e] = (uint32_t)fc_bf16_bits(a) | ((uint32_t)fc_bf16_bits(b) << 16);
        }
        *(uint4 *)(out + row * d + 8 * c) = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

// ---------------------------------------------------------------------------------------------
// Linear layer, block = (4 rows, 64 output columns); each wave owns every 4th column of the block and
// runs the dot products with lanes along the hidden dimension.  MODE 0: out = aux + x w^T
// (aux = residual or nullptr); MODE 1: out = silu(x w^T) * (x aux^T) (aux = second weight matrix).
constexpr int LG_ROWS = 4;

template <typename T, int MODE>
__global__ __launch_bounds__(256) void k_linear_generic(const T *__restrict__ X, const T *__restrict__ W,
                                                        const T *aux, int M, int K, int N, T *out)
{
    const int m0 = blockIdx.x * LG_ROWS, n0 = blockIdx.y * 64;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int c = wave; c < 64; c += 4) {
        const int n = n0 + c;
        if (n >= N) break;
        const T *w = W + (size_t)n * K;
        const T *w2 = MODE == 1 ? aux + (size_t)n * K : nullptr;
        float acc[LG_ROWS], acc2[LG_ROWS];
#pragma unroll
        for (int r = 0; r < LG_ROWS; ++r) acc[r] = acc2[r] = 0.f;
        for (int k = lane; k < K; k += 64) {
            const float wv = fc_to_float(w[k]);
            const float wv2 = MODE == 1 ? fc_to_float(w2[k]) : 0.f;
#pragma unroll
            for (int r = 0; r < LG_ROWS; ++r)
                if (m0 + r < M) {
                    const float xv = fc_to_float(X[(size_t)(m0 + r) * K + k]);
                    acc[r] += wv * xv;
                    if (MODE == 1) acc2[r] += wv2 * xv;
                }
        }
#pragma unroll
        for (int r = 0; r < LG_ROWS; ++r) {
            const float a = wave_sum(acc[r]);
            const float b = MODE == 1 ? wave_sum(acc2[r]) : 0.f;
            if (lane == 0 && m0 + r < M) {
                const size_t o = (size_t)(m0 + r) * N + n;
                float y;
                if (MODE == 1)
                    y = a / (1.0f + expf(-a)) * b;
                else
                    y = aux ? a + fc_to_float(aux[o]) : a;
                out[o] = fc_from_float<T>(y);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// KV drift diagnostic: cosine similarity over the head dimension between rows of the cache and an
// earlier snapshot of the same rows in the plain [B][Hkv][rows][Dh] layout.  One wave per
// (sequence, kv head, row); lanes run along the head dimension.
template <typename T>
__global__ __launch_bounds__(64) void k_kv_similarity(FcGeom G, const T *__restrict__ kc, const T *__restrict__ vc,
                                                      const T *__restrict__ k_prev, const T *__restrict__ v_prev,
                                                      int start, int rows, float *sim_k, float *sim_v)
{
    const int r = blockIdx.x, j = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const size_t old = (((size_t)b * G.Hkv + j) * rows + r) * G.Dh;
    float dk = 0.f, nk = 0.f, pk = 0.f, dv = 0.f, nv = 0.f, pv = 0.f;
    for (int i = lane; i < G.Dh; i += 64) {
        const float xk = fc_to_float(kc[fc_k_index(G, b, j, start + r, i)]), yk = fc_to_float(k_prev[old + i]);
        const float xv = fc_to_float(vc[fc_v_index(G, b, j, start + r, i)]), yv = fc_to_float(v_prev[old + i]);
        dk += xk * yk;
        nk += xk * xk;
        pk += yk * yk;
        dv += xv * yv;
        nv += xv * xv;
        pv += yv * yv;
    }
    dk = wave_sum(dk);
    nk = wave_sum(nk);
    pk = wave_sum(pk);
    dv = wave_sum(dv);
    nv = wave_sum(nv);
    pv = wave_sum(pv);
    if (lane == 0) {
        const size_t o = ((size_t)b * G.Hkv + j) * rows + r;
        sim_k[o] = (nk > 0.f && pk > 0.f) ? dk / (sqrtf(nk) * sqrtf(pk)) : 0.f;
        sim_v[o] = (nv > 0.f && pv > 0.f) ? dv / (sqrtf(nv) * sqrtf(pv)) : 0.f;
    }
}

}  // namespace

hipError_t fc_launch_kv_similarity(const FcGeom &G, int dtype, const void *k_layer, const void *v_layer,
                                   const void *k_prev, const void *v_prev, int start, int rows, float *sim_k,
                                   float *sim_v, hipStream_t s)
{
    const dim3 grid((unsigned)rows, (unsigned)G.Hkv, (unsigned)G.B);
    if (dtype == FC_F32)
        k_kv_similarity<float><<<grid, dim3(64), 0, s>>>(G, (const float *)k_layer, (const float *)v_layer,
                                                         (const float *)k_prev, (const float *)v_prev, start, rows, sim_k,
                                                         sim_v);
    else
        k_kv_similarity<bf16_t><<<grid, dim3(64), 0, s>>>(G, (const bf16_t *)k_layer, (const bf16_t *)v_layer,
                                                          (const bf16_t *)k_prev, (const bf16_t *)v_prev, start, rows,
                                                          sim_k, sim_v);
    return hipGetLastError();
}

hipError_t fc_launch_copy_rows(const FcGeom &G, int dtype, void *k_layer, void *v_layer, void *k_rows,
                               void *v_rows, int start, int rows, bool to_cache, hipStream_t s)
{
    const size_t total = (size_t)G.B * G.Hkv * rows * G.Dh;
    size_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (blocks == 0) return hipSuccess;
    if (dtype == FC_F32)
        k_copy_rows<float><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(
            G, (float *)k_layer, (float *)v_layer, (float *)k_rows, (float *)v_rows, start, rows, to_cache);
    else
        k_copy_rows<bf16_t><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(
            G, (bf16_t *)k_layer, (bf16_t *)v_layer, (bf16_t *)k_rows, (bf16_t *)v_rows, start, rows,
            to_cache);
    return hipGetLastError();
}

hipError_t fc_launch_project_generic(const FcGeom &G, int dtype, const void *x, const void *w,
                                     const void *bias, const int32_t *pos, int win_start, int A,
                                     void *q_out, void *k_layer, void *v_layer, hipStream_t s)
{
    const int M = G.B * A;
    dim3 grid((M + PG_ROWS - 1) / PG_ROWS, G.Hq + 2 * G.Hkv);
    if (dtype == FC_F32)
        k_project_generic<float><<<grid, dim3(256), 0, s>>>(G, (const float *)x, (const float *)w,
                                                            (const float *)bias, pos, win_start, A,
                                                            (float *)q_out, (float *)k_layer,
                                                            (float *)v_layer);
    else
        k_project_generic<bf16_t><<<grid, dim3(256), 0, s>>>(G, (const bf16_t *)x, (const bf16_t *)w,
                                                             (const bf16_t *)bias, pos, win_start, A,
                                                             (bf16_t *)q_out, (bf16_t *)k_layer,
                                                             (bf16_t *)v_layer);
    return hipGetLastError();
}

hipError_t fc_launch_attention_generic(const FcGeom &G, int dtype, const void *q, const void *k_layer,
                                       const void *v_layer, const int32_t *pos, int A, int kv_len,
                                       void *out, hipStream_t s)
{
    dim3 grid(A, G.Hq, G.B);
    if (dtype == FC_F32)
        k_attention_generic<float><<<grid, dim3(256), 0, s>>>(G, (const float *)q, (const float *)k_layer,
                                                              (const float *)v_layer, pos, A, kv_len,
                                                              (float *)out);
    else
        k_attention_generic<bf16_t><<<grid, dim3(256), 0, s>>>(G, (const bf16_t *)q,
                                                               (const bf16_t *)k_layer,
                                                               (const bf16_t *)v_layer, pos, A, kv_len,
                                                               (bf16_t *)out);
    return hipGetLastError();
}

hipError_t fc_launch_rmsnorm(int dtype, const void *x, const void *weight, float eps, int rows, int d,
                             void *out, hipStream_t s)
{
    if (dtype == FC_F32)
        k_rmsnorm<float><<<dim3((unsigned)rows), dim3(256), 0, s>>>((const float *)x, (const float *)weight, eps,
                                                                    d, (float *)out);
    else if (d % 8 == 0 && d <= 8192 && (((uintptr_t)x | (uintptr_t)weight | (uintptr_t)out) & 15) == 0) {
        const uint16_t *xb = (const uint16_t *)x, *wb = (const uint16_t *)weight;
        if (d <= 2048)
            k_rmsnorm_bf16_row<1><<<dim3((unsigned)rows), dim3(256), 0, s>>>(xb, wb, eps, d, (uint16_t *)out);
        else if (d <= 4096)
            k_rmsnorm_bf16_row<2><<<dim3((unsigned)rows), dim3(256), 0, s>>>(xb, wb, eps, d, (uint16_t *)out);
        else
            k_rmsnorm_bf16_row<4><<<dim3((unsigned)rows), dim3(256), 0, s>>>(xb, wb, eps, d, (uint16_t *)out);
    } else
        k_rmsnorm<bf16_t><<<dim3((unsigned)rows), dim3(256), 0, s>>>((const bf16_t *)x, (const bf16_t *)weight,
                                                                     eps, d, (bf16_t *)out);
    return hipGetLastError();
}

template <typename T>
static void launch_linear_t(int mode, const void *x, const void *w, const void *aux, int M, int K, int N,
                            void *out, hipStream_t s)
{
    const dim3 grid((unsigned)((M + LG_ROWS - 1) / LG_ROWS), (unsigned)((N + 63) / 64));
    if (mode == FC_LIN_GATE_UP)
        k_linear_generic<T, 1><<<grid, dim3(256), 0, s>>>((const T *)x, (const T *)w, (const T *)aux, M, K, N, (T *)out);
    else
        k_linear_generic<T, 0><<<grid, dim3(256), 0, s>>>((const T *)x, (const T *)w, (const T *)aux, M, K, N, (T *)out);
}

hipError_t fc_launch_linear_generic(int dtype, int mode, const void *x, const void *w, const void *aux,
                                    int M, int K, int N, void *out, hipStream_t s)
{
    if (dtype == FC_F32)
        launch_linear_t<float>(mode, x, w, aux, M, K, N, out, s);
    else
        launch_linear_t<bf16_t>(mode, x, w, aux, M, K, N, out, s);
    return hipGetLastError();
}
