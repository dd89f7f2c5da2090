// Row-wise pieces of the decoder forward pass on gfx950: embedding gather, RMSNorm, rotary
// embedding + KV append, SwiGLU, and the KV-length bookkeeping (the rollback of Sec. 3.3).
// All are bandwidth-trivial next to the weight streaming of the GEMMs; they exist so that no
// step of the forward pass leaves the GPU.
#include "common.h"
#include "kernels.h"
#include "prof.h"
#include "../../include/psd.h"

namespace psd {
namespace {

constexpr int kRowThreads = 256;
constexpr int kMaxV4 = 8;              // float4 per thread kept in registers: rows up to 8192 wide

// fixed-order block sum: butterfly inside each wavefront, then the four totals left to right
__device__ __forceinline__ float block_sum4(float v, float *red) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return ((red[0] + red[1]) + red[2]) + red[3];
}

__device__ __forceinline__ f32x4 load_gain4(const float *g, int i4) { return reinterpret_cast<const f32x4 *>(g)[i4]; }
__device__ __forceinline__ f32x4 load_gain4(const uint16_t *g, int i4) {
    const uint2 raw = reinterpret_cast<const uint2 *>(g)[i4];
    return f32x4{bf16_bits_to_f32(raw.x & 0xffffu), __uint_as_float(raw.x & 0xffff0000u),
                 bf16_bits_to_f32(raw.y & 0xffffu), __uint_as_float(raw.y & 0xffff0000u)};
}
__device__ __forceinline__ f32x4 load_row4(const float *row, int i4) { return reinterpret_cast<const f32x4 *>(row)[i4]; }
__device__ __forceinline__ f32x4 load_row4(const uint16_t *row, int i4) { return load_gain4(row, i4); }

// One block per row: x (+)= source, then xn = x * rsqrt(mean(x^2) + eps) * gain.  The source is either
// an embedding row (EMBED) or the split-K partial sums of the projection that feeds the residual
// stream, added in split order.  All loads of a row are issued before the first use.
template <typename TW, bool EMBED>
__global__ __launch_bounds__(kRowThreads) void residual_norm_kernel(const TW *embed, const int32_t *tokens, int vocab,
                                                                    const float *partial, int S, size_t split_stride,
                                                                    float *x, const TW *gain, float *xn, float *sumsq_out,
                                                                    int d, float eps, RopeTable rt, uint16_t *xn16,
                                                                    ZeroFill zf) {
    __shared__ float red[4];
    const int m = blockIdx.x, tid = threadIdx.x, n4 = d >> 2;
    if constexpr (EMBED) {
        // counters that later kernels of this forward pass expect at zero
        if (m == 0)
            for (int j = tid; j < zf.n; j += kRowThreads) zf.words[j] = 0u;
        // (cos, sin) of this row's position at every rotation frequency, once per forward pass for all layers;
        // the angle position * theta^(-2i/d_h) is evaluated in fp64
        if (rt.cs && tid < rt.d_h / 2) {
            const int pos = rt.lens[m / rt.R] + (rt.depth ? rt.depth[m % rt.R] : m % rt.R);
            const double inv_freq = exp2(-2.0 * (double)tid / (double)rt.d_h * log2((double)rt.theta));
            double sn, cs;
            sincos((double)pos * inv_freq, &sn, &cs);
            rt.cs[(size_t)m * (rt.d_h / 2) + tid] = make_float2((float)cs, (float)sn);
        }
    }
    f32x4 v[kMaxV4];
    float ss = 0.f;
    f32x4 *__restrict__ xrow = reinterpret_cast<f32x4 *>(x + (size_t)m * d);
    const TW *erow = nullptr;
    if constexpr (EMBED) {
        int tok = tokens[m];
        tok = min(max(tok, 0), vocab - 1);
        erow = embed + (size_t)tok * d;
    }
    // issue every load of the row first (x or the embedding row, then the partials four splits at a
    // time), add in split order, store afterwards
    const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < kMaxV4; ++j) {
        const int i4 = tid + j * kRowThreads;
        v[j] = zero;
        if (i4 < n4) {
            if constexpr (EMBED) v[j] = load_row4(erow, i4);
            else v[j] = xrow[i4];
        }
    }
    if constexpr (!EMBED) {
        const f32x4 *prow = reinterpret_cast<const f32x4 *>(partial + (size_t)m * d);
        const size_t stride4 = split_stride >> 2;
        int sp = 0;
        for (; sp + 4 <= S; sp += 4) {
            f32x4 t[4][kMaxV4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int j = 0; j < kMaxV4; ++j) {
                    const int i4 = tid + j * kRowThreads;
                    t[u][j] = i4 < n4 ? prow[(sp + u) * stride4 + i4] : zero;
                }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int j = 0; j < kMaxV4; ++j) v[j] += t[u][j];
        }
        for (; sp < S; ++sp) {
#pragma unroll
            for (int j = 0; j < kMaxV4; ++j) {
                const int i4 = tid + j * kRowThreads;
                if (i4 < n4) v[j] += prow[sp * stride4 + i4];
            }
        }
    }
#pragma unroll
    for (int j = 0; j < kMaxV4; ++j) {
        const int i4 = tid + j * kRowThreads;
        if (i4 < n4) {
            const f32x4 a = v[j];
            xrow[i4] = a;
            ss += a[0] * a[0] + a[1] * a[1] + a[2] * a[2] + a[3] * a[3];
        }
    }
    const float tot = block_sum4(ss, red);
    float scale = 1.0f / sqrtf(tot / (float)d + eps);
    if (sumsq_out) {                       // the norm scale is applied by the consumer of the next projection
        if (tid == 0) sumsq_out[m] = tot;
        scale = 1.0f;
    }
    f32x4 *orow = reinterpret_cast<f32x4 *>(xn + (size_t)m * d);
#pragma unroll
    for (int j = 0; j < kMaxV4; ++j) {
        const int i4 = tid + j * kRowThreads;
        if (i4 < n4) {
            const f32x4 r = v[j] * scale * load_gain4(gain, i4);
            orow[i4] = r;
            if (xn16)              // the same row rounded to fp16: the operand of the tiled projections
                reinterpret_cast<uint2 *>(xn16 + (size_t)m * d)[i4] =
                    make_uint2(f32_to_f16_bits(r[0]) | ((uint32_t)f32_to_f16_bits(r[1]) << 16),
                               f32_to_f16_bits(r[2]) | ((uint32_t)f32_to_f16_bits(r[3]) << 16));
        }
    }
}

// One block per (new row, head slot): slots 0..h_q-1 rotate a query head, the next h_kv rotate a
// key head into the cache, the last h_kv copy a value head into the transposed V cache.  The
// projection arrives as split-K partials and is summed here, in split order.  Thread i < d_h/2
// owns the rotation pair (i, i + d_h/2); the angle position * theta^(-2i/d_h) is evaluated in fp64.
template <typename TC>
__global__ __launch_bounds__(64) void reduce_rope_append_kernel(const float *partial, int S, size_t split_stride,
                                                                RowScale rs, float *q_out, TC *k_cache, TC *v_cache,
                                                                const int32_t *lens, int R, int h_q, int h_kv, int d_h,
                                                                int max_len, float theta) {
    const int m = blockIdx.x, slot = blockIdx.y, b = m / R, r = m % R;
    const int pos = lens[b] + r;
    if (pos >= max_len) return;            // capacity was checked on the host; never write outside
    // the sums of squares first, the projection's partials next, the reduction after both are in flight
    float ssq = 0.f;
    if (rs.sumsq)
        for (int t = threadIdx.x; t < rs.tiles; t += 64) ssq += rs.sumsq[(size_t)t * gridDim.x + m];
    const int half = d_h / 2;
    const int width = (h_q + 2 * h_kv) * d_h;
    const float *src = partial + (size_t)m * width + (size_t)slot * d_h;
    const int i = threadIdx.x;
    auto value = [&](int e) {                  // loads four splits at a time, adds in split order
        float a = 0.f;
        int sp = 0;
        for (; sp + 4 <= S; sp += 4) {
            const float t0 = src[sp * split_stride + e], t1 = src[(sp + 1) * split_stride + e];
            const float t2 = src[(sp + 2) * split_stride + e], t3 = src[(sp + 3) * split_stride + e];
            a += t0; a += t1; a += t2; a += t3;
        }
        for (; sp < S; ++sp) a += src[sp * split_stride + e];
        return a;
    };
    auto scale_of = [&]() { return rs.sumsq ? 1.0f / sqrtf(wave_sum(ssq) * rs.inv_d + rs.eps) : 1.0f; };
    if (slot < h_q + h_kv) {
        const float r1 = i < half ? value(i) : 0.f, r2 = i < half ? value(half + i) : 0.f;
        const float sc = scale_of();
        if (i >= half) return;
        const double inv_freq = exp2(-2.0 * (double)i / (double)d_h * log2((double)theta));
        double sn, cs;
        sincos((double)pos * inv_freq, &sn, &cs);
        const float c = (float)cs, s = (float)sn;
        const float x1 = r1 * sc, x2 = r2 * sc;
        const float y1 = x1 * c - x2 * s, y2 = x2 * c + x1 * s;
        if (slot < h_q) {
            float *dst = q_out + ((size_t)m * h_q + slot) * d_h;
            dst[i] = y1;
            dst[half + i] = y2;
        } else {
            TC *dst = k_cache + (((size_t)b * h_kv + (slot - h_q)) * max_len + pos) * d_h;
            store_elem(dst, i, y1);
            store_elem(dst, half + i, y2);
        }
    } else {
        // V is stored transposed: v_cache[b][h][d][pos]
        const int h = slot - h_q - h_kv;
        const float v0 = i < d_h ? value(i) : 0.f, v1 = i + 64 < d_h ? value(i + 64) : 0.f;     // d_h <= 128
        const float sc = scale_of();
        if (i < d_h) store_elem(v_cache, (((size_t)b * h_kv + h) * d_h + i) * max_len + pos, v0 * sc);
        if (i + 64 < d_h) store_elem(v_cache, (((size_t)b * h_kv + h) * d_h + i + 64) * max_len + pos, v1 * sc);
    }
}

// h = silu(g) * u, four columns per thread, one row per blockIdx.y; [g | u] arrive as split-K partials of
// the gate|up projection
__global__ __launch_bounds__(256) void reduce_swiglu_kernel(const float *partial, int S, size_t split_stride, RowScale rs,
                                                            float *h, int M, int f, uint16_t *h16) {
    __shared__ float red[4];
    const int m = blockIdx.y, f4 = f >> 2;
    float ssq = 0.f;
    if (rs.sumsq)
        for (int t = threadIdx.x; t < rs.tiles; t += 256) ssq += rs.sumsq[(size_t)t * M + m];
    const int j4 = blockIdx.x * 256 + threadIdx.x;
    f32x4 g = f32x4{0.f, 0.f, 0.f, 0.f}, u = g;
    if (j4 < f4)
        for (int sp = 0; sp < S; ++sp) {
            const f32x4 *row = reinterpret_cast<const f32x4 *>(partial + sp * split_stride + (size_t)m * 2 * f);
            g += row[j4];
            u += row[f4 + j4];
        }
    const float sc = rs.sumsq ? 1.0f / sqrtf(block_sum4(ssq, red) * rs.inv_d + rs.eps) : 1.0f;
    if (j4 >= f4) return;
    g *= sc;
    u *= sc;
    f32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = g[e] / (1.0f + expf(-g[e])) * u[e];
    reinterpret_cast<f32x4 *>(h + (size_t)m * f)[j4] = o;
    if (h16)
        reinterpret_cast<uint2 *>(h16 + (size_t)m * f)[j4] =
            make_uint2(f32_to_f16_bits(o[0]) | ((uint32_t)f32_to_f16_bits(o[1]) << 16),
                       f32_to_f16_bits(o[2]) | ((uint32_t)f32_to_f16_bits(o[3]) << 16));
}

__global__ void advance_lens_kernel(int32_t *lens, int B, int delta, int max_len) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) lens[b] = min(lens[b] + delta, max_len);
}

__global__ void truncate_kernel(int32_t *lens, const int32_t *base, const int32_t *keep, int offset, int cap, int B) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) lens[b] = max(0, min(min(lens[b], cap), base[b] + keep[b] + offset));
}

__global__ void truncate_to_kernel(int32_t *lens, int new_len, int B) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) lens[b] = max(0, min(lens[b], new_len));
}

}  // namespace

void launch_embed_norm(int dtype, const void *embed, const int32_t *tokens, float *x, const void *gain, float *xn,
                       float *sumsq_out, int M, int d, int vocab, float eps, RopeTable rt, uint16_t *xn16, ZeroFill zf,
                       hipStream_t stream) {
    ScopedProf sp(PSD_KIND_EMBED, stream);
    if (dtype == PSD_BF16)
        launch_kernel(residual_norm_kernel<uint16_t, true>, M, kRowThreads, 0, stream, (const uint16_t *)embed, tokens, vocab, nullptr, 0, 0,
                                                                           x, (const uint16_t *)gain, xn, sumsq_out, d, eps, rt, xn16, zf);
    else
        launch_kernel(residual_norm_kernel<float, true>, M, kRowThreads, 0, stream, (const float *)embed, tokens, vocab, nullptr, 0, 0, x,
                                                                        (const float *)gain, xn, sumsq_out, d, eps, rt, xn16, zf);
}

void launch_reduce_residual_norm(int dtype, const float *partial, int S, float *x, const void *gain, float *xn,
                                 int M, int d, float eps, uint16_t *xn16, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_RMSNORM, stream);
    const size_t stride = (size_t)M * d;
    if (dtype == PSD_BF16)
        launch_kernel(residual_norm_kernel<uint16_t, false>, M, kRowThreads, 0, stream, nullptr, nullptr, 0, partial, S, stride, x,
                                                                            (const uint16_t *)gain, xn, nullptr, d, eps, RopeTable{}, xn16, ZeroFill{});
    else
        launch_kernel(residual_norm_kernel<float, false>, M, kRowThreads, 0, stream, nullptr, nullptr, 0, partial, S, stride, x,
                                                                         (const float *)gain, xn, nullptr, d, eps, RopeTable{}, xn16, ZeroFill{});
}

void launch_reduce_rope_append(int dtype, const float *partial, int S, RowScale rs, float *q_out, void *k_cache,
                               void *v_cache, const int32_t *lens, int B, int R, int h_q, int h_kv, int d_h,
                               int max_len, float theta, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_ROPE_APPEND, stream);
    const size_t stride = (size_t)B * R * (h_q + 2 * h_kv) * d_h;
    const dim3 grid(B * R, h_q + 2 * h_kv);
    if (dtype == PSD_BF16)
        launch_kernel(reduce_rope_append_kernel<uint16_t>, grid, 64, 0, stream, partial, S, stride, rs, q_out, (uint16_t *)k_cache,
                                                                     (uint16_t *)v_cache, lens, R, h_q, h_kv, d_h, max_len, theta);
    else
        launch_kernel(reduce_rope_append_kernel<float>, grid, 64, 0, stream, partial, S, stride, rs, q_out, (float *)k_cache, (float *)v_cache,
                                                                  lens, R, h_q, h_kv, d_h, max_len, theta);
}

void launch_reduce_swiglu(const float *partial, int S, RowScale rs, float *h, int M, int f, uint16_t *h16, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_SWIGLU, stream);
    const dim3 grid((unsigned)((f / 4 + 255) / 256), (unsigned)M);
    launch_kernel(reduce_swiglu_kernel, grid, 256, 0, stream, partial, S, (size_t)M * 2 * f, rs, h, M, f, h16);
}

void launch_advance_lens(int32_t *lens, int B, int delta, int max_len, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_LENS, stream);
    launch_kernel(advance_lens_kernel, (B + 63) / 64, 64, 0, stream, lens, B, delta, max_len);
}
void launch_truncate(int32_t *lens, const int32_t *base, const int32_t *keep, int offset, int cap, int B,
                     hipStream_t stream) {
    ScopedProf sp(PSD_KIND_LENS, stream);
    launch_kernel(truncate_kernel, (B + 63) / 64, 64, 0, stream, lens, base, keep, offset, cap, B);
}
void launch_truncate_to(int32_t *lens, int new_len, int B, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_LENS, stream);
    launch_kernel(truncate_to_kernel, (B + 63) / 64, 64, 0, stream, lens, new_len, B);
}

}  // namespace psd
