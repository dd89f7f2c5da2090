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

template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T *embed, const int32_t *tokens, float *x,
                                                    int d, int vocab) {
    const int m = blockIdx.x;
    int tok = tokens[m];
    tok = min(max(tok, 0), vocab - 1);
    const T *row = embed + (size_t)tok * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)m * d + i] = load_elem(row, i);
}

// One block per row.  The sum of squares is taken in fp32 in a fixed order: per-thread strided
// partial, butterfly inside the wavefront, then the four wavefront totals left to right.
template <typename TW, typename TA>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float *x, const TW *gain, TA *out, int d,
                                                      float eps, int row_stride_x) {
    const int m = blockIdx.x, tid = threadIdx.x;
    const float *row = x + (size_t)m * row_stride_x;
    float ss = 0.f;
    for (int i = tid; i < d; i += 256) { const float v = row[i]; ss += v * v; }
    __shared__ float red[4];
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float tot = ((red[0] + red[1]) + red[2]) + red[3];
    const float scale = 1.0f / sqrtf(tot / (float)d + eps);
    for (int i = tid; i < d; i += 256) store_elem(out, (size_t)m * d + i, row[i] * scale * load_elem(gain, i));
}

// One block per (new row, head slot): slots 0..h_q-1 rotate a query head, the next h_kv rotate a
// key head into the cache, the last h_kv copy a value head into the transposed V cache.  Thread
// i < d_h/2 owns the rotation pair (i, i + d_h/2); the angle position * theta^(-2i/d_h) is
// evaluated in fp64.
template <typename TA, typename TC>
__global__ __launch_bounds__(64) void rope_append_kernel(const float *qkv, TA *q_out, TC *k_cache, TC *v_cache,
                                                         const int32_t *lens, int R, int h_q, int h_kv, int d_h,
                                                         int max_len, float theta) {
    const int m = blockIdx.x, slot = blockIdx.y, b = m / R, r = m % R;
    const int pos = lens[b] + r;
    if (pos >= max_len) return;            // capacity was checked on the host; never write outside
    const int half = d_h / 2;
    const int width = (h_q + 2 * h_kv) * d_h;
    const float *src = qkv + (size_t)m * width + (size_t)slot * d_h;
    const int i = threadIdx.x;
    if (slot < h_q + h_kv) {
        if (i >= half) return;
        const double inv_freq = exp2(-2.0 * (double)i / (double)d_h * log2((double)theta));
        double sn, cs;
        sincos((double)pos * inv_freq, &sn, &cs);
        const float c = (float)cs, s = (float)sn;
        const float x1 = src[i], x2 = src[half + i];
        const float y1 = x1 * c - x2 * s, y2 = x2 * c + x1 * s;
        if (slot < h_q) {
            TA *dst = q_out + ((size_t)m * h_q + slot) * d_h;
            store_elem(dst, i, y1);
            store_elem(dst, half + i, y2);
        } else {
            TC *dst = k_cache + (((size_t)b * h_kv + (slot - h_q)) * max_len + pos) * d_h;
            store_elem(dst, i, y1);
            store_elem(dst, half + i, y2);
        }
    } else {
        // V is stored transposed: v_cache[b][h][d][pos]
        const int h = slot - h_q - h_kv;
        for (int dd = i; dd < d_h; dd += 64)
            store_elem(v_cache, (((size_t)b * h_kv + h) * d_h + dd) * max_len + pos, src[dd]);
    }
}

template <typename TA>
__global__ __launch_bounds__(256) void swiglu_kernel(const float *gu, TA *h, int M, int f) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)M * f) return;
    const size_t m = idx / f, j = idx % f;
    const float g = gu[m * 2 * f + j], u = gu[m * 2 * f + f + j];
    store_elem(h, idx, g / (1.0f + expf(-g)) * u);
}

__global__ void advance_lens_kernel(int32_t *lens, int B, int delta, int max_len) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) lens[b] = min(lens[b] + delta, max_len);
}

__global__ void truncate_kernel(int32_t *lens, const int32_t *base, const int32_t *keep, int offset, int B) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) lens[b] = max(0, min(lens[b], base[b] + keep[b] + offset));
}

__global__ void truncate_to_kernel(int32_t *lens, int new_len, int B) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) lens[b] = max(0, min(lens[b], new_len));
}

}  // namespace

void launch_embed(int dtype, const void *embed, const int32_t *tokens, float *x, int M, int d, int vocab,
                  hipStream_t stream) {
    ScopedProf sp(PSD_KIND_EMBED, stream);
    if (dtype == PSD_BF16) embed_kernel<uint16_t><<<M, 256, 0, stream>>>((const uint16_t *)embed, tokens, x, d, vocab);
    else embed_kernel<float><<<M, 256, 0, stream>>>((const float *)embed, tokens, x, d, vocab);
}

void launch_rmsnorm(int dtype, const float *x, const void *gain, void *out, int M, int d, float eps,
                    int row_stride_x, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_RMSNORM, stream);
    if (dtype == PSD_BF16)
        rmsnorm_kernel<uint16_t, float><<<M, 256, 0, stream>>>(x, (const uint16_t *)gain, (float *)out, d, eps, row_stride_x);
    else
        rmsnorm_kernel<float, float><<<M, 256, 0, stream>>>(x, (const float *)gain, (float *)out, d, eps, row_stride_x);
}

void launch_rope_append(int dtype, const float *qkv, void *q_out, void *k_cache, void *v_cache,
                        const int32_t *lens, int B, int R, int h_q, int h_kv, int d_h, int max_len,
                        float theta, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_ROPE_APPEND, stream);
    if (dtype == PSD_BF16)
        rope_append_kernel<float, uint16_t><<<dim3(B * R, h_q + 2 * h_kv), 64, 0, stream>>>(qkv, (float *)q_out, (uint16_t *)k_cache,
                                                                      (uint16_t *)v_cache, lens, R, h_q, h_kv, d_h, max_len, theta);
    else
        rope_append_kernel<float, float><<<dim3(B * R, h_q + 2 * h_kv), 64, 0, stream>>>(qkv, (float *)q_out, (float *)k_cache, (float *)v_cache,
                                                                   lens, R, h_q, h_kv, d_h, max_len, theta);
}

void launch_swiglu(int dtype, const float *gu, void *h, int M, int f, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_SWIGLU, stream);
    const unsigned blocks = (unsigned)(((size_t)M * f + 255) / 256);
    (void)dtype;
    swiglu_kernel<float><<<blocks, 256, 0, stream>>>(gu, (float *)h, M, f);
}

void launch_advance_lens(int32_t *lens, int B, int delta, int max_len, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_LENS, stream);
    advance_lens_kernel<<<(B + 63) / 64, 64, 0, stream>>>(lens, B, delta, max_len);
}
void launch_truncate(int32_t *lens, const int32_t *base, const int32_t *keep, int offset, int B, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_LENS, stream);
    truncate_kernel<<<(B + 63) / 64, 64, 0, stream>>>(lens, base, keep, offset, B);
}
void launch_truncate_to(int32_t *lens, int new_len, int B, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_LENS, stream);
    truncate_to_kernel<<<(B + 63) / 64, 64, 0, stream>>>(lens, new_len, B);
}

}  // namespace psd
