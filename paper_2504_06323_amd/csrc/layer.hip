// The attention half of a LLaMA-style layer (the models of Table 2, Section 4.1.1), so that the inputs of the
// q / k / v, o and gate / up projections -- the activations the weight metric (Eq. 5) and the Hessian are taken
// from -- can come from a forward pass instead of being injected:
//   a = rmsnorm(x) * w;   q, k <- rotary embedding by position;   o_in = causal softmax(q k^T / sqrt(d)) v.
// rmsnorm and the rotary embedding are plain bandwidth-bound kernels; the attention here is the any-shape
// version (one wave per query), the matrix-core version for 128-wide bf16 heads lives in attention.hip.
#include "mfma_bf16.hpp"

namespace mp {

namespace {

template <typename T>
__device__ __forceinline__ T narrow_as(float f);
template <>
__device__ __forceinline__ float narrow_as<float>(float f) { return f; }
template <>
__device__ __forceinline__ bf16_t narrow_as<bf16_t>(float f) { return narrow_to_bf16(f); }

// y[t, :] = x[t, :] / sqrt(mean(x[t, :]^2) + eps) * weight ; one wave per token row
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_rows(const T *__restrict__ x, const T *__restrict__ weight,
                                                    T *__restrict__ y, int64_t tokens, int64_t channels, int64_t ld_x,
                                                    int64_t ld_y, float eps) {
    const int lane = threadIdx.x & 63;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6); t < tokens;
         t += static_cast<int64_t>(gridDim.x) * 4) {
        const T *row = x + t * ld_x;
        float s = 0.f;
        for (int64_t j = lane; j < channels; j += 64) {
            const float v = widen(row[j]);
            s = fmaf(v, v, s);
        }
        s = wave_sum(s);
        s = __shfl(s, 0);
        const float scale = 1.f / sqrtf(s / static_cast<float>(channels) + eps);
        for (int64_t j = lane; j < channels; j += 64)
            y[t * ld_y + j] = narrow_as<T>(widen(row[j]) * scale * widen(weight[j]));
    }
}

// the same with 16-byte accesses (8-element packets; channels and pitches multiples of 8, 16-byte aligned bases);
// the row is read twice, the second time from cache
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_rows_vec(const T *__restrict__ x, const T *__restrict__ weight,
                                                        T *__restrict__ y, int64_t tokens, int64_t channels,
                                                        int64_t ld_x, int64_t ld_y, float eps) {
    const int lane = threadIdx.x & 63;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6); t < tokens;
         t += static_cast<int64_t>(gridDim.x) * 4) {
        const T *row = x + t * ld_x;
        float s = 0.f;
        for (int64_t j = lane * 8; j < channels; j += 512) {
            Packet<T, 8> pk;
            pk.load(row + j);
            float v[8];
            pk.to_float(v);
#pragma unroll
            for (int e = 0; e < 8; ++e) s = fmaf(v[e], v[e], s);
        }
        s = wave_sum(s);
        s = __shfl(s, 0);
        const float scale = 1.f / sqrtf(s / static_cast<float>(channels) + eps);
        for (int64_t j = lane * 8; j < channels; j += 512) {
            Packet<T, 8> pk, pw;
            pk.load(row + j);
            pw.load(weight + j);
            float v[8], wv[8];
            pk.to_float(v);
            pw.to_float(wv);
            T out[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) out[e] = narrow_as<T>(v[e] * scale * wv[e]);
            *reinterpret_cast<Packet<T, 8> *>(y + t * ld_y + j) = *reinterpret_cast<const Packet<T, 8> *>(out);
        }
    }
}

// out[t, :] = a[t, :] + b[t, :] (the residual connections of the layer), fp32 sum rounded once
template <typename T>
__global__ __launch_bounds__(256) void add_rows(const T *__restrict__ a, const T *__restrict__ b, T *__restrict__ out,
                                                int64_t rows, int64_t cols, int64_t ld_a, int64_t ld_b, int64_t ld_out) {
    const int64_t n = rows * cols;
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; e < n;
         e += static_cast<int64_t>(gridDim.x) * 256) {
        const int64_t r = e / cols, c = e - r * cols;
        out[r * ld_out + c] = narrow_as<T>(widen(a[r * ld_a + c]) + widen(b[r * ld_b + c]));
    }
}

template <typename T>
__global__ __launch_bounds__(256) void add_rows_vec(const T *__restrict__ a, const T *__restrict__ b, T *__restrict__ out,
                                                    int64_t rows, int64_t cols, int64_t ld_a, int64_t ld_b,
                                                    int64_t ld_out) {
    const int64_t per_row = cols / 8, n = rows * per_row;
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; e < n;
         e += static_cast<int64_t>(gridDim.x) * 256) {
        const int64_t r = e / per_row, c = (e - r * per_row) * 8;
        Packet<T, 8> pa, pb;
        pa.load(a + r * ld_a + c);
        pb.load(b + r * ld_b + c);
        float va[8], vb[8];
        pa.to_float(va);
        pb.to_float(vb);
        T o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = narrow_as<T>(va[i] + vb[i]);
        *reinterpret_cast<Packet<T, 8> *>(out + r * ld_out + c) = *reinterpret_cast<const Packet<T, 8> *>(o);
    }
}

// Rotary embedding with 16-byte accesses: a thread takes 8 consecutive dimensions i of one token, computes their
// angles once and turns those dimensions (and their partners i + d/2) in every head of the token.
template <typename T>
__global__ __launch_bounds__(256) void rotary_rows_vec(T *__restrict__ x, int64_t tokens, int64_t heads, int64_t head_dim,
                                                       int64_t ld, int64_t seq_len, float log2_base) {
    const int64_t half = head_dim / 2, per_token = half / 8, n = tokens * per_token;
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; e < n;
         e += static_cast<int64_t>(gridDim.x) * 256) {
        const int64_t t = e / per_token, i0 = (e - t * per_token) * 8;
        const float pos = static_cast<float>(t % seq_len);
        float sn[8], cs[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float inv = exp2f(-2.f * static_cast<float>(i0 + i) / static_cast<float>(head_dim) * log2_base);
            sincosf(pos * inv, &sn[i], &cs[i]);
        }
        for (int64_t h = 0; h < heads; ++h) {
            T *p = x + t * ld + h * head_dim + i0;
            Packet<T, 8> pa, pb;
            pa.load(p);
            pb.load(p + half);
            float a[8], b[8];
            pa.to_float(a);
            pb.to_float(b);
            T oa[8], ob[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                oa[i] = narrow_as<T>(a[i] * cs[i] - b[i] * sn[i]);
                ob[i] = narrow_as<T>(b[i] * cs[i] + a[i] * sn[i]);
            }
            *reinterpret_cast<Packet<T, 8> *>(p) = *reinterpret_cast<const Packet<T, 8> *>(oa);
            *reinterpret_cast<Packet<T, 8> *>(p + half) = *reinterpret_cast<const Packet<T, 8> *>(ob);
        }
    }
}

// in place: dimension i < d/2 of every head is paired with i + d/2; the pair turns by position * base^(-2i/d)
template <typename T>
__global__ __launch_bounds__(256) void rotary_rows(T *__restrict__ x, int64_t tokens, int64_t heads, int64_t head_dim,
                                                   int64_t ld, int64_t seq_len, float log2_base) {
    const int64_t half = head_dim / 2, per_token = heads * half, n = tokens * per_token;
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; e < n;
         e += static_cast<int64_t>(gridDim.x) * 256) {
        const int64_t t = e / per_token, rem = e - t * per_token, h = rem / half, i = rem - h * half;
        const float pos = static_cast<float>(t % seq_len);
        const float inv = exp2f(-2.f * static_cast<float>(i) / static_cast<float>(head_dim) * log2_base);
        float sn, cs;
        sincosf(pos * inv, &sn, &cs);
        T *p = x + t * ld + h * head_dim + i;
        const float a = widen(p[0]), b = widen(p[half]);
        p[0] = narrow_as<T>(a * cs - b * sn);
        p[half] = narrow_as<T>(b * cs + a * sn);
    }
}

// One wave per (sequence, head, query): lanes share the head dimension, keys are walked in order with a running
// maximum (the usual streaming form of the softmax).  Any head width up to 256.
template <typename T>
__global__ __launch_bounds__(256) void attention_generic(const T *__restrict__ q, const T *__restrict__ k,
                                                         const T *__restrict__ v, T *__restrict__ o, int64_t n_seqs,
                                                         int64_t seq_len, int64_t heads, int64_t kv_heads,
                                                         int64_t head_dim, int64_t ld_q, int64_t ld_k, int64_t ld_v,
                                                         int64_t ld_o) {
    const int lane = threadIdx.x & 63;
    const int64_t n_items = n_seqs * heads * seq_len;
    const float scale = 1.f / sqrtf(static_cast<float>(head_dim));
    const int64_t group = heads / kv_heads;
    for (int64_t item = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6); item < n_items;
         item += static_cast<int64_t>(gridDim.x) * 4) {
        const int64_t s = item % seq_len, h = (item / seq_len) % heads, b = item / (seq_len * heads);
        const int64_t g = h / group, t0 = b * seq_len;
        float qv[4], acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int64_t d = lane + 64 * c;
            qv[c] = d < head_dim ? widen(q[(t0 + s) * ld_q + h * head_dim + d]) : 0.f;
        }
        float m = -INFINITY, l = 0.f;
        for (int64_t t = 0; t <= s; ++t) {
            float dot = 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int64_t d = lane + 64 * c;
                if (d < head_dim) dot = fmaf(qv[c], widen(k[(t0 + t) * ld_k + g * head_dim + d]), dot);
            }
            dot = wave_sum(dot);
            dot = __shfl(dot, 0) * scale;
            const float m_new = fmaxf(m, dot);
            const float fix = __expf(m - m_new), p = __expf(dot - m_new);
            l = l * fix + p;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int64_t d = lane + 64 * c;
                if (d < head_dim) acc[c] = fmaf(p, widen(v[(t0 + t) * ld_v + g * head_dim + d]), acc[c] * fix);
            }
            m = m_new;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int64_t d = lane + 64 * c;
            if (d < head_dim) o[(t0 + s) * ld_o + h * head_dim + d] = narrow_as<T>(acc[c] / l);
        }
    }
}

}  // namespace

// defined in attention.hip: the matrix-core version, for bf16 heads of width 128; returns false if the shapes do
// not fit (nothing launched)
bool launch_attention_tiles(const void *q, const void *k, const void *v, void *o, int dtype, int64_t n_seqs,
                            int64_t seq_len, int64_t heads, int64_t kv_heads, int64_t head_dim, int64_t ld_q,
                            int64_t ld_k, int64_t ld_v, int64_t ld_o, hipStream_t stream);

}  // namespace mp

extern "C" int prune_rmsnorm(const void *x, const void *weight, void *y, int dtype, int64_t tokens, int64_t channels,
                             int64_t ld_x, int64_t ld_y, float eps, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (tokens <= 0 || channels <= 0 || ld_x < channels || ld_y < channels) return PRUNE_ERR_SHAPE;
    if (!x || !weight || !y) return PRUNE_ERR_NULL;
    if (!(eps >= 0.f)) return PRUNE_ERR_RANGE;
    const size_t es = elem_size(dtype);
    if (!aligned_to(x, es) || !aligned_to(weight, es) || !aligned_to(y, es)) return PRUNE_ERR_ALIGNMENT;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const unsigned blocks = static_cast<unsigned>(ceil_div(tokens, 4) < 16384 ? ceil_div(tokens, 4) : 16384);
    if (packet_ok(x, channels, ld_x) && packet_ok(y, channels, ld_y) && aligned_to(weight, 16)) {
        if (dtype == PRUNE_BF16)
            hipLaunchKernelGGL(rmsnorm_rows_vec<bf16_t>, dim3(blocks), dim3(256), 0, stream, static_cast<const bf16_t *>(x),
                               static_cast<const bf16_t *>(weight), static_cast<bf16_t *>(y), tokens, channels, ld_x, ld_y,
                               eps);
        else
            hipLaunchKernelGGL(rmsnorm_rows_vec<float>, dim3(blocks), dim3(256), 0, stream, static_cast<const float *>(x),
                               static_cast<const float *>(weight), static_cast<float *>(y), tokens, channels, ld_x, ld_y,
                               eps);
        return launch_status();
    }
    if (dtype == PRUNE_BF16)
        hipLaunchKernelGGL(rmsnorm_rows<bf16_t>, dim3(blocks), dim3(256), 0, stream, static_cast<const bf16_t *>(x),
                           static_cast<const bf16_t *>(weight), static_cast<bf16_t *>(y), tokens, channels, ld_x, ld_y, eps);
    else
        hipLaunchKernelGGL(rmsnorm_rows<float>, dim3(blocks), dim3(256), 0, stream, static_cast<const float *>(x),
                           static_cast<const float *>(weight), static_cast<float *>(y), tokens, channels, ld_x, ld_y, eps);
    return launch_status();
}

extern "C" int prune_add(const void *a, const void *b, void *out, int dtype, int64_t rows, int64_t cols, int64_t ld_a,
                         int64_t ld_b, int64_t ld_out, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (rows <= 0 || cols <= 0 || ld_a < cols || ld_b < cols || ld_out < cols) return PRUNE_ERR_SHAPE;
    if (!a || !b || !out) return PRUNE_ERR_NULL;
    const size_t es = elem_size(dtype);
    if (!aligned_to(a, es) || !aligned_to(b, es) || !aligned_to(out, es)) return PRUNE_ERR_ALIGNMENT;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (packet_ok(a, cols, ld_a) && packet_ok(b, cols, ld_b) && packet_ok(out, cols, ld_out)) {
        if (dtype == PRUNE_BF16)
            hipLaunchKernelGGL(add_rows_vec<bf16_t>, dim3(8192), dim3(256), 0, stream, static_cast<const bf16_t *>(a),
                               static_cast<const bf16_t *>(b), static_cast<bf16_t *>(out), rows, cols, ld_a, ld_b, ld_out);
        else
            hipLaunchKernelGGL(add_rows_vec<float>, dim3(8192), dim3(256), 0, stream, static_cast<const float *>(a),
                               static_cast<const float *>(b), static_cast<float *>(out), rows, cols, ld_a, ld_b, ld_out);
        return launch_status();
    }
    if (dtype == PRUNE_BF16)
        hipLaunchKernelGGL(add_rows<bf16_t>, dim3(8192), dim3(256), 0, stream, static_cast<const bf16_t *>(a),
                           static_cast<const bf16_t *>(b), static_cast<bf16_t *>(out), rows, cols, ld_a, ld_b, ld_out);
    else
        hipLaunchKernelGGL(add_rows<float>, dim3(8192), dim3(256), 0, stream, static_cast<const float *>(a),
                           static_cast<const float *>(b), static_cast<float *>(out), rows, cols, ld_a, ld_b, ld_out);
    return launch_status();
}

extern "C" int prune_rotary(void *x, int dtype, int64_t tokens, int64_t heads, int64_t head_dim, int64_t ld,
                            int64_t seq_len, float base, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (tokens <= 0 || heads <= 0 || head_dim <= 0 || head_dim % 2 != 0 || ld < heads * head_dim || seq_len <= 0)
        return PRUNE_ERR_SHAPE;
    if (!x) return PRUNE_ERR_NULL;
    if (!(base > 1.f)) return PRUNE_ERR_RANGE;
    if (!aligned_to(x, elem_size(dtype))) return PRUNE_ERR_ALIGNMENT;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const float log2_base = log2f(base);
    if (head_dim % 16 == 0 && ld % 8 == 0 && aligned_to(x, 16)) {
        if (dtype == PRUNE_BF16)
            hipLaunchKernelGGL(rotary_rows_vec<bf16_t>, dim3(4096), dim3(256), 0, stream, static_cast<bf16_t *>(x), tokens,
                               heads, head_dim, ld, seq_len, log2_base);
        else
            hipLaunchKernelGGL(rotary_rows_vec<float>, dim3(4096), dim3(256), 0, stream, static_cast<float *>(x), tokens,
                               heads, head_dim, ld, seq_len, log2_base);
        return launch_status();
    }
    if (dtype == PRUNE_BF16)
        hipLaunchKernelGGL(rotary_rows<bf16_t>, dim3(4096), dim3(256), 0, stream, static_cast<bf16_t *>(x), tokens, heads,
                           head_dim, ld, seq_len, log2_base);
    else
        hipLaunchKernelGGL(rotary_rows<float>, dim3(4096), dim3(256), 0, stream, static_cast<float *>(x), tokens, heads,
                           head_dim, ld, seq_len, log2_base);
    return launch_status();
}

extern "C" int prune_causal_attention(const void *q, const void *k, const void *v, void *o, int dtype, int64_t n_seqs,
                                      int64_t seq_len, int64_t heads, int64_t kv_heads, int64_t head_dim, int64_t ld_q,
                                      int64_t ld_k, int64_t ld_v, int64_t ld_o, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (n_seqs <= 0 || seq_len <= 0 || heads <= 0 || kv_heads <= 0 || heads % kv_heads != 0 || head_dim <= 0 ||
        head_dim > 256 || ld_q < heads * head_dim || ld_o < heads * head_dim || ld_k < kv_heads * head_dim ||
        ld_v < kv_heads * head_dim)
        return PRUNE_ERR_SHAPE;
    if (!q || !k || !v || !o) return PRUNE_ERR_NULL;
    const size_t es = elem_size(dtype);
    if (!aligned_to(q, es) || !aligned_to(k, es) || !aligned_to(v, es) || !aligned_to(o, es)) return PRUNE_ERR_ALIGNMENT;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (launch_attention_tiles(q, k, v, o, dtype, n_seqs, seq_len, heads, kv_heads, head_dim, ld_q, ld_k, ld_v, ld_o,
                               stream))
        return launch_status();
    const int64_t items = n_seqs * heads * seq_len;
    const unsigned blocks = static_cast<unsigned>(ceil_div(items, 4) < 65536 ? ceil_div(items, 4) : 65536);
    if (dtype == PRUNE_BF16)
        hipLaunchKernelGGL(attention_generic<bf16_t>, dim3(blocks), dim3(256), 0, stream, static_cast<const bf16_t *>(q),
                           static_cast<const bf16_t *>(k), static_cast<const bf16_t *>(v), static_cast<bf16_t *>(o), n_seqs,
                           seq_len, heads, kv_heads, head_dim, ld_q, ld_k, ld_v, ld_o);
    else
        hipLaunchKernelGGL(attention_generic<float>, dim3(blocks), dim3(256), 0, stream, static_cast<const float *>(q),
                           static_cast<const float *>(k), static_cast<const float *>(v), static_cast<float *>(o), n_seqs,
                           seq_len, heads, kv_heads, head_dim, ld_q, ld_k, ld_v, ld_o);
    return launch_status();
}
