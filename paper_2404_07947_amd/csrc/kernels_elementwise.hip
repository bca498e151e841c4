// Bandwidth-bound helper kernels: embedding gather, LayerNorm / RMSNorm, K/V append, greedy argmax.
#include "common.h"
#include "kernels.h"

namespace exe {

// ---------------------------------------------------------------- embedding
// h[t][:] = tok_emb[tokens[t]][:] (+ pos_emb[pos[t]][:]); the residual stream h is float.
template <typename T>
__global__ void embed_kernel(const int32_t* __restrict__ tokens, const int32_t* __restrict__ pos, int d,
                             const T* __restrict__ tok_emb, const T* __restrict__ pos_emb, float* __restrict__ h)
{
    int t = blockIdx.x;
    const T* e = tok_emb + (int64_t)tokens[t] * d;
    const T* p = pos_emb ? pos_emb + (int64_t)pos[t] * d : nullptr;
    float* o = h + (int64_t)t * d;
    for (int k = threadIdx.x; k < d; k += blockDim.x) {
        float v = to_f32(e[k]);
        if (p) v += to_f32(p[k]);
        o[k] = v;
    }
}

template <typename T>
__global__ void load_hidden_kernel(const T* __restrict__ x, int64_t n, float* __restrict__ h)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) h[i] = to_f32(x[i]);
}

template <typename T>
__global__ void store_hidden_kernel(const float* __restrict__ h, int64_t n, T* __restrict__ out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) out[i] = from_f32<T>(h[i]);
}

hipError_t launch_embed(int dtype, const int32_t* tokens, const int32_t* pos, int T, int d, const void* tok_emb,
                        const void* pos_emb, float* h, hipStream_t s)
{
    if (T <= 0) return hipSuccess;
    if (dtype == DT_F32)
        embed_kernel<float><<<T, 256, 0, s>>>(tokens, pos, d, (const float*)tok_emb, (const float*)pos_emb, h);
    else
        embed_kernel<bf16_t><<<T, 256, 0, s>>>(tokens, pos, d, (const bf16_t*)tok_emb, (const bf16_t*)pos_emb, h);
    return hipGetLastError();
}

hipError_t launch_load_hidden(int dtype, const void* x, int64_t n, float* h, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    int blocks = (int)((n + 1023) / 1024 < 8192 ? (n + 1023) / 1024 : 8192);
    if (dtype == DT_F32) load_hidden_kernel<float><<<blocks, 256, 0, s>>>((const float*)x, n, h);
    else load_hidden_kernel<bf16_t><<<blocks, 256, 0, s>>>((const bf16_t*)x, n, h);
    return hipGetLastError();
}

hipError_t launch_store_hidden(int dtype, const float* h, int64_t n, void* out, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    int blocks = (int)((n + 1023) / 1024 < 8192 ? (n + 1023) / 1024 : 8192);
    if (dtype == DT_F32) store_hidden_kernel<float><<<blocks, 256, 0, s>>>(h, n, (float*)out);
    else store_hidden_kernel<bf16_t><<<blocks, 256, 0, s>>>(h, n, (bf16_t*)out);
    return hipGetLastError();
}

// ---------------------------------------------------------------- norms
// One workgroup per row.  The row is kept in LDS as float, statistics are exact two-pass in float:
// LayerNorm: mean, then the mean of squared deviations; RMSNorm: mean of squares.
__device__ __forceinline__ float block_sum(float v, float* red)
{
    v = wave_sum(v);
    int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < nw; ++i) t += red[i];
    return t;
}

// four consecutive elements (k is a multiple of 4, rows start at multiples of 4 elements) as one access
__device__ __forceinline__ f32x4 load4(const float* p) { return *(const f32x4*)p; }
__device__ __forceinline__ f32x4 load4(const bf16_t* p)
{
    uint2 u = *(const uint2*)p;
    return f32x4{bf16lo(u.x), bf16hi(u.x), bf16lo(u.y), bf16hi(u.y)};
}
__device__ __forceinline__ void store4(float* p, f32x4 v) { *(f32x4*)p = v; }
__device__ __forceinline__ void store4(bf16_t* p, f32x4 v)
{
    bf16x4 w;
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = (bf16_t)v[j];
    *(bf16x4*)p = w;
}

template <typename T, bool RMS>
__global__ void norm_kernel(const float* __restrict__ x, const int32_t* __restrict__ row_index, int d,
                            const T* __restrict__ gain, const T* __restrict__ shift, float eps, float out_scale,
                            T* __restrict__ out)
{
    extern __shared__ float row[];
    __shared__ float red[16];
    int r = blockIdx.x;
    int64_t src = row_index ? row_index[r] : r;
    const float* xr = x + src * d;
    float s = 0.f;
    for (int k = threadIdx.x * 4; k < d; k += blockDim.x * 4) {
        f32x4 v = *(const f32x4*)(xr + k);
        *(f32x4*)(row + k) = v;
        s += RMS ? (v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w) : (v.x + v.y + v.z + v.w);
    }
    float tot = block_sum(s, red);
    float mean = 0.f, rstd;
    if (RMS) {
        rstd = 1.f / sqrtf(tot / d + eps);
    } else {
        mean = tot / d;
        float q = 0.f;
        for (int k = threadIdx.x * 4; k < d; k += blockDim.x * 4) {
            f32x4 v = *(const f32x4*)(row + k);
            float a = v.x - mean, b = v.y - mean, c = v.z - mean, e = v.w - mean;
            q += a * a + b * b + c * c + e * e;
        }
        float var = block_sum(q, red) / d;
        rstd = 1.f / sqrtf(var + eps);
    }
    T* o = out + (int64_t)r * d;
    for (int k = threadIdx.x * 4; k < d; k += blockDim.x * 4) {
        f32x4 v = *(const f32x4*)(row + k);
        f32x4 g = load4(gain + k), b = RMS ? f32x4{0.f, 0.f, 0.f, 0.f} : load4(shift + k), y;
#pragma unroll
        for (int j = 0; j < 4; ++j) y[j] = ((v[j] - mean) * rstd * g[j] + b[j]) * out_scale;
        store4(o + k, y);
    }
}

hipError_t launch_norm(int dtype, int rms, const float* x, const int32_t* row_index, int rows, int d,
                       const void* gain, const void* shift, float eps, float out_scale, void* out, hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    if (d % 4 != 0 || d > 36864) return hipErrorInvalidValue;
    size_t lds = (size_t)d * sizeof(float);
    int threads = d >= 4096 ? 512 : 256;
#define EXE_NORM(T, R)                                                                                       \
    norm_kernel<T, R><<<rows, threads, lds, s>>>(x, row_index, d, (const T*)gain, (const T*)shift, eps,      \
                                                 out_scale, (T*)out)
    if (dtype == DT_F32) { if (rms) EXE_NORM(float, true); else EXE_NORM(float, false); }
    else { if (rms) EXE_NORM(bf16_t, true); else EXE_NORM(bf16_t, false); }
#undef EXE_NORM
    return hipGetLastError();
}

// ---------------------------------------------------------------- K/V append
// grid (T, 2): blockIdx.y = 0 keys, 1 values.  Each thread moves 16 bytes.
template <typename T>
__global__ void kv_append_kernel(const T* __restrict__ src, int ld, int k_off, int v_off,
                                 const int32_t* __restrict__ tok_b, const int32_t* __restrict__ tok_pos,
                                 const int64_t* __restrict__ base, const int32_t* __restrict__ cap, int layer, int H,
                                 int dh, T* __restrict__ pool)
{
    constexpr int EPL = 16 / sizeof(T);
    int t = blockIdx.x, kv = blockIdx.y;
    int b = tok_b ? tok_b[t] : t;
    int pos = tok_pos[t];
    int64_t c = cap[b];
    const T* s = src + (int64_t)t * ld + (kv ? v_off : k_off);
    T* dst = pool + base[b] + ((int64_t)(layer * 2 + kv) * H) * c * dh + (int64_t)pos * dh;
    int inner = H * dh;
    for (int e = threadIdx.x * EPL; e < inner; e += blockDim.x * EPL) {
        int head = e / dh, col = e - head * dh;
        *(uint4*)(dst + (int64_t)head * c * dh + col) = *(const uint4*)(s + e);
    }
}

hipError_t launch_kv_append(int dtype, const void* src, int ld, int k_off, int v_off, int T, const int32_t* tok_b,
                            const int32_t* tok_pos, const int64_t* base, const int32_t* cap, int layer, int H, int dh,
                            void* pool, hipStream_t s)
{
    if (T <= 0) return hipSuccess;
    int epl = dtype == DT_F32 ? 4 : 8;
    if (dh % epl || ld % epl || k_off % epl || v_off % epl) return hipErrorInvalidValue;
    dim3 grid(T, 2);
    if (dtype == DT_F32)
        kv_append_kernel<float><<<grid, 256, 0, s>>>((const float*)src, ld, k_off, v_off, tok_b, tok_pos, base, cap,
                                                     layer, H, dh, (float*)pool);
    else
        kv_append_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t*)src, ld, k_off, v_off, tok_b, tok_pos, base,
                                                      cap, layer, H, dh, (bf16_t*)pool);
    return hipGetLastError();
}

// Paged pool: the same rows into blocks of 2^shift positions.  `layer_pool` is the layer's slab of blocks, block b at
// b * 2*H*2^shift*dh elements holding [K|V][head][row][dh]; table [sequences][table_w] lists each sequence's blocks.
template <typename T>
__global__ void kv_append_paged_kernel(const T* __restrict__ src, int ld, int k_off, int v_off,
                                       const int32_t* __restrict__ tok_b, const int32_t* __restrict__ tok_pos,
                                       const int32_t* __restrict__ table, int table_w, int shift, int H, int dh,
                                       T* __restrict__ layer_pool)
{
    constexpr int EPL = 16 / sizeof(T);
    int t = blockIdx.x, kv = blockIdx.y;
    int b = tok_b ? tok_b[t] : t;
    int pos = tok_pos[t];
    int64_t rows = (int64_t)1 << shift;
    int blk = table[(int64_t)b * table_w + (pos >> shift)];
    const T* s = src + (int64_t)t * ld + (kv ? v_off : k_off);
    T* dst = layer_pool + ((int64_t)blk * 2 + kv) * H * rows * dh + (int64_t)(pos & (rows - 1)) * dh;
    int inner = H * dh;
    for (int e = threadIdx.x * EPL; e < inner; e += blockDim.x * EPL) {
        int head = e / dh, col = e - head * dh;
        *(uint4*)(dst + (int64_t)head * rows * dh + col) = *(const uint4*)(s + e);
    }
}

hipError_t launch_kv_append_paged(int dtype, const void* src, int ld, int k_off, int v_off, int T, const int32_t* tok_b,
                                  const int32_t* tok_pos, const int32_t* table, int table_w, int shift, int H, int dh,
                                  void* layer_pool, hipStream_t s)
{
    if (T <= 0) return hipSuccess;
    int epl = dtype == DT_F32 ? 4 : 8;
    if (dh % epl || ld % epl || k_off % epl || v_off % epl || !table || table_w < 1) return hipErrorInvalidValue;
    dim3 grid(T, 2);
    if (dtype == DT_F32)
        kv_append_paged_kernel<float><<<grid, 256, 0, s>>>((const float*)src, ld, k_off, v_off, tok_b, tok_pos, table, table_w,
                                                           shift, H, dh, (float*)layer_pool);
    else
        kv_append_paged_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t*)src, ld, k_off, v_off, tok_b, tok_pos, table,
                                                            table_w, shift, H, dh, (bf16_t*)layer_pool);
    return hipGetLastError();
}

// ---------------------------------------------------------------- greedy argmax
// One workgroup per row; ties resolve to the lowest index at every level of the reduction.
__global__ void argmax_kernel(const float* __restrict__ logits, int n, int32_t* __restrict__ out)
{
    __shared__ float bv[16];
    __shared__ int bi[16];
    const float* x = logits + (int64_t)blockIdx.x * n;
    float best = -INFINITY;
    int idx = 0x7fffffff;
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        float v = x[i];
        if (v > best || (v == best && i < idx)) { best = v; idx = i; }
    }
    if (idx == 0x7fffffff) { best = -INFINITY; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(best, o, WAVE);
        int oi = __shfl_xor(idx, o, WAVE);
        if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
    }
    int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { bv[w] = best; bi[w] = idx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < (int)(blockDim.x >> 6); ++i)
            if (bv[i] > best || (bv[i] == best && bi[i] < idx)) { best = bv[i]; idx = bi[i]; }
        out[blockIdx.x] = idx == 0x7fffffff ? 0 : idx;
    }
}

hipError_t launch_argmax(const float* logits, int rows, int n, int32_t* out, hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    argmax_kernel<<<rows, 1024, 0, s>>>(logits, n, out);
    return hipGetLastError();
}

}  // namespace exe
