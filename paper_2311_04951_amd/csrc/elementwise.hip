// Small row-wise kernels of the verify pass: embedding gather, RMSNorm (+ packing of the result as
// the activation planes the next GEMM reads), cache-length bookkeeping (Section 4.4: truncation is a
// length write) and the raw cache append used to build an existing context.
#include <cstdlib>
#include "ss_device.h"
#include "ss_kernels.h"
#include <algorithm>

namespace ss {

// h[r][:] = E[token[r]][:]
template <typename T>
__global__ void embed_kernel(const T *embed, const int32_t *tokens, int d, int vocab, float *h, int32_t *status) {
    const int r = blockIdx.x;
    int tok = tokens[r];
    if (tok < 0 || tok >= vocab) {
        if (threadIdx.x == 0) atomicOr(status, 1);
        tok = tok < 0 ? 0 : vocab - 1;
    }
    const T *src = embed + (size_t)tok * d;
    for (int e = threadIdx.x; e < d; e += blockDim.x) h[(size_t)r * d + e] = to_f32(src[e]);
}

void launch_embed(int dtype, const void *embed, const int32_t *tokens, int R, int d, int vocab, float *h,
                  int32_t *status, hipStream_t st) {
    if (dtype) hipLaunchKernelGGL((embed_kernel<bf16_t>), dim3(R), dim3(256), 0, st, (const bf16_t *)embed, tokens, d, vocab, h, status);
    else hipLaunchKernelGGL((embed_kernel<float>), dim3(R), dim3(256), 0, st, (const float *)embed, tokens, d, vocab, h, status);
}

// act[r][:] = h[src][:] * gain / sqrt(mean(h[src]^2) + eps) with src = row0 + r*row_stride.
// One workgroup per row; a row of up to 8192 elements stays in registers between the two passes (16-byte
// loads, 8-byte stores of four packed values per plane); longer or unaligned rows take the plain loops.
__device__ __forceinline__ void store_act4(const ActPlanes<bf16_t> &a, size_t off, const float (&x)[4]) {
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        hi[j] = bf16_rne(x[j]);
        lo[j] = bf16_rne(x[j] - bf16_bits_to_f32(hi[j]));
    }
    *reinterpret_cast<uint2 *>(a.base + off) = make_uint2(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16));
    *reinterpret_cast<uint2 *>(a.base + a.plane + off) = make_uint2(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16));
}
__device__ __forceinline__ void store_act4(const ActPlanes<float> &a, size_t off, const float (&x)[4]) {
    *reinterpret_cast<float4 *>(a.base + off) = make_float4(x[0], x[1], x[2], x[3]);
}
// SPLITK: the row is first completed, x = h[r] + (parts[0][r] + parts[1][r] + ...) with the splits added in order, and
// stored back to h; without a gain that is all (the norm below is the same code either way, so a fused launch and
// the two separate ones give the same bits).
constexpr int SPLITK_MAX = 4; // splits the fused form can sum (the wide GEMM never makes more)
template <typename T, bool SPLITK>
__global__ __launch_bounds__(256) void rmsnorm_pack_kernel(const float *h, const float *gain, int row0, int row_stride,
                                                           int d, float eps, ActPlanes<T> act, const float *parts,
                                                           int ksplit, size_t part_stride, float *h_out) {
    constexpr int MAXV = 8; // float4 per thread kept in registers
    const int r = blockIdx.x;
    const float *x = h + (size_t)(row0 + r * row_stride) * d;
    const bool vec = d % 4 == 0 && d <= 256 * 4 * MAXV && act.ld % 4 == 0 && act.plane % 4 == 0 &&
                     (reinterpret_cast<uintptr_t>(h) & 15) == 0 && (reinterpret_cast<uintptr_t>(gain) & 15) == 0 &&
                     (reinterpret_cast<uintptr_t>(act.base) & 15) == 0 &&
                     (!SPLITK || ((reinterpret_cast<uintptr_t>(parts) & 15) == 0 && part_stride % 4 == 0));
    float4 v[MAXV], gn[MAXV];
    float ss = 0.f;
    if (vec) {
#pragma unroll
        for (int j = 0; j < MAXV; ++j) {
            const int e4 = threadIdx.x + 256 * j;
            v[j] = e4 * 4 < d ? reinterpret_cast<const float4 *>(x)[e4] : make_float4(0.f, 0.f, 0.f, 0.f);
            // the gains are requested with the row, not behind the reduction (one memory round trip less)
            gn[j] = (gain && e4 * 4 < d) ? reinterpret_cast<const float4 *>(gain)[e4] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        if constexpr (SPLITK) {
            // every partial is requested before the first one is used (at most SPLITK_MAX splits)
            float4 p[MAXV][SPLITK_MAX];
#pragma unroll
            for (int j = 0; j < MAXV; ++j)
#pragma unroll
                for (int z = 0; z < SPLITK_MAX; ++z) {
                    const int e4 = threadIdx.x + 256 * j;
                    p[j][z] = (e4 * 4 < d && z < ksplit) ? reinterpret_cast<const float4 *>(parts + z * part_stride + (size_t)r * d)[e4]
                                                         : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
            for (int j = 0; j < MAXV; ++j) {
                const int e4 = threadIdx.x + 256 * j;
                if (e4 * 4 < d) {
                    float4 s4 = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int z = 0; z < SPLITK_MAX; ++z)
                        if (z < ksplit) {
                            s4.x += p[j][z].x; s4.y += p[j][z].y; s4.z += p[j][z].z; s4.w += p[j][z].w;
                        }
                    v[j].x += s4.x; v[j].y += s4.y; v[j].z += s4.z; v[j].w += s4.w;
                    reinterpret_cast<float4 *>(h_out + (size_t)r * d)[e4] = v[j];
                }
            }
            if (!gain) return;
        }
#pragma unroll
        for (int j = 0; j < MAXV; ++j) ss += (v[j].x * v[j].x + v[j].y * v[j].y) + (v[j].z * v[j].z + v[j].w * v[j].w);
    } else {
        if constexpr (SPLITK) {
            for (int e = threadIdx.x; e < d; e += 256) {
                float s1 = 0.f;
                for (int z = 0; z < ksplit; ++z) s1 += parts[z * part_stride + (size_t)r * d + e];
                h_out[(size_t)r * d + e] = x[e] + s1; // x is this row of h_out; the same thread reads it back below
            }
            if (!gain) return;
        }
        for (int e = threadIdx.x; e < d; e += 256) ss += x[e] * x[e];
    }
    ss = wave_sum(ss);
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = (part[0] + part[1]) + (part[2] + part[3]);
    const float scale = 1.0f / sqrtf(tot / (float)d + eps);
    if (vec) {
#pragma unroll
        for (int j = 0; j < MAXV; ++j) {
            const int e4 = threadIdx.x + 256 * j;
            if (e4 * 4 < d) {
                const float4 g = gn[j];
                const float o[4] = {v[j].x * scale * g.x, v[j].y * scale * g.y, v[j].z * scale * g.z, v[j].w * scale * g.w};
                store_act4(act, (size_t)r * act.ld + 4 * e4, o);
            }
        }
    } else {
        for (int e = threadIdx.x; e < d; e += 256) store_act(act, (size_t)r * act.ld + e, x[e] * scale * gain[e]);
    }
}

void launch_rmsnorm_pack_rows(int dtype, const float *h, const float *gain, int nrows, int row0, int row_stride,
                              int d, float eps, void *act, size_t act_plane, int ld_act, hipStream_t st) {
    if (dtype) {
        ActPlanes<bf16_t> ap{(bf16_t *)act, act_plane, ld_act};
        hipLaunchKernelGGL((rmsnorm_pack_kernel<bf16_t, false>), dim3(nrows), dim3(256), 0, st, h, gain, row0, row_stride, d, eps, ap, nullptr, 0, (size_t)0, nullptr);
    } else {
        ActPlanes<float> ap{(float *)act, act_plane, ld_act};
        hipLaunchKernelGGL((rmsnorm_pack_kernel<float, false>), dim3(nrows), dim3(256), 0, st, h, gain, row0, row_stride, d, eps, ap, nullptr, 0, (size_t)0, nullptr);
    }
}

void launch_rmsnorm_pack(int dtype, const float *h, const float *gain, int R, int d, float eps, void *act,
                         size_t act_plane, int ld_act, hipStream_t st) {
    launch_rmsnorm_pack_rows(dtype, h, gain, R, 0, 1, d, eps, act, act_plane, ld_act, st);
}

void launch_splitk_resid_norm(int dtype, float *h, const float *parts, int ksplit, const float *gain, int R, int d,
                              float eps, void *act, size_t act_plane, int ld_act, hipStream_t st) {
    if (ksplit > SPLITK_MAX) abort(); // the caller's split count is bounded by the same constant
    const size_t stride = (size_t)R * d;
    if (dtype) {
        ActPlanes<bf16_t> ap{(bf16_t *)act, act_plane, ld_act};
        hipLaunchKernelGGL((rmsnorm_pack_kernel<bf16_t, true>), dim3(R), dim3(256), 0, st, h, gain, 0, 1, d, eps, ap, parts, ksplit, stride, h);
    } else {
        ActPlanes<float> ap{(float *)act, act_plane, ld_act};
        hipLaunchKernelGGL((rmsnorm_pack_kernel<float, true>), dim3(R), dim3(256), 0, st, h, gain, 0, 1, d, eps, ap, parts, ksplit, stride, h);
    }
}

__global__ void len_add_kernel(int32_t *len, int batch, int delta) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < batch) len[b] += delta;
}
void launch_len_add(int32_t *len, int batch, int delta, hipStream_t st) {
    hipLaunchKernelGGL(len_add_kernel, dim3((batch + 63) / 64), dim3(64), 0, st, len, batch, delta);
}

// after the rejection step only the first n_accepted + 1 of the M appended rows stay
__global__ void len_rollback_kernel(int32_t *len, const int32_t *n_accepted, int batch, int M) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < batch) {
        int a = n_accepted[b];
        a = a < 0 ? 0 : (a > M - 1 ? M - 1 : a);
        len[b] -= M - 1 - a;
    }
}
void launch_len_rollback(int32_t *len, const int32_t *n_accepted, int batch, int M, hipStream_t st) {
    hipLaunchKernelGGL(len_rollback_kernel, dim3((batch + 63) / 64), dim3(64), 0, st, len, n_accepted, batch, M);
}

// The batched speculative step's token plumbing.  verify rows of sequence b = [its last committed token, d_1 .. d_K]
// (the draft's tokens arrive call-major, [K][batch]); the same tokens sequence-major for the rejection step.
__global__ void step_pack_tokens_kernel(const int32_t *feed, const int32_t *dtok, int batch, int K, int32_t *vt, int32_t *dbk) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= batch * (K + 1)) return;
    const int b = idx / (K + 1), j = idx - b * (K + 1);
    const int32_t v = j == 0 ? feed[2 * b + 1] : dtok[(size_t)(j - 1) * batch + b];
    vt[idx] = v;
    if (j > 0) dbk[b * K + j - 1] = v;
}
void launch_step_pack_tokens(const int32_t *feed, const int32_t *dtok, int batch, int K, int32_t *vt, int32_t *dbk, hipStream_t st) {
    const int n = batch * (K + 1);
    hipLaunchKernelGGL(step_pack_tokens_kernel, dim3((n + 63) / 64), dim3(64), 0, st, feed, dtok, batch, K, vt, dbk);
}
// the next step's draft feed of sequence b: its last two committed tokens = [verify row a_b, the token that followed]
__global__ void step_next_feed_kernel(const int32_t *vt, const int32_t *n_accepted, const int32_t *next, int batch, int K, int32_t *feed) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    int a = n_accepted[b];
    a = a < 0 ? 0 : (a > K ? K : a);
    feed[2 * b] = vt[b * (K + 1) + a];
    feed[2 * b + 1] = next[b];
}
void launch_step_next_feed(const int32_t *vt, const int32_t *n_accepted, const int32_t *next, int batch, int K, int32_t *feed, hipStream_t st) {
    hipLaunchKernelGGL(step_next_feed_kernel, dim3((batch + 63) / 64), dim3(64), 0, st, vt, n_accepted, next, batch, K, feed);
}

// truncation from a device array (Section 4.4: dropping the stale tail of a cache is a length write)
__global__ void len_truncate_kernel(int32_t *len, const int32_t *new_len, int batch, int32_t *status) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < batch) {
        const int want = new_len[b] < 0 ? 0 : new_len[b];
        if (want > len[b]) {
            if (status) atomicOr(status, 4);
        } else {
            len[b] = want;
        }
    }
}
void launch_len_truncate(int32_t *len, const int32_t *new_len, int batch, int32_t *status, hipStream_t st) {
    hipLaunchKernelGGL(len_truncate_kernel, dim3((batch + 63) / 64), dim3(64), 0, st, len, new_len, batch, status);
}

__global__ void fill_u32_kernel(uint32_t *p, size_t n, uint32_t value) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = value;
}
void launch_fill_u32(uint32_t *p, size_t n, uint32_t value, hipStream_t st) {
    if (!n) return;
    const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, 1024);
    hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks), dim3(256), 0, st, p, n, value);
}

// raw append: rows [n_rows][H*hd] of rotated keys / values into sequence `seq` at pos0..
template <typename T>
__global__ void kv_append_kernel(T *kc, T *vc, const T *k, const T *v, int seq, int pos0, int H, int hd, int S) {
    const int r = blockIdx.x, pos = pos0 + r;
    const int W = H * hd;
    for (int e = threadIdx.x; e < W; e += blockDim.x) {
        const int h = e / hd, j = e - h * hd;
        const size_t head = ((size_t)seq * H + h) * S * hd;
        kc[head + (size_t)pos * hd + j] = k[(size_t)r * W + e];
        vc[head + ((size_t)(pos >> 6) * hd + j) * 64 + (pos & 63)] = v[(size_t)r * W + e];
    }
}
void launch_kv_append(int dtype, void *kc, void *vc, const void *k, const void *v, int seq, int pos0, int n_rows,
                      int H, int hd, int S, hipStream_t st) {
    if (n_rows <= 0) return;
    if (dtype) hipLaunchKernelGGL((kv_append_kernel<bf16_t>), dim3(n_rows), dim3(256), 0, st, (bf16_t *)kc, (bf16_t *)vc, (const bf16_t *)k, (const bf16_t *)v, seq, pos0, H, hd, S);
    else hipLaunchKernelGGL((kv_append_kernel<float>), dim3(n_rows), dim3(256), 0, st, (float *)kc, (float *)vc, (const float *)k, (const float *)v, seq, pos0, H, hd, S);
}

// Row-wise int8 quantisation (one workgroup per row).  Every step is one IEEE fp32 operation (maximum of
// absolute values, a correctly rounded division by 127, a correctly rounded division by the scale, round to
// nearest even), so the bytes do not depend on how the row is split over threads.
template <typename T>
__global__ void __launch_bounds__(256) quantize_rows_int8_kernel(const T *__restrict__ W, long long K, int8_t *__restrict__ q, float *__restrict__ scale) {
    __shared__ float red[256];
    const size_t base = (size_t)blockIdx.x * (size_t)K;
    float amax = 0.f;
    for (long long k = threadIdx.x; k < K; k += 256) amax = fmaxf(amax, fabsf(to_f32(W[base + k])));
    red[threadIdx.x] = amax;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    amax = red[0];
    const float sc = amax > 0.f ? __fdiv_rn(amax, 127.0f) : 1.0f;
    if (threadIdx.x == 0) scale[blockIdx.x] = sc;
    for (long long k = threadIdx.x; k < K; k += 256) {
        float t = rintf(__fdiv_rn(to_f32(W[base + k]), sc));
        t = fminf(fmaxf(t, -127.0f), 127.0f);
        q[base + k] = (int8_t)(int)t;
    }
}
void launch_quantize_rows_int8(int dtype, const void *W, long long rows, long long K, int8_t *q, float *scale, hipStream_t st) {
    if (rows <= 0) return;
    if (dtype) hipLaunchKernelGGL((quantize_rows_int8_kernel<bf16_t>), dim3((unsigned)rows), dim3(256), 0, st, (const bf16_t *)W, K, q, scale);
    else hipLaunchKernelGGL((quantize_rows_int8_kernel<float>), dim3((unsigned)rows), dim3(256), 0, st, (const float *)W, K, q, scale);
}

// int4 with one scale per group of 128 entries: a wavefront per group, a lane per byte (two entries).  The
// same single IEEE operations as the int8 quantiser, with 7 in place of 127.
template <typename T>
__global__ void __launch_bounds__(256) quantize_rows_int4_kernel(const T *__restrict__ W, long long rows, long long K, uint8_t *__restrict__ q, float *__restrict__ scale) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t base = (size_t)blockIdx.x * (size_t)K;
    for (long long j = wave; j < K / 128; j += 4) {
        const size_t k = base + (size_t)j * 128 + 2 * lane;
        const float w0 = to_f32(W[k]), w1 = to_f32(W[k + 1]);
        float amax = fmaxf(fabsf(w0), fabsf(w1));
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
        const float sc = amax > 0.f ? __fdiv_rn(amax, 7.0f) : 1.0f;
        if (lane == 0) scale[(size_t)j * (size_t)rows + blockIdx.x] = sc;
        const float t0 = fminf(fmaxf(rintf(__fdiv_rn(w0, sc)), -7.0f), 7.0f), t1 = fminf(fmaxf(rintf(__fdiv_rn(w1, sc)), -7.0f), 7.0f);
        q[k / 2] = (uint8_t)(((int)t0 & 0xf) | (((int)t1 & 0xf) << 4));
    }
}
void launch_quantize_rows_int4(int dtype, const void *W, long long rows, long long K, uint8_t *q, float *scale, hipStream_t st) {
    if (rows <= 0) return;
    if (dtype) hipLaunchKernelGGL((quantize_rows_int4_kernel<bf16_t>), dim3((unsigned)rows), dim3(256), 0, st, (const bf16_t *)W, rows, K, q, scale);
    else hipLaunchKernelGGL((quantize_rows_int4_kernel<float>), dim3((unsigned)rows), dim3(256), 0, st, (const float *)W, rows, K, q, scale);
}

// Read-stream probe: every lane keeps eight independent 16-byte loads in flight, a wavefront instruction
// covers 1 KB contiguous, the grid walks the buffer once.  The loads are folded into a word that is stored
// only if it equals a value the data cannot be arranged to avoid checking, which keeps them alive.
typedef uint32_t probe_u32x4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) read_probe_kernel(const probe_u32x4 *__restrict__ src, size_t n16, uint32_t *sink) {
    constexpr int U = 8;
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    probe_u32x4 acc = {0u, 0u, 0u, 0u};
    size_t i = tid;
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        probe_u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = 1u;
}
void launch_read_probe(const void *buf, size_t bytes, uint32_t *sink, hipStream_t st) {
    hipLaunchKernelGGL(read_probe_kernel, dim3(4096), dim3(256), 0, st, (const probe_u32x4 *)buf, bytes / 16, sink);
}

} // namespace ss
