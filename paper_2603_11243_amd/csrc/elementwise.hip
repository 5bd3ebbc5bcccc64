// Memory-bound helpers of the decoder forward: input-row assembly, RMSNorm, weight re-layout,
// and the first-failing-token scan of the acceptance rule.
#include <algorithm>
#include <type_traits>

#include "device_utils.h"
#include "ssd_internal.h"

namespace ssd {

// ---------------------------------------------------------------------------------------------
// Input assembly (Sec. 2.2: the LLM sees the speech embeddings g, the prompt and the draft prefix):
// decoder row r <- speech_emb[src] or embed[token id], widened to the fp32 residual stream.
template <typename T>
__global__ void __launch_bounds__(256) embed_rows_kernel(const T* __restrict__ speech_emb, const T* __restrict__ embed,
                                                         const int32_t* __restrict__ prompt_ids,
                                                         const int32_t* __restrict__ draft_ids,
                                                         const int32_t* __restrict__ row_src, int M, int d, int vocab,
                                                         float* __restrict__ x, int32_t* __restrict__ flags) {
    const int r = blockIdx.x;
    const int32_t code = row_src[r];
    const T* src;
    if (code & (SRC_DRAFT | SRC_PROMPT)) {
        const int raw = (code & SRC_DRAFT) ? draft_ids[code & SRC_MASK] : prompt_ids[code & SRC_MASK];
        const int id = raw < 0 ? 0 : (raw >= vocab ? vocab - 1 : raw);
        if (id != raw && threadIdx.x == 0) raise_flag(flags, SSD_FLAG_TOKEN_CLAMPED);   // sticky until read
        src = embed + (int64_t)id * d;
    } else {
        src = speech_emb + (int64_t)code * d;
    }
    float* dst = x + (int64_t)r * d;
    for (int i = threadIdx.x; i < d; i += 256) {
        if constexpr (sizeof(T) == 2) dst[i] = bf16_to_f32(src[i]); else dst[i] = src[i];
    }
}

void launch_embed_rows(int dtype, const void* speech_emb, const void* embed, const int32_t* prompt_ids,
                       const int32_t* draft_ids, const int32_t* row_src, int M, int d, int vocab, float* x,
                       int32_t* flags, hipStream_t st) {
    if (M <= 0) return;
    if (dtype == SSD_BF16)
        hipLaunchKernelGGL(embed_rows_kernel<bf16_t>, dim3(M), dim3(256), 0, st, (const bf16_t*)speech_emb,
                           (const bf16_t*)embed, prompt_ids, draft_ids, row_src, M, d, vocab, x, flags);
    else
        hipLaunchKernelGGL(embed_rows_kernel<float>, dim3(M), dim3(256), 0, st, (const float*)speech_emb,
                           (const float*)embed, prompt_ids, draft_ids, row_src, M, d, vocab, x, flags);
}

// ---------------------------------------------------------------------------------------------
// dst[r] = src[row_idx[r]] for rows of row_bytes (a multiple of 16) bytes.
__global__ void __launch_bounds__(256) gather_rows_kernel(const uint4* __restrict__ src, const int32_t* __restrict__ row_idx,
                                                          int chunks, uint4* __restrict__ dst) {
    const uint4* s = src + (int64_t)row_idx[blockIdx.x] * chunks;
    uint4* d = dst + (int64_t)blockIdx.x * chunks;
    for (int i = threadIdx.x; i < chunks; i += 256) d[i] = s[i];
}

void launch_gather_rows(const void* src, const int32_t* row_idx, int n_rows, int64_t row_bytes, void* dst, hipStream_t st) {
    if (n_rows <= 0) return;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(n_rows), dim3(256), 0, st, static_cast<const uint4*>(src), row_idx,
                       (int)(row_bytes / 16), static_cast<uint4*>(dst));
}

// out[i] = table ? table[clamp(src[idx[i]], 0, n_table - 1)] : src[idx[i]]   (token-id gathers between the gate and
// the verification pass: prompt ids of the selected utterances, CTC draft symbols mapped to LLM token ids)
__global__ void __launch_bounds__(256) gather_ids_kernel(const int32_t* __restrict__ src, const int32_t* __restrict__ idx, int n,
                                                         const int32_t* __restrict__ table, int n_table, int32_t* __restrict__ out) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    int v = src[idx[i]];
    if (table) v = table[min(max(v, 0), n_table - 1)];
    out[i] = v;
}

void launch_gather_ids(const int32_t* src, const int32_t* idx, int n, const int32_t* table, int n_table, int32_t* out, hipStream_t st) {
    if (n <= 0) return;
    hipLaunchKernelGGL(gather_ids_kernel, dim3((n + 255) / 256), dim3(256), 0, st, src, idx, n, table, n_table, out);
}

// ---------------------------------------------------------------------------------------------
// RMSNorm: out[r] = x[row] * gain / sqrt(mean(x[row]^2) + eps), row = row_idx ? row_idx[r] : r.
// One wavefront per row; statistics in fp32.  d must be a multiple of 4.
// T = bf16 gain with f16 output (MFMA operand type), or fp32 gain with fp32 output.
template <typename T, int NV, bool BF>
__global__ void __launch_bounds__(256) rmsnorm_kernel(float* __restrict__ x, const T* __restrict__ gain,
                                                      const int32_t* __restrict__ row_idx, int n_rows, int d,
                                                      float eps, T* __restrict__ out, const float* __restrict__ partials,
                                                      int n_splits, int64_t split_stride, int32_t* __restrict__ flags) {
    // the row stays in registers between the statistic and the scaling: NV float4 per lane (d <= 256*NV)
    const int lane = threadIdx.x % 64;
    const int r = blockIdx.x * 4 + threadIdx.x / 64;
    if (r >= n_rows) return;
    const int64_t row = row_idx ? row_idx[r] : r;
    float4* src = reinterpret_cast<float4*>(x + row * d);
    const int n4 = d / 4;
    float4 v[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int i = lane + 64 * j;
        if (i < n4) {
            typedef float f32x4v __attribute__((ext_vector_type(4)));
            const f32x4v t = __builtin_nontemporal_load(reinterpret_cast<const f32x4v*>(src) + i);
            v[j] = make_float4(t[0], t[1], t[2], t[3]);
        } else {
            v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    if (n_splits > 1) {
        // pending K-split partial sums of the projection before this norm: add them in split order
        for (int s = 0; s < n_splits; ++s) {
            const float4* ps = reinterpret_cast<const float4*>(partials + s * split_stride + row * d);
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int i = lane + 64 * j;
                if (i < n4) {
                    const float4 p = ps[i];
                    v[j].x += p.x; v[j].y += p.y; v[j].z += p.z; v[j].w += p.w;
                }
            }
        }
        if (!row_idx) {
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int i = lane + 64 * j;
                if (i < n4) src[i] = v[j];
            }
        }
    }
    // the gain is fetched before the reduction, so that its cache round trip overlaps with it
    uint2 g16[sizeof(T) == 2 ? NV : 1];
    if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int i = lane + 64 * j;
            g16[j] = i < n4 ? reinterpret_cast<const uint2*>(gain)[i] : make_uint2(0u, 0u);
        }
    }
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) ss += v[j].x * v[j].x + v[j].y * v[j].y + v[j].z * v[j].z + v[j].w * v[j].w;
    ss = group_allreduce<64>(ss, OpSum());
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    T* dst = out + (int64_t)r * d;
    float peak = 0.f;
    auto store_row = [&](auto clamp_c) {
        constexpr bool CLAMP = decltype(clamp_c)::value;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int i = lane + 64 * j;
            if (i >= n4) continue;
            if constexpr (sizeof(T) == 2) {
                const uint2 g = g16[j];
                uint2 o;
                o.x = op_store2<BF, CLAMP>(v[j].x * inv * bf16_lo(g.x), v[j].y * inv * bf16_hi(g.x), peak);
                o.y = op_store2<BF, CLAMP>(v[j].z * inv * bf16_lo(g.y), v[j].w * inv * bf16_hi(g.y), peak);
                reinterpret_cast<uint2*>(dst)[i] = o;
            } else {
                const float4 g = reinterpret_cast<const float4*>(gain)[i];
                reinterpret_cast<float4*>(dst)[i] =
                    make_float4(v[j].x * inv * g.x, v[j].y * inv * g.y, v[j].z * inv * g.z, v[j].w * inv * g.w);
            }
        }
    };
    store_row(std::false_type());
    if (!(peak <= F16_MAX)) {                               // a gain large enough to leave the half range: store saturated
        store_row(std::true_type());
        raise_flag(flags, SSD_FLAG_ACT_OVERFLOW);
    }
}

// Same operation with one workgroup per row, for launches with few rows (there a wavefront per row
// leaves most of the chip idle and serialises the split sums): every thread owns d/1024 float4s
// and all its split loads are issued together.
template <typename T, int MAXV, bool BF>
__global__ void __launch_bounds__(256) rmsnorm_row_kernel(float* __restrict__ x, const T* __restrict__ gain,
                                                          const int32_t* __restrict__ row_idx, int d, float eps,
                                                          T* __restrict__ out, const float* __restrict__ partials,
                                                          int n_splits, int64_t split_stride, int32_t* __restrict__ flags) {
    __shared__ float red[4];
    const int r = blockIdx.x;
    const int64_t row = row_idx ? row_idx[r] : r;
    float4* src = reinterpret_cast<float4*>(x + row * d);
    const int n4 = d / 4;
    float4 v[MAXV];
    float ss = 0.f;
    // the gain is fetched up front: its cache round trip overlaps with the row loads and the reduction
    uint2 g16[sizeof(T) == 2 ? MAXV : 1];
    if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int k = 0; k < MAXV; ++k) {
            const int i = threadIdx.x + k * 256;
            g16[k] = i < n4 ? reinterpret_cast<const uint2*>(gain)[i] : make_uint2(0u, 0u);
        }
    }
#pragma unroll
    for (int k = 0; k < MAXV; ++k) {
        const int i = threadIdx.x + k * 256;
        v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < n4) {
            v[k] = src[i];
            float4 p[SKINNY_MAX_SPLITS];
#pragma unroll
            for (int s = 0; s < SKINNY_MAX_SPLITS; ++s)
                if (n_splits > 1 && s < n_splits) p[s] = reinterpret_cast<const float4*>(partials + s * split_stride + row * d)[i];
#pragma unroll
            for (int s = 0; s < SKINNY_MAX_SPLITS; ++s)
                if (n_splits > 1 && s < n_splits) { v[k].x += p[s].x; v[k].y += p[s].y; v[k].z += p[s].z; v[k].w += p[s].w; }
            if (n_splits > 1 && !row_idx) src[i] = v[k];
            ss += v[k].x * v[k].x + v[k].y * v[k].y + v[k].z * v[k].z + v[k].w * v[k].w;
        }
    }
    ss = group_allreduce<64>(ss, OpSum());
    if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = ss;
    __syncthreads();
    ss = (red[0] + red[1]) + (red[2] + red[3]);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    T* dst = out + (int64_t)r * d;
    float peak = 0.f;
    auto store_row = [&](auto clamp_c) {
        constexpr bool CLAMP = decltype(clamp_c)::value;
#pragma unroll
        for (int k = 0; k < MAXV; ++k) {
            const int i = threadIdx.x + k * 256;
            if (i >= n4) continue;
            if constexpr (sizeof(T) == 2) {
                const uint2 g = g16[k];
                uint2 o;
                o.x = op_store2<BF, CLAMP>(v[k].x * inv * bf16_lo(g.x), v[k].y * inv * bf16_hi(g.x), peak);
                o.y = op_store2<BF, CLAMP>(v[k].z * inv * bf16_lo(g.y), v[k].w * inv * bf16_hi(g.y), peak);
                reinterpret_cast<uint2*>(dst)[i] = o;
            } else {
                const float4 g = reinterpret_cast<const float4*>(gain)[i];
                reinterpret_cast<float4*>(dst)[i] = make_float4(v[k].x * inv * g.x, v[k].y * inv * g.y, v[k].z * inv * g.z, v[k].w * inv * g.w);
            }
        }
    };
    store_row(std::false_type());
    if (!(peak <= F16_MAX)) {
        store_row(std::true_type());
        raise_flag(flags, SSD_FLAG_ACT_OVERFLOW);
    }
}

void launch_rmsnorm(int dtype, float* x, const void* gain, const int32_t* row_idx, int n_rows, int d, float eps,
                    void* out, const float* partials, int n_splits, int64_t split_stride, int32_t* flags, bool bf16_ops,
                    hipStream_t st) {
    if (n_rows <= 0) return;
    if (n_rows <= 512 && d <= 4096 && n_splits <= SKINNY_MAX_SPLITS) {
#define SSD_RMSNORM_ROW(T, BF) \
        hipLaunchKernelGGL((rmsnorm_row_kernel<T, 4, BF>), dim3(n_rows), dim3(256), 0, st, x, (const T*)gain, row_idx, d, eps, (T*)out, partials, n_splits, split_stride, flags)
        if (dtype == SSD_BF16) { if (bf16_ops) SSD_RMSNORM_ROW(bf16_t, true); else SSD_RMSNORM_ROW(bf16_t, false); }
        else SSD_RMSNORM_ROW(float, false);
#undef SSD_RMSNORM_ROW
        return;
    }
    const dim3 grid((unsigned)((n_rows + 3) / 4)), block(256);
#define SSD_RMSNORM(T, NV, BF) \
    hipLaunchKernelGGL((rmsnorm_kernel<T, NV, BF>), grid, block, 0, st, x, (const T*)gain, row_idx, n_rows, d, eps, (T*)out, partials, n_splits, split_stride, flags)
#define SSD_RMSNORM_OP(NV) do { if (bf16_ops) SSD_RMSNORM(bf16_t, NV, true); else SSD_RMSNORM(bf16_t, NV, false); } while (0)
    if (dtype == SSD_BF16) {
        if (d <= 2048) SSD_RMSNORM_OP(8);
        else if (d <= 4096) SSD_RMSNORM_OP(16);
        else SSD_RMSNORM_OP(32);               // d_model <= 8192 is checked at context creation
    } else {
        SSD_RMSNORM(float, 4, false);          // fp32 models have d_model <= 1024
    }
#undef SSD_RMSNORM_OP
#undef SSD_RMSNORM
}

// ---------------------------------------------------------------------------------------------
// Weight re-layout (once, at context creation).
//
// bf16 weights become f16 MFMA operands: w * scale with scale a power of two chosen from the
// tensor's largest magnitude, so that bf16 values (8 significant bits) within 31 binades of it are
// represented exactly.  A scale of 0 keeps the bf16 bit pattern (contexts with bfloat16 operands).
// fp32 weights are copied unchanged.
template <typename T> struct Packed;
// `lost` counts the values whose half representation differs from w * scale: a bf16 value keeps all its 8
// significant bits only within 31 binades below the largest magnitude of its tensor (which lands just below
// 2^14, against the smallest half subnormal 2^-24); smaller ones are rounded to the subnormal grid.
template <> struct Packed<float> { typedef float type; static __device__ __forceinline__ float cvt(float v, float, unsigned& lost) { return v; } };
template <> struct Packed<bf16_t> {
    typedef f16_t type;
    static __device__ __forceinline__ f16_t cvt(bf16_t v, float scale, unsigned& lost) {
        if (scale <= 0.f) return v;                          // bfloat16 operands: the stored pattern is the operand
        const float t = bf16_to_f32(v) * scale;
        const f16_t h = f32_to_f16(t);
        lost += (f16_to_f32(h) != t) ? 1u : 0u;
        return h;
    }
};
// one atomic per wavefront that lost something (at context creation only)
__device__ __forceinline__ void add_lost(unsigned lost, unsigned long long* counter) {
    lost = (unsigned)group_allreduce_i<64>((int)lost, [] __device__(int a, int b) { return a + b; });
    if (counter && lost && threadIdx.x % 64 == 0) atomicAdd(counter, (unsigned long long)lost);
}

template <typename T>
__global__ void absmax_kernel(const T* __restrict__ w, int64_t n, unsigned int* __restrict__ out) {
    float m = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        float v;
        if constexpr (sizeof(T) == 2) v = bf16_to_f32(w[i]); else v = w[i];
        m = fmaxf(m, fabsf(v));
    }
    m = group_allreduce<64>(m, OpMax());
    if (threadIdx.x % 64 == 0) atomicMax(out, __float_as_uint(m));      // non-negative floats order like their bits
}

void launch_absmax(int dtype, const void* w, int64_t n, unsigned int* out, hipStream_t st) {
    const unsigned grid = (unsigned)std::min<int64_t>((n + 255) / 256, 2048);
    if (dtype == SSD_BF16) hipLaunchKernelGGL(absmax_kernel<bf16_t>, dim3(grid), dim3(256), 0, st, (const bf16_t*)w, n, out);
    else hipLaunchKernelGGL(absmax_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)w, n, out);
}

template <typename T>
__global__ void convert_rows_kernel(const T* __restrict__ w, typename Packed<T>::type* __restrict__ out, int cols, float scale,
                                    unsigned long long* __restrict__ inexact) {
    const T* src = w + (int64_t)blockIdx.x * cols;
    typename Packed<T>::type* dst = out + (int64_t)blockIdx.x * cols;
    unsigned lost = 0;
    for (int i = threadIdx.x; i < cols; i += blockDim.x) dst[i] = Packed<T>::cvt(src[i], scale, lost);
    add_lost(lost, inexact);
}

void launch_convert_weight(int dtype, const void* w, void* out, int rows, int cols, float scale, unsigned long long* inexact,
                           hipStream_t st) {
    if (dtype == SSD_BF16) hipLaunchKernelGGL(convert_rows_kernel<bf16_t>, dim3(rows), dim3(256), 0, st, (const bf16_t*)w, (f16_t*)out, cols, scale, inexact);
    else hipLaunchKernelGGL(convert_rows_kernel<float>, dim3(rows), dim3(256), 0, st, (const float*)w, (float*)out, cols, scale, inexact);
}
//
// Fused QKV: rows [q heads | k heads | v heads].  Inside every rotary head (q and k) rows are
// regrouped into blocks of 64 = [32 rows of the first half | their 32 rotation partners], so that
// the GEMM epilogue finds a column and its partner (i, i + head_dim/2) in the same lane of two
// neighbouring 32-wide accumulator blocks.  The f32 path keeps the natural order.
template <typename T>
__global__ void pack_qkv_kernel(const T* __restrict__ wq, const T* __restrict__ wk, const T* __restrict__ wv,
                                typename Packed<T>::type* __restrict__ out, int d_q, int d_kv, int d_model, int head_dim,
                                int permute, float scale, unsigned long long* __restrict__ inexact) {
    const int p = blockIdx.x;                       // packed row
    int orig = p;
    const int d_rot = d_q + d_kv;
    if (permute && p < d_rot) {
        const int half = head_dim / 2;
        const int head = p / head_dim, w = p % head_dim;
        const int grp = w / 64, in = w % 64;       // group of 64 packed rows inside the head
        const int blk = in / 32, o = in % 32;
        orig = head * head_dim + blk * half + grp * 32 + o;
    }
    const T* src = orig < d_q ? wq + (int64_t)orig * d_model
                 : orig < d_q + d_kv ? wk + (int64_t)(orig - d_q) * d_model
                 : wv + (int64_t)(orig - d_q - d_kv) * d_model;
    typename Packed<T>::type* dst = out + (int64_t)p * d_model;
    unsigned lost = 0;
    for (int i = threadIdx.x; i < d_model; i += blockDim.x) dst[i] = Packed<T>::cvt(src[i], scale, lost);
    add_lost(lost, inexact);
}

void launch_pack_qkv(int dtype, const void* wq, const void* wk, const void* wv, void* out, int d_q, int d_kv,
                     int d_model, int head_dim, float scale, unsigned long long* inexact, hipStream_t st) {
    const int rows = d_q + 2 * d_kv;
    if (dtype == SSD_BF16)
        hipLaunchKernelGGL(pack_qkv_kernel<bf16_t>, dim3(rows), dim3(256), 0, st, (const bf16_t*)wq, (const bf16_t*)wk,
                           (const bf16_t*)wv, (f16_t*)out, d_q, d_kv, d_model, head_dim, 1, scale, inexact);
    else
        hipLaunchKernelGGL(pack_qkv_kernel<float>, dim3(rows), dim3(256), 0, st, (const float*)wq, (const float*)wk,
                           (const float*)wv, (float*)out, d_q, d_kv, d_model, head_dim, 0, 1.0f, inexact);
}

// Fused gate/up: bf16 packs blocks of 64 rows = [32 gate rows | the same 32 up rows]; f32 packs
// [all gate rows | all up rows].
template <typename T>
__global__ void pack_gate_up_kernel(const T* __restrict__ wg, const T* __restrict__ wu,
                                    typename Packed<T>::type* __restrict__ out, int d_ff, int d_model, int interleave,
                                    float scale, unsigned long long* __restrict__ inexact) {
    const int p = blockIdx.x;
    const T* src;
    if (interleave) {
        const int grp = p / 64, in = p % 64;
        const int f = grp * 32 + in % 32;
        src = (in < 32 ? wg : wu) + (int64_t)f * d_model;
    } else {
        src = p < d_ff ? wg + (int64_t)p * d_model : wu + (int64_t)(p - d_ff) * d_model;
    }
    typename Packed<T>::type* dst = out + (int64_t)p * d_model;
    unsigned lost = 0;
    for (int i = threadIdx.x; i < d_model; i += blockDim.x) dst[i] = Packed<T>::cvt(src[i], scale, lost);
    add_lost(lost, inexact);
}

void launch_pack_gate_up(int dtype, const void* wg, const void* wu, void* out, int d_ff, int d_model, float scale,
                         unsigned long long* inexact, hipStream_t st) {
    if (dtype == SSD_BF16)
        hipLaunchKernelGGL(pack_gate_up_kernel<bf16_t>, dim3(2 * d_ff), dim3(256), 0, st, (const bf16_t*)wg,
                           (const bf16_t*)wu, (f16_t*)out, d_ff, d_model, 1, scale, inexact);
    else
        hipLaunchKernelGGL(pack_gate_up_kernel<float>, dim3(2 * d_ff), dim3(256), 0, st, (const float*)wg,
                           (const float*)wu, (float*)out, d_ff, d_model, 0, 1.0f, inexact);
}

// ---------------------------------------------------------------------------------------------
// Acceptance (Eq. 5 and the definition of j in Sec. 2.3): token i passes iff logp_i > ln(tau);
// accept_len = (index of the first failing token) - 1, or U when none fails.
// One wavefront per utterance.
__global__ void __launch_bounds__(64) accept_scan_kernel(const float* __restrict__ logp,
                                                         const int32_t* __restrict__ cu_draft, float ln_tau,
                                                         int32_t* __restrict__ accept_len,
                                                         uint8_t* __restrict__ all_accepted) {
    const int b = blockIdx.x;
    const int lo = cu_draft[b], hi = cu_draft[b + 1];
    const int U = hi - lo;
    int first_fail = U;                                  // 0-based index of the first failing token
    for (int i = threadIdx.x; i < U; i += 64) {
        if (!(logp[lo + i] > ln_tau)) { first_fail = i; break; }
    }
    first_fail = group_allreduce_i<64>(first_fail, OpMinI());
    if (threadIdx.x == 0) {
        accept_len[b] = first_fail;
        all_accepted[b] = first_fail == U ? 1 : 0;
    }
}

// Operating-point grids (Sec. 3.2): entropies and likelihoods do not depend on the thresholds, so the
// decisions for n thresholds are n applications of the single-threshold rule to the same numbers.
__global__ void __launch_bounds__(256) gate_grid_kernel(const float* __restrict__ max_entropy, int B,
                                                        const float* __restrict__ taus, int n_tau,
                                                        uint8_t* __restrict__ gate_pass) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= B * n_tau) return;
    gate_pass[i] = max_entropy[i % B] < taus[i / B] ? 1 : 0;
}

__global__ void __launch_bounds__(64) accept_grid_kernel(const float* __restrict__ logp, const int32_t* __restrict__ cu_draft,
                                                         int Bv, const float* __restrict__ ln_taus,
                                                         int32_t* __restrict__ accept_len, uint8_t* __restrict__ all_accepted) {
    const int b = blockIdx.x, a = blockIdx.y;
    const int lo = cu_draft[b], U = cu_draft[b + 1] - lo;
    const float ln_tau = ln_taus[a];
    int first_fail = U;
    for (int i = threadIdx.x; i < U; i += 64) {
        if (!(logp[lo + i] > ln_tau)) { first_fail = i; break; }
    }
    first_fail = group_allreduce_i<64>(first_fail, OpMinI());
    if (threadIdx.x == 0) {
        accept_len[a * Bv + b] = first_fail;
        all_accepted[a * Bv + b] = first_fail == U ? 1 : 0;
    }
}

void launch_gate_grid(const float* max_entropy, int B, const float* taus_dev, int n_tau, uint8_t* gate_pass, hipStream_t st) {
    hipLaunchKernelGGL(gate_grid_kernel, dim3((B * n_tau + 255) / 256), dim3(256), 0, st, max_entropy, B, taus_dev, n_tau, gate_pass);
}
void launch_accept_grid(const float* logp, const int32_t* cu_draft_dev, int Bv, const float* ln_taus_dev, int n_tau,
                        int32_t* accept_len, uint8_t* all_accepted, hipStream_t st) {
    hipLaunchKernelGGL(accept_grid_kernel, dim3(Bv, n_tau), dim3(64), 0, st, logp, cu_draft_dev, Bv, ln_taus_dev, accept_len, all_accepted);
}

void launch_accept_scan(const float* logp, const int32_t* cu_draft_dev, int Bv, float ln_tau, int32_t* accept_len,
                        uint8_t* all_accepted, hipStream_t st) {
    if (Bv <= 0) return;
    hipLaunchKernelGGL(accept_scan_kernel, dim3(Bv), dim3(64), 0, st, logp, cu_draft_dev, ln_tau, accept_len, all_accepted);
}

// ---------------------------------------------------------------------------------------------
// Measurement aid: what the matrix cores sustain on this device with nothing else going on.
// Every wavefront issues independent v_mfma_f32_16x16x32_f16 (the instruction of the big GEMMs, and the one
// that sustains the most flop/s under the power limit) on pseudo-random operands held in registers (no
// memory traffic in the loop), two wavefronts per SIMD; one wavefront also samples the shader clock
// against the 100 MHz constant clock.
typedef _Float16 peak_f16x8_t __attribute__((ext_vector_type(8)));
typedef float peak_f32x4_t __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(512) mfma_ceiling_kernel(float* __restrict__ sink, long long* __restrict__ clocks, int iters) {
    peak_f32x4_t acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[i][r] = 0.f;
    peak_f16x8_t a[8], b[2];
    unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) { h = h * 1664525u + 1013904223u; a[q][e] = (_Float16)(((h >> 8) & 0xffff) / 65536.0f - 0.5f); }
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) { h = h * 1664525u + 1013904223u; b[q][e] = (_Float16)(((h >> 8) & 0xffff) / 65536.0f - 0.5f); }
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i % 8], b[i / 8], acc[i], 0, 0, 0);
    }
    if (blockIdx.x == 3 && threadIdx.x == 0) { clocks[0] = clock64() - c0; clocks[1] = wall_clock64() - w0; }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) s += acc[i][r];
    sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// Streaming read of n 16-byte units, the access pattern that reads fastest on this chip: all wavefronts of the
// launch interleave 8 KB trips (eight 1 KB loads in flight per wavefront, consecutive wavefronts on consecutive
// trips) and the loads carry the non-temporal hint.  (Measured on 3 GiB: 7.0 TB/s; the same loop without the hint
// 6.2 TB/s, a contiguous share per workgroup 6.0 TB/s without and 6.6 TB/s with the hint.)  The values are folded
// into a word that is stored only if it has a particular value, so the loads cannot be dropped.
__global__ void __launch_bounds__(512) hbm_read_kernel(const uint4* __restrict__ p, int64_t n, uint32_t* __restrict__ sink) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4* q = reinterpret_cast<const u32x4*>(p);
    uint32_t acc = 0;
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int64_t gw = (int64_t)blockIdx.x * 8 + wave, nw = (int64_t)gridDim.x * 8;
    int64_t i = gw * 512 + lane;
    for (; i + 7 * 64 < n; i += nw * 512) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(q + i + u * 64);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (int u = 0; u < 8; ++u)
        if (i + u * 64 < n) { const u32x4 v = q[i + u * 64]; acc ^= v.x ^ v.y ^ v.z ^ v.w; }
    if (acc == 0x9e3779b9u) *sink = acc;
}
void launch_hbm_read(const void* buf, size_t bytes, uint32_t* sink, hipStream_t st) {
    hipLaunchKernelGGL(hbm_read_kernel, dim3(256), dim3(512), 0, st, static_cast<const uint4*>(buf), (int64_t)(bytes / 16), sink);
}

void launch_mfma_ceiling(float* sink, long long* clocks, int n_workgroups, int iters, hipStream_t st) {
    hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(n_workgroups), dim3(512), 0, st, sink, clocks, iters);
}

}  // namespace ssd
