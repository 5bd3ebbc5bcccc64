// Auto-regressive fallback (Sec. 2.3, Eq. 6): kernels that exist only for the token-by-token
// continuation from the accepted prefix -- storing keys/values of the verification pass into a
// cache, and attention of ONE new query row per utterance against its cached rows.
// Everything else of a decode step reuses the verification kernels on a batch of Br rows
// (RMSNorm, skinny weight-streaming GEMMs with split-K, LM head with argmax).
#include "device_utils.h"
#include "ssd_internal.h"

namespace ssd {

// ---------------------------------------------------------------------------------------------
// Copy the (rotated) K and V parts of qkv rows into the cache of one layer.
// qkv row layout: [q (d_q) | k (d_kv) | v (d_kv)]; cache: K [slots, d_kv], V [slots, d_kv].
template <typename T>
__global__ void __launch_bounds__(256) kv_store_kernel(const T* __restrict__ qkv, const int32_t* __restrict__ row_slot,
                                                       int d_q, int d_kv, T* __restrict__ kc, T* __restrict__ vc) {
    const int r = blockIdx.x;
    const int64_t slot = row_slot[r];
    if (slot < 0) return;
    const T* src = qkv + (int64_t)r * (d_q + 2 * d_kv) + d_q;
    constexpr int VEC = 16 / sizeof(T);
    const uint4* ks = reinterpret_cast<const uint4*>(src);
    const uint4* vs = reinterpret_cast<const uint4*>(src + d_kv);
    uint4* kd = reinterpret_cast<uint4*>(kc + slot * d_kv);
    uint4* vd = reinterpret_cast<uint4*>(vc + slot * d_kv);
    for (int i = threadIdx.x; i < d_kv / VEC; i += 256) { kd[i] = ks[i]; vd[i] = vs[i]; }
}

void launch_kv_store(int dtype, const void* qkv, const int32_t* row_slot, int n_rows, int d_q, int d_kv, void* kc,
                     void* vc, hipStream_t st) {
    if (n_rows <= 0) return;
    if (dtype == SSD_BF16)
        hipLaunchKernelGGL(kv_store_kernel<f16_t>, dim3(n_rows), dim3(256), 0, st, (const f16_t*)qkv, row_slot, d_q, d_kv, (f16_t*)kc, (f16_t*)vc);
    else
        hipLaunchKernelGGL(kv_store_kernel<float>, dim3(n_rows), dim3(256), 0, st, (const float*)qkv, row_slot, d_q, d_kv, (float*)kc, (float*)vc);
}

// ---------------------------------------------------------------------------------------------
// One query row per utterance: wavefront (b, head) attends to cache rows kv_start[b] .. +n_ctx[b]-1
// (the last of which is the row of the query token itself, stored just before).
// Keys are processed 64 at a time with an online softmax; lanes own keys for the scores and own
// output dimensions for P.V.  head_dim <= 128, multiple of 8.
template <typename T> __device__ __forceinline__ float elem_to_f32(T v);
template <> __device__ __forceinline__ float elem_to_f32<float>(float v) { return v; }
template <typename T> __device__ __forceinline__ T f32_to_elem(float v);
template <> __device__ __forceinline__ float f32_to_elem<float>(float v) { return v; }

// eight consecutive elements as fp32
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
    const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
// eight 16-bit operand patterns (IEEE half or bfloat16) as fp32
template <bool BF>
__device__ __forceinline__ void unpack8(const uint4& w, float (&v)[8]) {
    if constexpr (BF) {
        v[0] = bf16_lo(w.x); v[1] = bf16_hi(w.x); v[2] = bf16_lo(w.y); v[3] = bf16_hi(w.y);
        v[4] = bf16_lo(w.z); v[5] = bf16_hi(w.z); v[6] = bf16_lo(w.w); v[7] = bf16_hi(w.w);
    } else {
        typedef _Float16 h8 __attribute__((ext_vector_type(8)));
        const h8 a = __builtin_bit_cast(h8, w);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (float)a[e];
    }
}

template <typename T>
__global__ void __launch_bounds__(64) decode_attn_kernel(const T* __restrict__ qkv, const T* __restrict__ kc,
                                                         const T* __restrict__ vc, const int32_t* __restrict__ kv_start,
                                                         const int32_t* __restrict__ n_ctx, int n_q_heads, int n_kv_heads,
                                                         int head_dim, T* __restrict__ out) {
    __shared__ float q_s[128];
    __shared__ float p_s[64];
    const int lane = threadIdx.x;
    const int b = blockIdx.x, h = blockIdx.y;
    const int kvh = h / (n_q_heads / n_kv_heads);
    const int d_q = n_q_heads * head_dim, d_kv = n_kv_heads * head_dim;
    const T* q = qkv + (int64_t)b * (d_q + 2 * d_kv) + h * head_dim;
    for (int i = lane; i < head_dim; i += 64) q_s[i] = elem_to_f32<T>(q[i]);
    __builtin_amdgcn_wave_barrier();
    const int n = n_ctx[b];
    const T* kbase = kc + (int64_t)kv_start[b] * d_kv + kvh * head_dim;
    const T* vbase = vc + (int64_t)kv_start[b] * d_kv + kvh * head_dim;
    const float scale = 1.0f / sqrtf((float)head_dim);
    // P.V: lane = (key group kg of 4, chunk dc of 8 output dims)
    const int kg = lane / 16, dc = lane % 16;
    const bool dims_live = dc * 8 < head_dim;
    float m = -INFINITY, l = 0.f, o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < n; k0 += 64) {
        const int key = k0 + lane;
        float s = -INFINITY;
        if (key < n) {
            const T* kr = kbase + (int64_t)key * d_kv;
            float acc = 0.f;
            for (int i = 0; i < head_dim; i += 8) {
                float kv8[8];
                load8(kr + i, kv8);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc = fmaf(q_s[i + e], kv8[e], acc);
            }
            s = acc * scale;
        }
        const float m_new = fmaxf(m, group_allreduce<64>(s, OpMax()));
        const float p = expf(s - m_new);
        const float alpha = expf(m - m_new);
        l = l * alpha + group_allreduce<64>(p, OpSum());
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= alpha;
        p_s[lane] = p;
        __builtin_amdgcn_wave_barrier();
        const int n_keys = min(64, n - k0);
        if (dims_live) {
            for (int j = kg; j < n_keys; j += 4) {
                const float pj = p_s[j];
                float v8[8];
                load8(vbase + (int64_t)(k0 + j) * d_kv + dc * 8, v8);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = fmaf(pj, v8[e], o[e]);
            }
        }
        __builtin_amdgcn_wave_barrier();
        m = m_new;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        o[e] += __shfl_xor(o[e], 16);
        o[e] += __shfl_xor(o[e], 32);
    }
    if (kg == 0 && dims_live) {
        T* dst = out + (int64_t)b * d_q + h * head_dim + dc * 8;
        const float inv = 1.0f / l;
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[e] = f32_to_elem<T>(o[e] * inv);
    }
}

// head_dim 128 in half precision: lane = (key group kg of 4, chunk dc of 8 dims).  A block of 64 keys
// is 16 loads of K and 16 of V per lane, all issued before the first use (the rows are 256 bytes, a
// 16-lane group reads one row); a score is a 16-lane reduction, the softmax statistics are reduced over
// the four key groups, and P.V accumulates in the lane, reduced over the key groups at the end.
// A workgroup is DEC_WAVES wavefronts that take the 64-key blocks of one (utterance, head) in turn and
// merge their (max, sum, output) triples through LDS: the blocks of a context are then loaded at
// once instead of one after the other.
constexpr int DEC_WAVES = 4;

// Fused variant: the QKV projection of the step has been left as K-split partial sums
// part[split][row][packed column] (fp32, packed column order of the fused QKV weight: inside a head the
// rotary pairs (i, i+64) sit 32 columns apart in 64-column groups, V columns are in natural order).
// The kernel adds the splits, rotates q and the new k, appends the new k / v row to the cache (first query
// head of each K/V group) and treats that row as the last key without reading it back.
// a value as the cache / the next kernel will see it: rounded to the operand type, saturated for IEEE half
template <bool BF> __device__ __forceinline__ float round_like_stored(float v, bool& bad) {
    if constexpr (BF) return bf16_to_f32(f32_to_bf16(v));
    else return f16_to_f32(f32_to_f16_sat(v, bad));
}
template <bool BF> __device__ __forceinline__ uint32_t pack2_sat(float lo, float hi, bool& bad) {
    if constexpr (BF) return pack_bf16x2(lo, hi);
    else return pack_f16x2_sat(lo, hi, bad);
}

struct DecodeFused {
    const float* part; int n_splits; int64_t split_stride;    // split_stride = rows * (d_q + 2 d_kv)
    const float2* rope_tab;                                   // [position][64] (cos, sin)
    f16_t* kc_w; f16_t* vc_w;                                 // writable views of the cache
    int32_t* flags;                                           // sticky device flags (SSD_FLAG_ACT_OVERFLOW on a saturated store)
    // The new row's position is the number of rows its utterance has in the cache (cache row i of an
    // utterance is position i), and its slot is kv_start + that number: no further index arrays.
};
// sum over the splits (at most 8) of eight consecutive packed columns starting at `col` of row b; the loads
// of four splits are issued together
__device__ __forceinline__ void sum_splits8(const DecodeFused& f, int64_t row_off, int col, float (&v)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = 0.f;
#pragma unroll 1
    for (int s0 = 0; s0 < f.n_splits; s0 += 4) {
        float4 t[4][2];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const float4* src = reinterpret_cast<const float4*>(f.part + (s0 + s < f.n_splits ? s0 + s : 0) * f.split_stride + row_off + col);
            t[s][0] = src[0];
            t[s][1] = src[1];
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s0 + s < f.n_splits) {
                v[0] += t[s][0].x; v[1] += t[s][0].y; v[2] += t[s][0].z; v[3] += t[s][0].w;
                v[4] += t[s][1].x; v[5] += t[s][1].y; v[6] += t[s][1].z; v[7] += t[s][1].w;
            }
        }
    }
}
// the eight (cos, sin) pairs a lane needs at position p: dims (dc % 8) * 8 .. + 7 of the first half of a head
__device__ __forceinline__ void rope_entries(const DecodeFused& f, int dc, int p, float2 (&cs)[8]) {
    const int i0 = (dc % 8) * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) cs[e] = f.rope_tab[(int64_t)p * 64 + i0 + e];
}
// dims 8 dc .. 8 dc + 7 of rotated head `head_col0` (packed column of the head's first dim); cs from rope_entries,
// requested before the partial sums so that its round trip overlaps theirs
__device__ __forceinline__ void rotated_chunk(const DecodeFused& f, int64_t row_off, int head_col0, int dc, const float2 (&cs)[8], float (&v)[8]) {
    const int i0 = (dc % 8) * 8;                              // dim inside the first half of the head
    const int col_lo = head_col0 + (i0 / 32) * 64 + (i0 % 32);
    float lo[8], hi[8];
    sum_splits8(f, row_off, col_lo, lo);
    sum_splits8(f, row_off, col_lo + 32, hi);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = dc < 8 ? lo[e] * cs[e].x - hi[e] * cs[e].y : hi[e] * cs[e].x + lo[e] * cs[e].y;
}

template <bool FUSED, bool BF>
__global__ void __launch_bounds__(64 * DEC_WAVES) decode_attn_hd128_kernel(const f16_t* __restrict__ qkv, const f16_t* __restrict__ kc,
                                                               const f16_t* __restrict__ vc, const int32_t* __restrict__ kv_start,
                                                               const int32_t* __restrict__ n_ctx, int n_q_heads, int n_kv_heads,
                                                               f16_t* __restrict__ out, DecodeFused fu) {
    constexpr int HD = 128;
    __shared__ float merge_o[DEC_WAVES][16][8];
    __shared__ float merge_ml[DEC_WAVES][2];
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64, kg = lane / 16, dc = lane % 16;
    const int b = blockIdx.x, h = blockIdx.y;
    const int kvh = h / (n_q_heads / n_kv_heads);
    const int d_q = n_q_heads * HD, d_kv = n_kv_heads * HD;
    const float sc = 0.08838834764831845f * 1.4426950408889634f;      // log2(e) / sqrt(128)
    float qf[8];
    float m = -INFINITY, l = 0.f, o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const int n = n_ctx[b] - (FUSED ? 1 : 0);                // rows to read from the cache
    const f16_t* kbase = kc + (int64_t)kv_start[b] * d_kv + kvh * HD + dc * 8;
    const f16_t* vbase = vc + (int64_t)kv_start[b] * d_kv + kvh * HD + dc * 8;
    uint4 kr[16], vr[16];
    auto load_block = [&](int k0) {
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int key = min(k0 + it * 4 + kg, n - 1);
            kr[it] = *reinterpret_cast<const uint4*>(kbase + (int64_t)key * d_kv);
        }
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int key = min(k0 + it * 4 + kg, n - 1);
            vr[it] = *reinterpret_cast<const uint4*>(vbase + (int64_t)key * d_kv);
        }
    };
    // the first block of keys and values is requested before q is put together
    if (wave * 64 < n) load_block(wave * 64);
    if constexpr (FUSED) {
        // Key group 0 of every wavefront builds q (wavefront 0 also the new k / v row) and hands it to the
        // other key groups: the partial sums are read once per wavefront, not once per lane.
        const int64_t row_off = (int64_t)b * (d_q + 2 * d_kv);
        const int p = n;                                     // position of the new token
        float s_new = 0.f;
        bool bad = false;
        uint4 vw = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[e] = 0.f;
        if (kg == 0) {
            float2 cs[8];                                    // the same entries rotate q and the new k
            rope_entries(fu, dc, p, cs);
            rotated_chunk(fu, row_off, h * HD, dc, cs, qf);
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[e] = round_like_stored<BF>(qf[e], bad) * sc;      // q is rounded (and saturated) like a stored row
            if (wave == 0) {
                float kn[8], vn[8];
                rotated_chunk(fu, row_off, d_q + kvh * HD, dc, cs, kn);
                sum_splits8(fu, row_off, d_q + d_kv + kvh * HD + dc * 8, vn);
                // the cache holds half precision: the new row takes part in this step with the values later steps read
                uint4 kw;
                kw.x = pack2_sat<BF>(kn[0], kn[1], bad); kw.y = pack2_sat<BF>(kn[2], kn[3], bad); kw.z = pack2_sat<BF>(kn[4], kn[5], bad); kw.w = pack2_sat<BF>(kn[6], kn[7], bad);
                vw.x = pack2_sat<BF>(vn[0], vn[1], bad); vw.y = pack2_sat<BF>(vn[2], vn[3], bad); vw.z = pack2_sat<BF>(vn[4], vn[5], bad); vw.w = pack2_sat<BF>(vn[6], vn[7], bad);
                if (h % (n_q_heads / n_kv_heads) == 0) {
                    const int64_t so = ((int64_t)kv_start[b] + n) * d_kv + kvh * HD + dc * 8;
                    *reinterpret_cast<uint4*>(fu.kc_w + so) = kw;
                    *reinterpret_cast<uint4*>(fu.vc_w + so) = vw;
                }
                float kh[8];
                unpack8<BF>(kw, kh);
#pragma unroll
                for (int e = 0; e < 8; ++e) s_new = fmaf(qf[e], kh[e], s_new);
            }
        }
        if (bad) raise_flag(fu.flags, SSD_FLAG_ACT_OVERFLOW);
        s_new = group_allreduce<16>(s_new, OpSum());          // lanes 0..15 hold the score of the new row
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[e] = __shfl(qf[e], dc);
        s_new = __shfl(s_new, 0);
        if (wave == 0) {                                     // the new row is wavefront 0's first key
            m = s_new; l = 1.f;
            if (kg == 0) {
                unpack8<BF>(vw, o);
            }
        }
    } else {
        unpack8<BF>(*reinterpret_cast<const uint4*>(qkv + (int64_t)b * (d_q + 2 * d_kv) + h * HD + dc * 8), qf);
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[e] *= sc;
    }
    for (int k0 = wave * 64; k0 < n; k0 += 64 * DEC_WAVES) {
        float s[16];
        float cm = -INFINITY;
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            float kk[8];
            unpack8<BF>(kr[it], kk);
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = fmaf(qf[e], kk[e], acc);
            acc = group_allreduce<16>(acc, OpSum());
            s[it] = (k0 + it * 4 + kg < n) ? acc : -INFINITY;
            cm = fmaxf(cm, s[it]);
        }
        cm = fmaxf(cm, __shfl_xor(cm, 16));
        cm = fmaxf(cm, __shfl_xor(cm, 32));
        const float m_new = fmaxf(m, cm);                 // finite: key k0 exists
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= alpha;
        float ps = 0.f;
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const float p = __builtin_amdgcn_exp2f(s[it] - m_new);
            ps += p;
            float vv[8];
            unpack8<BF>(vr[it], vv);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = fmaf(p, vv[e], o[e]);
        }
        ps += __shfl_xor(ps, 16);
        ps += __shfl_xor(ps, 32);
        l = l * alpha + ps;
        m = m_new;
        if (k0 + 64 * DEC_WAVES < n) load_block(k0 + 64 * DEC_WAVES);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        o[e] += __shfl_xor(o[e], 16);
        o[e] += __shfl_xor(o[e], 32);
    }
    // merge the wavefronts: wave w's partial is (m, l, o) with o scaled by 2^-m; a wavefront without a block has l = 0
    if (kg == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) merge_o[wave][dc][e] = o[e];
        if (dc == 0) { merge_ml[wave][0] = m; merge_ml[wave][1] = l; }
    }
    __syncthreads();
    if (wave == 0 && kg == 0) {
        float mt = -INFINITY;
#pragma unroll
        for (int w = 0; w < DEC_WAVES; ++w) mt = fmaxf(mt, merge_ml[w][0]);     // finite: wave 0 saw key 0
        l = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
        for (int w = 0; w < DEC_WAVES; ++w) {
            const float lw = merge_ml[w][1];
            const float f = lw > 0.f ? __builtin_amdgcn_exp2f(merge_ml[w][0] - mt) : 0.f;
            l = fmaf(lw, f, l);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = fmaf(merge_o[w][dc][e], f, o[e]);
        }
        const float inv = 1.0f / l;
        uint4 w;
        w.x = op_pack2<BF>(o[0] * inv, o[1] * inv); w.y = op_pack2<BF>(o[2] * inv, o[3] * inv);
        w.z = op_pack2<BF>(o[4] * inv, o[5] * inv); w.w = op_pack2<BF>(o[6] * inv, o[7] * inv);
        *reinterpret_cast<uint4*>(out + (int64_t)b * d_q + h * HD + dc * 8) = w;
    }
}

void launch_decode_attn(int dtype, const void* qkv, const void* kc, const void* vc, const int32_t* kv_start,
                        const int32_t* n_ctx, int Br, int n_q_heads, int n_kv_heads, int head_dim, void* out,
                        bool bf16_ops, hipStream_t st) {
    if (Br <= 0) return;
    if (dtype == SSD_BF16) {                                 // 16-bit models always have head_dim 128
        if (bf16_ops)
            hipLaunchKernelGGL((decode_attn_hd128_kernel<false, true>), dim3(Br, n_q_heads), dim3(64 * DEC_WAVES), 0, st, (const f16_t*)qkv, (const f16_t*)kc,
                               (const f16_t*)vc, kv_start, n_ctx, n_q_heads, n_kv_heads, (f16_t*)out, DecodeFused{});
        else
            hipLaunchKernelGGL((decode_attn_hd128_kernel<false, false>), dim3(Br, n_q_heads), dim3(64 * DEC_WAVES), 0, st, (const f16_t*)qkv, (const f16_t*)kc,
                               (const f16_t*)vc, kv_start, n_ctx, n_q_heads, n_kv_heads, (f16_t*)out, DecodeFused{});
    } else {
        hipLaunchKernelGGL(decode_attn_kernel<float>, dim3(Br, n_q_heads), dim3(64), 0, st, (const float*)qkv, (const float*)kc,
                           (const float*)vc, kv_start, n_ctx, n_q_heads, n_kv_heads, head_dim, (float*)out);
    }
}

void launch_decode_attn_fused(const float* qkv_part, int n_splits, const float* rope_tab, void* kc, void* vc,
                              const int32_t* kv_start, const int32_t* n_ctx, int Br, int n_q_heads, int n_kv_heads,
                              void* out, int32_t* flags, bool bf16_ops, hipStream_t st) {
    if (Br <= 0) return;
    const int64_t stride = (int64_t)Br * (n_q_heads + 2 * n_kv_heads) * 128;
    DecodeFused fu{qkv_part, n_splits, stride, reinterpret_cast<const float2*>(rope_tab), (f16_t*)kc, (f16_t*)vc, flags};
    if (bf16_ops)
        hipLaunchKernelGGL((decode_attn_hd128_kernel<true, true>), dim3(Br, n_q_heads), dim3(64 * DEC_WAVES), 0, st, nullptr, (const f16_t*)kc,
                           (const f16_t*)vc, kv_start, n_ctx, n_q_heads, n_kv_heads, (f16_t*)out, fu);
    else
        hipLaunchKernelGGL((decode_attn_hd128_kernel<true, false>), dim3(Br, n_q_heads), dim3(64 * DEC_WAVES), 0, st, nullptr, (const f16_t*)kc,
                           (const f16_t*)vc, kv_start, n_ctx, n_q_heads, n_kv_heads, (f16_t*)out, fu);
}

}  // namespace ssd
