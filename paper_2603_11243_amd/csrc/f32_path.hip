// All-fp32 decoder kernels (used when the model dtype is SSD_F32, i.e. the small validation
// configuration).  Plain, LDS-tiled vector-ALU code: these shapes are tiny and launch-bound, the
// purpose of this path is a tight (1e-4) comparison with the float64 oracle.
#include "device_utils.h"
#include "ssd_internal.h"

namespace ssd {

// C[M,N] (+)= A[M,K] * W[N,K]^T.  64x64 tile, 256 threads, 4x4 outputs per thread, BK = 16.
// K must be a multiple of 16; M and N are arbitrary.
template <int EPI>
__global__ void __launch_bounds__(256) gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W,
                                                       float* __restrict__ C, int M, int N, int K) {
    __shared__ float As[16][64 + 4];
    __shared__ float Ws[16][64 + 4];
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int lr = threadIdx.x / 4, lk = (threadIdx.x % 4) * 4;     // loader: row in tile, k offset
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        {
            const int ar = min(m0 + lr, M - 1), wr = min(n0 + lr, N - 1);
            const float4 a = *reinterpret_cast<const float4*>(A + (int64_t)ar * K + k0 + lk);
            const float4 w = *reinterpret_cast<const float4*>(W + (int64_t)wr * K + k0 + lk);
            As[lk + 0][lr] = a.x; As[lk + 1][lr] = a.y; As[lk + 2][lr] = a.z; As[lk + 3][lr] = a.w;
            Ws[lk + 0][lr] = w.x; Ws[lk + 1][lr] = w.y; Ws[lk + 2][lr] = w.z; Ws[lk + 3][lr] = w.w;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; w[i] = Ws[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = m0 + ty * 4 + i;
        if (r >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = n0 + tx * 4 + j;
            if (c >= N) continue;
            float* p = C + (int64_t)r * N + c;
            if (EPI == F32_ADD) *p += acc[i][j]; else *p = acc[i][j];
        }
    }
}

void launch_gemm_f32(const float* A, const float* W, float* C, int M, int N, int K, int epilogue, hipStream_t st) {
    if (M <= 0 || N <= 0) return;
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    if (epilogue == F32_ADD) hipLaunchKernelGGL(gemm_f32_kernel<F32_ADD>, grid, dim3(256), 0, st, A, W, C, M, N, K);
    else hipLaunchKernelGGL(gemm_f32_kernel<F32_STORE>, grid, dim3(256), 0, st, A, W, C, M, N, K);
}

// Rotary embedding in place on the first n_heads_rot heads of every row of qkv
// (row layout [q heads | k heads | v heads], row_stride floats per row).
// rope_tab[pos][i] = (cos, sin) of pos * theta^(-2i/head_dim).
__global__ void __launch_bounds__(256) rope_f32_kernel(float* __restrict__ qkv, const int32_t* __restrict__ pos,
                                                       const float2* __restrict__ rope_tab, int M, int n_heads_rot,
                                                       int head_dim, int row_stride) {
    const int half = head_dim / 2;
    const int64_t total = (int64_t)M * n_heads_rot * half;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int i = (int)(idx % half);
    const int h = (int)((idx / half) % n_heads_rot);
    const int r = (int)(idx / ((int64_t)half * n_heads_rot));
    const float2 cs = rope_tab[(int64_t)pos[r] * half + i];
    float* p = qkv + (int64_t)r * row_stride + h * head_dim + i;
    const float a = p[0], b = p[half];
    p[0] = a * cs.x - b * cs.y;
    p[half] = b * cs.x + a * cs.y;
}

void launch_rope_f32(float* qkv, const int32_t* pos, const float* rope_tab, int M, int n_heads_rot, int head_dim,
                     int row_stride, hipStream_t st) {
    const int64_t total = (int64_t)M * n_heads_rot * (head_dim / 2);
    if (total <= 0) return;
    hipLaunchKernelGGL(rope_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, qkv, pos,
                       (const float2*)rope_tab, M, n_heads_rot, head_dim, row_stride);
}

// h = silu(gate) * up, gu rows are [gate (d_ff) | up (d_ff)].
__global__ void __launch_bounds__(256) swiglu_f32_kernel(const float* __restrict__ gu, float* __restrict__ h, int M,
                                                         int d_ff) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)M * d_ff) return;
    const int64_t r = idx / d_ff;
    const int c = (int)(idx % d_ff);
    const float g = gu[r * 2 * d_ff + c], u = gu[r * 2 * d_ff + d_ff + c];
    h[idx] = g / (1.0f + expf(-g)) * u;
}

void launch_swiglu_f32(const float* gu, float* h, int M, int d_ff, hipStream_t st) {
    const int64_t total = (int64_t)M * d_ff;
    if (total <= 0) return;
    hipLaunchKernelGGL(swiglu_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, gu, h, M, d_ff);
}

// Causal attention, one wavefront per (query row, query head).  Keys are processed 64 at a time
// with an online softmax; lanes own keys for the scores and own output dimensions for P.V.
// qkv rows: [q heads | k heads | v heads]; head_dim <= 128 and a multiple of 4.
__global__ void __launch_bounds__(256) attn_f32_kernel(const float* __restrict__ qkv, float* __restrict__ out,
                                                       const AttnTile* __restrict__ tiles, int n_q_heads,
                                                       int n_kv_heads, int head_dim) {
    __shared__ float q_s[4][128];
    __shared__ float p_s[4][64];
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const AttnTile t = tiles[blockIdx.x];
    const int h = blockIdx.y;
    const int kvh = h / (n_q_heads / n_kv_heads);
    const int d_q = n_q_heads * head_dim, d_kv = n_kv_heads * head_dim;
    const int stride = d_q + 2 * d_kv;
    const int qpos = t.q_start + wave;
    const bool live = qpos < t.seq_len;
    const float scale = 1.0f / sqrtf((float)head_dim);
    if (live) {
        const float* q = qkv + (int64_t)(t.seq_start + qpos) * stride + h * head_dim;
        for (int i = lane; i < head_dim; i += 64) q_s[wave][i] = q[i];
    }
    __syncthreads();
    if (!live) return;
    float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
    const float* kbase = qkv + (int64_t)t.seq_start * stride + d_q + kvh * head_dim;
    const float* vbase = kbase + d_kv;
    for (int k0 = 0; k0 <= qpos; k0 += 64) {
        const int key = k0 + lane;
        float s = -INFINITY;
        if (key <= qpos) {
            const float4* kr = reinterpret_cast<const float4*>(kbase + (int64_t)key * stride);
            float acc = 0.f;
            for (int i = 0; i < head_dim / 4; ++i) {
                const float4 kv = kr[i];
                acc += q_s[wave][4 * i] * kv.x + q_s[wave][4 * i + 1] * kv.y + q_s[wave][4 * i + 2] * kv.z +
                       q_s[wave][4 * i + 3] * kv.w;
            }
            s = acc * scale;
        }
        const float m_new = fmaxf(m, group_allreduce<64>(s, OpMax()));
        const float p = expf(s - m_new);                       // 0 for masked lanes
        const float alpha = expf(m - m_new);                   // 0 on the first chunk (m = -inf)
        l = l * alpha + group_allreduce<64>(p, OpSum());
        o0 *= alpha; o1 *= alpha;
        p_s[wave][lane] = p;
        __builtin_amdgcn_wave_barrier();
        const int n_keys = min(64, qpos - k0 + 1);
        for (int j = 0; j < n_keys; ++j) {
            const float pj = p_s[wave][j];
            const float* vr = vbase + (int64_t)(k0 + j) * stride;
            if (lane < head_dim) o0 = fmaf(pj, vr[lane], o0);
            if (lane + 64 < head_dim) o1 = fmaf(pj, vr[lane + 64], o1);
        }
        __builtin_amdgcn_wave_barrier();
        m = m_new;
    }
    float* o = out + (int64_t)(t.seq_start + qpos) * d_q + h * head_dim;
    if (lane < head_dim) o[lane] = o0 / l;
    if (lane + 64 < head_dim) o[lane + 64] = o1 / l;
}

void launch_attn_f32(const float* qkv, float* out, const AttnTile* tiles, int n_tiles, int n_q_heads, int n_kv_heads,
                     int head_dim, hipStream_t st) {
    if (n_tiles <= 0) return;
    hipLaunchKernelGGL(attn_f32_kernel, dim3(n_tiles, n_q_heads), dim3(256), 0, st, qkv, out, tiles, n_q_heads,
                       n_kv_heads, head_dim);
}

// LM head + log-softmax + target gather (Eq. 5's likelihood), one workgroup per verification row.
// Each wavefront walks vocabulary rows v = wave, wave+4, ...; lanes split the d-long dot product.
// The logits only ever live in registers.  d <= 64*16.
__global__ void __launch_bounds__(256) lmhead_f32_kernel(const float* __restrict__ hv, const float* __restrict__ w_lm,
                                                         const int32_t* __restrict__ targets, int d, int vocab,
                                                         float* __restrict__ logp, int32_t* __restrict__ greedy) {
    __shared__ float red_m[4], red_s[4], red_t[4], red_best[4];
    __shared__ int red_arg[4];
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int r = blockIdx.x;
    int tgt = targets[r];
    tgt = tgt < 0 ? 0 : (tgt >= vocab ? vocab - 1 : tgt);
    float h[16];
    int nh = 0;
    for (int i = lane; i < d; i += 64) h[nh++] = hv[(int64_t)r * d + i];
    float m = -INFINITY, s = 0.f, tl = 0.f, best = -INFINITY;
    int arg = 0x7fffffff;
    for (int v = wave; v < vocab; v += 4) {
        const float* w = w_lm + (int64_t)v * d;
        float acc = 0.f;
        for (int j = 0; j < nh; ++j) acc = fmaf(h[j], w[lane + 64 * j], acc);
        acc = group_allreduce<64>(acc, OpSum());
        if (acc > m) { s = s * expf(m - acc) + 1.0f; m = acc; } else { s += expf(acc - m); }
        if (acc > best) { best = acc; arg = v; }
        if (v == tgt) tl = acc;
    }
    if (lane == 0) { red_m[wave] = m; red_s[wave] = s; red_t[wave] = tl; red_best[wave] = best; red_arg[wave] = arg; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float M = red_m[0];
        for (int w = 1; w < 4; ++w) M = fmaxf(M, red_m[w]);
        float S = 0.f;
        for (int w = 0; w < 4; ++w) S += red_s[w] * expf(red_m[w] - M);
        logp[r] = red_t[tgt % 4] - (M + logf(S));
        if (greedy) {
            float b = red_best[0]; int a = red_arg[0];
            for (int w = 1; w < 4; ++w)
                if (red_best[w] > b || (red_best[w] == b && red_arg[w] < a)) { b = red_best[w]; a = red_arg[w]; }
            greedy[r] = a;
        }
    }
}

void launch_lmhead_f32(const float* hv, const float* w_lm, const int32_t* targets, int Mv, int d, int vocab,
                       float* logp, int32_t* greedy, hipStream_t st) {
    if (Mv <= 0) return;
    hipLaunchKernelGGL(lmhead_f32_kernel, dim3(Mv), dim3(256), 0, st, hv, w_lm, targets, d, vocab, logp, greedy);
}

}  // namespace ssd
