// CTC gate (Sec. 2.1): frame entropy (Eq. 3), greedy alignment (Eq. 2), collapse map B, decision.
//
// Kernel 1 (gate_frames_*): one CTC frame per group of LPR lanes.  The whole row of scores is
// loaded once with 16-byte loads and kept in registers; the row maximum, the lowest index that
// attains it, sum exp(z-m) and sum exp(z-m)(z-m) are reduced inside the lane group.
//     H = log S - W / S,   S = sum_a exp(z_a - m),   W = sum_a exp(z_a - m) (z_a - m)
// which equals -sum_a p_a log p_a for p = softmax(z).  The kernel streams the logits exactly once
// and is bound by HBM bandwidth (co-limited by vector ALU issue for bf16 input).
//
// Kernel 2 (gate_utterances): one workgroup per utterance: max_t H_t, threshold test, and a
// stable compaction of the frames kept by B (not blank, and different from the previous frame).
#include "device_utils.h"
#include "ssd_internal.h"

namespace ssd {

template <typename T> struct Chunk;          // 16 bytes of scores
template <> struct Chunk<float> {
    static constexpr int N = 4;
    static constexpr uint32_t NEG_INF = 0xff800000u;
    static __device__ __forceinline__ void unpack(const uint4& c, float* z) {
        z[0] = __uint_as_float(c.x); z[1] = __uint_as_float(c.y);
        z[2] = __uint_as_float(c.z); z[3] = __uint_as_float(c.w);
    }
};
template <> struct Chunk<bf16_t> {
    static constexpr int N = 8;
    static constexpr uint32_t NEG_INF = 0xff80ff80u;
    static __device__ __forceinline__ void unpack(const uint4& c, float* z) {
        z[0] = bf16_lo(c.x); z[1] = bf16_hi(c.x); z[2] = bf16_lo(c.y); z[3] = bf16_hi(c.y);
        z[4] = bf16_lo(c.z); z[5] = bf16_hi(c.z); z[6] = bf16_lo(c.w); z[7] = bf16_hi(c.w);
    }
};

// Rows are V scores with V*sizeof(T) a multiple of 16; a row has n_chunks <= LPR*NCH chunks.
// Lane g of a group owns chunks g, g+LPR, g+2*LPR, ...
template <typename T, int LPR, int NCH>
__global__ void __launch_bounds__(256) gate_frames_vec(const T* __restrict__ logits, int64_t n_rows,
                                                       int V, float* __restrict__ H_out,
                                                       int32_t* __restrict__ arg_out) {
    constexpr int EPC = Chunk<T>::N;
    constexpr int ROWS_PER_BLOCK = 256 / LPR;
    const int g = threadIdx.x % LPR;
    int64_t row = (int64_t)blockIdx.x * ROWS_PER_BLOCK + threadIdx.x / LPR;
    const bool live = row < n_rows;
    if (!live) row = n_rows - 1;                      // keep the lane group whole for the reductions
    const int n_chunks = V / EPC;
    const uint4* src = reinterpret_cast<const uint4*>(logits + row * (int64_t)V);

    uint4 c[NCH];
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        const int idx = g + k * LPR;
        if (idx < n_chunks) {
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + idx));
            c[k] = make_uint4(v.x, v.y, v.z, v.w);
        }
        else c[k] = make_uint4(Chunk<T>::NEG_INF, Chunk<T>::NEG_INF, Chunk<T>::NEG_INF, Chunk<T>::NEG_INF);
    }

    float m = -INFINITY;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        float z[EPC];
        Chunk<T>::unpack(c[k], z);
#pragma unroll
        for (int e = 0; e < EPC; e += 2) m = fmaxf(m, fmaxf(z[e], z[e + 1]));
    }
    m = group_allreduce<LPR>(m, OpMax());

    // Walk the lane's elements from the highest index down so the last match is the lowest index.
    float S = 0.f, W = 0.f;
    int arg = 0x7fffffff;
#pragma unroll
    for (int k = NCH - 1; k >= 0; --k) {
        float z[EPC];
        Chunk<T>::unpack(c[k], z);
        const int base = (g + k * LPR) * EPC;
#pragma unroll
        for (int e = EPC - 1; e >= 0; --e) {
            const float d = z[e] - m;
            const float ex = __expf(d);
            S += ex;
            W = fmaf(ex, d, W);
            arg = (z[e] == m) ? base + e : arg;
        }
    }
    if (W != W) {
        // a score of -inf gives 0 * -inf above; redo the weighted sum with such terms as 0
        W = 0.f;
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            float z[EPC];
            Chunk<T>::unpack(c[k], z);
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
                const float d = fmaxf(z[e] - m, -1e30f);
                W = fmaf(__expf(d), d, W);
            }
        }
    }
    S = group_allreduce<LPR>(S, OpSum());
    W = group_allreduce<LPR>(W, OpSum());
    arg = group_allreduce_i<LPR>(arg, OpMinI());
    if (live && g == 0) {
        H_out[row] = __logf(S) - W / S;
        arg_out[row] = arg;
    }
}

// bf16 fast path.  A bf16 score widened to fp32 has 16 zero bits at the bottom; the complement of
// the element index is put there while widening (one v_lshl_or / v_and_or per element, the same
// cost as the plain widening), so that ONE float maximum over these keys yields both the row maximum
// (top 16 bits) and, among equal scores, the lowest index (largest complement) -- no per-element
// compare/select.  That holds for a positive, normal maximum; rows whose maximum is negative, zero,
// denormal or non-finite take the generic route (compare/select per element), chosen per
// wavefront.  The second sweep is one fma (z*log2e - m*log2e), one v_exp_f32, one add, one fma per
// element:  H = ln2 * (log2 S - W2/S) with S = sum 2^t, W2 = sum 2^t t, which is shift invariant
// in t, so the rounding of m*log2e cancels.
// The kernel is persistent (grid-stride over row blocks) so the per-lane index constants are built
// once, and the loads of the next row block are issued before the arithmetic of the current one.
__device__ __forceinline__ float max3_bits(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));   // returns an operand bit-exactly
    return r;
}
__device__ __forceinline__ float max_bits(float a, float b) {
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
template <int W>
__device__ __forceinline__ float group_max_bits(float v) {
    v = max_bits(v, dpp_f<DPP_XOR1>(v));
    v = max_bits(v, dpp_f<DPP_XOR2>(v));
    v = max_bits(v, dpp_f<DPP_HALF_MIRROR>(v));
    v = max_bits(v, dpp_f<DPP_MIRROR>(v));
    if (W > 16) {
        v = max_bits(v, __shfl_xor(v, 16));
        v = max_bits(v, __shfl_xor(v, 32));
    }
    return v;
}

template <int LPR, int NCH, bool FULL>     // FULL: the row has exactly LPR*NCH chunks (no chunk predicate)
__global__ void __launch_bounds__(256) gate_frames_bf16_keyed(const bf16_t* __restrict__ logits, int64_t n_rows, int V,
                                                              float* __restrict__ H_out, int32_t* __restrict__ arg_out) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr int ROWS_PER_BLOCK = 256 / LPR;
    constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;
    const int g = threadIdx.x % LPR;
    const int n_chunks = V / 8;
    const int64_t n_blocks = (n_rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    // (~index) & 0xffff of the eight elements of this lane's first chunk.  Chunk k lies 128 k elements
    // further; for the row lengths served here (at most 8 chunks of 16 lanes) that only clears bits
    // 7.. of the complement, so the key of chunk k is the key of chunk 0 xor (k << 7): applied once
    // per chunk to the chunk's maximum, not per element.  Eight constants instead of one per element
    // keep the kernel at 150 registers, i.e. three wavefronts per SIMD instead of two (5.2 -> 5.6 TB/s).
    uint32_t low0[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) low0[e] = (~(uint32_t)(g * 8 + e)) & 0xffffu;
    auto load_block = [&](int64_t blk, u32x4 (&c)[NCH]) {
        int64_t row = blk * ROWS_PER_BLOCK + threadIdx.x / LPR;
        if (row >= n_rows) row = n_rows - 1;
        const u32x4* src = reinterpret_cast<const u32x4*>(logits + row * (int64_t)V) + g;
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            if (FULL || g + k * LPR < n_chunks) c[k] = __builtin_nontemporal_load(src + k * LPR);
            else c[k] = (u32x4){0xf14af14au, 0xf14af14au, 0xf14af14au, 0xf14af14au};   // about -1e30: finite, exp -> 0
        }
    };

    u32x4 buf0[NCH], buf1[NCH];
    if ((int64_t)blockIdx.x < n_blocks) load_block(blockIdx.x, buf0);
    // two row blocks per trip so that the register sets swap roles without copies
    for (int64_t blk0 = blockIdx.x; blk0 < n_blocks; blk0 += 2 * (int64_t)gridDim.x) {
      #pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int64_t blk = blk0 + half * (int64_t)gridDim.x;
        if (blk >= n_blocks) break;
        u32x4 (&cur)[NCH] = half ? buf1 : buf0;
        u32x4 (&nxt)[NCH] = half ? buf0 : buf1;
        const int64_t nblk = blk + gridDim.x;
        if (nblk < n_blocks) load_block(nblk, nxt);
        const int64_t row = blk * ROWS_PER_BLOCK + threadIdx.x / LPR;
        const bool live = row < n_rows;

        // ---- sweep 1: maximum of the keyed values
        float mk = __uint_as_float(0xff800000u);           // -inf
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            float mc = __uint_as_float(0xff800000u);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t x = cur[k][w];
                const float k_lo = __uint_as_float((x << 16) | low0[2 * w]);
                const float k_hi = __uint_as_float((x & 0xffff0000u) | low0[2 * w + 1]);
                mc = max3_bits(mc, k_lo, k_hi);
            }
            // (a chunk without any value above -inf turns into a non-number here, which the maximum ignores)
            mk = max_bits(mk, __uint_as_float(__float_as_uint(mc) ^ (uint32_t)(k * LPR * 8)));
        }
        mk = group_max_bits<LPR>(mk);
        const uint32_t mb = __float_as_uint(mk);
        const uint32_t expo = mb & 0x7f800000u;
        const bool easy = (mb >> 31) == 0 && expo != 0 && expo != 0x7f800000u;
        // generic route: plain maximum, then the lowest index that attains it by compare/select
        auto generic_max = [&](float& m, int& arg) {
            m = -INFINITY;
#pragma unroll
            for (int k = 0; k < NCH; ++k)
#pragma unroll
                for (int w = 0; w < 4; ++w) m = fmaxf(m, fmaxf(bf16_lo(cur[k][w]), bf16_hi(cur[k][w])));
            m = group_allreduce<LPR>(m, OpMax());
            arg = 0x7fffffff;
#pragma unroll
            for (int k = NCH - 1; k >= 0; --k)
#pragma unroll
                for (int w = 3; w >= 0; --w) {
                    const int base = (g + k * LPR) * 8 + 2 * w;
                    arg = (bf16_hi(cur[k][w]) == m) ? base + 1 : arg;
                    arg = (bf16_lo(cur[k][w]) == m) ? base : arg;
                }
            arg = group_allreduce_i<LPR>(arg, OpMinI());
        };
        float m, S = 0.f, W2 = 0.f;
        int arg;
        if (__all(easy)) {
            m = __uint_as_float(mb & 0xffff0000u);
            arg = (int)((~mb) & 0xffffu);
        } else {
            generic_max(m, arg);
        }
        // ---- sweep 2: S = sum 2^t, W2 = sum 2^t t,  t = (z - m) log2(e) up to a row constant
        float nml = -m * LOG2E;
#pragma unroll
        for (int k = 0; k < NCH; ++k)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float t0 = fmaf(bf16_lo(cur[k][w]), LOG2E, nml), t1 = fmaf(bf16_hi(cur[k][w]), LOG2E, nml);
                const float e0 = __builtin_amdgcn_exp2f(t0), e1 = __builtin_amdgcn_exp2f(t1);
                S += e0; W2 = fmaf(e0, t0, W2);
                S += e1; W2 = fmaf(e1, t1, W2);
            }
        if (__any(W2 != W2)) {
            // A score of -inf gives 0 * -inf above (and a non-number key in sweep 1): redo the rows of
            // this wavefront on the generic route, with such terms counted as 0.
            generic_max(m, arg);
            nml = -m * LOG2E;
            S = 0.f; W2 = 0.f;
#pragma unroll
            for (int k = 0; k < NCH; ++k)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float t0 = fmaxf(fmaf(bf16_lo(cur[k][w]), LOG2E, nml), -1e30f);
                    const float t1 = fmaxf(fmaf(bf16_hi(cur[k][w]), LOG2E, nml), -1e30f);
                    const float e0 = __builtin_amdgcn_exp2f(t0), e1 = __builtin_amdgcn_exp2f(t1);
                    S += e0; W2 = fmaf(e0, t0, W2);
                    S += e1; W2 = fmaf(e1, t1, W2);
                }
        }
        S = group_allreduce<LPR>(S, OpSum());
        W2 = group_allreduce<LPR>(W2, OpSum());
        if (live && g == 0) {
            H_out[row] = LN2 * (__builtin_amdgcn_logf(S) - W2 / S);
            arg_out[row] = arg;
        }
      }
    }
}

// Any V, any alignment: one wavefront per row, two passes over memory (second pass hits cache).
template <typename T>
__global__ void __launch_bounds__(256) gate_frames_generic(const T* __restrict__ logits, int64_t n_rows,
                                                           int V, float* __restrict__ H_out,
                                                           int32_t* __restrict__ arg_out) {
    const int lane = threadIdx.x % 64;
    int64_t row = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
    const bool live = row < n_rows;
    if (!live) row = n_rows - 1;
    const T* src = logits + row * (int64_t)V;
    auto ld = [&](int i) -> float {
        if constexpr (sizeof(T) == 2) return bf16_to_f32(src[i]); else return src[i];
    };
    float m = -INFINITY;
    for (int i = lane; i < V; i += 64) m = fmaxf(m, ld(i));
    m = group_allreduce<64>(m, OpMax());
    float S = 0.f, W = 0.f;
    int arg = 0x7fffffff;
    for (int i = lane; i < V; i += 64) {
        const float z = ld(i);
        const float d = fmaxf(z - m, -1e30f);
        const float ex = __expf(d);
        S += ex;
        W = fmaf(ex, d, W);
        if (z == m && i < arg) arg = i;
    }
    S = group_allreduce<64>(S, OpSum());
    W = group_allreduce<64>(W, OpSum());
    arg = group_allreduce_i<64>(arg, OpMinI());
    if (live && lane == 0) {
        H_out[row] = __logf(S) - W / S;
        arg_out[row] = arg;
    }
}

// One workgroup (256 threads) per utterance.  The frame range of an utterance is clamped into
// [0, n_rows], so that prefix sums that were never seen by the host cannot lead outside H / arg / draft.
__global__ void __launch_bounds__(256) gate_utterances(const float* __restrict__ H,
                                                       const int32_t* __restrict__ arg,
                                                       const int32_t* __restrict__ cu_frames, int n_rows, int blank,
                                                       float tau, float* __restrict__ max_entropy,
                                                       uint8_t* __restrict__ gate_pass,
                                                       int32_t* __restrict__ draft, int32_t* __restrict__ draft_len) {
    __shared__ int wave_cnt[4];
    __shared__ float wave_max[4];
    const int b = blockIdx.x;
    const int lo = min(max(cu_frames[b], 0), n_rows), hi = min(max(cu_frames[b + 1], lo), n_rows);
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    float mx = -INFINITY;
    int written = 0;                                   // same value in every thread
    for (int t0 = lo; t0 < hi; t0 += 256) {
        const int t = t0 + threadIdx.x;
        bool keep = false;
        int a = 0;
        if (t < hi) {
            a = arg[t];
            mx = fmaxf(mx, H[t]);
            keep = (a != blank) && (t == lo || a != arg[t - 1]);
        }
        const unsigned long long mask = __ballot(keep);
        const int before = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[wave] = __popcll(mask);
        __syncthreads();
        int wave_off = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int c = wave_cnt[w];
            if (w < wave) wave_off += c;
            total += c;
        }
        if (keep) draft[lo + written + wave_off + before] = a;
        written += total;
        __syncthreads();
    }
    mx = group_allreduce<64>(mx, OpMax());
    if (lane == 0) wave_max[wave] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float m = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
        max_entropy[b] = m;
        gate_pass[b] = (m < tau) ? 1 : 0;
        draft_len[b] = written;
    }
}

void launch_gate_utterances(const float* H, const int32_t* arg, const int32_t* cu_frames_dev, int64_t n_rows, int B, int blank,
                            float tau, float* max_entropy, uint8_t* gate_pass, int32_t* draft, int32_t* draft_len,
                            hipStream_t st) {
    hipLaunchKernelGGL(gate_utterances, dim3(B), dim3(256), 0, st, H, arg, cu_frames_dev, (int)n_rows, blank, tau,
                       max_entropy, gate_pass, draft, draft_len);
}

template <typename T, int LPR>
static void launch_vec(const T* logits, int64_t n_rows, int V, float* H, int32_t* arg, hipStream_t st) {
    const int n_chunks = V / Chunk<T>::N;
    const int nch = (n_chunks + LPR - 1) / LPR;
    const unsigned grid = (unsigned)((n_rows + (256 / LPR) - 1) / (256 / LPR));
    if constexpr (sizeof(T) == 2) {
        // persistent launch: enough workgroups to fill 256 CUs several times over, no more than there is work
        const unsigned pgrid = grid < 256u * 8u ? grid : 256u * 8u;
        const bf16_t* z = logits;
        const bool full = n_chunks == nch * LPR;
#define SSD_GATE_LAUNCH(NCH_)                                                                                          \
        if (full) hipLaunchKernelGGL((gate_frames_bf16_keyed<LPR, NCH_, true>), dim3(pgrid), dim3(256), 0, st, z, n_rows, V, H, arg); \
        else hipLaunchKernelGGL((gate_frames_bf16_keyed<LPR, NCH_, false>), dim3(pgrid), dim3(256), 0, st, z, n_rows, V, H, arg)
        if (nch <= 1) { SSD_GATE_LAUNCH(1); }
        else if (nch <= 2) { SSD_GATE_LAUNCH(2); }
        else if (nch <= 4) { SSD_GATE_LAUNCH(4); }
        else { SSD_GATE_LAUNCH(8); }
#undef SSD_GATE_LAUNCH
        return;
    }
    if (nch <= 1) hipLaunchKernelGGL((gate_frames_vec<T, LPR, 1>), dim3(grid), dim3(256), 0, st, logits, n_rows, V, H, arg);
    else if (nch <= 2) hipLaunchKernelGGL((gate_frames_vec<T, LPR, 2>), dim3(grid), dim3(256), 0, st, logits, n_rows, V, H, arg);
    else if (nch <= 4) hipLaunchKernelGGL((gate_frames_vec<T, LPR, 4>), dim3(grid), dim3(256), 0, st, logits, n_rows, V, H, arg);
    else hipLaunchKernelGGL((gate_frames_vec<T, LPR, 8>), dim3(grid), dim3(256), 0, st, logits, n_rows, V, H, arg);
}

template <typename T>
static void launch_frames(const T* logits, int64_t n_rows, int V, float* H, int32_t* arg, hipStream_t st) {
    constexpr int EPC = Chunk<T>::N;
    const bool vec_ok = (V % EPC == 0) && ((reinterpret_cast<uintptr_t>(logits) & 15) == 0);
    if (vec_ok && V <= 16 * 8 * EPC && V > 0) {
        if (V <= 16 * 4 * EPC || V > 64 * 4 * EPC / 2) launch_vec<T, 16>(logits, n_rows, V, H, arg, st);
        else launch_vec<T, 64>(logits, n_rows, V, H, arg, st);
    } else if (vec_ok && V <= 64 * 8 * EPC) {
        launch_vec<T, 64>(logits, n_rows, V, H, arg, st);
    } else {
        const unsigned grid = (unsigned)((n_rows + 3) / 4);
        hipLaunchKernelGGL((gate_frames_generic<T>), dim3(grid), dim3(256), 0, st, logits, n_rows, V, H, arg);
    }
}

void launch_gate(const void* logits, int dtype, int64_t n_rows, int V, const int32_t* cu_frames_dev, int B,
                 int blank, float tau, float* H, int32_t* arg, float* max_entropy, uint8_t* gate_pass,
                 int32_t* draft, int32_t* draft_len, hipStream_t st) {
    if (dtype == SSD_BF16) launch_frames<bf16_t>(static_cast<const bf16_t*>(logits), n_rows, V, H, arg, st);
    else launch_frames<float>(static_cast<const float*>(logits), n_rows, V, H, arg, st);
    launch_gate_utterances(H, arg, cu_frames_dev, n_rows, B, blank, tau, max_entropy, gate_pass, draft, draft_len, st);
}

}  // namespace ssd
