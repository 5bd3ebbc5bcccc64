// The three projection GEMMs of a decoder layer (Eq. 4's network), 16-bit MFMA (IEEE half or bfloat16 operands,
// a template parameter of every kernel here) with fused epilogues:
//   QKV      : a[M,d] x Wqkv^T  -> rotary embedding on q,k in fp32 -> f16 qkv[M, d_q + 2 d_kv]
//   residual : o[M,K] x W^T     -> x[M,N] += acc                (attention output and MLP down projection)
//   SwiGLU   : b[M,d] x Wgu^T   -> h[M,d_ff] = silu(gate) * up  (f16)
// Every epilogue first multiplies the accumulator by `descale`, the inverse of the power of two the
// weight tensor was scaled by when it was converted to f16.
// The fused weight layouts are produced by pack_qkv_kernel / pack_gate_up_kernel: a column and the
// column it must be combined with sit 32 packed columns apart inside a group of 64, i.e. in two
// accumulator blocks of the same lane.
// Three main loops feed these epilogues: big tiles on v_mfma_f32_16x16x32_f16 (gemm_core16.h), skinny
// LDS-ring tiles for 33..128 rows (gemm_core.h) and the register-streaming kernel for at most 32 rows
// (gemm_stream.h).
#include <type_traits>

#include "gemm_core.h"
#include "gemm_core16.h"
#include "gemm_stream.h"
#include "ssd_internal.h"

namespace ssd {

// Workgroup id -> tile: one XCD walks a contiguous run of tiles, and tiles are ordered in bands of
// GROUP_M row-tiles so that the run reuses few A and W panels.
__device__ __forceinline__ void tile_of_workgroup(int pid, int total, int tiles_m, int tiles_n, int& tm, int& tn) {
    constexpr int GROUP_M = 4;
    const int v = xcd_contiguous_index(pid, total);
    const int band = v / (GROUP_M * tiles_n);
    const int first_m = band * GROUP_M;
    const int rows = min(tiles_m - first_m, GROUP_M);
    const int in = v % (GROUP_M * tiles_n);
    tm = first_m + in % rows;
    tn = in / rows;
}

// The epilogues below read first and write afterwards, block by block: a load placed after a store
// through an unrelated pointer cannot be moved ahead of it by the compiler, and a read-modify-write
// written element by element degenerates into one exposed memory round trip per element.
// They are written against an accumulator layout L (Layout32: 32x32 blocks of v_mfma_f32_32x32x16,
// Layout16: 16x16 blocks of v_mfma_f32_16x16x32): L::row / L::col give the element a register holds and
// L::PAIR the distance, in blocks, to the block 32 columns further (where the fused weight layouts put
// the partner column).
constexpr int residual_batch(int tm, int g0) {             // largest divisor of tm that is at most g0 (at least 1)
    int g = 1;
    for (int c = 1; c <= tm; ++c)
        if (tm % c == 0 && c <= g0) g = c;
    return g;
}
template <bool BF_>
struct EpiResidual {
    // (not transposed: the fp32 read-modify-write measured 3-8 % slower with 16-byte accesses whose lanes of one
    // row segment are 16 lane ids apart, O projection 8.77 -> 8.95 ms per step at 15214 rows)
    static constexpr bool WANTS_SPLIT = false, BF = BF_, TRANSPOSE = false, USES_LDS = false;
    float* x; int ldx; float descale;
    template <int TM, int TN, class L = Layout32>
    __device__ __forceinline__ void operator()(typename L::vec_t (&acc)[TM][TN], int row0, int col0, int M, int lane) const {
        if constexpr (L::TRANSPOSED) {
            // a lane holds four consecutive columns of one row per block: 16-byte loads and stores
            constexpr int GT = residual_batch(TM, 96 / (4 * TN));
#pragma unroll
            for (int i0 = 0; i0 < TM; i0 += GT) {
                float4 old[GT][TN];
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    const int row = min(row0 + L::row(i0 + g, lane), M - 1);
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        old[g][j] = *reinterpret_cast<const float4*>(x + (int64_t)row * ldx + col0 + L::col4(j, lane));
                }
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    const int row = row0 + L::row(i0 + g, lane);
                    if (row >= M) continue;
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const f32x4_t a = acc[i0 + g][j];
                        *reinterpret_cast<float4*>(x + (int64_t)row * ldx + col0 + L::col4(j, lane)) =
                            make_float4(old[g][j].x + a[0] * descale, old[g][j].y + a[1] * descale, old[g][j].z + a[2] * descale,
                                        old[g][j].w + a[3] * descale);
                    }
                }
            }
            return;
        } else {
        // Row blocks per batch: all loads of a batch are in flight together, so a tile pays one memory
        // latency per batch.  Up to 96 registers of old values (the fragment registers are dead by now).
        constexpr int G0 = 96 / (L::REGS * TN);
        constexpr int G = residual_batch(TM, G0);
#pragma unroll
        for (int i0 = 0; i0 < TM; i0 += G) {
            float old[G][L::REGS][TN];
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int r = 0; r < L::REGS; ++r) {
                    const int row = min(row0 + L::row(i0 + g, r, lane), M - 1);
#pragma unroll
                    for (int j = 0; j < TN; ++j) old[g][r][j] = x[(int64_t)row * ldx + col0 + L::col(j, lane)];
                }
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int r = 0; r < L::REGS; ++r) {
                    const int row = row0 + L::row(i0 + g, r, lane);
                    if (row >= M) continue;
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        x[(int64_t)row * ldx + col0 + L::col(j, lane)] = old[g][r][j] + acc[i0 + g][j][r] * descale;
                }
        }
        }
    }
};

// The residual epilogue of the big tiles: x[M,N] += acc through the workgroup's LDS (free after the K loop).  With
// transposed accumulator blocks a lane writes its four consecutive columns of a row as one 16-byte LDS store; the
// wavefront's 64 x 64 half tile is then read back row by row, 16 lanes per 256-byte row, so that the old values of x
// are loaded and the sums stored with fully coalesced 16-byte accesses: 32 + 32 global instructions per wavefront
// instead of 128 + 128 four-byte ones that touch 64-byte pieces of four rows each.
constexpr int RES_LDS_STRIDE = 68;                           // floats per staged row: 64 + 4 (16-byte columns stay spread)
template <bool BF_>
struct EpiResidualLds {
    static constexpr bool WANTS_SPLIT = false, BF = BF_, TRANSPOSE = true, USES_LDS = true;
    float* x; int ldx; float descale;
    template <int TM> static constexpr int wave_lds_bytes() { return (TM / 2) * 16 * RES_LDS_STRIDE * 4; }
    template <int TM, int TN>
    __device__ __forceinline__ void run_lds(f32x4_t (&acc)[TM][TN], int row0, int col0, int M, int lane, float* stage) const {
        static_assert(TN == 4 && TM % 2 == 0, "a wavefront tile of 64 columns, two halves of row blocks");
        constexpr int HB = TM / 2;                           // row blocks per half
        constexpr int ROWS = HB * 16;                        // rows per half
        constexpr int NI = ROWS / 4;                         // instructions per half: 4 rows x 256 bytes each
        const int m = lane % 16, g = lane / 16;
        const int rr = lane / 16, cc = (lane % 16) * 4;      // read-back: row 4 it + rr of the half, columns cc .. cc + 3
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            // old values first: their round trip overlaps the LDS exchange
            float4 old[NI];
#pragma unroll
            for (int it = 0; it < NI; ++it) {
                const int row = min(row0 + half * ROWS + 4 * it + rr, M - 1);
                typedef float f32x4v __attribute__((ext_vector_type(4)));
                const f32x4v t = __builtin_nontemporal_load(reinterpret_cast<const f32x4v*>(x + (int64_t)row * ldx + col0 + cc));
                old[it] = make_float4(t[0], t[1], t[2], t[3]);
            }
            if (half) __builtin_amdgcn_wave_barrier();       // the reads of the first half are done (waited for below)
#pragma unroll
            for (int i = 0; i < HB; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const f32x4_t a = acc[half * HB + i][j];
                    *reinterpret_cast<float4*>(stage + (i * 16 + m) * RES_LDS_STRIDE + j * 16 + 4 * g) =
                        make_float4(a[0] * descale, a[1] * descale, a[2] * descale, a[3] * descale);
                }
            __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0): the stores have landed
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int it = 0; it < NI; ++it) {
                const int row = row0 + half * ROWS + 4 * it + rr;
                const float4 v = *reinterpret_cast<const float4*>(stage + (4 * it + rr) * RES_LDS_STRIDE + cc);
                if (row < M)
                    *reinterpret_cast<float4*>(x + (int64_t)row * ldx + col0 + cc) =
                        make_float4(old[it].x + v.x, old[it].y + v.y, old[it].z + v.z, old[it].w + v.w);
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);
        }
    }
};

template <bool BF_>
struct EpiQkvRope {
    static constexpr bool WANTS_SPLIT = false, BF = BF_, TRANSPOSE = true, USES_LDS = false;     // big tiles: transposed accumulator blocks
    f16_t* qkv; int ldq; int d_rot; float descale;            // d_rot = d_q + d_kv: columns that get rotated
    const int32_t* pos; const float2* rope_tab; // rope_tab[pos][i] = (cos, sin), i < 64
    // optional K/V cache: rows with row_slot[row] >= 0 also store their k and v parts at that slot
    const int32_t* row_slot; f16_t* kc; f16_t* vc; int d_q;
    // optional: the table rows already gathered per decoder row (rope_rows[row][i] = rope_tab[pos[row]][i]),
    // which takes the position lookup out of the dependency chain
    const float2* rope_rows;
    int32_t* flags;                             // sticky device flags: a saturated store raises SSD_FLAG_ACT_OVERFLOW
    template <int TM, int TN, class L = Layout32>
    __device__ __forceinline__ void operator()(typename L::vec_t (&acc)[TM][TN], int row0, int col0, int M, int lane) const {
        static_assert((TN * L::BLOCK) % 64 == 0, "rotation partners live 32 packed columns apart in groups of 64");
        if constexpr (L::TRANSPOSED) {
            // A lane holds one row and four consecutive packed columns per block: the four rotary entries are one
            // 32-byte read, the outputs two 8-byte stores (and two more into the K/V cache).
            const float2* tabT = rope_rows ? rope_rows : rope_tab;
            const int d_kvT = d_rot - d_q;
            float peak = 0.f;
            constexpr int NJT = TN / 2;
            constexpr int GT = residual_batch(TM, 64 / (NJT * 8) > 0 ? 64 / (NJT * 8) : 1);
#pragma unroll
            for (int i0 = 0; i0 < TM; i0 += GT) {
                int t_row[GT], slot[GT];
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    const int row = min(row0 + L::row(i0 + g, lane), M - 1);
                    t_row[g] = rope_rows ? row : pos[row];
                    slot[g] = row_slot ? row_slot[row] : -1;
                }
                float4 cs[GT][NJT][2];                      // (cos, sin) of four consecutive rotary indices
#pragma unroll
                for (int g = 0; g < GT; ++g)
#pragma unroll
                    for (int jj = 0; jj < NJT; ++jj) {
                        const int j = (jj / L::PAIR) * 2 * L::PAIR + jj % L::PAIR;
                        const int p = col0 + j * L::BLOCK;
                        const int i_rot = ((p % 128) / 64) * 32 + p % 32 + 4 * (lane / 16);
                        if (p < d_rot) {
                            const float4* src = reinterpret_cast<const float4*>(tabT + (int64_t)t_row[g] * 64 + i_rot);
                            cs[g][jj][0] = src[0];
                            cs[g][jj][1] = src[1];
                        } else {
                            cs[g][jj][0] = cs[g][jj][1] = make_float4(1.f, 0.f, 1.f, 0.f);
                        }
                    }
                auto store_batch = [&](auto clamp_c) {
                    constexpr bool CLAMP = decltype(clamp_c)::value;
#pragma unroll
                    for (int g = 0; g < GT; ++g) {
                        const int row = row0 + L::row(i0 + g, lane);
                        if (row >= M) continue;
#pragma unroll
                        for (int jj = 0; jj < NJT; ++jj) {
                            const int j = (jj / L::PAIR) * 2 * L::PAIR + jj % L::PAIR;
                            const int p = col0 + j * L::BLOCK;
                            const bool rot = p < d_rot;
                            const int head = p / 128, i_rot = ((p % 128) / 64) * 32 + p % 32 + 4 * (lane / 16);
                            const int c0 = rot ? head * 128 + i_rot : p + 4 * (lane / 16);
                            const int c1 = rot ? c0 + 64 : c0 + 32;
                            const f32x4_t a = acc[i0 + g][j], b = acc[i0 + g][j + L::PAIR];
                            const float cx[4] = {cs[g][jj][0].x, cs[g][jj][0].z, cs[g][jj][1].x, cs[g][jj][1].z};
                            const float sy[4] = {cs[g][jj][0].y, cs[g][jj][0].w, cs[g][jj][1].y, cs[g][jj][1].w};
                            uint16_t v0[4], v1[4];
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const float av = a[r] * descale, bv = b[r] * descale;
                                v0[r] = Op16<BF>::template store<CLAMP>(av * cx[r] - bv * sy[r], peak);
                                v1[r] = Op16<BF>::template store<CLAMP>(bv * cx[r] + av * sy[r], peak);
                            }
                            const uint2 w0 = make_uint2((uint32_t)v0[0] | ((uint32_t)v0[1] << 16), (uint32_t)v0[2] | ((uint32_t)v0[3] << 16));
                            const uint2 w1 = make_uint2((uint32_t)v1[0] | ((uint32_t)v1[1] << 16), (uint32_t)v1[2] | ((uint32_t)v1[3] << 16));
                            f16_t* o = qkv + (int64_t)row * ldq;
                            *reinterpret_cast<uint2*>(o + c0) = w0;
                            *reinterpret_cast<uint2*>(o + c1) = w1;
                            if (slot[g] >= 0 && c0 >= d_q) {
                                f16_t* dst = (rot ? kc : vc) + (int64_t)slot[g] * d_kvT - (rot ? d_q : d_rot);
                                *reinterpret_cast<uint2*>(dst + c0) = w0;
                                *reinterpret_cast<uint2*>(dst + c1) = w1;
                            }
                        }
                    }
                };
                const float before = peak;
                store_batch(std::false_type());
                if (!(peak <= F16_MAX)) {
                    peak = before;
                    store_batch(std::true_type());
                    raise_flag(flags, SSD_FLAG_ACT_OVERFLOW);
                }
            }
        } else {
        // Column blocks come in groups of 64 packed columns: the first half holds x[i], the second x[i+64]
        // of 32 rotation pairs (or 64 plain columns of v); block j is handled with its partner j + PAIR.
        constexpr int NJ = TN / 2;
        // All table loads of a batch of row blocks are issued before the first store of the batch (the
        // compiler cannot move a load above a store that might alias it), so a batch costs one memory
        // latency, not one per block: up to 32 (cos, sin) pairs, 64 registers, are held per lane.
        constexpr int G = residual_batch(TM, 32 / (NJ * L::REGS) > 0 ? 32 / (NJ * L::REGS) : 1);
        const float2* tab = rope_rows ? rope_rows : rope_tab;
        const int d_kv = d_rot - d_q;
        float peak = 0.f;                                   // largest magnitude stored by this lane
#pragma unroll
        for (int i0 = 0; i0 < TM; i0 += G) {
            int t_row[G][L::REGS], slot[G][L::REGS];
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int r = 0; r < L::REGS; ++r) {
                    const int row = min(row0 + L::row(i0 + g, r, lane), M - 1);
                    t_row[g][r] = rope_rows ? row : pos[row];
                    slot[g][r] = row_slot ? row_slot[row] : -1;
                }
            float2 cs[G][NJ][L::REGS];
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int jj = 0; jj < NJ; ++jj) {
                    const int j = (jj / L::PAIR) * 2 * L::PAIR + jj % L::PAIR;
                    const int p = col0 + j * L::BLOCK;
                    const int i_rot = ((p % 128) / 64) * 32 + p % 32 + lane % L::BLOCK;
#pragma unroll
                    for (int r = 0; r < L::REGS; ++r)
                        cs[g][jj][r] = p < d_rot ? tab[(int64_t)t_row[g][r] * 64 + i_rot] : make_float2(1.f, 0.f);
                }
            // stores of the batch; repeated with clamping by a lane that met a value beyond the half range
            auto store_batch = [&](auto clamp_c) {
                constexpr bool CLAMP = decltype(clamp_c)::value;
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int jj = 0; jj < NJ; ++jj) {
                        const int j = (jj / L::PAIR) * 2 * L::PAIR + jj % L::PAIR;
                        const int p = col0 + j * L::BLOCK;              // packed column of this block
                        const bool rot = p < d_rot;
                        const int head = p / 128, i_rot = ((p % 128) / 64) * 32 + p % 32 + lane % L::BLOCK;
                        const int c0 = rot ? head * 128 + i_rot : p + lane % L::BLOCK;
                        const int c1 = rot ? c0 + 64 : c0 + 32;
#pragma unroll
                        for (int r = 0; r < L::REGS; ++r) {
                            const int row = row0 + L::row(i0 + g, r, lane);
                            if (row >= M) continue;
                            const float a = acc[i0 + g][j][r] * descale, b = acc[i0 + g][j + L::PAIR][r] * descale;
                            const float2 c = cs[g][jj][r];
                            f16_t* o = qkv + (int64_t)row * ldq;
                            const f16_t v0 = Op16<BF>::template store<CLAMP>(a * c.x - b * c.y, peak), v1 = Op16<BF>::template store<CLAMP>(b * c.x + a * c.y, peak);
                            o[c0] = v0;
                            o[c1] = v1;
                            if (slot[g][r] >= 0 && c0 >= d_q) {           // a group of 64 lies inside q, k or v
                                f16_t* dst = (rot ? kc : vc) + (int64_t)slot[g][r] * d_kv - (rot ? d_q : d_rot);
                                dst[c0] = v0;
                                dst[c1] = v1;
                            }
                        }
                    }
            };
            const float before = peak;
            store_batch(std::false_type());
            if (!(peak <= F16_MAX)) {
                peak = before;                              // keep later batches on the plain pass unless they overflow too
                store_batch(std::true_type());
                raise_flag(flags, SSD_FLAG_ACT_OVERFLOW);
            }
        }
        }
    }
};

template <bool BF_>
struct EpiSwiglu {
    static constexpr bool WANTS_SPLIT = false, BF = BF_, TRANSPOSE = true, USES_LDS = false;
    f16_t* h; int d_ff; float descale; int32_t* flags;
    template <int TM, int TN, class L = Layout32>
    __device__ __forceinline__ void operator()(typename L::vec_t (&acc)[TM][TN], int row0, int col0, int M, int lane) const {
        static_assert((TN * L::BLOCK) % 64 == 0, "gate/up live 32 packed columns apart in groups of 64");
        float peak = 0.f;                                   // largest magnitude stored by this lane
        if constexpr (L::TRANSPOSED) {
            // a lane holds one row and four consecutive packed columns per block: four outputs, one 8-byte store
            auto store_allT = [&](auto clamp_c) {
                constexpr bool CLAMP = decltype(clamp_c)::value;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int row = row0 + L::row(i, lane);
                    if (row >= M) continue;
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        if ((j / L::PAIR) % 2 != 0) continue;
                        const int p = col0 + j * L::BLOCK;
                        const int f = (p / 64) * 32 + p % 32 + 4 * (lane / 16);
                        uint16_t v[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const float g = acc[i][j][r] * descale, u = acc[i][j + L::PAIR][r] * descale;
                            v[r] = Op16<BF>::template store<CLAMP>(g * u * __builtin_amdgcn_rcpf(1.0f + __expf(-g)), peak);
                        }
                        *reinterpret_cast<uint2*>(h + (int64_t)row * d_ff + f) =
                            make_uint2((uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16));
                    }
                }
            };
            store_allT(std::false_type());
            if (!(peak <= F16_MAX)) {
                store_allT(std::true_type());
                raise_flag(flags, SSD_FLAG_ACT_OVERFLOW);
            }
        } else {
        auto store_all = [&](auto clamp_c) {
            constexpr bool CLAMP = decltype(clamp_c)::value;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if ((j / L::PAIR) % 2 != 0) continue;
                const int p = col0 + j * L::BLOCK;
                const int f = (p / 64) * 32 + p % 32 + lane % L::BLOCK;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < L::REGS; ++r) {
                        const int row = row0 + L::row(i, r, lane);
                        if (row >= M) continue;
                        const float g = acc[i][j][r] * descale, u = acc[i][j + L::PAIR][r] * descale;
                        // silu(g) * u with the hardware reciprocal (1 ulp) instead of an IEEE division: the epilogue is
                        // 48 outputs per lane and the division was half of its instructions
                        h[(int64_t)row * d_ff + f] = Op16<BF>::template store<CLAMP>(g * u * __builtin_amdgcn_rcpf(1.0f + __expf(-g)), peak);
                    }
            }
        };
        store_all(std::false_type());
        if (!(peak <= F16_MAX)) {                           // rare: repeat this lane's stores saturated
            store_all(std::true_type());
            raise_flag(flags, SSD_FLAG_ACT_OVERFLOW);
        }
        }
    }
};

// Stores the scaled accumulator as an fp32 partial sum of one K split: part[split][row][col].
// Whoever consumes it (the RMSNorm that follows) adds the splits in a fixed order.
template <bool BF_>
struct EpiPartial {
    static constexpr bool WANTS_SPLIT = true, BF = BF_, TRANSPOSE = false, USES_LDS = false;
    float* part; int ld; int64_t split_stride; float descale;
    template <int TM, int TN, class L = Layout32>
    __device__ __forceinline__ void operator()(typename L::vec_t (&acc)[TM][TN], int row0, int col0, int M, int lane, int split) const {
        float* base = part + split * split_stride;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < L::REGS; ++r) {
                const int row = row0 + L::row(i, r, lane);
                if (row >= M) continue;
#pragma unroll
                for (int j = 0; j < TN; ++j) base[(int64_t)row * ld + col0 + L::col(j, lane)] = acc[i][j][r] * descale;
            }
    }
};

// Epilogues for products outside the decoder layer (the projector's windowed cross-attention).
// EpiScoresValues: the product [frames, 64 score columns | d_h value columns | padding] is split on the way out.
// The score columns stay fp32 (they go through an exponential), rows of 64; the value columns are rounded to IEEE
// half (2^-12 relative, an eighth of the bf16 rounding their weighted sums get afterwards; beyond 65504 they
// saturate and SSD_FLAG_ACT_OVERFLOW is raised), rows of d_h: 2.3 KB per frame instead of 5 KB of fp32.
template <bool BF_>
struct EpiScoresValues {
    static constexpr bool WANTS_SPLIT = false, BF = BF_, TRANSPOSE = true, USES_LDS = false;
    float* scores; uint16_t* vals; int d_h; int32_t* flags;
    template <int TM, int TN, class L = Layout32>
    __device__ __forceinline__ void operator()(typename L::vec_t (&acc)[TM][TN], int row0, int col0, int M, int lane) const {
        bool bad = false;
        if constexpr (L::TRANSPOSED) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = row0 + L::row(i, lane);
                if (row >= M) continue;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = col0 + L::col4(j, lane);           // blocks of 16 columns never straddle column 64
                    if (col < QF_SCORE_COLS)
                        *reinterpret_cast<float4*>(scores + (int64_t)row * QF_SCORE_COLS + col) =
                            make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
                    else if (col - QF_SCORE_COLS < d_h)
                        *reinterpret_cast<uint2*>(vals + (int64_t)row * d_h + (col - QF_SCORE_COLS)) =
                            make_uint2(pack_f16x2_sat(acc[i][j][0], acc[i][j][1], bad), pack_f16x2_sat(acc[i][j][2], acc[i][j][3], bad));
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < L::REGS; ++r) {
                    const int row = row0 + L::row(i, r, lane);
                    if (row >= M) continue;
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int col = col0 + L::col(j, lane);
                        if (col < QF_SCORE_COLS) scores[(int64_t)row * QF_SCORE_COLS + col] = acc[i][j][r];
                        else if (col - QF_SCORE_COLS < d_h) vals[(int64_t)row * d_h + (col - QF_SCORE_COLS)] = f32_to_f16_sat(acc[i][j][r], bad);
                    }
                }
        }
        if (bad) raise_flag(flags, SSD_FLAG_ACT_OVERFLOW);
    }
};
template <bool BF_>
struct EpiStore16 {
    static constexpr bool WANTS_SPLIT = false, BF = BF_, TRANSPOSE = true, USES_LDS = false;
    uint16_t* c; int ldc;
    template <int TM, int TN, class L = Layout32>
    __device__ __forceinline__ void operator()(typename L::vec_t (&acc)[TM][TN], int row0, int col0, int M, int lane) const {
        if constexpr (L::TRANSPOSED) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = row0 + L::row(i, lane);
                if (row >= M) continue;
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    *reinterpret_cast<uint2*>(c + (int64_t)row * ldc + col0 + L::col4(j, lane)) =
                        make_uint2(op_pack2<BF>(acc[i][j][0], acc[i][j][1]), op_pack2<BF>(acc[i][j][2], acc[i][j][3]));
            }
            return;
        } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < L::REGS; ++r) {
                const int row = row0 + L::row(i, r, lane);
                if (row >= M) continue;
#pragma unroll
                for (int j = 0; j < TN; ++j) c[(int64_t)row * ldc + col0 + L::col(j, lane)] = Op16<BF>::cvt(acc[i][j][r]);
            }
        }
    }
};

// grid = tiles * splits; split s of a tile accumulates K slices [s*KT/splits, (s+1)*KT/splits)
template <int BM, int BN, int WAVES_M, int WAVES_N, int NSTAGE, class Epi>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N)
gemm_mfma_kernel(const f16_t* __restrict__ A, const f16_t* __restrict__ W, int M, int N, int K, int splits, Epi epi) {
    using Tile = GemmTile<BM, BN, WAVES_M, WAVES_N, NSTAGE, Epi::BF>;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    const int split = blockIdx.x % splits;
    int tm, tn;
    tile_of_workgroup(blockIdx.x / splits, tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);
    const int KT = K / GEMM_BK;
    const int kt0 = (int)((int64_t)KT * split / splits), kt1 = (int)((int64_t)KT * (split + 1) / splits);
    f32x16_t acc[Tile::TM][Tile::TN];
#pragma unroll
    for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
        for (int j = 0; j < Tile::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    Tile::run(A, W, M, K, tm * BM, tn * BN, kt0, kt1, smem_raw, acc);
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    if constexpr (Epi::WANTS_SPLIT)
        epi.template operator()<Tile::TM, Tile::TN>(acc, tm * BM + wm * Tile::WTM, tn * BN + wn * Tile::WTN, M, lane, split);
    else
        epi.template operator()<Tile::TM, Tile::TN>(acc, tm * BM + wm * Tile::WTM, tn * BN + wn * Tile::WTN, M, lane);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int NSTAGE, class Epi>
static void launch_gemm(const f16_t* A, const f16_t* W, int M, int N, int K, int splits, const Epi& epi, hipStream_t st) {
    if (M <= 0) return;
    auto kern = gemm_mfma_kernel<BM, BN, WAVES_M, WAVES_N, NSTAGE, Epi>;
    constexpr size_t lds = gemm_lds_bytes<BM, BN, NSTAGE>();
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    const int tiles = ((M + BM - 1) / BM) * (N / BN);
    hipLaunchKernelGGL(kern, dim3(tiles * splits), dim3(64 * WAVES_M * WAVES_N), lds, st, A, W, M, N, K, splits, epi);
}

// One-wavefront tile with the K range split over KG wavefronts of the workgroup, each with its own LDS ring; the
// partial accumulators are added through LDS in group order (deterministic) and group 0 runs the epilogue.  For
// projections with few rows, few column tiles and an epilogue that needs whole sums (QKV + RoPE at 33-128 rows): a
// CU then keeps KG rings of weight and activation slices in flight instead of one.
template <int BM, int BN, int NSTAGE, int KG, class Epi>
__global__ void __launch_bounds__(64 * KG)
gemm_mfma_kgroups_kernel(const f16_t* __restrict__ A, const f16_t* __restrict__ W, int M, int N, int K, Epi epi) {
    using Tile = GemmTile<BM, BN, 1, 1, NSTAGE, Epi::BF>;
    constexpr int RING = (int)gemm_lds_bytes<BM, BN, NSTAGE>();
    constexpr int ACC_FLOATS = Tile::TM * Tile::TN * 16;               // per lane
    static_assert(ACC_FLOATS * 64 * 4 <= RING, "a group's partial tile must fit its ring");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    int tm, tn;
    tile_of_workgroup(blockIdx.x, tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);
    const int g = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
    const int per = K / GEMM_BK / KG;                                   // the launcher checks divisibility
    f32x16_t acc[Tile::TM][Tile::TN];
#pragma unroll
    for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
        for (int j = 0; j < Tile::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    Tile::run(A, W, M, K, tm * BM, tn * BN, g * per, (g + 1) * per, smem_raw + g * RING, acc);
    // a group's ring is read by that group only and all its reads have completed: it may hold the partial tile
    float* mine = reinterpret_cast<float*>(smem_raw + g * RING);
    if (g > 0) {
#pragma unroll
        for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
            for (int j = 0; j < Tile::TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) mine[((i * Tile::TN + j) * 16 + r) * 64 + lane] = acc[i][j][r];
    }
    __syncthreads();
    if (g == 0) {
        for (int o = 1; o < KG; ++o) {
            const float* theirs = reinterpret_cast<const float*>(smem_raw + o * RING);
#pragma unroll
            for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
                for (int j = 0; j < Tile::TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] += theirs[((i * Tile::TN + j) * 16 + r) * 64 + lane];
        }
        epi.template operator()<Tile::TM, Tile::TN>(acc, tm * BM, tn * BN, M, lane);
    }
}

template <int BM, int BN, int NSTAGE, int KG, class Epi>
static void launch_gemm_kgroups(const f16_t* A, const f16_t* W, int M, int N, int K, const Epi& epi, hipStream_t st) {
    if (M <= 0) return;
    auto kern = gemm_mfma_kgroups_kernel<BM, BN, NSTAGE, KG, Epi>;
    constexpr size_t lds = KG * gemm_lds_bytes<BM, BN, NSTAGE>();
    static_assert(lds <= 160 * 1024, "LDS of a compute unit");
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    const int tiles = ((M + BM - 1) / BM) * (N / BN);
    hipLaunchKernelGGL(kern, dim3(tiles), dim3(64 * KG), lds, st, A, W, M, N, K, epi);
}

// Big tiles on v_mfma_f32_16x16x32_f16 (gemm_core16.h): same tile shapes, workgroup order and epilogues.
template <int BM, int BN, int WAVES_M, int WAVES_N, class Epi>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N)
gemm_mfma16_kernel(const f16_t* __restrict__ A, const f16_t* __restrict__ W, int M, int N, int K, Epi epi) {
    using Tile = GemmTile16<BM, BN, WAVES_M, WAVES_N, Epi::BF, Epi::TRANSPOSE>;   // transposed accumulator blocks where the epilogue gains from them
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    int tm, tn;
    tile_of_workgroup(blockIdx.x, tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);
    f32x4_t acc[Tile::TM][Tile::TN];
#pragma unroll
    for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
        for (int j = 0; j < Tile::TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
    Tile::run(A, W, M, K, tm * BM, tn * BN, 0, K / GEMM_BK, smem_raw, acc);
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    if constexpr (Epi::USES_LDS)
        epi.template run_lds<Tile::TM, Tile::TN>(acc, tm * BM + wm * Tile::WTM, tn * BN + wn * Tile::WTN, M, lane,
                                                 reinterpret_cast<float*>(smem_raw + wave * Epi::template wave_lds_bytes<Tile::TM>()));
    else if constexpr (Epi::TRANSPOSE)
        epi.template operator()<Tile::TM, Tile::TN, Layout16T>(acc, tm * BM + wm * Tile::WTM, tn * BN + wn * Tile::WTN, M, lane);
    else
        epi.template operator()<Tile::TM, Tile::TN, Layout16>(acc, tm * BM + wm * Tile::WTM, tn * BN + wn * Tile::WTN, M, lane);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, class Epi>
static void launch_gemm16(const f16_t* A, const f16_t* W, int M, int N, int K, const Epi& epi, hipStream_t st) {
    if (M <= 0) return;
    auto kern = gemm_mfma16_kernel<BM, BN, WAVES_M, WAVES_N, Epi>;
    constexpr size_t ring = gemm_lds_bytes<BM, BN, 2>();
    constexpr size_t lds = [] {
        if constexpr (Epi::USES_LDS) {
            constexpr size_t stage = (size_t)WAVES_M * WAVES_N * Epi::template wave_lds_bytes<BM / WAVES_M / 16>();
            return stage > ring ? stage : ring;
        } else {
            return ring;
        }
    }();
    static_assert(lds <= 160 * 1024, "LDS of a compute unit");
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    const int tiles = ((M + BM - 1) / BM) * (N / BN);
    hipLaunchKernelGGL(kern, dim3(tiles), dim3(64 * WAVES_M * WAVES_N), lds, st, A, W, M, N, K, epi);
}

// Register-streaming kernel for at most 32 rows (gemm_stream.h); it reads the stream-layout copy of the
// weights.  A workgroup takes K/64/splits steps of 64; they must divide evenly over 8 or 4 wavefronts.
constexpr int STREAM_MAX_ROWS = 32;
template <int NW, int DEPTH, class Epi>
static void launch_stream_cfg(const f16_t* A, const void* Ws, int M, int N, int K, int splits, const Epi& epi, hipStream_t st) {
    auto kern = gemm_stream_kernel<NW, DEPTH, Epi::BF, Epi>;
    constexpr size_t lds = gemm_stream_lds_bytes<NW, DEPTH>();
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3((N / 64) * splits), dim3(64 * NW), lds, st, A, static_cast<const u32x4_t*>(Ws), M, N, K, splits, epi);
}
bool stream_layout_supported(int N, int K) { return N > 0 && K > 0 && N % 64 == 0 && K % 256 == 0; }
static bool stream_shape_ok(int M, int N, int K, int splits) {
    if (M <= 0 || M > STREAM_MAX_ROWS || !stream_layout_supported(N, K) || splits < 1) return false;
    if ((int64_t)M * K * 2 >= (int64_t)1 << 32) return false;
    const int KT = K / 64;
    return KT % splits == 0 && (KT / splits) % 4 == 0;
}
template <class Epi>
static bool try_launch_stream(const f16_t* A, const void* Ws, int M, int N, int K, int splits, const Epi& epi, hipStream_t st) {
    if (!Ws || !stream_shape_ok(M, N, K, splits)) return false;
    const int per = K / 64 / splits;
    const int nw = per % 8 == 0 ? 8 : 4;
    const int steps = per / nw;
    const int depth = steps % 4 == 0 ? 4 : steps % 3 == 0 ? 3 : steps % 2 == 0 ? 2 : 1;
#define SSD_STREAM_CASE(NW_, D_) if (nw == NW_ && depth == D_) { launch_stream_cfg<NW_, D_>(A, Ws, M, N, K, splits, epi, st); return true; }
    SSD_STREAM_CASE(8, 4) SSD_STREAM_CASE(8, 3) SSD_STREAM_CASE(8, 2) SSD_STREAM_CASE(8, 1)
    SSD_STREAM_CASE(4, 4) SSD_STREAM_CASE(4, 3) SSD_STREAM_CASE(4, 2) SSD_STREAM_CASE(4, 1)
#undef SSD_STREAM_CASE
    return false;
}
void launch_stream_layout(const uint16_t* w, void* out, int N, int K, hipStream_t st) {
    const int64_t units = (int64_t)N * K / 8;
    hipLaunchKernelGGL(stream_layout_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, st,
                       reinterpret_cast<const u32x4_t*>(w), static_cast<u32x4_t*>(out), N, K);
}

// Tile choice.  All candidates use eight wavefronts as 2 x 4 and a 256-wide tile (N is a multiple
// of 256 for every GEMM here) on the 16x16x32 matrix instruction; the tile height is picked per launch
// so that the number of tiles wastes as little of the last round over the 256 CUs as possible:
// cost = rounds * height / efficiency.
// With at most 128 rows the job is weight streaming and what counts is the number of weight bytes in
// flight: at most 32 rows go to the register-streaming kernel when the shape divides evenly; otherwise a
// skinny 128 x 64 tile (four wavefronts, each 32 rows x 64 columns) with a six-stage LDS ring
// (144 KB, five slices in flight), and for at most 32 rows a 32 x 64 tile of one wavefront, six stages
// of 12 KB, two workgroups per CU.
template <class Epi>
static void launch_skinny(const f16_t* A, const f16_t* W, const void* Ws, int M, int N, int K, int splits, const Epi& epi, hipStream_t st) {
    if (try_launch_stream(A, Ws, M, N, K, splits, epi, st)) return;
    // 33..128 rows: the launch should put a workgroup on every CU.  A projection with few column tiles and no K
    // split (QKV: 64-80 tiles) is cut into row tiles of 32 or 64 as well; the row tiles of a column slab then
    // read the same weights, which the L2 serves.
    const int col_tiles = (N / 64) * splits;
    if constexpr (!Epi::WANTS_SPLIT) {
        // whole sums wanted (no K split across workgroups) and few column tiles: split K inside the workgroup
        if (col_tiles <= 96 && M > 32 && (K / GEMM_BK) % 4 == 0 && K / GEMM_BK >= 16) {
            launch_gemm_kgroups<32, 64, 3, 4>(A, W, M, N, K, epi, st);
            return;
        }
    }
    if (M <= 32 || (col_tiles <= 96 && M > 32)) launch_gemm<32, 64, 1, 1, 6>(A, W, M, N, K, splits, epi, st);
    else if (col_tiles <= 160 && M > 64) launch_gemm<64, 64, 2, 1, 6>(A, W, M, N, K, splits, epi, st);
    else launch_gemm<128, 64, 4, 1, 6>(A, W, M, N, K, splits, epi, st);
}

template <class Epi>
static void launch_big(const f16_t* A, const f16_t* W, int M, int N, int K, const Epi& epi, hipStream_t st) {
    const int heights[3] = {256, 192, 128};
    const double eff[3] = {1.0, 0.97, 0.90};
    int best = 0;
    double best_cost = 1e30;
    for (int c = 0; c < 3; ++c) {
        const long tiles = (long)((M + heights[c] - 1) / heights[c]) * (N / 256);
        const double cost = (double)((tiles + 255) / 256) * heights[c] / eff[c];
        if (cost < best_cost - 1e-9) { best_cost = cost; best = c; }
    }
    if (best == 0) launch_gemm16<256, 256, 2, 4>(A, W, M, N, K, epi, st);
    else if (best == 1) launch_gemm16<192, 256, 2, 4>(A, W, M, N, K, epi, st);
    else launch_gemm16<128, 256, 2, 4>(A, W, M, N, K, epi, st);
}
template <class Epi>
static void launch_by_shape(const f16_t* A, const f16_t* W, const void* Ws, int M, int N, int K, const Epi& epi, hipStream_t st) {
    if (M <= SKINNY_MAX_ROWS) launch_skinny(A, W, Ws, M, N, K, 1, epi, st);
    else launch_big(A, W, M, N, K, epi, st);
}

void launch_gemm_qkv_rope(const uint16_t* A, const uint16_t* Wqkv_packed, const void* W_stream, uint16_t* qkv, const int32_t* pos,
                          const float* rope_tab, int M, int d_model, int d_q, int d_kv, float descale,
                          const int32_t* row_slot, uint16_t* kc, uint16_t* vc, const float* rope_rows, int32_t* flags,
                          bool bf16_ops, hipStream_t st) {
    const int N = d_q + 2 * d_kv;
    if (bf16_ops) {
        EpiQkvRope<true> epi{qkv, N, d_q + d_kv, descale, pos, reinterpret_cast<const float2*>(rope_tab), row_slot, kc, vc, d_q,
                             reinterpret_cast<const float2*>(rope_rows), flags};
        launch_by_shape(A, Wqkv_packed, W_stream, M, N, d_model, epi, st);
    } else {
        EpiQkvRope<false> epi{qkv, N, d_q + d_kv, descale, pos, reinterpret_cast<const float2*>(rope_tab), row_slot, kc, vc, d_q,
                              reinterpret_cast<const float2*>(rope_rows), flags};
        launch_by_shape(A, Wqkv_packed, W_stream, M, N, d_model, epi, st);
    }
}

int launch_gemm_qkv_partial(const uint16_t* A, const void* W_stream, float* part, int M, int d_model, int N, float descale,
                            bool bf16_ops, hipStream_t st) {
    if (!W_stream || M > STREAM_MAX_ROWS) return 0;
    int splits = 0;
    for (int s = SKINNY_MAX_SPLITS; s >= 2 && !splits; --s)                 // about one workgroup per CU
        if (stream_shape_ok(M, N, d_model, s) && (N / 64) * s <= 320) splits = s;
    if (!splits) return 0;
    if (bf16_ops) {
        EpiPartial<true> epi{part, N, (int64_t)M * N, descale};
        return try_launch_stream(A, W_stream, M, N, d_model, splits, epi, st) ? splits : 0;
    }
    EpiPartial<false> epi{part, N, (int64_t)M * N, descale};
    return try_launch_stream(A, W_stream, M, N, d_model, splits, epi, st) ? splits : 0;
}

int gemm_residual_splits(int M, int N, int K, bool have_stream) {
    if (M > SKINNY_MAX_ROWS) return 1;
    if (have_stream && M <= STREAM_MAX_ROWS) {
        // register-streaming kernel: the most splits (workgroups) whose K range still divides over 4 wavefronts
        for (int s = SKINNY_MAX_SPLITS; s >= 2; --s)
            if (stream_shape_ok(M, N, K, s) && (N / 64) * s <= 512) return s;
    }
    int splits = 1;
    while (splits < SKINNY_MAX_SPLITS && (N / 64) * splits < 256 && K / GEMM_BK / (splits * 2) >= 4) splits *= 2;
    return splits;
}

// x += A W^T.  With few rows the K range is split over several workgroups per tile to get enough
// of them for weight streaming; the splits land in `partials` ([splits][M][N] fp32) and the caller
// hands them to the next RMSNorm, which adds them to x in a fixed order.  Returns the split count
// (1: x has been updated in place).
template <bool BF>
static int gemm_residual_impl(const uint16_t* A, const uint16_t* W, const void* W_stream, float* x, float* partials, int M, int N, int K,
                              float descale, hipStream_t st) {
    const int splits = gemm_residual_splits(M, N, K, W_stream != nullptr);
    if (splits > 1) {
        EpiPartial<BF> epi{partials, N, (int64_t)M * N, descale};
        launch_skinny(A, W, W_stream, M, N, K, splits, epi, st);
        return splits;
    }
    if (M > SKINNY_MAX_ROWS) launch_big(A, W, M, N, K, EpiResidualLds<BF>{x, N, descale}, st);
    else launch_skinny(A, W, W_stream, M, N, K, 1, EpiResidual<BF>{x, N, descale}, st);
    return 1;
}
int launch_gemm_residual(const uint16_t* A, const uint16_t* W, const void* W_stream, float* x, float* partials, int M, int N, int K,
                         float descale, bool bf16_ops, hipStream_t st) {
    return bf16_ops ? gemm_residual_impl<true>(A, W, W_stream, x, partials, M, N, K, descale, st)
                    : gemm_residual_impl<false>(A, W, W_stream, x, partials, M, N, K, descale, st);
}

void launch_gemm_scores_values(const uint16_t* A, const uint16_t* W, float* scores, uint16_t* vals, int M, int N, int K, int d_h,
                               int32_t* flags, bool bf16_ops, hipStream_t st) {
    if (bf16_ops) launch_by_shape(A, W, nullptr, M, N, K, EpiScoresValues<true>{scores, vals, d_h, flags}, st);
    else launch_by_shape(A, W, nullptr, M, N, K, EpiScoresValues<false>{scores, vals, d_h, flags}, st);
}
void launch_gemm_store_16(const uint16_t* A, const uint16_t* W, uint16_t* C, int M, int N, int K, bool bf16_ops, hipStream_t st) {
    if (bf16_ops) launch_by_shape(A, W, nullptr, M, N, K, EpiStore16<true>{C, N}, st);
    else launch_by_shape(A, W, nullptr, M, N, K, EpiStore16<false>{C, N}, st);
}

void launch_gemm_swiglu(const uint16_t* A, const uint16_t* Wgu_packed, const void* W_stream, uint16_t* h, int M, int d_ff, int K,
                        float descale, int32_t* flags, bool bf16_ops, hipStream_t st) {
    if (bf16_ops) {
        EpiSwiglu<true> epi{h, d_ff, descale, flags};
        launch_by_shape(A, Wgu_packed, W_stream, M, 2 * d_ff, K, epi, st);
    } else {
        EpiSwiglu<false> epi{h, d_ff, descale, flags};
        launch_by_shape(A, Wgu_packed, W_stream, M, 2 * d_ff, K, epi, st);
    }
}

}  // namespace ssd
