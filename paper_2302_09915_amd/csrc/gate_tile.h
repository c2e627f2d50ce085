// Tile code of the gate (scores on the matrix cores, softmax, top-k, load statistics) shared by the
// translation units that instantiate it for one element type each (gate_bf16.hip, gate_f16.hip,
// gate_f32.hip) and by gate.hip (selection on given scores, finalize, host entry points).
#pragma once

#include <climits>
#include <type_traits>

#include "internal.h"

namespace tamoe {


typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kKC = 64;                 // K elements per chunk (128 bytes of a bf16 row)
constexpr int kLdsRow = kKC * 2 + 16;   // padded LDS row: 16-byte reads of 32 rows stay conflict-free

constexpr int kTileRow = 36;            // floats per row of a wavefront's 32 x 32 logits tile in LDS

__device__ __forceinline__ int expert_of(int nb, int v, int half) {
    return nb * 32 + ((v >> 2) << 3) + (half << 2) + (v & 3);
}

// value of lane (lane ^ MASK), MASK < 32.  Masks 1, 2, 4, 8 stay inside a row of 16 lanes and are
// composed from the data-parallel lane permutations of the vector unit, which cost an instruction
// or two and no wait: 1 and 2 are quad permutations, 4 = reverse within 8 lanes then reverse
// within 4, 8 = reverse within 16 then reverse within 8.  Mask 16 goes through the LDS crossbar
// (ds_swizzle), whose result has to be waited for like an LDS read.
template <int MASK>
__device__ __forceinline__ float swizzle_xor(float v) {
    const int x = __float_as_int(v);
    if constexpr (MASK == 1) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0xB1, 0xf, 0xf, true));    // quad_perm [1,0,3,2]
    } else if constexpr (MASK == 2) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x4E, 0xf, 0xf, true));    // quad_perm [2,3,0,1]
    } else if constexpr (MASK == 4) {
        const int h = __builtin_amdgcn_update_dpp(0, x, 0x141, 0xf, 0xf, true);            // row_half_mirror: i ^ 7
        return __int_as_float(__builtin_amdgcn_update_dpp(0, h, 0x1B, 0xf, 0xf, true));    // quad_perm [3,2,1,0]: ^ 3
    } else if constexpr (MASK == 8) {
        const int r = __builtin_amdgcn_update_dpp(0, x, 0x140, 0xf, 0xf, true);            // row_mirror: i ^ 15
        return __int_as_float(__builtin_amdgcn_update_dpp(0, r, 0x141, 0xf, 0xf, true));   // row_half_mirror: ^ 7
    } else {
        return __int_as_float(__builtin_amdgcn_ds_swizzle(x, (MASK << 10) | 0x1f));
    }
}

// One level of a transposed butterfly over the 32 token lanes: lanes that differ in bit S
// exchange half of their SIZE values and add, so that each keeps SIZE/2 partial sums (those
// whose index has bit 0 equal to the lane's bit S).  After log2 levels a lane holds the complete
// sums of SIZE/32 indices instead of every lane holding all of them: SIZE-1 exchanges instead of
// 5*SIZE.  The summation tree is fixed, so the result is the same on every run.
template <int SIZE, int S>
__device__ __forceinline__ void transpose_reduce(float (&a)[SIZE], int lane) {
    if constexpr (S < 5) {
        if constexpr (SIZE >= 2) {
            const bool up = (lane >> S) & 1;
            float nxt[SIZE / 2];
#pragma unroll
            for (int i = 0; i < SIZE / 2; ++i) {
                const float keep = up ? a[2 * i + 1] : a[2 * i];
                const float send = up ? a[2 * i] : a[2 * i + 1];
                nxt[i] = keep + swizzle_xor<(1 << S)>(send);
            }
            transpose_reduce<SIZE / 2, S + 1>(nxt, lane);
#pragma unroll
            for (int i = 0; i < SIZE / 2; ++i) a[i] = nxt[i];
        } else {
            a[0] += swizzle_xor<(1 << S)>(a[0]);
            transpose_reduce<SIZE, S + 1>(a, lane);
        }
    }
}

// (value, index) order of the selection: higher score first, equal scores to the lower index
__device__ __forceinline__ bool ranks_before(float av, int ai, float bv, int bi) {
    return av > bv || (av == bv && ai < bi);
}

// Writes the 32-token score tile of a wavefront to a row-major [S][N] matrix.  The accumulator
// layout has one token per lane, so a direct store would write 16 bytes per lane, 512 bytes apart.
// Each 32-expert block goes through a 32 x 32 tile of LDS owned by the wavefront (rows padded to 36
// floats) and leaves as whole 128-byte row segments: eight lanes per row, eight rows per store
// instruction.
template <int NB>
__device__ __forceinline__ void store_logits_tile(const float (&sc)[NB][16], int lane, int64_t token, int N,
                                                  float* __restrict__ logits, float* tile, int64_t S) {
    const int half = lane >> 5;
    const int r = lane & 31;
    const int64_t token0 = token - r;
    const bool vec = (N & 3) == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<float4*>(&tile[r * kTileRow + 8 * q + 4 * half]) =
                make_float4(sc[nb][4 * q], sc[nb][4 * q + 1], sc[nb][4 * q + 2], sc[nb][4 * q + 3]);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rr = i * 8 + (lane >> 3);
            const int e = nb * 32 + (lane & 7) * 4;
            const float4 v4 = *reinterpret_cast<const float4*>(&tile[rr * kTileRow + (lane & 7) * 4]);
            const int64_t tg = token0 + rr;
            if (tg < S && e < N) {
                float* dst = logits + tg * N + e;
                if (vec) {
                    // streamed: 32 MiB of dirty lines left in L2 would be written back at the
                    // end of the kernel, after the last wavefront, with nothing to overlap
                    typedef float f32x4 __attribute__((ext_vector_type(4)));
                    const f32x4 o = {v4.x, v4.y, v4.z, v4.w};
                    __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(dst));
                } else {
                    dst[0] = v4.x;
                    if (e + 1 < N) dst[1] = v4.y;
                    if (e + 2 < N) dst[2] = v4.z;
                    if (e + 3 < N) dst[3] = v4.w;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
}

// The reverse of store_logits_tile: reads the 32-token score tile of a wavefront from a row-major
// [S][N] matrix (the sum of n_parts matrices part_stride floats apart, added in ascending order) as
// whole 128-byte row segments and hands it over in the accumulator layout through the wavefront's
// LDS tile.  Entries beyond S or N come back as -infinity.
template <int NB>
__device__ __forceinline__ void load_logits_tile(float (&sc)[NB][16], int lane, int64_t token, int N,
                                                 const float* __restrict__ logits, int n_parts, size_t part_stride,
                                                 float* tile, int64_t S) {
    const int half = lane >> 5;
    const int r = lane & 31;
    const int64_t token0 = token - r;
    const bool vec = (N & 3) == 0 && (part_stride & 3) == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0;
    static_assert(kMaxKSplits <= 8, "the parts of a block are held in registers");
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        // every load of the block is issued before the first sum: a loop that adds each part as it
        // arrives pays one memory round trip per part
        float4 part[4][kMaxKSplits];
        bool inside[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rr = i * 8 + (lane >> 3);
            const int e = nb * 32 + (lane & 7) * 4;
            const int64_t tg = token0 + rr;
            inside[i] = tg < S && e < N;
            const float* src = logits + (inside[i] ? tg * N + e : 0);
#pragma unroll
            for (int p = 0; p < kMaxKSplits; ++p) {
                part[i][p] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (inside[i] && p < n_parts) {
                    if (vec) {
                        part[i][p] = *reinterpret_cast<const float4*>(src + p * part_stride);
                    } else {
                        part[i][p].x = src[p * part_stride];
                        if (e + 1 < N) part[i][p].y = src[p * part_stride + 1];
                        if (e + 2 < N) part[i][p].z = src[p * part_stride + 2];
                        if (e + 3 < N) part[i][p].w = src[p * part_stride + 3];
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rr = i * 8 + (lane >> 3);
            const int e = nb * 32 + (lane & 7) * 4;
            float4 v4 = part[i][0];
#pragma unroll
            for (int p = 1; p < kMaxKSplits; ++p) {  // ascending parts; absent parts are +0
                v4.x += part[i][p].x;
                v4.y += part[i][p].y;
                v4.z += part[i][p].z;
                v4.w += part[i][p].w;
            }
            if (!inside[i]) v4 = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (inside[i] && e + 1 >= N) v4.y = -INFINITY;
            if (inside[i] && e + 2 >= N) v4.z = -INFINITY;
            if (inside[i] && e + 3 >= N) v4.w = -INFINITY;
            *reinterpret_cast<float4*>(&tile[rr * kTileRow + (lane & 7) * 4]) = v4;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 v4 = *reinterpret_cast<const float4*>(&tile[r * kTileRow + 8 * q + 4 * half]);
            sc[nb][4 * q] = v4.x;
            sc[nb][4 * q + 1] = v4.y;
            sc[nb][4 * q + 2] = v4.z;
            sc[nb][4 * q + 3] = v4.w;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
}

// What a lane keeps of its token's selection for the block-wide step that follows (finish_block).
struct TokenPairs {
    int expert[TAMOE_MAX_K];   // selected expert of choice j, -1 if none (token beyond S, no valid score)
    int rank[TAMOE_MAX_K];     // earlier tokens of this wavefront with the same expert at choice j
};

// Selection on a 32-token tile held in the accumulator layout described above.
// sc[nb][v]: score of expert_of(nb, v, lane>>5) for token `token` (lane & 31 within the tile).
// m_wave: LDS, [>= NB*32] floats owned by this wavefront; pairs_wave: LDS, [>= k*NB*32] ints owned by this
// wavefront, receives the number of its tokens that chose expert e at choice j in [j*NB*32 + e].
template <int NB>
__device__ __forceinline__ void select_tile(float (&sc)[NB][16], int lane, int64_t token, bool token_ok, int N,
                                            int k, float* __restrict__ logits, int32_t* __restrict__ topk_idx,
                                            float* __restrict__ topk_w, float* m_wave, int32_t* pairs_wave,
                                            float* tile, int64_t S, TokenPairs& tp) {
    const int half = lane >> 5;
    constexpr int ROWS = NB * 32;
    for (int q = lane; q < k * ROWS; q += 64) pairs_wave[q] = 0;
    if (logits != nullptr) store_logits_tile<NB>(sc, lane, token, N, logits, tile, S);
    if (N < NB * 32) {  // uniform
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (expert_of(nb, v, half) >= N) sc[nb][v] = -INFINITY;
    }

    float sel_v[TAMOE_MAX_K];
    int sel_i[TAMOE_MAX_K];
#pragma unroll
    for (int j = 0; j < TAMOE_MAX_K; ++j) {
        sel_v[j] = -INFINITY;
        sel_i[j] = -1;
    }
    if (k <= 2) {
        // one pass keeps the best two of the lane (values are visited in ascending expert index,
        // so a strict '>' leaves equal scores with the lower index), then the two halves merge
        float b1v = -INFINITY, b2v = -INFINITY;
        int b1i = INT_MAX, b2i = INT_MAX;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float a = sc[nb][v];
                const int e = expert_of(nb, v, half);
                const bool g1 = a > b1v, g2 = a > b2v;
                b2v = g1 ? b1v : (g2 ? a : b2v);
                b2i = g1 ? b1i : (g2 ? e : b2i);
                b1v = g1 ? a : b1v;
                b1i = g1 ? e : b1i;
            }
        const float o1v = __shfl_xor(b1v, 32), o2v = __shfl_xor(b2v, 32);
        const int o1i = __shfl_xor(b1i, 32), o2i = __shfl_xor(b2i, 32);
        const bool mine = ranks_before(b1v, b1i, o1v, o1i);
        sel_v[0] = mine ? b1v : o1v;
        sel_i[0] = mine ? b1i : o1i;
        // runner-up: the loser of the two leaders against the winner's own second
        const float cv = mine ? o1v : b1v, dv = mine ? b2v : o2v;
        const int ci = mine ? o1i : b1i, di = mine ? b2i : o2i;
        const bool c_first = ranks_before(cv, ci, dv, di);
        sel_v[1] = c_first ? cv : dv;
        sel_i[1] = c_first ? ci : di;
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (sel_i[j] == INT_MAX) sel_i[j] = -1;
    } else {
        // k passes; each takes the best score that comes after the previous pick in the order
        // (score descending, expert index ascending)
        float last_v = INFINITY;
        int last_i = -1;
#pragma unroll
        for (int j = 0; j < TAMOE_MAX_K; ++j) {
            if (j < k) {
                float bv = -INFINITY;
                int bi = INT_MAX;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float a = sc[nb][v];
                        const int e = expert_of(nb, v, half);
                        const bool after = (a < last_v) || (a == last_v && e > last_i);
                        if (after && a > bv) {
                            bv = a;
                            bi = e;
                        }
                    }
                const float ov = __shfl_xor(bv, 32);
                const int oi = __shfl_xor(bi, 32);
                if (ranks_before(ov, oi, bv, bi)) {
                    bv = ov;
                    bi = oi;
                }
                last_v = bv;
                last_i = bi;
                sel_v[j] = bv;
                sel_i[j] = bi == INT_MAX ? -1 : bi;
            }
        }
    }

    // softmax: the first pick is the row maximum.  exp(l - max) = 2^(l*log2(e) - max*log2(e)) on the
    // hardware exponential, one fused multiply-add per score.  The rounding of the product max*log2(e)
    // shifts every exponent of the row by the same amount and cancels in the quotient; what is left is
    // the rounding of the fused operation, below 1e-5 relative for differences down to -100.
    constexpr float kLog2e = 1.44269504088896340736f;
    const float mx = sel_v[0];
    const float shift = -(mx * kLog2e);
    float part = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            sc[nb][v] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[nb][v], kLog2e, shift));
            part += sc[nb][v];
        }
    const float den = part + __shfl_xor(part, 32);
    const float inv = 1.0f / den;

    if (half == 0 && token_ok) {
#pragma unroll
        for (int j = 0; j < TAMOE_MAX_K; ++j) {
            if (j < k) {
                topk_idx[token * k + j] = sel_i[j];
                topk_w[token * k + j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sel_v[j], kLog2e, shift)) / den;
            }
        }
    }

    // Pairs per (choice, expert) of this wavefront, and for every pair the number of earlier tokens of
    // the wavefront with the same expert at the same choice (tokens are in lane order): what the
    // capacity-limited slot assignment needs from the gate.  Both halves hold the same selection.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the zeroes above before the atomics
    const int r_tok = lane & 31;
    constexpr int kExpertBits = NB == 1 ? 5 : NB == 2 ? 6 : 7;   // experts < NB * 32
#pragma unroll
    for (int j = 0; j < TAMOE_MAX_K; ++j) {
        tp.expert[j] = -1;
        tp.rank[j] = 0;
        if (j < k) {
            const int mine = (token_ok && sel_i[j] >= 0 && sel_i[j] < N) ? sel_i[j] : -1;
            // lanes (of the 32 token lanes; the upper half holds copies) with the same expert: one ballot
            // per bit of the expert index, and the lane keeps the mask or its complement
            uint32_t same = (uint32_t)__ballot(mine >= 0);
#pragma unroll
            for (int b = 0; b < kExpertBits; ++b) {
                const bool bit = (mine >> b) & 1;
                const uint32_t with_bit = (uint32_t)__ballot(bit);
                same &= bit ? with_bit : ~with_bit;
            }
            const int rank = __popc(same & ((1u << r_tok) - 1u));
            tp.expert[j] = mine;
            tp.rank[j] = rank;
            if (half == 0 && mine >= 0) atomicAdd(&pairs_wave[j * ROWS + mine], 1);
        }
    }

    // per-expert probability sums over the 32 tokens of the tile
    constexpr int V = NB * 16;
    float p[V];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) p[nb * 16 + v] = token_ok ? sc[nb][v] * inv : 0.f;
    transpose_reduce<V, 0>(p, lane);
    // lane r now holds the sums of the value indices q = r + 32*i (i < V/32), or, when V < 32, of
    // q = r mod V (in every lane that shares it)
    const int r = lane & 31;
    if constexpr (V >= 32) {
#pragma unroll
        for (int i = 0; i < V / 32; ++i) {
            const int q = r + 32 * i;
            const int e = expert_of(q >> 4, q & 15, half);
            if (e < N) m_wave[e] = p[i];
        }
    } else {
        const int e = expert_of(0, r & 15, half);
        if (r < 16 && e < N) m_wave[e] = p[0];
    }
}

// Block-wide end of the selection: per-workgroup probability sums and pair counts, and every pair's
// position among the pairs of its workgroup (pairs of earlier wavefronts + rank inside its own).
// pairs: LDS, wavefront w owns [w*pairs_stride, + k*NB*32).
template <int NB, int WAVES>
__device__ __forceinline__ void finish_block(const float (*m_w)[NB * 32], const int32_t* pairs, int pairs_stride,
                                             const TokenPairs& tp, int lane, int wave, int64_t token, bool token_ok,
                                             int N, int k, const GateStats& gs) {
    constexpr int ROWS = NB * 32;
    __syncthreads();
    if ((lane >> 5) == 0 && token_ok) {
#pragma unroll
        for (int j = 0; j < TAMOE_MAX_K; ++j) {
            if (j < k) {
                int before = 0;
                if (tp.expert[j] >= 0) {
#pragma unroll
                    for (int w = 0; w < WAVES; ++w)
                        if (w < wave) before += pairs[w * pairs_stride + j * ROWS + tp.expert[j]];
                }
                gs.local_pos[token * k + j] = before + tp.rank[j];
            }
        }
    }
    for (int e = threadIdx.x; e < N; e += WAVES * 64) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) s += m_w[w][e];
        gs.m_part[(size_t)e * gs.n_blocks + blockIdx.x] = s;
    }
    for (int q = threadIdx.x; q < k * ROWS; q += WAVES * 64) {
        const int j = q / ROWS, e = q - j * ROWS;
        if (e < N) {
            int32_t c = 0;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) c += pairs[w * pairs_stride + q];
            gs.tile_pairs[(size_t)e * gs.pitch + (size_t)j * gs.n_blocks + blockIdx.x] = c;
        }
    }
}

// KTAIL: d is not a multiple of the 64-element K chunk (the last chunk is partly out of range).
// ET: element type (TAMOE_BF16, TAMOE_F16, TAMOE_F32).  Rows are addressed in 2-byte units whatever the
// type (d counts those units: twice the hidden size for fp32), a K chunk is 128 bytes of a row, and
// tiles move as 16-byte pieces; only the MFMA differs.  For fp32 a piece holds four values and feeds
// four v_mfma_f32_32x32x2_f32 (fp32 operands, fp32 accumulation) instead of one 32x32x16.
// SPLIT: the workgroups of grid row blockIdx.y take the blockIdx.y-th share of the K chunks and write
// their partial scores to logits + blockIdx.y * S * N instead of selecting; a select_kernel adds the
// shares.  For batches so small that whole-K token tiles would leave most SIMDs idle.
template <int NB, int WAVES, bool KTAIL, int ET, bool SPLIT = false>
__device__ __forceinline__ void gate_mfma_tile(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, int64_t S, int d, int N, int k,
    float* __restrict__ logits, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, const GateStats gs) {
    constexpr int T = WAVES * 64;
    constexpr int ROWS = NB * 32;        // expert rows of the W tile
    constexpr int TOK = WAVES * 32;      // token rows of the x tile
    constexpr int WU = ROWS * 8 / T;     // 16-byte pieces of the W chunk per thread
    constexpr int XU = TOK * 8 / T;      // 16-byte pieces of the x chunk per thread (= 4)
    static_assert(ROWS * 8 % T == 0 && XU == 4, "tiles must split evenly over the threads");
    __shared__ __attribute__((aligned(16))) unsigned char w_lds[2][ROWS * kLdsRow];
    __shared__ __attribute__((aligned(16))) unsigned char x_lds[2][TOK * kLdsRow];
    __shared__ float m_w[WAVES][ROWS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int r = lane & 31;
    const int half = lane >> 5;
    const int64_t tile0 = (int64_t)blockIdx.x * TOK;
    const int64_t token = tile0 + wave * 32 + r;
    const bool token_ok = token < S;

    for (int q = tid; q < WAVES * ROWS; q += T) (&m_w[0][0])[q] = 0.f;

    const int all_chunks = (d + kKC - 1) / kKC;
    int c_begin = 0, n_chunks = all_chunks;   // this workgroup's chunks: c_begin .. c_begin + n_chunks - 1
    if constexpr (SPLIT) {
        const int per = (all_chunks + (int)gridDim.y - 1) / (int)gridDim.y;
        c_begin = (int)blockIdx.y * per;
        n_chunks = all_chunks - c_begin < per ? all_chunks - c_begin : per;
        if (n_chunks < 0) n_chunks = 0;       // a share past the end: its partial scores are zero
    }
    const int n_addr = n_chunks > 0 ? n_chunks : 1;  // for addresses only
    const vec16 zero = {0u, 0u, 0u, 0u};
    // Rows of x are a power-of-two pitch apart, so the same K chunk of every row falls into the
    // same few memory channels.  Workgroups would all walk K in step and queue on those channels;
    // instead workgroup b starts its walk at chunk (17 b) mod n_chunks and wraps around.  (A dot
    // product may be summed in any order; a token's scores depend on the order only in rounding.)
    const int rot = (int)(((int64_t)blockIdx.x * 17) % n_addr);

    // Both tiles go global -> registers -> LDS -> MFMA operands.  Unit u of a thread is the
    // 16-byte piece (unit & 7) of tile row (unit >> 3), unit = tid + u * T: eight consecutive
    // lanes read one 128-byte line, so every global load instruction is fully coalesced (loading
    // the x operand straight into its MFMA lane layout would touch 32 lines per instruction and
    // stall the address unit on the L1 tag rate).
    // Every load is unconditional so that the loop body is straight-line code and the loads of
    // later chunks stay in flight across the MFMAs of the current one:
    //  - a token row beyond S reads row S-1 (its results are discarded);
    //  - an expert row beyond N reads row N-1 (its scores are masked before the selection);
    //  - a chunk index beyond the last chunk reads the last chunk again (never consumed);
    //  - with KTAIL, a 16-byte piece beyond d reads the last piece of the row; the W piece is then
    //    replaced by zeros, so the finite x values it meets contribute nothing.
    const uint16_t* wsrc[WU];
    const uint16_t* xsrc[XU];
    int lds_off_w[WU], lds_off_x[XU];
#pragma unroll
    for (int u = 0; u < WU; ++u) {
        const int unit = tid + u * T;
        const int row = unit >> 3;
        wsrc[u] = w + (size_t)(row < N ? row : N - 1) * d + (unit & 7) * 8;
        lds_off_w[u] = row * kLdsRow + (unit & 7) * 16;
    }
#pragma unroll
    for (int u = 0; u < XU; ++u) {
        const int unit = tid + u * T;
        const int row = unit >> 3;
        const int64_t t = tile0 + row;
        xsrc[u] = x + (size_t)(t < S ? t : S - 1) * d + (unit & 7) * 8;
        lds_off_x[u] = row * kLdsRow + (unit & 7) * 16;
    }
    const int piece = tid & 7;  // (unit & 7) is the same for every unit of a thread: T % 8 == 0

    auto chunk_at = [&](int step) {  // K chunk visited at pipeline step `step` (clamped past the end)
        int c = (step < n_addr ? step : n_addr - 1) + rot;
        c = (c >= n_addr ? c - n_addr : c) + c_begin;
        return c < all_chunks ? c : all_chunks - 1;
    };
    auto load_w = [&](int kc, vec16 (&dst)[WU]) {
        kc = chunk_at(kc);
        int k0 = kc * kKC;
        bool in = true;
        if constexpr (KTAIL) {
            in = k0 + piece * 8 < d;
            k0 = in ? k0 : d - 8 - piece * 8;
        }
#pragma unroll
        for (int u = 0; u < WU; ++u) {
            const vec16 t = *reinterpret_cast<const vec16*>(wsrc[u] + k0);
            dst[u] = (!KTAIL || in) ? t : zero;
        }
    };
    // x is read with ordinary loads, not streaming (nontemporal) ones, although the gate uses every
    // byte once: an ordinary load leaves the line in the 256 MB last-level cache, and the dispatch
    // reads x again right after the gate.  On a 512 MiB x the scatter gets about half of its reads
    // from that cache (its kernel 307 -> 256 us) for 5 us more here.
    auto load_x = [&](int kc, vec16 (&dst)[XU]) {
        kc = chunk_at(kc);
        int k0 = kc * kKC;
        if constexpr (KTAIL) k0 = (k0 + piece * 8 < d) ? k0 : d - 8 - piece * 8;
#pragma unroll
        for (int u = 0; u < XU; ++u) dst[u] = *reinterpret_cast<const vec16*>(xsrc[u] + k0);
    };
    auto store_w = [&](const vec16 (&src)[WU], int buf) {
#pragma unroll
        for (int u = 0; u < WU; ++u) *reinterpret_cast<vec16*>(&w_lds[buf][lds_off_w[u]]) = src[u];
    };
    auto store_x = [&](const vec16 (&src)[XU], int buf) {
#pragma unroll
        for (int u = 0; u < XU; ++u) *reinterpret_cast<vec16*>(&x_lds[buf][lds_off_x[u]]) = src[u];
    };

    f32x16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0.f;

    // MFMA operands of lane (r, half) for K step i of a chunk: the 16-byte piece 4*half + i of
    // W row nb*32 + r (A) and of x row wave*32 + r (B).  Any order of the K pieces works as long
    // as A and B use the same one.
    auto compute = [&](int buf) {
        const unsigned char* wl = &w_lds[buf][r * kLdsRow + half * 64];
        const unsigned char* xl = &x_lds[buf][(wave * 32 + r) * kLdsRow + half * 64];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const vec16 b = *reinterpret_cast<const vec16*>(xl + i * 16);
            if constexpr (ET == TAMOE_F32) {
                vec16 a[NB];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) a[nb] = *reinterpret_cast<const vec16*>(wl + nb * 32 * kLdsRow + i * 16);
                // consecutive MFMAs go to different accumulators
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[nb][j]), __uint_as_float(b[j]),
                                                                       acc[nb], 0, 0, 0);
            } else {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const vec16 a = *reinterpret_cast<const vec16*>(wl + nb * 32 * kLdsRow + i * 16);
                    if constexpr (ET == TAMOE_F16)
                        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                                          __builtin_bit_cast(f16x8, b), acc[nb], 0, 0, 0);
                    else
                        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                                           __builtin_bit_cast(bf16x8, b), acc[nb], 0, 0, 0);
                }
            }
        }
    };

    // Software pipeline.  Chunk c of both tiles is requested four iterations before it is used
    // (four register sets each; two for W when a thread owns more than four pieces of it) and is
    // copied to the LDS double buffer one iteration before use.  Loads complete in order, so at
    // the point where an iteration waits for chunk c+1 the chunks c+2 .. c+4 are still in flight:
    // about 12 KiB of x per wavefront, which is what covers the HBM latency.
    constexpr int DW = WU <= 4 ? 4 : 2;
    vec16 wr[DW][WU];
    vec16 xr[4][XU];
    auto stage = [&](int kc, auto U) {   // u = kc mod 4, a compile-time constant at each call
        constexpr int u = decltype(U)::value;
        load_w(kc + DW, wr[u % DW]);
        load_x(kc + 4, xr[u]);
        __builtin_amdgcn_sched_barrier(0);  // keep the requests ahead of the MFMAs
        compute(u & 1);
        store_w(wr[(u + 1) % DW], (u + 1) & 1);
        store_x(xr[(u + 1) & 3], (u + 1) & 1);
        __syncthreads();
    };

#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if (c < DW) load_w(c, wr[c]);
        load_x(c, xr[c]);
    }
    store_w(wr[0], 0);
    store_x(xr[0], 0);
    __syncthreads();

    const int n_groups = n_chunks >> 2;
    for (int g = 0; g < n_groups; ++g) {
        stage(4 * g + 0, std::integral_constant<int, 0>{});
        stage(4 * g + 1, std::integral_constant<int, 1>{});
        stage(4 * g + 2, std::integral_constant<int, 2>{});
        stage(4 * g + 3, std::integral_constant<int, 3>{});
    }
    const int rem = n_chunks & 3;  // uniform
    if (rem > 0) stage(4 * n_groups + 0, std::integral_constant<int, 0>{});
    if (rem > 1) stage(4 * n_groups + 1, std::integral_constant<int, 1>{});
    if (rem > 2) stage(4 * n_groups + 2, std::integral_constant<int, 2>{});

    float sc[NB][16];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) sc[nb][v] = acc[nb][v];
    // the K loop is over (its last stage ended with a barrier): x_lds is free, 9216 bytes per wavefront:
    // the logits tile first, the wavefront's pair counts (at most 8 choices x 128 experts) behind it
    constexpr int kWaveWords = 2 * 32 * kLdsRow / 4;
    constexpr int kTileWords = 32 * kTileRow;
    static_assert(kWaveWords >= kTileWords + TAMOE_MAX_K * TAMOE_MAX_EXPERTS,
                  "logits tile and pair counts must fit the wavefront's share of x_lds");
    float* tile = reinterpret_cast<float*>(&x_lds[0][0]) + wave * kWaveWords;
    if constexpr (SPLIT) {
        store_logits_tile<NB>(sc, lane, token, N, logits + (size_t)blockIdx.y * (size_t)S * N, tile, S);
    } else {
        int32_t* pairs = reinterpret_cast<int32_t*>(&x_lds[0][0]) + kTileWords;
        TokenPairs tp;
        select_tile<NB>(sc, lane, token, token_ok, N, k, logits, topk_idx, topk_w, m_w[wave],
                        pairs + wave * kWaveWords, tile, S, tp);
        finish_block<NB, WAVES>(m_w, pairs, kWaveWords, tp, lane, wave, token, token_ok, N, k, gs);
    }
}

#define TAMOE_GATE_ARGS                                                                                     \
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ w, int64_t S, int d, int N, int k,         \
        float *__restrict__ logits, int32_t *__restrict__ topk_idx, float *__restrict__ topk_w,             \
        const GateStats gs

template <int NB, int WAVES, bool KTAIL>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu((NB == 4 && WAVES < 4) ? 1 : 2)))
void gate_bf16_kernel(TAMOE_GATE_ARGS) {
    gate_mfma_tile<NB, WAVES, KTAIL, TAMOE_BF16>(x, w, S, d, N, k, logits, topk_idx, topk_w, gs);
}

template <int NB, int WAVES, bool KTAIL>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu((NB == 4 && WAVES < 4) ? 1 : 2)))
void gate_f16_kernel(TAMOE_GATE_ARGS) {
    gate_mfma_tile<NB, WAVES, KTAIL, TAMOE_F16>(x, w, S, d, N, k, logits, topk_idx, topk_w, gs);
}

// fp32 storage: x and w point to floats, d counts 2-byte units (twice the hidden size)
template <int NB, int WAVES, bool KTAIL>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu((NB == 4 && WAVES < 4) ? 1 : 2)))
void gate_f32_kernel(TAMOE_GATE_ARGS) {
    gate_mfma_tile<NB, WAVES, KTAIL, TAMOE_F32>(x, w, S, d, N, k, logits, topk_idx, topk_w, gs);
}

// fp32 storage, small batches: one wavefront per workgroup, K split over grid rows (see SPLIT above)
template <int NB, bool KTAIL>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(1)))
void gate_f32_split_kernel(TAMOE_GATE_ARGS) {
    gate_mfma_tile<NB, 1, KTAIL, TAMOE_F32, true>(x, w, S, d, N, k, logits, topk_idx, topk_w, gs);
}
#undef TAMOE_GATE_ARGS

// ---- launches (host) ------------------------------------------------------------------------------

inline const char* gate_kernel_name(int et) {
    return et == TAMOE_F32 ? "gate_f32_kernel" : et == TAMOE_F16 ? "gate_f16_kernel" : "gate_bf16_kernel";
}

template <int NB, int ET>
inline void launch_gate_mfma(int waves, int64_t blocks, hipStream_t st, const uint16_t* x, const uint16_t* w,
                             int64_t S, int d, int N, int k, float* logits, int32_t* topk_idx, float* topk_w,
                             const GateStats& gs) {
    const dim3 grid((unsigned)blocks);
    const bool ktail = d % kKC != 0;
    TraceScope tr(gate_kernel_name(ET), st);
#define TAMOE_GATE_LAUNCH(WV, KT)                                                                                  \
    do {                                                                                                           \
        if constexpr (ET == TAMOE_F32)                                                                             \
            gate_f32_kernel<NB, WV, KT><<<grid, dim3(WV * 64), 0, st>>>(x, w, S, d, N, k, logits, topk_idx, topk_w, \
                                                                         gs);                                       \
        else if constexpr (ET == TAMOE_F16)                                                                        \
            gate_f16_kernel<NB, WV, KT><<<grid, dim3(WV * 64), 0, st>>>(x, w, S, d, N, k, logits, topk_idx, topk_w, \
                                                                         gs);                                       \
        else                                                                                                       \
            gate_bf16_kernel<NB, WV, KT><<<grid, dim3(WV * 64), 0, st>>>(x, w, S, d, N, k, logits, topk_idx,       \
                                                                          topk_w, gs);                              \
    } while (0)
    if (waves == 8) {
        if constexpr (NB >= 2) {
            if (ktail) TAMOE_GATE_LAUNCH(8, true); else TAMOE_GATE_LAUNCH(8, false);
        }
    } else if (waves == 4) {
        if (ktail) TAMOE_GATE_LAUNCH(4, true); else TAMOE_GATE_LAUNCH(4, false);
    } else if (waves == 2) {
        if (ktail) TAMOE_GATE_LAUNCH(2, true); else TAMOE_GATE_LAUNCH(2, false);
    } else {
        if (ktail) TAMOE_GATE_LAUNCH(1, true); else TAMOE_GATE_LAUNCH(1, false);
    }
#undef TAMOE_GATE_LAUNCH
}

// Everything tamoe_gate passes on to the launch of one element type.
struct GateLaunch {
    int waves;            // wavefronts per workgroup (gate_waves)
    int splits;           // K shares (gate_k_splits); > 1 only for fp32 storage
    int64_t blocks;       // token tiles
    hipStream_t st;
    const uint16_t* x;
    const uint16_t* w;
    int64_t S;
    int d_units;          // row length in 2-byte units
    int N, k;
    float* logits;        // caller's logits (may be NULL); for a split launch the partial-score buffer
    int32_t* topk_idx;
    float* topk_w;
    GateStats stats;      // n_blocks and pitch are those of this launch
};

template <int ET>
inline void launch_gate_typed(const GateLaunch& g) {
    if (g.N <= 32)
        launch_gate_mfma<1, ET>(g.waves, g.blocks, g.st, g.x, g.w, g.S, g.d_units, g.N, g.k, g.logits, g.topk_idx,
                                g.topk_w, g.stats);
    else if (g.N <= 64)
        launch_gate_mfma<2, ET>(g.waves, g.blocks, g.st, g.x, g.w, g.S, g.d_units, g.N, g.k, g.logits, g.topk_idx,
                                g.topk_w, g.stats);
    else
        launch_gate_mfma<4, ET>(g.waves, g.blocks, g.st, g.x, g.w, g.S, g.d_units, g.N, g.k, g.logits, g.topk_idx,
                                g.topk_w, g.stats);
}

// One definition each, in the translation unit of the element type.
void launch_gate_bf16(const GateLaunch& g);
void launch_gate_f16(const GateLaunch& g);
void launch_gate_f32(const GateLaunch& g);        // whole-K tiles
void launch_gate_f32_split(const GateLaunch& g);  // g.splits K shares, partial scores to g.logits

}  // namespace tamoe
