// HIP kernels for gfx950 (CDNA4, wave64) and the launch side of smha_forward.
//
// Block-wise kernel (Sec. 4.2.2, Algorithm 1 of the paper, re-designed for CDNA4):
//   one workgroup = one 64-row query tile (two waves of 32 rows), loop over the non-empty
//   64-key tiles of that tile row, K staged row-major and V staged transposed in LDS,
//   S^T = K Q^T and O^T = V^T P^T on v_mfma_f32_32x32x16 so that every lane owns one query
//   row: the softmax statistics are per-lane scalars and the score accumulators are already
//   a legal k-slice of the second MFMA's B operand (no LDS round trip for P).
// Row-wise kernel (Sec. 4.1): one wave per query row, groups of d/8 lanes gather one K/V
//   row each as a single contiguous 16-byte-per-lane segment, DPP/shuffle reductions, no
//   LDS and no barrier.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "smha_internal.hpp"

namespace smha {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct Strides {
    int64_t b, h, s;
};

struct FwdParams {
    const uint16_t *Q, *K, *V;
    void *O;
    Strides qs, ks, vs, os;
    int B, H, S, Bm, Hm;
    int out_dtype;  // smha_dtype_t
    float c;        // scale * log2(e)
    // block path
    const Item *items;
    const int32_t *item_off, *item_cnt;
    int max_items;
    const UEntry *uent;
    const uint64_t *kt_bitmap;
    float *scratch;
    int max_slots;
    const SplitRow *split_rows;
    const int32_t *split_off, *split_cnt;
    // row path
    const int32_t *row_ptr, *col_idx;
    const int64_t *col_off;
    int wgs_per_bh;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <bool BF16>
__device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c) {
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// two fp32 -> one dword of two 16-bit floats (round to nearest even), lo = a
template <bool BF16>
__device__ __forceinline__ uint32_t pack2(float a, float b) {
    if constexpr (BF16) {
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        bf2 v = {(__bf16)a, (__bf16)b};
        return __builtin_bit_cast(uint32_t, v);
    } else {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        h2 v = {(_Float16)a, (_Float16)b};
        return __builtin_bit_cast(uint32_t, v);
    }
}

template <bool BF16>
__device__ __forceinline__ float widen16(uint32_t bits16) {
    if constexpr (BF16) {
        return __builtin_bit_cast(float, bits16 << 16);
    } else {
        return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
    }
}

__device__ __forceinline__ void store_out4(void *O, int64_t elem_off, int out_dtype, float a, float b,
                                           float c, float d) {
    if (out_dtype == SMHA_F32) {
        f32x4 v = {a, b, c, d};
        *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(O) + elem_off) = v;
    } else if (out_dtype == SMHA_BF16) {
        u32x2 v = {pack2<true>(a, b), pack2<true>(c, d)};
        *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(O) + elem_off) = v;
    } else {
        u32x2 v = {pack2<false>(a, b), pack2<false>(c, d)};
        *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(O) + elem_off) = v;
    }
}

// ---------------------------------------------------------------------------------------
// Block-wise kernel
// ---------------------------------------------------------------------------------------
// One workgroup = two waves = one 128-row query supertile; wave w owns the 64-row tile row
// 2*super + w as two 32-row slices, so every K / V^T fragment read from LDS feeds two MFMAs.
// The workgroup walks the union of the two tile rows' key-tile lists; a wave skips the math
// of tiles that are empty for its own tile row but still helps staging them.
//
// LDS layouts (16-bit elements):
//   Ks[key][D + 8]         row-major, 16-byte pad per row -> conflict-free 16-byte operand reads
//   Vt[dcol][64 positions] transposed; the 64 keys of a tile are permuted inside each group of
//     16 (key = 16g + 8a + 4h + b  ->  position 16g + 8h + 4a + b) so that the 8 keys a lane
//     needs for one MFMA are one 16-byte chunk, and chunks are XOR-swizzled by
//     (dcol ^ dcol>>3) & 7 so that both the transposing writes and the operand reads spread
//     over the banks.
//
// Software pipeline (one wave per SIMD, so overlap has to come from inside the wave).  A
// tile is processed as two half tiles of 32 keys:
//     scores(0) | scores(1) + probabilities(0) | P V(0) + probabilities(1) | P V(1)
// so the vector ALU work of a half always has matrix work of its neighbour to hide under.
// K and V^T are double-buffered in LDS: tile t+1 is written while tile t is computed (one
// barrier per tile) and tile t+2 is already on its way from global memory into registers.
//
// Online softmax with a lazily raised reference: probabilities are formed against the
// running reference m_run without waiting for the half tile's own maximum; the maximum is
// gathered on the side and only if some row exceeds m_run by more than 2^8 is the half
// redone against the raised reference (and O, l rescaled).  Probabilities therefore stay
// below 2^8: exact enough in the fp32 sums and far inside the binary16 range.
__device__ __forceinline__ int vt_swz(int dcol) { return (dcol ^ (dcol >> 3)) & 7; }

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, int64_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load16(__amdgpu_buffer_rsrc_t r, int byte_off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0);  // out of range -> zeros
}

template <int V>
struct IC {
    static constexpr int value = V;
};

template <int D, bool BF16>
__global__ void __launch_bounds__(128) smha_block_fwd(const FwdParams p) {
    constexpr int NS = D / 16;            // k-steps of S^T = K Q^T
    constexpr int NDT = D / 32;           // 32-wide d tiles of O^T
    constexpr int KSTR = D + 8;           // padded K row, in elements
    constexpr int KBUF = 64 * KSTR;       // one K buffer, in elements
    constexpr int CPR = D / 8;            // 16-byte chunks per K/V row
    constexpr int KCH = 64 * CPR / 128;   // K chunks staged per thread
    constexpr int VSU = 16 * CPR / 128;   // V sub-units (4 keys x 8 columns) per thread
    constexpr int NP = BF16 ? 2 : 1;      // P operands per product (hi, lo for bfloat16)
    constexpr int PPM = 16 / (2 * NS);    // probability pairs handled per score MFMA
    constexpr int VBUF = D * 64;          // one V^T buffer, in elements
    __shared__ __attribute__((aligned(16))) uint16_t Ks[2 * KBUF];
    __shared__ __attribute__((aligned(16))) uint16_t Vt[2 * VBUF];

    // workgroup -> (batch*head, item).  Workgroups are dealt round-robin to the 8 XCDs, so
    // the low 3 bits pick the (b,h) pair inside a group of 8: each XCD's L2 then serves the
    // K/V of one head at a time.
    const int wg = blockIdx.x;
    const int xcd = wg & 7, rest = wg >> 3;
    const int grp = rest / p.max_items, it = rest - grp * p.max_items;
    const int bh = grp * 8 + xcd;
    if (bh >= p.B * p.H) return;
    const int b = bh / p.H, h = bh - b * p.H;
    const int mask = (p.Bm > 1 ? b : 0) * p.Hm + (p.Hm > 1 ? h : 0);
    if (it >= p.item_cnt[mask]) return;
    const Item item = p.items[p.item_off[mask] + it];
    const int n = item.end - item.begin;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, hh = lane >> 5;
    const int S = p.S;
    const float NEG_INF = -__builtin_inff();
    const float thr_raw = 8.0f / p.c;

    const __amdgpu_buffer_rsrc_t rQ = make_rsrc(p.Q + b * p.qs.b + h * p.qs.h, ((int64_t)(S - 1) * p.qs.s + D) * 2);
    const __amdgpu_buffer_rsrc_t rK = make_rsrc(p.K + b * p.ks.b + h * p.ks.h, ((int64_t)(S - 1) * p.ks.s + D) * 2);
    const __amdgpu_buffer_rsrc_t rV = make_rsrc(p.V + b * p.vs.b + h * p.vs.h, ((int64_t)(S - 1) * p.vs.s + D) * 2);
    const int ksb = (int)p.ks.s * 2, vsb = (int)p.vs.s * 2;  // row pitch in bytes

    // Q^T operands: slice a, lane (j, hh) holds Q[q0 + 32 a + j][16 s + 8 hh .. +8]
    const int q0 = (2 * item.qtile + w) * 64;
    u32x4 qf[2][NS];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int s = 0; s < NS; ++s)
            qf[a][s] = buf_load16(rQ, (q0 + 32 * a + j) * (int)p.qs.s * 2 + (16 * s + 8 * hh) * 2);

    // per-thread staging offsets
    int kvo[KCH], vvo[VSU];
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
        const int u = tid + 128 * i;
        kvo[i] = (u / CPR) * ksb + (u % CPR) * 16;
    }
#pragma unroll
    for (int i = 0; i < VSU; ++i) {
        const int u = tid + 128 * i;
        vvo[i] = 4 * (u / CPR) * vsb + (u % CPR) * 16;
    }
    u32x4 kreg[KCH];
    u32x4 vreg[VSU][4];
    auto gloadK = [&](int col) __attribute__((always_inline)) {
        const int base = col * 64 * ksb;
#pragma unroll
        for (int i = 0; i < KCH; ++i) kreg[i] = buf_load16(rK, kvo[i] + base);
    };
    auto gloadV = [&](int col) __attribute__((always_inline)) {
        const int base = col * 64 * vsb;
#pragma unroll
        for (int i = 0; i < VSU; ++i)
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) vreg[i][bb] = buf_load16(rV, vvo[i] + base + bb * vsb);
    };
    auto stageK = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            const int u = tid + 128 * i;
            *reinterpret_cast<u32x4 *>(&Ks[buf * KBUF + (u / CPR) * KSTR + 8 * (u % CPR)]) = kreg[i];
        }
    };
    auto stageV = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < VSU; ++i) {
            const int u = tid + 128 * i;
            const int c = u % CPR, kq = u / CPR;
            const int g = kq >> 2, a = (kq >> 1) & 1, hsel = kq & 1;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int mword = e >> 1;
                const uint32_t r0 = vreg[i][0][mword], r1 = vreg[i][1][mword];
                const uint32_t r2 = vreg[i][2][mword], r3 = vreg[i][3][mword];
                u32x2 out;
                if (e & 1) {
                    out[0] = (r0 >> 16) | (r1 & 0xFFFF0000u);
                    out[1] = (r2 >> 16) | (r3 & 0xFFFF0000u);
                } else {
                    out[0] = (r0 & 0xFFFFu) | (r1 << 16);
                    out[1] = (r2 & 0xFFFFu) | (r3 << 16);
                }
                const int dcol = 8 * c + e;
                const int chunk = (2 * g + hsel) ^ vt_swz(dcol);
                *reinterpret_cast<u32x2 *>(&Vt[buf * VBUF + dcol * 64 + chunk * 8 + a * 4]) = out;
            }
        }
    };
    auto entry_col = [&](int t) __attribute__((always_inline)) { return p.uent[item.begin + t].col; };
    auto entry_code = [&](int t) __attribute__((always_inline)) { return p.uent[item.begin + t].code[w]; };

    // LDS operand read offsets (elements)
    const int k_rd = j * KSTR + 8 * hh;  // + buf * KBUF + 32 kt * KSTR + 16 s
    int v_rd[2][4];                      // [dt parity][2 kt + u]; + (dt & ~1) * 32 * 64
#pragma unroll
    for (int par = 0; par < 2; ++par)
#pragma unroll
        for (int cu = 0; cu < 4; ++cu) {
            const int dcol = 32 * par + j;
            v_rd[par][cu] = dcol * 64 + (((2 * cu + hh) ^ vt_swz(dcol)) * 8);
        }

    float m_run[2] = {NEG_INF, NEG_INF}, l_run[2] = {0.f, 0.f};
    f32x16 o[2][NDT];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[a][dt][r] = 0.f;
    f32x16 Sh[2][2];        // [key half kt][slice a]: scores of the half tiles in flight
    u32x4 pf[2][2][NP];     // [slice a][u][hi/lo]: probabilities of the half tile being multiplied

    // ---- pieces of the pipeline ---------------------------------------------------------
    float mc[2], psum[2], mt[2];
    auto sm_begin = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            mc[a] = (m_run[a] == NEG_INF ? 0.f : m_run[a]) * p.c;
            psum[a] = 0.f;
            mt[a] = NEG_INF;
        }
    };
    auto sm_pair = [&](f32x16 (&Sc)[2], int pair, bool track_max) __attribute__((always_inline)) {
        const int a = pair >> 3, pr = pair & 7;
        const float s0 = Sc[a][2 * pr], s1 = Sc[a][2 * pr + 1];
        const float e0 = fast_exp2(fmaf(s0, p.c, -mc[a]));
        const float e1 = fast_exp2(fmaf(s1, p.c, -mc[a]));
        psum[a] += e0 + e1;
        if (track_max) mt[a] = fmaxf(fmaxf(s0, s1), mt[a]);
        if constexpr (BF16) {
            // bfloat16 keeps 8 significant bits: P is split into a truncated high part and a
            // rounded residual (p = hi + lo up to 2^-17) and the second product runs twice
            const uint32_t b0 = __builtin_bit_cast(uint32_t, e0) & 0xFFFF0000u;
            const uint32_t b1 = __builtin_bit_cast(uint32_t, e1) & 0xFFFF0000u;
            pf[a][pr >> 2][0][pr & 3] = (b0 >> 16) | b1;
            pf[a][pr >> 2][1][pr & 3] =
                pack2<true>(e0 - __builtin_bit_cast(float, b0), e1 - __builtin_bit_cast(float, b1));
        } else {
            pf[a][pr >> 2][0][pr & 3] = pack2<false>(e0, e1);
        }
    };
    // after the optimistic pass: raise the reference if some row overshot it, redo the half
    auto sm_end = [&](f32x16 (&Sc)[2]) __attribute__((always_inline)) {
        bool grow = (mt[0] > m_run[0] + thr_raw) || (mt[1] > m_run[1] + thr_raw);
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const float mrow = fmaxf(mt[a], __shfl_xor(mt[a], 32));
                const float m_new = fmaxf(m_run[a], mrow);
                const float m_use = (m_new == NEG_INF) ? 0.f : m_new;
                const float alpha = fast_exp2((m_run[a] - m_use) * p.c);
                m_run[a] = m_new;
                l_run[a] *= alpha;
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[a][dt][r] *= alpha;
                mc[a] = m_use * p.c;
                psum[a] = 0.f;
            }
#pragma unroll
            for (int pair = 0; pair < 16; ++pair) sm_pair(Sc, pair, false);
        }
        l_run[0] += psum[0];
        l_run[1] += psum[1];
    };
    auto apply_bitmap = [&](f32x16 (&Sx)[2], int code, int kt) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const uint64_t word = p.kt_bitmap[(size_t)code * 64 + 32 * a + j];
            const uint32_t bits = (uint32_t)(word >> (32 * kt)) >> (4 * hh);
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (!((bits >> (8 * (r / 4) + (r % 4))) & 1u)) Sx[a][r] = NEG_INF;
        }
    };
    // one tile for this wave: K at Ks + kbase, V^T at Vt + vbase
    auto compute_tile = [&](int kbase, int vbase, int code) __attribute__((always_inline)) {
        // scores of half 0
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int r = 0; r < 16; ++r) Sh[kt][a][r] = 0.f;
        const uint16_t *kp = &Ks[kbase + k_rd];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const u32x4 frag = *reinterpret_cast<const u32x4 *>(kp + 16 * s);
#pragma unroll
            for (int a = 0; a < 2; ++a) Sh[0][a] = mfma32<BF16>(frag, qf[a][s], Sh[0][a]);
        }
        if (code >= 0) apply_bitmap(Sh[0], code, 0);
        // scores of half 1 | probabilities of half 0
        sm_begin();
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const u32x4 frag = *reinterpret_cast<const u32x4 *>(kp + 32 * KSTR + 16 * s);
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                Sh[1][a] = mfma32<BF16>(frag, qf[a][s], Sh[1][a]);
#pragma unroll
                for (int q = 0; q < PPM; ++q) sm_pair(Sh[0], (s * 2 + a) * PPM + q, true);
            }
        }
        sm_end(Sh[0]);
        if (code >= 0) apply_bitmap(Sh[1], code, 1);
        // P V of half 0 | probabilities of half 1 (into a second set of P registers)
        const uint16_t *vp = &Vt[vbase];
        u32x4 pf0[2][2][NP];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int x = 0; x < NP; ++x) pf0[a][u][x] = pf[a][u][x];
        sm_begin();
        {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) {
                    const u32x4 frag =
                        *reinterpret_cast<const u32x4 *>(vp + v_rd[dt & 1][u] + (dt & ~1) * 32 * 64);
#pragma unroll
                    for (int a = 0; a < 2; ++a) {
                        o[a][dt] = mfma32<BF16>(frag, pf0[a][u][0], o[a][dt]);
                        if constexpr (BF16) o[a][dt] = mfma32<BF16>(frag, pf0[a][u][1], o[a][dt]);
#pragma unroll
                        for (int q = 0; q < 16 / (4 * NDT); ++q)
                            sm_pair(Sh[1], ((u * NDT + dt) * 2 + a) * (16 / (4 * NDT)) + q, true);
                    }
                }
        }
        sm_end(Sh[1]);
        // P V of half 1
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) {
                const u32x4 frag =
                    *reinterpret_cast<const u32x4 *>(vp + v_rd[dt & 1][2 + u] + (dt & ~1) * 32 * 64);
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    o[a][dt] = mfma32<BF16>(frag, pf[a][u][0], o[a][dt]);
                    if constexpr (BF16) o[a][dt] = mfma32<BF16>(frag, pf[a][u][1], o[a][dt]);
                }
            }
    };

    // ---- main loop: tile t from LDS buffer t&1, tile t+1 registers -> LDS, tile t+2 in flight
    if (n > 0) {
        gloadK(entry_col(0));
        gloadV(entry_col(0));
        stageK(0);
        stageV(0);
        if (n > 1) {
            gloadK(entry_col(1));
            gloadV(entry_col(1));
        }
        __syncthreads();
    }
    for (int t = 0; t < n; ++t) {
        const int buf = t & 1;
        if (t + 1 < n) {
            stageK(buf ^ 1);
            stageV(buf ^ 1);
        }
        if (t + 2 < n) {
            gloadK(entry_col(t + 2));
            gloadV(entry_col(t + 2));
        }
        const int code = entry_code(t);
        if (code != -2) compute_tile(buf * KBUF, buf * VBUF, code);
        __syncthreads();
    }

    // o[a][dt][r] = O[q = q0 + 32 a + j][d = 32 dt + 8 (r/4) + 4 hh + r%4]
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const float l_tot = l_run[a] + __shfl_xor(l_run[a], 32);
        const int qrow = q0 + 32 * a + j;
        if (item.slot < 0) {
            if (qrow < S) {
                const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
                const int64_t base = b * p.os.b + h * p.os.h + (int64_t)qrow * p.os.s;
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4)
                        store_out4(p.O, base + 32 * dt + 8 * g4 + 4 * hh, p.out_dtype, o[a][dt][4 * g4] * inv,
                                   o[a][dt][4 * g4 + 1] * inv, o[a][dt][4 * g4 + 2] * inv,
                                   o[a][dt][4 * g4 + 3] * inv);
            }
        } else {
            float *sc = p.scratch + ((size_t)bh * p.max_slots + item.slot) * (size_t)(128 * D + 256);
            const int row = 64 * w + 32 * a + j;
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    f32x4 v = {o[a][dt][4 * g4], o[a][dt][4 * g4 + 1], o[a][dt][4 * g4 + 2], o[a][dt][4 * g4 + 3]};
                    *reinterpret_cast<f32x4 *>(sc + row * D + 32 * dt + 8 * g4 + 4 * hh) = v;
                }
            if (hh == 0) {
                sc[128 * D + row] = m_run[a] * p.c;  // -inf stays -inf (c > 0)
                sc[128 * D + 128 + row] = l_tot;
            }
        }
    }
}

// Merge the partial (O, m, l) of supertiles that were split along keys.  One workgroup per
// (split supertile, 16-row slab, batch*head); thread = (row, 4 output columns).
template <int D>
__global__ void __launch_bounds__(16 * (D / 4)) smha_block_combine(const FwdParams p) {
    const int bh = blockIdx.z;
    const int b = bh / p.H, h = bh - b * p.H;
    const int mask = (p.Bm > 1 ? b : 0) * p.Hm + (p.Hm > 1 ? h : 0);
    if ((int)blockIdx.x >= p.split_cnt[mask]) return;
    const SplitRow sr = p.split_rows[p.split_off[mask] + blockIdx.x];
    const size_t stride = (size_t)(128 * D + 256);
    const float *base = p.scratch + ((size_t)bh * p.max_slots + sr.slot0) * stride;
    const int row = blockIdx.y * 16 + threadIdx.x / (D / 4), dq = threadIdx.x % (D / 4);
    const int qrow = sr.qtile * 128 + row;
    if (qrow >= p.S) return;
    float mstar = -__builtin_inff();
    for (int c = 0; c < sr.count; ++c) mstar = fmaxf(mstar, base[c * stride + 128 * D + row]);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float L = 0.f;
    if (mstar != -__builtin_inff()) {
#pragma unroll 4
        for (int c = 0; c < sr.count; ++c) {
            const float wgt = fast_exp2(base[c * stride + 128 * D + row] - mstar);
            L += wgt * base[c * stride + 128 * D + 128 + row];
            const f32x4 v = *reinterpret_cast<const f32x4 *>(base + c * stride + row * D + 4 * dq);
            acc += v * wgt;
        }
    }
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    store_out4(p.O, b * p.os.b + h * p.os.h + (int64_t)qrow * p.os.s + 4 * dq, p.out_dtype, acc[0] * inv,
               acc[1] * inv, acc[2] * inv, acc[3] * inv);
}

// ---------------------------------------------------------------------------------------
// Row-wise kernel
// ---------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false);
    return v + __builtin_bit_cast(float, moved);
}

// sum over the aligned group of LPK (8 or 16) lanes; every lane of the group gets the sum
template <int LPK>
__device__ __forceinline__ float group_sum(float v) {
    v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);  // row_half_mirror: the other quad of the 8
    if constexpr (LPK == 16) v = dpp_add<0x140>(v);  // row_mirror: the other half of the 16
    return v;
}

template <int D, bool BF16>
__global__ void __launch_bounds__(256) smha_row_fwd(const FwdParams p) {
    constexpr int LPK = D / 8;     // lanes that share one key (16 bytes of the row each)
    constexpr int KPS = 64 / LPK;  // keys a wave handles per step
    constexpr int U = 2;           // independent steps in flight
    const int wg = blockIdx.x;
    const int xcd = wg & 7, rest = wg >> 3;
    const int grp = rest / p.wgs_per_bh, rb = rest - grp * p.wgs_per_bh;
    const int bh = grp * 8 + xcd;
    if (bh >= p.B * p.H) return;
    const int b = bh / p.H, h = bh - b * p.H;
    const int mask = (p.Bm > 1 ? b : 0) * p.Hm + (p.Hm > 1 ? h : 0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = rb * 4 + wave;
    if (i >= p.S) return;
    const int sub = lane % LPK, g = lane / LPK;
    const float NEG_INF = -__builtin_inff();

    float qf[8];
    {
        u32x4 v = *reinterpret_cast<const u32x4 *>(p.Q + b * p.qs.b + h * p.qs.h + (int64_t)i * p.qs.s + 8 * sub);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            qf[2 * e] = widen16<BF16>(v[e] & 0xFFFFu) * p.c;
            qf[2 * e + 1] = widen16<BF16>(v[e] >> 16) * p.c;
        }
    }
    const int32_t *rp = p.row_ptr + (size_t)mask * (p.S + 1);
    const int beg = rp[i], end = rp[i + 1];
    const int32_t *ci = p.col_idx + p.col_off[mask];
    const uint16_t *Kb = p.K + b * p.ks.b + h * p.ks.h + 8 * sub;
    const uint16_t *Vb = p.V + b * p.vs.b + h * p.vs.h + 8 * sub;

    float m = NEG_INF, l = 0.f, acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;

    for (int base = beg; base < end; base += KPS * U) {
        u32x4 kv[U], vv[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int idx = base + u * KPS + g;
            ok[u] = idx < end;
            const int col = ci[ok[u] ? idx : beg];
            kv[u] = *reinterpret_cast<const u32x4 *>(Kb + (int64_t)col * p.ks.s);
            vv[u] = *reinterpret_cast<const u32x4 *>(Vb + (int64_t)col * p.vs.s);
        }
        float s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                d = fmaf(qf[2 * e], widen16<BF16>(kv[u][e] & 0xFFFFu), d);
                d = fmaf(qf[2 * e + 1], widen16<BF16>(kv[u][e] >> 16), d);
            }
            d = group_sum<LPK>(d);
            s[u] = ok[u] ? d : NEG_INF;
        }
        float m_new = m;
#pragma unroll
        for (int u = 0; u < U; ++u) m_new = fmaxf(m_new, s[u]);
        const float m_use = (m_new == NEG_INF) ? 0.f : m_new;
        const float alpha = fast_exp2(m - m_use);
        m = m_new;
        l *= alpha;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float pe = fast_exp2(s[u] - m_use);
            l += pe;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[2 * e] = fmaf(pe, widen16<BF16>(vv[u][e] & 0xFFFFu), acc[2 * e]);
                acc[2 * e + 1] = fmaf(pe, widen16<BF16>(vv[u][e] >> 16), acc[2 * e + 1]);
            }
        }
    }
    // merge the KPS lane groups (butterfly over lane bits >= LPK)
#pragma unroll
    for (int off = LPK; off < 64; off <<= 1) {
        const float m_o = __shfl_xor(m, off);
        const float l_o = __shfl_xor(l, off);
        const float m_new = fmaxf(m, m_o);
        const float m_use = (m_new == NEG_INF) ? 0.f : m_new;
        const float wa = fast_exp2(m - m_use), wb = fast_exp2(m_o - m_use);
        l = l * wa + l_o * wb;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = acc[e] * wa + __shfl_xor(acc[e], off) * wb;
        m = m_new;
    }
    if (g == 0) {
        const float inv = l > 0.f ? 1.0f / l : 0.f;
        const int64_t o = b * p.os.b + h * p.os.h + (int64_t)i * p.os.s + 8 * sub;
        store_out4(p.O, o, p.out_dtype, acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
        store_out4(p.O, o + 4, p.out_dtype, acc[4] * inv, acc[5] * inv, acc[6] * inv, acc[7] * inv);
    }
}

// ---------------------------------------------------------------------------------------
// Host side: device residency of a plan
// ---------------------------------------------------------------------------------------
int current_device_or_negative() {
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || n < 1) {
        (void)hipGetLastError();
        return -1;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return -1;
    }
    return dev;
}

smha_status_t copy_mask_to_host(const uint8_t *dev_mask, size_t bytes, uint8_t *host_dst) {
    if (hipMemcpy(host_dst, dev_mask, bytes, hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return SMHA_ERR_HIP;
    }
    return SMHA_OK;
}

template <typename T>
static bool to_device(T *&dst, const std::vector<T> &src) {
    dst = nullptr;
    const size_t bytes = std::max<size_t>(src.size(), 1) * sizeof(T);
    if (hipMalloc(reinterpret_cast<void **>(&dst), bytes) != hipSuccess) return false;
    if (!src.empty() && hipMemcpy(dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess)
        return false;
    return true;
}

smha_status_t upload_plan(smha_plan *p, int device_id) {
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device_id >= n) {
        (void)hipGetLastError();
        return SMHA_ERR_HIP;
    }
    int prev = 0;
    if (hipGetDevice(&prev) != hipSuccess || hipSetDevice(device_id) != hipSuccess) {
        (void)hipGetLastError();
        return SMHA_ERR_HIP;
    }
    bool ok = true;
    DeviceArrays &d = p->dev;
    p->device = device_id;
    if (p->has_row) {
        ok = ok && to_device(d.row_ptr, p->h_row_ptr) && to_device(d.col_idx, p->h_col_idx) &&
             to_device(d.col_off, p->h_col_off);
    }
    if (ok && p->has_block) {
        ok = to_device(d.uent, p->h_uent) && to_device(d.kt_bitmap, p->h_kt_bitmap) && to_device(d.items, p->h_items) &&
             to_device(d.item_off, p->h_item_off) && to_device(d.item_cnt, p->h_item_cnt) &&
             to_device(d.split_rows, p->h_split_rows) && to_device(d.split_off, p->h_split_off) &&
             to_device(d.split_cnt, p->h_split_cnt);
    }
    (void)hipSetDevice(prev);
    if (!ok) {
        (void)hipGetLastError();
        release_device(p);
        return SMHA_ERR_ALLOC;
    }
    return SMHA_OK;
}

void release_device(smha_plan *p) {
    if (p->device < 0) return;
    int prev = 0;
    (void)hipGetDevice(&prev);
    (void)hipSetDevice(p->device);
    DeviceArrays &d = p->dev;
    void *ptrs[] = {d.row_ptr, d.col_idx, d.col_off, d.uent, d.kt_bitmap, d.items,
                    d.item_off, d.item_cnt, d.split_rows, d.split_off, d.split_cnt, p->d_scratch};
    for (void *q : ptrs)
        if (q) (void)hipFree(q);
    d = DeviceArrays{};
    p->d_scratch = nullptr;
    p->scratch_bytes = 0;
    p->device = -1;
    (void)hipSetDevice(prev);
}

}  // namespace smha

// ---------------------------------------------------------------------------------------
// smha_forward
// ---------------------------------------------------------------------------------------
using namespace smha;

static bool strides_ok(const int64_t *s) { return !s || (s[0] % 8 == 0 && s[1] % 8 == 0 && s[2] % 8 == 0 && s[2] > 0); }

template <int D, bool BF16>
static hipError_t launch_block(const smha_plan *plan, FwdParams &fp, hipStream_t stream) {
    const int BH = fp.B * fp.H;
    const int groups = (BH + 7) / 8;
    const unsigned grid = (unsigned)(8 * groups * plan->max_items);
    if (grid == 0) return hipSuccess;
    hipLaunchKernelGGL((smha_block_fwd<D, BF16>), dim3(grid), dim3(128), 0, stream, fp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (plan->max_split_rows > 0) {
        hipLaunchKernelGGL((smha_block_combine<D>), dim3(plan->max_split_rows, 8, BH), dim3(16 * (D / 4)), 0, stream, fp);
        e = hipGetLastError();
    }
    return e;
}

template <int D, bool BF16>
static hipError_t launch_row(const smha_plan *plan, FwdParams &fp, hipStream_t stream) {
    const int BH = fp.B * fp.H;
    const int groups = (BH + 7) / 8;
    fp.wgs_per_bh = (fp.S + 3) / 4;
    const unsigned grid = (unsigned)(8 * groups * fp.wgs_per_bh);
    hipLaunchKernelGGL((smha_row_fwd<D, BF16>), dim3(grid), dim3(256), 0, stream, fp);
    return hipGetLastError();
}

extern "C" smha_status_t smha_forward(const smha_plan_t *plan, const void *Q, const void *K,
                                      const void *V, void *O, int B, int H, int d,
                                      smha_dtype_t in_dtype, smha_dtype_t out_dtype,
                                      const int64_t q_strides[3], const int64_t k_strides[3],
                                      const int64_t v_strides[3], const int64_t o_strides[3],
                                      float scale, smha_kernel_t kernel, void *hip_stream) {
    if (!plan || !Q || !K || !V || !O || B < 1 || H < 1) return SMHA_ERR_INVALID_ARG;
    if (in_dtype != SMHA_F16 && in_dtype != SMHA_BF16) return SMHA_ERR_UNSUPPORTED;
    if (out_dtype != in_dtype && out_dtype != SMHA_F32) return SMHA_ERR_UNSUPPORTED;
    if (d != 64 && d != 128) return SMHA_ERR_UNSUPPORTED;
    if (kernel < SMHA_KERNEL_AUTO || kernel > SMHA_KERNEL_BLOCK) return SMHA_ERR_INVALID_ARG;
    if ((plan->Bm != 1 && plan->Bm != B) || (plan->Hm != 1 && plan->Hm != H)) return SMHA_ERR_SHAPE;
    if (!strides_ok(q_strides) || !strides_ok(k_strides) || !strides_ok(v_strides) || !strides_ok(o_strides))
        return SMHA_ERR_UNSUPPORTED;
    const uintptr_t align = (uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O;
    if (align & 15) return SMHA_ERR_UNSUPPORTED;
    if ((int64_t)B * H > (1 << 24)) return SMHA_ERR_UNSUPPORTED;
    {   // the block kernel addresses one head's Q/K/V through 32-bit buffer offsets
        const int64_t lim = (int64_t)1 << 31;
        const int64_t rows = (int64_t)plan->S + 128;
        const int64_t qs = q_strides ? q_strides[2] : d, ks = k_strides ? k_strides[2] : d, vs = v_strides ? v_strides[2] : d;
        if ((rows * qs + d) * 2 >= lim || (rows * ks + d) * 2 >= lim || (rows * vs + d) * 2 >= lim) return SMHA_ERR_UNSUPPORTED;
    }
    int which = kernel == SMHA_KERNEL_AUTO ? plan->kernel : (int)kernel;
    if (which == SMHA_KERNEL_ROW && !plan->has_row) return SMHA_ERR_UNSUPPORTED;
    if (which == SMHA_KERNEL_BLOCK && !plan->has_block) return SMHA_ERR_UNSUPPORTED;
    if (plan->device < 0) return SMHA_ERR_HIP;
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess || cur != plan->device) {
        (void)hipGetLastError();
        return SMHA_ERR_HIP;
    }

    const int S = plan->S;
    auto packed = [&](Strides &s) { s.s = d; s.h = (int64_t)S * d; s.b = (int64_t)H * S * d; };
    auto take = [&](Strides &s, const int64_t *in) {
        if (in) { s.b = in[0]; s.h = in[1]; s.s = in[2]; } else packed(s);
    };
    FwdParams fp{};
    fp.Q = (const uint16_t *)Q; fp.K = (const uint16_t *)K; fp.V = (const uint16_t *)V; fp.O = O;
    take(fp.qs, q_strides); take(fp.ks, k_strides); take(fp.vs, v_strides); take(fp.os, o_strides);
    fp.B = B; fp.H = H; fp.S = S; fp.Bm = plan->Bm; fp.Hm = plan->Hm;
    fp.out_dtype = out_dtype;
    const float sc = scale > 0.f ? scale : 1.0f / std::sqrt((float)d);
    fp.c = sc * 1.4426950408889634f;
    const DeviceArrays &dv = plan->dev;
    fp.items = dv.items; fp.item_off = dv.item_off; fp.item_cnt = dv.item_cnt; fp.max_items = plan->max_items;
    fp.uent = dv.uent; fp.kt_bitmap = dv.kt_bitmap;
    fp.max_slots = plan->max_slots;
    fp.split_rows = dv.split_rows; fp.split_off = dv.split_off; fp.split_cnt = dv.split_cnt;
    fp.row_ptr = dv.row_ptr; fp.col_idx = dv.col_idx; fp.col_off = dv.col_off;

    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t e = hipSuccess;
    if (which == SMHA_KERNEL_BLOCK) {
        if (plan->max_slots > 0) {
            const size_t need = (size_t)B * H * plan->max_slots * (size_t)(128 * d + 256) * sizeof(float);
            std::lock_guard<std::mutex> lock(plan->scratch_mutex);
            if (need > plan->scratch_bytes) {
                if (plan->d_scratch) {
                    // earlier launches may still be reading the old buffer
                    if (hipDeviceSynchronize() != hipSuccess || hipFree(plan->d_scratch) != hipSuccess) {
                        (void)hipGetLastError();
                        return SMHA_ERR_HIP;
                    }
                    plan->d_scratch = nullptr;
                    plan->scratch_bytes = 0;
                }
                void *ptr = nullptr;
                if (hipMalloc(&ptr, need) != hipSuccess) {
                    (void)hipGetLastError();
                    return SMHA_ERR_ALLOC;
                }
                plan->d_scratch = (float *)ptr;
                plan->scratch_bytes = need;
            }
            fp.scratch = plan->d_scratch;
        }
        if (d == 64)
            e = in_dtype == SMHA_BF16 ? launch_block<64, true>(plan, fp, stream) : launch_block<64, false>(plan, fp, stream);
        else
            e = in_dtype == SMHA_BF16 ? launch_block<128, true>(plan, fp, stream) : launch_block<128, false>(plan, fp, stream);
    } else {
        if (d == 64)
            e = in_dtype == SMHA_BF16 ? launch_row<64, true>(plan, fp, stream) : launch_row<64, false>(plan, fp, stream);
        else
            e = in_dtype == SMHA_BF16 ? launch_row<128, true>(plan, fp, stream) : launch_row<128, false>(plan, fp, stream);
    }
    return e == hipSuccess ? SMHA_OK : SMHA_ERR_HIP;
}

extern "C" const char *smha_kernel_name(const smha_plan_t *plan, int d, smha_dtype_t in_dtype,
                                        smha_kernel_t kernel) {
    if (!plan) return "";
    const int which = kernel == SMHA_KERNEL_AUTO ? plan->kernel : (int)kernel;
    return which == SMHA_KERNEL_ROW ? "smha_row_fwd" : "smha_block_fwd";
}
