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

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <vector>

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
    int B, H, S, Sk, Bm, Hm;  // S queries, Sk keys
    int d;          // head size in memory: a multiple of 8, at most the kernel's D (columns d .. D-1 are read as zeros and never stored)
    int out_dtype;  // smha_dtype_t
    float c;        // scale * log2(e)
    // block path
    const Item *items;
    const int32_t *item_off, *item_cnt;
    // work order of the block kernel: for each XCD x a list of (batch*head, item index) pairs of the
    // heads with batch*head mod 8 = x; the workgroup of rank r on that XCD (of gridDim.x / 8) takes
    // positions r, r + gridDim.x / 8, ... until the list ends or a pair with batch*head < 0 comes up.
    // order_hdr = {start of each XCD's list (8), length (8)}
    const int32_t *order, *order_hdr;
    // second form: order_hdr = per workgroup {first step, steps, first item, items}, order = StepRec
    // records (step_bytes of them), order_items = ItemRec records (item_bytes)
    const int32_t *order_items;
    int64_t step_bytes, item_bytes;
    int form;    // 1: (batch*head, item) pairs in `order`; 2: WorkRec records
    int n_work;  // 8 * the longest list
    int per_xcd; // workgroups per XCD the order was made for (host side: the grid is 8 times this)
    const UEntry *uent;
    const int32_t *gidx;  // gathered tiles: 64 key numbers each
    int n_gidx;           // entries of gidx
    const uint64_t *kt_bitmap;
    int bmp_spare;  // index of an all-zero spare bitmap block (what fetch_word falls back to for a tile without a bitmap)
    // split 128-row groups: workspace slots of 128 D + 1024 floats per (batch*head), arrival counters
    // (8 per (batch*head, split group), zero between launches), and the groups' descriptions
    float *scratch;
    uint32_t *counters;
    int max_slots, max_splits;
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
// One workgroup = four waves = one 128-row query supertile (two vertically adjacent 64-row
// tile rows); wave w owns rows 32 w .. 32 w + 31.  The workgroup walks the union of the two
// tile rows' key-tile lists, so a staged K/V tile is shared by up to four waves; a wave skips
// the math of tiles that are empty for its own tile row (or, through the bitmap, for its own
// 32 rows).  Two workgroups fit a CU (two waves per SIMD): one workgroup's softmax (vector
// ALU) and memory waits overlap the other's MFMAs.
//
// K and V tiles go from global memory straight into LDS (buffer_load ... lds, 16 bytes per
// lane, no registers and no vector-ALU work), both row-major [64 keys][D] with the 16-byte
// chunks of a row XOR-swizzled so that operand reads spread over the 64 banks (256 bytes):
// a 16-byte K read is served 16 lanes (= 16 consecutive rows, one logical chunk) at a time, so
// swz_k must be a bijection of those rows onto the 16 chunk slots of a 256-byte window; a
// transposing V read is served 32 lanes at a time (4 consecutive rows x 4 consecutive chunks),
// so swz_v must send those rows to different aligned groups of 4 chunks.  The swizzle is
// applied on the global side: LDS chunk p of a row is filled with global chunk p ^ swz(row).
// Rows past S read as zeros (buffer bounds), so ragged S needs no branches.
// Both tiles are double-buffered: the loads of tile t+1 are issued at the top of tile t (right
// after the barrier that ends tile t-1 freed their buffers) and are waited for at the barrier
// that ends tile t.
//
// S^T = K Q^T reads K fragments with 16-byte LDS reads (a lane's 8 consecutive d values of
// one key).  O^T = V^T P^T needs, per lane, 8 keys of one d column: ds_read_b64_tr_b16
// delivers exactly that from the row-major tile (16 lanes read 4 keys x 16 columns, each lane
// receives 4 keys of one column), so V is never transposed in software.
//
// Online softmax with a lazily raised reference: the running reference m_run is only raised
// when a tile's row maximum exceeds it by more than 2^8, so the O rescale is rare and
// probabilities stay below 2^8 (exact enough in the fp32 sums, far inside the binary16 range).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, int64_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load16(__amdgpu_buffer_rsrc_t r, int byte_off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0);  // out of range -> zeros
}
// (rows of 256 bytes or more: a row's chunks are permuted inside each aligned group of 16)
template <int D> __device__ __forceinline__ int swz_k(int row) {
    if constexpr (D >= 128) return row & 15;
    else return (row / (128 / D)) & (D / 8 - 1);
}
template <int D> __device__ __forceinline__ int swz_v(int row) {
    if constexpr (D >= 128) return (row & 3) << 2;
    else return ((row / (128 / D)) & (D / 32 - 1)) << 2;
}
typedef __attribute__((address_space(3))) void lds_void;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Buffer descriptor as four dwords (base, no stride, size in bytes, raw 32-bit data format) for the
// loads below; out-of-range offsets return zeros.
__device__ __forceinline__ u32x4 make_rsrc4(const void *base, int64_t bytes) {
    const uint64_t a = (uint64_t)base;
    return u32x4{(uint32_t)a, (uint32_t)(a >> 32) & 0xFFFFu, (uint32_t)bytes, 0x00020000u};
}
// 64 lanes x 16 bytes from per-lane global offsets into 1 KiB of LDS at byte address `lds`
// (lane l -> lds + 16 l), bypassing registers.  Written as an instruction: the compiler's own
// form makes it track which LDS object each load in flight may write, which forces the two
// buffers of a pair to be compile-time objects (a loop body per buffer) and adds full waits
// wherever it cannot tell; here every wait for these loads is an explicit s_waitcnt in the
// kernel (memory operations retire in order, so the compiler's own vmcnt waits stay safe).
// M0 is written here without being listed as clobbered: the compiler reserves it, sets it right
// before each use of its own and rejects it on a clobber list with a warning.
__device__ __forceinline__ void load_to_lds(u32x4 rsrc, uint32_t lds, int byte_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds), "v"(byte_off), "s"(rsrc) : "memory");
}
// transposing LDS read: see the kernel comment; returns this lane's 4 keys of one column
__device__ __forceinline__ u32x2 lds_read_tr(const uint16_t *src) {
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)src);
    return __builtin_bit_cast(u32x2, v);
}

// Read-only plan data at a wave-uniform address: through the constant address space, so the
// load is a scalar one (a vector load would have to drain the wave's outstanding tile loads and
// output stores before its value could be used).
template <typename T>
__device__ __forceinline__ T uniform_load(const T *ptr) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8 || sizeof(T) == 16, "one, two or four dwords");
    if constexpr (sizeof(T) == 4) {
        typedef const uint32_t __attribute__((address_space(4))) *const_ptr;
        return __builtin_bit_cast(T, *(const_ptr)(uintptr_t)ptr);
    } else if constexpr (sizeof(T) == 8) {
        typedef const u32x2 __attribute__((address_space(4))) *const_ptr;
        return __builtin_bit_cast(T, *(const_ptr)(uintptr_t)ptr);
    } else {
        typedef const u32x4 __attribute__((address_space(4))) *const_ptr;
        return __builtin_bit_cast(T, *(const_ptr)(uintptr_t)ptr);
    }
}

template <int OUT>  // smha_dtype_t of the output
__device__ __forceinline__ void store4(void *O, int64_t elem_off, float a, float b, float c, float d) {
    if constexpr (OUT == SMHA_F32) {
        f32x4 v = {a, b, c, d};
        *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(O) + elem_off) = v;
    } else {
        u32x2 v = {pack2<OUT == SMHA_BF16>(a, b), pack2<OUT == SMHA_BF16>(c, d)};
        *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(O) + elem_off) = v;
    }
}


// The end of a work item that is one part of a split 128-row group (see Item), for one wave's 32 rows
// (quarter w of the group): o[dt][r] = unnormalised O[row j][d = 32 dt + 8 (r/4) + 4 hh + r%4], m_c the
// rows' running maximum in units of the exponent (-inf if none), l_tot their running sum.
// The partial result goes to the workspace, register by register (64 consecutive floats per wave
// instruction).  Parts run on any XCD and the XCDs' L2 caches are not coherent with each other, so these
// stores and the loads of the merge are device-scope atomic accesses (they go through to memory), and the
// wave waits for its stores before it counts itself in: when the counter reads count - 1, every other
// part's quarter is in memory.  The wave that finds it so owns the merge: it leaves its mark (its
// workgroup's number) in the counter and merges when it sees fit (merge_split_parts).
// The same for the kernel form whose eight waves own 16 rows each (an eighth of the group per wave): Acc is
// the accumulator vector (16 floats there, 4 here), NA how many a lane holds; a slot has room for eight
// waves' references and sums, and a group has eight counters, whichever form runs.
constexpr uint32_t kMergeMark = 0x80000000u;
constexpr int kSlotExtra = 1024;  // floats of a workspace slot after the 128 x D accumulators: 512 references, 512 sums
template <int D, typename Acc, int NA>
__device__ __forceinline__ bool put_split_part(const FwdParams &p, const Acc (&o)[NA], float m_c, float l_tot,
                                               int w, int lane, int b, int h, int bh, int slot, int split) {
    constexpr int E = sizeof(Acc) / 4;
    constexpr int NR = E * NA;                                 // accumulator registers per lane
    constexpr size_t SLOT = (size_t)(128 * D + kSlotExtra);  // floats per workspace slot
    float *mine = p.scratch + ((size_t)bh * p.max_slots + slot) * SLOT;
    auto put = [&](float *ptr, float v) __attribute__((always_inline)) {
        __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
#pragma unroll
    for (int dt = 0; dt < NA; ++dt)
#pragma unroll
        for (int r = 0; r < E; ++r) put(mine + ((size_t)w * NR + dt * E + r) * 64 + lane, o[dt][r]);
    put(mine + 128 * D + w * 64 + lane, m_c);
    put(mine + 128 * D + 512 + w * 64 + lane, l_tot);
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0): the stores above have completed
    const int mask = (p.Bm > 1 ? b : 0) * p.Hm + (p.Hm > 1 ? h : 0);
    const int count = uniform_load(&p.split_rows[uniform_load(p.split_off + mask) + split].count);
    uint32_t *counter = p.counters + ((size_t)bh * p.max_splits + split) * 8 + w;
    int last = 0;
    if (lane == 0) {
        const uint32_t seen = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        last = (int)seen == count - 1;
        if (last) __hip_atomic_store(counter, kMergeMark | blockIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return __builtin_amdgcn_readfirstlane(last) != 0;  // this wave owns the merge of its quarter
}

// The merge of a split group's quarter w, by the wave that owns it (see put_split_part; any other wave
// returns at once): all parts in list order (the owner's included, re-read: the result does not depend on
// which part came last), then O; the counter goes back to zero for the next launch.
// (owner_known: the caller remembers put_split_part's answer, and the counter need not be asked)
// (W16: the eight-wave form: register r of a lane is column 16 (r / 4) + 4 (lane / 16) + r % 4 of its row)
template <int D, int OUT, int PB, int RB, bool W16 = false>  // a batch of loads in flight: PB parts x RB accumulator registers
__device__ __forceinline__ void merge_split_parts(const FwdParams &p, int w, int lane, int b, int h, int bh, int qrow, int split,
                                                  bool owner_known = false) {
    constexpr int NR = W16 ? D / 4 : D / 2;
    constexpr size_t SLOT = (size_t)(128 * D + kSlotExtra);
    const int hh = lane >> 5;
    const float NEG_INF = -__builtin_inff();
    auto get = [&](const float *ptr) __attribute__((always_inline)) {
        return __hip_atomic_load(const_cast<float *>(ptr), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    uint32_t *counter = p.counters + ((size_t)bh * p.max_splits + split) * 8 + w;
    if (!owner_known) {
        uint32_t state = 0;
        if (lane == 0) state = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (__builtin_amdgcn_readfirstlane(state) != (kMergeMark | blockIdx.x)) return;
    }
    if (lane == 0) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int mask = (p.Bm > 1 ? b : 0) * p.Hm + (p.Hm > 1 ? h : 0);
    const SplitRow sr = uniform_load(p.split_rows + uniform_load(p.split_off + mask) + split);
    const float *base = p.scratch + ((size_t)bh * p.max_slots + sr.slot0) * SLOT;
    // Every batch of loads costs one trip to memory, so as much as the registers hold travels together:
    // RB accumulator registers of PB parts, with those parts' references (and, in the first batch, their
    // sums); RB registers are finished and stored before the next RB are begun.  A group of at most PB
    // parts finds its common reference in the first batch; longer ones take a pass over all references first.
    const bool one_block = sr.count <= PB;
    float mstar = NEG_INF;
    if (!one_block) {
        for (int c0 = 0; c0 < sr.count; c0 += 8) {
            float ms[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) ms[u] = get(base + (size_t)min(c0 + u, sr.count - 1) * SLOT + 128 * D + w * 64 + lane);
#pragma unroll
            for (int u = 0; u < 8; ++u) mstar = fmaxf(mstar, ms[u]);
        }
    }
    const float *mine_q = base + (size_t)w * NR * 64 + lane;  // this wave's quarter of part 0
    const int64_t obase = b * p.os.b + h * p.os.h + (int64_t)qrow * p.os.s;
    float L = 0.f, inv = 0.f;
#pragma unroll
    for (int r0 = 0; r0 < NR; r0 += RB) {
        float acc[RB];
#pragma unroll
        for (int i = 0; i < RB; ++i) acc[i] = 0.f;
        for (int c0 = 0; c0 < sr.count; c0 += PB) {
            float mu[PB], lu[PB], v[PB][RB];
            int at[PB];  // float offset of part c0 + u from part 0 (parts past the end: part c0 again, weight 0)
#pragma unroll
            for (int u = 0; u < PB; ++u) {
                at[u] = (c0 + u < sr.count ? c0 + u : c0) * (int)SLOT;
                mu[u] = get(base + at[u] + 128 * D + w * 64 + lane);
                if (r0 == 0) lu[u] = get(base + at[u] + 128 * D + 512 + w * 64 + lane);
            }
#pragma unroll
            for (int u = 0; u < PB; ++u)
#pragma unroll
                for (int i = 0; i < RB; ++i) v[u][i] = get(mine_q + at[u] + (r0 + i) * 64);
            if (r0 == 0 && one_block) {
#pragma unroll
                for (int u = 0; u < PB; ++u) mstar = fmaxf(mstar, mu[u]);  // (parts past the end repeat part c0)
            }
#pragma unroll
            for (int u = 0; u < PB; ++u) {
                // (a row with no key in any part has -inf everywhere: weight 0, never -inf - -inf)
                const float wgt = (c0 + u < sr.count && mu[u] != NEG_INF) ? fast_exp2(mu[u] - mstar) : 0.f;
                if (r0 == 0) L += wgt * lu[u];
#pragma unroll
                for (int i = 0; i < RB; ++i) acc[i] = fmaf(wgt, v[u][i], acc[i]);
            }
        }
        if (r0 == 0) inv = L > 0.f ? 1.0f / L : 0.f;
        if (qrow < p.S) {
#pragma unroll
            for (int i = 0; i < RB; i += 4) {
                const int r = r0 + i;
                const int col = W16 ? 16 * (r >> 2) + 4 * (lane >> 4) : 32 * (r >> 4) + 8 * ((r & 15) >> 2) + 4 * hh;
                if (col < p.d) store4<OUT>(p.O, obase + col, acc[i] * inv, acc[i + 1] * inv, acc[i + 2] * inv, acc[i + 3] * inv);
            }
        }
    }
}

// GATHER: the plan holds gathered tiles (staged rows that come from arbitrary key numbers, see
// UEntry); plans without any run the instantiation that does not know about them.
template <int D, int OUT>
__device__ __forceinline__ void finish_split_part(const FwdParams &p, const f32x16 (&o)[D / 32], float m_c, float l_tot,
                                                  int w, int lane, int b, int h, int bh, int qrow, int slot, int split) {
    if (put_split_part<D, f32x16, D / 32>(p, o, m_c, l_tot, w, lane, b, h, bh, slot, split))
        merge_split_parts<D, OUT, 4, 8>(p, w, lane, b, h, bh, qrow, split, true);
}

// SPLIT: the plan cuts some 128-row groups into parts (the instantiation for plans that do not carries
// none of the merge code: its registers would be paid for in every item's start and end).
template <int D, bool BF16, int OUT, bool GATHER, bool SPLIT>
__global__ void __launch_bounds__(256, D == 64 ? 4 : D == 128 ? 2 : 1) smha_block_fwd(const FwdParams p) {
    constexpr int NS = D / 16;            // k-steps of S^T = K Q^T
    constexpr int NDT = D / 32;           // 32-wide d tiles of O^T
    constexpr int TILE = 64 * D;          // one K or V tile, in elements
    constexpr int CPR = D / 8;            // 16-byte chunks per K/V row
    constexpr int LPW = CPR / 4;          // 1 KiB load instructions per wave, per tile, per tensor
    constexpr int NP = BF16 ? 2 : 1;      // P operands per product (hi, lo for bfloat16)
    constexpr int PF = D >= 128 ? 8 : 4;  // LDS fragment requests kept ahead of the MFMAs (d = 128 has the registers: 199 of 256;
                                          // 8 instead of 4 is worth 1.6 % there; at d = 64 more would spill)
    // K[0], K[1], V[0], V[1]: tile t lives in K[t & 1], V[t & 1]
    __shared__ __attribute__((aligned(1024))) uint16_t smem[4 * TILE];
    // key numbers of the current item's gathered tiles (64 each)
    __shared__ __attribute__((aligned(1024))) int32_t gix[GATHER ? kMaxGatherPerItem * 64 : 1];
    const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void *)smem;  // LDS byte address
    constexpr int TB = TILE * 2;                                        // bytes per tile

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, hh = lane >> 5;
    const int S = p.S;
    const float NEG_INF = -__builtin_inff();
    const float thr_raw = 8.0f / p.c;
    constexpr int OOB = 0x7FFFFF00;  // past every buffer: such loads return zeros without traffic
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // LDS operand read offsets (bytes inside a tile).
    // K fragment (kt, s): row 32 kt + j, logical chunk 2 s + hh -> physical chunk (2 s) ^ hh ^ swz_k(j):
    // byte offset k_rd ^ (32 s) (+ 64 kt D)
    const int k_rd = j * D * 2 + ((hh ^ swz_k<D>(j)) * 16);
    // V^T fragment (dt, key group of 4): lane reads 8 bytes of row 4 hh + (lane%16)/4 (+ 8 a + 16 cu),
    // logical chunk 4 dt + 2 ((lane/16)&1) + (lane%4)/2, second half of the chunk if lane%4 is odd:
    // byte offset v_rd ^ (64 dt) (+ 2 D (8 a + 16 cu))
    const int v_row = 4 * hh + ((lane & 15) >> 2);
    const int v_rd = v_row * D * 2 + ((swz_v<D>(v_row) + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) * 16) + (lane & 1) * 8;

    // Persistent workgroups: the grid is a multiple of 8 that fills the chip once, and each
    // workgroup walks the work list with that stride (so it stays on its XCD's heads).  Work
    // index -> XCD = index mod 8 -> (batch*head), so that each XCD's L2 serves the K/V of one
    // head at a time.  Items are software-pipelined: the next item's descriptor is fetched (scalar
    // loads) while the current one starts; its entries, Q fragments and first K/V tile are
    // requested right after the current item's last tile, before the current item's output
    // stores, so memory latency of an item's start hides behind the previous item's end.
    struct Work {  // wave-uniform
        int valid, b, h, bh, qtile, begin, n, slot, split, col0, code0[2], gid0;  // col0, code0, gid0: the first entry
        int gbegin, gcount;
    };
    const int xcd = blockIdx.x & 7, per_xcd = gridDim.x >> 3;
    const int list_at = uniform_load(p.order_hdr + xcd), list_len = uniform_load(p.order_hdr + 8 + xcd);
    auto fetch_work = [&](int pos) __attribute__((always_inline)) {  // position in this XCD's list
        Work wk;
        wk.valid = pos < list_len;
        wk.bh = wk.b = wk.h = 0;
        wk.qtile = wk.begin = wk.n = wk.col0 = wk.gid0 = wk.gbegin = wk.gcount = 0;
        wk.slot = wk.split = -1;
        wk.code0[0] = wk.code0[1] = -2;
        if (wk.valid) {
            struct Pair { int32_t bh, index; };
            const Pair pr = uniform_load(reinterpret_cast<const Pair *>(p.order) + list_at + pos);
            wk.valid = pr.bh >= 0;
            wk.bh = max(pr.bh, 0);
            wk.b = wk.bh / p.H;
            wk.h = wk.bh - wk.b * p.H;
            if (wk.valid) {
                const Item *ip = p.items + pr.index;
                struct ItemHead { int32_t qtile, begin, end, slot; };
                const ItemHead item = uniform_load(reinterpret_cast<const ItemHead *>(ip));
                if constexpr (GATHER) {
                    wk.gbegin = uniform_load(&ip->gbegin);
                    wk.gcount = uniform_load(&ip->gcount);
                }
                wk.qtile = item.qtile;
                wk.begin = item.begin;
                wk.n = item.end - item.begin;
                wk.slot = item.slot;
                if (item.slot >= 0) wk.split = uniform_load(&ip->split);
                const UEntry e0 = uniform_load(p.uent + item.begin);  // (the array ends with a spare entry)
                wk.col0 = e0.col;
                wk.gid0 = wk.n > 0 ? e0.gather : 0;
                wk.code0[0] = wk.n > 0 ? e0.code[0] : -2;
                wk.code0[1] = wk.n > 0 ? e0.code[1] : -2;
            }
        }
        return wk;
    };

    const int ksb = (int)p.ks.s * 2, vsb = (int)p.vs.s * 2;  // row pitch in bytes
    // global -> LDS: wave w fills the 1 KiB blocks w, w+4, ... of each tile; LDS chunk (row, pc)
    // receives global chunk pc ^ swz(row).  Block w + 4 i starts 64 i / CPR * 4 rows (a multiple
    // of 16) below block w, which leaves the swizzle alone: one per-lane offset serves all i.
    // (D = 256: the blocks are 8 rows apart, and the K swizzle of a wave's odd blocks differs from that of
    // its even ones in bit 3: a second offset)
    constexpr int RSTEP = 4 * 64 / CPR;  // rows between two of a wave's blocks
    constexpr int NKO = RSTEP % 16 ? 2 : 1;
    // A head narrower than D has no chunks d/8 .. CPR-1: a lane whose chunk is one of them carries kNoChunk
    // instead of its offset.  Offsets are unsigned 32-bit sums below 2^31 (the host checks the sizes), so with
    // kNoChunk added they stay past every buffer, the load returns zeros and a store is dropped.
    constexpr uint32_t kNoChunk = 0x80000000u;
    const int cpr_d = p.d >> 3;  // chunks a row has in memory
    uint32_t k_go[NKO], v_go;  // (block i of the wave: k_go[i % NKO] + i RSTEP rows)
    uint32_t g_kc[NKO], g_vc;  // with gathered tiles a staged row may come from any key: offset = key * pitch + chunk part
    const int g_row = (w * 64 + lane) / CPR;  // the lane's row in the wave's first block
    {
        const int pchunk = w * 64 + lane;
        const int row = pchunk / CPR, pc = pchunk % CPR;
        const int vc = pc ^ swz_v<D>(row);
        v_go = vc < cpr_d ? (uint32_t)(row * vsb + vc * 16) : kNoChunk;
        g_vc = vc < cpr_d ? (uint32_t)(vc * 16) : kNoChunk;
#pragma unroll
        for (int o = 0; o < NKO; ++o) {
            const int kc = pc ^ swz_k<D>(row + o * RSTEP);
            k_go[o] = kc < cpr_d ? (uint32_t)(row * ksb + kc * 16) : kNoChunk;
            g_kc[o] = kc < cpr_d ? (uint32_t)(kc * 16) : kNoChunk;
        }
    }
    const uint32_t gix_lds = (uint32_t)(uintptr_t)(lds_void *)gix;

    // state of the item being started / computed
    u32x4 rK, rV;
    // the item's entries, one per lane (at most 64, the planner cuts longer lists): requested
    // here, not touched before the item's first wait
    int raw_col = 0, raw_code0 = -2, raw_code1 = -2, raw_gid = 0;
    uint64_t raw_word = 0;  // bitmap word of the first tile (see fetch_word below)
    // Each wave has a private quarter of the second buffer pair (free between items): its 32 Q rows
    // are staged there (full-line requests instead of 32 partial lines per fragment load), and the
    // binary16 / bfloat16 output tile is transposed there into whole rows before it is stored.
    uint16_t *const priv = smem + (w < 2 ? 1 : 3) * TILE + (w & 1) * (32 * D);
    const uint32_t priv_lds = smem_base + ((w < 2 ? 1 : 3) * TILE + (w & 1) * (32 * D)) * 2;
    constexpr int NQL = CPR / 2;  // 1 KiB pieces of a 32-row slab
    // Request everything an item needs before its first tile can be computed.
    auto start_work = [&](const Work &wk) __attribute__((always_inline)) {
        const u32x4 rQ = make_rsrc4(p.Q + wk.b * p.qs.b + wk.h * p.qs.h, ((int64_t)(S - 1) * p.qs.s + p.d) * 2);
        rK = make_rsrc4(p.K + wk.b * p.ks.b + wk.h * p.ks.h, ((int64_t)(p.Sk - 1) * p.ks.s + p.d) * 2);
        rV = make_rsrc4(p.V + wk.b * p.vs.b + wk.h * p.vs.h, ((int64_t)(p.Sk - 1) * p.vs.s + p.d) * 2);
        {
            // (one 16-byte request per lane: every memory instruction here holds the wave ~100 cycles)
            typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
            static_assert(sizeof(UEntry) == 16, "an entry is loaded as one vector");
            const UEntry *u = p.uent + wk.begin + min(lane, max(wk.n - 1, 0));
            const i32x4 ev = __builtin_nontemporal_load(reinterpret_cast<const i32x4 *>(u));
            raw_col = ev[0];
            raw_code0 = ev[1];
            raw_code1 = ev[2];
            if constexpr (GATHER) raw_gid = ev[3];
            const int c0 = (w >> 1) ? wk.code0[1] : wk.code0[0];
            raw_word = 0;
            if (c0 >= 0) raw_word = p.kt_bitmap[(size_t)c0 * 64 + 32 * (w & 1) + j];
        }
        // Q rows q0 .. q0+31 -> private slab, chunks swizzled like a K tile's (rows past S: zeros)
        const int q0 = wk.qtile * 128 + 32 * w;
        int lane_o = lane;
        asm volatile("" : "+v"(lane_o));  // keeps the per-lane offsets below out of long-lived registers
#pragma unroll
        for (int i = 0; i < NQL; ++i) {
            const int pchunk = i * 64 + lane_o;
            const int row = pchunk / CPR, pc = pchunk % CPR;
            const int qc = pc ^ swz_k<D>(row);
            load_to_lds(rQ, priv_lds + i * 1024, qc < cpr_d ? (q0 + row) * (int)p.qs.s * 2 + qc * 16 : (int)kNoChunk);
        }
        if constexpr (GATHER) {
            // the key numbers of the item's gathered tiles -> LDS; wave w brings blocks 4 w .. 4 w + 3
            if (4 * w < wk.gcount) {
                const u32x4 rG = make_rsrc4(p.gidx, (int64_t)p.n_gidx * 4);
                load_to_lds(rG, gix_lds + w * 1024, ((wk.gbegin + 4 * w) * 64 + lane * 4) * 4);
            }
            // first tile: its key numbers, if it is a gathered one, come straight from memory (the
            // planner puts gathered tiles last, so this only happens in items that have no other)
            int key[LPW];
#pragma unroll
            for (int i = 0; i < LPW; ++i) key[i] = wk.col0 * 64 + g_row + i * RSTEP;
            if (wk.gid0 > 0) {
#pragma unroll
                for (int i = 0; i < LPW; ++i) key[i] = p.gidx[(size_t)(wk.gid0 - 1) * 64 + g_row + i * RSTEP];
            }
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                load_to_lds(rK, smem_base + (w + 4 * i) * 1024, g_kc[i % NKO] + (wk.n > 0 ? key[i] * ksb : OOB));
                load_to_lds(rV, smem_base + 2 * TB + (w + 4 * i) * 1024, g_vc + (wk.n > 0 ? key[i] * vsb : OOB));
            }
        } else {
            const int kb = wk.n > 0 ? wk.col0 * 64 * ksb : OOB, vb = wk.n > 0 ? wk.col0 * 64 * vsb : OOB;
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                load_to_lds(rK, smem_base + (w + 4 * i) * 1024, k_go[i % NKO] + (kb + i * RSTEP * ksb));
                load_to_lds(rV, smem_base + 2 * TB + (w + 4 * i) * 1024, v_go + (vb + i * RSTEP * vsb));
            }
        }
    };
    // Invariant at the top of the loop: everything requested for the item has landed (each way
    // into the loop ends with the wait that makes it so, which lets the compiler see it too).
    int pos = blockIdx.x >> 3;
    int turn = 0;        // how many items this workgroup has taken
    uint64_t owned = 0;  // wave-uniform: see put_split_part
    Work item = fetch_work(pos);
    if (item.valid) start_work(item);
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
    while (item.valid) {
    // the next item's descriptor: scalar loads that complete under this item's tiles
    pos += per_xcd;
    const Work nxt = fetch_work(pos);
    const int n = item.n;
    const int b = item.b, h = item.h, bh = item.bh;
    int e_col, e_code, e_gid = 0;
    const int q0 = item.qtile * 128 + 32 * w;

    auto entry_col = [&](int t) __attribute__((always_inline)) { return __builtin_amdgcn_readlane(e_col, t & 63); };
    auto entry_code = [&](int t) __attribute__((always_inline)) {
        return t < n ? __builtin_amdgcn_readlane(e_code, t & 63) : -2;
    };
    // bitmap word of this lane's query row for a part tile (callers skip full and empty tiles; the
    // spare block only keeps the index valid if one does not)
    auto fetch_word = [&](int code) __attribute__((always_inline)) {
        const int blk = code >= 0 ? code : p.bmp_spare;
        return p.kt_bitmap[(size_t)blk * 64 + 32 * (w & 1) + j];
    };

    // the wave's 2 LPW load instructions of one tile (K and V pieces alternate)
    int ld_kb = OOB, ld_vb = OOB;
    int ld_key[GATHER ? LPW : 1];  // with gathered tiles: the key each of the lane's staged rows comes from
    bool ld_live = false;
    auto load_begin = [&](int t) __attribute__((always_inline)) {  // past the end: zeros, no traffic
        const int col = entry_col(t);
        if constexpr (GATHER) {
            const int gid = t < n ? __builtin_amdgcn_readlane(e_gid, t & 63) : 0;
            const int slot = max(gid - 1 - item.gbegin, 0);
            ld_live = t < n;
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                const int from_list = gix[slot * 64 + g_row + i * RSTEP];
                ld_key[i] = gid > 0 ? from_list : col * 64 + g_row + i * RSTEP;
            }
        } else {
            ld_kb = t < n ? col * 64 * ksb : OOB;
            ld_vb = t < n ? col * 64 * vsb : OOB;
        }
    };
    auto load_piece = [&](int i, uint32_t Kd, uint32_t Vd) __attribute__((always_inline)) {  // i in [0, 2 LPW); LDS byte addresses
        if constexpr (GATHER) {
            if (i & 1)
                load_to_lds(rV, Vd + (w + 4 * (i >> 1)) * 1024, g_vc + (ld_live ? ld_key[i >> 1] * vsb : OOB));
            else
                load_to_lds(rK, Kd + (w + 4 * (i >> 1)) * 1024, g_kc[(i >> 1) % NKO] + (ld_live ? ld_key[i >> 1] * ksb : OOB));
        } else if (i & 1)
            load_to_lds(rV, Vd + (w + 4 * (i >> 1)) * 1024, v_go + (ld_vb + (i >> 1) * RSTEP * vsb));
        else
            load_to_lds(rK, Kd + (w + 4 * (i >> 1)) * 1024, k_go[(i >> 1) % NKO] + (ld_kb + (i >> 1) * RSTEP * ksb));
    };

    u32x4 qf[NS];  // Q^T operand: lane (j, hh) holds Q[q0 + j][16 s + 8 hh .. +8], read from the slab below
    float m_run = NEG_INF, l_run = 0.f;
    f32x16 o[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) o[dt] = zero16;

    // one tile for this wave
    auto compute_tile = [&](int k_off, int v_off, uint32_t Kn, uint32_t Vn, int code, uint64_t word) __attribute__((always_inline)) {
        // this tile's operand read addresses (bytes inside smem)
        const int krd = k_rd + k_off, vrd = v_rd + v_off;
        if (code >= 0 && __builtin_amdgcn_ballot_w64(word != 0) == 0) return;  // nothing for these 32 rows
        // scores, transposed: acc[kt][r] = S[q = j][key = 32 kt + 8 (r/4) + 4 hh + r%4].
        // Fragments are requested PF MFMAs ahead of their use (LDS latency is several MFMAs).
        f32x16 acc[2] = {zero16, zero16};
        auto k_addr = [&](int i) __attribute__((always_inline)) {  // i = 2 s + kt
            const int s = i >> 1, kt = i & 1;
            return reinterpret_cast<const char *>(smem) + ((krd ^ (32 * s)) + 64 * kt * D);
        };
        u32x4 kfrag[PF];
#pragma unroll
        for (int i = 0; i < PF; ++i) kfrag[i] = *reinterpret_cast<const u32x4 *>(k_addr(i));
        __builtin_amdgcn_sched_barrier(0);  // keep the requests ahead of the MFMAs that follow
#pragma unroll
        for (int i = 0; i < 2 * NS; ++i) {  // the two accumulator chains alternate
            acc[i & 1] = mfma32<BF16>(kfrag[i % PF], qf[i >> 1], acc[i & 1]);
            if (i + PF < 2 * NS) kfrag[i % PF] = *reinterpret_cast<const u32x4 *>(k_addr(i + PF));
            __builtin_amdgcn_sched_barrier(0);
        }
        // From here to the end of the tile the wave mixes vector-ALU work with its MFMAs: it gets issue
        // priority over waves that are in their pure-MFMA phase, whose MFMAs fill the gaps (measured:
        // 6 % on cfg4 with four waves per SIMD, nothing lost elsewhere).
        __builtin_amdgcn_s_setprio(1);
        if (code >= 0) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const uint32_t bits = (uint32_t)(word >> (32 * kt)) >> (4 * hh);
                // two instructions per score: the key's bit spread over a word (0 or all ones), then a
                // bitwise select between the score and -inf.  (Written on the whole vector: the same
                // expression element by element was compiled into code that used element 0 for every score.)
                typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
                u32x16 keep;
#pragma unroll
                for (int r = 0; r < 16; ++r) keep[r] = (uint32_t)__builtin_amdgcn_sbfe((int)bits, 8 * (r / 4) + (r % 4), 1);
                const u32x16 sc = __builtin_bit_cast(u32x16, acc[kt]);
                acc[kt] = __builtin_bit_cast(f32x16, (sc & keep) | (~keep & 0xFF800000u));
            }
        }
        // Lazily raised reference: probabilities are formed against the running reference m_run
        // as long as no score of the tile exceeds it by more than 8 / c (they then stay below 2^8:
        // safe in binary16, exact enough in the fp32 sums).  One test per tile, on the raw scores
        // (a test on the exponentials' sums, per key group, costs nothing in instructions but makes
        // every group's MFMAs wait for a branch on the last exponential: measured 330 instead of
        // 160 cycles per group).  Only when the test fires (always on an item's first tile, rarely
        // afterwards) is the reference raised to the tile's maximum and O and l rescaled.
        float mc = (m_run == NEG_INF ? 0.f : m_run) * p.c;
        u32x4 pf[4][NP];  // [cu = 2 kt + u: keys 16 cu .. 16 cu + 15][hi/lo]
        auto p_pair = [&](int cu, int q, float &gs) __attribute__((always_inline)) {  // pair q (0..3) of key group cu
            const int kt = cu >> 1, u = cu & 1;
            const float e0 = fast_exp2(fmaf(acc[kt][8 * u + 2 * q], p.c, -mc));
            const float e1 = fast_exp2(fmaf(acc[kt][8 * u + 2 * q + 1], p.c, -mc));
            if constexpr (BF16) {
                // bfloat16 keeps 8 significant bits: P is split into a truncated high part and a
                // rounded residual (p = hi + lo up to 2^-17); the product runs twice
                gs += e0 + e1;
                const uint32_t b0 = __builtin_bit_cast(uint32_t, e0) & 0xFFFF0000u;
                const uint32_t b1 = __builtin_bit_cast(uint32_t, e1) & 0xFFFF0000u;
                pf[cu][0][q] = (b0 >> 16) | b1;
                pf[cu][1][q] = pack2<true>(e0 - __builtin_bit_cast(float, b0), e1 - __builtin_bit_cast(float, b1));
            } else {
                // the row sum is formed from the rounded binary16 values the MFMA will use
                typedef _Float16 h2 __attribute__((ext_vector_type(2)));
                const uint32_t packed = pack2<false>(e0, e1);
                pf[cu][0][q] = packed;
                gs = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, packed), __builtin_bit_cast(h2, 0x3C003C00u), gs, false);
            }
        };
        float mt = NEG_INF;  // this lane's 32 of the row's 64 scores
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r) mt = fmaxf(mt, acc[kt][r]);
        // (m_run = -inf: any finite score fires; a row with nothing but masked keys never does)
        if (__builtin_amdgcn_ballot_w64(mt > m_run + thr_raw) != 0) {
            mt = fmaxf(mt, __shfl_xor(mt, 32));
            const float m_new = fmaxf(m_run, mt);
            const float m_use = (m_new == NEG_INF) ? 0.f : m_new;
            const float alpha = fast_exp2((m_run - m_use) * p.c);
            m_run = m_new;
            mc = m_use * p.c;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) o[dt] *= alpha;
        }
        // O^T += V^T P^T.  Fragment (cu, dt): keys 16 cu + 8 a + 4 hh + 0..3 (a = 0, 1) of columns
        // 32 dt + j: two transposing reads, requested PF MFMAs ahead.  The exponentials of key
        // group cu+1 are issued between the MFMAs of group cu, so they run under the matrix pipe.
        auto v_frag = [&](int i) __attribute__((always_inline)) {  // i = cu * NDT + dt
            const int cu = i / NDT, dt = i % NDT;
            const char *ptr = reinterpret_cast<const char *>(smem) + ((vrd ^ (64 * dt)) + 32 * cu * D);
            const u32x2 lo = lds_read_tr(reinterpret_cast<const uint16_t *>(ptr)), hi = lds_read_tr(reinterpret_cast<const uint16_t *>(ptr + 16 * D));
            return u32x4{lo[0], lo[1], hi[0], hi[1]};
        };
        u32x4 vfrag[PF];
#pragma unroll
        for (int i = 0; i < PF; ++i) vfrag[i] = v_frag(i);
        float gs = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) p_pair(0, q, gs);
#pragma unroll
        for (int cu = 0; cu < 4; ++cu) {
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) {
                const int i = cu * NDT + dt;
                o[dt] = mfma32<BF16>(vfrag[i % PF], pf[cu][0], o[dt]);
                if constexpr (BF16) o[dt] = mfma32<BF16>(vfrag[i % PF], pf[cu][1], o[dt]);
                if (i + PF < 4 * NDT) vfrag[i % PF] = v_frag(i + PF);
                if (cu < 3) {  // the next key group's four pairs, spread over this group's MFMAs
                    if constexpr (NDT <= 4) {
#pragma unroll
                        for (int q = dt * (4 / NDT); q < (dt + 1) * (4 / NDT); ++q) p_pair(cu + 1, q, gs);
                    } else {
                        if (dt % (NDT / 4) == 0) p_pair(cu + 1, dt / (NDT / 4), gs);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        l_run += gs;
        __builtin_amdgcn_s_setprio(0);
    };

    // ---- main loop: tile t is computed from one LDS buffer pair while the loads of tile t+1,
    // issued at the top of the iteration and outside every branch (with the loads inside the
    // arms of the branch below the compiler keeps the output accumulators in two register sets
    // and copies between them), land in the other pair, which every wave left at the previous
    // barrier; they are waited for at the barrier that ends tile t.  One loop body; the buffer
    // pair is a run-time offset.
    e_col = raw_col;
    if constexpr (GATHER) e_gid = raw_gid;
    e_code = lane < n ? ((w >> 1) ? raw_code1 : raw_code0) : -2;
    {
        int krd = k_rd;
        asm volatile("" : "+v"(krd));  // (the fragment addresses are made here, not kept across items)
#pragma unroll
        for (int s = 0; s < NS; ++s)
            qf[s] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(priv) + (krd ^ (32 * s)));
    }
    int code = entry_code(0);
    uint64_t word = raw_word;
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the slab is read before tile 1 may overwrite it
    __builtin_amdgcn_s_barrier();        // every wave's part of tile 0 is visible
    for (int t = 0; t < n; ++t) {
        const int par = t & 1;
        const int code_next = entry_code(t + 1);
        uint64_t word_next = 0;  // (only part tiles have a bitmap; the others never look at the word)
        if (code_next >= 0) word_next = fetch_word(code_next);
        load_begin(t + 1);
        const uint32_t Kn = smem_base + (par ^ 1) * TB, Vn = smem_base + (2 + (par ^ 1)) * TB;
#pragma unroll
        for (int i = 0; i < 2 * LPW; ++i) load_piece(i, Kn, Vn);
        if (code != -2) compute_tile(par * TB, (2 + par) * TB, Kn, Vn, code, word);
        __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0): tile t+1 landed, own LDS reads done
        __builtin_amdgcn_s_barrier();        // ... for every wave: tile t+1 visible, tile t free
        code = code_next;
        word = word_next;
    }

    // Every load issued for this item has landed and every wave is past its last LDS read (the
    // last barrier), so the next item's requests can go out now; the output stores follow them.
    // o[dt][r] = O[q = q0 + j][d = 32 dt + 8 (r/4) + 4 hh + r%4]
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const int qrow = q0 + j;
    if (item.slot < 0 && OUT != SMHA_F32) {
        // 16-bit output: the wave's 32 x D tile goes through its private LDS slab (chunk-swizzled
        // rows) and leaves as whole rows, 16 bytes per lane
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));  // (addresses below are made here, not kept in registers across the item)
        const int je = lane_e & 31, he = lane_e >> 5;
        const int o_wr = je * D * 2 + swz_k<D>(je) * 16 + he * 8;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const u32x2 v = {pack2<OUT == SMHA_BF16>(o[dt][4 * g4] * inv, o[dt][4 * g4 + 1] * inv),
                                 pack2<OUT == SMHA_BF16>(o[dt][4 * g4 + 2] * inv, o[dt][4 * g4 + 3] * inv)};
                *reinterpret_cast<u32x2 *>(reinterpret_cast<char *>(priv) + (o_wr ^ ((4 * dt + g4) * 16))) = v;
                __builtin_amdgcn_sched_barrier(0);  // (pack and write as we go: no second copy of the tile in registers)
            }
        u32x4 ov[NQL];
#pragma unroll
        for (int i = 0; i < NQL; ++i) ov[i] = *reinterpret_cast<const u32x4 *>(priv + (i * 64 + lane_e) * 8);
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the slab is read before the next Q may land in it
        if (nxt.valid) start_work(nxt);
        __builtin_amdgcn_sched_barrier(0);
        // NQL stores, every one issued by every wave (rows past S fall outside the buffer and are
        // dropped), so that the wait below can count them
        const __amdgpu_buffer_rsrc_t rO = make_rsrc(reinterpret_cast<const uint16_t *>(p.O) + b * p.os.b + h * p.os.h,
                                                    ((int64_t)(S - 1) * p.os.s + p.d) * 2);
#pragma unroll
        for (int i = 0; i < NQL; ++i) {
            const int pchunk = i * 64 + lane_e;
            const int row = pchunk / CPR, pc = pchunk % CPR;
            const int oc = pc ^ swz_k<D>(row);
            // (aux 2 = streaming: O is not read again here, and lines kept for it would push K and V out of the
            // XCD's L2: measured 144 -> 134 us on the 8k BigBird workload)
            __builtin_amdgcn_raw_buffer_store_b128(ov[i], rO, oc < cpr_d ? (q0 + row) * (int)p.os.s * 2 + oc * 16 : (int)kNoChunk, 0, 2);
        }
        // The next item's requests were issued before these stores and memory operations retire
        // in order: allowing NQL operations to stay outstanding waits for the requests only.
        __builtin_amdgcn_s_waitcnt(0x0070 | (NQL & 15) | ((NQL >> 4) << 14));  // vmcnt(NQL) lgkmcnt(0)
    } else {
        if (nxt.valid) start_work(nxt);
        __builtin_amdgcn_sched_barrier(0);
        if (item.slot < 0) {
            if (qrow < S) {
                const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
                const int64_t obase = b * p.os.b + h * p.os.h + (int64_t)qrow * p.os.s;
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4)
                        if (32 * dt + 8 * g4 + 4 * hh < p.d)
                            store4<OUT>(p.O, obase + 32 * dt + 8 * g4 + 4 * hh, o[dt][4 * g4] * inv, o[dt][4 * g4 + 1] * inv,
                                        o[dt][4 * g4 + 2] * inv, o[dt][4 * g4 + 3] * inv);
            }
        } else {
            if constexpr (SPLIT) {
                // (which of its items' groups this wave has to merge is kept as one bit per turn; from turn 63
                // on the bit only says that the counters of those turns have to be asked)
                const bool last = put_split_part<D, f32x16, NDT>(p, o, m_run * p.c /* -inf stays -inf (c > 0) */, l_tot, w, lane, b, h, bh,
                                                    item.slot, item.split);
                if (last || turn >= 63) owned |= 1ull << min(turn, 63);
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
    }
    item = nxt;
    ++turn;
    }  // persistent loop over work items
    if constexpr (SPLIT) {
        // Second walk over this workgroup's items: the split groups whose last part one of its waves wrote
        // are merged here, where nothing of the tile loop is alive any more (the merge needs many registers,
        // and inside the loop every item's start and end would pay for them).
        __builtin_amdgcn_s_waitcnt(0x0070);
        auto merge_at = [&](int pos2, bool owner_known) __attribute__((always_inline)) {
            struct Pair { int32_t bh, index; };
            const Pair pr = uniform_load(reinterpret_cast<const Pair *>(p.order) + list_at + pos2);
            if (pr.bh < 0) return;
            const Item *ip = p.items + pr.index;
            if (uniform_load(&ip->slot) < 0) return;
            const int qtile = uniform_load(&ip->qtile), split = uniform_load(&ip->split);
            const int b2 = pr.bh / p.H, h2 = pr.bh - b2 * p.H;
            merge_split_parts<D, OUT, (D == 128 ? 8 : 4), 16>(p, w, lane, b2, h2, pr.bh, qtile * 128 + 32 * w + j, split, owner_known);
        };
        while (owned) {
            const int k = __builtin_ctzll(owned);
            owned &= owned - 1;
            if (k < 63) {
                merge_at((blockIdx.x >> 3) + k * per_xcd, true);
            } else {
                for (int pos2 = (blockIdx.x >> 3) + 63 * per_xcd; pos2 < list_len; pos2 += per_xcd) merge_at(pos2, false);
            }
        }
    }
}

#include "block_fwd2.inc"
#include "block_fwd16.inc"

// ---------------------------------------------------------------------------------------
// Row-wise kernel
// ---------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false);
    return v + __builtin_bit_cast(float, moved);
}

// sum over the aligned group of LPK (8, 16 or 32) lanes; every lane of the group gets the sum
template <int LPK>
__device__ __forceinline__ float group_sum(float v) {
    v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);  // row_half_mirror: the other quad of the 8
    if constexpr (LPK >= 16) v = dpp_add<0x140>(v);  // row_mirror: the other half of the 16
    if constexpr (LPK == 32) v += __shfl_xor(v, 16);  // the other 16 of the 32
    return v;
}

// RPW query rows per wave: 1 (a whole wave per row: long rows) or 4 (16 lanes per row: rows with
// few keys, where a wave per row spends its time on set-up and on merging 8 mostly idle key groups).
template <int D, bool BF16, int RPW>
__global__ void __launch_bounds__(256) smha_row_fwd(const FwdParams p) {
    constexpr int LPK = D / 8;     // lanes that share one key (16 bytes of the row each)
    constexpr int LPR = 64 / RPW;  // lanes per query row
    constexpr int KPS = LPR / LPK; // keys a row handles per step
    constexpr int U = RPW == 1 ? 2 : 4;  // independent steps in flight
    const int wg = blockIdx.x;
    const int xcd = wg & 7, rest = wg >> 3;
    const int grp = rest / p.wgs_per_bh, rb = rest - grp * p.wgs_per_bh;
    const int bh = grp * 8 + xcd;
    if (bh >= p.B * p.H) return;
    const int b = bh / p.H, h = bh - b * p.H;
    const int mask = (p.Bm > 1 ? b : 0) * p.Hm + (p.Hm > 1 ? h : 0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i_raw = (rb * 4 + wave) * RPW + lane / LPR;
    if ((rb * 4 + wave) * RPW >= p.S) return;  // (whole waves leave together)
    const bool row_ok = i_raw < p.S;           // rows past the end stay for the shuffles below, with no keys
    const int i = row_ok ? i_raw : p.S - 1;
    const int sub_raw = lane % LPK, g = (lane % LPR) / LPK;
    // a head narrower than D: the lanes past its last column read column 0 again, with a zero query, and store nothing
    const bool col_ok = 8 * sub_raw < p.d;
    const int sub = col_ok ? sub_raw : 0;
    const float NEG_INF = -__builtin_inff();

    float qf[8];
    {
        u32x4 v = *reinterpret_cast<const u32x4 *>(p.Q + b * p.qs.b + h * p.qs.h + (int64_t)i * p.qs.s + 8 * sub);
        const float cq = col_ok ? p.c : 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            qf[2 * e] = widen16<BF16>(v[e] & 0xFFFFu) * cq;
            qf[2 * e + 1] = widen16<BF16>(v[e] >> 16) * cq;
        }
    }
    const int32_t *rp = p.row_ptr + (size_t)mask * (p.S + 1);
    const int beg = rp[i], end = row_ok ? rp[i + 1] : beg;
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
    // merge the row's KPS lane groups (butterfly over the lane bits between LPK and LPR)
#pragma unroll
    for (int off = LPK; off < LPR; off <<= 1) {
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
    if (g == 0 && row_ok && col_ok) {
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

// Mask intake on the device (Sec. 4.2.1: the mask is analysed once): a dense byte mask is
// packed into bit rows, one thread per 64-bit word = 64 mask bytes, so that only S*S/8 bytes
// cross to the host for the format analysis.  HBM-bound: S*S bytes read, S*S/8 written per mask.
// Rows have S entries (the key side); words[row * W + t] bit c = (row[64 t + c] != 0), entries
// past S are 0, where row runs over all query rows of all masks.
__global__ void __launch_bounds__(256) smha_mask_pack_bits(const uint8_t *__restrict__ mask, uint64_t *__restrict__ words,
                                                           int S, int W, long long n_words) {
    const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= n_words) return;
    const long long row = g / W;
    const int t = (int)(g - row * W);
    const uint8_t *src = mask + row * S + 64 * (long long)t;
    const int n = min(64, S - 64 * t);
    uint64_t out = 0;
    if (n == 64 && ((uintptr_t)src & 15) == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const u32x4 v = reinterpret_cast<const u32x4 *>(src)[q];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // any nonzero byte -> its bit 0, then gather the four bit-0s of the dword
                uint32_t x = v[e];
                x |= x >> 4;
                x |= x >> 2;
                x |= x >> 1;
                x &= 0x01010101u;
                out |= (uint64_t)((x * 0x10204080u) >> 28) << (16 * q + 4 * e);
            }
        }
    } else {
        for (int c = 0; c < n; ++c) out |= (uint64_t)(src[c] != 0) << c;
    }
    words[g] = out;
}

smha_status_t pack_device_mask(const uint8_t *dev_mask, int n_masks, int Sq, int Sk, uint64_t *host_words) {
    const int W = (Sk + 63) / 64;
    const long long n_words = (long long)n_masks * Sq * W;
    uint64_t *d_words = nullptr;
    if (hipMalloc(reinterpret_cast<void **>(&d_words), (size_t)n_words * 8) != hipSuccess) {
        (void)hipGetLastError();
        return SMHA_ERR_ALLOC;
    }
    const unsigned grid = (unsigned)((n_words + 255) / 256);
    hipLaunchKernelGGL(smha_mask_pack_bits, dim3(grid), dim3(256), 0, 0, dev_mask, d_words, Sk, W, n_words);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpy(host_words, d_words, (size_t)n_words * 8, hipMemcpyDeviceToHost);
    (void)hipFree(d_words);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return SMHA_ERR_HIP;
    }
    return SMHA_OK;
}

// Mask analysis on the device: one wave per 64x64 tile, lane r = row r of the tile.  Reads the
// dense mask once (HBM-bound), writes 16 bytes per tile and, for partially filled tiles only, the
// 64 bitmap words (word r = row r, bit c = key column c; entries outside the mask are 0) at a slot
// taken from a per-mask counter.  Full and empty tiles need no bitmap.
__global__ void __launch_bounds__(256) smha_mask_classify(const uint8_t *__restrict__ mask, TileInfo *__restrict__ info,
                                                          uint64_t *__restrict__ part_bits, uint32_t *__restrict__ counters,
                                                          int Sq, int Sk, int nqt, int nkt, long long n_tiles) {
    const long long tile = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= n_tiles) return;  // (whole waves leave together)
    const int lane = threadIdx.x & 63;
    const long long per_mask = (long long)nqt * nkt;
    const int mi = (int)(tile / per_mask);
    const int rem = (int)(tile - mi * per_mask);
    const int tr = rem / nkt, tc = rem - tr * nkt;
    const int row = tr * 64 + lane;
    uint64_t word = 0;
    if (row < Sq) {
        const uint8_t *src = mask + ((long long)mi * Sq + row) * Sk + 64ll * tc;
        const int n = min(64, Sk - 64 * tc);
        if (n == 64 && ((uintptr_t)src & 15) == 0) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u32x4 v = reinterpret_cast<const u32x4 *>(src)[q];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    uint32_t x = v[e];  // any nonzero byte -> its bit 0, then gather the four bit-0s
                    x |= x >> 4;
                    x |= x >> 2;
                    x |= x >> 1;
                    x &= 0x01010101u;
                    word |= (uint64_t)((x * 0x10204080u) >> 28) << (16 * q + 4 * e);
                }
            }
        } else {
            for (int c = 0; c < n; ++c) word |= (uint64_t)(src[c] != 0) << c;
        }
    }
    uint32_t cnt = __builtin_popcountll(word);
    uint64_t used = word, grp = word;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        cnt += __shfl_xor(cnt, off);
        used |= __shfl_xor(used, off);
        if (off < 16) grp |= __shfl_xor(grp, off);  // OR over the 16 rows of the lane's group
    }
    uint32_t q16 = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) q16 += ((grp >> (16 * q)) & 0xFFFFull) != 0;
    const uint32_t v16 = __shfl(q16, 0) + __shfl(q16, 16) + __shfl(q16, 32) + __shfl(q16, 48);
    uint32_t slot = 0;
    const bool part = cnt > 0 && cnt < 4096;
    if (part) {
        if (lane == 0) slot = atomicAdd(counters + mi, 1u);
        slot = __shfl(slot, 0);
        part_bits[((long long)mi * per_mask + slot) * 64 + lane] = word;
    }
    if (lane == 0) info[tile] = TileInfo{used, cnt | (v16 << 16), slot};
}

smha_status_t classify_device_mask(const uint8_t *dev_mask, int n_masks, int Sq, int Sk, std::vector<TileInfo> &info,
                                   std::vector<std::vector<uint64_t>> &part_bits) {
    const int nqt = (Sq + 63) / 64, nkt = (Sk + 63) / 64;
    const long long per_mask = (long long)nqt * nkt, n_tiles = per_mask * n_masks;
    info.resize((size_t)n_tiles);
    part_bits.assign((size_t)n_masks, {});
    // One scratch allocation {tile records, per-mask counters, bitmap slots}; it is kept for the next plan
    // (allocating and freeing tens of megabytes costs more than the analysis) unless it is very large.
    const size_t info_bytes = (size_t)n_tiles * sizeof(TileInfo), cnt_bytes = ((size_t)n_masks * 4 + 255) / 256 * 256;
    const size_t bits_at = (info_bytes + cnt_bytes + 255) / 256 * 256, total = bits_at + (size_t)n_tiles * 512;
    static std::mutex cache_mutex;
    static void *cache_ptr = nullptr;
    static size_t cache_bytes = 0;
    static int cache_device = -1;
    constexpr size_t kKeepAtMost = (size_t)128 << 20;
    std::lock_guard<std::mutex> lock(cache_mutex);  // (also serialises analyses that share the scratch)
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) {
        (void)hipGetLastError();
        return SMHA_ERR_HIP;
    }
    char *scratch_dev = nullptr;
    bool cached = false;
    if (cache_ptr && cache_device == device && cache_bytes >= total) {
        scratch_dev = (char *)cache_ptr;
        cached = true;
    } else {
        if (cache_ptr && total <= kKeepAtMost) {  // replaced by a larger one below
            int prev = device;
            (void)hipSetDevice(cache_device);
            (void)hipFree(cache_ptr);
            (void)hipSetDevice(prev);
            cache_ptr = nullptr;
            cache_bytes = 0;
        }
        if (hipMalloc(reinterpret_cast<void **>(&scratch_dev), total) != hipSuccess) {
            (void)hipGetLastError();
            return SMHA_ERR_ALLOC;
        }
        if (total <= kKeepAtMost) {
            cache_ptr = scratch_dev;
            cache_bytes = total;
            cache_device = device;
            cached = true;
        }
    }
    TileInfo *d_info = reinterpret_cast<TileInfo *>(scratch_dev);
    uint32_t *d_cnt = reinterpret_cast<uint32_t *>(scratch_dev + info_bytes);
    uint64_t *d_bits = reinterpret_cast<uint64_t *>(scratch_dev + bits_at);
    auto done = [&](smha_status_t st) {
        if (st != SMHA_OK) (void)hipGetLastError();
        if (!cached) (void)hipFree(scratch_dev);
        return st;
    };
    if (hipMemsetAsync(d_cnt, 0, (size_t)n_masks * 4, 0) != hipSuccess) return done(SMHA_ERR_HIP);
    const unsigned grid = (unsigned)((n_tiles + 3) / 4);
    hipLaunchKernelGGL(smha_mask_classify, dim3(grid), dim3(256), 0, 0, dev_mask, d_info, d_bits, d_cnt, Sq, Sk, nqt, nkt, n_tiles);
    if (hipGetLastError() != hipSuccess) return done(SMHA_ERR_HIP);
    // (tile records and counters are adjacent: one copy)
    std::vector<char> back(info_bytes + (size_t)n_masks * 4);
    if (hipMemcpy(back.data(), scratch_dev, back.size(), hipMemcpyDeviceToHost) != hipSuccess) return done(SMHA_ERR_HIP);
    std::memcpy(info.data(), back.data(), info_bytes);
    std::vector<uint32_t> n_part((size_t)n_masks);
    std::memcpy(n_part.data(), back.data() + info_bytes, (size_t)n_masks * 4);
    for (int mi = 0; mi < n_masks; ++mi) {
        if (!n_part[mi]) continue;
        part_bits[mi].resize((size_t)n_part[mi] * 64);
        if (hipMemcpy(part_bits[mi].data(), d_bits + (size_t)mi * per_mask * 64, (size_t)n_part[mi] * 512,
                      hipMemcpyDeviceToHost) != hipSuccess)
            return done(SMHA_ERR_HIP);
    }
    return done(SMHA_OK);
}

// Every index array of a plan lives in one device allocation, filled with one copy: a plan has up to 18
// arrays, and an allocation and a copy each cost more than the analysis of a small mask.
struct Arena {
    std::vector<char> host;
    std::vector<std::pair<void **, size_t>> fixups;  // (pointer to set, offset)
    template <typename T>
    void add(T *&dst, const std::vector<T> &src) {
        const size_t at = (host.size() + 255) / 256 * 256;
        host.resize(at + std::max<size_t>(src.size(), 1) * sizeof(T));
        if (!src.empty()) std::memcpy(host.data() + at, src.data(), src.size() * sizeof(T));
        fixups.push_back({reinterpret_cast<void **>(&dst), at});
    }
};

static int compute_units_of(int device_id) {
    static std::mutex m;
    static int cached[64] = {0};
    std::lock_guard<std::mutex> lock(m);
    if (device_id >= 0 && device_id < 64 && cached[device_id]) return cached[device_id];
    hipDeviceProp_t prop;
    int n = hipGetDeviceProperties(&prop, device_id) == hipSuccess ? prop.multiProcessorCount : 256;
    if (n < 8) n = 8;
    n = (n + 7) / 8 * 8;
    if (device_id >= 0 && device_id < 64) cached[device_id] = n;
    return n;
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
    DeviceArrays &d = p->dev;
    p->device = device_id;
    p->n_cu = compute_units_of(device_id);
    Arena arena;
    if (p->has_row) {
        arena.add(d.row_ptr, p->h_row_ptr);
        arena.add(d.col_idx, p->h_col_idx);
        arena.add(d.col_off, p->h_col_off);
    }
    if (p->has_block) {
        arena.add(d.uent, p->h_uent);
        arena.add(d.gidx, p->h_gidx);
        arena.add(d.kt_bitmap, p->h_kt_bitmap);
        for (int lvl = 0; lvl < (p->fine_differs ? 2 : 1); ++lvl) {
            const WorkLists &wl = p->lists[lvl];
            arena.add(d.items[lvl], wl.items);
            arena.add(d.item_off[lvl], wl.item_off);
            arena.add(d.item_cnt[lvl], wl.item_cnt);
            arena.add(d.split_rows[lvl], wl.split_rows);
            arena.add(d.split_off[lvl], wl.split_off);
            arena.add(d.split_cnt[lvl], wl.split_cnt);
        }
    }
    bool ok = true;
    if (!arena.host.empty()) {
        ok = hipMalloc(&d.arena, arena.host.size()) == hipSuccess &&
             hipMemcpy(d.arena, arena.host.data(), arena.host.size(), hipMemcpyHostToDevice) == hipSuccess;
        if (ok)
            for (auto &f : arena.fixups) *f.first = (char *)d.arena + f.second;
    }
    (void)hipSetDevice(prev);
    if (!ok) {
        (void)hipGetLastError();
        for (auto &f : arena.fixups) *f.first = nullptr;
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
    if (d.arena) (void)hipFree(d.arena);
    d = DeviceArrays{};
    for (smha_plan::Prepared *pr : p->prepared) {
        if (pr->order) (void)hipFree(pr->order);
        for (void *q : pr->ws)
            if (q) (void)hipFree(q);
        delete pr;
    }
    p->prepared.clear();
    p->device = -1;
    (void)hipSetDevice(prev);
}

}  // namespace smha

// ---------------------------------------------------------------------------------------
// smha_forward
// ---------------------------------------------------------------------------------------
using namespace smha;

static bool strides_ok(const int64_t *s) { return !s || (s[0] % 8 == 0 && s[1] % 8 == 0 && s[2] % 8 == 0 && s[2] > 0); }

// Which form of the block kernel runs a call: the plan's block_form option, else SMHA_BLOCK_FORM=1 or 2 in
// the environment (read once), else the first form (on the workloads measured so far it is the faster
// one).  Plans with gathered tiles, and bfloat16 at d = 128 (the second form's LDS does not hold two
// probability operands per step there), run the first form whatever is asked for.
static int block_form(const smha_plan *plan, int d, bool bf16) {
    static const int from_env = [] {
        const char *e = getenv("SMHA_BLOCK_FORM");
        return e ? atoi(e) : 0;
    }();
    const int asked = plan->opts.block_form ? plan->opts.block_form : from_env;
    if (plan->n_gathered > 0) return 1;
    if (d > 128) return asked == 1 ? 1 : 3;  // 256 columns: eight waves of 16 rows are two waves per SIMD, four of 32 are one
    if (asked == 3) return d == 128 ? 3 : 1;  // eight waves of 16 rows: 128 and 256 columns
    if (asked == 0) return d == 128 && !plan->dense_long_lists ? 3 : 1;  // the library's choice
    if (bf16 && d == 128) return 1;
    return asked == 2 ? 2 : 1;
}
static int workgroups_per_cu(int form, int d) { return form == 2 ? 1 : form == 3 ? (d > 128 ? 1 : 2) : (d == 64 ? 4 : d == 128 ? 2 : 1); }

template <int D, bool BF16, int OUT>
static hipError_t launch_block_out(const smha_plan *plan, FwdParams &fp, hipStream_t stream) {
    if (fp.n_work == 0) return hipSuccess;
    if constexpr (!(BF16 && D == 128) && D <= 128) {
        if (fp.form == 2) {
            hipLaunchKernelGGL((smha_block_fwd2<D, BF16, OUT>), dim3(8u * (unsigned)fp.per_xcd), dim3(512), 0, stream, fp);
            return hipGetLastError();
        }
    }
    // the grid fills the chip once (two workgroups fit a CU at d = 128, four at d = 64: LDS and
    // registers); the work order was made for exactly this many workgroups
    const unsigned grid = 8u * (unsigned)fp.per_xcd;
    const bool split = fp.max_slots > 0;
    if constexpr (D >= 128) {
        if (fp.form == 3) {  // eight waves of 16 rows (plans without gathered tiles; at 64 columns the form also
                             // works, but fits two workgroups per compute unit where the first form fits four,
                             // and was 10-20 % slower on every mask measured: not instantiated)
            if (split)
                hipLaunchKernelGGL((smha_block_fwd16<D, BF16, OUT, true>), dim3(grid), dim3(512), 0, stream, fp);
            else
                hipLaunchKernelGGL((smha_block_fwd16<D, BF16, OUT, false>), dim3(grid), dim3(512), 0, stream, fp);
            return hipGetLastError();
        }
    }
    if (plan->n_gathered > 0) {
        if (split)
            hipLaunchKernelGGL((smha_block_fwd<D, BF16, OUT, true, true>), dim3(grid), dim3(256), 0, stream, fp);
        else
            hipLaunchKernelGGL((smha_block_fwd<D, BF16, OUT, true, false>), dim3(grid), dim3(256), 0, stream, fp);
    } else {
        if (split)
            hipLaunchKernelGGL((smha_block_fwd<D, BF16, OUT, false, true>), dim3(grid), dim3(256), 0, stream, fp);
        else
            hipLaunchKernelGGL((smha_block_fwd<D, BF16, OUT, false, false>), dim3(grid), dim3(256), 0, stream, fp);
    }
    return hipGetLastError();
}

template <int D, bool BF16>
static hipError_t launch_block(const smha_plan *plan, FwdParams &fp, hipStream_t stream) {
    if (fp.out_dtype == SMHA_F32) return launch_block_out<D, BF16, SMHA_F32>(plan, fp, stream);
    return launch_block_out<D, BF16, BF16 ? SMHA_BF16 : SMHA_F16>(plan, fp, stream);
}

template <int D, bool BF16>
static hipError_t launch_row(const smha_plan *plan, FwdParams &fp, hipStream_t stream) {
    const int BH = fp.B * fp.H;
    const int groups = (BH + 7) / 8;
    // rows with few keys share a wave (see the kernel): decided from the mean row length of the plan
    const bool short_rows = plan->row_mean_nnz <= 32.0;
    constexpr int RPW = D <= 128 ? 4 : 2;  // rows of a wave when rows are short (a row needs D / 8 lanes per key)
    const int rows_per_wg = short_rows ? 4 * RPW : 4;
    fp.wgs_per_bh = (fp.S + rows_per_wg - 1) / rows_per_wg;
    const unsigned grid = (unsigned)(8 * groups * fp.wgs_per_bh);
    if (short_rows)
        hipLaunchKernelGGL((smha_row_fwd<D, BF16, RPW>), dim3(grid), dim3(256), 0, stream, fp);
    else
        hipLaunchKernelGGL((smha_row_fwd<D, BF16, 1>), dim3(grid), dim3(256), 0, stream, fp);
    return hipGetLastError();
}

// Which grain of work items a call walks: the coarse lists unless they leave more than half of the
// chip's workgroup slots empty for this batch and head count (then the longest list would be the launch).
static int grain_for(const smha_plan *plan, int B, int H, int d, int form) {
    if (!plan->fine_differs || !plan->has_block) return 0;
    int64_t n_items = 0;
    const WorkLists &w0 = plan->lists[0];
    if (plan->Bm == 1 && plan->Hm == 1)
        n_items = (int64_t)B * H * w0.item_cnt[0];
    else
        for (int bh = 0; bh < B * H; ++bh)
            n_items += w0.item_cnt[(plan->Bm > 1 ? bh / H : 0) * plan->Hm + (plan->Hm > 1 ? bh % H : 0)];
    return 2 * n_items < (int64_t)workgroups_per_cu(form, d) * plan->n_cu ? 1 : 0;
}

// The work order and workspaces for a call shape: found, or made now (allocates and copies; nothing
// that exists is freed or moved).  *ws receives the workspace for this call (null if the plan splits
// no group).
static smha_status_t prepared_for(const smha_plan *plan, int B, int H, int d, int lvl, int form,
                                  const smha_plan::Prepared **out, void **ws, bool may_allocate = true) {
    std::lock_guard<std::mutex> lock(plan->prepared_mutex);
    smha_plan::Prepared *hit = nullptr;
    for (smha_plan::Prepared *q : plan->prepared)
        if (q->B == B && q->H == H && q->d == d && q->lvl == lvl && q->form == form) hit = q;
    if (!hit && !may_allocate) return SMHA_ERR_UNSUPPORTED;
    if (!hit) {
        const WorkLists &wl = plan->lists[plan->fine_differs ? lvl : 0];
        if ((int64_t)B * H * wl.max_items > ((int64_t)1 << 28)) return SMHA_ERR_UNSUPPORTED;  // (the order table indexes items with 32 bits)
        std::vector<int32_t> table;
        int per_xcd = 0, longest = 0;
        int64_t step_words = 0, item_words = 0;
        const int slots = workgroups_per_cu(form, d) * plan->n_cu / 8;  // workgroups that fit an XCD at once
        smha_plan::Prepared *q = nullptr;
        try {
            build_work_order(plan, lvl, B, H, slots, table, per_xcd);
            longest = 0;
            for (int x = 0; x < 8; ++x) longest = std::max(longest, table[8 + x]);
            if (form == 2) {
                // The second form walks, per workgroup, one contiguous stream of steps and one of items
                // (see StepRec / ItemRec): {8 offsets} + per workgroup {first step, steps, first item,
                // items} + step records + item records.
                const int n_wg = 8 * per_xcd;
                std::vector<int32_t> hdr((size_t)4 * n_wg, 0), steps, items;
                for (int wg = 0; wg < n_wg; ++wg) {
                    const int x = wg & 7, r = wg >> 3;
                    hdr[4 * wg] = (int32_t)(steps.size() / 4);
                    hdr[4 * wg + 2] = (int32_t)(items.size() / 8);
                    int n_it = 0;
                    for (int pos = r; pos < table[8 + x]; pos += per_xcd) {
                        const int32_t bh = table[16 + 2 * (table[x] + pos)];
                        if (bh < 0) break;
                        const Item &it = wl.items[table[16 + 2 * (table[x] + pos) + 1]];
                        const int32_t rec[8] = {bh / H, bh % H, it.qtile, it.slot, it.split, 0, 0, 0};
                        items.insert(items.end(), rec, rec + 8);
                        const int n = it.end - it.begin;
                        for (int e = 0; e < std::max(n, 1); ++e) {  // (an item without entries is one step that loads and computes nothing)
                            const int32_t meta = n_it | (e == 0 ? kStepFirst : 0) | (e == std::max(n, 1) - 1 ? kStepLast : 0);
                            const UEntry none{-1, {-2, -2}, 0};
                            const UEntry &u = n > 0 ? plan->h_uent[it.begin + e] : none;
                            const int32_t st[4] = {u.col, u.code[0], u.code[1], meta};
                            steps.insert(steps.end(), st, st + 4);
                        }
                        ++n_it;
                    }
                    hdr[4 * wg + 1] = (int32_t)(steps.size() / 4) - hdr[4 * wg];
                    hdr[4 * wg + 3] = n_it;
                }
                if (items.size() / 8 > (size_t)kStepItemMask || steps.size() / 4 > (size_t)INT32_MAX / 16) return SMHA_ERR_UNSUPPORTED;
                std::vector<int32_t> all(8, 0);
                all[0] = 8;                                  // per-workgroup headers
                all[1] = all[0] + (int32_t)hdr.size();       // step records
                all[2] = all[1] + (int32_t)steps.size();     // item records
                all[3] = all[2] + (int32_t)items.size();     // end
                all.insert(all.end(), hdr.begin(), hdr.end());
                all.insert(all.end(), steps.begin(), steps.end());
                all.insert(all.end(), items.begin(), items.end());
                all.resize(all.size() + 256, 0);             // (whole 1 KiB requests past the last record stay inside the buffer's bounds check anyway; slack for tidiness)
                table.swap(all);
                step_words = (int64_t)steps.size();
                item_words = (int64_t)items.size();
            }
            q = new smha_plan::Prepared();
        } catch (const std::bad_alloc &) {
            return SMHA_ERR_ALLOC;
        }
        q->B = B; q->H = H; q->d = d; q->lvl = lvl; q->form = form; q->per_xcd = per_xcd;
        q->longest = longest;
        q->step_words = step_words;
        q->item_words = item_words;
        bool ok = hipMalloc((void **)&q->order, table.size() * sizeof(int32_t)) == hipSuccess &&
                  hipMemcpy(q->order, table.data(), table.size() * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess;
        if (ok && wl.max_slots > 0) {
            q->ws_bytes = workspace_bytes(plan, lvl, B, H, d, &q->counters_at);
            // (the counters start at zero and every launch leaves them at zero; the copy has completed on return)
            const std::vector<uint32_t> zeros((q->ws_bytes - q->counters_at) / sizeof(uint32_t), 0u);
            for (int i = 0; ok && i < smha_plan::kCallSlots; ++i)
                ok = hipMalloc(&q->ws[i], q->ws_bytes) == hipSuccess &&
                     hipMemcpy((char *)q->ws[i] + q->counters_at, zeros.data(), zeros.size() * sizeof(uint32_t),
                               hipMemcpyHostToDevice) == hipSuccess;
        }
        if (ok) {
            try {
                plan->prepared.push_back(q);
            } catch (const std::bad_alloc &) {
                ok = false;
            }
        }
        if (!ok) {
            (void)hipGetLastError();
            if (q->order) (void)hipFree(q->order);
            for (void *w : q->ws)
                if (w) (void)hipFree(w);
            delete q;
            return SMHA_ERR_ALLOC;
        }
        hit = q;
    }
    *out = hit;
    *ws = hit->ws_bytes ? hit->ws[hit->next++ % smha_plan::kCallSlots] : nullptr;
    return SMHA_OK;
}

// Head sizes: any multiple of 8 up to 256.  The kernels exist for 64, 128 and 256 columns; a narrower head
// runs on the next of the three, its missing columns read as zeros (which changes no score) and never stored.
static bool head_size_ok(int d) { return d >= 8 && d <= 256 && d % 8 == 0; }
static int kernel_head_size(int d) { return d <= 64 ? 64 : d <= 128 ? 128 : 256; }

static smha_status_t check_shape(const smha_plan *plan, int B, int H, int d) {
    if (!plan || B < 1 || H < 1) return SMHA_ERR_INVALID_ARG;
    if (!head_size_ok(d)) return SMHA_ERR_UNSUPPORTED;
    if ((plan->Bm != 1 && plan->Bm != B) || (plan->Hm != 1 && plan->Hm != H)) return SMHA_ERR_SHAPE;
    if ((int64_t)B * H > (1 << 24)) return SMHA_ERR_UNSUPPORTED;
    return SMHA_OK;
}

extern "C" smha_status_t smha_plan_prepare(const smha_plan_t *plan, int B, int H, int d) {
    const smha_status_t st = check_shape(plan, B, H, d);
    if (st != SMHA_OK) return st;
    if (!plan->has_block) return SMHA_OK;  // the row kernel needs nothing per shape
    if (plan->device < 0) return SMHA_ERR_HIP;
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess || cur != plan->device) {
        (void)hipGetLastError();
        return SMHA_ERR_HIP;
    }
    const int D = kernel_head_size(d);
    for (int bf16 = 0; bf16 < 2; ++bf16) {  // (the two input types may run different forms of the kernel)
        int form = block_form(plan, D, bf16 != 0);
        if (form == 2 && d != D) form = 1;  // (the second form has no narrower heads)
        const smha_plan::Prepared *pr = nullptr;
        void *ws = nullptr;
        const smha_status_t s2 = prepared_for(plan, B, H, D, grain_for(plan, B, H, D, form), form, &pr, &ws);
        if (s2 != SMHA_OK) return s2;
    }
    return SMHA_OK;
}

// Workspace in the library's own image, for callers that cannot allocate: one array per GPU, kept
// until the process ends.  Host code only ever uses the address hipGetSymbolAddress returns for the
// current device (the array's name is not a device address on the host side).
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex static_scratch_mutex;
static void *static_scratch_ptr[kMaxDevices];  // per device, null until asked for

static void *static_scratch_for(int device) {
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(static_scratch_mutex);
    if (!static_scratch_ptr[device]) {  // (the caller has made `device` current)
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        static_scratch_ptr[device] = ptr;
    }
    return static_scratch_ptr[device];
}

__global__ void smha_fill_zero(uint32_t *dst, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0u;
}

static smha_status_t forward_impl(const smha_plan_t *plan, const void *Q, const void *K,
                                      const void *V, void *O, int B, int H, int d,
                                      smha_dtype_t in_dtype, smha_dtype_t out_dtype,
                                      const int64_t q_strides[3], const int64_t k_strides[3],
                                      const int64_t v_strides[3], const int64_t o_strides[3],
                                      float scale, smha_kernel_t kernel, void *hip_stream, bool static_ws) {
    if (!plan || !Q || !K || !V || !O || B < 1 || H < 1) return SMHA_ERR_INVALID_ARG;
    if (in_dtype != SMHA_F16 && in_dtype != SMHA_BF16) return SMHA_ERR_UNSUPPORTED;
    if (out_dtype != in_dtype && out_dtype != SMHA_F32) return SMHA_ERR_UNSUPPORTED;
    if (!head_size_ok(d)) return SMHA_ERR_UNSUPPORTED;
    const int D = kernel_head_size(d);
    if (kernel < SMHA_KERNEL_AUTO || kernel > SMHA_KERNEL_BLOCK) return SMHA_ERR_INVALID_ARG;
    if ((plan->Bm != 1 && plan->Bm != B) || (plan->Hm != 1 && plan->Hm != H)) return SMHA_ERR_SHAPE;
    if (!strides_ok(q_strides) || !strides_ok(k_strides) || !strides_ok(v_strides) || !strides_ok(o_strides))
        return SMHA_ERR_UNSUPPORTED;
    const uintptr_t align = (uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O;
    if (align & 15) return SMHA_ERR_UNSUPPORTED;
    if ((int64_t)B * H > (1 << 24)) return SMHA_ERR_UNSUPPORTED;
    {   // the block kernel addresses one head's Q/K/V/O through 32-bit buffer offsets
        const int64_t lim = (int64_t)1 << 31;
        const int64_t rows = (int64_t)plan->S + 128, krows = (int64_t)plan->Sk + 128;
        const int64_t qs = q_strides ? q_strides[2] : d, ks = k_strides ? k_strides[2] : d, vs = v_strides ? v_strides[2] : d;
        const int64_t os = o_strides ? o_strides[2] : d;
        if (qs < d || ks < d || vs < d || os < d) return SMHA_ERR_UNSUPPORTED;  // rows must not overlap
        if ((rows * qs + d) * 2 >= lim || (krows * ks + d) * 2 >= lim || (krows * vs + d) * 2 >= lim ||
            (rows * os + d) * 2 >= lim)
            return SMHA_ERR_UNSUPPORTED;
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

    const int S = plan->S, Sk = plan->Sk;
    auto take = [&](Strides &s, const int64_t *in, int rows) {
        if (in) { s.b = in[0]; s.h = in[1]; s.s = in[2]; } else { s.s = d; s.h = (int64_t)rows * d; s.b = (int64_t)H * rows * d; }
    };
    FwdParams fp{};
    fp.Q = (const uint16_t *)Q; fp.K = (const uint16_t *)K; fp.V = (const uint16_t *)V; fp.O = O;
    take(fp.qs, q_strides, S); take(fp.ks, k_strides, Sk); take(fp.vs, v_strides, Sk); take(fp.os, o_strides, S);
    fp.B = B; fp.H = H; fp.S = S; fp.Sk = Sk; fp.Bm = plan->Bm; fp.Hm = plan->Hm;
    fp.d = d;
    fp.out_dtype = out_dtype;
    const float sc = scale > 0.f ? scale : 1.0f / std::sqrt((float)d);
    fp.c = sc * 1.4426950408889634f;
    const DeviceArrays &dv = plan->dev;
    int form = block_form(plan, D, in_dtype == SMHA_BF16);
    if (form == 2 && d != D) form = 1;  // (the second form has no narrower heads)
    const int lvl = grain_for(plan, B, H, D, form);
    const WorkLists &wl = plan->lists[lvl];
    fp.items = dv.items[lvl]; fp.item_off = dv.item_off[lvl]; fp.item_cnt = dv.item_cnt[lvl];
    fp.uent = dv.uent; fp.gidx = dv.gidx; fp.n_gidx = (int)plan->h_gidx.size(); fp.kt_bitmap = dv.kt_bitmap; fp.bmp_spare = (int)(plan->h_kt_bitmap.size() / 64) - 1;
    fp.max_slots = wl.max_slots;
    fp.split_rows = dv.split_rows[lvl]; fp.split_off = dv.split_off[lvl]; fp.split_cnt = dv.split_cnt[lvl];
    fp.row_ptr = dv.row_ptr; fp.col_idx = dv.col_idx; fp.col_off = dv.col_off;

    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t e = hipSuccess;
    if (which == SMHA_KERNEL_BLOCK) {
        if ((int64_t)B * H * wl.max_items > ((int64_t)1 << 28)) return SMHA_ERR_UNSUPPORTED;  // (the order table indexes items with 32 bits)
        const smha_plan::Prepared *pr = nullptr;
        void *ws = nullptr;
        const smha_status_t st = prepared_for(plan, B, H, D, lvl, form, &pr, &ws, !static_ws);
        fp.form = form;
        if (st != SMHA_OK) return st;
        if (static_ws && pr->ws_bytes) {
            // the library's own array instead of a workspace of the plan; its counters are cleared by a
            // small kernel ahead of the launch (the array is shared by every such call on this GPU)
            if (pr->ws_bytes > kStaticScratchBytes) return SMHA_ERR_UNSUPPORTED;
            ws = static_scratch_for(plan->device);
            if (!ws) return SMHA_ERR_HIP;
            const size_t n = (pr->ws_bytes - pr->counters_at) / sizeof(uint32_t);
            hipLaunchKernelGGL(smha_fill_zero, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                               (uint32_t *)((char *)ws + pr->counters_at), n);
            if (hipGetLastError() != hipSuccess) return SMHA_ERR_HIP;
        }
        fp.order_hdr = pr->order;
        fp.order = pr->order + 16;
        if (form == 2) {
            fp.order_hdr = pr->order + 8;
            fp.order = pr->order + 8 + 4 * 8 * (int64_t)pr->per_xcd;
            fp.order_items = fp.order + pr->step_words;
            fp.step_bytes = pr->step_words * 4;
            fp.item_bytes = pr->item_words * 4;
        }
        fp.n_work = 8 * pr->longest;
        fp.per_xcd = pr->per_xcd;
        fp.scratch = (float *)ws;
        fp.counters = ws ? (uint32_t *)((char *)ws + pr->counters_at) : nullptr;
        fp.max_splits = wl.max_split_rows;
        if (D == 64)
            e = in_dtype == SMHA_BF16 ? launch_block<64, true>(plan, fp, stream) : launch_block<64, false>(plan, fp, stream);
        else if (D == 128)
            e = in_dtype == SMHA_BF16 ? launch_block<128, true>(plan, fp, stream) : launch_block<128, false>(plan, fp, stream);
        else
            e = in_dtype == SMHA_BF16 ? launch_block<256, true>(plan, fp, stream) : launch_block<256, false>(plan, fp, stream);
    } else {
        if (D == 64)
            e = in_dtype == SMHA_BF16 ? launch_row<64, true>(plan, fp, stream) : launch_row<64, false>(plan, fp, stream);
        else if (D == 128)
            e = in_dtype == SMHA_BF16 ? launch_row<128, true>(plan, fp, stream) : launch_row<128, false>(plan, fp, stream);
        else
            e = in_dtype == SMHA_BF16 ? launch_row<256, true>(plan, fp, stream) : launch_row<256, false>(plan, fp, stream);
    }
    return e == hipSuccess ? SMHA_OK : SMHA_ERR_HIP;
}

extern "C" smha_status_t smha_forward(const smha_plan_t *plan, const void *Q, const void *K,
                                      const void *V, void *O, int B, int H, int d,
                                      smha_dtype_t in_dtype, smha_dtype_t out_dtype,
                                      const int64_t q_strides[3], const int64_t k_strides[3],
                                      const int64_t v_strides[3], const int64_t o_strides[3],
                                      float scale, smha_kernel_t kernel, void *hip_stream) {
    return forward_impl(plan, Q, K, V, O, B, H, d, in_dtype, out_dtype, q_strides, k_strides, v_strides, o_strides,
                        scale, kernel, hip_stream, false);
}

extern "C" smha_status_t smha_forward_static(const smha_plan_t *plan, const void *Q, const void *K,
                                             const void *V, void *O, int B, int H, int d,
                                             smha_dtype_t in_dtype, smha_dtype_t out_dtype,
                                             const int64_t q_strides[3], const int64_t k_strides[3],
                                             const int64_t v_strides[3], const int64_t o_strides[3],
                                             float scale, smha_kernel_t kernel, void *hip_stream) {
    return forward_impl(plan, Q, K, V, O, B, H, d, in_dtype, out_dtype, q_strides, k_strides, v_strides, o_strides,
                        scale, kernel, hip_stream, true);
}

extern "C" const char *smha_kernel_name(const smha_plan_t *plan, int d, smha_dtype_t in_dtype,
                                        smha_kernel_t kernel) {
    if (!plan) return "";
    const int which = kernel == SMHA_KERNEL_AUTO ? plan->kernel : (int)kernel;
    if (which == SMHA_KERNEL_ROW) return "smha_row_fwd";
    if (!head_size_ok(d)) return "smha_block_fwd";
    const int D = kernel_head_size(d);
    int form = block_form(plan, D, in_dtype == SMHA_BF16);
    if (form == 2 && d != D) form = 1;
    return form == 3 ? "smha_block_fwd16" : form == 2 ? "smha_block_fwd2" : "smha_block_fwd";
}
