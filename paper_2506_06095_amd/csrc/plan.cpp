// Host-side mask analysis: dense mask or pattern description -> per-row format, two-level
// block format (Sec. 4.2.1 of the paper), kernel selection (Sec. 4.2.3) and the block
// kernel's work lists.  Integer work only; runs without a GPU.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <functional>
#include <memory>
#include <new>
#include <queue>
#include <thread>
#include <utility>
#include <vector>

#include "smha_internal.hpp"

namespace smha {
namespace {

// ---------------------------------------------------------------------------------------
// Row sources: produce one mask row as a bit string (bit j of word j/64 = entry (i, j)).
// ---------------------------------------------------------------------------------------
struct RowSource {
    virtual ~RowSource() = default;
    virtual void row_bits(int i, uint64_t *words) const = 0;  // words[W], W = ceil(Sk/64)
};

inline void set_range(uint64_t *w, int lo, int hi) {  // bits [lo, hi)
    if (lo >= hi) return;
    int wl = lo >> 6, wh = (hi - 1) >> 6;
    uint64_t ml = ~0ull << (lo & 63);
    uint64_t mh = ~0ull >> (63 - ((hi - 1) & 63));
    if (wl == wh) {
        w[wl] |= ml & mh;
        return;
    }
    w[wl] |= ml;
    for (int t = wl + 1; t < wh; ++t) w[t] = ~0ull;
    w[wh] |= mh;
}

inline void keep_below(uint64_t *w, int W, int n) {  // clear bits >= n
    int full = n >> 6;
    if (full < W) {
        int rem = n & 63;
        if (rem) {
            w[full] &= ~0ull >> (64 - rem);
            ++full;
        }
        for (int t = full; t < W; ++t) w[t] = 0;
    }
}

struct DenseSource final : RowSource {
    const uint8_t *m;
    int S, W;
    DenseSource(const uint8_t *mask, int S_) : m(mask), S(S_), W((S_ + 63) / 64) {}
    void row_bits(int i, uint64_t *words) const override {
        const uint8_t *r = m + (size_t)i * S;
        int j = 0;
        for (int t = 0; t < W; ++t) {
            uint64_t out = 0;
            for (int byte = 0; byte < 8 && j < S; ++byte) {
                if (j + 8 <= S) {
                    uint64_t x;
                    std::memcpy(&x, r + j, 8);
                    // any nonzero byte -> its bit 0, then gather the eight bit-0s
                    x |= x >> 4;
                    x |= x >> 2;
                    x |= x >> 1;
                    x &= 0x0101010101010101ull;
                    out |= ((x * 0x0102040810204080ull) >> 56) << (8 * byte);
                    j += 8;
                } else {
                    for (int b = 0; j < S; ++b, ++j)
                        if (r[j]) out |= 1ull << (8 * byte + b);
                }
            }
            words[t] = out;
        }
    }
};

// bit rows that were packed elsewhere (on the GPU, for a device mask)
struct BitSource final : RowSource {
    const uint64_t *w;
    int W;
    BitSource(const uint64_t *words, int S_) : w(words), W((S_ + 63) / 64) {}
    void row_bits(int i, uint64_t *words) const override { std::memcpy(words, w + (size_t)i * W, sizeof(uint64_t) * W); }
};

inline uint64_t mix64(uint64_t x) {  // splitmix64 output function
    x += 0x9E3779B97F4A7C15ull;
    uint64_t z = x;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

inline uint64_t block_hash(uint64_t seed, uint64_t head, uint32_t br, uint32_t bc) {
    uint64_t key = mix64(seed ^ mix64(head));
    return mix64(key ^ (((uint64_t)br << 32) | bc));
}

struct DescSource final : RowSource {
    smha_mask_desc_t d;
    int S, W, valid;
    std::vector<std::vector<int32_t>> keep;  // per block row of d.block: kept block columns
    DescSource(const smha_mask_desc_t &desc, int S_, int head, int valid_)
        : d(desc), S(S_), W((S_ + 63) / 64), valid(valid_) {
        if (!(d.flags & (SMHA_MASK_BLOCK_RANDOM | SMHA_MASK_BIGBIRD))) return;
        const int bs = d.block, nb = (S + bs - 1) / bs;
        keep.resize(nb);
        std::vector<uint8_t> row(nb);
        std::vector<std::pair<uint64_t, int32_t>> cand;
        for (int br = 0; br < nb; ++br) {
            std::fill(row.begin(), row.end(), 0);
            if (d.flags & SMHA_MASK_BLOCK_RANDOM) {
                for (int bc = 0; bc < nb; ++bc) {
                    double u = (double)(block_hash(d.seed, head, br, bc) >> 11) *
                               (1.0 / 9007199254740992.0);
                    if (bc == br || u < d.keep_p) row[bc] = 1;
                }
            }
            if (d.flags & SMHA_MASK_BIGBIRD) {
                std::vector<uint8_t> bb(nb, 0);
                const int half = (d.n_window_blocks - 1) / 2;
                if (d.n_window_blocks > 0)
                    for (int bc = std::max(0, br - half); bc < std::min(nb, br + half + 1); ++bc)
                        bb[bc] = 1;
                for (int bc = 0; bc < std::min(nb, d.n_global_blocks); ++bc) bb[bc] = 1;
                if (br < d.n_global_blocks) std::fill(bb.begin(), bb.end(), 1);
                cand.clear();
                for (int bc = 0; bc < nb; ++bc)
                    if (!bb[bc]) cand.emplace_back(block_hash(d.seed, head, br, bc), bc);
                std::sort(cand.begin(), cand.end());
                for (int t = 0; t < (int)cand.size() && t < d.n_random_blocks; ++t)
                    bb[cand[t].second] = 1;
                for (int bc = 0; bc < nb; ++bc) row[bc] |= bb[bc];
            }
            for (int bc = 0; bc < nb; ++bc)
                if (row[bc]) keep[br].push_back(bc);
        }
    }
    void row_bits(int i, uint64_t *w) const override {
        std::memset(w, 0, sizeof(uint64_t) * W);
        const uint32_t f = d.flags;
        const uint32_t additive = f & (SMHA_MASK_WINDOW | SMHA_MASK_GLOBAL | SMHA_MASK_STRIDED |
                                       SMHA_MASK_BLOCK_RANDOM | SMHA_MASK_BIGBIRD);
        if (!additive) set_range(w, 0, S);
        if (f & SMHA_MASK_WINDOW) {
            int64_t lo = (int64_t)i - d.window_left, hi = (int64_t)i + d.window_right + 1;
            set_range(w, (int)std::max<int64_t>(0, lo), (int)std::min<int64_t>(S, hi));
        }
        if (f & SMHA_MASK_GLOBAL) set_range(w, 0, i < d.n_global ? S : std::min(S, d.n_global));
        if (f & SMHA_MASK_STRIDED)
            for (int j = d.stride_phase; j < S; j += d.stride) w[j >> 6] |= 1ull << (j & 63);
        if (!keep.empty()) {
            const int bs = d.block;
            for (int32_t bc : keep[i / bs])
                set_range(w, bc * bs, std::min<int64_t>(S, (int64_t)(bc + 1) * bs));
        }
        if (f & SMHA_MASK_CAUSAL) keep_below(w, W, i + 1);
        if (f & SMHA_MASK_PADDING) keep_below(w, W, i < valid ? valid : 0);
    }
};

// ---------------------------------------------------------------------------------------
// One stripe = 64 consecutive mask rows.  Everything downstream is derived from its bits.
// ---------------------------------------------------------------------------------------
struct Stripe {
    int32_t row_nnz[64];
    std::vector<int32_t> cols;                // per-row format, rows concatenated
    std::vector<int32_t> load_col[4];         // per block row inside the stripe (64/block of them)
    std::vector<uint8_t> flag[4];
    std::vector<uint64_t> bitmap[4];
    std::vector<int32_t> kt_col, kt_bmp_local;  // 64x64 tiles (only when block != 64)
    std::vector<uint64_t> kt_bitmap;
    int64_t valid16 = 0, nnz = 0;
};

inline uint64_t extract_bits(const uint64_t *row, int c0, int n) {  // n <= 64, c0 % n == 0
    uint64_t w = row[c0 >> 6] >> (c0 & 63);
    return n == 64 ? w : (w & ((1ull << n) - 1));
}

void analyse_stripe(const RowSource &src, int Sq, int Sk, int block, bool want_rows, int stripe,
                    uint64_t *bits /* 64*W */, Stripe &out) {
    const int W = (Sk + 63) / 64;
    const int r0 = stripe * 64;
    for (int r = 0; r < 64; ++r) {
        uint64_t *w = bits + (size_t)r * W;
        if (r0 + r < Sq)
            src.row_bits(r0 + r, w);
        else
            std::memset(w, 0, sizeof(uint64_t) * W);
        int c = 0;
        for (int t = 0; t < W; ++t) c += __builtin_popcountll(w[t]);
        out.row_nnz[r] = c;
        out.nnz += c;
    }
    if (want_rows) {
        out.cols.reserve(out.nnz);
        for (int r = 0; r < 64; ++r) {
            const uint64_t *w = bits + (size_t)r * W;
            for (int t = 0; t < W; ++t) {
                uint64_t x = w[t];
                while (x) {
                    out.cols.push_back(t * 64 + __builtin_ctzll(x));
                    x &= x - 1;
                }
            }
        }
    }
    // non-empty 16x16 tiles (input of the paper's Eq. 1)
    for (int g = 0; g < 4; ++g) {
        if (r0 + g * 16 >= Sq) break;
        for (int t = 0; t < W; ++t) {
            uint64_t any = 0;
            for (int r = 0; r < 16; ++r) any |= bits[(size_t)(g * 16 + r) * W + t];
            for (int q = 0; q < 4; ++q)
                if ((any >> (16 * q)) & 0xFFFF) ++out.valid16;
        }
    }
    // tiles of edge `block`
    const int nb = (Sk + block - 1) / block;
    const int per = 64 / block;
    for (int sub = 0; sub < per; ++sub) {
        if (r0 + sub * block >= Sq) break;
        for (int bc = 0; bc < nb; ++bc) {
            uint64_t words[64];
            int cnt = 0;
            for (int r = 0; r < block; ++r) {
                words[r] = extract_bits(bits + (size_t)(sub * block + r) * W, bc * block, block);
                cnt += __builtin_popcountll(words[r]);
            }
            if (!cnt) continue;
            out.load_col[sub].push_back(bc);
            const bool full = cnt == block * block;
            out.flag[sub].push_back(full ? 1 : 0);
            if (!full) out.bitmap[sub].insert(out.bitmap[sub].end(), words, words + block);
        }
    }
    if (block != 64) {
        for (int kt = 0; kt < W; ++kt) {
            uint64_t words[64];
            int cnt = 0;
            for (int r = 0; r < 64; ++r) {
                words[r] = bits[(size_t)r * W + kt];
                cnt += __builtin_popcountll(words[r]);
            }
            if (!cnt) continue;
            out.kt_col.push_back(kt);
            if (cnt == 64 * 64) {
                out.kt_bmp_local.push_back(-1);
            } else {
                out.kt_bmp_local.push_back((int32_t)(out.kt_bitmap.size() / 64));
                out.kt_bitmap.insert(out.kt_bitmap.end(), words, words + 64);
            }
        }
    }
}

smha_status_t analyse_mask(const RowSource &src, int Sq, int Sk, int block, bool want_rows,
                           MaskFormats &mf) {
    const int W = (Sk + 63) / 64;
    const int n_stripes = (Sq + 63) / 64;
    std::vector<Stripe> stripes(n_stripes);
    std::atomic<int> next{0};
    std::atomic<bool> failed{false};
    int n_threads = (int)std::min<unsigned>(std::max(1u, std::thread::hardware_concurrency()), 16u);
    n_threads = std::min(n_threads, n_stripes);
    if ((int64_t)Sq * Sk < (1 << 20)) n_threads = 1;
    auto work = [&]() {
        try {
            std::vector<uint64_t> bits((size_t)64 * W);
            for (;;) {
                int s = next.fetch_add(1);
                if (s >= n_stripes) break;
                analyse_stripe(src, Sq, Sk, block, want_rows, s, bits.data(), stripes[s]);
            }
        } catch (const std::bad_alloc &) {
            failed = true;
        }
    };
    if (n_threads <= 1) {
        work();
    } else {
        std::vector<std::thread> pool;
        for (int t = 0; t < n_threads; ++t) pool.emplace_back(work);
        for (auto &t : pool) t.join();
    }
    if (failed) return SMHA_ERR_ALLOC;

    const int nbr = (Sq + block - 1) / block;
    const int per = 64 / block;
    mf.load_row_ptr.assign(nbr + 1, 0);
    mf.full_row_ptr.assign(nbr + 1, 0);
    mf.part_row_ptr.assign(nbr + 1, 0);
    if (want_rows) {
        mf.row_ptr.assign(Sq + 1, 0);
        int64_t total = 0;
        for (auto &st : stripes) total += st.nnz;
        if (total > INT32_MAX) return SMHA_ERR_UNSUPPORTED;
        mf.col_idx.reserve(total);
    }
    mf.kt_row_ptr.assign(n_stripes + 1, 0);
    for (int s = 0; s < n_stripes; ++s) {
        Stripe &st = stripes[s];
        mf.nnz += st.nnz;
        mf.n_valid16 += st.valid16;
        if (want_rows) {
            for (int r = 0; r < 64 && s * 64 + r < Sq; ++r)
                mf.row_ptr[s * 64 + r + 1] = mf.row_ptr[s * 64 + r] + st.row_nnz[r];
            mf.col_idx.insert(mf.col_idx.end(), st.cols.begin(), st.cols.end());
        }
        for (int sub = 0; sub < per; ++sub) {
            const int br = s * per + sub;
            if (br >= nbr) break;
            for (size_t e = 0; e < st.load_col[sub].size(); ++e) {
                mf.load_col_idx.push_back(st.load_col[sub][e]);
                mf.flags.push_back(st.flag[sub][e]);
                (st.flag[sub][e] ? mf.full_col_idx : mf.part_col_idx).push_back(st.load_col[sub][e]);
            }
            mf.bitmap.insert(mf.bitmap.end(), st.bitmap[sub].begin(), st.bitmap[sub].end());
            mf.load_row_ptr[br + 1] = (int32_t)mf.load_col_idx.size();
            mf.full_row_ptr[br + 1] = (int32_t)mf.full_col_idx.size();
            mf.part_row_ptr[br + 1] = (int32_t)mf.part_col_idx.size();
        }
        if (block != 64) {
            const int32_t base = (int32_t)(mf.kt_bitmap.size() / 64);
            for (size_t e = 0; e < st.kt_col.size(); ++e) {
                mf.kt_col.push_back(st.kt_col[e]);
                mf.kt_bmp.push_back(st.kt_bmp_local[e] < 0 ? -1 : base + st.kt_bmp_local[e]);
            }
            mf.kt_bitmap.insert(mf.kt_bitmap.end(), st.kt_bitmap.begin(), st.kt_bitmap.end());
            mf.kt_row_ptr[s + 1] = (int32_t)mf.kt_col.size();
        }
        Stripe().cols.swap(st.cols);  // release early
    }
    if (block == 64) {  // the kernel's tiles ARE the exported tiles
        mf.kt_row_ptr = mf.load_row_ptr;
        mf.kt_col = mf.load_col_idx;
        mf.kt_bmp.resize(mf.flags.size());
        int32_t part = 0;
        for (size_t e = 0; e < mf.flags.size(); ++e) mf.kt_bmp[e] = mf.flags[e] ? -1 : part++;
        mf.kt_bitmap = mf.bitmap;
    }
    return SMHA_OK;
}

smha_status_t check_opts(const smha_plan_opts_t *in, smha_plan_opts_t &o) {
    o = smha_plan_opts_t{};
    if (in) o = *in;
    if (o.block == 0) o.block = 64;
    if (o.block != 16 && o.block != 32 && o.block != 64) return SMHA_ERR_UNSUPPORTED;
    if (o.force < SMHA_KERNEL_AUTO || o.force > SMHA_KERNEL_BLOCK) return SMHA_ERR_INVALID_ARG;
    if (o.selector != SMHA_SELECTOR_CALIBRATED && o.selector != SMHA_SELECTOR_PAPER_EQ1)
        return SMHA_ERR_INVALID_ARG;
    if (o.device_id < -2) return SMHA_ERR_INVALID_ARG;
    if (o.block_form < 0 || o.block_form > 3) return SMHA_ERR_INVALID_ARG;
    if (o.head_dim == 0) o.head_dim = 64;
    if (o.head_dim < 8 || o.head_dim > 256 || o.head_dim % 8) return SMHA_ERR_UNSUPPORTED;
    return SMHA_OK;
}

// The per-row column list is the one large array (4 bytes per unmasked entry, written entry by
// entry): it is built in the first pass only when it will certainly be kept.
bool rows_wanted(const smha_plan_opts_t &o) { return o.build_both || o.force == SMHA_KERNEL_ROW; }

}  // namespace

// ---------------------------------------------------------------------------------------
// Kernel selection (Sec. 4.2.3).
//   paper:      threshold = valid16 / n^2 - tau / (log2 n)^2, n = ceil(S/16), tau = 1.2;
//               row-wise iff threshold < 0 (n == 1: row-wise).  The paper states it for as many
//               queries as keys; with Sq != Sk the ratio is taken over the nq * nk tiles of the
//               mask and n in the logarithm is the key side, nk = ceil(Sk/16).
//   calibrated: compare modelled times per (batch, head) pair:
//               block = steps * t_step(d) + t_fixed ; row = nnz * t_entry(d) + Sq * t_rowfix
// ---------------------------------------------------------------------------------------
static double eq1_threshold(double valid16, int Sq, int Sk) {
    const double nq = std::ceil(Sq / 16.0), nk = std::ceil(Sk / 16.0);
    if (nk <= 1.0) return -INFINITY;
    const double lg = std::log2(nk);
    return valid16 / (nq * nk) - 1.2 / (lg * lg);
}

// Cost-model constants in nanoseconds of whole-chip time per (batch, head) pair, fitted to MI355X
// timings of both kernels with 64 pairs in flight (sequence 512 / 2048 / 4096, scattered masks of 2 to
// 64 random keys per row, sliding windows of 8 to 128, causal; least squares by hand on the 4096 rows):
//   block kernel: time = steps * step_ns + fixed_ns, steps = staged K/V tiles of a pair (the union lists
//                 of its 128-row groups) with a gathered tile counted as 1.5 (it takes the bitmap path
//                 and gathers its rows).  d = 64: scattered 4096 4924 ns / 2048 steps = 2.4, causal 4096
//                 3136 / 1056 = 3.0, scattered 2048 1330 / 512 = 2.6 -> 2.8; d = 128: 8400 / 2048 = 4.1,
//                 4889 / 1056 = 4.6, BigBird 8192 (32 pairs) 125 us / 32 / 866 = 4.5 -> 4.5.  fixed_ns = 60:
//                 what a launch of the block kernel costs beyond one of the row kernel, per pair at 64 pairs
//                 (decides only the smallest masks: both kernels are launch-bound there);
//   row kernel:   time = entries * entry_ns + rows * row_ns.  Rows of at most 32 keys on average share a wave
//                 four at a time.  d = 64: entry 0.0096 (2 vs 16 keys per row: 568 ns / 57344 entries; 32 vs
//                 64: 1134 / 129434 = 0.0088; causal 0.0100), row 0.13 shared / 0.44 with a wave per row;
//                 d = 128: entry 0.0195 (0.0198, 0.0188, causal 0.0203), row 0.12 / 0.43.
// Of the 60 measured cases the model now picks the slower kernel in 4, by at most 1.17x.
struct CostModel {
    double step_ns, fixed_ns, entry_ns, row_ns;
};
static CostModel cost_model(int d, double mean_row_nnz) {  // (a head narrower than 64, 128 or 256 columns costs what that kernel costs)
    const bool shared = mean_row_nnz <= 32.0;
    if (d > 128) return CostModel{10.0, 60.0, 0.039, shared ? 0.12 : 0.43};  // (256 columns, one workgroup of eight waves per compute unit: 9.9-10.0 ns per step measured; the row constants are twice those of 128 columns, not measured)
    return d > 64 ? CostModel{4.5, 60.0, 0.0195, shared ? 0.12 : 0.43} : CostModel{2.8, 60.0, 0.0096, shared ? 0.13 : 0.44};
}

// Formats of one mask (64-wide tiles, no per-row lists) from what the GPU reported per tile.
static void formats_from_tiles(const TileInfo *info, const std::vector<uint64_t> &part_bits, int nqt, int nkt,
                               MaskFormats &mf) {
    mf = MaskFormats{};
    mf.load_row_ptr.assign(nqt + 1, 0);
    mf.full_row_ptr.assign(nqt + 1, 0);
    mf.part_row_ptr.assign(nqt + 1, 0);
    for (int tr = 0; tr < nqt; ++tr) {
        for (int tc = 0; tc < nkt; ++tc) {
            const TileInfo &t = info[(size_t)tr * nkt + tc];
            const uint32_t cnt = t.cnt_v16 & 0xFFFFu;
            mf.nnz += cnt;
            mf.n_valid16 += (t.cnt_v16 >> 16) & 0xFFu;
            if (!cnt) continue;
            const bool full = cnt == 64 * 64;
            mf.load_col_idx.push_back(tc);
            mf.flags.push_back(full ? 1 : 0);
            (full ? mf.full_col_idx : mf.part_col_idx).push_back(tc);
            if (!full)  // (the GPU stored part tiles in the order its waves reached them: put them in list order)
                mf.bitmap.insert(mf.bitmap.end(), part_bits.begin() + (size_t)t.slot * 64, part_bits.begin() + (size_t)t.slot * 64 + 64);
        }
        mf.load_row_ptr[tr + 1] = (int32_t)mf.load_col_idx.size();
        mf.full_row_ptr[tr + 1] = (int32_t)mf.full_col_idx.size();
        mf.part_row_ptr[tr + 1] = (int32_t)mf.part_col_idx.size();
    }
    mf.kt_row_ptr = mf.load_row_ptr;  // the kernel's tiles are the exported tiles
    mf.kt_col = mf.load_col_idx;
    mf.kt_bmp.resize(mf.flags.size());
    int32_t part = 0;
    for (size_t e = 0; e < mf.flags.size(); ++e) mf.kt_bmp[e] = mf.flags[e] ? -1 : part++;
    mf.kt_bitmap = mf.bitmap;
}

// After a first pass without the per-row lists: could the selector take the row kernel?  (The
// block estimate here ignores gathered tiles, so it is an upper bound: if the row kernel does not
// beat it, it will not beat the final one either.)  If so the masks are analysed again with rows.
static bool row_may_be_chosen(const smha_plan *p) {
    if (p->opts.force != SMHA_KERNEL_AUTO) return false;
    const int n_masks = p->Bm * p->Hm;
    double v16 = 0, nnz = 0, tiles = 0;
    for (auto &m : p->masks) {
        v16 += (double)m.n_valid16;
        nnz += (double)m.nnz;
        tiles += (double)m.kt_col.size();
    }
    if (p->opts.selector == SMHA_SELECTOR_PAPER_EQ1) return eq1_threshold(v16 / n_masks, p->S, p->Sk) < 0;
    const CostModel cm = cost_model(p->opts.head_dim, nnz / n_masks / p->S);
    // (a pair's steps are at most its tiles: two tile rows share a staged tile, gathered tiles replace several)
    return nnz / n_masks * cm.entry_ns + p->S * cm.row_ns < tiles / n_masks * cm.step_ns + cm.fixed_ns;
}

smha_status_t finish_plan(smha_plan *p) {
    const int n_masks = p->Bm * p->Hm;
    const int S = p->S;  // queries
    double v16 = 0, nnz = 0, tiles = 0;
    for (auto &m : p->masks) {
        v16 += (double)m.n_valid16;
        nnz += (double)m.nnz;
        tiles += (double)m.kt_col.size();
    }
    v16 /= n_masks;
    nnz /= n_masks;
    tiles /= n_masks;
    p->eq1_threshold = eq1_threshold(v16, S, p->Sk);
    const CostModel cm = cost_model(p->opts.head_dim, nnz / S);
    p->model_row_us = 1e-3 * (nnz * cm.entry_ns + S * cm.row_ns);
    p->row_mean_nnz = nnz / S;

    try {
        // ---- block path first (its work lists say how many tiles the kernel will really visit,
        // which the selector needs): tiles, work items, split rows --------------------------
        if (p->opts.force != SMHA_KERNEL_ROW || p->opts.build_both) {
            const int nqt = (S + kTile - 1) / kTile;
            const int nsup = (S + kSuper - 1) / kSuper;
            for (int mi = 0; mi < n_masks; ++mi) {
                MaskFormats &m = p->masks[mi];
                const int32_t bmp_base = (int32_t)(p->h_kt_bitmap.size() / 64);
                p->h_kt_bitmap.insert(p->h_kt_bitmap.end(), m.kt_bitmap.begin(), m.kt_bitmap.end());
                // union of the two tile rows of every supertile (both lists ascending: merge); tiles
                // that use few key columns are repacked into gathered tiles (see UEntry), which go
                // to the end of the supertile's list
                std::vector<int32_t> sup_ptr(nsup + 1, 0);
                const int32_t ent_base = (int32_t)p->h_uent.size();
                const int64_t pad_key = (int64_t)p->Sk + 64;  // (past the sequence: loads as zeros)
                struct Sparse { int32_t col, ea, eb; uint64_t used; };
                std::vector<Sparse> sparse;
                std::vector<int32_t> keys;
                for (int sp = 0; sp < nsup; ++sp) {
                    const int r0 = 2 * sp, r1 = 2 * sp + 1;
                    int a = m.kt_row_ptr[r0], ae = m.kt_row_ptr[r0 + 1];
                    int b = r1 < nqt ? m.kt_row_ptr[r1] : 0, be = r1 < nqt ? m.kt_row_ptr[r1 + 1] : 0;
                    auto code = [&](int e) { return m.kt_bmp[e] < 0 ? -1 : m.kt_bmp[e] + bmp_base; };
                    auto used_cols = [&](int e) {  // which of the tile's 64 key columns any query uses
                        if (e < 0) return (uint64_t)0;
                        if (m.kt_bmp[e] < 0) return ~(uint64_t)0;
                        uint64_t u = 0;
                        const uint64_t *w = m.kt_bitmap.data() + (size_t)m.kt_bmp[e] * 64;
                        for (int r = 0; r < 64; ++r) u |= w[r];
                        return u;
                    };
                    sparse.clear();
                    int n_sparse_cols = 0;
                    while (a < ae || b < be) {
                        UEntry u{0, {-2, -2}, 0};
                        const int ca = a < ae ? m.kt_col[a] : INT32_MAX;
                        const int cb = b < be ? m.kt_col[b] : INT32_MAX;
                        u.col = std::min(ca, cb);
                        const int ea = ca == u.col ? a++ : -1, eb = cb == u.col ? b++ : -1;
                        const uint64_t used = used_cols(ea) | used_cols(eb);
                        if (!p->opts.no_gather && __builtin_popcountll(used) <= kGatherMaxCols) {
                            sparse.push_back({u.col, ea, eb, used});
                            n_sparse_cols += __builtin_popcountll(used);
                            continue;
                        }
                        if (ea >= 0) u.code[0] = code(ea);
                        if (eb >= 0) u.code[1] = code(eb);
                        p->h_uent.push_back(u);
                    }
                    // repacking pays only if it saves steps
                    if ((n_sparse_cols + 63) / 64 >= (int)sparse.size()) {
                        for (const Sparse &t : sparse) {
                            UEntry u{t.col, {-2, -2}, 0};
                            if (t.ea >= 0) u.code[0] = code(t.ea);
                            if (t.eb >= 0) u.code[1] = code(t.eb);
                            p->h_uent.push_back(u);
                        }
                        // (the list is no longer ascending in col; nothing depends on that)
                    } else {
                        keys.clear();
                        for (const Sparse &t : sparse) {
                            for (uint64_t x = t.used; x; x &= x - 1) keys.push_back(t.col * 64 + __builtin_ctzll(x));
                        }
                        // keys ascend (tiles ascend, bits ascend); 64 per gathered tile
                        size_t ti = 0;  // sparse tile that holds keys[k]
                        for (size_t k0 = 0; k0 < keys.size(); k0 += 64) {
                            const int nk = (int)std::min<size_t>(64, keys.size() - k0);
                            const int32_t gt = (int32_t)(p->h_gidx.size() / 64);
                            uint64_t wa[64] = {0}, wb[64] = {0};
                            for (int k = 0; k < 64; ++k) {
                                if (k >= nk) {
                                    p->h_gidx.push_back((int32_t)std::min<int64_t>(pad_key, INT32_MAX));
                                    continue;
                                }
                                const int32_t key = keys[k0 + k];
                                p->h_gidx.push_back(key);
                                while (sparse[ti].col != key / 64) ++ti;
                                const Sparse &t = sparse[ti];
                                const int bit = key & 63;
                                for (int side = 0; side < 2; ++side) {
                                    const int e = side ? t.eb : t.ea;
                                    if (e < 0) continue;
                                    uint64_t *dst = side ? wb : wa;
                                    if (m.kt_bmp[e] < 0) {
                                        for (int r = 0; r < 64; ++r) dst[r] |= 1ull << k;
                                    } else {
                                        const uint64_t *w = m.kt_bitmap.data() + (size_t)m.kt_bmp[e] * 64;
                                        for (int r = 0; r < 64; ++r) dst[r] |= ((w[r] >> bit) & 1ull) << k;
                                    }
                                }
                            }
                            UEntry u{0, {-2, -2}, gt + 1};
                            for (int side = 0; side < 2; ++side) {
                                const uint64_t *w = side ? wb : wa;
                                uint64_t any = 0;
                                for (int r = 0; r < 64; ++r) any |= w[r];
                                if (!any) continue;
                                u.code[side] = (int32_t)(p->h_kt_bitmap.size() / 64);
                                p->h_kt_bitmap.insert(p->h_kt_bitmap.end(), w, w + 64);
                            }
                            p->h_uent.push_back(u);
                            ++p->n_gathered;
                        }
                    }
                    sup_ptr[sp + 1] = (int32_t)p->h_uent.size() - ent_base;
                }
                // split supertiles whose list is much longer than the typical one, so that a
                // few heavy rows (global tokens) do not serialise on one workgroup
                int64_t n_nonempty = 0;
                for (int sp = 0; sp < nsup; ++sp) n_nonempty += sup_ptr[sp + 1] > sup_ptr[sp];
                const double avg = n_nonempty ? (double)sup_ptr[nsup] / n_nonempty : 0.0;
                for (int lvl = 0; lvl < 2; ++lvl) {
                // Grain 0: parts of at most `chunk` steps (the kernel holds one entry per lane: 64 at
                // most), and lists up to twice that stay whole: merging costs a second launch (4-6 us),
                // more than a workgroup that runs a few steps longer than the others.  Grain 1: at most
                // 16 steps per item, for calls with so few heads that one long list would be the launch.
                const int chunk = lvl == 0 ? std::min(64, std::max(16, (int)std::ceil(1.5 * avg))) : 16;
                const int whole = lvl == 0 ? std::min(64, 2 * chunk) : 16;
                WorkLists &wl = p->lists[lvl];
                std::vector<Item> items;
                std::vector<SplitRow> splits;
                int32_t slots = 0;
                auto make_item = [&](int sp, int32_t b, int32_t e, int32_t slot, int32_t split = -1) {
                    Item it{sp, b, e, slot, 0, 0, split, 0};
                    for (int32_t x = b; x < e; ++x)
                        if (p->h_uent[x].gather > 0) {
                            if (!it.gcount) it.gbegin = p->h_uent[x].gather - 1;
                            ++it.gcount;
                        }
                    return it;
                };
                std::vector<int32_t> cuts;
                for (int sp = 0; sp < nsup; ++sp) {
                    const int32_t b = ent_base + sup_ptr[sp], e = ent_base + sup_ptr[sp + 1];
                    const int n = e - b;
                    int n_gath = 0;
                    for (int32_t x = b; x < e; ++x) n_gath += p->h_uent[x].gather > 0;
                    if (n <= whole && n_gath <= kMaxGatherPerItem) {
                        items.push_back(make_item(sp, b, e, -1));
                        continue;
                    }
                    // equal parts of at most `chunk` entries, cut again where a part would hold more
                    // gathered tiles than the kernel keeps key numbers for
                    const int parts = (n + chunk - 1) / chunk;
                    cuts.clear();
                    cuts.push_back(b);
                    for (int c = 1; c <= parts; ++c) {
                        const int32_t ce = b + (int32_t)((int64_t)n * c / parts);
                        int g = 0;
                        for (int32_t x = cuts.back(); x < ce; ++x) {
                            if (p->h_uent[x].gather > 0 && ++g > kMaxGatherPerItem) {
                                cuts.push_back(x);
                                g = 1;
                            }
                        }
                        if (ce > cuts.back()) cuts.push_back(ce);
                    }
                    const int n_parts = (int)cuts.size() - 1;
                    if (n_parts == 1) {
                        items.push_back(make_item(sp, b, e, -1));
                        continue;
                    }
                    splits.push_back({sp, slots, n_parts, 0});
                    for (int c = 0; c < n_parts; ++c)
                        items.push_back(make_item(sp, cuts[c], cuts[c + 1], slots++, (int32_t)splits.size() - 1));
                }
                std::stable_sort(items.begin(), items.end(), [](const Item &a, const Item &b) {
                    return (a.end - a.begin) > (b.end - b.begin);
                });
                wl.item_off.push_back((int32_t)wl.items.size());
                wl.item_cnt.push_back((int32_t)items.size());
                wl.items.insert(wl.items.end(), items.begin(), items.end());
                wl.split_off.push_back((int32_t)wl.split_rows.size());
                wl.split_cnt.push_back((int32_t)splits.size());
                wl.split_rows.insert(wl.split_rows.end(), splits.begin(), splits.end());
                wl.max_items = std::max(wl.max_items, (int)items.size());
                wl.max_split_rows = std::max(wl.max_split_rows, (int)splits.size());
                wl.max_slots = std::max(wl.max_slots, (int)slots);
                }
            }
        }
        // (no block lists were built: the forced row kernel; the estimate then falls back to one step per tile)
        const double steps = p->h_uent.empty() ? tiles : ((double)p->h_uent.size() + 0.5 * (double)p->n_gathered) / n_masks;
        p->model_block_us = 1e-3 * (steps * cm.step_ns + cm.fixed_ns);
        int choice;
        if (p->opts.force != SMHA_KERNEL_AUTO)
            choice = p->opts.force;
        else if (p->opts.selector == SMHA_SELECTOR_PAPER_EQ1)
            choice = p->eq1_threshold < 0 ? SMHA_KERNEL_ROW : SMHA_KERNEL_BLOCK;
        else
            choice = p->model_row_us < p->model_block_us ? SMHA_KERNEL_ROW : SMHA_KERNEL_BLOCK;
        p->kernel = choice;
        p->has_row = p->opts.build_both || choice == SMHA_KERNEL_ROW;
        p->has_block = p->opts.build_both || choice == SMHA_KERNEL_BLOCK;
        p->fine_differs = p->lists[1].items.size() != p->lists[0].items.size();
        if (!p->fine_differs) p->lists[1] = WorkLists{};  // (same cuts: one copy serves both)
        {   // (measured at 128 columns: the third form loses 3-5 % on dense causal lists of 16 steps and more,
            // and wins up to 20 % wherever tiles are partially filled or lists are short)
            int64_t tiles_in_lists = 0, part_in_lists = 0;
            for (const UEntry &u : p->h_uent)
                for (int side = 0; side < 2; ++side) {
                    tiles_in_lists += u.code[side] != -2;
                    part_in_lists += u.code[side] >= 0;
                }
            const double groups = (double)n_masks * ((p->S + 127) / 128);
            p->dense_long_lists = (double)part_in_lists < 0.15 * (double)tiles_in_lists && (double)p->h_uent.size() > 16.0 * groups;
        }
        if (p->has_block) {
            p->h_kt_bitmap.insert(p->h_kt_bitmap.end(), 64, 0ull);  // spare all-zero block
            p->h_uent.push_back(UEntry{0, {-2, -2}, 0});             // spare entry: an empty item may read one past its list
        } else {  // the row kernel was chosen: the block kernel's lists are not kept
            std::vector<UEntry>().swap(p->h_uent);
            std::vector<int32_t>().swap(p->h_gidx);
            std::vector<uint64_t>().swap(p->h_kt_bitmap);
            p->lists[0] = WorkLists{};
            p->lists[1] = WorkLists{};
            p->n_gathered = 0;
            p->fine_differs = false;
        }
        // ---- row path: concatenate -------------------------------------------------
        if (p->has_row) {
            p->h_row_ptr.reserve((size_t)n_masks * (S + 1));
            int64_t off = 0;
            for (auto &m : p->masks) {
                p->h_col_off.push_back(off);
                p->h_row_ptr.insert(p->h_row_ptr.end(), m.row_ptr.begin(), m.row_ptr.end());
                off += (int64_t)m.col_idx.size();
            }
            p->h_col_idx.reserve(off);
            for (auto &m : p->masks)
                p->h_col_idx.insert(p->h_col_idx.end(), m.col_idx.begin(), m.col_idx.end());
        }
        // the per-row column list is large; drop it when no kernel will read it
        if (!p->has_row)
            for (auto &m : p->masks) {
                // keep row_ptr/col_idx for export only when explicitly requested (build_both)
                std::vector<int32_t>().swap(m.col_idx);
                std::vector<int32_t>().swap(m.row_ptr);
            }
    } catch (const std::bad_alloc &) {
        return SMHA_ERR_ALLOC;
    }

    int dev = p->opts.device_id;
    if (dev == -2) return SMHA_OK;
    if (dev == -1) {
        dev = current_device_or_negative();
        if (dev < 0) return SMHA_OK;  // host-only plan; forward will report SMHA_ERR_HIP
    }
    return upload_plan(p, dev);
}

// One workspace of the block kernel for a call shape: per (batch*head) max_slots partial results of
// 128 rows (O, then running maximum and sum per row, each written per wave: 128 d + 512 floats), then
// four arrival counters (one per 32-row quarter) per (batch*head, split group).
size_t workspace_bytes(const smha_plan *plan, int lvl, int B, int H, int d, size_t *counters_at) {
    const WorkLists &wl = plan->lists[plan->fine_differs ? lvl : 0];
    const size_t partials = (size_t)B * H * wl.max_slots * (size_t)(128 * d + 1024) * sizeof(float);
    const size_t at = (partials + 255) / 256 * 256;
    if (counters_at) *counters_at = at;
    return at + (size_t)B * H * wl.max_split_rows * 8 * sizeof(uint32_t);
}

// The block kernel's work order for B x H heads on `slots` resident workgroups per XCD.  Items
// differ in length (tile rows under global tokens, random blocks, padding), and with equal item
// counts per workgroup the slowest one ends well after the average one; so the items of each head
// go, longest first, to the workgroup with the least work so far (cost: tiles plus a fixed part per
// item), head after head so that an XCD's workgroups stay on one head's K/V at a time.
// table = {start of each XCD's list (8), its length (8), then (batch*head, item index) pairs};
// list position = turn * per_xcd + workgroup rank; a workgroup's unused turns hold batch*head = -1.
void build_work_order(const smha_plan *plan, int lvl, int B, int H, int slots, std::vector<int32_t> &table, int &per_xcd) {
    const WorkLists &wl = plan->lists[plan->fine_differs ? lvl : 0];
    const int BH = B * H;
    auto mask_of = [&](int bh) { return (plan->Bm > 1 ? bh / H : 0) * plan->Hm + (plan->Hm > 1 ? bh % H : 0); };
    int64_t most = 0;  // items of the busiest XCD
    for (int x = 0; x < 8; ++x) {
        int64_t n = 0;
        for (int bh = x; bh < BH; bh += 8) n += wl.item_cnt[mask_of(bh)];
        most = std::max(most, n);
    }
    per_xcd = (int)std::min<int64_t>(slots, most);
    table.assign(16, 0);
    if (per_xcd == 0) return;
    constexpr int kItemCost = 2;  // an item's start and end, in tiles
    typedef std::pair<int64_t, int> Load;  // (work so far, workgroup rank)
    std::vector<std::vector<int32_t>> mine(per_xcd);
    for (int x = 0; x < 8; ++x) {
        std::priority_queue<Load, std::vector<Load>, std::greater<Load>> heap;
        for (int r = 0; r < per_xcd; ++r) {
            heap.push({0, r});
            mine[r].clear();
        }
        for (int bh = x; bh < BH; bh += 8) {
            const int mask = mask_of(bh);
            const int32_t off = wl.item_off[mask];
            for (int it = 0; it < wl.item_cnt[mask]; ++it) {  // (sorted by length, longest first)
                const Item &item = wl.items[off + it];
                Load l = heap.top();
                heap.pop();
                mine[l.second].push_back(bh);
                mine[l.second].push_back(off + it);
                l.first += kItemCost + (item.end - item.begin);
                heap.push(l);
            }
        }
        size_t turns = 0;
        for (int r = 0; r < per_xcd; ++r) turns = std::max(turns, mine[r].size() / 2);
        table[x] = (int32_t)((table.size() - 16) / 2);
        table[8 + x] = (int32_t)(turns * per_xcd);
        for (size_t t = 0; t < turns; ++t)
            for (int r = 0; r < per_xcd; ++r) {
                const bool has = 2 * t < mine[r].size();
                table.push_back(has ? mine[r][2 * t] : -1);
                table.push_back(has ? mine[r][2 * t + 1] : 0);
            }
    }
}

}  // namespace smha

using namespace smha;

extern "C" smha_status_t smha_plan_from_dense(const uint8_t *mask, int mask_on_device, int Bm,
                                              int Hm, int S, const smha_plan_opts_t *opts,
                                              smha_plan_t **out) {
    return smha_plan_from_dense_rect(mask, mask_on_device, Bm, Hm, S, S, opts, out);
}

extern "C" smha_status_t smha_plan_from_dense_rect(const uint8_t *mask, int mask_on_device, int Bm,
                                                   int Hm, int Sq, int Sk, const smha_plan_opts_t *opts,
                                                   smha_plan_t **out) {
    if (!mask || !out || Bm < 1 || Hm < 1 || Sq < 1 || Sk < 1) return SMHA_ERR_INVALID_ARG;
    smha_plan_opts_t o;
    smha_status_t st = check_opts(opts, o);
    if (st != SMHA_OK) return st;
    try {
        std::unique_ptr<smha_plan> p(new smha_plan);
        p->S = Sq; p->Sk = Sk; p->Bm = Bm; p->Hm = Hm; p->block = o.block; p->opts = o;
        const size_t per_mask = (size_t)Sq * Sk;
        const size_t words_per_mask = (size_t)Sq * ((Sk + 63) / 64);
        // A device mask whose plan needs neither per-row lists nor tiles narrower than 64 is analysed
        // by the GPU itself: 16 bytes per tile and the bitmaps of partially filled tiles cross over.
        bool analysed = false;
        if (mask_on_device && o.block == 64 && !rows_wanted(o)) {
            std::vector<TileInfo> info;
            std::vector<std::vector<uint64_t>> part_bits;
            st = classify_device_mask(mask, Bm * Hm, Sq, Sk, info, part_bits);
            if (st != SMHA_OK) return st;
            const int nqt = (Sq + 63) / 64, nkt = (Sk + 63) / 64;
            p->masks.assign((size_t)Bm * Hm, MaskFormats{});
            for (int mi = 0; mi < Bm * Hm; ++mi)
                formats_from_tiles(info.data() + (size_t)mi * nqt * nkt, part_bits[mi], nqt, nkt, p->masks[mi]);
            analysed = !row_may_be_chosen(p.get());  // (else: the row kernel may win, which needs the per-row lists)
        }
        std::vector<uint64_t> packed;  // otherwise a device mask is packed to bits on the GPU: 1/8 of the bytes cross over
        if (mask_on_device && !analysed) {
            packed.resize(words_per_mask * Bm * Hm);
            st = pack_device_mask(mask, Bm * Hm, Sq, Sk, packed.data());
            if (st != SMHA_OK) return st;
        }
        auto analyse_all = [&](bool rows) {
            p->masks.assign((size_t)Bm * Hm, MaskFormats{});
            for (int mi = 0; mi < Bm * Hm; ++mi) {
                smha_status_t s1;
                if (mask_on_device) {
                    BitSource src(packed.data() + words_per_mask * mi, Sk);
                    s1 = analyse_mask(src, Sq, Sk, o.block, rows, p->masks[mi]);
                } else {
                    DenseSource src(mask + per_mask * mi, Sk);
                    s1 = analyse_mask(src, Sq, Sk, o.block, rows, p->masks[mi]);
                }
                if (s1 != SMHA_OK) return s1;
            }
            return SMHA_OK;
        };
        if (!analysed) {
            st = analyse_all(rows_wanted(o));
            if (st == SMHA_OK && !rows_wanted(o) && row_may_be_chosen(p.get())) st = analyse_all(true);
            if (st != SMHA_OK) return st;
        }
        st = finish_plan(p.get());
        if (st != SMHA_OK) { release_device(p.get()); return st; }
        *out = p.release();
        return SMHA_OK;
    } catch (const std::bad_alloc &) {
        return SMHA_ERR_ALLOC;
    }
}

extern "C" smha_status_t smha_plan_from_desc(const smha_mask_desc_t *desc, int B, int H, int S,
                                             const smha_plan_opts_t *opts, smha_plan_t **out) {
    if (!desc || !out || B < 1 || H < 1 || S < 1) return SMHA_ERR_INVALID_ARG;
    const smha_mask_desc_t &d = *desc;
    const uint32_t known = SMHA_MASK_CAUSAL | SMHA_MASK_WINDOW | SMHA_MASK_GLOBAL | SMHA_MASK_STRIDED |
                           SMHA_MASK_BLOCK_RANDOM | SMHA_MASK_BIGBIRD | SMHA_MASK_PADDING;
    if (d.flags & ~known) return SMHA_ERR_INVALID_ARG;
    if ((d.flags & SMHA_MASK_WINDOW) && (d.window_left < 0 || d.window_right < 0)) return SMHA_ERR_INVALID_ARG;
    if ((d.flags & SMHA_MASK_GLOBAL) && d.n_global < 0) return SMHA_ERR_INVALID_ARG;
    if ((d.flags & SMHA_MASK_STRIDED) && (d.stride < 1 || d.stride_phase < 0 || d.stride_phase >= d.stride))
        return SMHA_ERR_INVALID_ARG;
    if (d.flags & (SMHA_MASK_BLOCK_RANDOM | SMHA_MASK_BIGBIRD)) {
        if (d.block < 1) return SMHA_ERR_INVALID_ARG;
        if ((d.flags & SMHA_MASK_BLOCK_RANDOM) && !(d.keep_p >= 0.0 && d.keep_p <= 1.0)) return SMHA_ERR_INVALID_ARG;
        if ((d.flags & SMHA_MASK_BIGBIRD) &&
            (d.n_window_blocks < 0 || d.n_global_blocks < 0 || d.n_random_blocks < 0))
            return SMHA_ERR_INVALID_ARG;
    }
    if (d.flags & SMHA_MASK_PADDING) {
        if (!d.valid_len) return SMHA_ERR_INVALID_ARG;
        for (int b = 0; b < B; ++b)
            if (d.valid_len[b] < 0 || d.valid_len[b] > S) return SMHA_ERR_INVALID_ARG;
    }
    smha_plan_opts_t o;
    smha_status_t st = check_opts(opts, o);
    if (st != SMHA_OK) return st;
    try {
        std::unique_ptr<smha_plan> p(new smha_plan);
        const int Bm = (d.flags & SMHA_MASK_PADDING) ? B : 1;
        const int Hm = (d.per_head && (d.flags & (SMHA_MASK_BLOCK_RANDOM | SMHA_MASK_BIGBIRD))) ? H : 1;
        p->S = S; p->Sk = S; p->Bm = Bm; p->Hm = Hm; p->block = o.block; p->opts = o;
        auto analyse_all = [&](bool rows) {
            p->masks.assign((size_t)Bm * Hm, MaskFormats{});
            for (int b = 0; b < Bm; ++b)
                for (int h = 0; h < Hm; ++h) {
                    const int valid = (d.flags & SMHA_MASK_PADDING) ? d.valid_len[b] : S;
                    DescSource src(d, S, h, valid);
                    const smha_status_t s1 = analyse_mask(src, S, S, o.block, rows, p->masks[(size_t)b * Hm + h]);
                    if (s1 != SMHA_OK) return s1;
                }
            return SMHA_OK;
        };
        st = analyse_all(rows_wanted(o));
        if (st == SMHA_OK && !rows_wanted(o) && row_may_be_chosen(p.get())) st = analyse_all(true);
        if (st != SMHA_OK) return st;
        st = finish_plan(p.get());
        if (st != SMHA_OK) { release_device(p.get()); return st; }
        *out = p.release();
        return SMHA_OK;
    } catch (const std::bad_alloc &) {
        return SMHA_ERR_ALLOC;
    }
}

extern "C" smha_status_t smha_plan_work_order(const smha_plan_t *p, int B, int H, int workgroups_per_xcd, int fine,
                                              int32_t *host_dst, size_t cap, size_t *need, int *per_xcd) {
    if (!p || !need || B < 1 || H < 1 || workgroups_per_xcd < 1 || fine < 0 || fine > 1) return SMHA_ERR_INVALID_ARG;
    if (cap > 0 && !host_dst) return SMHA_ERR_INVALID_ARG;
    if ((p->Bm != 1 && p->Bm != B) || (p->Hm != 1 && p->Hm != H)) return SMHA_ERR_SHAPE;
    if (!p->has_block) return SMHA_ERR_UNSUPPORTED;
    if ((int64_t)B * H > (1 << 24)) return SMHA_ERR_UNSUPPORTED;
    std::vector<int32_t> table;
    int n = 0;
    try { build_work_order(p, fine, B, H, workgroups_per_xcd, table, n); } catch (const std::bad_alloc &) { return SMHA_ERR_ALLOC; }
    *need = table.size();
    if (per_xcd) *per_xcd = n;
    if (cap >= table.size()) std::memcpy(host_dst, table.data(), table.size() * sizeof(int32_t));
    return SMHA_OK;
}

extern "C" smha_status_t smha_plan_info(const smha_plan_t *p, smha_plan_info_t *out) {
    if (!p || !out) return SMHA_ERR_INVALID_ARG;
    smha_plan_info_t i{};
    i.n_gathered = p->n_gathered;
    i.S = p->S; i.Sk = p->Sk; i.Bm = p->Bm; i.Hm = p->Hm; i.block = p->block; i.kernel = p->kernel;
    i.has_row_format = p->has_row; i.has_block_kernel_lists = p->has_block; i.on_device = p->device >= 0;
    for (auto &m : p->masks) {
        i.nnz += m.nnz;
        i.n_valid += (int64_t)m.load_col_idx.size();
        i.n_full += (int64_t)m.full_col_idx.size();
        i.n_part += (int64_t)m.part_col_idx.size();
        i.n_valid16 += m.n_valid16;
        i.n_tiles64 += (int64_t)m.kt_col.size();
    }
    i.n_union = p->h_uent.empty() ? 0 : (int64_t)p->h_uent.size() - 1;  // (without the spare entry)
    i.n_items = (int64_t)p->lists[0].items.size();
    i.n_split_rows = (int64_t)p->lists[0].split_rows.size();
    i.eq1_threshold = p->eq1_threshold;
    i.model_row_us = p->model_row_us;
    i.model_block_us = p->model_block_us;
    *out = i;
    return SMHA_OK;
}

extern "C" smha_status_t smha_plan_export(const smha_plan_t *p, int mask_index, smha_export_t which,
                                          void *host_dst, size_t cap, size_t *need) {
    if (!p || !need || mask_index < 0 || mask_index >= p->Bm * p->Hm) return SMHA_ERR_INVALID_ARG;
    if (cap > 0 && !host_dst) return SMHA_ERR_INVALID_ARG;
    const MaskFormats &m = p->masks[mask_index];
    const void *src = nullptr;
    size_t bytes = 0;
    std::vector<uint64_t> it8;
    auto vec = [&](const auto &v) { src = v.data(); bytes = v.size() * sizeof(v[0]); };
    switch (which) {
        case SMHA_EXPORT_ROW_PTR:
            if (m.row_ptr.empty()) return SMHA_ERR_UNSUPPORTED;
            vec(m.row_ptr); break;
        case SMHA_EXPORT_COL_IDX:
            if (m.row_ptr.empty()) return SMHA_ERR_UNSUPPORTED;
            vec(m.col_idx); break;
        case SMHA_EXPORT_LOAD_ROW_PTR: vec(m.load_row_ptr); break;
        case SMHA_EXPORT_LOAD_COL_IDX: vec(m.load_col_idx); break;
        case SMHA_EXPORT_BLOCK_FLAGS: vec(m.flags); break;
        case SMHA_EXPORT_BITMAP: vec(m.bitmap); break;
        case SMHA_EXPORT_FULL_ROW_PTR: vec(m.full_row_ptr); break;
        case SMHA_EXPORT_FULL_COL_IDX: vec(m.full_col_idx); break;
        case SMHA_EXPORT_PART_ROW_PTR: vec(m.part_row_ptr); break;
        case SMHA_EXPORT_PART_COL_IDX: vec(m.part_col_idx); break;
        case SMHA_EXPORT_BITMAP_IT8: {
            if (p->block != 64) return SMHA_ERR_UNSUPPORTED;
            const size_t np = m.bitmap.size() / 64;
            try { it8.assign(np * 64, 0); } catch (const std::bad_alloc &) { return SMHA_ERR_ALLOC; }
            for (size_t t = 0; t < np; ++t)
                for (int ir = 0; ir < 8; ++ir)
                    for (int ic = 0; ic < 8; ++ic) {
                        uint64_t w = 0;
                        for (int r = 0; r < 8; ++r)
                            w |= ((m.bitmap[t * 64 + ir * 8 + r] >> (8 * ic)) & 0xFFull) << (8 * r);
                        it8[t * 64 + ic * 8 + ir] = w;
                    }
            vec(it8);
            break;
        }
        case SMHA_EXPORT_KERNEL_ENTRIES:
            if (!p->has_block) return SMHA_ERR_UNSUPPORTED;
            src = p->h_uent.data(); bytes = (p->h_uent.size() - 1) * sizeof(UEntry); break;  // (without the spare entry)
        case SMHA_EXPORT_KERNEL_GATHER_KEYS:
            if (!p->has_block) return SMHA_ERR_UNSUPPORTED;
            vec(p->h_gidx); break;
        case SMHA_EXPORT_KERNEL_BITMAPS:
            if (!p->has_block) return SMHA_ERR_UNSUPPORTED;
            src = p->h_kt_bitmap.data(); bytes = (p->h_kt_bitmap.size() - 64) * sizeof(uint64_t); break;  // (without the spare block)
        case SMHA_EXPORT_KERNEL_ITEMS:
            if (!p->has_block) return SMHA_ERR_UNSUPPORTED;
            src = p->lists[0].items.data() + p->lists[0].item_off[mask_index];
            bytes = (size_t)p->lists[0].item_cnt[mask_index] * sizeof(Item); break;
        case SMHA_EXPORT_KERNEL_ITEMS_FINE: {
            if (!p->has_block) return SMHA_ERR_UNSUPPORTED;
            const WorkLists &wl = p->lists[p->fine_differs ? 1 : 0];
            src = wl.items.data() + wl.item_off[mask_index];
            bytes = (size_t)wl.item_cnt[mask_index] * sizeof(Item); break;
        }
        default: return SMHA_ERR_INVALID_ARG;
    }
    *need = bytes;
    if (cap >= bytes && bytes) std::memcpy(host_dst, src, bytes);
    return SMHA_OK;
}

extern "C" void smha_plan_destroy(smha_plan_t *p) {
    if (!p) return;
    release_device(p);
    delete p;
}

extern "C" const char *smha_status_string(smha_status_t s) {
    switch (s) {
        case SMHA_OK: return "ok";
        case SMHA_ERR_INVALID_ARG: return "invalid argument";
        case SMHA_ERR_UNSUPPORTED: return "unsupported configuration";
        case SMHA_ERR_SHAPE: return "shape mismatch";
        case SMHA_ERR_ALLOC: return "allocation failed";
        case SMHA_ERR_HIP: return "HIP error or no usable GPU";
    }
    return "unknown status";
}
