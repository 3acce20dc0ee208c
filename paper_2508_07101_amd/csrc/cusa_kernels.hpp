// Device code of libcusa: gfx950 kernels for the CUSA decode hot path.
//
//   topk_kernel         per-head ranked top-k (Sec. 3.2): radix select on order-preserving keys;
//                       the ranking by a counting sort over value bins (quick_rank) or, where
//                       scores crowd, a bitonic sort held in registers (lane exchanges by DPP /
//                       permlane swaps, LDS across waves)
//   union_kernel        cross-head union, first-occurrence global rank, cut at
//                       K-W, recency window (Sec. 3.2, 3.3) -> ascending rho
//   attn_kernel         split-K flash-decode over all tokens or over rho
//                       (Eq. 1 / SparseAttention of Alg. 1), GQA group in registers; its
//                       scoring forms also make P = q.K^T over the candidate range (Alg. 1,
//                       selection layer): one lane per key row, K staged through LDS,
//                       products accumulated by k = 1 MFMA in column order
//   sample_threshold_kernel   per-head thresholds from a sample of the scores (filtered selection)
//   attn_reduce_kernel  merges the split-K partials and writes bf16
//   per_head_rho_kernel, rank_aggregate_kernel, recall_kernel   the head-to-head variant, the other
//                       two readings of the global ranking, the recall of Eq. 3
//   probe_*_kernel      traffic probes (benchmark support)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cusa {

constexpr int D = 128;        // head_dim
constexpr int PAGE = 16;      // tokens per page of a paged cache

struct KvView {
    const uint16_t* k;
    const uint16_t* v;
    int64_t sb, sh, st;       // contiguous: element strides (batch, kv head, token)
    const int32_t* bt;        // paged: block table [B][max_pages]
    int32_t max_pages;
    int32_t G;                // kv heads
    const int32_t* seq_lens;  // [B]
};

template <bool PAGED>
__device__ __forceinline__ int64_t row_offset(const KvView& kv, int b, int kvh, int pos) {
    if (PAGED) {
        int64_t page = kv.bt[(int64_t)b * kv.max_pages + (pos >> 4)];
        return ((page * kv.G + kvh) * PAGE + (pos & (PAGE - 1))) * D;
    }
    return (int64_t)b * kv.sb + (int64_t)kvh * kv.sh + (int64_t)pos * kv.st;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

// 16 bytes of a K or V row.  Every row is read once per pass, so the load carries the streaming
// (non-temporal) hint: the caches need not keep what will not be asked for again.  On this machine that
// is worth 7-11 % on every attention kernel (c3 full attention 90 -> 83 us, c5 sparse 99 -> 88 us): a
// pass no longer turns over the whole L2 with lines nobody returns to.
__device__ __forceinline__ u32x4 stream_load(const uint16_t* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

// With per-head token lists the heads of a group ask for many of the same rows from different
// workgroups: those loads stay ordinary, so that the second asker finds the row in L2.
template <bool SHARED_ROWS>
__device__ __forceinline__ u32x4 row_load(const uint16_t* p) {
    return SHARED_ROWS ? *reinterpret_cast<const u32x4*>(p) : stream_load(p);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ void unpack8(const uint4& w, float* f) {
    f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x);
    f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
    f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z);
    f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;   // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ---------------------------------------------------------------- scoring
//
// The selection scores P = q.K^T are made by the attention kernel's scoring forms (attn_kernel with
// SCORE; ONLY_SCORES for cusa_select and the second chance).  Their bit-exactness rests on the product
// chain: V_MFMA_F32_4X4X1_16B_F32 takes, per lane, one binary32 element of q (head = lane % 4) and one
// of K (the lane's row) and adds the 4 heads x 64 rows of single products to the accumulators.  With
// k = 1 there is exactly one product (exact: bf16 x bf16 has a 16-bit significand) and one rounded
// addition per instruction, so walking the 128 columns in order is the left-to-right binary32 sum --
// no reordering inside the instruction can occur.  (Checked bit for bit against a scalar fmaf chain
// on the device.)

constexpr int SCORE_ROWS = 64;                        // tokens of a sample tile

// ---------------------------------------------------------------- block helpers

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// number of set bits of a 64-bit ballot below this lane
__device__ __forceinline__ int mbcnt(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Exclusive prefix sum of one int per thread over a 1024-thread block.
// scratch: SEL_WAVES + 1 ints of LDS.  Returns the exclusive prefix; *total gets the sum.
__device__ __forceinline__ int block_scan_excl(int v, int* scratch, int* total) {
    const int lane = lane_id(), w = wave_id();
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int n = __shfl_up(inc, o);
        if (lane >= o) inc += n;
    }
    __syncthreads();                               // scratch may still be read from a previous call
    if (lane == 63) scratch[w] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int i = 0; i < SEL_WAVES; ++i) {
            int c = scratch[i];
            scratch[i] = run;
            run += c;
        }
        scratch[SEL_WAVES] = run;
    }
    __syncthreads();
    *total = scratch[SEL_WAVES];
    return scratch[w] + inc - v;
}

// Order-preserving map of a binary32 score to uint32 (larger score -> larger key);
// -0 is mapped like +0 so that the two compare equal.
__device__ __forceinline__ uint32_t score_key(float s) {
    uint32_t u = __float_as_uint(s);
    if (u == 0x80000000u) u = 0;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// State of the selection's filtered fast path (sample_threshold_kernel has the account).
struct FilterState {              // device memory of the fast path, all per (sequence, head) = row
    uint32_t* thr;                // threshold key; 0xffffffff: keep nothing (flagged, or nothing to select)
    int32_t* cand_cnt;            // candidates kept so far
    int32_t* fail;                // 1: this head takes the second chance
    int32_t* n_failed;            // number of flagged heads
    uint64_t* cand;               // [row][cap] composites (score key << 32 | ~position), in any order
    int32_t cap;
    int32_t n_sink;
};

// Flags are set wherever a head's guess turns out bad; the heads are counted in one place, the top-k over
// the kept candidates, which looks at every head once.
__device__ __forceinline__ void flag_failed(const FilterState& f, int64_t row) { f.fail[row] = 1; }

// Inverse of score_key.
__device__ __forceinline__ float key_score(uint32_t key) {
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// ---------------------------------------------------------------- per-head top-k
//
// One 1024-thread workgroup per (sequence, head).  The candidates are ordered by
// the 64-bit composite (score_key << 32 | ~position): larger composite = better
// score, or equal score and lower position -- a strict total order, so "the k best"
// is a unique set and a unique ranking.
//   1. radix select (11/11/10-bit digits, LDS histograms) finds the score key T
//      of the k-th best candidate and how many candidates tie with it;
//   2. if more candidates equal T than are still needed, a second radix select
//      over ~position finds the position bound among the ties;
//   3. the k survivors are compacted into LDS and bitonic-sorted (descending);
//   4. ranks are written rank-major: rho_head[b][j][h].
// With ITEMS > 0 a thread keeps its ITEMS candidates (positions i*1024 + tid) in
// registers, loaded once with independent loads; ITEMS <= 0 (streamed) re-reads the scores from
// memory in every pass, 32 independent loads at a time (any length).

struct SelectState {
    uint32_t prefix;     // digits fixed so far
    int need;            // how many of the candidates matching prefix are wanted
    int count_eq;        // candidates whose digit equals the chosen one (last pass)
};

// One radix-select pass over `hist` (NB bins, already filled): choose the digit
// in which the `need`-th largest lies.  All threads call; results via LDS `st`.
template <int NB>
__device__ __forceinline__ void pick_digit(int* hist, int* scratch, SelectState* st, int shift) {
    // thread i owns bins [i*PER, i*PER+PER) counted from the top (descending digits)
    constexpr int PER = (NB + SEL_THREADS - 1) / SEL_THREADS;
    int local[PER];
    int sum = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        int bin = NB - 1 - (threadIdx.x * PER + j);
        local[j] = bin >= 0 ? hist[bin] : 0;
        sum += local[j];
    }
    int total;
    int above = block_scan_excl(sum, scratch, &total);   // candidates with larger digits
    const int need = st->need;
    __syncthreads();                                     // everyone has read st->need
    if (above < need && need <= above + sum) {
        int run = above;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            if (run < need && need <= run + local[j]) {
                int bin = NB - 1 - (threadIdx.x * PER + j);
                st->prefix |= (uint32_t)bin << shift;
                st->need = need - run;
                st->count_eq = local[j];
            }
            run += local[j];
        }
    }
    __syncthreads();
}

// Radix select of the `need`-th largest 32-bit key among this workgroup's candidates.
// scan(f) must call f(key, t) for every candidate slot of the calling thread, the same
// number of times in every lane of a wave; slots past the candidate range carry key 0, which
// no real score maps to and which therefore never reaches the top k.  key_map(key, t, &out)
// narrows the candidates and chooses the key that is selected on.
// Leaves the key in st->prefix, the number still wanted among equal keys in st->need and
// their count in st->count_eq.
// Keys whose top digit is below min_digit0 are known not to matter and are not counted.
// first_pass > 0 resumes a selection whose leading digits *st already holds.
template <typename Scan, typename KeyMap>
__device__ __forceinline__ void radix_select(int first_pass, int need, uint32_t min_digit0, Scan scan, KeyMap key_map,
                                             int* hist, int* scratch, SelectState* st) {
    if (first_pass == 0 && threadIdx.x == 0) {
        st->prefix = 0;
        st->need = need;
        st->count_eq = 0;
    }
    const int shifts[3] = {21, 10, 0};
    const int bits[3] = {11, 11, 10};
    uint32_t mask = 0;
    for (int pass = 0; pass < first_pass; ++pass) mask |= ((1u << bits[pass]) - 1u) << shifts[pass];
    for (int pass = first_pass; pass < 3; ++pass) {
        for (int i = threadIdx.x; i < 2048; i += SEL_THREADS) hist[i] = 0;
        __syncthreads();
        const uint32_t prefix = st->prefix;
        const int shift = shifts[pass];
        const uint32_t dmask = (1u << bits[pass]) - 1u;
        const uint32_t floor_d = pass == 0 ? min_digit0 : 0u;
        scan([&](uint32_t skey, int t) {
            uint32_t key;
            if (key_map(skey, t, &key) && (key & mask) == prefix && ((key >> shift) & dmask) >= floor_d)
                atomicAdd(&hist[(key >> shift) & dmask], 1);
        });
        __syncthreads();
        if (pass < 2) pick_digit<2048>(hist, scratch, st, shift);
        else pick_digit<1024>(hist, scratch, st, shift);
        mask |= dmask << shift;
    }
}

// Adds this thread's count to a workgroup counter with one LDS atomic per wave; returns the first of
// the thread's slots.  The counter must be zero and visible before, and is complete after the next
// workgroup barrier.
__device__ __forceinline__ int wave_reserve(int mine, int* counter) {
    int inc = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int nb = __shfl_up(inc, o);
        if (lane_id() >= o) inc += nb;
    }
    int wave_base = 0;
    if (lane_id() == 63) wave_base = atomicAdd(counter, inc);
    return __shfl(wave_base, 63) + inc - mine;
}

// Entries of the LDS candidate list of topk_kernel<ITEMS, MTOP> (0: no list; short rows are
// cheap to walk again).
__host__ __device__ constexpr int topk_list_cap(int items, int mtop) {
    return (items > 0 && items < 8) ? 0 : (mtop <= 2 ? 6144 : 10240);
}
// 8-byte entries of LDS behind the sort buffer: the candidate list or the quick ranking's segments, and
// behind them its 2048 bin counters.
__host__ __device__ constexpr int topk_area_entries(int items, int mtop, bool merge = false) {
    int n = topk_list_cap(items, mtop) + 1024 > mtop * 1024 + 1024 ? topk_list_cap(items, mtop) + 1024 : mtop * 1024 + 1024;
    // short rows (no list): room to rank all their candidates at once
    if (items > 0 && items < 8 && items * 1024 + 1024 > n) n = items * 1024 + 1024;
    // ranking all composites of a merge at once: items * 1024 segments entries and the bins, sort buffer included
    if (merge && items * 1024 + 1024 - mtop * 1024 > n) n = items * 1024 + 1024 - mtop * 1024;
    return n;
}

// Value of lane (l ^ STRIDE) for STRIDE < 64 without the LDS crossbar: DPP moves inside a 16-lane
// row, row/half swaps beyond.
template <int CTRL, int BANK_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t old, uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)v, CTRL, 0xF, BANK_MASK, false);
}
template <int STRIDE>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v) {
    // every lane has a source lane, so a plain DPP move into a fresh register does it (one
    // instruction, no copy of the destination's previous value)
    if constexpr (STRIDE == 1) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);        // quad_perm [1,0,3,2]
    else if constexpr (STRIDE == 2) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
    else if constexpr (STRIDE == 4) {
        const uint32_t t = dpp_u32<0x104, 0x5>(v, v);                 // row_shl:4 into lanes 0-3, 8-11 of a row
        return dpp_u32<0x114, 0xA>(t, v);                             // row_shr:4 into lanes 4-7, 12-15
    } else if constexpr (STRIDE == 8) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x128, 0xF, 0xF, true);   // row_ror:8
    else if constexpr (STRIDE == 16) {
        const auto s = __builtin_amdgcn_permlane16_swap(v, v, false, false);   // s[0]: rows 0,0,2,2; s[1]: rows 1,1,3,3
        return (threadIdx.x & 16) ? s[0] : s[1];
    } else {
        static_assert(STRIDE == 32, "lane_xor: stride must be a power of two below 64");
        const auto s = __builtin_amdgcn_permlane32_swap(v, v, false, false);   // s[0]: lower half twice; s[1]: upper half twice
        return (threadIdx.x & 32) ? s[0] : s[1];
    }
}
__device__ __forceinline__ uint32_t lane_xor_any(uint32_t v, int stride) {
    switch (stride) {
        case 1: return lane_xor<1>(v);
        case 2: return lane_xor<2>(v);
        case 4: return lane_xor<4>(v);
        case 8: return lane_xor<8>(v);
        case 16: return lane_xor<16>(v);
        default: return lane_xor<32>(v);
    }
}

// Ranks the composites mine(0) .. mine(NPT - 1) of every thread (zero: none; all at or above the score s_lo)
// and writes the picks ranked below k_out, rank-major (out[rank * H]) -- without a sorting network:
// 2048 bins divide the score range evenly by value (monotone in the key, so bins are in rank order), a
// counting sort puts every composite into its bin's segment, and inside a segment -- a few entries,
// unless scores repeat -- a composite's rank is the number of entries that beat it.  The range is
// [s_lo, s_lo + 6 x the mean excess over s_lo], not up to the best score: a few very large scores
// (attention sinks, hot tokens) would otherwise stretch the bins over empty space and crowd the
// rest; whatever lies above shares the first bin, which may hold more.  About a fifth of the
// instructions of a sorting network.  Returns false, having written nothing, when a bin is crowded
// (more than RMAX entries among the bins that hold wanted ranks, RMAX_FIRST in the first: many equal
// scores) or the scores are not finite;
// the caller then ranks another way.  seg: room for seg_cap composites (more: false); rbin: 2048 ints; scratch: as for
// block_scan_excl.  Called by the whole workgroup.
template <int NPT, typename Mine>
__device__ __forceinline__ bool quick_rank(Mine mine, float s_lo, int k_out, uint64_t* seg, int seg_cap, int* rbin,
                                           int* scratch, int32_t* __restrict__ out, int H) {
    constexpr int RBINS = 2048, RMAX = 32, RMAX_FIRST = 512;
    __shared__ float rk_excess;
    __shared__ int rk_crowd, rk_first, rk_n;
    const int tid = threadIdx.x;
    __syncthreads();                                     // whatever the areas held before has been read
    if (tid == 0) {
        rk_excess = 0.0f;
        rk_crowd = rk_n = 0;
    }
    for (int i = tid; i < RBINS; i += SEL_THREADS) rbin[i] = 0;
    float excess = 0.0f;
    int n_mine = 0;
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
        if (mine(j) != 0) {
            excess += key_score((uint32_t)(mine(j) >> 32)) - s_lo;
            ++n_mine;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        excess += __shfl_xor(excess, o);
        n_mine += __shfl_xor(n_mine, o);
    }
    __syncthreads();                                     // the counters and rbin are cleared
    if (lane_id() == 0) {
        atomicAdd(&rk_excess, excess);
        atomicAdd(&rk_n, n_mine);
    }
    __syncthreads();
    const int n = rk_n;
    const float range = n > 0 ? 6.0f * rk_excess / (float)n : 0.0f;
    // workgroup-uniform (not so: all scores equal, or not finite, or more composites than seg holds)
    bool quick = range > 0.0f && range < 3.0e38f && n <= seg_cap;
    const float scale = quick ? (float)(RBINS - 1) / range : 0.0f;
    auto bin_of = [&](uint64_t cv) {                     // bin 0 holds the best scores
        const int up = (int)((key_score((uint32_t)(cv >> 32)) - s_lo) * scale);
        return RBINS - 1 - (up < 0 ? 0 : up > RBINS - 1 ? RBINS - 1 : up);
    };
    int slot[NPT];
    if (quick) {
#pragma unroll
        for (int j = 0; j < NPT; ++j)
            if (mine(j) != 0) slot[j] = atomicAdd(&rbin[bin_of(mine(j))], 1);
    }
    __syncthreads();
    {   // counts -> first indices (thread i owns bins 2i, 2i + 1); the most crowded bin
        const int c0 = rbin[2 * tid], c1 = rbin[2 * tid + 1];
        int total;
        const int first = block_scan_excl(c0 + c1, scratch, &total);
        // only segments that reach into the wanted ranks are walked: the others may be crowded; bin 0 is
        // looked at on its own
        int crowd = first + c0 < k_out ? c1 : 0;
        if (tid != 0 && first < k_out && c0 > crowd) crowd = c0;
        if (tid == 0) rk_first = c0;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const int other = __shfl_xor(crowd, o);
            crowd = other > crowd ? other : crowd;
        }
        if (lane_id() == 0) atomicMax(&rk_crowd, crowd);
        rbin[2 * tid] = first;
        rbin[2 * tid + 1] = first + c0;
    }
    __syncthreads();
    quick = quick && rk_crowd <= RMAX && rk_first <= RMAX_FIRST;
    if (!quick) return false;
#pragma unroll
    for (int j = 0; j < NPT; ++j)
        if (mine(j) != 0) seg[rbin[bin_of(mine(j))] + slot[j]] = mine(j);
    __syncthreads();
    // the composites ranked below k_out lie in the segments' first k_out entries or just behind them
    for (int i = tid; i < n; i += SEL_THREADS) {
        const uint64_t cv = seg[i];
        const int bn = bin_of(cv), lo = rbin[bn], hi = bn == RBINS - 1 ? n : rbin[bn + 1];
        if (lo >= k_out) break;                          // (segments are in rank order: nothing wanted from here on)
        int rank = lo;
        for (int q = lo; q < hi; ++q) rank += seg[q] > cv ? 1 : 0;
        if (rank < k_out) out[(int64_t)rank * H] = (int32_t)~(uint32_t)cv;
    }
    return true;
}

// ITEMS == -1 is the streamed kernel in a register-lean form (half the keys in flight, compiled for two
// resident workgroups per CU): with many more rows than CUs two rows overlap on a CU, which gains more
// than the shorter batches lose (c5, 2048 rows: 198 -> 147 us); with one row per CU it is twice as
// slow as the wide form (c4: 65 -> 134 us), so few long rows keep ITEMS == 0.
//
// Few long rows (fewer rows than CUs, more than 32768 candidates) are cut into slices, one workgroup
// each (blockIdx.z): a slice selects its own k best and leaves their composites, unsorted and padded
// with zeros, in parts[row][slice][k]; the k best of a row are among the k best of its slices, so a
// second launch (MERGE) selects and ranks among those n_slices * k composites instead of the row.
template <int ITEMS, int MTOP, bool MERGE = false>
__global__ __launch_bounds__(SEL_THREADS, ((ITEMS == -1 && MTOP <= 4) || (MERGE && ITEMS <= 4 && MTOP <= 2)) ? 8 : 4) void topk_kernel(const float* __restrict__ P, int64_t ldp,
                                                            const int32_t* __restrict__ seq_lens,
                                                            int32_t* __restrict__ rho_head, int H, int k,
                                                            int budget, int window, int raw_keys, int n_sink,
                                                            uint64_t* __restrict__ parts, int slice_len, int n_slices,
                                                            const int32_t* __restrict__ only_rows, FilterState flt) {
    static_assert(!MERGE || ITEMS > 0, "the composites of a merge are held in registers");
    constexpr int NSORT = MTOP * SEL_THREADS;         // k <= NSORT
    constexpr int CAP = topk_list_cap(ITEMS, MTOP);
    extern __shared__ uint64_t sort_buf[];            // NSORT composites (aliases the histogram), then CAP list entries
    uint64_t* const cand = sort_buf + NSORT;
    __shared__ int scratch[SEL_WAVES + 1];
    __shared__ SelectState st;
    __shared__ int n_out, n_list;
    int* hist = reinterpret_cast<int*>(sort_buf);     // 2048 ints = 8 KB <= NSORT * 8

    // Workgroups go to the 8 XCDs round-robin in launch order.  The heads of a sequence write the same
    // lines of the rank-major output (entry (j, h) next to (j, h+1)); with eight sequences or more, all
    // heads of a sequence are put on one XCD, whose L2 then merges their 4-byte stores into whole
    // lines instead of each XCD writing its own fragments of every line (c5: 104 MB written for a 13 MB
    // output before).
    int h = blockIdx.x, b = blockIdx.y;
    {
        const int B = gridDim.y, lin = blockIdx.x + H * blockIdx.y;
        if (lin < (B / 8) * 8 * H) {
            const int within = lin % (8 * H);
            b = (lin / (8 * H)) * 8 + (within & 7);
            h = within >> 3;
        }
    }
    // only_rows: the second chance of the filtered fast path ranks the flagged heads only
    if (only_rows && only_rows[(int64_t)b * H + h] == 0) return;
    const int L = seq_lens[b];
    if (L <= budget) return;
    const int Lc = L - window;
    // this workgroup's candidates: the positions [t_lo, t_hi) of the row (a slice of it), or -- MERGE --
    // the composites the slices left, or (flt.thr set) those the filtered pass kept for this head
    const bool slice = !MERGE && parts != nullptr;
    const int t_lo = slice ? (int)blockIdx.z * slice_len : 0;
    const int t_hi = slice ? min(Lc, t_lo + slice_len) : Lc;
    uint64_t* const my_parts = parts + (((int64_t)b * H + h) * n_slices + (slice ? (int)blockIdx.z : 0)) * k;
    // the first n_sink positions are kept in rho anyway and are no candidates (key 0, like the padding)
    const int k_eff = MERGE ? min(k, Lc - n_sink) : min(k, t_hi - max(t_lo, n_sink));
    if (slice && k_eff <= 0) {                        // nothing of the row falls into this slice
        for (int i = threadIdx.x; i < k; i += SEL_THREADS) my_parts[i] = 0;
        return;
    }
    const float* __restrict__ row = P + ((int64_t)b * H + h) * ldp;
    // raw_keys: the row already holds order-preserving uint32 keys (the aggregated ranking keys of
    // the votes / max-score readings) instead of binary32 scores
    auto key_of = [raw_keys](float v) { return raw_keys ? __float_as_uint(v) : score_key(v); };
    uint32_t keys[ITEMS > 0 ? ITEMS : 1];
    int pos_of[MERGE ? ITEMS : 1];                     // MERGE: the positions that come with the keys
    if constexpr (MERGE) {
        int n_cand = n_slices * k;
        const uint64_t* __restrict__ src = my_parts;
        if (flt.thr) {
            const int64_t row = (int64_t)b * H + h;
            n_cand = flt.cand_cnt[row];
            // fewer than k kept: the threshold was too high and some of the k best are missing; more than
            // the list holds: some were dropped.  Either way the head is ranked the ordinary way later.
            if (flt.fail[row] != 0 || n_cand > flt.cap || n_cand < k_eff) {
                if (threadIdx.x == 0) {
                    flag_failed(flt, row);
                    atomicAdd(flt.n_failed, 1);
                }
                return;
            }
            src = flt.cand + row * flt.cap;
        }
        uint64_t mcv[ITEMS];                           // this thread's composites (zero: none)
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int sl = i * SEL_THREADS + threadIdx.x;
            const uint64_t cv = src[sl < n_cand ? sl : n_cand - 1];
            mcv[i] = sl < n_cand ? cv : 0;
        }
        // These composites are few and most of them among the k best, so they are first ranked as they are:
        // quick_rank over all of them, of which only the ranks below k_eff are written.  A filtered pass's
        // candidates are all at or above the head's threshold; the slices' picks (zeros where a slice had
        // fewer than k) start at the lowest of their scores.  If that does not work out (crowded bins) they
        // are selected and sorted like any row.
        if constexpr (ITEMS <= 8 || MTOP <= 4) {       // (what fits the register file)
            if (!raw_keys) {
                float s_lo;
                if (flt.thr) {
                    s_lo = key_score(flt.thr[(int64_t)b * H + h]);
                } else {
                    __shared__ uint32_t merge_lowest;
                    uint32_t lowest = 0xffffffffu;
#pragma unroll
                    for (int i = 0; i < ITEMS; ++i) {
                        const uint32_t key = (uint32_t)(mcv[i] >> 32);
                        if (mcv[i] != 0 && key < lowest) lowest = key;
                    }
                    if (threadIdx.x == 0) merge_lowest = 0xffffffffu;
                    __syncthreads();
#pragma unroll
                    for (int o = 32; o > 0; o >>= 1) {
                        const uint32_t other = __shfl_xor(lowest, o);
                        lowest = other < lowest ? other : lowest;
                    }
                    if (lane_id() == 0) atomicMin(&merge_lowest, lowest);
                    __syncthreads();
                    s_lo = key_score(merge_lowest);
                }
                if (quick_rank<ITEMS>([&](int j) { return mcv[j]; }, s_lo, k_eff, sort_buf, ITEMS * SEL_THREADS,
                                      reinterpret_cast<int*>(sort_buf + ITEMS * SEL_THREADS), scratch,
                                      rho_head + (int64_t)b * k * H + h, H))
                    return;
            }
        }
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            keys[i] = (uint32_t)(mcv[i] >> 32);
            pos_of[i] = (int)~(uint32_t)mcv[i];
        }
    } else if constexpr (ITEMS > 0) {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int t = t_lo + i * SEL_THREADS + threadIdx.x;
            const uint32_t kv_ = key_of(row[t < t_hi ? t : t_hi - 1]);   // clamped: loads stay unconditional
            keys[i] = (t < t_hi && t >= n_sink) ? kv_ : 0u;
        }
    }
    // Streamed rows (ITEMS <= 0) are walked in batches of SB keys per thread covering the positions
    // [t0, t0 + SB * 1024): key u of a thread is position t0 + ((u / 4) * 1024 + thread) * 4 + u % 4, so a
    // thread fetches 16 bytes at a time and a wave 1 KB per load.  Rows start 256-byte aligned and are
    // padded to a multiple of 64 entries (ldp), so a load that starts below ldp stays inside the row;
    // the others are clamped and, like everything at or past t_hi, masked (loads stay unconditional).
    // A slice starts at a multiple of 4096 positions, so its loads are aligned like the row's.
    constexpr int SB = ITEMS == -1 ? 8 : 16;
    auto stream_pos = [&](int t0, int u) { return t0 + ((u >> 2) * SEL_THREADS + (int)threadIdx.x) * 4 + (u & 3); };
    // The loads of the next batch are issued before the current one is worked on.
    auto stream_issue = [&](f32x4 (&x)[SB / 4], int t0) {
#pragma unroll
        for (int v = 0; v < SB / 4; ++v) {
            const int t = stream_pos(t0, 4 * v);
            x[v] = *reinterpret_cast<const f32x4*>(row + (t < (int)ldp ? t : (int)ldp - 4));
        }
    };
    auto stream_take = [&](const f32x4 (&x)[SB / 4], uint32_t (&kk)[SB], int t0) {
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            const int t = stream_pos(t0, u);
            const uint32_t kv_ = key_of(x[u >> 2][u & 3]);
            kk[u] = (t < t_hi && t >= n_sink) ? kv_ : 0u;
        }
    };
    // f(keys of the batch, first position of the batch) for every batch of a streamed row
    auto stream_batches = [&](auto f) {
        f32x4 x[SB / 4];
        stream_issue(x, t_lo);
        for (int t0 = t_lo; t0 < t_hi; t0 += SB * SEL_THREADS) {
            uint32_t kk[SB];
            stream_take(x, kk, t0);
            stream_issue(x, t0 + SB * SEL_THREADS);    // past the row's end: clamped loads, never used
            __builtin_amdgcn_sched_barrier(0);
            f(kk, t0);
        }
    };
    auto scan = [&](auto f) {
        if constexpr (ITEMS > 0) {
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) {
                f(keys[i], MERGE ? pos_of[i] : t_lo + i * SEL_THREADS + (int)threadIdx.x);
            }
        } else {
            stream_batches([&](const uint32_t (&kk)[SB], int t0) {
#pragma unroll
                for (int u = 0; u < SB; ++u) f(kk[u], stream_pos(t0, u));
            });
        }
    };

    // 0. a cheap lower bound for the k_eff-th best key.  Each thread keeps the MTOP largest of
    //    its own candidates (MTOP * 1024 >= k); the k_eff-th largest of those values cannot
    //    exceed the k_eff-th largest of all candidates, so its top digit d0 bounds the answer's
    //    from below and the first histogram pass may skip every key under d0 -- most of them,
    //    which matters because LDS histogram atomics are what this kernel is bound by.
    //    A streamed row keeps the maxima of 8 disjoint groups of the thread's candidates instead
    //    (one instruction per key): distinct candidates again, so the same argument holds, and
    //    with 8192 group maxima the bound is about as tight.
    //    The candidates a filtered pass kept (when ranking them as they are did not work out, above): no
    //    bound (d0 = 0) and no list for them.
    const bool direct = MERGE && flt.thr != nullptr;
    constexpr int MG = ITEMS > 0 ? MTOP : ITEMS == -1 ? 4 : 8;
    uint32_t d0 = 0u;
    if (!direct) {
    uint32_t top[MG];
#pragma unroll
    for (int j = 0; j < MG; ++j) top[j] = 0u;
    if constexpr (ITEMS > 0) {
        scan([&](uint32_t key, int) {
            uint32_t x = key;
#pragma unroll
            for (int j = 0; j < MTOP; ++j) {
                const uint32_t hi = top[j] > x ? top[j] : x;
                x = top[j] > x ? x : top[j];
                top[j] = hi;
            }
        });
    } else {
        stream_batches([&](const uint32_t (&kk)[SB], int) {
#pragma unroll
            for (int u = 0; u < SB; ++u) top[u % MG] = top[u % MG] > kk[u] ? top[u % MG] : kk[u];
        });
    }
    for (int i = threadIdx.x; i < 2048; i += SEL_THREADS) hist[i] = 0;
    if (threadIdx.x == 0) {
        st.prefix = 0;
        st.need = k_eff;
        st.count_eq = 0;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < MG; ++j) atomicAdd(&hist[top[j] >> 21], 1);
    __syncthreads();
    pick_digit<2048>(hist, scratch, &st, 21);
    d0 = st.prefix >> 21;
    __syncthreads();
    }
    //    With the keys in registers, what lies at or above the bound -- typically 1.3 to 2 times k
    //    candidates -- is ranked as it is (quick_rank: only the segments that reach into the first k_eff
    //    ranks are walked); the selection below runs only if that does not work out.
    if constexpr (ITEMS > 0 && ITEMS <= 16 && !MERGE) {   // (32 keys per thread leave no registers for it)
        if (!slice && !raw_keys && d0 > 0u) {
            const uint32_t bound = d0 << 21;
            auto mine = [&](int i) -> uint64_t {
                const int t = t_lo + i * SEL_THREADS + (int)threadIdx.x;
                return keys[i] >= bound ? ((uint64_t)keys[i] << 32) | (uint32_t)~(uint32_t)t : 0;
            };
            constexpr int SEGS = topk_area_entries(ITEMS, MTOP) - 1024;
            if (quick_rank<ITEMS>(mine, key_score(bound), k_eff, cand, SEGS, reinterpret_cast<int*>(cand + SEGS), scratch,
                                  rho_head + (int64_t)b * k * H + h, H))
                return;
        }
    }
    // 1-3 for candidates delivered by scan_fn: the remaining digits of the k_eff-th best score key
    // T (its top digit is already in st), the position bound among the keys equal to T when they
    // straddle the cut (rare), and the survivors' composites compacted into sort_buf in any order.
    uint32_t sel_T = 0u;                               // the k_eff-th best score key, once finish has run
    auto finish = [&](auto scan_fn) {
        radix_select(1, k_eff, 0u, scan_fn, [](uint32_t skey, int, uint32_t* key) { *key = skey; return true; },
                     hist, scratch, &st);
        const uint32_t T = st.prefix;
        sel_T = T;
        const int need_eq = st.need, count_eq = st.count_eq;
        __syncthreads();
        uint32_t pos_bound = 0xffffffffu;              // take every tie
        if (count_eq > need_eq) {
            radix_select(0, need_eq, 0u, scan_fn,
                         [T](uint32_t skey, int t, uint32_t* key) { *key = ~(uint32_t)t; return skey == T; },
                         hist, scratch, &st);
            pos_bound = ~st.prefix;                    // need_eq-th smallest tying position
            __syncthreads();
        }
        if (threadIdx.x == 0) n_out = 0;
        __syncthreads();                               // also: histogram no longer needed
        // one reservation per wave: count this thread's survivors, scan the counts over the wave
        int mine = 0;
        scan_fn([&](uint32_t key, int t) {
            mine += (key > T || (key == T && (uint32_t)t <= pos_bound)) ? 1 : 0;
        });
        int slot = wave_reserve(mine, &n_out);
        scan_fn([&](uint32_t key, int t) {
            if (key > T || (key == T && (uint32_t)t <= pos_bound)) {
                if (slot < NSORT) sort_buf[slot] = ((uint64_t)key << 32) | (uint32_t)~(uint32_t)t;
                ++slot;
            }
        });
        __syncthreads();
    };

    // The top digit of T comes from one histogram pass over all candidates whose top digit is at
    // least d0.  Those are the only ones that can still matter; when they fit they are copied to
    // an LDS list and everything after this pass walks the list (a few entries per thread)
    // instead of every candidate again.
    for (int i = threadIdx.x; i < 2048; i += SEL_THREADS) hist[i] = 0;
    if (threadIdx.x == 0) {
        st.prefix = 0;
        st.need = k_eff;
        st.count_eq = 0;
        n_list = 0;
    }
    __syncthreads();
    int listable = 0;
    bool listed = false;
    if constexpr (ITEMS <= 0) {
        // one walk does both: each batch is counted into the histogram, the wave reserves list
        // slots for the batch's candidates and writes them (in arbitrary order; what is selected
        // from the list does not depend on it)
        stream_batches([&](const uint32_t (&kk)[SB], int t0) {
            int n_new = 0;
#pragma unroll
            for (int u = 0; u < SB; ++u) {
                const uint32_t dg = kk[u] >> 21;
                if (dg >= d0) {
                    atomicAdd(&hist[dg], 1);
                    ++n_new;
                }
            }
            int slot = wave_reserve(n_new, &n_list);
#pragma unroll
            for (int u = 0; u < SB; ++u) {
                if ((kk[u] >> 21) >= d0) {
                    if (slot < CAP) cand[slot] = ((uint64_t)kk[u] << 32) | (uint32_t)~(uint32_t)stream_pos(t0, u);
                    ++slot;
                }
            }
        });
        __syncthreads();
        pick_digit<2048>(hist, scratch, &st, 21);
        listed = n_list <= CAP;
    } else {
    scan([&](uint32_t key, int) {
        const uint32_t dg = key >> 21;
        if (dg >= d0) {
            atomicAdd(&hist[dg], 1);
            ++listable;
        }
    });
    __syncthreads();
    pick_digit<2048>(hist, scratch, &st, 21);
    if (CAP > 0 && !direct) {
        int slot = wave_reserve(listable, &n_list);
        __syncthreads();
        listed = n_list <= CAP;
        if (listed) {
            scan([&](uint32_t key, int t) {
                if ((key >> 21) >= d0) cand[slot++] = ((uint64_t)key << 32) | (uint32_t)~(uint32_t)t;
            });
            __syncthreads();
        }
    }
    }
    if (listed) {
        const int n = n_list;
        // Rows too long for the ranking from registers above: the list holds exactly what lies at or above
        // the bound, so it is ranked as it is (the entries move to registers first: the segments take the
        // list's place, but only once the attempt is known to work out).
        if constexpr ((ITEMS > 16 || ITEMS == 0) && CAP > 0) {   // (not the lean streamed form: 64 registers)
            if (!slice && !raw_keys && d0 > 0u) {
                constexpr int LPT = CAP / SEL_THREADS;
                uint64_t lv[LPT];
#pragma unroll
                for (int j = 0; j < LPT; ++j) {
                    const int i = (int)threadIdx.x + j * SEL_THREADS;
                    lv[j] = i < n ? cand[i] : 0;
                }
                if (quick_rank<LPT>([&](int j) { return lv[j]; }, key_score(d0 << 21), k_eff, cand, CAP,
                                    reinterpret_cast<int*>(cand + CAP), scratch, rho_head + (int64_t)b * k * H + h, H))
                    return;
            }
        }
        finish([&](auto f) {
            for (int i = threadIdx.x; i < n; i += SEL_THREADS) {
                const uint64_t cv = cand[i];
                f((uint32_t)(cv >> 32), (int)~(uint32_t)cv);
            }
        });
    } else {
        finish(scan);
    }
    if (slice) {                                      // the slice's k best, in any order; the merge ranks
        for (int i = threadIdx.x; i < k; i += SEL_THREADS) my_parts[i] = i < k_eff ? sort_buf[i] : 0;
        return;
    }
    // 3a. The ranking, the quick way (quick_rank); the network below remains for rows with crowded bins
    //     (many equal scores), non-finite scores and raw keys.
    if (!raw_keys) {
        uint64_t mine[MTOP];
#pragma unroll
        for (int j = 0; j < MTOP; ++j) {
            const int i = (int)threadIdx.x + j * SEL_THREADS;
            mine[j] = i < k_eff ? sort_buf[i] : 0;
        }
        if (quick_rank<MTOP>([&](int j) { return mine[j]; }, key_score(sel_T), k_eff, cand, NSORT,
                             reinterpret_cast<int*>(cand + NSORT), scratch, rho_head + (int64_t)b * k * H + h, H))
            return;
    }
    for (int i = k_eff + threadIdx.x; i < NSORT; i += SEL_THREADS) sort_buf[i] = 0;
    __syncthreads();
    // 3b. Bitonic network over NSORT = MTOP * 1024 composites, MTOP per thread in registers:
    // element j of thread (wave, lane) is index wave*64*MTOP + j*64 + lane.  A step with
    // stride < 64 exchanges between lanes of a wave, a stride of 64 .. 32*MTOP between the
    // thread's own registers, and only larger strides go through LDS with workgroup barriers.
    {
        const int lane = lane_id(), base = wave_id() * 64 * MTOP + lane;
        uint64_t v[MTOP];
#pragma unroll
        for (int j = 0; j < MTOP; ++j) v[j] = sort_buf[base + j * 64];
#pragma unroll
        for (int size = 2; size <= NSORT; size <<= 1) {
#pragma unroll
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                if (stride >= 64 * MTOP) {             // partner in another wave
                    __syncthreads();
#pragma unroll
                    for (int j = 0; j < MTOP; ++j) sort_buf[base + j * 64] = v[j];
                    __syncthreads();
#pragma unroll
                    for (int j = 0; j < MTOP; ++j) {
                        const int i = base + j * 64;
                        const uint64_t o = sort_buf[i ^ stride];
                        const bool keep_max = ((i & stride) == 0) == ((i & size) == 0);
                        v[j] = ((v[j] > o) == keep_max) ? v[j] : o;
                    }
                } else if (stride >= 64) {             // partner in this thread's registers
                    const int js = stride >> 6;
#pragma unroll
                    for (int j = 0; j < MTOP; ++j) {
                        if ((j & js) == 0 && (j | js) < MTOP) {
                            const int i = base + j * 64;
                            const bool desc = (i & size) == 0;
                            const uint64_t a = v[j], c = v[j | js];
                            const bool sw = (a < c) == desc;
                            v[j] = sw ? c : a;
                            v[j | js] = sw ? a : c;
                        }
                    }
                } else {                               // partner in another lane of this wave
#pragma unroll
                    for (int j = 0; j < MTOP; ++j) {
                        const int i = base + j * 64;
                        const uint32_t olo = lane_xor_any((uint32_t)v[j], stride);
                        const uint32_t ohi = lane_xor_any((uint32_t)(v[j] >> 32), stride);
                        const uint64_t o = ((uint64_t)ohi << 32) | olo;
                        const bool keep_max = ((i & stride) == 0) == ((i & size) == 0);
                        v[j] = ((v[j] > o) == keep_max) ? v[j] : o;
                    }
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < MTOP; ++j) sort_buf[base + j * 64] = v[j];
        __syncthreads();
    }
    // 4. rank-major output
    int32_t* __restrict__ out = rho_head + (int64_t)b * k * H + h;
    for (int j = threadIdx.x; j < k_eff; j += SEL_THREADS)
        out[(int64_t)j * H] = (int32_t)~(uint32_t)sort_buf[j];
}

// ---------------------------------------------------------------- union / rank / window
//
// One 1024-thread workgroup per sequence.  Slot s = j*H + h of the rank-major array is head h's
// rank-j pick; the historical part of rho is the set of the first K-W distinct tokens met when
// the slots are walked in order.  The set is a bitmap over the candidate positions in LDS (one bit
// per position: 16 KB for 131072 tokens).  A range of slots is added with one atomic OR per slot;
// the OR's return value tells whether the slot set its bit, so the number of new tokens in the
// range is exact even though, among slots of the range that name the same token, an arbitrary
// one sets it.  Ranges are taken in slot order, 8192 slots at a time; the range in which the
// count would pass K-W is taken back (the bits it set are cleared) and walked again in 1024-slot
// ranges, the crossing one of those in 64-slot groups by a single wave, and the crossing group is
// resolved exactly: a lane's pick counts if no lower lane of the group names the same token.
// What is left set is the answer; it is emitted in ascending position order, followed by the
// window {L-W .. L-1}.

// Adds the sink positions 0 .. n_sink-1 (never picked: they are no candidates) to the set in
// `bits` and writes the set's positions in ascending order, at most `limit` of them.  Thread i
// owns the words [i * wpt, i * wpt + wpt).  Returns n_sink.
__device__ __forceinline__ int emit_sinks_and_set(uint32_t* bits, int n_words, int n_sink, int limit, int* scratch,
                                                  int32_t* __restrict__ out) {
    const int tid = threadIdx.x;
    for (int t = tid; t < n_sink; t += SEL_THREADS) atomicOr(&bits[t >> 5], 1u << (t & 31));
    if (n_sink > 0) __syncthreads();
    const int wpt = (n_words + SEL_THREADS - 1) / SEL_THREADS;
    const int w_lo = tid * wpt, w_hi = (w_lo + wpt < n_words) ? w_lo + wpt : n_words;
    int mine = 0;
    for (int i = w_lo; i < w_hi; ++i) mine += __popc(bits[i]);
    int total;
    int off = block_scan_excl(mine, scratch, &total);
    for (int i = w_lo; i < w_hi; ++i) {
        uint32_t word = bits[i];
        while (word) {
            const int bpos = __ffs(word) - 1;
            if (off < limit) out[off] = i * 32 + bpos;
            ++off;
            word &= word - 1;
        }
    }
    return n_sink;
}

constexpr int UNION_UNROLL = 8;
constexpr int UNION_MAX_POSITIONS = 144 * 1024 * 8;   // candidate positions a 144 KB bitmap covers

__global__ __launch_bounds__(SEL_THREADS) void union_kernel(const int32_t* __restrict__ rho_head,
                                                             const int32_t* __restrict__ seq_lens,
                                                             int32_t* __restrict__ idx, int32_t* __restrict__ cnt,
                                                             int H, int k, int budget, int window, int n_sink) {
    extern __shared__ uint32_t bits[];                // ceil(Lc / 32) words
    __shared__ int wave_cnt[2 * SEL_WAVES];
    __shared__ int scratch[SEL_WAVES + 1];
    __shared__ int picks[SEL_THREADS];                // the picks of the crossing 1024-slot range, by slot
    __shared__ uint32_t idle[64];                     // where lanes with nothing to add send their atomic
    const int b = blockIdx.x, tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int L = seq_lens[b];
    int32_t* __restrict__ out = idx + (int64_t)b * budget;
    if (L <= budget) {
        for (int t = tid; t < L; t += SEL_THREADS) out[t] = t;
        if (tid == 0) cnt[b] = L;
        return;
    }
    const int Lc = L - window;
    const int k_eff = k < Lc - n_sink ? k : Lc - n_sink;
    const int S = k_eff * H;
    const int n_hist = budget - window - n_sink;      // picks to keep; the sink positions come on top
    const int32_t* __restrict__ rho = rho_head + (int64_t)b * k * H;
    const int n_words = (Lc + 31) >> 5;
    for (int i = tid; i < n_words; i += SEL_THREADS) bits[i] = 0u;
    __syncthreads();

    // The picks of the UNION_UNROLL slots s0 + u * 1024 + tid are requested with clamped,
    // unconditional loads (request_picks) and looked at later (take_picks: -1 past the end; a pick is
    // always a candidate position).  The empty asm keeps the compiler from turning the loads into one
    // branch each.
    auto request_picks = [&](int s0, int* raw) {
#pragma unroll
        for (int u = 0; u < UNION_UNROLL; ++u) raw[u] = rho[min(s0 + u * SEL_THREADS + tid, S - 1)];
    };
    auto take_picks = [&](int s0, int* raw, int* dst) {
#pragma unroll
        for (int u = 0; u < UNION_UNROLL; ++u) asm volatile("" : "+v"(raw[u]));
#pragma unroll
        for (int u = 0; u < UNION_UNROLL; ++u)
            dst[u] = (s0 + u * SEL_THREADS + tid < S && (uint32_t)raw[u] < (uint32_t)Lc) ? raw[u] : -1;
    };
    // workgroup total of per-wave counts (wave-uniform argument); wave_cnt alternates between two
    // halves so that one barrier per call is enough
    int parity = 0;
    auto block_total = [&](int wave_total) {
        int* const slot = wave_cnt + parity * SEL_WAVES;
        parity ^= 1;
        if (lane == 0) slot[w] = wave_total;
        __syncthreads();
        int sum = 0;
#pragma unroll
        for (int i = 0; i < SEL_WAVES; ++i) sum += slot[i];
        return sum;
    };
    int cum = 0;                                       // distinct tokens in the bitmap
    bool crossed = false;
    constexpr int CH = UNION_UNROLL * SEL_THREADS;
    int tok[UNION_UNROLL], raw[UNION_UNROLL];          // this range's picks; the next range's, requested early
    request_picks(0, raw);
    for (int c0 = 0; c0 < S && n_hist > 0; c0 += CH) {
        take_picks(c0, raw, tok);
        request_picks(c0 + CH, raw);
        uint32_t won = 0;
        int wave_added = 0;
#pragma unroll
        for (int u = 0; u < UNION_UNROLL; ++u) {
            // Neighbouring slots are neighbouring heads at one rank and often name the same token;
            // a lane whose left neighbour in its 16-lane row has the same pick leaves the atomic to it
            // (same-address LDS atomics of one instruction are carried out one after the other; for
            // the same reason the lanes that stay out add zero to a word of their own, not to a shared one).
            const int left = __builtin_amdgcn_update_dpp(-2, tok[u], 0x111, 0xF, 0xF, false);   // row_shr:1; -2 into lane 0 of a row
            const bool lead = tok[u] >= 0 && tok[u] != left;
            const uint32_t bit = 1u << (tok[u] & 31);
            const uint32_t old = atomicOr(lead ? &bits[tok[u] >> 5] : &idle[lane], lead ? bit : 0u);
            const bool wn = lead && !(old & bit);
            if (wn) won |= 1u << u;
            wave_added += __popcll(__ballot(wn));
        }
        const int added = block_total(wave_added);
        if (cum + added >= n_hist) {                   // take the range back and look closer
#pragma unroll
            for (int u = 0; u < UNION_UNROLL; ++u)
                if ((won >> u) & 1) atomicAnd(&bits[tok[u] >> 5], ~(1u << (tok[u] & 31)));
            __syncthreads();
            crossed = true;
            break;
        }
        cum += added;
    }

    int n_take = cum;                                  // fewer than K-W distinct picks in total (k < K-W only)
    if (crossed) {
        // tok[u] of thread i is slot u * 1024 + i of the crossing range
        n_take = n_hist;
        int my_pick = -1;                              // the thread's pick in the crossing 1024-slot range
        bool found = false;
#pragma unroll
        for (int u = 0; u < UNION_UNROLL; ++u) {
            if (!found) {                              // uniform
                const uint32_t bit = 1u << (tok[u] & 31);
                const uint32_t old = atomicOr(&bits[tok[u] >= 0 ? tok[u] >> 5 : 0], tok[u] >= 0 ? bit : 0u);
                const bool won = tok[u] >= 0 && !(old & bit);
                const int added = block_total(__popcll(__ballot(won)));
                if (cum + added >= n_hist) {
                    if (won) atomicAnd(&bits[tok[u] >> 5], ~bit);
                    my_pick = tok[u];
                    found = true;
                } else {
                    cum += added;
                }
            }
        }
        picks[tid] = my_pick;
        __syncthreads();
        if (w == 0) {                                  // one wave: its LDS accesses happen in program order
            int group_pick[SEL_WAVES];
#pragma unroll
            for (int g = 0; g < SEL_WAVES; ++g) group_pick[g] = picks[g * 64 + lane];
            int t = -1;                                // the lane's pick in the crossing group
            bool found = false;
#pragma unroll
            for (int g = 0; g < SEL_WAVES; ++g) {
                if (!found) {                          // uniform
                    const int tg = group_pick[g];
                    const uint32_t bit = 1u << (tg & 31);
                    uint32_t* const word = &bits[tg >= 0 ? tg >> 5 : 0];
                    const bool won = tg >= 0 && !(atomicOr(word, tg >= 0 ? bit : 0u) & bit);
                    const int c = __popcll(__ballot(won));
                    if (cum + c < n_hist) {
                        cum += c;
                    } else {                           // take the group back
                        if (won) atomicAnd(word, ~bit);
                        t = tg;
                        found = true;
                    }
                }
            }
            if (found) {
                // a pick of the crossing group counts only if no lower lane names its token
                bool dup = false;
#pragma unroll
                for (int l = 0; l < 63; ++l) {
                    const int tl = __builtin_amdgcn_readlane(t, l);
                    dup |= (l < lane) && (tl == t);
                }
                const uint32_t bit = 1u << (t & 31);
                uint32_t* const word = &bits[t >= 0 ? t >> 5 : 0];
                const bool is_new = t >= 0 && !dup && !(*word & bit);
                const uint64_t ballot = __ballot(is_new);
                if (is_new && cum + mbcnt(ballot) < n_hist) atomicOr(word, bit);
            }
        }
        __syncthreads();
    }
    n_take += emit_sinks_and_set(bits, n_words, n_sink, n_hist + n_sink, scratch, out);
    for (int j = tid; j < window; j += SEL_THREADS) out[n_take + j] = L - window + j;
    if (tid == 0) cnt[b] = n_take + window;
}

// ---------------------------------------------------------------- filtered selection: the threshold
//
// Writing a score for every (head, cached token) is what the selection layer's pass pays most for
// beyond its reads, and the per-head top-k then walks all of them again.  The fast path of a selection
// layer writes only the scores that can matter.  A first, small launch (this kernel) scores a SAMPLE
// of the tokens -- every 16th tile of 64, fewer of a very long sequence -- and takes, per head, a
// threshold theta from the sample such that with overwhelming probability at least k and not many more than k of the head's
// candidates score >= theta; the pass then keeps only those (as (score key, position) composites,
// compacted per head) and the top-k ranks among them.  theta is only a guess, so everything that
// depends on it is checked: a head whose kept candidates turn out fewer than k (theta too high) or more
// than the buffers hold (theta too low, or many equal scores) is flagged, and the flagged heads are
// scored and ranked again the ordinary way (the scores-only pass and topk_kernel in their flagged-only forms).
// The result never depends on theta; only the time does.
//
// The sample of a head has n_s candidates out of n (every position in a sampled tile that is a
// candidate); with the target fraction f = k / n, theta is at or just below the j-th largest of the
// sample, where
//   j = f n_s + FILTER_Z sqrt(f (1 - f) n_s) + 1:
// the number of sample members among the head's true top k is hypergeometric with mean f n_s and
// standard deviation below sqrt(f (1 - f) n_s), so it exceeds j - 1 with probability ~ 3e-7 at
// FILTER_Z = 5 for tokens in no particular order (ordered inputs can defeat any fixed sample; they cost
// the second chance, nothing else).  A head whose expected share of kept candidates is above
// FILTER_MAX_SHARE, or whose kept candidates would likely overflow its buffer, gains nothing from the
// filter and is flagged at once.
//
// One 1024-thread workgroup per (sequence, KV head).  Every wave scores sampled tiles on its own,
// straight from memory on the matrix cores (below); the keys of the sample stay in LDS, [head][slot].  Then a quarter of the workgroup works on each
// head: the sample's scores are counted into 2048 bins that divide [lowest, highest sample score]
// evenly (by value, not by key: keys are dense where scores are small and a digit of the key would
// put most of the sample into a handful of bins), the bin that holds the j-th largest is found by a
// scan from the top, and theta is the smallest sample key in that bin -- so the number of sample
// members at or above theta is known exactly (j' >= j), and the expected share is j' / (n_s + 1).
constexpr int SAMPLE_STEP = 16;                       // every 16th tile at least ...
constexpr int SAMPLE_MAX_TILES = 64;                  // ... and 64 tiles (4096 sample slots) per sequence at most
constexpr float FILTER_Z = 5.0f;
constexpr float FILTER_MAX_SHARE = 0.4f;
constexpr int THR_BINS = 2048;

// Expected number of kept candidates plus three standard deviations, for a head with n candidates,
// n_s of them sampled, jp sample members at or above the threshold.
__host__ __device__ inline float filter_kept_bound(float n, float n_s, float jp) {
    const float share = jp / (n_s + 1.0f);
    return n * (share + 3.0f * sqrtf(share * (1.0f - share) / (n_s > 1.0f ? n_s : 1.0f)));
}
// j of the account above.
__host__ __device__ inline int filter_sample_rank(float k_eff, float n, float n_s) {
    const float frac = k_eff / n;
    return (int)(frac * n_s + FILTER_Z * sqrtf(frac * (1.0f - frac) * n_s)) + 1;
}

template <int GQ, bool PAGED>
__global__ __launch_bounds__(SEL_THREADS) void sample_threshold_kernel(const uint16_t* __restrict__ q, int H, int k,
                                                                        int budget, int window,
                                                                        int n_slots_max, FilterState f, KvView kv) {
    static_assert(GQ <= 4, "a quarter of the workgroup per head");
    extern __shared__ uint32_t thr_lds_buf[];         // keys [GQ][n_slots_max], then bins [GQ][THR_BINS]
    uint32_t* const keys_all = thr_lds_buf;
    int* const hist_all = reinterpret_cast<int*>(thr_lds_buf + GQ * n_slots_max);
    __shared__ uint32_t red_min[4][4], red_max[4][4], thr_min[4];
    __shared__ int red_cnt[4][4], wave_sum[4][4], sel_bin[4], sel_jp[4];
    const int kvh = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row0 = (int64_t)b * H + kvh * GQ;     // first head of the group
    if (tid < GQ) {
        f.cand_cnt[row0 + tid] = 0;
        f.fail[row0 + tid] = 0;
    }
    if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) *f.n_failed = 0;   // counted by the top-k, a later launch
    const int L = kv.seq_lens[b];
    if (L <= budget) {                                  // rho is every token: nothing is selected
        if (tid < GQ) f.thr[row0 + tid] = 0xffffffffu;
        return;
    }
    const int Lc = L - window, n = Lc - f.n_sink, k_eff = k < n ? k : n;
    const int tiles_all = (Lc + 63) >> 6;
    // every SAMPLE_STEP-th tile of this sequence, or as many tiles as the launch has LDS for (a short
    // sequence in a cache laid out for long ones is still sampled densely)
    const int max_tiles = n_slots_max >> 6;
    const int tile_step = max(SAMPLE_STEP, (tiles_all + max_tiles - 1) / max_tiles);
    const int n_tiles = (tiles_all + tile_step - 1) / tile_step;
    const int n_slots = n_tiles * 64;

    // The sample's scores come from V_MFMA_F32_16X16X16_BF16, 16 tokens x 16 heads (GQ of them real) per
    // instruction: lane l holds, of token l % 16 and of head l % 16, the 16-byte chunks (4 j + l / 16) of
    // the 128 columns, j = 0 .. 3 -- the order in which columns are summed does not matter here, a sample
    // score only helps to guess a threshold and need not be the score the pass computes to the last bit.
    // A load instruction reads 64 contiguous bytes of each of 16 rows.
    const int m16 = lane & 15, kg = lane >> 4;
    u32x4 qreg[4];
#pragma unroll
    for (int jc = 0; jc < 4; ++jc) {
        qreg[jc] = u32x4{0u, 0u, 0u, 0u};
        if (m16 < GQ) qreg[jc] = *reinterpret_cast<const u32x4*>(q + (row0 + m16) * D + (jc * 4 + kg) * 8);
    }
    for (int s = wave; s < n_tiles; s += SEL_WAVES) {
        const int t0 = s * tile_step * 64;
#pragma unroll
        for (int pair = 0; pair < 2; ++pair) {
            u32x4 stage[2][4];
#pragma unroll
            for (int g2 = 0; g2 < 2; ++g2) {
                const int t = t0 + (pair * 2 + g2) * 16 + m16;
                const uint16_t* __restrict__ krow = kv.k + row_offset<PAGED>(kv, b, kvh, min(t, Lc - 1));
#pragma unroll
                // (plain loads: the sampled tiles are read again by the pass, from the last-level cache if still there)
                for (int jc = 0; jc < 4; ++jc) stage[g2][jc] = *reinterpret_cast<const u32x4*>(krow + (jc * 4 + kg) * 8);
            }
#pragma unroll
            for (int g2 = 0; g2 < 2; ++g2) {
                f32x4 acc = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int jc = 0; jc < 4; ++jc) {
                    const s16x4 a_lo = __builtin_bit_cast(s16x4, make_uint2(stage[g2][jc].x, stage[g2][jc].y));
                    const s16x4 a_hi = __builtin_bit_cast(s16x4, make_uint2(stage[g2][jc].z, stage[g2][jc].w));
                    const s16x4 b_lo = __builtin_bit_cast(s16x4, make_uint2(qreg[jc].x, qreg[jc].y));
                    const s16x4 b_hi = __builtin_bit_cast(s16x4, make_uint2(qreg[jc].z, qreg[jc].w));
                    acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_lo, b_lo, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_hi, b_hi, acc, 0, 0, 0);
                }
                // the lane holds, for head l % 16, the tokens 4 (l / 16) + i of this group of 16
                if (m16 < GQ) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int m = (pair * 2 + g2) * 16 + kg * 4 + i, t = t0 + m;
                        const bool valid = t < Lc && t >= f.n_sink;   // key 0 for what is no candidate
                        keys_all[m16 * n_slots_max + s * 64 + m] = valid ? score_key(acc[i]) : 0u;
                    }
                }
            }
        }
    }
    __syncthreads();

    // a quarter of the workgroup (4 waves) per head; quarters without a head only keep the barriers company
    const int hq = tid >> 8, tq = tid & 255, wq = tq >> 6;
    const bool has_head = hq < GQ;
    const uint32_t* const keys = keys_all + (has_head ? hq : 0) * n_slots_max;
    int* const hist = hist_all + (has_head ? hq : 0) * THR_BINS;
    {
        int cnt = 0;
        uint32_t lo = 0xffffffffu, hi = 0u;
        if (has_head) {
            for (int sl = tq; sl < n_slots; sl += 256) {
                const uint32_t key = keys[sl];
                if (key != 0u) {
                    ++cnt;
                    lo = key < lo ? key : lo;
                    hi = key > hi ? key : hi;
                }
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            cnt += __shfl_xor(cnt, o);
            const uint32_t lo2 = __shfl_xor(lo, o), hi2 = __shfl_xor(hi, o);
            lo = lo2 < lo ? lo2 : lo;
            hi = hi2 > hi ? hi2 : hi;
        }
        if (lane == 0) {
            red_cnt[hq][wq] = cnt;
            red_min[hq][wq] = lo;
            red_max[hq][wq] = hi;
        }
        for (int i = tq; i < THR_BINS; i += 256) hist[i] = 0;
        if (tq == 0) thr_min[hq] = 0xffffffffu;
    }
    __syncthreads();
    int n_s = 0;
    uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        n_s += red_cnt[hq][w];
        kmin = red_min[hq][w] < kmin ? red_min[hq][w] : kmin;
        kmax = red_max[hq][w] > kmax ? red_max[hq][w] : kmax;
    }
    const int j = filter_sample_rank((float)k_eff, (float)n, (float)n_s);
    const float smin = key_score(kmin), range = key_score(kmax) - smin;
    // no usable guess: too few in the sample, or scores that are not finite or all alike
    bool bad = !has_head || j >= n_s || !(range > 0.0f && range < 3.0e38f);
    const float scale = bad ? 0.0f : (float)(THR_BINS - 1) / range;
    auto bin_of = [&](uint32_t key) {
        const int bi = (int)((key_score(key) - smin) * scale);
        return bi < 0 ? 0 : bi > THR_BINS - 1 ? THR_BINS - 1 : bi;
    };
    if (!bad) {
        for (int sl = tq; sl < n_slots; sl += 256) {
            const uint32_t key = keys[sl];
            if (key != 0u) atomicAdd(&hist[bin_of(key)], 1);
        }
    }
    __syncthreads();
    {   // thread i of the quarter owns the 8 bins [2048 - 8 (i + 1), 2048 - 8 i), walked from the top
        int local[8], sum = 0;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            local[u] = hist[THR_BINS - 1 - (tq * 8 + u)];
            sum += local[u];
        }
        int inc = sum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(inc, o);
            if (lane >= o) inc += up;
        }
        if (lane == 63) wave_sum[hq][wq] = inc;
        __syncthreads();
        int above = inc - sum;                          // sample members in higher bins, owned by lower threads
        for (int w = 0; w < wq; ++w) above += wave_sum[hq][w];
        if (!bad && above < j && j <= above + sum) {
            int run = above;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (run < j && j <= run + local[u]) {
                    sel_bin[hq] = THR_BINS - 1 - (tq * 8 + u);
                    sel_jp[hq] = run + local[u];
                }
                run += local[u];
            }
        }
    }
    __syncthreads();
    if (!bad) {
        const int bsel = sel_bin[hq];
        uint32_t lo = 0xffffffffu;
        for (int sl = tq; sl < n_slots; sl += 256) {
            const uint32_t key = keys[sl];
            if (key != 0u && bin_of(key) == bsel) lo = key < lo ? key : lo;
        }
        if (lo != 0xffffffffu) atomicMin(&thr_min[hq], lo);
    }
    __syncthreads();
    if (has_head && tq == 0) {
        const int64_t row = row0 + hq;
        if (!bad) {
            const float jp = (float)sel_jp[hq];
            bad = jp / (float)(n_s + 1) > FILTER_MAX_SHARE || filter_kept_bound((float)n, (float)n_s, jp) > (float)f.cap;
        }
        f.thr[row] = bad ? 0xffffffffu : thr_min[hq];
        if (bad) flag_failed(f, row);
    }
}

// Aggregation for the other two readings of "globally ranked" (Sec. 3.2 names no ranking key):
// one key per candidate position, larger = better, 0 = proposed by no head.
//   votes     : (number of proposing heads) << 13 | (8191 - best rank among them)
//   max score : score_key of the largest score among the proposing heads
// The unified list is then the top K-W positions by (key descending, position ascending), which the
// per-head top-k kernel computes from the key row (raw_keys).  One workgroup per sequence walks
// the H * k_eff picks; key rows live in the workspace: agg[b][0][.] keys, agg[b][1][.] best ranks.
constexpr int RANK_VOTES_SHIFT = 13;                  // ranks are below 8192

__global__ __launch_bounds__(SEL_THREADS) void rank_aggregate_kernel(const int32_t* __restrict__ rho_head,
                                                                      const float* __restrict__ P, int64_t ldp,
                                                                      const int32_t* __restrict__ seq_lens,
                                                                      uint32_t* __restrict__ agg, int64_t ld_agg, int H,
                                                                      int k, int budget, int window, int by_score,
                                                                      int n_sink) {
    const int b = blockIdx.x, tid = threadIdx.x;
    const int L = seq_lens[b];
    if (L <= budget) return;
    const int Lc = L - window;
    const int k_eff = k < Lc - n_sink ? k : Lc - n_sink;
    const int S = k_eff * H;
    uint32_t* const key = agg + (int64_t)b * 2 * ld_agg;
    uint32_t* const best = key + ld_agg;
    for (int t = tid; t < Lc; t += SEL_THREADS) {
        key[t] = 0u;
        best[t] = 0u;
    }
    __threadfence();
    __syncthreads();
    const int32_t* __restrict__ rho = rho_head + (int64_t)b * k * H;
    for (int s = tid; s < S; s += SEL_THREADS) {
        const int j = s / H, h = s - j * H;
        const int t = rho[s];
        if ((uint32_t)t >= (uint32_t)Lc) continue;    // never: a pick is a candidate position
        if (by_score) {
            atomicMax(&key[t], score_key(P[((int64_t)b * H + h) * ldp + t]));
        } else {
            atomicAdd(&key[t], 1u << RANK_VOTES_SHIFT);
            atomicMax(&best[t], (uint32_t)(8191 - j));
        }
    }
    if (by_score) return;
    __threadfence();
    __syncthreads();
    for (int t = tid; t < Lc; t += SEL_THREADS) {
        // the atomics above were carried out in L2: read there, not in this CU's L1
        const uint32_t v = __hip_atomic_load(&key[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t r = __hip_atomic_load(&best[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (v) key[t] = v | r;
    }
}

// Head-to-head selection (the per-head variant the paper compares with, Sec. 3.2 and the
// generalization figure): head h of sequence b keeps ITS OWN first K-W ranked picks plus the window.
// One workgroup per (head, sequence): the picks (distinct positions) are set in an LDS bitmap over
// the candidate positions and emitted in ascending order like the unified set.
// idx_head [B][H][budget]; cnt[b] = min(K, L_b) is the same for every head.
__global__ __launch_bounds__(SEL_THREADS) void per_head_rho_kernel(const int32_t* __restrict__ rho_head,
                                                                    const int32_t* __restrict__ seq_lens,
                                                                    int32_t* __restrict__ idx_head,
                                                                    int32_t* __restrict__ cnt, int H, int k,
                                                                    int budget, int window, int n_sink) {
    extern __shared__ uint32_t bits[];                // ceil(Lc / 32) words
    __shared__ int scratch[SEL_WAVES + 1];
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int L = seq_lens[b];
    int32_t* __restrict__ out = idx_head + ((int64_t)b * H + h) * budget;
    if (L <= budget) {
        for (int t = tid; t < L; t += SEL_THREADS) out[t] = t;
        if (tid == 0 && h == 0) cnt[b] = L;
        return;
    }
    const int Lc = L - window;
    const int k_eff = k < Lc - n_sink ? k : Lc - n_sink;
    const int n_hist = min(budget - window - n_sink, k_eff);   // = K - W - n_sink: k is at least that, and so is Lc - n_sink
    const int n_words = (Lc + 31) >> 5;
    for (int i = tid; i < n_words; i += SEL_THREADS) bits[i] = 0u;
    __syncthreads();
    const int32_t* __restrict__ rho = rho_head + (int64_t)b * k * H + h;   // rank j at rho[j * H]
    for (int j = tid; j < n_hist; j += SEL_THREADS) {
        const int t = rho[(int64_t)j * H];
        if ((uint32_t)t < (uint32_t)Lc) atomicOr(&bits[t >> 5], 1u << (t & 31));
    }
    __syncthreads();
    const int n_take = n_hist + emit_sinks_and_set(bits, n_words, n_sink, n_hist + n_sink, scratch, out);
    for (int j = tid; j < window; j += SEL_THREADS) out[n_take + j] = L - window + j;
    if (tid == 0 && h == 0) cnt[b] = n_take + window;
}

// ---------------------------------------------------------------- attention (split-K flash-decode)
//
// grid (n_splits, G, B), 256 threads.  A workgroup owns a contiguous run of the
// sequence's token list (all tokens, or rho) for one KV head; the GQ query heads of
// that group sit in LDS as bf16.  A 256-byte K or V row is read by 16 lanes with one
// 16-byte load each; a wave therefore covers 4 rows per load instruction and TI*4
// rows per iteration.  The wave parks its K rows in LDS and re-reads them one row per
// lane, which is the operand layout of the 4x4x4 bf16 MFMA: 32 instructions give every
// lane the scores of its token for four heads.  Softmax is the usual running (max, sum)
// rescale per iteration with one exp per (token, head); the numerators go back through
// LDS to the lanes that hold that token's V row, and P.V accumulates 8 columns per lane.
// The four waves are merged through LDS into one partial (m, l, acc[128]) per
// head.  With one split that is the result and is written as bf16; otherwise the
// partial goes to the workspace and attn_reduce_kernel merges the splits.  (A merge
// inside this kernel by the last workgroup to arrive was measured and is slower: its
// device-coherent reads of the other workgroups' partials run at a few GB/s.)

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// max over the 16 lanes of a DPP row; every lane of the row gets the result
__device__ __forceinline__ float row_max16(float v) {
    v = fmaxf(v, dpp_move<0xB1>(v));
    v = fmaxf(v, dpp_move<0x4E>(v));
    v = fmaxf(v, dpp_move<0x141>(v));
    v = fmaxf(v, dpp_move<0x140>(v));
    return v;
}

// sum over the 16 lanes of a DPP row; every lane of the row gets the result
__device__ __forceinline__ float row_sum16(float v) {
    v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);   // row_half_mirror
    v += dpp_move<0x140>(v);   // row_mirror
    return v;
}

constexpr int ATTN_THREADS = 256;
constexpr int ATTN_WAVES = 4;
// Longest run of tokens a workgroup of the scoring variant may own: its scores wait in LDS (32 KB)
// until the run is done.
constexpr int ATTN_SCORE_CHUNK_CAP = 2048;
constexpr int ATTN_SCORE_CHUNK_CAP_G8 = 1024;

// Workgroup `split` of a (sequence, KV head) owns tokens [split*chunk, split*chunk + chunk) of
// the token list; a list of n tokens keeps ceil(n / chunk) workgroups busy (at least one) and
// the others leave at once, so short sequences of a ragged batch cost nothing.
__host__ __device__ inline int attn_active_splits(int n, int chunk) {
    const int a = (n + chunk - 1) / chunk;
    return a < 1 ? 1 : a;
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// V_PERMLANE32_SWAP / V_PERMLANE16_SWAP exchange halves (rows 2,3 of a with rows 0,1 of b) or
// odd/even 16-lane rows (rows 1,3 of a with rows 0,2 of b) of two registers.  Adding the two
// results folds a and b over that lane bit at once: the lanes whose bit is 0 end up with the
// sum of a, the others with the sum of b.
__device__ __forceinline__ float fold_halves(float a, float b) {
    const auto s = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(s[0]) + __uint_as_float(s[1]);
}
__device__ __forceinline__ float fold_rows(float a, float b) {
    const auto s = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(s[0]) + __uint_as_float(s[1]);
}
// max of a lane's value and the one 16 (32) lanes away, in every lane
__device__ __forceinline__ float max_with_row_neighbour(float v) {
    const auto s = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(s[0]), __uint_as_float(s[1]));
}
__device__ __forceinline__ float max_with_other_half(float v) {
    const auto s = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(s[0]), __uint_as_float(s[1]));
}
__device__ __forceinline__ float lane_value(float v, int lane) {
    return __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), lane));
}

__device__ __forceinline__ int wave_base_of(unsigned tid) { return (int)(tid >> 6); }

// LDS written by some lanes of a wave and read by others of the same wave: a wave's LDS
// accesses are performed in program order, so only the compiler has to be kept from
// reordering them.
// Workgroup barrier for data exchanged through LDS only: waits for this wave's LDS operations, not for
// its outstanding global loads (which a full __syncthreads() would drain first).
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// SCORE (selection layer, all tokens): the scores of the candidate range [0, L - window) are also
// written to P[b][head][t] (row stride ldp), so the layer's K is read once for both (Alg. 1 computes
// the layer's output and P from the same K).  q.k then runs as the k = 1 MFMA chain -- the pinned
// left-to-right binary32 sum (see "scoring" above) -- instead of the k = 4 bf16 MFMA, and the softmax
// uses those same values.
//
// lse (optional): log2 of each head's softmax denominator, M + log2(l) with scores scaled by
// sm_scale * log2(e); written by whoever writes the head's output (this kernel or the reduce).
//
// PER_HEAD (sparse, GQ = 1): every query head attends its own token list idx[b][head][0 .. cnt[b])
// -- the head-to-head selection the paper compares with (Sec. 3.2, the generalization figure) --
// so a workgroup serves one query head, blockIdx.y counts query heads (G of them) and head y reads
// KV head y >> hshift.  Nothing is shared inside a GQA group: each head fetches its own rows.
//
// ONLY_SCORES (a form of SCORE): the scores and nothing else -- no V rows, no softmax, no output.  This
// is cusa_select's scoring pass and the second chance of the filtered selection: with flt.fail set, only
// the groups that have a flagged head are scored, and nothing at all when the counter *flt.n_failed is 0.
template <int GQ, int TI, bool SPARSE, bool PAGED, bool SCORE = false, bool PER_HEAD = false, bool FILTER = false,
          bool ONLY_SCORES = false>
__global__ __launch_bounds__(ATTN_THREADS, 2) void attn_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ cnt, const int32_t* __restrict__ seq_lens,
    const uint16_t* __restrict__ q, int budget, int n_splits, int chunk, int G, float scale_log2e,
    float* __restrict__ part_acc, float* __restrict__ part_ml, uint16_t* __restrict__ out, float* __restrict__ lse,
    float* __restrict__ P, int64_t ldp, int window, int hshift, FilterState flt, KvView kv) {
    static_assert(!(SCORE && SPARSE), "scores are emitted by the pass over all tokens");
    static_assert(!FILTER || SCORE, "the filter is a form of the scoring variant");
    static_assert(!ONLY_SCORES || (SCORE && !FILTER), "scores only: the dense scoring variant without the attention");
    static_assert(!PER_HEAD || (SPARSE && GQ == 1), "per-head token lists: one query head per workgroup");
    constexpr int TILE = TI * 4;                      // tokens per wave iteration (<= 64)
    constexpr int WG_TILE = TILE * ATTN_WAVES;
    constexpr int SETS = (GQ + 3) / 4;                // groups of 4 heads, one MFMA accumulator each
    constexpr int QSB = 136;                          // padded head stride of q in LDS (bf16 elements)
    // A wave's K tile buffer (TILE rows of 256 bytes) also carries its partial accumulators
    // (GQ x 128 floats) into the final merge.
    // The scoring variant parks a tile's K rows in two halves of 64 columns, one after the other (its
    // product chain walks the columns in order anyway), which leaves LDS for the scores of the
    // workgroup's whole run (pstage below).
    constexpr int KSLOTS = SCORE ? 8 : 16;            // 16-byte slots of a K row held in LDS at a time
    constexpr int WAVE_LDS = TILE * KSLOTS * 16;      // bytes of a wave's tile buffer
    static_assert(WAVE_LDS >= GQ * D * 4, "the K tile buffer must hold a wave's partial accumulators");
    __shared__ __attribute__((aligned(16))) unsigned char smem_raw[ATTN_WAVES * WAVE_LDS];
    // this wave's K rows: chunk c of row r at slot c ^ (r & 7) (a swizzle over all sixteen slots, c ^ (r & 15),
    // removes the remaining two-way bank conflicts and was measured: no faster); scoring variant: chunk c
    // (of the half) at slot c ^ ((r >> 1) & 7)
    u32x4* const ktile = reinterpret_cast<u32x4*>(smem_raw) + wave_base_of(threadIdx.x) * (TILE * KSLOTS);
    __shared__ float sm_m[ATTN_WAVES][GQ];
    __shared__ float sm_l[ATTN_WAVES][GQ];
    // A wave's softmax numerators take the place of its K rows once those are scored.  They are
    // stored as bf16 in the operand order of the P.V products below: [row group r][four row loads ig]
    // [set][head][member k], so that the weights of one head for the four tokens a lane multiplies
    // together (rows 4ig .. 4ig+3 of its row group) are one 8-byte word.
    static_assert(TI % 4 == 0 && WAVE_LDS >= TI * SETS * 32, "the numerators must fit the K tile buffer");
    __bf16* const pbuf16 = reinterpret_cast<__bf16*>(ktile);
    // q in LDS: a private bf16 copy per wave, or -- in the scoring variant, whose product chain takes
    // binary32 operands -- one binary32 copy for the workgroup (every wave writes all of it with the
    // same values, so a wave depends on its own writes only and no workgroup barrier is needed).
    constexpr int QSF = 132;                          // padded head stride of the binary32 copy (floats)
    __shared__ __attribute__((aligned(16))) uint16_t qlds_all[SCORE ? 1 : ATTN_WAVES][SCORE ? 8 : SETS * 4 * QSB];
    __shared__ __attribute__((aligned(16))) float qf32[SCORE ? SETS * 4 * QSF : 4];
    // scoring variant: the scores of the workgroup's run (of its last STAGE_IT iterations, should a run be
    // longer: the host caps it at STAGE_TOK tokens), [head][token], on their way to P
    constexpr int STAGE_TOK = GQ >= 8 ? ATTN_SCORE_CHUNK_CAP_G8 : ATTN_SCORE_CHUNK_CAP;   // 32 KB at groups of 4 and 8
    constexpr int STAGE_IT = STAGE_TOK / WG_TILE;
    __shared__ __attribute__((aligned(16))) float pstage[SCORE ? GQ * STAGE_TOK : 4];
    // Filtered form of the scoring variant (FILTER; see sample_threshold_kernel): instead of every score,
    // the buffer takes the (score key, position) composites of the candidates at or above the head's
    // threshold, compacted per head -- STAGE_CAND of them per head at most, or the head is flagged.
    constexpr int STAGE_CAND = STAGE_TOK / 2;         // composites are twice a score's size
    uint64_t* const cstage = reinterpret_cast<uint64_t*>(pstage);
    __shared__ int cand_n[SCORE ? GQ : 1], cand_base[SCORE ? GQ : 1];
    __shared__ uint32_t thr_lds[SCORE ? GQ : 1];
    constexpr bool filtered = FILTER;
    // Workgroups go to the 8 XCDs round-robin in launch order (blockIdx.x fastest).  With ragged
    // lengths the low splits are the busy ones; starting each (sequence, KV head) at a different
    // block spreads them evenly over the XCDs instead of loading the first ones.
    if constexpr (ONLY_SCORES) {                         // the second chance with nothing flagged: out before any other load is asked for
        if (flt.fail && *flt.n_failed == 0) return;
    }
    const int gy = blockIdx.y, b = blockIdx.z, H = G * GQ;
    const int kvh = PER_HEAD ? gy >> hshift : gy;
    const int split = (int)((blockIdx.x + gy + G * b) % (unsigned)n_splits);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane >> 4, c = lane & 15;
    const int begin = split * chunk;
    const int32_t* __restrict__ my_idx = idx + (PER_HEAD ? (int64_t)b * G + gy : (int64_t)b) * budget;
    const int64_t head0 = (int64_t)b * H + gy * GQ;      // first query head of this group
    // Address pipeline.  A row's address is the end of a chain of dependent memory reads: the token
    // list (sparse), then the block table (paged), then the row.  The list entries (posA) of a tile
    // are requested one tile ahead, and so are the pool pages (pgA) of a pass over all tokens, whose
    // positions are arithmetic.  The first entries are fetched here, before the token count is
    // known: a row of idx has `budget` entries, so a read clamped to budget - 1 stays inside it, and
    // entries past the count are masked below like every row past the run's end.
    const int tile0 = begin + wave * TILE;
    int posA[TI], pgA[TI];
    auto idx_load = [&](int t_, int* p) {
        if (SPARSE) {
#pragma unroll
            for (int i = 0; i < TI; ++i) p[i] = my_idx[min(t_ + i * 4 + r, budget - 1)];
        }
    };
    idx_load(tile0, posA);

    // Every wave keeps its own bf16 copy of q in LDS (no workgroup barrier on the way in): lane l
    // fetches 16 bytes of head l / 16 per set now and parks them once the first tile's loads are
    // under way.  Heads beyond GQ score zero.
    uint16_t* const qlds = qlds_all[SCORE ? 0 : wave];
    u32x4 qv[SETS];
#pragma unroll
    for (int s = 0; s < SETS; ++s) {
        const int h = s * 4 + r;
        qv[s] = *reinterpret_cast<const u32x4*>(q + (head0 + (h < GQ ? h : 0)) * D + c * 8);
        if (h >= GQ) qv[s] = u32x4{0u, 0u, 0u, 0u};
    }
    bool q_parked = false;
    const int L = seq_lens[b];
    if constexpr (ONLY_SCORES) {
        if (L <= budget) return;                         // rho is every token: nothing is scored
        if (flt.fail) {                                  // the second chance: flagged heads' groups only
            int any = 0;
#pragma unroll
            for (int h = 0; h < GQ; ++h) any |= flt.fail[head0 + h];
            if (!any) return;
        }
    }
    const int n = SPARSE ? min(cnt[b], budget) : ONLY_SCORES ? L - window : L;   // scores only: the candidate range
    // Everything the first tile's addresses depend on is requested above and has to be here
    // before the first branch; otherwise the compiler sinks each load behind the branch that
    // precedes its first use and the kernel starts with a chain of dependent memory round trips.
    asm volatile("" ::"s"(L), "s"(n), "s"(kv.k), "s"(H));
    if (SPARSE) {
#pragma unroll
        for (int i = 0; i < TI; ++i) asm volatile("" ::"v"(posA[i]));
    }
    if (split > 0 && begin >= n) return;                 // split >= attn_active_splits(n, chunk)
    const int end = (begin + chunk < n) ? begin + chunk : n;

    // Scores come from V_MFMA_F32_4X4X4_16B_BF16: per lane four bf16 of q (head = lane % 4)
    // and four of K (the lane's token); after 32 instructions lane t holds q_h . k_t for the
    // heads of each set.  Lane t scores token t % TILE of the tile.
    const int tl = lane % TILE;
    const bool owner = lane < TILE;                   // lanes beyond TILE repeat a token; they add nothing to l
    // token tl is row load (tl / 4) of row group (tl % 4): where its numerators go (bf16 elements)
    const int p_slot = (((tl & 3) * (TI / 4) + (tl >> 4)) * SETS * 4) * 4 + ((tl >> 2) & 3);
    float m[GQ], l[GQ];
    f32x4 acc[SETS][8];                               // [set][column e of the lane's 8]: the four heads of the set
#pragma unroll
    for (int h = 0; h < GQ; ++h) {
        m[h] = -INFINITY;
        l[h] = 0.0f;
    }
#pragma unroll
    for (int s = 0; s < SETS; ++s)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[s][e] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // Rows past the end of the run read some token of the sequence (a valid row) so that all
    // loads are unconditional and issue back to back; their scores are masked below.
    // The next tile's K rows are requested as soon as this tile's are parked in LDS, i.e. before
    // this tile's arithmetic (not in the scoring variant, whose 64-token tiles leave no registers
    // for it; there the rows are requested at the top of the tile's own iteration).
    constexpr bool PREFETCH = !SCORE;
    // The scoring variant of a group of 8 has no registers for K and V rows at once (64 each at 64-token
    // tiles, beside 64 accumulators): its V rows are requested once the K rows are parked in LDS.
    constexpr bool V_LATE = !ONLY_SCORES && SCORE && (GQ >= 8 || (FILTER && GQ >= 4));
    u32x4 kreg[TI], vreg[TI];
    int64_t off[TI];
    // a valid position for row load i of the tile that starts at list entry t_ (an index outside the
    // sequence is a caller error; never fault on it)
    auto tile_pos = [&](int t_, int i, const int* p) {
        return SPARSE ? min(max(p[i], 0), L - 1) : min(t_ + i * 4 + r, end - 1);
    };
    // Pool pages of the tile's rows.  A pass over all tokens walks the table in order: tiles start at
    // multiples of 16 tokens, so row loads 4ig .. 4ig+3 of every lane fall into one page, entry
    // (t_ / 16 + ig) of the table (rows clamped to the run's last token: that token's page), and only
    // TI / 4 wave-uniform entries are fetched (g[ig]).
    auto page_load = [&](int t_, const int* p, int* g) {
        if constexpr (PAGED && SPARSE) {
#pragma unroll
            for (int i = 0; i < TI; ++i) g[i] = kv.bt[(int64_t)b * kv.max_pages + (tile_pos(t_, i, p) >> 4)];
        } else if constexpr (PAGED) {
#pragma unroll
            for (int ig = 0; ig < TI / 4; ++ig)
                g[ig] = kv.bt[(int64_t)b * kv.max_pages + min((t_ >> 4) + ig, (end - 1) >> 4)];
        }
    };
    auto make_off = [&](int t_, const int* p, int* g) {
        if constexpr (SPARSE && PAGED) page_load(t_, p, g);
#pragma unroll
        for (int i = 0; i < TI; ++i) {
            const int pos = tile_pos(t_, i, p);
            if (PAGED) off[i] = (((int64_t)g[SPARSE ? i : i >> 2] * kv.G + kvh) * PAGE + (pos & (PAGE - 1))) * D + c * 8;
            else off[i] = (int64_t)b * kv.sb + (int64_t)kvh * kv.sh + (int64_t)pos * kv.st + c * 8;
        }
    };
    auto request_k = [&]() {
#pragma unroll
        for (int i = 0; i < TI; ++i) kreg[i] = row_load<PER_HEAD>(kv.k + off[i]);
    };
    // After the rows of the tile at t_ have been requested: the lookups for the tile after it.
    auto advance = [&](int t_) {
        idx_load(t_ + WG_TILE, posA);
        if constexpr (!SPARSE) page_load(t_ + WG_TILE, posA, pgA);   // sparse: looked up where the offsets are made
    };
    if constexpr (!SPARSE) page_load(tile0, posA, pgA);
    if (PREFETCH && tile0 < end) {
        make_off(tile0, posA, pgA);
        request_k();
        advance(tile0);
    }
    // Scoring variant: the scores go to P through a staging buffer in LDS that the whole workgroup
    // writes out in one burst.  A few per cent of small writes scattered
    // through a streaming read cost this machine a sixth of its read rate; the same bytes written in
    // workgroup-sized bursts cost a third of that (measured with plain read / write kernels).  The
    // burst is issued at the end of the workgroup's run (the host caps a run at STAGE_TOK tokens; a
    // longer one would take a burst every STAGE_IT iterations, before the next tile's rows are
    // requested).  Measured on the selection pass, us without stores / scattered stores / bursts:
    // c3 95 / 106 / 99, c4 100 / 121 / 106, c5 867 / 1036 / 1008.  Giving every workgroup its own
    // burst phase, so that the chip's bursts do not coincide, was measured too and is slower.
    auto flush_scores = [&](int g0, int n_tok) {       // staged tokens [g0, g0 + n_tok) of this workgroup's run
        if constexpr (SCORE) {
            const int lim = min(end, L - window);      // candidates only; L <= budget: rho is every token, nothing is scored
            if (L > budget && g0 < lim) {
                const int quads = n_tok >> 2;
                for (int i = tid; i < GQ * quads; i += ATTN_THREADS) {
                    const int h = i / quads, w4 = (i - h * quads) * 4, t = g0 + w4;
                    const f32x4 v = *reinterpret_cast<const f32x4*>(&pstage[h * STAGE_TOK + w4]);
                    float* const dst = &P[(head0 + h) * ldp + t];
                    if (t + 3 < lim) {
                        __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(dst));
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (t + e < lim) dst[e] = v[e];
                    }
                }
            }
        }
    };
    // filtered form: the staged candidates of every head go to the head's list in memory, one reservation
    // per head and workgroup.  The reservation is a device-scope atomic whose answer takes microseconds:
    // reserve_candidates asks (thread h for head h; returns the answer, -1 if there is nothing to copy),
    // copy_candidates uses the answer and empties the buffer -- at the end of a run the workgroup merges
    // and writes its attention partials in between.  Both are called by the whole workgroup.
    auto reserve_candidates = [&]() -> int {
        int base = -1;
        if constexpr (SCORE) {
            lds_barrier();                               // every wave's candidates are staged
            if (tid < GQ) {
                const int n_h = cand_n[tid];
                if (n_h > STAGE_CAND) flag_failed(flt, head0 + tid);   // more candidates than the buffer held: some are lost
                else if (n_h > 0) base = atomicAdd(&flt.cand_cnt[head0 + tid], n_h);
            }
        }
        return base;
    };
    auto copy_candidates = [&](int base) {
        if constexpr (SCORE) {
            if (tid < GQ) {
                if (base >= 0 && base + cand_n[tid] > flt.cap) {   // the head's list is full (the count stays above cap: the ranking sees it too)
                    flag_failed(flt, head0 + tid);
                    base = -1;
                }
                cand_base[tid] = base;
            }
            lds_barrier();
#pragma unroll
            for (int h = 0; h < GQ; ++h) {
                const int n_h = cand_n[h], base_h = cand_base[h];
                if (base_h >= 0) {
                    uint64_t* const dst = flt.cand + (head0 + h) * flt.cap + base_h;
                    for (int i = tid; i < n_h; i += ATTN_THREADS) __builtin_nontemporal_store(cstage[h * STAGE_CAND + i], &dst[i]);
                }
            }
            lds_barrier();                               // all read, before the counters start again
            if (tid < GQ) cand_n[tid] = 0;
            lds_barrier();
        }
    };
    if constexpr (FILTER) {                              // the heads' thresholds wait in LDS, not in registers
        if (tid < GQ) {
            thr_lds[tid] = flt.thr[head0 + tid];
            cand_n[tid] = 0;
        }
        lds_barrier();
    }
    int t_opaque = 0;                                    // always zero, unknown to the compiler
    int it_staged = 0;                                   // first iteration whose scores are still in the staging buffer
    int it = 0;                                          // iterations of the workgroup so far
    for (int w0 = begin; w0 < end; w0 += WG_TILE, ++it) {
        const int t0 = w0 + wave * TILE;
        // Only the scoring variant has workgroup barriers inside the loop; there a wave whose tile lies
        // past the run's end still takes part in them.
        const bool active = t0 < end;
        // workgroup-uniform; the buffer holds STAGE_IT iterations at most
        const bool burst_due = SCORE && it - it_staged == STAGE_IT;
        if (burst_due) {
            if (filtered) {
                copy_candidates(reserve_candidates());
            } else {
                lds_barrier();                           // every wave's scores since the last burst are staged
                flush_scores(begin + it_staged * WG_TILE, (it - it_staged) * WG_TILE);
                lds_barrier();                           // ... and read, before the buffer is written again
            }
            it_staged = it;
        }
        if (!active) {
            if constexpr (!SCORE) break;
            continue;
        }
        if constexpr (!PREFETCH) {
            make_off(t0, posA, pgA);
            // K rows first: they are needed first (parked in LDS and scored), and loads return in
            // order, so the scores are under way while the V rows are still arriving.
            request_k();
        }
        if constexpr (!V_LATE && !ONLY_SCORES) {
#pragma unroll
            for (int i = 0; i < TI; ++i) vreg[i] = row_load<PER_HEAD>(kv.v + off[i]);
        }
        if constexpr (!PREFETCH && !V_LATE) advance(t0);
        __builtin_amdgcn_sched_barrier(0);               // keep every load above the arithmetic
        if (!q_parked) {
#pragma unroll
            for (int s = 0; s < SETS; ++s) {
                if constexpr (SCORE) {
                    float qf[8];
                    unpack8(make_uint4(qv[s].x, qv[s].y, qv[s].z, qv[s].w), qf);
                    float* const dst = &qf32[(s * 4 + r) * QSF + c * 8];
                    *reinterpret_cast<f32x4*>(dst) = f32x4{qf[0], qf[1], qf[2], qf[3]};
                    *reinterpret_cast<f32x4*>(dst + 4) = f32x4{qf[4], qf[5], qf[6], qf[7]};
                } else {
                    *reinterpret_cast<u32x4*>(&qlds[(s * 4 + r) * QSB + c * 8]) = qv[s];
                }
            }
            q_parked = true;
        }
        if constexpr (!SCORE) {
#pragma unroll
            for (int i = 0; i < TI; ++i) {
                const int row = i * 4 + r;
                ktile[row * 16 + (c ^ (row & 7))] = kreg[i];
            }
            wave_lds_sync();
        }
        if (PREFETCH && t0 + WG_TILE < end) {
            make_off(t0 + WG_TILE, posA, pgA);
            request_k();
            advance(t0 + WG_TILE);
            __builtin_amdgcn_sched_barrier(0);
        }

        f32x4 sc[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) sc[s] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if constexpr (SCORE) {
            // columns 0..63, then 64..127: the lanes holding that half of a row park it, every lane then
            // walks its own token's 64 columns in order
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                if (half) wave_lds_sync();            // the first half has been read
                if ((c >> 3) == half) {
#pragma unroll
                    for (int i = 0; i < TI; ++i) {
                        const int row = i * 4 + r;
                        ktile[row * 8 + ((c & 7) ^ ((row >> 1) & 7))] = kreg[i];
                    }
                }
                wave_lds_sync();
                if constexpr (V_LATE) {
                    if (half) {                       // the K rows' registers are free now
                        // the offsets are made again rather than kept in 32 registers since the K requests;
                        // the compiler must not see that they are the same values, or it keeps them
                        asm volatile("" : "+v"(t_opaque));
                        make_off(t0 + t_opaque, posA, pgA);
#pragma unroll
                        for (int i = 0; i < TI; ++i) vreg[i] = row_load<PER_HEAD>(kv.v + off[i]);
                        advance(t0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
#pragma unroll
                for (int c8 = 0; c8 < 8; ++c8) {
                    const int cc = half * 8 + c8;
                    const u32x4 kw = ktile[tl * 8 + (c8 ^ ((tl >> 1) & 7))];
                    float kf[8];
                    unpack8(make_uint4(kw.x, kw.y, kw.z, kw.w), kf);
                    float qf[SETS][8];
#pragma unroll
                    for (int s = 0; s < SETS; ++s) {
                        const float* const src = &qf32[(s * 4 + (lane & 3)) * QSF + cc * 8];
                        const f32x4 qa = *reinterpret_cast<const f32x4*>(src), qb = *reinterpret_cast<const f32x4*>(src + 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            qf[s][e] = qa[e];
                            qf[s][4 + e] = qb[e];
                        }
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e)
#pragma unroll
                        for (int s = 0; s < SETS; ++s)
                            sc[s] = __builtin_amdgcn_mfma_f32_4x4x1f32(qf[s][e], kf[e], sc[s], 0, 0, 0);
                }
            }
            if (filtered) {
                const int t = t0 + tl;
                const bool is_cand = lane < TILE && t >= flt.n_sink && t < min(end, L - window);
#pragma unroll
                for (int h = 0; h < GQ; ++h) {
                    const uint32_t key = score_key(sc[h >> 2][h & 3]), thr = thr_lds[h];
                    const bool keep = is_cand && thr != 0xffffffffu && key >= thr;
                    const uint64_t kept = __ballot(keep);
                    if (kept) {                          // wave-uniform: one reservation per wave and head
                        int base = 0;
                        if (lane == 0) base = atomicAdd(&cand_n[h], __popcll(kept));
                        base = __builtin_amdgcn_readfirstlane(base);
                        const int slot = base + mbcnt(kept);
                        if (keep && slot < STAGE_CAND) cstage[h * STAGE_CAND + slot] = ((uint64_t)key << 32) | (uint32_t)~(uint32_t)t;
                    }
                    asm volatile("" ::: "memory");       // one head at a time: nothing of the next is fetched early
                }
            } else if (lane < TILE) {
#pragma unroll
                for (int h = 0; h < GQ; ++h) pstage[h * STAGE_TOK + (it - it_staged) * WG_TILE + wave * TILE + tl] = sc[h >> 2][h & 3];
            }
        } else {
#pragma unroll
            for (int cc = 0; cc < 16; ++cc) {
                const u32x4 kw = ktile[tl * 16 + (cc ^ (tl & 7))];
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const uint2 kb = half == 0 ? make_uint2(kw.x, kw.y) : make_uint2(kw.z, kw.w);
                    const s16x4 bq = __builtin_bit_cast(s16x4, kb);
#pragma unroll
                    for (int s = 0; s < SETS; ++s) {
                        const s16x4 aq = *reinterpret_cast<const s16x4*>(&qlds[(s * 4 + (lane & 3)) * QSB + cc * 8 + half * 4]);
                        sc[s] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(aq, bq, sc[s], 0, 0, 0);
                    }
                }
            }
        }
        if constexpr (ONLY_SCORES) {
            wave_lds_sync();                              // the tile buffer is rewritten next iteration
            continue;
        }
        const bool valid = t0 + tl < end;
        float corr[GQ];
#pragma unroll
        for (int h = 0; h < GQ; ++h) {
            const float z = valid ? sc[h >> 2][h & 3] * scale_log2e : -INFINITY;
            float mt = row_max16(z);                  // lanes TILE apart hold the same token
            if (TILE > 16) mt = max_with_row_neighbour(mt);
            if (TILE > 32) mt = max_with_other_half(mt);
            const float m_new = fmaxf(m[h], mt);      // finite: token t0 of this tile is valid
            corr[h] = exp2f(m[h] - m_new);
            m[h] = m_new;
            // the weight enters numerator and denominator as the same bf16 value
            const __bf16 pb = (__bf16)exp2f(z - m_new);
            pbuf16[p_slot + h * 4] = pb;
            l[h] = l[h] * corr[h] + (owner ? (float)pb : 0.0f);
        }
#pragma unroll
        for (int s = 0; s < SETS; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                f32x4 a = acc[s][e];
#pragma unroll
                for (int hh = 0; hh < 4; ++hh)
                    if (s * 4 + hh < GQ) a[hh] *= corr[s * 4 + hh];
                acc[s][e] = a;
            }
        wave_lds_sync();
        // P.V on the matrix cores, four tokens per instruction.  A lane holds columns 8c .. 8c+7 of the
        // rows i*4 + r; the same column of four of its rows (4ig .. 4ig+3) is gathered into one bf16
        // quadruple (V_PERM_B32), which is this lane's column of the 4 x 4 B operand; the A operand is
        // the four tokens' weights of head (lane % 4).  One V_MFMA_F32_4X4X4_16B_BF16 then adds, for the
        // lane's column, the four tokens' products of four heads to the binary32 accumulator.
#pragma unroll
        for (int ig = 0; ig < TI / 4; ++ig) {
            s16x4 pa[SETS];
#pragma unroll
            for (int s = 0; s < SETS; ++s)
                pa[s] = *reinterpret_cast<const s16x4*>(pbuf16 + (((r * (TI / 4) + ig) * SETS + s) * 4 + (lane & 3)) * 4);
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) {
                const uint32_t r0 = vreg[4 * ig][w2], r1 = vreg[4 * ig + 1][w2], r2 = vreg[4 * ig + 2][w2], r3 = vreg[4 * ig + 3][w2];
                const uint2 lo = make_uint2(__builtin_amdgcn_perm(r1, r0, 0x05040100u), __builtin_amdgcn_perm(r3, r2, 0x05040100u));
                const uint2 hi = make_uint2(__builtin_amdgcn_perm(r1, r0, 0x07060302u), __builtin_amdgcn_perm(r3, r2, 0x07060302u));
                const s16x4 vlo = __builtin_bit_cast(s16x4, lo), vhi = __builtin_bit_cast(s16x4, hi);
#pragma unroll
                for (int s = 0; s < SETS; ++s) {
                    acc[s][2 * w2] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(pa[s], vlo, acc[s][2 * w2], 0, 0, 0);
                    acc[s][2 * w2 + 1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(pa[s], vhi, acc[s][2 * w2 + 1], 0, 0, 0);
                }
            }
        }
        wave_lds_sync();                              // the tile buffers are rewritten next iteration
    }
    int cand_reserved = -1;
    if constexpr (SCORE) {
        if (filtered) {
            cand_reserved = reserve_candidates();        // used after the merge below
        } else if (it > it_staged) {                   // the iterations staged since the last burst
            lds_barrier();
            flush_scores(begin + it_staged * WG_TILE, (it - it_staged) * WG_TILE);
        }
    }
    if constexpr (ONLY_SCORES) return;
    // Merge.  Inside the wave the four row groups are folded with lane swaps: of the N = 8 GQ
    // values of a lane, two folds leave N / 4 complete sums, those with flat index (head * 8 +
    // column) v0 .. v0 + N/4 - 1 where v0 depends on the row group.  The wave parks them in its
    // own tile buffer and the four waves meet in LDS.
    constexpr int N = GQ * 8;
    float* const wsum = reinterpret_cast<float*>(ktile);           // [GQ][D] of this wave
    {
        float y[N / 2], z[N / 4];
#pragma unroll
        for (int v = 0; v < N / 2; ++v) {
            constexpr int HALF = N / 2;                  // flat index = head * 8 + column
            y[v] = fold_halves(acc[v >> 5][v & 7][(v >> 3) & 3], acc[(v + HALF) >> 5][(v + HALF) & 7][((v + HALF) >> 3) & 3]);
        }
#pragma unroll
        for (int v = 0; v < N / 4; ++v) z[v] = fold_rows(y[v], y[v + N / 4]);
        const int v0 = (r >> 1) * (N / 2) + (r & 1) * (N / 4);
        if (N / 4 >= 4) {
#pragma unroll
            for (int j = 0; j < N / 16; ++j) {
                const int v = v0 + 4 * j;
                *reinterpret_cast<f32x4*>(&wsum[(v >> 3) * D + c * 8 + (v & 7)]) = f32x4{z[4 * j], z[4 * j + 1], z[4 * j + 2], z[4 * j + 3]};
            }
        } else {
            *reinterpret_cast<f32x2*>(&wsum[c * 8 + v0]) = f32x2{z[0], z[1]};
        }
    }
#pragma unroll
    for (int h = 0; h < GQ; ++h) {
        float ls = row_sum16(l[h]);                      // only lanes below TILE carry a sum
        float lt = lane_value(ls, 0);
        if (TILE > 16) lt += lane_value(ls, 16);
        if (TILE > 32) lt += lane_value(ls, 32) + lane_value(ls, 48);
        if (lane == 0) {
            sm_m[wave][h] = m[h];
            sm_l[wave][h] = lt;
        }
    }
    __syncthreads();
    const float* const sums = reinterpret_cast<const float*>(smem_raw);
    for (int o = tid; o < GQ * D; o += ATTN_THREADS) {
        const int h = o / D, col = o % D;
        float M = sm_m[0][h];
#pragma unroll
        for (int wv = 1; wv < ATTN_WAVES; ++wv) M = fmaxf(M, sm_m[wv][h]);
        float A = 0.0f, Ls = 0.0f;
#pragma unroll
        for (int wv = 0; wv < ATTN_WAVES; ++wv) {
            const float mw = sm_m[wv][h];
            const float f = (mw == -INFINITY) ? 0.0f : exp2f(mw - M);
            A = __builtin_fmaf(sums[wv * (WAVE_LDS / 4) + o], f, A);
            Ls = __builtin_fmaf(sm_l[wv][h], f, Ls);
        }
        if (n <= chunk) {                                // this workgroup saw the whole token list
            out[(head0 + h) * D + col] = f32_to_bf16_rne(Ls > 0.0f ? A / Ls : 0.0f);
            if (lse && col == 0) lse[head0 + h] = M + log2f(Ls);
        } else {
            const int64_t p = (head0 + h) * n_splits + split;
            part_acc[p * D + col] = A;
            if (col == 0) {
                part_ml[p * 2] = M;
                part_ml[p * 2 + 1] = Ls;
            }
        }
    }
    if constexpr (FILTER) copy_candidates(cand_reserved);
}

// Merge of the split-K partials of sequences that kept more than one workgroup busy.
// grid (H, B), 256 threads: thread (c4, sr) owns output
// columns 4*c4 .. 4*c4+3 and folds the splits sr, sr+8, ... into a running (m, l, a[4])
// with 16-byte loads; the eight split-rows then meet in LDS and the result is written as bf16.
// n_tok[b] is the sequence's token count (seq_lens, or cnt clipped to the budget when sparse).
__global__ __launch_bounds__(256) void attn_reduce_kernel(const float* __restrict__ part_acc,
                                                           const float* __restrict__ part_ml,
                                                           uint16_t* __restrict__ out,
                                                           const int32_t* __restrict__ n_tok, int n_clip,
                                                           int stride_splits, int chunk, int H,
                                                           float* __restrict__ lse) {
    __shared__ float red_a[8][D];
    __shared__ float red_m[8], red_l[8];
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, c4 = tid & 31, sr = tid >> 5;
    const int64_t base = ((int64_t)b * H + h) * stride_splits;
    constexpr int U = 4;
    // The first batch of partials is requested before the token count is known (any of the
    // stride_splits slots may be read); what lies beyond the active splits is dropped by select,
    // never by a multiplication, because those slots hold whatever was there before.
    f32x4 va[U];
    f32x2 vml[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int sv = sr + 8 * u;
        const int64_t p = base + (sv < stride_splits ? sv : 0);
        va[u] = *reinterpret_cast<const f32x4*>(&part_acc[p * D + c4 * 4]);
        vml[u] = *reinterpret_cast<const f32x2*>(&part_ml[p * 2]);
    }
    const int n_splits = attn_active_splits(min(n_tok[b], n_clip), chunk);
    // keep the requests above the branch (the compiler would sink them behind it)
    asm volatile("" ::"s"(n_splits));
#pragma unroll
    for (int u = 0; u < U; ++u) asm volatile("" ::"v"(va[u]), "v"(vml[u]));
    if (n_splits <= 1) return;                           // the attention kernel wrote the result itself
    float mo = -INFINITY, lo = 0.0f;
    f32x4 ao = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int s0 = sr; s0 < n_splits; s0 += 8 * U) {
        if (s0 != sr) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int sv = s0 + 8 * u;
                const int64_t p = base + (sv < n_splits ? sv : s0);
                va[u] = *reinterpret_cast<const f32x4*>(&part_acc[p * D + c4 * 4]);
                vml[u] = *reinterpret_cast<const f32x2*>(&part_ml[p * 2]);
            }
        }
        float mb = mo;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (s0 + 8 * u < n_splits) mb = fmaxf(mb, vml[u].x);
        if (mb == -INFINITY) continue;                   // nothing but empty splits so far
        const float f0 = (mo == -INFINITY) ? 0.0f : exp2f(mo - mb);
        ao *= f0;
        lo *= f0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float mu = vml[u].x;
            const bool live = s0 + 8 * u < n_splits && mu != -INFINITY;
            const float f = live ? exp2f(mu - mb) : 0.0f;
            const f32x4 a = live ? va[u] : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            ao += a * f;
            lo = __builtin_fmaf(live ? vml[u].y : 0.0f, f, lo);
        }
        mo = mb;
    }
    *reinterpret_cast<f32x4*>(&red_a[sr][c4 * 4]) = ao;
    if (c4 == 0) {
        red_m[sr] = mo;
        red_l[sr] = lo;
    }
    __syncthreads();
    if (tid < D) {
        float M = red_m[0];
#pragma unroll
        for (int j = 1; j < 8; ++j) M = fmaxf(M, red_m[j]);
        float A = 0.0f, Ls = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float mj = red_m[j];
            const float f = (mj == -INFINITY) ? 0.0f : exp2f(mj - M);
            A = __builtin_fmaf(red_a[j][tid], f, A);
            Ls = __builtin_fmaf(red_l[j], f, Ls);
        }
        out[((int64_t)b * H + h) * D + tid] = f32_to_bf16_rne(Ls > 0.0f ? A / Ls : 0.0f);
        if (lse && tid == 0) lse[(int64_t)b * H + h] = M + log2f(Ls);
    }
}

// Streaming-read probe (benchmark support): every thread folds 16-byte loads of a plain buffer,
// eight in flight per lane, consecutive lanes on consecutive addresses.  What this kernel reaches
// is the practical ceiling of a read-only pass on the machine, to set beside the nominal HBM peak.
constexpr int PROBE_THREADS = 256;
constexpr int PROBE_UNROLL = 8;

__global__ __launch_bounds__(PROBE_THREADS) void probe_stream_read_kernel(const u32x4* __restrict__ src, int64_t n_vec,
                                                                           uint32_t* __restrict__ sink) {
    const int64_t stride = (int64_t)gridDim.x * PROBE_THREADS;
    u32x4 fold = {0u, 0u, 0u, 0u};
    int64_t i = (int64_t)blockIdx.x * PROBE_THREADS + threadIdx.x;
    for (; i + (PROBE_UNROLL - 1) * stride < n_vec; i += PROBE_UNROLL * stride) {
        u32x4 v[PROBE_UNROLL];
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL; ++u) v[u] = __builtin_nontemporal_load(&src[i + u * stride]);
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL; ++u) fold ^= v[u];
    }
    for (; i < n_vec; i += stride) fold ^= __builtin_nontemporal_load(&src[i]);
    const uint32_t f = fold.x ^ fold.y ^ fold.z ^ fold.w;
    if (f == 0x9e3779b9u) *sink = f;                 // keeps the loads alive; practically never taken
}

// Traffic probes (benchmark support): the memory system's rate for the access patterns of the attention
// kernels, without their arithmetic.  A workgroup of four waves walks chunks of 32 tiles; a wave reads a
// tile of 32 KB with 32 streaming loads of 16 bytes per lane in flight (what K and V of 64 tokens are), then
//   PATTERN 0: nothing else (a plain streaming read in this shape);
//   PATTERN 1: nothing else -- but the tile is 128 rows of 256 bytes gathered from a region four times as
//              large: row 4 j + (hash(j) mod 4), ascending with irregular gaps like a sorted token list;
//   PATTERN 2: streams its tile and writes 1 KB of results as four runs of 256 bytes in rows far apart,
//              right away (what a scoring pass does that stores every tile's scores);
//   PATTERN 3: streams its tile and keeps the 1 KB in LDS; the workgroup writes the chunk's 32 KB in one
//              burst (four runs of 8 KB) when the chunk is done.
// dst takes the results of patterns 2 and 3: one float per 128 bytes read.
constexpr int PROBE_CHUNK_TILES = 32;

template <int PATTERN>
__global__ __launch_bounds__(256) void probe_traffic_kernel(const u32x4* __restrict__ src, float* __restrict__ dst,
                                                             int64_t n_chunks) {
    __shared__ f32x4 stage[PATTERN == 3 ? PROBE_CHUNK_TILES * 64 : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int64_t ch = blockIdx.x; ch < n_chunks; ch += gridDim.x) {
        for (int j = 0; j < PROBE_CHUNK_TILES / 4; ++j) {
            const int64_t t = ch * PROBE_CHUNK_TILES + j * 4 + wave;   // tile
            u32x4 v[32];
            if (PATTERN == 1) {
#pragma unroll
                for (int i = 0; i < 32; ++i) {
                    const int64_t jrow = t * 128 + i * 4 + (lane >> 4);
                    const uint32_t hsh = (uint32_t)jrow * 2654435761u;
                    v[i] = __builtin_nontemporal_load(&src[(jrow * 4 + (hsh >> 30)) * 16 + (lane & 15)]);
                }
            } else {
#pragma unroll
                for (int i = 0; i < 32; ++i) v[i] = __builtin_nontemporal_load(&src[t * 2048 + i * 64 + lane]);
            }
            u32x4 f = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < 32; ++i) f ^= v[i];
            const f32x4 o = {(float)f.x, (float)f.y, (float)f.z, (float)f.w};
            if (PATTERN == 2) {
                const int64_t g = t >> 9, col = (t & 511) * 64 + lane;
#pragma unroll
                for (int h = 0; h < 4; ++h) dst[(g * 4 + h) * 32768 + col] = o[h];
            } else if (PATTERN == 3) {
                stage[(j * 4 + wave) * 64 + lane] = o;
            } else if (f.x == 0x9e3779b9u) {
                dst[0] = o[0];                           // keeps the loads alive; practically never taken
            }
        }
        if (PATTERN == 3) {
            __syncthreads();
            constexpr int PER = PROBE_CHUNK_TILES * 64 / 4;   // 16-byte words per run: four runs of 8 KB
            for (int i = threadIdx.x; i < PROBE_CHUNK_TILES * 64; i += 256) {
                const int q = i / PER, w = i % PER;
                f32x4* const p = reinterpret_cast<f32x4*>(dst) + ((ch / 16) * 4 + q) * (16 * (int64_t)PER) + (ch % 16) * PER + w;
                __builtin_nontemporal_store(stage[i], p);
            }
            __syncthreads();
        }
    }
}

// Attention recall (Eq. 3): the share of a head's softmax mass that falls on its token set.  With
// lse = log2 of the softmax denominator (scores scaled by sm_scale * log2 e) over the set and over
// all tokens, the ratio of the two denominators is 2^(lse_set - lse_all).
__global__ void recall_kernel(const float* __restrict__ lse_set, const float* __restrict__ lse_all,
                              float* __restrict__ recall, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) recall[i] = exp2f(lse_set[i] - lse_all[i]);
}

}  // namespace cusa
