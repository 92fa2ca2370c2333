// Sub-graph construction (Algorithm 1 Step-2 with the intra-community probability knob of
// Section 4.2): per-layer fanout sampling, frontier de-duplication in first-appearance order,
// CSR blocks with local column ids and their transposes.  Integer arithmetic only; a whole group of
// mini-batches is sampled by one set of launches (blockIdx.y = batch within the group).
#include "cr_common.h"
#include <type_traits>

namespace cr {

constexpr uint64_t KEY_MAX = ~0ull;
constexpr uint64_t EMPTY = ~0ull;

// ---------------------------------------------------------------------------------------------
// integer exponential clock: E(r) = -log2((2r+1)/2^33) in Q24, one result bit per squaring
// ---------------------------------------------------------------------------------------------
// COMPACT: the squarings as a loop (for the rarely taken exact paths of kernels whose common path should keep its
// registers: unrolled, four of these chains side by side cost the weighted kernel half its occupancy)
template <bool COMPACT = false>
__device__ __forceinline__ uint32_t exp_clock_q24(uint32_t r)
{
    const uint64_t x = 2ull * r + 1ull;
    const int t = 63 - __clzll((long long)x);
    uint32_t y = (uint32_t)((x << (63 - t)) >> 32);
    uint32_t frac = 0;
    constexpr int UNROLL = COMPACT ? 1 : 24;
#pragma unroll UNROLL
    for (int i = 0; i < 24; ++i) {
        const uint32_t hi = __umulhi(y, y), lo = y * y;
        const bool top = (hi >> 31) != 0;
        y = top ? hi : ((hi << 1) | (lo >> 31));
        frac = (frac << 1) | (top ? 1u : 0u);
    }
    return ((uint32_t)(33 - t) << 24) - frac;
}

struct SelectArgs {
    const int64_t *g_indptr;
    const int32_t *g_indices;
    const int32_t *comm;
    const uint32_t *edge_intra;   // one bit per adjacency entry (same community), or NULL
    int64_t n_entries;
    const int32_t *dst_ids;   // roots, or the frontier of the layer above
    int64_t dst_stride;
    const int32_t *prev_hdr;  // header array of the layer above, NULL for the root layer
    int64_t n_roots_total;
    int32_t batch_size;
    int32_t fanout;
    uint32_t q_in, q_out;
    uint32_t strict_p1;       // drop inter-community picks (only meaningful when q_out == 0)
    uint32_t seed_lo, seed_hi, ctr3, first_batch;
    int32_t *sel;             // [G][cap_dst*fanout] chosen global neighbour ids, rows in slot order
    int64_t sel_stride;
    int32_t *cnt;             // [G][cap_dst]
    int64_t cnt_stride;
    uint32_t cand_target;     // long rows, uniform sampling: expected number of slots below the pre-filter threshold
    // Direct output (input-side block left in global ids, every row keeps min(fanout, degree) neighbours): the row
    // pointers are known before anything is selected, so the chosen ids go straight to their place in the block's
    // per-edge id array and the intermediate [row][fanout] array is not written at all.
    const int32_t *out_indptr;   // [G][out_indptr_stride] or NULL
    int64_t out_indptr_stride;
    int32_t *out_ids;            // [G][out_stride]
    int64_t out_stride;
    uint32_t exact_select;       // verification aid: no pre-filter thresholds, every ranking on full (key, slot) pairs
};

// where the chosen neighbours of a row go, and (when they go to the intermediate array) the row's count
__device__ __forceinline__ int32_t *sel_row_ptr(const SelectArgs &a, int g, int row)
{
    if (a.out_indptr) return a.out_ids + (int64_t)g * a.out_stride + a.out_indptr[(int64_t)g * a.out_indptr_stride + row];
    return a.sel + (int64_t)g * a.sel_stride + (int64_t)row * a.fanout;
}
__device__ __forceinline__ void set_row_count(const SelectArgs &a, int g, int row, int n)
{
    if (!a.out_indptr) a.cnt[(int64_t)g * a.cnt_stride + row] = n;
}

__device__ __forceinline__ int group_n_dst(const int32_t *prev_hdr, int g, int64_t n_roots_total, int batch_size)
{
    if (prev_hdr) return prev_hdr[(int64_t)g * CR_HDR_WORDS + CR_HDR_N_SRC];
    const int64_t left = n_roots_total - (int64_t)g * batch_size;
    return (int)(left < 0 ? 0 : (left > batch_size ? batch_size : left));
}

__device__ __forceinline__ uint32_t rl32(uint32_t v, int lane) { return (uint32_t)__builtin_amdgcn_readlane((int)v, lane); }
__device__ __forceinline__ uint64_t rl64(uint64_t v, int lane)
{
    return ((uint64_t)rl32((uint32_t)(v >> 32), lane) << 32) | rl32((uint32_t)v, lane);
}
__device__ __forceinline__ uint32_t push32(uint32_t v, int dst_lane) { return (uint32_t)__builtin_amdgcn_ds_permute(dst_lane << 2, (int)v); }
__device__ __forceinline__ uint64_t push64(uint64_t v, int dst_lane)
{
    return ((uint64_t)push32((uint32_t)(v >> 32), dst_lane) << 32) | push32((uint32_t)v, dst_lane);
}

__device__ __forceinline__ bool edge_is_intra(const SelectArgs &a, int64_t e) { return (a.edge_intra[e >> 5] >> (e & 31)) & 1u; }

__device__ __forceinline__ uint32_t pull32(uint32_t v, int src_lane) { return (uint32_t)__builtin_amdgcn_ds_bpermute(src_lane << 2, (int)v); }
__device__ __forceinline__ int lanes_below(uint64_t mask, int acc)      // acc + number of set bits below this lane
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, (uint32_t)acc));
}

// ordering key of slot j of node v given its random word: narrow mode (p = 0.5) uses the word itself
// MODE: 0 uniform (p = 0.5), 1 p = 1 (classes only, no clock), 2 weighted (0.5 < p < 1)
template <int MODE, bool COMPACT = false>
__device__ __forceinline__ uint64_t slot_key(const SelectArgs &a, uint32_t r, bool intra)
{
    if (MODE == 0) return r;
    if (MODE == 1) return (intra ? 0ull : (1ull << 62)) + (uint64_t)r;
    return (uint64_t)exp_clock_q24<COMPACT>(r) * (uint64_t)(intra ? a.q_out : a.q_in);
}

__device__ __forceinline__ uint32_t slot_word(const SelectArgs &a, int j, int32_t v, uint32_t batch)
{
    const u32x4 w = philox4x32_10((uint32_t)j >> 2, (uint32_t)v, batch, a.ctr3, a.seed_lo, a.seed_hi);
    const uint32_t pick = (uint32_t)j & 3u;
    return pick == 0 ? w.x : (pick == 1 ? w.y : (pick == 2 ? w.z : w.w));
}

// A row with more than 64 neighbours, handled by a whole wave.  A slot's ordering value is the pair
// (key, slot); with WIDE == false (p = 0.5, 32-bit keys) the pair is packed into one 64-bit word.
// Lanes 0..k-1 hold the k smallest pairs seen so far in ascending order: the first 64 slots are ranked
// by counting and permuted into place, later chunks of 64 slots are tested against the k-th pair and
// inserted by shifting.  Every pair is distinct, so the surviving set is unique.
template <int MODE, bool COMPACT = false>
__device__ __forceinline__ void select_big_row(const SelectArgs &a, int g, int row, int32_t v, int64_t base, int deg, int32_t cv,
                                            int lane)
{
    constexpr bool WIDE = MODE != 0;
    const int f = a.fanout;
    int32_t *sel_row = sel_row_ptr(a, g, row);
    const int k = f;
    const uint32_t batch = a.first_batch + (uint32_t)g;
    auto less = [&](uint64_t ka, uint32_t sa, uint64_t kb, uint32_t sb) -> bool {
        if (!WIDE) return ka < kb;
        return ka < kb || (ka == kb && sa < sb);
    };
    auto make_key = [&](uint32_t r, int j, bool intra, uint64_t &ck, uint32_t &cs) {
        if (!WIDE) {
            ck = ((uint64_t)r << 32) | (uint32_t)j;
            cs = 0;
        } else {
            ck = slot_key<MODE, COMPACT>(a, r, intra);
            cs = (uint32_t)j;
        }
    };
    // neighbour class look-ups are clamped to the row, so they can be issued ahead unconditionally
    auto load_u = [&](int j) -> int32_t { return a.g_indices[base + min(j, deg - 1)]; };

    // first chunk: rank the first 64 slots by counting, then move rank r to lane r
    uint64_t ck = KEY_MAX;
    uint32_t cs = 0xFFFFFFFFu;
    // class of slot j (clamped to the row): one bit when the graph carries them, else two dependent look-ups
    auto cls = [&](int j) -> bool {
        if (a.edge_intra) return edge_is_intra(a, base + min(j, deg - 1));
        return a.comm[load_u(j)] == cv;
    };
    {
        bool intra = false;
        if (WIDE) intra = cls(lane);
        make_key(slot_word(a, lane, v, batch), lane, intra, ck, cs);
        int rank = 0;
        for (int j = 0; j < WAVE; ++j) {
            const uint64_t kj = rl64(ck, j);
            const uint32_t sj = WIDE ? rl32(cs, j) : 0u;
            rank += less(kj, sj, ck, cs) ? 1 : 0;
        }
        ck = push64(ck, rank);
        if (WIDE) cs = push32(cs, rank);
    }

    // later chunks: a slot that beats the current k-th pair is inserted by shifting the sorted lanes
    uint64_t tk = rl64(ck, k - 1);
    uint32_t ts = WIDE ? rl32(cs, k - 1) : 0u;
    auto offer = [&](bool have, uint64_t nk, uint32_t ns) {
        uint64_t pass = __ballot(have && less(nk, ns, tk, ts));
        while (pass) {
            const int src = __ffsll((long long)pass) - 1;
            pass &= pass - 1;
            const uint64_t xk = rl64(nk, src);
            const uint32_t xs = WIDE ? rl32(ns, src) : 0u;
            if (less(xk, xs, tk, ts)) {
                const int pos = __popcll(__ballot(lane < k && less(ck, cs, xk, xs)));
                const uint64_t upk = __shfl_up(ck, 1);
                const uint32_t ups = WIDE ? __shfl_up(cs, 1) : 0u;
                if (lane > pos) { ck = upk; cs = ups; }
                if (lane == pos) { ck = xk; cs = xs; }
                tk = rl64(ck, k - 1);
                ts = WIDE ? rl32(cs, k - 1) : 0u;
            }
        }
    };
    if (!WIDE) {
        // uniform sampling needs no neighbour data at all: one Philox block gives a lane the words of
        // four consecutive slots, so an iteration covers 256 slots with arithmetic only
        for (int j0 = WAVE; j0 < deg; j0 += 4 * WAVE) {
            const int jb = j0 + 4 * lane;
            const u32x4 w = philox4x32_10((uint32_t)jb >> 2, (uint32_t)v, batch, a.ctr3, a.seed_lo, a.seed_hi);
            const uint32_t wr[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) offer(jb + i < deg, ((uint64_t)wr[i] << 32) | (uint32_t)(jb + i), 0u);
        }
    } else if (a.edge_intra) {
        // biased sampling needs the class of every neighbour; here it is one bit, fetched one chunk ahead
        bool c1 = cls(WAVE + lane);
        for (int j0 = WAVE; j0 < deg; j0 += WAVE) {
            const bool c2 = cls(j0 + WAVE + lane);
            const int j = j0 + lane;
            uint64_t nk = KEY_MAX;
            uint32_t ns = 0xFFFFFFFFu;
            if (j < deg) make_key(slot_word(a, j, v, batch), j, c1, nk, ns);
            offer(j < deg, nk, ns);
            c1 = c2;
        }
    } else {
        // without the bits: ids are fetched two chunks ahead and classes one chunk ahead, so the dependent
        // look-ups overlap the arithmetic
        int32_t u1 = load_u(WAVE + lane);
        int32_t c1 = a.comm[u1];
        int32_t u2 = load_u(2 * WAVE + lane);
        for (int j0 = WAVE; j0 < deg; j0 += WAVE) {
            const int32_t c2 = a.comm[u2];
            const int32_t u3 = load_u(j0 + 2 * WAVE + lane);
            const int j = j0 + lane;
            uint64_t nk = KEY_MAX;
            uint32_t ns = 0xFFFFFFFFu;
            if (j < deg) make_key(slot_word(a, j, v, batch), j, c1 == cv, nk, ns);
            offer(j < deg, nk, ns);
            c1 = c2;
            u2 = u3;
        }
    }

    // emit in ascending slot order
    const uint32_t slot = WIDE ? cs : (uint32_t)ck;
    const bool valid = lane < k && !(WIDE && a.strict_p1 && ck >= (1ull << 62));
    int32_t cu = 0;
    if (valid) cu = a.g_indices[base + slot];
    int rank = 0;
    for (int i = 0; i < k; ++i) {
        const uint32_t si = rl32(slot, i);
        const uint32_t vi = rl32(valid ? 1u : 0u, i);
        rank += (vi && si < slot) ? 1 : 0;
    }
    const uint64_t vmask = __ballot(valid);
    if (valid) sel_row[rank] = cu;
    if (lane == 0) set_row_count(a, g, row, __popcll(vmask));
}

// Uniform sampling of a row with more than 64 neighbours, the common way: slots whose random word falls
// below a threshold chosen so that about cand_target of them do (far more than the fanout, far fewer than
// the wave's candidate buffer holds) are compacted in slot order into LDS, ranked among themselves by
// counting, and the fanout smallest (word, slot) pairs are emitted in slot order.  Exact whenever it
// applies: every slot left out has a word >= the threshold > every candidate's word.  Returns false when
// the candidates are fewer than the fanout or more than the buffer holds (then the caller takes the
// general path, which needs no threshold).
constexpr int CAND_CAP = 128;

// rk[i] += (k < w[i]) for four words at once.  Written out by hand so that the four comparisons land in four different
// scalar register pairs and the four add-with-carry instructions follow them: the compiler routes every comparison
// through VCC and has to wait two cycles between each comparison and its add (three instructions lie between a
// comparison and the add that reads its result here, more than the two wait states the hardware asks for).
__device__ __forceinline__ void rank4(uint32_t k, const uint32_t (&w)[4], int (&rk)[4])
{
    uint64_t s0, s1, s2, s3;
    asm("v_cmp_lt_u32_e64 %4, %8, %9\n\t"
        "v_cmp_lt_u32_e64 %5, %8, %10\n\t"
        "v_cmp_lt_u32_e64 %6, %8, %11\n\t"
        "v_cmp_lt_u32_e64 %7, %8, %12\n\t"
        "v_addc_co_u32_e64 %0, %4, 0, %0, %4\n\t"
        "v_addc_co_u32_e64 %1, %5, 0, %1, %5\n\t"
        "v_addc_co_u32_e64 %2, %6, 0, %2, %6\n\t"
        "v_addc_co_u32_e64 %3, %7, 0, %3, %7"
        : "+v"(rk[0]), "+v"(rk[1]), "+v"(rk[2]), "+v"(rk[3]), "=&s"(s0), "=&s"(s1), "=&s"(s2), "=&s"(s3)
        : "v"(k), "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]));
}
// the same with the comparison turned round: rk[i] += (w[i] < k)
__device__ __forceinline__ void rank4_below(uint32_t k, const uint32_t (&w)[4], int (&rk)[4])
{
    uint64_t s0, s1, s2, s3;
    asm("v_cmp_gt_u32_e64 %4, %8, %9\n\t"
        "v_cmp_gt_u32_e64 %5, %8, %10\n\t"
        "v_cmp_gt_u32_e64 %6, %8, %11\n\t"
        "v_cmp_gt_u32_e64 %7, %8, %12\n\t"
        "v_addc_co_u32_e64 %0, %4, 0, %0, %4\n\t"
        "v_addc_co_u32_e64 %1, %5, 0, %1, %5\n\t"
        "v_addc_co_u32_e64 %2, %6, 0, %2, %6\n\t"
        "v_addc_co_u32_e64 %3, %7, 0, %3, %7"
        : "+v"(rk[0]), "+v"(rk[1]), "+v"(rk[2]), "+v"(rk[3]), "=&s"(s0), "=&s"(s1), "=&s"(s2), "=&s"(s3)
        : "v"(k), "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]));
}

//
// INTRA_ONLY is the same for p = 1 when the graph carries its edge-class bits: the pool is the row's
// intra-community slots (counted from the bits first); with fewer of them than the fanout the caller's general
// path fills up with inter-community ones.
template <bool INTRA_ONLY>
__device__ __forceinline__ bool select_big_row_filtered(const SelectArgs &a, int g, int row, int32_t v, int64_t base, int deg,
                                                        int lane, uint32_t *ckey /*[CAND_CAP + 4]*/, uint32_t *cslot /*[CAND_CAP]*/)
{
    const int k = a.fanout;
    const uint32_t batch = a.first_batch + (uint32_t)g;
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    int pool = deg;
    if (INTRA_ONLY) {
        const int64_t w_first = base >> 5, e_last = base + deg, w_last = (e_last - 1) >> 5;
        int n_in = 0;
        for (int64_t w = w_first + lane; w <= w_last; w += WAVE) {
            uint32_t bits = a.edge_intra[w];
            if (w == w_first) bits &= ~0u << (base & 31);
            if (w == w_last && (e_last & 31)) bits &= (1u << (e_last & 31)) - 1u;
            n_in += __popc(bits);
        }
#pragma unroll
        for (int o = 32; o; o >>= 1) n_in += __shfl_xor(n_in, o);
        if (n_in < k) return false;
        pool = n_in;
    }
    const int64_t w_max = (a.n_entries - 1) >> 5;
    // (float arithmetic: the threshold only steers how many candidates there are, any value gives the same result)
    const float thr_f = (float)a.cand_target * 4294967296.0f / (float)pool;
    const bool keep_all = thr_f >= 4294967040.0f;                  // every slot of the pool is to be a candidate
    const uint32_t thr = keep_all ? 0xFFFFFFFFu : (uint32_t)thr_f;
    int n = 0;
    // 256 slots from j0 on; a slot is a candidate iff its word is below thr and it belongs to the pool (of the right class,
    // and, in the row's last stretch, not beyond its end).  false: more candidates than the list holds.
    auto stretch = [&](int j0, auto is_last) -> bool {
        constexpr bool LAST = decltype(is_last)::value;
        const int jb = j0 + 4 * lane;
        const u32x4 w = philox4x32_10((uint32_t)jb >> 2, (uint32_t)v, batch, a.ctr3, a.seed_lo, a.seed_hi);
        const uint32_t wr[4] = {w.x, w.y, w.z, w.w};
        uint32_t nib = 0xFu;          // which of the lane's four slots belong to the pool
        if (INTRA_ONLY) {
            const int64_t e = base + min(jb, deg - 1);
            const int64_t wi = e >> 5;
            const uint64_t win = (uint64_t)a.edge_intra[wi] | ((uint64_t)a.edge_intra[min(wi + 1, w_max)] << 32);
            nib = (uint32_t)(win >> (e & 31)) & 0xFu;
        }
        if (LAST) {
            const int left = deg - jb;
            nib &= left >= 4 ? 0xFu : (left > 0 ? (1u << left) - 1u : 0u);
        }
        bool c[4];
        uint64_t b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t t = (INTRA_ONLY || LAST) ? (((nib >> i) & 1u) ? thr : 0u) : thr;
            c[i] = wr[i] < t;
            b[i] = __ballot(c[i]);
        }
        if ((b[0] | b[1] | b[2] | b[3]) == 0) return true;             // (most stretches of a very long row)
        int before = n;
#pragma unroll
        for (int i = 0; i < 4; ++i) before = lanes_below(b[i], before);
        const int total = __popcll(b[0]) + __popcll(b[1]) + __popcll(b[2]) + __popcll(b[3]);
        if (n + total > CAND_CAP) return false;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (c[i]) { ckey[before] = wr[i]; cslot[before] = (uint32_t)(jb + i); }
            before += c[i] ? 1 : 0;
        }
        n += total;
        return true;
    };
    int j0 = 0;
    for (; j0 + 4 * WAVE <= deg; j0 += 4 * WAVE)
        if (!stretch(j0, std::false_type{})) return false;
    if (j0 < deg && !stretch(j0, std::true_type{})) return false;
    // (a word of all ones is never below the threshold: with every slot wanted, leave such a row to the general path)
    if (keep_all && n != pool) return false;
    if (n < k) return false;
    if (lane < 4) ckey[n + lane] = ~0u;            // pad the words to a multiple of four with the largest one
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

    // candidate t sits at index t in slot order; a lane owns candidates lane and lane + 64.  Words only are compared: with
    // equal words at the boundary the kept count is off and the caller's general path takes the row.
    const bool have0 = lane < n, have1 = lane + WAVE < n;
    const uint32_t w0 = ckey[min(lane, n - 1)], w1 = ckey[min(lane + WAVE, n - 1)];
    int ra[4] = {0, 0, 0, 0}, rb[4] = {0, 0, 0, 0};
    if (n <= WAVE) {
        for (int t0 = 0; t0 < n; t0 += 4) {
            const uint4 kt = *reinterpret_cast<const uint4 *>(ckey + t0);
            const uint32_t ks[4] = {kt.x, kt.y, kt.z, kt.w};
            rank4_below(w0, ks, ra);
        }
    } else {
        for (int t0 = 0; t0 < n; t0 += 4) {
            const uint4 kt = *reinterpret_cast<const uint4 *>(ckey + t0);
            const uint32_t ks[4] = {kt.x, kt.y, kt.z, kt.w};
            rank4_below(w0, ks, ra);
            rank4_below(w1, ks, rb);
        }
    }
    const int r0 = ra[0] + ra[1] + ra[2] + ra[3], r1 = rb[0] + rb[1] + rb[2] + rb[3];
    const bool s0 = have0 && r0 < k, s1 = have1 && r1 < k;
    const uint64_t m0 = __ballot(s0), m1 = __ballot(s1);
    const bool exact = __popcll(m0) + __popcll(m1) == k;
    if (exact) {
        int32_t *sel_row = sel_row_ptr(a, g, row);
        if (s0) sel_row[__popcll(m0 & lt_mask)] = a.g_indices[base + cslot[lane]];
        if (s1) sel_row[__popcll(m0) + __popcll(m1 & lt_mask)] = a.g_indices[base + cslot[lane + WAVE]];
        if (lane == 0) set_row_count(a, g, row, k);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // the buffers are reused by this wave's next long row
    return exact;
}

// Long rows for 0.5 < p < 1, with the graph's edge-class bits.  A slot's key is E(r) * m with m = 1-p for an
// intra-community slot and p for an inter-community one, E a non-increasing function of the random word r, so
// "key below kappa" is "r at or above a per-class threshold".  kappa is chosen (float arithmetic, a few Newton steps
// on the expected candidate count; its value only affects how many candidates there are) so that about cand_target
// slots pass; only those get the 24-squaring clock.  The result is exact iff the fanout-th smallest candidate key
// is below the smallest key any left-out slot can have, E(threshold - 1) * m per class in integer arithmetic: that is
// checked, and otherwise (or with too few / too many candidates) the caller takes the general path.
template <bool COMPACT = false>
__device__ __forceinline__ bool select_big_row_weighted(const SelectArgs &a, int g, int row, int32_t v, int64_t base, int deg,
                                                        int lane, uint2 *cand, unsigned long long *ckey)
{
    const int k = a.fanout;
    const uint32_t batch = a.first_batch + (uint32_t)g;
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    const int64_t w_first = base >> 5, e_last = base + deg, w_last = (e_last - 1) >> 5;
    int n_in = 0;
    for (int64_t w = w_first + lane; w <= w_last; w += WAVE) {
        uint32_t bits = a.edge_intra[w];
        if (w == w_first) bits &= ~0u << (base & 31);
        if (w == w_last && (e_last & 31)) bits &= (1u << (e_last & 31)) - 1u;
        n_in += __popc(bits);
    }
#pragma unroll
    for (int o = 32; o; o >>= 1) n_in += __shfl_xor(n_in, o);
    const int n_out = deg - n_in;

    // per-class thresholds on the random word: candidate iff r >= t_class
    uint64_t t_in = 0, t_out = 0;
    if ((int)a.cand_target < deg) {
        const float ln2 = 0.69314718f, target = (float)a.cand_target;
        const float s_in = 1.0f / ((float)a.q_out * 16777216.0f), s_out = 1.0f / ((float)a.q_in * 16777216.0f);
        const float fi = (float)n_in, fo = (float)n_out;
        float kappa = target / (ln2 * (fi * s_in + fo * s_out));       // tangent at zero: never past the root
#pragma unroll
        for (int it = 0; it < 3; ++it) {
            const float ei = exp2f(-kappa * s_in), eo = exp2f(-kappa * s_out);
            const float gv = fi * (1.0f - ei) + fo * (1.0f - eo) - target;
            const float gd = ln2 * (fi * s_in * ei + fo * s_out * eo);
            if (gd > 0.0f) kappa -= gv / gd;
        }
        const float pi = exp2f(-kappa * s_in) * 4294967296.0f, po = exp2f(-kappa * s_out) * 4294967296.0f;
        t_in = pi >= 4294967296.0f ? 0x100000000ull : (uint64_t)(pi > 0.0f ? pi : 0.0f);
        t_out = po >= 4294967296.0f ? 0x100000000ull : (uint64_t)(po > 0.0f ? po : 0.0f);
    }
    // smallest key a slot that is left out can have (lane 0: intra, lane 1: inter), exact integers
    uint64_t bound;
    {
        const uint64_t t = lane == 0 ? t_in : t_out;
        const uint32_t m = lane == 0 ? a.q_out : a.q_in;
        const int pool = lane == 0 ? n_in : n_out;
        const uint64_t e = (uint64_t)exp_clock_q24<COMPACT>((uint32_t)(t > 0 ? t - 1 : 0)) * m;
        const uint64_t mine = (t == 0 || pool == 0) ? KEY_MAX : e;
        const uint64_t b0 = rl64(mine, 0), b1 = rl64(mine, 1);
        bound = b0 < b1 ? b0 : b1;
    }

    const int64_t w_max = (a.n_entries - 1) >> 5;
    int n = 0;
    for (int j0 = 0; j0 < deg; j0 += 4 * WAVE) {
        const int jb = j0 + 4 * lane;
        const u32x4 w = philox4x32_10((uint32_t)jb >> 2, (uint32_t)v, batch, a.ctr3, a.seed_lo, a.seed_hi);
        const uint32_t wr[4] = {w.x, w.y, w.z, w.w};
        const int64_t e = base + min(jb, deg - 1);
        const int64_t wi = e >> 5;
        const uint64_t win = (uint64_t)a.edge_intra[wi] | ((uint64_t)a.edge_intra[min(wi + 1, w_max)] << 32);
        const uint32_t nib = (uint32_t)(win >> (e & 31)) & 0xFu;
        bool c[4];
        uint64_t b[4];
        int before = n, total = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            c[i] = jb + i < deg && (uint64_t)wr[i] >= (((nib >> i) & 1u) ? t_in : t_out);
            b[i] = __ballot(c[i]);
            before += __popcll(b[i] & lt_mask);
            total += __popcll(b[i]);
        }
        if (n + total > CAND_CAP) return false;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (c[i]) cand[before] = make_uint2(wr[i], (uint32_t)(jb + i) | (((nib >> i) & 1u) << 31));
            before += c[i] ? 1 : 0;
        }
        n += total;
    }
    if (n < k) return false;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

    // keys of the candidates only; candidate t sits at index t in slot order, a lane owns candidates lane and lane + 64
    const uint2 c0 = cand[min(lane, n - 1)], c1 = cand[min(lane + WAVE, n - 1)];
    const bool have0 = lane < n, have1 = lane + WAVE < n;
    const uint64_t key0 = (uint64_t)exp_clock_q24<COMPACT>(c0.x) * ((c0.y >> 31) ? a.q_out : a.q_in);
    uint64_t key1 = KEY_MAX;
    if (n > WAVE) key1 = (uint64_t)exp_clock_q24<COMPACT>(c1.x) * ((c1.y >> 31) ? a.q_out : a.q_in);
    if (have0) ckey[lane] = key0;
    if (have1) ckey[lane + WAVE] = key1;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    int r0 = 0, r1 = 0;
    if (n <= WAVE) {
        for (int t = 0; t < n; ++t) {
            const uint64_t kt = ckey[t];
            r0 += (kt < key0 || (kt == key0 && t < lane)) ? 1 : 0;
        }
    } else {
        for (int t = 0; t < n; ++t) {
            const uint64_t kt = ckey[t];
            r0 += (kt < key0 || (kt == key0 && t < lane)) ? 1 : 0;
            r1 += (kt < key1 || (kt == key1 && t < lane + WAVE)) ? 1 : 0;
        }
    }
    // the fanout-th smallest candidate key must beat everything that was left out
    const uint64_t q0 = __ballot(have0 && r0 == k - 1), q1 = __ballot(have1 && r1 == k - 1);
    const uint64_t kth = q0 ? rl64(key0, __ffsll((long long)q0) - 1) : rl64(key1, __ffsll((long long)q1) - 1);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // both buffers are reused by this wave's next long row
    if (!(kth < bound)) return false;

    const bool s0 = have0 && r0 < k, s1 = have1 && r1 < k;
    const uint64_t m0 = __ballot(s0), m1 = __ballot(s1);
    int32_t *sel_row = sel_row_ptr(a, g, row);
    if (s0) sel_row[__popcll(m0 & lt_mask)] = a.g_indices[base + (c0.y & 0x7FFFFFFFu)];
    if (s1) sel_row[__popcll(m0) + __popcll(m1 & lt_mask)] = a.g_indices[base + (c1.y & 0x7FFFFFFFu)];
    if (lane == 0) set_row_count(a, g, row, k);
    return true;
}

// A wave takes SEL_ROWS consecutive destination rows.  Rows with at most 64 neighbours are packed side
// by side into the wave's lanes (lane = one neighbour slot of one row; as many consecutive rows per pass
// as fit), so that the random words, the keys and the ranking of several short rows cost one pass of
// instructions: a row with deg <= fanout keeps every neighbour, otherwise the slots whose (key, slot)
// pair ranks below the fanout inside their row survive; output keeps slot order.  Longer rows go through
// select_big_row one at a time.
constexpr int SEL_ROWS = 8;

template <int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 8))) void select_kernel(SelectArgs a)
{
    constexpr bool WIDE = MODE != 0;
    __shared__ uint2 cand[4][CAND_CAP];
    __shared__ unsigned long long ckey[MODE == 2 ? 4 : 1][MODE == 2 ? CAND_CAP : 1];
    const int g = blockIdx.y;
    const int n_dst = group_n_dst(a.prev_hdr, g, a.n_roots_total, a.batch_size);
    const int row0 = (int)(blockIdx.x * 4 + threadIdx.x / WAVE) * SEL_ROWS;
    if (row0 >= n_dst) return;
    const int lane = lane_id();
    const int f = a.fanout;
    const uint32_t batch = a.first_batch + (uint32_t)g;

    // lanes 0..SEL_ROWS-1 fetch one row's node id, adjacency range and community each
    int32_t mv = 0, mcv = 0;
    int64_t mbase = 0;
    int mdeg = 0;
    if (lane < SEL_ROWS && row0 + lane < n_dst) {
        mv = a.dst_ids[(int64_t)g * a.dst_stride + row0 + lane];
        mbase = a.g_indptr[mv];
        const int64_t d = a.g_indptr[mv + 1] - mbase;
        mdeg = (int)(d > 0x7FFFFFFF ? 0x7FFFFFFF : d);
        if (WIDE) mcv = a.comm[mv];
        if (mdeg == 0) set_row_count(a, g, row0 + lane, 0);
    }
    int32_t v[SEL_ROWS], cv[SEL_ROWS];
    int deg[SEL_ROWS], start[SEL_ROWS], pass[SEL_ROWS];
    int64_t base[SEL_ROWS];
    int off = 0, last_pass = 0;
#pragma unroll
    for (int i = 0; i < SEL_ROWS; ++i) {
        v[i] = (int32_t)rl32((uint32_t)mv, i);
        cv[i] = WIDE ? (int32_t)rl32((uint32_t)mcv, i) : 0;
        deg[i] = (int)rl32((uint32_t)mdeg, i);
        base[i] = (int64_t)rl64((uint64_t)mbase, i);
        // greedy packing of the short rows into passes of at most 64 lanes
        pass[i] = -1;
        start[i] = 0;
        if (deg[i] > 0 && deg[i] <= WAVE) {
            if (off + deg[i] > WAVE) { ++last_pass; off = 0; }
            pass[i] = last_pass;
            start[i] = off;
            off += deg[i];
        }
    }

    for (int p = 0; p <= last_pass; ++p) {
        int ri = -1, my_start = 0, my_len = 0, maxlen = 0;
        int32_t my_v = 0, my_cv = 0;
        int64_t my_base = 0;
#pragma unroll
        for (int i = 0; i < SEL_ROWS; ++i) {
            if (pass[i] != p) continue;                       // uniform
            if (deg[i] > f) maxlen = max(maxlen, deg[i]);
            if (lane >= start[i] && lane < start[i] + deg[i]) {
                ri = i; my_start = start[i]; my_len = deg[i]; my_v = v[i]; my_cv = cv[i]; my_base = base[i];
            }
        }
        const bool active = ri >= 0;
        if (__ballot(active) == 0) continue;
        const int j = lane - my_start;
        int32_t u = 0;
        if (active) u = a.g_indices[my_base + j];
        bool intra = false;
        if (WIDE && active && (maxlen > 0 || a.strict_p1)) intra = a.edge_intra ? edge_is_intra(a, my_base + j) : a.comm[u] == my_cv;
        bool survivor = active && !(WIDE && a.strict_p1 && !intra);
        if (maxlen > 0) {
            // every lane computes its slot's key; lanes of rows that keep all their neighbours ignore it
            const uint64_t ck = slot_key<MODE>(a, slot_word(a, j, my_v, batch), intra);
            int rank = 0;
            for (int d0 = 0; d0 < maxlen; d0 += 4) {          // four independent lane exchanges in flight per step
                uint64_t ok[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int src = my_start + d0 + q;
                    if (WIDE) ok[q] = ((uint64_t)pull32((uint32_t)(ck >> 32), src) << 32) | pull32((uint32_t)ck, src);
                    else ok[q] = pull32((uint32_t)ck, src);
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int d = d0 + q;
                    rank += (d < my_len && (ok[q] < ck || (ok[q] == ck && d < j))) ? 1 : 0;
                }
            }
            if (active && my_len > f) survivor = rank < f && !(WIDE && a.strict_p1 && ck >= (1ull << 62));
        }
        const uint64_t seg = (my_len >= WAVE ? ~0ull : ((1ull << my_len) - 1ull)) << my_start;
        const uint64_t smask = __ballot(survivor) & seg;
        if (active) {
            const int row = row0 + ri;
            if (survivor) sel_row_ptr(a, g, row)[__popcll(smask & ((1ull << lane) - 1ull))] = u;
            if (j == 0) set_row_count(a, g, row, __popcll(smask));
        }
    }

#pragma unroll
    for (int i = 0; i < SEL_ROWS; ++i)
        if (deg[i] > WAVE) {
            uint2 *buf = cand[threadIdx.x / WAVE];
            if (MODE == 2 && !a.exact_select && a.edge_intra &&
                select_big_row_weighted(a, g, row0 + i, v[i], base[i], deg[i], lane, buf, ckey[threadIdx.x / WAVE])) continue;
            select_big_row<MODE>(a, g, row0 + i, v[i], base[i], deg[i], cv[i], lane);
        }
}

// ---------------------------------------------------------------------------------------------
// Selection with four neighbour slots per lane: uniform sampling, and p = 1 on a graph that carries its edge-class bits
// ---------------------------------------------------------------------------------------------
// One Philox block yields the random words of four consecutive slots, so a lane owns a "quad" of slots and a pass of the
// wave covers 256 slots of consecutive destination rows laid side by side (a row of up to 256 slots never straddles two
// passes).  Both settings reduce to "keep the m smallest words of a pool of P slots, and all of the rest that is kept":
//   uniform        pool = the row, m = min(fanout, degree);
//   p = 1          with n_in >= fanout intra-community slots the pool is those and m = fanout; with fewer, all of them are
//                  kept and the pool is the inter-community slots with m = fanout - n_in (0 in strict mode).
// Slots whose word lies below a threshold of about (m + 3 sqrt(m) + 3) / P become candidates, are compacted in slot order
// into the row's stretch of an LDS list, and every lane ranks its four slots against that list (one broadcast read serves
// four comparisons per lane).  The ranking compares words only; a row whose kept count then differs from the count it must
// have (a threshold that let fewer than m slots through, or equal words at the boundary) is redone without threshold and
// with (word, slot) pairs compared in full, so the result is exact in every case.
//
// Weighted sampling (0.5 < p < 1) takes the same passes with single-precision keys: approx_clock(r) * m_class, compared
// through their bit patterns (all positive).  They decide only WHICH slots are kept (the output is in slot order), so the
// result is exact whenever the largest kept key and the smallest key left out are further apart than the keys' error
// bounds; that is checked per row, and a row that fails (or whose threshold let too few slots through) is redone with
// the exact integer keys.  The bound |approx_clock(r) * 2^24 - E(r)| <= CLOCK_ERR_ABS + CLOCK_ERR_REL * E(r) (E in its
// Q24 units) holds with a factor of two to spare for every one of the 2^32 words: cr_selftest_clock_approximation
// measures it on the device.
constexpr float CLOCK_ERR_ABS = 8.0f;             // Q24 units
constexpr float CLOCK_ERR_REL = 0x1p-17f;       // (measured: 3 units / 2^-19)

__device__ __forceinline__ float approx_clock(uint32_t r)
{
    // (2r+1) / 2^33 below one half: 33 - log2(2r+1), the argument rounded to 24 bits.  Above: the distance from one,
    // d = 2^33 - (2r+1), is converted instead, so that the small clocks -- the ones that get picked -- keep their
    // relative precision.
    // (one logarithm: the argument is chosen first; the instruction runs at a quarter of the rate of ordinary ones)
    const bool far = r < 0x80000000u;
    const float arg = far ? (float)(2u * r + 1u) : 1.0f - (float)(2u * ~r + 1u) * 0x1p-33f;
    const float lg = __builtin_amdgcn_logf(arg);
    return far ? 33.0f - lg : __builtin_fabsf(lg);
}

// Is every key of the kept side provably below every key of the left-out side?  hi = the largest approximate key kept
// (class weight m_hi), lo = the smallest approximate key left out (class weight m_lo; +infinity: nothing there).  A key's
// error: its clock's (CLOCK_ERR_ABS + CLOCK_ERR_REL * E, times the class weight) plus the rounding of the product; the
// last term covers the rounding of this comparison itself.
__device__ __forceinline__ bool keys_apart(float hi, float m_hi, float lo, float m_lo)
{
    if (!(lo < INFINITY)) return true;
    const float slack = (hi + lo) * (CLOCK_ERR_REL + 0x1p-21f) + CLOCK_ERR_ABS * 0x1p-24f * (m_hi + m_lo);
    return lo - hi > slack;
}

constexpr int QUAD_ROWS = 32;            // destination rows per wave
constexpr int QUAD_MAX_DEG = 4 * WAVE;   // longest row a pass holds

struct alignas(16) QuadRow {
    int32_t v, deg, startq, nq_row;      // node, degree, first quad in the wave's quad sequence, number of quads | which of
                                         // the wave's destination rows it is << 8
    int64_t base;                        // first adjacency entry
    int32_t *out;                        // where the row's chosen ids go
};

// One pass; returns the rows that have to be redone exactly (bit r = the r-th row of the wave's quad sequence: the rows
// are laid out in the order the packing placed them, not in the order of the block).  rowmask: rows to process.
template <int MODE, bool EXACT>
__device__ __forceinline__ uint32_t quad_pass(const SelectArgs &a, int g, int row0, int p, uint32_t rowmask, const QuadRow *rows,
                                              const int *startq, uint32_t *klist, uint32_t *clist, uint32_t *rowinfo,
                                              unsigned long long *k64, uint32_t *rowstat, int lane)
{
    const int f = a.fanout;
    const uint32_t batch = a.first_batch + (uint32_t)g;
    const int gq = p * WAVE + lane;
    // the row of this lane's quad: the last one that starts at or before it (startq is non-decreasing, startq[0] = 0)
    static_assert(QUAD_ROWS == 32, "the bisection below takes five steps");
    int r = startq[16] <= gq ? 16 : 0;
    r += startq[r + 8] <= gq ? 8 : 0;
    r += startq[r + 4] <= gq ? 4 : 0;
    r += startq[r + 2] <= gq ? 2 : 0;
    r += startq[r + 1] <= gq ? 1 : 0;
    const QuadRow R = rows[r];
    const int qi = gq - R.startq;
    const int nq = R.nq_row & 0xFF;
    const bool active = qi < nq && ((rowmask >> r) & 1u);
    if (__ballot(active) == 0) return 0u;
    const int first = R.startq - p * WAVE, last = first + nq - 1;         // the row's lanes in this pass
    const int jb = 4 * qi;
    const int left = active ? R.deg - jb : 0;
    const uint32_t vmask = left >= 4 ? 0xFu : ((1u << left) - 1u);        // the quad's slots that exist
    const u32x4 w = philox4x32_10((uint32_t)qi, (uint32_t)R.v, batch, a.ctr3, a.seed_lo, a.seed_hi);
    const uint32_t wr[4] = {w.x, w.y, w.z, w.w};

    // number of set flags of this row in the lanes before this one, and in the whole row (flags of lanes outside any
    // row are zero)
    // (in_pass: the same count over all the lanes before this one, whatever their row)
    auto seg = [&](uint32_t m4, int &excl, int &total, int &in_pass) {
        int e = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) e = lanes_below(__ballot((m4 >> i) & 1u), e);
        const int before_row = (int)pull32((uint32_t)e, first);
        const int upto_last = (int)pull32((uint32_t)(e + __popc(m4)), last);
        excl = e - before_row;
        total = upto_last - before_row;
        in_pass = e;
    };

    uint32_t pool = vmask, take = 0u;
    int m = min(f, R.deg), P = R.deg, expect = m;
    uint32_t nib = 0u;
    int n_in = 0;
    if (MODE >= 1) {
        if (active) {
            const int64_t e = R.base + jb, wi = e >> 5, w_max = (a.n_entries - 1) >> 5;
            const uint64_t win = (uint64_t)a.edge_intra[wi] | ((uint64_t)a.edge_intra[min(wi + 1, w_max)] << 32);
            nib = (uint32_t)(win >> (e & 31)) & 0xFu;
        }
        int unused, unused2;
        seg(nib & vmask, unused, n_in, unused2);
    }
    if (MODE == 1) {
        const uint32_t in4 = nib & vmask;
        if (n_in >= f) {
            pool = in4; m = f; P = n_in; expect = f;
        } else {
            take = in4; pool = vmask & ~nib; P = R.deg - n_in;
            m = a.strict_p1 ? 0 : min(f - n_in, P);
            expect = n_in + m;
        }
    }
    // the ordering words of the lane's four slots: the random words themselves, or (weighted) the bit patterns of the
    // single-precision keys
    uint32_t kw[4] = {wr[0], wr[1], wr[2], wr[3]};
    if (MODE == 2 && !EXACT) {
#pragma unroll
        for (int i = 0; i < 4; ++i) kw[i] = __float_as_uint(approx_clock(wr[i]) * (float)(((nib >> i) & 1u) ? a.q_out : a.q_in));
    }
    const bool ranked = active && m > 0 && m < P;
    if (!ranked) {
        if (m >= P) take |= pool;           // the whole pool is kept
        pool = 0u;
    }
    uint32_t cm = pool;                      // candidates among this lane's slots
    float kappa = INFINITY;                  // weighted: every slot that is no candidate has a key of at least this
    if (!EXACT && ranked) {
        // (float arithmetic: the threshold only steers how many candidates there are)
        const float mf = (float)m;
        const float target = mf + 3.0f * __builtin_amdgcn_sqrtf(mf) + 3.0f;
        uint32_t T = 0xFFFFFFFFu;
        bool all = true;
        if (MODE == 2) {
            // expected number of keys below kappa: n_in (1 - 2^(-kappa / q_out)) + n_out (1 - 2^(-kappa / q_in)); three
            // Newton steps from the tangent at zero (never past the root)
            if (target < (float)P) {
                const float ln2 = 0.69314718f, fi = (float)n_in, fo = (float)(P - n_in);
                const float s_in = __builtin_amdgcn_rcpf((float)a.q_out), s_out = __builtin_amdgcn_rcpf((float)a.q_in);
                float kp = target / (ln2 * (fi * s_in + fo * s_out));
#pragma unroll
                for (int it = 0; it < 3; ++it) {
                    const float ei = __builtin_amdgcn_exp2f(-kp * s_in), eo = __builtin_amdgcn_exp2f(-kp * s_out);
                    const float gv = fi * (1.0f - ei) + fo * (1.0f - eo) - target;
                    const float gd = ln2 * (fi * s_in * ei + fo * s_out * eo);
                    if (gd > 0.0f) kp -= gv / gd;
                }
                if (kp > 0.0f && kp < 3.0e38f) { kappa = kp; T = __float_as_uint(kp); all = false; }
            }
        } else {
            const float tf = target * 4294967296.0f * __builtin_amdgcn_rcpf((float)P);
            if (tf < 4294967040.0f) { T = (uint32_t)tf; all = false; }
        }
        if (!all) {
            uint32_t below = 0u;
#pragma unroll
            for (int i = 0; i < 4; ++i) below |= (kw[i] < T ? 1u : 0u) << i;
            cm &= below;
        }
    }
    int cpos, n_c, cglob;
    seg(cm, cpos, n_c, cglob);
    int rk[4] = {0, 0, 0, 0};
    uint32_t below_m = 0u;                   // candidates among this lane's slots with fewer than m candidates in front
    const int nc_mine = ranked ? n_c : 0;
    if constexpr (MODE == 2 && EXACT) {
        // the exact integer keys, 64 bits each: every slot of the row is a candidate, (key, slot) pairs compared in full
        unsigned long long ek[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) ek[i] = (uint64_t)exp_clock_q24<true>(wr[i]) * (uint64_t)(((nib >> i) & 1u) ? a.q_out : a.q_in);
        unsigned long long *kl = k64 + 4 * first;
        if (ranked) {
            int k = cpos;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if ((cm >> i) & 1u) kl[k++] = ek[i];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        for (int t = 0; __ballot(t < nc_mine) != 0; ++t) {
            if (t < nc_mine) {
                const unsigned long long kt = kl[t];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    rk[i] += (kt < ek[i] || (kt == ek[i] && t < cpos + (int)__popc(cm & ((1u << i) - 1u)))) ? 1 : 0;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) below_m |= rk[i] < m ? 1u << i : 0u;
    } else {
        // the row's list: candidates' words in slot order, padded with the largest word to a multiple of four
        uint32_t *kl = klist + 4 * first;
        if (active) *reinterpret_cast<uint4 *>(klist + 4 * lane) = make_uint4(~0u, ~0u, ~0u, ~0u);
        // With at most 64 candidates in the whole pass a lane ranks ONE candidate (the lane-th of the pass, in slot order)
        // against its row's list, two instructions per list entry, instead of its own four slots against it, eight per
        // entry: in rows much longer than their list most slots are no candidates.  clist[c]: where candidate c sits in the
        // lists (bits 0..7) and its row (bits 8..11); rowinfo[r]: start of the row's list, its length << 8, m << 20.
        const int n_pass_cand = (int)rl32((uint32_t)(cglob + (int)__popc(cm)), WAVE - 1);
        const bool by_candidate = !EXACT && n_pass_cand <= WAVE;
        if (ranked) {
            int k = cpos, c = cglob;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if ((cm >> i) & 1u) {
                    kl[k] = kw[i];
                    if (by_candidate) clist[c++] = (uint32_t)(4 * first + k) | ((uint32_t)r << 8);
                    ++k;
                }
            if (by_candidate && qi == 0) rowinfo[r] = (uint32_t)(4 * first) | ((uint32_t)n_c << 8) | ((uint32_t)m << 20);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (by_candidate) {
            const bool have = lane < n_pass_cand;
            const uint32_t ce = clist[lane];                       // (stale beyond the pass's candidates: masked below)
            const uint32_t ri = rowinfo[(ce >> 8) & (QUAD_ROWS - 1)];
            const uint32_t mine = klist[ce & 0xFFu];
            const uint32_t *rl = klist + (ri & 0xFCu);
            const int nc = have ? (int)((ri >> 8) & 0xFFFu) : 0;
            int ra[4] = {0, 0, 0, 0};
            for (int t0 = 0; __ballot(t0 < nc) != 0; t0 += 4) {
                if (t0 < nc) {
                    const uint4 kt = *reinterpret_cast<const uint4 *>(rl + t0);
                    const uint32_t ks[4] = {kt.x, kt.y, kt.z, kt.w};
                    rank4_below(mine, ks, ra);
                }
            }
            const uint64_t low = __ballot(have && ra[0] + ra[1] + ra[2] + ra[3] < (int)(ri >> 20));
            // this lane's candidates are numbers cglob, cglob + 1, .. of the pass: hand their bits back to its slots
            uint32_t b = (uint32_t)(low >> (cglob & (WAVE - 1)));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t is_c = (cm >> i) & 1u;
                below_m |= (b & is_c) << i;
                b >>= is_c;
            }
        } else {
            for (int t0 = 0; __ballot(t0 < nc_mine) != 0; t0 += 4) {
                if (t0 < nc_mine) {
                    const uint4 kt = *reinterpret_cast<const uint4 *>(kl + t0);
                    const uint32_t ks[4] = {kt.x, kt.y, kt.z, kt.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (!EXACT) {
                            rank4(ks[q], kw, rk);
                        } else {
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                rk[i] += (ks[q] < kw[i] || (ks[q] == kw[i] && t0 + q < cpos + (int)__popc(cm & ((1u << i) - 1u)))) ? 1 : 0;
                        }
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) below_m |= rk[i] < m ? 1u << i : 0u;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // the lists are reused by the next pass
    const uint32_t emit = take | (cm & below_m);
    int epos, total, unused3;
    seg(emit, epos, total, unused3);
    bool ok = total == expect;            // (always true in the exact pass)
    if constexpr (MODE == 2 && !EXACT) {
        // largest kept key and smallest key left out, per row and class (LDS atomics on the bit patterns):
        // rowstat[4 r + ..] = max kept intra, max kept inter, min left-out intra, min left-out inter
        rowstat[lane] = rowstat[lane + WAVE] = (lane & 2) ? 0x7F800000u : 0u;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (ranked) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if ((cm >> i) & 1u) {
                    const int cls = ((nib >> i) & 1u) ? 0 : 1;
                    if ((below_m >> i) & 1u) atomicMax(&rowstat[4 * r + cls], kw[i]);
                    else atomicMin(&rowstat[4 * r + 2 + cls], kw[i]);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (ranked) {
            const uint4 st = *reinterpret_cast<const uint4 *>(&rowstat[4 * r]);
            const float m_in = (float)a.q_out, m_out = (float)a.q_in;      // an intra-community slot's clock is scaled by 1 - p
            const float hi_in = __uint_as_float(st.x), hi_out = __uint_as_float(st.y);
            const float lo_in = __uint_as_float(st.z), lo_out = __uint_as_float(st.w);
            // (a slot that is no candidate has an approximate key of at least kappa, whatever its class)
            ok = ok && keys_apart(hi_in, m_in, lo_in, m_in) && keys_apart(hi_in, m_in, lo_out, m_out) &&
                 keys_apart(hi_out, m_out, lo_in, m_in) && keys_apart(hi_out, m_out, lo_out, m_out) &&
                 keys_apart(hi_in, m_in, kappa, m_out) && keys_apart(hi_out, m_out, kappa, m_out);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
    if (active && ok) {
        int k = epos;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if ((emit >> i) & 1u) R.out[k++] = a.g_indices[R.base + jb + i];
        if (qi == 0) set_row_count(a, g, row0 + (R.nq_row >> 8), total);
    }
    uint64_t bad = __ballot(active && qi == 0 && !ok);
    uint32_t redo = 0u;
    while (bad) {
        redo |= 1u << rl32((uint32_t)r, __ffsll((long long)bad) - 1);
        bad &= bad - 1;
    }
    return redo;
}

// Long rows, weighted, with single-precision keys: the row's slots are filtered by per-class thresholds on the random word
// (chosen so that about cand_target keys lie below a common kappa), the candidates' keys approx_clock(r) * m_class are
// ranked through their bit patterns, and the result is accepted if the largest kept key and the smallest key left out
// (among the candidates, and the smallest a filtered-out slot can have) are further apart than the keys' error bounds.
// Returns false otherwise (too few or too many candidates, check failed): the caller goes on to the exact paths.
__device__ __forceinline__ bool select_big_row_weighted_f32(const SelectArgs &a, int g, int row, int32_t v, int64_t base, int deg,
                                                            int lane, uint32_t *ckey /*[CAND_CAP + 4]*/, uint32_t *cslot /*[CAND_CAP]*/)
{
    const int k = a.fanout;
    const uint32_t batch = a.first_batch + (uint32_t)g;
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    const int64_t w_first = base >> 5, e_last = base + deg, w_last = (e_last - 1) >> 5;
    int n_in = 0;
    for (int64_t w = w_first + lane; w <= w_last; w += WAVE) {
        uint32_t bits = a.edge_intra[w];
        if (w == w_first) bits &= ~0u << (base & 31);
        if (w == w_last && (e_last & 31)) bits &= (1u << (e_last & 31)) - 1u;
        n_in += __popc(bits);
    }
#pragma unroll
    for (int o = 32; o; o >>= 1) n_in += __shfl_xor(n_in, o);
    const int n_out = deg - n_in;
    const float m_in = (float)a.q_out, m_out = (float)a.q_in;       // an intra-community slot's clock is scaled by 1 - p

    // candidate iff r >= t_class; lo_non: the smallest key a slot below its class's threshold can have
    uint32_t t_in = 0u, t_out = 0u;
    float non_in = INFINITY, non_out = INFINITY;
    if ((int)a.cand_target < deg) {
        const float ln2 = 0.69314718f, target = (float)a.cand_target, fi = (float)n_in, fo = (float)n_out;
        const float s_in = __builtin_amdgcn_rcpf(m_in), s_out = __builtin_amdgcn_rcpf(m_out);
        float kp = target / (ln2 * (fi * s_in + fo * s_out));
#pragma unroll
        for (int it = 0; it < 3; ++it) {
            const float ei = __builtin_amdgcn_exp2f(-kp * s_in), eo = __builtin_amdgcn_exp2f(-kp * s_out);
            const float gv = fi * (1.0f - ei) + fo * (1.0f - eo) - target;
            const float gd = ln2 * (fi * s_in * ei + fo * s_out * eo);
            if (gd > 0.0f) kp -= gv / gd;
        }
        const float pi = __builtin_amdgcn_exp2f(-kp * s_in) * 4294967296.0f, po = __builtin_amdgcn_exp2f(-kp * s_out) * 4294967296.0f;
        t_in = pi >= 4294967040.0f ? 0xFFFFFFFFu : (uint32_t)(pi > 0.0f ? pi : 0.0f);
        t_out = po >= 4294967040.0f ? 0xFFFFFFFFu : (uint32_t)(po > 0.0f ? po : 0.0f);
        if (t_in > 0u && n_in > 0) non_in = approx_clock(t_in - 1u) * m_in;
        if (t_out > 0u && n_out > 0) non_out = approx_clock(t_out - 1u) * m_out;
    }

    const int64_t w_max = (a.n_entries - 1) >> 5;
    int n = 0;
    // 256 slots from j0 on; a slot is a candidate iff its word is at or above its class's threshold (in the row's last
    // stretch: and it is not beyond the row's end).  false: more candidates than the list holds.
    auto stretch = [&](int j0, auto is_last) -> bool {
        constexpr bool LAST = decltype(is_last)::value;
        const int jb = j0 + 4 * lane;
        const u32x4 w = philox4x32_10((uint32_t)jb >> 2, (uint32_t)v, batch, a.ctr3, a.seed_lo, a.seed_hi);
        const uint32_t wr[4] = {w.x, w.y, w.z, w.w};
        const int64_t e = base + min(jb, deg - 1);
        const int64_t wi = e >> 5;
        const uint64_t win = (uint64_t)a.edge_intra[wi] | ((uint64_t)a.edge_intra[min(wi + 1, w_max)] << 32);
        const uint32_t nib = (uint32_t)(win >> (e & 31)) & 0xFu;
        bool c[4];
        uint64_t b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            c[i] = wr[i] >= (((nib >> i) & 1u) ? t_in : t_out);
            if (LAST) c[i] = c[i] && jb + i < deg;
            b[i] = __ballot(c[i]);
        }
        if ((b[0] | b[1] | b[2] | b[3]) == 0) return true;             // (most stretches of a very long row)
        int before = n;
#pragma unroll
        for (int i = 0; i < 4; ++i) before = lanes_below(b[i], before);
        const int total = __popcll(b[0]) + __popcll(b[1]) + __popcll(b[2]) + __popcll(b[3]);
        if (n + total > CAND_CAP) return false;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (c[i]) {
                ckey[before] = wr[i];               // (the key is computed once per candidate, after the loop)
                cslot[before] = (uint32_t)(jb + i) | (((nib >> i) & 1u) << 31);
            }
            before += c[i] ? 1 : 0;
        }
        n += total;
        return true;
    };
    int j0 = 0;
    for (; j0 + 4 * WAVE <= deg; j0 += 4 * WAVE)
        if (!stretch(j0, std::false_type{})) return false;
    if (j0 < deg && !stretch(j0, std::true_type{})) return false;
    if (n < k) return false;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

    // candidate t sits at index t in slot order; a lane owns candidates lane and lane + 64 and turns their random words
    // into keys
    const bool have0 = lane < n, have1 = lane + WAVE < n;
    const uint32_t q0 = cslot[min(lane, n - 1)], q1 = cslot[min(lane + WAVE, n - 1)];
    const bool in0 = q0 >> 31, in1 = q1 >> 31;
    const uint32_t w0 = __float_as_uint(approx_clock(ckey[min(lane, n - 1)]) * (in0 ? m_in : m_out));
    uint32_t w1 = 0x7F800000u;
    if (n > WAVE) w1 = __float_as_uint(approx_clock(ckey[min(lane + WAVE, n - 1)]) * (in1 ? m_in : m_out));
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // every lane has read its words
    if (have0) ckey[lane] = w0;
    if (have1) ckey[lane + WAVE] = w1;
    if (lane < 4) ckey[n + lane] = ~0u;            // pad the keys to a multiple of four with the largest pattern
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    int ra[4] = {0, 0, 0, 0}, rb[4] = {0, 0, 0, 0};
    for (int t0 = 0; t0 < n; t0 += 4) {
        const uint4 kt = *reinterpret_cast<const uint4 *>(ckey + t0);
        const uint32_t ks[4] = {kt.x, kt.y, kt.z, kt.w};
        rank4_below(w0, ks, ra);
        if (n > WAVE) rank4_below(w1, ks, rb);
    }
    const int r0 = ra[0] + ra[1] + ra[2] + ra[3], r1 = rb[0] + rb[1] + rb[2] + rb[3];
    const bool s0 = have0 && r0 < k, s1 = have1 && r1 < k;
    const uint64_t m0 = __ballot(s0), m1 = __ballot(s1);
    // largest kept key and smallest candidate key left out, per class (x: intra, y: inter)
    uint32_t hi_x = max((s0 && in0) ? w0 : 0u, (s1 && in1) ? w1 : 0u), hi_y = max((s0 && !in0) ? w0 : 0u, (s1 && !in1) ? w1 : 0u);
    uint32_t lo_x = min((have0 && !s0 && in0) ? w0 : 0x7F800000u, (have1 && !s1 && in1) ? w1 : 0x7F800000u);
    uint32_t lo_y = min((have0 && !s0 && !in0) ? w0 : 0x7F800000u, (have1 && !s1 && !in1) ? w1 : 0x7F800000u);
#pragma unroll
    for (int o = 32; o; o >>= 1) {
        hi_x = max(hi_x, (uint32_t)__shfl_xor((int)hi_x, o));
        hi_y = max(hi_y, (uint32_t)__shfl_xor((int)hi_y, o));
        lo_x = min(lo_x, (uint32_t)__shfl_xor((int)lo_x, o));
        lo_y = min(lo_y, (uint32_t)__shfl_xor((int)lo_y, o));
    }
    const float hx = __uint_as_float(hi_x), hy = __uint_as_float(hi_y);
    const float lx = fminf(__uint_as_float(lo_x), non_in), ly = fminf(__uint_as_float(lo_y), non_out);
    const bool exact = __popcll(m0) + __popcll(m1) == k && keys_apart(hx, m_in, lx, m_in) && keys_apart(hx, m_in, ly, m_out) &&
                       keys_apart(hy, m_out, lx, m_in) && keys_apart(hy, m_out, ly, m_out);
    if (exact) {
        int32_t *sel_row = sel_row_ptr(a, g, row);
        if (s0) sel_row[__popcll(m0 & lt_mask)] = a.g_indices[base + (q0 & 0x7FFFFFFFu)];
        if (s1) sel_row[__popcll(m0) + __popcll(m1 & lt_mask)] = a.g_indices[base + (q1 & 0x7FFFFFFFu)];
        if (lane == 0) set_row_count(a, g, row, k);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // the buffers are reused by this wave's next long row
    return exact;
}

// (occupancy targets: the weighted instantiation takes 85 registers when left alone, which leaves five waves per SIMD and
// measures 5 % slower on a sampled group than 80 registers -- six waves, as many workgroups as its LDS allows -- with two
// words spilled; the other two fit 64 registers, eight waves: 3 % on a group at p = 1)
template <int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(MODE == 2 ? 6 : 8, 8))) void select_quad_kernel(SelectArgs a)
{
    __shared__ QuadRow rows_s[4][QUAD_ROWS];
    __shared__ int startq_s[4][QUAD_ROWS];
    __shared__ __align__(16) uint32_t klist_s[4][4 * WAVE];
    __shared__ uint32_t cslot_s[4][CAND_CAP];              // (long rows: candidates' slots; passes: the pass's candidates)
    __shared__ uint32_t rowinfo_s[4][QUAD_ROWS];
    __shared__ unsigned long long k64_s[MODE == 2 ? 4 : 1][MODE == 2 ? 4 * WAVE : 1];     // weighted: exact 64-bit keys
    __shared__ __align__(16) uint32_t rowstat_s[MODE == 2 ? 4 : 1][4 * QUAD_ROWS];
    const int wv = (int)threadIdx.x / WAVE;
    unsigned long long *k64 = k64_s[MODE == 2 ? wv : 0];
    uint32_t *rowstat = rowstat_s[MODE == 2 ? wv : 0];
    const int g = blockIdx.y;
    const int n_dst = group_n_dst(a.prev_hdr, g, a.n_roots_total, a.batch_size);
    const int row0 = (int)(blockIdx.x * 4 + wv) * QUAD_ROWS;
    if (row0 >= n_dst) return;
    const int lane = lane_id();

    // lanes 0..QUAD_ROWS-1 fetch one row's node id, adjacency range and output place each
    int32_t mv = 0;
    int64_t mbase = 0;
    int mdeg = 0;
    int32_t *mout = nullptr;
    if (lane < QUAD_ROWS && row0 + lane < n_dst) {
        mv = a.dst_ids[(int64_t)g * a.dst_stride + row0 + lane];
        mbase = a.g_indptr[mv];
        const int64_t d = a.g_indptr[mv + 1] - mbase;
        mdeg = (int)(d > 0x7FFFFFFF ? 0x7FFFFFFF : d);
        mout = sel_row_ptr(a, g, row0 + lane);
        if (mdeg == 0) set_row_count(a, g, row0 + lane, 0);
    }
    const int mq = (mdeg > 0 && mdeg <= QUAD_MAX_DEG) ? (mdeg + 3) >> 2 : 0;
    // Packing of the rows' quads into passes of 64 (a row never straddles two passes): a pass takes, again and again, the
    // first row not yet placed that still fits (first fit over the rows; filling the passes with the rows in their own
    // order leaves them three quarters full on the degree mixes of sampled frontiers, this gets them to ~85 %).  The rows
    // are stored in the order they were placed, so that their first quads ascend and a lane finds its row by bisection;
    // rows without quads (empty, or longer than a pass) come last with a start no lane reaches.
    uint32_t waiting = (uint32_t)__ballot(mq > 0);       // (lanes from QUAD_ROWS on hold no row: mq = 0)
    int my_start = 0x3FFFFFFF, my_place = 0, placed = 0, n_pass = 0;
    while (waiting) {
        int room = WAVE;
        for (;;) {
            const uint32_t fits = (uint32_t)__ballot(mq <= room) & waiting;
            if (!fits) break;
            const int i = __builtin_ctz(fits);
            if (lane == i) { my_start = n_pass * WAVE + (WAVE - room); my_place = placed; }
            room -= (int)rl32((uint32_t)mq, i);
            waiting &= ~(1u << i);
            ++placed;
        }
        ++n_pass;
    }
    {
        const uint32_t rest = (uint32_t)__ballot(lane < QUAD_ROWS && mq == 0);
        if (lane < QUAD_ROWS && mq == 0) my_place = placed + (int)__popc(rest & ((1u << lane) - 1u));
    }
    if (lane < QUAD_ROWS) {
        QuadRow R;
        R.v = mv; R.deg = mdeg; R.startq = my_start; R.nq_row = mq | (lane << 8); R.base = mbase; R.out = mout;
        rows_s[wv][my_place] = R;
        startq_s[wv][my_place] = my_start;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

    uint32_t exact_rows = a.exact_select ? ~0u : 0u;
    if (!a.exact_select)
        for (int p = 0; p < n_pass; ++p)
            exact_rows |= quad_pass<MODE, false>(a, g, row0, p, ~0u, rows_s[wv], startq_s[wv], klist_s[wv], cslot_s[wv], rowinfo_s[wv], k64, rowstat, lane);
    if (exact_rows)
        for (int p = 0; p < n_pass; ++p)
            quad_pass<MODE, true>(a, g, row0, p, exact_rows, rows_s[wv], startq_s[wv], klist_s[wv], cslot_s[wv], rowinfo_s[wv], k64, rowstat, lane);

    // longer rows, one at a time
#pragma unroll 1
    for (int i = 0; i < QUAD_ROWS; ++i) {
        const int deg = (int)rl32((uint32_t)mdeg, i);
        if (deg <= QUAD_MAX_DEG) continue;
        const int32_t v = (int32_t)rl32((uint32_t)mv, i);
        const int64_t base = (int64_t)rl64((uint64_t)mbase, i);
        if constexpr (MODE == 2) {
            if (!a.exact_select && select_big_row_weighted_f32(a, g, row0 + i, v, base, deg, lane, klist_s[wv], cslot_s[wv])) continue;
            if (!a.exact_select &&
                select_big_row_weighted<true>(a, g, row0 + i, v, base, deg, lane, reinterpret_cast<uint2 *>(klist_s[wv]), k64)) continue;
        } else {
            if (!a.exact_select && select_big_row_filtered<MODE == 1>(a, g, row0 + i, v, base, deg, lane, klist_s[wv], cslot_s[wv])) continue;
        }
        select_big_row<MODE, true>(a, g, row0 + i, v, base, deg, MODE >= 1 ? a.comm[v] : 0, lane);
    }
}

// rows of a block that keep min(fanout, degree) neighbours each (no strict mode): the counts need no selection
__global__ __launch_bounds__(256) void row_counts_kernel(const int64_t *__restrict__ g_indptr, const int32_t *__restrict__ dst_ids,
                                                         int64_t dst_stride, const int32_t *__restrict__ prev_hdr, int64_t n_roots_total,
                                                         int32_t batch_size, int32_t fanout, int32_t *__restrict__ cnt, int64_t cnt_stride)
{
    const int g = blockIdx.y;
    const int n_dst = group_n_dst(prev_hdr, g, n_roots_total, batch_size);
    const int row = (int)(blockIdx.x * 256 + threadIdx.x);
    if (row >= n_dst) return;
    const int32_t v = dst_ids[(int64_t)g * dst_stride + row];
    const int64_t d = g_indptr[v + 1] - g_indptr[v];
    cnt[(int64_t)g * cnt_stride + row] = (int32_t)(d < fanout ? d : fanout);
}

// Error of approx_clock against the integer clock over every 32-bit word: out[0] = largest |error| (Q24 units) among the
// words of the upper half (small clocks), out[1] = largest |error| / E over the lower half, out[2] = largest
// |error| / (CLOCK_ERR_ABS + CLOCK_ERR_REL * E) over all words (the selection relies on this being at most 1).
__global__ __launch_bounds__(256) void clock_selftest_kernel(float *out)
{
    float worst_abs = 0.f, worst_rel = 0.f, worst_ratio = 0.f;
    const uint32_t stride = gridDim.x * 256u;
    uint32_t r = blockIdx.x * 256u + threadIdx.x;
    for (uint64_t n = r; n < 0x100000000ull; n += stride, r += stride) {
        const uint32_t exact = exp_clock_q24(r);
        // (the single-precision value times 2^24 and the 30-bit integer are both exact in double precision)
        const float err = (float)fabs((double)approx_clock(r) * 16777216.0 - (double)exact);
        const float ef = (float)exact;
        const bool small_clock = r >= 0x80000000u;
        worst_abs = fmaxf(worst_abs, small_clock ? err : 0.f);
        worst_rel = fmaxf(worst_rel, small_clock ? 0.f : err / ef);
        worst_ratio = fmaxf(worst_ratio, err / (CLOCK_ERR_ABS + CLOCK_ERR_REL * ef));
    }
    // (non-negative floats order like their bit patterns)
    atomicMax(reinterpret_cast<unsigned int *>(out + 0), __float_as_uint(worst_abs));
    atomicMax(reinterpret_cast<unsigned int *>(out + 1), __float_as_uint(worst_rel));
    atomicMax(reinterpret_cast<unsigned int *>(out + 2), __float_as_uint(worst_ratio));
}

struct ScanArgs {
    const int32_t *prev_hdr;
    int64_t n_roots_total;
    int32_t batch_size;
    int32_t mode;          // 0: row counts -> indptr ; 1: new-node counts -> offsets ; 2: source counts -> t_indptr ;
                           // 3: n_fixed values per batch, no header involved
    const int32_t *in;
    int64_t in_stride;
    int32_t *out;
    int64_t out_stride;
    int32_t *out_copy;     // mode 2: fill cursors
    int64_t copy_stride;
    int32_t *hdr;
    int32_t n_fixed;
    const int32_t *tile_before;   // optional (one batch only): sum of everything in front of each tile, computed beforehand
    int32_t cap_src;              // mode 1: entries the frontier array holds
    int64_t *async_status;        // mode 1: status words of the caller's context, or NULL
};

// out[0..n] = exclusive prefix sums of in[0..n) per batch (blockIdx.y).  A workgroup owns one tile of 256 x 16
// elements (blockIdx.x): it first adds up everything in front of its tile (the input is a few hundred KB at most and
// sits in L2, so the tiles of a batch need no hand-off between workgroups and all of them run at once), then scans
// its own tile.  The workgroup of the last tile also writes out[n] and the block header.
constexpr int SCAN_ITEMS = 16;
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;

__global__ __launch_bounds__(SCAN_THREADS) void scan_kernel(ScanArgs a)
{
    __shared__ int lds[17];
    const int g = blockIdx.y;
    int32_t *hdr = a.hdr + (int64_t)g * CR_HDR_WORDS;
    const int n_dst = group_n_dst(a.prev_hdr, g, a.n_roots_total, a.batch_size);
    const int n = a.mode == 3 ? a.n_fixed : (a.mode == 2 ? hdr[CR_HDR_N_SRC] : n_dst);
    const int first = (int)blockIdx.x * SCAN_TILE;
    if (first >= n && blockIdx.x != 0) return;              // (the first workgroup also handles an empty batch)
    const int32_t *in = a.in + (int64_t)g * a.in_stride;
    int32_t *out = a.out + (int64_t)g * a.out_stride;
    int32_t *out_copy = a.out_copy ? a.out_copy + (int64_t)g * a.copy_stride : nullptr;

    int before = 0;                                          // sum of in[0..first)
    if (a.tile_before) {
        before = a.tile_before[blockIdx.x];
    } else if (first > 0) {
        int part = 0;
        int i0 = (int)threadIdx.x;                               // (first is a multiple of the tile size)
        // four tiles' loads in flight at a time: the loop is a chain of round trips to the L2, not of additions
        for (; i0 + 3 * SCAN_TILE < first; i0 += 4 * SCAN_TILE) {
            int x[4][SCAN_ITEMS];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int k = 0; k < SCAN_ITEMS; ++k) x[u][k] = in[i0 + u * SCAN_TILE + k * SCAN_THREADS];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int k = 0; k < SCAN_ITEMS; ++k) part += x[u][k];
        }
        for (; i0 < first; i0 += SCAN_TILE) {
            int x[SCAN_ITEMS];
#pragma unroll
            for (int k = 0; k < SCAN_ITEMS; ++k) x[k] = in[i0 + k * SCAN_THREADS];
#pragma unroll
            for (int k = 0; k < SCAN_ITEMS; ++k) part += x[k];
        }
        block_exclusive_scan<SCAN_THREADS / WAVE>(part, lds, before);
        __syncthreads();                                     // lds is reused below
    }
    // A thread scans sixteen consecutive elements, but the tile travels between memory and the threads through LDS, so
    // that a wave's loads and stores touch consecutive words (a thread reading its own sixteen words straight from memory
    // makes every load instruction touch 64 different cache lines).  Sixteen words are followed by one of padding: the
    // threads' stretches start 17 words apart, on different banks.
    __shared__ int tile[SCAN_TILE + SCAN_TILE / SCAN_ITEMS];
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        const int j = k * SCAN_THREADS + (int)threadIdx.x;
        tile[j + j / SCAN_ITEMS] = first + j < n ? in[first + j] : 0;
    }
    __syncthreads();
    int *mine = tile + (int)threadIdx.x * (SCAN_ITEMS + 1);
    int x[SCAN_ITEMS];
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) x[i] = mine[i];
    int sum = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) sum += x[i];
    int tile_total;
    int run = before + block_exclusive_scan<SCAN_THREADS / WAVE>(sum, lds, tile_total);
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        mine[i] = run;
        run += x[i];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        const int j = k * SCAN_THREADS + (int)threadIdx.x;
        if (first + j < n) {
            const int v = tile[j + j / SCAN_ITEMS];
            out[first + j] = v;
            if (out_copy) out_copy[first + j] = v;
        }
    }
    if (threadIdx.x == 0 && n <= first + SCAN_TILE) {        // the last tile
        const int total = before + tile_total;
        out[n] = total;
        if (a.mode == 0) {
            hdr[CR_HDR_N_DST] = n_dst;
            hdr[CR_HDR_NNZ] = total;
            // a block sampled below a frontier that was cut short is as invalid as that frontier
            hdr[CR_HDR_STATUS] = a.prev_hdr ? a.prev_hdr[(int64_t)g * CR_HDR_WORDS + CR_HDR_STATUS] : 0;
            hdr[4] = hdr[5] = hdr[6] = hdr[7] = 0;
        } else if (a.mode == 1) {
            const int need = n_dst + total;
            if (need > a.cap_src) {        // only possible with capacities below the bound: cut the frontier, mark the block
                hdr[CR_HDR_N_SRC] = a.cap_src;
                atomicOr(&hdr[CR_HDR_STATUS], CR_ASYNC_FRONTIER_OVERFLOW);
                if (a.async_status) {
                    atomicOr(reinterpret_cast<unsigned long long *>(a.async_status), (unsigned long long)CR_ASYNC_FRONTIER_OVERFLOW);
                    atomicMax(reinterpret_cast<long long *>(a.async_status + 1), (long long)need);
                }
            } else {
                hdr[CR_HDR_N_SRC] = need;
            }
        }
    }
}

// For long inputs (the cells of a group-level row order: several hundred thousand) summing everything in front of
// every tile would read the input a hundred times over; two small kernels give the tiles their starting sums instead.
__global__ __launch_bounds__(SCAN_THREADS) void scan_tile_sums_kernel(const int32_t *in, int n, int32_t *tile_sum)
{
    __shared__ int lds[17];
    const int start = (int)blockIdx.x * SCAN_TILE + (int)threadIdx.x;
    int part = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        const int i = start + k * SCAN_THREADS;
        part += i < n ? in[i] : 0;
    }
    int total;
    block_exclusive_scan<SCAN_THREADS / WAVE>(part, lds, total);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
}

// exclusive prefix sums of at most 1024 * 16 tile sums, in place, by one workgroup
__global__ __launch_bounds__(1024) void scan_tile_offsets_kernel(int32_t *tile_sum, int n_tiles)
{
    __shared__ int lds[17];
    int x[16], sum = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int i = (int)threadIdx.x * 16 + k;
        x[k] = i < n_tiles ? tile_sum[i] : 0;
        sum += x[k];
    }
    int total;
    int run = block_exclusive_scan_1024(sum, lds, total);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int i = (int)threadIdx.x * 16 + k;
        if (i < n_tiles) tile_sum[i] = run;
        run += x[k];
    }
}

// ---------------------------------------------------------------------------------------------
// Processing order of a block's destination rows (cr_block_set.row_order): rows grouped by the community of their
// node, a counting sort per batch over at most ORDER_BUCKETS buckets (communities are folded onto the buckets in
// order when there are more).  No global atomics (they resolve at the memory side on this part and cost ~200 ns
// each): a workgroup counts its ORDER_TILE rows per bucket in LDS and writes the counts bucket-major, one prefix sum
// per batch over (bucket, workgroup) gives every workgroup its first position in every bucket, and a second pass
// hands out positions from LDS cursors.  The order inside a (bucket, workgroup) cell follows the LDS atomics and is
// not reproducible, which is fine: the order only says which workgroup of the gather handles a row and when.
// ---------------------------------------------------------------------------------------------
constexpr int ORDER_BUCKETS = 4096;
constexpr int ORDER_TILE = 8192;          // rows per workgroup of 256 threads

struct OrderArgs {
    const int32_t *prev_hdr;
    int64_t n_roots_total;
    int32_t batch_size;
    const int32_t *dst_ids;
    int64_t dst_stride;
    const int32_t *comm;
    int32_t n_comm;
    int32_t n_buckets;        // min(n_comm, ORDER_BUCKETS)
    int32_t n_tiles;          // workgroups per batch (gridDim.x)
    int32_t *cells;           // [n_batches][n_buckets * n_tiles + 1]: counts, then (scanned, in `offsets`) first positions
    int32_t *offsets;
    int32_t *order;
    int64_t order_stride;
    int32_t grouped;          // 1: one order over all batches of the group, entries batch * cap_dst + row, count at the end
    int32_t cap_dst;
    uint16_t *bucket;         // [n_batches][bucket_stride]: a row's bucket, kept from the counting pass for the scatter pass
    int64_t bucket_stride;
};

__device__ __forceinline__ int order_bucket(const OrderArgs &a, int node)
{
    const int cm = a.comm[node];
    const int c = a.n_comm <= ORDER_BUCKETS ? cm : (int)((int64_t)cm * ORDER_BUCKETS / a.n_comm);
    return min(max(c, 0), a.n_buckets - 1);
}

template <bool SCATTER>
__global__ __launch_bounds__(256) void order_pass_kernel(OrderArgs a)
{
    __shared__ int lds[ORDER_BUCKETS];
    const int g = blockIdx.y, tile = blockIdx.x;
    const int n_dst = group_n_dst(a.prev_hdr, g, a.n_roots_total, a.batch_size);
    // per batch: cells [bucket][tile] of this batch; grouped: cells [bucket][batch][tile] of the whole group
    const int col = a.grouped ? g * a.n_tiles + tile : tile;
    const int cols = a.grouped ? (int)gridDim.y * a.n_tiles : a.n_tiles;
    const int64_t cell0 = a.grouped ? 0 : (int64_t)g * ((int64_t)a.n_buckets * a.n_tiles + 1);
    for (int b = threadIdx.x; b < a.n_buckets; b += 256) lds[b] = SCATTER ? a.offsets[cell0 + (int64_t)b * cols + col] : 0;
    if (SCATTER && a.grouped && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0)
        a.order[(int64_t)gridDim.y * a.cap_dst] = a.offsets[(int64_t)a.n_buckets * cols];      // number of entries
    __syncthreads();
    constexpr int PER = ORDER_TILE / 256;
    // the counting pass looks the rows' communities up (one scattered read per row) and leaves their buckets behind; the
    // scatter pass reads those in row order
    uint16_t *kept = a.bucket + (int64_t)g * a.bucket_stride;
    int bkt[PER];
    if (SCATTER) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int r = tile * ORDER_TILE + i * 256 + (int)threadIdx.x;
            bkt[i] = kept[min(r, max(n_dst - 1, 0))];
        }
    } else {
        int node[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int r = tile * ORDER_TILE + i * 256 + (int)threadIdx.x;
            node[i] = a.dst_ids[(int64_t)g * a.dst_stride + min(r, max(n_dst - 1, 0))];
        }
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int r = tile * ORDER_TILE + i * 256 + (int)threadIdx.x;
            bkt[i] = order_bucket(a, node[i]);
            if (r < n_dst) kept[r] = (uint16_t)bkt[i];
        }
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int r = tile * ORDER_TILE + i * 256 + (int)threadIdx.x;
        if (r < n_dst) {
            const int pos = atomicAdd(&lds[bkt[i]], 1);
            if (SCATTER) {
                if (a.grouped) a.order[pos] = g * a.cap_dst + r;
                else a.order[(int64_t)g * a.order_stride + pos] = r;
            }
        }
    }
    if (!SCATTER) {
        __syncthreads();
        for (int b = threadIdx.x; b < a.n_buckets; b += 256) a.cells[cell0 + (int64_t)b * cols + col] = lds[b];
    }
}

// ---------------------------------------------------------------------------------------------
// frontier de-duplication: open-addressing table of (id << 32 | position), min position wins
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t hash_slot(uint32_t id, int bits) { return (id * 0x9E3779B1u) >> (32 - bits); }

__device__ __forceinline__ bool table_insert(unsigned long long *table, int bits, uint32_t id, uint32_t pos)
{
    const uint32_t mask = (1u << bits) - 1u;
    const unsigned long long mine = ((unsigned long long)id << 32) | pos;
    uint32_t h = hash_slot(id, bits);
    for (uint32_t probe = 0; probe <= mask; ++probe) {
        const unsigned long long old = atomicCAS(&table[h], EMPTY, mine);
        if (old == EMPTY) return true;
        if ((uint32_t)(old >> 32) == id) {
            atomicMin(&table[h], mine);
            return true;
        }
        h = (h + 1) & mask;
    }
    return false;
}

// returns the table slot of id (which must be present), or -1
__device__ __forceinline__ int table_find(const unsigned long long *table, int bits, uint32_t id, uint32_t &value)
{
    const uint32_t mask = (1u << bits) - 1u;
    uint32_t h = hash_slot(id, bits);
    for (uint32_t probe = 0; probe <= mask; ++probe) {
        const unsigned long long e = table[h];
        if ((uint32_t)(e >> 32) == id) { value = (uint32_t)e; return (int)h; }
        if (e == EMPTY) break;
        h = (h + 1) & mask;
    }
    value = 0;
    return -1;
}

// clears the first n (even) entries of every batch's table slice
__global__ __launch_bounds__(256) void fill_u64_kernel(unsigned long long *base, int64_t slice_stride, int64_t n, unsigned long long v)
{
    unsigned long long *p = base + (int64_t)blockIdx.y * slice_stride;
    int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 2;
    const int64_t stride = (int64_t)gridDim.x * 256 * 2;
    for (; i + 1 < n; i += stride) *reinterpret_cast<ulonglong2 *>(p + i) = make_ulonglong2(v, v);
    if (i < n) p[i] = v;
}

// Direct-address variant for graphs whose node count is within a small factor of the frontier
// capacity: one int32 per node holding the smallest position seen (INT_MAX = absent).  Insertion is a
// single no-return atomic, look-ups are single loads; touched entries are reset after the hop.
constexpr int32_t ABSENT = 0x7FFFFFFF;

struct DedupArgs {
    int32_t direct;           // 1: table is int32[n_nodes] per batch, 0: open-addressing table
    const int32_t *prev_hdr;
    int64_t n_roots_total;
    int32_t batch_size;
    int32_t fanout;
    int32_t gw;               // lanes per row: power of two >= fanout
    const int32_t *dst_ids;
    int64_t dst_stride;
    const int32_t *sel;
    int64_t sel_stride;
    unsigned long long *table;
    int64_t table_stride;
    int32_t table_bits;
    int32_t *hdr;
    int32_t *src_ids;
    int64_t src_stride;
    int32_t cap_src;          // entries the frontier array holds per batch
    int64_t *async_status;    // status words of the caller's context, or NULL
    int32_t *indptr;
    int64_t indptr_stride;
    int32_t *indices;
    int64_t indices_stride;
    int32_t *gather_ids;      // [G][cap_nnz] or NULL
    int32_t *newcnt;          // [G][cap_dst]
    int32_t *newoff;          // [G][cap_dst+1]
    unsigned long long *newmask;
    int64_t row_stride;       // stride of newcnt / newmask
    int64_t off_stride;
    int32_t *tcount;          // [G][cap_src] or NULL
    int32_t *tfill;           // [G][cap_src+1]
    int64_t t_stride;
    int32_t *t_indptr;
    int64_t t_indptr_stride;
    int32_t *t_indices;
    int32_t *t_tmp;           // [G][cap_nnz] destination rows in arrival order
    int32_t *t_pos;           // [G][cap_nnz] where each edge landed in t_tmp
    int64_t tt_stride;        // stride of t_tmp / t_pos
};

// maps a thread to (row, j): gw lanes per row
#define CR_ROW_LANE()                                                                 \
    const int g = blockIdx.y;                                                         \
    const int n_dst = group_n_dst(a.prev_hdr, g, a.n_roots_total, a.batch_size);      \
    const int64_t gt = (int64_t)blockIdx.x * 256 + threadIdx.x;                       \
    const int row = (int)(gt / a.gw);                                                 \
    const int j = (int)(gt % a.gw);                                                   \
    const int32_t *indptr = a.indptr + (int64_t)g * a.indptr_stride;                  \
    const bool in_row = row < n_dst;                                                  \
    const int rstart = in_row ? indptr[row] : 0;                                      \
    const int k = in_row ? indptr[row + 1] - rstart : 0;                              \
    const bool active = in_row && j < k;                                              \
    const int64_t ell = (int64_t)row * a.fanout + j;                                  \
    unsigned long long *table = a.table + (int64_t)g * a.table_stride;                \
    int32_t *hdr = a.hdr + (int64_t)g * CR_HDR_WORDS;                                 \
    (void)hdr; (void)table; (void)ell; (void)rstart

__global__ __launch_bounds__(256) void insert_kernel(DedupArgs a)
{
    CR_ROW_LANE();
    bool ok = true;
    int32_t *dtab = reinterpret_cast<int32_t *>(table);
    if (in_row && j == 0) {
        const int32_t v = a.dst_ids[(int64_t)g * a.dst_stride + row];
        a.src_ids[(int64_t)g * a.src_stride + row] = v;
        if (a.direct) atomicMin(&dtab[v], row);
        else ok = table_insert(table, a.table_bits, (uint32_t)v, (uint32_t)row);
    }
    if (active) {
        const int32_t u = a.sel[(int64_t)g * a.sel_stride + ell];
        if (a.direct) atomicMin(&dtab[u], (int32_t)(n_dst + ell));
        else ok = table_insert(table, a.table_bits, (uint32_t)u, (uint32_t)(n_dst + ell)) && ok;
    }
    if (!ok) {
        atomicOr(&hdr[CR_HDR_STATUS], CR_ASYNC_TABLE_FULL);
        if (a.async_status) atomicOr(reinterpret_cast<unsigned long long *>(a.async_status), (unsigned long long)CR_ASYNC_TABLE_FULL);
    }
}

// which chosen neighbours are seen here for the first time (and are not destination nodes)
__global__ __launch_bounds__(256) void mark_new_kernel(DedupArgs a)
{
    CR_ROW_LANE();
    bool isnew = false;
    if (active) {
        const int32_t u = a.sel[(int64_t)g * a.sel_stride + ell];
        if (a.direct) {
            isnew = reinterpret_cast<const int32_t *>(table)[u] == (int32_t)(n_dst + ell);
        } else {
            uint32_t pos;
            const int h = table_find(table, a.table_bits, (uint32_t)u, pos);
            isnew = h >= 0 && pos == (uint32_t)(n_dst + ell);
        }
    }
    const uint64_t m = __ballot(isnew);
    if (in_row && j == 0) {
        const int sub = lane_id() / a.gw;
        const uint64_t rowmask = a.gw == 64 ? m : ((m >> (sub * a.gw)) & ((1ull << a.gw) - 1ull));
        a.newcnt[(int64_t)g * a.row_stride + row] = __popcll(rowmask);
        a.newmask[(int64_t)g * a.row_stride + row] = rowmask;
    }
}

// new nodes get consecutive frontier positions after the destination nodes; the table entry of a
// node now holds its position in the frontier
__global__ __launch_bounds__(256) void assign_kernel(DedupArgs a)
{
    CR_ROW_LANE();
    if (a.tcount) {   // clear the per-source counters of the transposed block
        const int n_src = hdr[CR_HDR_N_SRC];
        int32_t *tc = a.tcount + (int64_t)g * a.t_stride;
        for (int64_t i = gt; i < n_src; i += (int64_t)gridDim.x * 256) tc[i] = 0;
    }
    if (!active) return;
    const uint64_t rowmask = a.newmask[(int64_t)g * a.row_stride + row];
    if (!((rowmask >> j) & 1ull)) return;
    const int32_t u = a.sel[(int64_t)g * a.sel_stride + ell];
    const int local = n_dst + a.newoff[(int64_t)g * a.off_stride + row] + __popcll(rowmask & ((1ull << j) - 1ull));
    if (local < a.cap_src) a.src_ids[(int64_t)g * a.src_stride + local] = u;      // (a frontier cut short: the block is marked invalid)
    if (a.direct) {
        reinterpret_cast<int32_t *>(table)[u] = local;
    } else {
        uint32_t pos;
        const int h = table_find(table, a.table_bits, (uint32_t)u, pos);
        if (h >= 0) table[h] = ((unsigned long long)(uint32_t)u << 32) | (uint32_t)local;
    }
}

__global__ __launch_bounds__(256) void relabel_kernel(DedupArgs a)
{
    CR_ROW_LANE();
    if (!active) return;
    const int32_t u = a.sel[(int64_t)g * a.sel_stride + ell];
    uint32_t local;
    if (a.direct) local = (uint32_t)reinterpret_cast<const int32_t *>(table)[u];
    else table_find(table, a.table_bits, (uint32_t)u, local);
    if (local >= (uint32_t)a.cap_src) local = 0;       // only in a block that is marked invalid: keeps every later access in range
    a.indices[(int64_t)g * a.indices_stride + rstart + j] = (int32_t)local;
    if (a.gather_ids) a.gather_ids[(int64_t)g * a.indices_stride + rstart + j] = u;
    if (a.tcount) atomicAdd(&a.tcount[(int64_t)g * a.t_stride + local], 1);
}

// input-side block left in global ids: compact the chosen neighbours into CSR order, copy the
// destination nodes into the head of the frontier, mark the frontier size as not computed
__global__ __launch_bounds__(256) void compact_ids_kernel(DedupArgs a)
{
    CR_ROW_LANE();
    if (blockIdx.x == 0 && threadIdx.x == 0) hdr[CR_HDR_N_SRC] = -1;
    if (in_row && j == 0) a.src_ids[(int64_t)g * a.src_stride + row] = a.dst_ids[(int64_t)g * a.dst_stride + row];
    if (!active) return;
    a.gather_ids[(int64_t)g * a.indices_stride + rstart + j] = a.sel[(int64_t)g * a.sel_stride + ell];
}

// the same when the selection has already written the ids in place: only the destination nodes are left to copy, one
// thread per row
__global__ __launch_bounds__(256) void frontier_head_kernel(DedupArgs a)
{
    const int g = blockIdx.y;
    const int n_dst = group_n_dst(a.prev_hdr, g, a.n_roots_total, a.batch_size);
    const int row = (int)(blockIdx.x * 256 + threadIdx.x);
    if (blockIdx.x == 0 && threadIdx.x == 0) a.hdr[(int64_t)g * CR_HDR_WORDS + CR_HDR_N_SRC] = -1;
    if (row < n_dst) a.src_ids[(int64_t)g * a.src_stride + row] = a.dst_ids[(int64_t)g * a.dst_stride + row];
}

// direct-address table: put the entries this hop touched back to "absent"
__global__ __launch_bounds__(256) void reset_kernel(DedupArgs a)
{
    const int g = blockIdx.y;
    const int n_src = a.hdr[(int64_t)g * CR_HDR_WORDS + CR_HDR_N_SRC];
    int32_t *dtab = reinterpret_cast<int32_t *>(a.table + (int64_t)g * a.table_stride);
    const int32_t *src = a.src_ids + (int64_t)g * a.src_stride;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_src; i += (int64_t)gridDim.x * 256) dtab[src[i]] = ABSENT;
}

// transposed block: scatter the destination row of every edge into its source's segment in arrival
// order, then rank inside the segment so that the stored order is ascending (hence reproducible)
__global__ __launch_bounds__(256) void t_fill_kernel(DedupArgs a)
{
    CR_ROW_LANE();
    if (!active) return;
    const int64_t e = (int64_t)g * a.indices_stride + rstart + j;
    const int local = a.indices[e];
    const int p = atomicAdd(&a.tfill[(int64_t)g * a.t_stride + local], 1);
    a.t_tmp[(int64_t)g * a.tt_stride + p] = row;
    a.t_pos[(int64_t)g * a.tt_stride + rstart + j] = p;
}

__global__ __launch_bounds__(256) void t_rank_kernel(DedupArgs a)
{
    CR_ROW_LANE();
    if (!active) return;
    const int64_t e = (int64_t)g * a.indices_stride + rstart + j;
    const int local = a.indices[e];
    const int32_t *tp = a.t_indptr + (int64_t)g * a.t_indptr_stride;
    const int s0 = tp[local], s1 = tp[local + 1];
    const int32_t *tmp = a.t_tmp + (int64_t)g * a.tt_stride;
    const int mine = a.t_pos[(int64_t)g * a.tt_stride + rstart + j];
    int rank = 0;
    for (int q = s0; q < s1; ++q) {
        const int r = tmp[q];
        rank += (r < row || (r == row && q < mine)) ? 1 : 0;
    }
    a.t_indices[(int64_t)g * a.indices_stride + s0 + rank] = row;
}

// one thread per 32 adjacency entries: find the row of the first one, then walk
__global__ __launch_bounds__(256) void edge_classes_kernel(const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                                                           const int32_t *__restrict__ comm, int64_t n_nodes, int64_t n_entries,
                                                           uint32_t *__restrict__ out)
{
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t e0 = w * 32;
    if (e0 >= n_entries) return;
    int64_t lo = 0, hi = n_nodes;            // last row r with indptr[r] <= e0
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (indptr[mid] <= e0) lo = mid; else hi = mid;
    }
    int64_t r = lo, r_end = indptr[r + 1];
    int32_t cr = comm[r];
    uint32_t bits = 0;
    for (int b = 0; b < 32 && e0 + b < n_entries; ++b) {
        const int64_t e = e0 + b;
        while (e >= r_end) { ++r; r_end = indptr[r + 1]; cr = comm[r]; }
        if (comm[indices[e]] == cr) bits |= 1u << b;
    }
    out[w] = bits;
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct SamplePlan {
    int L;
    int32_t cap_dst[CR_MAX_LAYERS], cap_src[CR_MAX_LAYERS], cap_nnz[CR_MAX_LAYERS];
    int table_bits[CR_MAX_LAYERS];
    int64_t max_dst = 0, max_src_t = 0, max_nnz = 0, max_nnz_t = 0, max_table = 0;
    bool direct = false;      // direct-address de-duplication table (one int32 per node) instead of hashing
    int64_t table_stride = 0; // per batch, in 8-byte units
    // workspace slices
    int32_t *sel, *cnt, *newoff, *tcount, *tfill, *t_tmp, *t_pos, *order_hist, *order_cursor, *order_tiles;
    uint16_t *order_bucket;
    unsigned long long *newmask, *table;
    size_t bytes;
};

static cr_status make_plan(const cr_sample_cfg *cfg, int64_t n_nodes, int32_t batch_size, int32_t n_batches,
                           void *ws, SamplePlan &p)
{
    CR_REQUIRE(cfg != nullptr, CR_ERR_INVALID_ARG, "cfg is NULL");
    CR_REQUIRE(cfg->n_layers >= 1 && cfg->n_layers <= CR_MAX_LAYERS, CR_ERR_INVALID_ARG,
               "n_layers = %d outside 1..%d", cfg->n_layers, CR_MAX_LAYERS);
    CR_REQUIRE(n_nodes >= 1 && n_nodes <= 0x7FFFFFFF, CR_ERR_INVALID_ARG, "n_nodes must be in 1..2^31-1");
    CR_REQUIRE(batch_size >= 1, CR_ERR_INVALID_ARG, "batch_size must be positive");
    CR_REQUIRE(n_batches >= 1 && n_batches <= 65535, CR_ERR_INVALID_ARG, "n_batches must be in 1..65535");
    CR_REQUIRE(cfg->p_intra >= 0.5 && cfg->p_intra <= 1.0, CR_ERR_INVALID_ARG, "p_intra = %g outside [0.5, 1]", cfg->p_intra);
    CR_REQUIRE(cfg->epoch < (1u << 24), CR_ERR_INVALID_ARG, "epoch must be below 2^24");
    CR_REQUIRE(!((cfg->flags & CR_SAMPLE_TRANSPOSE_INPUT) && (cfg->flags & CR_SAMPLE_INPUT_GLOBAL_IDS)), CR_ERR_INVALID_ARG,
               "CR_SAMPLE_TRANSPOSE_INPUT and CR_SAMPLE_INPUT_GLOBAL_IDS exclude each other");
    p.L = cfg->n_layers;
    int64_t dst = batch_size;
    for (int l = p.L - 1; l >= 0; --l) {
        const int f = cfg->fanout[l];
        CR_REQUIRE(f >= 1 && f <= CR_MAX_FANOUT, CR_ERR_INVALID_ARG, "fanout[%d] = %d outside 1..%d", l, f, CR_MAX_FANOUT);
        const int64_t nnz = dst * f;
        int64_t src = dst * (1 + f);
        if (src > n_nodes) src = n_nodes;
        if (src < dst) src = dst;
        CR_REQUIRE(nnz <= 0x7FFFFFFF / 2, CR_ERR_UNSUPPORTED, "layer %d would hold %lld edges per batch", l, (long long)nnz);
        p.cap_dst[l] = (int32_t)dst;
        p.cap_src[l] = (int32_t)src;
        p.cap_nnz[l] = (int32_t)nnz;
        int bits = 4;
        while ((1ll << bits) < 2 * src) ++bits;
        CR_REQUIRE(bits <= 31, CR_ERR_UNSUPPORTED, "layer %d frontier too large for the de-duplication table", l);
        p.table_bits[l] = bits;
        p.max_dst = dst > p.max_dst ? dst : p.max_dst;
        p.max_nnz = nnz > p.max_nnz ? nnz : p.max_nnz;
        p.max_table = (1ll << bits) > p.max_table ? (1ll << bits) : p.max_table;
        if (l >= 1 || (cfg->flags & CR_SAMPLE_TRANSPOSE_INPUT)) {
            p.max_src_t = src > p.max_src_t ? src : p.max_src_t;
            p.max_nnz_t = nnz > p.max_nnz_t ? nnz : p.max_nnz_t;
        }
        dst = src;
    }
    const size_t G = (size_t)n_batches;
    Carver c(ws);
    p.sel = c.take<int32_t>(G * p.max_nnz);
    p.cnt = c.take<int32_t>(G * p.max_dst);
    p.newoff = c.take<int32_t>(G * (p.max_dst + 1));
    p.newmask = c.take<unsigned long long>(G * p.max_dst);
    p.direct = n_nodes <= 4 * p.max_table && !(cfg->flags & CR_SAMPLE_HASH_DEDUP);
    p.table_stride = p.direct ? round_up(ceil_div(n_nodes, 2), 2) : p.max_table;
    p.table = c.take<unsigned long long>(G * (size_t)p.table_stride);
    p.tcount = c.take<int32_t>(G * (p.max_src_t + 1));
    p.tfill = c.take<int32_t>(G * (p.max_src_t + 1));
    p.t_tmp = c.take<int32_t>(G * (p.max_nnz_t + 1));
    p.t_pos = c.take<int32_t>(G * (p.max_nnz_t + 1));
    if (cfg->flags & CR_SAMPLE_ROW_ORDER) {          // cells of the row-order counting sort, sized for 4096 buckets
        const size_t cells = (size_t)ORDER_BUCKETS * (size_t)ceil_div(p.max_dst, ORDER_TILE) + 1;
        p.order_hist = c.take<int32_t>(G * cells);
        p.order_cursor = c.take<int32_t>(G * cells);
        p.order_tiles = c.take<int32_t>(16384);
        p.order_bucket = c.take<uint16_t>(G * p.max_dst);
    } else {
        p.order_hist = p.order_cursor = p.order_tiles = nullptr;
        p.order_bucket = nullptr;
    }
    p.bytes = c.bytes();
    return CR_OK;
}

}  // namespace cr

using namespace cr;

extern "C" cr_status cr_block_capacities(const cr_sample_cfg *cfg, int64_t n_nodes, int32_t batch_size,
                                         int32_t *cap_dst, int32_t *cap_src, int32_t *cap_nnz)
{
    SamplePlan p;
    cr_status st = make_plan(cfg, n_nodes, batch_size, 1, nullptr, p);
    if (st != CR_OK) return st;
    CR_REQUIRE(cap_dst && cap_src && cap_nnz, CR_ERR_INVALID_ARG, "output arrays must not be NULL");
    for (int l = 0; l < p.L; ++l) {
        cap_dst[l] = p.cap_dst[l];
        cap_src[l] = p.cap_src[l];
        cap_nnz[l] = p.cap_nnz[l];
    }
    return CR_OK;
}

extern "C" cr_status cr_sample_blocks_workspace_bytes(const cr_sample_cfg *cfg, int64_t n_nodes, int32_t batch_size,
                                                      int32_t n_batches, size_t *bytes)
{
    SamplePlan p;
    cr_status st = make_plan(cfg, n_nodes, batch_size, n_batches, nullptr, p);
    if (st != CR_OK) return st;
    CR_REQUIRE(bytes != nullptr, CR_ERR_INVALID_ARG, "bytes is NULL");
    *bytes = p.bytes;
    return CR_OK;
}

extern "C" cr_status cr_selftest_clock_approximation(float *result, void *stream)
{
    CR_REQUIRE(result != nullptr, CR_ERR_INVALID_ARG, "result must not be NULL");
    if (dry_run()) return CR_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(fill_u64_kernel, dim3(1), dim3(256), 0, s, reinterpret_cast<unsigned long long *>(result), (int64_t)0, (int64_t)2, 0ull);
    hipLaunchKernelGGL(clock_selftest_kernel, dim3(4096), dim3(256), 0, s, result);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_sample_blocks_dedup_table(const cr_sample_cfg *cfg, int64_t n_nodes, int32_t batch_size, int32_t *kind)
{
    SamplePlan p;
    cr_status st = make_plan(cfg, n_nodes, batch_size, 1, nullptr, p);
    if (st != CR_OK) return st;
    CR_REQUIRE(kind != nullptr, CR_ERR_INVALID_ARG, "kind is NULL");
    *kind = p.direct ? CR_DEDUP_DIRECT : CR_DEDUP_HASH;
    return CR_OK;
}

extern "C" cr_status cr_graph_edge_classes(const cr_graph *graph, uint32_t *edge_intra, void *stream)
{
    CR_REQUIRE(graph != nullptr, CR_ERR_INVALID_ARG, "graph is NULL");
    CR_REQUIRE(graph->indptr && graph->indices && graph->comm, CR_ERR_INVALID_ARG, "graph has a NULL array");
    CR_REQUIRE(graph->n_nodes >= 1 && graph->n_entries >= 0, CR_ERR_INVALID_ARG, "graph sizes must be positive");
    CR_REQUIRE(edge_intra != nullptr, CR_ERR_INVALID_ARG, "edge_intra must not be NULL");
    if (dry_run() || graph->n_entries == 0) return CR_OK;
    const int64_t words = ceil_div(graph->n_entries, 32);
    hipLaunchKernelGGL(edge_classes_kernel, dim3((unsigned)ceil_div(words, 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       graph->indptr, graph->indices, graph->comm, graph->n_nodes, graph->n_entries, edge_intra);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_sample_blocks(const cr_graph *graph, const cr_sample_cfg *cfg, const int32_t *roots,
                                      int64_t n_roots_total, int32_t batch_size, int32_t n_batches, void *ws,
                                      size_t ws_bytes, cr_block_set *layers, void *stream)
{
    CR_REQUIRE(graph != nullptr, CR_ERR_INVALID_ARG, "graph is NULL");
    CR_REQUIRE(graph->indptr && graph->indices && graph->comm, CR_ERR_INVALID_ARG, "graph has a NULL array");
    CR_REQUIRE(graph->n_comm >= 1, CR_ERR_INVALID_ARG, "n_comm must be positive");
    SamplePlan p;
    cr_status st = make_plan(cfg, graph->n_nodes, batch_size, n_batches, ws, p);
    if (st != CR_OK) return st;
    CR_REQUIRE(roots != nullptr && layers != nullptr, CR_ERR_INVALID_ARG, "roots / layers must not be NULL");
    CR_REQUIRE(n_roots_total > (int64_t)(n_batches - 1) * batch_size && n_roots_total <= (int64_t)n_batches * batch_size,
               CR_ERR_INVALID_ARG, "n_roots_total = %lld does not fill %d batches of %d (only the last may be short)",
               (long long)n_roots_total, n_batches, batch_size);
    CR_REQUIRE((uint64_t)cfg->first_batch + (uint64_t)n_batches <= 0xFFFFFFFFull, CR_ERR_INVALID_ARG, "batch index overflows 32 bits");
    CR_REQUIRE(ws != nullptr && aligned16(ws), CR_ERR_INVALID_ARG, "workspace must be a 16-byte aligned device pointer");
    CR_REQUIRE(ws_bytes >= p.bytes, CR_ERR_CAPACITY, "workspace of %zu bytes, %zu needed", ws_bytes, p.bytes);
    for (int l = 0; l < p.L; ++l) {
        const cr_block_set &b = layers[l];
        CR_REQUIRE(b.n_batches == n_batches && b.fanout == cfg->fanout[l], CR_ERR_INVALID_ARG,
                   "layers[%d]: n_batches / fanout do not match the request", l);
        if (!(cfg->flags & CR_SAMPLE_SMALL_FRONTIER)) {
            CR_REQUIRE(b.cap_dst >= p.cap_dst[l] && b.cap_src >= p.cap_src[l] && b.cap_nnz >= p.cap_nnz[l], CR_ERR_CAPACITY,
                       "layers[%d]: capacities (%d, %d, %d) below the bound (%d, %d, %d)", l, b.cap_dst, b.cap_src, b.cap_nnz,
                       p.cap_dst[l], p.cap_src[l], p.cap_nnz[l]);
        } else {
            // the rows of layer l are the frontier of layer l+1, which is cut at that layer's cap_src
            const int64_t rows = l == p.L - 1 ? (int64_t)batch_size
                                              : (layers[l + 1].cap_src < p.cap_dst[l] ? layers[l + 1].cap_src : p.cap_dst[l]);
            CR_REQUIRE(b.cap_dst >= rows && b.cap_src >= b.cap_dst && (int64_t)b.cap_nnz >= rows * cfg->fanout[l], CR_ERR_CAPACITY,
                       "layers[%d]: capacities (%d, %d, %d) cannot hold %lld rows of fanout %d and their own ids", l, b.cap_dst,
                       b.cap_src, b.cap_nnz, (long long)rows, cfg->fanout[l]);
        }
        CR_REQUIRE(b.hdr && b.src_ids && b.indptr && b.indices, CR_ERR_INVALID_ARG, "layers[%d] has a NULL array", l);
        CR_REQUIRE((b.t_indptr == nullptr) == (b.t_indices == nullptr), CR_ERR_INVALID_ARG,
                   "layers[%d]: t_indptr and t_indices must be given together", l);
        CR_REQUIRE(l >= 1 || b.t_indptr == nullptr || (cfg->flags & CR_SAMPLE_TRANSPOSE_INPUT), CR_ERR_UNSUPPORTED,
                   "layer 0 takes a transposed block only with CR_SAMPLE_TRANSPOSE_INPUT");
        CR_REQUIRE(l >= 1 || !(cfg->flags & CR_SAMPLE_INPUT_GLOBAL_IDS) || b.gather_ids != nullptr, CR_ERR_INVALID_ARG,
                   "CR_SAMPLE_INPUT_GLOBAL_IDS needs layers[0].gather_ids");
        CR_REQUIRE((b.row_order == nullptr && b.group_order == nullptr) || (cfg->flags & CR_SAMPLE_ROW_ORDER), CR_ERR_INVALID_ARG,
                   "layers[%d].row_order / group_order need CR_SAMPLE_ROW_ORDER (it sizes the workspace)", l);
        CR_REQUIRE(b.group_order == nullptr || (int64_t)n_batches * b.cap_dst < 0x7FFFFFFF, CR_ERR_UNSUPPORTED,
                   "layers[%d].group_order: n_batches * cap_dst does not fit 31 bits", l);
    }
    if (dry_run()) return CR_OK;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t q_in = (uint32_t)llround(cfg->p_intra * 65536.0);
    const uint32_t q_out = 65536u - q_in;
    const dim3 blk(256);
    for (int l = p.L - 1; l >= 0; --l) {
        const cr_block_set &b = layers[l];
        const int f = cfg->fanout[l];
        const bool root = l == p.L - 1;
        const int32_t *prev_hdr = root ? nullptr : layers[l + 1].hdr;
        const int32_t *dst_ids = root ? roots : layers[l + 1].src_ids;
        const int64_t dst_stride = root ? batch_size : layers[l + 1].cap_src;
        const int cap_dst = p.cap_dst[l];

        SelectArgs sa;
        sa.g_indptr = graph->indptr; sa.g_indices = graph->indices; sa.comm = graph->comm;
        sa.edge_intra = graph->edge_intra; sa.n_entries = graph->n_entries;
        sa.dst_ids = dst_ids; sa.dst_stride = dst_stride; sa.prev_hdr = prev_hdr;
        sa.n_roots_total = n_roots_total; sa.batch_size = batch_size; sa.fanout = f;
        sa.q_in = q_in; sa.q_out = q_out;
        sa.strict_p1 = (q_out == 0 && (cfg->flags & CR_SAMPLE_STRICT_INTRA)) ? 1u : 0u;
        sa.seed_lo = (uint32_t)cfg->seed; sa.seed_hi = (uint32_t)(cfg->seed >> 32);
        sa.ctr3 = (cfg->epoch << 8) | (DOMAIN_NEIGHBOUR << 4) | (uint32_t)l;
        sa.first_batch = cfg->first_batch;
        sa.sel = p.sel; sa.sel_stride = p.max_nnz; sa.cnt = p.cnt; sa.cnt_stride = p.max_dst;
        {   // fanout + four standard deviations and a little more: short about once in a few thousand long rows (those
            // take the general path), never near the buffer's end
            int target = f + (int)(4.0 * sqrt((double)f)) + 4;
            sa.cand_target = (uint32_t)(target > 96 ? 96 : target);
        }
        sa.exact_select = (cfg->flags & CR_SAMPLE_EXACT_RANKING) ? 1u : 0u;
        const dim3 sel_grid((unsigned)ceil_div(cap_dst, 4 * SEL_ROWS), n_batches);
        const dim3 quad_grid((unsigned)ceil_div(cap_dst, 4 * QUAD_ROWS), n_batches);
        // Input-side block in global ids, every row keeps min(fanout, degree) neighbours: counts and row pointers first
        // (they need no selection), then the selection writes the chosen ids straight into the block.
        const bool direct_out = l == 0 && (cfg->flags & CR_SAMPLE_INPUT_GLOBAL_IDS) && !sa.strict_p1;
        ScanArgs sc;
        sc.tile_before = nullptr;
        sc.prev_hdr = prev_hdr; sc.n_roots_total = n_roots_total; sc.batch_size = batch_size;
        sc.mode = 0; sc.in = p.cnt; sc.in_stride = p.max_dst; sc.out = b.indptr; sc.out_stride = b.cap_dst + 1;
        sc.out_copy = nullptr; sc.copy_stride = 0; sc.hdr = b.hdr;
        sc.cap_src = b.cap_src; sc.async_status = async_status();
        const dim3 scan_grid((unsigned)ceil_div(cap_dst, SCAN_TILE), n_batches);
        sa.out_indptr = nullptr; sa.out_indptr_stride = 0; sa.out_ids = nullptr; sa.out_stride = 0;
        if (direct_out) {
            hipLaunchKernelGGL(row_counts_kernel, dim3((unsigned)ceil_div(cap_dst, 256), n_batches), blk, 0, s, graph->indptr, dst_ids, dst_stride,
                               prev_hdr, n_roots_total, batch_size, f, p.cnt, (int64_t)p.max_dst);
            hipLaunchKernelGGL(scan_kernel, scan_grid, dim3(SCAN_THREADS), 0, s, sc);
            sa.out_indptr = b.indptr; sa.out_indptr_stride = b.cap_dst + 1; sa.out_ids = b.gather_ids; sa.out_stride = b.cap_nnz;
        }
        if (q_in == q_out) hipLaunchKernelGGL(select_quad_kernel<0>, quad_grid, blk, 0, s, sa);
        else if (q_out == 0 && graph->edge_intra) hipLaunchKernelGGL(select_quad_kernel<1>, quad_grid, blk, 0, s, sa);
        else if (graph->edge_intra) hipLaunchKernelGGL(select_quad_kernel<2>, quad_grid, blk, 0, s, sa);
        else if (q_out == 0) hipLaunchKernelGGL(select_kernel<1>, sel_grid, blk, 0, s, sa);
        else hipLaunchKernelGGL(select_kernel<2>, sel_grid, blk, 0, s, sa);

        for (int grouped = 0; grouped < 2; ++grouped) {       // processing orders of this layer's destination rows
            int32_t *order = grouped ? b.group_order : b.row_order;
            if (!order) continue;
            OrderArgs oa;
            oa.prev_hdr = prev_hdr; oa.n_roots_total = n_roots_total; oa.batch_size = batch_size;
            oa.dst_ids = dst_ids; oa.dst_stride = dst_stride; oa.comm = graph->comm; oa.n_comm = graph->n_comm;
            oa.n_buckets = graph->n_comm < ORDER_BUCKETS ? graph->n_comm : ORDER_BUCKETS;
            oa.n_tiles = (int32_t)ceil_div(cap_dst, ORDER_TILE);
            oa.cells = p.order_hist; oa.offsets = p.order_cursor; oa.order = order; oa.order_stride = b.cap_dst;
            oa.grouped = grouped; oa.cap_dst = b.cap_dst;
            oa.bucket = p.order_bucket; oa.bucket_stride = p.max_dst;
            const int n_cells = oa.n_buckets * oa.n_tiles * (grouped ? n_batches : 1);
            const dim3 og((unsigned)oa.n_tiles, n_batches);
            hipLaunchKernelGGL(order_pass_kernel<false>, og, blk, 0, s, oa);
            ScanArgs so;
            so.prev_hdr = prev_hdr; so.n_roots_total = n_roots_total; so.batch_size = batch_size;
            so.mode = 3; so.n_fixed = n_cells; so.in = p.order_hist; so.in_stride = n_cells + 1; so.out = p.order_cursor;
            so.out_stride = n_cells + 1; so.out_copy = nullptr; so.copy_stride = 0; so.hdr = b.hdr;
            so.tile_before = nullptr; so.cap_src = 0; so.async_status = nullptr;
            const int scan_tiles = (int)ceil_div(n_cells, SCAN_TILE);
            if (grouped && scan_tiles > 8 && scan_tiles <= 16384) {
                hipLaunchKernelGGL(scan_tile_sums_kernel, dim3((unsigned)scan_tiles), dim3(SCAN_THREADS), 0, s, p.order_hist, n_cells, p.order_tiles);
                hipLaunchKernelGGL(scan_tile_offsets_kernel, dim3(1), dim3(1024), 0, s, p.order_tiles, scan_tiles);
                so.tile_before = p.order_tiles;
            }
            hipLaunchKernelGGL(scan_kernel, dim3((unsigned)scan_tiles, grouped ? 1 : n_batches), dim3(SCAN_THREADS), 0, s, so);
            hipLaunchKernelGGL(order_pass_kernel<true>, og, blk, 0, s, oa);
        }

        if (!direct_out) hipLaunchKernelGGL(scan_kernel, scan_grid, dim3(SCAN_THREADS), 0, s, sc);

        DedupArgs da;
        da.prev_hdr = prev_hdr; da.n_roots_total = n_roots_total; da.batch_size = batch_size; da.fanout = f;
        da.gw = f <= 16 ? 16 : (f <= 32 ? 32 : 64);
        da.dst_ids = dst_ids; da.dst_stride = dst_stride; da.sel = p.sel; da.sel_stride = p.max_nnz;
        da.direct = p.direct ? 1 : 0;
        da.table = p.table; da.table_stride = p.table_stride; da.table_bits = p.table_bits[l];
        da.hdr = b.hdr; da.src_ids = b.src_ids; da.src_stride = b.cap_src; da.cap_src = b.cap_src; da.async_status = async_status();
        da.indptr = b.indptr; da.indptr_stride = b.cap_dst + 1; da.indices = b.indices; da.indices_stride = b.cap_nnz; da.gather_ids = b.gather_ids;
        da.newcnt = p.cnt; da.newoff = p.newoff; da.newmask = p.newmask; da.row_stride = p.max_dst; da.off_stride = p.max_dst + 1;
        const dim3 grid((unsigned)ceil_div((int64_t)cap_dst * da.gw, 256), n_batches);
        if (l == 0 && (cfg->flags & CR_SAMPLE_INPUT_GLOBAL_IDS)) {
            da.tcount = nullptr; da.tfill = nullptr; da.t_stride = 0; da.t_indptr = nullptr; da.t_indptr_stride = 0;
            da.t_indices = nullptr; da.t_tmp = nullptr; da.t_pos = nullptr; da.tt_stride = 0;
            if (direct_out) hipLaunchKernelGGL(frontier_head_kernel, dim3((unsigned)ceil_div(cap_dst, 256), n_batches), blk, 0, s, da);
            else hipLaunchKernelGGL(compact_ids_kernel, grid, blk, 0, s, da);
            continue;
        }

        if (!p.direct) {
            const int64_t table_size = 1ll << p.table_bits[l];
            hipLaunchKernelGGL(fill_u64_kernel, dim3((unsigned)(ceil_div(table_size, 512) < 4096 ? ceil_div(table_size, 512) : 4096), n_batches), blk, 0, s,
                               p.table, p.table_stride, table_size, EMPTY);
        } else if (root) {   // once per call; every hop puts the entries it touched back
            hipLaunchKernelGGL(fill_u64_kernel, dim3((unsigned)(ceil_div(p.table_stride, 512) < 4096 ? ceil_div(p.table_stride, 512) : 4096), n_batches), blk, 0, s,
                               p.table, p.table_stride, p.table_stride, 0x7FFFFFFF7FFFFFFFull);
        }

        const bool tr = b.t_indptr != nullptr;
        da.tcount = tr ? p.tcount : nullptr; da.tfill = p.tfill; da.t_stride = p.max_src_t + 1;
        da.t_indptr = b.t_indptr; da.t_indptr_stride = b.cap_src + 1; da.t_indices = b.t_indices;
        da.t_tmp = p.t_tmp; da.t_pos = p.t_pos; da.tt_stride = p.max_nnz_t + 1;
        hipLaunchKernelGGL(insert_kernel, grid, blk, 0, s, da);
        hipLaunchKernelGGL(mark_new_kernel, grid, blk, 0, s, da);
        sc.mode = 1; sc.in = p.cnt; sc.in_stride = p.max_dst; sc.out = p.newoff; sc.out_stride = p.max_dst + 1;
        hipLaunchKernelGGL(scan_kernel, scan_grid, dim3(SCAN_THREADS), 0, s, sc);
        hipLaunchKernelGGL(assign_kernel, grid, blk, 0, s, da);
        hipLaunchKernelGGL(relabel_kernel, grid, blk, 0, s, da);
        if (p.direct)
            hipLaunchKernelGGL(reset_kernel, dim3((unsigned)ceil_div(p.cap_src[l], 1024), n_batches), blk, 0, s, da);
        if (tr) {
            sc.mode = 2; sc.in = p.tcount; sc.in_stride = p.max_src_t + 1; sc.out = b.t_indptr; sc.out_stride = b.cap_src + 1;
            sc.out_copy = p.tfill; sc.copy_stride = p.max_src_t + 1;
            hipLaunchKernelGGL(scan_kernel, dim3((unsigned)ceil_div(b.cap_src, SCAN_TILE), n_batches), dim3(SCAN_THREADS), 0, s, sc);
            hipLaunchKernelGGL(t_fill_kernel, grid, blk, 0, s, da);
            hipLaunchKernelGGL(t_rank_kernel, grid, blk, 0, s, da);
        }
    }
    CR_LAUNCH_CHECK();
    return CR_OK;
}
