// Centroid scoring and budgeted cluster selection for gfx950 (Eq. 1, Sec. 3.1; two levels: Sec. 3.4).
//
// One launch per decode step, one workgroup of 512 threads per unit; the coarse level and the fine
// level run back to back in the same workgroup.  The launch moves a few per cent of the step's
// bytes and nothing can overlap it (the value pass needs its result), so what counts is the length
// of the chain a wave executes: per level one trip to memory for the centroid rows, all requested at
// once, then a handful of short phases between workgroup barriers.  Two measured facts shape it:
//   * one compute unit pulls only about 20 GB/s out of a cold HBM (the chip's bandwidth is the sum
//     over its 256 units), so the 64-128 KiB of centroid rows per level are the largest single cost;
//   * with one workgroup per compute unit every instruction of the chain costs 8-9 cycles, so the
//     chain is kept short: the products run on the fp64 matrix pipe, every thread then owns ONE entry
//     (no loops at the benchmark's sizes), one exponential per (entry, head), no logarithm, and what
//     is the same for the whole workgroup (one value per head) is worked out once per wave, the heads
//     side by side in the lanes.  (More waves would shorten the per-entry part and lengthen that one:
//     512 threads is where the two balance for levels of 256-512 entries.)
//
// Logits l[h,i] = scale * q_h . Kc_i are accumulated in fp64 (products of bf16 numbers are exact,
// so the sum carries ~1e-16 relative error and the ranking agrees with an fp64 reference except on
// ties far below any tolerance) with v_mfma_f64_4x4x4 (four independent 4x4x4 blocks per
// instruction: 16 entries x 4 heads per wave and round).  The score of an entry is
// sum_h e^{l[h,i] - LSE_h}, G times Eq. 1 averaged over the query heads of the group; it is compared
// in the linear domain (same order as its logarithm, the rank key the getters report).  Selection =
// "take clusters in descending score order (ties: lower id) while the running token count stays
// within the budget, stop at the first that does not fit"; token counts are positive, so this is a
// threshold on (score, id): one 256-bucket histogram over the leading bits of the score and a direct
// comparison among the entries of the boundary bucket (a most-significant-digit radix search takes
// over where that bucket is crowded).
//
// Per-entry working arrays (logits, keys, counts, ids, row starts, flags) live in LDS when a level
// has at most lds_cap entries and in a global scratch area otherwise (separate template
// instantiations: LDS instructions and LDS-only barriers in the first case).
//
// Shadow workgroups: with spare compute units (2 U <= units of the chip, U a multiple of eight: the
// blocks of a launch go round the eight L2 slices), a second workgroup per unit, placed on the same
// L2 slice, runs the same code without storing anything and asks for the centroid rows in the
// opposite order, so that each of the two finds part of its rows already in the shared L2.  It never
// communicates with the first.
//
// Outputs for the value pass: the flat list of stored rows of the selected clusters' keys, and one
// "centroid term" entry (value-centroid row + ready-made logits) per cluster that stays behind at
// either level (unpromising coarse clusters, unselected fine candidates).
#include <type_traits>

#include "mp_device.h"
#include "mp_internal.h"

namespace mp {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kInFlight = 4;                          // rounds (16 entries per wave) whose centroid rows are requested ahead
constexpr int kHistBits = 8;                          // first (and normally only) digit of the selection
constexpr int kHistBuckets = 1 << kHistBits;
constexpr int kListCap = 64;                          // boundary-bucket entries ordered by direct comparison
static_assert(kThreads == 512, "a thread carries one element per head group of the 512-element query operand");
static_assert(kWaves <= 16, "the (head, wave) lane layout below uses rows of 16 lanes");
constexpr int kKeep = 2;                              // chunks of kThreads entries whose e^{l - M} stay in registers

// Order-preserving 64-bit image of a rank key r, ascending = descending r.
__device__ __forceinline__ uint64_t descending_key(double r)
{
    uint64_t b = (uint64_t)__double_as_longlong(r);
    b = (b >> 63) ? ~b : (b | 0x8000000000000000ull);   // ascending in r
    return ~b;                                           // ascending key = descending r
}

struct Scratch {
    unsigned long long hist[3][256];  // radix digit histograms: entry count << 40 | token count
    unsigned long long hkey[3][256];  // a key that fell into each bucket (THE key where the bucket holds one entry)
    unsigned long long rk_min[kWaves], rk_max[kWaves];  // per wave: smallest / largest key that takes part
    uint32_t rk_wt[kWaves], rk_cn[kWaves];              // ... their token total and their number
    uint32_t wsum[2][kWaves][2];      // per-wave totals of the two-value scan, double-buffered
    double wm[kWaves][8];             // per wave and head: largest logit of an entry that takes part
    double ws[kWaves][8];             // per wave and head: sum of N e^{l - M_h}
    double bm[8], bs[8];              // what stayed behind at the coarse level, per head: shift and sum of N e^{l - shift}
    // extremes of the keys, token total, "some score too small" flag and boundary-list length of the
    // level in progress, maintained with LDS atomics
    unsigned long long key_min, key_max;
    uint32_t key_total, key_tiny, bl_count;
};

struct Arrays {
    double* lg;            // [G][lg_stride]
    long long lg_stride;
    uint64_t* keys;
    uint32_t* wts;
    int32_t* ids;          // candidate fine ids (fine level of two)
    int32_t* aux;          // fine: first stored row; coarse: first child
    int32_t* aux2;         // coarse: end of children; fine: offset of the cluster's rows in the row list
    uint8_t* flags;
};

// Barrier between phases.  With the working arrays in LDS nothing written to global memory is read
// back inside the kernel, so only LDS traffic has to be ordered and outstanding global stores may
// stay in flight.
template <bool kLds>
__device__ __forceinline__ void phase_sync()
{
    if constexpr (kLds) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    } else {
        __syncthreads();
    }
}

// Exclusive prefix sums of two values per thread over one chunk of kThreads threads, with running
// totals carried in registers (every thread adds the same chunk totals, so they stay uniform).
// One barrier per call: the per-wave totals are double-buffered by the parity of `calls`; after the
// barrier the first 16 lanes of every wave scan them.
struct ScanState {
    uint32_t carry_a = 0, carry_b = 0, calls = 0;
};
template <bool kLds>
__device__ __forceinline__ void chunk_excl_scan2(uint32_t a, uint32_t b, Scratch& s, ScanState& st, uint32_t& ex_a,
                                                 uint32_t& ex_b)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t ia = wave_incl_scan_u32(a), ib = wave_incl_scan_u32(b);
    const int par = st.calls & 1;
    ++st.calls;
    if (lane == 63) {
        s.wsum[par][wave][0] = ia;
        s.wsum[par][wave][1] = ib;
    }
    phase_sync<kLds>();
    const uint32_t wa = lane < kWaves ? s.wsum[par][lane][0] : 0u, wb = lane < kWaves ? s.wsum[par][lane][1] : 0u;
    const uint32_t sa = wave_incl_scan_u32(wa), sb = wave_incl_scan_u32(wb);
    const int w = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t off_a = (uint32_t)__builtin_amdgcn_readlane((int)(sa - wa), w);
    const uint32_t off_b = (uint32_t)__builtin_amdgcn_readlane((int)(sb - wb), w);
    const uint32_t tot_a = (uint32_t)__builtin_amdgcn_readlane((int)sa, kWaves - 1);
    const uint32_t tot_b = (uint32_t)__builtin_amdgcn_readlane((int)sb, kWaves - 1);
    ex_a = st.carry_a + off_a + ia - a;
    ex_b = st.carry_b + off_b + ib - b;
    st.carry_a += tot_a;
    st.carry_b += tot_b;
}

template <typename T, typename Op>
__device__ __forceinline__ T wave_reduce(T v, Op op)
{
    auto moved = [](T x, auto ctrl) {
        constexpr int kCtrl = decltype(ctrl)::value;
        if constexpr (sizeof(T) == 4) {
            return (T)__builtin_amdgcn_mov_dpp((int)x, kCtrl, 0xf, 0xf, true);
        } else {
            const uint32_t lo = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)x, kCtrl, 0xf, 0xf, true);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)(x >> 32), kCtrl, 0xf, 0xf, true);
            return (T)(((uint64_t)hi << 32) | lo);
        }
    };
    auto lane_value = [](T x, int src) {
        if constexpr (sizeof(T) == 4) {
            return (T)__builtin_amdgcn_readlane((int)x, src);
        } else {
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, src);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), src);
            return (T)(((uint64_t)hi << 32) | lo);
        }
    };
    v = op(v, moved(v, std::integral_constant<int, kDppXor1>{}));
    v = op(v, moved(v, std::integral_constant<int, kDppXor2>{}));
    v = op(v, moved(v, std::integral_constant<int, kDppHalfMirror>{}));
    v = op(v, moved(v, std::integral_constant<int, kDppMirror>{}));
    return op(op(lane_value(v, 0), lane_value(v, 16)), op(lane_value(v, 32), lane_value(v, 48)));
}

// Weighted radix select.  keys[i] ascending = rank order, wts[i] > 0 for entries that take part
// (entries with wts == 0 are never selected).  Finds the key K* of the first entry (in (key, index)
// order) at which the running weight exceeds `budget`, the weight `acc` of all entries with key <
// K*, and how many entries carry exactly K*.  Returns false if everything fits.
//
// Digits are taken from key - min(key), starting at the top bit of max - min, so that the first
// digit already spreads the entries over the histogram instead of piling them onto a few LDS
// addresses.  One barrier per digit of up to 8 bits: the histogram (entry count and token count
// packed in one 64-bit LDS atomic) is scanned by every wave for itself, which leaves the chosen
// digit wave-uniform in registers.  Next to each bucket's counts sits the key of an entry that fell
// into it, so that the pass in which the boundary bucket is down to one entry ends the search
// without another sweep.  Three histogram buffers rotate: pass p fills buffer p%3 and
// clears buffer (p+1)%3, whose last readers (pass p-2) all finished before the barrier of pass p-1.
template <bool kLds>
__device__ __forceinline__ bool radix_select(const uint64_t* keys, const uint32_t* wts, int n, long long budget,
                                             Scratch& s, uint64_t& kstar, uint64_t& acc_out, uint32_t& ties_out)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr unsigned long long kWtMask = (1ull << 40) - 1;
    // token totals fit 31 bits
    const uint32_t bud = budget < 0 ? 0u : (budget > 0xffffffffll ? 0xffffffffu : (uint32_t)budget);
    {
        uint64_t kmin = ~0ull, kmax = 0;
        uint32_t wt = 0, cn = 0;
        for (int i = tid; i < n; i += kThreads) {
            const uint32_t w = wts[i];
            if (w == 0) continue;
            const uint64_t k = keys[i];
            kmin = k < kmin ? k : kmin;
            kmax = k > kmax ? k : kmax;
            wt += w;
            ++cn;
        }
        kmin = wave_reduce(kmin, [](uint64_t a, uint64_t b) { return a < b ? a : b; });
        kmax = wave_reduce(kmax, [](uint64_t a, uint64_t b) { return a > b ? a : b; });
        wt = wave_reduce(wt, [](uint32_t a, uint32_t b) { return a + b; });
        cn = wave_reduce(cn, [](uint32_t a, uint32_t b) { return a + b; });
        if (lane == 0) {
            s.rk_min[wave] = kmin;
            s.rk_max[wave] = kmax;
            s.rk_wt[wave] = wt;
            s.rk_cn[wave] = cn;
        }
    }
    if (tid < 256) s.hist[0][tid] = 0;
    phase_sync<kLds>();
    uint64_t kmin = ~0ull, kmax = 0;
    uint32_t total = 0, cnt = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint64_t a = s.rk_min[w], b = s.rk_max[w];
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
        total += s.rk_wt[w];
        cnt += s.rk_cn[w];
    }
    if (total <= bud) return false;           // everything fits
    const uint64_t range = kmax - kmin;
    int hi = range ? 64 - __clzll((long long)range) : 0;   // number of low bits of key - kmin still undecided
    uint64_t prefix = 0;                                   // the decided bits of K* - kmin
    uint32_t acc = 0;
    for (int pass = 0; hi > 0; ++pass) {
        const int bits = hi < 8 ? hi : 8, shift = hi - bits;
        const uint32_t dmask = (1u << bits) - 1u;
        unsigned long long* H = s.hist[pass % 3];
        unsigned long long* HK = s.hkey[pass % 3];
        if (tid < 256) s.hist[(pass + 1) % 3][tid] = 0;
        for (int i = tid; i < n; i += kThreads) {
            const uint32_t w = wts[i];
            if (w == 0) continue;
            const uint64_t k = keys[i] - kmin;
            if (hi >= 64 || (k >> hi) == prefix) {
                const uint32_t b = (uint32_t)(k >> shift) & dmask;
                atomicAdd(&H[b], (1ull << 40) | w);
                HK[b] = keys[i];        // plain store: only read back where this entry is alone in its bucket
            }
        }
        phase_sync<kLds>();
        unsigned long long h4[4];
        uint32_t sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            h4[j] = H[4 * lane + j];
            sum += (uint32_t)(h4[j] & kWtMask);
        }
        const uint32_t incl = wave_incl_scan_u32(sum);
        // the bucket being split weighs more than what is left of the budget, so some lane crosses
        const unsigned long long mask = __ballot((unsigned long long)acc + incl > bud);
        const int first = mask ? __ffsll((long long)mask) - 1 : 63;
        uint32_t a = acc + incl - sum, d = 4 * lane, c = 0;
        bool done = false;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t wj = (uint32_t)(h4[j] & kWtMask);
            if (!done) {
                if ((unsigned long long)a + wj > bud) {
                    d = 4 * lane + j;
                    c = (uint32_t)(h4[j] >> 40);
                    done = true;
                } else {
                    a += wj;
                }
            }
        }
        acc = (uint32_t)__builtin_amdgcn_readlane((int)a, first);
        cnt = (uint32_t)__builtin_amdgcn_readlane((int)c, first);
        prefix = (prefix << bits) | (uint32_t)__builtin_amdgcn_readlane((int)d, first);
        hi = shift;
        if (cnt == 1 && hi > 0) {
            // a single entry carries the boundary: its full key is K*, and it left that key in the
            // bucket's slot (nobody else wrote there in this pass)
            kstar = HK[(uint32_t)prefix & dmask];
            acc_out = acc;
            ties_out = 1;
            return true;
        }
    }
    kstar = kmin + prefix;
    acc_out = acc;
    ties_out = cnt;
    return true;
}

// ------------------------------------------------------------------------------------------------
// Dynamic LDS behind the Scratch block: the query in matrix-operand order, the selection's
// histogram and boundary list, then the per-entry working arrays (cap = p.lds_cap entries each).
// ------------------------------------------------------------------------------------------------
struct Lds {
    double* qB;                 // [GH][32][16]: slice s, dim group k, head j (see query_operand_element)
    unsigned long long* hist;   // [kHistBuckets] entry count << 40 | token count
    unsigned long long* blist;  // [kListCap][2]: key, position << 32 | token count
    Arrays A;
};

__host__ __device__ constexpr size_t align16(size_t x) { return (x + 15) & ~size_t(15); }

template <int G>
__device__ __forceinline__ Lds carve_lds(unsigned char* lds, int cap)
{
    constexpr int GH = (G + 3) / 4;
    Lds L;
    L.qB = reinterpret_cast<double*>(lds);
    L.hist = reinterpret_cast<unsigned long long*>(L.qB + GH * 512);
    L.blist = L.hist + kHistBuckets;
    L.A.lg = reinterpret_cast<double*>(L.blist + 2 * kListCap);
    L.A.lg_stride = cap;
    L.A.keys = reinterpret_cast<uint64_t*>(L.A.lg + (size_t)G * cap);
    L.A.wts = reinterpret_cast<uint32_t*>(L.A.keys + cap);
    L.A.ids = reinterpret_cast<int32_t*>(L.A.wts + cap);
    L.A.aux = L.A.ids + cap;
    L.A.aux2 = L.A.aux + cap;
    L.A.flags = reinterpret_cast<uint8_t*>(L.A.aux2 + cap);
    return L;
}

template <int G>
__device__ __forceinline__ Arrays global_arrays(const ScoreParams& p, int u)
{
    Arrays A;
    A.lg = p.lg + (long long)u * G * p.lg_stride;
    A.lg_stride = p.lg_stride;
    A.keys = reinterpret_cast<uint64_t*>(p.g_keys) + (long long)u * p.g_stride;
    A.wts = p.g_wts + (long long)u * p.g_stride;
    A.ids = p.cand + (long long)u * p.f_stride;       // the candidate list itself
    A.aux = p.g_aux + (long long)u * p.g_stride;
    A.aux2 = p.g_aux2 + (long long)u * p.g_stride;
    A.flags = p.g_flags + (long long)u * p.g_stride;
    return A;
}

// ------------------------------------------------------------------------------------------------
// The matrix product.
//
// v_mfma_f64_4x4x4 computes four independent blocks D_b[i][j] += sum_k A_b[i][k] * B_b[k][j] with
// (measured lane map) A_b[i][k] in lane 16k + 4b + i, B_b[k][j] in lane 16k + 4b + j and D_b[i][j]
// in lane 16i + 4b + j.  Here i = entry inside a block, j = head, k = one of four groups of 32
// dimensions: lane (k, e = 4b + i) holds, for entry e of the wave's 16, the dimensions
// {32c + 8k + r : c < 4, r < 8} (four 16-byte pieces of the row, so that one load instruction of the
// wave covers 64 contiguous bytes of 16 rows), and 32 instructions, one per (c, r), add up the whole
// product.  The B operand (the query, the same for every block) is read from LDS: element x of qB,
// x = (hg * 32 + 8c + r) * 16 + 4k + j, is dimension 32c + 8k + r of head 4 hg + j.
// After the product lane (i, b, j) owns the logit of entry 4b + i and head j.
// ------------------------------------------------------------------------------------------------
template <int G>
__device__ __forceinline__ double query_operand_element(const ScoreParams& p, int u, int x)
{
    const int hg = x >> 9, s = (x >> 4) & 31, k = (x >> 2) & 3, j = x & 3;
    const int h = 4 * hg + j, d = 32 * (s >> 3) + 8 * k + (s & 7);
    return h < G ? (double)bf16_to_f32(p.q[((long long)u * G + h) * kHeadDim + d]) : 0.0;
}

__device__ __forceinline__ double shfl_xor_f64(double v, int m)
{
    const long long b = __double_as_longlong(v);
    const int lo = __shfl_xor((int)(b & 0xffffffffll), m, 64), hi = __shfl_xor((int)(b >> 32), m, 64);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
constexpr int kDppRowRor4 = 0x124, kDppRowRor8 = 0x128;
// Largest value over the 16 lanes of a wave that own the same head (lanes equal modulo 4).
__device__ __forceinline__ double max_same_head(double x)
{
    x = fmax(x, dpp_f64<kDppRowRor4>(x));
    x = fmax(x, dpp_f64<kDppRowRor8>(x));
    x = fmax(x, shfl_xor_f64(x, 16));
    x = fmax(x, shfl_xor_f64(x, 32));
    return x;
}
__device__ __forceinline__ double row_min_f64(double v)
{
    v = fmin(v, dpp_f64<kDppXor1>(v));
    v = fmin(v, dpp_f64<kDppXor2>(v));
    v = fmin(v, dpp_f64<kDppHalfMirror>(v));
    v = fmin(v, dpp_f64<kDppMirror>(v));
    return v;
}

// One value per head from a [kWaves][8] table of per-wave values: lane 16 hh + w of every wave takes
// the value of (wave w, head 4 hg + hh), the row is combined, `post` (head group, head, combined value) is applied
// -- once per head group, the heads side by side in the lanes -- and every lane receives the G results.
template <int G, typename RowOp, typename Post>
__device__ __forceinline__ void combine_waves(const double (&tab)[kWaves][8], double neutral, RowOp row_op, Post post,
                                              double (&out)[G])
{
    constexpr int GH = (G + 3) / 4;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int hg = 0; hg < GH; ++hg) {
        const int h = 4 * hg + (lane >> 4), w = lane & 15;
        const int hc = h < G ? h : G - 1;
        const double v = post(hg, hc, row_op((h < G && w < kWaves) ? tab[w][h] : neutral));
#pragma unroll
        for (int hh = 0; hh < 4; ++hh)
            if (4 * hg + hh < G) out[4 * hg + hh] = readlane_f64(v, 16 * hh);
    }
}

// The value itself, but the compiler can neither move its evaluation out of the branch it stands in nor
// evaluate it ahead of time (used to keep rarely needed logarithms out of the common path).
__device__ __forceinline__ double not_hoisted(double v)
{
    asm volatile("" : "+v"(v));
    return v;
}

// One centroid-term entry (Eq. 2): the row of the value centroid and log2( N_i e^{l[h,i]} ) per head.
template <int G>
__device__ __forceinline__ void emit_term(const ScoreParams& p, const Arrays& A, int u, int i, int row, uint32_t slot)
{
    const long long o = (long long)u * p.mp_stride + slot;
    p.mp_rows[o] = row;
    const float lgN = __builtin_amdgcn_logf((float)A.wts[i]);
#pragma unroll
    for (int h = 0; h < G; ++h) p.mp_scores[o * G + h] = (float)(A.lg[h * A.lg_stride + i] * 1.4426950408889634) + lgN;
}

// One level: logits, Eq. 1 normaliser, scores, budgeted selection.
// Entry x stands for cluster id (use_ids ? A.ids[x] : x).  `with_behind`: the normaliser also covers
// the coarse clusters that stayed behind (S.bm / S.bs).  `meanwhile` runs (in every thread) once the
// level's centroid rows have been asked for: work of the previous level that the requests did not
// have to wait for.  `q_pending`: the
// query operand still has to go to LDS (first level of the launch; qv = this thread's element).
// `quiet`: store nothing in global memory (shadow workgroup); `reverse`: ask for the rows last round
// first.  On return A holds logits, keys, member counts (0 = takes no part), row starts and flags,
// all published by a barrier.  Returns 1 if the keys are linear-domain scores, 0 if they are
// logarithmic rank keys (the rare case of scores below the range of a double).
// What a level keeps of its own entries after the selection: the shift per head, and for the first
// kKeep chunks of kThreads entries the member count and e^{l - shift} of this thread's entry.
template <int G>
struct LevelState {
    double M[G];
    double ek[kKeep][G];
    uint32_t wk[kKeep];
};

template <int G, bool kLds, typename Meanwhile>
__device__ __forceinline__ int score_level(const ScoreParams& p, const Lds& L, const Arrays& A, Scratch& S, int u, int n,
                                           bool use_ids, bool coarse, long long budget, bool with_behind,
                                           bool q_pending, const double (&qv)[(G + 3) / 4], bool quiet, bool reverse,
                                           unsigned long long* key_out, uint8_t* flag_out, LevelState<G>& state,
                                           Meanwhile meanwhile)
{
    constexpr int GH = (G + 3) / 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double ninf = -INFINITY;
    const int row_off = coarse ? p.fcap : 0;
    const int32_t* Nu = p.N + (long long)u * p.tab_rows + row_off;
    const uint16_t* Kcu = p.Kc + ((long long)u * p.tab_rows + row_off) * kHeadDim;
    const int32_t* st = coarse ? p.cstart + (long long)u * p.cstart_stride : p.fstart + (long long)u * p.fstart_stride;
    const int chunks = (n + kThreads - 1) / kThreads;

    // ================= logits: matrix layout, 16 entries per wave and round =================
    {
        const int kA = lane >> 4, eA = lane & 15;                       // operand layout: dim group, entry
        const int jD = lane & 3, eD = ((lane >> 2) & 3) * 4 + (lane >> 4);   // result layout: head, entry
        const int bsel = kA * 4 + jD;                                   // this lane's slot in a slice of qB
        const int rounds = (n + 16 * kWaves - 1) / (16 * kWaves);
        uint4 raw[kInFlight][4];
        int cntD[kInFlight], auxD[kInFlight], aux2D[kInFlight];
        auto request = [&](int t, uint4 (&r)[4], int& cnt, int& a1, int& a2) {
            const int base = ((reverse ? rounds - 1 - t : t) * kWaves + wave) * 16;
            const int xa = base + eA, xd = base + eD;
#pragma unroll
            for (int c = 0; c < 4; ++c) r[c] = make_uint4(0, 0, 0, 0);
            cnt = a1 = a2 = 0;
            if (xa < n) {
                const int id = use_ids ? A.ids[xa] : xa;
                const uint4* kp = reinterpret_cast<const uint4*>(Kcu + (long long)id * kHeadDim) + kA;
#pragma unroll
                for (int c = 0; c < 4; ++c) r[c] = kp[4 * c];
            }
            if (xd < n) {
                const int id = use_ids ? A.ids[xd] : xd;
                cnt = Nu[id];
                a1 = st[id];
                if (coarse) a2 = st[id + 1];
            }
        };
#pragma unroll
        for (int t = 0; t < kInFlight; ++t) {
            if (t < rounds) request(t, raw[t], cntD[t], auxD[t], aux2D[t]);
            else {
#pragma unroll
                for (int c = 0; c < 4; ++c) raw[t][c] = make_uint4(0, 0, 0, 0);
                cntD[t] = auxD[t] = aux2D[t] = 0;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // while the rows travel: empty histogram and extremes for this level's selection (their last
        // readers passed a barrier long ago), and the query operand
        if (tid < kHistBuckets) L.hist[tid] = 0;
        if (tid == 0) {
            S.bl_count = 0;
            S.key_min = ~0ull;
            S.key_max = 0;
            S.key_total = 0;
            S.key_tiny = 0;
        }
        if (q_pending) {
#pragma unroll
            for (int hg = 0; hg < GH; ++hg) L.qB[tid + hg * kThreads] = qv[hg];
            phase_sync<true>();
        }
        meanwhile();

        double mx[GH];
#pragma unroll
        for (int hg = 0; hg < GH; ++hg) mx[hg] = ninf;
#pragma unroll 1
        for (int t0 = 0; t0 < rounds; t0 += kInFlight) {
#pragma unroll
            for (int j = 0; j < kInFlight; ++j) {
                const int t = t0 + j;
                if (t < rounds) {
                    double acc[GH];
#pragma unroll
                    for (int hg = 0; hg < GH; ++hg) acc[hg] = 0.0;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const uint32_t w4[4] = {raw[j][c].x, raw[j][c].y, raw[j][c].z, raw[j][c].w};
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const double a = (double)((e & 1) ? bf16hi_to_f32(w4[e >> 1]) : bf16lo_to_f32(w4[e >> 1]));
#pragma unroll
                            for (int hg = 0; hg < GH; ++hg)
                                acc[hg] = __builtin_amdgcn_mfma_f64_4x4x4f64(a, L.qB[(hg * 32 + 8 * c + e) * 16 + bsel], acc[hg], 0, 0, 0);
                        }
                    }
                    const int xd = ((reverse ? rounds - 1 - t : t) * kWaves + wave) * 16 + eD;
                    const bool part = xd < n && cntD[j] > 0;
                    if (xd < n && jD == 0) {
                        A.wts[xd] = part ? (uint32_t)cntD[j] : 0u;
                        A.aux[xd] = auxD[j];
                        if (coarse) A.aux2[xd] = aux2D[j];
                    }
#pragma unroll
                    for (int hg = 0; hg < GH; ++hg) {
                        const double l = acc[hg] * p.scale;
                        if (xd < n && 4 * hg + jD < G) {
                            A.lg[(4 * hg + jD) * A.lg_stride + xd] = l;
                            if (part) mx[hg] = fmax(mx[hg], l);
                        }
                    }
                    if (t + kInFlight < rounds) request(t + kInFlight, raw[j], cntD[j], auxD[j], aux2D[j]);
                }
            }
        }
#pragma unroll
        for (int hg = 0; hg < GH; ++hg) {
            mx[hg] = max_same_head(mx[hg]);
            if (lane < 4 && 4 * hg + lane < G) S.wm[wave][4 * hg + lane] = mx[hg];
        }
    }
    phase_sync<kLds>();

    // ================= from here on thread tid owns entry tid (+ kThreads per further chunk) =================
    // shift of the level: the largest logit that takes part (and the shift of what stayed behind)
    double (&M)[G] = state.M;
    combine_waves<G>(S.wm, ninf, [](double v) { return row_max_f64(v); },
                     [&](int, int h, double v) { return (with_behind && S.bs[h] > 0.0) ? fmax(v, S.bm[h]) : v; }, M);
    // e^{l - M_h} of the own entries (kept in registers for the first kKeep chunks) and the sums of N e^{l - M_h}
    double (&ek)[kKeep][G] = state.ek;
    uint32_t (&wk)[kKeep] = state.wk;
    double sm[G];
#pragma unroll
    for (int h = 0; h < G; ++h) sm[h] = 0.0;
#pragma unroll
    for (int c = 0; c < kKeep; ++c) {
        wk[c] = 0;
#pragma unroll
        for (int h = 0; h < G; ++h) ek[c][h] = 0.0;
        const int i = tid + c * kThreads;
        if (i < n) wk[c] = A.wts[i];
        if (wk[c]) {
#pragma unroll
            for (int h = 0; h < G; ++h) {
                ek[c][h] = exp_shifted(A.lg[h * A.lg_stride + i] - M[h]);
                sm[h] += (double)wk[c] * ek[c][h];
            }
        }
    }
    for (int c = kKeep; c < chunks; ++c) {
        const int i = tid + c * kThreads;
        const uint32_t w = i < n ? A.wts[i] : 0u;
        if (w) {
#pragma unroll
            for (int h = 0; h < G; ++h) sm[h] += (double)w * exp_shifted(A.lg[h * A.lg_stride + i] - M[h]);
        }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const double t = wave_sum_f64(sm[h]);
        if (lane == 0) S.ws[wave][h] = t;
    }
    phase_sync<kLds>();
    // 1 / sum_i N_i e^{l - M_h} per head (0 where nothing takes part)
    double inv[G];
    combine_waves<G>(S.ws, 0.0, [](double v) { return row_sum_f64(v); },
                     [&](int, int h, double v) {
                         if (with_behind && S.bs[h] > 0.0) {
                             // this row's head: its shift once more, from the table (cheaper than routing M here)
                             const int w = lane & 15;
                             const double m = fmax(row_max_f64(w < kWaves ? S.wm[w][h] : ninf), S.bm[h]);
                             v += S.bs[h] * exp_shifted(S.bm[h] - m);
                         }
                         return v > 0.0 ? 1.0 / v : 0.0;
                     }, inv);

    // ---- keys.  Linear domain: the complement of the bit pattern of sum_h e^{l - LSE_h} (ascending
    // key = descending score).  If a score leaves the range of a double, the whole level ranks by
    // log mean_h e^{l - LSE_h} worked out in the log domain instead (second trip; uniform). ----
    int linear = 1;
    constexpr double kLogGs[9] = {0.0, 0.0, 0.6931471805599453094, 1.0986122886681097821, 1.3862943611198906188,
                                  1.6094379124341002818, 1.7917594692280549573, 1.9459101090932196052, 2.0794415416798357477};
    constexpr double kLogG = kLogGs[G];
    for (;;) {
        double smin = INFINITY, smax = ninf;     // extremes of the score (linear) / of the rank key (log)
        uint32_t wsum = 0;
        bool tiny = false;
        auto one_key = [&](int i, uint32_t w, const double (&e)[G], bool kept) {
            uint64_t key = ~0ull;
            if (w) {
                double sc;
                if (linear) {
                    sc = 0.0;
#pragma unroll
                    for (int h = 0; h < G; ++h)
                        sc += (kept ? e[h] : exp_shifted(A.lg[h * A.lg_stride + i] - M[h])) * inv[h];
                    tiny |= !(sc >= 1e-280);
                    key = ~(uint64_t)__double_as_longlong(sc);
                } else {
                    double th[G], tm = ninf;
#pragma unroll
                    for (int h = 0; h < G; ++h) {
                        th[h] = A.lg[h * A.lg_stride + i] - (M[h] - log(not_hoisted(inv[h])));
                        tm = fmax(tm, th[h]);
                    }
                    double ss = 0.0;
#pragma unroll
                    for (int h = 0; h < G; ++h) ss += exp_shifted(th[h] - tm);
                    sc = tm - kLogG + log(ss);
                    key = descending_key(sc);
                }
                smin = fmin(smin, sc);
                smax = fmax(smax, sc);
                wsum += w;
            }
            if (i < n) {
                A.keys[i] = key;
                if (!quiet) key_out[i] = key;
            }
        };
#pragma unroll
        for (int c = 0; c < kKeep; ++c)
            if (c < chunks) one_key(tid + c * kThreads, wk[c], ek[c], true);
        for (int c = kKeep; c < chunks; ++c) {
            const int i = tid + c * kThreads;
            one_key(i, i < n ? A.wts[i] : 0u, ek[0], false);
        }
        smin = row_min_f64(smin);
        smax = row_max_f64(smax);
        smin = fmin(fmin(readlane_f64(smin, 0), readlane_f64(smin, 16)), fmin(readlane_f64(smin, 32), readlane_f64(smin, 48)));
        smax = fmax(fmax(readlane_f64(smax, 0), readlane_f64(smax, 16)), fmax(readlane_f64(smax, 32), readlane_f64(smax, 48)));
        wsum = wave_reduce(wsum, [](uint32_t a, uint32_t b) { return a + b; });
        if (lane == 0 && wsum) {
            // the largest score carries the smallest key
            const uint64_t klo = linear ? ~(uint64_t)__double_as_longlong(smax) : descending_key(smax);
            const uint64_t khi = linear ? ~(uint64_t)__double_as_longlong(smin) : descending_key(smin);
            atomicMin(&S.key_min, (unsigned long long)klo);
            atomicMax(&S.key_max, (unsigned long long)khi);
            atomicAdd(&S.key_total, wsum);
        }
        if (__any(tiny) && lane == 0) atomicOr(&S.key_tiny, 1u);
        phase_sync<kLds>();
        if (!linear || !S.key_tiny) break;
        linear = 0;
        phase_sync<kLds>();       // everyone has seen the flag
        if (tid == 0) {
            S.key_min = ~0ull;
            S.key_max = 0;
            S.key_total = 0;
            S.key_tiny = 0;
        }
        phase_sync<kLds>();
    }

    // ---- budgeted selection ----
    const uint64_t kmin = S.key_min, kmax = S.key_max;
    const uint32_t total = S.key_total;
    const uint32_t bud = budget < 0 ? 0u : (budget > 0xffffffffll ? 0xffffffffu : (uint32_t)budget);
    constexpr unsigned long long kWtMask = (1ull << 40) - 1;
    if (total <= bud) {
        for (int c = 0; c < chunks; ++c) {
            const int i = tid + c * kThreads;
            if (i < n) {
                const uint8_t f = A.wts[i] ? 1 : 0;
                A.flags[i] = f;
                if (!quiet) flag_out[i] = f;
            }
        }
    } else {
        const uint64_t range = kmax - kmin;
        const int hi = range ? 64 - __clzll((long long)range) : 0;
        const int bits = hi < kHistBits ? hi : kHistBits, shift = hi - bits;
        for (int c = 0; c < chunks; ++c) {
            const int i = tid + c * kThreads;
            const uint32_t w = i < n ? A.wts[i] : 0u;
            if (w) atomicAdd(&L.hist[(uint32_t)((A.keys[i] - kmin) >> shift)], (1ull << 40) | w);
        }
        phase_sync<kLds>();
        // every wave scans the histogram for itself: kHistBuckets / 64 buckets per lane
        constexpr int BPL = kHistBuckets / 64;
        unsigned long long hb[BPL];
        uint32_t sum = 0;
#pragma unroll
        for (int j = 0; j < BPL; ++j) {
            hb[j] = L.hist[BPL * lane + j];
            sum += (uint32_t)(hb[j] & kWtMask);
        }
        const uint32_t incl = wave_incl_scan_u32(sum);
        const unsigned long long crossing = __ballot((unsigned long long)incl > bud);
        const int first = crossing ? __ffsll((long long)crossing) - 1 : 63;
        uint32_t a = incl - sum, d = BPL * lane, cn = 0;
        bool done = false;
#pragma unroll
        for (int j = 0; j < BPL; ++j) {
            const uint32_t wj = (uint32_t)(hb[j] & kWtMask);
            if (!done) {
                if ((unsigned long long)a + wj > bud) {
                    d = BPL * lane + j;
                    cn = (uint32_t)(hb[j] >> 40);
                    done = true;
                } else {
                    a += wj;
                }
            }
        }
        const uint32_t acc = (uint32_t)__builtin_amdgcn_readlane((int)a, first);
        const uint32_t bcnt = (uint32_t)__builtin_amdgcn_readlane((int)cn, first);
        const uint32_t bstar = (uint32_t)__builtin_amdgcn_readlane((int)d, first);
        if (bcnt <= (uint32_t)kListCap) {
            // entries before the boundary bucket are taken, entries behind it are not; those inside it
            // (often one: the first that does not fit) queue up to be ordered by (key, position)
            for (int c = 0; c < chunks; ++c) {
                const int i = tid + c * kThreads;
                if (i >= n) continue;
                const uint32_t w = A.wts[i];
                const uint32_t b = w ? (uint32_t)((A.keys[i] - kmin) >> shift) : ~0u;
                if (b == bstar && bcnt > 1) {
                    const uint32_t slot = atomicAdd(&S.bl_count, 1u);
                    L.blist[2 * slot] = A.keys[i];
                    L.blist[2 * slot + 1] = ((unsigned long long)(uint32_t)i << 32) | w;
                    continue;
                }
                const uint8_t f = (w && b < bstar) ? 1 : 0;
                A.flags[i] = f;
                if (!quiet) flag_out[i] = f;
            }
            if (bcnt > 1) {
                phase_sync<kLds>();
                if ((uint32_t)tid < bcnt) {
                    const unsigned long long mk = L.blist[2 * tid], mv = L.blist[2 * tid + 1];
                    const uint32_t mpos = (uint32_t)(mv >> 32);
                    unsigned long long run = (unsigned long long)acc + (uint32_t)mv;
                    for (uint32_t m = 0; m < bcnt; ++m) {
                        const unsigned long long ok = L.blist[2 * m], ov = L.blist[2 * m + 1];
                        if (ok < mk || (ok == mk && (uint32_t)(ov >> 32) < mpos)) run += (uint32_t)ov;
                    }
                    const uint8_t f = run <= bud ? 1 : 0;
                    A.flags[mpos] = f;
                    if (!quiet) flag_out[mpos] = f;
                }
            }
        } else {
            // a crowded boundary bucket (many equal or nearly equal scores): the general search
            uint64_t kstar = 0, acc2 = 0;
            uint32_t ties = 0;
            const bool bounded = radix_select<kLds>(A.keys, A.wts, n, budget, S, kstar, acc2, ties);
            for (int i = tid; i < n; i += kThreads) {
                uint8_t f = 0;
                if (A.wts[i]) {
                    if (!bounded) f = 1;
                    else {
                        const uint64_t k = A.keys[i];
                        if (k < kstar) f = 1;
                        else if (k == kstar && ties > 1) {
                            // exactly equal keys: lower position first, keep while the running count still fits
                            uint64_t run = acc2;
                            for (int j = 0; j <= i; ++j)
                                if (A.wts[j] && A.keys[j] == kstar) run += A.wts[j];
                            f = ((long long)run <= budget) ? 1 : 0;
                        }
                    }
                }
                A.flags[i] = f;
                if (!quiet) flag_out[i] = f;
            }
        }
    }
    phase_sync<kLds>();

    return linear;
}

// The clusters a level did not take enter the next level's normaliser through their centroid: their
// shift and their sum of N e^{l - shift} per head go to S.bm / S.bs (published by the caller's next barrier).
template <int G, bool kLds>
__device__ __forceinline__ void leave_behind(const Arrays& A, Scratch& S, int n, const LevelState<G>& st)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunks = (n + kThreads - 1) / kThreads;
    double sm[G];
#pragma unroll
    for (int h = 0; h < G; ++h) sm[h] = 0.0;
#pragma unroll
    for (int c = 0; c < kKeep; ++c) {
        const int i = tid + c * kThreads;
        if (st.wk[c] && !A.flags[i]) {
#pragma unroll
            for (int h = 0; h < G; ++h) sm[h] += (double)st.wk[c] * st.ek[c][h];
        }
    }
    for (int c = kKeep; c < chunks; ++c) {
        const int i = tid + c * kThreads;
        const uint32_t w = i < n ? A.wts[i] : 0u;
        if (w && !A.flags[i]) {
#pragma unroll
            for (int h = 0; h < G; ++h) sm[h] += (double)w * exp_shifted(A.lg[h * A.lg_stride + i] - st.M[h]);
        }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const double t = wave_sum_f64(sm[h]);
        if (lane == 0) S.ws[wave][h] = t;
    }
    phase_sync<kLds>();
    double bsum[G];
    combine_waves<G>(S.ws, 0.0, [](double v) { return row_sum_f64(v); }, [](int, int, double v) { return v; }, bsum);
    if (tid == 0) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
            S.bm[h] = st.M[h];
            S.bs[h] = bsum[h];
        }
    }
}

// Coarse level (Sec. 3.4), after scoring and selection: the candidate list (children of the promising
// clusters, ascending fine id) goes to global memory and, as far as it fits, to the LDS slot the fine
// level reads its ids from; every cluster that stays behind gets the slot of its centroid term (left
// in C.aux, which only promising clusters need otherwise).  The terms themselves are written later,
// by emit_coarse_terms, while the fine level's rows travel.
template <int G, bool kLds>
__device__ __forceinline__ void coarse_candidates(const ScoreParams& p, const Arrays& C, int32_t* cand_l, Scratch& S,
                                                  ScanState& sc, int u, bool quiet, int& n_cand, uint32_t& n_terms)
{
    const int tid = threadIdx.x;
    const int n_c = p.n_coarse;
    int32_t* cand_g = p.cand + (long long)u * p.f_stride;
    sc.carry_a = sc.carry_b = 0;
    for (int i0 = 0; i0 < n_c; i0 += kThreads) {
        const int i = i0 + tid;
        const bool part = i < n_c && C.wts[i] != 0;
        const bool keep = part && C.flags[i];
        const bool emit = part && !keep && p.use_mp;
        int c0 = 0, c1 = 0;
        if (keep) { c0 = C.aux[i]; c1 = C.aux2[i]; }
        uint32_t pos, slot;
        chunk_excl_scan2<kLds>((uint32_t)(c1 - c0), emit ? 1u : 0u, S, sc, pos, slot);
        for (int f = c0; f < c1; ++f) {
            const uint32_t o = pos + (uint32_t)(f - c0);
            if (!quiet) cand_g[o] = f;
            if (o < (uint32_t)p.lds_cap) cand_l[o] = f;
        }
        if (emit) C.aux[i] = (int32_t)slot;
    }
    n_cand = (int)sc.carry_a;
    n_terms = sc.carry_b;
    if (tid == 0 && !quiet) {
        p.n_cand[u] = n_cand;
        p.counters[4 * u + 2] = n_c;
    }
}

template <int G>
__device__ __forceinline__ void emit_coarse_terms(const ScoreParams& p, const Arrays& C, int u)
{
    if (!p.use_mp) return;
    for (int i = threadIdx.x; i < p.n_coarse; i += kThreads)
        if (C.wts[i] != 0 && !C.flags[i]) emit_term<G>(p, C, u, i, p.fcap + i, (uint32_t)C.aux[i]);
}

// Fine level, after scoring and selection: emit centroid terms for the unselected candidates and
// the flat list of stored rows of the selected clusters.
template <int G, bool kLds>
__device__ __forceinline__ void fine_epilogue(const ScoreParams& p, const Arrays& F, Scratch& S, ScanState& sc, int u,
                                              int n_f, bool two, uint32_t n_terms)
{
    const int tid = threadIdx.x;
    // One scan gives every selected cluster (ascending fine id) its slot in a compact list and the
    // offset of its rows in the flat row list, and every unselected candidate its centroid-term slot.
    // The compact list reuses the storage of the keys, which nobody reads any more.
    int2* sel_rc = reinterpret_cast<int2*>(F.keys);      // (first stored row, count)
    int32_t* sel_off = F.aux2;
    sc.carry_a = sc.carry_b = 0;
    for (int i0 = 0; i0 < n_f; i0 += kThreads) {
        const int i = i0 + tid;
        const bool part = i < n_f && F.wts[i] != 0;
        const bool sel = part && F.flags[i];
        const bool emit = part && !sel && p.use_mp;
        const uint32_t w = sel ? F.wts[i] : 0u;
        const int r0 = sel ? F.aux[i] : 0;
        uint32_t off, packed;       // packed: selected clusters in the low half, terms in the high half
        chunk_excl_scan2<kLds>(w, (sel ? 1u : 0u) | (emit ? 0x10000u : 0u), S, sc, off, packed);
        if (sel) {
            sel_rc[packed & 0xffffu] = make_int2(r0, (int)w);
            sel_off[packed & 0xffffu] = (int32_t)off;
            if (p.sel_base) {
                // q . centroid of a selected cluster, log2 units, for a value pass over keys stored as residuals
                // from it: eight columns per cluster, head h in column h (groups of up to five heads) or, for
                // larger groups, which the value pass splits over two waves, in column 4 * half + h % ceil(G / 2)
                constexpr int kHalf = G > 5 ? (G + 1) / 2 : 8;
                float b[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int h = 0; h < G; ++h)
                    b[h < kHalf ? h : 4 + h - kHalf] = (float)(F.lg[h * F.lg_stride + i] * 1.4426950408889634);
                float4* dst = reinterpret_cast<float4*>(p.sel_base + ((long long)u * p.f_stride + (packed & 0xffffu)) * 8);
                dst[0] = make_float4(b[0], b[1], b[2], b[3]);
                dst[1] = make_float4(b[4], b[5], b[6], b[7]);
            }
        }
        if (emit) emit_term<G>(p, F, u, i, two ? F.ids[i] : i, n_terms + (packed >> 16));
    }
    const uint32_t total = sc.carry_a, n_sel = sc.carry_b & 0xffffu;
    n_terms += sc.carry_b >> 16;
    phase_sync<kLds>();
    // expansion: one row of 16 lanes per selected cluster, the next cluster's entry fetched early
    int32_t* ro = p.rows + (long long)u * p.rows_stride;
    int32_t* so = p.row_slot ? p.row_slot + (long long)u * p.rows_stride : nullptr;   // compact slot of each row's cluster
    const int grp = tid >> 4, sub = tid & 15;
    int2 rc_n = make_int2(0, 0);
    int off_n = 0;
    if ((uint32_t)grp < n_sel) {
        rc_n = sel_rc[grp];
        off_n = sel_off[grp];
    }
    for (uint32_t k = grp; k < n_sel; k += kThreads / 16) {
        const int2 rc = rc_n;
        const int off = off_n;
        const uint32_t kn = k + kThreads / 16;
        if (kn < n_sel) {
            rc_n = sel_rc[kn];
            off_n = sel_off[kn];
        }
        for (int j = sub; j < rc.y; j += 16) ro[off + j] = rc.x + j;
        if (so)
            for (int j = sub; j < rc.y; j += 16) so[off + j] = (int32_t)k;
    }
    if (tid == 0) {
        p.n_rows[u] = (int32_t)total;
        p.n_mp[u] = (int32_t)n_terms;
        p.counters[4 * u + 0] = (int32_t)total + p.n_tail;
        p.counters[4 * u + 1] = n_f;
        if (!two) p.counters[4 * u + 2] = 0;
        p.counters[4 * u + 3] = (int32_t)n_terms;
    }
}

// What a shadow workgroup does at the last level: ask for the centroid rows of the second half of
// the level's entries, last entry first, and drop them.
__device__ __forceinline__ void touch_rows(const ScoreParams& p, const int32_t* ids, int u, int n)
{
    const uint16_t* Kcu = p.Kc + (long long)u * p.tab_rows * kHeadDim;
    const int grp = threadIdx.x >> 4, sub = threadIdx.x & 15;
    uint32_t x = 0;
    for (int k = n - 1 - grp; k >= n / 2; k -= kThreads / 16) {
        const int id = ids ? ids[k] : k;
        const uint4 v = reinterpret_cast<const uint4*>(Kcu + (long long)id * kHeadDim)[sub];
        x ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    // (keeps the loads alive: the condition never holds, and the slot would be the unit's own)
    if (x == 0xfff1fff2u && p.U < 0) p.counters[4 * u] = 0;
}

template <int G>
__global__ __launch_bounds__(kThreads) void score_select_kernel(const ScoreParams p)
{
    constexpr int GH = (G + 3) / 4;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    Scratch& S = *reinterpret_cast<Scratch*>(smem_raw);
    const Lds L = carve_lds<G>(smem_raw + align16(sizeof(Scratch)), p.lds_cap);
    const int u = blockIdx.x % p.U, tid = threadIdx.x;
    const bool shadow = blockIdx.x >= (unsigned)p.U;     // second workgroup of the unit: warms the shared L2, stores nothing

    double qv[GH];      // this thread's elements of the query operand (one per head group)
#pragma unroll
    for (int hg = 0; hg < GH; ++hg) qv[hg] = query_operand_element<G>(p, u, tid + hg * kThreads);
    if (!shadow && tid < 16 * p.app_n) {       // the step's new rows go to their place in the tail buffers
        const int a = tid >> 4, c = tid & 15;
        const uint4 w = reinterpret_cast<const uint4*>(p.app_src[a])[(long long)u * 16 + c];
        reinterpret_cast<uint4*>(p.app_dst[a])[((long long)u * p.app_dst_rows + p.app_row) * 16 + c] = w;
    }

    const bool two = p.levels == 2;
    const Arrays Ag = global_arrays<G>(p, u);
    ScanState sc;
    LevelState<G> stc, stf;
    const auto nothing = [] {};
    uint32_t n_terms = 0;
    int n_f = p.n_fine;
    const bool coarse_lds = p.n_coarse <= p.lds_cap;
    if (two) {
        unsigned long long* kc = p.key_c + (long long)u * p.c_stride;
        uint8_t* fc = p.flag_c + (long long)u * p.c_stride;
        if (coarse_lds) {
            const int lin = score_level<G, true>(p, L, L.A, S, u, p.n_coarse, false, true, p.coarse_budget, false, true, qv,
                                                 shadow, shadow, kc, fc, stc, nothing);
            if (tid == 0 && !shadow) p.key_mode[2 * u] = lin;
            coarse_candidates<G, true>(p, L.A, L.A.ids, S, sc, u, shadow, n_f, n_terms);
        } else {
            // (a shadow workgroup would race with the first one on the global working arrays: it leaves)
            if (shadow) return;
            const int lin = score_level<G, false>(p, L, Ag, S, u, p.n_coarse, false, true, p.coarse_budget, false, true, qv,
                                                  false, false, kc, fc, stc, nothing);
            if (tid == 0) p.key_mode[2 * u] = lin;
            coarse_candidates<G, false>(p, Ag, L.A.ids, S, sc, u, false, n_f, n_terms);
        }
        // the fine level reads the candidate list: from LDS, or back from global memory where it is long
        __syncthreads();
    }
    if (shadow) {
        if (n_f <= p.lds_cap) touch_rows(p, two ? L.A.ids : nullptr, u, n_f);
        return;
    }
    // What the coarse level still owes -- the centroid terms of the clusters that stayed behind and
    // their share of the fine level's normaliser -- is done while the fine level's rows travel.  It
    // reads the coarse level's working arrays, which the fine level is about to reuse: the barrier
    // inside leave_behind stands between the two.
    const auto coarse_rest = [&] {
        if (!two) return;
        if (coarse_lds) {
            emit_coarse_terms<G>(p, L.A, u);
            leave_behind<G, true>(L.A, S, p.n_coarse, stc);
        } else {
            emit_coarse_terms<G>(p, Ag, u);
            leave_behind<G, false>(Ag, S, p.n_coarse, stc);
        }
    };
    unsigned long long* kf = p.key_f + (long long)u * p.f_stride;
    uint8_t* ff = p.flag_f + (long long)u * p.f_stride;
    if (n_f <= p.lds_cap) {
        const int lin = score_level<G, true>(p, L, L.A, S, u, n_f, two, false, p.key_budget, two, !two, qv, false, false, kf, ff,
                                             stf, coarse_rest);
        if (tid == 0) p.key_mode[2 * u + 1] = lin;
        fine_epilogue<G, true>(p, L.A, S, sc, u, n_f, two, n_terms);
    } else {
        const int lin = score_level<G, false>(p, L, Ag, S, u, n_f, two, false, p.key_budget, two, !two, qv, false, false, kf, ff,
                                              stf, coarse_rest);
        if (tid == 0) p.key_mode[2 * u + 1] = lin;
        fine_epilogue<G, false>(p, Ag, S, sc, u, n_f, two, n_terms);
    }
}

}  // namespace

size_t score_smem_bytes(int G, int lds_cap)
{
    const size_t GH = (size_t)(G + 3) / 4;
    return align16(sizeof(Scratch)) + GH * 512 * 8 + (size_t)kHistBuckets * 8 + (size_t)kListCap * 16 +
           (size_t)lds_cap * (8 * (size_t)G + 8 + 4 * 4 + 1) + 32;
}

template <int G>
static hipError_t launch_score_g(const ScoreParams& p, int copies, hipStream_t s)
{
    static size_t configured = 48 * 1024;
    const size_t smem = score_smem_bytes(G, p.lds_cap);
    if (smem > configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_select_kernel<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = smem;
    }
    hipLaunchKernelGGL((score_select_kernel<G>), dim3(p.U * copies), dim3(kThreads), smem, s, p);
    return hipGetLastError();
}

hipError_t launch_score_select(const ScoreParams& p, int n_compute_units, hipStream_t s)
{
    // a shadow workgroup per unit where the chip has compute units to spare and the second workgroup
    // of unit u (block u + U) lands on the same L2 slice as the first (blocks go round the 8 slices)
    const int copies = (p.U % 8 == 0 && 2 * p.U <= n_compute_units) ? 2 : 1;
    switch (p.G) {
        case 1: return launch_score_g<1>(p, copies, s);
        case 2: return launch_score_g<2>(p, copies, s);
        case 3: return launch_score_g<3>(p, copies, s);
        case 4: return launch_score_g<4>(p, copies, s);
        case 5: return launch_score_g<5>(p, copies, s);
        case 6: return launch_score_g<6>(p, copies, s);
        case 7: return launch_score_g<7>(p, copies, s);
        case 8: return launch_score_g<8>(p, copies, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace mp
