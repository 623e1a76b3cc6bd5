// Centroid scoring and budgeted cluster selection for gfx950 (Eq. 1, Sec. 3.1; two levels: Sec. 3.4).
//
// One launch per decode step, one workgroup of 512 threads per unit; the coarse level and the fine
// level run back to back in the same workgroup.
//
// Logits l[h,i] = scale * q_h . Kc_i are accumulated in fp64 (products of bf16 numbers are exact,
// so the sum carries ~1e-16 relative error and the ranking agrees with an fp64 reference except on
// ties far below any tolerance).  A group of 8 lanes (16 for more than 4 heads) shares one centroid
// row with coalesced 16-byte loads; each lane keeps its slice of every query head in registers as
// doubles and partial sums are combined with DPP.  The rank key is log(mean_h exp(l[h,i] - LSE_h)),
// the logarithm of Eq. 1 averaged over the query heads of the group.  Selection = "take clusters in
// descending key order (ties: lower id) while the running token count stays within the budget, stop
// at the first that does not fit"; token counts are positive, so this is a threshold on (key, id),
// found by a weighted most-significant-digit radix select instead of a sort.
//
// Per-entry working arrays (logits, keys, counts, ids, row starts, flags) live in LDS when a level
// has at most lds_cap entries and in a global scratch area otherwise.  The two cases are separate
// template instantiations, so that the LDS case uses LDS instructions and LDS-only barriers (the
// kernel's global stores are never read back by the same workgroup in that case).
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

__device__ __forceinline__ uint64_t descending_key(double r)
{
    uint64_t b = (uint64_t)__double_as_longlong(r);
    b = (b >> 63) ? ~b : (b | 0x8000000000000000ull);   // ascending in r
    return ~b;                                           // ascending key = descending r
}
__device__ __forceinline__ double key_to_rank(uint64_t key)
{
    uint64_t b = ~key;
    b = (b >> 63) ? (b & 0x7fffffffffffffffull) : ~b;
    return __longlong_as_double((long long)b);
}

struct Scratch {
    float gmax[kWaves * 8];           // per wave, per head: largest logit of an entry that takes part
    double red_s[kWaves * 8];         // per wave, per head: sum of N e^{l - shift}
    double extra[8];                  // log-sum of the unpromising coarse clusters' N e^l, per head
    unsigned long long hist[3][256];  // radix digit histograms: entry count << 40 | token count
    unsigned long long hkey[3][256];  // a key that fell into each bucket (THE key where the bucket holds one entry)
    unsigned long long rk_min[kWaves], rk_max[kWaves];  // per wave: smallest / largest key that takes part
    uint32_t rk_wt[kWaves], rk_cn[kWaves];              // ... their token total and their number
    uint32_t wsum[2][kWaves][2];      // per-wave totals of the two-value scan, double-buffered
};

struct Arrays {
    double* lg;            // [G][lg_stride]
    long long lg_stride;
    uint64_t* keys;
    uint32_t* wts;
    int32_t* ids;
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

// What a level hands from its log-sum-exp to later sums over subsets of its entries: the shift per
// head (the largest logit of an entry that takes part, rounded to float) and, for levels of up to
// 2 * kThreads entries, this thread's terms N_i e^{l[h,i] - shift_h} of entries tid and tid + kThreads.
template <int G>
struct LevelTerms {
    double shift[G];
    double e[2][G];
    bool kept;
};

// lse[h] = shift_h + log( sum over the workgroup of sm[h]  [+ e^{extra_h - shift_h}] ) for every head,
// where sm[h] is this thread's sum of terms already divided by e^{shift_h}.  One barrier: per-wave sums
// via DPP, then every wave adds the eight of them itself (one row of 16 lanes per head), so the
// result needs no second barrier.  S.red_s is reused by the next call: callers have a barrier
// between two calls.
template <int G, bool kLds>
__device__ __forceinline__ void combine_lse(Scratch& S, const double (&shift)[G], const double (&sm)[G], bool with_extra,
                                            double (&lse)[G])
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const double t = wave_sum_f64(sm[h]);
        if (lane == 0) S.red_s[wave * 8 + h] = t;
    }
    phase_sync<kLds>();
#pragma unroll
    for (int h0 = 0; h0 < G; h0 += 4) {
        const int h = h0 + (lane >> 4), w = lane & 15;
        const bool live = h < G && w < kWaves;
        double t = row_sum_f64(live ? S.red_s[w * 8 + h] : 0.0);
        double sh = -INFINITY;
#pragma unroll
        for (int hh = 0; hh < 4; ++hh)
            if (h0 + hh < G && (lane >> 4) == hh) sh = shift[h0 + hh];
        double r;
        if (with_extra && h < G) {
            const double ex = S.extra[h];
            const double M = fmax(sh, ex);
            if (M == -INFINITY) {
                r = -INFINITY;
            } else {
                const double a = (t > 0.0) ? t * exp_shifted(sh - M) : 0.0;
                r = M + log(a + exp_shifted(ex - M));
            }
        } else {
            r = (t > 0.0) ? sh + log(t) : -INFINITY;
        }
#pragma unroll
        for (int hh = 0; hh < 4; ++hh)
            if (h0 + hh < G) lse[h0 + hh] = readlane_f64(r, 16 * hh);
    }
}

// Exclusive prefix sums of two values per thread over one chunk of kThreads threads, with running
// totals carried in registers (every thread adds the same chunk totals, so they stay uniform).
// One barrier per call: the per-wave totals are double-buffered by the parity of `calls`.
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
    uint32_t off_a = 0, off_b = 0, tot_a = 0, tot_b = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t wa = s.wsum[par][w][0], wb = s.wsum[par][w][1];
        off_a += (w < wave) ? wa : 0u;
        off_b += (w < wave) ? wb : 0u;
        tot_a += wa;
        tot_b += wb;
    }
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

template <int kLanes>
__device__ __forceinline__ double group_sum_f64(double v)
{
    v += dpp_f64<kDppXor1>(v);
    v += dpp_f64<kDppXor2>(v);
    v += dpp_f64<kDppHalfMirror>(v);
    if constexpr (kLanes == 16) v += dpp_f64<kDppMirror>(v);
    return v;
}

// One level: logits, Eq. 1 normaliser, rank keys, budgeted selection.  On return A.flags holds the
// selected / promising mask, A.wts the member counts (0 = takes no part), A.lg the logits, A.keys
// the rank keys.  Entry i stands for cluster id (use_ids ? A.ids[i] : i).
template <int G, bool kLds, int LPE>
__device__ __forceinline__ void score_level(const ScoreParams& p, const Arrays& A, Scratch& S, int u, int n,
                                            bool use_ids, bool coarse, const double (&qreg)[G][128 / LPE],
                                            long long budget, bool with_extra, LevelTerms<G>& T)
{
    constexpr int DPL = 128 / LPE;           // dims per lane: 16 or 8
    constexpr int EPI = kThreads / LPE;      // entries per pass of the workgroup
    const int tid = threadIdx.x;
    const int row_off = coarse ? p.fcap : 0;
    const int32_t* Nu = p.N + (long long)u * p.tab_rows + row_off;
    const uint16_t* Kcu = p.Kc + ((long long)u * p.tab_rows + row_off) * kHeadDim;
    const int32_t* st = coarse ? p.cstart + (long long)u * p.cstart_stride : p.fstart + (long long)u * p.fstart_stride;

    // member counts and row starts of the first 2*kThreads entries: loads issued now, stored after the logits
    int pre_w[2] = {0, 0}, pre_a[2] = {0, 0}, pre_b[2] = {0, 0};
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int i = tid + k * kThreads;
        if (i < n) {
            const int id = use_ids ? A.ids[i] : i;
            pre_w[k] = Nu[id];
            pre_a[k] = st[id];
            if (coarse) pre_b[k] = st[id + 1];
        }
    }
    // ---- logits: LPE lanes per entry, DPL dims per lane; two entries per lane and pass, the rows of
    // the next pass are requested before the current ones are used ----
    {
        const int sub = tid % LPE, grp = tid / LPE;
        uint4 nxt[2][DPL / 8];
        int nxt_w[2];
        float mxf[G];        // largest logit, per head, of the entries with members that this lane finishes
#pragma unroll
        for (int h = 0; h < G; ++h) mxf[h] = -INFINITY;
        auto request = [&](int i0) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int i = i0 + j * EPI + grp;
#pragma unroll
                for (int v = 0; v < DPL / 8; ++v) nxt[j][v] = make_uint4(0, 0, 0, 0);
                nxt_w[j] = 0;
                if (i < n) {
                    const int id = use_ids ? A.ids[i] : i;
                    const uint4* kp = reinterpret_cast<const uint4*>(Kcu + (long long)id * kHeadDim + DPL * sub);
#pragma unroll
                    for (int v = 0; v < DPL / 8; ++v) nxt[j][v] = kp[v];
                    nxt_w[j] = Nu[id];
                }
            }
        };
        request(0);
        for (int i0 = 0; i0 < n; i0 += 2 * EPI) {
            uint4 kv[2][DPL / 8];
            int kw[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int v = 0; v < DPL / 8; ++v) kv[j][v] = nxt[j][v];
                kw[j] = nxt_w[j];
            }
            if (i0 + 2 * EPI < n) request(i0 + 2 * EPI);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int i = i0 + j * EPI + grp;
                double kd[DPL];
#pragma unroll
                for (int v = 0; v < DPL / 8; ++v) {
                    const uint32_t w[4] = {kv[j][v].x, kv[j][v].y, kv[j][v].z, kv[j][v].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        kd[8 * v + 2 * e] = (double)bf16lo_to_f32(w[e]);
                        kd[8 * v + 2 * e + 1] = (double)bf16hi_to_f32(w[e]);
                    }
                }
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    double a = 0.0;
#pragma unroll
                    for (int e = 0; e < DPL; ++e) a = fma(qreg[h][e], kd[e], a);
                    a = group_sum_f64<LPE>(a) * p.scale;
                    if (sub == 0 && i < n) {
                        A.lg[h * A.lg_stride + i] = a;
                        if (kw[j] > 0) mxf[h] = fmaxf(mxf[h], (float)a);
                    }
                }
            }
        }
        const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float m = wave_max_f32(mxf[h]);
            if (lane == 0) S.gmax[wave * 8 + h] = m;
        }
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int i = tid + k * kThreads;
        if (i < n) {
            A.wts[i] = (uint32_t)(pre_w[k] > 0 ? pre_w[k] : 0);
            A.aux[i] = pre_a[k];
            if (coarse) A.aux2[i] = pre_b[k];
        }
    }
    for (int i = tid + 2 * kThreads; i < n; i += kThreads) {
        const int id = use_ids ? A.ids[i] : i;
        const int w = Nu[id];
        A.wts[i] = (uint32_t)(w > 0 ? w : 0);
        A.aux[i] = st[id];
        if (coarse) A.aux2[i] = st[id + 1];
    }
    phase_sync<kLds>();

    // ---- per-head normaliser of Eq. 1: LSE_h = log( sum_i N_i e^{l[h,i]} + e^{extra_h} ) ----
    // shift: the largest logit of the level (the waves left theirs in S.gmax before the barrier above)
    double lse[G];
    {
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float m = S.gmax[h];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) m = fmaxf(m, S.gmax[w * 8 + h]);
            T.shift[h] = (double)m;
        }
        T.kept = (G <= 6) && n <= 2 * kThreads;     // (larger groups have no registers to spare for the kept terms)
        double sm[G];
#pragma unroll
        for (int h = 0; h < G; ++h) sm[h] = T.e[0][h] = T.e[1][h] = 0.0;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int i = tid + k * kThreads;
            if (i < n && A.wts[i] != 0) {
                const double w = (double)A.wts[i];
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const double e = w * exp_shifted(A.lg[h * A.lg_stride + i] - T.shift[h]);
                    if constexpr (G <= 6) T.e[k][h] = e;
                    sm[h] += e;
                }
            }
        }
        for (int i = tid + 2 * kThreads; i < n; i += kThreads)
            if (A.wts[i] != 0) {
                const double w = (double)A.wts[i];
#pragma unroll
                for (int h = 0; h < G; ++h) sm[h] += w * exp_shifted(A.lg[h * A.lg_stride + i] - T.shift[h]);
            }
        combine_lse<G, kLds>(S, T.shift, sm, with_extra, lse);
    }

    // ---- rank keys ----
    const double logG = log((double)G);
    for (int i = tid; i < n; i += kThreads) {
        uint64_t key = ~0ull;
        if (A.wts[i]) {
            double t[G], tm = -INFINITY;
#pragma unroll
            for (int h = 0; h < G; ++h) {
                t[h] = A.lg[h * A.lg_stride + i] - lse[h];
                tm = fmax(tm, t[h]);
            }
            double r = tm - logG;
            if constexpr (G > 1) {
                double ssum = 0.0;
#pragma unroll
                for (int h = 0; h < G; ++h) ssum += exp_shifted(t[h] - tm);
                r += log(ssum);
            }
            key = descending_key(r);
        }
        A.keys[i] = key;
    }
    // (the barrier that publishes the keys is the first one inside radix_select)

    // ---- budgeted selection ----
    uint64_t kstar = 0, acc = 0;
    uint32_t ties = 0;
    const bool bounded = radix_select<kLds>(A.keys, A.wts, n, budget, S, kstar, acc, ties);
    for (int i = tid; i < n; i += kThreads) {
        uint8_t f = 0;
        if (A.wts[i]) {
            if (!bounded) f = 1;
            else {
                const uint64_t k = A.keys[i];
                if (k < kstar) f = 1;
                else if (k == kstar && ties > 1) {
                    // exactly equal keys: lower position first, keep while the running count still fits
                    uint64_t run = acc;
                    for (int j = 0; j <= i; ++j)
                        if (A.wts[j] && A.keys[j] == kstar) run += A.wts[j];
                    f = ((long long)run <= budget) ? 1 : 0;
                }
            }
        }
        A.flags[i] = f;
    }
    phase_sync<kLds>();
}

// Per-position views for the getters: rank key (NaN where the entry took no part) and flag.
__device__ __forceinline__ void write_views(const Arrays& A, int n, double* r_out, uint8_t* flag_out)
{
    for (int i = threadIdx.x; i < n; i += kThreads) {
        r_out[i] = A.wts[i] ? key_to_rank(A.keys[i]) : __longlong_as_double(0x7ff8000000000000ll);
        flag_out[i] = A.flags[i];
    }
}

// One centroid-term entry (Eq. 2): the row of the value centroid and log2( N_i e^{l[h,i]} ) per head.
template <int G>
__device__ __forceinline__ void emit_term(const ScoreParams& p, const Arrays& A, int u, int i, int row, uint32_t slot)
{
    const double kLog2e = 1.4426950408889634;
    const long long o = (long long)u * p.mp_stride + slot;
    p.mp_rows[o] = row;
    const double lnN = log((double)A.wts[i]);
#pragma unroll
    for (int h = 0; h < G; ++h) p.mp_scores[o * G + h] = (float)((A.lg[h * A.lg_stride + i] + lnN) * kLog2e);
}

template <int G, bool kLds>
__device__ __forceinline__ Arrays make_arrays(unsigned char* lds, const ScoreParams& p, int u)
{
    Arrays A;
    if constexpr (kLds) {
        A.lg = reinterpret_cast<double*>(lds);
        A.lg_stride = p.lds_cap;
        A.keys = reinterpret_cast<uint64_t*>(A.lg + (size_t)G * p.lds_cap);
        A.wts = reinterpret_cast<uint32_t*>(A.keys + p.lds_cap);
        A.ids = reinterpret_cast<int32_t*>(A.wts + p.lds_cap);
        A.aux = A.ids + p.lds_cap;
        A.aux2 = A.aux + p.lds_cap;
        A.flags = reinterpret_cast<uint8_t*>(A.aux2 + p.lds_cap);
    } else {
        A.lg = p.lg + (long long)u * G * p.lg_stride;
        A.lg_stride = p.lg_stride;
        A.keys = reinterpret_cast<uint64_t*>(p.g_keys) + (long long)u * p.g_stride;
        A.wts = p.g_wts + (long long)u * p.g_stride;
        A.ids = p.cand + (long long)u * p.f_stride;       // the candidate list itself
        A.aux = p.g_aux + (long long)u * p.g_stride;
        A.aux2 = p.g_aux2 + (long long)u * p.g_stride;
        A.flags = p.g_flags + (long long)u * p.g_stride;
    }
    return A;
}

// Coarse level (Sec. 3.4): score all coarse clusters, keep the promising ones, emit centroid terms
// for the others, leave the log-sum of their N e^l in S.extra and the candidate list (children of
// the promising clusters, ascending fine id) in global memory and, as far as it fits, in the LDS
// slot the fine level reads its ids from (unused by the coarse level, whose entries are 0..n-1).
template <int G, bool kLds, int LPE>
__device__ __forceinline__ void coarse_phase(const ScoreParams& p, unsigned char* lds, Scratch& S, ScanState& sc,
                                             int u, const double (&qreg)[G][128 / LPE], int& n_cand,
                                             uint32_t& n_terms)
{
    const int tid = threadIdx.x;
    const int n_c = p.n_coarse;
    const Arrays C = make_arrays<G, kLds>(lds, p, u);
    LevelTerms<G> T;
    score_level<G, kLds, LPE>(p, C, S, u, n_c, false, true, qreg, p.coarse_budget, false, T);
    // log-sum of the unpromising clusters: the same terms as in the level's own normaliser, so the
    // exponentials are not taken again where they were kept
    double ex[G];
    {
        double sm[G];
#pragma unroll
        for (int h = 0; h < G; ++h) sm[h] = 0.0;
        if (G <= 6 && T.kept) {
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int i = tid + k * kThreads;
                if (i < n_c && C.wts[i] != 0 && !C.flags[i])
#pragma unroll
                    for (int h = 0; h < G; ++h) sm[h] += T.e[k][h];
            }
        } else {
            for (int i = tid; i < n_c; i += kThreads)
                if (C.wts[i] != 0 && !C.flags[i]) {
                    const double w = (double)C.wts[i];
#pragma unroll
                    for (int h = 0; h < G; ++h) sm[h] += w * exp_shifted(C.lg[h * C.lg_stride + i] - T.shift[h]);
                }
        }
        combine_lse<G, kLds>(S, T.shift, sm, false, ex);
    }
#pragma unroll
    for (int h = 0; h < G; ++h)
        if (tid == h) S.extra[h] = ex[h];
    int32_t* cand_g = p.cand + (long long)u * p.f_stride;
    int32_t* cand_l = make_arrays<G, true>(lds, p, u).ids;
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
            cand_g[o] = f;
            if (o < (uint32_t)p.lds_cap) cand_l[o] = f;
        }
        if (emit) emit_term<G>(p, C, u, i, p.fcap + i, slot);
    }
    n_cand = (int)sc.carry_a;
    n_terms = sc.carry_b;
    write_views(C, n_c, p.r_c + (long long)u * p.c_stride, p.flag_c + (long long)u * p.c_stride);
    if (tid == 0) {
        p.n_cand[u] = n_cand;
        p.counters[4 * u + 2] = n_c;
    }
    // the fine level reuses the coarse level's working arrays; with more candidates than fit in LDS
    // it also reads the candidate list back from global memory
    __syncthreads();
}

// Fine level: score the candidates, select within the key budget, emit centroid terms for the
// unselected candidates and the flat list of stored rows of the selected clusters.
template <int G, bool kLds, int LPE>
__device__ __forceinline__ void fine_phase(const ScoreParams& p, unsigned char* lds, Scratch& S, ScanState& sc,
                                           int u, const double (&qreg)[G][128 / LPE], int n_f, bool two,
                                           uint32_t n_terms)
{
    const int tid = threadIdx.x;
    const Arrays F = make_arrays<G, kLds>(lds, p, u);
    LevelTerms<G> T;
    score_level<G, kLds, LPE>(p, F, S, u, n_f, two, false, qreg, p.key_budget, two, T);
    write_views(F, n_f, p.r_f + (long long)u * p.f_stride, p.flag_f + (long long)u * p.f_stride);

    // One scan gives every selected cluster (ascending fine id) its slot in a compact list and the
    // offset of its rows in the flat row list, and every unselected candidate its centroid-term slot.
    // The compact list reuses the storage of the keys, which nobody reads after the views above.
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
        }
        if (emit) emit_term<G>(p, F, u, i, two ? F.ids[i] : i, n_terms + (packed >> 16));
    }
    const uint32_t total = sc.carry_a, n_sel = sc.carry_b & 0xffffu;
    n_terms += sc.carry_b >> 16;
    phase_sync<kLds>();
    // expansion: one row of 16 lanes per selected cluster, the next cluster's entry fetched early
    int32_t* ro = p.rows + (long long)u * p.rows_stride;
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

template <int G>
__global__ __launch_bounds__(kThreads) void score_select_kernel(const ScoreParams p)
{
    constexpr int LPE = (G <= 4) ? 8 : 16;   // lanes per entry in the logits phase
    constexpr int DPL = 128 / LPE;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    Scratch& S = *reinterpret_cast<Scratch*>(smem_raw);
    unsigned char* lds = smem_raw + ((sizeof(Scratch) + 15) & ~size_t(15));
    const int u = blockIdx.x, tid = threadIdx.x;

    if (tid < 16 * p.app_n) {       // the step's new rows go to their place in the tail buffers
        const int a = tid >> 4, c = tid & 15;
        const uint4 w = reinterpret_cast<const uint4*>(p.app_src[a])[(long long)u * 16 + c];
        reinterpret_cast<uint4*>(p.app_dst[a])[((long long)u * p.app_dst_rows + p.app_row) * 16 + c] = w;
    }

    // query slice of this lane: dims [DPL*sub, DPL*sub + DPL) of every head, as doubles
    double qreg[G][DPL];
    {
        const int sub = tid % LPE;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const uint4* qp = reinterpret_cast<const uint4*>(p.q + ((long long)u * G + h) * kHeadDim + DPL * sub);
#pragma unroll
            for (int v = 0; v < DPL / 8; ++v) {
                const uint4 qv = qp[v];
                const uint32_t w[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    qreg[h][8 * v + 2 * e] = (double)bf16lo_to_f32(w[e]);
                    qreg[h][8 * v + 2 * e + 1] = (double)bf16hi_to_f32(w[e]);
                }
            }
        }
    }

    const bool two = p.levels == 2;
    ScanState sc;
    uint32_t n_terms = 0;
    int n_f = p.n_fine;
    if (two) {
        if (p.n_coarse <= p.lds_cap) coarse_phase<G, true, LPE>(p, lds, S, sc, u, qreg, n_f, n_terms);
        else coarse_phase<G, false, LPE>(p, lds, S, sc, u, qreg, n_f, n_terms);
    }
    if (n_f <= p.lds_cap) fine_phase<G, true, LPE>(p, lds, S, sc, u, qreg, n_f, two, n_terms);
    else fine_phase<G, false, LPE>(p, lds, S, sc, u, qreg, n_f, two, n_terms);
}

}  // namespace

size_t score_smem_bytes(int G, int lds_cap)
{
    return ((sizeof(Scratch) + 15) & ~size_t(15)) + (size_t)lds_cap * (8 * (size_t)G + 8 + 4 * 4 + 1) + 32;
}

template <int G>
static hipError_t launch_score_g(const ScoreParams& p, hipStream_t s)
{
    static size_t configured = 48 * 1024;
    const size_t smem = score_smem_bytes(G, p.lds_cap);
    if (smem > configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_select_kernel<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = smem;
    }
    hipLaunchKernelGGL((score_select_kernel<G>), dim3(p.U), dim3(kThreads), smem, s, p);
    return hipGetLastError();
}

hipError_t launch_score_select(const ScoreParams& p, hipStream_t s)
{
    switch (p.G) {
        case 1: return launch_score_g<1>(p, s);
        case 2: return launch_score_g<2>(p, s);
        case 3: return launch_score_g<3>(p, s);
        case 4: return launch_score_g<4>(p, s);
        case 5: return launch_score_g<5>(p, s);
        case 6: return launch_score_g<6>(p, s);
        case 7: return launch_score_g<7>(p, s);
        case 8: return launch_score_g<8>(p, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace mp
