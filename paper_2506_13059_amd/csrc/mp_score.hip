// Centroid scoring and budgeted cluster selection for gfx950 (Eq. 1, Sec. 3.1; two levels: Sec. 3.4).
//
// One launch per decode step, one workgroup of 512 threads per unit; the coarse level and the fine
// level run back to back in the same workgroup, so candidate ids, counts and the unpromising
// clusters' log-sum never leave the chip.
//
// Logits l[h,i] = scale * q_h . Kc_i are accumulated in fp64 (products of bf16 numbers are exact,
// so the sum carries ~1e-16 relative error and the ranking agrees with an fp64 reference except on
// ties far below any tolerance).  16 lanes share one centroid row (one coalesced 16-byte load per
// lane), each lane keeps its 8 query dims of every head in registers as doubles, partial sums are
// combined with DPP.  The rank key is log(mean_h exp(l[h,i] - LSE_h)), the logarithm of Eq. 1
// averaged over the query heads of the group.  Selection = "take clusters in descending key order
// (ties: lower id) while the running token count stays within the budget, stop at the first that
// does not fit"; token counts are positive, so this is a threshold on (key, id), found by a
// weighted most-significant-digit radix select instead of a sort.
//
// Per-entry working arrays (logits, keys, counts, ids, row starts, flags) live in LDS when a level
// has at most lds_cap entries and in a global scratch area otherwise; they are reached through
// generic pointers chosen per level at run time.
//
// Outputs for the value pass: the flat list of stored rows of the selected clusters' keys, and one
// "centroid term" entry (value-centroid row + ready-made logits) per cluster that stays behind at
// either level (unpromising coarse clusters, unselected fine candidates).
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

struct Scratch {
    double red[kWaves * 8];      // cross-wave reductions, up to 8 heads
    double bc[8];                // broadcast values (per head)
    double extra[8];             // log-sum of the unpromising coarse clusters' N e^l, per head
    uint32_t hist_w[256];
    uint32_t hist_c[256];
    uint32_t wsum[kWaves];
    uint32_t carry;
    uint32_t sel_digit, sel_found, sel_cnt;
    unsigned long long sel_acc;
    unsigned long long sel_key;
};

struct Arrays {
    double* lg;            // [G][lg_stride]
    long long lg_stride;
    uint64_t* keys;
    uint32_t* wts;
    int32_t* ids;
    int32_t* aux;          // fine: first stored row; coarse: first child
    int32_t* aux2;         // coarse: end of children
    uint8_t* flags;
};

template <int G>
__device__ __forceinline__ void block_max(double (&v)[G], Scratch& s)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const double w = wave_max_f64(v[h]);
        if (lane == 0) s.red[wave * 8 + h] = w;
    }
    __syncthreads();
    if (threadIdx.x < G) {
        double m = s.red[threadIdx.x];
        for (int w = 1; w < kWaves; ++w) m = fmax(m, s.red[w * 8 + threadIdx.x]);
        s.bc[threadIdx.x] = m;
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < G; ++h) v[h] = s.bc[h];
    __syncthreads();
}

// sum over the workgroup in a fixed order (bit-reproducible)
template <int G>
__device__ __forceinline__ void block_sum(double (&v)[G], Scratch& s)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const double w = wave_sum_f64(v[h]);
        if (lane == 0) s.red[wave * 8 + h] = w;
    }
    __syncthreads();
    if (threadIdx.x < G) {
        double m = 0.0;
        for (int w = 0; w < kWaves; ++w) m += s.red[w * 8 + threadIdx.x];
        s.bc[threadIdx.x] = m;
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < G; ++h) v[h] = s.bc[h];
    __syncthreads();
}

// Exclusive prefix sum over one chunk of kThreads values (one per thread) with a running carry in
// s.carry; returns the exclusive prefix including the carry.  All threads must call.
__device__ __forceinline__ uint32_t chunk_excl_scan(uint32_t v, Scratch& s)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t incl = wave_incl_scan_u32(v);
    if (lane == 63) s.wsum[wave] = incl;
    __syncthreads();
    uint32_t woff = 0;
    for (int w = 0; w < wave; ++w) woff += s.wsum[w];
    const uint32_t carry = s.carry;
    const uint32_t excl = carry + woff + incl - v;
    __syncthreads();
    if (threadIdx.x == kThreads - 1) s.carry = carry + woff + incl;
    __syncthreads();
    return excl;
}

// Weighted radix select.  keys[i] ascending = rank order, wts[i] > 0 for entries that take part
// (entries with wts == 0 are never selected).  Finds the key K* of the first entry (in (key, index)
// order) at which the running weight exceeds `budget`, the weight `acc` of all entries with key <
// K*, and how many entries carry exactly K*.  Returns false if everything fits.
__device__ __forceinline__ bool radix_select(const uint64_t* keys, const uint32_t* wts, int n, long long budget,
                                             Scratch& s, uint64_t& kstar, uint64_t& acc_out, uint32_t& ties_out)
{
    const int tid = threadIdx.x;
    uint64_t prefix = 0;
    uint64_t acc = 0;
    for (int pass = 0; pass < 8; ++pass) {
        const int shift = 56 - 8 * pass;
        if (tid < 256) {
            s.hist_w[tid] = 0;
            s.hist_c[tid] = 0;
        }
        __syncthreads();
        for (int i = tid; i < n; i += kThreads) {
            const uint32_t w = wts[i];
            if (w == 0) continue;
            const uint64_t k = keys[i];
            if (pass == 0 || (k >> (shift + 8)) == prefix) {
                const uint32_t d = (uint32_t)(k >> shift) & 255u;
                atomicAdd(&s.hist_w[d], w);
                atomicAdd(&s.hist_c[d], 1u);
            }
        }
        __syncthreads();
        if (tid < 64) {
            const uint4 w4 = *reinterpret_cast<const uint4*>(&s.hist_w[4 * tid]);
            const uint32_t sum = w4.x + w4.y + w4.z + w4.w;
            const uint32_t incl = wave_incl_scan_u32(sum);
            const bool cross = (long long)(acc + incl) > budget;
            const unsigned long long mask = __ballot(cross);
            if (mask == 0ull) {
                if (tid == 0) s.sel_found = 0;
            } else {
                const int first = __ffsll((long long)mask) - 1;
                if (tid == first) {
                    uint64_t a = acc + incl - sum;
                    uint32_t d = 4 * tid;
                    const uint32_t ws[4] = {w4.x, w4.y, w4.z, w4.w};
                    for (int j = 0; j < 4; ++j) {
                        if ((long long)(a + ws[j]) > budget) { d = 4 * tid + j; break; }
                        a += ws[j];
                    }
                    s.sel_found = 1;
                    s.sel_digit = d;
                    s.sel_acc = a;
                    s.sel_cnt = s.hist_c[d];
                }
            }
        }
        __syncthreads();
        if (!s.sel_found) return false;       // only possible in pass 0: everything fits
        acc = s.sel_acc;
        prefix = (prefix << 8) | s.sel_digit;
        const uint32_t cnt = s.sel_cnt;
        __syncthreads();
        if (cnt == 1 && pass < 7) {
            // a single entry carries the boundary: its full key is K*
            for (int i = tid; i < n; i += kThreads) {
                if (wts[i] == 0) continue;
                const uint64_t k = keys[i];
                if ((k >> shift) == prefix) s.sel_key = k;
            }
            __syncthreads();
            kstar = s.sel_key;
            acc_out = acc;
            ties_out = 1;
            __syncthreads();
            return true;
        }
    }
    kstar = prefix;
    acc_out = acc;
    ties_out = s.sel_cnt;
    return true;
}

__device__ __forceinline__ double sum16_f64(double v)
{
    v += dpp_f64<kDppXor1>(v);
    v += dpp_f64<kDppXor2>(v);
    v += dpp_f64<kDppHalfMirror>(v);
    v += dpp_f64<kDppMirror>(v);
    return v;
}

// One level: logits, Eq. 1 normaliser, rank keys, budgeted selection.  On return A.flags holds the
// selected / promising mask, A.wts the member counts (0 = takes no part), A.lg the logits.
// Entry i stands for cluster id (use_ids ? A.ids[i] : i).
template <int G>
__device__ __forceinline__ void score_level(const ScoreParams& p, const Arrays& A, Scratch& S, int u, int n,
                                            bool use_ids, bool coarse, const double (&qreg)[G][8], long long budget,
                                            bool with_extra, double* r_out, uint8_t* flag_out)
{
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
    // ---- logits: 16 lanes per entry, 8 dims per lane, 4 entries in flight per lane ----
    {
        const int sub = tid & 15, grp = tid >> 4;
        for (int i0 = 0; i0 < n; i0 += 4 * (kThreads / 16)) {
            uint4 kv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = i0 + j * (kThreads / 16) + grp;
                kv[j] = make_uint4(0, 0, 0, 0);
                if (i < n) {
                    const int id = use_ids ? A.ids[i] : i;
                    kv[j] = reinterpret_cast<const uint4*>(Kcu + (long long)id * kHeadDim)[sub];
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = i0 + j * (kThreads / 16) + grp;
                const uint32_t w[4] = {kv[j].x, kv[j].y, kv[j].z, kv[j].w};
                double kd[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    kd[2 * e] = (double)bf16lo_to_f32(w[e]);
                    kd[2 * e + 1] = (double)bf16hi_to_f32(w[e]);
                }
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    double a = 0.0;
#pragma unroll
                    for (int e = 0; e < 8; ++e) a = fma(qreg[h][e], kd[e], a);
                    a = sum16_f64(a);
                    if (sub == 0 && i < n) A.lg[h * A.lg_stride + i] = a * p.scale;
                }
            }
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
    __syncthreads();

    // ---- per-head normaliser of Eq. 1: LSE_h = log( sum_i N_i e^{l[h,i]} + e^{extra_h} ) ----
    double lse[G];
    {
        double mx[G];
#pragma unroll
        for (int h = 0; h < G; ++h) mx[h] = with_extra ? S.extra[h] : -INFINITY;
        for (int i = tid; i < n; i += kThreads)
            if (A.wts[i])
#pragma unroll
                for (int h = 0; h < G; ++h) mx[h] = fmax(mx[h], A.lg[h * A.lg_stride + i]);
        block_max<G>(mx, S);
        double sm[G];
#pragma unroll
        for (int h = 0; h < G; ++h) sm[h] = 0.0;
        for (int i = tid; i < n; i += kThreads) {
            const uint32_t w = A.wts[i];
            if (w)
#pragma unroll
                for (int h = 0; h < G; ++h) sm[h] += (double)w * exp(A.lg[h * A.lg_stride + i] - mx[h]);
        }
        if (tid == 0 && with_extra)
#pragma unroll
            for (int h = 0; h < G; ++h)
                if (S.extra[h] != -INFINITY) sm[h] += exp(S.extra[h] - mx[h]);
        block_sum<G>(sm, S);
#pragma unroll
        for (int h = 0; h < G; ++h) lse[h] = (mx[h] == -INFINITY) ? -INFINITY : mx[h] + log(sm[h]);
    }

    // ---- rank keys ----
    const double logG = log((double)G);
    for (int i = tid; i < n; i += kThreads) {
        double r = __longlong_as_double(0x7ff8000000000000ll);
        uint64_t key = ~0ull;
        if (A.wts[i]) {
            double t[G], tm = -INFINITY;
#pragma unroll
            for (int h = 0; h < G; ++h) {
                t[h] = A.lg[h * A.lg_stride + i] - lse[h];
                tm = fmax(tm, t[h]);
            }
            double ssum = 0.0;
#pragma unroll
            for (int h = 0; h < G; ++h) ssum += exp(t[h] - tm);
            r = tm + log(ssum) - logG;
            key = descending_key(r);
        }
        A.keys[i] = key;
        r_out[i] = r;
    }
    __syncthreads();

    // ---- budgeted selection ----
    uint64_t kstar = 0, acc = 0;
    uint32_t ties = 0;
    const bool bounded = radix_select(A.keys, A.wts, n, budget, S, kstar, acc, ties);
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
        flag_out[i] = f;
    }
    __syncthreads();
}

// Centroid-term entries for every entry that takes part but was not kept at this level.
template <int G>
__device__ __forceinline__ uint32_t emit_terms(const ScoreParams& p, const Arrays& A, Scratch& S, int u, int n,
                                               bool use_ids, int row_off, uint32_t base)
{
    const int tid = threadIdx.x;
    const double kLog2e = 1.4426950408889634;
    if (tid == 0) S.carry = 0;
    __syncthreads();
    for (int i0 = 0; i0 < n; i0 += kThreads) {
        const int i = i0 + tid;
        const bool emit = (i < n) && A.wts[i] && !A.flags[i];
        const uint32_t pos = chunk_excl_scan(emit ? 1u : 0u, S);
        if (emit) {
            const int id = use_ids ? A.ids[i] : i;
            const long long o = (long long)u * p.mp_stride + base + pos;
            p.mp_rows[o] = row_off + id;
            const double lnN = log((double)A.wts[i]);
#pragma unroll
            for (int h = 0; h < G; ++h) p.mp_scores[o * G + h] = (float)((A.lg[h * A.lg_stride + i] + lnN) * kLog2e);
        }
    }
    const uint32_t cnt = S.carry;
    __syncthreads();
    return cnt;
}

template <int G>
__global__ __launch_bounds__(kThreads) void score_select_kernel(const ScoreParams p)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    Scratch& S = *reinterpret_cast<Scratch*>(smem_raw);
    // LDS working arrays for a level with at most lds_cap entries
    unsigned char* base = smem_raw + ((sizeof(Scratch) + 15) & ~size_t(15));
    Arrays L;
    L.lg = reinterpret_cast<double*>(base);
    L.lg_stride = p.lds_cap;
    L.keys = reinterpret_cast<uint64_t*>(L.lg + (size_t)G * p.lds_cap);
    L.wts = reinterpret_cast<uint32_t*>(L.keys + p.lds_cap);
    L.ids = reinterpret_cast<int32_t*>(L.wts + p.lds_cap);
    L.aux = L.ids + p.lds_cap;
    L.aux2 = L.aux + p.lds_cap;
    L.flags = reinterpret_cast<uint8_t*>(L.aux2 + p.lds_cap);
    const int u = blockIdx.x, tid = threadIdx.x;
    // the same arrays in global scratch, for levels that do not fit
    Arrays Gm;
    Gm.lg = p.lg + (long long)u * G * p.lg_stride;
    Gm.lg_stride = p.lg_stride;
    Gm.keys = reinterpret_cast<uint64_t*>(p.g_keys) + (long long)u * p.g_stride;
    Gm.wts = p.g_wts + (long long)u * p.g_stride;
    Gm.ids = p.g_ids + (long long)u * p.g_stride;
    Gm.aux = p.g_aux + (long long)u * p.g_stride;
    Gm.aux2 = p.g_aux2 + (long long)u * p.g_stride;
    Gm.flags = p.g_flags + (long long)u * p.g_stride;

    // query slice of this lane: dims [8*sub, 8*sub+8) of every head, as doubles
    double qreg[G][8];
    {
        const int sub = tid & 15;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const uint4 qv = reinterpret_cast<const uint4*>(p.q + ((long long)u * G + h) * kHeadDim)[sub];
            const uint32_t w[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                qreg[h][2 * e] = (double)bf16lo_to_f32(w[e]);
                qreg[h][2 * e + 1] = (double)bf16hi_to_f32(w[e]);
            }
        }
    }
    if (tid == 0) S.carry = 0;
    __syncthreads();

    const bool two = p.levels == 2;
    uint32_t n_terms = 0;
    int n_f = p.n_fine;
    bool fine_ids = false;
    Arrays F = (p.n_fine <= p.lds_cap) ? L : Gm;
    if (two) {
        const int n_c = p.n_coarse;
        const Arrays C = (n_c <= p.lds_cap) ? L : Gm;
        score_level<G>(p, C, S, u, n_c, false, true, qreg, p.coarse_budget, false, p.r_c + (long long)u * p.c_stride,
                       p.flag_c + (long long)u * p.c_stride);
        // log-sum of the unpromising clusters' N e^{l}: joins the fine level's Eq. 1 denominator
        {
            double mx[G], sm[G];
#pragma unroll
            for (int h = 0; h < G; ++h) { mx[h] = -INFINITY; sm[h] = 0.0; }
            for (int i = tid; i < n_c; i += kThreads)
                if (C.wts[i] && !C.flags[i])
#pragma unroll
                    for (int h = 0; h < G; ++h) mx[h] = fmax(mx[h], C.lg[h * C.lg_stride + i]);
            block_max<G>(mx, S);
            for (int i = tid; i < n_c; i += kThreads)
                if (C.wts[i] && !C.flags[i])
#pragma unroll
                    for (int h = 0; h < G; ++h) sm[h] += (double)C.wts[i] * exp(C.lg[h * C.lg_stride + i] - mx[h]);
            block_sum<G>(sm, S);
            if (tid < G) {
                double v = -INFINITY;
#pragma unroll
                for (int h = 0; h < G; ++h)
                    if (h == tid) v = (mx[h] == -INFINITY) ? -INFINITY : mx[h] + log(sm[h]);
                S.extra[tid] = v;
            }
        }
        if (p.use_mp) n_terms = emit_terms<G>(p, C, S, u, n_c, false, p.fcap, 0);
        // candidates: the children of the promising clusters, ascending fine id, written to the global
        // candidate list first (the coarse arrays may share LDS with the fine ones and are still read).
        if (tid == 0) S.carry = 0;
        __syncthreads();
        int32_t* cand_g = p.cand + (long long)u * p.f_stride;
        for (int i0 = 0; i0 < n_c; i0 += kThreads) {
            const int i = i0 + tid;
            int c0 = 0, c1 = 0;
            if (i < n_c && C.flags[i]) { c0 = C.aux[i]; c1 = C.aux2[i]; }
            const uint32_t pos = chunk_excl_scan((uint32_t)(c1 - c0), S);
            for (int f = c0; f < c1; ++f) cand_g[pos + (f - c0)] = f;
        }
        n_f = (int)S.carry;
        __syncthreads();               // every read of the coarse arrays is done, the candidate list is written
        F = (n_f <= p.lds_cap) ? L : Gm;
        for (int i = tid; i < n_f; i += kThreads) F.ids[i] = cand_g[i];
        fine_ids = true;
        if (tid == 0) {
            p.n_cand[u] = n_f;
            p.counters[4 * u + 2] = n_c;
        }
        __syncthreads();
    } else if (tid == 0) {
        p.counters[4 * u + 2] = 0;
    }

    score_level<G>(p, F, S, u, n_f, fine_ids, false, qreg, p.key_budget, two, p.r_f + (long long)u * p.f_stride,
                   p.flag_f + (long long)u * p.f_stride);
    if (p.use_mp) n_terms += emit_terms<G>(p, F, S, u, n_f, fine_ids, 0, n_terms);

    // flat list of stored rows of the selected clusters, ascending fine id
    if (tid == 0) S.carry = 0;
    __syncthreads();
    uint32_t* offs = reinterpret_cast<uint32_t*>(F.keys);   // keys are no longer needed
    for (int i0 = 0; i0 < n_f; i0 += kThreads) {
        const int i = i0 + tid;
        const uint32_t w = (i < n_f && F.flags[i]) ? F.wts[i] : 0u;
        const uint32_t pos = chunk_excl_scan(w, S);
        if (i < n_f) offs[i] = pos;
    }
    const uint32_t total = S.carry;
    __syncthreads();
    int32_t* ro = p.rows + (long long)u * p.rows_stride;
    const int wave = tid >> 6, lane = tid & 63;
    for (int i = wave; i < n_f; i += kWaves) {
        if (!F.flags[i]) continue;
        const int r0 = F.aux[i];
        const int cnt = (int)F.wts[i];
        const uint32_t o = offs[i];
        for (int j = lane; j < cnt; j += 64) ro[o + j] = r0 + j;
    }
    if (tid == 0) {
        p.n_rows[u] = (int32_t)total;
        p.n_mp[u] = (int32_t)n_terms;
        p.counters[4 * u + 0] = (int32_t)total + p.n_tail;
        p.counters[4 * u + 1] = n_f;
        p.counters[4 * u + 3] = (int32_t)n_terms;
    }
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
