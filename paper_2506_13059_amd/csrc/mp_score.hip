// Centroid scoring and budgeted cluster selection for gfx950 (Eq. 1, Sec. 3.1; two levels: Sec. 3.4).
//
// One workgroup of 1024 threads per unit and level.  Logits l[h,i] = scale * q_h . Kc_i are
// accumulated in fp64 (products of bf16 numbers are exact, so the sum carries ~1e-16 relative
// error and the ranking agrees with an fp64 reference except on ties far below any tolerance).
// The rank key is log(mean_h exp(l[h,i] - LSE_h)), i.e. the logarithm of Eq. 1 averaged over the
// query heads of the group.  Selection = "take clusters in descending key order (ties: lower id)
// while the running token count stays within the budget, stop at the first that does not fit";
// because token counts are positive this equals a threshold on (key, id), found by a weighted
// most-significant-digit radix select instead of a sort.
//
// The coarse launch leaves: the promising mask, the candidate list (children of promising
// clusters), the log-sum of the unpromising clusters' N*exp(l) per head, and one "centroid term"
// entry per unpromising cluster.  The fine launch leaves: the selected mask, the flat list of
// stored row numbers of the selected clusters' keys, and centroid-term entries for the unselected
// candidates.  The value pass consumes the row list and the centroid-term list.
#include "mp_device.h"
#include "mp_internal.h"

namespace mp {

namespace {

constexpr int kThreads = 1024;
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
    uint32_t hist_w[256];
    uint32_t hist_c[256];
    uint32_t wsum[kWaves];
    uint32_t carry;
    uint32_t sel_digit, sel_found, sel_cnt;
    unsigned long long sel_acc;
    unsigned long long sel_key;
};

// max over the workgroup of v[h] for h < G; result in out[h] for every thread
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

// sum over the workgroup, fixed order (deterministic)
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

// Exclusive prefix sum over one chunk of 1024 values (one per thread) with a running carry kept
// in s.carry; returns the exclusive prefix including the carry.  All threads must call.
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
// (entries with wts == 0 must carry key ~0 and are never selected).  Finds the key K* of the
// first entry (in (key, index) order) at which the running weight exceeds `budget`, and the
// weight `acc` of all entries with key < K*.  Returns false if everything fits.
__device__ __forceinline__ bool radix_select(const uint64_t* keys, const uint32_t* wts, int n, long long budget,
                                             Scratch& s, uint64_t& kstar, uint64_t& acc_out, uint32_t& ties_out)
{
    const int tid = threadIdx.x;
    uint64_t prefix = 0;      // digits fixed so far (high bits)
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
    ties_out = s.sel_cnt;   // entries whose key equals K* exactly
    return true;
}

template <int G, bool kCoarse>
__global__ __launch_bounds__(kThreads) void score_select_kernel(const ScoreParams p)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    Scratch& S = *reinterpret_cast<Scratch*>(smem_raw);
    double* qs = reinterpret_cast<double*>(smem_raw + ((sizeof(Scratch) + 15) & ~size_t(15)));   // [G][128]
    uint64_t* keys = reinterpret_cast<uint64_t*>(qs + G * kHeadDim);                               // [cap]
    uint32_t* wts = reinterpret_cast<uint32_t*>(keys + p.smem_cap);                                // [cap]
    uint8_t* flags = reinterpret_cast<uint8_t*>(wts + p.smem_cap);                                 // [cap]

    const int u = blockIdx.x, tid = threadIdx.x;
    int n = p.n_cand_fixed;
    if (p.n_cand_dev) n = p.n_cand_dev[u];
    if (n > p.smem_cap) n = p.smem_cap;   // cannot happen: the host sizes smem_cap from the table capacity
    const int32_t* cand = p.cand ? p.cand + (long long)u * p.cand_stride : nullptr;
    const int32_t* Nu = p.N + (long long)u * p.tab_rows;
    const uint16_t* Kcu = p.Kc + (long long)u * p.tab_rows * kHeadDim;
    double* lg = p.lg + (long long)u * G * p.lg_stride;
    const double kLog2e = 1.4426950408889634;

    if (tid == 0) S.carry = 0;
    for (int i = tid; i < G * kHeadDim; i += kThreads)
        qs[i] = (double)bf16_to_f32(p.q[(long long)u * G * kHeadDim + i]);
    __syncthreads();

    // ---- logits: 4 lanes per candidate, 32 dims each ----
    {
        const int part = tid & 3;
        for (int i0 = 0; i0 < n; i0 += kThreads / 4) {
            const int i = i0 + (tid >> 2);
            const bool live = i < n;
            const int id = live ? (cand ? cand[i] : i) : 0;
            const int row = p.row_off + id;
            const int nw = live ? Nu[row] : 0;
            double acc[G];
#pragma unroll
            for (int h = 0; h < G; ++h) acc[h] = 0.0;
            if (live && nw > 0) {
                const uint4* kp = reinterpret_cast<const uint4*>(Kcu + (long long)row * kHeadDim + 32 * part);
                uint4 kv[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) kv[j] = kp[j];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t w[4] = {kv[j].x, kv[j].y, kv[j].z, kv[j].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const double k0 = (double)bf16lo_to_f32(w[e]);
                        const double k1 = (double)bf16hi_to_f32(w[e]);
                        const int d = 32 * part + 8 * j + 2 * e;
#pragma unroll
                        for (int h = 0; h < G; ++h) {
                            const double2 qq = *reinterpret_cast<const double2*>(&qs[h * kHeadDim + d]);
                            acc[h] = fma(qq.x, k0, acc[h]);
                            acc[h] = fma(qq.y, k1, acc[h]);
                        }
                    }
                }
            }
#pragma unroll
            for (int h = 0; h < G; ++h) acc[h] = sum4_f64(acc[h]);
            if (live && part == 0) {
#pragma unroll
                for (int h = 0; h < G; ++h) lg[h * p.lg_stride + i] = (nw > 0) ? acc[h] * p.scale : -INFINITY;
                wts[i] = (uint32_t)(nw > 0 ? nw : 0);
            }
        }
    }
    __syncthreads();

    // ---- per-head normaliser of Eq. 1: LSE_h = log( sum_i N_i e^{l[h,i]} + e^{extra_h} ) ----
    double lse[G];
    {
        double mx[G];
#pragma unroll
        for (int h = 0; h < G; ++h) mx[h] = p.extra_lse ? p.extra_lse[(long long)u * G + h] : -INFINITY;
        for (int i = tid; i < n; i += kThreads)
            if (wts[i])
#pragma unroll
                for (int h = 0; h < G; ++h) mx[h] = fmax(mx[h], lg[h * p.lg_stride + i]);
        block_max<G>(mx, S);
        double sm[G];
#pragma unroll
        for (int h = 0; h < G; ++h) sm[h] = 0.0;
        for (int i = tid; i < n; i += kThreads)
            if (wts[i])
#pragma unroll
                for (int h = 0; h < G; ++h) sm[h] += (double)wts[i] * exp(lg[h * p.lg_stride + i] - mx[h]);
        if (tid == 0 && p.extra_lse)
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const double e = p.extra_lse[(long long)u * G + h];
                if (e != -INFINITY) sm[h] += exp(e - mx[h]);
            }
        block_sum<G>(sm, S);
#pragma unroll
        for (int h = 0; h < G; ++h) lse[h] = (mx[h] == -INFINITY) ? -INFINITY : mx[h] + log(sm[h]);
    }

    // ---- rank keys ----
    const double logG = log((double)G);
    for (int i = tid; i < n; i += kThreads) {
        double r = __longlong_as_double(0x7ff8000000000000ll);
        uint64_t key = ~0ull;
        if (wts[i]) {
            double t[G], tm = -INFINITY;
#pragma unroll
            for (int h = 0; h < G; ++h) {
                t[h] = lg[h * p.lg_stride + i] - lse[h];
                tm = fmax(tm, t[h]);
            }
            double ssum = 0.0;
#pragma unroll
            for (int h = 0; h < G; ++h) ssum += exp(t[h] - tm);
            r = tm + log(ssum) - logG;
            key = descending_key(r);
        }
        keys[i] = key;
        p.r_out[(long long)u * p.r_stride + i] = r;
    }
    __syncthreads();

    // ---- budgeted selection ----
    uint64_t kstar = 0, acc = 0;
    uint32_t ties = 0;
    const bool bounded = radix_select(keys, wts, n, p.budget, S, kstar, acc, ties);
    for (int i = tid; i < n; i += kThreads) {
        uint8_t f = 0;
        if (wts[i]) {
            if (!bounded) f = 1;
            else {
                const uint64_t k = keys[i];
                if (k < kstar) f = 1;
                else if (k == kstar && ties > 1) {
                    // equal keys: lower position first; keep while the running count still fits
                    uint64_t run = acc;
                    for (int j = 0; j <= i; ++j)
                        if (wts[j] && keys[j] == kstar) run += wts[j];
                    f = ((long long)run <= p.budget) ? 1 : 0;
                }
            }
        }
        flags[i] = f;
        p.flag_out[(long long)u * p.r_stride + i] = f;
    }
    __syncthreads();

    // ---- centroid-term entries for everything that stays behind at this level ----
    int mp_base = 0;
    if (p.mp_append) mp_base = p.n_mp[u];
    if (tid == 0) S.carry = 0;
    __syncthreads();
    uint32_t n_mp_here = 0;
    if (p.use_mp) {
        for (int i0 = 0; i0 < n; i0 += kThreads) {
            const int i = i0 + tid;
            const bool emit = (i < n) && wts[i] && !flags[i];
            const uint32_t pos = chunk_excl_scan(emit ? 1u : 0u, S);
            if (emit) {
                const int id = cand ? cand[i] : i;
                const long long o = (long long)u * p.mp_stride + mp_base + pos;
                p.mp_rows[o] = p.row_off + id;
                const double lnN = log((double)wts[i]);
#pragma unroll
                for (int h = 0; h < G; ++h)
                    p.mp_scores[o * G + h] = (float)((lg[h * p.lg_stride + i] + lnN) * kLog2e);
            }
        }
        n_mp_here = S.carry;
    }
    __syncthreads();

    if constexpr (kCoarse) {
        // log-sum of the unpromising clusters' N e^{l}: joins the fine level's Eq. 1 denominator
        double mx[G], sm[G];
#pragma unroll
        for (int h = 0; h < G; ++h) { mx[h] = -INFINITY; sm[h] = 0.0; }
        for (int i = tid; i < n; i += kThreads)
            if (wts[i] && !flags[i])
#pragma unroll
                for (int h = 0; h < G; ++h) mx[h] = fmax(mx[h], lg[h * p.lg_stride + i]);
        block_max<G>(mx, S);
        for (int i = tid; i < n; i += kThreads)
            if (wts[i] && !flags[i])
#pragma unroll
                for (int h = 0; h < G; ++h) sm[h] += (double)wts[i] * exp(lg[h * p.lg_stride + i] - mx[h]);
        block_sum<G>(sm, S);
        if (tid < G) {
            double v = -INFINITY;
#pragma unroll
            for (int h = 0; h < G; ++h)
                if (h == tid) v = (mx[h] == -INFINITY) ? -INFINITY : mx[h] + log(sm[h]);
            p.unprom_lse_out[(long long)u * G + tid] = v;
        }
        // candidate list: children of the promising clusters, ascending fine id
        if (tid == 0) S.carry = 0;
        __syncthreads();
        const int32_t* cs = p.cstart + (long long)u * p.cstart_stride;
        int32_t* co = p.cand_out + (long long)u * p.cand_out_stride;
        for (int i0 = 0; i0 < n; i0 += kThreads) {
            const int i = i0 + tid;
            int c0 = 0, c1 = 0;
            if (i < n && flags[i]) { c0 = cs[i]; c1 = cs[i + 1]; }
            const uint32_t pos = chunk_excl_scan((uint32_t)(c1 - c0), S);
            for (int f = c0; f < c1; ++f) co[pos + (f - c0)] = f;
        }
        if (tid == 0) {
            p.n_cand_out[u] = (int32_t)S.carry;
            p.n_mp[u] = (int32_t)n_mp_here;
            p.counters[4 * u + 2] = n;
        }
    } else {
        // flat list of stored rows of the selected clusters, ascending fine id
        if (tid == 0) S.carry = 0;
        __syncthreads();
        uint32_t* offs = reinterpret_cast<uint32_t*>(keys);   // keys are no longer needed
        for (int i0 = 0; i0 < n; i0 += kThreads) {
            const int i = i0 + tid;
            const uint32_t w = (i < n && flags[i]) ? wts[i] : 0u;
            const uint32_t pos = chunk_excl_scan(w, S);
            if (i < n) offs[i] = pos;
        }
        const uint32_t total = S.carry;
        __syncthreads();
        const int32_t* fs = p.fstart + (long long)u * p.fstart_stride;
        int32_t* ro = p.rows_out + (long long)u * p.rows_stride;
        const int wave = tid >> 6, lane = tid & 63;
        for (int i = wave; i < n; i += kWaves) {
            if (!flags[i]) continue;
            const int id = cand ? cand[i] : i;
            const int r0 = fs[id];
            const int cnt = (int)wts[i];
            const uint32_t o = offs[i];
            for (int j = lane; j < cnt; j += 64) ro[o + j] = r0 + j;
        }
        if (tid == 0) {
            p.n_rows_out[u] = (int32_t)total;
            p.n_mp[u] = (int32_t)(mp_base + n_mp_here);
            p.counters[4 * u + 0] = (int32_t)total + p.n_tail;
            p.counters[4 * u + 1] = n;
            if (!p.mp_append) p.counters[4 * u + 2] = 0;
            p.counters[4 * u + 3] = (int32_t)(mp_base + n_mp_here);
        }
    }
}

}  // namespace

size_t score_smem_bytes(int G, int cap)
{
    return ((sizeof(Scratch) + 15) & ~size_t(15)) + sizeof(double) * G * kHeadDim + (size_t)cap * (8 + 4 + 1) + 16;
}

template <int G, bool kCoarse>
static hipError_t launch_score_gc(const ScoreParams& p, hipStream_t s)
{
    static size_t configured = 48 * 1024;
    const size_t smem = score_smem_bytes(G, p.smem_cap);
    if (smem > configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_select_kernel<G, kCoarse>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = smem;
    }
    hipLaunchKernelGGL((score_select_kernel<G, kCoarse>), dim3(p.U), dim3(kThreads), smem, s, p);
    return hipGetLastError();
}

template <int G>
static hipError_t launch_score_g(const ScoreParams& p, hipStream_t s)
{
    return p.coarse ? launch_score_gc<G, true>(p, s) : launch_score_gc<G, false>(p, s);
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
