// Value pass and merge for gfx950.
//
// The value pass is the byte mover of the decode step: it streams 256-byte key rows and value rows
// (the keys of the selected clusters, the unclustered tail, or all keys for the dense comparison)
// and, in the same launch, the value-centroid rows of the clusters that enter the softmax through
// their centroid term N*exp(q.Kc) (Eq. 2).  Every workgroup writes one online-softmax partial
// (m, l, acc[128]) per query head of the group; the merge kernel combines them (Sec. 4: split over
// the KV dimension followed by a reduction of the intermediate results).
//
// Lane layout inside a wave: lane = 8*r + c.  A group of 8 lanes (fixed r) owns one row at a
// time; lane c holds dims [8c, 8c+8) and [64+8c, 64+8c+8) of that row, so that each 16-byte load
// instruction of the wave covers eight full 128-byte lines.  A query-key product is 8 packed bf16
// dot instructions per head followed by a 3-step DPP sum over the 8 lanes; the value update keeps
// 16 fp32 accumulators per head and lane.  All G heads of the group share every loaded row.
//
// 8-bit rows (a source with row_scale): a row is 128 one-byte e4m3 codes and lane c holds the 16
// contiguous dims [16c, 16c+16) of it, one 16-byte load for the key and one for the value.  Key
// codes are widened to bf16 pairs (exact: a code has four significant bits) and go through the same
// packed dot instructions; value codes are widened to fp32.  The row's two fp32 scales multiply the
// logit and the probability that weighs the value row, so the arithmetic equals that on code * scale.
#include "mp_device.h"
#include "mp_internal.h"

namespace mp {

namespace {

struct RowRegs {
    uint4 klo, khi, vlo, vhi;
};

// 16-byte global load issued through inline assembly: the compiler neither moves it towards its
// use nor waits for it, so the software pipeline below stays as written.  Every use of the result
// must be preceded by wait_rows<N>(), N = number of such loads issued after the ones needed
// (vector memory loads return in order).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// Cache policy of the row loads: non-temporal where a row is used once per step (kOnce).  Loads marked
// so move 7 % more bytes per second in the dense kernel (5.9 -> 6.3 TB/s) and 12 % more over the
// scattered runs of selected keys than plain loads; the scope bits (sc0, sc1) change nothing.  Where two
// waves ask for the same row (groups of more than five heads, split over pairs of waves) the row has to
// stay for the second request: plain loads there (4.8 against 3.7 TB/s at eight heads).
#ifndef MP_LOAD_BITS
#define MP_LOAD_BITS " nt"
#endif
template <bool kOnce = true>
__device__ __forceinline__ void issue_load16(u32x4& d, const void* p)
{
    if constexpr (kOnce) asm volatile("global_load_dwordx4 %0, %1, off" MP_LOAD_BITS : "=&v"(d) : "v"(p) : "memory");
    else asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(d) : "v"(p) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_rows(u32x4 (&b)[8])
{
    asm volatile("s_waitcnt vmcnt(%8)"
                 : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7])
                 : "n"(N));
}
__device__ __forceinline__ RowRegs as_row(const u32x4& klo, const u32x4& khi, const u32x4& vlo, const u32x4& vhi)
{
    RowRegs t;
    t.klo = make_uint4(klo.x, klo.y, klo.z, klo.w);
    t.khi = make_uint4(khi.x, khi.y, khi.z, khi.w);
    t.vlo = make_uint4(vlo.x, vlo.y, vlo.z, vlo.w);
    t.vhi = make_uint4(vhi.x, vhi.y, vhi.z, vhi.w);
    return t;
}

// kWide: the lane holds the 16 contiguous dims [16c, 16c+16) of the row (the layout of a workgroup
// that streams 8-bit rows) instead of [8c, 8c+8) and [64+8c, 64+8c+8).
template <bool kWide>
__device__ __forceinline__ void load_vrow(RowRegs& t, const uint16_t* __restrict__ V, long long row, int c)
{
    if constexpr (kWide) {
        const uint4* vp = reinterpret_cast<const uint4*>(V + row * kHeadDim) + 2 * c;
        t.vlo = vp[0];
        t.vhi = vp[1];
    } else {
        const uint4* vp = reinterpret_cast<const uint4*>(V + row * kHeadDim) + c;
        t.vlo = vp[0];
        t.vhi = vp[8];
    }
}

template <int G>
struct HeadState {
    float m[G];
    float l[G];
    float acc[G][16];
};

template <int G>
__device__ __forceinline__ void qk_scores(const RowRegs& t, const uint4 (&qlo)[G], const uint4 (&qhi)[G], float scale,
                                          bool valid, float (&s)[G])
{
#pragma unroll
    for (int h = 0; h < G; ++h) {
        float a = 0.f;
        a = dot2_bf16(t.klo.x, qlo[h].x, a);
        a = dot2_bf16(t.klo.y, qlo[h].y, a);
        a = dot2_bf16(t.klo.z, qlo[h].z, a);
        a = dot2_bf16(t.klo.w, qlo[h].w, a);
        a = dot2_bf16(t.khi.x, qhi[h].x, a);
        a = dot2_bf16(t.khi.y, qhi[h].y, a);
        a = dot2_bf16(t.khi.z, qhi[h].z, a);
        a = dot2_bf16(t.khi.w, qhi[h].w, a);
        a = sum8(a);
        s[h] = valid ? a * scale : -INFINITY;
    }
}

template <int G>
__device__ __forceinline__ void accumulate_v(HeadState<G>& st, const RowRegs& t, const float (&p)[G])
{
    const uint32_t w[8] = {t.vlo.x, t.vlo.y, t.vlo.z, t.vlo.w, t.vhi.x, t.vhi.y, t.vhi.z, t.vhi.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float va = bf16lo_to_f32(w[i]);
        const float vb = bf16hi_to_f32(w[i]);
#pragma unroll
        for (int h = 0; h < G; ++h) {
            st.acc[h][2 * i] = fmaf(p[h], va, st.acc[h][2 * i]);
            st.acc[h][2 * i + 1] = fmaf(p[h], vb, st.acc[h][2 * i + 1]);
        }
    }
}

// Online-softmax bookkeeping for the scores of two rows: running maximum and denominator of `st` are
// brought up to date (accumulators rescaled when the maximum moves) and the rows' probabilities
// relative to that maximum are returned.
template <int G>
__device__ __forceinline__ void softmax_probs(HeadState<G>& st, const float (&s0)[G], const float (&s1)[G], float (&p0)[G],
                                              float (&p1)[G])
{
    float mn[G];
    bool grow = false;
#pragma unroll
    for (int h = 0; h < G; ++h) {
        mn[h] = fmaxf(st.m[h], fmaxf(s0[h], s1[h]));
        grow |= (mn[h] > st.m[h]);
    }
    if (__any(grow)) {   // rescale lazily: the running maximum settles after a few rows
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float ms = (mn[h] == -INFINITY) ? 0.f : mn[h];
            const float a = __builtin_amdgcn_exp2f(st.m[h] - ms);
            st.l[h] *= a;
#pragma unroll
            for (int e = 0; e < 16; ++e) st.acc[h][e] *= a;
            st.m[h] = mn[h];
        }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float ms = (st.m[h] == -INFINITY) ? 0.f : st.m[h];
        p0[h] = __builtin_amdgcn_exp2f(s0[h] - ms);
        p1[h] = __builtin_amdgcn_exp2f(s1[h] - ms);
        st.l[h] += p0[h] + p1[h];
    }
}

// Online-softmax update with the scores of two rows (s0, s1) and their value rows.
template <int G>
__device__ __forceinline__ void softmax_step(HeadState<G>& st, const float (&s0)[G], const float (&s1)[G],
                                             const RowRegs& t0, const RowRegs& t1)
{
    float p0[G], p1[G];
    softmax_probs<G>(st, s0, s1, p0, p1);
    accumulate_v<G>(st, t0, p0);
    accumulate_v<G>(st, t1, p1);
}

// ---- 8-bit rows -------------------------------------------------------------------------------
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void issue_load8(u32x2& d, const void* p)
{
    asm volatile("global_load_dwordx2 %0, %1, off" : "=&v"(d) : "v"(p) : "memory");   // (plain: neighbouring rows' scales share a line)
}
// (plain: for data that many rows share, such as a cluster's logit shares)
__device__ __forceinline__ void issue_load16_shared(u32x4& d, const void* p)
{
    asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(d) : "v"(p) : "memory");
}
// kBase: 16-byte loads of ready-made logit shares per row (1 for up to four heads, 2 for five).
template <int N, int kBase>
__device__ __forceinline__ void wait_rows8(u32x4 (&b)[4], u32x2 (&sc)[2], u32x4 (&bs)[2 * kBase])
{
    if constexpr (kBase == 1)
        asm volatile("s_waitcnt vmcnt(%8)"
                     : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(sc[0]), "+v"(sc[1]), "+v"(bs[0]), "+v"(bs[1])
                     : "n"(N));
    else
        asm volatile("s_waitcnt vmcnt(%10)"
                     : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(sc[0]), "+v"(sc[1]), "+v"(bs[0]), "+v"(bs[1]),
                       "+v"(bs[2]), "+v"(bs[3])
                     : "n"(N));
}

// Two e4m3 codes (the low or the high half of w) as one dword of two bf16 values.
template <bool kHigh>
__device__ __forceinline__ uint32_t e4m3_pair_to_bf16(uint32_t w)
{
    const auto f = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, kHigh);
    return __builtin_amdgcn_perm(__float_as_uint(f[1]), __float_as_uint(f[0]), 0x07060302u);   // upper halves of both
}

// Logits of one 8-bit key row (16 codes per lane) against the G queries; qa / qb hold this lane's
// dims [16c, 16c+8) and [16c+8, 16c+16) of every query.  `scale` already includes the row's key scale;
// base[h] is the share of the row's cluster centroid (the codes are the key's residual from it).
template <int G>
__device__ __forceinline__ void qk_scores8(const u32x4& kc, const uint4 (&qa)[G], const uint4 (&qb)[G], float scale,
                                           const float (&base)[G], bool valid, float (&s)[G])
{
    const uint32_t k0 = e4m3_pair_to_bf16<false>(kc.x), k1 = e4m3_pair_to_bf16<true>(kc.x);
    const uint32_t k2 = e4m3_pair_to_bf16<false>(kc.y), k3 = e4m3_pair_to_bf16<true>(kc.y);
    const uint32_t k4 = e4m3_pair_to_bf16<false>(kc.z), k5 = e4m3_pair_to_bf16<true>(kc.z);
    const uint32_t k6 = e4m3_pair_to_bf16<false>(kc.w), k7 = e4m3_pair_to_bf16<true>(kc.w);
#pragma unroll
    for (int h = 0; h < G; ++h) {
        float a = 0.f;
        a = dot2_bf16(k0, qa[h].x, a);
        a = dot2_bf16(k1, qa[h].y, a);
        a = dot2_bf16(k2, qa[h].z, a);
        a = dot2_bf16(k3, qa[h].w, a);
        a = dot2_bf16(k4, qb[h].x, a);
        a = dot2_bf16(k5, qb[h].y, a);
        a = dot2_bf16(k6, qb[h].z, a);
        a = dot2_bf16(k7, qb[h].w, a);
        a = sum8(a);
        s[h] = valid ? fmaf(a, scale, base[h]) : -INFINITY;
    }
}

// acc += (p * vscale) * value codes; accumulator e of a lane is dim 16c + e.
template <int G>
__device__ __forceinline__ void accumulate_v8(HeadState<G>& st, const u32x4& vc, const float (&p)[G], float vscale)
{
    float pv[G];
#pragma unroll
    for (int h = 0; h < G; ++h) pv[h] = p[h] * vscale;
    const uint32_t w[4] = {vc.x, vc.y, vc.z, vc.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);
        const auto hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
#pragma unroll
        for (int h = 0; h < G; ++h) {
            st.acc[h][4 * i] = fmaf(pv[h], lo[0], st.acc[h][4 * i]);
            st.acc[h][4 * i + 1] = fmaf(pv[h], lo[1], st.acc[h][4 * i + 1]);
            st.acc[h][4 * i + 2] = fmaf(pv[h], hi[0], st.acc[h][4 * i + 2]);
            st.acc[h][4 * i + 3] = fmaf(pv[h], hi[1], st.acc[h][4 * i + 3]);
        }
    }
}

// The 8-bit counterpart of stream_rows<G, false, kIters> below: same strips, same masking, a software
// pipeline of kStages stages (the loads of the next iteration are in flight while one is consumed).  Loads per iteration (two rows): key codes, value codes, the two scales
// and the cluster's ready-made logit shares of each row, 6 + 2 * kBase in all.
template <int G, int kIters, bool kOnce>
__device__ __forceinline__ void stream_rows8(HeadState<G>& st, const RowSource& S, const ValuePassParams& p, int u,
                                             int w0, int w1, int end, int r, int c, int lane, int gt, int h0)
{
    auto head = [&](int h) { return h0 + h < gt ? h0 + h : gt - 1; };
    const uint8_t* __restrict__ Kb = reinterpret_cast<const uint8_t*>(S.K) + (long long)u * S.unit_rows * kHeadDim;
    const uint8_t* __restrict__ Vb = reinterpret_cast<const uint8_t*>(S.V) + (long long)u * S.unit_rows * kHeadDim;
    const float* __restrict__ Sb = S.row_scale + (long long)u * S.unit_rows * 2;
    const int32_t* __restrict__ rows = S.rows + (long long)u * S.rows_stride;
    const int32_t* __restrict__ slots = S.row_slot + (long long)u * S.rows_stride;
    // this wave's columns of the logit-share table: the second half of a split group starts at column 4
    const float* __restrict__ Bb = S.slot_base + (long long)u * S.base_stride * 8 + (h0 > 0 ? 4 : 0);
    constexpr int kStrip = 16 * kIters;
    constexpr int kBase = (G + 3) / 4;
    constexpr int kLoads = 6 + 2 * kBase;
    uint4 qa[G], qb[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const uint4* qp = reinterpret_cast<const uint4*>(p.q + ((long long)u * gt + head(h)) * kHeadDim) + 2 * c;
        qa[h] = qp[0];
        qb[h] = qp[1];
    }
    const float scale = p.scale_log2e;
    auto strip_rows = [&](int j0, int& ia, int& ib, int& sa, int& sb) {
        int pa = j0 + lane, pb = j0 + 64 + lane;
        pa = pa < end ? pa : end - 1;
        pb = pb < end ? pb : end - 1;
        ia = rows[pa];
        ib = rows[pb];
        sa = slots[pa];
        sb = slots[pb];
    };
    int na, nb, nsa, nsb;
    strip_rows(w0, na, nb, nsa, nsb);
    constexpr int kStages = 2;     // (measured at four heads: one iteration ahead 72 us, two ahead 76 us per launch)
    for (int j0 = w0; j0 < w1; j0 += kStrip) {
        const int ia = na, ib = nb, sa = nsa, sb = nsb;
        if (j0 + kStrip < w1) strip_rows(j0 + kStrip, na, nb, nsa, nsb);
        u32x4 buf[kStages][4];
        u32x2 scl[kStages][2];
        u32x4 bas[kStages][2 * kBase];
        auto issue = [&](int it, u32x4 (&b)[4], u32x2 (&sc)[2], u32x4 (&bs)[2 * kBase]) {
            const int slot = it * 16 + r;
            const bool first = slot < 64;                 // resolved at compile time after unrolling
            const long long i0 = __shfl(first ? ia : ib, slot & 63, 64);
            const long long i1 = __shfl(first ? ia : ib, (slot + 8) & 63, 64);
            const long long s0 = __shfl(first ? sa : sb, slot & 63, 64);
            const long long s1 = __shfl(first ? sa : sb, (slot + 8) & 63, 64);
            issue_load16<kOnce>(b[0], reinterpret_cast<const uint4*>(Kb + i0 * kHeadDim) + c);
            issue_load16<kOnce>(b[1], reinterpret_cast<const uint4*>(Vb + i0 * kHeadDim) + c);
            issue_load8(sc[0], Sb + i0 * 2);
#pragma unroll
            for (int k = 0; k < kBase; ++k) issue_load16_shared(bs[k], Bb + s0 * 8 + 4 * k);
            issue_load16<kOnce>(b[2], reinterpret_cast<const uint4*>(Kb + i1 * kHeadDim) + c);
            issue_load16<kOnce>(b[3], reinterpret_cast<const uint4*>(Vb + i1 * kHeadDim) + c);
            issue_load8(sc[1], Sb + i1 * 2);
#pragma unroll
            for (int k = 0; k < kBase; ++k) issue_load16_shared(bs[kBase + k], Bb + s1 * 8 + 4 * k);
        };
#pragma unroll
        for (int it = 0; it < kStages - 1; ++it)
            if (it < kIters) issue(it, buf[it], scl[it], bas[it]);
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const int jj = j0 + it * 16;
            constexpr int kA = kStages - 1;
            if (it + kA < kIters) issue(it + kA, buf[(it + kA) % kStages], scl[(it + kA) % kStages], bas[(it + kA) % kStages]);
            u32x4(&b)[4] = buf[it % kStages];
            u32x2(&sc)[2] = scl[it % kStages];
            u32x4(&bs)[2 * kBase] = bas[it % kStages];
            // loads issued after this iteration's: kLoads for each later iteration already under way
            if (kStages > 3 && it + 3 < kIters) wait_rows8<3 * kLoads, kBase>(b, sc, bs);
            else if (kStages > 2 && it + 2 < kIters) wait_rows8<2 * kLoads, kBase>(b, sc, bs);
            else if (it + 1 < kIters) wait_rows8<kLoads, kBase>(b, sc, bs);
            else wait_rows8<0, kBase>(b, sc, bs);
            if (jj < w1) {
                float s0[G], s1[G], p0[G], p1[G], b0[G], b1[G];
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    b0[h] = __uint_as_float(bs[h >> 2][h & 3]);
                    b1[h] = __uint_as_float(bs[kBase + (h >> 2)][h & 3]);
                }
                qk_scores8<G>(b[0], qa, qb, scale * __uint_as_float(sc[0].x), b0, jj + r < w1, s0);
                qk_scores8<G>(b[2], qa, qb, scale * __uint_as_float(sc[1].x), b1, jj + 8 + r < w1, s1);
                softmax_probs<G>(st, s0, s1, p0, p1);
                accumulate_v8<G>(st, b[1], p0, __uint_as_float(sc[0].y));
                accumulate_v8<G>(st, b[3], p1, __uint_as_float(sc[1].y));
            }
        }
    }
}

// Stream the rows [w0, w1) of a source through one wave, 16 rows per iteration (two per group of 8
// lanes), in strips of 128 rows whose row numbers are fetched with two coalesced loads.
//
// kScored = false (exact rows, the hot path): a software pipeline of three stages (two for a wave
// that holds five heads; a wave never holds more, larger groups are split over two waves).  The loads of
// iterations it+1 and it+2 are in flight while iteration it is consumed; they are issued through
// inline assembly and waited for by count, because the compiler would otherwise sink each load
// next to its use.  All eight iterations of a strip issue their loads (rows past the end are
// clamped to the last valid row and masked), so the counts are static.
// kScored = true (centroid terms): logits are read ready-made (log2 units, ln N included) and
// only the value-centroid row is loaded; this stream is short and uses plain loads.
// The G heads of `st` are the heads h0, h0 + 1, ... of the unit's gt heads (clamped to the last one:
// a wave that owns fewer than G heads computes the last one again and its caller drops the copy).
template <int G, bool kScored, int kIters, bool kWide = false, bool kOnce = true>
__device__ __forceinline__ void stream_rows(HeadState<G>& st, const RowSource& S, const ValuePassParams& p, int u,
                                            int w0, int w1, int end, int r, int c, int lane, int gt, int h0)
{
    auto head = [&](int h) { return h0 + h < gt ? h0 + h : gt - 1; };
    const uint16_t* __restrict__ Vb = S.V + (long long)u * S.unit_rows * kHeadDim;
    const int32_t* __restrict__ rows = S.rows ? S.rows + (long long)u * S.rows_stride : nullptr;
    constexpr int kStrip = 16 * kIters;   // rows a wave handles between two refills of its index registers
    if constexpr (kScored) {
        const float* __restrict__ sc = S.scores + (long long)u * S.rows_stride * gt;
        for (int j0 = w0; j0 < w1; j0 += 16) {
            const int ja = j0 + r, jb = j0 + 8 + r;
            const bool va = ja < w1, vb = jb < w1;
            const int pa = va ? ja : w1 - 1, pb = vb ? jb : w1 - 1;
            const int ia = rows ? rows[pa] : pa, ib = rows ? rows[pb] : pb;
            RowRegs t0, t1;
            load_vrow<kWide>(t0, Vb, ia, c);
            load_vrow<kWide>(t1, Vb, ib, c);
            float s0[G], s1[G];
#pragma unroll
            for (int h = 0; h < G; ++h) {
                s0[h] = va ? sc[(long long)pa * gt + head(h)] : -INFINITY;
                s1[h] = vb ? sc[(long long)pb * gt + head(h)] : -INFINITY;
            }
            softmax_step<G>(st, s0, s1, t0, t1);
        }
    } else {
        const uint16_t* __restrict__ Kb = S.K + (long long)u * S.unit_rows * kHeadDim;
        uint4 qlo[G], qhi[G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const uint4* qp = reinterpret_cast<const uint4*>(p.q + ((long long)u * gt + head(h)) * kHeadDim) + c;
            qlo[h] = qp[0];
            qhi[h] = qp[8];
        }
        const float scale = p.scale_log2e;
        // row numbers of a strip: requested one strip ahead, so that a strip starts with one memory
        // latency (its first rows) instead of two (row numbers, then rows)
        auto strip_rows = [&](int j0, int& ia, int& ib) {
            int pa = j0 + lane, pb = j0 + 64 + lane;
            pa = pa < end ? pa : end - 1;
            pb = pb < end ? pb : end - 1;
            ia = rows ? rows[pa] : pa;
            ib = rows ? rows[pb] : pb;
        };
        int na, nb;
        strip_rows(w0, na, nb);
        for (int j0 = w0; j0 < w1; j0 += kStrip) {
            const int ia = na, ib = nb;
            if (j0 + kStrip < w1) strip_rows(j0 + kStrip, na, nb);
            static_assert(G <= 5, "a wave holds at most five heads (larger groups are split over two waves)");
            {
                // loads of kStages - 1 later iterations are in flight while one is consumed: three
                // stages where the registers allow it, two for the group of five
                constexpr int kStages = G <= 4 ? 3 : 2;
                u32x4 buf[kStages][8];
                auto issue = [&](int it, u32x4 (&b)[8]) {
                    const int slot = it * 16 + r;
                    const int src_reg = (slot < 64) ? ia : ib;   // resolved at compile time after unrolling
                    const long long i0 = __shfl(src_reg, slot & 63, 64);
                    const long long i1 = __shfl(src_reg, (slot + 8) & 63, 64);
                    const uint4* k0 = reinterpret_cast<const uint4*>(Kb + i0 * kHeadDim) + c;
                    const uint4* v0 = reinterpret_cast<const uint4*>(Vb + i0 * kHeadDim) + c;
                    const uint4* k1 = reinterpret_cast<const uint4*>(Kb + i1 * kHeadDim) + c;
                    const uint4* v1 = reinterpret_cast<const uint4*>(Vb + i1 * kHeadDim) + c;
                    issue_load16<kOnce>(b[0], k0);
                    issue_load16<kOnce>(b[1], k0 + 8);
                    issue_load16<kOnce>(b[2], v0);
                    issue_load16<kOnce>(b[3], v0 + 8);
                    issue_load16<kOnce>(b[4], k1);
                    issue_load16<kOnce>(b[5], k1 + 8);
                    issue_load16<kOnce>(b[6], v1);
                    issue_load16<kOnce>(b[7], v1 + 8);
                };
                issue(0, buf[0]);
                if (kStages > 2 && kIters > 1) issue(1, buf[1 % kStages]);
#pragma unroll
                for (int it = 0; it < kIters; ++it) {
                    const int jj = j0 + it * 16;
                    if (it + kStages - 1 < kIters) issue(it + kStages - 1, buf[(it + kStages - 1) % kStages]);
                    u32x4(&b)[8] = buf[it % kStages];
                    if (kStages > 2 && it + 2 < kIters) wait_rows<16>(b);
                    else if (it + 1 < kIters) wait_rows<8>(b);
                    else wait_rows<0>(b);
                    if (jj < w1) {
                        const RowRegs cur0 = as_row(b[0], b[1], b[2], b[3]);
                        const RowRegs cur1 = as_row(b[4], b[5], b[6], b[7]);
                        float s0[G], s1[G];
                        qk_scores<G>(cur0, qlo, qhi, scale, jj + r < w1, s0);
                        qk_scores<G>(cur1, qlo, qhi, scale, jj + 8 + r < w1, s1);
                        softmax_step<G>(st, s0, s1, cur0, cur1);
                    }
                }
            }
        }
    }
}

// kBytes: the launch has a source of 8-bit rows.  Such launches get a kernel of their own, so that
// the registers of one row format's pipeline never cost the other its second wave per SIMD.
template <int G, bool kBytes>
__global__ __launch_bounds__(256) void value_pass_kernel(const ValuePassParams p)
{
    constexpr int HB = G < 4 ? G : 4;   // heads combined per round of the epilogue
    extern __shared__ float smem[];

    // chunk-major order: the first chunks of every unit are dispatched first, so the workgroups that
    // run last are the (often partly filled) last chunks of the longest source
    const int cidx = blockIdx.x / p.n_units;
    const int u = blockIdx.x - cidx * p.n_units;
    int si = 0;
#pragma unroll
    for (int i = 1; i < kMaxSources; ++i)
        if (i < p.n_sources && cidx >= p.src[i].chunk0) si = i;
    const RowSource& S = p.src[si];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int r = lane >> 3, c = lane & 7;

    int count = S.row0 + S.count_max;
    if (S.count_dev) {
        const int cd = S.count_dev[u];
        count = cd < count ? cd : count;
    }
    const int chunk_rows = S.chunk_rows;
    const int begin = S.row0 + (cidx - S.chunk0) * chunk_rows;
    const int end = (begin + chunk_rows < count) ? begin + chunk_rows : count;
    float* part = p.partials + ((long long)u * p.chunks_per_unit + cidx) * G * kPartStride;
    // A scored source may ride along instead of having workgroups of its own: its rows are shared out
    // evenly over this source's chunks and go through the same online softmax after the chunk's own rows.
    const bool bytes = kBytes && S.row_scale != nullptr;   // 8-bit rows: accumulator e of lane c is dim 16c + e
    const RowSource* T = S.guest ? &p.src[0] : nullptr;     // (always the launch's first source)
    int g0 = 0, g1 = 0;
    if (T) {
        int nt = T->count_max;
        if (T->count_dev) {
            const int cd = T->count_dev[u];
            nt = cd < nt ? cd : nt;
        }
        const long long k = cidx - S.chunk0;
        g0 = (int)(nt * k / S.n_chunks);
        g1 = (int)(nt * (k + 1) / S.n_chunks);
    }
    if (begin >= end && g0 >= g1) {   // nothing to do for this chunk: an empty partial
        if (tid < G) {
            part[tid * kPartStride + 0] = -INFINITY;
            part[tid * kPartStride + 1] = 0.f;
        }
        return;
    }

    // Groups of more than five heads do not fit one wave's registers next to the load pipeline: the
    // waves then work in pairs on the same rows, each wave of a pair on one half of the heads (the
    // second request for a row is served by the cache), two row streams per workgroup instead of four.
    constexpr bool kSplit = G > 5;
    constexpr int GH = kSplit ? (G + 1) / 2 : G;        // heads per wave
    const int half = kSplit ? (wave & 1) : 0;           // which heads: [0, GH) or [GH, G)
    HeadState<GH> st;
#pragma unroll
    for (int h = 0; h < GH; ++h) {
        st.m[h] = -INFINITY;
        st.l[h] = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) st.acc[h][e] = 0.f;
    }

    const int wave_rows = kSplit ? chunk_rows >> 1 : chunk_rows >> 2;
    const int w0 = begin + (kSplit ? wave >> 1 : wave) * wave_rows;
    const int w1 = (w0 + wave_rows < end) ? w0 + wave_rows : end;
    const int h0 = half * GH;
    if (begin >= end) {
        // (only the guest's rows)
    } else if (S.scores != nullptr) {
        stream_rows<GH, true, 8>(st, S, p, u, w0, w1, end, r, c, lane, G, h0);
    } else if constexpr (kBytes) {
        if (bytes && chunk_rows >= 512)
            stream_rows8<GH, 8, !kSplit>(st, S, p, u, w0, w1, end, r, c, lane, G, h0);
        else if (bytes)
            stream_rows8<GH, 2, !kSplit>(st, S, p, u, w0, w1, end, r, c, lane, G, h0);
        else   // (the bf16 rows of such a launch are the short unclustered tail)
            stream_rows<GH, false, 2, false, !kSplit>(st, S, p, u, w0, w1, end, r, c, lane, G, h0);
    } else {
        if (chunk_rows >= 512)
            stream_rows<GH, false, 8, false, !kSplit>(st, S, p, u, w0, w1, end, r, c, lane, G, h0);
        else
            stream_rows<GH, false, 2, false, !kSplit>(st, S, p, u, w0, w1, end, r, c, lane, G, h0);
    }

    if (g0 < g1) {
        const int streams = kSplit ? 2 : 4, wi = kSplit ? wave >> 1 : wave;
        const int per = (((g1 - g0) + streams - 1) / streams + 15) & ~15;
        const int a = g0 + wi * per, b = (a + per < g1) ? a + per : g1;
        if (a < b) {
            if (bytes) {
                if constexpr (kBytes) stream_rows<GH, true, 8, true>(st, *T, p, u, a, b, g1, r, c, lane, G, h0);
            } else {
                stream_rows<GH, true, 8>(st, *T, p, u, a, b, g1, r, c, lane, G, h0);
            }
        }
    }

    // -------- combine the 32 row groups of the workgroup (4 waves x 8 groups), HB heads per round ----
    float* sm_m = smem;             // [32][HB]
    float* sm_l = smem + 128;       // [32][HB]
    float* sm_w = smem + 256;       // [32][HB]
    float* sm_ml = smem + 384;      // [HB][2] : merged m and l
    float* sm_acc = smem + 400;     // [32][HB][128]
    const int sid = wave * 8 + r;
#pragma unroll
    for (int hb = 0; hb < G; hb += HB) {
        if (hb) __syncthreads();
#pragma unroll
        for (int hh = 0; hh < HB; ++hh) {
            const int h = hb + hh;
            if (h < G) {
                // this wave's state of head h, or nothing (m = -inf, zeros) for a head of the other half
                const int ia = h < GH ? h : 0, ib = h >= GH ? h - GH : 0;      // index as half 0 / half 1
                const bool own = !kSplit || (half == 0 ? h < GH : h >= GH);
                const float hm = half == 0 ? st.m[ia] : st.m[ib], hl = half == 0 ? st.l[ia] : st.l[ib];
                float a[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) a[e] = own ? (half == 0 ? st.acc[ia][e] : st.acc[ib][e]) : 0.f;
                if (c == 0) {
                    sm_m[sid * HB + hh] = own ? hm : -INFINITY;
                    sm_l[sid * HB + hh] = own ? hl : 0.f;
                }
                float4* dst = reinterpret_cast<float4*>(sm_acc + ((sid * HB + hh) * kHeadDim));
                const int lo = bytes ? 4 * c : 2 * c, hi = bytes ? 4 * c + 2 : 16 + 2 * c;
                dst[lo] = make_float4(a[0], a[1], a[2], a[3]);
                dst[lo + 1] = make_float4(a[4], a[5], a[6], a[7]);
                dst[hi] = make_float4(a[8], a[9], a[10], a[11]);
                dst[hi + 1] = make_float4(a[12], a[13], a[14], a[15]);
            }
        }
        __syncthreads();
        if (wave < HB && hb + wave < G) {
            // wave hh handles head hh: lane s < 32 holds the state of row group s
            const int hh = wave;
            const float mi = (lane < 32) ? sm_m[lane * HB + hh] : -INFINITY;
            float M = mi;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
            const float Ms = (M == -INFINITY) ? 0.f : M;
            const float w = (lane < 32) ? __builtin_amdgcn_exp2f(mi - Ms) : 0.f;
            float L = (lane < 32) ? sm_l[lane * HB + hh] * w : 0.f;
            if (lane < 32) sm_w[lane * HB + hh] = w;
            // fixed-order sum over the 32 groups (butterfly: the same order on every run)
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) L += __shfl_xor(L, off, 64);
            if (lane == 0) {
                sm_ml[2 * hh] = M;
                sm_ml[2 * hh + 1] = L;
            }
        }
        __syncthreads();
        for (int o = tid; o < HB * 64; o += 256) {
            const int hh = o >> 6, dp = o & 63;
            if (hb + hh < G) {
                float a0 = 0.f, a1 = 0.f;
#pragma unroll 8
                for (int s = 0; s < 32; ++s) {
                    const float w = sm_w[s * HB + hh];
                    const float2 v = *reinterpret_cast<const float2*>(sm_acc + ((s * HB + hh) * kHeadDim) + 2 * dp);
                    a0 = fmaf(w, v.x, a0);
                    a1 = fmaf(w, v.y, a1);
                }
                float* ph = part + (hb + hh) * kPartStride;
                *reinterpret_cast<float2*>(ph + 4 + 2 * dp) = make_float2(a0, a1);
                if (dp == 0) {
                    ph[0] = sm_ml[2 * hh];
                    ph[1] = sm_ml[2 * hh + 1];
                }
            }
        }
    }
}

// One workgroup of 128 threads per (unit, head); thread d combines dimension d over the chunks in
// chunk order (bit-reproducible).  Every thread reads the (m, l) pairs of all chunks itself (the
// same addresses across a wave: one transaction) and works out the weights 2^(m_i - M) on its own,
// so nothing is exchanged and nothing waited for except memory: kBatch chunks are fetched at a
// time, all loads of a batch in flight together, with an online rescale between batches (the
// launch picks the batch that covers all chunks in one trip to memory where it can).
template <int kBatch>
__global__ __launch_bounds__(128) void merge_kernel(const float* __restrict__ partials, int chunks_per_unit, int G,
                                                    uint16_t* __restrict__ out, float* __restrict__ lse)
{
    const int uh = blockIdx.x;
    const int u = uh / G, h = uh - u * G;
    const int d = threadIdx.x;
    const float* base = partials + ((long long)u * chunks_per_unit * G + h) * kPartStride;
    const long long cs = (long long)G * kPartStride;
    float M = -INFINITY, L = 0.f, a = 0.f;
    for (int i0 = 0; i0 < chunks_per_unit; i0 += kBatch) {
        float m[kBatch], l[kBatch], v[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int i = i0 + j < chunks_per_unit ? i0 + j : chunks_per_unit - 1;    // always a valid address
            m[j] = base[i * cs];
            l[j] = base[i * cs + 1];
            v[j] = base[i * cs + 4 + d];
        }
        float bm = -INFINITY;
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            if (i0 + j >= chunks_per_unit) m[j] = -INFINITY;
            bm = fmaxf(bm, m[j]);
        }
        const float Mn = fmaxf(M, bm);
        if (Mn == -INFINITY) continue;                       // only empty chunks so far
        const float keep = (M == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(M - Mn);
        a *= keep;
        L *= keep;
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const float w = (m[j] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m[j] - Mn);
            if (w > 0.f) {                                   // (an empty chunk's row is never looked at)
                a = fmaf(v[j], w, a);
                L = fmaf(l[j], w, L);
            }
        }
        M = Mn;
    }
    const float o = (L > 0.f) ? a / L : 0.f;
    out[(long long)uh * kHeadDim + d] = f32_to_bf16_rne(o);
    if (lse && d == 0) lse[uh] = (L > 0.f) ? (M + log2f(L)) * 0.6931471805599453f : -INFINITY;
}

template <int G>
hipError_t launch_vp(const ValuePassParams& p, hipStream_t stream)
{
    constexpr int HB = G < 4 ? G : 4;
    const size_t smem = sizeof(float) * (size_t)(400 + 32 * HB * kHeadDim);
    const long long blocks = (long long)p.n_units * p.chunks_per_unit;
    if (blocks <= 0) return hipSuccess;
    bool bytes = false;
    for (int i = 0; i < p.n_sources; ++i) bytes |= p.src[i].row_scale != nullptr;
    if (bytes)
        hipLaunchKernelGGL((value_pass_kernel<G, true>), dim3((unsigned)blocks), dim3(256), smem, stream, p);
    else
        hipLaunchKernelGGL((value_pass_kernel<G, false>), dim3((unsigned)blocks), dim3(256), smem, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_value_pass(const ValuePassParams& p, int G, hipStream_t stream)
{
    switch (G) {
        case 1: return launch_vp<1>(p, stream);
        case 2: return launch_vp<2>(p, stream);
        case 3: return launch_vp<3>(p, stream);
        case 4: return launch_vp<4>(p, stream);
        case 5: return launch_vp<5>(p, stream);
        case 6: return launch_vp<6>(p, stream);
        case 7: return launch_vp<7>(p, stream);
        case 8: return launch_vp<8>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_merge(const float* partials, int n_units, int chunks_per_unit, int G, uint16_t* out, float* lse,
                        hipStream_t stream)
{
    const long long blocks = (long long)n_units * G;
    if (blocks <= 0) return hipSuccess;
    if (chunks_per_unit <= 16)
        hipLaunchKernelGGL(merge_kernel<16>, dim3((unsigned)blocks), dim3(128), 0, stream, partials, chunks_per_unit, G, out, lse);
    else if (chunks_per_unit <= 32)
        hipLaunchKernelGGL(merge_kernel<32>, dim3((unsigned)blocks), dim3(128), 0, stream, partials, chunks_per_unit, G, out, lse);
    else
        hipLaunchKernelGGL(merge_kernel<64>, dim3((unsigned)blocks), dim3(128), 0, stream, partials, chunks_per_unit, G, out, lse);
    return hipGetLastError();
}

}  // namespace mp
