// Index construction kernels for gfx950: member lists (stable counting sort by cluster id),
// cluster-contiguous gather of the KV rows, and the per-cluster tables (N, key centroid, value
// centroid = bf16-rounded fp64 means of the member keys / values, Sec. 3.1 and 3.2).
//
// Member sums run over the members in sequence order, one wave per cluster, in fp64: the result
// does not depend on the launch shape and repeats bit for bit.
#include <type_traits>

#include "mp_device.h"
#include "mp_internal.h"

namespace mp {

namespace {

// cnt[u][id[u][t]] += 1
__global__ void histogram_kernel(const int32_t* __restrict__ ids, long long ids_stride, int n,
                                 int32_t* __restrict__ cnt, long long cnt_stride)
{
    const int u = blockIdx.y;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) atomicAdd(cnt + u * cnt_stride + ids[u * ids_stride + t], 1);
}

// start[u][0..k] = exclusive prefix sum of cnt[u][0..k), one workgroup of 1024 threads per unit.
__global__ __launch_bounds__(1024) void exclusive_scan_kernel(const int32_t* __restrict__ cnt, long long cnt_stride,
                                                              int k, int32_t* __restrict__ start,
                                                              long long start_stride)
{
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t carry_s;
    const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    for (int base = 0; base < k; base += 1024) {
        const int i = base + tid;
        const uint32_t v = (i < k) ? (uint32_t)cnt[u * cnt_stride + i] : 0u;
        const uint32_t incl = wave_incl_scan_u32(v);
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        uint32_t woff = 0;
        for (int w = 0; w < wave; ++w) woff += wsum[w];
        const uint32_t carry = carry_s;
        if (i < k) start[u * start_stride + i] = (int32_t)(carry + woff + incl - v);
        __syncthreads();
        if (tid == 1023) carry_s = carry + woff + incl;
        __syncthreads();
    }
    if (tid == 0) start[u * start_stride + k] = (int32_t)carry_s;
}

// Member lists: list[u][start[id] + rank] = point index, points of a cluster in ascending order.
// One thread per cluster walks the ids of its block (staged through LDS, every lane reads the same
// word, which LDS serves as a broadcast) and appends its own members.
// grid = (ceil(max clusters per block / 256), n_blocks, U)
constexpr int kListTile = 4096;
__global__ __launch_bounds__(256) void member_list_kernel(const int32_t* __restrict__ ids, long long ids_stride,
                                                          const int32_t* __restrict__ blocks /*[nb][4]: x0,x1,k0,k1*/,
                                                          const int32_t* __restrict__ start, long long start_stride,
                                                          int32_t* __restrict__ list, long long list_stride)
{
    __shared__ int32_t tile[kListTile];
    const int u = blockIdx.z, b = blockIdx.y;
    const int x0 = blocks[4 * b + 0], x1 = blocks[4 * b + 1], k0 = blocks[4 * b + 2], k1 = blocks[4 * b + 3];
    const int kbase = k0 + blockIdx.x * 256;
    if (kbase >= k1) return;
    const int my = kbase + threadIdx.x;
    const bool live = my < k1;
    int wr = live ? start[u * start_stride + my] : 0;
    const int32_t* idp = ids + u * ids_stride;
    int32_t* lp = list + u * list_stride;
    for (int t0 = x0; t0 < x1; t0 += kListTile) {
        const int nt = (x1 - t0 < kListTile) ? x1 - t0 : kListTile;
        __syncthreads();
        for (int i = threadIdx.x; i < nt; i += 256) tile[i] = idp[t0 + i];
        __syncthreads();
        if (live) {
            int i = 0;
            for (; i + 4 <= nt; i += 4) {
                const int4 v = *reinterpret_cast<const int4*>(&tile[i]);
                if (v.x == my) lp[wr++] = t0 + i;
                if (v.y == my) lp[wr++] = t0 + i + 1;
                if (v.z == my) lp[wr++] = t0 + i + 2;
                if (v.w == my) lp[wr++] = t0 + i + 3;
            }
            for (; i < nt; ++i)
                if (tile[i] == my) lp[wr++] = t0 + i;
        }
    }
}

// Member lists and their offsets for every block of a unit in one launch: a stable counting sort of
// the block's points by cluster id.  One workgroup of 16 waves per (block, unit); `waves` of them
// walk one contiguous segment of the block's points each, 64 points at a time.
//   Among the 64 points of a step, the lanes that share this lane's id are found with one ballot per
//   id bit; a point's rank among them is the number of such lanes below it, and the lowest of them
//   adds their number to the segment's counter of that id (LDS, touched by this wave only).
//   walk 1 counts; then counter[w][id] becomes the position of the first member of id in segment w
//   (block offset + exclusive prefix over ids + members in earlier segments); walk 2 writes the
//   members at counter + rank.  Within a cluster the members end up in ascending point order.
// start[u][id] = first list position of cluster id (positions count from the first point of the
// launch, `p_first`); the last block also writes the end position after its last cluster.
// Dynamic LDS: (waves + 1) * max clusters per block int32.
constexpr int kListWaves = 16;
__global__ __launch_bounds__(1024) void block_lists_kernel(const int32_t* __restrict__ ids, long long ids_stride,
                                                           const int32_t* __restrict__ blocks /*[nb][4]: x0,x1,k0,k1*/,
                                                           int p_first, int waves, int32_t* __restrict__ start,
                                                           long long start_stride, int32_t* __restrict__ list,
                                                           long long list_stride)
{
    extern __shared__ int32_t lists_lds[];
    __shared__ int32_t wave_tot[kListWaves];
    const int b = blockIdx.x, u = blockIdx.y;
    const int x0 = blocks[4 * b + 0], x1 = blocks[4 * b + 1], k0 = blocks[4 * b + 2], k1 = blocks[4 * b + 3];
    const int k = k1 - k0, n = x1 - x0;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int32_t* ctr = lists_lds;                  // [waves][k]
    int32_t* tot = lists_lds + waves * k;      // [k]
    const int32_t* idp = ids + u * ids_stride;
    int32_t* lp = list + u * list_stride;
    const int bits = k > 1 ? 32 - __clz(k - 1) : 0;
    const int seg = (((n + waves - 1) / waves) + 63) & ~63;
    const int s0 = x0 + wave * seg, s1 = (s0 + seg < x1) ? s0 + seg : x1;
    const unsigned long long below = (1ull << lane) - 1ull;

    for (int i = tid; i < waves * k; i += 1024) ctr[i] = 0;
    __syncthreads();
    // one walk over the wave's segment; kWrite = false: count, true: place
    auto walk = [&](auto write_tag) {
        constexpr bool kWrite = decltype(write_tag)::value;
        if (wave >= waves) return;
        int32_t* my = ctr + wave * k;
        for (int t0 = s0; t0 < s1; t0 += 256) {
            int id4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int t = t0 + 64 * r + lane;
                id4[r] = t < s1 ? idp[t] - k0 : -1;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int t = t0 + 64 * r + lane;
                const int id = id4[r];
                const bool valid = id >= 0;
                unsigned long long same = __ballot(valid);
                for (int bit = 0; bit < bits; ++bit) {
                    const bool one = (id >> bit) & 1;
                    const unsigned long long m = __ballot(valid && one);
                    same &= one ? m : ~m;
                }
                const int rank = __popcll(same & below);
                if (valid) {
                    const int base = my[id];
                    if (kWrite) lp[base + rank] = t;
                    if (rank == 0) my[id] = base + __popcll(same);
                }
            }
        }
    };
    walk(std::false_type{});
    __syncthreads();
    // counts per segment -> first positions: totals per id, exclusive prefix over ids, segments in order
    const int per = (k + 1023) / 1024;          // consecutive ids per thread
    const int i0 = tid * per, i1 = (i0 + per < k) ? i0 + per : k;
    int run = 0;
    for (int id = i0; id < i1; ++id) {
        int c = 0;
        for (int w = 0; w < waves; ++w) c += ctr[w * k + id];
        tot[id] = c;
        run += c;
    }
    const int incl = (int)wave_incl_scan_u32((uint32_t)run);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int pos = x0 - p_first + incl - run;
    for (int w = 0; w < wave; ++w) pos += wave_tot[w];
    for (int id = i0; id < i1; ++id) {
        start[u * start_stride + k0 + id] = pos;
        int q = pos;
        for (int w = 0; w < waves; ++w) {
            const int c = ctr[w * k + id];
            ctr[w * k + id] = q;
            q += c;
        }
        pos += tot[id];
    }
    if (b == (int)gridDim.x - 1 && tid == 0) start[u * start_stride + k1] = x1 - p_first;
    __syncthreads();
    walk(std::true_type{});
}

// dst[u][p] = src[u][list[u][p]] for 256-byte rows; one thread moves 16 bytes.
__global__ void gather_rows_kernel(const uint4* __restrict__ srcK, const uint4* __restrict__ srcV,
                                   long long src_unit_rows, const int32_t* __restrict__ list, long long list_stride,
                                   int n, uint4* __restrict__ dstK, uint4* __restrict__ dstV, long long dst_unit_rows,
                                   int dst_row0)
{
    const int u = blockIdx.y;
    const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long p = g >> 4;
    const int c = (int)(g & 15);
    if (p >= n) return;
    const long long s = list[u * list_stride + p];
    // (a pure stream: every line is read once and written once)
    store_once(&dstK[((long long)u * dst_unit_rows + dst_row0 + p) * 16 + c], load_once(&srcK[((long long)u * src_unit_rows + s) * 16 + c]));
    store_once(&dstV[((long long)u * dst_unit_rows + dst_row0 + p) * 16 + c], load_once(&srcV[((long long)u * src_unit_rows + s) * 16 + c]));
}

// The same gather into 8-bit storage.  A value row becomes 128 e4m3 codes (OCP format: bias 7,
// largest magnitude 448, no infinities) and one fp32 scale, scale = max|x| / 448 (1 for a zero row),
// code = x / scale rounded to nearest even; both divisions are IEEE fp32.  A key row is stored the
// same way as its residual from the key centroid of its fine cluster, x = fp32(k) - fp32(centroid):
// the decode step already has q . centroid, and the residual is small where the key itself is not.
// Sixteen threads share a row (8 elements of the key and 8 of the value each);
// scales[u][row] = {key scale, value scale}.
// Elementwise fp32 difference of two groups of eight bf16 values.
struct F8 { float v[8]; };
__device__ __forceinline__ F8 widen8(const uint4& w)
{
    const uint32_t d[4] = {w.x, w.y, w.z, w.w};
    F8 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o.v[2 * i] = bf16lo_to_f32(d[i]);
        o.v[2 * i + 1] = bf16hi_to_f32(d[i]);
    }
    return o;
}
__device__ __forceinline__ float absmax8(const F8& x)
{
    float a = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf(x.v[i]));
    return a;
}
__device__ __forceinline__ uint2 e4m3_codes8(const F8& x, float scale)
{
    // (the quotient of the row's largest entry may exceed 448 by an ulp: clamp, so that the conversion never overflows)
    auto q = [&](float v) { return fminf(fmaxf(v / scale, -448.f), 448.f); };
    int out[2] = {0, 0};
    out[0] = __builtin_amdgcn_cvt_pk_fp8_f32(q(x.v[0]), q(x.v[1]), out[0], false);
    out[0] = __builtin_amdgcn_cvt_pk_fp8_f32(q(x.v[2]), q(x.v[3]), out[0], true);
    out[1] = __builtin_amdgcn_cvt_pk_fp8_f32(q(x.v[4]), q(x.v[5]), out[1], false);
    out[1] = __builtin_amdgcn_cvt_pk_fp8_f32(q(x.v[6]), q(x.v[7]), out[1], true);
    return make_uint2((uint32_t)out[0], (uint32_t)out[1]);
}
__global__ void gather_quantize_rows_kernel(const uint4* __restrict__ srcK, const uint4* __restrict__ srcV,
                                            long long src_unit_rows, const int32_t* __restrict__ list,
                                            long long list_stride, const int32_t* __restrict__ ids, long long ids_stride,
                                            const uint4* __restrict__ Kc, long long kc_unit_rows, int n,
                                            uint2* __restrict__ dstK, uint2* __restrict__ dstV,
                                            float2* __restrict__ scales, long long dst_unit_rows, int dst_row0)
{
    const int u = blockIdx.y;
    const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long p = g >> 4;
    const int c = (int)(g & 15);
    if (p >= n) return;   // (all sixteen threads of a row leave together)
    const long long s = list[u * list_stride + p];
    const long long f = ids[u * ids_stride + s];
    F8 k = widen8(srcK[((long long)u * src_unit_rows + s) * 16 + c]);
    const F8 cen = widen8(Kc[((long long)u * kc_unit_rows + f) * 16 + c]);
    const F8 v = widen8(srcV[((long long)u * src_unit_rows + s) * 16 + c]);
#pragma unroll
    for (int i = 0; i < 8; ++i) k.v[i] -= cen.v[i];
    float ka = absmax8(k), va = absmax8(v);
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
        ka = fmaxf(ka, __shfl_xor(ka, off, 64));
        va = fmaxf(va, __shfl_xor(va, off, 64));
    }
    const float ks = ka > 0.f ? ka / 448.f : 1.f, vs = va > 0.f ? va / 448.f : 1.f;
    const long long row = (long long)u * dst_unit_rows + dst_row0 + p;
    dstK[row * 16 + c] = e4m3_codes8(k, ks);
    dstV[row * 16 + c] = e4m3_codes8(v, vs);
    if (c == 0) scales[row] = make_float2(ks, vs);
}

// One wave per cluster of [k0, k): fp64 sum of the member rows in list order, mean rounded once to bf16.
// Lane l owns dims 2l and 2l+1.  Empty cluster: `fallback` row if given (else zeros).
// mean_out row index = out_row0 + cluster id.  count_out optional.
__global__ __launch_bounds__(256) void cluster_mean_kernel(const uint16_t* __restrict__ X, long long x_unit_rows,
                                                           const int32_t* __restrict__ list, long long list_stride,
                                                           const int32_t* __restrict__ start, long long start_stride,
                                                           int k0, int k, uint16_t* __restrict__ mean_out,
                                                           long long out_unit_rows, int out_row0,
                                                           const uint16_t* __restrict__ fallback,
                                                           long long fb_unit_rows, int32_t* __restrict__ count_out,
                                                           long long count_stride, int count_off,
                                                           double* __restrict__ sum_out, long long sum_unit_rows)
{
    const int u = blockIdx.y;
    const int f = k0 + blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (f >= k) return;
    const int s0 = start[u * start_stride + f], s1 = start[u * start_stride + f + 1];
    const uint32_t* Xu = reinterpret_cast<const uint32_t*>(X + (long long)u * x_unit_rows * kHeadDim);
    const int32_t* lp = list ? list + u * list_stride : nullptr;
    double a0 = 0.0, a1 = 0.0;
    // 64 member indices at a time (one per lane), then their rows kBatch at a time: the row numbers
    // reach every lane through a lane broadcast, so that kBatch row loads are in flight at once while
    // the additions keep the members' order (a wave's time is the number of trips to memory it makes:
    // with 8 rows a trip the means of coarse clusters of some hundred rows took 160 us per call in an
    // online refresh, with 32 rows a trip a third of that)
    constexpr int kBatch = 32;
    for (int base = s0; base < s1; base += 64) {
        const int nm = (s1 - base < 64) ? s1 - base : 64;
        const int mine = (lane < nm) ? (lp ? lp[base + lane] : base + lane) : 0;
        for (int m = 0; m < nm; m += kBatch) {
            uint32_t w[kBatch];
#pragma unroll
            for (int q = 0; q < kBatch; ++q) {
                const long long r = __builtin_amdgcn_readlane(mine, (m + q) & 63);
                w[q] = (m + q < nm) ? load_once(&Xu[r * 64 + lane]) : 0u;
            }
#pragma unroll
            for (int q = 0; q < kBatch; ++q) {
                if (m + q < nm) {
                    a0 += (double)bf16lo_to_f32(w[q]);
                    a1 += (double)bf16hi_to_f32(w[q]);
                }
            }
        }
    }
    const int n = s1 - s0;
    uint32_t outw;
    if (n > 0) {
        const double inv = (double)n;
        outw = (uint32_t)f64_to_bf16_rne(a0 / inv) | ((uint32_t)f64_to_bf16_rne(a1 / inv) << 16);
    } else if (fallback) {
        outw = reinterpret_cast<const uint32_t*>(fallback + ((long long)u * fb_unit_rows + f) * kHeadDim)[lane];
    } else {
        outw = 0u;
    }
    reinterpret_cast<uint32_t*>(mean_out + ((long long)u * out_unit_rows + out_row0 + f) * kHeadDim)[lane] = outw;
    if (count_out && lane == 0) count_out[u * count_stride + count_off + f] = n;
    if (sum_out) reinterpret_cast<double2*>(sum_out + ((long long)u * sum_unit_rows + f) * kHeadDim)[lane] = make_double2(a0, a1);
}

// Stored tables of the coarse clusters [c0, c1) from those of their fine clusters (Sec. 3.4: a coarse
// centroid is the mean of all rows below it): one wave per coarse cluster adds its children's fp64 member
// sums in ascending fine id, starting from zero, divides by the children's member count and rounds once
// to bf16.  The sum of fine cluster f is row (map ? map[f - map_f0] : f) of `sums` (sums taken before a
// renumbering sit at the old ids).  Empty cluster: `fallback` row if given (else zeros).  Lane l owns
// dims 2l and 2l+1, as in cluster_mean_kernel.
__global__ __launch_bounds__(256) void coarse_from_children_kernel(const double* __restrict__ sums, long long sum_unit_rows,
                                                                   const int32_t* __restrict__ map, long long map_stride,
                                                                   int map_f0, const int32_t* __restrict__ cstart,
                                                                   long long cstart_stride,
                                                                   const int32_t* __restrict__ fine_count,
                                                                   long long count_stride, int c0, int c1,
                                                                   uint16_t* __restrict__ mean_out, long long out_unit_rows,
                                                                   int out_row0, const uint16_t* __restrict__ fallback,
                                                                   long long fb_unit_rows, int32_t* __restrict__ count_out,
                                                                   int count_off)
{
    const int u = blockIdx.y;
    const int c = c0 + blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (c >= c1) return;
    const int f_begin = cstart[u * cstart_stride + c], f_end = cstart[u * cstart_stride + c + 1];
    const double2* Su = reinterpret_cast<const double2*>(sums + (long long)u * sum_unit_rows * kHeadDim);
    double a0 = 0.0, a1 = 0.0;
    long long n = 0;
    for (int base = f_begin; base < f_end; base += 8) {      // eight children's rows in flight, added in order
        double2 w[8];
        int cnt[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int f = base + q;
            w[q] = make_double2(0.0, 0.0);
            cnt[q] = 0;
            if (f < f_end) {
                const long long src = map ? map[u * map_stride + (f - map_f0)] : f;
                w[q] = Su[src * 64 + lane];
                cnt[q] = fine_count[u * count_stride + f];
            }
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            if (base + q < f_end) {
                a0 += w[q].x;
                a1 += w[q].y;
                n += cnt[q];
            }
        }
    }
    uint32_t outw;
    if (n > 0) {
        const double inv = (double)n;
        outw = (uint32_t)f64_to_bf16_rne(a0 / inv) | ((uint32_t)f64_to_bf16_rne(a1 / inv) << 16);
    } else if (fallback) {
        outw = reinterpret_cast<const uint32_t*>(fallback + ((long long)u * fb_unit_rows + c) * kHeadDim)[lane];
    } else {
        outw = 0u;
    }
    reinterpret_cast<uint32_t*>(mean_out + ((long long)u * out_unit_rows + out_row0 + c) * kHeadDim)[lane] = outw;
    if (count_out && lane == 0) count_out[u * count_stride + count_off + c] = (int32_t)n;
}

// For the fine range [f0, f1) whose coarse ids lie in [c0, c1) and are non-decreasing in the fine id:
// cstart[u][c] = first fine id of the range whose coarse id is >= c, for c in [c0, c1]; cstart[c1] = f1.
__global__ void coarse_start_kernel(const int32_t* __restrict__ cof, long long cof_stride, int f0, int f1, int c0,
                                    int c1, int32_t* __restrict__ cstart, long long cstart_stride)
{
    const int u = blockIdx.y;
    const int f = f0 + blockIdx.x * blockDim.x + threadIdx.x;
    if (f > f1) return;
    const int cur = (f < f1) ? cof[u * cof_stride + f] : c1;
    const int prev = (f > f0) ? cof[u * cof_stride + f - 1] : c0 - 1;
    for (int c = prev + 1; c <= cur; ++c) cstart[u * cstart_stride + c] = f;
}

// Stored-order tables from member lists built on local point indices:
// fstart[u][f] = pt0 + start[u][f] for f in [f0, f1];  perm[u][pt0 + p] = pt0 + list[u][p] for p < n_pts.
__global__ void offset_lists_kernel(const int32_t* __restrict__ start, long long start_stride, int f0, int f1,
                                    const int32_t* __restrict__ list, long long list_stride, int n_pts, int pt0,
                                    int32_t* __restrict__ fstart, long long fstart_stride, int32_t* __restrict__ perm,
                                    long long perm_stride)
{
    const int u = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_pts) perm[u * perm_stride + pt0 + i] = pt0 + list[u * list_stride + i];
    if (i <= f1 - f0) fstart[u * fstart_stride + f0 + i] = pt0 + start[u * start_stride + f0 + i];
}

// fot[u][list[p]] = f for p in [start[f], start[f+1])  (inverse of the member lists)
__global__ void ids_from_lists_kernel(const int32_t* __restrict__ list, long long list_stride,
                                      const int32_t* __restrict__ start, long long start_stride, int k,
                                      int32_t* __restrict__ ids, long long ids_stride)
{
    const int u = blockIdx.y;
    const int f = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (f >= k) return;
    const int s0 = start[u * start_stride + f], s1 = start[u * start_stride + f + 1];
    for (int p = s0 + lane; p < s1; p += 64) ids[u * ids_stride + list[u * list_stride + p]] = f;
}

// Dense per-cluster views of the last decode call's selection, from the per-candidate arrays:
// sel[u][id] = flag of the candidate with that id (0 if it was no candidate), r[u][id] = its rank
// key (NaN if it was no candidate).  One workgroup per unit.
__global__ __launch_bounds__(256) void scatter_selection_kernel(const int32_t* __restrict__ cand,
                                                                long long cand_stride,
                                                                const int32_t* __restrict__ n_cand_dev,
                                                                int n_cand_fixed, const uint8_t* __restrict__ flag,
                                                                const unsigned long long* __restrict__ keys,
                                                                const int32_t* __restrict__ key_mode, int level, int G,
                                                                long long pos_stride, int n_ids,
                                                                uint8_t* __restrict__ sel_out, double* __restrict__ r_out)
{
    const int u = blockIdx.x;
    const int n = n_cand_dev ? n_cand_dev[u] : n_cand_fixed;
    const double nan = __longlong_as_double(0x7ff8000000000000ll);
    const int mode = key_mode[2 * u + level];
    const double logG = log((double)G);
    for (int i = threadIdx.x; i < n_ids; i += 256) {
        if (sel_out) sel_out[(long long)u * n_ids + i] = 0;
        if (r_out) r_out[(long long)u * n_ids + i] = nan;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += 256) {
        const int id = cand ? cand[u * cand_stride + i] : i;
        if (sel_out) sel_out[(long long)u * n_ids + id] = flag[u * pos_stride + i];
        if (r_out) {
            const unsigned long long key = keys[u * pos_stride + i];
            double r = nan;
            if (key != ~0ull) {
                if (mode == 1) {
                    r = log(__longlong_as_double((long long)~key)) - logG;
                } else {    // undo the order-preserving map of the rank key
                    unsigned long long b = ~key;
                    b = (b >> 63) ? (b & 0x7fffffffffffffffull) : ~b;
                    r = __longlong_as_double((long long)b);
                }
            }
            r_out[(long long)u * n_ids + id] = r;
        }
    }
}

}  // namespace

hipError_t launch_scatter_selection(const int32_t* cand, long long cand_stride, const int32_t* n_cand_dev,
                                    int n_cand_fixed, const uint8_t* flag, const unsigned long long* keys,
                                    const int32_t* key_mode, int level, int G, long long pos_stride, int n_ids, int U,
                                    uint8_t* sel_out, double* r_out, hipStream_t s)
{
    if (n_ids <= 0) return hipSuccess;
    hipLaunchKernelGGL(scatter_selection_kernel, dim3(U), dim3(256), 0, s, cand, cand_stride, n_cand_dev,
                       n_cand_fixed, flag, keys, key_mode, level, G, pos_stride, n_ids, sel_out, r_out);
    return hipGetLastError();
}

// ---- host launchers ----------------------------------------------------------------------------
hipError_t launch_histogram(const int32_t* ids, long long ids_stride, int n, int U, int32_t* cnt,
                            long long cnt_stride, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(histogram_kernel, dim3((n + 255) / 256, U), dim3(256), 0, s, ids, ids_stride, n, cnt,
                       cnt_stride);
    return hipGetLastError();
}

hipError_t launch_exclusive_scan(const int32_t* cnt, long long cnt_stride, int k, int U, int32_t* start,
                                 long long start_stride, hipStream_t s)
{
    hipLaunchKernelGGL(exclusive_scan_kernel, dim3(U), dim3(1024), 0, s, cnt, cnt_stride, k, start, start_stride);
    return hipGetLastError();
}

hipError_t launch_member_lists(const int32_t* ids, long long ids_stride, const int32_t* blocks_dev, int nb,
                               int max_k_per_block, int U, const int32_t* start, long long start_stride,
                               int32_t* list, long long list_stride, hipStream_t s)
{
    if (nb <= 0 || max_k_per_block <= 0) return hipSuccess;
    hipLaunchKernelGGL(member_list_kernel, dim3((max_k_per_block + 255) / 256, nb, U), dim3(256), 0, s, ids,
                       ids_stride, blocks_dev, start, start_stride, list, list_stride);
    return hipGetLastError();
}

hipError_t launch_block_lists(const int32_t* ids, long long ids_stride, const int32_t* blocks_dev, int nb,
                              int max_k_per_block, int p_first, int U, int32_t* start, long long start_stride,
                              int32_t* list, long long list_stride, hipStream_t s)
{
    if (nb <= 0 || max_k_per_block <= 0) return hipSuccess;
    constexpr int kLdsInts = 16384;            // 64 KiB
    if (2 * max_k_per_block > kLdsInts) return hipErrorInvalidValue;
    int waves = kLdsInts / max_k_per_block - 1;
    if (waves > kListWaves) waves = kListWaves;
    const size_t smem = (size_t)(waves + 1) * max_k_per_block * sizeof(int32_t);
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&block_lists_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsInts * 4);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(block_lists_kernel, dim3(nb, U), dim3(1024), smem, s, ids, ids_stride, blocks_dev, p_first,
                       waves, start, start_stride, list, list_stride);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const void* srcK, const void* srcV, long long src_unit_rows, const int32_t* list,
                              long long list_stride, int n, int U, void* dstK, void* dstV, long long dst_unit_rows,
                              int dst_row0, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const long long threads = (long long)n * 16;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((threads + 255) / 256), U), dim3(256), 0, s,
                       (const uint4*)srcK, (const uint4*)srcV, src_unit_rows, list, list_stride, n, (uint4*)dstK,
                       (uint4*)dstV, dst_unit_rows, dst_row0);
    return hipGetLastError();
}

hipError_t launch_gather_quantize_rows(const void* srcK, const void* srcV, long long src_unit_rows, const int32_t* list,
                                       long long list_stride, const int32_t* ids, long long ids_stride,
                                       const uint16_t* Kc, long long kc_unit_rows, int n, int U, void* dstK, void* dstV,
                                       float* scales, long long dst_unit_rows, int dst_row0, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const long long threads = (long long)n * 16;
    hipLaunchKernelGGL(gather_quantize_rows_kernel, dim3((unsigned)((threads + 255) / 256), U), dim3(256), 0, s,
                       (const uint4*)srcK, (const uint4*)srcV, src_unit_rows, list, list_stride, ids, ids_stride,
                       (const uint4*)Kc, kc_unit_rows, n, (uint2*)dstK, (uint2*)dstV, (float2*)scales, dst_unit_rows,
                       dst_row0);
    return hipGetLastError();
}

hipError_t launch_cluster_means(const uint16_t* X, long long x_unit_rows, const int32_t* list, long long list_stride,
                                const int32_t* start, long long start_stride, int k0, int k, int U,
                                uint16_t* mean_out, long long out_unit_rows, int out_row0, const uint16_t* fallback,
                                long long fb_unit_rows, int32_t* count_out, long long count_stride, int count_off,
                                double* sum_out, long long sum_unit_rows, hipStream_t s)
{
    if (k <= k0) return hipSuccess;
    hipLaunchKernelGGL(cluster_mean_kernel, dim3((k - k0 + 3) / 4, U), dim3(256), 0, s, X, x_unit_rows, list,
                       list_stride, start, start_stride, k0, k, mean_out, out_unit_rows, out_row0, fallback,
                       fb_unit_rows, count_out, count_stride, count_off, sum_out, sum_unit_rows);
    return hipGetLastError();
}

hipError_t launch_coarse_from_children(const double* sums, long long sum_unit_rows, const int32_t* map, long long map_stride,
                                       int map_f0, const int32_t* cstart, long long cstart_stride,
                                       const int32_t* fine_count, long long count_stride, int c0, int c1, int U,
                                       uint16_t* mean_out, long long out_unit_rows, int out_row0, const uint16_t* fallback,
                                       long long fb_unit_rows, int32_t* count_out, int count_off, hipStream_t s)
{
    if (c1 <= c0) return hipSuccess;
    hipLaunchKernelGGL(coarse_from_children_kernel, dim3((c1 - c0 + 3) / 4, U), dim3(256), 0, s, sums, sum_unit_rows, map,
                       map_stride, map_f0, cstart, cstart_stride, fine_count, count_stride, c0, c1, mean_out, out_unit_rows,
                       out_row0, fallback, fb_unit_rows, count_out, count_off);
    return hipGetLastError();
}

hipError_t launch_coarse_start(const int32_t* cof, long long cof_stride, int f0, int f1, int c0, int c1, int U,
                               int32_t* cstart, long long cstart_stride, hipStream_t s)
{
    hipLaunchKernelGGL(coarse_start_kernel, dim3((f1 - f0 + 1 + 255) / 256, U), dim3(256), 0, s, cof, cof_stride, f0,
                       f1, c0, c1, cstart, cstart_stride);
    return hipGetLastError();
}

hipError_t launch_offset_lists(const int32_t* start, long long start_stride, int f0, int f1, const int32_t* list,
                               long long list_stride, int n_pts, int pt0, int U, int32_t* fstart,
                               long long fstart_stride, int32_t* perm, long long perm_stride, hipStream_t s)
{
    const int n = n_pts > f1 - f0 + 1 ? n_pts : f1 - f0 + 1;
    hipLaunchKernelGGL(offset_lists_kernel, dim3((n + 255) / 256, U), dim3(256), 0, s, start, start_stride, f0, f1,
                       list, list_stride, n_pts, pt0, fstart, fstart_stride, perm, perm_stride);
    return hipGetLastError();
}

hipError_t launch_ids_from_lists(const int32_t* list, long long list_stride, const int32_t* start,
                                 long long start_stride, int k, int U, int32_t* ids, long long ids_stride,
                                 hipStream_t s)
{
    if (k <= 0) return hipSuccess;
    hipLaunchKernelGGL(ids_from_lists_kernel, dim3((k + 3) / 4, U), dim3(256), 0, s, list, list_stride, start,
                       start_stride, k, ids, ids_stride);
    return hipGetLastError();
}

}  // namespace mp
