// Nearest-centroid assignment of blockwise k-means (Sec. 3.2: assignment step of Lloyd's iterations
// inside each block of the sequence; also the one-shot assignment of appended tokens, Sec. 3.3).
//
// The result is defined in fp64: a[t] = argmin_j sum_i (x_t[i] - c_j[i])^2 with the sum taken in
// index order and the lowest j among equal distances.  Points and centroids are bf16 values, so the
// bulk of the work is a bf16 contraction and runs on the matrix cores; fp64 is only spent where it
// can change the answer:
//
//   1. assign_mfma_kernel: s[t,j] = x_t.c_j - |c_j|^2/2 (argmax = nearest centroid) with
//      v_mfma_f32_32x32x16_bf16, fp32 accumulation.  Per point it keeps the best and the second
//      best score.  The products are exact and every one of the 128 accumulation steps loses at
//      most one unit in the last place of a partial sum bounded by |x||c|, so each score is within
//      2^-16 max(|x|^2, max_j |c_j|^2) of its exact value.  A point whose two best scores are
//      further apart than 2^-13 of that scale has a unique nearest centroid in exact arithmetic
//      too (and by far more than fp64 rounding), which is the fp64 answer.
//   2. Every other point (near-equal or equal distances) goes onto a per-block list and
//      assign_exact_list_kernel recomputes it exactly as defined above, over all centroids of the
//      block, in fp64 without fused multiply-adds.
#include "mp_device.h"
#include "mp_internal.h"

namespace mp {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kTile = 32;                 // centroids per tile = rows of the MFMA A operand
constexpr int kRowBytes = 256 + 16;       // padded LDS row of one centroid
constexpr float kMarginScale = 1.0f / 8192.0f;   // 2^-13

// grid = (ceil(max points per block / 128), nb, U); 256 threads = 4 waves of 32 points.
// blocks: int32 [nb][4] = {first point, end point, first centroid, end centroid}.
// assign[u][t] receives the best centroid of stage 1; amb_list[u][first point + i], i < amb_cnt[u][b],
// the points of block b that stage 2 has to recompute.
__global__ __launch_bounds__(256) void assign_mfma_kernel(const uint16_t* __restrict__ X, long long x_unit_rows,
                                                          const int32_t* __restrict__ blocks,
                                                          const uint16_t* __restrict__ C, long long c_unit_rows,
                                                          int32_t* __restrict__ assign, long long assign_stride,
                                                          int32_t* __restrict__ amb_list, long long list_stride,
                                                          int32_t* __restrict__ amb_cnt, int cnt_stride)
{
    __shared__ __align__(16) unsigned char tile[kTile * kRowBytes];
    __shared__ __align__(16) float tile_c2[kTile];       // -|c|^2 / 2, -inf past the last centroid
    const int u = blockIdx.z, b = blockIdx.y;
    const int x0 = blocks[4 * b + 0], x1 = blocks[4 * b + 1], k0 = blocks[4 * b + 2], k1 = blocks[4 * b + 3];
    const int p0 = x0 + (int)blockIdx.x * 128;
    if (p0 >= x1) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int t = p0 + wave * 32 + col;
    const bool live = t < x1;

    // B operand: this lane's point, dims [16 ks + 8 half, +8) for ks = 0..7
    bf16x8_t xb[8];
    float x2 = 0.f;
    {
        const uint4* xp = reinterpret_cast<const uint4*>(X + ((long long)u * x_unit_rows + (live ? t : x0)) * kHeadDim);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const uint4 w = xp[2 * ks + half];
            xb[ks] = __builtin_bit_cast(bf16x8_t, w);
            const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = bf16lo_to_f32(ww[e]), hi = bf16hi_to_f32(ww[e]);
                x2 = fmaf(lo, lo, x2);
                x2 = fmaf(hi, hi, x2);
            }
        }
    }
    float best = -INFINITY, second = -INFINITY, c2max = 0.f;
    int bj = k0;
    for (int j0 = k0; j0 < k1; j0 += kTile) {
        const int nj = (k1 - j0 < kTile) ? k1 - j0 : kTile;
        __syncthreads();
        // centroid tile -> LDS (zero rows past the end) and its squared norms: 8 threads per row
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int e = pass * 256 + tid;
            const int row = e >> 4, seg = e & 15;
            uint4 w = make_uint4(0, 0, 0, 0);
            if (row < nj) w = reinterpret_cast<const uint4*>(C + ((long long)u * c_unit_rows + j0 + row) * kHeadDim)[seg];
            *reinterpret_cast<uint4*>(tile + row * kRowBytes + seg * 16) = w;
            const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
            float s = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float lo = bf16lo_to_f32(ww[q]), hi = bf16hi_to_f32(ww[q]);
                s = fmaf(lo, lo, s);
                s = fmaf(hi, hi, s);
            }
            s = sum8(s);
            s += dpp_f32<kDppMirror>(s);      // the other 8 lanes of the row of 16
            if (seg == 0) tile_c2[row] = row < nj ? -0.5f * s : -INFINITY;
        }
        __syncthreads();
        // accumulator rows of this lane: m(i) = 8 (i / 4) + 4 half + i % 4
        f32x16_t acc;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float4 c = *reinterpret_cast<const float4*>(&tile_c2[8 * g + 4 * half]);
            acc[4 * g + 0] = c.x; acc[4 * g + 1] = c.y; acc[4 * g + 2] = c.z; acc[4 * g + 3] = c.w;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (acc[i] != -INFINITY) c2max = fmaxf(c2max, -2.f * acc[i]);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(tile + col * kRowBytes + 32 * ks + 16 * half);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xb[ks], acc, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float v = acc[i];
            const int j = j0 + 8 * (i >> 2) + 4 * half + (i & 3);
            second = fmaxf(second, fminf(best, v));
            bj = v > best ? j : bj;
            best = fmaxf(best, v);
        }
    }
    // the two halves of the wave hold the other rows of the same point
    {
        const float ob = __shfl_xor(best, 32, 64), os = __shfl_xor(second, 32, 64), oc = __shfl_xor(c2max, 32, 64);
        const int oj = __shfl_xor(bj, 32, 64);
        const float ox = __shfl_xor(x2, 32, 64);
        second = fmaxf(fmaxf(second, os), fminf(best, ob));
        if (ob > best || (ob == best && oj < bj)) bj = oj;
        best = fmaxf(best, ob);
        c2max = fmaxf(c2max, oc);
        x2 += ox;
    }
    if (live && half == 0) {
        assign[u * assign_stride + t] = bj;
        const float margin = kMarginScale * fmaxf(x2, c2max);
        // (written so that a NaN score also sends the point to the exact pass)
        if (!(best - second > margin)) {
            const int pos = atomicAdd(&amb_cnt[u * cnt_stride + b], 1);
            amb_list[u * list_stride + x0 + pos] = t;
        }
    }
}

// Exact assignment of the listed points.  A workgroup takes 32 listed points; the 8 threads that
// share a point split every tile of 32 centroids among them (thread s takes centroids s, s+8, ...),
// each computing whole distances in the defining order, and the 8 partial results are merged with
// the lower centroid index winning equal distances.  The block's centroids pass through LDS as
// doubles, 32 at a time.  grid = (nb, U, ceil(max points per block / 32)): the list position is the
// slowest grid dimension, so that the few workgroups that have work (short lists) are neighbours
// in dispatch order and spread over the whole chip; the others leave at once.
constexpr int kExactPts = 32;
__global__ __launch_bounds__(256) void assign_exact_list_kernel(const uint16_t* __restrict__ X, long long x_unit_rows,
                                                                const int32_t* __restrict__ blocks,
                                                                const uint16_t* __restrict__ C, long long c_unit_rows,
                                                                int32_t* __restrict__ assign, long long assign_stride,
                                                                const int32_t* __restrict__ amb_list, long long list_stride,
                                                                const int32_t* __restrict__ amb_cnt, int cnt_stride)
{
    __shared__ double ct[kTile * kHeadDim];
    __shared__ double part_d[8][kExactPts];
    __shared__ int part_j[8][kExactPts];
    const int b = blockIdx.x, u = blockIdx.y;
    const int x0 = blocks[4 * b + 0], x1 = blocks[4 * b + 1], k0 = blocks[4 * b + 2], k1 = blocks[4 * b + 3];
    int n = amb_cnt[u * cnt_stride + b];
    if (n > x1 - x0) n = x1 - x0;
    const int e0 = (int)blockIdx.z * kExactPts;
    if (e0 >= n) return;
    const int pt = threadIdx.x & (kExactPts - 1), slice = threadIdx.x / kExactPts;
    const bool live = e0 + pt < n;
    const int t = amb_list[u * list_stride + x0 + (live ? e0 + pt : e0)];
    float x[kHeadDim];
    {
        const uint4* xp = reinterpret_cast<const uint4*>(X + ((long long)u * x_unit_rows + t) * kHeadDim);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint4 w = xp[i];
            x[8 * i + 0] = bf16lo_to_f32(w.x); x[8 * i + 1] = bf16hi_to_f32(w.x);
            x[8 * i + 2] = bf16lo_to_f32(w.y); x[8 * i + 3] = bf16hi_to_f32(w.y);
            x[8 * i + 4] = bf16lo_to_f32(w.z); x[8 * i + 5] = bf16hi_to_f32(w.z);
            x[8 * i + 6] = bf16lo_to_f32(w.w); x[8 * i + 7] = bf16hi_to_f32(w.w);
        }
    }
    double best = INFINITY;
    int bj = k0;
    for (int j0 = k0; j0 < k1; j0 += kTile) {
        const int nj = (k1 - j0 < kTile) ? k1 - j0 : kTile;
        __syncthreads();
        for (int e = threadIdx.x; e < nj * (kHeadDim / 2); e += 256) {
            const int j = e >> 6, w = e & 63;
            const uint32_t cw = reinterpret_cast<const uint32_t*>(C + ((long long)u * c_unit_rows + j0 + j) * kHeadDim)[w];
            ct[j * kHeadDim + 2 * w] = (double)bf16lo_to_f32(cw);
            ct[j * kHeadDim + 2 * w + 1] = (double)bf16hi_to_f32(cw);
        }
        __syncthreads();
        for (int j = slice; j < nj; j += 8) {
            double s = 0.0;
#pragma unroll
            for (int i = 0; i < kHeadDim; i += 2) {
                const double2 c2 = *reinterpret_cast<const double2*>(&ct[j * kHeadDim + i]);
                const double d0 = __dsub_rn((double)x[i], c2.x);
                const double d1 = __dsub_rn((double)x[i + 1], c2.y);
                s = __dadd_rn(s, __dmul_rn(d0, d0));
                s = __dadd_rn(s, __dmul_rn(d1, d1));
            }
            if (s < best) {
                best = s;
                bj = j0 + j;
            }
        }
    }
    part_d[slice][pt] = best;
    part_j[slice][pt] = bj;
    __syncthreads();
    if (slice == 0 && live) {
#pragma unroll
        for (int sl = 1; sl < 8; ++sl) {
            const double od = part_d[sl][pt];
            const int oj = part_j[sl][pt];
            if (od < best || (od == best && oj < bj)) {
                best = od;
                bj = oj;
            }
        }
        assign[u * assign_stride + t] = bj;
    }
}

}  // namespace

hipError_t launch_assign(const uint16_t* X, long long x_unit_rows, const int32_t* blocks_dev, int nb, int max_pts,
                         int U, const uint16_t* C, long long c_unit_rows, int32_t* assign, long long assign_stride,
                         int32_t* amb_list, long long list_stride, int32_t* amb_cnt, int cnt_stride, hipStream_t s)
{
    if (nb <= 0 || max_pts <= 0 || U <= 0) return hipSuccess;
    if (nb > cnt_stride || U > 65535 || (max_pts + kExactPts - 1) / kExactPts > 65535) return hipErrorInvalidValue;
    hipError_t e = launch_fill_i32(amb_cnt, (long long)U * cnt_stride, 0, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(assign_mfma_kernel, dim3((max_pts + 127) / 128, nb, U), dim3(256), 0, s, X, x_unit_rows,
                       blocks_dev, C, c_unit_rows, assign, assign_stride, amb_list, list_stride, amb_cnt, cnt_stride);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(assign_exact_list_kernel, dim3(nb, U, (max_pts + kExactPts - 1) / kExactPts), dim3(256), 0, s, X, x_unit_rows,
                       blocks_dev, C, c_unit_rows, assign, assign_stride, amb_list, list_stride, amb_cnt, cnt_stride);
    return hipGetLastError();
}

}  // namespace mp
