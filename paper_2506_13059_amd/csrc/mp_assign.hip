// Nearest-centroid assignment of k-means on the keys (Sec. 3.1: assignment step of Lloyd's iterations;
// Sec. 3.3: run inside each block of the sequence, and as the one-shot assignment of appended tokens).
//
// The result is defined in fp64: a[t] = argmin_j sum_i (x_t[i] - c_j[i])^2 with the sum taken in
// index order and the lowest j among equal distances.  Points and centroids are bf16 values, so the
// bulk of the work is a bf16 contraction and runs on the matrix cores; fp64 is only spent where it
// can change the answer:
//
//   1. assign_mfma_kernel: s[t,j] = x_t.c_j - |c_j|^2/2 (argmax = nearest centroid) with
//      v_mfma_f32_32x32x16_bf16, fp32 accumulation.  The offset -|c_j|^2/2 is part of the
//      contraction: split exactly into three bf16 values, it sits in three extra slots of the
//      reduction dimension against ones on the point side, so the scores leave the matrix cores
//      complete.  Per point the kernel keeps the best and the second best score.  The products
//      are exact and every one of the 131 accumulation steps loses at most one unit in the last
//      place of a partial sum bounded by max(|x||c|, |c|^2/2), so each score is within
//      2^-16 max(|x|^2, max_j |c_j|^2) of its exact value (2^-19 more for four mantissa bits that
//      carry an index during the comparison).  A point whose two best scores are
//      further apart than 2^-14 of that scale has a unique nearest centroid in exact arithmetic
//      too (and by far more than fp64 rounding), which is the fp64 answer.
//   2. Every other point (near-equal or equal distances) goes onto a per-block list and
//      assign_recheck_kernel decides it exactly as defined above: it collects the centroids whose
//      score is within the same margin of the best one and evaluates their distances in fp64
//      without fused multiply-adds.
#include <algorithm>

#include "mp_device.h"
#include "mp_internal.h"

namespace mp {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kTile = 32;                 // centroids per tile = rows of the MFMA A operand
constexpr int kRowBytes = 256 + 16;       // LDS row of one centroid: 128 dims, then -|c|^2/2 as three bf16 and five zeros
constexpr float kMarginScale = 1.0f / 16384.0f;  // 2^-14: 1.8 times the sum of two scores' error bounds
constexpr float kNoCentroid = -3.0e38f;          // score of a padded row (finite: index bits are packed into scores)

// Scores of 32 centroids (one LDS tile: rows of kRowBytes, -|c|^2/2 in three bf16 pieces behind the
// 128 dims) against this wave's 2 x 32 points, folded into the running best / second best of every
// point.  Accumulator rows of a lane: m(i) = 8 (i / 4) + 4 half + i % 4.  The slot i of a score
// inside the tile rides in its four lowest mantissa bits (a change of at most 2^-19 of its
// magnitude), so that a pair of scores costs one max3, one med3 and one max; the tile of the best
// score is noted per tile.
__device__ __forceinline__ void fold_scores(const f32x16_t (&acc)[2], int j0, float (&best)[2], float (&second)[2],
                                            int (&btile)[2])
{
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const float before = best[c];
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            const float va = __uint_as_float((__float_as_uint(acc[c][i]) & ~15u) | (uint32_t)i);
            const float vb = __uint_as_float((__float_as_uint(acc[c][i + 1]) & ~15u) | (uint32_t)(i + 1));
            second[c] = fmaxf(second[c], __builtin_amdgcn_fmed3f(best[c], va, vb));
            best[c] = fmaxf(fmaxf(va, vb), best[c]);
        }
        btile[c] = best[c] != before ? j0 : btile[c];
    }
}

// The nine operand fragments a lane takes from one tile: the offset slots, then dims [16 ks + 8 half, +8).
__device__ __forceinline__ void read_fragments(const unsigned char* tile, int col, int half, bf16x8_t (&f)[9])
{
    const unsigned char* row = tile + col * kRowBytes;
    f[8] = *reinterpret_cast<const bf16x8_t*>(row + 256);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) f[ks] = *reinterpret_cast<const bf16x8_t*>(row + 32 * ks + 16 * half);
}

__device__ __forceinline__ void multiply_tile(const bf16x8_t (&f)[9], const bf16x8_t (&xb)[2][8], bf16x8_t ones,
                                              bf16x8_t ones_too, f32x16_t (&acc)[2])
{
    const f32x16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[8], ones, zero, 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[8], ones_too, zero, 0, 0, 0);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[ks], xb[0][ks], acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[ks], xb[1][ks], acc[1], 0, 0, 0);
    }
}

__device__ __forceinline__ void tile_scores(const unsigned char* tile, int col, int half, const bf16x8_t (&xb)[2][8],
                                            bf16x8_t ones, bf16x8_t ones_too, int j0, float (&best)[2],
                                            float (&second)[2], int (&btile)[2])
{
    f32x16_t acc[2];
    {
        const f32x16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(tile + col * kRowBytes + 256);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, ones, zero, 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, ones_too, zero, 0, 0, 0);
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(tile + col * kRowBytes + 32 * ks + 16 * half);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xb[0][ks], acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xb[1][ks], acc[1], 0, 0, 0);
    }
    fold_scores(acc, j0, best, second, btile);
}

// One 16-byte piece of a centroid row goes to its place in an LDS tile; the 16 lanes that hold a
// row add up |c|^2 (exact products, a dozen fp32 roundings: at most 2^-20 of its value, far below
// the bound on a score), and the lane with the first piece writes -|c|^2/2 behind the row, split
// exactly into three bf16 values (24 significant bits in three pieces of 8).  Returns |c|^2.
__device__ __forceinline__ float deposit_piece(unsigned char* tile_row, int seg, uint4 w, bool exists)
{
    *reinterpret_cast<uint4*>(tile_row + seg * 16) = w;
    float s = dot2_bf16(w.x, w.x, 0.f);
    s = dot2_bf16(w.y, w.y, s);
    s = dot2_bf16(w.z, w.z, s);
    s = dot2_bf16(w.w, w.w, s);
    s = sum8(s);
    s += dpp_f32<kDppMirror>(s);      // the other 8 lanes of the row of 16
    if (seg == 0) {
        const float v = exists ? -0.5f * s : kNoCentroid;
        const uint32_t hi = __float_as_uint(v) & 0xffff0000u;
        const float r1 = v - __uint_as_float(hi);
        const uint32_t mid = __float_as_uint(r1) & 0xffff0000u;
        const uint32_t lo = __float_as_uint(r1 - __uint_as_float(mid)) & 0xffff0000u;
        *reinterpret_cast<uint4*>(tile_row + 256) = make_uint4((hi >> 16) | mid, lo >> 16, 0u, 0u);
    }
    return s;
}

// The two halves of a wave hold the other accumulator rows of the same points: combine them, write
// the stage-1 assignment, and list the point for the exact pass unless its two best scores are
// further apart than the margin.
__device__ __forceinline__ void finish_points(int half, const float (&best)[2], const float (&second)[2],
                                              const int (&btile)[2], const float (&x2)[2], const int (&tpt)[2], int x0,
                                              int x1, float c2max, int32_t* assign_u, int32_t* amb_list_u,
                                              int32_t* amb_cnt_ub)
{
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int slot = (int)(__float_as_uint(best[c]) & 15u);
        const int bj = btile[c] + 8 * (slot >> 2) + 4 * half + (slot & 3);
        const float ob = __shfl_xor(best[c], 32, 64), os = __shfl_xor(second[c], 32, 64);
        const int oj = __shfl_xor(bj, 32, 64);
        const float ox = __shfl_xor(x2[c], 32, 64);
        const float sec = fmaxf(fmaxf(second[c], os), fminf(best[c], ob));
        int j = bj;
        if (ob > best[c] || (ob == best[c] && oj < j)) j = oj;
        const float bst = fmaxf(best[c], ob);
        const float xx = x2[c] + ox;
        const int t = tpt[c];
        if (t < x1 && half == 0) {
            assign_u[t] = j;
            const float margin = kMarginScale * fmaxf(xx, c2max);
            // (written so that a point without any comparable score also goes to the exact pass)
            if (!(bst - sec > margin)) {
                const int pos = atomicAdd(amb_cnt_ub, 1);
                amb_list_u[x0 + pos] = t;
            }
        }
    }
}

// grid = (ceil(max points per block / 256), nb, U); 256 threads = 4 waves of 64 points (two MFMA
// column tiles that share every centroid fragment).  Centroid tiles are double-buffered in LDS; their
// rows are requested two tiles ahead and wait in registers until the buffer they go to is free.
// blocks: int32 [nb][4] = {first point, end point, first centroid, end centroid}.
// assign[u][t] receives the best centroid of stage 1; amb_list[u][first point + i], i < amb_cnt[u][b],
// the points of block b that stage 2 has to decide.
constexpr int kPtsPerWg = 256;
__global__ __launch_bounds__(256) void assign_mfma_kernel(const uint16_t* __restrict__ X, long long x_unit_rows,
                                                          const int32_t* __restrict__ blocks,
                                                          const uint16_t* __restrict__ C, long long c_unit_rows,
                                                          int32_t* __restrict__ assign, long long assign_stride,
                                                          int32_t* __restrict__ amb_list, long long list_stride,
                                                          int32_t* __restrict__ amb_cnt, int cnt_stride)
{
    __shared__ __align__(16) unsigned char tile[2][kTile * kRowBytes];
    __shared__ float wave_c2max[4];
    const int u = blockIdx.z, b = blockIdx.y;
    const int x0 = blocks[4 * b + 0], x1 = blocks[4 * b + 1], k0 = blocks[4 * b + 2], k1 = blocks[4 * b + 3];
    const int p0 = x0 + (int)blockIdx.x * kPtsPerWg;
    if (p0 >= x1) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;

    // B operands: this lane's two points, dims [16 ks + 8 half, +8) for ks = 0..7
    bf16x8_t xb[2][8];
    float x2[2];
    int tpt[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        tpt[c] = p0 + wave * 64 + 32 * c + col;
        const int tl = tpt[c] < x1 ? tpt[c] : x0;
        const uint4* xp = reinterpret_cast<const uint4*>(X + ((long long)u * x_unit_rows + tl) * kHeadDim);
        x2[c] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const uint4 w = xp[2 * ks + half];
            xb[c][ks] = __builtin_bit_cast(bf16x8_t, w);
            x2[c] = dot2_bf16(w.x, w.x, x2[c]);      // |x|^2 only scales the margin
            x2[c] = dot2_bf16(w.y, w.y, x2[c]);
            x2[c] = dot2_bf16(w.z, w.z, x2[c]);
            x2[c] = dot2_bf16(w.w, w.w, x2[c]);
        }
    }
    // point side of the three offset slots: ones in the slots of the lower half-wave, zeros elsewhere
    const bf16x8_t ones = __builtin_bit_cast(bf16x8_t, half == 0 ? make_uint4(0x3f803f80u, 0x00003f80u, 0u, 0u)
                                                                  : make_uint4(0u, 0u, 0u, 0u));
    bf16x8_t ones_too = ones;      // a second copy the compiler cannot see through: two multiplications
    asm volatile("" : "+v"(ones_too));   // on the otherwise idle matrix pipe instead of sixteen register moves
    // this thread's share of a centroid tile: two 16-byte pieces, 16 threads per row
    const uint16_t* Cu = C + (long long)u * c_unit_rows * kHeadDim;
    uint4 pre_a[2], pre_b[2];     // rows on their way to LDS: the next tile and the one after it
    float c2max = 0.f;
    auto request = [&](int j0, uint4 (&pre)[2]) {
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int e = pass * 256 + tid;
            const int row = e >> 4, seg = e & 15;
            // always a load (of the last centroid when the row does not exist; deposit stores zeros for
            // it): the count of loads in flight is then the same on every path, which is what lets
            // the compiler wait for the older request only
            const int j = j0 + row < k1 ? j0 + row : k1 - 1;
            pre[pass] = reinterpret_cast<const uint4*>(Cu + (long long)j * kHeadDim)[seg];
        }
    };
    auto deposit = [&](int j0, int buf, const uint4 (&pre)[2]) {
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int e = pass * 256 + tid;
            const int row = e >> 4, seg = e & 15;
            const bool exists = j0 + row < k1;
            const uint4 w = exists ? pre[pass] : make_uint4(0, 0, 0, 0);
            c2max = fmaxf(c2max, deposit_piece(tile[buf] + row * kRowBytes, seg, w, exists));   // (absent rows are zeros)
        }
    };
    float best[2] = {-INFINITY, -INFINITY}, second[2] = {-INFINITY, -INFINITY};
    int btile[2] = {k0, k0};
    // Rows are requested two tiles ahead: a tile's multiplications take less time than a load from
    // L2 under the traffic of the other workgroups' point loads.
    request(k0, pre_a);
    request(k0 + kTile, pre_b);
    deposit(k0, 0, pre_a);
    __syncthreads();
    // one tile: `next` holds the rows of the following tile, `after` receives those of the one after it
    auto step = [&](int j0, int buf, uint4 (&after)[2], const uint4 (&next)[2]) {
        const bool more = j0 + kTile < k1;
        request(j0 + 2 * kTile, after);
        __builtin_amdgcn_sched_barrier(0);      // (the compiler would sink the loads below the multiplications)
        tile_scores(tile[buf], col, half, xb, ones, ones_too, j0, best, second, btile);
        if (more) deposit(j0 + kTile, buf ^ 1, next);
        __syncthreads();
    };
    // (two tiles per trip, so that the two register sets swap roles without being copied: a copy
    // would have to wait for the load)
    for (int j0 = k0; j0 < k1; j0 += 2 * kTile) {
        step(j0, 0, pre_a, pre_b);
        if (j0 + kTile < k1) step(j0 + kTile, 1, pre_b, pre_a);
    }
    // largest |c|^2 of the block: every thread saw the rows it deposited
    c2max = wave_max_f32(c2max);
    if (lane == 0) wave_c2max[wave] = c2max;
    __syncthreads();
    c2max = fmaxf(fmaxf(wave_c2max[0], wave_c2max[1]), fmaxf(wave_c2max[2], wave_c2max[3]));
    finish_points(half, best, second, btile, x2, tpt, x0, x1, c2max, assign + u * assign_stride,
                  amb_list + u * list_stride, amb_cnt + u * cnt_stride + b);
}

// The same stage for blocks of at most kResidentK centroids (every blockwise build with one centroid
// per 32 tokens and blocks of 8192): all centroids of the block stay in LDS, a workgroup walks
// several chunks of 256 points of its (block, unit), and the points of the next chunk are on their
// way from memory while the current ones are multiplied.  No barrier after the centroids are in
// place.  grid = (workgroups per (block, unit), nb, U), dynamic LDS = kResidentK rows.
constexpr int kResidentK = 256;
__global__ __launch_bounds__(256) void assign_resident_kernel(const uint16_t* __restrict__ X, long long x_unit_rows,
                                                              const int32_t* __restrict__ blocks,
                                                              const uint16_t* __restrict__ C, long long c_unit_rows,
                                                              int32_t* __restrict__ assign, long long assign_stride,
                                                              int32_t* __restrict__ amb_list, long long list_stride,
                                                              int32_t* __restrict__ amb_cnt, int cnt_stride)
{
    extern __shared__ __align__(16) unsigned char ctile[];      // [kResidentK][kRowBytes]
    __shared__ float wave_c2max[4];
    const int u = blockIdx.z, b = blockIdx.y;
    const int x0 = blocks[4 * b + 0], x1 = blocks[4 * b + 1], k0 = blocks[4 * b + 2];
    const int k1 = min(blocks[4 * b + 3], k0 + kResidentK);     // (the launch guarantees the block has no more)
    const int n_chunks = (x1 - x0 + kPtsPerWg - 1) / kPtsPerWg;
    int chunk = blockIdx.x;
    if (chunk >= n_chunks) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const uint16_t* Xu = X + (long long)u * x_unit_rows * kHeadDim;

    bf16x8_t xb[2][8], xn[2][8];
    auto load_points = [&](int ch, bf16x8_t (&dst)[2][8]) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int t = x0 + ch * kPtsPerWg + wave * 64 + 32 * c + col;
            const uint4* xp = reinterpret_cast<const uint4*>(Xu + (long long)(t < x1 ? t : x0) * kHeadDim);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) dst[c][ks] = __builtin_bit_cast(bf16x8_t, xp[2 * ks + half]);
        }
    };
    load_points(chunk, xb);

    // ---- the block's centroids: 16 lanes per row, rows past the last centroid are zeros that can never win ----
    const int ntiles = (k1 - k0 + kTile - 1) / kTile;
    float c2max = 0.f;
    {
        const uint16_t* Cu = C + (long long)u * c_unit_rows * kHeadDim;
        for (int e = tid; e < ntiles * kTile * 16; e += 256) {
            const int row = e >> 4, seg = e & 15;
            const bool exists = k0 + row < k1;
            uint4 w = make_uint4(0, 0, 0, 0);
            if (exists) w = reinterpret_cast<const uint4*>(Cu + (long long)(k0 + row) * kHeadDim)[seg];
            c2max = fmaxf(c2max, deposit_piece(ctile + row * kRowBytes, seg, w, exists));
        }
    }
    c2max = wave_max_f32(c2max);
    if (lane == 0) wave_c2max[wave] = c2max;
    __syncthreads();
    c2max = fmaxf(fmaxf(wave_c2max[0], wave_c2max[1]), fmaxf(wave_c2max[2], wave_c2max[3]));

    const bf16x8_t ones = __builtin_bit_cast(bf16x8_t, half == 0 ? make_uint4(0x3f803f80u, 0x00003f80u, 0u, 0u)
                                                                  : make_uint4(0u, 0u, 0u, 0u));
    bf16x8_t ones_too = ones;
    asm volatile("" : "+v"(ones_too));
    while (true) {
        const int next = chunk + (int)gridDim.x;
        const bool has_next = next < n_chunks;
        if (has_next) load_points(next, xn);
        float x2[2] = {0.f, 0.f};
        int tpt[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            tpt[c] = x0 + chunk * kPtsPerWg + wave * 64 + 32 * c + col;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const uint4 w = __builtin_bit_cast(uint4, xb[c][ks]);
                x2[c] = dot2_bf16(w.x, w.x, x2[c]);      // |x|^2 only scales the margin
                x2[c] = dot2_bf16(w.y, w.y, x2[c]);
                x2[c] = dot2_bf16(w.z, w.z, x2[c]);
                x2[c] = dot2_bf16(w.w, w.w, x2[c]);
            }
        }
        float best[2] = {-INFINITY, -INFINITY}, second[2] = {-INFINITY, -INFINITY};
        int btile[2] = {k0, k0};
        // The comparison of one tile's scores runs while the next tile is multiplied: two accumulator
        // sets, and an instruction order that puts a few comparison instructions behind every pair of
        // matrix instructions (a matrix instruction waits for its predecessor on the same accumulators
        // anyway) and keeps one LDS read in flight.
        auto multiply_and_fold = [&](int t, f32x16_t (&cur)[2], const f32x16_t (&prev)[2]) {
            bf16x8_t f[9];
            read_fragments(ctile + t * kTile * kRowBytes, col, half, f);
            multiply_tile(f, xb, ones, ones_too, cur);
            fold_scores(prev, k0 + (t - 1) * kTile, best, second, btile);
            // order: fragment reads run one step ahead of the pair of matrix instructions that use them,
            // eight comparison instructions follow every pair
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
            for (int q = 0; q < 9; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);     // two matrix instructions
                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);     // eight vector instructions
                if (q < 7) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // the read after next
            }
        };
        f32x16_t acc_a[2], acc_b[2];
        {
            bf16x8_t f[9];
            read_fragments(ctile, col, half, f);
            multiply_tile(f, xb, ones, ones_too, acc_a);
        }
        for (int t = 1; t < ntiles; t += 2) {
            multiply_and_fold(t, acc_b, acc_a);
            if (t + 1 < ntiles) multiply_and_fold(t + 1, acc_a, acc_b);
        }
        if (ntiles & 1) fold_scores(acc_a, k0 + (ntiles - 1) * kTile, best, second, btile);
        else fold_scores(acc_b, k0 + (ntiles - 1) * kTile, best, second, btile);
        finish_points(half, best, second, btile, x2, tpt, x0, x1, c2max, assign + u * assign_stride,
                      amb_list + u * list_stride, amb_cnt + u * cnt_stride + b);
        if (!has_next) break;
        for (int c = 0; c < 2; ++c)
            for (int ks = 0; ks < 8; ++ks) xb[c][ks] = xn[c][ks];
        chunk = next;
    }
}

// Stage 2.  One wave per listed point, three passes over the block's centroids:
//   1. fp32 scores s_j = x.c_j - |c_j|^2/2 again (8 lanes per centroid, 16 dims each, sequential
//      fused multiply-adds: error far below the bound of stage 1), their maximum and max_j |c_j|^2;
//   2. every centroid whose score (kept in LDS, or computed once more for blocks with more than
//      kScoreCache centroids) is within the margin of the maximum is a candidate: the nearest
//      centroid in exact arithmetic, and everything tied with it, is among them;
//   3. the candidates' distances exactly as defined, one lane per candidate, fp64, no fused
//      multiply-adds, sum in index order; smallest distance wins, equal distances -> lowest index.
// More than kCandCap candidates (many coinciding centroids): every centroid is treated as one.
// grid = (nb, U, Z): the waves of a (block, unit) walk its list with stride 4 Z.  The list position
// is the slowest grid dimension, so that the few workgroups that have work are neighbours in
// dispatch order and spread over the whole chip.
constexpr int kCandCap = 64;
constexpr int kScoreCache = 2048;     // scores of pass 1 kept in LDS for pass 2 when the block has no more centroids

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// |x - c|^2 in fp64, dims in index order, rounding after every operation
__device__ __forceinline__ double exact_distance(const uint16_t* xrow /*LDS*/, const uint16_t* crow /*global*/)
{
    double s = 0.0;
    const uint4* cp = reinterpret_cast<const uint4*>(crow);
    const uint4* xp = reinterpret_cast<const uint4*>(xrow);
#pragma unroll 2
    for (int i = 0; i < 16; ++i) {
        const uint4 cw = cp[i], xw = xp[i];
        const uint32_t c4[4] = {cw.x, cw.y, cw.z, cw.w}, x4[4] = {xw.x, xw.y, xw.z, xw.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const double d0 = __dsub_rn((double)bf16lo_to_f32(x4[e]), (double)bf16lo_to_f32(c4[e]));
            const double d1 = __dsub_rn((double)bf16hi_to_f32(x4[e]), (double)bf16hi_to_f32(c4[e]));
            s = __dadd_rn(s, __dmul_rn(d0, d0));
            s = __dadd_rn(s, __dmul_rn(d1, d1));
        }
    }
    return s;
}

__global__ __launch_bounds__(256) void assign_recheck_kernel(const uint16_t* __restrict__ X, long long x_unit_rows,
                                                             const int32_t* __restrict__ blocks,
                                                             const uint16_t* __restrict__ C, long long c_unit_rows,
                                                             int32_t* __restrict__ assign, long long assign_stride,
                                                             const int32_t* __restrict__ amb_list, long long list_stride,
                                                             const int32_t* __restrict__ amb_cnt, int cnt_stride,
                                                             int32_t* __restrict__ cnt_next)
{
    __shared__ __align__(16) uint16_t xrow[4][kHeadDim];
    __shared__ int cand[4][kCandCap];
    __shared__ int ncand[4];
    __shared__ float sc_cache[4][kScoreCache];
    const int b = blockIdx.x, u = blockIdx.y;
    // the counters the next assignment step will count into (nobody reads them in this launch): all of the unit's
    if (b == 0 && blockIdx.z == 0)
        for (int i = threadIdx.x; i < cnt_stride; i += blockDim.x) cnt_next[u * cnt_stride + i] = 0;
    const int x0 = blocks[4 * b + 0], x1 = blocks[4 * b + 1], k0 = blocks[4 * b + 2], k1 = blocks[4 * b + 3];
    int n = amb_cnt[u * cnt_stride + b];
    if (n > x1 - x0) n = x1 - x0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 7, grp = lane >> 3;
    const uint16_t* Cu = C + (long long)u * c_unit_rows * kHeadDim;
    for (int e = (int)blockIdx.z * 4 + wave; e < n; e += (int)gridDim.z * 4) {
        const int t = amb_list[u * list_stride + x0 + e];
        const uint16_t* xg = X + ((long long)u * x_unit_rows + t) * kHeadDim;
        float xs[16];
        float x2 = 0.f;
        {
            const uint4 a = reinterpret_cast<const uint4*>(xg)[2 * sub], bq = reinterpret_cast<const uint4*>(xg)[2 * sub + 1];
            if (grp == 0) {
                reinterpret_cast<uint4*>(xrow[wave])[2 * sub] = a;
                reinterpret_cast<uint4*>(xrow[wave])[2 * sub + 1] = bq;
            }
            const uint32_t w[8] = {a.x, a.y, a.z, a.w, bq.x, bq.y, bq.z, bq.w};
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                xs[2 * q] = bf16lo_to_f32(w[q]);
                xs[2 * q + 1] = bf16hi_to_f32(w[q]);
                x2 = fmaf(xs[2 * q], xs[2 * q], x2);
                x2 = fmaf(xs[2 * q + 1], xs[2 * q + 1], x2);
            }
            x2 = sum8(x2);
        }
        // s_j and |c_j|^2 of four centroids j, j+8, j+16, j+24 by the 8 lanes of a group (every lane of
        // the group gets them); all eight row loads are issued before the first is used
        auto scores4 = [&](int j, float (&sc)[4], float (&cc)[4]) {
            uint4 a[4], bq[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int jr = (j + 8 * r < k1) ? j + 8 * r : k1 - 1;
                const uint4* cp = reinterpret_cast<const uint4*>(Cu + (long long)jr * kHeadDim);
                a[r] = cp[2 * sub];
                bq[r] = cp[2 * sub + 1];
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t w[8] = {a[r].x, a[r].y, a[r].z, a[r].w, bq[r].x, bq[r].y, bq[r].z, bq[r].w};
                float dot = 0.f, c2 = 0.f;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const float lo = bf16lo_to_f32(w[q]), hi = bf16hi_to_f32(w[q]);
                    dot = fmaf(xs[2 * q], lo, dot);
                    dot = fmaf(xs[2 * q + 1], hi, dot);
                    c2 = fmaf(lo, lo, c2);
                    c2 = fmaf(hi, hi, c2);
                }
                dot = sum8(dot);
                c2 = sum8(c2);
                cc[r] = c2;
                sc[r] = (j + 8 * r < k1) ? fmaf(-0.5f, c2, dot) : -INFINITY;
            }
        };
        const bool cached = k1 - k0 <= kScoreCache;
        float best = -INFINITY, c2max = 0.f;
        for (int j = k0 + grp; j < k1; j += 32) {
            float sc[4], cc[4];
            scores4(j, sc, cc);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                best = fmaxf(best, sc[r]);
                c2max = fmaxf(c2max, cc[r]);        // (a clamped row repeats a real one)
                if (cached && sub == 0 && j + 8 * r < k1) sc_cache[wave][j + 8 * r - k0] = sc[r];
            }
        }
        best = wave_max_f32(best);
        c2max = wave_max_f32(c2max);
        const float thr = best - kMarginScale * fmaxf(x2, c2max);
        if (lane == 0) ncand[wave] = 0;
        wave_lds_sync();
        auto consider = [&](int j, float sc) {
            if (!(sc < thr)) {                       // also true for NaN
                const int pos = atomicAdd(&ncand[wave], 1);
                if (pos < kCandCap) cand[wave][pos] = j;
            }
        };
        if (cached) {
            for (int j = k0 + lane; j < k1; j += 64) consider(j, sc_cache[wave][j - k0]);
        } else {
            for (int j = k0 + grp; j < k1; j += 32) {
                float sc[4], cc[4];
                scores4(j, sc, cc);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (sub == 0 && j + 8 * r < k1) consider(j + 8 * r, sc[r]);
            }
        }
        wave_lds_sync();
        const int nc = ncand[wave];
        double bd = INFINITY;
        int bj = k0;
        if (nc <= kCandCap) {
            if (lane < nc) {
                const int j = cand[wave][lane];
                const double d = exact_distance(xrow[wave], Cu + (long long)j * kHeadDim);
                if (d < bd) { bd = d; bj = j; }
            }
        } else {
            for (int j = k0 + lane; j < k1; j += 64) {
                const double d = exact_distance(xrow[wave], Cu + (long long)j * kHeadDim);
                if (d < bd) { bd = d; bj = j; }
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const double od = __shfl_xor(bd, off, 64);
            const int oj = __shfl_xor(bj, off, 64);
            if (od < bd || (od == bd && oj < bj)) { bd = od; bj = oj; }
        }
        if (lane == 0) assign[u * assign_stride + t] = bj;
        wave_lds_sync();       // xrow / cand are reused by the next point
    }
}

}  // namespace

hipError_t launch_assign(const uint16_t* X, long long x_unit_rows, const int32_t* blocks_dev, int nb, int max_pts,
                         int max_k, int U, const uint16_t* C, long long c_unit_rows, int32_t* assign,
                         long long assign_stride, int32_t* amb_list, long long list_stride, int32_t* amb_cnt,
                         int32_t* amb_cnt_next, int cnt_stride, hipStream_t s)
{
    if (nb <= 0 || max_pts <= 0 || U <= 0) return hipSuccess;
    if (nb > cnt_stride || U > 65535) return hipErrorInvalidValue;
    hipError_t e = hipSuccess;
    const int n_chunks = (max_pts + kPtsPerWg - 1) / kPtsPerWg;
    if (max_k > 0 && max_k <= kResidentK && n_chunks >= 4) {
        // enough workgroups to fill the chip, several chunks each where the blocks are long enough
        static bool configured = false;
        const int smem = kResidentK * kRowBytes;
        if (!configured) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&assign_resident_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (e != hipSuccess) return e;
            configured = true;
        }
        const long long groups = (long long)nb * U;
        const int gx = (int)std::min<long long>(n_chunks, std::max<long long>(4, (1024 + groups - 1) / groups));
        hipLaunchKernelGGL(assign_resident_kernel, dim3(gx, nb, U), dim3(256), smem, s, X, x_unit_rows, blocks_dev, C,
                           c_unit_rows, assign, assign_stride, amb_list, list_stride, amb_cnt, cnt_stride);
    } else {
        hipLaunchKernelGGL(assign_mfma_kernel, dim3(n_chunks, nb, U), dim3(256), 0, s, X, x_unit_rows, blocks_dev, C,
                           c_unit_rows, assign, assign_stride, amb_list, list_stride, amb_cnt, cnt_stride);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int z = std::min(32, (max_pts + 3) / 4);      // (deeper grids only add workgroups that find nothing to do)
    hipLaunchKernelGGL(assign_recheck_kernel, dim3(nb, U, z), dim3(256), 0, s, X, x_unit_rows,
                       blocks_dev, C, c_unit_rows, assign, assign_stride, amb_list, list_stride, amb_cnt, cnt_stride,
                       amb_cnt_next);
    return hipGetLastError();
}

}  // namespace mp
