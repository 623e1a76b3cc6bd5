// k-means index construction (Sec. 3.1, 3.3, 3.4) and the online cluster update (Sec. 3.3):
// kernels that are specific to clustering, and the host-side sequencing of all clustering launches.
//
// A "problem" is a set of points X (bf16 rows), split into blocks; block b owns the points
// [x0,x1) and the clusters [k0,k1) (global ids).  Fine level: points = keys of the unit, blocks =
// the clustering blocks.  Coarse level: points = the fine k-means centroids, one block per
// clustering block.
//
// Assignment is decided in fp64 on the exact squared Euclidean distance, accumulated dimension by
// dimension without fused multiply-add, scanning centroids in ascending id with a strict "<":
// equal distances keep the lowest id.
#include <algorithm>
#include <vector>

#include "mp_ctx.h"
#include "mp_device.h"
#include "mp_internal.h"

namespace mp {

namespace {

// C[u][k] = X[u][x0(block of k) + seed[u][k]]   grid = (nb, U)
__global__ __launch_bounds__(256) void init_centroids_kernel(const uint16_t* __restrict__ X, long long x_unit_rows,
                                                             const int32_t* __restrict__ blocks,
                                                             const int32_t* __restrict__ seeds, long long seed_stride,
                                                             uint16_t* __restrict__ C, long long c_unit_rows)
{
    const int b = blockIdx.x, u = blockIdx.y;
    const int x0 = blocks[4 * b + 0], k0 = blocks[4 * b + 2], k1 = blocks[4 * b + 3];
    const int lane16 = threadIdx.x & 15;
    for (int k = k0 + (threadIdx.x >> 4); k < k1; k += 16) {
        const long long src = x0 + seeds[u * seed_stride + k];
        reinterpret_cast<uint4*>(C + ((long long)u * c_unit_rows + k) * kHeadDim)[lane16] =
            reinterpret_cast<const uint4*>(X + ((long long)u * x_unit_rows + src) * kHeadDim)[lane16];
    }
}

// Exact nearest-centroid assignment.  One thread per point, 256 points per workgroup; the block's
// centroids pass through LDS as doubles, 32 at a time.  grid = (ceil(max points per block/256), nb, U)
constexpr int kAssignTile = 32;
__global__ __launch_bounds__(256) void assign_exact_kernel(const uint16_t* __restrict__ X, long long x_unit_rows,
                                                           const int32_t* __restrict__ blocks,
                                                           const uint16_t* __restrict__ C, long long c_unit_rows,
                                                           int32_t* __restrict__ assign, long long assign_stride)
{
    __shared__ double ct[kAssignTile * kHeadDim];
    const int u = blockIdx.z, b = blockIdx.y;
    const int x0 = blocks[4 * b + 0], x1 = blocks[4 * b + 1], k0 = blocks[4 * b + 2], k1 = blocks[4 * b + 3];
    const int t = x0 + blockIdx.x * 256 + threadIdx.x;
    if (x0 + (int)blockIdx.x * 256 >= x1) return;
    const bool live = t < x1;
    float x[kHeadDim];
    {
        const uint4* xp = reinterpret_cast<const uint4*>(X + ((long long)u * x_unit_rows + (live ? t : x0)) * kHeadDim);
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
    for (int j0 = k0; j0 < k1; j0 += kAssignTile) {
        const int nj = (k1 - j0 < kAssignTile) ? k1 - j0 : kAssignTile;
        __syncthreads();
        for (int e = threadIdx.x; e < nj * (kHeadDim / 2); e += 256) {
            const int j = e >> 6, w = e & 63;
            const uint32_t cw = reinterpret_cast<const uint32_t*>(C + ((long long)u * c_unit_rows + j0 + j) * kHeadDim)[w];
            ct[j * kHeadDim + 2 * w] = (double)bf16lo_to_f32(cw);
            ct[j * kHeadDim + 2 * w + 1] = (double)bf16hi_to_f32(cw);
        }
        __syncthreads();
        for (int j = 0; j < nj; ++j) {
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
    if (live) assign[u * assign_stride + t] = bj;
}

// inv[u][perm[u][p]] = p for p in [0, n)
__global__ void invert_perm_kernel(const int32_t* __restrict__ perm, long long perm_stride, int n,
                                   int32_t* __restrict__ inv, long long inv_stride)
{
    const int u = blockIdx.y;
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) inv[u * inv_stride + perm[u * perm_stride + p]] = p;
}

// out[u][i] = map[u][in[u][i]]
__global__ void map_ids_kernel(const int32_t* __restrict__ in, long long in_stride, int n,
                               const int32_t* __restrict__ map, long long map_stride, int32_t* __restrict__ out,
                               long long out_stride)
{
    const int u = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[u * out_stride + i] = map[u * map_stride + in[u * in_stride + i]];
}

// dst[u][dst_row0 + p] = src[u][list ? list[u][p] : p]  (256-byte rows, one array)
__global__ void gather1_rows_kernel(const uint4* __restrict__ src, long long src_unit_rows,
                                    const int32_t* __restrict__ list, long long list_stride, int n,
                                    uint4* __restrict__ dst, long long dst_unit_rows, int dst_row0)
{
    const int u = blockIdx.y;
    const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long p = g >> 4;
    const int c = (int)(g & 15);
    if (p >= n) return;
    const long long s = list ? list[u * list_stride + p] : p;
    dst[((long long)u * dst_unit_rows + dst_row0 + p) * 16 + c] = src[((long long)u * src_unit_rows + s) * 16 + c];
}

#define MP_HIPC(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) return fail(ctx, MP_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

struct Problem {
    const uint16_t* X;
    long long x_unit_rows;
    int n_points;                 // points per unit (all blocks)
    const int32_t* blocks_dev;    // [nb][4]
    int nb;
    int max_pts, max_k;           // per block
    int k_total;                  // clusters per unit (all blocks)
    uint16_t* C;                  // centroids, row = global cluster id
    long long c_unit_rows;
    int32_t* assign;              // [U, assign_stride] global cluster id of each point
    long long assign_stride;
    int32_t* list;                // [U, list_stride] member lists
    long long list_stride;
    int32_t* cnt;                 // [U, cnt_stride]
    int32_t* start;               // [U, cnt_stride + 1]
    long long cnt_stride;
};

// One Lloyd iteration: assign, member lists, centroid <- bf16(mean of members); empty keeps.
mp_status lloyd_iteration(mp_ctx* ctx, const Problem& pr, hipStream_t s)
{
    const int U = ctx->U;
    hipLaunchKernelGGL(assign_exact_kernel, dim3((pr.max_pts + 255) / 256, pr.nb, U), dim3(256), 0, s, pr.X,
                       pr.x_unit_rows, pr.blocks_dev, pr.C, pr.c_unit_rows, pr.assign, pr.assign_stride);
    MP_HIPC(hipGetLastError());
    MP_HIPC(launch_fill_i32(pr.cnt, (long long)U * pr.cnt_stride, 0, s));
    MP_HIPC(launch_histogram(pr.assign, pr.assign_stride, pr.n_points, U, pr.cnt, pr.cnt_stride, s));
    MP_HIPC(launch_exclusive_scan(pr.cnt, pr.cnt_stride, pr.k_total, U, pr.start, pr.cnt_stride + 1, s));
    MP_HIPC(launch_member_lists(pr.assign, pr.assign_stride, pr.blocks_dev, pr.nb, pr.max_k, U, pr.start,
                                pr.cnt_stride + 1, pr.list, pr.list_stride, s));
    MP_HIPC(launch_cluster_means(pr.X, pr.x_unit_rows, pr.list, pr.list_stride, pr.start, pr.cnt_stride + 1,
                                 pr.k_total, U, pr.C, pr.c_unit_rows, 0, pr.C, pr.c_unit_rows, nullptr, 0, 0, s));
    return MP_OK;
}

// splitmix64: the documented generator behind seeds drawn from a 64-bit seed
inline uint64_t splitmix64(uint64_t& x)
{
    uint64_t z = (x += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}

// k distinct integers of [0, n): partial Fisher-Yates driven by splitmix64(seed)
void draw_distinct(uint64_t seed, int n, int k, int32_t* out)
{
    std::vector<int32_t> idx((size_t)n);
    for (int i = 0; i < n; ++i) idx[i] = i;
    uint64_t st = seed;
    for (int i = 0; i < k; ++i) {
        const int j = i + (int)(splitmix64(st) % (uint64_t)(n - i));
        std::swap(idx[i], idx[j]);
        out[i] = idx[i];
    }
}

}  // namespace

mp_status cluster_kv_impl(mp_ctx* ctx, const void* k, const void* v, int32_t n_tokens, int32_t n_fine,
                          int32_t n_coarse, int32_t iters, uint64_t seed, const int32_t* init_fine,
                          const int32_t* init_coarse, hipStream_t s)
{
    const int U = ctx->U;
    const bool two = ctx->cfg.levels == 2;
    const std::vector<BlockPlan> blocks = plan_blocks(n_tokens, ctx->cfg.block_w, ctx->cfg.block_alpha, n_fine, n_coarse);
    const int nb = (int)blocks.size();

    // seeds: explicit, or drawn per (unit, block) from the 64-bit seed
    std::vector<int32_t>& gen_f = ctx->stage_seed_f;
    std::vector<int32_t>& gen_c = ctx->stage_seed_c;
    if (!init_fine) {
        gen_f.resize((size_t)U * n_fine);
        for (int u = 0; u < U; ++u)
            for (int b = 0; b < nb; ++b)
                draw_distinct(seed ^ (0x51ed270b0ull + (uint64_t)u * 1000003ull + (uint64_t)b * 2ull), blocks[b].t1 - blocks[b].t0,
                              blocks[b].f1 - blocks[b].f0, gen_f.data() + (size_t)u * n_fine + blocks[b].f0);
        init_fine = gen_f.data();
    }
    if (two && !init_coarse) {
        gen_c.resize((size_t)U * n_coarse);
        for (int u = 0; u < U; ++u)
            for (int b = 0; b < nb; ++b)
                draw_distinct(seed ^ (0x51ed270b0ull + (uint64_t)u * 1000003ull + (uint64_t)b * 2ull + 1ull),
                              blocks[b].f1 - blocks[b].f0, blocks[b].c1 - blocks[b].c0,
                              gen_c.data() + (size_t)u * n_coarse + blocks[b].c0);
        init_coarse = gen_c.data();
    }
    MP_HIPC(hipMemcpy2DAsync(ctx->km_seed_f, (size_t)ctx->Fcap * 4, init_fine, (size_t)n_fine * 4, (size_t)n_fine * 4, U,
                             hipMemcpyHostToDevice, s));
    if (two)
        MP_HIPC(hipMemcpy2DAsync(ctx->km_seed_c, (size_t)std::max(ctx->Ccap, 1) * 4, init_coarse, (size_t)n_coarse * 4,
                                 (size_t)n_coarse * 4, U, hipMemcpyHostToDevice, s));

    // block descriptors: [0] fine problem, [1] coarse problem
    std::vector<int32_t>& bd = ctx->stage_blocks2;
    bd.assign(8 * (size_t)ctx->max_blocks, 0);
    int max_pts = 0, max_kf = 0, max_kc = 0;
    for (int b = 0; b < nb; ++b) {
        const BlockPlan& p = blocks[b];
        int32_t* f = &bd[4 * b];
        f[0] = p.t0; f[1] = p.t1; f[2] = p.f0; f[3] = p.f1;
        int32_t* c = &bd[4 * (size_t)ctx->max_blocks + 4 * b];
        c[0] = p.f0; c[1] = p.f1; c[2] = p.c0; c[3] = p.c1;
        max_pts = std::max(max_pts, p.t1 - p.t0);
        max_kf = std::max(max_kf, p.f1 - p.f0);
        max_kc = std::max(max_kc, p.c1 - p.c0);
    }
    int32_t* bdev_f = ctx->blocks_dev + 4 * (size_t)ctx->max_blocks;          // slot 1
    int32_t* bdev_c = ctx->blocks_dev + 8 * (size_t)ctx->max_blocks;          // slot 2
    MP_HIPC(hipMemcpyAsync(bdev_f, bd.data(), bd.size() * sizeof(int32_t), hipMemcpyHostToDevice, s));

    // ---- fine level ----
    Problem pf{};
    pf.X = (const uint16_t*)k; pf.x_unit_rows = n_tokens; pf.n_points = n_tokens; pf.blocks_dev = bdev_f; pf.nb = nb;
    pf.max_pts = max_pts; pf.max_k = max_kf; pf.k_total = n_fine; pf.C = ctx->km_Cf; pf.c_unit_rows = ctx->Fcap;
    pf.assign = ctx->km_assign; pf.assign_stride = ctx->Ncap; pf.list = ctx->km_list; pf.list_stride = ctx->Ncap;
    pf.cnt = ctx->km_cnt; pf.start = ctx->km_start; pf.cnt_stride = ctx->tab_rows;
    hipLaunchKernelGGL(init_centroids_kernel, dim3(nb, U), dim3(256), 0, s, pf.X, pf.x_unit_rows, pf.blocks_dev,
                       ctx->km_seed_f, (long long)ctx->Fcap, pf.C, pf.c_unit_rows);
    MP_HIPC(hipGetLastError());
    for (int it = 0; it < iters; ++it) {
        const mp_status st = lloyd_iteration(ctx, pf, s);
        if (st != MP_OK) return st;
    }

    if (two) {
        // ---- coarse level: k-means on the fine centroids ----
        Problem pc{};
        pc.X = ctx->km_Cf; pc.x_unit_rows = ctx->Fcap; pc.n_points = n_fine; pc.blocks_dev = bdev_c; pc.nb = nb;
        pc.max_pts = max_kf; pc.max_k = max_kc; pc.k_total = n_coarse; pc.C = ctx->km_Cc; pc.c_unit_rows = std::max(ctx->Ccap, 1);
        pc.assign = ctx->km_parent; pc.assign_stride = ctx->Fcap; pc.list = ctx->km_plist; pc.list_stride = ctx->Fcap;
        pc.cnt = ctx->km_cnt; pc.start = ctx->km_start; pc.cnt_stride = ctx->tab_rows;
        hipLaunchKernelGGL(init_centroids_kernel, dim3(nb, U), dim3(256), 0, s, pc.X, pc.x_unit_rows, pc.blocks_dev,
                           ctx->km_seed_c, (long long)std::max(ctx->Ccap, 1), pc.C, pc.c_unit_rows);
        MP_HIPC(hipGetLastError());
        for (int it = 0; it < iters; ++it) {
            const mp_status st = lloyd_iteration(ctx, pc, s);
            if (st != MP_OK) return st;
        }
        // km_plist = fine ids grouped by coarse cluster (ascending inside): the new fine numbering.
        hipLaunchKernelGGL(invert_perm_kernel, dim3((n_fine + 255) / 256, U), dim3(256), 0, s, ctx->km_plist,
                           (long long)ctx->Fcap, n_fine, ctx->km_newid, (long long)ctx->Fcap);
        MP_HIPC(hipGetLastError());
        // coarse id of each fine cluster in the new numbering; token ids in the new numbering
        hipLaunchKernelGGL(map_ids_kernel, dim3((n_fine + 255) / 256, U), dim3(256), 0, s, ctx->km_plist,
                           (long long)ctx->Fcap, n_fine, ctx->km_parent, (long long)ctx->Fcap, ctx->cof, (long long)ctx->Fcap);
        MP_HIPC(hipGetLastError());
        hipLaunchKernelGGL(map_ids_kernel, dim3((n_tokens + 255) / 256, U), dim3(256), 0, s, ctx->km_assign,
                           (long long)ctx->Ncap, n_tokens, ctx->km_newid, (long long)ctx->Fcap, ctx->fot, (long long)ctx->Ncap);
        MP_HIPC(hipGetLastError());
        // key centroids kept by empty clusters: the k-means centroids, in the new numbering
        hipLaunchKernelGGL(gather1_rows_kernel, dim3((unsigned)(((long long)n_fine * 16 + 255) / 256), U), dim3(256), 0, s,
                           (const uint4*)ctx->km_Cf, (long long)ctx->Fcap, ctx->km_plist, (long long)ctx->Fcap, n_fine,
                           (uint4*)ctx->Kc, ctx->tab_rows, 0);
        MP_HIPC(hipGetLastError());
        hipLaunchKernelGGL(gather1_rows_kernel, dim3((unsigned)(((long long)n_coarse * 16 + 255) / 256), U), dim3(256), 0, s,
                           (const uint4*)ctx->km_Cc, (long long)std::max(ctx->Ccap, 1), nullptr, 0, n_coarse, (uint4*)ctx->Kc,
                           ctx->tab_rows, ctx->Fcap);
        MP_HIPC(hipGetLastError());
    } else {
        MP_HIPC(hipMemcpy2DAsync(ctx->fot, (size_t)ctx->Ncap * 4, ctx->km_assign, (size_t)ctx->Ncap * 4, (size_t)n_tokens * 4, U,
                                 hipMemcpyDeviceToDevice, s));
        hipLaunchKernelGGL(gather1_rows_kernel, dim3((unsigned)(((long long)n_fine * 16 + 255) / 256), U), dim3(256), 0, s,
                           (const uint4*)ctx->km_Cf, (long long)ctx->Fcap, nullptr, 0, n_fine, (uint4*)ctx->Kc, ctx->tab_rows, 0);
        MP_HIPC(hipGetLastError());
    }
    return finalize_index(ctx, k, v, n_tokens, n_fine, n_coarse, blocks, true, s);
}

mp_status update_clusters_impl(mp_ctx* ctx, const void*, const void*, int32_t, int32_t, int32_t, int32_t, int32_t,
                               uint64_t, const int32_t*, hipStream_t)
{
    return fail(ctx, MP_ESTATE, "mp_update_clusters: not implemented yet");
}

}  // namespace mp
