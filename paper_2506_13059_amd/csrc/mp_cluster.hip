// k-means index construction (Sec. 3.1, 3.3, 3.4) and the online cluster update (Sec. 3.3):
// kernels that are specific to clustering, and the host-side sequencing of all clustering launches.
//
// A "problem" is a set of points X (bf16 rows), split into blocks; block b owns the points
// [x0,x1) and the clusters [k0,k1) (global ids).  Fine level: points = keys, blocks = the
// clustering blocks.  Coarse level: points = the fine k-means centroids, one block per clustering
// block.  The same code serves the full build (points = the caller's keys in sequence order) and
// the online update (points = the last block, kept in sequence order in Kfb / Vfb).
//
// Assignment is decided in fp64 on the exact squared Euclidean distance, accumulated dimension by
// dimension without fused multiply-add, scanning centroids in ascending id with a strict "<":
// equal distances keep the lowest id.
#include <algorithm>
#include <cstring>
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

// inv[u][perm[u][p0 + p]] = v0 + p for p in [0, n)
__global__ void invert_perm_kernel(const int32_t* __restrict__ perm, long long perm_stride, int p0, int n, int v0,
                                   int32_t* __restrict__ inv, long long inv_stride)
{
    const int u = blockIdx.y;
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) inv[u * inv_stride + perm[u * perm_stride + p0 + p]] = v0 + p;
}

// out[u][o0 + i] = map[u][in[u][i0 + i]] for i in [0, n)
__global__ void map_ids_kernel(const int32_t* __restrict__ in, long long in_stride, int i0, int n,
                               const int32_t* __restrict__ map, long long map_stride, int32_t* __restrict__ out,
                               long long out_stride, int o0)
{
    const int u = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[u * out_stride + o0 + i] = map[u * map_stride + in[u * in_stride + i0 + i]];
}

// dst[u][dst_row0 + p] = src[u][list ? list[u][list0 + p] : src_row0 + p]  (256-byte rows, one array)
__global__ void gather1_rows_kernel(const uint4* __restrict__ src, long long src_unit_rows, int src_row0,
                                    const int32_t* __restrict__ list, long long list_stride, int list0, int n,
                                    uint4* __restrict__ dst, long long dst_unit_rows, int dst_row0)
{
    const int u = blockIdx.y;
    const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long p = g >> 4;
    const int c = (int)(g & 15);
    if (p >= n) return;
    const long long s = list ? list[u * list_stride + list0 + p] : src_row0 + p;
    dst[((long long)u * dst_unit_rows + dst_row0 + p) * 16 + c] = src[((long long)u * src_unit_rows + s) * 16 + c];
}

// Running-mean move of the centroids touched by the one-shot assignment of the appended points
// (Sec. 3.3): c_j <- bf16((N_j c_j + sum of the appended points assigned to j, in sequence order)
// / (N_j + n_j)).  One wave per cluster j in [k0, k1); N_j = Nold[j] for j < k_old_end, else 0.
__global__ __launch_bounds__(256) void running_mean_kernel(const uint16_t* __restrict__ X, long long x_unit_rows,
                                                           int x0, int x1, const int32_t* __restrict__ assign,
                                                           long long assign_stride, int k0, int k1, int k_old_end,
                                                           const int32_t* __restrict__ Nold, long long n_stride,
                                                           uint16_t* __restrict__ C, long long c_unit_rows)
{
    const int u = blockIdx.y;
    const int j = k0 + blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (j >= k1) return;
    const long long nold = (j < k_old_end) ? Nold[u * n_stride + j] : 0;
    uint32_t* crow = reinterpret_cast<uint32_t*>(C + ((long long)u * c_unit_rows + j) * kHeadDim);
    const uint32_t cw = crow[lane];
    double s0 = (double)nold * (double)bf16lo_to_f32(cw), s1 = (double)nold * (double)bf16hi_to_f32(cw);
    const uint32_t* Xu = reinterpret_cast<const uint32_t*>(X + (long long)u * x_unit_rows * kHeadDim);
    int n = 0;
    for (int t0 = x0; t0 < x1; t0 += 64) {      // 64 appended points at a time: who of them belongs to j?
        const int t = t0 + lane;
        unsigned long long mine = __ballot(t < x1 && assign[u * assign_stride + t] == j);
        while (mine) {                           // ascending bit order = sequence order
            const int b = __ffsll((long long)mine) - 1;
            mine &= mine - 1;
            const uint32_t w = Xu[(long long)(t0 + b) * 64 + lane];
            s0 += (double)bf16lo_to_f32(w);
            s1 += (double)bf16hi_to_f32(w);
            ++n;
        }
    }
    if (n == 0) return;
    const double den = (double)(nold + n);
    crow[lane] = (uint32_t)f64_to_bf16_rne(s0 / den) | ((uint32_t)f64_to_bf16_rne(s1 / den) << 16);
}

#define MP_HIPC(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) return fail(ctx, MP_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

#define MP_TRY(expr)                       \
    do {                                   \
        const mp_status st_ = (expr);      \
        if (st_ != MP_OK) return st_;      \
    } while (0)

inline unsigned blocks_for(long long n, int per) { return (unsigned)((n + per - 1) / per); }

// Start of an entry point that uploads small host arrays: the pinned staging buffer may be reused
// once the copies of the previous call have been carried out.
mp_status stage_open(mp_ctx* ctx)
{
    if (ctx->pin_pending) {
        MP_HIPC(hipEventSynchronize(ctx->pin_ev));
        ctx->pin_pending = false;
    }
    ctx->pin_used = 0;
    ctx->n_up = 0;
    return MP_OK;
}

// Host -> device copy of `height` rows of `width` bytes.  What fits goes through the pinned staging
// buffer (packed there at once, so the caller's array is free again on return; the copy itself is
// asynchronous); larger arrays are copied directly from the caller's memory.
struct UploadBatch { mp_ctx::UploadSeg seg[mp_ctx::kMaxUploadSegs]; };

// grid = (word blocks, segments): row r of segment g goes from the pinned buffer to dst + r * dpitch.
__global__ void scatter_uploads_kernel(const char* __restrict__ pin, const UploadBatch b)
{
    const mp_ctx::UploadSeg sg = b.seg[blockIdx.y];
    const unsigned wpr = sg.width / 4;                                   // words per row
    const unsigned long long n = (unsigned long long)wpr * sg.height;
    for (unsigned long long i = (unsigned long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (unsigned long long)gridDim.x * blockDim.x) {
        const unsigned long long r = i / wpr, c = i - r * wpr;
        reinterpret_cast<uint32_t*>(static_cast<char*>(sg.dst) + r * sg.dpitch)[c] =
            reinterpret_cast<const uint32_t*>(pin + sg.src_off + r * sg.width)[c];
    }
}

// Carry out the uploads staged so far (before the first kernel that reads them is launched).
mp_status flush_uploads(mp_ctx* ctx, hipStream_t s)
{
    if (ctx->n_up == 0) return MP_OK;
    UploadBatch b{};
    unsigned long long most = 0;
    for (int i = 0; i < ctx->n_up; ++i) {
        b.seg[i] = ctx->up_seg[i];
        most = std::max<unsigned long long>(most, (unsigned long long)(b.seg[i].width / 4) * b.seg[i].height);
    }
    const unsigned gx = (unsigned)std::min<unsigned long long>(64, (most + 255) / 256);
    hipLaunchKernelGGL(scatter_uploads_kernel, dim3(std::max(gx, 1u), ctx->n_up), dim3(256), 0, s, ctx->pin, b);
    ctx->n_up = 0;
    MP_HIPC(hipGetLastError());
    MP_HIPC(hipEventRecord(ctx->pin_ev, s));
    ctx->pin_pending = true;
    return MP_OK;
}

// Stage a small host array (rows of `width` bytes, a multiple of 4) for the device; it arrives with the
// next flush_uploads.  What does not fit the pinned buffer is copied the ordinary way at once.
mp_status upload_2d(mp_ctx* ctx, void* dst, size_t dpitch, const void* src, size_t spitch, size_t width, size_t height,
                    hipStream_t s)
{
    if (width == 0 || height == 0) return MP_OK;
    const size_t bytes = width * height;
    if (ctx->pin && ctx->pin_used + bytes <= ctx->pin_bytes && width % 4 == 0 && dpitch % 4 == 0) {
        if (ctx->n_up == mp_ctx::kMaxUploadSegs) MP_TRY(flush_uploads(ctx, s));
        char* p = ctx->pin + ctx->pin_used;
        for (size_t r = 0; r < height; ++r) memcpy(p + r * width, (const char*)src + r * spitch, width);
        ctx->up_seg[ctx->n_up++] = mp_ctx::UploadSeg{dst, (unsigned long long)dpitch, (unsigned long long)ctx->pin_used,
                                                     (unsigned)width, (unsigned)height};
        ctx->pin_used += (bytes + 255) & ~(size_t)255;
    } else {
        MP_TRY(flush_uploads(ctx, s));      // (keeps the order of the writes)
        MP_HIPC(hipMemcpy2DAsync(dst, dpitch, src, spitch, width, height, hipMemcpyHostToDevice, s));
    }
    return MP_OK;
}
mp_status upload(mp_ctx* ctx, void* dst, const void* src, size_t bytes, hipStream_t s)
{
    return upload_2d(ctx, dst, bytes, src, bytes, bytes, 1, s);
}
struct Problem {
    const uint16_t* X;
    long long x_unit_rows;
    int n_points;                 // points per unit covered by the blocks (indices < n_points)
    const int32_t* blocks_dev;    // [nb][4]
    int nb;
    int max_pts, max_k;           // per block
    int k_total;                  // end of the cluster id range
    uint16_t* C;                  // centroids, row = global cluster id
    long long c_unit_rows;
    int32_t* assign;              // [U, assign_stride] global cluster id of each point
    long long assign_stride;
    int32_t* list;                // [U, list_stride] member lists
    long long list_stride;
    int32_t* cnt;                 // [U, cnt_stride]
    int32_t* start;               // [U, cnt_stride + 1]
    long long cnt_stride;
    int k_first;                  // first cluster id of the blocks
    int p_first;                  // first point index of the blocks
    double* sum_out;              // optional [U, sum_unit_rows, 128]: the fp64 member sums behind the new centroids
    long long sum_unit_rows;
};

// The counter array of the near-tie lists to use now (which = 0) and the one to leave zeroed for the next step (1).
inline int32_t* amb_counters(mp_ctx* ctx, int which)
{
    return ctx->km_amb + (size_t)((ctx->amb_turn ^ which) & 1) * ctx->U * ctx->max_blocks;
}

mp_status launch_assign(mp_ctx* ctx, const Problem& pr, hipStream_t s)
{
    // the member-list array is free during the assignment step and holds the points of the exact pass
    MP_HIPC(mp::launch_assign(pr.X, pr.x_unit_rows, pr.blocks_dev, pr.nb, pr.max_pts, pr.max_k, ctx->U, pr.C, pr.c_unit_rows,
                              pr.assign, pr.assign_stride, pr.list, pr.list_stride, amb_counters(ctx, 0), amb_counters(ctx, 1),
                              ctx->max_blocks, s));
    ctx->amb_turn ^= 1;
    return MP_OK;
}

// Member lists of the current assignment: cnt, start (positions relative to the first point), list.
mp_status build_lists(mp_ctx* ctx, const Problem& pr, hipStream_t s)
{
    const int U = ctx->U;
    MP_HIPC(launch_block_lists(pr.assign, pr.assign_stride, pr.blocks_dev, pr.nb, pr.max_k, pr.p_first, U, pr.start,
                               pr.cnt_stride + 1, pr.list, pr.list_stride, s));
    return MP_OK;
}

// One Lloyd iteration: assign, member lists, centroid <- bf16(mean of members); empty keeps.
// keep_sums: also store the member sums (pr.sum_out), which the coarse tables are built from when this was
// the last iteration.
mp_status lloyd_iteration(mp_ctx* ctx, const Problem& pr, bool keep_sums, hipStream_t s)
{
    mp_status st = launch_assign(ctx, pr, s);
    if (st != MP_OK) return st;
    st = build_lists(ctx, pr, s);
    if (st != MP_OK) return st;
    MP_HIPC(launch_cluster_means(pr.X, pr.x_unit_rows, pr.list, pr.list_stride, pr.start, pr.cnt_stride + 1,
                                 pr.k_first, pr.k_total, ctx->U, pr.C, pr.c_unit_rows, 0, pr.C, pr.c_unit_rows,
                                 nullptr, 0, 0, keep_sums ? pr.sum_out : nullptr, pr.sum_unit_rows, s));
    return MP_OK;
}

// splitmix64: the generator behind seeds drawn from a 64-bit seed
inline uint64_t splitmix64(uint64_t& x)
{
    uint64_t z = (x += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}

// k distinct integers of [0, n): partial Fisher-Yates driven by splitmix64(seed).  The identity
// array it shuffles is kept between calls and put back after each (only the 2k touched places), so
// a call costs O(k), not O(n): a build draws thousands of short lists from long ranges.
void draw_distinct(uint64_t seed, int n, int k, int32_t* out)
{
    static thread_local std::vector<int32_t> idx;
    if ((int)idx.size() < n) {
        const int old = (int)idx.size();
        idx.resize((size_t)n);
        for (int i = old; i < n; ++i) idx[i] = i;
    }
    uint64_t st = seed;
    for (int i = 0; i < k; ++i) {
        const int j = i + (int)(splitmix64(st) % (uint64_t)(n - i));
        std::swap(idx[i], idx[j]);
        out[i] = idx[i];
    }
    st = seed;
    for (int i = 0; i < k; ++i) {
        const int j = i + (int)(splitmix64(st) % (uint64_t)(n - i));
        idx[j] = j;
    }
    for (int i = 0; i < k; ++i) idx[i] = i;
}

bool distinct_in_range(const int32_t* v, int k, int n)
{
    std::vector<char> seen((size_t)std::max(n, 1), 0);
    for (int i = 0; i < k; ++i) {
        if (v[i] < 0 || v[i] >= n || seen[v[i]]) return false;
        seen[v[i]] = 1;
    }
    return true;
}

// A contiguous run of clustering blocks whose points live in X at local indices [0, n_pts).
struct Range {
    const uint16_t* Xk;             // keys the clusters are formed on (lookup keys when the context uses them)
    const uint16_t* Xs;             // keys to store and attend exactly (== Xk without lookup keys)
    const uint16_t* Xv;
    long long x_unit_rows;
    int pt0;                        // token / stored-row index of local point 0
    int n_pts;
    std::vector<BlockPlan> blocks;  // t0/t1 = LOCAL point ranges; f*/c* = global cluster ids
    int f0, f1, c0, c1;
};

void upload_descs(const Range& r, int max_blocks, std::vector<int32_t>& bd, int& max_pts, int& max_kf, int& max_kc)
{
    bd.assign(8 * (size_t)max_blocks, 0);
    max_pts = max_kf = max_kc = 0;
    for (size_t b = 0; b < r.blocks.size(); ++b) {
        const BlockPlan& p = r.blocks[b];
        int32_t* f = &bd[4 * b];
        f[0] = p.t0; f[1] = p.t1; f[2] = p.f0; f[3] = p.f1;
        int32_t* c = &bd[4 * (size_t)max_blocks + 4 * b];
        c[0] = p.f0; c[1] = p.f1; c[2] = p.c0; c[3] = p.c1;
        max_pts = std::max(max_pts, p.t1 - p.t0);
        max_kf = std::max(max_kf, p.f1 - p.f0);
        max_kc = std::max(max_kc, p.c1 - p.c0);
    }
}

}  // namespace

// Stored layout and tables of a range from: ids (final fine id of each local point), ctx->cof for
// [f0,f1) (non-decreasing per block), and -- for empty clusters -- the key centroids already sitting
// in ctx->Kc when key_fallback is set.  Block descriptors of the range must be in blocks_dev slot 1.
// fine_keys_are_means: the fine key centroids in ctx->Kc are the member means already and ctx->sumK holds the
// member sums behind them, at the fine ids of before the renumbering when sum_map (new id - f0 -> old id) is given.
mp_status finalize_range(mp_ctx* ctx, const void* Xk, const void* Xs, const void* Xv, long long x_unit_rows, int pt0,
                         int n_pts, const int32_t* ids, long long ids_stride, int f0, int f1, int c0, int c1, int nb,
                         int max_kf, bool key_fallback, bool fine_keys_are_means, const int32_t* sum_map, hipStream_t s)
{
    const int U = ctx->U;
    const long long Ncap = ctx->Ncap, tab = ctx->tab_rows;
    const int32_t* bdev = ctx->blocks_dev + 4 * (size_t)ctx->max_blocks;
    if (ids != ctx->fot + pt0)
        MP_HIPC(hipMemcpy2DAsync(ctx->fot + pt0, (size_t)Ncap * 4, ids, (size_t)ids_stride * 4, (size_t)n_pts * 4, U,
                                 hipMemcpyDeviceToDevice, s));
    MP_HIPC(launch_block_lists(ids, ids_stride, bdev, nb, max_kf, 0, U, ctx->km_start, tab + 1, ctx->km_list, Ncap, s));
    MP_HIPC(launch_offset_lists(ctx->km_start, tab + 1, f0, f1, ctx->km_list, Ncap, n_pts, pt0, U, ctx->fstart,
                                ctx->Fcap + 1, ctx->perm, Ncap, s));
    const bool bytes = ctx->cfg.kv_format == MP_KV_E4M3;
    if (!bytes)
        MP_HIPC(launch_gather_rows(Xs, Xv, x_unit_rows, ctx->km_list, Ncap, n_pts, U, ctx->Kp, ctx->Vp, Ncap, pt0, s));
    // (after a Lloyd iteration the working centroids already sitting in ctx->Kc ARE the member means of the
    // final assignment -- same members, same order of summation, same rounding: nothing to recompute)
    const bool two = ctx->cfg.levels == 2;
    if (!fine_keys_are_means)
        MP_HIPC(launch_cluster_means((const uint16_t*)Xk, x_unit_rows, ctx->km_list, Ncap, ctx->km_start, tab + 1, f0, f1, U,
                                     ctx->Kc, tab, 0, key_fallback ? ctx->Kc : nullptr, tab, nullptr, 0, 0,
                                     two ? ctx->sumK : nullptr, ctx->Fcap, s));
    MP_HIPC(launch_cluster_means((const uint16_t*)Xv, x_unit_rows, ctx->km_list, Ncap, ctx->km_start, tab + 1, f0, f1, U,
                                 ctx->Vc, tab, 0, nullptr, 0, ctx->Ncl, tab, 0, two ? ctx->sumV : nullptr, ctx->Fcap, s));
    if (bytes)   // (8-bit keys are residuals from the fine key centroids, which are final only now)
        MP_HIPC(launch_gather_quantize_rows(Xs, Xv, x_unit_rows, ctx->km_list, Ncap, ids, ids_stride, ctx->Kc, tab, n_pts, U,
                                            ctx->Kq, ctx->Vq, ctx->kv_scale, Ncap, pt0, s));
    if (two) {
        // the coarse tables: sums of the children's sums, in ascending fine id (no further pass over the rows)
        MP_HIPC(launch_coarse_start(ctx->cof, ctx->Fcap, f0, f1, c0, c1, U, ctx->cstart, ctx->Ccap + 1, s));
        const uint16_t* kfb = key_fallback ? ctx->Kc + (long long)ctx->Fcap * kHeadDim : nullptr;
        const int32_t* kmap = fine_keys_are_means ? sum_map : nullptr;
        MP_HIPC(launch_coarse_from_children(ctx->sumK, ctx->Fcap, kmap, ctx->Fcap, f0, ctx->cstart, ctx->Ccap + 1, ctx->Ncl, tab,
                                            c0, c1, U, ctx->Kc, tab, ctx->Fcap, kfb, tab, nullptr, 0, s));
        MP_HIPC(launch_coarse_from_children(ctx->sumV, ctx->Fcap, nullptr, 0, f0, ctx->cstart, ctx->Ccap + 1, ctx->Ncl, tab,
                                            c0, c1, U, ctx->Vc, tab, ctx->Fcap, nullptr, 0, ctx->Ncl, ctx->Fcap, s));
    }
    return MP_OK;
}

namespace {

// After the fine level of a range has its working centroids in km_Cf[f0,f1) and the assignment of
// its points in km_assign (old numbering), and -- two levels -- the coarse working centroids in
// km_Cc[c0,c1): run the coarse Lloyd iterations (coarse_iters >= 1), renumber, and finalize.
mp_status coarse_and_finalize(mp_ctx* ctx, const Range& r, int coarse_iters, bool init_coarse_from_seeds,
                              bool fine_keys_are_means, int max_kf, int max_kc, hipStream_t s)
{
    const int U = ctx->U;
    const bool two = ctx->cfg.levels == 2;
    const int nb = (int)r.blocks.size();
    const int kf = r.f1 - r.f0, kc = r.c1 - r.c0;
    const int32_t* bdev_c = ctx->blocks_dev + 8 * (size_t)ctx->max_blocks;
    const long long Fcap = ctx->Fcap, Ccap1 = std::max(ctx->Ccap, 1);
    if (two) {
        Problem pc{};
        pc.X = ctx->km_Cf; pc.x_unit_rows = Fcap; pc.n_points = r.f1; pc.p_first = r.f0; pc.blocks_dev = bdev_c; pc.nb = nb;
        pc.max_pts = max_kf; pc.max_k = max_kc; pc.k_total = r.c1; pc.k_first = r.c0; pc.C = ctx->km_Cc; pc.c_unit_rows = Ccap1;
        pc.assign = ctx->km_parent; pc.assign_stride = Fcap; pc.list = ctx->km_plist; pc.list_stride = Fcap;
        pc.cnt = ctx->km_cnt; pc.start = ctx->km_start; pc.cnt_stride = ctx->tab_rows;
        if (init_coarse_from_seeds) {
            hipLaunchKernelGGL(init_centroids_kernel, dim3(nb, U), dim3(256), 0, s, pc.X, pc.x_unit_rows, pc.blocks_dev,
                               ctx->km_seed_c, Ccap1, pc.C, pc.c_unit_rows);
            MP_HIPC(hipGetLastError());
        }
        for (int it = 0; it < coarse_iters; ++it) {
            const mp_status st = lloyd_iteration(ctx, pc, false, s);
            if (st != MP_OK) return st;
        }
        // km_plist[0..kf) = fine ids of the range grouped by coarse cluster (ascending inside): new order
        hipLaunchKernelGGL(invert_perm_kernel, dim3(blocks_for(kf, 256), U), dim3(256), 0, s, ctx->km_plist, Fcap, 0, kf,
                           r.f0, ctx->km_newid, Fcap);
        MP_HIPC(hipGetLastError());
        hipLaunchKernelGGL(map_ids_kernel, dim3(blocks_for(kf, 256), U), dim3(256), 0, s, ctx->km_plist, Fcap, 0, kf,
                           ctx->km_parent, Fcap, ctx->cof, Fcap, r.f0);
        MP_HIPC(hipGetLastError());
        hipLaunchKernelGGL(map_ids_kernel, dim3(blocks_for(r.n_pts, 256), U), dim3(256), 0, s, ctx->km_assign,
                           (long long)ctx->Ncap, 0, r.n_pts, ctx->km_newid, Fcap, ctx->km_assign, (long long)ctx->Ncap, 0);
        MP_HIPC(hipGetLastError());
        // key centroids kept by empty clusters: the working centroids, in the new numbering
        hipLaunchKernelGGL(gather1_rows_kernel, dim3(blocks_for((long long)kf * 16, 256), U), dim3(256), 0, s,
                           (const uint4*)ctx->km_Cf, Fcap, 0, ctx->km_plist, Fcap, 0, kf, (uint4*)ctx->Kc, ctx->tab_rows, r.f0);
        MP_HIPC(hipGetLastError());
        hipLaunchKernelGGL(gather1_rows_kernel, dim3(blocks_for((long long)kc * 16, 256), U), dim3(256), 0, s,
                           (const uint4*)ctx->km_Cc, Ccap1, r.c0, nullptr, 0, 0, kc, (uint4*)ctx->Kc, ctx->tab_rows,
                           ctx->Fcap + r.c0);
        MP_HIPC(hipGetLastError());
    } else {
        hipLaunchKernelGGL(gather1_rows_kernel, dim3(blocks_for((long long)kf * 16, 256), U), dim3(256), 0, s,
                           (const uint4*)ctx->km_Cf, Fcap, r.f0, nullptr, 0, 0, kf, (uint4*)ctx->Kc, ctx->tab_rows, r.f0);
        MP_HIPC(hipGetLastError());
    }
    return finalize_range(ctx, r.Xk, r.Xs, r.Xv, r.x_unit_rows, r.pt0, r.n_pts, ctx->km_assign, ctx->Ncap, r.f0, r.f1, r.c0,
                          r.c1, nb, max_kf, true, fine_keys_are_means, two ? ctx->km_plist : nullptr, s);
}

// Fresh clustering of a range: seeds are on the device (km_seed_f / km_seed_c at the range's ids).
mp_status cluster_range(mp_ctx* ctx, const Range& r, int iters, hipStream_t s)
{
    const int U = ctx->U;
    const int nb = (int)r.blocks.size();
    int max_pts, max_kf, max_kc;
    upload_descs(r, ctx->max_blocks, ctx->stage_blocks2, max_pts, max_kf, max_kc);
    int32_t* bdev_f = ctx->blocks_dev + 4 * (size_t)ctx->max_blocks;
    MP_TRY(upload(ctx, bdev_f, ctx->stage_blocks2.data(), ctx->stage_blocks2.size() * sizeof(int32_t), s));
    MP_TRY(flush_uploads(ctx, s));      // (the seeds staged by the caller included)
    Problem pf{};
    pf.X = r.Xk; pf.x_unit_rows = r.x_unit_rows; pf.n_points = r.n_pts; pf.p_first = 0; pf.blocks_dev = bdev_f; pf.nb = nb;
    pf.max_pts = max_pts; pf.max_k = max_kf; pf.k_total = r.f1; pf.k_first = r.f0; pf.C = ctx->km_Cf; pf.c_unit_rows = ctx->Fcap;
    pf.assign = ctx->km_assign; pf.assign_stride = ctx->Ncap; pf.list = ctx->km_list; pf.list_stride = ctx->Ncap;
    pf.cnt = ctx->km_cnt; pf.start = ctx->km_start; pf.cnt_stride = ctx->tab_rows;
    hipLaunchKernelGGL(init_centroids_kernel, dim3(nb, U), dim3(256), 0, s, pf.X, pf.x_unit_rows, pf.blocks_dev,
                       ctx->km_seed_f, (long long)ctx->Fcap, pf.C, pf.c_unit_rows);
    MP_HIPC(hipGetLastError());
    pf.sum_out = ctx->sumK; pf.sum_unit_rows = ctx->Fcap;
    for (int it = 0; it < iters; ++it) {
        const mp_status st = lloyd_iteration(ctx, pf, it == iters - 1, s);
        if (st != MP_OK) return st;
    }
    return coarse_and_finalize(ctx, r, iters, true, iters > 0, max_kf, max_kc, s);
}

}  // namespace

mp_status cluster_kv_impl(mp_ctx* ctx, const void* k, const void* k_lookup, const void* v, int32_t n_tokens, int32_t n_fine,
                          int32_t n_coarse, int32_t iters, uint64_t seed, const int32_t* init_fine,
                          const int32_t* init_coarse, hipStream_t s)
{
    MP_TRY(stage_open(ctx));
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
    MP_TRY(upload_2d(ctx, ctx->km_seed_f, (size_t)ctx->Fcap * 4, init_fine, (size_t)n_fine * 4, (size_t)n_fine * 4, U, s));
    if (two)
        MP_TRY(upload_2d(ctx, ctx->km_seed_c, (size_t)std::max(ctx->Ccap, 1) * 4, init_coarse, (size_t)n_coarse * 4,
                         (size_t)n_coarse * 4, U, s));

    Range r;
    r.Xk = (const uint16_t*)(k_lookup ? k_lookup : k); r.Xs = (const uint16_t*)k; r.Xv = (const uint16_t*)v;
    r.x_unit_rows = n_tokens; r.pt0 = 0; r.n_pts = n_tokens;
    r.blocks = blocks; r.f0 = 0; r.f1 = n_fine; r.c0 = 0; r.c1 = n_coarse;
    const mp_status st = cluster_range(ctx, r, iters, s);
    if (st != MP_OK) return st;

    // keep the last block in sequence order for the online update
    const BlockPlan& lb = blocks.back();
    const int nlast = lb.t1 - lb.t0;
    if (nlast <= ctx->FBcap) {
        const size_t row = kHeadDim * sizeof(uint16_t);
        MP_HIPC(hipMemcpy2DAsync(ctx->Kfb, (size_t)ctx->FBcap * row, (const char*)r.Xk + (size_t)lb.t0 * row,
                                 (size_t)n_tokens * row, (size_t)nlast * row, U, hipMemcpyDeviceToDevice, s));
        if (k_lookup)
            MP_HIPC(hipMemcpy2DAsync(ctx->Kfs, (size_t)ctx->FBcap * row, (const char*)k + (size_t)lb.t0 * row,
                                     (size_t)n_tokens * row, (size_t)nlast * row, U, hipMemcpyDeviceToDevice, s));
        MP_HIPC(hipMemcpy2DAsync(ctx->Vfb, (size_t)ctx->FBcap * row, (const char*)v + (size_t)lb.t0 * row,
                                 (size_t)n_tokens * row, (size_t)nlast * row, U, hipMemcpyDeviceToDevice, s));
    }
    ctx->n_tokens = n_tokens;
    ctx->n_fine = n_fine;
    ctx->n_coarse = two ? n_coarse : 0;
    ctx->blocks = blocks;
    ctx->has_index = true;
    ctx->decoded = false;
    ctx->updatable = nlast <= ctx->FBcap;
    return MP_OK;
}

mp_status set_clustering_impl(mp_ctx* ctx, const void* k, const void* k_lookup, const void* v, int32_t n_tokens, const int32_t* fine_of_token,
                              int32_t n_fine, const int32_t* coarse_of_fine, int32_t n_coarse, hipStream_t s)
{
    MP_TRY(stage_open(ctx));
    const int U = ctx->U;
    const bool two = ctx->cfg.levels == 2;
    MP_HIPC(hipMemcpy2DAsync(ctx->fot, (size_t)ctx->Ncap * 4, fine_of_token, (size_t)n_tokens * 4, (size_t)n_tokens * 4, U,
                             hipMemcpyDeviceToDevice, s));
    if (two)
        MP_HIPC(hipMemcpy2DAsync(ctx->cof, (size_t)ctx->Fcap * 4, coarse_of_fine, (size_t)n_fine * 4, (size_t)n_fine * 4, U,
                                 hipMemcpyDeviceToDevice, s));
    Range r;
    r.blocks.assign(1, BlockPlan{0, n_tokens, 0, n_fine, 0, n_coarse});
    int max_pts, max_kf, max_kc;
    upload_descs(r, ctx->max_blocks, ctx->stage_blocks2, max_pts, max_kf, max_kc);
    MP_TRY(upload(ctx, ctx->blocks_dev + 4 * (size_t)ctx->max_blocks, ctx->stage_blocks2.data(),
                  ctx->stage_blocks2.size() * sizeof(int32_t), s));
    MP_TRY(flush_uploads(ctx, s));
    const void* xk = k_lookup ? k_lookup : k;
    const mp_status st = finalize_range(ctx, xk, k, v, n_tokens, 0, n_tokens, ctx->fot, ctx->Ncap, 0, n_fine, 0, n_coarse, 1,
                                        max_kf, false, false, nullptr, s);
    if (st != MP_OK) return st;
    if (n_tokens <= ctx->FBcap) {
        const size_t row = kHeadDim * sizeof(uint16_t);
        MP_HIPC(hipMemcpy2DAsync(ctx->Kfb, (size_t)ctx->FBcap * row, xk, (size_t)n_tokens * row, (size_t)n_tokens * row, U,
                                 hipMemcpyDeviceToDevice, s));
        if (k_lookup)
            MP_HIPC(hipMemcpy2DAsync(ctx->Kfs, (size_t)ctx->FBcap * row, k, (size_t)n_tokens * row, (size_t)n_tokens * row, U,
                                     hipMemcpyDeviceToDevice, s));
        MP_HIPC(hipMemcpy2DAsync(ctx->Vfb, (size_t)ctx->FBcap * row, v, (size_t)n_tokens * row, (size_t)n_tokens * row, U,
                                 hipMemcpyDeviceToDevice, s));
    }
    ctx->n_tokens = n_tokens;
    ctx->n_fine = n_fine;
    ctx->n_coarse = two ? n_coarse : 0;
    ctx->blocks = r.blocks;
    ctx->has_index = true;
    ctx->decoded = false;
    ctx->updatable = n_tokens <= ctx->FBcap;
    return MP_OK;
}

void update_seed_counts(const mp_ctx* ctx, int n_new, int n_new_fine, int n_new_coarse, int32_t counts[6])
{
    const BlockPlan& lb = ctx->blocks.back();
    const bool two = ctx->cfg.levels == 2;
    const long long nb = lb.t1 - lb.t0 + n_new;
    const long long kf = lb.f1 - lb.f0 + n_new_fine;
    const long long kc = two ? lb.c1 - lb.c0 + n_new_coarse : 0;
    counts[0] = n_new_fine;
    counts[1] = two ? n_new_coarse : 0;
    counts[2] = counts[3] = counts[4] = counts[5] = 0;
    const int W = ctx->cfg.block_w;
    if (W > 0 && nb >= (long long)W + ctx->cfg.block_alpha) {
        counts[2] = (int32_t)(kf * W / nb);
        counts[3] = (int32_t)(kf - counts[2]);
        counts[4] = (int32_t)(kc * W / nb);
        counts[5] = (int32_t)(kc - counts[4]);
    }
}

mp_status update_clusters_impl(mp_ctx* ctx, const void* k_new, const void* k_new_lookup, const void* v_new, int32_t n_new, int32_t n_new_fine,
                               int32_t n_new_coarse, int32_t refine_iters, int32_t split_iters, uint64_t seed,
                               const int32_t* seeds, hipStream_t s)
{
    MP_TRY(stage_open(ctx));
    const int U = ctx->U;
    const bool two = ctx->cfg.levels == 2;
    if (!ctx->updatable) return fail(ctx, MP_ESTATE, "mp_update_clusters: the last block does not fit the update workspace");
    BlockPlan lb = ctx->blocks.back();
    const int t0 = lb.t0, f0 = lb.f0, c0 = lb.c0;
    const int nb_old = lb.t1 - lb.t0, nb = nb_old + n_new;
    const int kf_old = lb.f1 - lb.f0, kf = kf_old + n_new_fine;
    const int kc_old = lb.c1 - lb.c0, kc = two ? kc_old + n_new_coarse : 0;
    const int f1 = f0 + kf, c1 = c0 + kc;
    if (ctx->n_tokens + n_new > ctx->Ncap) return fail(ctx, MP_ECAPACITY, "mp_update_clusters: %d tokens > max_tokens %d", ctx->n_tokens + n_new, ctx->Ncap);
    if (nb > ctx->FBcap) return fail(ctx, MP_ECAPACITY, "mp_update_clusters: last block would hold %d tokens > %d", nb, ctx->FBcap);
    if (f1 > ctx->Fcap) return fail(ctx, MP_ECAPACITY, "mp_update_clusters: %d fine clusters > max_fine %d", f1, ctx->Fcap);
    if (two && c1 > ctx->Ccap) return fail(ctx, MP_ECAPACITY, "mp_update_clusters: %d coarse clusters > max_coarse %d", c1, ctx->Ccap);
    if ((int)ctx->blocks.size() + 1 > ctx->max_blocks) return fail(ctx, MP_ECAPACITY, "mp_update_clusters: too many blocks");

    int32_t cnts[6];
    update_seed_counts(ctx, n_new, n_new_fine, n_new_coarse, cnts);
    const bool split = cnts[2] > 0 || cnts[3] > 0;
    const int W = ctx->cfg.block_w;
    if (split) {
        if (cnts[2] < 1 || cnts[3] < 1 || cnts[2] > W || cnts[3] > nb - W)
            return fail(ctx, MP_EINVAL, "mp_update_clusters: cannot split %d fine clusters over %d + %d tokens", kf, W, nb - W);
        if (two && (cnts[4] < 1 || cnts[5] < 1 || cnts[4] > cnts[2] || cnts[5] > cnts[3]))
            return fail(ctx, MP_EINVAL, "mp_update_clusters: cannot split %d coarse clusters", kc);
    }
    int total = 0, off[7];
    for (int i = 0; i < 6; ++i) { off[i] = total; total += cnts[i]; }
    off[6] = total;
    const int lim[6] = {n_new, n_new_fine, W, nb - W, cnts[2], cnts[3]};
    std::vector<int32_t>& gen = ctx->stage_seed_f;
    if (!seeds) {
        gen.resize((size_t)U * std::max(total, 1));
        for (int u = 0; u < U; ++u)
            for (int i = 0; i < 6; ++i)
                if (cnts[i] > 0)
                    draw_distinct(seed ^ (0x7f4a7c15ull + (uint64_t)u * 1000003ull + (uint64_t)i * 7919ull + (uint64_t)ctx->n_tokens),
                                  lim[i], cnts[i], gen.data() + (size_t)u * total + off[i]);
        seeds = gen.data();
    } else {
        for (int u = 0; u < U; ++u)
            for (int i = 0; i < 6; ++i)
                if (cnts[i] > 0 && !distinct_in_range(seeds + (size_t)u * total + off[i], cnts[i], lim[i]))
                    return fail(ctx, MP_EINVAL, "mp_update_clusters: seed list %d of unit %d is not a set of distinct indices below %d", i, u, lim[i]);
    }
    const size_t row = kHeadDim * sizeof(uint16_t);
    const long long Fcap = ctx->Fcap, Ccap1 = std::max(ctx->Ccap, 1), Ncap = ctx->Ncap;

    // ---- append the new tokens to the sequence-ordered copy of the last block ----
    MP_HIPC(hipMemcpy2DAsync((char*)ctx->Kfb + (size_t)nb_old * row, (size_t)ctx->FBcap * row,
                             k_new_lookup ? k_new_lookup : k_new, (size_t)n_new * row, (size_t)n_new * row, U,
                             hipMemcpyDeviceToDevice, s));
    if (k_new_lookup)
        MP_HIPC(hipMemcpy2DAsync((char*)ctx->Kfs + (size_t)nb_old * row, (size_t)ctx->FBcap * row, k_new, (size_t)n_new * row,
                                 (size_t)n_new * row, U, hipMemcpyDeviceToDevice, s));
    MP_HIPC(hipMemcpy2DAsync((char*)ctx->Vfb + (size_t)nb_old * row, (size_t)ctx->FBcap * row, v_new, (size_t)n_new * row,
                             (size_t)n_new * row, U, hipMemcpyDeviceToDevice, s));
    // seeds of the new clusters, at their global ids
    if (n_new_fine > 0)
        MP_TRY(upload_2d(ctx, ctx->km_seed_f + lb.f1, (size_t)Fcap * 4, seeds + off[0], (size_t)total * 4,
                         (size_t)n_new_fine * 4, U, s));
    if (two && n_new_coarse > 0)
        MP_TRY(upload_2d(ctx, ctx->km_seed_c + lb.c1, (size_t)Ccap1 * 4, seeds + off[1], (size_t)total * 4,
                         (size_t)n_new_coarse * 4, U, s));

    // block descriptors: slot 1 = [fine: all points of the last block | coarse], slot 0 (scratch) = appended points / new clusters
    Range r;
    r.Xk = ctx->Kfb; r.Xs = k_new_lookup ? ctx->Kfs : ctx->Kfb; r.Xv = ctx->Vfb; r.x_unit_rows = ctx->FBcap; r.pt0 = t0; r.n_pts = nb;
    r.blocks.assign(1, BlockPlan{0, nb, f0, f1, c0, c1});
    r.f0 = f0; r.f1 = f1; r.c0 = c0; r.c1 = c1;
    int max_pts, max_kf, max_kc;
    upload_descs(r, ctx->max_blocks, ctx->stage_blocks2, max_pts, max_kf, max_kc);
    int32_t* bdev_f = ctx->blocks_dev + 4 * (size_t)ctx->max_blocks;
    MP_TRY(upload(ctx, bdev_f, ctx->stage_blocks2.data(), ctx->stage_blocks2.size() * sizeof(int32_t), s));
    std::vector<int32_t>& sd = ctx->stage_blocks;
    sd.assign(12, 0);
    sd[0] = nb_old; sd[1] = nb; sd[2] = f0; sd[3] = f1;             // appended points vs all fine centroids
    sd[4] = nb_old; sd[5] = nb; sd[6] = lb.f1; sd[7] = f1;          // new fine centroids seeded from appended points
    sd[8] = lb.f1; sd[9] = f1; sd[10] = lb.c1; sd[11] = c1;         // new coarse centroids seeded from new fine centroids
    MP_TRY(upload(ctx, ctx->blocks_dev, sd.data(), sd.size() * sizeof(int32_t), s));
    MP_TRY(flush_uploads(ctx, s));

    // ---- working fine centroids: the stored key centroids, then the new seeds ----
    hipLaunchKernelGGL(gather1_rows_kernel, dim3(blocks_for((long long)kf_old * 16, 256), U), dim3(256), 0, s,
                       (const uint4*)ctx->Kc, ctx->tab_rows, f0, nullptr, 0, 0, kf_old, (uint4*)ctx->km_Cf, Fcap, f0);
    MP_HIPC(hipGetLastError());
    if (n_new_fine > 0) {
        hipLaunchKernelGGL(init_centroids_kernel, dim3(1, U), dim3(256), 0, s, ctx->Kfb, (long long)ctx->FBcap,
                           ctx->blocks_dev + 4, ctx->km_seed_f, Fcap, ctx->km_Cf, Fcap);
        MP_HIPC(hipGetLastError());
    }
    // ---- one-shot assignment of the appended tokens + running mean of the touched centroids ----
    MP_HIPC(mp::launch_assign(ctx->Kfb, (long long)ctx->FBcap, ctx->blocks_dev, 1, n_new, 0, U, ctx->km_Cf, Fcap,
                              ctx->km_assign, Ncap, ctx->km_list, Ncap, amb_counters(ctx, 0), amb_counters(ctx, 1),
                              ctx->max_blocks, s));
    ctx->amb_turn ^= 1;
    MP_HIPC(hipMemcpy2DAsync(ctx->km_assign, (size_t)Ncap * 4, ctx->fot + t0, (size_t)Ncap * 4, (size_t)nb_old * 4, U,
                             hipMemcpyDeviceToDevice, s));
    hipLaunchKernelGGL(running_mean_kernel, dim3((kf + 3) / 4, U), dim3(256), 0, s, ctx->Kfb, (long long)ctx->FBcap,
                       nb_old, nb, ctx->km_assign, Ncap, f0, f1, lb.f1, ctx->Ncl, ctx->tab_rows, ctx->km_Cf, Fcap);
    MP_HIPC(hipGetLastError());
    // ---- refinement: full Lloyd iterations over the last block ----
    Problem pf{};
    pf.X = ctx->Kfb; pf.x_unit_rows = ctx->FBcap; pf.n_points = nb; pf.p_first = 0; pf.blocks_dev = bdev_f; pf.nb = 1;
    pf.max_pts = nb; pf.max_k = kf; pf.k_total = f1; pf.k_first = f0; pf.C = ctx->km_Cf; pf.c_unit_rows = Fcap;
    pf.assign = ctx->km_assign; pf.assign_stride = Ncap; pf.list = ctx->km_list; pf.list_stride = Ncap;
    pf.cnt = ctx->km_cnt; pf.start = ctx->km_start; pf.cnt_stride = ctx->tab_rows;
    pf.sum_out = ctx->sumK; pf.sum_unit_rows = ctx->Fcap;
    for (int it = 0; it < refine_iters; ++it) {
        const mp_status st = lloyd_iteration(ctx, pf, it == refine_iters - 1, s);
        if (st != MP_OK) return st;
    }
    // ---- coarse level: stored coarse key centroids, plus seeds taken from the new fine centroids ----
    if (two) {
        hipLaunchKernelGGL(gather1_rows_kernel, dim3(blocks_for((long long)kc_old * 16, 256), U), dim3(256), 0, s,
                           (const uint4*)ctx->Kc, ctx->tab_rows, ctx->Fcap + c0, nullptr, 0, 0, kc_old, (uint4*)ctx->km_Cc,
                           Ccap1, c0);
        MP_HIPC(hipGetLastError());
        if (n_new_coarse > 0) {
            hipLaunchKernelGGL(init_centroids_kernel, dim3(1, U), dim3(256), 0, s, ctx->km_Cf, Fcap, ctx->blocks_dev + 8,
                               ctx->km_seed_c, Ccap1, ctx->km_Cc, Ccap1);
            MP_HIPC(hipGetLastError());
        }
    }
    mp_status st = coarse_and_finalize(ctx, r, std::max(1, refine_iters), false, refine_iters > 0, max_kf, max_kc, s);
    if (st != MP_OK) return st;
    lb.t1 = t0 + nb; lb.f1 = f1; lb.c1 = c1;
    ctx->blocks.back() = lb;
    ctx->n_tokens += n_new;
    ctx->n_fine += n_new_fine;
    ctx->n_coarse += two ? n_new_coarse : 0;
    ctx->decoded = false;

    if (split) {
        // ---- the last block reached W + alpha tokens: cluster its first W tokens and the rest afresh ----
        MP_TRY(upload_2d(ctx, ctx->km_seed_f + f0, (size_t)Fcap * 4, seeds + off[2], (size_t)total * 4,
                         (size_t)(cnts[2] + cnts[3]) * 4, U, s));
        if (two)
            MP_TRY(upload_2d(ctx, ctx->km_seed_c + c0, (size_t)Ccap1 * 4, seeds + off[4], (size_t)total * 4,
                             (size_t)(cnts[4] + cnts[5]) * 4, U, s));
        Range r2 = r;
        r2.blocks.clear();
        r2.blocks.push_back(BlockPlan{0, W, f0, f0 + cnts[2], c0, c0 + cnts[4]});
        r2.blocks.push_back(BlockPlan{W, nb, f0 + cnts[2], f1, c0 + cnts[4], c1});
        st = cluster_range(ctx, r2, split_iters, s);
        if (st != MP_OK) return st;
        // the remaining tokens become the new last block: move them to the front of the sequence-ordered
        // copies, W rows at a time (a piece never overlaps its destination, W rows further down)
        uint16_t* bufs[3] = {ctx->Kfb, ctx->Vfb, k_new_lookup ? ctx->Kfs : nullptr};
        for (uint16_t* b : bufs) {
            if (!b) continue;
            for (int done = 0; done < nb - W; done += W) {
                const int rows_now = std::min(W, nb - W - done);
                MP_HIPC(hipMemcpy2DAsync((char*)b + (size_t)done * row, (size_t)ctx->FBcap * row,
                                         (const char*)b + (size_t)(W + done) * row, (size_t)ctx->FBcap * row,
                                         (size_t)rows_now * row, U, hipMemcpyDeviceToDevice, s));
            }
        }
        ctx->blocks.back() = BlockPlan{t0, t0 + W, f0, f0 + cnts[2], c0, c0 + cnts[4]};
        ctx->blocks.push_back(BlockPlan{t0 + W, t0 + nb, f0 + cnts[2], f1, c0 + cnts[4], c1});
    }
    return MP_OK;
}

}  // namespace mp
