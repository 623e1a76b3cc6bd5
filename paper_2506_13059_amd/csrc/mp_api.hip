// C-ABI layer: argument checks, error strings, memory ownership, launch sequencing.
#include "../../include/mp.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "mp_ctx.h"
#include "mp_internal.h"

using namespace mp;

namespace mp {
// implemented in mp_cluster.hip
mp_status cluster_kv_impl(mp_ctx* ctx, const void* k, const void* k_lookup, const void* v, int32_t n_tokens, int32_t n_fine,
                          int32_t n_coarse, int32_t iters, uint64_t seed, const int32_t* init_fine,
                          const int32_t* init_coarse, hipStream_t s);
mp_status update_clusters_impl(mp_ctx* ctx, const void* k_new, const void* k_new_lookup, const void* v_new, int32_t n_new,
                               int32_t n_new_fine, int32_t n_new_coarse, int32_t refine_iters, int32_t split_iters,
                               uint64_t seed, const int32_t* seeds, hipStream_t s);
mp_status set_clustering_impl(mp_ctx* ctx, const void* k, const void* k_lookup, const void* v, int32_t n_tokens,
                              const int32_t* fine_of_token, int32_t n_fine, const int32_t* coarse_of_fine, int32_t n_coarse,
                              hipStream_t s);
void update_seed_counts(const mp_ctx* ctx, int n_new, int n_new_fine, int n_new_coarse, int32_t counts[6]);
hipError_t resolve_static_scratch();   // further down in this file

thread_local std::string g_err;   // errors of context-free calls

mp_status fail(mp_ctx* ctx, mp_status st, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf;
    else g_err = buf;
    return st;
}

// Rows per workgroup of the value pass for a stream of n rows per unit: large enough that the
// partials stay a small fraction of the traffic, small enough that there are many workgroups.
// Two workgroups of the value pass are resident per compute unit, 512 on the chip.
constexpr int kResidentWgs = 512;

int pick_chunk_rows(long long n_rows_per_unit, int n_units)
{
    int cr = kChunkRowsMin;
    while (cr < 4096 && n_units * ((n_rows_per_unit + cr - 1) / cr) > 8192) cr *= 2;
    return cr;
}

// Rows per workgroup for one stream of the value pass (selected keys: largest = 2048; centroid terms
// and tail: largest = 512).  Long chunks spread the prologue and epilogue of a workgroup over more
// bytes, but only pay off while the stream still has a workgroup for every resident slot; so: the
// largest size that does, else the smallest (measured on cfg3: 2048 at key budget 8192 = 512
// workgroups, 512 at budget 4096 = 1024 workgroups; on one sequence of 32K tokens, 8 units, 128-row
// chunks instead of 512-row ones fill 4 times as many compute units).
int pick_stream_chunk_rows(int rows_max, int n_units, int largest)
{
    static const int kChoices[] = {2048, 512, 256, 128};
    for (int c : kChoices)
        if (c <= largest && (long long)n_units * ((rows_max + c - 1) / c) >= kResidentWgs) return c;
    return 128;
}

// Most chunks a stream of up to rows_cap rows can be cut into under that rule.
int max_stream_chunks(int rows_cap, int n_units, int largest)
{
    int m = 1;
    for (int r = 1; r <= rows_cap; ++r) {
        const int c = pick_stream_chunk_rows(r, n_units, largest);
        m = std::max(m, (r + c - 1) / c);
    }
    return m;
}

}  // namespace mp

namespace {

#define MP_HIP(ctx, expr)                                                                           \
    do {                                                                                            \
        hipError_t e_ = (expr);                                                                     \
        if (e_ != hipSuccess) return fail((ctx), MP_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }

// k distinct values, all in [0, n)?
bool distinct_in_range(const int32_t* v, int k, int n)
{
    std::vector<char> seen((size_t)std::max(n, 1), 0);
    for (int i = 0; i < k; ++i) {
        if (v[i] < 0 || v[i] >= n || seen[v[i]]) return false;
        seen[v[i]] = 1;
    }
    return true;
}

template <typename T>
hipError_t dev_alloc(mp_ctx* ctx, T** p, size_t count)
{
    const size_t bytes = std::max<size_t>(count, 1) * sizeof(T);
    void* q = nullptr;
    hipError_t e = hipMalloc(&q, bytes);
    if (e != hipSuccess) return e;
    ctx->allocs.push_back(q);
    ctx->device_bytes += bytes;
    *p = (T*)q;
    return hipSuccess;
}

void free_all(mp_ctx* ctx)
{
    for (void* p : ctx->allocs) (void)hipFree(p);
    ctx->allocs.clear();
}

}  // namespace

// A context created with lookup_keys expects lookup keys wherever keys are handed over, any other none.
static bool lookup_arg_ok(const mp_ctx* ctx, const void* k_lookup) { return (ctx->cfg.lookup_keys != 0) == (k_lookup != nullptr); }

extern "C" {

const char* mp_version(void) { return "mp-gfx950 0.1"; }

const char* mp_last_error(const mp_ctx* ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

size_t mp_device_bytes(const mp_ctx* ctx) { return ctx ? ctx->device_bytes : 0; }

int32_t mp_plan_blocks(int32_t n_tokens, int32_t block_w, int32_t block_alpha, int32_t n_fine, int32_t n_coarse,
                       int32_t* out, int32_t max_blocks)
{
    if (n_tokens <= 0 || block_w < 0 || block_alpha < 0 || n_fine < 0 || n_coarse < 0) return -1;
    std::vector<BlockPlan> b = plan_blocks(n_tokens, block_w, block_alpha, n_fine, n_coarse);
    if (out) {
        for (int i = 0; i < (int)b.size() && i < max_blocks; ++i) {
            out[6 * i + 0] = b[i].t0; out[6 * i + 1] = b[i].t1;
            out[6 * i + 2] = b[i].f0; out[6 * i + 3] = b[i].f1;
            out[6 * i + 4] = b[i].c0; out[6 * i + 5] = b[i].c1;
        }
    }
    return (int32_t)b.size();
}

mp_status mp_create(const mp_config* cfg, mp_ctx** out)
{
    if (!cfg || !out) return fail(nullptr, MP_EINVAL, "mp_create: null pointer");
    *out = nullptr;
    const mp_config& c = *cfg;
    if (c.batch < 1 || c.n_kv_heads < 1 || c.n_q_heads < 1 || c.n_q_heads % c.n_kv_heads)
        return fail(nullptr, MP_EINVAL, "mp_create: bad head counts B=%d Hq=%d Hkv=%d", c.batch, c.n_q_heads,
                    c.n_kv_heads);
    if (c.head_dim != kHeadDimHost) return fail(nullptr, MP_EINVAL, "mp_create: head_dim must be 128, got %d", c.head_dim);
    const int G = c.n_q_heads / c.n_kv_heads;
    if (G > 8) return fail(nullptr, MP_EINVAL, "mp_create: group size %d > 8 is not supported", G);
    if (c.levels != 1 && c.levels != 2) return fail(nullptr, MP_EINVAL, "mp_create: levels must be 1 or 2");
    if (c.max_tokens < 1) return fail(nullptr, MP_EINVAL, "mp_create: max_tokens must be >= 1");
    if (c.max_fine < 1 || c.max_fine > kMaxClustersPerLevel)
        return fail(nullptr, MP_EINVAL, "mp_create: max_fine must be in [1, %d]", kMaxClustersPerLevel);
    if (c.levels == 2 && (c.max_coarse < 1 || c.max_coarse > c.max_fine))
        return fail(nullptr, MP_EINVAL, "mp_create: max_coarse must be in [1, max_fine] when levels == 2");
    if (c.levels == 1 && c.max_coarse < 0) return fail(nullptr, MP_EINVAL, "mp_create: max_coarse < 0");
    if (c.block_w < 0 || c.block_alpha < 0 || (c.block_w > 0 && (c.block_alpha < 1 || c.block_alpha > c.block_w)))
        return fail(nullptr, MP_EINVAL, "mp_create: need block_w >= 0 and, with block_w > 0, 1 <= block_alpha <= block_w");
    if (c.max_tail < 0) return fail(nullptr, MP_EINVAL, "mp_create: max_tail < 0");
    if (!(c.softmax_scale >= 0.f)) return fail(nullptr, MP_EINVAL, "mp_create: softmax_scale must be >= 0");
    if (c.kv_format != MP_KV_BF16 && c.kv_format != MP_KV_E4M3) return fail(nullptr, MP_EINVAL, "mp_create: unknown kv_format %d", c.kv_format);
    if (c.kv_format == MP_KV_E4M3 && c.lookup_keys)
        return fail(nullptr, MP_EINVAL, "mp_create: 8-bit keys are residuals from the centroids of the stored keys; not available with lookup_keys");
    if ((long long)c.batch * c.n_kv_heads > 65535) return fail(nullptr, MP_EINVAL, "mp_create: more than 65535 units");

    mp_ctx* ctx = new (std::nothrow) mp_ctx();
    if (!ctx) return fail(nullptr, MP_ENOMEM, "mp_create: host allocation failed");
    ctx->cfg = c;
    ctx->U = c.batch * c.n_kv_heads;
    ctx->G = G;
    ctx->scale_d = c.softmax_scale > 0.f ? (double)c.softmax_scale : 1.0 / std::sqrt((double)kHeadDimHost);
    ctx->scale = (float)ctx->scale_d;
    ctx->Ncap = c.max_tokens;
    ctx->Fcap = c.max_fine;
    ctx->Ccap = c.levels == 2 ? c.max_coarse : 0;
    ctx->Tcap = c.max_tail;
    ctx->tab_rows = (long long)ctx->Fcap + ctx->Ccap;
    ctx->FBcap = c.block_w > 0 ? (int32_t)std::min<long long>(c.max_tokens, 2ll * c.block_w) : c.max_tokens;
    ctx->max_blocks = std::max(4, c.block_w > 0 ? c.max_tokens / c.block_w + 2 : 2);
    ctx->Pcap = mp::max_stream_chunks(ctx->Ncap, ctx->U, 2048) + mp::max_stream_chunks(std::max(ctx->Tcap, 1), ctx->U, 512) +
                mp::max_stream_chunks((int)ctx->tab_rows, ctx->U, 512);

    hipError_t e = hipGetDevice(&ctx->device);
    if (e == hipSuccess) e = mp::resolve_static_scratch();
    if (e == hipSuccess) e = hipDeviceGetAttribute(&ctx->n_cus, hipDeviceAttributeMultiprocessorCount, ctx->device);
    const size_t U = ctx->U, N = ctx->Ncap, F = ctx->Fcap, Cc = std::max(ctx->Ccap, 1), T = ctx->tab_rows, D = kHeadDimHost;
#define A(ptr, count) if (e == hipSuccess) e = dev_alloc(ctx, &ctx->ptr, (count))
    if (c.kv_format == MP_KV_E4M3) { A(Kq, U * N * D); A(Vq, U * N * D); A(kv_scale, U * N * 2); A(sel_base, U * F * 8); A(row_slot, U * N); }
    else { A(Kp, U * N * D); A(Vp, U * N * D); }
    A(perm, U * N); A(fot, U * N);
    A(fstart, U * (F + 1)); A(cof, U * F); A(cstart, U * (Cc + 1));
    if (c.levels == 2) { A(sumK, U * F * D); A(sumV, U * F * D); }
    A(Kc, U * T * D); A(Vc, U * T * D); A(Ncl, U * T);
    A(Kfb, U * (size_t)ctx->FBcap * D); A(Vfb, U * (size_t)ctx->FBcap * D);
    if (c.lookup_keys) A(Kfs, U * (size_t)ctx->FBcap * D);
    A(km_assign, U * N); A(km_list, U * N); A(km_cnt, U * T); A(km_start, U * (T + 2));
    A(km_Cf, U * F * D); A(km_Cc, U * Cc * D); A(km_parent, U * F); A(km_plist, U * F); A(km_newid, U * F);
    A(km_seed_f, U * F); A(km_seed_c, U * Cc); A(blocks_dev, 3 * (size_t)ctx->max_blocks * 4);
    A(km_amb, 2 * U * (size_t)ctx->max_blocks);
    ctx->Lcap = (int32_t)std::max(F, Cc);
    const size_t Lc = ctx->Lcap;
    A(lg, U * G * Lc); A(sc_keys, U * Lc); A(sc_wts, U * Lc); A(sc_ids, U * Lc); A(sc_aux, U * Lc); A(sc_aux2, U * Lc);
    A(sc_flags, U * Lc); A(key_c, U * Cc); A(key_f, U * F); A(key_mode, U * 2); A(flag_c, U * Cc); A(flag_f, U * F);
    A(cand, U * F); A(n_cand, U); A(unprom_lse, U * G); A(rows, U * N); A(n_rows, U);
    A(mp_rows, U * T); A(mp_scores, U * T * G); A(n_mp, U); A(counters, U * 4);
    A(partials, U * (size_t)ctx->Pcap * G * kPartStride);
    if (ctx->Tcap > 0) {
        const size_t Tc = ctx->Tcap;
        A(Kt, U * Tc * D); A(Vt, U * Tc * D); A(Kts, U * Tc * D); A(Vts, U * Tc * D);
        if (c.lookup_keys) { A(Ktl, U * Tc * D); A(Ktls, U * Tc * D); }
    }
#undef A
    if (e == hipSuccess) {
        ctx->pin_bytes = 1u << 20;
        e = hipHostMalloc((void**)&ctx->pin, ctx->pin_bytes, hipHostMallocDefault);
        if (e != hipSuccess) ctx->pin = nullptr;
    }
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->pin_ev, hipEventDisableTiming);
    if (e == hipSuccess) e = hipMemset(ctx->counters, 0, U * 4 * sizeof(int32_t));
    if (e == hipSuccess) e = hipMemset(ctx->km_amb, 0, 2 * U * (size_t)ctx->max_blocks * sizeof(int32_t));
    if (e == hipSuccess) e = hipMemset(ctx->n_mp, 0, U * sizeof(int32_t));
    if (e == hipSuccess) e = hipMemset(ctx->n_rows, 0, U * sizeof(int32_t));
    if (e == hipSuccess) e = hipMemset(ctx->n_cand, 0, U * sizeof(int32_t));
    if (e != hipSuccess) {
        const mp_status st = (e == hipErrorOutOfMemory) ? MP_ENOMEM : MP_EHIP;
        fail(nullptr, st, "mp_create: %s (after %zu bytes)", hipGetErrorString(e), ctx->device_bytes);
        if (ctx->pin_ev) (void)hipEventDestroy(ctx->pin_ev);
        if (ctx->pin) (void)hipHostFree(ctx->pin);
        free_all(ctx);
        delete ctx;
        return st;
    }
    *out = ctx;
    return MP_OK;
}

void mp_destroy(mp_ctx* ctx)
{
    if (!ctx) return;
    (void)hipDeviceSynchronize();
    for (hipEvent_t e : ctx->ev)
        if (e) (void)hipEventDestroy(e);
    if (ctx->pin_ev) (void)hipEventDestroy(ctx->pin_ev);
    if (ctx->pin) (void)hipHostFree(ctx->pin);
    free_all(ctx);
    delete ctx;
}

mp_status mp_cluster_kv(mp_ctx* ctx, const void* k, const void* k_lookup, const void* v, int32_t n_tokens, int32_t n_fine, int32_t n_coarse,
                        int32_t iters, uint64_t seed, const int32_t* init_fine, const int32_t* init_coarse,
                        void* stream)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_cluster_kv: null context");
    if (!k || !v) return fail(ctx, MP_EINVAL, "mp_cluster_kv: null k/v");
    if (n_tokens < 1 || n_fine < 1 || iters < 1) return fail(ctx, MP_EINVAL, "mp_cluster_kv: n_tokens, n_fine, iters must be >= 1");
    if (n_tokens > ctx->Ncap) return fail(ctx, MP_ECAPACITY, "mp_cluster_kv: n_tokens %d > max_tokens %d", n_tokens, ctx->Ncap);
    if (n_fine > ctx->Fcap) return fail(ctx, MP_ECAPACITY, "mp_cluster_kv: n_fine %d > max_fine %d", n_fine, ctx->Fcap);
    if (ctx->cfg.levels == 2) {
        if (n_coarse < 1) return fail(ctx, MP_EINVAL, "mp_cluster_kv: n_coarse must be >= 1 with two levels");
        if (n_coarse > ctx->Ccap) return fail(ctx, MP_ECAPACITY, "mp_cluster_kv: n_coarse %d > max_coarse %d", n_coarse, ctx->Ccap);
    } else {
        n_coarse = 0;
    }
    const std::vector<BlockPlan> blocks = plan_blocks(n_tokens, ctx->cfg.block_w, ctx->cfg.block_alpha, n_fine, n_coarse);
    if ((int)blocks.size() > ctx->max_blocks) return fail(ctx, MP_ECAPACITY, "mp_cluster_kv: too many blocks");
    for (const BlockPlan& b : blocks) {
        const int kf = b.f1 - b.f0, kc = b.c1 - b.c0, nt = b.t1 - b.t0;
        if (kf < 1 || kf > nt) return fail(ctx, MP_EINVAL, "mp_cluster_kv: block [%d,%d) gets %d fine clusters", b.t0, b.t1, kf);
        if (ctx->cfg.levels == 2 && (kc < 1 || kc > kf))
            return fail(ctx, MP_EINVAL, "mp_cluster_kv: block [%d,%d) gets %d coarse clusters for %d fine", b.t0, b.t1, kc, kf);
    }
    const int U = ctx->U;
    if (init_fine)
        for (int u = 0; u < U; ++u)
            for (const BlockPlan& b : blocks)
                if (!distinct_in_range(init_fine + (size_t)u * n_fine + b.f0, b.f1 - b.f0, b.t1 - b.t0))
                    return fail(ctx, MP_EINVAL, "mp_cluster_kv: init_fine of unit %d, block [%d,%d) is not a set of distinct token indices inside the block", u, b.t0, b.t1);
    if (init_coarse && ctx->cfg.levels == 2)
        for (int u = 0; u < U; ++u)
            for (const BlockPlan& b : blocks)
                if (!distinct_in_range(init_coarse + (size_t)u * n_coarse + b.c0, b.c1 - b.c0, b.f1 - b.f0))
                    return fail(ctx, MP_EINVAL, "mp_cluster_kv: init_coarse of unit %d, block [%d,%d) is not a set of distinct fine-cluster indices inside the block", u, b.t0, b.t1);
    if (!lookup_arg_ok(ctx, k_lookup)) return fail(ctx, MP_EINVAL, "mp_cluster_kv: k_lookup must be given exactly when the context was created with lookup_keys");
    const mp_status st = cluster_kv_impl(ctx, k, k_lookup, v, n_tokens, n_fine, n_coarse, iters, seed, init_fine, init_coarse, (hipStream_t)stream);
    if (st == MP_EHIP) ctx->has_index = false;      // the launch sequence broke off part-way: no usable index
    return st;
}

mp_status mp_set_clustering(mp_ctx* ctx, const void* k, const void* k_lookup, const void* v, int32_t n_tokens,
                            const int32_t* fine_of_token, int32_t n_fine, const int32_t* coarse_of_fine, int32_t n_coarse,
                            void* stream)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_set_clustering: null context");
    if (!k || !v || !fine_of_token) return fail(ctx, MP_EINVAL, "mp_set_clustering: null pointer");
    if (n_tokens < 1 || n_fine < 1) return fail(ctx, MP_EINVAL, "mp_set_clustering: n_tokens and n_fine must be >= 1");
    if (n_tokens > ctx->Ncap) return fail(ctx, MP_ECAPACITY, "mp_set_clustering: n_tokens %d > max_tokens %d", n_tokens, ctx->Ncap);
    if (n_fine > ctx->Fcap) return fail(ctx, MP_ECAPACITY, "mp_set_clustering: n_fine %d > max_fine %d", n_fine, ctx->Fcap);
    if (ctx->cfg.levels == 2) {
        if (!coarse_of_fine || n_coarse < 1) return fail(ctx, MP_EINVAL, "mp_set_clustering: two levels need coarse_of_fine and n_coarse >= 1");
        if (n_coarse > ctx->Ccap) return fail(ctx, MP_ECAPACITY, "mp_set_clustering: n_coarse %d > max_coarse %d", n_coarse, ctx->Ccap);
    } else {
        n_coarse = 0;
    }
    if (!lookup_arg_ok(ctx, k_lookup)) return fail(ctx, MP_EINVAL, "mp_set_clustering: k_lookup must be given exactly when the context was created with lookup_keys");
    const mp_status st = set_clustering_impl(ctx, k, k_lookup, v, n_tokens, fine_of_token, n_fine, coarse_of_fine, n_coarse, (hipStream_t)stream);
    if (st == MP_EHIP) ctx->has_index = false;
    return st;
}

int32_t mp_update_seed_counts(const mp_ctx* ctx, int32_t n_new, int32_t n_new_fine, int32_t n_new_coarse, int32_t* counts)
{
    if (!ctx || !counts || !ctx->has_index || n_new < 1 || n_new_fine < 0 || n_new_coarse < 0) return -1;
    update_seed_counts(ctx, n_new, n_new_fine, n_new_coarse, counts);
    int32_t t = 0;
    for (int i = 0; i < 6; ++i) t += counts[i];
    return t;
}

mp_status mp_update_clusters(mp_ctx* ctx, const void* k_new, const void* k_new_lookup, const void* v_new, int32_t n_new,
                             int32_t n_new_fine, int32_t n_new_coarse, int32_t refine_iters, int32_t split_iters,
                             uint64_t seed, const int32_t* seeds, void* stream)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_update_clusters: null context");
    if (!ctx->has_index) return fail(ctx, MP_ESTATE, "mp_update_clusters: no index yet (call mp_cluster_kv first)");
    if (!k_new || !v_new) return fail(ctx, MP_EINVAL, "mp_update_clusters: null k_new/v_new");
    if (n_new < 1 || n_new_fine < 0 || n_new_fine > n_new || refine_iters < 0 || split_iters < 1)
        return fail(ctx, MP_EINVAL, "mp_update_clusters: bad counts n_new=%d n_new_fine=%d refine=%d split=%d", n_new, n_new_fine,
                    refine_iters, split_iters);
    if (ctx->cfg.levels == 2 && (n_new_coarse < 0 || n_new_coarse > n_new_fine))
        return fail(ctx, MP_EINVAL, "mp_update_clusters: n_new_coarse must be in [0, n_new_fine]");
    if (!lookup_arg_ok(ctx, k_new_lookup)) return fail(ctx, MP_EINVAL, "mp_update_clusters: k_new_lookup must be given exactly when the context was created with lookup_keys");
    const mp_status st = update_clusters_impl(ctx, k_new, k_new_lookup, v_new, n_new, n_new_fine, ctx->cfg.levels == 2 ? n_new_coarse : 0,
                                              refine_iters, split_iters, seed, seeds, (hipStream_t)stream);
    if (st == MP_EHIP) ctx->has_index = false;      // the launch sequence broke off part-way: no usable index
    return st;
}

}  // extern "C"

namespace {
// Rows that join the tail buffers at the start of a step (see ScoreParams::app_*).
struct AppendRows {
    int n = 0;
    const void* src[3] = {nullptr, nullptr, nullptr};
    void* dst[3] = {nullptr, nullptr, nullptr};
    long long dst_rows = 0;
    int row = 0;
};
}  // namespace

static mp_status decode_impl(mp_ctx* ctx, const void* q, const void* q_lookup, const void* k_tail, const void* v_tail,
                             int32_t n_tail, int32_t tail_stride, int32_t key_budget, int32_t coarse_budget, uint32_t flags,
                             void* out, float* lse, void* stream, const AppendRows* app)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_decode_attention: null context");
    if (!ctx->has_index) return fail(ctx, MP_ESTATE, "mp_decode_attention: no index yet (call mp_cluster_kv first)");
    if (!q || !out) return fail(ctx, MP_EINVAL, "mp_decode_attention: null q/out");
    if (n_tail < 0 || key_budget < 0 || coarse_budget < 0) return fail(ctx, MP_EINVAL, "mp_decode_attention: negative size or budget");
    if (n_tail > 0 && (!k_tail || !v_tail)) return fail(ctx, MP_EINVAL, "mp_decode_attention: null tail with n_tail > 0");
    if (tail_stride != 0 && tail_stride < n_tail) return fail(ctx, MP_EINVAL, "mp_decode_attention: tail_stride %d < n_tail %d", tail_stride, n_tail);
    if (n_tail > ctx->Tcap) return fail(ctx, MP_ECAPACITY, "mp_decode_attention: n_tail %d > max_tail %d", n_tail, ctx->Tcap);
    if (flags & ~MP_DECODE_NO_MULTIPOLE) return fail(ctx, MP_EINVAL, "mp_decode_attention: unknown flags 0x%x", flags);
    if (q_lookup && ctx->cfg.kv_format == MP_KV_E4M3)
        return fail(ctx, MP_EINVAL, "mp_decode_attention: a lookup query cannot be combined with 8-bit keys (residuals from the centroids q itself must meet)");
    hipStream_t s = (hipStream_t)stream;
    const int U = ctx->U, G = ctx->G;
    const bool two = ctx->cfg.levels == 2;
    const int use_mp = (flags & MP_DECODE_NO_MULTIPOLE) ? 0 : 1;

    ScoreParams sp{};
    sp.q = (const uint16_t*)(q_lookup ? q_lookup : q); sp.Kc = ctx->Kc; sp.N = ctx->Ncl; sp.tab_rows = ctx->tab_rows; sp.fcap = ctx->Fcap;
    sp.levels = ctx->cfg.levels; sp.n_fine = ctx->n_fine; sp.n_coarse = ctx->n_coarse;
    sp.key_budget = key_budget; sp.coarse_budget = coarse_budget; sp.scale = ctx->scale_d;
    sp.cstart = ctx->cstart; sp.cstart_stride = ctx->Ccap + 1; sp.fstart = ctx->fstart; sp.fstart_stride = ctx->Fcap + 1;
    sp.lg = ctx->lg; sp.lg_stride = ctx->Lcap; sp.g_keys = ctx->sc_keys; sp.g_wts = ctx->sc_wts; sp.g_ids = ctx->sc_ids;
    sp.g_aux = ctx->sc_aux; sp.g_aux2 = ctx->sc_aux2; sp.g_flags = ctx->sc_flags; sp.g_stride = ctx->Lcap;
    sp.key_c = ctx->key_c; sp.flag_c = ctx->flag_c; sp.c_stride = std::max(ctx->Ccap, 1);
    sp.key_f = ctx->key_f; sp.key_mode = ctx->key_mode; sp.flag_f = ctx->flag_f; sp.f_stride = ctx->Fcap; sp.cand = ctx->cand; sp.n_cand = ctx->n_cand;
    sp.rows = ctx->rows; sp.rows_stride = ctx->Ncap; sp.n_rows = ctx->n_rows;
    sp.sel_base = ctx->sel_base; sp.row_slot = ctx->row_slot;     // (null unless the keys are stored as residuals)
    sp.mp_rows = ctx->mp_rows; sp.mp_scores = ctx->mp_scores; sp.mp_stride = ctx->tab_rows; sp.n_mp = ctx->n_mp;
    sp.use_mp = use_mp; sp.counters = ctx->counters; sp.n_tail = n_tail;
    sp.lds_cap = std::min(1024, std::max(ctx->n_fine, std::max(ctx->n_coarse, 1)));
    sp.G = G; sp.U = U;
    if (app) {
        sp.app_n = app->n; sp.app_dst_rows = app->dst_rows; sp.app_row = app->row;
        for (int a = 0; a < app->n; ++a) { sp.app_src[a] = app->src[a]; sp.app_dst[a] = app->dst[a]; }
    }
    // the plan of the value pass first: every check that can fail is made before anything is enqueued

    ValuePassParams vp{};
    vp.q = (const uint16_t*)q;
    vp.partials = ctx->partials;
    vp.n_units = U;
    vp.scale_log2e = (float)(ctx->scale_d * 1.4426950408889634);
    const int main_max = std::min(key_budget, ctx->n_tokens);
    int ns = 0, chunk0 = 0;
    // order: centroid terms, tail, selected keys -- the longest stream goes last (see the kernel's block mapping)
    // The centroid terms ride along with the selected keys where there are any: shared out over that
    // stream's workgroups they cost each a few per cent more rows, instead of workgroups of their own -- most of
    // them empty, since only the host-known upper bound of their number can size the grid -- that take their
    // turn on the compute units before the long streams start.
    const bool terms_ride = use_mp && main_max > 0;
    int terms_src = -1;         // (the terms are the launch's first source: what a rider has to be)
    if (use_mp) {
        const int mp_max = ctx->n_fine + ctx->n_coarse;
        const int cr = pick_stream_chunk_rows(mp_max, U, 512);
        terms_src = ns;
        RowSource& r = vp.src[ns++];
        r.K = nullptr; r.V = ctx->Vc; r.unit_rows = ctx->tab_rows; r.rows = ctx->mp_rows; r.rows_stride = ctx->tab_rows;
        r.count_dev = ctx->n_mp; r.count_max = mp_max; r.scores = ctx->mp_scores; r.chunk0 = chunk0;
        r.chunk_rows = cr; r.row0 = 0; r.n_chunks = terms_ride ? 0 : ceil_div(mp_max, cr); chunk0 += r.n_chunks;
    }
    if (n_tail > 0) {
        const int cr = pick_stream_chunk_rows(n_tail, U, 512);
        RowSource& r = vp.src[ns++];
        r.K = (const uint16_t*)k_tail; r.V = (const uint16_t*)v_tail; r.unit_rows = tail_stride ? tail_stride : n_tail; r.rows = nullptr; r.rows_stride = 0;
        r.count_dev = nullptr; r.count_max = n_tail; r.scores = nullptr; r.chunk0 = chunk0;
        r.chunk_rows = cr; r.row0 = 0; r.n_chunks = ceil_div(n_tail, cr); chunk0 += r.n_chunks;
    }
    if (main_max > 0) {
        const int crm = pick_stream_chunk_rows(main_max, U, 2048);
        RowSource& r = vp.src[ns++];
        if (ctx->cfg.kv_format == MP_KV_E4M3) {
            r.K = (const uint16_t*)ctx->Kq; r.V = (const uint16_t*)ctx->Vq; r.row_scale = ctx->kv_scale;
            r.row_slot = ctx->row_slot; r.slot_base = ctx->sel_base; r.base_stride = ctx->Fcap;
        }
        else { r.K = ctx->Kp; r.V = ctx->Vp; }
        r.unit_rows = ctx->Ncap; r.rows = ctx->rows; r.rows_stride = ctx->Ncap;
        r.count_dev = ctx->n_rows; r.count_max = main_max; r.scores = nullptr; r.chunk0 = chunk0;
        r.chunk_rows = crm; r.row0 = 0; r.n_chunks = ceil_div(main_max, crm); chunk0 += r.n_chunks;
        r.guest = (terms_ride && terms_src == 0) ? 1 : 0;
    }
    vp.n_sources = ns;
    vp.chunks_per_unit = chunk0;
    if (chunk0 > ctx->Pcap) return fail(ctx, MP_ECAPACITY, "mp_decode_attention: %d chunks > workspace %d", chunk0, ctx->Pcap);
    if (ctx->timing) MP_HIP(ctx, hipEventRecord(ctx->ev[0], s));
    if (ctx->timing) MP_HIP(ctx, hipEventRecord(ctx->ev[1], s));
    MP_HIP(ctx, launch_score_select(sp, ctx->n_cus, s));
    if (ctx->timing) MP_HIP(ctx, hipEventRecord(ctx->ev[2], s));
    if (chunk0 > 0) MP_HIP(ctx, launch_value_pass(vp, G, s));
    if (ctx->timing) MP_HIP(ctx, hipEventRecord(ctx->ev[3], s));
    MP_HIP(ctx, launch_merge(ctx->partials, U, chunk0, G, (uint16_t*)out, lse, s));
    if (ctx->timing) MP_HIP(ctx, hipEventRecord(ctx->ev[4], s));
    ctx->timed_levels = two ? 2 : 1;
    ctx->decoded = true;
    return MP_OK;
}

extern "C" {

mp_status mp_decode_attention(mp_ctx* ctx, const void* q, const void* q_lookup, const void* k_tail, const void* v_tail,
                              int32_t n_tail, int32_t tail_stride,
                              int32_t key_budget, int32_t coarse_budget, uint32_t flags, void* out, float* lse, void* stream)
{
    return decode_impl(ctx, q, q_lookup, k_tail, v_tail, n_tail, tail_stride, key_budget, coarse_budget, flags, out, lse,
                       stream, nullptr);
}

// ------------------------------------------------------------------------------------------------
// Library-managed local buffer (Sec. 4: the newest L .. 2L tokens stay unclustered and are attended
// exactly; every L steps the oldest L of them go into the clusters) and sink tokens
// ------------------------------------------------------------------------------------------------
mp_status mp_local_buffer_init(mp_ctx* ctx, int32_t window, const void* k_sink, const void* v_sink, int32_t n_sink,
                               const void* k_recent, const void* k_recent_lookup, const void* v_recent, int32_t n_recent,
                               void* stream)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_local_buffer_init: null context");
    if (window < 1 || n_sink < 0 || n_recent < 0 || n_recent >= 2 * window)
        return fail(ctx, MP_EINVAL, "mp_local_buffer_init: need window >= 1, n_sink >= 0, 0 <= n_recent < 2 * window");
    if ((n_sink > 0 && (!k_sink || !v_sink)) || (n_recent > 0 && (!k_recent || !v_recent)))
        return fail(ctx, MP_EINVAL, "mp_local_buffer_init: null rows with a positive count");
    if (n_recent > 0 && !lookup_arg_ok(ctx, k_recent_lookup))
        return fail(ctx, MP_EINVAL, "mp_local_buffer_init: k_recent_lookup must be given exactly when the context was created with lookup_keys");
    if ((long long)n_sink + 2ll * window > ctx->Tcap)
        return fail(ctx, MP_ECAPACITY, "mp_local_buffer_init: n_sink + 2 * window = %lld > max_tail %d", (long long)n_sink + 2ll * window, ctx->Tcap);
    hipStream_t s = (hipStream_t)stream;
    const size_t row = kHeadDimHost * sizeof(uint16_t), pitch = (size_t)ctx->Tcap * row;
    if (n_sink > 0) {
        MP_HIP(ctx, hipMemcpy2DAsync(ctx->Kt, pitch, k_sink, n_sink * row, n_sink * row, ctx->U, hipMemcpyDeviceToDevice, s));
        MP_HIP(ctx, hipMemcpy2DAsync(ctx->Vt, pitch, v_sink, n_sink * row, n_sink * row, ctx->U, hipMemcpyDeviceToDevice, s));
    }
    if (n_recent > 0) {
        MP_HIP(ctx, hipMemcpy2DAsync((char*)ctx->Kt + n_sink * row, pitch, k_recent, n_recent * row, n_recent * row, ctx->U, hipMemcpyDeviceToDevice, s));
        MP_HIP(ctx, hipMemcpy2DAsync((char*)ctx->Vt + n_sink * row, pitch, v_recent, n_recent * row, n_recent * row, ctx->U, hipMemcpyDeviceToDevice, s));
        if (k_recent_lookup)
            MP_HIP(ctx, hipMemcpy2DAsync((char*)ctx->Ktl + n_sink * row, pitch, k_recent_lookup, n_recent * row, n_recent * row, ctx->U, hipMemcpyDeviceToDevice, s));
    }
    ctx->lb_window = window;
    ctx->lb_sink = n_sink;
    ctx->lb_recent = n_recent;
    return MP_OK;
}

mp_status mp_local_buffer_size(const mp_ctx* ctx, int32_t* window, int32_t* n_sink, int32_t* n_recent)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_local_buffer_size: null context");
    if (ctx->lb_window == 0) return fail(const_cast<mp_ctx*>(ctx), MP_ESTATE, "mp_local_buffer_size: no local buffer (call mp_local_buffer_init first)");
    if (window) *window = ctx->lb_window;
    if (n_sink) *n_sink = ctx->lb_sink;
    if (n_recent) *n_recent = ctx->lb_recent;
    return MP_OK;
}

namespace {
// The oldest L tokens of the local buffer go into the clusters; the newer L move down.
mp_status refresh_local_buffer(mp_ctx* ctx, int32_t n_new_fine, int32_t n_new_coarse, int32_t refine_iters,
                               int32_t split_iters, uint64_t seed, const int32_t* seeds, hipStream_t s)
{
    const int L = ctx->lb_window, ns = ctx->lb_sink;
    if (n_new_fine < 0 || n_new_fine > L || refine_iters < 0 || split_iters < 1)
        return fail(ctx, MP_EINVAL, "mp_decode_step: bad update counts n_new_fine=%d refine=%d split=%d", n_new_fine, refine_iters, split_iters);
    if (ctx->cfg.levels == 2 && (n_new_coarse < 0 || n_new_coarse > n_new_fine))
        return fail(ctx, MP_EINVAL, "mp_decode_step: n_new_coarse must be in [0, n_new_fine]");
    const size_t row = kHeadDimHost * sizeof(uint16_t), pitch = (size_t)ctx->Tcap * row;
    MP_HIP(ctx, hipMemcpy2DAsync(ctx->Kts, L * row, (char*)ctx->Kt + ns * row, pitch, L * row, ctx->U, hipMemcpyDeviceToDevice, s));
    MP_HIP(ctx, hipMemcpy2DAsync(ctx->Vts, L * row, (char*)ctx->Vt + ns * row, pitch, L * row, ctx->U, hipMemcpyDeviceToDevice, s));
    const bool lookup = ctx->cfg.lookup_keys != 0;
    if (lookup)
        MP_HIP(ctx, hipMemcpy2DAsync(ctx->Ktls, L * row, (char*)ctx->Ktl + ns * row, pitch, L * row, ctx->U, hipMemcpyDeviceToDevice, s));
    const mp_status st = update_clusters_impl(ctx, ctx->Kts, lookup ? ctx->Ktls : nullptr, ctx->Vts, L, n_new_fine,
                                              ctx->cfg.levels == 2 ? n_new_coarse : 0, refine_iters, split_iters, seed, seeds, s);
    if (st != MP_OK) return st;
    if (lookup)
        MP_HIP(ctx, hipMemcpy2DAsync((char*)ctx->Ktl + ns * row, pitch, (char*)ctx->Ktl + (ns + L) * row, pitch, L * row, ctx->U, hipMemcpyDeviceToDevice, s));
    MP_HIP(ctx, hipMemcpy2DAsync((char*)ctx->Kt + ns * row, pitch, (char*)ctx->Kt + (ns + L) * row, pitch, L * row, ctx->U, hipMemcpyDeviceToDevice, s));
    MP_HIP(ctx, hipMemcpy2DAsync((char*)ctx->Vt + ns * row, pitch, (char*)ctx->Vt + (ns + L) * row, pitch, L * row, ctx->U, hipMemcpyDeviceToDevice, s));
    ctx->lb_recent = L;
    return MP_OK;
}
}  // namespace

mp_status mp_decode_step(mp_ctx* ctx, const void* q, const void* q_lookup, const void* k_new, const void* k_new_lookup,
                         const void* v_new, int32_t key_budget, int32_t coarse_budget, uint32_t flags, int32_t n_new_fine,
                         int32_t n_new_coarse, int32_t refine_iters, int32_t split_iters, uint64_t seed,
                         const int32_t* seeds, void* out, float* lse, void* stream)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_decode_step: null context");
    if (!ctx->has_index) return fail(ctx, MP_ESTATE, "mp_decode_step: no index yet (call mp_cluster_kv first)");
    if (ctx->lb_window == 0) return fail(ctx, MP_ESTATE, "mp_decode_step: no local buffer (call mp_local_buffer_init first)");
    if (!q || !k_new || !v_new || !out) return fail(ctx, MP_EINVAL, "mp_decode_step: null q/k_new/v_new/out");
    if (!lookup_arg_ok(ctx, k_new_lookup)) return fail(ctx, MP_EINVAL, "mp_decode_step: k_new_lookup must be given exactly when the context was created with lookup_keys");
    hipStream_t s = (hipStream_t)stream;
    const int L = ctx->lb_window, ns = ctx->lb_sink;
    if (ctx->lb_recent >= 2 * L) {      // a refresh that failed in an earlier call (e.g. capacity) is due first
        const mp_status st = refresh_local_buffer(ctx, n_new_fine, n_new_coarse, refine_iters, split_iters, seed, seeds, s);
        if (st != MP_OK) return st;
    }
    // the new token joins the buffer first (a decoding step attends to its own key and value): the
    // scoring launch of the step copies its rows in, one launch less than a copy of its own
    AppendRows app;
    app.dst_rows = ctx->Tcap; app.row = ns + ctx->lb_recent;
    app.src[app.n] = k_new; app.dst[app.n++] = ctx->Kt;
    app.src[app.n] = v_new; app.dst[app.n++] = ctx->Vt;
    if (k_new_lookup) { app.src[app.n] = k_new_lookup; app.dst[app.n++] = ctx->Ktl; }
    ctx->lb_recent += 1;
    const mp_status st = decode_impl(ctx, q, q_lookup, ctx->Kt, ctx->Vt, ns + ctx->lb_recent, ctx->Tcap, key_budget,
                                     coarse_budget, flags, out, lse, stream, &app);
    if (st != MP_OK) {
        ctx->lb_recent -= 1;
        return st;
    }
    if (ctx->lb_recent == 2 * L)
        return refresh_local_buffer(ctx, n_new_fine, n_new_coarse, refine_iters, split_iters, seed, seeds, s);
    return MP_OK;
}

// ------------------------------------------------------------------------------------------------
// Stage timing
// ------------------------------------------------------------------------------------------------
mp_status mp_enable_stage_timing(mp_ctx* ctx, int32_t enable)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_enable_stage_timing: null context");
    if (enable && !ctx->ev[0])
        for (hipEvent_t& e : ctx->ev) MP_HIP(ctx, hipEventCreate(&e));
    ctx->timing = enable != 0;
    ctx->timed_levels = 0;
    return MP_OK;
}

mp_status mp_get_stage_timing(mp_ctx* ctx, float* ms)
{
    if (!ctx || !ms) return fail(ctx, MP_EINVAL, "mp_get_stage_timing: null pointer");
    if (!ctx->timing || !ctx->timed_levels) return fail(ctx, MP_ESTATE, "mp_get_stage_timing: no timed decode call yet");
    MP_HIP(ctx, hipEventSynchronize(ctx->ev[4]));
    ms[0] = 0.f;
    MP_HIP(ctx, hipEventElapsedTime(&ms[1], ctx->ev[1], ctx->ev[2]));
    MP_HIP(ctx, hipEventElapsedTime(&ms[2], ctx->ev[2], ctx->ev[3]));
    MP_HIP(ctx, hipEventElapsedTime(&ms[3], ctx->ev[3], ctx->ev[4]));
    return MP_OK;
}

// ------------------------------------------------------------------------------------------------
// Introspection
// ------------------------------------------------------------------------------------------------
mp_status mp_get_sizes(const mp_ctx* ctx, int32_t* n_tokens, int32_t* n_fine, int32_t* n_coarse, int32_t* n_blocks)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_get_sizes: null context");
    if (!ctx->has_index) return fail(const_cast<mp_ctx*>(ctx), MP_ESTATE, "mp_get_sizes: no index yet");
    if (n_tokens) *n_tokens = ctx->n_tokens;
    if (n_fine) *n_fine = ctx->n_fine;
    if (n_coarse) *n_coarse = ctx->n_coarse;
    if (n_blocks) *n_blocks = (int32_t)ctx->blocks.size();
    return MP_OK;
}

mp_status mp_get_assignments(mp_ctx* ctx, int32_t* fine_of_token, int32_t* coarse_of_fine, void* stream)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_get_assignments: null context");
    if (!ctx->has_index) return fail(ctx, MP_ESTATE, "mp_get_assignments: no index yet");
    hipStream_t s = (hipStream_t)stream;
    if (fine_of_token)
        MP_HIP(ctx, hipMemcpy2DAsync(fine_of_token, (size_t)ctx->n_tokens * 4, ctx->fot, (size_t)ctx->Ncap * 4,
                                     (size_t)ctx->n_tokens * 4, ctx->U, hipMemcpyDeviceToDevice, s));
    if (coarse_of_fine && ctx->cfg.levels == 2)
        MP_HIP(ctx, hipMemcpy2DAsync(coarse_of_fine, (size_t)ctx->n_fine * 4, ctx->cof, (size_t)ctx->Fcap * 4,
                                     (size_t)ctx->n_fine * 4, ctx->U, hipMemcpyDeviceToDevice, s));
    return MP_OK;
}

mp_status mp_get_centroids(mp_ctx* ctx, int32_t level, void* kc, void* vc, int32_t* n_members, void* stream)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_get_centroids: null context");
    if (!ctx->has_index) return fail(ctx, MP_ESTATE, "mp_get_centroids: no index yet");
    if (level != 0 && !(level == 1 && ctx->cfg.levels == 2)) return fail(ctx, MP_EINVAL, "mp_get_centroids: no level %d", level);
    hipStream_t s = (hipStream_t)stream;
    const int n = level == 0 ? ctx->n_fine : ctx->n_coarse;
    const size_t off = level == 0 ? 0 : (size_t)ctx->Fcap;
    const size_t row = kHeadDimHost * 2;
    if (kc)
        MP_HIP(ctx, hipMemcpy2DAsync(kc, n * row, (const char*)ctx->Kc + off * row, (size_t)ctx->tab_rows * row, n * row, ctx->U,
                                     hipMemcpyDeviceToDevice, s));
    if (vc)
        MP_HIP(ctx, hipMemcpy2DAsync(vc, n * row, (const char*)ctx->Vc + off * row, (size_t)ctx->tab_rows * row, n * row, ctx->U,
                                     hipMemcpyDeviceToDevice, s));
    if (n_members)
        MP_HIP(ctx, hipMemcpy2DAsync(n_members, (size_t)n * 4, ctx->Ncl + off, (size_t)ctx->tab_rows * 4, (size_t)n * 4, ctx->U,
                                     hipMemcpyDeviceToDevice, s));
    return MP_OK;
}

mp_status mp_get_selection(mp_ctx* ctx, uint8_t* fine_selected, uint8_t* coarse_promising, double* r_fine, double* r_coarse,
                           void* stream)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_get_selection: null context");
    if (!ctx->has_index || !ctx->decoded) return fail(ctx, MP_ESTATE, "mp_get_selection: no decode call on this index yet");
    hipStream_t s = (hipStream_t)stream;
    const bool two = ctx->cfg.levels == 2;
    if (fine_selected || r_fine)
        MP_HIP(ctx, launch_scatter_selection(two ? ctx->cand : nullptr, ctx->Fcap, two ? ctx->n_cand : nullptr, ctx->n_fine,
                                             ctx->flag_f, ctx->key_f, ctx->key_mode, 1, ctx->G, ctx->Fcap, ctx->n_fine, ctx->U,
                                             fine_selected, r_fine, s));
    if (two && (coarse_promising || r_coarse))
        MP_HIP(ctx, launch_scatter_selection(nullptr, 0, nullptr, ctx->n_coarse, ctx->flag_c, ctx->key_c, ctx->key_mode, 0, ctx->G,
                                             std::max(ctx->Ccap, 1), ctx->n_coarse, ctx->U, coarse_promising, r_coarse, s));
    return MP_OK;
}

mp_status mp_get_counters(mp_ctx* ctx, int32_t* counters, void* stream)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_get_counters: null context");
    if (!counters) return fail(ctx, MP_EINVAL, "mp_get_counters: null pointer");
    if (!ctx->has_index || !ctx->decoded) return fail(ctx, MP_ESTATE, "mp_get_counters: no decode call on this index yet");
    MP_HIP(ctx, hipMemcpyAsync(counters, ctx->counters, (size_t)ctx->U * 4 * sizeof(int32_t), hipMemcpyDeviceToDevice,
                               (hipStream_t)stream));
    return MP_OK;
}

mp_status mp_get_layout(mp_ctx* ctx, void* k_perm, void* v_perm, int32_t* perm, int32_t* fine_start, void* stream)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_get_layout: null context");
    if (!ctx->has_index) return fail(ctx, MP_ESTATE, "mp_get_layout: no index yet");
    if (ctx->cfg.kv_format != MP_KV_BF16 && (k_perm || v_perm))
        return fail(ctx, MP_EINVAL, "mp_get_layout: this context stores 8-bit rows (use mp_get_kv_codes)");
    hipStream_t s = (hipStream_t)stream;
    const size_t row = kHeadDimHost * 2, n = ctx->n_tokens;
    if (k_perm)
        MP_HIP(ctx, hipMemcpy2DAsync(k_perm, n * row, ctx->Kp, (size_t)ctx->Ncap * row, n * row, ctx->U, hipMemcpyDeviceToDevice, s));
    if (v_perm)
        MP_HIP(ctx, hipMemcpy2DAsync(v_perm, n * row, ctx->Vp, (size_t)ctx->Ncap * row, n * row, ctx->U, hipMemcpyDeviceToDevice, s));
    if (perm)
        MP_HIP(ctx, hipMemcpy2DAsync(perm, n * 4, ctx->perm, (size_t)ctx->Ncap * 4, n * 4, ctx->U, hipMemcpyDeviceToDevice, s));
    if (fine_start)
        MP_HIP(ctx, hipMemcpy2DAsync(fine_start, (size_t)(ctx->n_fine + 1) * 4, ctx->fstart, (size_t)(ctx->Fcap + 1) * 4,
                                     (size_t)(ctx->n_fine + 1) * 4, ctx->U, hipMemcpyDeviceToDevice, s));
    return MP_OK;
}

mp_status mp_get_kv_codes(mp_ctx* ctx, void* k_codes, void* v_codes, float* scales, void* stream)
{
    if (!ctx) return fail(nullptr, MP_EINVAL, "mp_get_kv_codes: null context");
    if (ctx->cfg.kv_format != MP_KV_E4M3) return fail(ctx, MP_EINVAL, "mp_get_kv_codes: this context does not store 8-bit rows");
    if (!ctx->has_index) return fail(ctx, MP_ESTATE, "mp_get_kv_codes: no index yet");
    hipStream_t s = (hipStream_t)stream;
    const size_t row = kHeadDimHost, n = ctx->n_tokens;
    if (k_codes)
        MP_HIP(ctx, hipMemcpy2DAsync(k_codes, n * row, ctx->Kq, (size_t)ctx->Ncap * row, n * row, ctx->U, hipMemcpyDeviceToDevice, s));
    if (v_codes)
        MP_HIP(ctx, hipMemcpy2DAsync(v_codes, n * row, ctx->Vq, (size_t)ctx->Ncap * row, n * row, ctx->U, hipMemcpyDeviceToDevice, s));
    if (scales)
        MP_HIP(ctx, hipMemcpy2DAsync(scales, n * 8, ctx->kv_scale, (size_t)ctx->Ncap * 8, n * 8, ctx->U, hipMemcpyDeviceToDevice, s));
    return MP_OK;
}

// ------------------------------------------------------------------------------------------------
// Dense comparison kernel
// ------------------------------------------------------------------------------------------------
size_t mp_dense_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t n)
{
    if (batch <= 0 || n_q_heads <= 0 || n_kv_heads <= 0 || n < 0 || n_q_heads % n_kv_heads) return 0;
    const int U = batch * n_kv_heads, G = n_q_heads / n_kv_heads;
    const int cr = pick_chunk_rows(n, U);
    const int chunks = ceil_div(n > 0 ? n : 1, cr);
    return sizeof(float) * (size_t)U * chunks * G * kPartStride;
}

}  // extern "C"

namespace {

// Split-KV launch sequence of the dense kernel; `partials` holds mp_dense_workspace_bytes() bytes.
mp_status dense_impl(const char* who, const void* q, const void* k, const void* v, int32_t batch, int32_t n_q_heads,
                     int32_t n_kv_heads, int32_t n, float softmax_scale, void* out, float* lse, float* partials,
                     hipStream_t s)
{
    const int U = batch * n_kv_heads, G = n_q_heads / n_kv_heads;
    const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)kHeadDimHost);
    ValuePassParams p{};
    p.q = (const uint16_t*)q;
    p.partials = partials;
    p.n_units = U;
    const int dcr = pick_chunk_rows(n, U);
    p.chunks_per_unit = ceil_div(n > 0 ? n : 1, dcr);
    p.src[0].chunk_rows = dcr;
    p.src[0].row0 = 0;
    p.n_sources = 1;
    p.scale_log2e = scale * 1.4426950408889634f;
    p.src[0].K = (const uint16_t*)k;
    p.src[0].V = (const uint16_t*)v;
    p.src[0].unit_rows = n;
    p.src[0].count_max = n;
    p.src[0].chunk0 = 0;
    p.src[0].n_chunks = p.chunks_per_unit;
    hipError_t e = launch_value_pass(p, G, s);
    if (e == hipSuccess) e = launch_merge(p.partials, U, p.chunks_per_unit, G, (uint16_t*)out, lse, s);
    if (e != hipSuccess) return fail(nullptr, MP_EHIP, "%s: %s", who, hipGetErrorString(e));
    return MP_OK;
}

mp_status dense_args_ok(const char* who, const void* q, const void* k, const void* v, int32_t batch, int32_t n_q_heads,
                        int32_t n_kv_heads, int32_t n, const void* out)
{
    if (!q || !out) return fail(nullptr, MP_EINVAL, "%s: null pointer", who);
    if (batch <= 0 || n_q_heads <= 0 || n_kv_heads <= 0 || n < 0 || n_q_heads % n_kv_heads)
        return fail(nullptr, MP_EINVAL, "%s: bad shape B=%d Hq=%d Hkv=%d n=%d", who, batch, n_q_heads, n_kv_heads, n);
    if (n > 0 && (!k || !v)) return fail(nullptr, MP_EINVAL, "%s: null k/v with n > 0", who);
    if (n_q_heads / n_kv_heads > 8) return fail(nullptr, MP_EINVAL, "%s: group size %d > 8 is not supported", who, n_q_heads / n_kv_heads);
    return MP_OK;
}

// Partial results of mp_dense_attention_static: one array per GPU, part of the library's image on
// that GPU for the life of the process.  Host code never uses the name `scratch` as an address:
// scratch_on_device() asks the runtime for the array's address on the current device once and
// hands out that pointer.
constexpr size_t kStaticScratchBytes = MP_DENSE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

hipError_t scratch_on_device(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

namespace mp {
// The library's set-up call (mp_create) resolves the array on its device, so that a later
// mp_dense_attention_static on that device makes no runtime query at all.
hipError_t resolve_static_scratch()
{
    void* p = nullptr;
    return scratch_on_device(&p);
}
}  // namespace mp

extern "C" {

mp_status mp_dense_attention(const void* q, const void* k, const void* v, int32_t batch, int32_t n_q_heads,
                             int32_t n_kv_heads, int32_t n, float softmax_scale, void* out, float* lse, void* workspace,
                             size_t workspace_bytes, void* stream)
{
    if (!workspace) return fail(nullptr, MP_EINVAL, "mp_dense_attention: null pointer");
    const mp_status st = dense_args_ok("mp_dense_attention", q, k, v, batch, n_q_heads, n_kv_heads, n, out);
    if (st != MP_OK) return st;
    const size_t need = mp_dense_workspace_bytes(batch, n_q_heads, n_kv_heads, n);
    if (workspace_bytes < need) return fail(nullptr, MP_EINVAL, "mp_dense_attention: workspace %zu < %zu bytes", workspace_bytes, need);
    return dense_impl("mp_dense_attention", q, k, v, batch, n_q_heads, n_kv_heads, n, softmax_scale, out, lse,
                      (float*)workspace, (hipStream_t)stream);
}

size_t mp_dense_static_scratch_bytes(void) { return kStaticScratchBytes; }

mp_status mp_dense_attention_static(const void* q, const void* k, const void* v, int32_t batch, int32_t n_q_heads,
                                    int32_t n_kv_heads, int32_t n, float softmax_scale, void* out, float* lse, void* stream)
{
    const mp_status st = dense_args_ok("mp_dense_attention_static", q, k, v, batch, n_q_heads, n_kv_heads, n, out);
    if (st != MP_OK) return st;
    const size_t need = mp_dense_workspace_bytes(batch, n_q_heads, n_kv_heads, n);
    if (need > kStaticScratchBytes)
        return fail(nullptr, MP_ECAPACITY, "mp_dense_attention_static: this shape needs %zu bytes of partial results, the built-in "
                    "scratch array holds %zu (use mp_dense_attention with a workspace)", need, kStaticScratchBytes);
    void* base = nullptr;
    const hipError_t e = scratch_on_device(&base);
    if (e != hipSuccess) return fail(nullptr, MP_EHIP, "mp_dense_attention_static: hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    // every chunk of every unit writes its partial (an empty chunk writes an empty one) before the
    // merge reads it, so nothing of the previous call's contents is ever read: no clearing needed
    return dense_impl("mp_dense_attention_static", q, k, v, batch, n_q_heads, n_kv_heads, n, softmax_scale, out, lse,
                      (float*)base, (hipStream_t)stream);
}

}  // extern "C"
