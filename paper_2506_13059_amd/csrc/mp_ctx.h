// The context object behind the opaque mp_ctx handle, and small host-side helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/mp.h"

namespace mp {

constexpr int kHeadDimHost = 128;
constexpr int kMaxClustersPerLevel = 8192;   // candidates of one level must fit the scoring kernel's LDS

// Token / cluster ranges of one clustering block (Sec. 3.3).
struct BlockPlan {
    int32_t t0, t1;   // tokens
    int32_t f0, f1;   // fine cluster ids
    int32_t c0, c1;   // coarse cluster ids
};

// Blocks of block_w tokens; the last one takes the remaining block_alpha .. block_w+block_alpha-1
// tokens.  Cluster totals are split by cumulative integer division.
inline std::vector<BlockPlan> plan_blocks(int32_t n_tokens, int32_t block_w, int32_t block_alpha, int32_t n_fine,
                                          int32_t n_coarse)
{
    std::vector<int32_t> bounds;
    bounds.push_back(0);
    if (block_w > 0 && n_tokens >= block_w + block_alpha) {
        const int32_t m = (n_tokens - block_alpha) / block_w;
        for (int32_t i = 1; i <= m; ++i) bounds.push_back(i * block_w);
    }
    if (bounds.back() != n_tokens) bounds.push_back(n_tokens);
    std::vector<BlockPlan> out;
    for (size_t b = 0; b + 1 < bounds.size(); ++b) {
        const long long t0 = bounds[b], t1 = bounds[b + 1];
        BlockPlan p;
        p.t0 = (int32_t)t0;
        p.t1 = (int32_t)t1;
        p.f0 = (int32_t)((long long)n_fine * t0 / n_tokens);
        p.f1 = (int32_t)((long long)n_fine * t1 / n_tokens);
        p.c0 = (int32_t)((long long)n_coarse * t0 / n_tokens);
        p.c1 = (int32_t)((long long)n_coarse * t1 / n_tokens);
        out.push_back(p);
    }
    return out;
}

}  // namespace mp

// The handle of the C ABI.  All device arrays have a leading unit axis; "cap" sizes come from cfg.
struct mp_ctx {
    mp_config cfg{};
    std::string err;
    int device = 0;
    int n_cus = 0;                 // compute units of that device
    int U = 0, G = 0;
    float scale = 0.f;
    double scale_d = 0.0;          // softmax scale in double (0 in cfg => exactly 1/sqrt(128) in fp64)
    size_t device_bytes = 0;
    std::vector<void*> allocs;     // everything to hipFree at destroy

    int32_t Ncap = 0, Fcap = 0, Ccap = 0, Tcap = 0, FBcap = 0;
    long long tab_rows = 0;        // Fcap + Ccap: rows per unit of the centroid tables

    // ---- clustered cache and index tables ----
    uint16_t* Kp = nullptr;        // bf16 [U, Ncap, 128] keys, cluster after cluster
    uint16_t* Vp = nullptr;        // bf16 [U, Ncap, 128]
    // (8-bit storage, cfg.kv_format == MP_KV_E4M3: Kp / Vp stay null and these hold the rows instead)
    uint8_t* Kq = nullptr;         // e4m3 codes [U, Ncap, 128]
    uint8_t* Vq = nullptr;
    float* kv_scale = nullptr;     // fp32 [U, Ncap, 2]: key scale and value scale of each stored row
    float* sel_base = nullptr;     // fp32 [U, Fcap, 8]: q . centroid of the clusters selected by the last decode call
    int32_t* row_slot = nullptr;   // [U, Ncap]: for each entry of `rows`, its cluster's position in sel_base
    int32_t* perm = nullptr;       // [U, Ncap] sequence index of each stored row
    int32_t* fot = nullptr;        // [U, Ncap] fine cluster of each token (sequence order)
    int32_t* fstart = nullptr;     // [U, Fcap+1] first stored row of each fine cluster
    int32_t* cof = nullptr;        // [U, Fcap] coarse cluster of each fine cluster
    int32_t* cstart = nullptr;     // [U, Ccap+1] first fine cluster of each coarse cluster
    double* sumK = nullptr;        // fp64 [U, Fcap, 128] member sums of the fine clusters (two levels: what the coarse
    double* sumV = nullptr;        // tables are added up from); sumK may sit at the ids of before a renumbering
    uint16_t* Kc = nullptr;        // bf16 [U, tab_rows, 128] key centroids: fine rows, coarse rows from Fcap
    uint16_t* Vc = nullptr;        // bf16 [U, tab_rows, 128] value centroids
    int32_t* Ncl = nullptr;        // [U, tab_rows] member counts

    // ---- last block in sequence order (working set of the online update) ----
    uint16_t* Kfb = nullptr;       // bf16 [U, FBcap, 128] keys the clusters are formed on (lookup keys if in use)
    uint16_t* Kfs = nullptr;       // bf16 [U, FBcap, 128] the stored keys of the same tokens (only with lookup keys)
    uint16_t* Vfb = nullptr;

    // ---- k-means workspace ----
    int32_t* km_assign = nullptr;  // [U, Ncap] block-local cluster of each point
    int32_t* km_list = nullptr;    // [U, Ncap] member lists (during an assignment step: points of the exact pass)
    int32_t* km_amb = nullptr;     // [2][U, max_blocks] number of such points per block: two arrays used in turn, the one
    int amb_turn = 0;              // not in use is all zero (see launch_assign)
    int32_t* km_cnt = nullptr;     // [U, tab_rows]
    int32_t* km_start = nullptr;   // [U, tab_rows + 2]
    uint16_t* km_Cf = nullptr;     // bf16 [U, Fcap, 128] fine k-means centroids
    uint16_t* km_Cc = nullptr;     // bf16 [U, Ccap, 128] coarse k-means centroids
    int32_t* km_parent = nullptr;  // [U, Fcap] coarse assignment of the fine centroids
    int32_t* km_plist = nullptr;   // [U, Fcap] fine ids ordered by parent
    int32_t* km_newid = nullptr;   // [U, Fcap]
    int32_t* km_seed_f = nullptr;  // [U, Fcap]
    int32_t* km_seed_c = nullptr;  // [U, Ccap]
    int32_t* blocks_dev = nullptr; // [3][max_blocks][4] block descriptors (fine level, coarse level, scratch)
    int32_t max_blocks = 0;

    // ---- decode workspace ----
    double* lg = nullptr;          // [U, G, Lcap] logits of a level that does not fit LDS (Lcap = max(Fcap, Ccap))
    unsigned long long* sc_keys = nullptr;   // [U, Lcap] and the other per-entry arrays of such a level
    uint32_t* sc_wts = nullptr;
    int32_t* sc_ids = nullptr;
    int32_t* sc_aux = nullptr;
    int32_t* sc_aux2 = nullptr;
    uint8_t* sc_flags = nullptr;
    int32_t Lcap = 0;
    unsigned long long* key_c = nullptr;   // [U, Ccap] keys the coarse clusters were ranked by in the last call
    unsigned long long* key_f = nullptr;   // [U, Fcap] the same for the fine level, by candidate position
    int32_t* key_mode = nullptr;   // [U, 2] what those keys are (see launch_scatter_selection)
    uint8_t* flag_c = nullptr;     // [U, Ccap] promising
    uint8_t* flag_f = nullptr;     // [U, Fcap] selected, by candidate position
    int32_t* cand = nullptr;       // [U, Fcap]
    int32_t* n_cand = nullptr;     // [U]
    double* unprom_lse = nullptr;  // [U, G]
    int32_t* rows = nullptr;       // [U, Ncap] stored rows of the selected keys
    int32_t* n_rows = nullptr;     // [U]
    int32_t* mp_rows = nullptr;    // [U, tab_rows]
    float* mp_scores = nullptr;    // [U, tab_rows, G]
    int32_t* n_mp = nullptr;       // [U]
    int32_t* counters = nullptr;   // [U, 4]
    float* partials = nullptr;     // [U, Pcap, G, 132]
    int32_t Pcap = 0;

    // library-managed local buffer (mp_local_buffer_init / mp_decode_step): rows [0, lb_sink) are sink
    // tokens, rows [lb_sink, lb_sink + lb_recent) the newest tokens in sequence order
    uint16_t* Kt = nullptr;        // bf16 [U, Tcap, 128]
    uint16_t* Vt = nullptr;
    uint16_t* Kts = nullptr;       // bf16 [U, Tcap, 128] staging: the rows handed to the cluster update, packed
    uint16_t* Vts = nullptr;
    uint16_t* Ktl = nullptr;       // lookup keys of the buffered tokens and their staging (only with lookup keys)
    uint16_t* Ktls = nullptr;
    int32_t lb_window = 0, lb_sink = 0, lb_recent = 0;

    // ---- current index (host copies of sizes) ----
    bool has_index = false;
    bool decoded = false;
    bool updatable = false;        // the last block fits Kfb / Vfb
    int32_t n_tokens = 0, n_fine = 0, n_coarse = 0;
    std::vector<mp::BlockPlan> blocks;

    // optional stage timing of mp_decode_attention: events before coarse, fine, value pass, merge, and after
    bool timing = false;
    int timed_levels = 0;
    hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};

    // host staging for small uploads (kept alive until the next call that uploads)
    std::vector<int32_t> stage_blocks, stage_blocks2, stage_seed_f, stage_seed_c;
    // Pinned staging buffer: small host arrays (block descriptors, seed lists) are packed into it
    // and copied from there, so that the copies are asynchronous and the stream never drains for
    // them.  pin_ev marks the last such copy; the next call that stages waits for it first.
    char* pin = nullptr;
    size_t pin_bytes = 0, pin_used = 0;
    hipEvent_t pin_ev = nullptr;
    bool pin_pending = false;
    // Uploads staged there are carried out together, by one kernel that reads the pinned buffer itself
    // (a refresh's four small host-to-device copies took 60 us of idle stream between them).
    struct UploadSeg { void* dst; unsigned long long dpitch, src_off; unsigned width, height; };   // bytes, multiples of 4
    static constexpr int kMaxUploadSegs = 8;
    UploadSeg up_seg[kMaxUploadSegs];
    int n_up = 0;
};

namespace mp {
// Record an error message on the context (or, with ctx == nullptr, for the calling thread) and
// return the status.
mp_status fail(mp_ctx* ctx, mp_status st, const char* fmt, ...) __attribute__((format(printf, 3, 4)));
int pick_chunk_rows(long long n_rows_per_unit, int n_units);
}  // namespace mp
