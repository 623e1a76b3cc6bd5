// Host-side declarations shared by the kernel translation units and the C-ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mp {

// ------------------------------------------------------------------------------------------------
// Value pass: streams rows (keys + values, or value centroids with ready-made scores) and produces
// one online-softmax partial (m, l, acc[128]) per (unit, chunk, head).  A stream may be cut into two
// sources with different chunk sizes (large chunks first, small ones last) to shorten the drain.
// ------------------------------------------------------------------------------------------------
constexpr int kChunkRowsMin = 512;     // smallest chunk of the dense kernel: 4 waves, one strip of 128 rows each
constexpr int kPartStride = 132;       // floats per (unit, chunk, head): m, l, pad, pad, acc[128]
constexpr int kMaxSources = 4;

// One stream of rows.  Row j of unit u lives at K + (u*unit_rows + idx)*128 (elements) where idx = rows ?
// rows[u*rows_stride + j] : j.  The number of rows is *count_dev (clamped to count_max) or count_max.
struct RowSource {
    const uint16_t* K;         // bf16 keys; unused when scores != nullptr
    const uint16_t* V;         // bf16 values (or value centroids)
    long long unit_rows;       // rows per unit in K / V
    const int32_t* rows;       // optional gather list
    long long rows_stride;     // entries per unit in rows / scores
    const int32_t* count_dev;  // optional per-unit row count on the device
    int32_t count_max;         // upper bound of the row count (fixes the chunk count)
    const float* scores;       // optional [U, rows_stride, G] ready-made logits in log2 units
    // optional, all three or none: K and V hold 128-byte rows of e4m3 codes; the value row idx stands for
    // code * row_scale[idx][1], the key row for (its cluster's centroid) + code * row_scale[idx][0], and the
    // centroid's share of the logit is read ready-made: slot_base[row_slot[j]] for list position j
    const float* row_scale;    // [U, unit_rows, 2]
    const int32_t* row_slot;   // [U, rows_stride]
    const float* slot_base;    // [U, base_stride, 8] log2 units, column layout as written by the scoring kernel
    long long base_stride;
    int32_t chunk0;            // first chunk id of this source inside a unit
    int32_t n_chunks;          // ceil(count_max / chunk_rows)
    int32_t chunk_rows;        // rows per workgroup of this source, a multiple of 64
    int32_t row0;              // first list position this source covers: [row0, row0 + count_max)
    int32_t guest;             // 1: src[0] of the launch, a scored source with n_chunks == 0, rides along: its rows
                               // are shared out evenly over this source's chunks
};

struct ValuePassParams {
    const uint16_t* q;         // bf16 [U*G, 128]
    float* partials;           // [U, chunks_per_unit, G, kPartStride]
    int32_t n_units;
    int32_t chunks_per_unit;
    int32_t n_sources;
    float scale_log2e;         // softmax scale * log2(e)
    RowSource src[kMaxSources];
};

hipError_t launch_value_pass(const ValuePassParams& p, int G, hipStream_t stream);

// Merge of the partials of a unit into the output: out bf16 [U*G, 128], lse fp32 [U*G] (optional).
hipError_t launch_merge(const float* partials, int n_units, int chunks_per_unit, int G, uint16_t* out,
                        float* lse, hipStream_t stream);

// ------------------------------------------------------------------------------------------------
// Centroid scoring + budgeted selection (one launch per level)
// ------------------------------------------------------------------------------------------------
struct ScoreParams {
    const uint16_t* q;          // bf16 [U*G, 128]
    const uint16_t* Kc;         // bf16 [U, tab_rows, 128]: fine rows, then coarse rows from row fcap
    const int32_t* N;           // [U, tab_rows]
    long long tab_rows;
    int fcap;
    int levels, n_fine, n_coarse;
    long long key_budget, coarse_budget;
    double scale;
    const int32_t* cstart;      // [U, cstart_stride] first child of each coarse cluster
    long long cstart_stride;
    const int32_t* fstart;      // [U, fstart_stride] first stored row of each fine cluster
    long long fstart_stride;
    // working arrays in global memory, used by a level with more than lds_cap entries
    double* lg;                 // [U, G, lg_stride]
    long long lg_stride;
    unsigned long long* g_keys; // [U, g_stride]
    uint32_t* g_wts;
    int32_t* g_ids;
    int32_t* g_aux;
    int32_t* g_aux2;
    uint8_t* g_flags;
    long long g_stride;
    // per-position views of the last call (for the getters): the key each entry was ranked by (all
    // ones: took no part) and, per unit and level, what the keys are (key_mode, see launch_scatter_selection)
    unsigned long long* key_c;  // [U, c_stride] coarse
    uint8_t* flag_c;            // [U, c_stride] promising
    long long c_stride;
    unsigned long long* key_f;  // [U, f_stride] fine, by candidate position
    uint8_t* flag_f;            // [U, f_stride] selected, by candidate position
    long long f_stride;
    int32_t* key_mode;          // [U, 2] coarse, fine
    int32_t* cand;              // [U, f_stride] candidate fine ids (two levels)
    int32_t* n_cand;            // [U]
    // outputs for the value pass
    int32_t* rows;              // [U, rows_stride] stored rows of the selected keys
    long long rows_stride;
    int32_t* n_rows;            // [U]
    // optional (both or none; keys stored as residuals from their cluster's centroid): per selected cluster, in
    // the order of a compact list, q . centroid in log2 units, eight columns (see fine_epilogue), and per row of
    // `rows` the position of its cluster in that list
    float* sel_base;            // [U, f_stride, 8]
    int32_t* row_slot;          // [U, rows_stride]
    int32_t* mp_rows;           // [U, mp_stride] centroid-table row of each centroid term
    float* mp_scores;           // [U, mp_stride, G] (l + ln N) * log2(e)
    long long mp_stride;
    int32_t* n_mp;              // [U]
    int use_mp;
    int32_t* counters;          // [U, 4]
    int n_tail;
    // optional: rows the caller hands over with this step (a generation loop's new token) are copied
    // into the tail buffers by the workgroup of their unit before anything else; the value pass,
    // a later launch, then finds them there.  app_n arrays (0 = none), 256-byte rows.
    int app_n;
    const void* app_src[3];     // [U, 128] bf16 each
    void* app_dst[3];           // [U, app_dst_rows, 128] bf16 each
    long long app_dst_rows;
    int app_row;
    int lds_cap;                // entries of a level that fit the LDS working arrays
    int G, U;
};

// n_compute_units: of the device the launch goes to (decides whether units get a second, shadow workgroup).
hipError_t launch_score_select(const ScoreParams& p, int n_compute_units, hipStream_t stream);
size_t score_smem_bytes(int G, int cap);

// ------------------------------------------------------------------------------------------------
// Index construction helpers (member lists, gathers, per-cluster means)
// ------------------------------------------------------------------------------------------------
// Nearest-centroid assignment (fp64 definition, lowest index among equal distances) of the points of
// nb blocks per unit.  blocks_dev: int32 [nb][4] = {first point, end point, first centroid, end
// centroid}; assign[u][t] receives the centroid row of point t.  amb_list [U, list_stride] (at least
// as long as the point range) and amb_cnt [U, cnt_stride >= nb] are workspace; amb_cnt must be all zero on
// entry, and the call leaves amb_cnt_next [U, cnt_stride] all zero for the next one (two arrays used in turn
// save a fill launch per step).  max_pts / max_k: the
// largest point / centroid count of a block (max_k = 0: not known; it only selects the kernel).
hipError_t launch_assign(const uint16_t* X, long long x_unit_rows, const int32_t* blocks_dev, int nb, int max_pts,
                         int max_k, int U, const uint16_t* C, long long c_unit_rows, int32_t* assign,
                         long long assign_stride, int32_t* amb_list, long long list_stride, int32_t* amb_cnt,
                         int32_t* amb_cnt_next, int cnt_stride, hipStream_t s);
hipError_t launch_histogram(const int32_t* ids, long long ids_stride, int n, int U, int32_t* cnt,
                            long long cnt_stride, hipStream_t s);
hipError_t launch_exclusive_scan(const int32_t* cnt, long long cnt_stride, int k, int U, int32_t* start,
                                 long long start_stride, hipStream_t s);
// Member lists of all blocks in one launch (stable counting sort by cluster id):
// start[u][id] = first list position of cluster id, counted from point p_first; the entry after the
// last block's last cluster receives the end position; list[u][position] = point index.
hipError_t launch_block_lists(const int32_t* ids, long long ids_stride, const int32_t* blocks_dev, int nb,
                              int max_k_per_block, int p_first, int U, int32_t* start, long long start_stride,
                              int32_t* list, long long list_stride, hipStream_t s);
// blocks_dev: int32 [nb][4] = {first point, end point, first cluster, end cluster}
hipError_t launch_member_lists(const int32_t* ids, long long ids_stride, const int32_t* blocks_dev, int nb,
                               int max_k_per_block, int U, const int32_t* start, long long start_stride,
                               int32_t* list, long long list_stride, hipStream_t s);
hipError_t launch_gather_rows(const void* srcK, const void* srcV, long long src_unit_rows, const int32_t* list,
                              long long list_stride, int n, int U, void* dstK, void* dstV, long long dst_unit_rows,
                              int dst_row0, hipStream_t s);
// The same into 8-bit storage: dstK / dstV receive 128 e4m3 codes per row, scales [U, dst_unit_rows, 2] the
// rows' fp32 scales {key, value} (scale = max|x| / 448, 1 for a zero row; code = round-to-nearest-even(x / scale)).
// For a value row x is the row; for a key row x = fp32(key) - fp32(Kc[ids[point]]), the residual from the key
// centroid of the point's fine cluster (ids [U, ids_stride] by local point, Kc [U, kc_unit_rows, 128] bf16).
hipError_t launch_gather_quantize_rows(const void* srcK, const void* srcV, long long src_unit_rows, const int32_t* list,
                                       long long list_stride, const int32_t* ids, long long ids_stride,
                                       const uint16_t* Kc, long long kc_unit_rows, int n, int U, void* dstK, void* dstV,
                                       float* scales, long long dst_unit_rows, int dst_row0, hipStream_t s);
// mean_out row (out_row0 + id) = bf16(fp64 sum of the member rows in list order / count); sum_out (optional)
// receives the fp64 sums themselves, row = id.
hipError_t launch_cluster_means(const uint16_t* X, long long x_unit_rows, const int32_t* list, long long list_stride,
                                const int32_t* start, long long start_stride, int k0, int k, int U,
                                uint16_t* mean_out, long long out_unit_rows, int out_row0, const uint16_t* fallback,
                                long long fb_unit_rows, int32_t* count_out, long long count_stride, int count_off,
                                double* sum_out, long long sum_unit_rows, hipStream_t s);
// Coarse clusters [c0, c1) from their children: sums [U, sum_unit_rows, 128] fp64 member sums of the fine clusters
// (row = map ? map[f - map_f0] : f), cstart = first child of each coarse cluster, fine_count[f] members.
hipError_t launch_coarse_from_children(const double* sums, long long sum_unit_rows, const int32_t* map, long long map_stride,
                                       int map_f0, const int32_t* cstart, long long cstart_stride,
                                       const int32_t* fine_count, long long count_stride, int c0, int c1, int U,
                                       uint16_t* mean_out, long long out_unit_rows, int out_row0, const uint16_t* fallback,
                                       long long fb_unit_rows, int32_t* count_out, int count_off, hipStream_t s);
hipError_t launch_coarse_start(const int32_t* cof, long long cof_stride, int f0, int f1, int c0, int c1, int U,
                               int32_t* cstart, long long cstart_stride, hipStream_t s);
hipError_t launch_offset_lists(const int32_t* start, long long start_stride, int f0, int f1, const int32_t* list,
                               long long list_stride, int n_pts, int pt0, int U, int32_t* fstart,
                               long long fstart_stride, int32_t* perm, long long perm_stride, hipStream_t s);
hipError_t launch_ids_from_lists(const int32_t* list, long long list_stride, const int32_t* start,
                                 long long start_stride, int k, int U, int32_t* ids, long long ids_stride,
                                 hipStream_t s);
// Views of the last scoring launch, by cluster id.  keys [U, pos_stride] by position; key_mode[2*u + level]
// says what they are: 0 = order-preserving image of the rank key r = log mean_h e^{l - LSE_h}; 1 = complement
// of the bit pattern of sum_h e^{l - LSE_h} (then r = log(sum) - log G).  r_out receives r (NaN: took no part).
hipError_t launch_scatter_selection(const int32_t* cand, long long cand_stride, const int32_t* n_cand_dev,
                                    int n_cand_fixed, const uint8_t* flag, const unsigned long long* keys,
                                    const int32_t* key_mode, int level, int G, long long pos_stride, int n_ids, int U,
                                    uint8_t* sel_out, double* r_out, hipStream_t s);

}  // namespace mp
