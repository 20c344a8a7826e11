// Kernel parameter blocks and launch entry points (host side sees only this header).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lkv {

// Rows of a [heads, rows, d] tensor with element strides; d contiguous.
struct RowSrc {
  const char* base;
  int64_t stride_head;  // bytes
  int64_t stride_row;   // bytes
};

struct PassParams {
  RowSrc q;        // [H_q, W, d]
  RowSrc kb;       // [H_kv, S, d]
  RowSrc kc;       // [H_kv, T, d] (base may be null when T == 0)
  const char* planes;   // [L*K, d] contiguous
  int q_linear;    // q.stride_head >= W * q.stride_row and a KV head's G query heads span < 2 GiB: window row
                   // m = g*W + j of KV head h sits at 32-bit offset g * stride_head + j * stride_row from the
                   // first row of query head h*G, and one buffer descriptor covers the group
  int group;       // G
  int w;           // W
  uint32_t w_magic;  // ceil(2^32 / W) (0 for W == 1): row / W, see div_w
  int m_rows;      // M = G * W
  int s_t;         // S
  int t_ctx;       // T
  // key ranges of sweep 1: n_ctx_ranges ranges of ctx_per_range look-back keys, then ranges of blk_per_range block keys
  int keys_per_range;   // key rows a workgroup's LDS holds (multiple of 32, <= score_max_range())
  int blk_per_range;    // block keys per block range (multiple of 32)
  int ctx_per_range;    // look-back keys per look-back range (multiple of 32)
  int n_ctx_ranges;     // ceil(T / ctx_per_range)
  int n_ranges;         // n_ctx_ranges + ceil(S / blk_per_range)
  int n_parts;          // sweep-1 partials per window row (= sweep 1's n_ranges)
  // key ranges of sweep 2 (block keys only); the launcher rewrites the fields above from these
  int s2_blk_per_range; // multiple of 32
  int s2_ranges;        // ceil(S / s2_blk_per_range)
  int n_qgroups;        // ceil(M / sweep_rows_per_group())
  int n_kv_heads;
  int causal;
  int lim0;        // key index kidx is visible to window row j iff kidx <= lim0 + j (when causal)
  float scale2;    // log2(e) / sqrt(d)
  float2* part;    // [H_kv, m_pad, r_pad] sweep-1 partials (reference, sum) in the exp2 domain
  int m_pad;       // rows per head in part
  int r_pad;       // partials per row in part: n_ranges rounded up to a multiple of 8
  int lds_tail_offset;  // byte offset of the per-row LDS arrays (set by the launcher)
  float* s_part;   // [n_qgroups, H_kv, S] sweep-2 pooled probabilities (sum over the group's rows)
  const float* row_lse;  // [H_kv, M] natural-log sum of exp(logit) over keys outside this call, or null
  int lse_complete;      // row_lse is every window row's COMPLETE log-sum-exp: sweep 1 computes no row statistics
  // hashing (sweep 1)
  int n_tables, n_bits, n_planes;  // L, K, L*K (<= 512)
  int tables_per_split; // tables of the KEY codes computed by one query-row group's workgroups: ceil(L / n_qgroups)
  int q_tab_per_wg;     // tables of the QUERY codes (of its own window rows) owned by workgroup (range, group): ceil(L / NR)
  int q_tab_per_tile;   // whole tables per 32-plane tile of that job: floor(32 / K)
  int q_tiles;          // ceil(q_tab_per_wg / q_tab_per_tile)
  int hist_lds_words;   // q_tab_per_wg * 2^K / 2 when the query histograms are built, else 0
  uint16_t* sig_k;      // [H_kv, S, L]
  uint16_t* sig_q;      // [H_q, W, L] = [H_kv, M, L]
  int32_t* cnt;         // with qhist: [n_qgroups, H_kv, S] written by sweep 2; else [H_kv, S] zeroed in sweep 1
                        // for the count kernel's atomics
  uint32_t* qhist;      // [H_kv, L, 2^K / 2, n_qgroups] histograms of the query codes of each row group, two 16-bit
                        // bins per word, every word rewritten by sweep 1; null: separate count kernel
};

struct CountParams {
  const uint16_t* sig_k;  // [H_kv, S, L]
  const uint16_t* sig_q;  // [H_q, W, L]
  int32_t* cnt;           // [H_kv, S]
  int group, w, s_t;
  int n_tables, n_bits;
  int tables_per_group;   // TG: tables whose histograms share the LDS at one time
  int groups_per_wg;      // table groups a workgroup takes one after the other
  int keys_per_range;     // <= count_max_keys_per_range()
};

struct SelectParams {
  const float* s_part;  // [n_qgroups, H_kv, S]
  int n_qgroups;
  int n_kv_heads;
  float inv_m;          // 1 / (G * W)
  const int32_t* cnt;   // [n_cnt_parts, H_kv, S]
  int n_cnt_parts;
  int32_t* cnt_out;     // [H_kv, S] summed counts (optional, for the stage outputs)
  int s_t;
  int n_anchor, n_local, k_exact, k_lsh;
  int cnt_bits;         // bits needed to hold G * W * L
  float* s_exact;       // [H_kv, S] final scores (optional, for the stage outputs)
  int32_t* keep;        // [H_kv, B_t]
};

// Adds one layer's scores and counts, summed over its KV heads, into [S] accumulators.
struct AccumParams {
  const float* s_part;  // [n_qgroups, H_kv, S]
  const int32_t* cnt;   // [n_cnt_parts, H_kv, S]
  int n_qgroups, n_cnt_parts, n_kv_heads, s_t;
  float inv_m;          // 1 / (G * W)
  float* score;         // [S]
  int32_t* count;       // [S]
  int accumulate;       // 0: overwrite, else add
};

struct AppendParams {
  RowSrc kb, vb;        // [H_kv, S, d]
  const int32_t* keep;  // [H_kv, B_t], or [B_t] shared by all heads when keep_stride_head == 0
  int keep_stride_head; // elements between two heads' index lists
  int b_t;
  int s_t;              // rows in the block: indices are clamped into it
  int row_bytes;        // d * elem size
  char* k_cache;
  char* v_cache;
  int64_t cache_stride_head;  // bytes
  int64_t* cache_pos;
  int64_t pos_stride_head;    // elements
  int64_t cache_len;
  int64_t block_pos0;
};

// The single sweep of a block whose window rows come with their complete log-sum-exp.
struct SingleParams {
  RowSrc q;        // [H_q, W, d]; stride_head >= W * stride_row, a KV head's G query heads within 2 GiB
  RowSrc kb;       // [H_kv, S, d]
  const char* planes;  // [L*K, d] contiguous
  int group, w;
  uint32_t w_magic;
  int m_rows;      // M = G * W <= single_max_rows()
  int s_t;
  int keys_per_range;  // multiple of 32, <= single_max_keys()
  int n_ranges;        // ceil(S / keys_per_range)
  int n_kv_heads;
  int causal, lim0;    // block key i is visible to window row j iff i <= lim0 + j (when causal)
  float scale2;
  const float* row_lse;  // [H_kv, M] complete natural-log normaliser of every window row
  int n_tables, n_bits, n_planes;
  int q_tab_per_wg;    // tables whose window-row codes and histogram workgroup (range, head) owns: ceil(L / n_ranges)
  int q_tab_per_tile;  // floor(32 / K)
  int q_tiles;         // ceil(q_tab_per_wg / q_tab_per_tile) <= single_max_qtiles()
  float* s_part;       // [H_kv, S] pooled probabilities (sum over the rows)
  int32_t* cnt;        // [H_kv, S]
  uint16_t* sig_k;     // [H_kv, S, L] or null: key codes only for the stage outputs
  uint16_t* sig_q;     // [H_kv, M, L]
  uint32_t* qhist;     // [H_kv, L, 2^K / 2] histograms of the window-row codes, two 16-bit bins per word
  uint32_t* flags;     // [H_kv, L]: epoch + 1 of the launch that published the table's histogram
  uint32_t* sync;      // [0] epoch, [1] workgroups of the running launch that have finished; both zero at first
  int spin_limit;      // polls of a flag before the workgroup computes the table itself
};
size_t single_lds_bytes(int dtype, int head_dim, int keys_per_range, int q_tiles, int q_tab_per_wg, int n_bits, int n_tables);
int single_max_rows();
int single_max_keys();
int single_max_qtiles();
bool single_supports(int dtype, int head_dim);
hipError_t launch_single(int dtype, int head_dim, const SingleParams& p, hipStream_t st);
hipError_t init_single_attributes();

// Attention of n_q queries per query head over the first cache_len rows of each KV head's compacted cache.
struct AttendParams {
  RowSrc q;            // [H_q, n_q, d]
  int group, n_q;
  uint32_t nq_magic;   // ceil(2^32 / n_q) (0 for n_q == 1): row / n_q, see div_w
  int m_rows;          // M = G * n_q rows per KV head, row m = g * n_q + j
  const char* k_cache; // [H_kv, cap, d] rows contiguous
  const char* v_cache;
  int64_t cache_stride_head;  // bytes
  int row_bytes;       // d * elem size
  int cache_len;       // rows
  // the block's own keys and values, behind the cache rows in key order (none: s_t == 0)
  const char* k_blk;   // [H_kv, s_t, d]
  const char* v_blk;
  int64_t kb_stride_head, vb_stride_head;  // bytes
  int kb_stride_row, vb_stride_row;        // bytes
  int s_t;
  int diag;            // block key i is visible to query j iff i <= diag + j (>= s_t: no mask); |diag| <= 2^30
  int keys_per_split;  // cache rows per split, multiple of 32
  int blk_keys_per_split;  // block keys per split, multiple of 32
  int n_splits;        // every split takes its share of both segments; 0: no key at all
  int direct;          // one split and a wave per row tile: attend_kernel writes out / out_lse itself
  int wprt_log;        // log2 of the waves that share a 32-row tile (over different key tiles)
  int n_parts;         // partials per row: one per key split
  int n_qgroups;       // ceil(M / 256)
  int n_kv_heads;
  float scale2;        // log2(e) / sqrt(d)
  float* part_o;       // [H_kv, n_parts, M, d] unnormalised partial outputs
  float2* part_ml;     // [H_kv, n_parts, M] (reference, sum) in the exp2 domain
  float* out;          // [H_kv * M, d]
  float* out_lse;      // [H_kv * M] natural log
};
struct AttendPlan {
  int n_qgroups, wprt_log, n_splits, keys_per_split, blk_keys_per_split, n_parts, direct;
};
void attend_plan(int m_rows, int64_t cache_len, int s_t, int n_kv_heads, int n_cu, AttendPlan* plan);
size_t attend_workspace_bytes(const AttendPlan& plan, int m_rows, int n_kv_heads, int head_dim);  // part_o, then part_ml
hipError_t launch_attend(int dtype, int head_dim, const AttendParams& p, hipStream_t st);
// the normaliser alone (out unused): 512 rows per workgroup, keys only
void attend_lse_plan(int m_rows, int64_t cache_len, int n_kv_heads, int n_cu, AttendPlan* plan);
hipError_t launch_attend_lse(int dtype, int head_dim, const AttendParams& p, hipStream_t st);
hipError_t init_attend_attributes();

hipError_t launch_sweep1(int dtype, int head_dim, const PassParams& p, hipStream_t st);
hipError_t launch_sweep2(int dtype, int head_dim, const PassParams& p, hipStream_t st);
hipError_t launch_count(const CountParams& p, int n_kv_heads, hipStream_t st);
hipError_t launch_select(const SelectParams& p, hipStream_t st);
// split_override > 0: workgroups per head (tuning); otherwise n_cu / heads
hipError_t launch_select_append(const SelectParams& p, const AppendParams& ap, int n_cu, int split_override, hipStream_t st);
hipError_t launch_append(const AppendParams& p, int n_kv_heads, hipStream_t st);
hipError_t launch_accumulate(const AccumParams& p, hipStream_t st);
hipError_t init_kernel_attributes();
size_t sweep_lds_bytes(int dtype, int head_dim, bool pass2, int range_keys, int q_tiles, int hist_lds_words);
int sweep_rows_per_group();  // window rows one sweep workgroup covers
int score_max_range();  // most keys one score workgroup takes (its LDS holds the whole range)
int count_max_keys_per_range();
// LDS of a count workgroup: the histogram of one table group plus the staged query and key codes of all its tables
size_t count_lds_bytes(int n_bits, int tables_per_group, int groups_per_wg, int n_query_rows, int keys_per_range);

}  // namespace lkv
