// HIP kernels of the LASER-KV block-selection path for gfx950 (wave64, MFMA, LDS).
//
//   pass_kernel<PASS2=false>   sweep 1: per window row, partial (reference, sum) of 2^(logit) over each
//                              key range (Alg. 1 step 3, normaliser), and in the same workgroups the
//                              SimHash codes of keys and window queries (Sec. 3.3 "Recall") plus the
//                              per-table histograms of the query codes                          [MFMA]
//   pass_kernel<PASS2=true>    sweep 2: pooled softmax probability per key (Alg. 1 step 3), and the
//                              collision counts by histogram lookup (Alg. 1 step 6)              [MFMA]
//   count_kernel               collision counts via LDS histograms, for code widths whose histograms
//                              are too large to keep resident in global memory
//   select_kernel              Alg. 1 steps 4-8 + Sec. 3.1 partition: two rank selections and
//                              compaction; FUSED also gathers the kept K/V rows onto the cache tail
//   append_kernel              the gather alone
#include "laserkv_device.h"
#include "laserkv_kernels.h"

#include <limits.h>

namespace lkv {

// ---------------------------------------------------------------------------------------------
// The two sweeps over a block's keys.  Workgroup = (key range, query-row group of 256 rows, KV
// head); 16 waves, one workgroup per compute unit.
//
//   sweep 1 (PASS2 = false): waves 0-7 compute, per window row, partial softmax statistics over the
//            range (Alg. 1 step 3, normaliser); waves 8-15 compute the SimHash sign bits of the
//            range's keys (Sec. 3.3 "Recall") from the SAME LDS rows, so the block's keys are read
//            from HBM once for both contractions and the two roles overlap on every SIMD.  Waves 0-7
//            then hash their own window rows (already in registers) for the few tables this workgroup
//            owns and histogram the codes in LDS; the histograms leave as plain stores.
//   sweep 2 (PASS2 = true):  pooled softmax probability of every key of the range (Alg. 1 step 3);
//            wave = (row tile, half of the range).  Before that loop: collision counts of the range's
//            keys by lookup in the histograms (Alg. 1 step 6).
//
// The whole range (<= SCORE_MAX_RANGE keys) is fetched into LDS up front: a range is microseconds
// of work, so what matters is having all of its loads in flight at once.  After one barrier each
// wave walks its 32-key tiles on its own: A fragments of ONE 32-row tile (queries, or hyperplanes
// for the hashing waves) stay in registers, B fragments come from LDS (row pitch padded by one
// 16-byte chunk: conflict-free reads at base + immediate addresses).  Four waves share a SIMD
// (<= 128 registers per lane): one wave alone issues a vector instruction only every ~10 clocks.
//
// Sweep 1 multiplies keys (A) by window rows (B), so a lane owns one window row and keeps its
// sum_i 2^(x_i - ref) privately, ref being the lane's maximum over the range's first tile.  The common
// case costs one fma, one exp and one add per logit; a range whose later logits exceed that reference
// by more than 2^7 overflows the sum, which is detected after the loop and redone with a
// running-maximum reference.  Sweep 2 multiplies window rows (A) by keys (B), so a lane owns one key
// and its pooled probability is an in-lane sum: one fma, one exp and one add per logit.
//
// Hashing: lane = vector, accumulator register = plane, with the planes fed in an order that makes
// a lane's 16 registers 16 consecutive planes: one v_alignbit per register shifts its sign bit into
// the lane's word, and one exchange with the partner lane completes the 32-bit word of that 32-plane
// tile.  With several query-row groups the tables are split between their workgroups.
// ---------------------------------------------------------------------------------------------
constexpr int PASS_WAVES = 16;
constexpr int PASS_ROWS = 256;        // window rows per workgroup: 8 row tiles
constexpr int SCORE_MAX_RANGE = 288;  // keys per workgroup at most
constexpr int BITS_PITCH = 17;        // words per vector row in the sign-bit scratch (<= 16 plane tiles)

template <int DT, int D>
__host__ __device__ constexpr int row_pitch_chunks() { return D * (DT == DT_BF16 ? 2 : 4) / 16 + 1; }

template <int DT, int D, bool PASS2>
__global__ __launch_bounds__(PASS_WAVES * 64) void pass_kernel(PassParams p) {
  constexpr int ES = DT == DT_BF16 ? 2 : 4;
  constexpr int CH = D * ES / 16;  // 16-byte chunks per row
  constexpr int NCH = CH / 2;      // chunk pairs per tile
  constexpr int CHP = CH + 1;      // LDS row pitch in chunks
  constexpr int NTHR = PASS_WAVES * 64;
  constexpr int MQ = PASS_ROWS;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, rl = lane & 31, kg = lane >> 5;
  // work item: heads are the slow index of the XCD-major order, so one head's keys, queries and
  // query histograms are fetched into one L2 (or as few as the head count allows)
  const int n_qg = p.n_qgroups;
  int kr, qg, h;
  {
    const int per_head = p.n_ranges * n_qg;
    const int lin = xcd_major(blockIdx.x, per_head * p.n_kv_heads);
    h = lin / per_head;
    const int rem = lin - h * per_head;
    kr = rem / n_qg;
    qg = rem - kr * n_qg;
  }
  const int nkr = p.keys_per_range;  // key rows the LDS holds
  // The first n_ctx_ranges ranges of sweep 1 hold look-back keys (ctx_per_range each; they only enter the
  // normaliser), the others blk_per_range consecutive block keys each; sweep 2 has block ranges only, of a
  // length of its own.  In LDS, rows [0, nb) are block keys b0 .., rows [nb, nb + nc) look-back keys c0 ...
  const int kb = kr - p.n_ctx_ranges;
  const int b0 = max(kb, 0) * p.blk_per_range;
  const int nb = kb < 0 ? 0 : min(p.blk_per_range, p.s_t - b0);    // block keys of this range
  const int c0 = kr * p.ctx_per_range;
  const int nc = kb < 0 ? min(p.ctx_per_range, p.t_ctx - c0) : 0;  // look-back keys of this range
  const int n_rows = nb + nc;
  const int k0 = p.t_ctx + b0;  // key index of block row 0 (look-back keys count first): key k is visible
  const int k1 = k0 + nb;       // to window row j iff k <= lim0 + j
  const char* kb_ptr = p.kb.base + (int64_t)h * p.kb.stride_head;
  const char* kc_ptr = p.kc.base + (int64_t)h * p.kc.stride_head;  // null base when there are no look-back keys
  const int kb_stride = (int)p.kb.stride_row, kc_stride = (int)p.kc.stride_row;
  const int n_tiles = (n_rows + 31) >> 5;
  // sweep 1: the tables whose QUERY codes (for the window rows of group qg) this workgroup owns ...
  const int qt0 = kr * p.q_tab_per_wg;
  const int n_qt = PASS2 ? 0 : max(0, min(p.q_tab_per_wg, p.n_tables - qt0));
  const int n_qpt = (n_qt + p.q_tab_per_tile - 1) / p.q_tab_per_tile;  // 32-plane tiles of whole tables
  // ... and its share of the tables of the KEY codes
  const int tab0 = qg * p.tables_per_split;
  const int n_tab = PASS2 ? 0 : max(0, min(p.tables_per_split, p.n_tables - tab0));
  const int plane0 = tab0 * p.n_bits;
  const int n_pl = n_tab * p.n_bits;
  const int n_mt = (n_pl + 31) >> 5;
  // roles
  const bool hash_wave = !PASS2 && wave >= 8;
  const int rt = wave & 7;  // row tile of a score wave; index of a hashing wave

  extern __shared__ uint4 smem[];
  uint4* sK = smem;                                                    // [nkr][CHP]
  uint4* after_rows = smem + (size_t)nkr * CHP;
  float* sCol = reinterpret_cast<float*>(after_rows);                  // sweep 2: [8][nkr]
  uint32_t* sBits = reinterpret_cast<uint32_t*>(after_rows);           // sweep 1: [nkr][BITS_PITCH]
  uint4* sQP = after_rows + (nkr * BITS_PITCH + 3) / 4;                // sweep 1: [q_tiles * 32][CHP] planes of the query job
  uint32_t* sHist = reinterpret_cast<uint32_t*>(sQP + (size_t)p.q_tiles * 32 * CHP);  // sweep 1: [hist_lds_words]
  uint4* sQst = after_rows + 2 * nkr;                                  // sweep 2: [256][CHP] query panel (past sCol)
  // row limits and lse sit past both the steady-state arrays and the A-operand staging area
  int* sLim = reinterpret_cast<int*>(reinterpret_cast<char*>(smem) + p.lds_tail_offset);  // [MQ]
  float* sLse = reinterpret_cast<float*>(sLim + MQ);                   // [MQ]

  // 1. everything this workgroup reads from memory, issued back to back.  The A operands (256 window
  // rows; in sweep 1 also up to 256 hyperplanes) are fetched as whole rows by all threads and passed
  // through LDS into the fragment layout: a wave fetching its own 32 rows 16 bytes per lane would
  // touch 32 cache lines per instruction and dominate the kernel.  The key rows wait in registers
  // meanwhile and then take over the same LDS space.
  constexpr bool STAGE_A = CH <= 16;                 // wider rows: fragments straight from memory
  constexpr int QL = STAGE_A ? MQ * CH / NTHR : 1;   // 16-byte chunks per thread: query panel
  constexpr int KL = STAGE_A ? ((SCORE_MAX_RANGE + 32) * CH + NTHR - 1) / NTHR : 1;  // keys + one tile of planes
  const int n_kchunks = n_tiles * 32 * CH;           // rows past the range: any readable row, masked later
  const int n_chunks = n_kchunks + n_qpt * 32 * CH;
  auto key_chunk = [&](int q) -> uint4 {
    if (q < n_kchunks) {
      const int row = q / CH, c = q % CH;
      if (row < nb || nc == 0) return ld16(kb_ptr + (uint32_t)(min(b0 + row, p.s_t - 1) * kb_stride + c * 16));
      return ld16(kc_ptr + (uint32_t)(min(c0 + row - nb, p.t_ctx - 1) * kc_stride + c * 16));
    }
    // planes of the query job: tile t holds the planes of whole tables qt0 + t*q_tab_per_tile ..., padded
    // with copies of its last plane
    const int qq = q - n_kchunks;
    const int row = qq / CH, c = qq % CH;
    const int t_tab0 = qt0 + (row >> 5) * p.q_tab_per_tile;
    const int t_planes = min(p.q_tab_per_tile, qt0 + n_qt - t_tab0) * p.n_bits;
    const int pm = t_tab0 * p.n_bits + min(row & 31, t_planes - 1);
    return ld16(p.planes + (size_t)pm * (D * ES) + c * 16);
  };
  auto key_slot = [&](int q) -> int {
    if (q < n_kchunks) return (q / CH) * CHP + q % CH;
    const int qq = q - n_kchunks;
    return (int)(sQP - smem) + (qq / CH) * CHP + qq % CH;
  };

  // sweep 2: four threads per window row, each a quarter of the row's sweep-1 partials (consecutive in
  // memory); the first eight are prefetched here
  uint4 pv[PASS2 ? 4 : 1];
  const int pr_per = p.r_pad >> 2;  // partials per thread, even
  const int pr_beg = (tid & 3) * pr_per;
  const float2* pr_ptr = nullptr;
  if (PASS2 && !p.lse_complete) {
    const int m = min(qg * MQ + (tid >> 2), p.m_rows - 1);
    pr_ptr = p.part + ((size_t)h * p.m_pad + m) * p.r_pad + pr_beg;
#pragma unroll
    for (int u = 0; u < 4; ++u) pv[u] = ld16(pr_ptr + min(2 * u, pr_per - 2));
  }
  // Sweep 2, collision counts (Alg. 1 step 6) of this range's keys over this workgroup's share of the
  // tables: 1, 2 or 4 lanes per key, eight tables per lane and step.  In the common shape (two row
  // groups, one step per lane, aligned codes) the job rides along with the main loop: the key's eight
  // codes are fetched here with the other loads, each loop iteration issues the histogram lookups of
  // two tables and adds up those of the iteration before, so their latency costs nothing.
  const int tab0c = qg * p.tables_per_split;
  const int n_tabc = PASS2 && p.qhist ? max(0, min(p.tables_per_split, p.n_tables - tab0c)) : 0;
  int lpk_log = n_tabc > 16 ? 2 : (n_tabc > 8 ? 1 : 0);
  while (lpk_log > 0 && (nb << lpk_log) > NTHR) --lpk_log;
  const bool cnt_piped = NCH <= 8 && n_tabc > 0 && n_tabc == (8 << lpk_log) && (p.n_tables & 7) == 0 && (tab0c & 7) == 0 &&
                         (nb << lpk_log) <= NTHR && n_qg == 2;
  const bool cnt_lane = cnt_piped && tid < (nb << lpk_log);
  const int cnt_key = tid >> lpk_log, cnt_tb = (tid & ((1 << lpk_log) - 1)) * 8;
  uint4 cnt_codes = make_uint4(0u, 0u, 0u, 0u);  // two 16-bit codes per word, consumed from .x upwards
  if (cnt_lane) cnt_codes = ld16(p.sig_k + ((size_t)h * p.s_t + b0 + cnt_key) * p.n_tables + tab0c + cnt_tb);

  uint4 a[NCH];  // A operand: this wave's 32 window rows, or (hashing waves) its first 32 planes
  if (STAGE_A) {
    // Load u of a thread is chunk tid % CH of row tid / CH + u * (NTHR / CH): one byte offset per thread
    // and tensor, one add per load; rows past the end of a tensor read as zero (they are masked, or their
    // results are never stored).
    uint4 qpre[QL], ppre[QL], kpre[KL];
    constexpr int ROWS_PER_LOAD = NTHR / CH;
    const uint32_t trow = tid / CH, tcol = (tid % CH) * 16;
    if (p.q_linear) {
      // row m = g * W + j of the KV head's group at g * stride_head + j * stride_row from the group's first row;
      // rows past M land at or past the descriptor's end (stride_head >= W * stride_row) and read as zero
      const uint32_t qstride = (uint32_t)p.q.stride_row, hstride = (uint32_t)p.q.stride_head;
      const __amdgpu_buffer_rsrc_t qsrd = make_srd(p.q.base + (int64_t)h * p.group * p.q.stride_head,
                                                   (uint32_t)(p.group - 1) * hstride + (uint32_t)p.w * qstride);
#pragma unroll
      for (int u = 0; u < QL; ++u) {
        const int m = qg * MQ + trow + u * ROWS_PER_LOAD;
        const int g = div_w(m, p.w_magic);
        qpre[u] = buf_ld16(qsrd, (uint32_t)g * hstride + (uint32_t)(m - g * p.w) * qstride + tcol);
      }
    } else {
#pragma unroll
      for (int u = 0; u < QL; ++u) {
        const int q = tid + NTHR * u;
        const int row = q / CH, c = q % CH;
        const int m = min(qg * MQ + row, p.m_rows - 1);
        const int g = div_w(m, p.w_magic), j = m - g * p.w;
        qpre[u] = ld16(p.q.base + (int64_t)(h * p.group + g) * p.q.stride_head + (int64_t)j * p.q.stride_row + c * 16);
      }
    }
    if (!PASS2) {
      const __amdgpu_buffer_rsrc_t psrd = make_srd(p.planes, (uint32_t)p.n_planes * (D * ES));
      const uint32_t poff = (plane0 + trow) * (D * ES) + tcol;
#pragma unroll
      for (int u = 0; u < QL; ++u) ppre[u] = buf_ld16(psrd, poff + u * ROWS_PER_LOAD * (D * ES));
    }
    {
      const __amdgpu_buffer_rsrc_t kb_srd = make_srd(kb_ptr, (uint32_t)p.s_t * (uint32_t)kb_stride);
      const __amdgpu_buffer_rsrc_t kc_srd = make_srd(kc_ptr, (uint32_t)p.t_ctx * (uint32_t)kc_stride);
#pragma unroll
      for (int u = 0; u < KL; ++u) {
        const int q = tid + NTHR * u;
        const int row = (int)trow + u * ROWS_PER_LOAD;  // LDS row of this chunk
        if (q < n_kchunks) {
          // two loads under complementary lane masks (a select between the descriptors would be looped over)
          if (PASS2 || row < nb) kpre[u] = buf_ld16(kb_srd, (uint32_t)(b0 + row) * (uint32_t)kb_stride + tcol);
          else kpre[u] = buf_ld16(kc_srd, (uint32_t)(c0 + row - nb) * (uint32_t)kc_stride + tcol);
        } else if (q < n_chunks) {
          kpre[u] = key_chunk(q);
        }
      }
    }
    if (PASS2) {
      // sweep 2 has room for the query panel beside the keys: both go to their LDS places as they
      // arrive and the fragments are read after the one barrier further down
#pragma unroll
      for (int u = 0; u < QL; ++u) {
        const int q = tid + NTHR * u;
        sQst[(q / CH) * CHP + q % CH] = qpre[u];
      }
    } else {
      // staging area: rows [0, 256) queries, rows [256, 512) planes, pitch CHP
#pragma unroll
      for (int u = 0; u < QL; ++u) {
        const int q = tid + NTHR * u;
        smem[(q / CH) * CHP + q % CH] = qpre[u];
        smem[(MQ + q / CH) * CHP + q % CH] = ppre[u];
      }
      __syncthreads();
      {
        const uint4* arow = smem + (size_t)(hash_wave ? MQ + rt * 32 + plane_row(rl) : rt * 32 + rl) * CHP + kg;
#pragma unroll
        for (int i = 0; i < NCH; ++i) a[i] = arow[2 * i];
      }
      __syncthreads();  // fragments are in registers: the key rows may take the space
    }
#pragma unroll
    for (int u = 0; u < KL; ++u) {
      const int q = tid + NTHR * u;
      if (q < n_chunks) sK[key_slot(q)] = kpre[u];
    }
    for (int q = tid + NTHR * KL; q < n_chunks; q += NTHR) sK[key_slot(q)] = key_chunk(q);  // further plane tiles
  } else {
    if (hash_wave) {
      const int pm = min(plane0 + min(rt * 32 + plane_row(rl), max(n_pl - 1, 0)), p.n_planes - 1);
      const char* ptr = p.planes + (size_t)pm * (D * ES);
#pragma unroll
      for (int i = 0; i < NCH; ++i) a[i] = ld16(ptr + (2 * i + kg) * 16);
    } else {
      const int mc = min(qg * MQ + rt * 32 + rl, p.m_rows - 1);
      const int g = div_w(mc, p.w_magic), j = mc - g * p.w;
      const char* ptr = p.q.base + (int64_t)(h * p.group + g) * p.q.stride_head + (int64_t)j * p.q.stride_row;
#pragma unroll
      for (int i = 0; i < NCH; ++i) a[i] = ld16(ptr + (2 * i + kg) * 16);
    }
    constexpr int LDB = 4;
    for (int c0 = 0; c0 < n_chunks; c0 += NTHR * LDB) {
      uint4 pre[LDB];
#pragma unroll
      for (int u = 0; u < LDB; ++u) {
        const int q = c0 + tid + NTHR * u;
        if (q < n_chunks) pre[u] = key_chunk(q);
      }
#pragma unroll
      for (int u = 0; u < LDB; ++u) {
        const int q = c0 + tid + NTHR * u;
        if (q < n_chunks) sK[key_slot(q)] = pre[u];
      }
    }
  }
  if (!PASS2)
    for (int i = tid; i < p.hist_lds_words; i += NTHR) sHist[i] = 0u;
  for (int t = tid; t < MQ; t += NTHR) {
    const int m = min(qg * MQ + t, p.m_rows - 1);
    const int j = m - div_w(m, p.w_magic) * p.w;
    sLim[t] = p.causal ? p.lim0 + j : INT_MAX;
  }
  if (PASS2 && p.lse_complete) {
    // the caller knows every row's complete log-sum-exp (natural log -> exp2 domain): nothing to merge
    if ((tid & 3) == 0) {
      const int t = tid >> 2, m = qg * MQ + t;
      sLse[t] = m < p.m_rows ? p.row_lse[(size_t)h * p.m_rows + m] * 1.4426950408889634f : 1.0e30f;
    }
  } else if (PASS2) {
    // row log-sum-exp from the sweep-1 partials: maximum reference first, then one exp per partial
    float mm = NEG_BIG, ss = 0.0f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int r = pr_beg + 2 * u;
      if (2 * u < pr_per && r < p.n_parts) mm = fmaxf(mm, __uint_as_float(pv[u].x));
      if (2 * u < pr_per && r + 1 < p.n_parts) mm = fmaxf(mm, __uint_as_float(pv[u].z));
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int r = pr_beg + 2 * u;
      if (2 * u < pr_per && r < p.n_parts) ss = fmaf(__uint_as_float(pv[u].y), fast_exp2(__uint_as_float(pv[u].x) - mm), ss);
      if (2 * u < pr_per && r + 1 < p.n_parts) ss = fmaf(__uint_as_float(pv[u].w), fast_exp2(__uint_as_float(pv[u].z) - mm), ss);
    }
    for (int e = 8; e < pr_per; ++e) {  // more than 32 ranges per head: the rest, not prefetched
      const float2 v = pr_ptr[e];
      if (pr_beg + e < p.n_parts) lse_merge(mm, ss, v.x, v.y);
    }
    // keys outside this call, summarised by the caller as one log-sum-exp per window row, join the
    // normaliser like one more partial (natural log -> exp2 domain)
    if (p.row_lse && (tid & 3) == 0 && qg * MQ + (tid >> 2) < p.m_rows)
      lse_merge(mm, ss, p.row_lse[(size_t)h * p.m_rows + qg * MQ + (tid >> 2)] * 1.4426950408889634f, 1.0f);
    lse_merge(mm, ss, lane_xor1(mm), lane_xor1(ss));
    lse_merge(mm, ss, lane_xor2(mm), lane_xor2(ss));
    const int t = tid >> 2;
    if ((tid & 3) == 0) sLse[t] = (qg * MQ + t < p.m_rows) ? mm + fast_log2(ss) : 1.0e30f;  // padding rows: probability 0
  }
  __syncthreads();
  if (PASS2 && STAGE_A) {
    const uint4* arow = sQst + (size_t)(rt * 32 + rl) * CHP + kg;
#pragma unroll
    for (int i = 0; i < NCH; ++i) a[i] = arow[2 * i];
  }

  if (PASS2 && n_tabc > 0 && !cnt_piped) {
    // the general shape: the whole job before the main loop, eight tables at a time from the L2-resident
    // query histograms
    const int lpk = 1 << lpk_log;
    for (int kq = tid; kq < (nb << lpk_log); kq += NTHR) {
      const int key = kq >> lpk_log, sub = kq & (lpk - 1);
      const uint16_t* sk = p.sig_k + ((size_t)h * p.s_t + b0 + key) * p.n_tables + tab0c;
      int sum = 0;
      for (int tb = sub * 8; tb < n_tabc; tb += 8 * lpk) {
        uint32_t cw[4];
        const bool vec = tb + 8 <= n_tabc && ((reinterpret_cast<uintptr_t>(sk + tb) & 15) == 0);
        if (vec) {
          const uint4 v = *reinterpret_cast<const uint4*>(sk + tb);
          cw[0] = v.x; cw[1] = v.y; cw[2] = v.z; cw[3] = v.w;
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const uint32_t lo = tb + 2 * u < n_tabc ? sk[tb + 2 * u] : 0u;
            const uint32_t hi = tb + 2 * u + 1 < n_tabc ? sk[tb + 2 * u + 1] : 0u;
            cw[u] = lo | (hi << 16);
          }
        }
        const size_t hist_w = (size_t)(1 << p.n_bits) >> 1;
        // a bin's counts over the query-row groups sit in consecutive words
        const uint32_t* hist = p.qhist + (size_t)h * p.n_tables * hist_w * n_qg;
        if (n_qg == 2) {
          uint2 hv[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const uint32_t code = (cw[u >> 1] >> ((u & 1) * 16)) & 0xffffu;
            const size_t at = (size_t)(tab0c + min(tb + u, n_tabc - 1)) * hist_w + (code >> 1);
            hv[u] = *reinterpret_cast<const uint2*>(hist + at * 2);
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const uint32_t sh = (cw[u >> 1] >> ((u & 1) * 16)) & 1u ? 16 : 0;
            sum += (tb + u < n_tabc) ? (int)(((hv[u].x >> sh) & 0xffffu) + ((hv[u].y >> sh) & 0xffffu)) : 0;
          }
        } else {
          for (int g2 = 0; g2 < n_qg; ++g2) {
            uint32_t hv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              const uint32_t code = (cw[u >> 1] >> ((u & 1) * 16)) & 0xffffu;
              const size_t at = (size_t)(tab0c + min(tb + u, n_tabc - 1)) * hist_w + (code >> 1);
              hv[u] = (hist[at * n_qg + g2] >> ((code & 1u) * 16)) & 0xffffu;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) sum += (tb + u < n_tabc) ? (int)hv[u] : 0;
          }
        }
      }
      if (lpk > 1) sum += lane_xor1(sum);
      if (lpk > 2) sum += lane_xor2(sum);
      if (sub == 0) p.cnt[((size_t)qg * p.n_kv_heads + h) * p.s_t + b0 + key] = sum;
    }
  }

  if (PASS2) {
    // lane = key column, registers = window rows: a key's pooled probability is an in-lane sum
    float lse[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) lse[r] = sLse[rt * 32 + acc_row(r, kg)];
    const int t_half = (n_tiles + 1) >> 1;  // this wave's half of the tiles
    const int nt_beg = (wave >> 3) * t_half;
    const int nt_end = min(n_tiles, nt_beg + t_half);
    // pipelined count job: step s looks up tables cnt_tb + 2s and + 2s + 1 (both row groups' bins in one
    // 8-byte word pair) and adds up the pair fetched by step s - 1
    const uint32_t* cnt_hist =
        cnt_piped ? p.qhist + ((size_t)h * p.n_tables + tab0c + cnt_tb) * ((size_t)(1 << p.n_bits) >> 1) * 2 : nullptr;
    const uint32_t cnt_hw2 = (uint32_t)(1 << p.n_bits);  // words per table: 2^K / 2 bins x 2 row groups
    uint2 cnt_pa = make_uint2(0u, 0u), cnt_pb = make_uint2(0u, 0u);
    uint32_t cnt_psh = 0u;  // shifts (0 / 16) of the pending pair, packed
    int cnt_sum = 0, cnt_step = 0;
    auto cnt_advance = [&]() {
      // add up the pending pair (zeros before the first step) ...
      cnt_sum += (int)(((cnt_pa.x >> (cnt_psh & 31u)) & 0xffffu) + ((cnt_pa.y >> (cnt_psh & 31u)) & 0xffffu) +
                       ((cnt_pb.x >> (cnt_psh >> 8)) & 0xffffu) + ((cnt_pb.y >> (cnt_psh >> 8)) & 0xffffu));
      cnt_pa = make_uint2(0u, 0u);
      cnt_pb = make_uint2(0u, 0u);
      // ... and issue the next one
      if (cnt_lane && cnt_step < 4) {
        const uint32_t c0 = cnt_codes.x & 0xffffu, c1 = cnt_codes.x >> 16;
        cnt_pa = *reinterpret_cast<const uint2*>(cnt_hist + (size_t)(2 * cnt_step) * cnt_hw2 + (c0 >> 1) * 2);
        cnt_pb = *reinterpret_cast<const uint2*>(cnt_hist + (size_t)(2 * cnt_step + 1) * cnt_hw2 + (c1 >> 1) * 2);
        cnt_psh = ((c0 & 1u) * 16u) | (((c1 & 1u) * 16u) << 8);
        cnt_codes = make_uint4(cnt_codes.y, cnt_codes.z, cnt_codes.w, 0u);
      }
      ++cnt_step;
    };
    // rolled on purpose (microsecond kernels start from a cold instruction cache)
#pragma unroll 1
    for (int nt = nt_beg; nt < nt_end; ++nt) {
      const int kbase = k0 + nt * 32;
      if (cnt_piped) cnt_advance();
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
      const uint4* brow = sK + (size_t)(nt * 32 + rl) * CHP + kg;
#pragma unroll
      for (int i = 0; i < NCH; ++i) Mma<DT>::run(acc, a[i], brow[2 * i]);
      const int kidx = kbase + rl;
      const bool partial = (kbase + 32 > k1) || (p.causal && (kbase + 31 > p.lim0));  // wave-uniform
      float col = 0.0f;
      if (!partial) {
#pragma unroll
        for (int r = 0; r < 16; ++r) col += fast_exp2(fmaf(acc[r], p.scale2, -lse[r]));
      } else {
        // registers 4g .. 4g+3 of a lane are four consecutive window rows: their limits come as one 16-byte read
        const bool in_range = kidx < k1;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int4 lim4 = *reinterpret_cast<const int4*>(&sLim[rt * 32 + acc_row(4 * g4, kg)]);
          const int lims[4] = {lim4.x, lim4.y, lim4.z, lim4.w};
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float e = fast_exp2(fmaf(acc[4 * g4 + u], p.scale2, -lse[4 * g4 + u]));
            col += (in_range & (kidx <= lims[u])) ? e : 0.0f;
          }
        }
      }
      col = half_pair_sum(col);
      if (kg == 0) sCol[rt * nkr + nt * 32 + rl] = col;
    }
    if (cnt_piped) {
      // the last pending pair, and the steps a short loop did not reach, all issued before any is added
      cnt_advance();
      uint2 ra[4], rb[4];
      uint32_t rsh[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        ra[u] = cnt_pa;  // u == 0: what the call above may have issued; otherwise replaced or zero
        rb[u] = cnt_pb;
        rsh[u] = cnt_psh;
        if (u > 0) {
          ra[u] = make_uint2(0u, 0u);
          rb[u] = make_uint2(0u, 0u);
          if (cnt_lane && cnt_step < 4) {
            const uint32_t c0 = cnt_codes.x & 0xffffu, c1 = cnt_codes.x >> 16;
            ra[u] = *reinterpret_cast<const uint2*>(cnt_hist + (size_t)(2 * cnt_step) * cnt_hw2 + (c0 >> 1) * 2);
            rb[u] = *reinterpret_cast<const uint2*>(cnt_hist + (size_t)(2 * cnt_step + 1) * cnt_hw2 + (c1 >> 1) * 2);
            rsh[u] = ((c0 & 1u) * 16u) | (((c1 & 1u) * 16u) << 8);
            cnt_codes = make_uint4(cnt_codes.y, cnt_codes.z, cnt_codes.w, 0u);
          }
          ++cnt_step;
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        cnt_sum += (int)(((ra[u].x >> (rsh[u] & 31u)) & 0xffffu) + ((ra[u].y >> (rsh[u] & 31u)) & 0xffffu) +
                         ((rb[u].x >> (rsh[u] >> 8)) & 0xffffu) + ((rb[u].y >> (rsh[u] >> 8)) & 0xffffu));
      if (lpk_log > 0) cnt_sum += lane_xor1(cnt_sum);
      if (lpk_log > 1) cnt_sum += lane_xor2(cnt_sum);
      if (cnt_lane && (tid & ((1 << lpk_log) - 1)) == 0)
        p.cnt[((size_t)qg * p.n_kv_heads + h) * p.s_t + b0 + cnt_key] = cnt_sum;
    }
  } else if (!hash_wave) {
    // Sweep 1 multiplies the other way round (keys as the A operand, window rows as B): lane = window
    // row rt*32 + rl, registers = 16 keys of the tile, so a row's statistics never leave the lane.
    // Each lane keeps (ref, sum) with sum = sum_i 2^(x_i - ref) over its keys; ref is the lane's
    // maximum over the first tile and is not raised afterwards (see the overflow check below).
    const int lim = sLim[rt * 32 + rl];
    const int row = qg * MQ + rt * 32 + rl;
    if (!p.lse_complete) {  // workgroup-uniform: with complete row statistics from the caller only the hashing remains
    auto tile = [&](int nt, f32x16& acc) {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
      const uint4* krow = sK + (size_t)(nt * 32 + rl) * CHP + kg;
#pragma unroll
      for (int i = 0; i < NCH; ++i) Mma<DT>::run(acc, krow[2 * i], a[i]);
    };
    // scaled logits of a tile whose tail may be outside the range or hidden by the causal mask
    const int last_blk = min(lim - k0, nb - 1);  // last block row this window row may see (negative: none)
    auto masked = [&](int nt, f32x16& acc) {
      // register r holds the key in LDS row rb + 8*(r/4) + (r&3); the look-back rows [nb, n_rows) are always visible
      const int rb = nt * 32 + 4 * kg;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = rb + 8 * (r >> 2) + (r & 3);
        const bool vis = (row <= last_blk) | ((unsigned)(row - nb) < (unsigned)nc);  // no short circuit: straight-line code
        acc[r] = vis ? acc[r] * p.scale2 : NEG_BIG;
      }
    };
    // tiles that need the masks (wave-uniform): rows past the range, or block keys beyond the first window row's limit
    auto needs_mask = [&](int nt) {
      const int t0 = nt * 32;
      return t0 + 32 > n_rows || (p.causal && t0 < nb && k0 + min(t0 + 31, nb - 1) > p.lim0);
    };
    float ref, sum = 0.0f;
    {
      f32x16 acc;
      tile(0, acc);
      masked(0, acc);
      float mx = acc[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[r]);
      ref = mx;  // NEG_BIG when the row sees none of the lane's keys: its junk sum gets weight 0 in every merge
#pragma unroll
      for (int r = 0; r < 16; ++r) sum += fast_exp2(acc[r] - ref);
    }
#pragma unroll 1
    for (int nt = 1; nt < n_tiles; ++nt) {
      f32x16 acc;
      tile(nt, acc);
      if (!needs_mask(nt)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(acc[r], p.scale2, -ref));
      } else {
        masked(nt, acc);
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += fast_exp2(acc[r] - ref);
      }
    }
    // A later logit more than 2^7 above the first tile's maximum (exp2 domain) overflows the sum.
    // The wave then redoes its rows with a reference that follows the running maximum.
    if (__any(!(sum < 3.0e38f))) {
      ref = NEG_BIG;
      sum = 0.0f;
#pragma unroll 1
      for (int nt = 0; nt < n_tiles; ++nt) {
        f32x16 acc;
        tile(nt, acc);
        masked(nt, acc);
        float mx = ref;
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[r]);
        float add = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) add += fast_exp2(acc[r] - mx);
        sum = sum * fast_exp2(ref - mx) + add;
        ref = mx;
      }
    }
    // the two halves of the wave hold the same rows over different keys
    lse_merge(ref, sum, half_other(ref, kg), half_other(sum, kg));
    if (kg == 0 && row < p.m_rows) p.part[((size_t)h * p.m_pad + row) * p.r_pad + kr] = make_float2(ref, sum);
    }

    // SimHash codes of this wave's 32 window rows for the tables this workgroup owns (Sec. 3.3 "Recall"):
    // planes as the A operand (in plane_row order), the rows already in registers as B, so lane = row
    // and a lane's registers are 16 consecutive planes.  The codes go to sig_q and into the workgroup's
    // LDS histograms of (table, code) over the 256 rows of its query-row group.
    const uint32_t code_mask = (1u << p.n_bits) - 1u;
    const int hist_w = p.hist_lds_words ? (1 << p.n_bits) >> 1 : 0;  // words per table, 0: no histograms
#pragma unroll 1
    for (int t = 0; t < n_qpt; ++t) {
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
      const uint4* prow = sQP + (size_t)(t * 32 + plane_row(rl)) * CHP + kg;
#pragma unroll
      for (int i = 0; i < NCH; ++i) Mma<DT>::run(acc, prow[2 * i], a[i]);
      uint32_t neg = 0u;
#pragma unroll
      for (int r = 15; r >= 0; --r) neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[r]), 31);
      const uint32_t pos = ~neg & 0xffffu;
      const uint32_t other = half_other(pos, kg);
      const uint32_t word = kg ? (other | (pos << 16)) : (pos | (other << 16));
      // the tile's tables alternate between the two lanes that hold the row
      const int t_tab0 = qt0 + t * p.q_tab_per_tile;
      const int t_tabs = min(p.q_tab_per_tile, qt0 + n_qt - t_tab0);
      if (row < p.m_rows)
        for (int tt = kg; tt < t_tabs; tt += 2) {
          const uint32_t code = (word >> (tt * p.n_bits)) & code_mask;
          p.sig_q[((size_t)h * p.m_rows + row) * p.n_tables + t_tab0 + tt] = (uint16_t)code;
          if (hist_w) atomicAdd(sHist + (t_tab0 + tt - qt0) * hist_w + (code >> 1), 1u << ((code & 1u) * 16));
        }
    }
  } else {
    // hashing waves: SimHash sign bits of the range's block keys
    const int n_vt = (nb + 31) >> 5;  // look-back keys are never candidates: not hashed
#pragma unroll 1
    for (int mt = rt; mt < n_mt; mt += 8) {
      if (mt != rt) {
        const int pm = plane0 + min(mt * 32 + plane_row(rl), n_pl - 1);
        const char* ptr = p.planes + (size_t)pm * (D * ES);
#pragma unroll
        for (int i = 0; i < NCH; ++i) a[i] = ld16(ptr + (2 * i + kg) * 16);
      }
#pragma unroll 1
      for (int vt = 0; vt < n_vt; ++vt) {
        const int base = vt * 32;
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        const uint4* brow = sK + (size_t)(base + rl) * CHP + kg;
#pragma unroll
        for (int i = 0; i < NCH; ++i) Mma<DT>::run(acc, a[i], brow[2 * i]);
        // the lane's 16 accumulators are planes 16*kg .. 16*kg+15 of the tile in register order (see
        // plane_row); shifting their sign bits in from the top register down leaves plane r at bit r
        uint32_t neg = 0u;
#pragma unroll
        for (int r = 15; r >= 0; --r) neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[r]), 31);
        const uint32_t pos = ~neg & 0xffffu;  // bit = projection >= 0 (an accumulator is never -0)
        const uint32_t mask = pos | (half_other(pos, kg) << 16);
        if (kg == 0) sBits[(size_t)(base + rl) * BITS_PITCH + mt] = mask;
      }
    }
  }

  if (PASS2) {
    __syncthreads();
    for (int t = tid; t < nb; t += NTHR) {
      float v = 0.0f;
#pragma unroll
      for (int w = 0; w < 8; ++w) v += sCol[w * nkr + t];
      p.s_part[((size_t)qg * p.n_kv_heads + h) * p.s_t + b0 + t] = v;
    }
  } else {
    __syncthreads();
    // key codes: one item = (key, group of 8 tables) -> one 16-byte store where aligned
    const uint32_t code_mask = (1u << p.n_bits) - 1u;
    const int n_tg8 = (n_tab + 7) >> 3;
    const int n_items = nb * n_tg8;
    for (int it = tid; it < n_items; it += NTHR) {
      const int vr = it / n_tg8, tb = (it - vr * n_tg8) * 8;
      const uint32_t* bits = sBits + (size_t)vr * BITS_PITCH;
      uint32_t codes[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int bitpos = min(tb + u, n_tab - 1) * p.n_bits;
        const int w0 = bitpos >> 5, sh = bitpos & 31;
        const uint64_t two = (uint64_t)bits[w0] | ((uint64_t)bits[w0 + 1] << 32);
        codes[u] = (uint32_t)(two >> sh) & code_mask;
      }
      uint16_t* dst = p.sig_k + ((size_t)h * p.s_t + b0 + vr) * p.n_tables + tab0 + tb;
      if (tb + 8 <= n_tab && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0)) {
        const uint4 cv = make_uint4(codes[0] | (codes[1] << 16), codes[2] | (codes[3] << 16),
                                    codes[4] | (codes[5] << 16), codes[6] | (codes[7] << 16));
        *reinterpret_cast<uint4*>(dst) = cv;
      } else {
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (tb + u < n_tab) dst[u] = (uint16_t)codes[u];
      }
    }
    // the finished histograms of this workgroup's (row group, tables), interleaved with the other
    // groups' word by word: every word is rewritten each block, so nothing has to be cleared and no
    // global atomics are needed
    if (p.hist_lds_words && n_qt > 0) {
      const int hist_w = (1 << p.n_bits) >> 1;
      uint32_t* dst = p.qhist + ((size_t)h * p.n_tables + qt0) * hist_w * n_qg + qg;
      for (int i = tid; i < n_qt * hist_w; i += NTHR) dst[(size_t)i * n_qg] = sHist[i];
    }
    if (!p.qhist && qg == 0)  // the separate count kernel accumulates with atomics
      for (int t = tid; t < nb; t += NTHR) p.cnt[(size_t)h * p.s_t + b0 + t] = 0;
  }
}

// ---------------------------------------------------------------------------------------------
// Collision counts as a kernel of their own (codes too wide for resident histograms).  Workgroup =
// (key range, set of table groups, KV head).  All codes the workgroup needs -- its tables' codes of
// the G*W window queries and of the range's keys -- are fetched into LDS once, so that only one
// round trip to memory lies on the kernel's critical path.  Then, one table group after the other
// through the same LDS histogram (two 16-bit bins per word): the query codes are histogrammed, every
// key looks its own codes up, and the bins that were touched are cleared again.  A key's count over
// all the workgroup's tables meets in a register and costs one global atomic.
// ---------------------------------------------------------------------------------------------
constexpr int COUNT_THREADS = 1024;
constexpr int COUNT_KEYS_PER_THREAD = 8;  // keys_per_range <= COUNT_THREADS * COUNT_KEYS_PER_THREAD
__global__ __launch_bounds__(COUNT_THREADS) void count_kernel(CountParams p) {
  extern __shared__ uint32_t bins[];  // [tables_per_group << n_bits] / 2 words, then the staged codes
  const int tid = threadIdx.x;
  const int kr = blockIdx.x, h = blockIdx.z;
  const int nq = p.group * p.w;
  const int i0 = kr * p.keys_per_range;
  const int i1 = min(i0 + p.keys_per_range, p.s_t);
  const int n_keys = i1 - i0;
  const int t_first = blockIdx.y * p.groups_per_wg * p.tables_per_group;            // the workgroup's tables
  const int ntw = min(p.groups_per_wg * p.tables_per_group, p.n_tables - t_first);  // > 0 by the grid's construction
  const int n_bin_words = (p.tables_per_group << p.n_bits) >> 1;
  uint16_t* sQ = reinterpret_cast<uint16_t*>(bins + ((n_bin_words + 3) & ~3));  // [ntw][nq]
  uint16_t* sKc = sQ + ((ntw * nq + 7) & ~7);                                   // [n_keys][ntw]
  // 1. everything from memory, issued back to back: query codes (transposed to table-major), key codes
  const uint16_t* gq = p.sig_q + (size_t)h * nq * p.n_tables + t_first;
  const uint16_t* gk = p.sig_k + ((size_t)h * p.s_t + i0) * p.n_tables + t_first;
  const bool vec8 = (ntw & 7) == 0 && (p.n_tables & 7) == 0 && (t_first & 7) == 0;  // rows of whole aligned 16-byte groups
  if (vec8) {
    const int g8 = ntw >> 3;
    for (int e = tid; e < nq * g8; e += COUNT_THREADS) {
      const int qrow = e / g8, gi = e - qrow * g8;
      const uint4 v = ld16(gq + (size_t)qrow * p.n_tables + gi * 8);
      const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int u = 0; u < 8; ++u) sQ[(gi * 8 + u) * nq + qrow] = (uint16_t)(wv[u >> 1] >> ((u & 1) * 16));
    }
    for (int e = tid; e < n_keys * g8; e += COUNT_THREADS) {
      const int key = e / g8, gi = e - key * g8;
      *reinterpret_cast<uint4*>(sKc + (size_t)key * ntw + gi * 8) = ld16(gk + (size_t)key * p.n_tables + gi * 8);
    }
  } else {
    for (int e = tid; e < nq * ntw; e += COUNT_THREADS) {
      const int qrow = e / ntw, tl = e - qrow * ntw;
      sQ[tl * nq + qrow] = gq[(size_t)qrow * p.n_tables + tl];
    }
    for (int e = tid; e < n_keys * ntw; e += COUNT_THREADS) {
      const int key = e / ntw, tl = e - key * ntw;
      sKc[(size_t)key * ntw + tl] = gk[(size_t)key * p.n_tables + tl];
    }
  }
  if ((n_bin_words & 3) == 0) {
    uint4* b4 = reinterpret_cast<uint4*>(bins);
    for (int i = tid; i < n_bin_words / 4; i += COUNT_THREADS) b4[i] = make_uint4(0u, 0u, 0u, 0u);
  } else {
    for (int i = tid; i < n_bin_words; i += COUNT_THREADS) bins[i] = 0u;
  }
  int sum[COUNT_KEYS_PER_THREAD];
#pragma unroll
  for (int k = 0; k < COUNT_KEYS_PER_THREAD; ++k) sum[k] = 0;
  __syncthreads();
  // 2. the table groups, one after the other, in LDS only
  for (int g0 = 0; g0 < ntw; g0 += p.tables_per_group) {
    const int tga = min(p.tables_per_group, ntw - g0);
    for (int e = tid; e < nq * tga; e += COUNT_THREADS) {
      const int tl = e / nq, qrow = e - tl * nq;
      const uint32_t idx = ((uint32_t)tl << p.n_bits) | sQ[(g0 + tl) * nq + qrow];
      atomicAdd(&bins[idx >> 1], 1u << ((idx & 1u) * 16));
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < COUNT_KEYS_PER_THREAD; ++k) {
      const int key = tid + k * COUNT_THREADS;
      if (key < n_keys) {
        const uint16_t* kc = sKc + (size_t)key * ntw + g0;
        for (int tl = 0; tl < tga; ++tl) {
          const uint32_t idx = ((uint32_t)tl << p.n_bits) | kc[tl];
          sum[k] += (bins[idx >> 1] >> ((idx & 1u) * 16)) & 0xffffu;
        }
      }
    }
    if (g0 + p.tables_per_group < ntw) {  // block-uniform: another group follows
      __syncthreads();                    // lookups done before the bins are cleared
      // only the bins of this group's query codes are non-zero
      for (int e = tid; e < nq * tga; e += COUNT_THREADS) {
        const int tl = e / nq, qrow = e - tl * nq;
        const uint32_t idx = ((uint32_t)tl << p.n_bits) | sQ[(g0 + tl) * nq + qrow];
        bins[idx >> 1] = 0u;
      }
      __syncthreads();
    }
  }
#pragma unroll
  for (int k = 0; k < COUNT_KEYS_PER_THREAD; ++k) {
    const int key = tid + k * COUNT_THREADS;
    if (key < n_keys) atomicAdd(&p.cnt[(size_t)h * p.s_t + i0 + key], sum[k]);
  }
}

// ---------------------------------------------------------------------------------------------
// Selection.  One 1024-thread workgroup per KV head; thread t owns the EPT consecutive positions
// starting at t*EPT, so thread order is index order.  The k-th largest key is found by a radix
// descent over 8-bit digits from the top (LDS histogram, four interleaved copies against same-
// address atomics), which also yields how many keys equal to the threshold are still needed; those
// are taken in index order via a prefix count.
//
// The kernel is a chain of short workgroup-wide phases, so each round of the descent is kept to ONE
// barrier: after the histogram is complete every wave scans it redundantly (lane l owns digits
// 4l..4l+3) and learns the chosen digit through a wave broadcast; nothing goes back through LDS.  Three
// histogram buffers rotate, the one read in round r being cleared during round r + 1 and reused in
// round r + 3.
// ---------------------------------------------------------------------------------------------
//
// FUSED = true also appends: a head's selection is then computed redundantly by `split` workgroups
// (the inputs are L2-resident and the compute units would idle otherwise), and each of them copies
// its share of the kept K/V rows to the cache tail.  That saves a kernel boundary, which on this
// chip costs about as much as the whole copy.
constexpr int SEL_COPIES = 4;
constexpr int SEL_BUFFERS = 3;

template <int EPT, bool FUSED>
__global__ __launch_bounds__(1024) void select_kernel(SelectParams p, AppendParams ap, int split) {
  __shared__ __align__(16) uint32_t sHist[SEL_BUFFERS][SEL_COPIES][256];
  __shared__ int sWave[16];
  __shared__ uint32_t sList[64];  // keys that share the threshold's leading digits
  __shared__ int sListN;
  __shared__ uint32_t sMaxCnt;  // largest collision count among the candidates
  __shared__ int sKeep[FUSED ? 1024 : 1];  // FUSED: the kept indices this workgroup copies
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n_sel_wg = p.n_kv_heads * split;
  // the workgroups that share a head (and read the same scores and counts) sit on one XCD
  const int sel_id = xcd_major(blockIdx.x, n_sel_wg);
  const int h = FUSED ? sel_id / split : sel_id;
  const int part = FUSED ? sel_id - h * split : 0;
  uint32_t key[EPT], c2[EPT];
  bool inr[EPT], cand[EPT], sel[EPT];
  {
    // scores and counts arrive in up to two parts in the common cases: issue every load before the
    // first use (a loop with a run-time part count would serialise one memory round trip per load)
    float sc[EPT];
    int cc[EPT];
    const size_t hoff = (size_t)h * p.s_t, poff = (size_t)p.n_kv_heads * p.s_t;
    // 16-byte loads when a thread's EPT positions are whole aligned quads inside the block
    const bool quads = EPT % 4 == 0 && (p.s_t & 3) == 0 && (tid + 1) * EPT <= p.s_t;
    if (p.n_qgroups <= 2 && p.n_cnt_parts <= 2 && __all(quads)) {
      constexpr int NQ = EPT >= 4 ? EPT / 4 : 1;
      const bool s2 = p.n_qgroups > 1, c2p = p.n_cnt_parts > 1;
      uint4 a0[NQ], a1[NQ], b0[NQ], b1[NQ];
      const uint4* ps = reinterpret_cast<const uint4*>(p.s_part + hoff + (size_t)tid * EPT);
      const uint4* pc = reinterpret_cast<const uint4*>(p.cnt + hoff + (size_t)tid * EPT);
      const size_t pq = poff / 4;
#pragma unroll
      for (int v = 0; v < NQ; ++v) {
        a0[v] = ps[v];
        a1[v] = s2 ? ps[pq + v] : make_uint4(0u, 0u, 0u, 0u);
        b0[v] = pc[v];
        b1[v] = c2p ? pc[pq + v] : make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int v = 0; v < NQ; ++v) {
        const uint32_t x0[4] = {a0[v].x, a0[v].y, a0[v].z, a0[v].w}, x1[4] = {a1[v].x, a1[v].y, a1[v].z, a1[v].w};
        const uint32_t y0[4] = {b0[v].x, b0[v].y, b0[v].z, b0[v].w}, y1[4] = {b1[v].x, b1[v].y, b1[v].z, b1[v].w};
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (4 * v + u < EPT) {
            sc[4 * v + u] = __uint_as_float(x0[u]) + __uint_as_float(x1[u]);
            cc[4 * v + u] = (int)(y0[u] + y1[u]);
          }
      }
    } else if (EPT == 2 && p.n_qgroups <= 2 && p.n_cnt_parts <= 2 &&
               __all((p.s_t & 1) == 0 && (tid + 1) * EPT <= p.s_t)) {
      // two positions per thread: 8-byte loads
      const bool s2 = p.n_qgroups > 1, c2p = p.n_cnt_parts > 1;
      const uint2* ps = reinterpret_cast<const uint2*>(p.s_part + hoff + (size_t)tid * 2);
      const uint2* pc = reinterpret_cast<const uint2*>(p.cnt + hoff + (size_t)tid * 2);
      const size_t pq = poff / 2;
      const uint2 a0 = ps[0], a1 = s2 ? ps[pq] : make_uint2(0u, 0u);
      const uint2 b0 = pc[0], b1 = c2p ? pc[pq] : make_uint2(0u, 0u);
      sc[0] = __uint_as_float(a0.x) + __uint_as_float(a1.x);
      sc[EPT - 1] = __uint_as_float(a0.y) + __uint_as_float(a1.y);
      cc[0] = (int)(b0.x + b1.x);
      cc[EPT - 1] = (int)(b0.y + b1.y);
    } else if (p.n_qgroups <= 2 && p.n_cnt_parts <= 2) {
      const bool s2 = p.n_qgroups > 1, c2p = p.n_cnt_parts > 1;
      float a0[EPT], a1[EPT];
      int b0[EPT], b1[EPT];
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const int i = min(tid * EPT + e, p.s_t - 1);
        a0[e] = p.s_part[hoff + i];
        a1[e] = s2 ? p.s_part[poff + hoff + i] : 0.0f;
        b0[e] = p.cnt[hoff + i];
        b1[e] = c2p ? p.cnt[poff + hoff + i] : 0;
      }
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        sc[e] = a0[e] + a1[e];
        cc[e] = b0[e] + b1[e];
      }
    } else {
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const int i = min(tid * EPT + e, p.s_t - 1);
        float sacc = 0.0f;
        int cacc = 0;
        for (int q = 0; q < p.n_qgroups; ++q) sacc += p.s_part[(size_t)q * poff + hoff + i];
        for (int q = 0; q < p.n_cnt_parts; ++q) cacc += p.cnt[(size_t)q * poff + hoff + i];
        sc[e] = sacc;
        cc[e] = cacc;
      }
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const int i = tid * EPT + e;
      inr[e] = i < p.s_t;
      cand[e] = inr[e] && i >= p.n_anchor && i < p.s_t - p.n_local;
      sel[e] = false;
      const float sv = sc[e] * p.inv_m;
      key[e] = inr[e] ? __float_as_uint(sv) : 0u;  // scores are >= 0: their bit patterns order like the values
      c2[e] = inr[e] ? (uint32_t)cc[e] : 0u;
      if (inr[e] && part == 0) {
        if (p.s_exact) p.s_exact[hoff + i] = sv;
        if (p.cnt_out) p.cnt_out[hoff + i] = cc[e];
      }
    }
  }

  // exclusive prefix of per-thread counts over the block, in thread (= index) order
  auto block_excl_scan = [&](int v) -> int {
    const int inc = wave_incl_scan(v);
    __syncthreads();  // sWave free again
    if (lane == 63) sWave[wave] = inc;
    __syncthreads();
    // the 16 wave totals, one per lane of every 16-lane row, prefix-summed inside the row
    int wt = sWave[lane & 15];
    wt += __builtin_amdgcn_update_dpp(0, wt, 0x111, 0xf, 0xf, true);  // row_shr:1
    wt += __builtin_amdgcn_update_dpp(0, wt, 0x112, 0xf, 0xf, true);  // row_shr:2
    wt += __builtin_amdgcn_update_dpp(0, wt, 0x114, 0xf, 0xf, true);  // row_shr:4
    wt += __builtin_amdgcn_update_dpp(0, wt, 0x118, 0xf, 0xf, true);  // row_shr:8
    const int base = wave ? __builtin_amdgcn_readlane(wt, wave - 1) : 0;
    return base + inc - v;
  };
  int round_no = 0;  // rounds of both descents so far: selects the histogram buffer
  // The k-th largest value among the active elements (val < 2^(8*n_digits)): returns it in thr, with `need`
  // = how many of the `in_bin` active elements equal to it belong to the top k.  All three block-uniform.
  auto kth_largest = [&](const uint32_t* val, const bool* active, int k, int n_digits, uint32_t& thr, int& need, int& in_bin) {
    uint32_t prefix = 0u, pmask = 0u;
    need = k;
    in_bin = 0;
    for (int dg = n_digits - 1; dg >= 0; --dg) {
      const int shift = 8 * dg;
      const int buf = round_no % SEL_BUFFERS;
      // buffer `buf` is zero here: cleared at kernel start or two rounds ago
#pragma unroll
      for (int e = 0; e < EPT; ++e)
        if (active[e] && (val[e] & pmask) == prefix) atomicAdd(&sHist[buf][lane & 3][(val[e] >> shift) & 255u], 1u);
      __syncthreads();
      // the buffer of the round before has been read by every wave: clear it for the round after next
      if (round_no > 0) sHist[(round_no - 1) % SEL_BUFFERS][tid >> 8][tid & 255] = 0u;
      ++round_no;
      // every wave: lane l owns digits 4l..4l+3; walk from the top digit down
      uint4 q[SEL_COPIES];
#pragma unroll
      for (int b = 0; b < SEL_COPIES; ++b) q[b] = *reinterpret_cast<const uint4*>(&sHist[buf][b][4 * lane]);
      const uint32_t c[4] = {q[0].x + q[1].x + q[2].x + q[3].x, q[0].y + q[1].y + q[2].y + q[3].y,
                             q[0].z + q[1].z + q[2].z + q[3].z, q[0].w + q[1].w + q[2].w + q[3].w};
      const int mine = (int)(c[0] + c[1] + c[2] + c[3]);
      const int incl = wave_incl_scan(mine);
      const int total = __builtin_amdgcn_readlane(incl, 63);
      int above = total - incl;  // keys in digits owned by higher lanes
      // the digit holding the need-th largest key: above < need <= above + count (one lane, one digit)
      int p_dig = -1, p_need = 0, p_cnt = 0;
#pragma unroll
      for (int b = 3; b >= 0; --b) {
        const bool hit = above < need && need <= above + (int)c[b];
        p_dig = hit ? 4 * lane + b : p_dig;
        p_need = hit ? need - above : p_need;
        p_cnt = hit ? (int)c[b] : p_cnt;
        above += (int)c[b];
      }
      const uint64_t hit_mask = __ballot(p_dig >= 0);
      const int src = hit_mask ? __builtin_ctzll(hit_mask) : 0;
      prefix |= (uint32_t)__builtin_amdgcn_readlane(p_dig, src) << shift;
      pmask |= 255u << shift;
      need = __builtin_amdgcn_readlane(p_need, src);
      in_bin = __builtin_amdgcn_readlane(p_cnt, src);
      if (dg > 0 && in_bin <= 64) {  // block-uniform
        // few keys share the chosen digits: every wave ranks them against each other (one key per
        // lane) instead of descending through the remaining digits
#pragma unroll
        for (int e = 0; e < EPT; ++e)
          if (active[e] && (val[e] & pmask) == prefix) sList[atomicAdd(&sListN, 1)] = val[e];
        __syncthreads();
        if (tid == 0) sListN = 0;  // next used after at least one more barrier
        const uint32_t v = lane < in_bin ? sList[lane] : 0u;
        int gt = 0, ge = 0;
        for (int j = 0; j < in_bin; ++j) {
          const uint32_t u = (uint32_t)__builtin_amdgcn_readlane((int)v, j);
          gt += u > v ? 1 : 0;
          ge += u >= v ? 1 : 0;
        }
        const uint64_t m2 = __ballot(lane < in_bin && gt < need && need <= ge);  // equal keys agree on the values
        const int s2 = m2 ? __builtin_ctzll(m2) : 0;
        prefix = (uint32_t)__builtin_amdgcn_readlane((int)v, s2);
        const int gt_s = __builtin_amdgcn_readlane(gt, s2), ge_s = __builtin_amdgcn_readlane(ge, s2);
        need -= gt_s;
        in_bin = ge_s - gt_s;
        break;
      }
    }
    thr = prefix;
  };

  for (int i = tid; i < SEL_BUFFERS * SEL_COPIES * 256; i += 1024) (&sHist[0][0][0])[i] = 0u;
  if (tid == 0) {
    sMaxCnt = 0u;
    sListN = 0;
  }
  __syncthreads();
  {
    // Collision counts are mostly tiny, so their top byte is usually zero for every candidate: the
    // block-wide maximum (one LDS atomic per wave, ordered by the barriers of the first stage) tells
    // how many digits the second stage really needs.
    uint32_t mx = 0u;
#pragma unroll
    for (int e = 0; e < EPT; ++e) mx = max(mx, cand[e] ? c2[e] : 0u);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, off));
    if (lane == 0 && mx) atomicMax(&sMaxCnt, mx);
  }
  // stage 1 (Alg. 1 step 4): the k_exact candidates ranked first by (score descending, index ascending)
  if (p.k_exact > 0) {  // block-uniform
    uint32_t thr;
    int need, in_bin;
    kth_largest(key, cand, p.k_exact, 4, thr, need, in_bin);
    int rank = 0;
    if (need < in_bin) {  // ties at the threshold (rare for scores): the lowest indices win
      int n_eq = 0;
#pragma unroll
      for (int e = 0; e < EPT; ++e) n_eq += (cand[e] && key[e] == thr) ? 1 : 0;
      rank = block_excl_scan(n_eq);
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if (cand[e]) {
        if (key[e] > thr) {
          sel[e] = true;
        } else if (key[e] == thr) {
          if (need >= in_bin || rank < need) sel[e] = true;
          ++rank;
        }
      }
    }
  } else {
    __syncthreads();  // orders the atomicMax above before its read below
  }
  // stage 2 (Alg. 1 steps 5-7): the k_lsh remaining candidates ranked first by (count descending, index
  // ascending).  Only the threshold is found here; its ties are resolved inside the compaction below.
  bool act2[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) act2[e] = cand[e] && !sel[e];
  uint32_t thr2 = 0xffffffffu;  // k_lsh == 0: nothing of the residual is kept
  int need2 = 0, in2 = 0;
  if (p.k_lsh > 0) {
    const int cnt_digits = sMaxCnt < 256u ? 1 : (sMaxCnt < 65536u ? 2 : (sMaxCnt < (1u << 24) ? 3 : 4));
    kth_largest(c2, act2, p.k_lsh, min(cnt_digits, (p.cnt_bits + 7) >> 3), thr2, need2, in2);
  }

  // Compaction (Alg. 1 step 8 and the Sec. 3.1 partition).  Kept for certain: protected positions, stage-1
  // winners, residual candidates with a count above the threshold.  Of the residual candidates AT the
  // threshold the first need2 in index order are kept.  One packed prefix count (certain << 16 | ties) gives
  // every element its output rank: certain ones before it plus min(ties before it, need2).
  int packed = 0;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const bool tie = act2[e] && c2[e] == thr2;
    sel[e] = inr[e] && (!cand[e] || sel[e] || (act2[e] && c2[e] > thr2 && p.k_lsh > 0));
    act2[e] = tie;
    packed += (sel[e] ? 1 << 16 : 0) + (tie ? 1 : 0);
  }
  const int pre = block_excl_scan(packed);
  int n_sure = pre >> 16, n_tie = pre & 0xffff;
  const int b_t = p.n_anchor + p.n_local + p.k_exact + p.k_lsh;
  // FUSED: this workgroup copies output ranks [r0, r1)
  const int per = (b_t + split - 1) / split;
  const int r0 = FUSED ? min(part * per, b_t) : 0, r1 = FUSED ? min(r0 + per, b_t) : b_t;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const bool kept = sel[e] || (act2[e] && n_tie < need2);
    if (kept) {
      const int pos = n_sure + min(n_tie, need2);
      if (pos >= r0 && pos < r1) {
        p.keep[(size_t)h * b_t + pos] = tid * EPT + e;
        if (FUSED) sKeep[pos - r0] = tid * EPT + e;
      }
    }
    n_sure += sel[e] ? 1 : 0;
    n_tie += act2[e] ? 1 : 0;
  }
  if (FUSED) {
    __syncthreads();
    const int cpr = ap.row_bytes / 16;
    const int n_copy = (r1 - r0) * cpr;
    // two chunk pairs per thread and step, all four loads in flight before the first store
    for (int t0 = tid; t0 < n_copy; t0 += 2048) {
      const int t1 = t0 + 1024;
      const bool two = t1 < n_copy;
      const int row0 = t0 / cpr, c0 = t0 - row0 * cpr;
      const int row1 = two ? t1 / cpr : row0, c1 = two ? t1 - row1 * cpr : c0;
      const int src0 = sKeep[row0], src1 = sKeep[row1];
      const char* kh = ap.kb.base + (int64_t)h * ap.kb.stride_head;
      const char* vh = ap.vb.base + (int64_t)h * ap.vb.stride_head;
      const uint4 k0v = ld16(kh + (int64_t)src0 * ap.kb.stride_row + c0 * 16);
      const uint4 v0v = ld16(vh + (int64_t)src0 * ap.vb.stride_row + c0 * 16);
      const uint4 k1v = ld16(kh + (int64_t)src1 * ap.kb.stride_row + c1 * 16);
      const uint4 v1v = ld16(vh + (int64_t)src1 * ap.vb.stride_row + c1 * 16);
      const int64_t dst_h = (int64_t)h * ap.cache_stride_head + (ap.cache_len + r0) * (int64_t)ap.row_bytes;
      const int64_t pos_h = (int64_t)h * ap.pos_stride_head + ap.cache_len + r0;
      st16_stream(ap.k_cache + dst_h + (int64_t)row0 * ap.row_bytes + c0 * 16, k0v);
      st16_stream(ap.v_cache + dst_h + (int64_t)row0 * ap.row_bytes + c0 * 16, v0v);
      if (c0 == 0) ap.cache_pos[pos_h + row0] = ap.block_pos0 + src0;
      if (two) {
        st16_stream(ap.k_cache + dst_h + (int64_t)row1 * ap.row_bytes + c1 * 16, k1v);
        st16_stream(ap.v_cache + dst_h + (int64_t)row1 * ap.row_bytes + c1 * 16, v1v);
        if (c1 == 0) ap.cache_pos[pos_h + row1] = ap.block_pos0 + src1;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Append: every thread moves one 16-byte chunk of one kept K row and the matching V chunk.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void append_kernel(AppendParams p) {
  const int h = blockIdx.y;
  const int cpr = p.row_bytes / 16;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int row = (int)(t / cpr), c = (int)(t % cpr);
  if (row >= p.b_t) return;
  const int src = min(max(p.keep[(size_t)h * p.keep_stride_head + row], 0), p.s_t - 1);
  const int64_t dst_off = (int64_t)h * p.cache_stride_head + (p.cache_len + row) * (int64_t)p.row_bytes + c * 16;
  const uint4 kv = ld16(p.kb.base + (int64_t)h * p.kb.stride_head + (int64_t)src * p.kb.stride_row + c * 16);
  const uint4 vv = ld16(p.vb.base + (int64_t)h * p.vb.stride_head + (int64_t)src * p.vb.stride_row + c * 16);
  *reinterpret_cast<uint4*>(p.k_cache + dst_off) = kv;
  *reinterpret_cast<uint4*>(p.v_cache + dst_off) = vv;
  if (c == 0) p.cache_pos[(int64_t)h * p.pos_stride_head + p.cache_len + row] = p.block_pos0 + src;
}

// ---------------------------------------------------------------------------------------------
// Global-consensus accumulation (Alg. 1 step 3 summed over layers and heads; likewise the counts of
// step 6): one layer's pooled scores and counts, summed over its KV heads in head order, are written
// to or added onto [S] accumulators.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void accumulate_kernel(AccumParams p) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= p.s_t) return;
  const size_t poff = (size_t)p.n_kv_heads * p.s_t;
  float s = 0.0f;
  int c = 0;
  for (int h = 0; h < p.n_kv_heads; ++h) {
    float sh = 0.0f;
    for (int q = 0; q < p.n_qgroups; ++q) sh += p.s_part[q * poff + (size_t)h * p.s_t + i];
    s += sh * p.inv_m;
    for (int q = 0; q < p.n_cnt_parts; ++q) c += p.cnt[q * poff + (size_t)h * p.s_t + i];
  }
  p.score[i] = p.accumulate ? p.score[i] + s : s;
  p.count[i] = p.accumulate ? p.count[i] + c : c;
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
// offset of the small per-row arrays = size of the larger of the two big LDS layouts of a sweep
size_t sweep_lds_tail_offset(int dtype, int head_dim, bool pass2, int range_keys, int q_tiles, int hist_lds_words) {
  const int es = dtype == DT_BF16 ? 2 : 4;
  const int ch = head_dim * es / 16;
  const size_t pitch = (size_t)(ch + 1) * 16;
  const size_t bits = (((size_t)range_keys * BITS_PITCH + 3) / 4) * 16;
  // sweep 2 keeps its query panel beside the keys; sweep 1 stages queries and planes in the space its
  // steady-state arrays take over afterwards
  const size_t panel = ch <= 16 ? (size_t)PASS_ROWS * pitch : 0;
  const size_t steady = range_keys * pitch + (pass2 ? (size_t)8 * range_keys * 4 + panel
                                                     : bits + (size_t)q_tiles * 32 * pitch + (size_t)hist_lds_words * 4);
  const size_t staging = pass2 ? 0 : 2 * panel;
  return ((steady > staging ? steady : staging) + 15) & ~(size_t)15;
}

size_t sweep_lds_bytes(int dtype, int head_dim, bool pass2, int range_keys, int q_tiles, int hist_lds_words) {
  return sweep_lds_tail_offset(dtype, head_dim, pass2, range_keys, q_tiles, hist_lds_words) + (size_t)PASS_ROWS * 8;
}

template <int DT, int D, bool PASS2>
static hipError_t launch_pass_t(const PassParams& p, hipStream_t st) {
  dim3 grid((PASS2 ? p.s2_ranges : p.n_ranges) * p.n_qgroups * p.n_kv_heads);
  PassParams q = p;
  if (PASS2) {  // sweep 2 has its own ranges over the block keys only
    q.n_ranges = p.s2_ranges;
    q.n_ctx_ranges = 0;
    q.blk_per_range = q.keys_per_range = p.s2_blk_per_range;
    q.ctx_per_range = 0;
  }
  q.lds_tail_offset = (int)sweep_lds_tail_offset(DT, D, PASS2, q.keys_per_range, p.q_tiles, p.hist_lds_words);
  const size_t lds = sweep_lds_bytes(DT, D, PASS2, q.keys_per_range, p.q_tiles, p.hist_lds_words);
  hipLaunchKernelGGL((pass_kernel<DT, D, PASS2>), grid, dim3(PASS_WAVES * 64), lds, st, q);
  return hipGetLastError();
}

template <bool PASS2>
static hipError_t launch_pass_any(int dtype, int head_dim, const PassParams& p, hipStream_t st) {
  if (dtype == DT_BF16 && head_dim == 128) return launch_pass_t<DT_BF16, 128, PASS2>(p, st);
  if (dtype == DT_BF16 && head_dim == 64) return launch_pass_t<DT_BF16, 64, PASS2>(p, st);
  if (dtype == DT_F32 && head_dim == 128) return launch_pass_t<DT_F32, 128, PASS2>(p, st);
  if (dtype == DT_F32 && head_dim == 64) return launch_pass_t<DT_F32, 64, PASS2>(p, st);
  return hipErrorInvalidValue;
}

hipError_t launch_sweep1(int dtype, int head_dim, const PassParams& p, hipStream_t st) {
  return launch_pass_any<false>(dtype, head_dim, p, st);
}
hipError_t launch_sweep2(int dtype, int head_dim, const PassParams& p, hipStream_t st) {
  return launch_pass_any<true>(dtype, head_dim, p, st);
}

template <int DT, int D>
static hipError_t pass_attrs() {
  const void* fns[] = {reinterpret_cast<const void*>(&pass_kernel<DT, D, false>), reinterpret_cast<const void*>(&pass_kernel<DT, D, true>)};
  for (const void* f : fns) {
    hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t init_kernel_attributes() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&count_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e == hipSuccess) e = pass_attrs<DT_BF16, 128>();
  if (e == hipSuccess) e = pass_attrs<DT_BF16, 64>();
  if (e == hipSuccess) e = pass_attrs<DT_F32, 128>();
  if (e == hipSuccess) e = pass_attrs<DT_F32, 64>();
  return e;
}

int score_max_range() { return SCORE_MAX_RANGE; }
int sweep_rows_per_group() { return PASS_ROWS; }

size_t count_lds_bytes(int n_bits, int tables_per_group, int groups_per_wg, int n_query_rows, int keys_per_range) {
  const size_t bin_words = (((size_t)tables_per_group << n_bits) / 2 + 3) & ~(size_t)3;
  const size_t ntw = (size_t)groups_per_wg * tables_per_group;
  return bin_words * 4 + ((ntw * n_query_rows + 7) & ~(size_t)7) * 2 + ntw * keys_per_range * 2 + 16;
}

hipError_t launch_count(const CountParams& p, int n_kv_heads, hipStream_t st) {
  const int n_tg = (p.n_tables + p.tables_per_group - 1) / p.tables_per_group;
  const int n_wg_t = (n_tg + p.groups_per_wg - 1) / p.groups_per_wg;
  const int n_kr = (p.s_t + p.keys_per_range - 1) / p.keys_per_range;
  if (p.keys_per_range > COUNT_THREADS * COUNT_KEYS_PER_THREAD) return hipErrorInvalidValue;
  const size_t lds = count_lds_bytes(p.n_bits, p.tables_per_group, p.groups_per_wg, p.group * p.w, p.keys_per_range);
  if (lds > 160 * 1024) return hipErrorInvalidValue;
  dim3 grid(n_kr, n_wg_t, n_kv_heads);
  hipLaunchKernelGGL(count_kernel, grid, dim3(COUNT_THREADS), lds, st, p);
  return hipGetLastError();
}

int count_max_keys_per_range() { return COUNT_THREADS * COUNT_KEYS_PER_THREAD; }

hipError_t launch_accumulate(const AccumParams& p, hipStream_t st) {
  hipLaunchKernelGGL(accumulate_kernel, dim3((p.s_t + 255) / 256), dim3(256), 0, st, p);
  return hipGetLastError();
}

template <bool FUSED>
static hipError_t launch_select_t(const SelectParams& p, const AppendParams& ap, int split, hipStream_t st) {
  const int ept = (p.s_t + 1023) / 1024;
  // `split` workgroups per head select (and, fused, copy)
  dim3 grid(p.n_kv_heads * split);
  if (ept <= 1) hipLaunchKernelGGL((select_kernel<1, FUSED>), grid, dim3(1024), 0, st, p, ap, split);
  else if (ept <= 2) hipLaunchKernelGGL((select_kernel<2, FUSED>), grid, dim3(1024), 0, st, p, ap, split);
  else if (ept <= 4) hipLaunchKernelGGL((select_kernel<4, FUSED>), grid, dim3(1024), 0, st, p, ap, split);
  else if (ept <= 8) hipLaunchKernelGGL((select_kernel<8, FUSED>), grid, dim3(1024), 0, st, p, ap, split);
  else if (ept <= 16) hipLaunchKernelGGL((select_kernel<16, FUSED>), grid, dim3(1024), 0, st, p, ap, split);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_select(const SelectParams& p, hipStream_t st) {
  AppendParams none = {};
  return launch_select_t<false>(p, none, 1, st);
}

hipError_t launch_select_append(const SelectParams& p, const AppendParams& ap, int n_cu, int split_override, hipStream_t st) {
  // enough workgroups per head to fill the chip, each copying at most 1024 rows
  const int b_t = p.n_anchor + p.n_local + p.k_exact + p.k_lsh;
  int split = split_override > 0 ? split_override : n_cu / p.n_kv_heads;
  if (split < 1) split = 1;
  while ((b_t + split - 1) / split > 1024) ++split;
  return launch_select_t<true>(p, ap, split, st);
}

hipError_t launch_append(const AppendParams& p, int n_kv_heads, hipStream_t st) {
  const int64_t n_chunks = (int64_t)p.b_t * (p.row_bytes / 16);
  if (n_chunks == 0) return hipSuccess;
  dim3 grid((unsigned)((n_chunks + 255) / 256), n_kv_heads);
  hipLaunchKernelGGL(append_kernel, grid, dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace lkv
