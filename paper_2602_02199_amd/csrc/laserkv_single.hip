// One sweep per block when the caller supplies every window row's complete log-sum-exp (Sec. 3.3 "Precision":
// the exact score is the attention the model already computes): the block's keys are read once and, from the
// same LDS rows, hashed (Sec. 3.3 "Recall"), scored (Alg. 1 step 3) and counted (Alg. 1 step 6).
//
// Workgroup = (range of <= 128 block keys, KV head), 16 waves; wave w keeps window rows 32w .. 32w+31 (up to
// 512 rows: the whole GQA group's window) and, for the key hashing, one 32-plane tile in registers.
//
//   1. SimHash codes of the window rows for the few tables this workgroup owns, histogrammed in LDS and
//      published to global memory with a per-table flag;
//   2. sign bits of the range's keys for every table; pooled probabilities exp(logit - row_lse) of the keys;
//   3. collision counts: every key looks its codes up in the 32 (L) published histograms.
//
// Step 3 depends on other workgroups of the same head, which normally published long before.  The wait on a
// flag is bounded: a workgroup that does not see a table in time hashes the window rows for that table itself
// (they are in its registers), writes the same histogram and sets the flag, so no workgroup ever depends on
// another one being resident.  Flags carry an epoch that the last workgroup of a launch advances on the
// device, so replays of a captured launch never see the flags of an earlier one.
#include "laserkv_device.h"
#include "laserkv_kernels.h"

#include <limits.h>

namespace lkv {

constexpr int SG_WAVES = 16;
constexpr int SG_THREADS = SG_WAVES * 64;
constexpr int SG_ROWS = 32 * SG_WAVES;  // window rows per workgroup
constexpr int SG_MAX_KEYS = 128;        // block keys per workgroup at most
constexpr int SG_MAX_QTILES = 4;        // 32-plane tiles of the workgroup's own tables
constexpr int SG_BITS_PITCH = 17;       // words per key in the sign-bit scratch (<= 16 plane tiles)
constexpr int SG_LPK = 8;               // lanes per key in the count step

// Histograms and flags travel between workgroups (possibly on different XCDs, whose L2s are not coherent with
// each other) as device-scope atomic stores and loads, which are served at the memory side instead of from an
// XCD's L2: no L2 write-back or invalidation is needed, only the order "histogram words acknowledged, then the
// flag" at the producer and "flag seen, then the look-ups issued" at the consumer.
__device__ __forceinline__ void sg_store(uint32_t* p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ uint32_t sg_load(const uint32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

__device__ __forceinline__ bool sg_wait_flag(const uint32_t* flag, uint32_t target, int spin_limit) {
  for (int i = 0;; ++i) {
    if (sg_load(flag) == target) return true;
    if (i >= spin_limit) return false;
    __builtin_amdgcn_s_sleep(32);
  }
}

template <int DT, int D>
__global__ __launch_bounds__(SG_THREADS) void single_sweep_kernel(SingleParams p) {
  constexpr int ES = DT == DT_BF16 ? 2 : 4;
  constexpr int CH = D * ES / 16;
  static_assert(CH <= 16, "rows wider than 256 bytes take the two-sweep path");
  constexpr int NCH = CH / 2;
  constexpr int CHP = CH + 1;
  constexpr int NTHR = SG_THREADS;
  constexpr int RPL = NTHR / CH;              // rows per load instruction of the workgroup
  constexpr int QL = SG_ROWS / RPL;           // loads per thread: window rows (and as many planes)
  constexpr int KL = (SG_MAX_KEYS + RPL - 1) / RPL;
  constexpr int TL = SG_MAX_QTILES * 32 * CH / NTHR;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, rl = lane & 31, kg = lane >> 5;
  const int lin = xcd_major(blockIdx.x, p.n_ranges * p.n_kv_heads);
  const int h = lin / p.n_ranges, kr = lin - h * p.n_ranges;
  const int nk = p.keys_per_range;
  const int b0 = kr * nk;
  const int nb = min(nk, p.s_t - b0);
  const int n_kt = (nb + 31) >> 5;
  const int n_bits = p.n_bits, n_tables = p.n_tables;
  const int hist_w = (1 << n_bits) >> 1;  // words per table: two 16-bit bins each
  const uint32_t code_mask = (1u << n_bits) - 1u;
  const int qt0 = kr * p.q_tab_per_wg;
  const int n_qt = max(0, min(p.q_tab_per_wg, n_tables - qt0));
  const int n_qpt = (n_qt + p.q_tab_per_tile - 1) / p.q_tab_per_tile;
  const int n_mt = (p.n_planes + 31) >> 5;
  // key hashing: plane tile mt of the wave, key tiles kt0, kt0 + kstep, ...
  const int kstep = max(1, SG_WAVES / n_mt);
  const int mt = wave % n_mt, kt0 = wave / n_mt;
  const bool hash_active = kt0 < kstep;

  extern __shared__ uint4 smem[];
  uint4* sK = smem;                                                         // [nk][CHP]
  uint32_t* sBits = reinterpret_cast<uint32_t*>(sK + (size_t)nk * CHP);     // [nk][SG_BITS_PITCH]
  uint4* sQP = reinterpret_cast<uint4*>(sBits + (((size_t)nk * SG_BITS_PITCH + 3) & ~(size_t)3));  // [q_tiles * 32][CHP]
  uint32_t* sHist = reinterpret_cast<uint32_t*>(sQP + (size_t)max(p.q_tiles, 1) * 32 * CHP);       // [q_tab_per_wg][hist_w]
  float* sCol = reinterpret_cast<float*>(sHist + (((size_t)max(p.q_tab_per_wg, 1) * hist_w + 3) & ~(size_t)3));  // [16][nk]
  int* sLim = reinterpret_cast<int*>(sCol + SG_WAVES * nk);                 // [SG_ROWS]
  float* sLse = reinterpret_cast<float*>(sLim + SG_ROWS);                   // [SG_ROWS]
  int* sMiss = reinterpret_cast<int*>(sLse + SG_ROWS);                      // [0]: count, [1 ..]: tables not seen in time

  // 1. everything from memory, issued back to back
  const uint32_t epoch = p.sync[0];
  const uint32_t target = epoch + 1u;
  const uint32_t trow = tid / CH, tcol = (tid % CH) * 16;
  uint4 qpre[QL], ppre[QL], kpre[KL], tpre[TL];
  {
    // window row m = g * W + j at g * stride_head + j * stride_row from the group's first row; rows past M land at
    // or past the descriptor's end (stride_head >= W * stride_row) and read as zero
    const uint32_t qstride = (uint32_t)p.q.stride_row, hstride = (uint32_t)p.q.stride_head;
    const __amdgpu_buffer_rsrc_t qsrd = make_srd(p.q.base + (int64_t)h * p.group * p.q.stride_head,
                                                 (uint32_t)(p.group - 1) * hstride + (uint32_t)p.w * qstride);
    const __amdgpu_buffer_rsrc_t psrd = make_srd(p.planes, (uint32_t)p.n_planes * (D * ES));
    const __amdgpu_buffer_rsrc_t ksrd = make_srd(p.kb.base + (int64_t)h * p.kb.stride_head, (uint32_t)p.s_t * (uint32_t)p.kb.stride_row);
#pragma unroll
    for (int u = 0; u < QL; ++u) {
      const int m = trow + u * RPL;
      const int g = div_w(m, p.w_magic);
      qpre[u] = buf_ld16(qsrd, (uint32_t)g * hstride + (uint32_t)(m - g * p.w) * qstride + tcol);
    }
#pragma unroll
    for (int u = 0; u < QL; ++u) ppre[u] = buf_ld16(psrd, (trow + u * RPL) * (D * ES) + tcol); // planes past L*K read as zero
#pragma unroll
    for (int u = 0; u < KL; ++u) kpre[u] = buf_ld16(ksrd, (uint32_t)(b0 + trow + u * RPL) * (uint32_t)p.kb.stride_row + tcol);
#pragma unroll
    for (int u = 0; u < TL; ++u) {
      // tile t of the own-table job holds the planes of whole tables qt0 + t * q_tab_per_tile ..., padded with
      // copies of its last plane
      const int q = tid + NTHR * u;
      tpre[u] = make_uint4(0u, 0u, 0u, 0u);
      if (q < n_qpt * 32 * CH) {
        const int row = q / CH, c = q % CH;
        const int t_tab0 = qt0 + (row >> 5) * p.q_tab_per_tile;
        const int t_planes = min(p.q_tab_per_tile, qt0 + n_qt - t_tab0) * n_bits;
        const int pm = t_tab0 * n_bits + min(row & 31, t_planes - 1);
        tpre[u] = ld16(p.planes + (size_t)pm * (D * ES) + c * 16);
      }
    }
  }
  float my_lse = 1.0e30f;  // padding rows: probability 0
  if (tid < SG_ROWS && tid < p.m_rows) my_lse = p.row_lse[(size_t)h * p.m_rows + tid] * 1.4426950408889634f;

  // 2. the A/B operands pass through LDS into the fragment layout: window rows first, then the planes
  uint4 a_q[NCH], a_p[NCH];
#pragma unroll
  for (int u = 0; u < QL; ++u) smem[(trow + u * RPL) * CHP + tid % CH] = qpre[u];
  __syncthreads();
  {
    const uint4* arow = smem + (size_t)(wave * 32 + rl) * CHP + kg;
#pragma unroll
    for (int i = 0; i < NCH; ++i) a_q[i] = arow[2 * i];
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < QL; ++u) smem[(trow + u * RPL) * CHP + tid % CH] = ppre[u];
  __syncthreads();
  {
    const uint4* arow = smem + (size_t)(mt * 32 + plane_row(rl)) * CHP + kg;
#pragma unroll
    for (int i = 0; i < NCH; ++i) a_p[i] = arow[2 * i];
  }
  __syncthreads();
  // the steady-state arrays take the space over
#pragma unroll
  for (int u = 0; u < KL; ++u)
    if ((int)trow + u * RPL < n_kt * 32) sK[(trow + u * RPL) * CHP + tid % CH] = kpre[u];
#pragma unroll
  for (int u = 0; u < TL; ++u) {
    const int q = tid + NTHR * u;
    if (q < n_qpt * 32 * CH) sQP[(q / CH) * CHP + q % CH] = tpre[u];
  }
  for (int i = tid; i < n_qt * hist_w; i += NTHR) sHist[i] = 0u;
  if (tid < SG_ROWS) {
    const int m = min(tid, p.m_rows - 1);
    const int j = m - div_w(m, p.w_magic) * p.w;
    sLim[tid] = p.causal ? p.lim0 + j : INT_MAX;
    sLse[tid] = my_lse;
  }
  if (tid == 0) sMiss[0] = 0;
  __syncthreads();

  const int row = wave * 32 + rl;  // this lane's window row in the operand fragments

  // Hashes the workgroup's window rows against the 32-plane tile at LDS rows prow0 .. and adds the codes of
  // its n_tt tables (first one t_tab0) to the LDS histograms starting at hist0; optionally stores the codes.
  auto hash_rows = [&](const uint4* tile, int t_tab0, int n_tt, uint32_t* hist0, bool store_codes) {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
    const uint4* prow = tile + (size_t)plane_row(rl) * CHP + kg;
#pragma unroll
    for (int i = 0; i < NCH; ++i) Mma<DT>::run(acc, prow[2 * i], a_q[i]);
    uint32_t neg = 0u;
#pragma unroll
    for (int r = 15; r >= 0; --r) neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[r]), 31);
    const uint32_t pos = ~neg & 0xffffu;  // bit = projection >= 0
    const uint32_t other = half_other(pos, kg);
    const uint32_t word = kg ? (other | (pos << 16)) : (pos | (other << 16));
    if (row < p.m_rows)
      for (int tt = kg; tt < n_tt; tt += 2) {  // the tile's tables alternate between the two lanes that hold the row
        const uint32_t code = (word >> (tt * n_bits)) & code_mask;
        if (store_codes) p.sig_q[((size_t)h * p.m_rows + row) * n_tables + t_tab0 + tt] = (uint16_t)code;
        atomicAdd(hist0 + (size_t)tt * hist_w + (code >> 1), 1u << ((code & 1u) * 16));
      }
  };
  // Publishing the finished LDS histograms of n_tt tables (first one t_tab0): the words go to global memory, and
  // once every wave has seen its stores acknowledged (an explicit wait, then a workgroup barrier) the tables' flags
  // are raised.
  auto publish_words = [&](const uint32_t* hist0, int t_tab0, int n_tt) {
    __syncthreads();
    uint32_t* dst = p.qhist + ((size_t)h * n_tables + t_tab0) * hist_w;
    for (int i = tid; i < n_tt * hist_w; i += NTHR) sg_store(dst + i, hist0[i]);
  };
  auto publish_flags = [&](int t_tab0, int n_tt) {
    // every wave first waits until its own stores are acknowledged (the barrier alone waits for LDS traffic only)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid < n_tt) sg_store(p.flags + (size_t)h * n_tables + t_tab0 + tid, target);
  };

  // 3. window-row codes of the tables this workgroup owns
#pragma unroll 1
  for (int t = 0; t < n_qpt; ++t) {
    const int t_tab0 = qt0 + t * p.q_tab_per_tile;
    hash_rows(sQP + (size_t)t * 32 * CHP, t_tab0, min(p.q_tab_per_tile, qt0 + n_qt - t_tab0),
              sHist + (size_t)(t_tab0 - qt0) * hist_w, true);
  }
  if (n_qt > 0) publish_words(sHist, qt0, n_qt);  // acknowledged while the keys are hashed

  // 4. sign bits of the range's keys: plane tile in registers, key rows from LDS
  if (hash_active) {
#pragma unroll 1
    for (int vt = kt0; vt < n_kt; vt += kstep) {
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
      const uint4* brow = sK + (size_t)(vt * 32 + rl) * CHP + kg;
#pragma unroll
      for (int i = 0; i < NCH; ++i) Mma<DT>::run(acc, a_p[i], brow[2 * i]);
      uint32_t neg = 0u;
#pragma unroll
      for (int r = 15; r >= 0; --r) neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[r]), 31);
      const uint32_t pos = ~neg & 0xffffu;
      const uint32_t mask = pos | (half_other(pos, kg) << 16);
      if (kg == 0) sBits[(size_t)(vt * 32 + rl) * SG_BITS_PITCH + mt] = mask;
    }
  }

  publish_flags(qt0, n_qt);
  // the other tables' flags are fetched now and looked at after the scores
  uint32_t flag_seen = target;
  if (tid < n_tables) flag_seen = sg_load(p.flags + (size_t)h * n_tables + tid);

  // 5. pooled probabilities: window rows (A) times keys (B), lane = key, registers = rows
  {
    float lse[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) lse[r] = sLse[wave * 32 + acc_row(r, kg)];
#pragma unroll 1
    for (int nt = 0; nt < n_kt; ++nt) {
      const int kbase = b0 + nt * 32;  // block index of the tile's first key; key i is visible to row j iff i <= lim0 + j
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
      const uint4* brow = sK + (size_t)(nt * 32 + rl) * CHP + kg;
#pragma unroll
      for (int i = 0; i < NCH; ++i) Mma<DT>::run(acc, a_q[i], brow[2 * i]);
      const int kidx = kbase + rl;
      const bool partial = (kbase + 32 > b0 + nb) || (p.causal && (kbase + 31 > p.lim0));  // wave-uniform
      float col = 0.0f;
      if (!partial) {
#pragma unroll
        for (int r = 0; r < 16; ++r) col += fast_exp2(fmaf(acc[r], p.scale2, -lse[r]));
      } else {
        const bool in_range = kidx < b0 + nb;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int4 lim4 = *reinterpret_cast<const int4*>(&sLim[wave * 32 + acc_row(4 * g4, kg)]);
          const int lims[4] = {lim4.x, lim4.y, lim4.z, lim4.w};
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float e = fast_exp2(fmaf(acc[4 * g4 + u], p.scale2, -lse[4 * g4 + u]));
            col += (in_range & (kidx <= lims[u])) ? e : 0.0f;
          }
        }
      }
      col = half_pair_sum(col);
      if (kg == 0) sCol[wave * nk + nt * 32 + rl] = col;
    }
  }
  __syncthreads();
  for (int t = tid; t < nb; t += NTHR) {
    float v = 0.0f;
#pragma unroll
    for (int w = 0; w < SG_WAVES; ++w) v += sCol[w * nk + t];
    p.s_part[(size_t)h * p.s_t + b0 + t] = v;
  }

  // 6. which tables' histograms are there?  Each flag is waited for by one thread; what is missing is listed.
  for (int t = tid; t < n_tables; t += NTHR)
    if (!(t == tid && flag_seen == target) && !sg_wait_flag(p.flags + (size_t)h * n_tables + t, target, p.spin_limit))
      sMiss[1 + atomicAdd(&sMiss[0], 1)] = t;
  __syncthreads();
  const int n_miss = sMiss[0];
  for (int mi = 0; mi < n_miss; ++mi) {  // workgroup-uniform; normally never entered
    const int t = sMiss[1 + mi];
    // the table's planes into tile 0 of the own-table area (padded with copies of its last plane), its histogram at sHist
    for (int q = tid; q < 32 * CH; q += NTHR) {
      const int prow = q / CH, c = q % CH;
      sQP[prow * CHP + c] = ld16(p.planes + (size_t)(t * n_bits + min(prow, n_bits - 1)) * (D * ES) + c * 16);
    }
    for (int i = tid; i < hist_w; i += NTHR) sHist[i] = 0u;
    __syncthreads();
    hash_rows(sQP, t, 1, sHist, false);
    publish_words(sHist, t, 1);
    publish_flags(t, 1);
    __syncthreads();
  }
  // 7. collision counts (Alg. 1 step 6): SG_LPK lanes per key, tables sub, sub + SG_LPK, ...
  {
    const uint32_t* hist = p.qhist + (size_t)h * n_tables * hist_w;
    for (int kq = tid; kq < nb * SG_LPK; kq += NTHR) {
      const int key = kq / SG_LPK, sub = kq % SG_LPK;
      const uint32_t* bits = sBits + (size_t)key * SG_BITS_PITCH;
      int sum = 0;
      for (int tb = sub; tb < n_tables; tb += 4 * SG_LPK) {
        uint32_t hv[4], sh[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int t = min(tb + u * SG_LPK, n_tables - 1);
          const int bitpos = t * n_bits;
          const int w0 = bitpos >> 5, s0 = bitpos & 31;
          const uint64_t two = (uint64_t)bits[w0] | ((uint64_t)bits[w0 + 1] << 32);
          const uint32_t code = (uint32_t)(two >> s0) & code_mask;
          hv[u] = sg_load(hist + (size_t)t * hist_w + (code >> 1));
          sh[u] = (code & 1u) * 16;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) sum += (tb + u * SG_LPK < n_tables) ? (int)((hv[u] >> sh[u]) & 0xffffu) : 0;
      }
      sum += lane_xor1(sum);
      sum += lane_xor2(sum);
      sum += lane_xor4(sum, (tid & 4) != 0);
      if (sub == 0) p.cnt[(size_t)h * p.s_t + b0 + key] = sum;
    }
  }
  // key codes for the stage outputs, on request
  if (p.sig_k) {
    for (int it = tid; it < nb * n_tables; it += NTHR) {
      const int key = it / n_tables, t = it - key * n_tables;
      const uint32_t* bits = sBits + (size_t)key * SG_BITS_PITCH;
      const int bitpos = t * n_bits;
      const int w0 = bitpos >> 5, s0 = bitpos & 31;
      const uint64_t two = (uint64_t)bits[w0] | ((uint64_t)bits[w0 + 1] << 32);
      p.sig_k[((size_t)h * p.s_t + b0 + key) * n_tables + t] = (uint16_t)((uint32_t)(two >> s0) & code_mask);
    }
  }
  // the last workgroup of the launch advances the epoch for the next one
  if (tid == 0) {
    const uint32_t done = atomicAdd(p.sync + 1, 1u);
    if (done == gridDim.x - 1) {
      p.sync[1] = 0u;
      p.sync[0] = target;
    }
  }
}

// ---- host side ----
size_t single_lds_bytes(int dtype, int head_dim, int keys_per_range, int q_tiles, int q_tab_per_wg, int n_bits, int n_tables) {
  const int es = dtype == DT_BF16 ? 2 : 4;
  const size_t pitch = (size_t)(head_dim * es / 16 + 1) * 16;
  const size_t hist_w = ((size_t)1 << n_bits) >> 1;
  const size_t staging = (size_t)SG_ROWS * pitch;
  const size_t steady = keys_per_range * pitch + (((size_t)keys_per_range * SG_BITS_PITCH + 3) & ~(size_t)3) * 4 +
                        (size_t)(q_tiles > 1 ? q_tiles : 1) * 32 * pitch + (((size_t)(q_tab_per_wg > 1 ? q_tab_per_wg : 1) * hist_w + 3) & ~(size_t)3) * 4 +
                        (size_t)SG_WAVES * keys_per_range * 4 + (size_t)SG_ROWS * 8 + ((size_t)n_tables + 4) * 4;
  return ((steady > staging ? steady : staging) + 15) & ~(size_t)15;
}
int single_max_rows() { return SG_ROWS; }
int single_max_keys() { return SG_MAX_KEYS; }
int single_max_qtiles() { return SG_MAX_QTILES; }

template <int DT, int D>
static hipError_t launch_single_t(const SingleParams& p, hipStream_t st) {
  const size_t lds = single_lds_bytes(DT, D, p.keys_per_range, p.q_tiles, p.q_tab_per_wg, p.n_bits, p.n_tables);
  if (lds > 160 * 1024 || p.m_rows > SG_ROWS || p.keys_per_range > SG_MAX_KEYS || p.q_tiles > SG_MAX_QTILES || p.n_planes > 512)
    return hipErrorInvalidValue;
  hipLaunchKernelGGL((single_sweep_kernel<DT, D>), dim3(p.n_ranges * p.n_kv_heads), dim3(SG_THREADS), lds, st, p);
  return hipGetLastError();
}

hipError_t launch_single(int dtype, int head_dim, const SingleParams& p, hipStream_t st) {
  if (dtype == DT_BF16 && head_dim == 128) return launch_single_t<DT_BF16, 128>(p, st);
  if (dtype == DT_BF16 && head_dim == 64) return launch_single_t<DT_BF16, 64>(p, st);
  if (dtype == DT_F32 && head_dim == 64) return launch_single_t<DT_F32, 64>(p, st);
  return hipErrorInvalidValue;
}
bool single_supports(int dtype, int head_dim) { return dtype == DT_BF16 || head_dim == 64; }

hipError_t init_single_attributes() {
  const void* fns[] = {reinterpret_cast<const void*>(&single_sweep_kernel<DT_BF16, 128>),
                       reinterpret_cast<const void*>(&single_sweep_kernel<DT_BF16, 64>),
                       reinterpret_cast<const void*>(&single_sweep_kernel<DT_F32, 64>)};
  for (const void* f : fns) {
    hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace lkv
